// Causal GQA attention on the gfx950 matrix cores (16-bit operands), varlen-packed: no token attends across
// sequences (paper Sec. 2.2) and the work list is rebuilt whenever pruning shrinks the batch.
//
// A work item is (one sequence, one block of queries, one KV head).  The workgroup has 8
// wavefronts; wavefront w serves query head kvh*G + w % G (G = query heads per KV head) and the
// 32-query block w / G of the item, so one K/V tile staged in LDS is shared by all G heads.
//
// Everything is computed transposed so that a lane owns ONE query:
//   S^T[key, query] = K Q^T      (A operand = K tile rows from LDS, B operand = Q from registers)
//   O^T[d, query]  += V^T P^T    (A operand = V^T tile from LDS,   B operand = P^T = the S^T
//                                 accumulator registers themselves, converted to f16)
// The 32x32 accumulator layout gives lane l the column l % 32 and rows (e/4)*8 + (l/32)*4 + e%4;
// those rows, read as the 16 contraction slots of the next MFMA, are keys {0-3, 8-11} for the low
// half-wave and {4-7, 12-15} for the high one.  The V^T tile is stored in LDS with the keys of every group of
// 16 in exactly that order (0-3, 8-11, 4-7, 12-15), so a lane's operand is ONE 16-byte chunk, and the chunks
// are XOR-swizzled by bits 1..3 of the row, which spreads the 16 lanes served per cycle over all 64 banks.
// Online softmax needs one cross-lane exchange (l <-> l ^ 32) per K/V tile.
// q and k come from the finished [T, (nq + nkv) * hd] buffer in the operand type OT (bf16 or IEEE half).
// V^T comes from the [kv head][d][column] buffer of the V finishing step, always IEEE half: the
// second contraction runs on the f16 MFMA in both modes so that the probabilities keep 11
// significand bits.  A sequence's columns
// start at a multiple of 64 so every 16-byte chunk is aligned.
#include <type_traits>

#include "common.h"

namespace prism {

static constexpr int HD = 128;           // head_dim served by this kernel
static constexpr int BKV = 64;           // keys per staged tile

template <typename OT, int G>
__global__ __launch_bounds__(512) void attention_16_kernel(const OT *__restrict__ QK, const f16 *__restrict__ Vt,
                                                           int64_t vt_stride, const AttnTile *__restrict__ tiles,
                                                           int nq, int nkv, OT *__restrict__ out) {
  typedef typename Mfma<OT>::vec8 vec8;
  typedef typename Mfma<OT>::vec4 vec4;
  constexpr int QB = 8 / G;              // 32-query blocks per item
  constexpr int BQ = 32 * QB;
  __shared__ __align__(16) OT lK[2][BKV * HD];       // [key][d], 16 chunks per row, swizzled
  __shared__ __align__(16) f16 lV[2][HD * BKV];      // [d][key, permuted within groups of 16], 8 chunks per row, swizzled

  const AttnTile it = tiles[blockIdx.x];
  const int kvh = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int hq = kvh * G + wave % G, qb = wave / G;
  const int row_elems = (nq + nkv) * HD;
  const int L = it.seq_len;
  const int q_lo = it.q0 + qb * 32;                               // first query of this wave
  const int q_last_blk = (it.q0 + BQ < L ? it.q0 + BQ : L) - 1;   // last valid query of the item
  const int n_kt = q_last_blk / BKV + 1;

  // ---- Q fragments: B operand, lane -> query (lane % 32), d = kk*16 + (lane/32)*8 .. +8
  int qi = q_lo + (lane & 31);
  const int qi_ld = qi < L ? qi : L - 1;
  vec8 qf[HD / 16];
  {
    const OT *qp = QK + (int64_t)(it.seq_row0 + qi_ld) * row_elems + (int64_t)hq * HD + (lane >> 5) * 8;
#pragma unroll
    for (int kk = 0; kk < HD / 16; ++kk) qf[kk] = *reinterpret_cast<const vec8 *>(qp + kk * 16);
  }

  // ---- staging addresses: 1024 chunks of K and 1024 of V^T per tile, 2 + 2 per thread
  const OT *gK[2];
  const f16 *gV[2];
  int sK[2], sV[2], krow[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = tid + i * 512;
    const int kr = c / 16, kc = c % 16;                            // K: key row, chunk
    krow[i] = kr;
    gK[i] = QK + (int64_t)(nq + kvh) * HD + kc * 8;               // + (seq_row0 + key) * row_elems later
    sK[i] = kr * HD + ((kc ^ (kr & 15)) * 8);
    const int vr = c / 8, vc = c % 8;                              // V^T: d row, 8 consecutive keys
    gV[i] = Vt + ((int64_t)kvh * HD + vr) * vt_stride + it.vt_col0 + vc * 8;
    // keys 0-3 of the 8 go to chunk 2*(vc/2), keys 4-7 to chunk 2*(vc/2)+1, both at half vc % 2
    sV[i] = vr * BKV + ((((vc & ~1)) ^ ((vr >> 1) & 7)) * 8) + (vc & 1) * 4;
  }
  auto load_tile = [&](int kt, vec8 (&rk)[2], f16x8 (&rv)[2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      int key = kt * BKV + krow[i];
      key = key < L ? key : L - 1;
      rk[i] = *reinterpret_cast<const vec8 *>(gK[i] + (int64_t)(it.seq_row0 + key) * row_elems);
      rv[i] = *reinterpret_cast<const f16x8 *>(gV[i] + kt * BKV);
    }
  };
  auto store_tile = [&](int buf, const vec8 (&rk)[2], const f16x8 (&rv)[2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      *reinterpret_cast<vec8 *>(&lK[buf][sK[i]]) = rk[i];
      f16x4 lo4, hi4;
      lo4[0] = rv[i][0]; lo4[1] = rv[i][1]; lo4[2] = rv[i][2]; lo4[3] = rv[i][3];
      hi4[0] = rv[i][4]; hi4[1] = rv[i][5]; hi4[2] = rv[i][6]; hi4[3] = rv[i][7];
      *reinterpret_cast<f16x4 *>(&lV[buf][sV[i]]) = lo4;
      *reinterpret_cast<f16x4 *>(&lV[buf][sV[i] ^ 8]) = hi4;          // the neighbouring chunk (chunk index ^ 1)
    }
  };

  f32x16 o[HD / 32];
#pragma unroll
  for (int t = 0; t < HD / 32; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[t][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c_exp = 1.4426950408889634f / sqrtf((float)HD);      // log2(e) / sqrt(hd)

  vec8 rk[2];
  f16x8 rv[2];
  load_tile(0, rk, rv);
  store_tile(0, rk, rv);
  __syncthreads();

  const int q_hi_wave = q_lo + 31;
  for (int kt = 0; kt < n_kt; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < n_kt;
    if (more) load_tile(kt + 1, rk, rv);

    // One K/V tile for this wave.  MASK: the tile holds keys after some query of the wave (the causal diagonal); the
    // two variants are separate code so that tiles below the diagonal carry no masking arithmetic at all.
    auto tile_step = [&](auto mask_tag) {
      constexpr bool MASK = decltype(mask_tag)::value;
      // ---- S^T = K Q^T for the 2 key blocks of the tile
      f32x16 s[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int e = 0; e < 16; ++e) s[kb][e] = 0.f;
        const int r = kb * 32 + (lane & 31);
#pragma unroll
        for (int kk = 0; kk < HD / 16; ++kk) {
          const int ch = kk * 2 + (lane >> 5);
          const vec8 kf = *reinterpret_cast<const vec8 *>(&lK[cur][r * HD + ((ch ^ (r & 15)) * 8)]);
          s[kb] = Mfma<OT>::mma(kf, qf[kk], s[kb]);
        }
      }
      // ---- causal mask + online softmax (lane owns query qi; partner lane ^ 32 owns the other keys)
      float mx = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          if (MASK) {
            const int key = kt * BKV + kb * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
            if (key > qi) s[kb][e] = -INFINITY;
          }
          mx = fmaxf(mx, s[kb][e]);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run, mx);
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c_exp);
      const float mb = m_new * c_exp;
      float psum = 0.f;
      f16x8 pf[4];                                    // P^T as B operands: 4 contraction steps of 16 keys
      typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
      const f16x2 ones = {(f16)1.0f, (f16)1.0f};
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
          f16x2 ph;
          ph[0] = (f16)__builtin_amdgcn_exp2f(s[kb][e] * c_exp - mb);       // p <= 1: no overflow
          ph[1] = (f16)__builtin_amdgcn_exp2f(s[kb][e + 1] * c_exp - mb);
          // the denominator sums the ROUNDED weights the numerator uses (one dot-product instruction per pair): the output
          // stays an exactly normalised average of V rows and the rounding of p cancels to first order
          psum = __builtin_amdgcn_fdot2(ph, ones, psum, false);
          pf[kb * 2 + (e >> 3)][e & 7] = ph[0];
          pf[kb * 2 + (e >> 3)][(e & 7) + 1] = ph[1];
        }
      l_run = l_run * alpha + psum;
      m_run = m_new;
      // the running maxima usually settle after a few tiles.  The ballot goes through an opaque asm so that the
      // compiler cannot turn the branch back into an unconditional multiply (x * 1 == x makes the two equivalent).
      unsigned long long moved = __builtin_amdgcn_ballot_w64(alpha != 1.0f);
      asm volatile("" : "+s"(moved));
      if (moved != 0) {
#pragma unroll
        for (int t = 0; t < HD / 32; ++t)
#pragma unroll
          for (int e = 0; e < 16; ++e) o[t][e] *= alpha;
      }
      // ---- O^T += V^T P^T
#pragma unroll
      for (int t = 0; t < HD / 32; ++t) {
        const int r = t * 32 + (lane & 31);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          // contraction slots 0-3 <- keys ks*16 + (lane/32)*4 .. +4 ; slots 4-7 <- the same + 8: chunk 2 ks + lane/32
          const int ch = ks * 2 + (lane >> 5);
          const f16x8 vf = *reinterpret_cast<const f16x8 *>(&lV[cur][r * BKV + ((ch ^ ((r >> 1) & 7)) * 8)]);
          o[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf[ks], o[t], 0, 0, 0);
        }
      }
        };
    if (kt * BKV <= q_hi_wave && q_lo < L) {       // wave-uniform: tile not entirely in this wave's future
      if (kt * BKV + BKV - 1 > q_lo) tile_step(std::true_type{});
      else tile_step(std::false_type{});
    }
    if (more) store_tile(cur ^ 1, rk, rv);
    __syncthreads();
  }

  // ---- normalise and store: lane holds d = t*32 + (e/4)*8 + (lane/32)*4 + e%4 of query qi
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (qi < L) {
    const float inv = 1.0f / l_tot;
    OT *op = out + (int64_t)(it.seq_row0 + qi) * nq * HD + (int64_t)hq * HD + (lane >> 5) * 4;
#pragma unroll
    for (int t = 0; t < HD / 32; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        vec4 v;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = from_f32<OT>(o[t][g * 4 + j] * inv);
        *reinterpret_cast<vec4 *>(op + t * 32 + g * 8) = v;
      }
  }
}

bool attention_16_supported(int nq, int nkv, int hd) {
  if (hd != HD || nkv <= 0 || nq % nkv != 0) return false;
  const int g = nq / nkv;
  return g == 1 || g == 2 || g == 4 || g == 8;
}

template <typename OT>
static void launch_typed(dim3 grid, int g, const OT *QK, const f16 *Vt, int64_t vt_stride, const AttnTile *tiles, int nq,
                         int nkv, OT *out, hipStream_t s) {
  switch (g) {
    case 1: attention_16_kernel<OT, 1><<<grid, 512, 0, s>>>(QK, Vt, vt_stride, tiles, nq, nkv, out); break;
    case 2: attention_16_kernel<OT, 2><<<grid, 512, 0, s>>>(QK, Vt, vt_stride, tiles, nq, nkv, out); break;
    case 4: attention_16_kernel<OT, 4><<<grid, 512, 0, s>>>(QK, Vt, vt_stride, tiles, nq, nkv, out); break;
    default: attention_16_kernel<OT, 8><<<grid, 512, 0, s>>>(QK, Vt, vt_stride, tiles, nq, nkv, out); break;
  }
}

int launch_attention_16(int dtype, const void *QK, const void *Vt, int64_t vt_stride, const AttnTile *tiles, int n_tiles,
                        int T, int nq, int nkv, int hd, void *out, hipStream_t s) {
  PRISM_REQUIRE(QK && Vt && tiles && out && n_tiles >= 0 && T >= 0 && is16(dtype), PRISM_EINVAL, "attention: bad arguments");
  PRISM_REQUIRE(attention_16_supported(nq, nkv, hd), PRISM_EUNSUPPORTED,
                "attention: 16-bit modes need head_dim 128 and 1, 2, 4 or 8 query heads per KV head (got hd %d, %d/%d)", hd, nq, nkv);
  PRISM_REQUIRE(vt_stride % 8 == 0, PRISM_EINVAL, "attention: V^T row stride must be a multiple of 8");
  if (n_tiles == 0) return PRISM_OK;
  dim3 grid(n_tiles, nkv);
  if (dtype == PRISM_DTYPE_BF16)
    launch_typed<bf16>(grid, nq / nkv, (const bf16 *)QK, (const f16 *)Vt, vt_stride, tiles, nq, nkv, (bf16 *)out, s);
  else
    launch_typed<f16>(grid, nq / nkv, (const f16 *)QK, (const f16 *)Vt, vt_stride, tiles, nq, nkv, (f16 *)out, s);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

}  // namespace prism
