// Causal GQA attention on the gfx950 matrix cores, varlen-packed: no token attends across
// sequences (paper Sec. 2.2) and the work list is rebuilt whenever pruning shrinks the batch.
//
// A work item is (one sequence, one block of queries, one KV head).  The workgroup has 8
// wavefronts; wavefront w serves query head kvh*G + w % G (G = query heads per KV head) and the
// 32-query block w / G of the item, so one K/V tile staged in LDS is shared by all G heads.
//
// Everything is computed transposed so that a lane owns ONE query:
//   S^T[key, query] = K Q^T      (A operand = K tile rows from LDS, B operand = Q from registers)
//   O^T[d, query]  += V^T P^T    (A operand = V^T tile from LDS,   B operand = P^T = the S^T
//                                 accumulator registers themselves, converted to bf16)
// The 32x32 accumulator layout gives lane l the column l % 32 and rows (e/4)*8 + (l/32)*4 + e%4;
// those rows, read as the 16 contraction slots of the next MFMA, are keys {0-3, 8-11} for the low
// half-wave and {4-7, 12-15} for the high one, so the V^T operand is fetched in that key order.
// Online softmax needs one cross-lane exchange (l <-> l ^ 32) per K/V tile.
// V^T comes from the [kv head][d][column] buffer written by the V transposition step; a sequence's
// columns start at a multiple of 64 so every 16-byte chunk is aligned.
#include "common.h"

namespace prism {

static constexpr int HD = 128;           // head_dim served by this kernel
static constexpr int BKV = 64;           // keys per staged tile

template <int G>
__global__ __launch_bounds__(512) void attention_bf16_kernel(const bf16 *__restrict__ QKV, const bf16 *__restrict__ Vt,
                                                             int64_t vt_stride, const AttnTile *__restrict__ tiles,
                                                             int nq, int nkv, bf16 *__restrict__ out) {
  constexpr int QB = 8 / G;              // 32-query blocks per item
  constexpr int BQ = 32 * QB;
  __shared__ __align__(16) bf16 lK[2][BKV * HD];     // [key][d], 16 chunks per row, swizzled
  __shared__ __align__(16) bf16 lV[2][HD * BKV];     // [d][key], 8 chunks per row, swizzled

  const AttnTile it = tiles[blockIdx.x];
  const int kvh = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int hq = kvh * G + wave % G, qb = wave / G;
  const int row_elems = (nq + 2 * nkv) * HD;
  const int L = it.seq_len;
  const int q_lo = it.q0 + qb * 32;                               // first query of this wave
  const int q_last_blk = (it.q0 + BQ < L ? it.q0 + BQ : L) - 1;   // last valid query of the item
  const int n_kt = q_last_blk / BKV + 1;

  // ---- Q fragments: B operand, lane -> query (lane % 32), d = kk*16 + (lane/32)*8 .. +8
  int qi = q_lo + (lane & 31);
  const int qi_ld = qi < L ? qi : L - 1;
  bf16x8 qf[HD / 16];
  {
    const bf16 *qp = QKV + (int64_t)(it.seq_row0 + qi_ld) * row_elems + (int64_t)hq * HD + (lane >> 5) * 8;
#pragma unroll
    for (int kk = 0; kk < HD / 16; ++kk) qf[kk] = *reinterpret_cast<const bf16x8 *>(qp + kk * 16);
  }

  // ---- staging addresses: 1024 chunks of K and 1024 of V^T per tile, 2 + 2 per thread
  const bf16 *gK[2], *gV[2];
  int sK[2], sV[2], krow[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = tid + i * 512;
    const int kr = c / 16, kc = c % 16;                            // K: key row, chunk
    krow[i] = kr;
    gK[i] = QKV + (int64_t)(nq + kvh) * HD + kc * 8;               // + (seq_row0 + key) * row_elems later
    sK[i] = kr * HD + ((kc ^ (kr & 15)) * 8);
    const int vr = c / 8, vc = c % 8;                              // V^T: d row, chunk of 8 keys
    gV[i] = Vt + ((int64_t)kvh * HD + vr) * vt_stride + it.vt_col0 + vc * 8;
    sV[i] = vr * BKV + ((vc ^ (vr & 7)) * 8);
  }
  auto load_tile = [&](int kt, bf16x8 (&rk)[2], bf16x8 (&rv)[2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      int key = kt * BKV + krow[i];
      key = key < L ? key : L - 1;
      rk[i] = *reinterpret_cast<const bf16x8 *>(gK[i] + (int64_t)(it.seq_row0 + key) * row_elems);
      rv[i] = *reinterpret_cast<const bf16x8 *>(gV[i] + kt * BKV);
    }
  };
  auto store_tile = [&](int buf, const bf16x8 (&rk)[2], const bf16x8 (&rv)[2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      *reinterpret_cast<bf16x8 *>(&lK[buf][sK[i]]) = rk[i];
      *reinterpret_cast<bf16x8 *>(&lV[buf][sV[i]]) = rv[i];
    }
  };

  f32x16 o[HD / 32];
#pragma unroll
  for (int t = 0; t < HD / 32; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[t][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c_exp = 1.4426950408889634f / sqrtf((float)HD);      // log2(e) / sqrt(hd)

  bf16x8 rk[2], rv[2];
  load_tile(0, rk, rv);
  store_tile(0, rk, rv);
  __syncthreads();

  const int q_hi_wave = q_lo + 31;
  for (int kt = 0; kt < n_kt; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < n_kt;
    if (more) load_tile(kt + 1, rk, rv);

    if (kt * BKV <= q_hi_wave && q_lo < L) {       // wave-uniform: tile not entirely in this wave's future
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
          const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(&lK[cur][r * HD + ((ch ^ (r & 15)) * 8)]);
          s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s[kb], 0, 0, 0);
        }
      }
      // ---- causal mask + online softmax (lane owns query qi; partner lane ^ 32 owns the other keys)
      const bool diag = kt * BKV + BKV - 1 > q_lo;   // tile may contain keys after some query of the wave
      float mx = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          if (diag) {
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
      bf16x8 pf[4];                                   // P^T as B operands: 4 contraction steps of 16 keys
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float p = __builtin_amdgcn_exp2f(s[kb][e] * c_exp - mb);
          psum += p;
          pf[kb * 2 + (e >> 3)][e & 7] = (bf16)p;
        }
      l_run = l_run * alpha + psum;
      m_run = m_new;
#pragma unroll
      for (int t = 0; t < HD / 32; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[t][e] *= alpha;
      // ---- O^T += V^T P^T
#pragma unroll
      for (int t = 0; t < HD / 32; ++t) {
        const int r = t * 32 + (lane & 31);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          // contraction slots 0-3 <- keys ks*16 + (lane/32)*4 .. +4 ; slots 4-7 <- the same + 8
          const int c0 = ks * 2, c1 = ks * 2 + 1, half = (lane >> 5) * 4;
          const bf16x4 v0 = *reinterpret_cast<const bf16x4 *>(&lV[cur][r * BKV + ((c0 ^ (r & 7)) * 8) + half]);
          const bf16x4 v1 = *reinterpret_cast<const bf16x4 *>(&lV[cur][r * BKV + ((c1 ^ (r & 7)) * 8) + half]);
          bf16x8 vf;
          vf[0] = v0[0]; vf[1] = v0[1]; vf[2] = v0[2]; vf[3] = v0[3];
          vf[4] = v1[0]; vf[5] = v1[1]; vf[6] = v1[2]; vf[7] = v1[3];
          o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[ks], o[t], 0, 0, 0);
        }
      }
    }
    if (more) store_tile(cur ^ 1, rk, rv);
    __syncthreads();
  }

  // ---- normalise and store: lane holds d = t*32 + (e/4)*8 + (lane/32)*4 + e%4 of query qi
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (qi < L) {
    const float inv = 1.0f / l_tot;
    bf16 *op = out + (int64_t)(it.seq_row0 + qi) * nq * HD + (int64_t)hq * HD + (lane >> 5) * 4;
#pragma unroll
    for (int t = 0; t < HD / 32; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 v;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = (bf16)(o[t][g * 4 + j] * inv);
        *reinterpret_cast<bf16x4 *>(op + t * 32 + g * 8) = v;
      }
  }
}

bool attention_bf16_supported(int nq, int nkv, int hd) {
  if (hd != HD || nkv <= 0 || nq % nkv != 0) return false;
  const int g = nq / nkv;
  return g == 1 || g == 2 || g == 4 || g == 8;
}

int attention_bf16_block_queries(int nq, int nkv) { return 32 * (8 / (nq / nkv)); }

int launch_attention_bf16(const bf16 *QKV, const bf16 *Vt, int64_t vt_stride, const AttnTile *tiles, int n_tiles,
                          int T, int nq, int nkv, int hd, bf16 *out, hipStream_t s) {
  PRISM_REQUIRE(QKV && Vt && tiles && out && n_tiles >= 0 && T >= 0, PRISM_EINVAL, "attention bf16: bad arguments");
  PRISM_REQUIRE(attention_bf16_supported(nq, nkv, hd), PRISM_EUNSUPPORTED,
                "attention bf16: needs head_dim 128 and 1, 2, 4 or 8 query heads per KV head (got hd %d, %d/%d)", hd, nq, nkv);
  PRISM_REQUIRE(vt_stride % 8 == 0, PRISM_EINVAL, "attention bf16: V^T row stride must be a multiple of 8");
  if (n_tiles == 0) return PRISM_OK;
  dim3 grid(n_tiles, nkv);
  switch (nq / nkv) {
    case 1: attention_bf16_kernel<1><<<grid, 512, 0, s>>>(QKV, Vt, vt_stride, tiles, nq, nkv, out); break;
    case 2: attention_bf16_kernel<2><<<grid, 512, 0, s>>>(QKV, Vt, vt_stride, tiles, nq, nkv, out); break;
    case 4: attention_bf16_kernel<4><<<grid, 512, 0, s>>>(QKV, Vt, vt_stride, tiles, nq, nkv, out); break;
    default: attention_bf16_kernel<8><<<grid, 512, 0, s>>>(QKV, Vt, vt_stride, tiles, nq, nkv, out); break;
  }
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

}  // namespace prism
