// Causal GQA attention on the gfx950 matrix cores (16-bit operands), varlen-packed: no token attends across
// sequences (paper Sec. 2.2) and the work list is rebuilt whenever pruning shrinks the batch.
//
// A work item is (one sequence, one block of queries, one KV head).  The workgroup has NW = 4
// wavefronts (8 when G = 8); wavefront w serves query head kvh*G + w % G (G = query heads per KV head) and the
// 32-query block w / G of the item, so one K/V tile staged in LDS is shared by all G heads.
//
// Everything is computed transposed so that a lane owns ONE query:
//   S^T[key, query] = K Q^T      (A operand = K tile rows from LDS, B operand = Q from registers)
//   O^T[d, query]  += V^T P^T    (A operand = V^T tile from LDS,   B operand = P^T = the S^T
//                                 accumulator registers themselves, converted to f16)
// The 32x32 accumulator layout gives lane l the column l % 32 and rows (e/4)*8 + (l/32)*4 + e%4;
// those rows, read as the 16 contraction slots of the next MFMA, are keys {0-3, 8-11} for the low
// half-wave and {4-7, 12-15} for the high one.  The V^T buffer in memory already holds the keys of every group of
// 16 in exactly that order (0-3, 8-11, 4-7, 12-15: key p of a sequence sits at column p with bits 2 and 3 swapped), so
// a lane's operand is ONE 16-byte chunk and a tile is staged as it is.  K and V^T tiles go from memory to LDS without
// passing through registers; chunks are XOR-swizzled by the row, which spreads the 16 lanes served per cycle over all
// 64 banks.
// Online softmax needs one cross-lane exchange (l <-> l ^ 32) per K/V tile.
// q and k come from the finished [T, (nq + nkv) * hd] buffer in the operand type OT (bf16 or IEEE half).
// V^T comes from the [kv head][d][column] buffer of the V finishing step, always IEEE half: the
// second contraction runs on the f16 MFMA in both modes so that the probabilities keep 11
// significand bits.  A sequence's columns
// start at a multiple of 64 so every 16-byte chunk is aligned.
// Shared prefix (paper Sec. 3.3: every (query, candidate) sequence begins with the same query): positions below
// pre_len of a work item's sequence have their q/k rows stored once, at pre_row0 + position, for all sequences of the
// launch; the K staging picks the row per key.  V^T needs no such case: every sequence's columns cover all its
// positions.  The output row base is a field of its own (out_base), so that a launch can read q and k in one row layout
// and write its output in another.
#include <type_traits>

#include "common.h"

namespace prism {

static constexpr int HD = 128;           // head_dim served by this kernel
static constexpr int BKV = 64;           // keys per staged tile
#define PRISM_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define PRISM_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

// A lane's value and the value of lane l ^ 32, as an unordered pair: one register swap between the two half-waves (no
// LDS round trip, nothing to wait for).  v_permlane32_swap exchanges the upper half of its first operand with the lower
// half of its second; with the same value in both, the two results hold the lower half-wave's and the upper half-wave's
// value in every lane.
__device__ __forceinline__ void half_wave_pair(float x, float &lo, float &hi) {
  typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
  const unsigned u = __float_as_uint(x);
  const u32x2 r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  lo = __uint_as_float(r[0]);
  hi = __uint_as_float(r[1]);
}

template <typename OT, int G, int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attention_16_kernel(const OT *__restrict__ QK, const f16 *__restrict__ Vt, int64_t vt_stride,
                         const AttnTile *__restrict__ tiles, int nq, int nkv, OT *__restrict__ out) {
  typedef typename Mfma<OT>::vec8 vec8;
  typedef typename Mfma<OT>::vec4 vec4;
  constexpr int QB = NW / G;             // 32-query blocks per item
  constexpr int NT = NW * 64;            // threads
  constexpr int BQ = 32 * QB;
  // Two stages, each its own LDS object and chosen at compile time: the compiler then knows that the loads in flight
  // towards one stage cannot alias the reads of the other and does not wait for them before those reads.
  __shared__ __align__(16) OT lK0[BKV * HD], lK1[BKV * HD];   // [key][d]: 16 chunks of 16 bytes per row, XOR-swizzled by the row
  __shared__ __align__(16) f16 lV0[HD * BKV], lV1[HD * BKV];  // [d][column of the tile]: 8 chunks per row, XOR-swizzled by the row

  // consecutive workgroup ids go to consecutive XCDs: with the KV head in the low digits of the id, all query blocks
  // of one (sequence, KV head) run on one XCD when nkv is a multiple of 8, one after the other, so its L2 holds their K/V
  const int kvh = blockIdx.x % nkv;
  const AttnTile it = tiles[blockIdx.x / nkv];
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
    const OT *qp = QK + (int64_t)(it.row_base + qi_ld) * row_elems + (int64_t)hq * HD + (lane >> 5) * 8;   // queries are never prefix positions
#pragma unroll
    for (int kk = 0; kk < HD / 16; ++kk) qf[kk] = *reinterpret_cast<const vec8 *>(qp + kk * 16);
  }

  // ---- staging without registers (global_load_lds_dwordx4): a wave instruction moves 64 chunks of 16 bytes to 1 KiB of
  // consecutive LDS, i.e. 4 key rows of K or 8 d rows of V^T; the tile takes 16 + 16 of them, NI + NI per wave.  The
  // swizzle is applied on the source side: LDS slot p of K row r receives chunk p ^ (r % 16), slot p of V^T row r chunk
  // p ^ ((r / 2) % 8), so that the 16 lanes served per cycle, which read one logical chunk of 16 consecutive rows,
  // touch all 64 banks.
  constexpr int NI = 16 / NW;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  // Byte offsets of this lane's chunks from the tile's first K row and first V^T column: fixed for the whole item, so
  // a tile costs one wave-uniform base address per operand and no per-lane address arithmetic.
  uint32_t oK[NI], oV[NI];
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    const int kr = (wave * NI + j) * 4 + (lane >> 4);
    oK[j] = ((uint32_t)kr * (uint32_t)row_elems + (uint32_t)(((lane & 15) ^ (kr & 15)) * 8)) * 2u;
    const int vr = (wave * NI + j) * 8 + (lane >> 3);
    oV[j] = ((uint32_t)vr * (uint32_t)vt_stride + (uint32_t)(((lane & 7) ^ ((vr >> 1) & 7)) * 8)) * 2u;   // < 4 GiB: checked by the launcher
  }
  const char *const kcol = reinterpret_cast<const char *>(QK + (int64_t)(nq + kvh) * HD);
  const char *const vrow = reinterpret_cast<const char *>(Vt + (int64_t)kvh * HD * vt_stride + it.vt_col0);
  auto stage_tile = [&](int kt, auto buf_tag) {
    constexpr int BUF = decltype(buf_tag)::value;
    OT *const lK = BUF ? lK1 : lK0;
    f16 *const lV = BUF ? lV1 : lV0;
    const int k0 = kt * BKV;
    if (k0 + BKV <= L && (k0 >= it.pre_len || k0 + BKV <= it.pre_len)) {
      // all 64 keys exist and sit in one row range (the shared prefix or the sequence's own rows)
      const char *kb = kcol + (int64_t)((k0 < it.pre_len ? it.pre_row0 : it.row_base) + k0) * row_elems * 2;
#pragma unroll
      for (int j = 0; j < NI; ++j)
        __builtin_amdgcn_global_load_lds(PRISM_GLOBAL_PTR(kb + oK[j]), PRISM_LDS_PTR(&lK[(wave_u * NI + j) * 4 * HD]), 16, 0, 0);
    } else {
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        const int kr = (wave * NI + j) * 4 + (lane >> 4);
        int key = k0 + kr;
        key = key < L ? key : L - 1;
        const char *src = kcol + ((int64_t)((key < it.pre_len ? it.pre_row0 : it.row_base) + key) * row_elems + (((lane & 15) ^ (kr & 15)) * 8)) * 2;
        __builtin_amdgcn_global_load_lds(PRISM_GLOBAL_PTR(src), PRISM_LDS_PTR(&lK[(wave_u * NI + j) * 4 * HD]), 16, 0, 0);
      }
    }
    const char *vb = vrow + (int64_t)k0 * 2;
#pragma unroll
    for (int j = 0; j < NI; ++j)
      __builtin_amdgcn_global_load_lds(PRISM_GLOBAL_PTR(vb + oV[j]), PRISM_LDS_PTR(&lV[(wave_u * NI + j) * 8 * BKV]), 16, 0, 0);
  };

  f32x16 o[HD / 32];
#pragma unroll
  for (int t = 0; t < HD / 32; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[t][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c_exp = 1.4426950408889634f / sqrtf((float)HD);      // log2(e) / sqrt(hd)

  stage_tile(0, std::integral_constant<int, 0>{});
  __syncthreads();                                   // also waits for this wave's own loads (vmcnt)

  const int q_hi_wave = q_lo + 31;
  // a lane reads row lane % 32 of a 32-row block and chunk 2 k + lane / 32 of it: slot (2 k + lane / 32) ^ swizzle(row),
  // which is the k = 0 address with k's bits flipped
  const int rdK = (lane & 31) * HD + (((lane >> 5) ^ (lane & 15)) * 8);
  const int rdV = (lane & 31) * BKV + (((lane >> 5) ^ ((lane >> 1) & 7)) * 8);
  // one tile: stage CUR holds tile kt, the other stage receives tile kt + 1 meanwhile
  auto step = [&](int kt, auto cur_tag) {
    constexpr int CUR = decltype(cur_tag)::value;
    const OT *const lK = CUR ? lK1 : lK0;
    const f16 *const lV = CUR ? lV1 : lV0;
    if (kt + 1 < n_kt) stage_tile(kt + 1, std::integral_constant<int, CUR ^ 1>{});

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
#pragma unroll
        for (int kk = 0; kk < HD / 16; ++kk) {
          const vec8 kf = *reinterpret_cast<const vec8 *>(&lK[(rdK ^ (kk * 16)) + kb * 32 * HD]);
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
      {
        float lo, hi;
        half_wave_pair(mx, lo, hi);
        mx = fmaxf(lo, hi);
      }
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
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          // contraction slots 0-3 <- keys ks*16 + (lane/32)*4 .. +4 ; slots 4-7 <- the same + 8: chunk 2 ks + lane/32
          const f16x8 vf = *reinterpret_cast<const f16x8 *>(&lV[(rdV ^ (ks * 16)) + t * 32 * BKV]);
          o[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf[ks], o[t], 0, 0, 0);
        }
      }
        };
    if (kt * BKV <= q_hi_wave && q_lo < L) {       // wave-uniform: tile not entirely in this wave's future
      if (kt * BKV + BKV - 1 > q_lo) tile_step(std::true_type{});
      else tile_step(std::false_type{});
    }
    __syncthreads();                                 // next tile landed (vmcnt) and everyone is done with this one
  };
  for (int kt = 0; kt < n_kt; kt += 2) {
    step(kt, std::integral_constant<int, 0>{});
    if (kt + 1 < n_kt) step(kt + 1, std::integral_constant<int, 1>{});
  }

  // ---- normalise and store: lane holds d = t*32 + (e/4)*8 + (lane/32)*4 + e%4 of query qi
  float l_lo, l_hi;
  half_wave_pair(l_run, l_lo, l_hi);
  const float l_tot = l_lo + l_hi;
  if (qi < L) {
    const float inv = 1.0f / l_tot;
    OT *op = out + (int64_t)(it.out_base + qi) * nq * HD + (int64_t)hq * HD + (lane >> 5) * 4;
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

// Waves per workgroup: 4 wherever the head grouping allows it, so that two workgroups share a compute unit (64 KiB of
// LDS and two waves per SIMD each) and one's matrix work overlaps the other's softmax and its start-up and drain.
static int waves_per_group(int g) { return g <= 4 ? 4 : 8; }

int attention_16_block_queries(int nq, int nkv) {
  const int g = nq / nkv;
  return 32 * (waves_per_group(g) / g);
}

template <typename OT, int G, int NW>
static hipError_t launch_one(int n_groups, const OT *QK, const f16 *Vt, int64_t vt_stride, const AttnTile *tiles, int nq, int nkv,
                             OT *out, hipStream_t s) {
  attention_16_kernel<OT, G, NW><<<n_groups, NW * 64, 0, s>>>(QK, Vt, vt_stride, tiles, nq, nkv, out);
  return hipGetLastError();
}

template <typename OT>
static hipError_t launch_typed(int n_groups, int g, const OT *QK, const f16 *Vt, int64_t vt_stride, const AttnTile *tiles, int nq,
                               int nkv, OT *out, hipStream_t s) {
  switch (g) {
    case 1: return launch_one<OT, 1, 4>(n_groups, QK, Vt, vt_stride, tiles, nq, nkv, out, s);
    case 2: return launch_one<OT, 2, 4>(n_groups, QK, Vt, vt_stride, tiles, nq, nkv, out, s);
    case 4: return launch_one<OT, 4, 4>(n_groups, QK, Vt, vt_stride, tiles, nq, nkv, out, s);
    default: return launch_one<OT, 8, 8>(n_groups, QK, Vt, vt_stride, tiles, nq, nkv, out, s);
  }
}

int launch_attention_16(int dtype, const void *QK, const void *Vt, int64_t vt_stride, const AttnTile *tiles, int n_tiles,
                        int T, int nq, int nkv, int hd, void *out, hipStream_t s) {
  PRISM_REQUIRE(QK && Vt && tiles && out && n_tiles >= 0 && T >= 0 && is16(dtype), PRISM_EINVAL, "attention: bad arguments");
  PRISM_REQUIRE(attention_16_supported(nq, nkv, hd), PRISM_EUNSUPPORTED,
                "attention: 16-bit modes need head_dim 128 and 1, 2, 4 or 8 query heads per KV head (got hd %d, %d/%d)", hd, nq, nkv);
  PRISM_REQUIRE(vt_stride % 8 == 0, PRISM_EINVAL, "attention: V^T row stride must be a multiple of 8");
  // the kernel addresses the 128 V^T rows of a KV head with 32-bit byte offsets
  PRISM_REQUIRE(vt_stride > 0 && (int64_t)HD * vt_stride * 2 < ((int64_t)1 << 32), PRISM_EUNSUPPORTED,
                "attention: V^T row stride %lld too large (128 rows must stay below 4 GiB)", (long long)vt_stride);
  PRISM_REQUIRE((int64_t)n_tiles * nkv < (int64_t)1 << 31, PRISM_EINVAL, "attention: too many work items (%d x %d)", n_tiles, nkv);
  if (n_tiles == 0) return PRISM_OK;
  const int n_groups = n_tiles * nkv;
  if (dtype == PRISM_DTYPE_BF16)
    PRISM_HIP(launch_typed<bf16>(n_groups, nq / nkv, (const bf16 *)QK, (const f16 *)Vt, vt_stride, tiles, nq, nkv, (bf16 *)out, s));
  else
    PRISM_HIP(launch_typed<f16>(n_groups, nq / nkv, (const f16 *)QK, (const f16 *)Vt, vt_stride, tiles, nq, nkv, (f16 *)out, s));
  return PRISM_OK;
}

}  // namespace prism
