// 16-bit-operand layer contractions on the gfx950 matrix cores (paper Sec. 2.2: the reranker's latency is
// dominated by the matrix multiplications of its transformer blocks).
//
// C = A W^T, A [M,K] and W [N,K] row-major, both bf16 or both IEEE half (K-contiguous, which is what
// the MFMA operand registers want: 8 consecutive k per lane), fp32 accumulation in
// v_mfma_f32_32x32x16_{bf16,f16} (same dense rate).
//
// Workgroup tile BM x BN x 64, WM x WN wavefronts, each owning a (BM/WM) x (BN/WN) block of 32x32
// accumulator tiles.  The production shape is 256 x 256 with 2 x 2 wavefronts (one per SIMD, 128 x 128 each,
// 256 accumulator registers in AGPRs) and a hand-scheduled K loop (gen_gemm_kloop.py); edge tiles and the
// small 128 x 128 configuration take the compiler-scheduled loop described next.  A and W tiles are staged in LDS (double-buffered; 16-byte chunks XOR-swizzled
// by row so that the 32-row operand reads spread over the banks) by direct global->LDS loads, which
// need no staging registers; the next K-slice lands while the current one feeds the MFMAs, one
// barrier per slice.  Inside a slice the operand fragments of step kk+1 are read while step kk's
// matrix instructions issue.
//
// Epilogues: plain store (bf16 or fp32), residual add into the fp32 stream, and SwiGLU, where the B tile is
// made of BN/2 gate rows and the BN/2 matching up rows so that a lane holds g and u of one element.
//
// Workgroup ids are remapped so that each XCD (ids are dealt round-robin over the 8 XCDs) owns a
// contiguous range of tiles, walked in groups of 8 (4 for the residual epilogue) row-tiles, to keep the operand panels in its L2.
#include <algorithm>
#include <mutex>

#include "common.h"
#include "gemm_16_kloop.inc"

namespace prism {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;
static constexpr int BK = 64;            // K-slice per stage (elements)
static constexpr int kChunks = BK / 8;   // 16-byte chunks per tile row

// LDS serves a 16-byte read of 16 consecutive lanes per cycle out of 64 banks; with 128-byte rows the bank
// half is the row's parity, so the chunk is rotated by bits 1..3 of the row.
__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

#define PRISM_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define PRISM_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

template <typename OT, int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(WM *WN * 64) void gemm_16_kernel(const OT *__restrict__ A,
                                                               const OT *__restrict__ W, void *__restrict__ out_,
                                                               int M, int N, int K, int nM, int nN, QkvEpilogue qe) {
  constexpr int NW = WM * WN;
  constexpr int WMT = BM / WM, WNT = BN / WN;      // wave tile
  constexpr int TM = WMT / 32, TN = WNT / 32;      // 32x32 accumulator tiles per wave
  // one direct-to-LDS instruction of a wave moves 64 x 16 B = 8 tile rows
  constexpr int A_ITERS = BM / 8 / NW, B_ITERS = BN / 8 / NW;
  static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile/waves mismatch");
  static_assert(EPI != PRISM_EPI_SWIGLU || TN % 2 == 0, "SwiGLU pairs gate and up tiles");
  typedef typename Mfma<OT>::vec8 vec8;
  extern __shared__ __align__(16) unsigned char smem[];
  OT *lA = reinterpret_cast<OT *>(smem);                     // [2][BM][BK]
  OT *lB = lA + 2 * BM * BK;                                 // [2][BN][BK]

  // ---- tile mapping: XCD-contiguous ranges, grouped walk ----
  const int n_tiles = nM * nN;
  int bid = blockIdx.x;
  {
    const int per = (n_tiles + 7) / 8, x = bid % 8, r = bid / 8;
    // XCD x owns logical ids [x*per, ...); ids beyond n_tiles idle
    bid = x * per + r;
    if (r >= per || bid >= n_tiles) return;
  }
  // measured: 8 row-tiles per group is best where the row panel is small (K = hidden); the down projection's row
  // panels are three times as long and the O projection's few column tiles leave little to share: 4 is 2 % faster there
  constexpr int GM = EPI == PRISM_EPI_RESIDUAL ? 4 : 8;
  const int group = bid / (GM * nN), first_m = group * GM;
  const int gsz = (nM - first_m) < GM ? (nM - first_m) : GM;
  const int tile_m = first_m + (bid % (GM * nN)) % gsz, tile_n = (bid % (GM * nN)) / gsz;
  const int m0 = tile_m * BM;
  const int F = EPI == PRISM_EPI_SWIGLU ? N / 2 : N;         // output columns
  constexpr int BNO = EPI == PRISM_EPI_SWIGLU ? BN / 2 : BN; // output columns per tile
  const int n0 = tile_n * (EPI == PRISM_EPI_SWIGLU ? BN / 2 : BN);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // ---- global -> LDS staging without registers (global_load_lds_dwordx4).  Instruction j of wave w
  //      fills tile rows (w * ITERS + j) * 8 .. + 8, lane l landing at row l / 8, chunk slot l % 8.
  //      The XOR swizzle is applied on the source side: slot p of row r receives chunk swz(r, p).
  const int lrow = lane >> 3;
  // byte offsets from A / W (both operands are below 4 GiB: checked by the launcher)
  uint32_t gA[A_ITERS], gB[B_ITERS];
#pragma unroll
  for (int j = 0; j < A_ITERS; ++j) {
    const int row = (wave * A_ITERS + j) * 8 + lrow;
    int gr = m0 + row;
    gr = gr < M ? gr : M - 1;
    gA[j] = ((uint32_t)gr * (uint32_t)K + swz(row, lane & 7) * 8) * 2u;
  }
#pragma unroll
  for (int j = 0; j < B_ITERS; ++j) {
    const int row = (wave * B_ITERS + j) * 8 + lrow;
    int gr;
    if (EPI == PRISM_EPI_SWIGLU) {
      const int half = row / (BN / 2), rr = row % (BN / 2);
      gr = n0 + rr; gr = gr < F ? gr : F - 1;
      gr += half * F;
    } else {
      gr = n0 + row; gr = gr < N ? gr : N - 1;
    }
    gB[j] = ((uint32_t)gr * (uint32_t)K + swz(row, lane & 7) * 8) * 2u;
  }
  auto stage_loads = [&](int kt, int buf) {
    const char *baseA = reinterpret_cast<const char *>(A) + (size_t)kt * BK * 2;   // uniform
    const char *baseB = reinterpret_cast<const char *>(W) + (size_t)kt * BK * 2;
#pragma unroll
    for (int j = 0; j < A_ITERS; ++j)
      __builtin_amdgcn_global_load_lds(PRISM_GLOBAL_PTR(baseA + gA[j]),
                                       PRISM_LDS_PTR(lA + buf * BM * BK + (wave * A_ITERS + j) * 8 * BK), 16, 0, 0);
#pragma unroll
    for (int j = 0; j < B_ITERS; ++j)
      __builtin_amdgcn_global_load_lds(PRISM_GLOBAL_PTR(baseB + gB[j]),
                                       PRISM_LDS_PTR(lB + buf * BN * BK + (wave * B_ITERS + j) * 8 * BK), 16, 0, 0);
  };

  // ---- LDS rows this lane reads as MFMA operands ----
  int rA[TM], rB[TN];
#pragma unroll
  for (int t = 0; t < TM; ++t) rA[t] = wm * WMT + t * 32 + (lane & 31);
#pragma unroll
  for (int t = 0; t < TN; ++t) {
    if (EPI == PRISM_EPI_SWIGLU)
      rB[t] = (t / (TN / 2)) * (BN / 2) + wn * (WNT / 2) + (t % (TN / 2)) * 32 + (lane & 31);
    else
      rB[t] = wn * WNT + t * 32 + (lane & 31);
  }
  const int khalf = lane >> 5;                               // which 8 of the 16 k of an MFMA this lane feeds

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nk = K / BK;

  // ---- epilogue geometry (see the epilogue): everything it reads or writes goes along the rows, 16 bytes per lane.
  //      Residual epilogue: the old values of a 32-row block are requested one block ahead.  (Requesting the first
  //      block before the K loop was tried: holding 64 registers across the loop makes the compiler spill.)
  constexpr bool kF32Out = EPI == PRISM_EPI_RESIDUAL || EPI == PRISM_EPI_STORE_F32;
  constexpr int ES = kF32Out ? 4 : 2;                               // bytes per output element
  constexpr int OUTW = EPI == PRISM_EPI_SWIGLU ? WNT / 2 : WNT;    // output columns of the wave
  constexpr int RB = OUTW * ES, CPR = RB / 16;                      // bytes / 16-byte chunks per staged row
  constexpr int NR = 1024 / RB, NI = 32 / NR;                       // rows per instruction, instructions per 32-row block
  const int f_row = lane / CPR, f_chunk = lane % CPR;               // lane -> (row within an instruction, chunk)
  const bool full_n = n0 + BNO <= F && (F * ES) % 16 == 0;
  f32x4 old[2][EPI == PRISM_EPI_RESIDUAL ? NI : 1];
  float *xo = reinterpret_cast<float *>(out_) + n0 + wn * OUTW + f_chunk * 4;
  auto load_old = [&](int i) __attribute__((always_inline)) {
    if constexpr (EPI == PRISM_EPI_RESIDUAL) {
#pragma unroll
      for (int rr = 0; rr < NI; ++rr) {
        const int row = m0 + wm * WMT + i * 32 + rr * NR + f_row;
        old[i & 1][rr] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(xo + (int64_t)(row < M ? row : M - 1) * N));
      }
    }
  };


  // ---- epilogue.  The W fragment was the instruction's first operand, so the 32x32 accumulator tile is
  //      transposed: a lane holds ONE row of A, m = lane % 32, and the output columns
  //      n = (e / 4) * 8 + (lane / 32) * 4 + e % 4, e = 0..15: four runs of 4 consecutive columns.
  //      Written straight from that layout, one store instruction touches 32 rows with 16-32 bytes in each, and
  //      the number of cache lines an instruction touches - not the bytes - is what the memory path charges for
  //      (measured: 12-29 us per 256 x 256 tile, a tenth to a fifth of the tile's time).  So every block of 32 rows goes
  //      through LDS, which is free once the K loop is done: lanes write their row's values, then read back 16 bytes
  //      each along the rows, so that an instruction reads or writes whole lines (2-8 complete rows of the wave's
  //      columns).  LDS requests of one wave are served in order, so no barrier is needed between the two phases.
  //      The epilogue is a lambda expanded after EACH of the two K loops below rather than once behind their join: the
  //      accumulators then stay wherever the loop left them (with one copy behind the join the register allocator parks
  //      dozens of them in scratch memory to reconcile the two loops' assignments).
  auto epilogue = [&]() __attribute__((always_inline)) {
  // Accumulator element (i, j, e), fetched from its accumulation register when it is needed: behind the hand-scheduled
  // loop all 256 of them sit in AGPRs, and read as plain values the compiler would copy the whole set into vector
  // registers at once, leaving none for the epilogue's own arithmetic.
  // (The compiler does not look inside these statements, so the wait between a matrix instruction and the first read
  // of its result is spelled out: every accumulator tile passes through an empty statement, which puts all matrix
  // instructions before it, then 32 idle cycles - more than the deepest instruction needs to retire.  All of these are
  // volatile, which keeps them in this order.)
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) asm volatile("" : "+a"(acc[i][j]));
  asm volatile("s_nop 15\n\ts_nop 15");
  auto AC = [&](int i, int j, int e) __attribute__((always_inline)) {
    float r;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(r) : "a"(acc[i][j][e]));
    return r;
  };
  __syncthreads();              // every wave's operand loads have landed and nobody reads operands any more
  const int m_in = lane & 31, n_in = (lane >> 5) * 4;
  constexpr int SWZ = CPR >= 16 ? 15 : CPR - 1;                     // chunk rotation by row: spreads a column of 16-byte
                                                                    // writes (one per row) over the banks
  static_assert(32 * RB <= 2 * (BM + BN) * BK * (int)sizeof(OT) / NW, "staging block must fit the wave's share of LDS");
  unsigned char *stg = smem + wave * (2 * (BM + BN) * BK * (int)sizeof(OT) / NW);
  // values for columns n .. n + 3 (n a multiple of 4, within the wave's columns) of staged row m
  auto put32 = [&](int m, int n, const f32x4 &v) __attribute__((always_inline)) {
    *reinterpret_cast<f32x4 *>(stg + m * RB + (((n >> 2) ^ (m & SWZ)) << 4)) = v;
  };
  auto put16 = [&](int m, int n, const typename Mfma<OT>::vec4 &v) __attribute__((always_inline)) {
    *reinterpret_cast<typename Mfma<OT>::vec4 *>(stg + m * RB + (((n >> 3) ^ (m & SWZ)) << 4) + (n & 4) * 2) = v;
  };
  auto staged = [&](int rr) __attribute__((always_inline)) {
    const int r = rr * NR + f_row;
    return *reinterpret_cast<const uint4 *>(stg + r * RB + ((f_chunk ^ (r & SWZ)) << 4));
  };
  // Flushes the staged block to rows row0 + r of a row-major destination (row pitch `pitch` bytes, the wave's first
  // column at byte col_byte0 of a row).
  auto flush_store = [&](unsigned char *dst, int64_t pitch, int64_t col_byte0, int row0) __attribute__((always_inline)) {
#pragma unroll
    for (int rr = 0; rr < NI; ++rr) {
      const int row = row0 + rr * NR + f_row;
      const uint4 v = staged(rr);
      if (row < M) __builtin_nontemporal_store(__builtin_bit_cast(u32x4_t, v), reinterpret_cast<u32x4_t *>(dst + (int64_t)row * pitch + col_byte0 + f_chunk * 16));
    }
  };

  if constexpr (EPI == kEpiQkv) {
    // The wave's 128 columns are one head.  A row's 128 values sit in lanes l and l ^ 32 (64 each); the rotate-half
    // partner of column d is d + 64 = the same register of accumulator tile j + 2, so the per-head RMSNorm (one
    // cross-lane add), the rotation and the single rounding all happen on the accumulators.  What the memory path
    // charges for is cache lines touched per instruction, so the cos/sin pairs come from the TRANSPOSED table (the 32
    // tokens of a row block are consecutive positions of a sequence almost always: two to four lines per load instead of
    // one or two per lane) and the finished q / k rows go through the staging block like the other epilogues' outputs.
    static_assert(WNT == 128 && TN == 4, "one head per wavefront");
    typedef typename Mfma<OT>::vec4 vec4;
    const int head = (n0 + wn * WNT) >> 7;                 // wave-uniform
    if (head < qe.nq + qe.nkv) {
      const OT *gain = reinterpret_cast<const OT *>(head < qe.nq ? qe.q_gain : qe.k_gain);
      vec4 ga[2][4], gb[2][4];
      if (qe.qk_norm) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            ga[j][g] = *reinterpret_cast<const vec4 *>(gain + j * 32 + g * 8 + n_in);
            gb[j][g] = *reinterpret_cast<const vec4 *>(gain + j * 32 + g * 8 + n_in + 64);
          }
      }
      const int64_t pitch = (int64_t)(qe.nq + qe.nkv) * 128 * 2;
      // (cos, sin) of (pos, d) sits at [d * stride + pos]: a wave-uniform base per column plus one 32-bit lane offset.
      // The positions of all four row blocks are fetched first and the 32 pairs of block i + 1 are requested before
      // block i is worked on, so the tile pays the two memory latencies once, not once per block.
      unsigned lane_off[TM];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = m0 + wm * WMT + i * 32 + m_in;
        lane_off[i] = (unsigned)n_in * (unsigned)qe.rope_stride + (unsigned)qe.pos[row < M ? row : M - 1];
      }
      float2 cs[2][2][4][4];
      auto load_cs = [&](int i) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int q = 0; q < 4; ++q)
              cs[i & 1][j][g][q] = (qe.rope_tab_t + (int64_t)(j * 32 + g * 8 + q) * qe.rope_stride)[lane_off[i]];
      };
      load_cs(0);
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row0 = m0 + wm * WMT + i * 32;
        if (i + 1 < TM) load_cs(i + 1);
        float r = 1.f;
        if (qe.qk_norm) {
          float ss = 0.f;
#pragma unroll
          for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              const float v = AC(i, j, e);
              ss += v * v;
            }
          ss += __shfl_xor(ss, 32);
          r = 1.0f / sqrtf(ss / 128.f + qe.eps);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int d = j * 32 + g * 8 + n_in;
            vec4 lo, hi;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const float2 c = cs[i & 1][j][g][q];
              float a = AC(i, j, g * 4 + q), b = AC(i, j + 2, g * 4 + q);
              if (qe.qk_norm) {
                a = a * r * to_f32(ga[j][g][q]);
                b = b * r * to_f32(gb[j][g][q]);
              }
              lo[q] = from_f32<OT>(a * c.x - b * c.y);
              hi[q] = from_f32<OT>(b * c.x + a * c.y);
            }
            put16(m_in, d, lo);
            put16(m_in, d + 64, hi);
          }
        }
        flush_store(reinterpret_cast<unsigned char *>(qe.QK), pitch, (int64_t)head * 128 * 2, row0);
      }
    } else {
      // v head: rounded to the operand type, stored as half, transposed (32 consecutive tokens of one d are contiguous)
      int vcol[TM];                                          // all four blocks' columns first: one memory latency, not four
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = m0 + wm * WMT + i * 32 + m_in;
        vcol[i] = qe.vt_col[row < M ? row : M - 1];
      }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = m0 + wm * WMT + i * 32 + m_in;
        if (row >= M) continue;
        f16 *vt = reinterpret_cast<f16 *>(qe.Vt) + (int64_t)(head - qe.nq - qe.nkv) * 128 * qe.vt_stride + vcol[i];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int d = j * 32 + (e >> 2) * 8 + n_in + (e & 3);
            vt[(int64_t)d * qe.vt_stride] = from_f32<f16>(to_f32(from_f32<OT>(AC(i, j, e))));
          }
      }
    }
    return;
  }

  if (full_n) {
    load_old(0);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int row0 = m0 + wm * WMT + i * 32;                       // first row of the block
      if (EPI == PRISM_EPI_SWIGLU) {
#pragma unroll
        for (int j = 0; j < TN / 2; ++j)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            typename Mfma<OT>::vec4 v;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const float gt = AC(i, j, g * 4 + q), up = AC(i, j + TN / 2, g * 4 + q);
              v[q] = from_f32<OT>(gt / (1.0f + __expf(-gt)) * up);
            }
            put16(m_in, j * 32 + g * 8 + n_in, v);
          }
        flush_store(reinterpret_cast<unsigned char *>(out_), (int64_t)F * 2, (int64_t)(n0 + wn * OUTW) * 2, row0);
      } else if (EPI == PRISM_EPI_RESIDUAL) {
        // read-modify-write of the fp32 stream, whole lines per instruction; the loads of the next block are requested
        // before this block is staged, so the tile pays the memory latency once, not per block
        if (i + 1 < TM) load_old(i + 1);
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            f32x4 v;
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = AC(i, j, g * 4 + q);
            put32(m_in, j * 32 + g * 8 + n_in, v);
          }
#pragma unroll
        for (int rr = 0; rr < NI; ++rr) {
          const int row = row0 + rr * NR + f_row;
          const uint4 u = staged(rr);
          f32x4 v = old[i & 1][rr];
          v[0] += __uint_as_float(u.x); v[1] += __uint_as_float(u.y); v[2] += __uint_as_float(u.z); v[3] += __uint_as_float(u.w);
          if (row < M) __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(xo + (int64_t)row * N));
        }
      } else {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            if (EPI == PRISM_EPI_STORE_F32) {
              f32x4 v;
#pragma unroll
              for (int q = 0; q < 4; ++q) v[q] = AC(i, j, g * 4 + q);
              put32(m_in, j * 32 + g * 8 + n_in, v);
            } else {
              typename Mfma<OT>::vec4 v;
#pragma unroll
              for (int q = 0; q < 4; ++q) v[q] = from_f32<OT>(AC(i, j, g * 4 + q));
              put16(m_in, j * 32 + g * 8 + n_in, v);
            }
          }
        flush_store(reinterpret_cast<unsigned char *>(out_), (int64_t)N * ES, (int64_t)(n0 + wn * OUTW) * ES, row0);
      }
    }
    return;
  }

  // ---- ragged last column tile (N not a multiple of the tile, or rows not 16-byte aligned): element by element
  if constexpr (EPI != kEpiQkv) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int row = m0 + wm * WMT + i * 32 + m_in;
      if (row >= M) continue;
#pragma unroll
      for (int j = 0; j < (EPI == PRISM_EPI_SWIGLU ? TN / 2 : TN); ++j)
        for (int g = 0; g < 4; ++g)
          for (int q = 0; q < 4; ++q) {
            const int col = n0 + wn * OUTW + j * 32 + g * 8 + n_in + q;
            if (col >= F) continue;
            if (EPI == PRISM_EPI_SWIGLU) {
              const float gt = AC(i, j, g * 4 + q), up = AC(i, j + TN / 2, g * 4 + q);
              reinterpret_cast<OT *>(out_)[(int64_t)row * F + col] = from_f32<OT>(gt / (1.0f + __expf(-gt)) * up);
            } else if (EPI == PRISM_EPI_RESIDUAL) {
              reinterpret_cast<float *>(out_)[(int64_t)row * N + col] += AC(i, j, g * 4 + q);
            } else if (EPI == PRISM_EPI_STORE_F32) {
              reinterpret_cast<float *>(out_)[(int64_t)row * N + col] = AC(i, j, g * 4 + q);
            } else {
              reinterpret_cast<OT *>(out_)[(int64_t)row * N + col] = from_f32<OT>(AC(i, j, g * 4 + q));
            }
          }
    }
  }
  };

  // The 256x256 / 2x2-wave configuration runs the hand-scheduled loop; other shapes take the compiler's schedule.
  constexpr bool kHandScheduled = BM == 256 && BN == 256 && WM == 2 && WN == 2;
  // interior tiles only: the hand-scheduled loop assumes that the tile's rows of A and W all exist
  const bool interior = m0 + BM <= M && n0 + (EPI == PRISM_EPI_SWIGLU ? BN / 2 : BN) <= F;
  if (kHandScheduled && interior) {
    if constexpr (kHandScheduled) {
      const unsigned ldsA = (unsigned)(uintptr_t)PRISM_LDS_PTR(lA), ldsB = (unsigned)(uintptr_t)PRISM_LDS_PTR(lB);
      const unsigned aA0 = ldsA + (unsigned)(rA[0] * BK + swz(rA[0], khalf) * 8) * 2u;
      const unsigned aB0 = ldsB + (unsigned)(rB[0] * BK + swz(rB[0], khalf) * 8) * 2u;
      // wave w's load instruction j fills tile rows (8 w + j) * 8 .. + 8 of each operand (1 KiB of LDS)
      const unsigned stride8 = 8u * (unsigned)K * 2u;
      const unsigned ldsA_w = __builtin_amdgcn_readfirstlane(ldsA + (unsigned)wave * A_ITERS * 8 * BK * 2);
      const unsigned ldsB_w = __builtin_amdgcn_readfirstlane(ldsB + (unsigned)wave * B_ITERS * 8 * BK * 2);
      const uint64_t baseA = (uint64_t)(uintptr_t)A, baseB = (uint64_t)(uintptr_t)W;
#define PRISM_RUN_KLOOP(TEXT)                                                                                           \
  asm volatile(TEXT                                                                                                     \
               : "+a"(acc[0][0]), "+a"(acc[0][1]), "+a"(acc[0][2]), "+a"(acc[0][3]), "+a"(acc[1][0]), "+a"(acc[1][1]), \
                 "+a"(acc[1][2]), "+a"(acc[1][3]), "+a"(acc[2][0]), "+a"(acc[2][1]), "+a"(acc[2][2]), "+a"(acc[2][3]), \
                 "+a"(acc[3][0]), "+a"(acc[3][1]), "+a"(acc[3][2]), "+a"(acc[3][3])                                    \
               : "v"(aA0), "v"(aB0), "v"(gA[0]), "v"(gB[0]), "s"(ldsA_w), "s"(ldsB_w), "s"(stride8), "s"(baseA),       \
                 "s"(baseB), "s"(nk)                                                                                   \
               : PRISM_KLOOP4_CLOBBERS)
      constexpr bool kF16 = Mfma<OT>::kIsF16;
      if constexpr (EPI == PRISM_EPI_SWIGLU) {
        if constexpr (kF16) PRISM_RUN_KLOOP(PRISM_KLOOP4_F16_SWIGLU);
        else PRISM_RUN_KLOOP(PRISM_KLOOP4_BF16_SWIGLU);
      } else {
        if constexpr (kF16) PRISM_RUN_KLOOP(PRISM_KLOOP4_F16_PLAIN);
        else PRISM_RUN_KLOOP(PRISM_KLOOP4_BF16_PLAIN);
      }
#undef PRISM_RUN_KLOOP
      epilogue();
    }
  } else {
    vec8 af[2][TM], bfr[2][TN];
    auto load_frags = [&](int set, const OT *cA, const OT *cB, int kk) {
#pragma unroll
      for (int t = 0; t < TM; ++t)
        af[set][t] = *reinterpret_cast<const vec8 *>(cA + rA[t] * BK + swz(rA[t], kk * 2 + khalf) * 8);
#pragma unroll
      for (int t = 0; t < TN; ++t)
        bfr[set][t] = *reinterpret_cast<const vec8 *>(cB + rB[t] * BK + swz(rB[t], kk * 2 + khalf) * 8);
    };
    stage_loads(0, 0);
    __syncthreads();                                           // waits for the loads (vmcnt) and the workgroup
    for (int kt = 0; kt < nk; ++kt) {
      const int cur = kt & 1;
      if (kt + 1 < nk) stage_loads(kt + 1, cur ^ 1);           // lands while this slice feeds the MFMAs
      const OT *cA = lA + cur * BM * BK, *cB = lB + cur * BN * BK;
      load_frags(0, cA, cB, 0);
#pragma unroll
      for (int kk = 0; kk < BK / 16; ++kk) {
        if (kk + 1 < BK / 16) load_frags((kk + 1) & 1, cA, cB, kk + 1);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = Mfma<OT>::mma(bfr[kk & 1][j], af[kk & 1][i], acc[i][j]);   // transposed tile, see the epilogue
      }
      __syncthreads();                                         // next slice landed (vmcnt) and everyone is done with this one
    }
    epilogue();
  }
}

bool gemm_16_supported(int epilogue, int N, int K) {
  if (K <= 0 || K % BK != 0 || N <= 0) return false;
  if (epilogue == PRISM_EPI_SWIGLU && N % 2 != 0) return false;
  return epilogue >= PRISM_EPI_STORE && epilogue <= PRISM_EPI_STORE_F32;
}

template <typename OT, int BM, int BN, int WM, int WN, int EPI>
static int launch_cfg(const OT *A, const OT *W, void *out, int M, int N, int K, hipStream_t s,
                      const QkvEpilogue &qe = QkvEpilogue{}) {
  constexpr size_t lds = 2 * (size_t)(BM + BN) * BK * sizeof(OT);
  auto kern = gemm_16_kernel<OT, BM, BN, WM, WN, EPI>;
  // the attribute is per function: set once per process, also when several contexts launch from different threads
  static std::once_flag attr_once;
  static hipError_t attr_rc = hipSuccess;
  std::call_once(attr_once, [&] {
    attr_rc = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  });
  PRISM_HIP(attr_rc);
  const int ncols = EPI == PRISM_EPI_SWIGLU ? N / 2 : N, bn_out = EPI == PRISM_EPI_SWIGLU ? BN / 2 : BN;
  const int nM = cdiv(M, BM), nN = cdiv(ncols, bn_out);
  const int grid = cdiv((int64_t)nM * nN, 8) * 8;
  kern<<<grid, WM * WN * 64, lds, s>>>(A, W, out, M, N, K, nM, nN, qe);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

// Cost of a round of small tiles relative to a round of big ones: a quarter of the work at about two thirds of the rate
// (the 128 x 128 loop is compiler-scheduled).  Only used to decide how a launch is tiled, never for results.
#ifndef PRISM_SMALL_TILE_COST
#define PRISM_SMALL_TILE_COST 0.4
#endif

template <typename OT, int EPI>
static int launch_epi(const OT *A, const OT *W, void *out, int M, int N, int K, hipStream_t s) {
  // A launch runs its tiles in rounds of one per compute unit, and a last round that fills only a few of them costs a
  // whole tile's time.  Rows are independent and both tile sizes give a row the same bits, so the launcher compares three
  // ways of tiling by their rounds: small tiles only, big tiles only, or the row tiles that fill whole rounds with big
  // tiles and the remaining rows in a second launch with small ones.
  constexpr int kCus = 256;
  constexpr bool kGlu = EPI == PRISM_EPI_SWIGLU;
  const int ncols = kGlu ? N / 2 : N;
  const int nN = cdiv(ncols, kGlu ? 128 : 256), nM = cdiv(M, 256), nN_small = cdiv(ncols, kGlu ? 64 : 128);
  const int64_t big_tiles = (int64_t)nM * nN;
  const double cost_small = PRISM_SMALL_TILE_COST * (double)cdiv((int64_t)cdiv(M, 128) * nN_small, kCus);
  const double cost_big = (double)cdiv(big_tiles, kCus);
  const int full_rounds = (int)(big_tiles / kCus);
  const int rows_big = (int)std::min<int64_t>(nM, (int64_t)full_rounds * kCus / nN);      // row tiles that fit whole rounds
  const int rest_rows = M - rows_big * 256;
  double cost_split = 1e30;
  if (rows_big >= 1 && rest_rows > 0)
    cost_split = (double)cdiv((int64_t)rows_big * nN, kCus) + PRISM_SMALL_TILE_COST * (double)cdiv((int64_t)cdiv(rest_rows, 128) * nN_small, kCus);
  if (cost_small <= cost_big && cost_small <= cost_split) return launch_cfg<OT, 128, 128, 2, 2, EPI>(A, W, out, M, N, K, s);
  if (cost_split < cost_big - 0.05) {
    const size_t out_elem = EPI == PRISM_EPI_RESIDUAL || EPI == PRISM_EPI_STORE_F32 ? 4 : 2;
    PRISM_TRY((launch_cfg<OT, 256, 256, 2, 2, EPI>(A, W, out, rows_big * 256, N, K, s)));
    return launch_cfg<OT, 128, 128, 2, 2, EPI>(A + (size_t)rows_big * 256 * K, W,
                                                reinterpret_cast<char *>(out) + (size_t)rows_big * 256 * ncols * out_elem, rest_rows, N, K, s);
  }
  return launch_cfg<OT, 256, 256, 2, 2, EPI>(A, W, out, M, N, K, s);
}

template <typename OT>
static int launch_typed(int epilogue, const OT *A, const OT *W, void *out, int M, int N, int K, hipStream_t s) {
  switch (epilogue) {
    case PRISM_EPI_STORE: return launch_epi<OT, PRISM_EPI_STORE>(A, W, out, M, N, K, s);
    case PRISM_EPI_RESIDUAL: return launch_epi<OT, PRISM_EPI_RESIDUAL>(A, W, out, M, N, K, s);
    case PRISM_EPI_STORE_F32: return launch_epi<OT, PRISM_EPI_STORE_F32>(A, W, out, M, N, K, s);
    default: return launch_epi<OT, PRISM_EPI_SWIGLU>(A, W, out, M, N, K, s);
  }
}

// The kernel addresses its operands with 32-bit byte offsets.  W has to fit that; A (and the output rows with it) is
// cut into row panels that do: rows of a GEMM are independent, so the panels are separate launches.
static int rows_per_launch(int K) {
  const int64_t rows = (((int64_t)1 << 32) - 1) / ((int64_t)K * 2);
  return (int)std::max<int64_t>(256, rows / 256 * 256);
}

int launch_gemm_16(int dtype, int epilogue, const void *A, const void *W, void *out, int M, int N, int K, hipStream_t s) {
  PRISM_REQUIRE(A && W && out && M >= 0 && is16(dtype), PRISM_EINVAL, "gemm: bad arguments");
  PRISM_REQUIRE(gemm_16_supported(epilogue, N, K), PRISM_EUNSUPPORTED,
                "gemm: N = %d, K = %d, epilogue %d not supported (K must be a multiple of %d)", N, K, epilogue, BK);
  PRISM_REQUIRE((int64_t)N * K * 2 < ((int64_t)1 << 32) && (int64_t)256 * K * 2 < ((int64_t)1 << 32), PRISM_EUNSUPPORTED,
                "gemm: a weight operand of %d x %d 16-bit elements exceeds 4 GiB", N, K);
  const int step = rows_per_launch(K);
  const int out_cols = epilogue == PRISM_EPI_SWIGLU ? N / 2 : N;
  const size_t out_elem = epilogue == PRISM_EPI_RESIDUAL || epilogue == PRISM_EPI_STORE_F32 ? 4 : 2;
  for (int m0 = 0; m0 < M; m0 += step) {
    const int rows = std::min(step, M - m0);
    const char *a = reinterpret_cast<const char *>(A) + (size_t)m0 * K * 2;
    char *o = reinterpret_cast<char *>(out) + (size_t)m0 * out_cols * out_elem;
    if (dtype == PRISM_DTYPE_BF16) PRISM_TRY(launch_typed<bf16>(epilogue, (const bf16 *)a, (const bf16 *)W, o, rows, N, K, s));
    else PRISM_TRY(launch_typed<f16>(epilogue, (const f16 *)a, (const f16 *)W, o, rows, N, K, s));
  }
  return PRISM_OK;
}

bool gemm_16_qkv_supported(int M, int nq, int nkv, int hd, int K) {
  // one head per wavefront of the 256 x 256 tile; smaller problems take the unfused path
  return hd == 128 && nq > 0 && nkv > 0 && (nq + 2 * nkv) % 2 == 0 && K > 0 && K % BK == 0 &&
         (int64_t)cdiv(M, 256) * ((nq + 2 * nkv) / 2) >= 256;
}

int launch_gemm_16_qkv(int dtype, const void *Xn, const void *Wqkv, int M, int K, int hd, const QkvEpilogue &e, hipStream_t s) {
  PRISM_REQUIRE(Xn && Wqkv && M >= 0 && is16(dtype) && e.pos && e.vt_col && e.rope_tab_t && e.rope_stride > 0 && e.QK && e.Vt, PRISM_EINVAL,
                "qkv gemm: bad arguments");
  PRISM_REQUIRE(!e.qk_norm || (e.q_gain && e.k_gain), PRISM_EINVAL, "qkv gemm: gains missing");
  PRISM_REQUIRE(gemm_16_qkv_supported(M, e.nq, e.nkv, hd, K), PRISM_EUNSUPPORTED, "qkv gemm: shape not supported by the fused epilogue");
  const int N = (e.nq + 2 * e.nkv) * 128;
  PRISM_REQUIRE((int64_t)N * K * 2 < ((int64_t)1 << 32) && (int64_t)256 * K * 2 < ((int64_t)1 << 32), PRISM_EUNSUPPORTED,
                "qkv gemm: the weight operand exceeds 4 GiB");
  const int step = rows_per_launch(K);
  for (int m0 = 0; m0 < M; m0 += step) {
    const int rows = std::min(step, M - m0);
    QkvEpilogue p = e;                       // row panel: every per-row array moves with the rows
    p.pos = e.pos + m0;
    p.vt_col = e.vt_col + m0;
    p.QK = reinterpret_cast<char *>(e.QK) + (size_t)m0 * (e.nq + e.nkv) * 128 * 2;
    const char *a = reinterpret_cast<const char *>(Xn) + (size_t)m0 * K * 2;
    if (dtype == PRISM_DTYPE_BF16)
      PRISM_TRY((launch_cfg<bf16, 256, 256, 2, 2, kEpiQkv>((const bf16 *)a, (const bf16 *)Wqkv, p.QK, rows, N, K, s, p)));
    else
      PRISM_TRY((launch_cfg<f16, 256, 256, 2, 2, kEpiQkv>((const f16 *)a, (const f16 *)Wqkv, p.QK, rows, N, K, s, p)));
  }
  return PRISM_OK;
}

}  // namespace prism
