// 16-bit-operand layer contractions on the gfx950 matrix cores (paper Sec. 2.2: the reranker's latency is
// dominated by the matrix multiplications of its transformer blocks).
//
// C = A W^T, A [M,K] and W [N,K] row-major, both bf16 or both IEEE half (K-contiguous, which is what
// the MFMA operand registers want: 8 consecutive k per lane), fp32 accumulation in
// v_mfma_f32_32x32x16_{bf16,f16} (same dense rate).
//
// Workgroup tile BM x BN x 64, WM x WN wavefronts, each owning a (BM/WM) x (BN/WN) block of 32x32
// accumulator tiles.  A and W tiles are staged in LDS (double-buffered; 16-byte chunks XOR-swizzled
// by row so that the 32-row operand reads spread over the banks).  The next K-slice is fetched into
// registers while the current one feeds the MFMAs, one barrier per slice.
//
// Epilogues: plain store (bf16 or fp32), residual add into the fp32 stream, and SwiGLU, where the B tile is
// made of BN/2 gate rows and the BN/2 matching up rows so that a lane holds g and u of one element.
//
// Workgroup ids are remapped so that each XCD (ids are dealt round-robin over the 8 XCDs) owns a
// contiguous range of tiles, walked in groups of 8 row-tiles, to keep the operand panels in its L2.
#include "common.h"

namespace prism {

static constexpr int BK = 64;            // K-slice per stage (elements)
static constexpr int kChunks = BK / 8;   // 16-byte chunks per tile row

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ (row & 7); }

template <typename OT, int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(WM *WN * 64) void gemm_16_kernel(const OT *__restrict__ A,
                                                               const OT *__restrict__ W, void *__restrict__ out_,
                                                                 int M, int N, int K, int nM, int nN) {
  constexpr int NT = WM * WN * 64;
  constexpr int WMT = BM / WM, WNT = BN / WN;      // wave tile
  constexpr int TM = WMT / 32, TN = WNT / 32;      // 32x32 accumulator tiles per wave
  constexpr int A_ITERS = BM * kChunks / NT, B_ITERS = BN * kChunks / NT;
  static_assert(BM * kChunks % NT == 0 && BN * kChunks % NT == 0, "tile/threads mismatch");
  static_assert(EPI != PRISM_EPI_SWIGLU || TN % 2 == 0, "SwiGLU pairs gate and up tiles");
  extern __shared__ __align__(16) unsigned char smem[];
  typedef typename Mfma<OT>::vec8 vec8;
  OT *lA = reinterpret_cast<OT *>(smem);                 // [2][BM][BK]
  OT *lB = lA + 2 * BM * BK;                               // [2][BN][BK]

  // ---- tile mapping: XCD-contiguous ranges, grouped walk ----
  const int n_tiles = nM * nN;
  int bid = blockIdx.x;
  {
    const int per = (n_tiles + 7) / 8, x = bid % 8, r = bid / 8;
    // XCD x owns logical ids [x*per, ...); ids beyond n_tiles idle
    bid = x * per + r;
    if (r >= per || bid >= n_tiles) return;
  }
  constexpr int GM = 8;
  const int group = bid / (GM * nN), first_m = group * GM;
  const int gsz = (nM - first_m) < GM ? (nM - first_m) : GM;
  const int tile_m = first_m + (bid % (GM * nN)) % gsz, tile_n = (bid % (GM * nN)) / gsz;
  const int m0 = tile_m * BM;
  const int F = EPI == PRISM_EPI_SWIGLU ? N / 2 : N;         // output columns
  const int n0 = tile_n * (EPI == PRISM_EPI_SWIGLU ? BN / 2 : BN);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // ---- global source pointers of this thread's 16-byte chunks ----
  const OT *gA[A_ITERS], *gB[B_ITERS];
  int sA[A_ITERS], sB[B_ITERS];                              // LDS element offsets (within one stage)
#pragma unroll
  for (int i = 0; i < A_ITERS; ++i) {
    const int c = tid + i * NT, row = c / kChunks, ch = c % kChunks;
    int gr = m0 + row; gr = gr < M ? gr : M - 1;
    gA[i] = A + (int64_t)gr * K + ch * 8;
    sA[i] = row * BK + swz(row, ch) * 8;
  }
#pragma unroll
  for (int i = 0; i < B_ITERS; ++i) {
    const int c = tid + i * NT, row = c / kChunks, ch = c % kChunks;
    int gr;
    if (EPI == PRISM_EPI_SWIGLU) {
      const int half = row / (BN / 2), rr = row % (BN / 2);
      gr = n0 + rr; gr = gr < F ? gr : F - 1;
      gr += half * F;
    } else {
      gr = n0 + row; gr = gr < N ? gr : N - 1;
    }
    gB[i] = W + (int64_t)gr * K + ch * 8;
    sB[i] = row * BK + swz(row, ch) * 8;
  }

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

  vec8 ra[A_ITERS], rb[B_ITERS];
  const int nk = K / BK;
#pragma unroll
  for (int i = 0; i < A_ITERS; ++i) ra[i] = *reinterpret_cast<const vec8 *>(gA[i]);
#pragma unroll
  for (int i = 0; i < B_ITERS; ++i) rb[i] = *reinterpret_cast<const vec8 *>(gB[i]);
#pragma unroll
  for (int i = 0; i < A_ITERS; ++i) *reinterpret_cast<vec8 *>(lA + sA[i]) = ra[i];
#pragma unroll
  for (int i = 0; i < B_ITERS; ++i) *reinterpret_cast<vec8 *>(lB + sB[i]) = rb[i];
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < nk;
    if (more) {
#pragma unroll
      for (int i = 0; i < A_ITERS; ++i) ra[i] = *reinterpret_cast<const vec8 *>(gA[i] + (int64_t)(kt + 1) * BK);
#pragma unroll
      for (int i = 0; i < B_ITERS; ++i) rb[i] = *reinterpret_cast<const vec8 *>(gB[i] + (int64_t)(kt + 1) * BK);
    }
    const OT *cA = lA + cur * BM * BK, *cB = lB + cur * BN * BK;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      vec8 af[TM], bfr[TN];
#pragma unroll
      for (int t = 0; t < TM; ++t)
        af[t] = *reinterpret_cast<const vec8 *>(cA + rA[t] * BK + swz(rA[t], kk * 2 + khalf) * 8);
#pragma unroll
      for (int t = 0; t < TN; ++t)
        bfr[t] = *reinterpret_cast<const vec8 *>(cB + rB[t] * BK + swz(rB[t], kk * 2 + khalf) * 8);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = Mfma<OT>::mma(af[i], bfr[j], acc[i][j]);
    }
    if (more) {
      OT *nA = lA + (cur ^ 1) * BM * BK, *nB = lB + (cur ^ 1) * BN * BK;
#pragma unroll
      for (int i = 0; i < A_ITERS; ++i) *reinterpret_cast<vec8 *>(nA + sA[i]) = ra[i];
#pragma unroll
      for (int i = 0; i < B_ITERS; ++i) *reinterpret_cast<vec8 *>(nB + sB[i]) = rb[i];
    }
    __syncthreads();
  }

  // ---- epilogue.  Accumulator layout of the 32x32 tile: lane holds column (lane % 32) and rows
  //      (e / 4) * 8 + (lane / 32) * 4 + e % 4 for e = 0..15.
  const int col_in = lane & 31, row_in = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int row = m0 + wm * WMT + i * 32 + (e >> 2) * 8 + row_in + (e & 3);
      if (row >= M) continue;
      if (EPI == PRISM_EPI_SWIGLU) {
#pragma unroll
        for (int j = 0; j < TN / 2; ++j) {
          const int col = n0 + wn * (WNT / 2) + j * 32 + col_in;
          if (col < F) {
            const float g = acc[i][j][e], u = acc[i][j + TN / 2][e];
            reinterpret_cast<OT *>(out_)[(int64_t)row * F + col] = from_f32<OT>(g / (1.0f + __expf(-g)) * u);
          }
        }
      } else {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int col = n0 + wn * WNT + j * 32 + col_in;
          if (col < N) {
            if (EPI == PRISM_EPI_STORE)
              reinterpret_cast<OT *>(out_)[(int64_t)row * N + col] = from_f32<OT>(acc[i][j][e]);
            else if (EPI == PRISM_EPI_STORE_F32)
              reinterpret_cast<float *>(out_)[(int64_t)row * N + col] = acc[i][j][e];
            else
              reinterpret_cast<float *>(out_)[(int64_t)row * N + col] += acc[i][j][e];
          }
        }
      }
    }
  }
}

bool gemm_16_supported(int epilogue, int N, int K) {
  if (K <= 0 || K % BK != 0 || N <= 0) return false;
  if (epilogue == PRISM_EPI_SWIGLU && N % 2 != 0) return false;
  return epilogue >= PRISM_EPI_STORE && epilogue <= PRISM_EPI_STORE_F32;
}

template <typename OT, int BM, int BN, int WM, int WN, int EPI>
static int launch_cfg(const OT *A, const OT *W, void *out, int M, int N, int K, hipStream_t s) {
  constexpr size_t lds = 2 * (size_t)(BM + BN) * BK * sizeof(OT);
  auto kern = gemm_16_kernel<OT, BM, BN, WM, WN, EPI>;
  static bool attr_set = false;   // the attribute is per function; set it once per process
  if (!attr_set) {
    PRISM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)lds));
    attr_set = true;
  }
  const int ncols = EPI == PRISM_EPI_SWIGLU ? N / 2 : N, bn_out = EPI == PRISM_EPI_SWIGLU ? BN / 2 : BN;
  const int nM = cdiv(M, BM), nN = cdiv(ncols, bn_out);
  const int grid = cdiv((int64_t)nM * nN, 8) * 8;
  kern<<<grid, WM * WN * 64, lds, s>>>(A, W, out, M, N, K, nM, nN);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

template <typename OT, int EPI>
static int launch_epi(const OT *A, const OT *W, void *out, int M, int N, int K, hipStream_t s) {
  // big tile when there is enough work to fill 256 CUs with it, else a 128x128 tile
  const int64_t big_tiles = (int64_t)cdiv(M, 256) * cdiv(EPI == PRISM_EPI_SWIGLU ? N / 2 : N, EPI == PRISM_EPI_SWIGLU ? 128 : 256);
  if (big_tiles >= 256) return launch_cfg<OT, 256, 256, 2, 4, EPI>(A, W, out, M, N, K, s);
  return launch_cfg<OT, 128, 128, 2, 2, EPI>(A, W, out, M, N, K, s);
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

int launch_gemm_16(int dtype, int epilogue, const void *A, const void *W, void *out, int M, int N, int K, hipStream_t s) {
  PRISM_REQUIRE(A && W && out && M >= 0 && is16(dtype), PRISM_EINVAL, "gemm: bad arguments");
  PRISM_REQUIRE(gemm_16_supported(epilogue, N, K), PRISM_EUNSUPPORTED,
                "gemm: N = %d, K = %d, epilogue %d not supported (K must be a multiple of %d)", N, K, epilogue, BK);
  if (M == 0) return PRISM_OK;
  if (dtype == PRISM_DTYPE_BF16) return launch_typed<bf16>(epilogue, (const bf16 *)A, (const bf16 *)W, out, M, N, K, s);
  return launch_typed<f16>(epilogue, (const f16 *)A, (const f16 *)W, out, M, N, K, s);
}

}  // namespace prism
