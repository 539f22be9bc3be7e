// fp32 layer contractions for the fp32 mode (small models, 1e-4 parity runs): a plain LDS-tiled
// kernel on the vector ALUs with every edge bounds-checked, so any M, N, K works.
// C = A W^T with A [M,K], W [N,K] row-major.  64x64 output tile, 256 threads, 4x4 per thread.
#include "common.h"

namespace prism {

template <int EPI>
__global__ __launch_bounds__(256) void gemm_fp32_kernel(const float *__restrict__ A, const float *__restrict__ W,
                                                        float *__restrict__ out, int M, int N, int K) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 1];
  __shared__ float Bs[BK][BN + 1];
  __shared__ float Us[EPI == PRISM_EPI_SWIGLU ? BK : 1][BN + 1];
  const int F = EPI == PRISM_EPI_SWIGLU ? N / 2 : N;       // output columns
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {}, accu[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
    for (int idx = threadIdx.x; idx < BM * BK; idx += 256) {
      const int r = idx / BK, c = idx % BK;
      As[c][r] = (m0 + r < M && k0 + c < K) ? A[(int64_t)(m0 + r) * K + k0 + c] : 0.f;
      Bs[c][r] = (n0 + r < F && k0 + c < K) ? W[(int64_t)(n0 + r) * K + k0 + c] : 0.f;
      if (EPI == PRISM_EPI_SWIGLU)
        Us[c][r] = (n0 + r < F && k0 + c < K) ? W[(int64_t)(F + n0 + r) * K + k0 + c] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4], u[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = As[kk][ty * 4 + i];
        b[i] = Bs[kk][tx * 4 + i];
        if (EPI == PRISM_EPI_SWIGLU) u[i] = Us[kk][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[i][j] += a[i] * b[j];
          if (EPI == PRISM_EPI_SWIGLU) accu[i][j] += a[i] * u[j];
        }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < M && n < F) {
        float *o = out + (int64_t)m * F + n;
        if (EPI == PRISM_EPI_STORE) *o = acc[i][j];
        else if (EPI == PRISM_EPI_RESIDUAL) *o += acc[i][j];
        else {
          const float g = acc[i][j];
          *o = g / (1.0f + expf(-g)) * accu[i][j];
        }
      }
    }
}

int launch_gemm_fp32(int epilogue, const float *A, const float *W, void *out, int M, int N, int K, hipStream_t s) {
  PRISM_REQUIRE(A && W && out && M >= 0 && N > 0 && K > 0, PRISM_EINVAL, "gemm fp32: bad arguments");
  PRISM_REQUIRE(epilogue != PRISM_EPI_SWIGLU || N % 2 == 0, PRISM_EINVAL, "gemm fp32: SwiGLU needs an even row count");
  if (M == 0) return PRISM_OK;
  const int F = epilogue == PRISM_EPI_SWIGLU ? N / 2 : N;
  dim3 grid(cdiv(F, 64), cdiv(M, 64));
  if (epilogue == PRISM_EPI_STORE) gemm_fp32_kernel<PRISM_EPI_STORE><<<grid, 256, 0, s>>>(A, W, (float *)out, M, N, K);
  else if (epilogue == PRISM_EPI_RESIDUAL) gemm_fp32_kernel<PRISM_EPI_RESIDUAL><<<grid, 256, 0, s>>>(A, W, (float *)out, M, N, K);
  else if (epilogue == PRISM_EPI_SWIGLU) gemm_fp32_kernel<PRISM_EPI_SWIGLU><<<grid, 256, 0, s>>>(A, W, (float *)out, M, N, K);
  else PRISM_REQUIRE(false, PRISM_EINVAL, "gemm: unknown epilogue %d", epilogue);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

}  // namespace prism
