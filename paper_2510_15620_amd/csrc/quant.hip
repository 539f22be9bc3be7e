// 4-bit weights for the streamed layers (the quantised variant of the paper's Sec. 6 evaluation; the paper names the
// format "W4A16" without detail, so the format is this build's reading): symmetric codes q in [-7, 7] for groups of 128
// consecutive input features of one output row, one bf16 scale per group (max|w| / 7, rounded to nearest even; 1 for an
// all-zero group), q = w / scale rounded to nearest even and clamped.  A bf16 scale times |q| <= 7 has at most 11
// significant bits, so the dequantised weight q * scale is exact in IEEE half: the matrix-core kernels see ordinary
// half (or bf16) weights, expanded layer by layer right before use, and only a quarter of the bytes travel.
//
// Blob of an [N, K] matrix: N * K / 2 code bytes (row-major; byte k / 2 of a row holds code k in its low nibble for
// even k, in its high nibble for odd k; a nibble is q + 8), then N * K / 128 bf16 scales (row-major).
#include <algorithm>

#include "common.h"

namespace prism {

static constexpr int kGroup = 128;

__device__ __forceinline__ float bf16_rne(float x) {
  unsigned u = __float_as_uint(x);
  u = (u + 0x7fffu + ((u >> 16) & 1u)) & 0xffff0000u;
  return __uint_as_float(u);
}

// one wavefront per (row, group): lane l owns elements 2l and 2l + 1 of the group
__global__ __launch_bounds__(256) void quantize_w4_kernel(const unsigned short *__restrict__ W, int64_t n_groups, int gpr /* groups per row */,
                                                          unsigned char *__restrict__ codes, unsigned short *__restrict__ scales) {
  const int64_t g = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (g >= n_groups) return;
  const int lane = threadIdx.x & 63;
  const unsigned pair = *reinterpret_cast<const unsigned *>(W + g * kGroup + 2 * lane);
  const float w0 = __uint_as_float(pair << 16), w1 = __uint_as_float(pair & 0xffff0000u);
  float amax = fmaxf(fabsf(w0), fabsf(w1));
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, 64));
  float scale = bf16_rne(amax / 7.0f);
  if (scale == 0.f) scale = 1.0f;
  const float q0 = fminf(fmaxf(rintf(w0 / scale), -7.f), 7.f), q1 = fminf(fmaxf(rintf(w1 / scale), -7.f), 7.f);
  codes[g * (kGroup / 2) + lane] = (unsigned char)(((int)q0 + 8) | (((int)q1 + 8) << 4));
  if (lane == 0) scales[g] = (unsigned short)(__float_as_uint(scale) >> 16);
  (void)gpr;
}

// one thread per 8 codes (4 bytes in, 16 bytes out)
template <typename OT>
__global__ __launch_bounds__(256) void dequantize_w4_kernel(const unsigned *__restrict__ codes, const unsigned short *__restrict__ scales,
                                                            int64_t n_words, OT *__restrict__ out) {
  typedef typename Mfma<OT>::vec8 vec8;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n_words; i += stride) {
    const unsigned c = codes[i];
    const float s = __uint_as_float((unsigned)scales[i / (kGroup / 8)] << 16);
    vec8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = from_f32<OT>((float)((int)((c >> (4 * e)) & 15u) - 8) * s);
    *reinterpret_cast<vec8 *>(out + i * 8) = v;
  }
}

// n elements of bf16 -> the operand type (norm gains that travel beside the quantised matrices)
template <typename OT>
__global__ void convert_bf16_kernel(const unsigned short *__restrict__ src, OT *__restrict__ dst, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = from_f32<OT>(__uint_as_float((unsigned)src[i] << 16));
}

int64_t w4_blob_bytes(int64_t N, int64_t K) { return N * K / 2 + N * (K / kGroup) * 2; }

int launch_quantize_w4(const void *W, int N, int K, void *blob, hipStream_t s) {
  PRISM_REQUIRE(W && blob && N > 0 && K > 0 && K % kGroup == 0, PRISM_EINVAL, "quantize_w4: K must be a positive multiple of %d", kGroup);
  const int64_t n_groups = (int64_t)N * (K / kGroup);
  unsigned char *codes = reinterpret_cast<unsigned char *>(blob);
  quantize_w4_kernel<<<(unsigned)cdiv(n_groups, 4), 256, 0, s>>>((const unsigned short *)W, n_groups, K / kGroup, codes,
                                                                  reinterpret_cast<unsigned short *>(codes + (int64_t)N * K / 2));
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

int launch_dequantize_w4(const void *blob, int N, int K, int dtype, void *out, hipStream_t s) {
  PRISM_REQUIRE(blob && out && N > 0 && K > 0 && K % kGroup == 0 && is16(dtype), PRISM_EINVAL,
                "dequantize_w4: K must be a positive multiple of %d and the output a 16-bit type", kGroup);
  const int64_t n_words = (int64_t)N * K / 8;
  const unsigned char *codes = reinterpret_cast<const unsigned char *>(blob);
  const unsigned short *scales = reinterpret_cast<const unsigned short *>(codes + (int64_t)N * K / 2);
  const int grid = (int)std::min<int64_t>(cdiv(n_words, 256), 16384);
  if (dtype == PRISM_DTYPE_BF16)
    dequantize_w4_kernel<bf16><<<grid, 256, 0, s>>>((const unsigned *)codes, scales, n_words, (bf16 *)out);
  else
    dequantize_w4_kernel<f16><<<grid, 256, 0, s>>>((const unsigned *)codes, scales, n_words, (f16 *)out);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

int launch_convert_bf16(const void *src, int64_t n, int dtype, void *dst, hipStream_t s) {
  PRISM_REQUIRE(src && dst && n >= 0 && is16(dtype), PRISM_EINVAL, "convert_bf16: bad arguments");
  if (n == 0) return PRISM_OK;
  if (dtype == PRISM_DTYPE_BF16) convert_bf16_kernel<bf16><<<(unsigned)cdiv(n, 256), 256, 0, s>>>((const unsigned short *)src, (bf16 *)dst, n);
  else convert_bf16_kernel<f16><<<(unsigned)cdiv(n, 256), 256, 0, s>>>((const unsigned short *)src, (f16 *)dst, n);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

}  // namespace prism
