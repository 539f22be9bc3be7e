// Causal GQA attention for the fp32 mode: the definition, one workgroup per (token, query head).
// Any head_dim; sequences up to PRISM_MAX_SEQ tokens (the score row lives in LDS).
#include "common.h"

namespace prism {

__global__ __launch_bounds__(128) void attention_fp32_kernel(const float *__restrict__ QKV,
                                                             const int32_t *__restrict__ pos, int nq, int nkv, int hd,
                                                             float *__restrict__ out) {
  extern __shared__ float p[];          // [pos + 1] scores, then [hd] the query
  __shared__ float red[2];
  const int t = blockIdx.x, h = blockIdx.y;
  const int i = pos[t], n_keys = i + 1;
  const int row = (nq + 2 * nkv) * hd, kvh = h / (nq / nkv);
  const float *q = QKV + (int64_t)t * row + (int64_t)h * hd;
  const float *kbase = QKV + (int64_t)(t - i) * row + (int64_t)(nq + kvh) * hd;
  const float *vbase = kbase + (int64_t)nkv * hd;
  float *qs = p + n_keys;
  for (int d = threadIdx.x; d < hd; d += 128) qs[d] = q[d];
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)hd);
  float mx = -INFINITY;
  for (int j = threadIdx.x; j < n_keys; j += 128) {
    const float *k = kbase + (int64_t)j * row;
    float dot = 0.f;
    for (int d = 0; d < hd; ++d) dot += qs[d] * k[d];
    dot *= scale;
    p[j] = dot;
    mx = fmaxf(mx, dot);
  }
  mx = wave_max(mx);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = fmaxf(red[0], red[1]);
  __syncthreads();
  float sum = 0.f;
  for (int j = threadIdx.x; j < n_keys; j += 128) {
    const float e = expf(p[j] - mx);
    p[j] = e;
    sum += e;
  }
  sum = wave_sum(sum);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sum;
  __syncthreads();
  sum = red[0] + red[1];
  for (int d = threadIdx.x; d < hd; d += 128) {
    float acc = 0.f;
    for (int j = 0; j < n_keys; ++j) acc += p[j] * vbase[(int64_t)j * row + d];
    out[(int64_t)t * nq * hd + (int64_t)h * hd + d] = acc / sum;
  }
}

int launch_attention_fp32(const float *QKV, const int32_t *pos, int T, int nq, int nkv, int hd, float *out,
                          hipStream_t s) {
  PRISM_REQUIRE(QKV && pos && out && T >= 0 && nq > 0 && nkv > 0 && nq % nkv == 0 && hd > 0, PRISM_EINVAL,
                "attention fp32: bad arguments");
  if (T == 0) return PRISM_OK;
  const size_t lds = (size_t)(PRISM_MAX_SEQ + hd) * sizeof(float);
  PRISM_REQUIRE(lds <= 64 * 1024, PRISM_EUNSUPPORTED, "attention fp32: head_dim %d too large", hd);
  attention_fp32_kernel<<<dim3(T, nq), 128, lds, s>>>(QKV, pos, nq, nkv, hd, out);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

}  // namespace prism
