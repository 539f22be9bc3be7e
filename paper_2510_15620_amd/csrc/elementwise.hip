// Bandwidth- and latency-bound steps of the path: embedding gather, RMSNorm, q/k norm + RoPE,
// V rounding + transposition, the intermediate scorer, compaction and the final top-K.
#include "common.h"

namespace prism {

// ------------------------------------------------------------------------------------------------
// Pack + embed: X[t,:] = table[tokens[t],:]            (paper Sec. 4.5: forwarding begins at the embedding)
// One workgroup per token row; HBM-bound (T*H*4 B written).
template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const int32_t *__restrict__ tokens, const T *__restrict__ table,
                                                    int hidden, float *__restrict__ X) {
  const int64_t t = blockIdx.x;
  const T *src = table + (int64_t)tokens[t] * hidden;
  float *dst = X + t * hidden;
  for (int i = threadIdx.x * 4; i < hidden; i += blockDim.x * 4) {
    if (i + 3 < hidden) {
      float4 v = make_float4(to_f32(src[i]), to_f32(src[i + 1]), to_f32(src[i + 2]), to_f32(src[i + 3]));
      *reinterpret_cast<float4 *>(dst + i) = v;
    } else {
      for (int j = i; j < hidden; ++j) dst[j] = to_f32(src[j]);
    }
  }
}

int launch_embed(const int32_t *tokens, int T, const void *table, int hidden, int dtype, float *X, hipStream_t s) {
  PRISM_REQUIRE(tokens && table && X && T >= 0 && hidden > 0 && hidden % 4 == 0, PRISM_EINVAL, "embed: bad arguments");
  if (T == 0) return PRISM_OK;
  if (dtype == PRISM_DTYPE_FP32)
    embed_kernel<float><<<T, 256, 0, s>>>(tokens, (const float *)table, hidden, X);
  else
    embed_kernel<bf16><<<T, 256, 0, s>>>(tokens, (const bf16 *)table, hidden, X);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

// ------------------------------------------------------------------------------------------------
// RMSNorm of the fp32 residual into the GEMM operand type.  One workgroup per row.  HBM-bound: T*H*(4 + sizeof(T)) bytes.
__device__ __forceinline__ float block_sum_256(float v, float *red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = red[0] + red[1] + red[2] + red[3];
  __syncthreads();
  return t;
}

template <typename T, int NV>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float *__restrict__ X, const T *__restrict__ gain,
                                                      int hidden, float eps, T *__restrict__ out) {
  typedef __attribute__((ext_vector_type(4))) float f32x4_t;
  __shared__ float red[4];
  const float *x = X + (int64_t)blockIdx.x * hidden;
  T *o = out + (int64_t)blockIdx.x * hidden;
  // NV > 0: the row (at most NV * 1024 values) stays in registers between the two passes; it is not needed again before
  // the layer's next GEMM epilogue, so the loads bypass the caches' retention.  NV == 0: any width, the row is read twice.
  f32x4_t keep[NV > 0 ? NV : 1];
  float ss = 0.f;
  if (NV > 0) {
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int i = threadIdx.x * 4 + k * 1024;
      if (i < hidden) {
        keep[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(x + i));
        ss += keep[k][0] * keep[k][0] + keep[k][1] * keep[k][1] + keep[k][2] * keep[k][2] + keep[k][3] * keep[k][3];
      }
    }
  } else {
    for (int i = threadIdx.x * 4; i < hidden; i += 1024) {
      float4 v = *reinterpret_cast<const float4 *>(x + i);
      ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
  }
  ss = block_sum_256(ss, red);
  const float r = 1.0f / sqrtf(ss / (float)hidden + eps);
  auto emit = [&](int i, float a, float b, float c, float d) {
    struct alignas(sizeof(T) * 4) Quad { T v[4]; } q, g = *reinterpret_cast<const Quad *>(gain + i);
    q.v[0] = from_f32<T>(a * r * to_f32(g.v[0]));
    q.v[1] = from_f32<T>(b * r * to_f32(g.v[1]));
    q.v[2] = from_f32<T>(c * r * to_f32(g.v[2]));
    q.v[3] = from_f32<T>(d * r * to_f32(g.v[3]));
    *reinterpret_cast<Quad *>(o + i) = q;
  };
  if (NV > 0) {
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int i = threadIdx.x * 4 + k * 1024;
      if (i < hidden) emit(i, keep[k][0], keep[k][1], keep[k][2], keep[k][3]);
    }
  } else {
    for (int i = threadIdx.x * 4; i < hidden; i += 1024) {
      float4 v = *reinterpret_cast<const float4 *>(x + i);
      emit(i, v.x, v.y, v.z, v.w);
    }
  }
}

template <typename T>
static void launch_rmsnorm_typed(const float *X, const void *gain, int T_, int hidden, float eps, void *out, hipStream_t s) {
  if (hidden <= 4096) rmsnorm_kernel<T, 4><<<T_, 256, 0, s>>>(X, (const T *)gain, hidden, eps, (T *)out);
  else if (hidden <= 8192) rmsnorm_kernel<T, 8><<<T_, 256, 0, s>>>(X, (const T *)gain, hidden, eps, (T *)out);
  else rmsnorm_kernel<T, 0><<<T_, 256, 0, s>>>(X, (const T *)gain, hidden, eps, (T *)out);
}

int launch_rmsnorm(const float *X, const void *gain, int T, int hidden, float eps, int dtype, void *out, hipStream_t s) {
  PRISM_REQUIRE(X && gain && out && T >= 0 && hidden > 0 && hidden % 4 == 0, PRISM_EINVAL, "rmsnorm: bad arguments");
  const size_t quad = 4 * dtype_size(dtype);        // the kernel moves four values at a time
  PRISM_REQUIRE((uintptr_t)X % 16 == 0 && (uintptr_t)gain % quad == 0 && (uintptr_t)out % quad == 0, PRISM_EINVAL,
                "rmsnorm: X must be 16-byte aligned, gain and out %zu-byte aligned", quad);
  if (T == 0) return PRISM_OK;
  if (dtype == PRISM_DTYPE_FP32) launch_rmsnorm_typed<float>(X, gain, T, hidden, eps, out, s);
  else if (dtype == PRISM_DTYPE_BF16) launch_rmsnorm_typed<bf16>(X, gain, T, hidden, eps, out, s);
  else launch_rmsnorm_typed<f16>(X, gain, T, hidden, eps, out, s);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

// ------------------------------------------------------------------------------------------------
// RoPE table, evaluated in fp64 and rounded once: (cos, sin)(pos * base^(-2 i / hd)) at tab[pos * half + i], or, transposed,
// at tab[i * n_pos + pos] (the layout the fused q/k/v epilogue reads: consecutive tokens of a sequence are then neighbours).
__global__ void rope_table_kernel(float2 *tab, int n_pos, int half, double log2_base, int transposed) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_pos * half) return;
  const int pos = transposed ? idx % n_pos : idx / half, i = transposed ? idx / n_pos : idx % half;
  const double theta = exp2(-(double)i / (double)half * log2_base);
  const double a = (double)pos * theta;
  tab[idx] = make_float2((float)cos(a), (float)sin(a));
}

int launch_rope_table(float2 *tab, int n_pos, int head_dim, float rope_base, hipStream_t s, bool transposed) {
  PRISM_REQUIRE(tab && n_pos > 0 && head_dim > 0 && head_dim % 2 == 0 && rope_base > 0, PRISM_EINVAL, "rope table: bad arguments");
  const int half = head_dim / 2, n = n_pos * half;
  rope_table_kernel<<<cdiv(n, 256), 256, 0, s>>>(tab, n_pos, half, log2((double)rope_base), transposed ? 1 : 0);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

// Row copy between two tables by index lists: one workgroup per row, 16 bytes per lane and step.
__global__ __launch_bounds__(256) void copy_rows_kernel(const uint4 *__restrict__ src, const int32_t *__restrict__ src_idx,
                                                        uint4 *__restrict__ dst, const int32_t *__restrict__ dst_idx, int vecs) {
  const uint4 *a = src + (int64_t)src_idx[blockIdx.x] * vecs;
  uint4 *b = dst + (int64_t)(dst_idx ? dst_idx[blockIdx.x] : (int)blockIdx.x) * vecs;   // no list: row i -> row i
  for (int i = threadIdx.x; i < vecs; i += 256) b[i] = a[i];
}

int launch_copy_rows(const void *src, const int32_t *src_idx, void *dst, const int32_t *dst_idx, int n, size_t row_bytes,
                     hipStream_t s) {
  PRISM_REQUIRE(src && src_idx && dst && n >= 0 && row_bytes % 16 == 0, PRISM_EINVAL, "copy_rows: bad arguments");
  if (n == 0) return PRISM_OK;
  copy_rows_kernel<<<n, 256, 0, s>>>((const uint4 *)src, src_idx, (uint4 *)dst, dst_idx, (int)(row_bytes / 16));
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

// Per-head RMSNorm (optional) then rotate-half RoPE on the q and k parts of the fp32 projection
// QKV [T, (nq + 2 nkv) * hd].  One wavefront per (token, head); lane i owns pairs (i, i + hd/2),
// (i + 64, i + 64 + hd/2), ...  The result is rounded ONCE, to the operand type of the QK^T
// contraction: fp32 mode rewrites QKV in place, bf16 mode writes QK [T, (nq + nkv) * hd].
template <typename T>
__global__ __launch_bounds__(256) void qk_finish_kernel(float *__restrict__ QKV, const int32_t *__restrict__ pos,
                                                        const T *__restrict__ q_gain, const T *__restrict__ k_gain,
                                                        int n_tok, int nq, int nkv, int hd, float eps, int qk_norm,
                                                        const float2 *__restrict__ rope_tab, T *__restrict__ out,
                                                        int out_row) {
  const int heads = nq + nkv;
  const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= (int64_t)n_tok * heads) return;
  const int t = (int)(item / heads), h = (int)(item % heads);
  const int lane = threadIdx.x & 63, half = hd / 2;
  const float *x = QKV + (int64_t)t * (nq + 2 * nkv) * hd + (int64_t)h * hd;
  T *o = out + (int64_t)t * out_row + (int64_t)h * hd;
  const T *g = h < nq ? q_gain : k_gain;
  const float2 *tab = rope_tab + (int64_t)pos[t] * half;
  float ss = 0.f;
  for (int i = lane; i < half; i += 64) {
    const float a = x[i], b = x[i + half];
    ss += a * a + b * b;
  }
  float r = 1.f;
  if (qk_norm) {
    ss = wave_sum(ss);
    r = 1.0f / sqrtf(ss / (float)hd + eps);
  }
  for (int i = lane; i < half; i += 64) {
    float a = x[i], b = x[i + half];
    if (qk_norm) {
      a = a * r * to_f32(g[i]);
      b = b * r * to_f32(g[i + half]);
    }
    const float2 cs = tab[i];
    o[i] = from_f32<T>(a * cs.x - b * cs.y);
    o[i + half] = from_f32<T>(b * cs.x + a * cs.y);
  }
}

int launch_qk_finish(int dtype, float *QKV, const int32_t *pos, const void *q_gain, const void *k_gain, int T,
                     int nq, int nkv, int hd, float eps, int qk_norm, const float2 *rope_tab, void *QK, hipStream_t s) {
  PRISM_REQUIRE(QKV && pos && rope_tab && T >= 0 && nq > 0 && nkv > 0 && hd > 0 && hd % 2 == 0, PRISM_EINVAL,
                "qk_finish: bad arguments");
  PRISM_REQUIRE(!qk_norm || (q_gain && k_gain), PRISM_EINVAL, "qk_finish: gains missing");
  PRISM_REQUIRE(dtype == PRISM_DTYPE_FP32 || QK, PRISM_EINVAL, "qk_finish: 16-bit modes need the QK output");
  if (T == 0) return PRISM_OK;
  const int64_t items = (int64_t)T * (nq + nkv);
  const int grid = cdiv(items, 4);
  if (dtype == PRISM_DTYPE_FP32)
    qk_finish_kernel<float><<<grid, 256, 0, s>>>(QKV, pos, (const float *)q_gain, (const float *)k_gain, T, nq, nkv, hd,
                                                  eps, qk_norm, rope_tab, QKV, (nq + 2 * nkv) * hd);
  else if (dtype == PRISM_DTYPE_BF16)
    qk_finish_kernel<bf16><<<grid, 256, 0, s>>>(QKV, pos, (const bf16 *)q_gain, (const bf16 *)k_gain, T, nq, nkv, hd,
                                                 eps, qk_norm, rope_tab, (bf16 *)QK, (nq + nkv) * hd);
  else
    qk_finish_kernel<f16><<<grid, 256, 0, s>>>(QKV, pos, (const f16 *)q_gain, (const f16 *)k_gain, T, nq, nkv, hd,
                                                eps, qk_norm, rope_tab, (f16 *)QK, (nq + nkv) * hd);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

// V part of the fp32 projection -> Vt [nkv][hd][vt_stride], column vt_col[t]: the P V contraction runs
// over keys, so the MFMA operand wants keys contiguous.  P V always runs on the f16 matrix-core
// instruction (the probabilities keep 11 significand bits), so Vt is IEEE half; in bf16-operand mode
// the values are rounded to bf16 first (half holds every bf16 value of normal half range exactly).
// Tile of 64 tokens x hd through LDS.
template <typename OT>
__global__ __launch_bounds__(256) void v_finish_kernel(const float *__restrict__ QKV, int n_tok, int nq, int nkv, int hd,
                                                       f16 *__restrict__ Vt, const int32_t *__restrict__ vt_col,
                                                       int64_t vt_stride) {
  __shared__ f16 tile[64][128 + 2];
  const int t0 = blockIdx.x * 64, h = blockIdx.y;
  const int row_elems = (nq + 2 * nkv) * hd;
  const float *src = QKV + (int64_t)(nq + nkv + h) * hd;
  for (int idx = threadIdx.x; idx < 64 * hd; idx += 256) {
    const int r = idx / hd, d = idx % hd;
    if (t0 + r < n_tok) tile[r][d] = from_f32<f16>(to_f32(from_f32<OT>(src[(int64_t)(t0 + r) * row_elems + d])));
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < 64 * hd; idx += 256) {
    const int d = idx / 64, r = idx % 64;
    if (t0 + r < n_tok) Vt[((int64_t)h * hd + d) * vt_stride + vt_col[t0 + r]] = tile[r][d];
  }
}

int launch_v_finish(int dtype, const float *QKV, int T, int nq, int nkv, int hd, void *Vt, const int32_t *vt_col,
                    int64_t vt_stride, hipStream_t s) {
  PRISM_REQUIRE(QKV && Vt && vt_col && T >= 0 && hd > 0 && hd <= 128 && is16(dtype), PRISM_EINVAL, "v_finish: bad arguments");
  if (T == 0) return PRISM_OK;
  if (dtype == PRISM_DTYPE_BF16)
    v_finish_kernel<bf16><<<dim3(cdiv(T, 64), nkv), 256, 0, s>>>(QKV, T, nq, nkv, hd, (f16 *)Vt, vt_col, vt_stride);
  else
    v_finish_kernel<f16><<<dim3(cdiv(T, 64), nkv), 256, 0, s>>>(QKV, T, nq, nkv, hd, (f16 *)Vt, vt_col, vt_stride);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

// ------------------------------------------------------------------------------------------------
// Intermediate scorer (Sec. 4.1): last-token state -> final RMSNorm -> yes/no head rows.
// One workgroup per live candidate; reads H floats; latency-bound.
template <typename T>
__global__ __launch_bounds__(256) void score_kernel(const float *__restrict__ X, const int32_t *__restrict__ last_row,
                                                    int hidden, const T *__restrict__ gain, const T *__restrict__ w_yes,
                                                    const T *__restrict__ w_no, float eps, float *__restrict__ scores) {
  __shared__ float red[4];
  const float *x = X + (int64_t)(last_row ? last_row[blockIdx.x] : (int)blockIdx.x) * hidden;   // no list: state c is row c
  float ss = 0.f, dy = 0.f, dn = 0.f;
  for (int i = threadIdx.x; i < hidden; i += 256) {
    const float v = x[i];
    ss += v * v;
    const float z = v * to_f32(gain[i]);
    dy += z * to_f32(w_yes[i]);
    dn += z * to_f32(w_no[i]);
  }
  ss = block_sum_256(ss, red);
  dy = block_sum_256(dy, red);
  dn = block_sum_256(dn, red);
  if (threadIdx.x == 0) {
    const float r = 1.0f / sqrtf(ss / (float)hidden + eps);
    scores[blockIdx.x] = dy * r - dn * r;
  }
}

int launch_score(const float *X, const int32_t *last_row, int n, int hidden, const void *final_norm,
                 const void *w_yes, const void *w_no, int dtype, float eps, float *scores, hipStream_t s) {
  PRISM_REQUIRE(X && final_norm && w_yes && w_no && scores && n >= 0 && hidden > 0, PRISM_EINVAL, "score: bad arguments");
  if (n == 0) return PRISM_OK;
  if (dtype == PRISM_DTYPE_FP32)
    score_kernel<float><<<n, 256, 0, s>>>(X, last_row, hidden, (const float *)final_norm, (const float *)w_yes,
                                           (const float *)w_no, eps, scores);
  else
    score_kernel<bf16><<<n, 256, 0, s>>>(X, last_row, hidden, (const bf16 *)final_norm, (const bf16 *)w_yes,
                                          (const bf16 *)w_no, eps, scores);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

// ------------------------------------------------------------------------------------------------
// Compaction (Sec. 4.1: continue only on the remaining candidates): each kept sequence's rows move
// to their new offset in a second buffer, order preserved.  HBM-bound: 2 * T' * H * 4 bytes.
__global__ __launch_bounds__(256) void compact_kernel(const float *__restrict__ Xs, float *__restrict__ Xd,
                                                      const int32_t *__restrict__ src_start,
                                                      const int32_t *__restrict__ dst_start,
                                                      const int32_t *__restrict__ len, int hidden) {
  const int c = blockIdx.x;
  const int n = len[c], h4 = hidden / 4;
  const float4 *src = reinterpret_cast<const float4 *>(Xs + (int64_t)src_start[c] * hidden);
  float4 *dst = reinterpret_cast<float4 *>(Xd + (int64_t)dst_start[c] * hidden);
  for (int r = blockIdx.y; r < n; r += gridDim.y)
    for (int i = threadIdx.x; i < h4; i += 256) dst[(int64_t)r * h4 + i] = src[(int64_t)r * h4 + i];
}

int launch_compact(const float *Xs, float *Xd, const int32_t *src_start, const int32_t *dst_start,
                   const int32_t *len, int n_keep, int hidden, hipStream_t s) {
  PRISM_REQUIRE(Xs && Xd && Xs != Xd && src_start && dst_start && len && n_keep >= 0 && hidden % 4 == 0, PRISM_EINVAL,
                "compact: bad arguments");
  if (n_keep == 0) return PRISM_OK;
  compact_kernel<<<dim3(n_keep, 32), 256, 0, s>>>(Xs, Xd, src_start, dst_start, len, hidden);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

// ------------------------------------------------------------------------------------------------
// Shared query: its V^T columns, written once per chunk, are copied into every sequence's column range.
__global__ __launch_bounds__(256) void vt_prefix_broadcast_kernel(f16 *__restrict__ Vt, int64_t vt_stride, int rows, int ql,
                                                                   const int32_t *__restrict__ seq_col0) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  f16 *v = Vt + (int64_t)row * vt_stride;
  const int col0 = seq_col0[blockIdx.y];
  const int ncol = (ql + 15) & ~15;
  for (int cidx = threadIdx.x & 63; cidx < ncol; cidx += 64)
    if (vt_column_of_key(cidx) < ql) v[col0 + cidx] = v[cidx];        // the mapping is its own inverse
}

int launch_vt_prefix_broadcast(void *Vt, int64_t vt_stride, int rows, int ql, const int32_t *seq_col0, int n_seq, hipStream_t s) {
  PRISM_REQUIRE(Vt && seq_col0 && vt_stride > 0 && rows > 0 && ql > 0 && n_seq >= 0, PRISM_EINVAL, "vt prefix broadcast: bad arguments");
  if (n_seq == 0) return PRISM_OK;
  vt_prefix_broadcast_kernel<<<dim3(cdiv(rows, 4), n_seq), 256, 0, s>>>((f16 *)Vt, vt_stride, rows, ql, seq_col0);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

// ------------------------------------------------------------------------------------------------
// Final top-K (Sec. 2.1): rank by counting (score descending, lower position first on ties).
__global__ __launch_bounds__(1024) void topk_kernel(const float *__restrict__ scores, const int8_t *__restrict__ tag,
                                                    int want, int n, int K, int32_t *__restrict__ out_pos,
                                                    float *__restrict__ out_scores) {
  // entries whose tag differs from `want` do not take part (tag == nullptr: all take part)
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    if (tag && tag[i] != want) continue;
    const float si = scores[i];
    int rank = 0;
    for (int j = 0; j < n; ++j) {
      if (tag && tag[j] != want) continue;
      const float sj = scores[j];
      rank += (sj > si) || (sj == si && j < i);
    }
    if (rank < K) {
      out_pos[rank] = i;
      out_scores[rank] = si;
    }
  }
}

int launch_topk_masked(const float *scores, const int8_t *tag, int want, int n, int K, int32_t *out_pos,
                       float *out_scores, hipStream_t s) {
  PRISM_REQUIRE(scores && out_pos && out_scores && n >= 0 && K >= 0, PRISM_EINVAL, "topk: bad arguments");
  if (n == 0 || K == 0) return PRISM_OK;
  topk_kernel<<<1, 1024, 0, s>>>(scores, tag, want, n, K, out_pos, out_scores);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

int launch_topk(const float *scores, int n, int K, int32_t *out_pos, float *out_scores, hipStream_t s) {
  return launch_topk_masked(scores, nullptr, 0, n, K, out_pos, out_scores, s);
}

__global__ void fill_zero_kernel(uint4 *p, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

// In place, 8 elements (16 bytes) per lane and step over the first n8 * 8 elements, one element per lane over the rest.
__global__ __launch_bounds__(256) void bf16_to_f16_kernel(unsigned short *p, size_t n, size_t n8) {
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
  auto half_bits = [](unsigned bf16_in_high_half) -> unsigned {
    const f16 h = from_f32<f16>(__uint_as_float(bf16_in_high_half));
    return (unsigned)*reinterpret_cast<const unsigned short *>(&h);
  };
  uint4 *q = reinterpret_cast<uint4 *>(p);
  for (size_t i = t; i < n8; i += stride) {
    const uint4 v = q[i];
    unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) w[k] = half_bits(w[k] << 16) | (half_bits(w[k] & 0xffff0000u) << 16);
    q[i] = make_uint4(w[0], w[1], w[2], w[3]);
  }
  for (size_t i = n8 * 8 + t; i < n; i += stride) p[i] = (unsigned short)half_bits((unsigned)p[i] << 16);
}

int launch_bf16_to_f16(void *p, size_t n, hipStream_t s) {
  PRISM_REQUIRE(p, PRISM_EINVAL, "bf16_to_f16: null pointer");
  if (n == 0) return PRISM_OK;
  const size_t n8 = (reinterpret_cast<uintptr_t>(p) % 16 == 0) ? n / 8 : 0;      // 16-byte steps need a 16-byte aligned buffer
  const size_t work = n8 ? n8 : n, blocks = (work + 255) / 256;
  bf16_to_f16_kernel<<<(int)(blocks < 8192 ? blocks : 8192), 256, 0, s>>>((unsigned short *)p, n, n8);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

int launch_fill_zero(void *p, size_t bytes, hipStream_t s) {
  PRISM_REQUIRE(p && bytes % 16 == 0, PRISM_EINVAL, "fill_zero: bad arguments");
  if (bytes == 0) return PRISM_OK;
  const size_t n16 = bytes / 16;
  const int grid = (int)((n16 + 255) / 256 < 4096 ? (n16 + 255) / 256 : 4096);
  fill_zero_kernel<<<grid, 256, 0, s>>>((uint4 *)p, n16);
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

}  // namespace prism
