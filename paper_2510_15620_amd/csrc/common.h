// Shared declarations of the HIP library: error plumbing, element types, kernel launchers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "prism.h"

namespace prism {

// ---- error plumbing --------------------------------------------------------------------------
void set_error(const char *fmt, ...);
int hip_fail(hipError_t e, const char *what, const char *file, int line);

#define PRISM_HIP(call)                                                        \
  do {                                                                         \
    hipError_t e_ = (call);                                                    \
    if (e_ != hipSuccess) return ::prism::hip_fail(e_, #call, __FILE__, __LINE__); \
  } while (0)

#define PRISM_REQUIRE(cond, code, ...)                                         \
  do {                                                                         \
    if (!(cond)) { ::prism::set_error(__VA_ARGS__); return (code); }           \
  } while (0)

#define PRISM_TRY(call)                                                        \
  do { int rc_ = (call); if (rc_ != PRISM_OK) return rc_; } while (0)

// ---- element types ---------------------------------------------------------------------------
typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef _Float16 f16;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }  // round-to-nearest-even
__device__ __forceinline__ float to_f32(f16 v) { return (float)v; }
// IEEE half, round-to-nearest-even, saturating at the largest finite half instead of overflowing to infinity
template <> __device__ __forceinline__ f16 from_f32<f16>(float v) { return (f16)fminf(fmaxf(v, -65504.0f), 65504.0f); }

// matrix-core instruction of a 16-bit operand type: D(32x32, fp32) += A(32x16) B(16x32)
template <typename T> struct Mfma;
template <> struct Mfma<bf16> {
  static constexpr bool kIsF16 = false;
  typedef bf16x8 vec8;
  typedef bf16x4 vec4;
  static __device__ __forceinline__ f32x16 mma(vec8 a, vec8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
};
template <> struct Mfma<f16> {
  static constexpr bool kIsF16 = true;
  typedef f16x8 vec8;
  typedef f16x4 vec4;
  static __device__ __forceinline__ f32x16 mma(vec8 a, vec8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }
};

static inline size_t dtype_size(int dtype) { return dtype == PRISM_DTYPE_FP32 ? 4 : 2; }
static inline bool is16(int dtype) { return dtype == PRISM_DTYPE_BF16 || dtype == PRISM_DTYPE_F16; }
static inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
static inline int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---- launchers (each validates shapes, launches on `s`, never synchronises) -------------------
int launch_embed(const int32_t *tokens, int T, const void *table, int hidden, int dtype, float *X, hipStream_t s);
int launch_rmsnorm(const float *X, const void *gain, int T, int hidden, float eps, int dtype, void *out, hipStream_t s);
int launch_gemm_fp32(int epilogue, const float *A, const float *W, void *out, int M, int N, int K, hipStream_t s);
// 16-bit operands (dtype PRISM_DTYPE_BF16 or PRISM_DTYPE_F16) on the matrix cores
int launch_gemm_16(int dtype, int epilogue, const void *A, const void *W, void *out, int M, int N, int K, hipStream_t s);
bool gemm_16_supported(int epilogue, int N, int K);
// The q/k/v projection with everything that follows it fused into the GEMM epilogue (head_dim 128): per-head RMSNorm
// (optional) and rotate-half RoPE on the q and k heads, rounded once into QK [T, (nq+nkv)*128]; the v heads rounded to the
// operand type and written transposed, as IEEE half, to Vt [nkv][128][vt_stride] at column vt_col[t].
struct QkvEpilogue {
  const int32_t *pos, *vt_col;
  const void *q_gain, *k_gain;
  const float2 *rope_tab_t;   // transposed table: (cos, sin) of (pos, i) at [i * rope_stride + pos]
  int rope_stride;            // positions the table was built for
  void *QK;
  void *Vt;
  int64_t vt_stride;
  int nq, nkv, qk_norm;
  float eps;
};
static const int kEpiQkv = 4;   // internal epilogue code of launch_gemm_16_qkv
bool gemm_16_qkv_supported(int M, int nq, int nkv, int hd, int K);
int launch_gemm_16_qkv(int dtype, const void *Xn, const void *Wqkv, int M, int K, int hd, const QkvEpilogue &e, hipStream_t s);

// dst row dst_idx[i] (i itself if dst_idx is null) = src row src_idx[i], i < n; rows of row_bytes (a multiple of 16) bytes.  src may be pinned host
// memory (its device-visible address): the embedding-table cache fetches its misses this way (Sec. 4.4).
int launch_copy_rows(const void *src, const int32_t *src_idx, void *dst, const int32_t *dst_idx, int n, size_t row_bytes,
                     hipStream_t s);

// 4-bit weight blobs (quant.hip): codes then bf16 scales, groups of 128 along K
int64_t w4_blob_bytes(int64_t N, int64_t K);
int launch_quantize_w4(const void *W_bf16, int N, int K, void *blob, hipStream_t s);
int launch_dequantize_w4(const void *blob, int N, int K, int dtype, void *out, hipStream_t s);
int launch_convert_bf16(const void *src, int64_t n, int dtype, void *dst, hipStream_t s);

// cos/sin table for RoPE: tab[pos * (hd/2) + i] = (cos, sin)(pos * base^(-2i/hd)), evaluated in fp64; transposed:
// tab[i * n_pos + pos]
int launch_rope_table(float2 *tab, int n_pos, int head_dim, float rope_base, hipStream_t s, bool transposed = false);
// q/k per-head RMSNorm + RoPE from the fp32 projection.  fp32 mode: in place (QK == nullptr).  bf16 mode:
// q,k -> QK [T, (nq+nkv)*hd] bf16.
int launch_qk_finish(int dtype, float *QKV, const int32_t *pos, const void *q_gain, const void *k_gain, int T,
                     int nq, int nkv, int hd, float eps, int qk_norm, const float2 *rope_tab, void *QK, hipStream_t s);
// v part of the fp32 projection -> Vt [nkv][hd][vt_stride], IEEE half (in bf16-operand mode: bf16-rounded values)
int launch_v_finish(int dtype, const float *QKV, int T, int nq, int nkv, int hd, void *Vt, const int32_t *vt_col,
                    int64_t vt_stride, hipStream_t s);
// Copies the V^T columns of a chunk's shared query (positions [0, ql): columns vt_column_of_key(position) of the chunk,
// whose query sequence starts at column 0) into the column range of each of n_seq sequences (first columns seq_col0[i],
// [device]); rows = nkv * hd rows of Vt.  Columns of positions >= ql are left alone.
int launch_vt_prefix_broadcast(void *Vt, int64_t vt_stride, int rows, int ql, const int32_t *seq_col0, int n_seq, hipStream_t s);

// generic fp32 attention: one workgroup per (token, q head); pos[t] = position of t in its sequence
int launch_attention_fp32(const float *QKV, const int32_t *pos, int T, int nq, int nkv, int hd, float *out,
                          hipStream_t s);
// matrix-core attention (hd == 128).  tiles: per work item {row base of the sequence, sequence length, first query of
// the tile, column of the sequence's first key in Vt, length and first row of a shared prefix}; see attn_16.hip.
// Positions below pre_len are a prefix whose q/k rows are stored once, at pre_row0 + position, and shared by several
// sequences (Sec. 3.3 batches (query, candidate) pairs that all begin with the same query; under a causal mask the
// query tokens' states do not depend on the candidate); position p >= pre_len has row row_base + p.  Without a prefix
// pre_len = 0 and row_base is the sequence's first row.  V^T columns are per sequence for ALL its positions.
// out_base: the tile's output for position p goes to row out_base + p (normally row_base; it differs when the layout the
// q/k rows were projected in is not the one the layer continues in).
struct AttnTile { int32_t row_base, seq_len, q0, vt_col0, pre_len, pre_row0, out_base, reserved; };
int launch_attention_16(int dtype, const void *QK, const void *Vt, int64_t vt_stride, const AttnTile *tiles, int n_tiles,
                        int T, int nq, int nkv, int hd, void *out, hipStream_t s);
bool attention_16_supported(int nq, int nkv, int hd);
int attention_16_block_queries(int nq, int nkv);   // queries per AttnTile for this head grouping
// Column of key p of a sequence in the V^T buffer, relative to the sequence's first column: within every group of 16
// the keys are stored in the order 0-3, 8-11, 4-7, 12-15 (the order in which the matrix cores' accumulator layout hands
// the probabilities to the second contraction), i.e. bits 2 and 3 of p are swapped.
__host__ __device__ inline int vt_column_of_key(int p) { return (p & ~12) | ((p & 4) << 1) | ((p & 8) >> 1); }
static const int kAttnBQ = 64;   // query rows per attention work item

int launch_score(const float *X, const int32_t *last_row, int n, int hidden, const void *final_norm,
                 const void *w_yes, const void *w_no, int dtype, float eps, float *scores, hipStream_t s);
size_t route_workspace_bytes(int n, int k);
int launch_route(const float *scores, int n, int K_rem, int n_clusters, float tau, int8_t *fate, double *stats,
                 void *workspace, hipStream_t s);
int launch_compact(const float *Xs, float *Xd, const int32_t *src_start, const int32_t *dst_start,
                   const int32_t *len, int n_keep, int hidden, hipStream_t s);
int launch_topk(const float *scores, int n, int K, int32_t *out_pos, float *out_scores, hipStream_t s);
// same, restricted to the entries whose tag equals `want` (tag may be null: all entries)
int launch_topk_masked(const float *scores, const int8_t *tag, int want, int n, int K, int32_t *out_pos,
                       float *out_scores, hipStream_t s);
int launch_fill_zero(void *p, size_t bytes, hipStream_t s);
// in place: n bf16 values -> the same values in IEEE half (exact for every bf16 value of normal half range)
int launch_bf16_to_f16(void *p, size_t n, hipStream_t s);

}  // namespace prism
