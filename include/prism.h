/*
 * prism.h - C ABI of the MI355X (gfx950) monolithic-forwarding reranker library.
 *
 * The library selects the top-K of N candidate documents for a query (paper Sec. 2.1,
 * problem statement) with ONE batched forward of a decoder-only cross-encoder over all
 * (query, candidate) sequences (Sec. 3.3, monolithic forwarding) and progressive cluster
 * pruning between layers (Sec. 4.1).  Every step runs in HIP kernels; the host side only
 * sequences launches and reads back the per-checkpoint keep mask.
 *
 * Conventions
 *   - Plain C types only.  Every pointer is tagged [host] or [device] below.
 *   - Matrices are row-major [out_features, in_features]; a projection is y = x W^T.
 *   - prism_model.dtype, PRISM_DTYPE_FP32 or PRISM_DTYPE_BF16, is the storage type of all weights.
 *     fp32 weights: every step in fp32.  bf16 weights: the operands of the matrix-core contractions
 *     (normalised GEMM inputs, q, k, v, attention output, SwiGLU output, and the layer weights) are
 *     16-bit, prism_options.operand says which 16-bit type; accumulation, softmax, norms and the
 *     residual stream are fp32.  IEEE half operands (the default) hold every bf16 weight exactly
 *     (down to 2^-17 in magnitude, below that to within 2^-25) and round activations 8x finer than
 *     bf16, at the same matrix-core rate; bf16 operands trade that precision for range.
 *   - All entry points return PRISM_OK (0) or a negative PRISM_E* code; nothing throws,
 *     aborts or exits; outputs are untouched on error (of a prism_report only n_events is defined then: 0; its
 *     arrays may hold events recorded before the failure).  prism_last_error() gives detail.
 *   - Conversions to IEEE half saturate at +-65504 (no infinity is ever produced, and nothing is counted or
 *     reported): the default half operands suit activations within that range - true of the synthetic N(0, 0.02)
 *     models here by orders of magnitude - and a model whose normalised inputs, q/k/v, attention output or SwiGLU output
 *     can exceed it should run with prism_options.operand = PRISM_DTYPE_BF16, which has fp32's range.
 *   - A context is single-caller.  Different contexts may run concurrently.
 */
#ifndef PRISM_H_
#define PRISM_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PRISM_OK            0
#define PRISM_EINVAL       (-1)  /* null / negative / zero-length input, token id out of range, K <= 0 */
#define PRISM_ECAP         (-2)  /* pool does not fit under hbm_cap_bytes even with chunking */
#define PRISM_EHIP         (-3)  /* a HIP call failed; see prism_last_error() */
#define PRISM_ENOMEM       (-4)  /* device or host allocation failed */
#define PRISM_EUNSUPPORTED (-5)  /* shape not supported by the kernels of the chosen dtype */

#define PRISM_DTYPE_FP32 0
#define PRISM_DTYPE_BF16 1
#define PRISM_DTYPE_F16  2  /* IEEE half: an operand type (prism_options.operand, kernel-level calls), not a weight type */

#define PRISM_MODE_DROP_ONLY  0  /* Sec. 7: only hopeless candidates are pruned; survivors reach full depth */
#define PRISM_MODE_THREE_WAY  1  /* Sec. 4.1: selected leave early, deferred continue, early termination */
#define PRISM_MODE_NO_PRUNING 2  /* plain full-depth forward of every candidate */

#define PRISM_MAX_CANDS    4096  /* candidates per call */
#define PRISM_MAX_CLUSTERS 8
#define PRISM_MAX_SEQ      8192  /* tokens per (query + candidate) sequence */
#define PRISM_N_KINDS      6     /* kernel kinds timed in prism_report */

/* fates written to prism_report.ev_fate (Sec. 4.1) */
#define PRISM_FATE_NOT_LIVE (-1)
#define PRISM_FATE_DROPPED    0
#define PRISM_FATE_DEFERRED   1
#define PRISM_FATE_SELECTED   2

typedef struct prism_ctx prism_ctx;

/* Layer weight formats.  W4G128 is this library's reading of the paper's 4-bit-weight / 16-bit-activation variant
 * (Sec. 6), which the paper names without detail: symmetric codes q in [-7, 7] for groups of 128 consecutive input
 * features of one output row, one bf16 scale per group (max|w| / 7 rounded to nearest even; 1 for an all-zero group),
 * q = w / scale rounded to nearest even and clamped; the weight used is q * scale, which is exact in IEEE half.
 * Blob of an [N, K] matrix (K % 128 == 0): N*K/2 code bytes, row-major, code k of a row in the low (k even) or high
 * (k odd) nibble of byte k/2, stored as q + 8; then N*K/128 bf16 scales, row-major. */
#define PRISM_WFMT_PLAIN  0
#define PRISM_WFMT_W4G128 1

/* Architecture of the reranker (decoder-only, causal; Sec. 2.1).  Sizes in elements. */
typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  float   rms_eps, rope_base;
  int32_t dtype;    /* PRISM_DTYPE_* */
  int32_t qk_norm;  /* 1: per-head RMSNorm on q and k (over head_dim) before RoPE */
} prism_model;

/* One transformer layer.  attn_norm, ffn_norm: [hidden]; wq: [n_q_heads*head_dim, hidden];
 * wk, wv: [n_kv_heads*head_dim, hidden]; q_norm, k_norm: [head_dim] (ignored if !qk_norm);
 * wo: [hidden, n_q_heads*head_dim]; w_gate, w_up: [ffn, hidden]; w_down: [hidden, ffn]. */
typedef struct {
  const void *attn_norm, *wq, *wk, *wv, *q_norm, *k_norm, *wo, *ffn_norm, *w_gate, *w_up, *w_down;
} prism_layer_weights;

typedef struct {
  const void *embed;                  /* [vocab, hidden]; [device] if embed_residency == 0, [pinned host] if 1 */
  const prism_layer_weights *layers;  /* [host] array of n_layers structs; the tensor pointers inside are
                                         [device] if layer_residency == 0, [pinned host] if 1 */
  const void *final_norm;             /* [device] [hidden] */
  const void *w_yes, *w_no;           /* [device] [hidden] each (a tied head points into embed rows, or at device
                                         copies of the two rows when the table stays on the host) */
  int32_t layer_residency;            /* 0: device; 1: pinned host, streamed one layer ahead (Sec. 4.2) */
  int32_t embed_residency;            /* 0: device; 1: pinned host (allocated by hipHostMalloc, so that kernels can read
                                         it), rows fetched on demand into a device LRU cache (Sec. 4.4) */
  int32_t layer_format;               /* PRISM_WFMT_PLAIN: tensors in the model dtype.  PRISM_WFMT_W4G128 (bf16 models):
                                         the seven matrices of a layer are 4-bit blobs as written by
                                         prism_op_quantize_w4 (the norm gains stay bf16); a layer is expanded into
                                         one of two device slots right before it runs, so device-resident blobs are
                                         borrowed in place for the context's lifetime, and streamed ones move a
                                         quarter of the bytes.  Needs hidden, ffn, n_q_heads*head_dim % 128 == 0 */
} prism_weights;

typedef struct {
  const int32_t *checkpoint_layers;   /* [host] 1-indexed: the check runs on the output of layer l, before l+1 */
  int32_t n_checkpoints;
  float   cv_threshold;               /* dispersion threshold tau (Sec. 4.1); gate opens iff std > tau*|mean| */
  int32_t n_clusters;                 /* k of the K-Means step, 2..PRISM_MAX_CLUSTERS; 0 -> 3 */
  int32_t mode;                       /* PRISM_MODE_* */
  int32_t chunk_cands;                /* Sec. 4.3 chunked execution: candidates per chunk; 0 = whole pool */
  int64_t hbm_cap_bytes;              /* cap on library-owned device memory; 0 = unlimited */
  void   *stream;                     /* hipStream_t of the caller, or NULL for a library-owned stream */
  int32_t operand;                    /* bf16 weights only: 0 or PRISM_DTYPE_F16 = IEEE half operands (default),
                                         PRISM_DTYPE_BF16 = bf16 operands */
  int32_t offload_hidden;             /* Sec. 4.3, second half: 1 = the residual stream of the whole pool lives in
                                         library-owned pinned host memory and at most three chunks of it are on the
                                         device (computing / being written back / being prefetched); needs chunk_cands > 0 */
  int32_t embed_cache_rows;           /* embed_residency == 1: rows of the device LRU cache; 0 -> vocab / 10 */
  int32_t stream_slots;               /* streamed or 4-bit layers: layer buffers in the ring, 0 or 2 = the paper's double
                                         buffer (Sec. 4.2); more lets the stream run ahead while the pool is large, which
                                         pays back after pruning, when a layer computes faster than it arrives */
  int32_t no_query_sharing;           /* 0 (default): the query's tokens, with which every (query, candidate) sequence
                                         begins (Sec. 3.3) and whose states under the causal mask do not depend on the
                                         candidate, are held and computed once per chunk, and every candidate's tokens
                                         attend to those rows; results are those of the unshared computation.  Applies
                                         to the 16-bit matrix-core path with a device-resident residual stream.
                                         1: every sequence carries and computes its own copy of the query */
  int32_t single_pass_checks;         /* 0 (default): a layer whose output is checked (Sec. 3.4) runs in two passes: first
                                         what the scores need (keys and values of every token; attention, O projection
                                         and FFN for each candidate's last token), then, after the decision, the rest of
                                         the layer for the survivors only.  Scores and results are those of the one-pass
                                         order.  Applies with a device-resident residual stream.
                                         1: the whole layer runs on every live candidate before the check */
} prism_options;

/* Optional per-call record.  The caller allocates every array ([host]); an "event" is one
 * scoring of the live set: each evaluated checkpoint plus the final scoring.  Rows of
 * ev_scores / ev_fate are indexed by ORIGINAL candidate index. */
typedef struct {
  int32_t  cap_events;      /* in: capacity of the ev_* arrays, in events (n_checkpoints + 1 suffices) */
  int32_t  n_cands;         /* in: row length of ev_scores / ev_fate (>= n_cands of the call) */
  int32_t  n_events;        /* out */
  int32_t *ev_layer;        /* out [cap_events] layer whose output was scored (n_layers = final) */
  int32_t *ev_n_before;     /* out [cap_events] live candidates scored */
  int32_t *ev_n_after;      /* out [cap_events] live candidates that continue */
  int32_t *ev_tokens_after; /* out [cap_events] live tokens that continue */
  int32_t *ev_gate;         /* out [cap_events] 1 if the dispersion gate fired */
  int32_t *ev_n_clusters;   /* out [cap_events] clusters used (0 if no clustering ran) */
  double  *ev_mean;         /* out [cap_events] mean of the live scores */
  double  *ev_std;          /* out [cap_events] population std of the live scores */
  float   *ev_scores;       /* out [cap_events * n_cands]; NaN where the candidate was not live */
  int8_t  *ev_fate;         /* out [cap_events * n_cands]; PRISM_FATE_* */
  double   ms_total;        /* out: GPU time of the call, first launch to last (HIP events) */
  double   ms_layers;       /* out: GPU time inside transformer layers */
  double   ms_checks;       /* out: GPU time in scoring + pruning + compaction */
  int64_t  token_layers;    /* out: sum over executed layers of live tokens */
  int64_t  peak_hbm_bytes;  /* out: library-owned device memory at its peak (what hbm_cap_bytes caps); the caller's own
                               device buffers - a device-resident embedding table, final_norm, the head rows - are
                               not in it */
  int64_t  bytes_streamed;  /* out: host->device weight bytes copied during the call */
  int32_t  layers_run;      /* out */
  /* out: per-kernel-kind totals over the call, from HIP events around each launch on the compute stream.
   * kinds: 0 fused QKV GEMM, 1 O-projection GEMM, 2 gate/up GEMM with SwiGLU, 3 down GEMM, 4 attention,
   * 5 the elementwise steps of a layer (RMSNorm, q/k norm + RoPE, V transposition where not fused) and the last layer's
 * one-row-per-candidate tail.
   * kind_flops is the ALGORITHMIC work: 2*M*N*K per GEMM (live tokens only), 2*nq*hd*L*(L+1) per sequence
   * of attention (causal triangle only); 0 for kind 5. */
  int32_t  kind_launches[PRISM_N_KINDS];
  double   kind_ms[PRISM_N_KINDS];
  double   kind_flops[PRISM_N_KINDS];
  int64_t  bytes_hidden_moved;  /* out: residual-stream bytes copied device->host and host->device (offload_hidden) */
  int64_t  embed_rows_hit;      /* out: token occurrences whose embedding row was in the device cache (embed_residency 1) */
  int64_t  embed_rows_missed;   /* out: token occurrences whose row was fetched from the host table during the call */
  /* Optional per-launch detail behind the kind_* totals, in launch order: the caller sets span_cap and the four arrays
   * ([host], span_cap entries each), or span_cap = 0 and NULL pointers.  rows = tokens (GEMM rows) the launch covered. */
  int32_t  span_cap;            /* in */
  int32_t  n_spans;             /* out: spans recorded (the first span_cap of the call) */
  int32_t *span_kind;           /* out */
  int32_t *span_rows;           /* out */
  float   *span_ms;             /* out */
  double  *span_flops;          /* out */
  /* in: which kinds get HIP-event spans (bit k = kind k); 0 means all.  Every span costs two event records on the
   * compute stream (about 3 ms per call at 36 layers with all kinds on), so a caller that times the call as a whole
   * can restrict the spans to the kinds it reads; the other kinds' totals then stay 0. */
  int32_t  kind_mask;
  /* out, only when kind_mask has PRISM_KIND_MASK_TRANSFERS set (it is not part of "0 means all"): time the side stream
   * spent moving streamed layer weights over the host link, summed over the layers, first copy start to last copy end
   * (HIP events on that stream); bytes_streamed / ms_transfers is the rate of the link while it is in use.  The records
   * behind the copies can delay compute kernels that share the side stream's hardware queue, so a call timed this way
   * is not the call to take the latency from.  0 otherwise. */
  double   ms_transfers;
} prism_report;
#define PRISM_KIND_MASK_TRANSFERS (1 << 8)

/* Build a context.  Device-resident layer weights are repacked once into library-owned HBM
 * (fused [wq;wk;wv] and [w_gate;w_up] operands): plain (not 4-bit) device-resident layer tensors are
 * not read again after prism_create returns, so a caller short of memory may release its own copies
 * then instead of holding the layers twice; pinned-host layer weights are borrowed and
 * read asynchronously by every prism_select, so they must stay mapped and unmodified until
 * prism_destroy.  embed, final_norm, w_yes, w_no are borrowed in place.  The option arrays
 * are copied. */
int prism_create(const prism_model *model, const prism_weights *weights, const prism_options *options,
                 prism_ctx **out_ctx);

/* Top-K selection (Sec. 2.1).  All pointers [host].  Sequence c is query ++ cand_tokens[c], positions
 * restart at 0 for every sequence.  out_idx / out_scores hold >= K entries; *out_count = min(K, n_cands).
 * Order: best first, ties by lower candidate index.  Synchronous: returns after the results are on the
 * host.  K >= n_cands disables pruning.  report may be NULL. */
int prism_select(prism_ctx *ctx, const int32_t *query_tokens, int32_t query_len,
                 const int32_t *const *cand_tokens, const int32_t *cand_lens, int32_t n_cands,
                 int32_t K, int32_t *out_idx, float *out_scores, int32_t *out_count,
                 prism_report *report);

/* Teacher forcing for parity tests: masks [host] is [n_events][n_cands] of 0/1 by ORIGINAL candidate index
 * (copied); at the e-th evaluated checkpoint the library still scores and routes, but keeps exactly the
 * candidates with mask 1 among the live ones.  NULL clears it. */
int prism_set_forced_keep(prism_ctx *ctx, const int8_t *masks, int32_t n_events, int32_t n_cands);

void prism_destroy(prism_ctx *ctx);
const char *prism_strerror(int code);
const char *prism_last_error(void);   /* thread-local detail of the last failure */

/* ------------------------------------------------------------------------------------------------
 * Kernel-level entry points: one call per step of the path, on caller-owned [device] buffers, on the
 * given hipStream_t (NULL = default stream).  They launch exactly the kernels prism_select uses and
 * return without synchronising unless stated.  Used by the parity tests and micro-benchmarks.
 * ------------------------------------------------------------------------------------------------ */

/* Pack + embed (Sec. 4.5: the forward begins at the embedding layer): X[t,:] = table[tokens[t],:] as fp32. */
int prism_op_embed(const int32_t *tokens, int32_t T, const void *table, int32_t hidden, int32_t dtype,
                   float *X, void *stream);

/* RMSNorm of the fp32 residual into the GEMM operand type (dtype FP32, BF16 or F16; gain in the same type): out[t,:] = X[t,:]/sqrt(mean(X[t,:]^2)+eps)*gain. */
int prism_op_rmsnorm(const float *X, const void *gain, int32_t T, int32_t hidden, float eps, int32_t dtype,
                     void *out, void *stream);

#define PRISM_EPI_STORE    0  /* C[M,N] (operand dtype) = A W^T */
#define PRISM_EPI_RESIDUAL 1  /* X[M,N] (fp32) += A W^T */
#define PRISM_EPI_SWIGLU   2  /* W is [2F,K] = [W_gate; W_up]; S[M,F] (operand dtype) = silu(A Wg^T) * (A Wu^T) */
#define PRISM_EPI_STORE_F32 3 /* C[M,N] (fp32) = A W^T: the q/k/v projection, normalised and rotated before rounding */
/* Layer contraction (Sec. 2.2: latency is dominated by the matrix multiplications of the blocks).
 * A [M,K], W [N,K] in dtype (FP32, BF16 or F16); N is the row count of W (2F for SWIGLU).  STORE_F32 exists for
 * the 16-bit types only (with FP32, STORE already writes fp32). */
int prism_op_gemm(int32_t dtype, int32_t epilogue, const void *A, const void *W, void *out,
                  int32_t M, int32_t N, int32_t K, void *stream);

/* Finishes the fused q/k/v projection QKV [T, (nq+2nkv)*hd] (fp32, [device]): per-head RMSNorm (optional,
 * over head_dim, gains q_gain / k_gain [head_dim]) then rotate-half RoPE (pair i with i + head_dim/2, angle
 * pos * rope_base^(-2i/head_dim)) on q and k.  pos[t] [device] is the position of token t in its sequence,
 * 0 <= pos[t] < max_pos <= PRISM_MAX_SEQ.
 *   fp32 mode: q and k are rewritten in place; QK and Vt are ignored (pass NULL).
 *   BF16 / F16: q and k go to QK [T, (nq+nkv)*hd] in that type; v is rounded to that type and written
 *     transposed to Vt [nkv][hd][vt_stride], always in IEEE half format (the operand type of the P V
 *     contraction; it holds bf16 values exactly) at column vt_col[t] [device].  The caller lays the sequences out so that
 *     each starts at a multiple of 64 columns, and zero-fills Vt once (pad columns must be finite).  For
 *     prism_op_attention, the token at position p of a sequence belongs at column
 *     first column + prism_vt_column_of_key(p): within every group of 16 positions the order is 0-3, 8-11, 4-7, 12-15,
 *     the order in which the matrix cores hand the attention weights to the P V contraction.
 * Synchronises the stream before returning. */
int32_t prism_vt_column_of_key(int32_t p);   /* p with bits 2 and 3 swapped; negative p is returned unchanged */
int prism_op_qkv_finish(int32_t dtype, void *QKV, const int32_t *pos, int32_t max_pos, const void *q_gain,
                        const void *k_gain, int32_t T, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                        float eps, float rope_base, int32_t qk_norm, void *QK, void *Vt, const int32_t *vt_col,
                        int64_t vt_stride, void *stream);

/* The fused form of prism_op_gemm (fp32 store) + prism_op_qkv_finish for the 16-bit modes, which is what prism_select
 * runs whenever it applies: [Q|K|V] = Xn Wqkv^T with Xn [T, hidden] and Wqkv [(nq+2nkv)*hd, hidden] ([device], dtype),
 * then per-head RMSNorm (optional) and RoPE on q and k and the transposed half-precision V, all applied to the fp32
 * accumulators in the GEMM's epilogue (one rounding, no fp32 intermediate in memory).  Outputs, pos, vt_col, gains as
 * in prism_op_qkv_finish.  Needs head_dim == 128, hidden % 64 == 0 and ceil(T / 256) * (nq + 2 nkv) / 2 >= 256 (one
 * head per wavefront of a 256 x 256 tile, enough tiles to fill the chip); PRISM_EUNSUPPORTED otherwise.
 * Synchronises the stream before returning. */
int prism_op_qkv_project(int32_t dtype, const void *Xn, const void *Wqkv, const int32_t *pos, int32_t max_pos,
                         const void *q_gain, const void *k_gain, int32_t T, int32_t hidden, int32_t n_q_heads,
                         int32_t n_kv_heads, int32_t head_dim, float eps, float rope_base, int32_t qk_norm,
                         void *QK, void *Vt, const int32_t *vt_col, int64_t vt_stride, void *stream);

/* 4-bit weight blobs (PRISM_WFMT_W4G128).  prism_w4_bytes: size of the blob of an [N, K] matrix.
 * prism_op_quantize_w4: W [N, K] bf16 [device] -> blob [device].  prism_op_dequantize_w4: blob -> out [N, K] [device] in
 * dtype BF16 or F16 (what a layer slot holds before the layer runs). */
int64_t prism_w4_bytes(int32_t N, int32_t K);
int prism_op_quantize_w4(const void *W, int32_t N, int32_t K, void *blob, void *stream);
int prism_op_dequantize_w4(const void *blob, int32_t N, int32_t K, int32_t dtype, void *out, void *stream);

/* Causal GQA attention within each sequence (no token attends across sequences; Sec. 2.2).
 * cu_seqlens [n_seqs+1] [host]: token offsets of the sequences; out [T, nq*hd] [device] in dtype.
 *   fp32 mode: QK = the finished QKV buffer [T, (nq+2nkv)*hd] (fp32); Vt, vt_col0 ignored.
 *   BF16 / F16: QK [T, (nq+nkv)*hd] in that type and Vt / vt_stride as written by prism_op_qkv_finish;
 *     vt_col0 [n_seqs] [host]: first Vt column of each sequence (multiples of 64); the key at position p of sequence
 *     i is read from column vt_col0[i] + prism_vt_column_of_key(p).
 * Synchronises the stream before returning. */
int prism_op_attention(int32_t dtype, const void *QK, const void *Vt, int64_t vt_stride,
                       const int32_t *cu_seqlens_host, const int32_t *vt_col0_host, int32_t n_seqs,
                       int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, void *out, void *stream);

/* Intermediate scorer (Sec. 4.1): for each sequence c, the last token's state through the final RMSNorm and
 * the yes/no head: scores[c] = z . w_yes - z . w_no.  last_row[c] = row of that token in X (NULL: row c). */
int prism_op_score(const float *X, const int32_t *last_row, int32_t n_seqs, int32_t hidden,
                   const void *final_norm, const void *w_yes, const void *w_no, int32_t dtype, float eps,
                   float *scores, void *stream);

/* One pruning check (Sec. 4.1): dispersion gate, exact 1-D K-Means, boundary-cluster routing.
 * scores [n] fp32 in, fate [n] int8 out (PRISM_FATE_*), stats [4] double out = {mean, std, gate, n_clusters}.
 * With n <= K_rem, a closed gate or a single distinct score every fate is DEFERRED.  All pointers [device].
 * Synchronises the stream before returning. */
int prism_op_route(const float *scores, int32_t n, int32_t K_rem, int32_t n_clusters, float tau,
                   int8_t *fate, double *stats, void *stream);

/* prism_op_route for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernel, same results as prism_op_route; the kernel's workspace
 * (328 192 bytes, enough for n = PRISM_MAX_CANDS and n_clusters = PRISM_MAX_CLUSTERS; larger requests are rejected with
 * PRISM_EINVAL) is a static device array of the library, one copy per device, held until the process ends.  The call
 * allocates and frees nothing and does NOT synchronise: fate and stats are ready when `stream` has drained.  Every
 * call on a device uses that device's one workspace, so calls that overlap on a device (different streams or threads)
 * race; the kernel overwrites every workspace entry before reading it, so consecutive calls need no clearing. */
int prism_op_route_static(const float *scores, int32_t n, int32_t K_rem, int32_t n_clusters, float tau,
                          int8_t *fate, double *stats, void *stream);

/* Stream compaction of the packed residual (Sec. 4.1: continue only on the remaining candidates):
 * rows [src_start[c], src_start[c]+len[c]) of X_src go to rows starting at dst_start[c] of X_dst for
 * each of the n_keep kept sequences; the arrays are [device]; X_dst must not alias X_src. */
int prism_op_compact(const float *X_src, float *X_dst, const int32_t *src_start, const int32_t *dst_start,
                     const int32_t *len, int32_t n_keep, int32_t hidden, void *stream);

/* Final top-K (Sec. 2.1): ranks n scores (descending, ties by lower position) and writes the first K
 * positions and scores. */
int prism_op_topk(const float *scores, int32_t n, int32_t K, int32_t *out_pos, float *out_scores, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PRISM_H_ */
