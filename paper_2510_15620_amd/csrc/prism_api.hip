// Host orchestrator and C ABI: the layer loop of monolithic forwarding (paper Sec. 3.3), the pruning
// checkpoints between layers (Sec. 3.4, 4.1), chunked execution within a layer (Sec. 4.3) and
// overlapped layer streaming from pinned host memory on a side stream (Sec. 4.2).
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <limits>
#include <new>
#include <string>
#include <vector>

#include "common.h"

namespace prism {

// ------------------------------------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int hip_fail(hipError_t e, const char *what, const char *file, int line) {
  set_error("HIP error %d (%s) in %s at %s:%d", (int)e, hipGetErrorString(e), what, file, line);
  return e == hipErrorOutOfMemory ? PRISM_ENOMEM : PRISM_EHIP;
}

// ------------------------------------------------------------------------------------------------ layer layout
// One layer's operands in one contiguous device buffer, so that a streamed layer is a handful of
// copies into a slot and the fused operands [wq;wk;wv] and [w_gate;w_up] come for free.
struct LayerLayout {
  size_t attn_norm, wqkv, wk, wv, q_norm, k_norm, wo, ffn_norm, wgu, wu, wd, bytes;
};

static LayerLayout make_layout(const prism_model &m) {
  const size_t e = dtype_size(m.dtype);
  const size_t H = m.hidden, Dq = (size_t)m.n_q_heads * m.head_dim, Dkv = (size_t)m.n_kv_heads * m.head_dim, F = m.ffn;
  LayerLayout L;
  size_t o = 0;
  auto take = [&](size_t elems) { size_t at = o; o = (size_t)round_up(o + elems * e, 256); return at; };
  L.attn_norm = take(H);
  L.wqkv = take((Dq + 2 * Dkv) * H);
  L.wk = L.wqkv + Dq * H * e;
  L.wv = L.wk + Dkv * H * e;
  L.q_norm = take(m.head_dim);
  L.k_norm = take(m.head_dim);
  L.wo = take(H * Dq);
  L.ffn_norm = take(H);
  L.wgu = take(2 * F * H);
  L.wu = L.wgu + F * H * e;
  L.wd = take(H * F);
  L.bytes = o;
  return L;
}

struct CopyItem { size_t dst_off; const void *src; size_t bytes; int64_t N, K; /* K = 0: a vector of N elements */ };

static void layer_copy_items(const prism_model &m, const LayerLayout &L, const prism_layer_weights &w,
                             std::vector<CopyItem> &items) {
  const size_t e = dtype_size(m.dtype);
  const size_t H = m.hidden, Dq = (size_t)m.n_q_heads * m.head_dim, Dkv = (size_t)m.n_kv_heads * m.head_dim, F = m.ffn;
  items.clear();
  const int64_t hd = m.head_dim;
  items.push_back({L.attn_norm, w.attn_norm, H * e, (int64_t)H, 0});
  items.push_back({L.wqkv, w.wq, Dq * H * e, (int64_t)Dq, (int64_t)H});
  items.push_back({L.wk, w.wk, Dkv * H * e, (int64_t)Dkv, (int64_t)H});
  items.push_back({L.wv, w.wv, Dkv * H * e, (int64_t)Dkv, (int64_t)H});
  if (m.qk_norm) {
    items.push_back({L.q_norm, w.q_norm, (size_t)hd * e, hd, 0});
    items.push_back({L.k_norm, w.k_norm, (size_t)hd * e, hd, 0});
  }
  items.push_back({L.wo, w.wo, H * Dq * e, (int64_t)H, (int64_t)Dq});
  items.push_back({L.ffn_norm, w.ffn_norm, H * e, (int64_t)H, 0});
  items.push_back({L.wgu, w.w_gate, F * H * e, (int64_t)F, (int64_t)H});
  items.push_back({L.wu, w.w_up, F * H * e, (int64_t)F, (int64_t)H});
  items.push_back({L.wd, w.w_down, H * F * e, (int64_t)H, (int64_t)F});
}

}  // namespace prism

using namespace prism;

// ------------------------------------------------------------------------------------------------ context
struct prism_ctx {
  prism_model m;
  prism_options opt;
  int op = PRISM_DTYPE_FP32;                      // operand type of the contractions: FP32, BF16 or F16
  std::vector<int32_t> checkpoints;
  LayerLayout lay;
  const void *embed = nullptr, *final_norm = nullptr, *w_yes = nullptr, *w_no = nullptr;
  bool streamed = false;                          // layer weights arrive from pinned host memory during every call
  bool w4 = false;                                // layer matrices are 4-bit blobs, expanded into a slot right before use
  bool two_slot = false;                          // streamed or w4: two layer slots, layer l + 2 prepared while l + 1 computes
  std::vector<char *> packed_buf;                 // streamed + w4: landing buffers of the 4-bit layers (2)
  size_t packed_bytes = 0;
  std::vector<prism_layer_weights> host_layers;   // the caller's tensors (pinned host when streamed)
  std::vector<char *> layer_buf;                  // n_layers slots (resident) or 2 (streamed)
  hipStream_t stream = nullptr, copy_stream = nullptr;
  bool own_stream = false;
  int ring = 2;                                   // layer slots of the streaming ring (two_slot); 2 is the paper's double buffer
  std::vector<hipEvent_t> ev_ready, ev_free;      // per ring slot
  hipEvent_t ev_t[4] = {nullptr, nullptr, nullptr, nullptr};
  std::vector<hipEvent_t> ev_layer;               // 4 per layer (two intervals: a layer may run in two passes), for the report
  std::vector<hipEvent_t> ev_xfer;                // 2 per layer on the side stream around a streamed layer's transfers, for the report
  // per-launch spans for the report: events come from a pool that only grows
  struct Span { int kind; hipEvent_t a, b; double flops; int rows; };
  std::vector<hipEvent_t> ev_pool; size_t ev_used = 0;
  std::vector<Span> spans;
  bool profiling = false;
  int span_mask = ~0;                             // kinds that get event spans while profiling
  float2 *rope_tab = nullptr, *rope_tab_t = nullptr;   // [pos][i] for the stand-alone finishing kernel, [i][pos] for the fused epilogue

  // scratch, grown on demand
  float *X[2] = {nullptr, nullptr};
  int64_t x_cap[2] = {0, 0};                      // tokens
  char *Xn = nullptr, *QKV = nullptr, *QK = nullptr, *Vt = nullptr, *AO = nullptr, *S = nullptr;
  // last layer: only the last token of a sequence is ever looked at again, so everything after the attention runs on
  // one row per candidate
  char *AOl = nullptr, *Xnl = nullptr, *Sl = nullptr; float *Xl = nullptr; int64_t last_cap = 0;   // candidates
  int64_t chunk_cap = 0, vt_cap = 0;              // tokens / V^T columns
  int32_t *d_meta = nullptr; int64_t meta_cap = 0;   // int32 words
  int32_t *h_meta = nullptr; int64_t h_meta_cap = 0; // pinned staging
  float *d_scores = nullptr; int8_t *d_fate = nullptr; double *d_stats = nullptr; void *route_ws = nullptr;
  int32_t *d_top_pos = nullptr; float *d_top_scores = nullptr;
  char *h_res = nullptr;                          // pinned: scores, fate, stats, topk
  std::vector<int8_t> forced; int forced_events = 0, forced_cands = 0;
  int64_t bytes_now = 0, bytes_peak = 0;

  // hidden-state offload (Sec. 4.3): the residual stream of the whole pool in pinned host memory, three chunk-sized
  // device slots: one computing, one being written back, one being prefetched
  bool offload = false;
  float *Xo[3] = {nullptr, nullptr, nullptr};
  int64_t xo_cap = 0;                             // tokens per slot
  float *h_X = nullptr; int64_t hx_cap = 0;       // pinned, tokens
  std::vector<int64_t> hrow;                      // first row in h_X of every ORIGINAL candidate
  hipStream_t xin_stream = nullptr, xout_stream = nullptr;
  hipEvent_t ev_in[3] = {nullptr, nullptr, nullptr}, ev_done[3] = {nullptr, nullptr, nullptr}, ev_out[3] = {nullptr, nullptr, nullptr};
  int64_t ostep = 0;                              // pipeline step = chunk visits so far; slot = ostep % 3
  bool primed = false;                            // the next step's prefetch has been issued
  int64_t bytes_hidden = 0;

  // embedding-table cache (Sec. 4.4): table in pinned host memory, least-recently-used rows on the device
  bool embed_cached = false;
  const void *embed_dev_alias = nullptr;          // device-visible address of the pinned table
  int cache_rows = 0;
  char *d_cache = nullptr;                        // [cache_rows, hidden] in the model dtype
  std::vector<int32_t> slot_of, tok_of, lru_prev, lru_next;   // token -> slot, slot -> token, recency list
  int lru_head = -1, lru_tail = -1;               // most / least recently used slot
  std::vector<int64_t> pin;                       // slot -> pass that last touched it
  int64_t pass_id = 0;
  int32_t *h_estage = nullptr, *d_estage = nullptr; int64_t estage_cap = 0, h_estage_cap = 0;   // [slot per row | miss tokens | miss slots]
  int64_t embed_hit = 0, embed_miss = 0;
};

namespace prism {

static int dev_alloc(prism_ctx *c, void **p, size_t bytes) {
  bytes = (size_t)round_up(bytes ? bytes : 256, 256);
  if (c->opt.hbm_cap_bytes > 0 && c->bytes_now + (int64_t)bytes > c->opt.hbm_cap_bytes) {
    set_error("device memory cap: %lld bytes in use + %zu requested exceeds hbm_cap_bytes = %lld",
              (long long)c->bytes_now, bytes, (long long)c->opt.hbm_cap_bytes);
    return PRISM_ECAP;
  }
  hipError_t e = hipMalloc(p, bytes);
  if (e != hipSuccess) { *p = nullptr; return hip_fail(e, "hipMalloc", __FILE__, __LINE__); }
  c->bytes_now += bytes;
  c->bytes_peak = std::max(c->bytes_peak, c->bytes_now);
  return PRISM_OK;
}

static void dev_free(prism_ctx *c, void *p, size_t bytes) {
  if (!p) return;
  (void)hipFree(p);
  c->bytes_now -= (int64_t)round_up(bytes ? bytes : 256, 256);
}

template <typename T>
static int grow(prism_ctx *c, T **p, int64_t *cap, int64_t need, size_t unit) {
  if (need <= *cap) return PRISM_OK;
  if (*p) { PRISM_HIP(hipStreamSynchronize(c->stream)); dev_free(c, *p, (size_t)*cap * unit); *p = nullptr; *cap = 0; }
  void *q = nullptr;
  PRISM_TRY(dev_alloc(c, &q, (size_t)need * unit));
  *p = (T *)q;
  *cap = need;
  return PRISM_OK;
}

static int validate_model(const prism_model *m) {
  PRISM_REQUIRE(m->n_layers > 0 && m->hidden > 0 && m->n_q_heads > 0 && m->n_kv_heads > 0 && m->head_dim > 0 &&
                    m->ffn > 0 && m->vocab > 0,
                PRISM_EINVAL, "model: sizes must be positive");
  PRISM_REQUIRE(m->n_q_heads % m->n_kv_heads == 0, PRISM_EINVAL, "model: n_q_heads must be a multiple of n_kv_heads");
  PRISM_REQUIRE(m->head_dim % 2 == 0 && m->hidden % 4 == 0, PRISM_EINVAL, "model: head_dim must be even, hidden a multiple of 4");
  PRISM_REQUIRE(m->dtype == PRISM_DTYPE_FP32 || m->dtype == PRISM_DTYPE_BF16, PRISM_EINVAL, "model: unknown dtype %d", m->dtype);
  PRISM_REQUIRE(m->rms_eps >= 0.f && m->rope_base > 0.f, PRISM_EINVAL, "model: rms_eps / rope_base out of range");
  if (m->dtype == PRISM_DTYPE_BF16) {
    const int Dq = m->n_q_heads * m->head_dim, Dkv = m->n_kv_heads * m->head_dim;
    PRISM_REQUIRE(attention_16_supported(m->n_q_heads, m->n_kv_heads, m->head_dim), PRISM_EUNSUPPORTED,
                  "bf16 mode needs head_dim 128 and 1, 2, 4 or 8 query heads per KV head");
    PRISM_REQUIRE(gemm_16_supported(PRISM_EPI_STORE, Dq + 2 * Dkv, m->hidden) &&
                      gemm_16_supported(PRISM_EPI_RESIDUAL, m->hidden, Dq) &&
                      gemm_16_supported(PRISM_EPI_SWIGLU, 2 * m->ffn, m->hidden) &&
                      gemm_16_supported(PRISM_EPI_RESIDUAL, m->hidden, m->ffn),
                  PRISM_EUNSUPPORTED, "bf16 mode needs hidden, n_q_heads*head_dim and ffn to be multiples of 64");
    PRISM_REQUIRE(m->hidden % 8 == 0 && m->ffn % 8 == 0, PRISM_EUNSUPPORTED, "bf16 mode: rows must be 16-byte aligned");
  }
  return PRISM_OK;
}

static size_t packed_layer_bytes(const prism_model &m, const LayerLayout &L, const prism_layer_weights &w) {
  std::vector<CopyItem> items;
  layer_copy_items(m, L, w, items);
  size_t b = 0;
  for (const CopyItem &it : items) b += (size_t)round_up(it.K ? w4_blob_bytes(it.N, it.K) : it.N * 2, 256);
  return b;
}

// Fills layer slot `slot` with layer `layer` on stream s, in two parts that can be issued apart.  kLayerTransfer: what
// crosses the host link (pinned host to device when streamed; device to device at create; nothing for resident 4-bit
// blobs).  kLayerFinish: the kernels that turn what arrived into operands - bf16 -> half in place if the operands are
// half; 4-bit blobs expanded into the slot, the norm gains converted beside them.
enum { kLayerTransfer = 1, kLayerFinish = 2, kLayerBoth = 3 };
static int issue_layer_copy(prism_ctx *c, int layer, int slot, hipStream_t s, hipMemcpyKind kind, int64_t *bytes, int parts = kLayerBoth) {
  std::vector<CopyItem> items;
  layer_copy_items(c->m, c->lay, c->host_layers[layer], items);
  if (c->w4) {
    size_t poff = 0;
    for (const CopyItem &it : items) {
      const size_t sb = it.K ? (size_t)w4_blob_bytes(it.N, it.K) : (size_t)it.N * 2;
      const void *src = it.src;
      if (c->streamed) {
        char *land = c->packed_buf[slot] + poff;
        if (parts & kLayerTransfer) {
          PRISM_HIP(hipMemcpyAsync(land, it.src, sb, hipMemcpyHostToDevice, s));
          if (bytes) *bytes += (int64_t)sb;
        }
        src = land;
        poff += (size_t)round_up(sb, 256);
      }
      if (!(parts & kLayerFinish)) continue;
      if (it.K) PRISM_TRY(launch_dequantize_w4(src, (int)it.N, (int)it.K, c->op, c->layer_buf[slot] + it.dst_off, s));
      else PRISM_TRY(launch_convert_bf16(src, it.N, c->op, c->layer_buf[slot] + it.dst_off, s));
    }
    return PRISM_OK;
  }
  if (parts & kLayerTransfer)
    for (const CopyItem &it : items) {
      PRISM_HIP(hipMemcpyAsync(c->layer_buf[slot] + it.dst_off, it.src, it.bytes, kind, s));
      if (bytes) *bytes += (int64_t)it.bytes;
    }
  // half operands: the bf16 weights become the same numbers in IEEE half, in place, on the same stream
  if ((parts & kLayerFinish) && c->op == PRISM_DTYPE_F16) PRISM_TRY(launch_bf16_to_f16(c->layer_buf[slot], c->lay.bytes / 2, s));
  return PRISM_OK;
}

}  // namespace prism

// ------------------------------------------------------------------------------------------------ create / destroy
extern "C" int prism_create(const prism_model *model, const prism_weights *weights, const prism_options *options,
                            prism_ctx **out_ctx) {
  PRISM_REQUIRE(model && weights && options && out_ctx, PRISM_EINVAL, "prism_create: null argument");
  PRISM_TRY(validate_model(model));
  PRISM_REQUIRE(weights->embed && weights->layers && weights->final_norm && weights->w_yes && weights->w_no,
                PRISM_EINVAL, "prism_create: null weight pointer");
  PRISM_REQUIRE(weights->layer_residency == 0 || weights->layer_residency == 1, PRISM_EINVAL, "prism_create: layer_residency");
  PRISM_REQUIRE(options->n_checkpoints >= 0 && (options->n_checkpoints == 0 || options->checkpoint_layers),
                PRISM_EINVAL, "prism_create: checkpoint list");
  PRISM_REQUIRE(options->mode >= 0 && options->mode <= 2, PRISM_EINVAL, "prism_create: mode %d", options->mode);
  PRISM_REQUIRE(options->cv_threshold >= 0.f, PRISM_EINVAL, "prism_create: cv_threshold must be >= 0");
  PRISM_REQUIRE(options->n_clusters == 0 || (options->n_clusters >= 2 && options->n_clusters <= PRISM_MAX_CLUSTERS),
                PRISM_EINVAL, "prism_create: n_clusters %d outside 2..%d", options->n_clusters, PRISM_MAX_CLUSTERS);
  PRISM_REQUIRE(options->chunk_cands >= 0 && options->hbm_cap_bytes >= 0, PRISM_EINVAL, "prism_create: negative option");
  PRISM_REQUIRE(options->operand == 0 || options->operand == PRISM_DTYPE_F16 || options->operand == PRISM_DTYPE_BF16,
                PRISM_EINVAL, "prism_create: operand must be 0, PRISM_DTYPE_F16 or PRISM_DTYPE_BF16");
  PRISM_REQUIRE(weights->embed_residency == 0 || weights->embed_residency == 1, PRISM_EINVAL, "prism_create: embed_residency");
  PRISM_REQUIRE(weights->layer_format == PRISM_WFMT_PLAIN || weights->layer_format == PRISM_WFMT_W4G128, PRISM_EINVAL,
                "prism_create: layer_format");
  if (weights->layer_format == PRISM_WFMT_W4G128) {
    PRISM_REQUIRE(model->dtype == PRISM_DTYPE_BF16, PRISM_EUNSUPPORTED, "prism_create: 4-bit layer weights need the bf16 model type");
    PRISM_REQUIRE(model->hidden % 128 == 0 && model->ffn % 128 == 0 && (model->n_q_heads * model->head_dim) % 128 == 0,
                  PRISM_EUNSUPPORTED, "prism_create: 4-bit layer weights need hidden, ffn and n_q_heads*head_dim to be multiples of 128");
  }
  PRISM_REQUIRE(options->offload_hidden == 0 || options->offload_hidden == 1, PRISM_EINVAL, "prism_create: offload_hidden");
  PRISM_REQUIRE(!options->offload_hidden || options->chunk_cands > 0, PRISM_EINVAL,
                "prism_create: offload_hidden needs chunked execution (chunk_cands > 0)");
  PRISM_REQUIRE(options->embed_cache_rows >= 0, PRISM_EINVAL, "prism_create: embed_cache_rows");
  PRISM_REQUIRE(options->stream_slots >= 0, PRISM_EINVAL, "prism_create: stream_slots");
  const void *embed_alias = nullptr;
  if (weights->embed_residency == 1) {
    // kernels read the table in place, so it has to be pinned memory that is mapped into the device's address space
    hipPointerAttribute_t at;
    hipError_t pe = hipPointerGetAttributes(&at, weights->embed);
    if (pe != hipSuccess) (void)hipGetLastError();
    PRISM_REQUIRE(pe == hipSuccess && at.type == hipMemoryTypeHost, PRISM_EINVAL,
                  "prism_create: embed_residency = 1 needs a table in pinned host memory (hipHostMalloc)");
    void *dp = nullptr;
    pe = hipHostGetDevicePointer(&dp, const_cast<void *>(weights->embed), 0);
    if (pe != hipSuccess) (void)hipGetLastError();
    PRISM_REQUIRE(pe == hipSuccess && dp, PRISM_EINVAL, "prism_create: the pinned embedding table is not mapped for the device");
    embed_alias = dp;
    for (const void *hp : {weights->w_yes, weights->w_no}) {
      pe = hipPointerGetAttributes(&at, hp);
      if (pe != hipSuccess) (void)hipGetLastError();
      PRISM_REQUIRE(pe == hipSuccess && at.type == hipMemoryTypeDevice, PRISM_EINVAL,
                    "prism_create: w_yes / w_no must be device memory when the embedding table stays on the host");
    }
  }
  for (int l = 0; l < model->n_layers; ++l) {
    const prism_layer_weights &w = weights->layers[l];
    PRISM_REQUIRE(w.attn_norm && w.wq && w.wk && w.wv && w.wo && w.ffn_norm && w.w_gate && w.w_up && w.w_down &&
                      (!model->qk_norm || (w.q_norm && w.k_norm)),
                  PRISM_EINVAL, "prism_create: null tensor in layer %d", l);
  }
  for (int i = 0; i < options->n_checkpoints; ++i)
    PRISM_REQUIRE(options->checkpoint_layers[i] >= 1 && options->checkpoint_layers[i] <= model->n_layers, PRISM_EINVAL,
                  "prism_create: checkpoint layer %d outside 1..%d", options->checkpoint_layers[i], model->n_layers);

  prism_ctx *c = new (std::nothrow) prism_ctx();
  PRISM_REQUIRE(c, PRISM_ENOMEM, "prism_create: out of host memory");
  c->m = *model;
  c->opt = *options;
  if (c->opt.n_clusters == 0) c->opt.n_clusters = 3;
  c->checkpoints.assign(options->checkpoint_layers, options->checkpoint_layers + options->n_checkpoints);
  std::sort(c->checkpoints.begin(), c->checkpoints.end());
  c->checkpoints.erase(std::unique(c->checkpoints.begin(), c->checkpoints.end()), c->checkpoints.end());
  c->opt.checkpoint_layers = nullptr;
  c->op = model->dtype == PRISM_DTYPE_FP32 ? PRISM_DTYPE_FP32
                                            : (options->operand == PRISM_DTYPE_BF16 ? PRISM_DTYPE_BF16 : PRISM_DTYPE_F16);
  c->lay = make_layout(*model);
  c->embed = weights->embed; c->final_norm = weights->final_norm; c->w_yes = weights->w_yes; c->w_no = weights->w_no;
  c->streamed = weights->layer_residency == 1;
  c->w4 = weights->layer_format == PRISM_WFMT_W4G128;
  c->two_slot = c->streamed || c->w4;
  c->host_layers.assign(weights->layers, weights->layers + model->n_layers);
  c->offload = options->offload_hidden == 1;
  c->embed_cached = weights->embed_residency == 1;
  c->embed_dev_alias = embed_alias;

  auto fail = [&](int rc) { prism_destroy(c); return rc; };
#define CREATE_TRY(x) do { int rc__ = (x); if (rc__ != PRISM_OK) return fail(rc__); } while (0)
#define CREATE_HIP(x) do { hipError_t e__ = (x); if (e__ != hipSuccess) return fail(hip_fail(e__, #x, __FILE__, __LINE__)); } while (0)
  if (options->stream) c->stream = (hipStream_t)options->stream;
  else { CREATE_HIP(hipStreamCreateWithFlags(&c->stream, hipStreamNonBlocking)); c->own_stream = true; }
  CREATE_HIP(hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking));
  c->ring = std::min(std::max(options->stream_slots, 2), model->n_layers > 1 ? model->n_layers : 2);
  c->ev_ready.assign(c->ring, nullptr);
  c->ev_free.assign(c->ring, nullptr);
  for (int i = 0; i < c->ring; ++i) {
    CREATE_HIP(hipEventCreateWithFlags(&c->ev_ready[i], hipEventDisableTiming));
    CREATE_HIP(hipEventCreateWithFlags(&c->ev_free[i], hipEventDisableTiming));
  }
  for (int i = 0; i < 4; ++i) CREATE_HIP(hipEventCreate(&c->ev_t[i]));

  const int n_slots = c->two_slot ? std::min(c->ring, model->n_layers) : model->n_layers;
  c->layer_buf.assign(n_slots, nullptr);
  for (int s = 0; s < n_slots; ++s) CREATE_TRY(dev_alloc(c, (void **)&c->layer_buf[s], c->lay.bytes));
  if (c->w4 && c->streamed) {
    c->packed_bytes = packed_layer_bytes(*model, c->lay, c->host_layers[0]);
    c->packed_buf.assign(n_slots, nullptr);
    for (int s = 0; s < n_slots; ++s) CREATE_TRY(dev_alloc(c, (void **)&c->packed_buf[s], c->packed_bytes));
  }
  if (!c->two_slot) {
    for (int l = 0; l < model->n_layers; ++l) CREATE_TRY(issue_layer_copy(c, l, l, c->stream, hipMemcpyDeviceToDevice, nullptr));
  }
  CREATE_TRY(dev_alloc(c, (void **)&c->rope_tab, (size_t)PRISM_MAX_SEQ * (model->head_dim / 2) * sizeof(float2)));
  CREATE_TRY(launch_rope_table(c->rope_tab, PRISM_MAX_SEQ, model->head_dim, model->rope_base, c->stream));
  CREATE_TRY(dev_alloc(c, (void **)&c->rope_tab_t, (size_t)PRISM_MAX_SEQ * (model->head_dim / 2) * sizeof(float2)));
  CREATE_TRY(launch_rope_table(c->rope_tab_t, PRISM_MAX_SEQ, model->head_dim, model->rope_base, c->stream, true));
  CREATE_TRY(dev_alloc(c, (void **)&c->d_scores, PRISM_MAX_CANDS * sizeof(float)));
  CREATE_TRY(dev_alloc(c, (void **)&c->d_fate, PRISM_MAX_CANDS));
  CREATE_TRY(dev_alloc(c, (void **)&c->d_stats, 4 * sizeof(double)));
  CREATE_TRY(dev_alloc(c, &c->route_ws, route_workspace_bytes(PRISM_MAX_CANDS, PRISM_MAX_CLUSTERS)));
  CREATE_TRY(dev_alloc(c, (void **)&c->d_top_pos, PRISM_MAX_CANDS * sizeof(int32_t)));
  CREATE_TRY(dev_alloc(c, (void **)&c->d_top_scores, PRISM_MAX_CANDS * sizeof(float)));
  CREATE_HIP(hipHostMalloc((void **)&c->h_res, PRISM_MAX_CANDS * 16 + 256, hipHostMallocDefault));
  if (c->offload) {
    CREATE_HIP(hipStreamCreateWithFlags(&c->xin_stream, hipStreamNonBlocking));
    CREATE_HIP(hipStreamCreateWithFlags(&c->xout_stream, hipStreamNonBlocking));
    for (int i = 0; i < 3; ++i) {
      CREATE_HIP(hipEventCreateWithFlags(&c->ev_in[i], hipEventDisableTiming));
      CREATE_HIP(hipEventCreateWithFlags(&c->ev_done[i], hipEventDisableTiming));
      CREATE_HIP(hipEventCreateWithFlags(&c->ev_out[i], hipEventDisableTiming));
    }
  }
  if (c->embed_cached) {
    c->cache_rows = options->embed_cache_rows > 0 ? std::min(options->embed_cache_rows, model->vocab) : std::max(model->vocab / 10, 1);
    CREATE_TRY(dev_alloc(c, (void **)&c->d_cache, (size_t)c->cache_rows * model->hidden * dtype_size(model->dtype)));
    c->slot_of.assign(model->vocab, -1);
    c->tok_of.assign(c->cache_rows, -1);
    c->pin.assign(c->cache_rows, -1);
    c->lru_prev.resize(c->cache_rows);
    c->lru_next.resize(c->cache_rows);
    for (int i = 0; i < c->cache_rows; ++i) { c->lru_prev[i] = i - 1; c->lru_next[i] = i + 1 < c->cache_rows ? i + 1 : -1; }
    c->lru_head = 0;
    c->lru_tail = c->cache_rows - 1;
  }
  CREATE_HIP(hipStreamSynchronize(c->stream));
#undef CREATE_TRY
#undef CREATE_HIP
  *out_ctx = c;
  return PRISM_OK;
}

extern "C" void prism_destroy(prism_ctx *c) {
  if (!c) return;
  if (c->stream) (void)hipStreamSynchronize(c->stream);
  if (c->copy_stream) (void)hipStreamSynchronize(c->copy_stream);
  if (c->xin_stream) (void)hipStreamSynchronize(c->xin_stream);
  if (c->xout_stream) (void)hipStreamSynchronize(c->xout_stream);
  for (char *p : c->layer_buf) if (p) (void)hipFree(p);
  for (char *p : c->packed_buf) if (p) (void)hipFree(p);
  for (void *p : {(void *)c->Xo[0], (void *)c->Xo[1], (void *)c->Xo[2], (void *)c->d_cache, (void *)c->d_estage}) if (p) (void)hipFree(p);
  if (c->h_X) (void)hipHostFree(c->h_X);
  if (c->h_estage) (void)hipHostFree(c->h_estage);
  for (int i = 0; i < 3; ++i)
    for (hipEvent_t e : {c->ev_in[i], c->ev_done[i], c->ev_out[i]}) if (e) (void)hipEventDestroy(e);
  if (c->xin_stream) (void)hipStreamDestroy(c->xin_stream);
  if (c->xout_stream) (void)hipStreamDestroy(c->xout_stream);
  void *ptrs[] = {c->AOl, c->Xnl, c->Sl, c->Xl, c->rope_tab, c->rope_tab_t, c->X[0], c->X[1], c->Xn, c->QKV, c->QK, c->Vt, c->AO, c->S, c->d_meta, c->d_scores, c->d_fate,
                  c->d_stats, c->route_ws, c->d_top_pos, c->d_top_scores};
  for (void *p : ptrs) if (p) (void)hipFree(p);
  if (c->h_meta) (void)hipHostFree(c->h_meta);
  if (c->h_res) (void)hipHostFree(c->h_res);
  for (hipEvent_t e : c->ev_ready) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->ev_free) if (e) (void)hipEventDestroy(e);
  for (int i = 0; i < 4; ++i) if (c->ev_t[i]) (void)hipEventDestroy(c->ev_t[i]);
  for (hipEvent_t e : c->ev_layer) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->ev_xfer) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->ev_pool) if (e) (void)hipEventDestroy(e);
  if (c->copy_stream) (void)hipStreamDestroy(c->copy_stream);
  if (c->own_stream && c->stream) (void)hipStreamDestroy(c->stream);
  delete c;
}

extern "C" int prism_set_forced_keep(prism_ctx *c, const int8_t *masks, int32_t n_events, int32_t n_cands) {
  PRISM_REQUIRE(c, PRISM_EINVAL, "prism_set_forced_keep: null context");
  if (!masks) { c->forced.clear(); c->forced_events = c->forced_cands = 0; return PRISM_OK; }
  PRISM_REQUIRE(n_events > 0 && n_cands > 0, PRISM_EINVAL, "prism_set_forced_keep: sizes must be positive");
  c->forced.assign(masks, masks + (size_t)n_events * n_cands);
  c->forced_events = n_events;
  c->forced_cands = n_cands;
  return PRISM_OK;
}

extern "C" const char *prism_strerror(int code) {
  switch (code) {
    case PRISM_OK: return "ok";
    case PRISM_EINVAL: return "invalid argument";
    case PRISM_ECAP: return "pool does not fit under the device-memory cap";
    case PRISM_EHIP: return "HIP runtime error";
    case PRISM_ENOMEM: return "out of memory";
    case PRISM_EUNSUPPORTED: return "shape not supported by the kernels of this dtype";
    default: return "unknown error code";
  }
}

extern "C" const char *prism_last_error(void) { return g_err; }

// ------------------------------------------------------------------------------------------------ select
namespace prism {

struct Chunk { int c0, c1; int64_t r0, r1; int tile0, n_tiles; int64_t vt_cols; };

// Per-call host state: the live set and the metadata derived from it.
struct Plan {
  std::vector<int> live;           // original candidate indices, batch order
  std::vector<int> len;            // sequence length per live candidate (query + document)
  std::vector<int64_t> row0;       // first row per live candidate: of its sequence, or of its document when the query is shared
  // Shared query (ql > 0): under the causal mask the query tokens' states do not depend on the candidate, so every chunk
  // holds the query's rows ONCE, in front (rows [chunk.r0, chunk.r0 + ql)), followed by the candidates' document rows;
  // attention reads keys below ql from the chunk's query rows.  ql = 0: every sequence carries its own copy of the query.
  int ql = 0;
  int own(int i) const { return len[i] - ql; }   // rows candidate i owns
  int64_t seq_tokens = 0;          // sum of the live sequences' lengths (what the paper counts as live tokens)
  int64_t T = 0;                   // rows actually held and computed
  std::vector<Chunk> chunks;
  std::vector<AttnTile> tiles;
  std::vector<AttnTile> last_tiles;   // per live candidate: the query block that holds its last token
  std::vector<int64_t> col0;          // per live candidate: first V^T column of its sequence (within its chunk)
  // second pass of a checked layer after a prune (single chunk): attention work items that read q, k and V^T where the
  // first pass projected them (the layout before the prune) and write their output in this plan's layout
  std::vector<AttnTile> xtiles;
  int64_t max_chunk_tokens = 0, max_vt_cols = 0;
};

static void build_plan(const prism_ctx *c, Plan &p) {
  const int n = (int)p.live.size();
  p.row0.resize(n);
  p.chunks.clear();
  p.tiles.clear();
  p.last_tiles.assign(n, AttnTile{0, 0, 0, 0, 0, 0, 0, 0});
  p.col0.assign(n, 0);
  p.xtiles.clear();
  p.max_chunk_tokens = p.max_vt_cols = 0;
  p.seq_tokens = 0;
  const int step = c->opt.chunk_cands > 0 ? c->opt.chunk_cands : std::max(n, 1);
  const bool mfma = is16(c->op);
  const int bq = mfma ? attention_16_block_queries(c->m.n_q_heads, c->m.n_kv_heads) : 0;
  const int ql = p.ql;
  int64_t r = 0;
  for (int c0 = 0; c0 < n; c0 += step) {
    Chunk ch;
    ch.c0 = c0; ch.c1 = std::min(n, c0 + step);
    ch.r0 = r;
    ch.tile0 = (int)p.tiles.size();
    int64_t col = 0;
    if (ql > 0) {
      // the shared query: an ordinary sequence of its own (rows [0, ql) of the chunk, columns [0, round_up(ql, 64)))
      for (int q0 = (ql - 1) / bq * bq; q0 >= 0; q0 -= bq) p.tiles.push_back({0, ql, q0, 0, 0, 0, 0, 0});   // row_base = out_base = 0
      col = round_up(ql, 64);
      r += ql;
    }
    for (int i = ch.c0; i < ch.c1; ++i) {
      p.row0[i] = r;
      r += p.own(i);
      p.seq_tokens += p.len[i];
      if (mfma) {
        // rows relative to the chunk; position t >= ql of the sequence is row row_base + t
        const int32_t row_base = (int32_t)(p.row0[i] - ch.r0) - ql;
        // a sequence's query blocks stay together (they share its K/V in one XCD's L2), the late ones, which loop
        // over the most keys, first
        for (int q0 = p.own(i) > 0 ? ql + (p.own(i) - 1) / bq * bq : -1; q0 >= ql; q0 -= bq)
          p.tiles.push_back({row_base, p.len[i], q0, (int32_t)col, ql, 0, row_base, 0});
        p.last_tiles[i] = {row_base, p.len[i], ql + (p.own(i) - 1) / bq * bq, (int32_t)col, ql, 0, row_base, 0};
        p.col0[i] = col;
        col += round_up(p.len[i], 64);
      }
    }
    ch.r1 = r;
    ch.n_tiles = (int)p.tiles.size() - ch.tile0;
    ch.vt_cols = col;
    p.chunks.push_back(ch);
    p.max_chunk_tokens = std::max(p.max_chunk_tokens, ch.r1 - ch.r0);
    p.max_vt_cols = std::max(p.max_vt_cols, col);
  }
  p.T = r;
}

// meta buffer (int32 words): [pos T][vtcol T][lastrow n][seqcol n][src 2n][dst 2n][len 2n][tiles][last tiles][xtiles][tokens T]
// (src/dst/len: one compaction entry per kept candidate plus one per chunk for the shared query's rows)
struct MetaOff { int64_t pos, vtcol, lastrow, seqcol, src, dst, len, tiles, ltiles, xtiles, tokens, words; };

static MetaOff meta_offsets(int64_t T, int n, int64_t n_tiles) {
  MetaOff o;
  int64_t w = 0;
  auto take = [&](int64_t k) { int64_t at = w; w = round_up(w + k, 64); return at; };
  constexpr int64_t tw = sizeof(AttnTile) / 4;
  o.pos = take(T); o.vtcol = take(T); o.lastrow = take(n); o.seqcol = take(n);
  o.src = take(2 * (int64_t)n); o.dst = take(2 * (int64_t)n); o.len = take(2 * (int64_t)n);
  o.tiles = take(tw * n_tiles); o.ltiles = take(tw * (int64_t)n); o.xtiles = take(tw * n_tiles); o.tokens = take(T);
  o.words = w;
  return o;
}

static int ensure_scratch(prism_ctx *c, const Plan &p, bool need_second_x, int n_cands, int64_t max_tiles) {
  const prism_model &m = c->m;
  const size_t e = dtype_size(m.dtype);
  const int64_t Dq = (int64_t)m.n_q_heads * m.head_dim, Dkv = (int64_t)m.n_kv_heads * m.head_dim;
  if (c->offload) {
    if (p.max_chunk_tokens > c->xo_cap) {
      PRISM_HIP(hipDeviceSynchronize());
      for (int i = 0; i < 3; ++i) { dev_free(c, c->Xo[i], (size_t)c->xo_cap * m.hidden * 4); c->Xo[i] = nullptr; }
      c->xo_cap = 0;
      for (int i = 0; i < 3; ++i) PRISM_TRY(dev_alloc(c, (void **)&c->Xo[i], (size_t)p.max_chunk_tokens * m.hidden * 4));
      c->xo_cap = p.max_chunk_tokens;
    }
    if (p.T > c->hx_cap) {
      PRISM_HIP(hipDeviceSynchronize());
      if (c->h_X) { (void)hipHostFree(c->h_X); c->h_X = nullptr; c->hx_cap = 0; }
      PRISM_HIP(hipHostMalloc((void **)&c->h_X, (size_t)p.T * m.hidden * 4, hipHostMallocDefault));
      c->hx_cap = p.T;
    }
  } else {
    PRISM_TRY(grow(c, &c->X[0], &c->x_cap[0], p.T, (size_t)m.hidden * 4));
    if (need_second_x) PRISM_TRY(grow(c, &c->X[1], &c->x_cap[1], p.T, (size_t)m.hidden * 4));
  }
  if (c->embed_cached) {
    const int64_t words = 3 * round_up(p.T, 64);
    PRISM_TRY(grow(c, &c->d_estage, &c->estage_cap, words, 4));
    if (words > c->h_estage_cap) {
      if (c->h_estage) { PRISM_HIP(hipStreamSynchronize(c->stream)); (void)hipHostFree(c->h_estage); c->h_estage = nullptr; c->h_estage_cap = 0; }
      PRISM_HIP(hipHostMalloc((void **)&c->h_estage, (size_t)words * 4, hipHostMallocDefault));
      c->h_estage_cap = words;
    }
  }
  if (p.max_chunk_tokens > c->chunk_cap) {
    PRISM_HIP(hipStreamSynchronize(c->stream));
    const int64_t old = c->chunk_cap, cap = p.max_chunk_tokens;
    const bool bf = is16(c->op);
    dev_free(c, c->Xn, (size_t)old * m.hidden * e); dev_free(c, c->QKV, (size_t)old * (Dq + 2 * Dkv) * 4);
    if (bf) dev_free(c, c->QK, (size_t)old * (Dq + Dkv) * e);
    dev_free(c, c->AO, (size_t)old * Dq * e); dev_free(c, c->S, (size_t)old * m.ffn * e);
    c->Xn = c->QKV = c->QK = c->AO = c->S = nullptr; c->chunk_cap = 0;
    PRISM_TRY(dev_alloc(c, (void **)&c->Xn, (size_t)cap * m.hidden * e));
    PRISM_TRY(dev_alloc(c, (void **)&c->QKV, (size_t)cap * (Dq + 2 * Dkv) * 4));     // fp32 projection
    if (bf) PRISM_TRY(dev_alloc(c, (void **)&c->QK, (size_t)cap * (Dq + Dkv) * e));   // finished q, k
    PRISM_TRY(dev_alloc(c, (void **)&c->AO, (size_t)cap * Dq * e));
    PRISM_TRY(dev_alloc(c, (void **)&c->S, (size_t)cap * m.ffn * e));
    c->chunk_cap = cap;
  }
  if (is16(c->op) && p.max_vt_cols > c->vt_cap) {
    const int64_t old = c->vt_cap;
    PRISM_TRY(grow(c, &c->Vt, &c->vt_cap, p.max_vt_cols, (size_t)Dkv * 2));
    (void)old;
    // pad columns are multiplied by exact zeros; they only have to be finite
    PRISM_TRY(launch_fill_zero(c->Vt, (size_t)round_up((size_t)c->vt_cap * Dkv * 2, 256), c->stream));
  }
  if (n_cands > c->last_cap) {
    PRISM_HIP(hipStreamSynchronize(c->stream));
    const int64_t old = c->last_cap;
    dev_free(c, c->AOl, (size_t)old * Dq * e); dev_free(c, c->Xnl, (size_t)old * m.hidden * e);
    dev_free(c, c->Sl, (size_t)old * m.ffn * e); dev_free(c, c->Xl, (size_t)old * m.hidden * 4);
    c->AOl = c->Xnl = c->Sl = nullptr; c->Xl = nullptr; c->last_cap = 0;
    PRISM_TRY(dev_alloc(c, (void **)&c->AOl, (size_t)n_cands * Dq * e));
    PRISM_TRY(dev_alloc(c, (void **)&c->Xnl, (size_t)n_cands * m.hidden * e));
    PRISM_TRY(dev_alloc(c, (void **)&c->Sl, (size_t)n_cands * m.ffn * e));
    PRISM_TRY(dev_alloc(c, (void **)&c->Xl, (size_t)n_cands * m.hidden * 4));
    c->last_cap = n_cands;
  }
  const MetaOff mo = meta_offsets(p.T, n_cands, max_tiles);
  PRISM_TRY(grow(c, &c->d_meta, &c->meta_cap, mo.words, 4));
  if (mo.words > c->h_meta_cap) {
    if (c->h_meta) { PRISM_HIP(hipStreamSynchronize(c->stream)); (void)hipHostFree(c->h_meta); c->h_meta = nullptr; }
    PRISM_HIP(hipHostMalloc((void **)&c->h_meta, (size_t)mo.words * 4, hipHostMallocDefault));
    c->h_meta_cap = mo.words;
  }
  return PRISM_OK;
}

// Writes pos / vtcol / lastrow / tiles for the current live set into the pinned staging buffer and
// uploads them.  The staging buffer is only rewritten after a stream synchronisation.
static int upload_meta(prism_ctx *c, const Plan &p, const MetaOff &mo, bool with_tokens) {
  int32_t *h = c->h_meta;
  const int n = (int)p.live.size();
  const int ql = p.ql;
  for (const Chunk &ch : p.chunks) {
    int64_t col = 0;
    if (ql > 0) {
      int32_t *pos = h + mo.pos + ch.r0, *vc = h + mo.vtcol + ch.r0;
      for (int t = 0; t < ql; ++t) { pos[t] = t; vc[t] = (int32_t)vt_column_of_key(t); }
      col = round_up(ql, 64);
    }
    for (int i = ch.c0; i < ch.c1; ++i) {
      int32_t *pos = h + mo.pos + p.row0[i], *vc = h + mo.vtcol + p.row0[i];
      for (int t = ql; t < p.len[i]; ++t) { pos[t - ql] = t; vc[t - ql] = (int32_t)(col + vt_column_of_key(t)); }
      h[mo.seqcol + i] = (int32_t)col;
      col += round_up(p.len[i], 64);
    }
  }
  for (int i = 0; i < n; ++i) h[mo.lastrow + i] = (int32_t)(p.row0[i] + p.own(i) - 1);
  if (!p.tiles.empty()) memcpy(h + mo.tiles, p.tiles.data(), p.tiles.size() * sizeof(AttnTile));
  if (!p.last_tiles.empty()) memcpy(h + mo.ltiles, p.last_tiles.data(), p.last_tiles.size() * sizeof(AttnTile));
  if (!p.xtiles.empty()) memcpy(h + mo.xtiles, p.xtiles.data(), p.xtiles.size() * sizeof(AttnTile));
  // one copy for [pos .. tiles], a second for the tokens (first upload only)
  PRISM_HIP(hipMemcpyAsync(c->d_meta, h, (size_t)mo.tokens * 4, hipMemcpyHostToDevice, c->stream));
  if (with_tokens)
    PRISM_HIP(hipMemcpyAsync(c->d_meta + mo.tokens, h + mo.tokens, (size_t)p.T * 4, hipMemcpyHostToDevice, c->stream));
  return PRISM_OK;
}

static int span_event(prism_ctx *c, hipEvent_t *e) {
  if (c->ev_used == c->ev_pool.size()) {
    hipEvent_t n = nullptr;
    PRISM_HIP(hipEventCreate(&n));
    c->ev_pool.push_back(n);
  }
  *e = c->ev_pool[c->ev_used++];
  PRISM_HIP(hipEventRecord(*e, c->stream));
  return PRISM_OK;
}

// Times the launches issued by `body` as one span of the given kind (only when a report was asked for).
template <typename Fn>
static int timed_span(prism_ctx *c, int kind, double flops, Fn body, int rows = 0) {
  if (!c->profiling || !((c->span_mask >> kind) & 1)) return body();
  prism_ctx::Span sp{kind, nullptr, nullptr, flops, rows};
  PRISM_TRY(span_event(c, &sp.a));
  PRISM_TRY(body());
  PRISM_TRY(span_event(c, &sp.b));
  c->spans.push_back(sp);
  return PRISM_OK;
}

// ---- embedding (Sec. 4.5 step 1), optionally through the device row cache (Sec. 4.4)
static void lru_touch(prism_ctx *c, int s) {          // slot s becomes the most recently used
  if (c->lru_head == s) return;
  const int a = c->lru_prev[s], b = c->lru_next[s];
  if (a >= 0) c->lru_next[a] = b;
  if (b >= 0) c->lru_prev[b] = a; else c->lru_tail = a;
  c->lru_prev[s] = -1;
  c->lru_next[s] = c->lru_head;
  c->lru_prev[c->lru_head] = s;
  c->lru_head = s;
}

// X[0 .. n) = embedding rows of the packed tokens [r0, r0 + n) (host copy tok, device copy d_tok), on stream s.
// With the cache: a textbook LRU over the token stream.  Rows are gathered from the cache in passes: a pass ends when
// the least recently used slot is one that this pass still needs, so no row is evicted before it has been gathered.
static int embed_range(prism_ctx *c, const int32_t *tok, const int32_t *d_tok, int64_t r0, int64_t n, int64_t T, float *X,
                       hipStream_t s) {
  const prism_model &m = c->m;
  if (!c->embed_cached) return launch_embed(d_tok + r0, (int)n, c->embed, m.hidden, m.dtype, X, s);
  const int64_t Tp = round_up(T, 64);
  int32_t *h_slot = c->h_estage, *h_mtok = c->h_estage + Tp, *h_mslot = c->h_estage + 2 * Tp;
  int32_t *d_slot = c->d_estage, *d_mtok = c->d_estage + Tp, *d_mslot = c->d_estage + 2 * Tp;
  // the miss lists of this range live at [r0, r0 + n) of their regions too (a range has at most n misses), so ranges
  // and passes never share staging memory and nothing has to be synchronised before the call returns
  int64_t pass_begin = r0, miss_begin = r0, miss_end = r0;
  auto flush = [&](int64_t end) -> int {
    if (end == pass_begin) return PRISM_OK;
    const int64_t nm = miss_end - miss_begin;
    PRISM_HIP(hipMemcpyAsync(d_slot + pass_begin, h_slot + pass_begin, (size_t)(end - pass_begin) * 4, hipMemcpyHostToDevice, s));
    if (nm > 0) {
      PRISM_HIP(hipMemcpyAsync(d_mtok + miss_begin, h_mtok + miss_begin, (size_t)nm * 4, hipMemcpyHostToDevice, s));
      PRISM_HIP(hipMemcpyAsync(d_mslot + miss_begin, h_mslot + miss_begin, (size_t)nm * 4, hipMemcpyHostToDevice, s));
      PRISM_TRY(launch_copy_rows(c->embed_dev_alias, d_mtok + miss_begin, c->d_cache, d_mslot + miss_begin, (int)nm,
                                 (size_t)m.hidden * dtype_size(m.dtype), s));
    }
    PRISM_TRY(launch_embed(d_slot + pass_begin, (int)(end - pass_begin), c->d_cache, m.hidden, m.dtype, X + (pass_begin - r0) * m.hidden, s));
    pass_begin = end;
    miss_begin = miss_end;
    ++c->pass_id;
    return PRISM_OK;
  };
  for (int64_t t = r0; t < r0 + n; ++t) {
    const int32_t tk = tok[t];
    int sl = c->slot_of[tk];
    if (sl >= 0) {
      ++c->embed_hit;
    } else {
      ++c->embed_miss;
      sl = c->lru_tail;
      if (c->pin[sl] == c->pass_id) PRISM_TRY(flush(t));       // the victim is still needed by this pass: gather first
      if (c->tok_of[sl] >= 0) c->slot_of[c->tok_of[sl]] = -1;
      c->tok_of[sl] = tk;
      c->slot_of[tk] = sl;
      h_mtok[miss_end] = tk;
      h_mslot[miss_end] = sl;
      ++miss_end;
    }
    lru_touch(c, sl);
    c->pin[sl] = c->pass_id;
    h_slot[t] = sl;
  }
  return flush(r0 + n);
}

// ---- hidden-state offload: chunk copies between the pinned host copy of the residual stream and a device slot, one
//      copy per run of candidates that are adjacent in the host layout (which never changes: pruning only drops runs)
static int copy_chunk(prism_ctx *c, const Plan &p, const Chunk &ch, int slot, bool to_device, hipStream_t st) {
  const int64_t H = c->m.hidden;
  int i = ch.c0;
  while (i < ch.c1) {
    int j = i;
    int64_t rows = p.len[i];
    while (j + 1 < ch.c1 && c->hrow[p.live[j + 1]] == c->hrow[p.live[j]] + p.len[j]) { ++j; rows += p.len[j]; }
    float *dev = c->Xo[slot] + (p.row0[i] - ch.r0) * H;
    float *host = c->h_X + c->hrow[p.live[i]] * H;
    if (to_device) PRISM_HIP(hipMemcpyAsync(dev, host, (size_t)rows * H * 4, hipMemcpyHostToDevice, st));
    else PRISM_HIP(hipMemcpyAsync(host, dev, (size_t)rows * H * 4, hipMemcpyDeviceToHost, st));
    c->bytes_hidden += rows * H * 4;
    i = j + 1;
  }
  return PRISM_OK;
}

// Requests chunk ci of plan p into the slot of pipeline step `step`.  The slot is free once its previous content has
// been written back; the chunk's data is on the host once its own last write-back is done.  wait_all (first request
// after the live set or the partition changed): wait for every write-back issued so far.
static int prefetch_chunk(prism_ctx *c, const Plan &p, int ci, int64_t step, bool wait_all) {
  const int slot = (int)(step % 3), nch = (int)p.chunks.size();
  if (wait_all) {
    for (int i = 0; i < 3; ++i) PRISM_HIP(hipStreamWaitEvent(c->xin_stream, c->ev_out[i], 0));
  } else {
    // steady state on one plan: chunk ci was last written back nch steps ago; with three or more chunks that is not
    // later than the slot's previous write-back (three steps ago) on the in-order write-back stream
    PRISM_HIP(hipStreamWaitEvent(c->xin_stream, c->ev_out[slot], 0));
    if (nch < 3 && step >= nch) PRISM_HIP(hipStreamWaitEvent(c->xin_stream, c->ev_out[(step - nch) % 3], 0));
  }
  PRISM_TRY(copy_chunk(c, p, p.chunks[ci], slot, true, c->xin_stream));
  PRISM_HIP(hipEventRecord(c->ev_in[slot], c->xin_stream));
  return PRISM_OK;
}

// Writes the slot of the current step back to the host once the compute stream is done with it (copy == false: only
// marks the slot as free, for results that are not needed again).
static int retire_chunk(prism_ctx *c, const Plan &p, const Chunk &ch, int slot, bool copy) {
  PRISM_HIP(hipEventRecord(c->ev_done[slot], c->stream));
  PRISM_HIP(hipStreamWaitEvent(c->xout_stream, c->ev_done[slot], 0));
  if (copy) PRISM_TRY(copy_chunk(c, p, ch, slot, false, c->xout_stream));
  PRISM_HIP(hipEventRecord(c->ev_out[slot], c->xout_stream));
  return PRISM_OK;
}

// One transformer layer over every chunk.  Offload mode additionally: score_after = score the chunk's candidates while
// the chunk is on the device (checkpoint layers and the last one); write_back = the layer's output is needed again;
// next_layer_same_plan = the next layer runs on the same live set, so its first chunk may be prefetched.
// last_only (the model's last layer): nothing but the final scores is read from this layer's output, and a score needs the
// last token's state only.  Keys and values are still needed for every token, so the q/k/v projection runs in full; the
// attention runs for the query block that holds the last token, and the O projection and the whole FFN block run on one
// gathered row per candidate, whose final scores are taken right there.
// resume: the chunk scratch still holds this plan's finished q, k and V^T of this layer (left by a last_only pass over the
// same single chunk): the layer continues at the attention step.
static int run_layer(prism_ctx *c, const Plan &p, const MetaOff &mo, float *X, const char *wbuf, bool score_after = false,
                     bool write_back = true, bool next_layer_same_plan = false, bool last_only = false, bool resume = false) {
  const prism_model &m = c->m;
  const LayerLayout &L = c->lay;
  const int H = m.hidden, Dq = m.n_q_heads * m.head_dim, Dkv = m.n_kv_heads * m.head_dim, F = m.ffn;
  hipStream_t s = c->stream;
  const bool bf = is16(c->op);
  auto gemm = [&](int epi, const void *A, const void *W, void *out, int M, int N, int K) {
    return bf ? launch_gemm_16(c->op, epi, A, W, out, M, N, K, s)
              : launch_gemm_fp32(epi, (const float *)A, (const float *)W, out, M, N, K, s);
  };
  const int nch = (int)p.chunks.size();
  for (int ci = 0; ci < nch; ++ci) {
    const Chunk &ch = p.chunks[ci];
    const int Tc = (int)(ch.r1 - ch.r0);
    float *Xc = c->offload ? nullptr : X + ch.r0 * H;
    int slot = 0;
    // offload pipeline: the next chunk visit (next chunk of this layer, or the first chunk of the next layer)
    const int next_ci = ci + 1 < nch ? ci + 1 : (next_layer_same_plan ? 0 : -1);
    if (c->offload) {
      slot = (int)(c->ostep % 3);
      if (!c->primed) PRISM_TRY(prefetch_chunk(c, p, ci, c->ostep, true));
      c->primed = false;
      // with one chunk per layer the next visit needs THIS visit's write-back, so it is requested afterwards
      if (nch >= 2 && next_ci >= 0) { PRISM_TRY(prefetch_chunk(c, p, next_ci, c->ostep + 1, false)); c->primed = true; }
      PRISM_HIP(hipStreamWaitEvent(s, c->ev_in[slot], 0));
      Xc = c->Xo[slot];
    }
    const int32_t *pos = c->d_meta + mo.pos + ch.r0;
    double attn_flops = 0.0;
    // causal triangle of every sequence; with a shared query its own triangle is computed once per chunk
    const double tri_q = (double)p.ql * (p.ql + 1.0);
    for (int i = ch.c0; i < ch.c1; ++i) attn_flops += 2.0 * m.n_q_heads * m.head_dim * ((double)p.len[i] * (p.len[i] + 1.0) - tri_q);
    attn_flops += 2.0 * m.n_q_heads * m.head_dim * tri_q;
    const double tk = 2.0 * Tc;
    // ---- attention block: X += Attn(RMSNorm(X)) Wo^T
    if (!resume) {
    PRISM_TRY(timed_span(c, 5, 0.0, [&] { return launch_rmsnorm(Xc, wbuf + L.attn_norm, Tc, H, m.rms_eps, c->op, c->Xn, s); }));
    // 16-bit modes at head_dim 128 with enough rows: norm, RoPE, rounding and the V transposition happen in the
    // projection's epilogue; otherwise the projection is stored in fp32 and finished by separate kernels
    const bool fused_qkv = bf && gemm_16_qkv_supported(Tc, m.n_q_heads, m.n_kv_heads, m.head_dim, H);
    PRISM_TRY(timed_span(c, 0, tk * (Dq + 2 * Dkv) * H, [&] {
      if (fused_qkv) {
        QkvEpilogue e;
        e.pos = pos; e.vt_col = c->d_meta + mo.vtcol + ch.r0;
        e.q_gain = wbuf + L.q_norm; e.k_gain = wbuf + L.k_norm;
        e.rope_tab_t = c->rope_tab_t; e.rope_stride = PRISM_MAX_SEQ; e.QK = c->QK; e.Vt = c->Vt; e.vt_stride = c->vt_cap;
        e.nq = m.n_q_heads; e.nkv = m.n_kv_heads; e.qk_norm = m.qk_norm; e.eps = m.rms_eps;
        return launch_gemm_16_qkv(c->op, c->Xn, wbuf + L.wqkv, Tc, H, m.head_dim, e, s);
      }
      return gemm(bf ? PRISM_EPI_STORE_F32 : PRISM_EPI_STORE, c->Xn, wbuf + L.wqkv, c->QKV, Tc, Dq + 2 * Dkv, H);
    }, Tc));
    if (!fused_qkv) PRISM_TRY(timed_span(c, 5, 0.0, [&] {
      PRISM_TRY(launch_qk_finish(c->op, (float *)c->QKV, pos, wbuf + L.q_norm, wbuf + L.k_norm, Tc, m.n_q_heads,
                                 m.n_kv_heads, m.head_dim, m.rms_eps, m.qk_norm, c->rope_tab, c->QK, s));
      if (bf)
        PRISM_TRY(launch_v_finish(c->op, (const float *)c->QKV, Tc, m.n_q_heads, m.n_kv_heads, m.head_dim, c->Vt,
                                  c->d_meta + mo.vtcol + ch.r0, c->vt_cap, s));
      return (int)PRISM_OK;
    }));
    if (p.ql > 0)   // every sequence's V^T columns cover all its positions: the query's part is copied in (a few MB)
      PRISM_TRY(timed_span(c, 5, 0.0, [&] {
        return launch_vt_prefix_broadcast(c->Vt, c->vt_cap, Dkv, p.ql, c->d_meta + mo.seqcol + ch.c0, ch.c1 - ch.c0, s);
      }));
    }
    if (last_only) {
      const int nc = ch.c1 - ch.c0;
      const size_t e = dtype_size(m.dtype);
      double last_attn = 0.0;                                    // one query per head: 2 contractions of length L
      for (int i = ch.c0; i < ch.c1; ++i) last_attn += 2.0 * m.n_q_heads * m.head_dim * 2.0 * p.len[i];
      PRISM_TRY(timed_span(c, 4, last_attn, [&] {
        if (bf)
          return launch_attention_16(c->op, c->QK, c->Vt, c->vt_cap, (const AttnTile *)(c->d_meta + mo.ltiles) + ch.c0, nc, Tc,
                                     m.n_q_heads, m.n_kv_heads, m.head_dim, c->AO, s);
        return launch_attention_fp32((const float *)c->QKV, pos, Tc, m.n_q_heads, m.n_kv_heads, m.head_dim, (float *)c->AO, s);
      }));
      // last_row holds rows of the packed pool; this chunk's rows start at ch.r0
      const int32_t *last_row = c->d_meta + mo.lastrow + ch.c0;
      char *AOl = c->AOl + (size_t)ch.c0 * Dq * e, *Xnl = c->Xnl + (size_t)ch.c0 * H * e, *Sl = c->Sl + (size_t)ch.c0 * F * e;
      float *Xl = c->Xl + (size_t)ch.c0 * H;
      PRISM_TRY(timed_span(c, 5, 0.0, [&] {
        PRISM_TRY(launch_copy_rows(c->AO - ch.r0 * (int64_t)Dq * (int64_t)e, last_row, AOl, nullptr, nc, (size_t)Dq * e, s));
        return launch_copy_rows(Xc - ch.r0 * H, last_row, Xl, nullptr, nc, (size_t)H * 4, s);
      }));
      // (timed with the elementwise kind: these launches are a different, tiny kernel configuration and would blur the
      // per-launch figures of the layer GEMMs)
      PRISM_TRY(timed_span(c, 5, 0.0, [&] {
        PRISM_TRY(gemm(PRISM_EPI_RESIDUAL, AOl, wbuf + L.wo, Xl, nc, H, Dq));
        PRISM_TRY(launch_rmsnorm(Xl, wbuf + L.ffn_norm, nc, H, m.rms_eps, c->op, Xnl, s));
        PRISM_TRY(gemm(PRISM_EPI_SWIGLU, Xnl, wbuf + L.wgu, Sl, nc, 2 * F, H));
        return gemm(PRISM_EPI_RESIDUAL, Sl, wbuf + L.wd, Xl, nc, H, F);
      }));
      PRISM_TRY(launch_score(Xl, nullptr, nc, m.hidden, c->final_norm, c->w_yes, c->w_no, m.dtype, m.rms_eps,
                             c->d_scores + ch.c0, s));
    } else {
    PRISM_TRY(timed_span(c, 4, attn_flops, [&] {
      if (bf) {
        if (resume && !p.xtiles.empty())      // q, k and V^T sit where the first pass left them
          return launch_attention_16(c->op, c->QK, c->Vt, c->vt_cap, (const AttnTile *)(c->d_meta + mo.xtiles),
                                     (int)p.xtiles.size(), Tc, m.n_q_heads, m.n_kv_heads, m.head_dim, c->AO, s);
        return launch_attention_16(c->op, c->QK, c->Vt, c->vt_cap, (const AttnTile *)(c->d_meta + mo.tiles) + ch.tile0,
                                   ch.n_tiles, Tc, m.n_q_heads, m.n_kv_heads, m.head_dim, c->AO, s);
      }
      return launch_attention_fp32((const float *)c->QKV, pos, Tc, m.n_q_heads, m.n_kv_heads, m.head_dim, (float *)c->AO, s);
    }, Tc));
    PRISM_TRY(timed_span(c, 1, tk * H * Dq, [&] { return gemm(PRISM_EPI_RESIDUAL, c->AO, wbuf + L.wo, Xc, Tc, H, Dq); }, Tc));
    // ---- FFN block: X += (silu(Xn Wg^T) * (Xn Wu^T)) Wd^T
    PRISM_TRY(timed_span(c, 5, 0.0, [&] { return launch_rmsnorm(Xc, wbuf + L.ffn_norm, Tc, H, m.rms_eps, c->op, c->Xn, s); }));
    PRISM_TRY(timed_span(c, 2, tk * 2 * F * H, [&] { return gemm(PRISM_EPI_SWIGLU, c->Xn, wbuf + L.wgu, c->S, Tc, 2 * F, H); }, Tc));
    PRISM_TRY(timed_span(c, 3, tk * H * F, [&] { return gemm(PRISM_EPI_RESIDUAL, c->S, wbuf + L.wd, Xc, Tc, H, F); }, Tc));
    }
    if (c->offload) {
      if (score_after && !last_only)   // last_row holds rows of the packed pool; this chunk's rows start at ch.r0
        PRISM_TRY(launch_score(Xc - ch.r0 * H, c->d_meta + mo.lastrow + ch.c0, ch.c1 - ch.c0, m.hidden, c->final_norm, c->w_yes,
                               c->w_no, m.dtype, m.rms_eps, c->d_scores + ch.c0, s));
      PRISM_TRY(retire_chunk(c, p, ch, slot, write_back));
      if (nch < 2 && next_ci >= 0) { PRISM_TRY(prefetch_chunk(c, p, next_ci, c->ostep + 1, false)); c->primed = true; }
      ++c->ostep;
    }
  }
  return PRISM_OK;
}

}  // namespace prism

static int select_impl(prism_ctx *c, const int32_t *query_tokens, int32_t query_len,
                       const int32_t *const *cand_tokens, const int32_t *cand_lens, int32_t n_cands, int32_t K,
                       int32_t *out_idx, float *out_scores, int32_t *out_count, prism_report *rep);

extern "C" int prism_select(prism_ctx *c, const int32_t *query_tokens, int32_t query_len,
                            const int32_t *const *cand_tokens, const int32_t *cand_lens, int32_t n_cands, int32_t K,
                            int32_t *out_idx, float *out_scores, int32_t *out_count, prism_report *rep) {
  const int rc = select_impl(c, query_tokens, query_len, cand_tokens, cand_lens, n_cands, K, out_idx, out_scores, out_count, rep);
  if (rc != PRISM_OK && c) {
    // A call that failed midway leaves work queued on the library's streams and a half-filled report: drain the
    // streams (errors here are secondary to rc), restart the offload pipeline from a clean state, and hand back an
    // empty report.  out_idx / out_scores / out_count are only written by a call that succeeds.
    for (hipStream_t st : {c->stream, c->copy_stream, c->xin_stream, c->xout_stream})
      if (st && hipStreamSynchronize(st) != hipSuccess) (void)hipGetLastError();
    c->primed = false;
    c->profiling = false;
    if (rep) rep->n_events = 0;
  }
  return rc;
}

static int select_impl(prism_ctx *c, const int32_t *query_tokens, int32_t query_len,
                       const int32_t *const *cand_tokens, const int32_t *cand_lens, int32_t n_cands, int32_t K,
                       int32_t *out_idx, float *out_scores, int32_t *out_count, prism_report *rep) {
  PRISM_REQUIRE(c && query_tokens && cand_tokens && cand_lens && out_idx && out_scores && out_count, PRISM_EINVAL,
                "prism_select: null argument");
  PRISM_REQUIRE(query_len > 0 && n_cands > 0 && K > 0, PRISM_EINVAL, "prism_select: query_len, n_cands and K must be positive");
  PRISM_REQUIRE(n_cands <= PRISM_MAX_CANDS, PRISM_EINVAL, "prism_select: more than %d candidates", PRISM_MAX_CANDS);
  const prism_model &m = c->m;
  for (int t = 0; t < query_len; ++t)
    PRISM_REQUIRE(query_tokens[t] >= 0 && query_tokens[t] < m.vocab, PRISM_EINVAL, "prism_select: query token %d out of range", t);
  Plan p;
  p.live.resize(n_cands);
  p.len.resize(n_cands);
  for (int i = 0; i < n_cands; ++i) {
    PRISM_REQUIRE(cand_lens[i] > 0 && cand_tokens[i], PRISM_EINVAL, "prism_select: candidate %d is empty", i);
    PRISM_REQUIRE((int64_t)query_len + cand_lens[i] <= PRISM_MAX_SEQ, PRISM_EINVAL,
                  "prism_select: sequence %d longer than %d tokens", i, PRISM_MAX_SEQ);
    for (int t = 0; t < cand_lens[i]; ++t)
      PRISM_REQUIRE(cand_tokens[i][t] >= 0 && cand_tokens[i][t] < m.vocab, PRISM_EINVAL,
                    "prism_select: token %d of candidate %d out of range", t, i);
    p.live[i] = i;
    p.len[i] = query_len + cand_lens[i];
  }
  if (rep) {
    PRISM_REQUIRE(rep->cap_events > 0 && rep->n_cands >= n_cands && rep->ev_layer && rep->ev_n_before && rep->ev_n_after &&
                      rep->ev_tokens_after && rep->ev_gate && rep->ev_n_clusters && rep->ev_mean && rep->ev_std &&
                      rep->ev_scores && rep->ev_fate,
                  PRISM_EINVAL, "prism_select: report arrays missing or too small");
  }
  const int Kc = std::min(K, n_cands);
  const int mode = K >= n_cands ? PRISM_MODE_NO_PRUNING : c->opt.mode;
  // the query is held and computed once per chunk where the path supports it: the matrix-core attention kernel (the
  // fp32 kernel finds sequences by their positions) and a device-resident residual stream
  p.ql = (!c->opt.no_query_sharing && is16(c->op) && !c->offload && n_cands > 1 &&
          attention_16_supported(m.n_q_heads, m.n_kv_heads, m.head_dim)) ? query_len : 0;
  build_plan(c, p);
  PRISM_REQUIRE(p.T < (int64_t)1 << 30, PRISM_EINVAL, "prism_select: pool of %lld tokens is too large", (long long)p.T);
  const bool may_prune = mode != PRISM_MODE_NO_PRUNING && !c->checkpoints.empty();
  const int64_t max_tiles = (int64_t)p.tiles.size();   // the live set only shrinks
  PRISM_TRY(ensure_scratch(c, p, may_prune, n_cands, max_tiles));
  const MetaOff mo = meta_offsets(p.T, n_cands, max_tiles);
  hipStream_t s = c->stream;

  // tokens, packed: sequence i = query ++ candidate i; with a shared query the query's tokens once per chunk
  {
    int32_t *tok = c->h_meta + mo.tokens;
    if (p.ql > 0)
      for (const Chunk &ch : p.chunks) memcpy(tok + ch.r0, query_tokens, (size_t)query_len * 4);
    for (int i = 0; i < n_cands; ++i) {
      if (p.ql == 0) memcpy(tok + p.row0[i], query_tokens, (size_t)query_len * 4);
      memcpy(tok + p.row0[i] + (p.ql == 0 ? query_len : 0), cand_tokens[i], (size_t)cand_lens[i] * 4);
    }
  }
  const bool timed = rep != nullptr;
  c->profiling = timed;
  c->span_mask = timed && rep->kind_mask ? rep->kind_mask : ~0;
  c->spans.clear();
  c->ev_used = 0;
  // opt-in: the end-of-transfer records wait for the copies in the side stream's hardware queue, which holds back compute
  // kernels behind them if the compute stream shares that queue
  const bool timed_xfer = timed && c->streamed && (rep->kind_mask & PRISM_KIND_MASK_TRANSFERS) != 0;
  if (timed_xfer && (int)c->ev_xfer.size() < 2 * m.n_layers) {
    const size_t old = c->ev_xfer.size();
    c->ev_xfer.resize(2 * m.n_layers, nullptr);
    for (size_t i = old; i < c->ev_xfer.size(); ++i) PRISM_HIP(hipEventCreate(&c->ev_xfer[i]));
  }
  int n_xfer_timed = 0;
  if (timed && (int)c->ev_layer.size() < 4 * m.n_layers) {
    const size_t old = c->ev_layer.size();
    c->ev_layer.resize(4 * m.n_layers, nullptr);
    for (size_t i = old; i < c->ev_layer.size(); ++i) PRISM_HIP(hipEventCreate(&c->ev_layer[i]));
  }
  if (timed) PRISM_HIP(hipEventRecord(c->ev_t[0], s));
  PRISM_TRY(upload_meta(c, p, mo, true));
  int cur = 0;
  c->embed_hit = c->embed_miss = 0;
  c->bytes_hidden = 0;
  if (c->offload) {
    // the pool's residual stream is born chunk by chunk and leaves for the host right away
    c->hrow.assign(p.row0.begin(), p.row0.end());
    c->primed = false;
    for (const Chunk &ch : p.chunks) {
      const int slot = (int)(c->ostep % 3);
      PRISM_HIP(hipStreamWaitEvent(s, c->ev_out[slot], 0));      // the slot's previous content has been written back
      PRISM_TRY(embed_range(c, c->h_meta + mo.tokens, c->d_meta + mo.tokens, ch.r0, ch.r1 - ch.r0, p.T, c->Xo[slot], s));
      PRISM_TRY(retire_chunk(c, p, ch, slot, true));
      ++c->ostep;
    }
  } else {
    PRISM_TRY(embed_range(c, c->h_meta + mo.tokens, c->d_meta + mo.tokens, 0, p.T, p.T, c->X[cur], s));
  }

  int64_t bytes_streamed = 0, token_layers = 0;
  // A layer's transfers and its finishing kernels (conversion or expansion, then the slot's ready event) are issued at
  // different times: whatever waits for a transfer to complete is queued only after a full layer of compute kernels
  // has been queued behind the transfer.  The side stream and the compute stream may be served by one hardware queue
  // (the runtime maps streams onto a few of them, and which share one depends on what else the process has created); a
  // queue is consumed in order, so a wait for the copy queued right behind it would hold back the compute kernels that
  // follow, and the copy would not overlap anything.  With the wait a layer later the order in the shared queue is
  // transfer, a layer of compute, wait: the overlap no longer depends on the mapping.
  auto transfer_layer = [&](int layer, int slot) -> int {
    if (timed_xfer) PRISM_HIP(hipEventRecord(c->ev_xfer[2 * layer], c->copy_stream));
    PRISM_TRY(issue_layer_copy(c, layer, slot, c->copy_stream, hipMemcpyHostToDevice, &bytes_streamed, kLayerTransfer));
    if (timed_xfer) { PRISM_HIP(hipEventRecord(c->ev_xfer[2 * layer + 1], c->copy_stream)); n_xfer_timed = layer + 1; }
    return PRISM_OK;
  };
  auto finish_layer = [&](int layer) -> int {
    const int slot = layer % c->ring;
    PRISM_TRY(issue_layer_copy(c, layer, slot, c->copy_stream, hipMemcpyHostToDevice, nullptr, kLayerFinish));
    PRISM_HIP(hipEventRecord(c->ev_ready[slot], c->copy_stream));
    return PRISM_OK;
  };
  if (c->two_slot) {
    // Sec. 4.2: a ring of layer buffers (two in the paper); layer l computes from slot l % ring while the layers
    // after it arrive (or are expanded) in the others
    for (int l = 0; l < std::min(c->ring, m.n_layers); ++l) PRISM_TRY(transfer_layer(l, l));
    for (int l = 0; l < std::min(c->ring - 1, m.n_layers); ++l) PRISM_TRY(finish_layer(l));
  }

  std::vector<int> early_idx;          // three-way mode: candidates selected before the end, in output order
  std::vector<float> early_scores;
  int K_rem = Kc, n_events = 0, n_forced_seen = 0, layers_run = 0;
  bool terminated = false;
  std::vector<int> final_idx;
  std::vector<float> final_scores;
  size_t next_ckpt = 0;
  double ms_checks = 0.0;
  float *h_scores = (float *)c->h_res;
  int8_t *h_fate = (int8_t *)(c->h_res + PRISM_MAX_CANDS * 4);
  double *h_stats = (double *)(c->h_res + PRISM_MAX_CANDS * 5);
  int32_t *h_top_pos = (int32_t *)(c->h_res + PRISM_MAX_CANDS * 5 + 64);
  float *h_top_scores = (float *)(c->h_res + PRISM_MAX_CANDS * 9 + 64);

  auto record_event = [&](int layer, int n_before, const std::vector<int> &live_before, bool gate, int n_clusters,
                          double mean, double sd, const int8_t *fate /* may be null */, const std::vector<char> *keep) {
    if (!rep || n_events >= rep->cap_events) { ++n_events; return; }
    const int e = n_events++;
    rep->ev_layer[e] = layer; rep->ev_n_before[e] = n_before; rep->ev_gate[e] = gate; rep->ev_n_clusters[e] = n_clusters;
    rep->ev_mean[e] = mean; rep->ev_std[e] = sd;
    float *sc = rep->ev_scores + (size_t)e * rep->n_cands;
    int8_t *ft = rep->ev_fate + (size_t)e * rep->n_cands;
    for (int i = 0; i < rep->n_cands; ++i) { sc[i] = std::numeric_limits<float>::quiet_NaN(); ft[i] = PRISM_FATE_NOT_LIVE; }
    int n_after = 0; int64_t tok_after = 0;
    for (int i = 0; i < n_before; ++i) {
      sc[live_before[i]] = h_scores[i];
      ft[live_before[i]] = fate ? fate[i] : (int8_t)PRISM_FATE_DEFERRED;
      if (!keep || (*keep)[i]) { ++n_after; tok_after += p.len[i]; }
    }
    rep->ev_n_after[e] = n_after; rep->ev_tokens_after[e] = (int32_t)tok_after;
  };

  std::vector<char> second_pass(m.n_layers, 0);
  for (int l = 0; l < m.n_layers && !terminated; ++l) {
    const int slot = c->two_slot ? l % c->ring : l;
    if (c->two_slot) PRISM_HIP(hipStreamWaitEvent(s, c->ev_ready[slot], 0));
    if (timed) PRISM_HIP(hipEventRecord(c->ev_layer[4 * l], s));
    // known before the layer runs: will its output be scored for pruning, and is it the last one
    while (next_ckpt < c->checkpoints.size() && c->checkpoints[next_ckpt] < l + 1) ++next_ckpt;
    const bool check_after = next_ckpt < c->checkpoints.size() && c->checkpoints[next_ckpt] == l + 1 && l + 1 < m.n_layers &&
                             may_prune && (int)p.live.size() > K_rem;
    const bool last_layer = l + 1 == m.n_layers;
    // A layer whose output is checked runs in two passes: first only what the scores need (keys and values of every
    // token, then attention, O projection and FFN for each candidate's last token, exactly as in the last layer), then,
    // after the decision, the rest of the layer for the survivors alone - the candidates the check drops never get
    // their layer finished.  The scores are the same bits either way (the GEMM variants and the other kernels compute a
    // row identically wherever it sits).
    const bool peek = check_after && !c->offload && !c->opt.single_pass_checks;
    second_pass[l] = false;
    PRISM_TRY(run_layer(c, p, mo, c->X[cur], c->layer_buf[slot], check_after || last_layer, !last_layer,
                        !last_layer && !check_after, last_layer || peek));
    if (timed) PRISM_HIP(hipEventRecord(c->ev_layer[4 * l + 1], s));
    token_layers += p.seq_tokens;
    layers_run = l + 1;
    // this layer's kernels are queued: the layer that arrived last (the one the ring's newest slot holds) can be finished
    if (c->two_slot && l + c->ring - 1 < m.n_layers) PRISM_TRY(finish_layer(l + c->ring - 1));
    auto release_slot = [&]() -> int {       // the layer's weights are no longer needed: the ring moves on
      if (c->two_slot && l + c->ring < m.n_layers) {
        PRISM_HIP(hipEventRecord(c->ev_free[slot], s));
        PRISM_HIP(hipStreamWaitEvent(c->copy_stream, c->ev_free[slot], 0));
        PRISM_TRY(transfer_layer(l + c->ring, slot));
      }
      return PRISM_OK;
    };
    if (!peek) PRISM_TRY(release_slot());
    const int n_live = (int)p.live.size();
    if (!check_after) continue;
    bool compacted = false;

    // ---- pruning check on the output of layer l + 1, before layer l + 2 runs (Sec. 3.4, 4.1)
    if (timed) PRISM_HIP(hipEventRecord(c->ev_t[2], s));
    if (!c->offload && !peek)   // offload mode scored every chunk while it was on the device, the first pass its last rows
      PRISM_TRY(launch_score(c->X[cur], c->d_meta + mo.lastrow, n_live, m.hidden, c->final_norm, c->w_yes, c->w_no, m.dtype,
                             m.rms_eps, c->d_scores, s));
    PRISM_TRY(launch_route(c->d_scores, n_live, K_rem, c->opt.n_clusters, c->opt.cv_threshold, c->d_fate, c->d_stats,
                           c->route_ws, s));
    PRISM_HIP(hipMemcpyAsync(h_scores, c->d_scores, (size_t)n_live * 4, hipMemcpyDeviceToHost, s));
    PRISM_HIP(hipMemcpyAsync(h_fate, c->d_fate, (size_t)n_live, hipMemcpyDeviceToHost, s));
    PRISM_HIP(hipMemcpyAsync(h_stats, c->d_stats, 4 * sizeof(double), hipMemcpyDeviceToHost, s));
    PRISM_HIP(hipStreamSynchronize(s));
    const bool gate = h_stats[2] != 0.0;
    const int n_clu = (int)h_stats[3];
    std::vector<char> keep(n_live, 1);
    int n_sel = 0, n_def = 0;
    for (int i = 0; i < n_live; ++i) {
      n_sel += h_fate[i] == PRISM_FATE_SELECTED;
      n_def += h_fate[i] == PRISM_FATE_DEFERRED;
      if (n_clu > 0) keep[i] = mode == PRISM_MODE_DROP_ONLY ? h_fate[i] != PRISM_FATE_DROPPED : h_fate[i] == PRISM_FATE_DEFERRED;
    }
    if (!c->forced.empty() && n_forced_seen < c->forced_events && mode == PRISM_MODE_DROP_ONLY) {
      const int8_t *fm = c->forced.data() + (size_t)n_forced_seen * c->forced_cands;
      for (int i = 0; i < n_live; ++i) keep[i] = p.live[i] < c->forced_cands ? fm[p.live[i]] != 0 : 1;
    }
    ++n_forced_seen;
    const std::vector<int> live_before = p.live;
    record_event(l + 1, n_live, live_before, gate, n_clu, h_stats[0], h_stats[1], h_fate, &keep);
    if (mode == PRISM_MODE_THREE_WAY && n_clu > 0) {
      if (n_sel > 0) {
        // selected candidates leave with their exit-time score, best first
        PRISM_TRY(launch_topk_masked(c->d_scores, c->d_fate, PRISM_FATE_SELECTED, n_live, n_sel, c->d_top_pos, c->d_top_scores, s));
        PRISM_HIP(hipMemcpyAsync(h_top_pos, c->d_top_pos, (size_t)n_sel * 4, hipMemcpyDeviceToHost, s));
        PRISM_HIP(hipMemcpyAsync(h_top_scores, c->d_top_scores, (size_t)n_sel * 4, hipMemcpyDeviceToHost, s));
        PRISM_HIP(hipStreamSynchronize(s));
        for (int i = 0; i < n_sel; ++i) { early_idx.push_back(p.live[h_top_pos[i]]); early_scores.push_back(h_top_scores[i]); }
        K_rem -= n_sel;
      }
      if (n_def == K_rem) {
        // Sec. 4.1: the deferred set fills the remaining slots exactly -> the forward stops here
        PRISM_TRY(launch_topk_masked(c->d_scores, c->d_fate, PRISM_FATE_DEFERRED, n_live, n_def, c->d_top_pos, c->d_top_scores, s));
        PRISM_HIP(hipMemcpyAsync(h_top_pos, c->d_top_pos, (size_t)n_def * 4, hipMemcpyDeviceToHost, s));
        PRISM_HIP(hipMemcpyAsync(h_top_scores, c->d_top_scores, (size_t)n_def * 4, hipMemcpyDeviceToHost, s));
        PRISM_HIP(hipStreamSynchronize(s));
        for (int i = 0; i < n_def; ++i) { final_idx.push_back(p.live[h_top_pos[i]]); final_scores.push_back(h_top_scores[i]); }
        terminated = true;
      }
    }
    int n_keep = 0;
    for (int i = 0; i < n_live; ++i) n_keep += keep[i];
    if (n_keep < n_live && !terminated) {
      // ---- compaction: kept sequences move to the other X buffer, order preserved; metadata is rebuilt
      int32_t *h = c->h_meta;
      Plan q;
      q.ql = p.ql;
      std::vector<int> from;
      for (int i = 0; i < n_live; ++i) {
        if (!keep[i]) continue;
        q.live.push_back(p.live[i]); q.len.push_back(p.len[i]); from.push_back(i);
      }
      build_plan(c, q);
      if (peek && is16(c->op) && p.chunks.size() == 1 && q.chunks.size() == 1) {
        const int bq = attention_16_block_queries(m.n_q_heads, m.n_kv_heads);
        const int ql = q.ql;
        if (ql > 0)
          for (int q0 = (ql - 1) / bq * bq; q0 >= 0; q0 -= bq) q.xtiles.push_back({0, ql, q0, 0, 0, 0, 0, 0});
        for (int k = 0; k < n_keep; ++k) {
          const int i = from[k];
          const int32_t old_base = (int32_t)p.row0[i] - ql, new_base = (int32_t)q.row0[k] - ql;
          for (int q0 = ql + (q.own(k) - 1) / bq * bq; q0 >= ql; q0 -= bq)
            q.xtiles.push_back({old_base, q.len[k], q0, (int32_t)p.col0[i], ql, 0, new_base, 0});
        }
      }
      int n_moves = 0;
      for (int k = 0; k < n_keep; ++k, ++n_moves) {
        h[mo.src + n_moves] = (int32_t)p.row0[from[k]]; h[mo.dst + n_moves] = (int32_t)q.row0[k]; h[mo.len + n_moves] = q.own(k);
      }
      if (q.ql > 0)      // every new chunk gets the query's rows (all copies are identical: take the first chunk's)
        for (const Chunk &ch : q.chunks) {
          h[mo.src + n_moves] = (int32_t)p.chunks[0].r0; h[mo.dst + n_moves] = (int32_t)ch.r0; h[mo.len + n_moves] = q.ql;
          ++n_moves;
        }
      // regrouping the survivors can produce a chunk with more tokens than any chunk before it
      PRISM_TRY(ensure_scratch(c, q, may_prune, n_cands, max_tiles));
      PRISM_TRY(upload_meta(c, q, mo, false));   // also carries src/dst/len, which sit between lastrow and tiles
      if (!c->offload) {   // offload mode: the host copy keeps its layout, dropped candidates are simply never fetched again
        PRISM_TRY(launch_compact(c->X[cur], c->X[cur ^ 1], c->d_meta + mo.src, c->d_meta + mo.dst, c->d_meta + mo.len, n_moves,
                                 m.hidden, s));
        cur ^= 1;
      }
      p = q;
      compacted = true;
    }
    if (timed) {
      PRISM_HIP(hipEventRecord(c->ev_t[3], s));
      PRISM_HIP(hipEventSynchronize(c->ev_t[3]));
      float ms = 0.f;
      PRISM_HIP(hipEventElapsedTime(&ms, c->ev_t[2], c->ev_t[3]));
      ms_checks += ms;
    }
    if (peek) {
      if (!terminated) {
        // second pass: the layer for the survivors.  If the pool is one chunk, the scratch still holds this layer's q, k
        // and V^T (in the layout before the prune) and the pass starts at the attention step, which writes its output
        // in the survivors' layout
        if (timed) PRISM_HIP(hipEventRecord(c->ev_layer[4 * l + 2], s));
        PRISM_TRY(run_layer(c, p, mo, c->X[cur], c->layer_buf[slot], false, true, false, false,
                            p.chunks.size() == 1 && (!compacted || !p.xtiles.empty())));
        p.xtiles.clear();
        if (timed) PRISM_HIP(hipEventRecord(c->ev_layer[4 * l + 3], s));
        second_pass[l] = true;
      }
      PRISM_TRY(release_slot());
    }
  }

  if (!terminated) {
    // ---- final scoring and top-K (Sec. 2.1)
    const int n_live = (int)p.live.size();
    const int k_out = std::min(K_rem, n_live);
    // (the last layer has scored every candidate from its gathered last-token state)
    PRISM_TRY(launch_topk(c->d_scores, n_live, k_out, c->d_top_pos, c->d_top_scores, s));
    PRISM_HIP(hipMemcpyAsync(h_scores, c->d_scores, (size_t)n_live * 4, hipMemcpyDeviceToHost, s));
    PRISM_HIP(hipMemcpyAsync(h_top_pos, c->d_top_pos, (size_t)k_out * 4, hipMemcpyDeviceToHost, s));
    PRISM_HIP(hipMemcpyAsync(h_top_scores, c->d_top_scores, (size_t)k_out * 4, hipMemcpyDeviceToHost, s));
    if (timed) PRISM_HIP(hipEventRecord(c->ev_t[1], s));
    PRISM_HIP(hipStreamSynchronize(s));
    for (int i = 0; i < k_out; ++i) { final_idx.push_back(p.live[h_top_pos[i]]); final_scores.push_back(h_top_scores[i]); }
    record_event(m.n_layers, n_live, p.live, false, 0, 0.0, 0.0, nullptr, nullptr);
  } else {
    if (timed) PRISM_HIP(hipEventRecord(c->ev_t[1], s));
    PRISM_HIP(hipStreamSynchronize(s));
  }
  if (c->two_slot) PRISM_HIP(hipStreamSynchronize(c->copy_stream));
  if (c->offload) {
    PRISM_HIP(hipStreamSynchronize(c->xin_stream));
    PRISM_HIP(hipStreamSynchronize(c->xout_stream));
  }

  int n_out = 0;
  for (size_t i = 0; i < early_idx.size() && n_out < Kc; ++i, ++n_out) { out_idx[n_out] = early_idx[i]; out_scores[n_out] = early_scores[i]; }
  for (size_t i = 0; i < final_idx.size() && n_out < Kc; ++i, ++n_out) { out_idx[n_out] = final_idx[i]; out_scores[n_out] = final_scores[i]; }
  *out_count = n_out;
  if (rep) {
    rep->n_events = std::min(n_events, rep->cap_events);
    float ms = 0.f;
    PRISM_HIP(hipEventElapsedTime(&ms, c->ev_t[0], c->ev_t[1]));
    rep->ms_total = ms;
    double ml = 0.0;
    for (int l = 0; l < layers_run; ++l) {
      PRISM_HIP(hipEventElapsedTime(&ms, c->ev_layer[4 * l], c->ev_layer[4 * l + 1]));
      ml += ms;
      if (second_pass[l]) {
        PRISM_HIP(hipEventElapsedTime(&ms, c->ev_layer[4 * l + 2], c->ev_layer[4 * l + 3]));
        ml += ms;
      }
    }
    rep->ms_layers = ml;
    double mx = 0.0;
    for (int l = 0; l < n_xfer_timed; ++l) {
      PRISM_HIP(hipEventElapsedTime(&ms, c->ev_xfer[2 * l], c->ev_xfer[2 * l + 1]));
      mx += ms;
    }
    rep->ms_transfers = mx;
    rep->ms_checks = ms_checks;
    rep->token_layers = token_layers;
    rep->peak_hbm_bytes = c->bytes_peak;
    rep->bytes_streamed = bytes_streamed;
    rep->layers_run = layers_run;
    rep->bytes_hidden_moved = c->bytes_hidden;
    rep->embed_rows_hit = c->embed_hit;
    rep->embed_rows_missed = c->embed_miss;
    for (int k = 0; k < PRISM_N_KINDS; ++k) { rep->kind_launches[k] = 0; rep->kind_ms[k] = 0.0; rep->kind_flops[k] = 0.0; }
    const bool detail = rep->span_cap > 0 && rep->span_kind && rep->span_rows && rep->span_ms && rep->span_flops;
    rep->n_spans = 0;
    for (const prism_ctx::Span &sp : c->spans) {
      PRISM_HIP(hipEventElapsedTime(&ms, sp.a, sp.b));
      rep->kind_launches[sp.kind] += 1;
      rep->kind_ms[sp.kind] += ms;
      rep->kind_flops[sp.kind] += sp.flops;
      if (detail && rep->n_spans < rep->span_cap) {
        const int i = rep->n_spans++;
        rep->span_kind[i] = sp.kind; rep->span_rows[i] = sp.rows; rep->span_ms[i] = ms; rep->span_flops[i] = sp.flops;
      }
    }
  }
  return PRISM_OK;
}

extern "C" int32_t prism_vt_column_of_key(int32_t p) { return p < 0 ? p : vt_column_of_key(p); }

// ------------------------------------------------------------------------------------------------ kernel-level entry points
namespace prism {

struct TmpDev {            // stream-ordered temporary: freed after the stream has drained
  void *p = nullptr;
  int alloc(size_t bytes) { hipError_t e = hipMalloc(&p, bytes ? bytes : 256); return e == hipSuccess ? PRISM_OK : hip_fail(e, "hipMalloc", __FILE__, __LINE__); }
  ~TmpDev() { if (p) (void)hipFree(p); }
};

}  // namespace prism

extern "C" int prism_op_embed(const int32_t *tokens, int32_t T, const void *table, int32_t hidden, int32_t dtype, float *X,
                              void *stream) {
  return launch_embed(tokens, T, table, hidden, dtype, X, (hipStream_t)stream);
}

extern "C" int prism_op_rmsnorm(const float *X, const void *gain, int32_t T, int32_t hidden, float eps, int32_t dtype,
                                void *out, void *stream) {
  return launch_rmsnorm(X, gain, T, hidden, eps, dtype, out, (hipStream_t)stream);
}

extern "C" int prism_op_gemm(int32_t dtype, int32_t epilogue, const void *A, const void *W, void *out, int32_t M, int32_t N,
                             int32_t K, void *stream) {
  PRISM_REQUIRE(epilogue >= PRISM_EPI_STORE && epilogue <= PRISM_EPI_STORE_F32, PRISM_EINVAL, "gemm: unknown epilogue %d", epilogue);
  PRISM_REQUIRE(dtype != PRISM_DTYPE_FP32 || epilogue != PRISM_EPI_STORE_F32, PRISM_EINVAL, "gemm: STORE_F32 is a bf16-mode epilogue");
  if (dtype == PRISM_DTYPE_FP32) return launch_gemm_fp32(epilogue, (const float *)A, (const float *)W, out, M, N, K, (hipStream_t)stream);
  PRISM_REQUIRE(is16(dtype), PRISM_EINVAL, "gemm: unknown dtype %d", dtype);
  return launch_gemm_16(dtype, epilogue, A, W, out, M, N, K, (hipStream_t)stream);
}

extern "C" int prism_op_qkv_finish(int32_t dtype, void *QKV, const int32_t *pos, int32_t max_pos, const void *q_gain,
                                   const void *k_gain, int32_t T, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                   float eps, float rope_base, int32_t qk_norm, void *QK, void *Vt, const int32_t *vt_col,
                                   int64_t vt_stride, void *stream) {
  PRISM_REQUIRE(max_pos > 0 && max_pos <= PRISM_MAX_SEQ && head_dim > 0 && head_dim % 2 == 0, PRISM_EINVAL, "qkv_finish: max_pos / head_dim");
  PRISM_REQUIRE(dtype == PRISM_DTYPE_FP32 || (is16(dtype) && QK && Vt && vt_col && vt_stride > 0), PRISM_EINVAL, "qkv_finish: 16-bit modes need QK, Vt, vt_col");
  hipStream_t s = (hipStream_t)stream;
  TmpDev tab;
  PRISM_TRY(tab.alloc((size_t)max_pos * (head_dim / 2) * sizeof(float2)));
  PRISM_TRY(launch_rope_table((float2 *)tab.p, max_pos, head_dim, rope_base, s));
  PRISM_TRY(launch_qk_finish(dtype, (float *)QKV, pos, q_gain, k_gain, T, n_q_heads, n_kv_heads, head_dim, eps, qk_norm,
                             (const float2 *)tab.p, QK, s));
  if (is16(dtype))
    PRISM_TRY(launch_v_finish(dtype, (const float *)QKV, T, n_q_heads, n_kv_heads, head_dim, Vt, vt_col, vt_stride, s));
  PRISM_HIP(hipStreamSynchronize(s));   // the table is freed on return
  return PRISM_OK;
}

extern "C" int prism_op_qkv_project(int32_t dtype, const void *Xn, const void *Wqkv, const int32_t *pos, int32_t max_pos,
                                    const void *q_gain, const void *k_gain, int32_t T, int32_t hidden, int32_t n_q_heads,
                                    int32_t n_kv_heads, int32_t head_dim, float eps, float rope_base, int32_t qk_norm,
                                    void *QK, void *Vt, const int32_t *vt_col, int64_t vt_stride, void *stream) {
  PRISM_REQUIRE(max_pos > 0 && max_pos <= PRISM_MAX_SEQ, PRISM_EINVAL, "qkv_project: max_pos");
  PRISM_REQUIRE(is16(dtype) && Xn && Wqkv && pos && QK && Vt && vt_col && vt_stride > 0 && T >= 0, PRISM_EINVAL, "qkv_project: bad arguments");
  PRISM_REQUIRE(gemm_16_qkv_supported(T, n_q_heads, n_kv_heads, head_dim, hidden), PRISM_EUNSUPPORTED,
                "qkv_project: needs head_dim 128, hidden a multiple of 64 and at least 256 tiles of 256 x 256 "
                "(use prism_op_gemm + prism_op_qkv_finish otherwise)");
  hipStream_t s = (hipStream_t)stream;
  TmpDev tab;
  PRISM_TRY(tab.alloc((size_t)max_pos * (head_dim / 2) * sizeof(float2)));
  PRISM_TRY(launch_rope_table((float2 *)tab.p, max_pos, head_dim, rope_base, s, true));
  QkvEpilogue e;
  e.pos = pos; e.vt_col = vt_col; e.q_gain = q_gain; e.k_gain = k_gain; e.rope_tab_t = (const float2 *)tab.p; e.rope_stride = max_pos;
  e.QK = QK; e.Vt = Vt; e.vt_stride = vt_stride; e.nq = n_q_heads; e.nkv = n_kv_heads; e.qk_norm = qk_norm; e.eps = eps;
  PRISM_TRY(launch_gemm_16_qkv(dtype, Xn, Wqkv, T, hidden, head_dim, e, s));
  PRISM_HIP(hipStreamSynchronize(s));   // the table is freed on return
  return PRISM_OK;
}

extern "C" int64_t prism_w4_bytes(int32_t N, int32_t K) { return N > 0 && K > 0 && K % 128 == 0 ? w4_blob_bytes(N, K) : -1; }

extern "C" int prism_op_quantize_w4(const void *W, int32_t N, int32_t K, void *blob, void *stream) {
  return launch_quantize_w4(W, N, K, blob, (hipStream_t)stream);
}

extern "C" int prism_op_dequantize_w4(const void *blob, int32_t N, int32_t K, int32_t dtype, void *out, void *stream) {
  return launch_dequantize_w4(blob, N, K, dtype, out, (hipStream_t)stream);
}

extern "C" int prism_op_attention(int32_t dtype, const void *QK, const void *Vt, int64_t vt_stride, const int32_t *cu,
                                  const int32_t *vt_col0, int32_t n_seqs, int32_t nq, int32_t nkv, int32_t hd, void *out,
                                  void *stream) {
  PRISM_REQUIRE(QK && cu && out && n_seqs >= 0 && nq > 0 && nkv > 0 && nq % nkv == 0, PRISM_EINVAL, "attention: bad arguments");
  hipStream_t s = (hipStream_t)stream;
  if (n_seqs == 0) return PRISM_OK;
  const int T = cu[n_seqs];
  for (int i = 0; i < n_seqs; ++i)
    PRISM_REQUIRE(cu[i + 1] > cu[i] && cu[i + 1] - cu[i] <= PRISM_MAX_SEQ, PRISM_EINVAL, "attention: sequence %d has bad length", i);
  const bool bf = is16(dtype);
  PRISM_REQUIRE(bf || dtype == PRISM_DTYPE_FP32, PRISM_EINVAL, "attention: unknown dtype %d", dtype);
  if (!bf) {
    std::vector<int32_t> pos(T);
    for (int i = 0; i < n_seqs; ++i) for (int t = cu[i]; t < cu[i + 1]; ++t) pos[t] = t - cu[i];
    TmpDev d_pos;
    PRISM_TRY(d_pos.alloc((size_t)T * 4));
    PRISM_HIP(hipMemcpyAsync(d_pos.p, pos.data(), (size_t)T * 4, hipMemcpyHostToDevice, s));
    PRISM_TRY(launch_attention_fp32((const float *)QK, (const int32_t *)d_pos.p, T, nq, nkv, hd, (float *)out, s));
    PRISM_HIP(hipStreamSynchronize(s));
    return PRISM_OK;
  }
  PRISM_REQUIRE(attention_16_supported(nq, nkv, hd), PRISM_EUNSUPPORTED, "attention bf16: unsupported head shape");
  PRISM_REQUIRE(Vt && vt_col0 && vt_stride > 0, PRISM_EINVAL, "attention bf16: Vt / vt_col0 missing");
  std::vector<AttnTile> tiles;
  const int bq = attention_16_block_queries(nq, nkv);
  for (int i = 0; i < n_seqs; ++i) {
    const int L = cu[i + 1] - cu[i];
    PRISM_REQUIRE(vt_col0[i] >= 0 && vt_col0[i] % 64 == 0 && vt_col0[i] + round_up(L, 64) <= vt_stride, PRISM_EINVAL,
                  "attention bf16: sequence %d: V^T columns must start at a multiple of 64 and fit the row stride", i);
    for (int q0 = L > 0 ? (L - 1) / bq * bq : -1; q0 >= 0; q0 -= bq) tiles.push_back({cu[i], L, q0, vt_col0[i], 0, 0, cu[i], 0});
  }
  TmpDev d_tiles;
  PRISM_TRY(d_tiles.alloc(tiles.size() * sizeof(AttnTile)));
  PRISM_HIP(hipMemcpyAsync(d_tiles.p, tiles.data(), tiles.size() * sizeof(AttnTile), hipMemcpyHostToDevice, s));
  PRISM_TRY(launch_attention_16(dtype, QK, Vt, vt_stride, (const AttnTile *)d_tiles.p, (int)tiles.size(), T, nq, nkv, hd, out, s));
  PRISM_HIP(hipStreamSynchronize(s));   // temporaries are released on return
  return PRISM_OK;
}

extern "C" int prism_op_score(const float *X, const int32_t *last_row, int32_t n_seqs, int32_t hidden, const void *final_norm,
                              const void *w_yes, const void *w_no, int32_t dtype, float eps, float *scores, void *stream) {
  return launch_score(X, last_row, n_seqs, hidden, final_norm, w_yes, w_no, dtype, eps, scores, (hipStream_t)stream);
}

extern "C" int prism_op_route(const float *scores, int32_t n, int32_t K_rem, int32_t n_clusters, float tau, int8_t *fate,
                              double *stats, void *stream) {
  PRISM_REQUIRE(n >= 1 && n <= PRISM_MAX_CANDS && n_clusters >= 2 && n_clusters <= PRISM_MAX_CLUSTERS, PRISM_EINVAL,
                "route: n = %d or n_clusters = %d out of range", n, n_clusters);
  hipStream_t s = (hipStream_t)stream;
  TmpDev ws;
  PRISM_TRY(ws.alloc(route_workspace_bytes(n, n_clusters)));
  PRISM_TRY(launch_route(scores, n, K_rem, n_clusters, tau, fate, stats, ws.p, s));
  PRISM_HIP(hipStreamSynchronize(s));
  return PRISM_OK;
}

extern "C" int prism_op_compact(const float *X_src, float *X_dst, const int32_t *src_start, const int32_t *dst_start,
                                const int32_t *len, int32_t n_keep, int32_t hidden, void *stream) {
  return launch_compact(X_src, X_dst, src_start, dst_start, len, n_keep, hidden, (hipStream_t)stream);
}

extern "C" int prism_op_topk(const float *scores, int32_t n, int32_t K, int32_t *out_pos, float *out_scores, void *stream) {
  PRISM_REQUIRE(n <= PRISM_MAX_CANDS && K <= n, PRISM_EINVAL, "topk: n = %d, K = %d", n, K);
  return launch_topk(scores, n, K, out_pos, out_scores, (hipStream_t)stream);
}
