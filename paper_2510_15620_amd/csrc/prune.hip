// One pruning check on the live candidates' provisional scores (paper Sec. 4.1, worked example
// Sec. 4.5): dispersion gate on the coefficient of variation, K-Means of the scalar scores, routing
// around the boundary cluster.
//
// The paper runs K-Means on the CPU (~1 ms); here it is one workgroup on the device so the scores
// never leave HBM before the decision.  K-Means of scalars is solved exactly: every optimum of the
// within-cluster sum of squares is a partition of the ranked scores into consecutive runs, so a
// dynamic programme over split positions finds it, with no seed and no iteration count.
//
// All decisions are taken in fp64 with a fixed operation order (sequential sums, no fused
// multiply-add: this file is compiled with -ffp-contract=off), so that a host implementation that
// follows the same order reaches the same bits.
#include <mutex>

#include "common.h"

namespace prism {

struct RouteWs {
  double *ranked, *P, *Q, *E0, *E1;
  int32_t *order, *arg;  // arg: [k+1][n+1]
};

__device__ __forceinline__ double run_cost(const double *P, const double *Q, int i, int j) {
  const double sp = P[j] - P[i];
  return (Q[j] - Q[i]) - sp * sp / (double)(j - i);
}

__global__ __launch_bounds__(1024) void route_kernel(const float *__restrict__ scores, int n, int K_rem, int k_req,
                                                     float tau, int8_t *__restrict__ fate, double *__restrict__ stats,
                                                     RouteWs ws) {
  __shared__ double sh_val[1024];
  __shared__ int sh_idx[1024];
  __shared__ int sh_flag;      // 1: clustering runs
  __shared__ int sh_distinct;
  __shared__ int sh_splits[PRISM_MAX_CLUSTERS + 1];
  __shared__ double sh_means[PRISM_MAX_CLUSTERS];
  __shared__ int sh_k, sh_b;
  const int tid = threadIdx.x, nt = blockDim.x;

  for (int i = tid; i < n; i += nt) fate[i] = PRISM_FATE_DEFERRED;
  if (tid == 0) {
    // mean and population std, sequential in index order
    double tot = 0.0;
    for (int i = 0; i < n; ++i) tot = tot + (double)scores[i];
    const double mean = n > 0 ? tot / (double)n : 0.0;
    double acc = 0.0;
    for (int i = 0; i < n; ++i) {
      const double d = (double)scores[i] - mean;
      acc = acc + d * d;
    }
    const double sd = n > 0 ? sqrt(acc / (double)n) : 0.0;
    const int gate = (n > K_rem) && (sd > (double)tau * fabs(mean));   // CV > tau, division-free
    stats[0] = mean;
    stats[1] = sd;
    stats[2] = (double)gate;
    stats[3] = 0.0;
    sh_flag = gate;
    sh_distinct = 0;
  }
  __syncthreads();
  if (!sh_flag) return;

  // rank: score descending, lower index first on ties
  for (int i = tid; i < n; i += nt) {
    const float si = scores[i];
    int r = 0;
    for (int j = 0; j < n; ++j) {
      const float sj = scores[j];
      r += (sj > si) || (sj == si && j < i);
    }
    ws.order[r] = i;
    ws.ranked[r] = (double)si;
  }
  __syncthreads();
  {
    int local = 0;
    for (int r = tid; r < n; r += nt) local += (r == 0) || (ws.ranked[r] != ws.ranked[r - 1]);
    if (local) atomicAdd(&sh_distinct, local);
  }
  __syncthreads();
  if (tid == 0) {
    int k = k_req < sh_distinct ? k_req : sh_distinct;
    sh_k = k;
    if (k <= 1) sh_flag = 0;
    // sequential prefix sums of x and x^2
    ws.P[0] = 0.0;
    ws.Q[0] = 0.0;
    for (int i = 0; i < n; ++i) {
      const double x = ws.ranked[i];
      ws.P[i + 1] = ws.P[i] + x;
      ws.Q[i + 1] = ws.Q[i] + x * x;
    }
  }
  __syncthreads();
  if (!sh_flag) return;
  const int k = sh_k;

  // E[m][i]: best cost of cutting ranked[i:] into m runs.  E[1][i] = cost(i, n).
  double *Eprev = ws.E0, *Ecur = ws.E1;
  for (int i = tid; i < n; i += nt) Eprev[i] = run_cost(ws.P, ws.Q, i, n);
  __syncthreads();
  for (int m = 2; m <= k; ++m) {
    int32_t *arg = ws.arg + (int64_t)m * (n + 1);
    if (m < k) {
      for (int i = tid; i <= n - m; i += nt) {
        double best = INFINITY;
        int best_s = -1;
        for (int s = i + 1; s <= n - (m - 1); ++s) {
          const double c = run_cost(ws.P, ws.Q, i, s) + Eprev[s];
          if (c < best) { best = c; best_s = s; }
        }
        Ecur[i] = best;
        arg[i] = best_s;
      }
    } else {
      // last stage is only read at i = 0: spread the candidates for s over the workgroup and
      // reduce to the smallest cost, smallest s among equals
      double best = INFINITY;
      int best_s = 0x7fffffff;
      for (int s = 1 + tid; s <= n - (m - 1); s += nt) {
        const double c = run_cost(ws.P, ws.Q, 0, s) + Eprev[s];
        if (c < best) { best = c; best_s = s; }
      }
      sh_val[tid] = best;
      sh_idx[tid] = best_s;
      __syncthreads();
      for (int off = nt >> 1; off > 0; off >>= 1) {
        if (tid < off) {
          const double c = sh_val[tid + off];
          const int s = sh_idx[tid + off];
          if (c < sh_val[tid] || (c == sh_val[tid] && s < sh_idx[tid])) { sh_val[tid] = c; sh_idx[tid] = s; }
        }
        __syncthreads();
      }
      if (tid == 0) arg[0] = sh_idx[0];
    }
    __syncthreads();
    double *t = Eprev; Eprev = Ecur; Ecur = t;
  }

  if (tid == 0) {
    // split positions, cluster means (sequential sums), boundary cluster
    sh_splits[0] = 0;
    int i = 0;
    for (int m = k, c = 1; m >= 2; --m, ++c) {
      i = ws.arg[(int64_t)m * (n + 1) + i];
      sh_splits[c] = i;
    }
    sh_splits[k] = n;
    int b = 0;
    for (int c = 0; c < k; ++c) {
      double tot = 0.0;
      for (int r = sh_splits[c]; r < sh_splits[c + 1]; ++r) tot = tot + ws.ranked[r];
      sh_means[c] = tot / (double)(sh_splits[c + 1] - sh_splits[c]);
      if (sh_splits[c] <= K_rem - 1 && K_rem - 1 < sh_splits[c + 1]) b = c;
    }
    sh_b = b;
    stats[3] = (double)k;
  }
  __syncthreads();
  const double mb = sh_means[sh_b];
  for (int r = tid; r < n; r += nt) {
    int c = 0;
    while (r >= sh_splits[c + 1]) ++c;
    const double mc = sh_means[c];
    fate[ws.order[r]] = mc > mb ? PRISM_FATE_SELECTED : (mc < mb ? PRISM_FATE_DROPPED : PRISM_FATE_DEFERRED);
  }
}

static RouteWs carve(void *workspace, int n, int k) {
  RouteWs ws;
  char *p = (char *)workspace;
  const size_t dn = (size_t)round_up((n + 1) * sizeof(double), 256);
  ws.ranked = (double *)p; p += dn;
  ws.P = (double *)p; p += dn;
  ws.Q = (double *)p; p += dn;
  ws.E0 = (double *)p; p += dn;
  ws.E1 = (double *)p; p += dn;
  ws.order = (int32_t *)p; p += round_up((n + 1) * sizeof(int32_t), 256);
  ws.arg = (int32_t *)p;
  (void)k;
  return ws;
}

size_t route_workspace_bytes(int n, int k) {
  return 5 * (size_t)round_up((n + 1) * sizeof(double), 256) + (size_t)round_up((n + 1) * sizeof(int32_t), 256) +
         (size_t)round_up((size_t)(k + 1) * (n + 1) * sizeof(int32_t), 256);
}

int launch_route(const float *scores, int n, int K_rem, int n_clusters, float tau, int8_t *fate, double *stats,
                 void *workspace, hipStream_t s) {
  PRISM_REQUIRE(scores && fate && stats && workspace, PRISM_EINVAL, "route: null argument");
  PRISM_REQUIRE(n >= 1 && n <= PRISM_MAX_CANDS, PRISM_EINVAL, "route: n = %d outside 1..%d", n, PRISM_MAX_CANDS);
  PRISM_REQUIRE(n_clusters >= 2 && n_clusters <= PRISM_MAX_CLUSTERS, PRISM_EINVAL, "route: n_clusters = %d outside 2..%d",
                n_clusters, PRISM_MAX_CLUSTERS);
  PRISM_REQUIRE(K_rem >= 1 && tau >= 0.f, PRISM_EINVAL, "route: K_rem = %d, tau = %g", K_rem, (double)tau);
  route_kernel<<<1, 1024, 0, s>>>(scores, n, K_rem, n_clusters, tau, fate, stats, carve(workspace, n, n_clusters));
  PRISM_HIP(hipGetLastError());
  return PRISM_OK;
}

// ---- the same check for callers that cannot allocate --------------------------------------------------------------
// The kernel's workspace (ranked scores, prefix sums, two cost rows, rank order, the argmin table) lives in a
// file-scope device array sized for the largest check the library accepts.  Every device that loads the library holds
// its own copy at its own address, looked up once per device.  The kernel writes every workspace entry before it reads
// it, so nothing has to be cleared between calls; calls that overlap on one device share the array and race.
static constexpr size_t up256(size_t v) { return (v + 255) / 256 * 256; }
static constexpr size_t kRouteScratchBytes =
    5 * up256((PRISM_MAX_CANDS + 1) * sizeof(double)) + up256((PRISM_MAX_CANDS + 1) * sizeof(int32_t)) +
    up256((size_t)(PRISM_MAX_CLUSTERS + 1) * (PRISM_MAX_CANDS + 1) * sizeof(int32_t));
static __device__ __align__(256) unsigned char scratch[kRouteScratchBytes];

static constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (the array's name is only a host-side handle).
static int scratch_of_current_device(void **out) {
  int dev = -1;
  PRISM_HIP(hipGetDevice(&dev));
  PRISM_REQUIRE(dev >= 0 && dev < kMaxDevices, PRISM_EUNSUPPORTED, "route: device ordinal %d not supported", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    PRISM_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    PRISM_REQUIRE(p, PRISM_EHIP, "route: the static workspace has no device address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return PRISM_OK;
}

}  // namespace prism

extern "C" int prism_op_route_static(const float *scores, int32_t n, int32_t K_rem, int32_t n_clusters, float tau,
                                     int8_t *fate, double *stats, void *stream) {
  using namespace prism;
  PRISM_REQUIRE(n >= 1 && n <= PRISM_MAX_CANDS, PRISM_EINVAL, "route (static workspace): n = %d outside 1..%d", n, PRISM_MAX_CANDS);
  PRISM_REQUIRE(n_clusters >= 2 && n_clusters <= PRISM_MAX_CLUSTERS, PRISM_EINVAL,
                "route (static workspace): n_clusters = %d outside 2..%d", n_clusters, PRISM_MAX_CLUSTERS);
  PRISM_REQUIRE(route_workspace_bytes(n, n_clusters) <= kRouteScratchBytes, PRISM_EINVAL,
                "route (static workspace): the check needs more than the %zu bytes of the static workspace", kRouteScratchBytes);
  void *ws = nullptr;
  PRISM_TRY(scratch_of_current_device(&ws));
  return launch_route(scores, n, K_rem, n_clusters, tau, fate, stats, ws, (hipStream_t)stream);
}
