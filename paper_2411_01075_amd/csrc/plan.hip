// Host-side planner: how the global batch and the training state are divided over the GPUs of a cluster
// (Sec. 3.4 "Optimizer": optimization formulation, dynamic-programming solution, training-state partition;
// supplementary Algorithm 1).  Plain C++ on the host; nothing here touches a device.
#include "common.h"
#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <vector>

using namespace cephalo;

namespace {

constexpr double kInf = std::numeric_limits<double>::infinity();

int check_plan_args(int32_t n, const cephalo_gpu_perf* g, int32_t B, const cephalo_cluster_model* c) {
  if (n <= 0 || B <= 0) return fail(CEPHALO_EINVAL, "plan: %d GPUs and batch %d must be positive", n, B);
  if (!g || !c) return fail(CEPHALO_EINVAL, "plan: null model");
  if ((int64_t)n * B * B > ((int64_t)1 << 31)) return fail(CEPHALO_EUNSUPPORTED, "plan: table of %d x %d x %d entries is too large", n, B, B);
  for (int i = 0; i < n; ++i) {
    if (!g[i].t_fwd || !g[i].t_bwd) return fail(CEPHALO_EINVAL, "plan: GPU %d has no latency table", i);
    if (g[i].max_m < 1) return fail(CEPHALO_EINVAL, "plan: GPU %d: latency tables must cover micro-batch size 1", i);
    if (!(g[i].mem_cap > 0)) return fail(CEPHALO_EINVAL, "plan: GPU %d: memory capacity must be positive", i);
  }
  if (!(c->mem_per_sample >= 0) || !(c->mem_base >= 0) || !(c->state_bytes >= 0))
    return fail(CEPHALO_EINVAL, "plan: memory model and training-state size must be non-negative");
  return CEPHALO_OK;
}

// latency of one micro-batch of size m: the profiled table, extended linearly through its last two points
double latency(const double* table, int max_m, int m) {
  if (m <= max_m) return table[m];
  const double slope = max_m >= 2 ? table[max_m] - table[max_m - 1] : table[1];
  return table[max_m] + slope * (m - max_m);
}

}  // namespace

extern "C" int cephalo_plan_compute(int32_t n, const cephalo_gpu_perf* gpus, int32_t B, const cephalo_cluster_model* c,
                                    int32_t* m_out, int32_t* l_out, double* latency_out) {
  {
    const int rc = check_plan_args(n, gpus, B, c);
    if (rc != CEPHALO_OK) return rc;
  }
  if (!m_out || !l_out) return fail(CEPHALO_EINVAL, "plan: null output");
  const double state_even = c->state_bytes / n;       // an even share of the training state
  auto mem = [&](int m) { return c->mem_base + c->mem_per_sample * m; };
  // D[i][j][k]: least achievable layer latency for the first i GPUs to take batch j with micro-batch sizes summing to k
  const size_t stride_i = (size_t)(B + 1) * (B + 1), stride_j = (size_t)(B + 1);
  std::vector<double> D((size_t)(n + 1) * stride_i, kInf);
  std::vector<int32_t> choice_m((size_t)(n + 1) * stride_i, 0), choice_l((size_t)(n + 1) * stride_i, 0);
  D[0] = 0.0;
  for (int i = 1; i <= n; ++i) {
    const cephalo_gpu_perf& g = gpus[i - 1];
    for (int j = 1; j <= B; ++j)
      for (int k = 1; k <= j; ++k) {
        double best = kInf;
        int bm = 0, bl = 0;
        for (int m = 1; m <= k; ++m) {
          if (mem(m) > g.mem_cap) break;              // compute memory alone must fit (and it grows with m)
          const bool uneven = mem(m) + state_even > g.mem_cap;    // then this GPU cannot hold an even share of the state
          const double ag = uneven ? c->allgather_uneven : c->allgather, rs = uneven ? c->reducescatter_uneven : c->reducescatter;
          const double tf1 = latency(g.t_fwd, g.max_m, m), tb1 = latency(g.t_bwd, g.max_m, m);
          for (int l = 1; l * m <= j; ++l) {
            const double prev = D[(size_t)(i - 1) * stride_i + (size_t)(j - l * m) * stride_j + (k - m)];
            if (prev == kInf) continue;
            const double t = std::max(l * tf1, ag) + std::max(l * tb1, ag + rs);
            const double r = std::max(prev, t);
            if (r < best) { best = r; bm = m; bl = l; }
          }
        }
        const size_t at = (size_t)i * stride_i + (size_t)j * stride_j + k;
        D[at] = best; choice_m[at] = bm; choice_l[at] = bl;
      }
  }
  // the total micro-batch size k fixes the aggregate compute memory: keep the k whose cluster-wide memory fits
  double cap_sum = 0.0;
  for (int i = 0; i < n; ++i) cap_sum += gpus[i].mem_cap;
  double best = kInf;
  int best_k = -1;
  for (int k = 1; k <= B; ++k) {
    const double aggregate = c->state_bytes + n * c->mem_base + c->mem_per_sample * k;
    if (aggregate > cap_sum) continue;
    const double v = D[(size_t)n * stride_i + (size_t)B * stride_j + k];
    if (v < best) { best = v; best_k = k; }
  }
  if (best_k < 0) return fail(CEPHALO_EUNSUPPORTED, "plan: no assignment of batch %d to %d GPUs fits in memory", B, n);
  int j = B, k = best_k;
  for (int i = n; i >= 1; --i) {
    const size_t at = (size_t)i * stride_i + (size_t)j * stride_j + k;
    m_out[i - 1] = choice_m[at]; l_out[i - 1] = choice_l[at];
    j -= choice_m[at] * choice_l[at]; k -= choice_m[at];
  }
  if (latency_out) *latency_out = best;
  return CEPHALO_OK;
}

extern "C" int cephalo_plan_state(int32_t n, const cephalo_gpu_perf* gpus, const int32_t* m, const cephalo_cluster_model* c,
                                  double* ratio_out) {
  if (n <= 0 || !gpus || !m || !c || !ratio_out) return fail(CEPHALO_EINVAL, "plan_state: bad arguments");
  // Start from each GPU's compute memory and hand the training state to whichever GPU has the lowest memory
  // utilisation, raising it until it meets the next lowest, and so on (a water-filling over the utilisations).
  std::vector<double> used(n), cap(n), state(n, 0.0);
  for (int i = 0; i < n; ++i) {
    if (!(gpus[i].mem_cap > 0) || m[i] < 1) return fail(CEPHALO_EINVAL, "plan_state: GPU %d: capacity and micro-batch size must be positive", i);
    cap[i] = gpus[i].mem_cap;
    used[i] = c->mem_base + c->mem_per_sample * m[i];
  }
  std::vector<int> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::sort(order.begin(), order.end(), [&](int a, int b) { return used[a] / cap[a] < used[b] / cap[b]; });
  double remaining = c->state_bytes, level = used[order[0]] / cap[order[0]], cap_active = 0.0;
  for (int p = 0; p < n && remaining > 0; ++p) {
    cap_active += cap[order[p]];                      // GPUs order[0..p] now sit at the common level
    const double next = p + 1 < n ? used[order[p + 1]] / cap[order[p + 1]] : kInf;
    const double need = (next - level) * cap_active;  // bytes that lift all of them to the next GPU's utilisation
    const double give = std::min(need, remaining);
    level += give / cap_active;
    remaining -= give;
  }
  double total = 0.0;
  for (int i = 0; i < n; ++i) {
    state[i] = std::max(0.0, level * cap[i] - used[i]);
    total += state[i];
  }
  for (int i = 0; i < n; ++i) ratio_out[i] = total > 0 ? state[i] / total : 1.0 / n;
  return CEPHALO_OK;
}

extern "C" int cephalo_plan_units(int32_t n, const double* ratio, int32_t units, int64_t L, int64_t* offset_out, int64_t* len_out,
                                  int32_t* n_even_out) {
  if (n <= 0 || units <= 0 || L <= 0 || !ratio || !offset_out || !len_out) return fail(CEPHALO_EINVAL, "plan_units: bad arguments");
  double sum = 0.0;
  for (int i = 0; i < n; ++i) {
    if (!(ratio[i] >= 0.0)) return fail(CEPHALO_EINVAL, "plan_units: ratio[%d] = %g is negative", i, ratio[i]);
    sum += ratio[i];
  }
  if (!(std::fabs(sum - 1.0) <= 1e-9)) return fail(CEPHALO_EINVAL, "plan_units: the ratios sum to %.12g, not 1", sum);
  const int64_t total = (int64_t)units * L;
  // whole-element targets: floor, then the largest remainders take what is left (ties to the lower index)
  std::vector<int64_t> target(n);
  std::vector<double> rem(n);
  int64_t given = 0;
  for (int i = 0; i < n; ++i) {
    const double want = ratio[i] / sum * (double)total;
    target[i] = std::min((int64_t)std::floor(want), total);
    rem[i] = want - (double)target[i];
    given += target[i];
  }
  std::vector<int> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return rem[a] > rem[b]; });
  for (int p = 0; given < total; p = (p + 1) % n) { ++target[order[p]]; ++given; }
  // even shares of one unit, and how many even units every target can carry
  std::vector<int64_t> even_off(n + 1);
  for (int i = 0; i <= n; ++i) even_off[i] = (int64_t)((__int128)i * L / n);
  int64_t n_even = units;
  for (int i = 0; i < n; ++i) {
    const int64_t share = even_off[i + 1] - even_off[i];
    if (share > 0) n_even = std::min(n_even, target[i] / share);
  }
  for (int64_t u = 0; u < n_even; ++u)
    for (int i = 0; i < n; ++i) {
      offset_out[u * n + i] = even_off[i];
      len_out[u * n + i] = even_off[i + 1] - even_off[i];
    }
  // the remaining units as one flat run divided in GPU order
  int64_t start = 0;                                   // position in the run, in elements
  for (int i = 0; i < n; ++i) {
    const int64_t lack = target[i] - n_even * (even_off[i + 1] - even_off[i]);
    const int64_t end = start + lack;
    for (int64_t u = n_even; u < units; ++u) {
      const int64_t u0 = (u - n_even) * L, u1 = u0 + L;
      const int64_t lo = std::max(start, u0), hi = std::min(end, u1);
      offset_out[u * n + i] = hi > lo ? lo - u0 : std::min(std::max(start - u0, (int64_t)0), L);
      len_out[u * n + i] = hi > lo ? hi - lo : 0;
    }
    start = end;
  }
  if (n_even_out) *n_even_out = (int32_t)n_even;
  return CEPHALO_OK;
}
