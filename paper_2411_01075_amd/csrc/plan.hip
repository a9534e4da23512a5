// Host-side planner: how the global batch and the training state are divided over the GPUs of a cluster
// (Sec. 3.4 "Optimizer": optimization formulation, dynamic-programming solution, training-state partition;
// supplementary Algorithm 1).  Plain C++ on the host; nothing here touches a device.
#include "common.h"
#include <algorithm>
#include <cmath>
#include <limits>
#include <new>
#include <numeric>
#include <vector>

using namespace cephalo;

namespace {

constexpr double kInf = std::numeric_limits<double>::infinity();

int check_plan_args(int32_t n, const cephalo_gpu_perf* g, int32_t B, const cephalo_cluster_model* c) {
  if (n <= 0 || B <= 0) return fail(CEPHALO_EINVAL, "plan: %d GPUs and batch %d must be positive", n, B);
  if (!g || !c) return fail(CEPHALO_EINVAL, "plan: null model");
  if ((int64_t)n * B > ((int64_t)1 << 26)) return fail(CEPHALO_EUNSUPPORTED, "plan: %d GPUs x batch %d is beyond the planner's tables (2^26 entries)", n, B);
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

// One way for a GPU to take a share: l micro-batches of m samples, and what a layer then costs on that GPU.
struct Option {
  double t;      // max(l T_f(m), AG') + max(l T_b(m), AG' + RS')
  int32_t m, l;
};

// The compute partition as a bottleneck problem.  The objective is the largest per-GPU latency, so the optimum is one
// of the finitely many option latencies, and "is there a plan in which no GPU exceeds tau" is monotone in tau.  For a
// given tau a GPU's admissible options reduce to cost(b) = the smallest micro-batch size with which it can take a
// share of b samples within tau; the cluster-wide memory (constraint III) grows with the sum of the micro-batch sizes
// and with nothing else, so a plan exists iff the least sum over all ways to split the batch fits:
//   least[i][j] = min over b of least[i-1][j-b] + cost_i(b)          (first i GPUs take j samples between them)
// The threshold is found by bisection over the sorted option latencies.  O(N B^2) per probe, O(log(N B log B))
// probes, tables of N x B entries (the supplementary algorithm's table has N x B x B and its loops N B^4 steps).
struct Planner {
  int n, B;
  const cephalo_gpu_perf* gpus;
  const cephalo_cluster_model* c;
  std::vector<std::vector<Option>> options;      // per GPU, every (m, l) whose compute memory fits that GPU
  std::vector<int32_t> least, pick_m, pick_l;    // [(n + 1) x (B + 1)]; least = kNone where no split exists
  std::vector<int32_t> cost, cost_l;             // [B + 1], of the GPU at hand
  double cap_sum = 0.0;
  static constexpr int32_t kNone = std::numeric_limits<int32_t>::max();

  Planner(int n_, int B_, const cephalo_gpu_perf* g, const cephalo_cluster_model* c_) : n(n_), B(B_), gpus(g), c(c_) {
    const double state_even = c->state_bytes / n;
    options.resize(n);
    for (int i = 0; i < n; ++i) {
      cap_sum += g[i].mem_cap;
      for (int m = 1; m <= B; ++m) {
        const double mem = c->mem_base + c->mem_per_sample * m;
        if (mem > g[i].mem_cap) break;                          // constraint II; the compute memory grows with m
        const bool uneven = mem + state_even > g[i].mem_cap;    // this GPU cannot hold an even share of the state as well
        const double ag = uneven ? c->allgather_uneven : c->allgather, rs = uneven ? c->reducescatter_uneven : c->reducescatter;
        const double tf = latency(g[i].t_fwd, g[i].max_m, m), tb = latency(g[i].t_bwd, g[i].max_m, m);
        for (int l = 1; l * m <= B; ++l) options[i].push_back({std::max(l * tf, ag) + std::max(l * tb, ag + rs), m, l});
      }
    }
    least.assign((size_t)(n + 1) * (B + 1), kNone);
    pick_m.assign(least.size(), 0);
    pick_l.assign(least.size(), 0);
    cost.resize(B + 1);
    cost_l.resize(B + 1);
  }
  bool memory_fits(int64_t sum_m) const { return !(c->state_bytes + n * c->mem_base + c->mem_per_sample * (double)sum_m > cap_sum); }

  // Is there a plan with every GPU within tau?  Leaves the tables filled for read_plan().
  bool feasible(double tau) {
    std::fill(least.begin(), least.end(), kNone);
    least[0] = 0;
    for (int i = 1; i <= n; ++i) {
      std::fill(cost.begin(), cost.end(), kNone);
      for (const Option& o : options[i - 1]) {
        const int b = o.m * o.l;
        if (o.t <= tau && o.m < cost[b]) { cost[b] = o.m; cost_l[b] = o.l; }
      }
      const int32_t* prev = &least[(size_t)(i - 1) * (B + 1)];
      int32_t* cur = &least[(size_t)i * (B + 1)];
      for (int j = i; j <= B - (n - i); ++j) {        // every GPU takes at least one sample
        int32_t best = kNone, bm = 0, bl = 0;
        for (int b = 1; b <= j - (i - 1); ++b) {
          if (cost[b] == kNone || prev[j - b] == kNone) continue;
          const int32_t v = prev[j - b] + cost[b];
          if (v < best) { best = v; bm = cost[b]; bl = cost_l[b]; }
        }
        cur[j] = best;
        pick_m[(size_t)i * (B + 1) + j] = bm;
        pick_l[(size_t)i * (B + 1) + j] = bl;
      }
    }
    const int32_t total = least[(size_t)n * (B + 1) + B];
    return total != kNone && memory_fits(total);
  }
  void read_plan(int32_t* m_out, int32_t* l_out) const {
    int j = B;
    for (int i = n; i >= 1; --i) {
      const size_t at = (size_t)i * (B + 1) + j;
      m_out[i - 1] = pick_m[at];
      l_out[i - 1] = pick_l[at];
      j -= pick_m[at] * pick_l[at];
    }
  }
};

}  // namespace

extern "C" int cephalo_plan_compute(int32_t n, const cephalo_gpu_perf* gpus, int32_t B, const cephalo_cluster_model* c,
                                    int32_t* m_out, int32_t* l_out, double* latency_out) {
  {
    const int rc = check_plan_args(n, gpus, B, c);
    if (rc != CEPHALO_OK) return rc;
  }
  if (!m_out || !l_out) return fail(CEPHALO_EINVAL, "plan: null output");
  if (B < n) return fail(CEPHALO_EUNSUPPORTED, "plan: batch %d cannot give each of %d GPUs a sample", B, n);
  try {
    Planner P(n, B, gpus, c);
    std::vector<double> taus;
    for (const auto& v : P.options)
      for (const Option& o : v) taus.push_back(o.t);
    std::sort(taus.begin(), taus.end());
    taus.erase(std::unique(taus.begin(), taus.end()), taus.end());
    if (taus.empty() || !P.feasible(taus.back()))
      return fail(CEPHALO_EUNSUPPORTED, "plan: no assignment of batch %d to %d GPUs fits in memory", B, n);
    size_t lo = 0, hi = taus.size() - 1;            // the least feasible threshold lies in [lo, hi]
    while (lo < hi) {
      const size_t mid = lo + (hi - lo) / 2;
      if (P.feasible(taus[mid])) hi = mid; else lo = mid + 1;
    }
    P.feasible(taus[lo]);                           // (the tables of the answer)
    P.read_plan(m_out, l_out);
    if (latency_out) *latency_out = taus[lo];
  } catch (const std::bad_alloc&) {
    return fail(CEPHALO_EUNSUPPORTED, "plan: out of host memory for %d GPUs x batch %d", n, B);
  }
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
