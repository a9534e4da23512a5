// A whole GPT-style stack on one GPU's batch share, in the layered order (every micro-batch passes
// through a layer before the next layer runs, forward and backward): token + position embedding,
// L layers, final LayerNorm, tied LM head with mean cross-entropy, and the matching backward with the
// parameter-gradient pass of every layer taken once over all b*S tokens.
#include <cstring>
#include "layer_impl.h"

namespace cephalo {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ int clamp_id(int id, int V) { return id < 0 ? 0 : (id >= V ? V - 1 : id); }

// x0[t] = wte[id[t]] + wpe[t % S] (wpe null: no learned positions); one wavefront per token.  Ids outside [0, V) are clamped.
template <typename T>
__global__ void __launch_bounds__(kThreads)
embed_fwd_kernel(const int* __restrict__ ids, const T* __restrict__ wte, const T* __restrict__ wpe, float* __restrict__ x0,
                 int tokens, int S, int H, int V) {
  constexpr int VN = Vec<T>::N;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (t >= tokens) return;
  const T* e = wte + (int64_t)clamp_id(ids[t], V) * H;
  const T* p = wpe ? wpe + (int64_t)(t % S) * H : nullptr;
  for (int v = lane; v < H / VN; v += 64) {
    float a[VN], b[VN];
    load_vec<T>(e + v * VN, a);
    if (p) {
      load_vec<T>(p + v * VN, b);
#pragma unroll
      for (int i = 0; i < VN; ++i) a[i] += b[i];
    }
#pragma unroll
    for (int i = 0; i < VN; ++i) x0[(int64_t)t * H + v * VN + i] = a[i];
  }
}

__device__ __forceinline__ float block_reduce(float v, bool is_max, float* red) {
  v = is_max ? wave_max(v) : wave_sum(v);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  const float a = red[0], b = red[1], c = red[2], d = red[3];
  return is_max ? fmaxf(fmaxf(a, b), fmaxf(c, d)) : (a + b) + (c + d);
}

// One block per token row of the fp32 logits [rows, ld] (V valid columns).  loss[row] = logsumexp - logit[target];
// dlogits[row] = coef * (softmax - onehot(target)) in the activation type, columns V..ld-1 set to zero.
// Two passes over the row: a running (max, sum of exp) pair per thread, merged across the block, then the gradient.
template <typename T>
__global__ void __launch_bounds__(kThreads)
cross_entropy_kernel(const float* __restrict__ logits, T* __restrict__ dlogits, const int* __restrict__ targets,
                     float* __restrict__ loss, int V, int ld, float coef) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  __shared__ float red[4];
  const float* row = logits + (int64_t)blockIdx.x * ld;
  T* drow = dlogits + (int64_t)blockIdx.x * ld;
  const int nv = ld / 4;
  float mx = -INFINITY, sum = 0.f;
  for (int v = threadIdx.x; v < nv; v += kThreads) {
    const f32x4 a = *reinterpret_cast<const f32x4*>(row + v * 4);
    float m4 = -INFINITY;
#pragma unroll
    for (int i = 0; i < 4; ++i) if (v * 4 + i < V) m4 = fmaxf(m4, a[i]);
    if (m4 > mx) { sum *= __expf(mx - m4); mx = m4; }      // exp(-inf) = 0 covers the first step
#pragma unroll
    for (int i = 0; i < 4; ++i) if (v * 4 + i < V) sum += __expf(a[i] - mx);
  }
  const float bmx = block_reduce(mx, true, red);
  sum = block_reduce(mx == -INFINITY ? 0.f : sum * __expf(mx - bmx), false, red);
  const float lse = bmx + __logf(sum);
  const int tgt = clamp_id(targets[blockIdx.x], V);
  if (threadIdx.x == 0) loss[blockIdx.x] = lse - row[tgt];
  constexpr int VN = Vec<T>::N;
  for (int v = threadIdx.x; v < ld / VN; v += kThreads) {
    float a[VN];
#pragma unroll
    for (int q = 0; q < VN / 4; ++q) {
      const f32x4 r = *reinterpret_cast<const f32x4*>(row + v * VN + 4 * q);
#pragma unroll
      for (int i = 0; i < 4; ++i) a[4 * q + i] = r[i];
    }
#pragma unroll
    for (int i = 0; i < VN; ++i) {
      const int c = v * VN + i;
      a[i] = c < V ? coef * (__expf(a[i] - lse) - (c == tgt ? 1.f : 0.f)) : 0.f;
    }
    store_vec<T>(drow + v * VN, a);
  }
}

// The same with the row held in registers: a block of 1024 threads reads its row once (thread t keeps groups t,
// t + 1024, ... of 16 bytes of output each), so the logits cross the memory bus once instead of twice.  Rows of up to
// 1024 * MAXG groups, 64 Ki columns in all; wider ones take the two-pass kernel above.
constexpr int kCeThreads = 1024;
template <typename T, int MAXG>
__global__ void __launch_bounds__(kCeThreads)
cross_entropy_row_kernel(const float* __restrict__ logits, T* __restrict__ dlogits, const int* __restrict__ targets,
                         float* __restrict__ loss, int V, int ld, float coef) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  constexpr int VN = Vec<T>::N, NW = kCeThreads / 64;
  __shared__ float red[2][NW];
  const float* row = logits + (int64_t)blockIdx.x * ld;
  T* drow = dlogits + (int64_t)blockIdx.x * ld;
  const int ng = ld / VN;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float a[MAXG][VN];
  float mx = -INFINITY;
#pragma unroll
  for (int j = 0; j < MAXG; ++j) {
    const int g = threadIdx.x + kCeThreads * j;
    if (g < ng) {
#pragma unroll
      for (int q = 0; q < VN / 4; ++q) {
        const f32x4 r = *reinterpret_cast<const f32x4*>(row + g * VN + 4 * q);
#pragma unroll
        for (int i = 0; i < 4; ++i) a[j][4 * q + i] = r[i];
      }
#pragma unroll
      for (int i = 0; i < VN; ++i) if (g * VN + i < V) mx = fmaxf(mx, a[j][i]);
    }
  }
  mx = wave_max(mx);
  if (lane == 0) red[0][wave] = mx;
  __syncthreads();
  float bmx = red[0][0];
#pragma unroll
  for (int w = 1; w < NW; ++w) bmx = fmaxf(bmx, red[0][w]);
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < MAXG; ++j) {
    const int g = threadIdx.x + kCeThreads * j;
    if (g < ng) {
#pragma unroll
      for (int i = 0; i < VN; ++i) if (g * VN + i < V) sum += __expf(a[j][i] - bmx);
    }
  }
  sum = wave_sum(sum);
  if (lane == 0) red[1][wave] = sum;
  __syncthreads();
  float bsum = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) bsum += red[1][w];
  const float lse = bmx + __logf(bsum);
  const int tgt = clamp_id(targets[blockIdx.x], V);
  if (threadIdx.x == 0) loss[blockIdx.x] = lse - row[tgt];
#pragma unroll
  for (int j = 0; j < MAXG; ++j) {
    const int g = threadIdx.x + kCeThreads * j;
    if (g < ng) {
      float o[VN];
#pragma unroll
      for (int i = 0; i < VN; ++i) {
        const int c = g * VN + i;
        o[i] = c < V ? coef * (__expf(a[j][i] - lse) - (c == tgt ? 1.f : 0.f)) : 0.f;
      }
      store_vec<T>(drow + g * VN, o);
    }
  }
}

template <typename T>
void launch_cross_entropy(const float* logits, T* dlogits, const int* targets, float* loss, int rows, int V, int ld, float coef, hipStream_t s) {
  // (a thread of a 1024-thread block has 128 registers: at most 64 of them hold the row)
  constexpr int kMost = 64 / Vec<T>::N;
  const int per_thread = (ld / Vec<T>::N + kCeThreads - 1) / kCeThreads;
  if (per_thread <= 4) cross_entropy_row_kernel<T, 4><<<rows, kCeThreads, 0, s>>>(logits, dlogits, targets, loss, V, ld, coef);
  else if (per_thread <= 8) cross_entropy_row_kernel<T, 8><<<rows, kCeThreads, 0, s>>>(logits, dlogits, targets, loss, V, ld, coef);
  else if (per_thread <= kMost) cross_entropy_row_kernel<T, kMost><<<rows, kCeThreads, 0, s>>>(logits, dlogits, targets, loss, V, ld, coef);
  else cross_entropy_kernel<T><<<rows, kThreads, 0, s>>>(logits, dlogits, targets, loss, V, ld, coef);
}

// out[0] = (1/n) * sum loss[0..n), one block, fixed order
__global__ void __launch_bounds__(kThreads) mean_kernel(const float* __restrict__ loss, int n, float* __restrict__ out) {
  __shared__ float red[4];
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += kThreads) s += loss[i];
  s = block_reduce(s, false, red);
  if (threadIdx.x == 0) out[0] = s / (float)n;
}

// ---- sort of the tokens by id.  A key is (id << 32) | token index: all keys differ, so any sorting network gives the
// one ascending order, which inside a run of equal ids is ascending token index.  Bitonic network over npad = a power
// of two >= n keys (the padding holds the largest key and stays at the end): compare-exchange partners at distance
// j < kSortTile are handled inside LDS, a tile of kSortTile keys per block; larger distances take one pass over global
// memory each.  b*S <= 2^24 tokens: at most 24 stages.
typedef unsigned long long u64;
constexpr int kSortTile = 2048;                 // keys per block (16 KiB of LDS), two per thread
constexpr int kSortThreads = kSortTile / 2;

__global__ void __launch_bounds__(kThreads) sort_keys_kernel(const int* __restrict__ ids, u64* __restrict__ keys, int n, int npad, int V) {
  const int i = blockIdx.x * kThreads + threadIdx.x;
  if (i < npad) keys[i] = i < n ? ((u64)(unsigned)clamp_id(ids[i], V) << 32) | (unsigned)i : ~(u64)0;
}

// Stages k = k_lo, 2 k_lo, .. k_hi of the network, each from partner distance min(k / 2, kSortTile / 2) down to 1.
// (2 .. kSortTile: sorts every tile; k_lo = k_hi > kSortTile: the tail of stage k after its global passes.)
__global__ void __launch_bounds__(kSortThreads) bitonic_tile_kernel(u64* __restrict__ keys, int k_lo, int k_hi) {
  __shared__ u64 tile[kSortTile];
  const int t = threadIdx.x, base = blockIdx.x * kSortTile;
  tile[t] = keys[base + t];
  tile[t + kSortThreads] = keys[base + t + kSortThreads];
  __syncthreads();
  for (int k = k_lo; k <= k_hi; k <<= 1) {
    for (int j = (k >> 1) < kSortThreads ? (k >> 1) : kSortThreads; j > 0; j >>= 1) {
      const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1)), l = i | j;
      const bool ascending = ((base + i) & k) == 0;
      const u64 a = tile[i], b = tile[l];
      if ((a > b) == ascending) { tile[i] = b; tile[l] = a; }
      __syncthreads();
    }
  }
  keys[base + t] = tile[t];
  keys[base + t + kSortThreads] = tile[t + kSortThreads];
}

// One pass of stage k at partner distance j >= kSortTile, straight on global memory; one pair per thread.
__global__ void __launch_bounds__(kThreads) bitonic_pass_kernel(u64* __restrict__ keys, int k, int j, int pairs) {
  const int t = blockIdx.x * kThreads + threadIdx.x;
  if (t >= pairs) return;
  const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1)), l = i | j;
  const bool ascending = (i & k) == 0;
  const u64 a = keys[i], b = keys[l];
  if ((a > b) == ascending) { keys[i] = b; keys[l] = a; }
}

int sort_pad(int n) {
  int p = kSortTile;
  while (p < n) p <<= 1;
  return p;
}

int launch_sort_tokens(const int* ids, u64* keys, int n, int V, hipStream_t s) {
  const int npad = sort_pad(n);
  sort_keys_kernel<<<(npad + kThreads - 1) / kThreads, kThreads, 0, s>>>(ids, keys, n, npad, V);
  CEPHALO_CHECK_LAUNCH("sort_keys");
  bitonic_tile_kernel<<<npad / kSortTile, kSortThreads, 0, s>>>(keys, 2, kSortTile);
  CEPHALO_CHECK_LAUNCH("bitonic_tile");
  for (int k = 2 * kSortTile; k <= npad; k <<= 1) {
    for (int j = k >> 1; j >= kSortTile; j >>= 1) {
      bitonic_pass_kernel<<<(npad / 2 + kThreads - 1) / kThreads, kThreads, 0, s>>>(keys, k, j, npad / 2);
      CEPHALO_CHECK_LAUNCH("bitonic_pass");
    }
    bitonic_tile_kernel<<<npad / kSortTile, kSortThreads, 0, s>>>(keys, k, k);
    CEPHALO_CHECK_LAUNCH("bitonic_tile");
  }
  return CEPHALO_OK;
}

// Token-embedding gradient.  The tokens are sorted by (id, token index), so the rows of dx0 that belong to one id form
// a run of the sorted order.  The sorted order is cut into segments of kEmbedSeg positions with one wavefront each
// (however often an id occurs, no wavefront walks more than a segment).  Pass 1: a wavefront sums each piece of a run
// inside its segment in order; a run that lies wholly inside the segment is added to its row of the gradient at once
// (the row already holds the head's part where the head is tied; nobody else writes that row), the piece that came in
// from the previous segment and the piece that goes on into the next are parked in part[segment][0 / 1].  Pass 2: the
// wavefront of the segment in which a cut run starts adds up its parked pieces, segment after segment, and adds the
// total to the row.  Every sum has a fixed order: reproducible.
constexpr int kEmbedSeg = 32;

__device__ __forceinline__ unsigned key_id(u64 k) { return (unsigned)(k >> 32); }

__global__ void __launch_bounds__(kThreads)
embed_bwd_segments_kernel(const u64* __restrict__ sorted, const float* __restrict__ dx0, float* __restrict__ g_wte,
                          float* __restrict__ part, int n, int H) {
  constexpr int VN = 4;
  const int seg = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int p0 = seg * kEmbedSeg;
  if (p0 >= n) return;
  const int p1 = min(n, p0 + kEmbedSeg);
  int i = p0;
  while (i < p1) {
    const unsigned id = key_id(sorted[i]);
    int e = i + 1;
    while (e < p1 && key_id(sorted[e]) == id) ++e;
    const bool from_before = i == p0 && p0 > 0 && key_id(sorted[p0 - 1]) == id;
    const bool goes_on = e == p1 && p1 < n && key_id(sorted[p1]) == id;
    float* dst = from_before ? part + ((size_t)seg * 2 + 0) * H : (goes_on ? part + ((size_t)seg * 2 + 1) * H : g_wte + (size_t)id * H);
    const bool add = !from_before && !goes_on;      // a whole run: onto the row; a piece: stored
    for (int v = lane; v < H / VN; v += 64) {
      float acc[VN] = {0.f, 0.f, 0.f, 0.f};
      for (int j = i; j < e; ++j) {
        float a[VN];
        load_vec<float>(dx0 + (int64_t)(unsigned)sorted[j] * H + v * VN, a);
#pragma unroll
        for (int c = 0; c < VN; ++c) acc[c] += a[c];
      }
#pragma unroll
      for (int c = 0; c < VN; ++c) dst[v * VN + c] = add ? dst[v * VN + c] + acc[c] : acc[c];
    }
    i = e;
  }
}

__global__ void __launch_bounds__(kThreads)
embed_bwd_joins_kernel(const u64* __restrict__ sorted, float* __restrict__ g_wte, const float* __restrict__ part, int n, int H) {
  constexpr int VN = 4;
  const int seg = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int p0 = seg * kEmbedSeg;
  if (p0 >= n) return;
  const int p1 = min(n, p0 + kEmbedSeg);
  if (p1 >= n) return;                                       // nothing goes on past the last segment
  const unsigned id = key_id(sorted[p1 - 1]);
  if (key_id(sorted[p1]) != id) return;                      // the last run of this segment ends here
  if (key_id(sorted[p0]) == id && p0 > 0 && key_id(sorted[p0 - 1]) == id) return;   // the run started in an earlier segment: its wavefront joins it
  // the run starts in this segment: its piece here is part[seg][1] -- unless it fills the segment from its first
  // position (then pass 1 saw no difference from "came in from before" only if p0 > 0, excluded above), and the
  // following segments hold part[.][0] while the run lasts
  int last = seg + 1;                                        // last segment the run reaches
  while ((int64_t)(last + 1) * kEmbedSeg < n && key_id(sorted[(last + 1) * kEmbedSeg]) == id && key_id(sorted[(last + 1) * kEmbedSeg - 1]) == id) ++last;
  for (int v = lane; v < H / VN; v += 64) {
    float acc[VN];
#pragma unroll
    for (int c = 0; c < VN; ++c) acc[c] = part[((size_t)seg * 2 + 1) * H + v * VN + c];
    for (int q = seg + 1; q <= last; ++q) {
#pragma unroll
      for (int c = 0; c < VN; ++c) acc[c] += part[((size_t)q * 2 + 0) * H + v * VN + c];
    }
    float* g = g_wte + (size_t)id * H + v * VN;
#pragma unroll
    for (int c = 0; c < VN; ++c) g[c] += acc[c];
  }
}

int embed_segments(int n) { return (n + kEmbedSeg - 1) / kEmbedSeg; }

// Position-embedding gradient: g_wpe[s] = sum over the b samples of dx0[n, s], samples in order.
__global__ void __launch_bounds__(kThreads)
wpe_bwd_kernel(const float* __restrict__ dx0, float* __restrict__ g_wpe, int b, int S, int H) {
  typedef float T;
  constexpr int VN = Vec<T>::N;
  const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;    // vector index inside [S, H]
  if (v * VN >= (int64_t)S * H) return;
  float acc[VN];
#pragma unroll
  for (int c = 0; c < VN; ++c) acc[c] = 0.f;
  for (int n = 0; n < b; ++n) {
    float a[VN];
    load_vec<T>(dx0 + (int64_t)n * S * H + v * VN, a);
#pragma unroll
    for (int c = 0; c < VN; ++c) acc[c] += a[c];
  }
#pragma unroll
  for (int c = 0; c < VN; ++c) g_wpe[v * VN + c] = acc[c];
}

// Input gradient of the tied LM head, duf = dlogits wte.  bf16: through wte^T [H, ldv] (zero-padded columns), made once
// per step, so that both operands are contiguous along the contracted vocabulary axis.
template <typename T> GemmArgs<T> head_dgrad_args(const T* dlg, const T* wte, const T* wteT, int Tm, int V, int H, int ldv);
template <> GemmArgs<float> head_dgrad_args<float>(const float* dlg, const float* wte, const float*, int Tm, int V, int H, int ldv) {
  GemmArgs<float> a = linear_dgrad<float>(dlg, wte, Tm, V, H);
  a.a_rs = ldv;
  return a;
}
template <> GemmArgs<bf16> head_dgrad_args<bf16>(const bf16* dlg, const bf16*, const bf16* wteT, int Tm, int V, int H, int ldv) {
  GemmArgs<bf16> a = linear_dgrad_wt<bf16>(dlg, wteT, Tm, V, H);
  a.a_rs = ldv; a.b_rs = ldv;
  return a;
}
template <typename T> int prepare_head_weights(const T* wte, T* wteT, int V, int H, int ldv, hipStream_t s);
template <> int prepare_head_weights<float>(const float*, float*, int, int, int, hipStream_t) { return CEPHALO_OK; }
template <> int prepare_head_weights<bf16>(const bf16* wte, bf16* wteT, int V, int H, int ldv, hipStream_t s) {
  return launch_transpose_bf16(wte, wteT, V, H, s, ldv);
}

__global__ void __launch_bounds__(kThreads) zero_kernel(float* __restrict__ p, int64_t n4) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < n4) reinterpret_cast<float4*>(p)[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

// Flat layout of a stack.  GPT-style: wte[V,H] wpe[S,H] layers lnf.gamma[H] lnf.beta[H], the head tied to wte.
// Llama-style: wte[V,H] layers normf.gamma[H] w_head[V,H] (no learned positions, no beta, a head of its own).
struct StackOffsets {
  int64_t wte, wpe, layers, normf, head, total;
  bool tied, positions;
};
StackOffsets stack_offsets(const cephalo_stack_desc& d) {
  const int64_t H = d.layer.hidden, V = d.vocab, PL = param_offsets(d.layer).total;
  StackOffsets o;
  o.tied = o.positions = !is_llama(d.layer);
  o.wte = 0;
  o.wpe = V * H;
  o.layers = o.wpe + (o.positions ? (int64_t)d.layer.seq * H : 0);
  o.normf = o.layers + d.layers * PL;
  o.head = o.tied ? o.wte : o.normf + H;
  o.total = o.tied ? o.normf + 2 * H : o.head + V * H;
  return o;
}

int check_stack(const cephalo_stack_desc* d) {
  if (!d) return fail(CEPHALO_EINVAL, "stack desc is null");
  TRY(check_desc(&d->layer));
  if (d->layers <= 0 || d->vocab <= 0) return fail(CEPHALO_EINVAL, "stack desc: layers %d and vocab %d must be positive", d->layers, d->vocab);
  if (d->checkpoint != 0 && d->checkpoint != 1) return fail(CEPHALO_EINVAL, "stack desc: checkpoint must be 0 or 1");
  if (d->offload < 0 || d->offload > 2) return fail(CEPHALO_EINVAL, "stack desc: offload must be 0, 1 or 2");
  if (d->offload && !d->checkpoint) return fail(CEPHALO_EINVAL, "stack desc: offload needs checkpoint = 1 (only boundary activations are offloaded)");
  if (d->interleave != 0 && d->interleave != 1) return fail(CEPHALO_EINVAL, "stack desc: interleave must be 0 or 1");
  if (d->interleave && d->offload) return fail(CEPHALO_EUNSUPPORTED, "stack desc: interleave and offload do not go together");
  if (d->offload == 2 && d->layer.dtype == CEPHALO_F32)
    return fail(CEPHALO_EUNSUPPORTED, "stack desc: offload = 2 needs the bf16 mode (in fp32 mode the weight gradients read the whole share's fp32 "
                "gradient of the residual stream, which therefore stays on the device)");
  return CEPHALO_OK;
}

struct StackLayout {
  size_t xs, xdump, saves, save_each, scratch, dxa, dxb, dxal, dxbl, uf, meanf, rstdf, duf, logits, dlogits, wteT, loss, lnf_part, keys, embed_part, total;
  int ldv;            // padded pitch of the logits
  size_t lnf_rows;
};

StackLayout stack_layout(const cephalo_stack_desc& d, int b, int m) {
  const cephalo_layer_desc& ld = d.layer;
  const size_t es = ld.dtype == CEPHALO_F32 ? 4 : 2;
  const size_t n = (size_t)b * ld.seq, Tm = (size_t)m * ld.seq, H = ld.hidden;
  StackLayout L;
  L.ldv = (d.vocab + 63) / 64 * 64;    // rows of the logits start on 128-byte lines (a pitch that is only a multiple of 16 bytes makes every
                                       // 128-byte slab of a row straddle two cache lines: measured 658 against 893 TFLOP/s for the head's input gradient)
  size_t p = 0;
  auto take = [&](size_t bytes) { size_t at = p; p += align_up(bytes); return at; };
  // layer-boundary activations, the fp32 residual stream: all of them, or (offload) two micro-batches coming in from the
  // host and two going out; with checkpointing also one micro-batch where the recomputed layer output is dropped
  L.xs = take(d.offload ? 4 * Tm * H * 4 : (size_t)(d.layers + 1) * n * H * 4);
  L.xdump = d.checkpoint ? take((d.interleave ? 2 : 1) * Tm * H * 4) : 0;
  L.save_each = align_up(save_layout(ld, b).total);
  L.saves = take((size_t)(d.checkpoint ? 1 : d.layers) * L.save_each);   // checkpointing: one layer's internals at a time
  L.scratch = take(scratch_layout(ld, m, b, d.interleave ? 2 : 1).total);
  // gradient of the residual stream, ping-pong between layers; offload = 2: the first buffer only takes the last result
  // (the gradient with respect to the embedding output), everything before passes through four micro-batch slots
  L.dxa = take(n * H * 4); L.dxb = take(d.offload == 2 ? 4 * Tm * H * 4 : n * H * 4);
  L.dxal = es == 4 ? L.dxa : take(n * H * es); L.dxbl = es == 4 ? L.dxb : take(n * H * es);   // and its copy in the activation type
  L.uf = take(n * H * es); L.meanf = take(n * 4); L.rstdf = take(n * 4);
  L.duf = take((d.interleave ? 2 : 1) * Tm * H * 4);
  L.logits = take((d.interleave ? 2 : 1) * Tm * (size_t)L.ldv * 4);   // one micro-batch of fp32 logits, reused (interleave: one per stream)
  L.dlogits = take(n * (size_t)L.ldv * es);       // their gradient for the whole share (an operand of the weight gradient)
  L.wteT = es == 4 ? 0 : take(H * (size_t)L.ldv * es);   // wte^T [H, ldv] for the input gradient of the LM head
  L.loss = take(n * 4);
  L.lnf_rows = (size_t)(b / m) * ln_bwd_blocks((int)Tm);
  L.lnf_part = take(3 * L.lnf_rows * H * 4);      // d gamma, d beta, and the column sums of the gradient the last layer receives
  L.keys = take((size_t)sort_pad((int)n) * sizeof(u64));      // (id, token index) keys of the embedding gradient's sort
  L.embed_part = take((size_t)embed_segments((int)n) * 2 * H * 4);   // pieces of runs of equal ids that cross a segment boundary
  L.total = p;
  return L;
}

// Where the layer-boundary activations [layers+1][b*S][H] live.  Resident: in the work area.  Offloaded (Sec. 3.2
// "Activation Checkpointing and Offloading" and the supplementary figure on offloading): in pinned host memory; a
// micro-batch's boundary activation goes to the host on the copy stream as soon as it is computed, while the next
// micro-batch runs, and comes back (two micro-batches of look-ahead) before it is needed, in the forward as the next
// layer's input and in the backward for the recomputation.  Accesses are sequential, so two device slots per direction
// and a handful of events order the streams; copies to the host and copies to the device have a stream each, so that
// both directions of the link are in use at once.
struct Boundary {
  bool offload = false;
  float* base = nullptr;           // resident: device [layers+1][n][H]; offload: host, same layout
  float* in_slot[2] = {nullptr, nullptr};
  float* out_slot[2] = {nullptr, nullptr};
  size_t n = 0, Tm = 0, H = 0;
  hipStream_t c = nullptr, xin = nullptr, xout = nullptr;   // compute, host-to-device copies, device-to-host copies
  hipEvent_t pre[2], free_in[2], comp[2], off[2], written, last;
  long issued = 0, consumed = 0, produced = 0;
  int err = CEPHALO_OK;

  float* at(int k, int j) const { return base + ((size_t)k * n + (size_t)j * Tm) * H; }
  void check(hipError_t e, const char* what) {
    if (e != hipSuccess && err == CEPHALO_OK) err = fail(CEPHALO_EHIP, "stack_step (offload): %s: %s", what, hipGetErrorString(e));
  }
  int open() {
    if (!offload) return CEPHALO_OK;
    for (hipEvent_t* e : {&pre[0], &pre[1], &free_in[0], &free_in[1], &comp[0], &comp[1], &off[0], &off[1], &written, &last})
      check(hipEventCreateWithFlags(e, hipEventDisableTiming), "event");
    return err;
  }
  // start bringing boundary k of micro-batch j to the device (no-op when resident or when j is past the share)
  void prefetch(int k, int j, int l) {
    if (!offload || j >= l) return;
    const int slot = (int)(issued % 2);
    check(hipStreamWaitEvent(xin, free_in[slot], 0), "wait");         // the slot's previous reader is done
    check(hipStreamWaitEvent(xin, written, 0), "wait");               // every copy to the host enqueued so far has landed
    check(hipMemcpyAsync(in_slot[slot], at(k, j), Tm * H * 4, hipMemcpyHostToDevice, xin), "copy to device");
    check(hipEventRecord(pre[slot], xin), "record");
    ++issued;
  }
  const float* in(int k, int j, int l) {
    if (!offload) return at(k, j);
    if (consumed == issued) prefetch(k, j, l);
    check(hipStreamWaitEvent(c, pre[consumed % 2], 0), "wait");
    return in_slot[consumed % 2];
  }
  void in_done() {
    if (!offload) return;
    check(hipEventRecord(free_in[consumed % 2], c), "record");
    ++consumed;
  }
  float* out(int k, int j) {
    if (!offload) return at(k, j);
    check(hipStreamWaitEvent(c, off[produced % 2], 0), "wait");        // the slot's previous content has left
    return out_slot[produced % 2];
  }
  void out_done(int k, int j) {
    if (!offload) return;
    const int slot = (int)(produced % 2);
    check(hipEventRecord(comp[slot], c), "record");
    check(hipStreamWaitEvent(xout, comp[slot], 0), "wait");
    check(hipMemcpyAsync(at(k, j), out_slot[slot], Tm * H * 4, hipMemcpyDeviceToHost, xout), "copy to host");
    check(hipEventRecord(off[slot], xout), "record");
    check(hipEventRecord(written, xout), "record");
    ++produced;
  }
  // the compute stream ends behind the copy streams, so that a caller who waits for it may release the host area
  int close() {
    if (!offload) return CEPHALO_OK;
    check(hipEventRecord(last, xin), "record");
    check(hipStreamWaitEvent(c, last, 0), "wait");
    check(hipStreamWaitEvent(c, written, 0), "wait");
    for (hipEvent_t e : {pre[0], pre[1], free_in[0], free_in[1], comp[0], comp[1], off[0], off[1], written, last}) check(hipEventDestroy(e), "event");
    return err;
  }
};

template <typename T>
int run_stack(const cephalo_stack_desc& d, const void* Pv, const int* ids, const int* targets, int b, int m,
              float* G, float scale, float* loss_out, void* ws, float* host_area, hipStream_t s, hipStream_t copy_in, hipStream_t copy_out,
              hipStream_t side) {
  const cephalo_layer_desc& ld = d.layer;
  const T* P = static_cast<const T*>(Pv);
  const int S = ld.seq, H = ld.hidden, V = d.vocab, NL = d.layers, l = b / m;
  const int n = b * S, Tm = m * S;
  const int64_t PL = param_offsets(ld).total;
  const StackOffsets SO = stack_offsets(d);
  const int64_t o_wte = SO.wte, o_wpe = SO.wpe, o_layers = SO.layers, o_lnf = SO.normf, o_head = SO.head;
  const bool rms = is_llama(ld);
  const StackLayout L = stack_layout(d, b, m);
  const SaveLayout SL = save_layout(ld, b);
  const int nst = d.interleave ? 2 : 1;
  const ScratchLayout WL = scratch_layout(ld, m, b, nst);
  void* scratch = at<char>(ws, L.scratch);
  // Interleave: micro-batch j runs on stream j % 2, so that the bandwidth-bound kernels of one micro-batch overlap the
  // matrix-core kernels of the other and GEMMs with few output tiles share the compute units.  A micro-batch's whole
  // chain through the layers stays on its stream; the streams meet where the share is handled as one (weight
  // gradients, shared weight transposes, the embeddings), through fork / join events.
  hipStream_t st[2] = {s, d.interleave ? side : s};
  Streams J;
  J.main = s; J.side = side; J.on = d.interleave != 0;
  TRY(J.open());
  struct JCloser { Streams& j; bool done = false; ~JCloser() { if (!done) (void)j.close(); } } jcloser{J};   // early exits still join
  const size_t act = (size_t)Tm * H;
  Boundary X;
  X.offload = d.offload != 0;
  X.n = n; X.Tm = Tm; X.H = H; X.c = s; X.xin = copy_in; X.xout = copy_out;
  if (X.offload) {
    X.base = host_area;
    for (int i = 0; i < 2; ++i) { X.in_slot[i] = at<float>(ws, L.xs) + i * act; X.out_slot[i] = at<float>(ws, L.xs) + (2 + i) * act; }
  } else {
    X.base = at<float>(ws, L.xs);
  }
  TRY(X.open());
  struct Closer { Boundary& x; bool done = false; ~Closer() { if (!done) (void)x.close(); } } closer{X};   // events are released on every path
  // offload = 2: the gradient of the residual stream takes the same road (the supplementary figure's GC^g / CG^g): the
  // gradient with respect to boundary k of micro-batch j goes to the host as soon as layer k's backward has produced it
  // and comes back, one micro-batch ahead, when layer k-1's backward of that micro-batch needs it.  Two boundaries are
  // alive at a time, so the host keeps two [b*S][H] images (boundary k in image k mod 2) after the activations.
  Boundary Gx;
  Gx.offload = d.offload == 2;
  Gx.n = n; Gx.Tm = Tm; Gx.H = H; Gx.c = s; Gx.xin = copy_in; Gx.xout = copy_out;
  if (Gx.offload) {
    Gx.base = host_area + (size_t)(NL + 1) * n * H;
    for (int i = 0; i < 2; ++i) { Gx.in_slot[i] = at<float>(ws, L.dxb) + i * act; Gx.out_slot[i] = at<float>(ws, L.dxb) + (2 + i) * act; }
  }
  TRY(Gx.open());
  struct GCloser { Boundary& x; bool done = false; ~GCloser() { if (!done) (void)x.close(); } } gcloser{Gx};

  // ---- forward
  TRY(prepare_head_weights<T>(P + o_head, at<T>(ws, L.wteT), V, H, L.ldv, s));
  J.fork();
  GemmSideBySide hint(nst);     // until the join: two kernels share the device
  for (int j = 0; j < l; ++j) {
    embed_fwd_kernel<T><<<(Tm + 3) / 4, kThreads, 0, st[j % nst]>>>(ids + (size_t)j * Tm, P + o_wte, SO.positions ? P + o_wpe : (const T*)nullptr, X.out(0, j), Tm, S, H, V);
    CEPHALO_CHECK_LAUNCH("embed_fwd");
    X.out_done(0, j);
  }
  auto save_of = [&](int layer) { return at<char>(ws, L.saves + (d.checkpoint ? 0 : (size_t)layer * L.save_each)); };
  for (int li = 0; li < NL; ++li) {
    void* save = save_of(li);
    X.prefetch(li, 0, l);
    for (int j = 0; j < l; ++j) {
      const float* xi = X.in(li, j, l);
      X.prefetch(li, j + 1, l);
      float* xo = X.out(li + 1, j);
      TRY(layer_fwd_t<T>(ld, P + o_layers + li * PL, xi, xo, m, saved_at<T>(save, SL, ld, j * m), st[j % nst]));
      X.in_done();
      X.out_done(li + 1, j);
    }
  }
  // ---- head: final LN, tied logits (fp32, one micro-batch at a time), cross-entropy and its gradient, back to the last layer's output
  T* uf = at<T>(ws, L.uf); float* logits = at<float>(ws, L.logits); T* dlogits = at<T>(ws, L.dlogits); float* duf = at<float>(ws, L.duf);
  float* meanf = at<float>(ws, L.meanf); float* rstdf = at<float>(ws, L.rstdf);
  float* lnf_g = at<float>(ws, L.lnf_part); float* lnf_b = lnf_g + L.lnf_rows * H; float* lnf_s = lnf_b + L.lnf_rows * H;
  float* dx_cur = at<float>(ws, L.dxa); float* dx_nxt = at<float>(ws, L.dxb);
  T* dxl_cur = at<T>(ws, L.dxal); T* dxl_nxt = at<T>(ws, L.dxbl);
  const float coef = scale / (float)n;
  const int nb = ln_bwd_blocks(Tm);
  X.prefetch(NL, 0, l);
  for (int j = 0; j < l; ++j) {
    const size_t t0 = (size_t)j * Tm;
    hipStream_t sj = st[j % nst];
    float* logits_j = logits + (size_t)(j % nst) * Tm * L.ldv;
    float* duf_j = duf + (size_t)(j % nst) * Tm * H;
    const float* xL = X.in(NL, j, l);
    X.prefetch(NL, j + 1, l);
    TRY(launch_ln_fwd<T>(xL, P + o_lnf, rms ? (const T*)nullptr : P + o_lnf + H, uf + t0 * H, meanf + t0, rstdf + t0, Tm, H, ld.ln_eps, sj, rms));
    T* dlg = dlogits + t0 * L.ldv;
    {
      GemmArgs<T> a = linear_fwd<T>(uf + t0 * H, P + o_head, Tm, V, H);
      a.epi = EPI_NONE_HEAD; a.Cf = logits_j; a.ldc = L.ldv;
      TRY(gemm<T>(a, sj));
    }
    launch_cross_entropy<T>(logits_j, dlg, targets + t0, at<float>(ws, L.loss) + t0, Tm, V, L.ldv, coef, sj);
    CEPHALO_CHECK_LAUNCH("cross_entropy");
    {
      GemmArgs<T> a = head_dgrad_args<T>(dlg, P + o_head, at<T>(ws, L.wteT), Tm, V, H, L.ldv);   // duf = dlogits W_head
      a.epi = EPI_NONE_HEAD; a.Cf = duf_j;
      TRY(gemm<T>(a, sj));
    }
    float* dxo = Gx.offload ? Gx.out(NL % 2, j) : dx_cur + t0 * H;
    TRY(launch_ln_bwd<T>(duf_j, xL, meanf + t0, rstdf + t0, P + o_lnf, (const float*)nullptr, dxo,
                         lowp_out<T>(dxl_cur + t0 * H), lnf_g + (size_t)j * nb * H, lnf_b + (size_t)j * nb * H, Tm, H, sj, rms,
                         rms ? (float*)nullptr : lnf_s + (size_t)j * nb * H));
    Gx.out_done(NL % 2, j);
    X.in_done();
  }
  J.join();
  hint.now(1);
  mean_kernel<<<1, kThreads, 0, s>>>(at<float>(ws, L.loss), n, loss_out);
  CEPHALO_CHECK_LAUNCH("mean_loss");
  {
    Work<T> w = work_at<T>(scratch, WL, ld, 0, 0, m);
    TRY(wgrad<T>(dlogits, uf, n, V, H, G + o_head, 1.0f, 0, (float*)nullptr, s, L.ldv));       // the head's gradient (tied: the head's part of d wte), whole share
    TRY(launch_reduce_partials(lnf_g, l * nb, H, G + o_lnf, 1.0f, 0, w.col_part, w.col_part_bytes, s));
    if (!rms) TRY(launch_reduce_partials(lnf_b, l * nb, H, G + o_lnf + H, 1.0f, 0, w.col_part, w.col_part_bytes, s));
    // The bias gradient of a layer's second feed-forward projection is the column sum of the gradient arriving at the
    // layer's output.  Whoever produces that gradient (the final norm's backward here, the layer above further down)
    // sums it block by block as it writes it.
    if (!rms) TRY(launch_reduce_partials(lnf_s, l * nb, H, G + o_layers + (size_t)(NL - 1) * PL + param_offsets(ld).b_fc2, 1.0f, 0, w.col_part, w.col_part_bytes, s));
  }
  // ---- backward through the layers
  for (int li = NL - 1; li >= 0; --li) {
    void* save = save_of(li);
    const T* Pl = P + o_layers + li * PL;
    TRY(prepare_dgrad_weights<T>(ld, Pl, work_at<T>(scratch, WL, ld, 0, 0, m).wT, s));
    J.fork();        // (after the previous layer's weight gradients too: they read what this layer's data pass overwrites)
    hint.now(nst);
    // Checkpointing: a micro-batch's internals are recomputed from its boundary input right before its backward (the
    // last layer's are still there from the forward); the recomputed output, the same values again, is dropped.
    const bool recompute = d.checkpoint && li != NL - 1;
    X.prefetch(li, 0, l);
    Gx.prefetch((li + 1) % 2, 0, l);
    for (int j = 0; j < l; ++j) {
      const float* xi = X.in(li, j, l);
      X.prefetch(li, j + 1, l);
      if (recompute) TRY(layer_fwd_t<T>(ld, Pl, xi, at<float>(ws, L.xdump) + (size_t)(j % nst) * act, m, saved_at<T>(save, SL, ld, j * m), st[j % nst]));
      // the fp32 gradient arriving at this layer's output and the one leaving at its input: resident buffers, or (offload = 2)
      // a slot just fetched from the host and a slot about to leave for it; layer 0's result stays on the device for the embeddings
      const float* dyj = Gx.offload ? Gx.in((li + 1) % 2, j, l) : dx_cur + j * act;
      Gx.prefetch((li + 1) % 2, j + 1, l);
      float* dxj = !Gx.offload ? dx_nxt + j * act : (li == 0 ? at<float>(ws, L.dxa) + j * act : Gx.out(li % 2, j));
      TRY(layer_bwd_data_t<T>(ld, Pl, xi, dyj, dxl_cur + j * act, dxj,
                              dxl_nxt + j * act, m, saved_at<T>(save, SL, ld, j * m), work_at<T>(scratch, WL, ld, j * m, j, m, j % nst), st[j % nst]));
      Gx.in_done();
      if (Gx.offload && li > 0) Gx.out_done(li % 2, j);
      X.in_done();
    }
    J.join();
    hint.now(1);
    J.fork();        // the parameter pass: weight-gradient GEMMs on the main stream, the bandwidth-bound reductions beside them
    TRY(layer_bwd_params_t<T>(ld, (const float*)nullptr, Gx.offload ? dxl_cur : lowp_of<T>(dx_cur, dxl_cur), n, l * nb,
                              saved_at<T>(save, SL, ld, 0), work_at<T>(scratch, WL, ld, 0, 0, m), G + o_layers + li * PL, 1.0f, 0, s, st[1],
                              (!rms && li > 0) ? G + o_layers + (size_t)(li - 1) * PL + param_offsets(ld).b_fc2 : (float*)nullptr));
    J.join();
    { float* t = dx_cur; dx_cur = dx_nxt; dx_nxt = t; }
    { T* t = dxl_cur; dxl_cur = dxl_nxt; dxl_nxt = t; }
  }
  // ---- embeddings
  if (Gx.offload) dx_cur = at<float>(ws, L.dxa);      // layer 0 left its result there
  if (SO.positions) {
    wpe_bwd_kernel<<<(int)(((int64_t)S * H / 4 + kThreads - 1) / kThreads), kThreads, 0, s>>>(dx_cur, G + o_wpe, b, S, H);
    CEPHALO_CHECK_LAUNCH("wpe_bwd");
  }
  if (!SO.tied) {      // the rows of d wte do not hold a head's part: they start at zero (rows of unused ids stay there)
    const int64_t n4 = (int64_t)V * H / 4;
    zero_kernel<<<(int)((n4 + kThreads - 1) / kThreads), kThreads, 0, s>>>(G + o_wte, n4);
    CEPHALO_CHECK_LAUNCH("zero_wte_grad");
  }
  u64* keys = at<u64>(ws, L.keys);
  TRY(launch_sort_tokens(ids, keys, n, V, s));
  const int nseg = embed_segments(n);
  embed_bwd_segments_kernel<<<(nseg + 3) / 4, kThreads, 0, s>>>(keys, dx_cur, G + o_wte, at<float>(ws, L.embed_part), n, H);
  CEPHALO_CHECK_LAUNCH("embed_bwd_segments");
  embed_bwd_joins_kernel<<<(nseg + 3) / 4, kThreads, 0, s>>>(keys, G + o_wte, at<float>(ws, L.embed_part), n, H);
  CEPHALO_CHECK_LAUNCH("embed_bwd_joins");
  closer.done = true;
  gcloser.done = true;
  jcloser.done = true;
  const int rc_join = J.close(), rc_grad = Gx.close(), rc_copy = X.close();      // errors of the final join and of the event releases are the call's result
  return rc_join != CEPHALO_OK ? rc_join : (rc_grad != CEPHALO_OK ? rc_grad : rc_copy);
}

}  // namespace
}  // namespace cephalo

using namespace cephalo;

extern "C" int64_t cephalo_stack_param_count(const cephalo_stack_desc* d) {
  const int rc = check_stack(d);
  if (rc != CEPHALO_OK) return rc;
  return stack_offsets(*d).total;
}

extern "C" int cephalo_stack_param_offsets(const cephalo_stack_desc* d, int64_t* offsets) {
  TRY(check_stack(d));
  if (!offsets) return fail(CEPHALO_EINVAL, "stack_param_offsets: null output");
  const StackOffsets o = stack_offsets(*d);
  offsets[0] = o.wte; offsets[1] = o.wpe; offsets[2] = o.layers; offsets[3] = o.normf; offsets[4] = o.head;
  return CEPHALO_OK;
}

extern "C" int cephalo_stack_workspace_bytes(const cephalo_stack_desc* d, int32_t batch_share, int32_t micro_batch, size_t* bytes) {
  TRY(check_stack(d));
  if (micro_batch <= 0 || batch_share <= 0 || batch_share % micro_batch != 0)
    return fail(CEPHALO_EINVAL, "stack_workspace_bytes: batch share b = %d is not a positive multiple of micro-batch size m = %d",
                batch_share, micro_batch);
  if (!bytes) return fail(CEPHALO_EINVAL, "stack_workspace_bytes: null output");
  *bytes = stack_layout(*d, batch_share, micro_batch).total;
  return CEPHALO_OK;
}

extern "C" int cephalo_op_cross_entropy(int32_t dtype, const float* logits, int32_t ld, const int32_t* targets, void* dlogits,
                                        float* loss_rows, int32_t rows, int32_t V, float coef, void* stream) {
  if (dtype != CEPHALO_F32 && dtype != CEPHALO_BF16) return fail(CEPHALO_EINVAL, "cross_entropy: unknown dtype %d", dtype);
  if (rows <= 0 || V <= 0 || ld < V) return fail(CEPHALO_EINVAL, "cross_entropy: %d rows, %d classes, pitch %d", rows, V, ld);
  if (ld % 8 != 0) return fail(CEPHALO_EUNSUPPORTED, "cross_entropy: the pitch %d must be a multiple of 8", ld);
  if (!logits || !targets || !dlogits || !loss_rows) return fail(CEPHALO_EINVAL, "cross_entropy: null buffer");
  if (!aligned16(logits) || !aligned16(dlogits)) return fail(CEPHALO_EINVAL, "cross_entropy: buffers must be 16-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == CEPHALO_F32) launch_cross_entropy<float>(logits, static_cast<float*>(dlogits), targets, loss_rows, rows, V, ld, coef, s);
  else launch_cross_entropy<bf16>(logits, static_cast<bf16*>(dlogits), targets, loss_rows, rows, V, ld, coef, s);
  CEPHALO_CHECK_LAUNCH("cross_entropy");
  return CEPHALO_OK;
}

extern "C" int cephalo_stack_workspace_regions(const cephalo_stack_desc* d, int32_t batch_share, int32_t micro_batch, size_t* offsets) {
  TRY(check_stack(d));
  if (micro_batch <= 0 || batch_share <= 0 || batch_share % micro_batch != 0)
    return fail(CEPHALO_EINVAL, "stack_workspace_regions: batch share b = %d is not a positive multiple of micro-batch size m = %d",
                batch_share, micro_batch);
  if (!offsets) return fail(CEPHALO_EINVAL, "stack_workspace_regions: null output");
  const StackLayout L = stack_layout(*d, batch_share, micro_batch);
  // the residual-stream gradient alternates between two buffers, one swap per layer, starting in the first
  const bool even = d->layers % 2 == 0;
  offsets[0] = L.xs;
  offsets[1] = d->offload == 2 ? L.dxa : (even ? L.dxa : L.dxb);
  offsets[2] = even ? L.dxb : L.dxa;      // (offload = 2: not resident; the host area's gradient image 1 holds it)
  return CEPHALO_OK;
}

namespace {
int stack_step_checked(const cephalo_stack_desc* d, const void* flat_param, const int32_t* ids, const int32_t* targets,
                       int32_t batch_share, int32_t micro_batch, float* flat_grad, float grad_scale, float* loss,
                       void* workspace, size_t workspace_bytes, void* host_area, size_t host_bytes, void* stream, void* copy_in, void* copy_out,
                       void* side = nullptr) {
  TRY(check_stack(d));
  if (micro_batch <= 0 || batch_share <= 0 || batch_share % micro_batch != 0)
    return fail(CEPHALO_EINVAL, "stack_step: batch share b = %d is not a positive multiple of micro-batch size m = %d",
                batch_share, micro_batch);
  if ((int64_t)batch_share * d->layer.seq > (1 << 24)) return fail(CEPHALO_EUNSUPPORTED, "stack_step: b*S is too many tokens");
  for (const void* p : {flat_param, (const void*)ids, (const void*)targets, (const void*)flat_grad, (const void*)loss, (const void*)workspace}) {
    if (!p) return fail(CEPHALO_EINVAL, "stack_step: null pointer argument");
  }
  if (!aligned16(flat_param) || !aligned16(flat_grad) || !aligned16(workspace))
    return fail(CEPHALO_EINVAL, "stack_step: flat_param, flat_grad and workspace must be 16-byte aligned");
  const size_t need = stack_layout(*d, batch_share, micro_batch).total;
  if (workspace_bytes < need) return fail(CEPHALO_EWORKSPACE, "stack_step: workspace %zu B < %zu B", workspace_bytes, need);
  if (d->offload) {
    size_t host_need = 0;
    TRY(cephalo_stack_host_bytes(d, batch_share, micro_batch, &host_need));
    if (!host_area || host_bytes < host_need) return fail(CEPHALO_EWORKSPACE, "stack_step: host area %zu B < %zu B", host_bytes, host_need);
    if (!copy_in || !copy_out || copy_in == stream || copy_out == stream)
      return fail(CEPHALO_EINVAL, "stack_step: offload needs copy streams other than the compute stream");
  }
  if (d->interleave && (!side || side == stream))
    return fail(CEPHALO_EINVAL, "stack_step: interleave needs a side stream other than the compute stream");
  hipStream_t s = static_cast<hipStream_t>(stream), ci = static_cast<hipStream_t>(copy_in), co = static_cast<hipStream_t>(copy_out);
  hipStream_t sd = static_cast<hipStream_t>(side);
  if (d->layer.dtype == CEPHALO_F32)
    return run_stack<float>(*d, flat_param, ids, targets, batch_share, micro_batch, flat_grad, grad_scale, loss, workspace,
                            static_cast<float*>(host_area), s, ci, co, sd);
  return run_stack<bf16>(*d, flat_param, ids, targets, batch_share, micro_batch, flat_grad, grad_scale, loss, workspace,
                         static_cast<float*>(host_area), s, ci, co, sd);
}
}  // namespace

extern "C" int cephalo_stack_host_bytes(const cephalo_stack_desc* d, int32_t batch_share, int32_t micro_batch, size_t* bytes) {
  TRY(check_stack(d));
  if (micro_batch <= 0 || batch_share <= 0 || batch_share % micro_batch != 0)
    return fail(CEPHALO_EINVAL, "stack_host_bytes: batch share b = %d is not a positive multiple of micro-batch size m = %d",
                batch_share, micro_batch);
  if (!bytes) return fail(CEPHALO_EINVAL, "stack_host_bytes: null output");
  // the layer-boundary activations; offload = 2: and two images of the residual stream's gradient behind them
  *bytes = d->offload ? (size_t)(d->layers + 1 + (d->offload == 2 ? 2 : 0)) * batch_share * d->layer.seq * d->layer.hidden * sizeof(float) : 0;
  return CEPHALO_OK;
}

extern "C" int cephalo_stack_step(const cephalo_stack_desc* d, const void* flat_param, const int32_t* ids, const int32_t* targets,
                                  int32_t batch_share, int32_t micro_batch, float* flat_grad, float grad_scale, float* loss,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  if (d && d->offload) return fail(CEPHALO_EINVAL, "stack_step: a desc with offload = 1 goes to cephalo_stack_step_offload");
  if (d && d->interleave) return fail(CEPHALO_EINVAL, "stack_step: a desc with interleave = 1 goes to cephalo_stack_step_interleaved");
  return stack_step_checked(d, flat_param, ids, targets, batch_share, micro_batch, flat_grad, grad_scale, loss,
                            workspace, workspace_bytes, nullptr, 0, stream, nullptr, nullptr);
}

extern "C" int cephalo_stack_step_offload(const cephalo_stack_desc* d, const void* flat_param, const int32_t* ids, const int32_t* targets,
                                          int32_t batch_share, int32_t micro_batch, float* flat_grad, float grad_scale, float* loss,
                                          void* workspace, size_t workspace_bytes, void* host_area, size_t host_bytes,
                                          void* stream, void* copy_in_stream, void* copy_out_stream) {
  if (d && !d->offload) return fail(CEPHALO_EINVAL, "stack_step_offload: the desc has offload = 0");
  return stack_step_checked(d, flat_param, ids, targets, batch_share, micro_batch, flat_grad, grad_scale, loss,
                            workspace, workspace_bytes, host_area, host_bytes, stream, copy_in_stream, copy_out_stream);
}

extern "C" int cephalo_stack_step_interleaved(const cephalo_stack_desc* d, const void* flat_param, const int32_t* ids, const int32_t* targets,
                                              int32_t batch_share, int32_t micro_batch, float* flat_grad, float grad_scale, float* loss,
                                              void* workspace, size_t workspace_bytes, void* stream, void* side_stream) {
  if (d && !d->interleave) return fail(CEPHALO_EINVAL, "stack_step_interleaved: the desc has interleave = 0");
  return stack_step_checked(d, flat_param, ids, targets, batch_share, micro_batch, flat_grad, grad_scale, loss,
                            workspace, workspace_bytes, nullptr, 0, stream, nullptr, nullptr, side_stream);
}
