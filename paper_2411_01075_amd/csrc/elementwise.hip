// LayerNorm forward/backward and column sums (bias gradients): HBM-bound row kernels.
// Forward: one 64-lane wavefront owns a row; its lanes hold the row in registers as 16-byte
// vectors, and row statistics are wavefront reductions (no LDS, no block barrier).
// Backward: a block of four wavefronts shares each row (see ln_bwd_kernel).
// The residual stream (x, x1, y and their gradients) and the gradients entering LayerNorm's
// backward are fp32; LayerNorm outputs are in the activation type T.
#include "kernels.h"

namespace cephalo {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

// N consecutive floats (N = 4 or 8) as 16-byte loads / stores
template <int N> __device__ __forceinline__ void load_f32(const float* p, float (&out)[N]) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
  for (int q = 0; q < N / 4; ++q) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(p + 4 * q);
#pragma unroll
    for (int i = 0; i < 4; ++i) out[4 * q + i] = v[i];
  }
}
template <int N> __device__ __forceinline__ void store_f32(float* p, const float (&in)[N]) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
  for (int q = 0; q < N / 4; ++q) {
    f32x4 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = in[4 * q + i];
    *reinterpret_cast<f32x4*>(p + 4 * q) = v;
  }
}

// RMS: root-mean-square norm instead (no mean subtraction, no beta: u = gamma * x / sqrt(mean(x^2) + eps)); the mean
// written is 0.
template <typename T, int MAXV, bool RMS>
__global__ void __launch_bounds__(kThreads)
ln_fwd_kernel(const float* __restrict__ x, const T* __restrict__ gamma, const T* __restrict__ beta,
              T* __restrict__ u, float* __restrict__ mean, float* __restrict__ rstd,
              int rows, int H, float eps) {
  constexpr int VN = Vec<T>::N;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nv = H / VN;
  const float inv_h = 1.0f / (float)H;
  // Straight-line code: a lane whose 16-byte group lies past the row reads the row's first group instead and its
  // values are replaced by zeros; only the stores are predicated.  (With each group's loads under its own bounds
  // branch the compiler waited for one group before it asked for the next, and for every group's store before the next
  // group's gamma and beta: eight memory round trips in a row per row of the matrix.)
  typedef typename Vec<T>::raw RawT;
  for (int row = blockIdx.x * kWaves + wave; row < rows; row += gridDim.x * kWaves) {
    const float* xr = x + (int64_t)row * H;
    float vals[MAXV][VN];
    RawT gr[MAXV], br[MAXV];
#pragma unroll
    for (int j = 0; j < MAXV; ++j) {
      const int v = lane + 64 * j, vc = v < nv ? v : 0;
      load_f32<VN>(xr + vc * VN, vals[j]);
    }
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < MAXV; ++j) {
      const bool ok = lane + 64 * j < nv;
#pragma unroll
      for (int i = 0; i < VN; ++i) { vals[j][i] = ok ? vals[j][i] : 0.f; sum += vals[j][i]; }
    }
    const float mu = RMS ? 0.f : wave_sum(sum) * inv_h;
    // gamma and beta (in L2: every row reads the same) are asked for here, all at once, and arrive under the second
    // reduction; asked for with the row they cost 50 registers more and a third of the rows in flight per SIMD
    constexpr bool EARLY = MAXV <= 8;      // (the widest rows: no registers for that either, they load them group by group)
    if (EARLY) {
#pragma unroll
      for (int j = 0; j < MAXV; ++j) {
        const int v = lane + 64 * j;
        int vc = v < nv ? v : 0;
        asm volatile("" : "+v"(vc));      // (kept here: they do not depend on the row, and the compiler would move them above the row's own loads)
        gr[j] = *reinterpret_cast<const RawT*>(gamma + vc * VN);
        if (!RMS) br[j] = *reinterpret_cast<const RawT*>(beta + vc * VN);
      }
    }
    float sq = 0.f;
#pragma unroll
    for (int j = 0; j < MAXV; ++j) {
      const bool ok = lane + 64 * j < nv;
#pragma unroll
      for (int i = 0; i < VN; ++i) { const float d = ok ? vals[j][i] - mu : 0.f; sq += d * d; }
    }
    const float rs = 1.0f / sqrtf(wave_sum(sq) * inv_h + eps);
    T* ur = u + (int64_t)row * H;
#pragma unroll
    for (int j = 0; j < MAXV; ++j) {
      const int v = lane + 64 * j, vc = v < nv ? v : 0;
      if (!EARLY) {
        gr[j] = *reinterpret_cast<const RawT*>(gamma + vc * VN);
        if (!RMS) br[j] = *reinterpret_cast<const RawT*>(beta + vc * VN);
      }
      float o[VN];
#pragma unroll
      for (int i = 0; i < VN; ++i) o[i] = (float)gr[j][i] * ((vals[j][i] - mu) * rs) + (RMS ? 0.f : (float)br[j][i]);
      if (v < nv) store_vec<T>(ur + v * VN, o);
    }
    if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
  }
}

constexpr int kLnBwdRowsPerBlock = 8;

// out = resid + rstd * (g - mean(g) - xhat * mean(g*xhat)),  g = du * gamma
// part_g[blk][h] = sum over the block's rows of du*xhat, part_b[blk][h] = sum of du
// RMS: backward of the root-mean-square norm, out = resid + rstd * (g - xhat * mean(g*xhat)) with xhat = x * rstd
// (part_b is still written, and not used).
//
// A block of four wavefronts works on its 8 rows together, two rows at a time: a thread owns the same MV 16-byte
// column groups of every row, so the column sums of the parameter gradients stay in its registers from the first row to
// the last (no reduction across wavefronts at the end) and a row costs it 3 x MV vectors.  With so few registers per
// row the loads of the next two rows are in flight while these two are reduced and written.  (One wavefront per row,
// the row in registers, needed 234 registers at H = 2048 and left two wavefronts per SIMD taking turns between a burst
// of loads and a burst of stores: 0.50-0.57 of the memory's rate.)  The two row sums go through LDS: one barrier per
// pair of rows, the slots alternate so that a second one is not needed.
// SUMS: the block's column sums of `out` go to part_s as well (the bias gradient of a projection that writes into the
// residual stream is the column sum of the stream's gradient, which is this kernel's result).
// RESID: there is a residual to add (otherwise `resid` is not read).
template <typename T, int MV, bool RMS, bool SUMS, bool RESID>
__global__ void __launch_bounds__(kThreads)
ln_bwd_kernel(const float* __restrict__ du, const float* __restrict__ x, const float* __restrict__ mean,
              const float* __restrict__ rstd, const T* __restrict__ gamma, const float* __restrict__ resid,
              float* __restrict__ out, T* __restrict__ out_lowp, float* __restrict__ part_g, float* __restrict__ part_b,
              float* __restrict__ part_s, int rows, int H) {
  constexpr int VN = Vec<T>::N;
  constexpr int R = 2;                                   // rows per step
  constexpr int STEPS = kLnBwdRowsPerBlock / R;
  constexpr bool AHEAD = MV <= 2;                        // wide rows: no room for the next step's rows
  __shared__ float red[2][R][2][kWaves];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nv = H / VN;
  const float inv_h = 1.0f / (float)H;
  const int row0 = blockIdx.x * kLnBwdRowsPerBlock;

  float gm[MV][VN], dg[MV][VN], db[MV][VN], ds[SUMS ? MV : 1][VN];
#pragma unroll
  for (int j = 0; j < MV; ++j) {
    const int v = threadIdx.x + kThreads * j;
    if (v < nv) {
      load_vec<T>(gamma + v * VN, gm[j]);
    } else {
#pragma unroll
      for (int i = 0; i < VN; ++i) gm[j][i] = 0.f;
    }
#pragma unroll
    for (int i = 0; i < VN; ++i) { dg[j][i] = 0.f; db[j][i] = 0.f; }
    if (SUMS) {
#pragma unroll
      for (int i = 0; i < VN; ++i) ds[j][i] = 0.f;
    }
  }

  struct Rows { float d[R][MV][VN], xv[R][MV][VN], rr[R][MV][VN]; };
  auto fetch = [&](Rows& b, int step) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int row = row0 + step * R + r;
#pragma unroll
      for (int j = 0; j < MV; ++j) {
        // (no branch around the loads: a group past the last row or the row's end reads a valid one instead and is
        // replaced by zeros -- it contributes nothing and is not stored; with the loads under bounds branches the
        // compiler waits for all of them at once and the rows asked for ahead do not overlap the arithmetic)
        const int v = threadIdx.x + kThreads * j;
        const bool ok = row < rows && v < nv;
        const int64_t o = (int64_t)min(row, rows - 1) * H + (v < nv ? v : 0) * VN;
        load_f32<VN>(du + o, b.d[r][j]);
        load_f32<VN>(x + o, b.xv[r][j]);
        if (RESID) {
          load_f32<VN>(resid + o, b.rr[r][j]);
        } else {
#pragma unroll
          for (int i = 0; i < VN; ++i) b.rr[r][j][i] = 0.f;
        }
        // a zero gradient is all it takes: every sum below has it as a factor, and the result of such a group is not stored
#pragma unroll
        for (int i = 0; i < VN; ++i) b.d[r][j][i] = ok ? b.d[r][j][i] : 0.f;
      }
    }
  };
  auto reduce_and_store = [&](Rows& b, int step) {
    float rs[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int row = min(row0 + step * R + r, rows - 1);
      const float mu = RMS ? 0.f : mean[row];
      rs[r] = rstd[row];
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int j = 0; j < MV; ++j)
#pragma unroll
        for (int i = 0; i < VN; ++i) {
          const float d = b.d[r][j][i];
          const float xh = (b.xv[r][j][i] - mu) * rs[r];
          const float g = d * gm[j][i];
          s1 += g;
          s2 += g * xh;
          dg[j][i] += d * xh;
          db[j][i] += d;
          b.xv[r][j][i] = xh;
          b.d[r][j][i] = g;
        }
      s1 = wave_sum(s1);
      s2 = wave_sum(s2);
      if (lane == 0) { red[step & 1][r][0][wave] = s1; red[step & 1][r][1][wave] = s2; }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int row = row0 + step * R + r;
      float c1 = 0.f, c2 = 0.f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) { c1 += red[step & 1][r][0][w]; c2 += red[step & 1][r][1][w]; }
      c1 = RMS ? 0.f : c1 * inv_h;
      c2 *= inv_h;
      if (row < rows) {
#pragma unroll
        for (int j = 0; j < MV; ++j) {
          const int v = threadIdx.x + kThreads * j;
          if (v < nv) {
            float o[VN];
#pragma unroll
            for (int i = 0; i < VN; ++i) o[i] = b.rr[r][j][i] + rs[r] * (b.d[r][j][i] - c1 - b.xv[r][j][i] * c2);
            if (SUMS) {
#pragma unroll
              for (int i = 0; i < VN; ++i) ds[j][i] += o[i];
            }
            store_f32<VN>(out + (int64_t)row * H + v * VN, o);
            if (out_lowp) store_vec<T>(out_lowp + (int64_t)row * H + v * VN, o);
          }
        }
      }
    }
  };
  if constexpr (AHEAD) {
    Rows b0, b1;
    fetch(b0, 0);
#pragma unroll
    for (int step = 0; step < STEPS; step += 2) {
      fetch(b1, step + 1);
      reduce_and_store(b0, step);
      if (step + 2 < STEPS) fetch(b0, step + 2);
      reduce_and_store(b1, step + 1);
    }
  } else {
    Rows b0;
#pragma unroll 1
    for (int step = 0; step < STEPS; ++step) {
      fetch(b0, step);
      reduce_and_store(b0, step);
    }
  }
  float* pg = part_g + (int64_t)blockIdx.x * H;
  float* pb = part_b + (int64_t)blockIdx.x * H;
#pragma unroll
  for (int j = 0; j < MV; ++j) {
    const int v = threadIdx.x + kThreads * j;
    if (v < nv) {
      store_f32<VN>(pg + v * VN, dg[j]);
      store_f32<VN>(pb + v * VN, db[j]);
      if (SUMS) store_f32<VN>(part_s + (int64_t)blockIdx.x * H + v * VN, ds[j]);
    }
  }
}

// out[y][n] = (accumulate ? out[y][n] : 0) + scale * sum over the chunks c of group y of partials[c][n], group y =
// chunks [y*per_group, (y+1)*per_group).  A block owns 64 columns of one group; its four wavefronts take chunks
// w, w+4, ... and their sums are combined in a fixed order, so the result does not depend on scheduling.
__global__ void __launch_bounds__(kThreads)
reduce_partials_kernel(const float* __restrict__ partials, int nchunks, int per_group, int N, float* __restrict__ out,
                       float scale, int accumulate) {
  __shared__ float red[kWaves][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = blockIdx.x * 64 + lane;
  const int c0 = blockIdx.y * per_group, c1 = min(nchunks, c0 + per_group);
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  if (n < N) {
    int c = c0 + wave;
    for (; c + 3 * kWaves < c1; c += 4 * kWaves) {
      s0 += partials[(int64_t)c * N + n];
      s1 += partials[(int64_t)(c + kWaves) * N + n];
      s2 += partials[(int64_t)(c + 2 * kWaves) * N + n];
      s3 += partials[(int64_t)(c + 3 * kWaves) * N + n];
    }
    for (; c < c1; c += kWaves) s0 += partials[(int64_t)c * N + n];
  }
  red[wave][lane] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (wave == 0 && n < N) {
    const float s = (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
    float* o = out + (int64_t)blockIdx.y * N + n;
    *o = (accumulate ? *o : 0.f) + scale * s;
  }
}

constexpr int kReduceGroup = 32;    // chunks per first-stage group of a two-stage reduction

constexpr int kColsumRowsPerChunk = 64;

template <typename T>
__global__ void __launch_bounds__(kThreads)
colsum_kernel(const T* __restrict__ dY, float* __restrict__ partials, int rows, int N) {
  constexpr int VN = Vec<T>::N;
  const int v = blockIdx.x * kThreads + threadIdx.x;  // vector column
  if (v * VN >= N) return;
  const int r0 = blockIdx.y * kColsumRowsPerChunk;
  const int r1 = min(rows, r0 + kColsumRowsPerChunk);
  float acc[VN];
#pragma unroll
  for (int i = 0; i < VN; ++i) acc[i] = 0.f;
  for (int r = r0; r < r1; ++r) {
    float d[VN];
    load_vec<T>(dY + (int64_t)r * N + v * VN, d);
#pragma unroll
    for (int i = 0; i < VN; ++i) acc[i] += d[i];
  }
  float* p = partials + (int64_t)blockIdx.y * N + v * VN;
#pragma unroll
  for (int i = 0; i < VN; ++i) p[i] = acc[i];
}

// 64x64 tile transposed through LDS: 16-byte global reads along the input rows, 16-byte global
// writes along the output rows; the LDS tile is padded so that the column walk is conflict-free.
// out has row pitch `pitch` >= rows; its columns [rows, pitch) are written with zeros.
__global__ void __launch_bounds__(kThreads)
transpose_bf16_kernel(const bf16* __restrict__ in, bf16* __restrict__ out, int rows, int cols, int pitch) {
  __shared__ bf16 tile[64][64 + 2];
  typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int v = threadIdx.x + kThreads * p;
    const int r = v >> 3, c = (v & 7) * 8;
    bf16x8 val = {0, 0, 0, 0, 0, 0, 0, 0};
    if (r0 + r < rows && c0 + c < cols) val = *reinterpret_cast<const bf16x8*>(in + (int64_t)(r0 + r) * cols + c0 + c);
#pragma unroll
    for (int i = 0; i < 8; ++i) tile[r][c + i] = val[i];
  }
  __syncthreads();
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int v = threadIdx.x + kThreads * p;
    const int c = v >> 3, r = (v & 7) * 8;       // output row c, output columns r..r+7
    if (c0 + c < cols && r0 + r < pitch) {
      bf16x8 val;
#pragma unroll
      for (int i = 0; i < 8; ++i) val[i] = tile[r + i][c];
      *reinterpret_cast<bf16x8*>(out + (int64_t)(c0 + c) * pitch + r0 + r) = val;
    }
  }
}

template <typename T> int maxv_for(int H) {
  const int nv = H / Vec<T>::N;
  const int need = (nv + 63) / 64;
  int m = 1;
  while (m < need) m *= 2;
  return m;
}

}  // namespace

template <typename T>
int launch_ln_fwd(const float* x, const T* gamma, const T* beta, T* u, float* mean, float* rstd,
                  int rows, int H, float eps, hipStream_t s, bool rms) {
  const int grid = (rows + kWaves - 1) / kWaves;
#define LN_FWD_CASE(MV)                                                                             \
  case MV:                                                                                          \
    if (rms) ln_fwd_kernel<T, MV, true><<<grid, kThreads, 0, s>>>(x, gamma, beta, u, mean, rstd, rows, H, eps);    \
    else ln_fwd_kernel<T, MV, false><<<grid, kThreads, 0, s>>>(x, gamma, beta, u, mean, rstd, rows, H, eps);    \
    break;
  switch (maxv_for<T>(H)) {
    LN_FWD_CASE(1) LN_FWD_CASE(2) LN_FWD_CASE(4) LN_FWD_CASE(8) LN_FWD_CASE(16)
    default: return fail(CEPHALO_EUNSUPPORTED, "layer norm: hidden width %d too large", H);
  }
#undef LN_FWD_CASE
  CEPHALO_CHECK_LAUNCH("ln_fwd");
  return CEPHALO_OK;
}

int ln_bwd_blocks(int rows) { return (rows + kLnBwdRowsPerBlock - 1) / kLnBwdRowsPerBlock; }

template <typename T>
int launch_ln_bwd(const float* du, const float* x, const float* mean, const float* rstd, const T* gamma,
                  const float* resid, float* out, T* out_lowp, float* part_g, float* part_b, int rows, int H, hipStream_t s, bool rms,
                  float* part_s) {
  if (rms && part_s) return fail(CEPHALO_EINVAL, "norm backward: column sums of the result go with the LayerNorm form only");
  const int nblocks = ln_bwd_blocks(rows);
  const int nv = H / Vec<T>::N;
  int mv = 1;
  while (mv * kThreads < nv) mv *= 2;          // 16-byte column groups per thread
#define LN_BWD_FORMS(MV, RESID)                                                                                      \
    { if (rms) ln_bwd_kernel<T, MV, true, false, RESID><<<nblocks, kThreads, 0, s>>>(du, x, mean, rstd, gamma, resid, out, out_lowp, part_g, part_b, nullptr, rows, H); \
      else if (part_s) ln_bwd_kernel<T, MV, false, true, RESID><<<nblocks, kThreads, 0, s>>>(du, x, mean, rstd, gamma, resid, out, out_lowp, part_g, part_b, part_s, rows, H); \
      else ln_bwd_kernel<T, MV, false, false, RESID><<<nblocks, kThreads, 0, s>>>(du, x, mean, rstd, gamma, resid, out, out_lowp, part_g, part_b, nullptr, rows, H); }
#define LN_BWD_CASE(MV)                                                                                               \
  case MV:                                                                                                            \
    if (resid) LN_BWD_FORMS(MV, true) else LN_BWD_FORMS(MV, false)                                                    \
    break;
  switch (mv) {
    LN_BWD_CASE(1) LN_BWD_CASE(2) LN_BWD_CASE(4)
    default: return fail(CEPHALO_EUNSUPPORTED, "layer norm: hidden width %d too large", H);
  }
#undef LN_BWD_CASE
#undef LN_BWD_FORMS
  CEPHALO_CHECK_LAUNCH("ln_bwd");
  return CEPHALO_OK;
}

size_t reduce_tmp_bytes(int nchunks, int N) {
  return nchunks > 2 * kReduceGroup ? (size_t)((nchunks + kReduceGroup - 1) / kReduceGroup) * N * sizeof(float) : 0;
}

int launch_reduce_partials(const float* partials, int nchunks, int N, float* g, float scale, int accumulate,
                           float* tmp, size_t tmp_bytes, hipStream_t s) {
  const size_t need = reduce_tmp_bytes(nchunks, N);
  if (need && tmp && tmp_bytes >= need) {     // many chunks: groups of 32 first (one block per group and 64 columns), then the groups
    const int groups = (nchunks + kReduceGroup - 1) / kReduceGroup;
    reduce_partials_kernel<<<dim3((N + 63) / 64, groups), kThreads, 0, s>>>(partials, nchunks, kReduceGroup, N, tmp, 1.0f, 0);
    reduce_partials_kernel<<<dim3((N + 63) / 64, 1), kThreads, 0, s>>>(tmp, groups, groups, N, g, scale, accumulate);
  } else {
    reduce_partials_kernel<<<dim3((N + 63) / 64, 1), kThreads, 0, s>>>(partials, nchunks, nchunks, N, g, scale, accumulate);
  }
  CEPHALO_CHECK_LAUNCH("reduce_partials");
  return CEPHALO_OK;
}

size_t colsum_partial_bytes(int rows, int N) {
  const size_t nchunks = (rows + kColsumRowsPerChunk - 1) / kColsumRowsPerChunk;
  return nchunks * (size_t)N * sizeof(float) + reduce_tmp_bytes((int)nchunks, N);   // chunk sums, then room for the group sums
}

template <typename T>
int launch_colsum(const T* dY, float* partials, size_t partial_bytes, float* g, float scale,
                  int accumulate, int rows, int N, hipStream_t s) {
  if (partial_bytes < colsum_partial_bytes(rows, N)) return fail(CEPHALO_EWORKSPACE, "colsum: partial buffer too small");
  const int nchunks = (rows + kColsumRowsPerChunk - 1) / kColsumRowsPerChunk;
  const int nvec = N / Vec<T>::N;
  dim3 grid((nvec + kThreads - 1) / kThreads, nchunks);
  colsum_kernel<T><<<grid, kThreads, 0, s>>>(dY, partials, rows, N);
  CEPHALO_CHECK_LAUNCH("colsum");
  return launch_reduce_partials(partials, nchunks, N, g, scale, accumulate, partials + (size_t)nchunks * N, reduce_tmp_bytes(nchunks, N), s);
}

int launch_transpose_bf16(const bf16* in, bf16* out, int rows, int cols, hipStream_t s, int out_pitch) {
  if (out_pitch == 0) out_pitch = rows;
  if (out_pitch % 8 != 0 || out_pitch < rows || cols % 8 != 0)
    return fail(CEPHALO_EINVAL, "transpose: %d x %d into pitch %d: columns and pitch must be multiples of 8", rows, cols, out_pitch);
  dim3 grid((cols + 63) / 64, (out_pitch + 63) / 64);
  transpose_bf16_kernel<<<grid, kThreads, 0, s>>>(in, out, rows, cols, out_pitch);
  CEPHALO_CHECK_LAUNCH("transpose");
  return CEPHALO_OK;
}

// ---- rotary position embedding (Llama-style layer)
// Within each head the pair (2i, 2i+1) of the token at position t is rotated by the angle t * base^(-2i/d).
// The angles' cosines and sines are tabulated once per call, tab[t][i] = (cos, sin) in fp32 (fp32 power, accurate
// sincos), and every kernel that rotates (the GEMM epilogue that produces q and k, the attention backward's stores of
// dq and dk, the stand-alone kernel below) reads the same table.
static __global__ void __launch_bounds__(kThreads)
rotary_table_kernel(float* __restrict__ tab, int S, int d, float log2_base) {
  const int idx = blockIdx.x * kThreads + threadIdx.x;
  if (idx >= S * (d / 2)) return;
  const int t = idx / (d / 2), i = idx % (d / 2);
  const float inv = exp2f(-2.0f * (float)i / (float)d * log2_base);
  float sn, cs;
  sincosf((float)t * inv, &sn, &cs);
  tab[2 * idx] = cs;
  tab[2 * idx + 1] = sn;
}

int launch_rotary_table(float* tab, int S, int d, float base, hipStream_t s) {
  if (d % 8 != 0) return fail(CEPHALO_EUNSUPPORTED, "rotary: head dim %d must be a multiple of 8", d);
  const int n = S * (d / 2);
  rotary_table_kernel<<<(n + kThreads - 1) / kThreads, kThreads, 0, s>>>(tab, S, d, log2f(base));
  CEPHALO_CHECK_LAUNCH("rotary_table");
  return CEPHALO_OK;
}

// In place on the Q and K thirds of qkv [rows, 3H], position t = row % S; sign = -1 turns back (the gradient's way).
// One thread per 4 consecutive values (2 pairs).
template <typename T>
static __global__ void __launch_bounds__(kThreads)
rotary_kernel(T* __restrict__ qkv, const float* __restrict__ tab, int rows, int S, int H, int d, float sign) {
  const int per_row = 2 * H / 4;                           // groups of the Q and K parts of a row
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= (int64_t)rows * per_row) return;
  const int row = (int)(idx / per_row), col = (int)(idx % per_row) * 4;     // column within [0, 2H): Q then K
  const int t = row % S;
  T* p = qkv + (int64_t)row * 3 * H + col;
  const float* r = tab + ((int64_t)t * (d / 2) + (col % d) / 2) * 2;
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const float cs = r[2 * q], sn = sign * r[2 * q + 1];
    const float e = (float)p[2 * q], o = (float)p[2 * q + 1];
    p[2 * q] = (T)(e * cs - o * sn);
    p[2 * q + 1] = (T)(e * sn + o * cs);
  }
}

template <typename T>
int launch_rotary(T* qkv, const float* tab, int rows, int S, int H, int heads, int inverse, hipStream_t s) {
  const int d = H / heads;
  if (H % 8 != 0 || d % 8 != 0) return fail(CEPHALO_EUNSUPPORTED, "rotary: head dim %d must be a multiple of 8", d);
  const int64_t n = (int64_t)rows * (2 * H / 4);
  rotary_kernel<T><<<(int)((n + kThreads - 1) / kThreads), kThreads, 0, s>>>(qkv, tab, rows, S, H, d, inverse ? -1.0f : 1.0f);
  CEPHALO_CHECK_LAUNCH("rotary");
  return CEPHALO_OK;
}

// ---- gated SiLU feed-forward: gu [rows, 2F] = [gate | up];  h = silu(gate) * up (the backward is an epilogue of the GEMM that produces dh)
__device__ __forceinline__ float sigmoidf_(float z) { return 1.0f / (1.0f + __expf(-z)); }

template <typename T>
static __global__ void __launch_bounds__(kThreads)
swiglu_fwd_kernel(const T* __restrict__ gu, T* __restrict__ h, int64_t rows, int F) {
  constexpr int VN = Vec<T>::N;
  const int per_row = F / VN;
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= rows * per_row) return;
  const int64_t row = idx / per_row;
  const int c = (int)(idx % per_row) * VN;
  float g[VN], u[VN], o[VN];
  load_vec<T>(gu + row * 2 * F + c, g);
  load_vec<T>(gu + row * 2 * F + F + c, u);
#pragma unroll
  for (int i = 0; i < VN; ++i) o[i] = g[i] * sigmoidf_(g[i]) * u[i];
  store_vec<T>(h + row * F + c, o);
}


template <typename T>
int launch_swiglu_fwd(const T* gu, T* h, int64_t rows, int F, hipStream_t s) {
  const int64_t n = rows * (F / Vec<T>::N);
  swiglu_fwd_kernel<T><<<(int)((n + kThreads - 1) / kThreads), kThreads, 0, s>>>(gu, h, rows, F);
  CEPHALO_CHECK_LAUNCH("swiglu_fwd");
  return CEPHALO_OK;
}

#define INSTANTIATE(T)                                                                                          \
  template int launch_ln_fwd<T>(const float*, const T*, const T*, T*, float*, float*, int, int, float, hipStream_t, bool); \
  template int launch_ln_bwd<T>(const float*, const float*, const float*, const float*, const T*, const float*, float*, \
                                T*, float*, float*, int, int, hipStream_t, bool, float*);                         \
  template int launch_rotary<T>(T*, const float*, int, int, int, int, int, hipStream_t);                          \
  template int launch_swiglu_fwd<T>(const T*, T*, int64_t, int, hipStream_t);                                     \
  template int launch_colsum<T>(const T*, float*, size_t, float*, float, int, int, int, hipStream_t);
INSTANTIATE(float)
INSTANTIATE(bf16)
#undef INSTANTIATE

}  // namespace cephalo
