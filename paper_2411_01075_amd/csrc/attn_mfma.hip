// Tiled attention forward and backward on the gfx950 matrix cores (bf16 operands, fp32 softmax
// and accumulation).  The S x S score matrix never reaches HBM: forward keeps a running row
// maximum and row sum (online softmax) and stores only the per-row log-sum-exp; backward
// recomputes the probabilities from Q, K and that log-sum-exp.
//
// Orientation.  v_mfma_f32_32x32x16_bf16 leaves each lane with ONE column of the 32x32 result
// (column lane%32) and 16 of its rows.  Every product is arranged so that the column is the
// index whose per-row statistics are needed and the rows are the index contracted next:
//   forward / dQ : S^T[t][q] = K Q^T  -> lane owns query q: max, sum, lse[q], rowsum(dO*O)[q] are
//                  lane scalars; the rows t feed the next product (O^T = V^T P^T, dQ^T = K^T dS^T)
//                  straight from registers as its B operand.
//   dK / dV      : S[q][t] = Q K^T    -> lane owns key t; rows q feed dV^T = dO^T P, dK^T = Q^T dS.
// The other operand of those second products (V^T, K^T, dO^T, Q^T: d-major views of row-major
// [token][d] tiles) is fetched from LDS with the transposing read ds_read_b64_tr_b16.
#include <type_traits>
#include "kernels.h"
#include <cstdlib>

namespace cephalo {
namespace {

typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
#define LDS_AS __attribute__((address_space(3)))
typedef LDS_AS bf16 lds_bf16;

constexpr int kThreads = 256;
constexpr int TILE = 64;            // tokens per LDS tile
constexpr float kLog2e = 1.44269504088896340736f;
constexpr float kLn2 = 0.69314718055994530942f;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
// the same descriptor as four words (base, base high half with stride 0, extent, flags), for inline assembly
typedef int i32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ i32x4 make_rsrc_words(const void* p, unsigned bytes) {
  const uint64_t addr = (uint64_t)(uintptr_t)p;
  return i32x4{(int)(unsigned)addr, (int)(unsigned)((addr >> 32) & 0xffffu), (int)bytes, 0x00020000};
}

// ROWS tokens by D values of one operand in LDS, staged by THREADS threads (through registers, or straight from
// global memory).
//
// Two layouts.  D = 64: rows padded to 72 elements (pitch 36 banks: a 16-byte fragment read has 16 lanes on 16
// consecutive rows, a transposing read has each group of 16 lanes on 4 consecutive rows; both fall on distinct banks).
// D = 128: rows of exactly 256 bytes (all 64 banks) with the 16-byte chunks of a row permuted,
//     chunk c of row r lives at chunk  c ^ swz(r),   swz(r) = ((r & 7) << 1) | ((r >> 3) & 1),
// so that 16 consecutive rows put the same chunk on 16 different places (fragment reads) and 4 consecutive rows put a
// pair of neighbouring chunks on 4 different pairs (transposing reads).  Without padding a direct-to-LDS load of 16
// bytes per lane fills 1 KiB = 4 whole rows at once; the permutation is applied by the address each lane fetches.
// (With padded rows only 4-byte-per-lane loads fit a row, and those run at a quarter of the rate: at 64 KB per key
// tile the forward pass spent more time staging than multiplying.)
template <int D, int ROWS = TILE, int THREADS = kThreads> struct Tile {
  static constexpr bool DIRECT = D == 128;
  static constexpr int LD = DIRECT ? D : D + 8;
  static constexpr int ELEMS = ROWS * LD;
  static constexpr int PER_THREAD = ROWS * D / 8 / THREADS;
  __device__ static constexpr int swz(int r) { return ((r & 7) << 1) | ((r >> 3) & 1); }

  // rows [row0, row0+ROWS) of a [*, ld] matrix, columns [0, D); rows >= nrows and columns >= d (the head's own width,
  // a multiple of 8, when it is narrower than the tile) read as zero
  __device__ static void load_global(const bf16* __restrict__ g, int64_t ld, int row0, int nrows, bf16x8 (&reg)[PER_THREAD], int d) {
#pragma unroll
    for (int p = 0; p < PER_THREAD; ++p) {
      const int v = threadIdx.x + THREADS * p;
      const int row = v / (D / 8), c = (v % (D / 8)) * 8;
      bf16x8 val = {0, 0, 0, 0, 0, 0, 0, 0};
      if (row0 + row < nrows && c < d) val = *reinterpret_cast<const bf16x8*>(g + (int64_t)(row0 + row) * ld + c);
      reg[p] = val;
    }
  }
  // The same rows straight from global memory into LDS, no registers in between (D = 128): 16 bytes per lane, a load
  // instruction fills 4 rows.  rsrc covers exactly one sample of the [*, ld_bytes/2] matrix, col_bytes is the head's
  // column offset.  Rows past the sample's end and chunks past the head's own width d are beyond the buffer's range
  // (every part of the address is in the range-checked offset): the hardware makes them zeros; callers mask such keys.
  // The loads are asynchronous: wait for vmcnt(0) and a workgroup barrier before reading the tile.
  static constexpr int NW = THREADS / 64, LOADS = ROWS / 4, PER_WAVE = LOADS / NW;
  // the part of the offset that belongs to the lane (the same for every tile: the compiler keeps it out of the loops)
  // (wave: this wavefront's place among the THREADS / 64 that stage the tile; by default its place in the block)
  __device__ static unsigned stage_lane(int j, unsigned ld_bytes, int d, int wave = -1) {
    if (wave < 0) wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int row = (wave * PER_WAVE + j) * 4 + (lane >> 4);
    const int c = (lane & 15) ^ swz(row);
    return c * 8 < d ? (unsigned)row * ld_bytes + (unsigned)c * 16 : 0x80000000u;
  }
  // The loads are issued behind the compiler's back: it tracks loads that write LDS, cannot tell one buffer from
  // another, and makes later LDS reads of the tile being multiplied wait for them (the whole memory latency, every
  // tile).  Callers wait (vmcnt(0)) and synchronise before they read what was staged.
  __device__ static void stage_one(i32x4 rsrc, int j, unsigned tile_bytes, unsigned ld_bytes, lds_bf16* lds, int d) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned dst = (unsigned)(uintptr_t)(lds + (wave * PER_WAVE + j) * 4 * LD);
    const unsigned off = stage_lane(j, ld_bytes, d) + tile_bytes;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" :: "s"(dst), "v"(off), "s"(rsrc) : "m0");
  }
  __device__ static void stage(i32x4 rsrc, unsigned col_bytes, unsigned ld_bytes, int row0, lds_bf16* lds, int d) {
    static_assert(DIRECT && LOADS % NW == 0, "rows of 256 bytes, loads split evenly over the wavefronts");
#pragma unroll
    for (int j = 0; j < PER_WAVE; ++j) stage_one(rsrc, j, (unsigned)row0 * ld_bytes + col_bytes, ld_bytes, lds, d);
  }
  __device__ static void store_lds(lds_bf16* lds, const bf16x8 (&reg)[PER_THREAD]) {
#pragma unroll
    for (int p = 0; p < PER_THREAD; ++p) {
      const int v = threadIdx.x + THREADS * p;
      const int row = v / (D / 8), c = v % (D / 8);
      *reinterpret_cast<LDS_AS bf16x8*>(lds + row * LD + (DIRECT ? c ^ swz(row) : c) * 8) = reg[p];
    }
  }
  // operand with MFMA rows = tile rows [rb, rb+32), contraction over d in [kk, kk+16)   (rb: a multiple of 16 rows from
  // the tile's first row, so that a row's place in its group of 16 is the lane's)
  __device__ static bf16x8 frag_rows(const lds_bf16* lds, int rb, int kk) {
    const int lane = threadIdx.x & 63;
    if constexpr (DIRECT) {
      // chunk (kk/8 + h) ^ swz = (kk/8) ^ (h ^ swz): the lane's part once, the fragment's part as an XOR of the byte address
      const unsigned own = (unsigned)(lane & 31) * (LD * 2) + (unsigned)(((lane >> 5) ^ swz(lane & 15)) << 4);
      return *reinterpret_cast<const LDS_AS bf16x8*>((const LDS_AS char*)lds + rb * (LD * 2) + (own ^ (unsigned)(kk * 2)));
    } else {
      return *reinterpret_cast<const LDS_AS bf16x8*>(lds + (rb + (lane & 31)) * LD + kk + (lane >> 5) * 8);
    }
  }
  // operand with MFMA rows = d in [db, db+32), contraction over 16 tile rows in the order the
  // accumulator of a preceding 32x32 product holds them: slot 4c+i of half-wave h is tile row
  // tb + 8c + 4h + i  (tb = first of the 16 rows, a multiple of 16 rows from the tile's first row)
  __device__ static bf16x8 frag_cols(const lds_bf16* lds, int db, int tb) {
    const int lane = threadIdx.x & 63;
    const int g = lane >> 4, i = lane & 15;
    s16x4 lo, hi;
    if constexpr (DIRECT) {
      // rows r and r + 8 (r < 8): swz(r + 8) = swz(r) | 1, so the second read is the first with chunk bit 0 flipped
      const int r = 4 * (g >> 1) + (i >> 2);
      const unsigned own = (unsigned)r * (LD * 2) + (unsigned)(((2 * (g & 1) + ((i & 3) >> 1)) ^ swz(r)) << 4) + 8u * (i & 1);
      const LDS_AS char* p0 = (const LDS_AS char*)lds + tb * (LD * 2);
      lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(p0 + (own ^ (unsigned)(db * 2))));
      hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(p0 + 8 * (LD * 2) + ((own ^ 16u) ^ (unsigned)(db * 2))));
    } else {
      const lds_bf16* p0 = lds + (tb + 4 * (g >> 1) + (i >> 2)) * LD + db + 16 * (g & 1) + 4 * (i & 3);
      lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(p0));
      hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(p0 + 8 * LD));
    }
    union { struct { s16x4 a, b; } s; bf16x8 v; } u;
    u.s.a = lo; u.s.b = hi;
    return u.v;
  }
};

// Which (tile pair, head, sample) a block works on.  Blocks are dealt round-robin to the 8 XCDs, each with an L2 of its
// own, and the blocks of one head (its query-tile pairs) all stream that head's keys and values: dealt out in launch
// order they land on 8 different XCDs, every XCD fetches every head's keys and values from memory and every staged
// tile pays the full memory latency.  Give each XCD a contiguous run of the (pair, head, sample) order instead, so the
// blocks of a head sit behind one L2: the first to ask for a tile brings it in, the others hit.
struct BlockCoords { int x, y, z; };
__device__ __forceinline__ BlockCoords block_coords() {
  const int gx = gridDim.x, gy = gridDim.y, n = gx * gy * gridDim.z;
  int l = blockIdx.x + gx * (blockIdx.y + gy * blockIdx.z);
  if (n % 8 == 0) l = (l % 8) * (n / 8) + l / 8;
  // (the divisions run on the vector unit; readfirstlane tells the compiler that the results are uniform)
  return {__builtin_amdgcn_readfirstlane(l % gx), __builtin_amdgcn_readfirstlane((l / gx) % gy), __builtin_amdgcn_readfirstlane(l / (gx * gy))};
}

// fragment of 32 rows of a row-major [*, ld] matrix straight from global memory (rows = MFMA rows)
template <int D>
__device__ void load_row_frags(const bf16* __restrict__ g, int64_t ld, int row0, int nrows, bf16x8 (&f)[D / 16], int d) {
  const int lane = threadIdx.x & 63;
  const int row = row0 + (lane & 31);
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) {
    bf16x8 val = {0, 0, 0, 0, 0, 0, 0, 0};
    const int c = kk * 16 + (lane >> 5) * 8;
    if (row < nrows && c < d) val = *reinterpret_cast<const bf16x8*>(g + (int64_t)row * ld + c);
    f[kk] = val;
  }
}

// Order hint for a run of N1 products whose LDS fragment is R1 ds_read instructions each, followed by N2 products
// with R2 reads each: the fragments of the first kAhead products are requested before the first product, then each
// product is followed by the request for the product kAhead places later.  (Left alone, the compiler waits for each
// fragment right before the product that uses it, and the matrix core idles for an LDS round trip every time.)
template <int N1, int R1, int N2 = 0, int R2 = 0, int kAhead = 4>
__device__ __forceinline__ void lds_ahead_schedule() {
  constexpr int N = N1 + N2;
  static_assert(N1 >= kAhead, "the first run covers the look-ahead");
  __builtin_amdgcn_sched_group_barrier(0x100, kAhead * R1, 0);
#pragma unroll
  for (int i = 0; i < N; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if (i + kAhead < N1) __builtin_amdgcn_sched_group_barrier(0x100, R1, 0);
    else if (i + kAhead < N) __builtin_amdgcn_sched_group_barrier(0x100, R2, 0);
  }
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int e0) {
  bf16x8 r;
#pragma unroll
  for (int i = 0; i < 8; ++i) r[i] = (bf16)v[e0 + i];
  return r;
}

// accumulator rows d (4 consecutive per group) of column token -> out[token][d0 + d], scaled
template <int D>
__device__ void store_transposed(const f32x16 (&acc)[D / 32], bf16* __restrict__ out, int64_t ld, int token, int ntokens, float mul, int d) {
  if (token >= ntokens) return;
  const int h = (threadIdx.x & 63) >> 5;
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bf16x4 v;
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = (bf16)(acc[dt][4 * j + i] * mul);
      const int d0 = dt * 32 + 8 * j + 4 * h;
      if (d0 < d) *reinterpret_cast<bf16x4*>(out + (int64_t)token * ld + d0) = v;      // (d is a multiple of 8: a group of 4 is in or out)
    }
}

// The same store for a gradient with respect to rotated queries or keys: each pair (2i, 2i+1) is first turned back by
// the angle of its position, rot[token][i] = (cos, sin), so that what is stored is the gradient before the rotation.
template <int D>
__device__ void store_transposed_unrotated(const f32x16 (&acc)[D / 32], bf16* __restrict__ out, int64_t ld, int token, int ntokens, float mul,
                                           const float* __restrict__ rot, int d) {
  if (token >= ntokens) return;
  const int h = (threadIdx.x & 63) >> 5;
  const f32x4* cs = reinterpret_cast<const f32x4*>(rot + (int64_t)token * d);      // d/2 pairs of (cos, sin) per position
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int d0 = dt * 32 + 8 * j + 4 * h;
      if (d0 >= d) continue;
      const f32x4 r = cs[d0 / 4];                                                   // pairs d0/2 and d0/2 + 1
      const float e0 = acc[dt][4 * j] * mul, o0 = acc[dt][4 * j + 1] * mul, e1 = acc[dt][4 * j + 2] * mul, o1 = acc[dt][4 * j + 3] * mul;
      bf16x4 v;
      v[0] = (bf16)(e0 * r[0] + o0 * r[1]);
      v[1] = (bf16)(o0 * r[0] - e0 * r[1]);
      v[2] = (bf16)(e1 * r[2] + o1 * r[3]);
      v[3] = (bf16)(o1 * r[2] - e1 * r[3]);
      *reinterpret_cast<bf16x4*>(out + (int64_t)token * ld + d0) = v;
    }
}

// ------------------------------------------------------------------------------------ forward
template <int D, bool CAUSAL>
__global__ void __launch_bounds__(kThreads, 2)
attn_fwd_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ O, float* __restrict__ lse, int S, int H, int A, float scale) {
  typedef Tile<D> TL;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  lds_bf16* smem = (lds_bf16*)smem_raw;
  auto Ks = [&](int st) { return smem + st * 2 * TL::ELEMS; };
  auto Vs = [&](int st) { return smem + st * 2 * TL::ELEMS + TL::ELEMS; };

  const BlockCoords blk = block_coords();
  const int a = blk.y, n = blk.z;
  const int d = H / A;        // the head's own width: D, or less (a multiple of 8) with the tiles' further columns held at zero
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: tests on a wavefront's rows become real branches
  const int lane = threadIdx.x & 63, h = lane >> 5;
  const int64_t ld = 3 * (int64_t)H;
  const bf16* base = qkv + (int64_t)n * S * ld + a * d;
  const float c2 = scale * kLog2e;
  // Under a causal mask the work of a query tile grows with its index, and a launch has about as many blocks as the
  // chip has slots, so nothing would even the load out: each block takes tile x and then tile ntq-1-x, whose key
  // ranges add up to the same length for every x.
  const int ntq = (S + 127) / 128;
  for (int pass = 0; pass < (CAUSAL ? 2 : 1); ++pass) {
  const int qt = pass == 0 ? blk.x : ntq - 1 - blk.x;
  if (pass == 1 && qt == blk.x) break;   // odd tile count: the middle tile is its own partner
  const int q0 = qt * 128 + wave * 32;             // this wavefront's 32 query rows
  const int q = q0 + (lane & 31);

  bf16x8 qf[D / 16];
  load_row_frags<D>(base, ld, q0, S, qf, d);

  f32x16 o[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[dt][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const int kv_end = CAUSAL ? min(S, qt * 128 + 128) : S;
  const int ntiles = (kv_end + TILE - 1) / TILE;
  bf16x8 rk[TL::PER_THREAD], rv[TL::PER_THREAD];
  TL::load_global(base + H, ld, 0, S, rk, d);
  TL::load_global(base + 2 * H, ld, 0, S, rv, d);
  TL::store_lds(Ks(0), rk);
  TL::store_lds(Vs(0), rv);
  __syncthreads();

  for (int kt = 0; kt < ntiles; ++kt) {
    const int cur = kt & 1, t0 = kt * TILE;
    if (kt + 1 < ntiles) {
      TL::load_global(base + H, ld, t0 + TILE, S, rk, d);
      TL::load_global(base + 2 * H, ld, t0 + TILE, S, rv, d);
    }
    if (!CAUSAL || t0 <= q0 + 31) {
      // All K fragments of the tile are read before the first MFMA needs one, and the two 32-key blocks accumulate
      // in turn, so neither an LDS round trip nor a dependent accumulator sits between consecutive MFMAs.
      bf16x8 kfr[2][D / 16];
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) kfr[tb][kk] = TL::frag_rows(Ks(cur), tb * 32, kk * 16);
      f32x16 s[2];
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int e = 0; e < 16; ++e) s[tb][e] = 0.f;
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
          s[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[tb][kk], qf[kk], s[tb], 0, 0, 0);
      // Only tiles that touch the diagonal or the ragged end need per-element masking (wave-uniform test).
      if ((CAUSAL && t0 + TILE - 1 > q0) || t0 + TILE > S) {
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int t = t0 + tb * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
            if (t >= S || (CAUSAL && t > q)) s[tb][e] = -INFINITY;
          }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[tb][e]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * c2;          // scores enter the exponent as s*c2 (c2 > 0)
      // Running maximum, in the log2 domain.  It is only raised when some row of the wavefront would otherwise see
      // an exponent above 8 (probabilities up to 2^8 are harmless in fp32 / bf16 and cancel in the final division);
      // raising it costs a pass over the output accumulators, and after the first tiles it is rarely needed.
      if (__any(mx > m_run + 8.0f)) {
        const float m_new = fmaxf(m_run, mx);
        const float alpha = (m_new == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m_run - m_new);
        l_run *= alpha;
        m_run = m_new;
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
          for (int e = 0; e < 16; ++e) o[dt][e] *= alpha;
      }
      const float neg_m = (m_run == -INFINITY) ? 0.f : -m_run;
      float psum = 0.f;
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[tb][e], c2, neg_m));
          s[tb][e] = p;
          psum += p;
        }
      l_run += psum;
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
          bf16x8 vfr[D / 32];
#pragma unroll
          for (int dt = 0; dt < D / 32; ++dt) vfr[dt] = TL::frag_cols(Vs(cur), dt * 32, tb * 32 + 16 * jj);
          const bf16x8 pf = pack8(s[tb], 8 * jj);
#pragma unroll
          for (int dt = 0; dt < D / 32; ++dt)
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[dt], pf, o[dt], 0, 0, 0);
        }
    }
    if (kt + 1 < ntiles) {
      TL::store_lds(Ks(cur ^ 1), rk);
      TL::store_lds(Vs(cur ^ 1), rv);
    }
    __syncthreads();
  }
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.0f / l_tot;
  store_transposed<D>(o, O + (int64_t)n * S * H + a * d, H, q, S, inv, d);
  if (h == 0 && q < S) lse[((int64_t)n * A + a) * S + q] = (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2;
  }   // pass
}

// ------------------------------------------------------------------------------------ forward, 8 wavefronts
// The same computation with two wavefronts per SIMD: 512 threads stage 128 keys per step, wavefronts 0-3 take the
// first 64 of them and wavefronts 4-7 the second 64, for the same four blocks of 32 queries.  Each half keeps its own
// running maximum, sum and output; at the end the second half hands them over through LDS and the first half merges
// (o = o0 2^(m0-m) + o1 2^(m1-m), likewise the sums).  While one wavefront of a SIMD runs its softmax on the vector
// unit the other's MFMAs keep the matrix core busy.
constexpr int kThreads8 = 512;

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(kThreads8)
attn_fwd8_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ O, float* __restrict__ lse, int S, int H, int A, float scale) {
  typedef Tile<D, 128, kThreads8> TL;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  lds_bf16* smem = (lds_bf16*)smem_raw;
  auto Ks = [&](int st) { return smem + st * 2 * TL::ELEMS; };
  auto Vs = [&](int st) { return smem + st * 2 * TL::ELEMS + TL::ELEMS; };

  const BlockCoords blk = block_coords();
  const int a = blk.y, n = blk.z;
  const int d = H / A;        // the head's own width: D, or less (a multiple of 8) with the tiles' further columns held at zero
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: tests on a wavefront's rows become real branches
  const int lane = threadIdx.x & 63, h = lane >> 5;
  const int qsub = wave & 3, kh = wave >> 2;        // block of 32 queries, half of the staged keys
  const int64_t ld = 3 * (int64_t)H;
  const bf16* base = qkv + (int64_t)n * S * ld + a * d;
  const i32x4 rs_qkv = make_rsrc_words(qkv + (int64_t)n * S * ld, (unsigned)(S * ld * 2));
  const unsigned k_bytes = (unsigned)((H + a * d) * 2), v_bytes = (unsigned)((2 * H + a * d) * 2);
  const float c2 = scale * kLog2e;
  const int ntq = (S + 127) / 128;                  // causal: query tile x, then its mirror tile (equal work per block)
  for (int pass = 0; pass < (CAUSAL ? 2 : 1); ++pass) {
    const int qt = pass == 0 ? blk.x : ntq - 1 - blk.x;
    if (pass == 1 && qt == blk.x) break;
    const int q0 = qt * 128 + qsub * 32;
    const int q = q0 + (lane & 31);

    bf16x8 qf[D / 16];
    load_row_frags<D>(base, ld, q0, S, qf, d);
    f32x16 o[D / 32];
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[dt][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const int kv_end = CAUSAL ? min(S, qt * 128 + 128) : S;
    const int ntiles = (kv_end + 127) / 128;
    bf16x8 rk[TL::DIRECT ? 1 : TL::PER_THREAD], rv[TL::DIRECT ? 1 : TL::PER_THREAD];   // register staging (D = 64)
    if constexpr (TL::DIRECT) {
      TL::stage(rs_qkv, k_bytes, (unsigned)ld * 2, 0, Ks(0), d);
      TL::stage(rs_qkv, v_bytes, (unsigned)ld * 2, 0, Vs(0), d);
    } else {
      TL::load_global(base + H, ld, 0, S, rk, d);
      TL::load_global(base + 2 * H, ld, 0, S, rv, d);
      TL::store_lds(Ks(0), rk);
      TL::store_lds(Vs(0), rv);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                // vmcnt(0): this wavefront's rows have landed
    __syncthreads();

    for (int kt = 0; kt < ntiles; ++kt) {
      const int cur = kt & 1;
      if (kt + 1 < ntiles) {                           // the next stage flies meanwhile
        if constexpr (TL::DIRECT) {
          TL::stage(rs_qkv, k_bytes, (unsigned)ld * 2, (kt + 1) * 128, Ks(cur ^ 1), d);
          TL::stage(rs_qkv, v_bytes, (unsigned)ld * 2, (kt + 1) * 128, Vs(cur ^ 1), d);
        } else {
          TL::load_global(base + H, ld, (kt + 1) * 128, S, rk, d);
          TL::load_global(base + 2 * H, ld, (kt + 1) * 128, S, rv, d);
        }
      }
      const int t0 = kt * 128 + kh * 64;            // this wavefront's 64 keys
      const lds_bf16* Kt = Ks(cur) + kh * 64 * TL::LD;
      const lds_bf16* Vt = Vs(cur) + kh * 64 * TL::LD;
      if (t0 < S && (!CAUSAL || t0 <= q0 + 31)) {
        f32x16 s[2];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
          for (int e = 0; e < 16; ++e) s[tb][e] = 0.f;
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk)
#pragma unroll
          for (int tb = 0; tb < 2; ++tb)     // the two key blocks accumulate in turn: no dependent accumulator back to back
            s[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_rows(Kt, tb * 32, kk * 16), qf[kk], s[tb], 0, 0, 0);
        lds_ahead_schedule<D / 8, 1>();
        if ((CAUSAL && t0 + 63 > q0) || t0 + 64 > S) {      // diagonal or ragged end: per-element masking
#pragma unroll
          for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              const int t = t0 + tb * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
              if (t >= S || (CAUSAL && t > q)) s[tb][e] = -INFINITY;
            }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
          for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[tb][e]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * c2;
        if (__any(mx > m_run + 8.0f)) {                       // lazy raise of the running maximum (log2 domain)
          const float m_new = fmaxf(m_run, mx);
          const float alpha = (m_new == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m_run - m_new);
          l_run *= alpha;
          m_run = m_new;
#pragma unroll
          for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[dt][e] *= alpha;
        }
        const float neg_m = (m_run == -INFINITY) ? 0.f : -m_run;
        float psum = 0.f;
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[tb][e], c2, neg_m));
            s[tb][e] = p;
            psum += p;
          }
        l_run += psum;
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) {
            const bf16x8 pf = pack8(s[tb], 8 * jj);
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt)
              o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_cols(Vt, dt * 32, tb * 32 + 16 * jj), pf, o[dt], 0, 0, 0);
          }
        lds_ahead_schedule<D / 8, 2>();
      }
      if constexpr (!TL::DIRECT) {
        if (kt + 1 < ntiles) {
          TL::store_lds(Ks(cur ^ 1), rk);
          TL::store_lds(Vs(cur ^ 1), rv);
        }
      }
      __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0)
      __syncthreads();
    }
    // merge the two key halves: [value index][lane] floats per block of queries, lanes contiguous
    constexpr int NV = D / 32 * 16 + 2;
    LDS_AS float* mrg = (LDS_AS float*)smem_raw + qsub * NV * 64 + lane;
    if (kh == 1) {
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) mrg[(dt * 16 + e) * 64] = o[dt][e];
      mrg[(NV - 2) * 64] = m_run;
      mrg[(NV - 1) * 64] = l_run;
    }
    __syncthreads();
    if (kh == 0) {
      const float m1 = mrg[(NV - 2) * 64], l1 = mrg[(NV - 1) * 64];
      const float m = fmaxf(m_run, m1);
      const float a0 = (m_run == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_run - m);
      const float a1 = (m1 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m1 - m);
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[dt][e] = o[dt][e] * a0 + mrg[(dt * 16 + e) * 64] * a1;
      const float l = l_run * a0 + l1 * a1;
      const float l_tot = l + __shfl_xor(l, 32, 64);
      const float inv = 1.0f / l_tot;
      store_transposed<D>(o, O + (int64_t)n * S * H + a * d, H, q, S, inv, d);
      if (h == 0 && q < S) lse[((int64_t)n * A + a) * S + q] = (m + __builtin_amdgcn_logf(l_tot)) * kLn2;
    }
    __syncthreads();     // the merge area is staged over again by the next pass
  }
}

// The matrix-core step of one wavefront, written as an explicit pipeline: the LDS fragment of product i + kAhead is
// requested right after product i is issued, into the register product i just freed.  PV: the 16 products
// O^T += V^T P^T of the tile before (fragments by transposing reads); QK: the 16 products S^T = K Q^T of this tile.
// `between(i)` runs after product i is issued (the staging loads of the next tiles are dealt out there, a few at a time:
// issued in one bunch they hold the wavefront until the memory pipeline has taken them all).
template <int D, bool PV, bool QK, typename TL, typename Between>
__device__ __forceinline__ void turn_products(const lds_bf16* Vt, const lds_bf16* Kt, const bf16x8 (&pf)[2][2], const bf16x8 (&qf)[D / 16],
                                              f32x16 (&o)[D / 32], f32x16 (&s)[2], Between between) {
  static_assert(D == 128, "16 + 16 products");
  constexpr int NPV = PV ? 16 : 0, N = NPV + (QK ? 16 : 0), kAhead = 4;      // (3 to 8 ahead measure the same)
  auto fetch = [&](int i) -> bf16x8 {
    if (i < NPV) return TL::frag_cols(Vt, (i % 4) * 32, (i / 8) * 32 + 16 * ((i / 4) % 2));
    const int j = i - NPV;
    return TL::frag_rows(Kt, (j % 2) * 32, (j / 2) * 16);
  };
  bf16x8 f[kAhead];
#pragma unroll
  for (int i = 0; i < kAhead; ++i) f[i] = fetch(i);
  if (QK) {
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
      for (int e = 0; e < 16; ++e) s[tb][e] = 0.f;
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < N; ++i) {
    if (i < NPV) {
      o[i % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i % kAhead], pf[i / 8][(i / 4) % 2], o[i % 4], 0, 0, 0);
    } else {
      const int j = i - NPV;
      s[j % 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i % kAhead], qf[j / 2], s[j % 2], 0, 0, 0);
    }
    if (i + kAhead < N) f[i % kAhead] = fetch(i + kAhead);
    between(i);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// ------------------------------------------------------------------------------------ forward, two groups in turns
// The eight-wavefront forward above leaves its two groups in step: the barrier of every key tile starts them together,
// so both multiply at the same time (sharing the matrix core) and then both run their softmax at the same time (sharing
// the vector unit) -- a tile costs the sum of the two, not the larger.  Here the groups take turns.  Time is cut into
// phases closed by a barrier; in a phase one group multiplies (the products of its softmax of the tile before, then the
// scores of the next tile) while the other runs its softmax, and in the next phase they swap:
//   step 2k   of a group:  O^T += V_{k-1}^T P_{k-1}^T ;  S_k^T = K_k Q^T        (matrix core, LDS reads)
//   step 2k+1 of a group:  P_k = softmax piece of S_k                            (vector unit)
// group 0 runs step p in phase p, group 1 runs step p-1.  K_{k+1} and V_k are staged during phases 2k and 2k+1 (V is
// wanted one tile later than K now) into the buffers that K_{k-1} and V_{k-2} left at the end of phase 2k-1: group 0
// issues the loads between the products of its step 2k and waits for them at the end of phase 2k+1.  The staging
// loads are issued behind the compiler's back (it would make the next transposing LDS read wait for them).
template <int D, bool CAUSAL>
__global__ void __launch_bounds__(kThreads8)
attn_fwd_turns_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ O, float* __restrict__ lse, int S, int H, int A, float scale) {
  typedef Tile<D, 128, kThreads8> TL;
  static_assert(TL::DIRECT, "rows of 256 bytes");
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  lds_bf16* smem = (lds_bf16*)smem_raw;
  auto Ks = [&](int st) { return smem + st * 2 * TL::ELEMS; };
  auto Vs = [&](int st) { return smem + st * 2 * TL::ELEMS + TL::ELEMS; };

  const BlockCoords blk = block_coords();
  const int a = blk.y, n = blk.z;
  const int d = H / A;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63, h = lane >> 5;
  const int qsub = wave & 3, kh = wave >> 2;
  const int64_t ld = 3 * (int64_t)H;
  const bf16* base = qkv + (int64_t)n * S * ld + a * d;
  const unsigned ld_bytes = (unsigned)ld * 2;
  const unsigned k_bytes = (unsigned)((H + a * d) * 2), v_bytes = (unsigned)((2 * H + a * d) * 2);
  const i32x4 rsrc = make_rsrc_words(qkv + (int64_t)n * S * ld, (unsigned)(S * ld * 2));
  // Staging is group 0's job (its four wavefronts split a tile's 32 load instructions: 8 each per operand), dealt out
  // between the products of its matrix-core step.  Load q of a tile pair: q < 8 the keys, else the values.
  typedef Tile<D, 128, 256> TS;
  unsigned lane_part[TS::PER_WAVE];
#pragma unroll
  for (int j = 0; j < TS::PER_WAVE; ++j) lane_part[j] = kh == 0 ? TS::stage_lane(j, ld_bytes, d) : 0x80000000u;
  auto stage_one = [&](int j, unsigned col_bytes, int row0, lds_bf16* lds) {
    const unsigned dst = (unsigned)(uintptr_t)(lds + (wave * TS::PER_WAVE + j) * 4 * TL::LD);
    const unsigned off = lane_part[j] + ((unsigned)row0 * ld_bytes + col_bytes);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" :: "s"(dst), "v"(off), "s"(rsrc) : "m0");
  };
  const float c2 = scale * kLog2e;
  const int ntq = (S + 127) / 128;
  for (int pass = 0; pass < (CAUSAL ? 2 : 1); ++pass) {
    const int qt = pass == 0 ? blk.x : ntq - 1 - blk.x;
    if (pass == 1 && qt == blk.x) break;
    const int q0 = qt * 128 + qsub * 32;
    const int q = q0 + (lane & 31);

    bf16x8 qf[D / 16];
    load_row_frags<D>(base, ld, q0, S, qf, d);
    f32x16 o[D / 32];
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[dt][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const int kv_end = CAUSAL ? min(S, qt * 128 + 128) : S;
    const int ntiles = (kv_end + 127) / 128;
    // this wavefront's 64 keys of tile k start at t0(k); the piece is skipped when it lies wholly past the queries
    auto first_key = [&](int k) { return k * 128 + kh * 64; };
    auto wanted = [&](int k) { const int t0 = first_key(k); return k < ntiles && t0 < S && (!CAUSAL || t0 <= q0 + 31); };

    if (kh == 0) {
#pragma unroll
      for (int j = 0; j < TS::PER_WAVE; ++j) stage_one(j, k_bytes, 0, Ks(0));
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                // vmcnt(0)
    __syncthreads();

    f32x16 s[2];
    bf16x8 pf[2][2];
    // the matrix-core step for tile k (products of tile k-1's probabilities, then tile k's scores)
    // (tile k's scores come from K buffer k & 1, tile k-1's values from V buffer (k - 1) & 1)
    auto Vprev = [&](int k) { return Vs((k + 1) & 1) + kh * 64 * TL::LD; };
    auto Kcur = [&](int k) { return Ks(k & 1) + kh * 64 * TL::LD; };
    // the vector-unit step for tile k
    auto soften = [&](int k) {
      if (!wanted(k)) {       // this wavefront's keys lie past its queries (or past the sequence): its products add nothing
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) pf[tb][jj] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        return;
      }
      const int t0 = first_key(k);
      if ((CAUSAL && t0 + 63 > q0) || t0 + 64 > S) {      // diagonal or ragged end: per-element masking
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int t = t0 + tb * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
            if (t >= S || (CAUSAL && t > q)) s[tb][e] = -INFINITY;
          }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[tb][e]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * c2;
      if (__any(mx > m_run + 8.0f)) {                       // lazy raise of the running maximum (log2 domain)
        const float m_new = fmaxf(m_run, mx);
        const float alpha = (m_new == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m_run - m_new);
        l_run *= alpha;
        m_run = m_new;
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
          for (int e = 0; e < 16; ++e) o[dt][e] *= alpha;
      }
      const float neg_m = (m_run == -INFINITY) ? 0.f : -m_run;
      float psum = 0.f;
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[tb][e], c2, neg_m));
          s[tb][e] = p;
          psum += p;
        }
      l_run += psum;
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) pf[tb][jj] = pack8(s[tb], 8 * jj);
    };
    // load q (0..15) of the pair staged while tile k is multiplied: K of tile k+1, V of tile k
    auto stage_next = [&](int k, int q) {
      if (q < TS::PER_WAVE) { if (k + 1 < ntiles) stage_one(q, k_bytes, (k + 1) * 128, Ks((k + 1) & 1)); }
      else if (k < ntiles) stage_one(q - TS::PER_WAVE, v_bytes, k * 128, Vs(k & 1));
    };
    auto close_phase = [&](bool landed) {
      if (landed) __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the tiles staged in the phase before have landed
      __syncthreads();
    };
    // Every wavefront runs every product of the schedule (an unwanted piece multiplies zeros: it occurs only on the
    // diagonal tile), so the loop body is one straight line per group.
    auto nothing = [](int) {};
    if (kh == 0) {
      turn_products<D, false, true, TL>(nullptr, Kcur(0), pf, qf, o, s, [&](int i) { stage_next(0, i); });
      close_phase(false);
      soften(0);
      close_phase(true);
      for (int k = 1; k < ntiles; ++k) {
        turn_products<D, true, true, TL>(Vprev(k), Kcur(k), pf, qf, o, s, [&](int i) { if (i & 1) stage_next(k, i >> 1); });
        close_phase(false);
        soften(k);
        close_phase(true);
      }
      turn_products<D, true, false, TL>(Vprev(ntiles), nullptr, pf, qf, o, s, nothing);
      close_phase(false);
      close_phase(false);
    } else {
      close_phase(false);
      turn_products<D, false, true, TL>(nullptr, Kcur(0), pf, qf, o, s, nothing);
      close_phase(false);
      for (int k = 1; k < ntiles; ++k) {
        soften(k - 1);
        close_phase(false);
        turn_products<D, true, true, TL>(Vprev(k), Kcur(k), pf, qf, o, s, nothing);
        close_phase(false);
      }
      soften(ntiles - 1);
      close_phase(false);
      turn_products<D, true, false, TL>(Vprev(ntiles), nullptr, pf, qf, o, s, nothing);
      close_phase(false);
    }
    // merge the two key halves: [value index][lane] floats per block of queries, lanes contiguous
    constexpr int NV = D / 32 * 16 + 2;
    LDS_AS float* mrg = (LDS_AS float*)smem_raw + qsub * NV * 64 + lane;
    if (kh == 1) {
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) mrg[(dt * 16 + e) * 64] = o[dt][e];
      mrg[(NV - 2) * 64] = m_run;
      mrg[(NV - 1) * 64] = l_run;
    }
    __syncthreads();
    if (kh == 0) {
      const float m1 = mrg[(NV - 2) * 64], l1 = mrg[(NV - 1) * 64];
      const float m = fmaxf(m_run, m1);
      const float a0 = (m_run == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_run - m);
      const float a1 = (m1 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m1 - m);
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[dt][e] = o[dt][e] * a0 + mrg[(dt * 16 + e) * 64] * a1;
      const float l = l_run * a0 + l1 * a1;
      const float l_tot = l + __shfl_xor(l, 32, 64);
      const float inv = 1.0f / l_tot;
      store_transposed<D>(o, O + (int64_t)n * S * H + a * d, H, q, S, inv, d);
      if (h == 0 && q < S) lse[((int64_t)n * A + a) * S + q] = (m + __builtin_amdgcn_logf(l_tot)) * kLn2;
    }
    __syncthreads();     // the merge area is staged over again by the next pass
  }
}

// ------------------------------------------------------------------------------------ rowsum(dO * O)
// dvec[n, a, s] = sum_d dO[s, a*D + d] * O[s, a*D + d]; a head's D values sit in D/8 consecutive lanes
template <int D>
__global__ void __launch_bounds__(kThreads)
attn_dvec_kernel(const bf16* __restrict__ O, const bf16* __restrict__ dO, float* __restrict__ dvec, int rows, int S, int H, int A) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + wave;
  if (row >= rows) return;
  const int n = row / S, s = row % S;
  for (int v = lane; v < H / 8; v += 64) {
    float a8[8], b8[8];
    load_vec<bf16>(O + (int64_t)row * H + v * 8, a8);
    load_vec<bf16>(dO + (int64_t)row * H + v * 8, b8);
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc += a8[i] * b8[i];
#pragma unroll
    for (int o = 1; o < D / 8; o <<= 1) acc += __shfl_xor(acc, o, 64);
    if ((lane & (D / 8 - 1)) == 0) dvec[((int64_t)n * A + (v * 8) / D) * S + s] = acc;
  }
}

// the same for a head width d that is not a power of two: one thread per (token, head), d/8 vectors each
__global__ void __launch_bounds__(kThreads)
attn_dvec_any_kernel(const bf16* __restrict__ O, const bf16* __restrict__ dO, float* __restrict__ dvec, int rows, int S, int H, int A) {
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= (int64_t)rows * A) return;
  const int row = (int)(idx / A), a = (int)(idx % A), d = H / A;
  const int n = row / S, s = row % S;
  float acc = 0.f;
  for (int v = 0; v < d / 8; ++v) {
    float a8[8], b8[8];
    load_vec<bf16>(O + (int64_t)row * H + a * d + v * 8, a8);
    load_vec<bf16>(dO + (int64_t)row * H + a * d + v * 8, b8);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc += a8[i] * b8[i];
  }
  dvec[((int64_t)n * A + a) * S + s] = acc;
}

// ------------------------------------------------------------------------------------ dQ
// A block owns 128 queries (causal: tile x, then its mirror tile) and walks the keys they see in stages of 128.  Eight
// wavefronts, as in the forward kernel: wavefront w takes the 32 queries of block w & 3 and the 64 keys of half w >> 2
// of every stage; each half accumulates its own dQ and the second hands it over through LDS at the end of the pass.
// The products are taken transposed (S^T = K Q^T, dP^T = V dO^T), so that a lane's 16 values belong to one query and
// its statistics are two scalars, and dS^T is at once the operand of dQ^T += K^T dS^T.
template <int D, bool CAUSAL, bool ROT>
__global__ void __launch_bounds__(kThreads8)
attn_dq_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ dO, const float* __restrict__ lse,
               const float* __restrict__ dvec, bf16* __restrict__ dqkv, int S, int H, int A, float scale,
                const float* __restrict__ rot) {
  typedef Tile<D, 128, kThreads8> TL;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  lds_bf16* smem = (lds_bf16*)smem_raw;
  auto Ks = [&](int st) { return smem + st * 2 * TL::ELEMS; };
  auto Vs = [&](int st) { return smem + st * 2 * TL::ELEMS + TL::ELEMS; };

  const BlockCoords blk = block_coords();
  const int a = blk.y, n = blk.z;
  const int d = H / A;        // the head's own width: D, or less (a multiple of 8) with the tiles' further columns held at zero
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: tests on a wavefront's rows become real branches
  const int lane = threadIdx.x & 63, h = lane >> 5;
  const int qsub = wave & 3, kh = wave >> 2;        // block of 32 queries, half of the staged keys
  const int64_t ld = 3 * (int64_t)H;
  const bf16* base = qkv + (int64_t)n * S * ld + a * d;
  const i32x4 rs_qkv = make_rsrc_words(qkv + (int64_t)n * S * ld, (unsigned)(S * ld * 2));
  const unsigned k_bytes = (unsigned)((H + a * d) * 2), v_bytes = (unsigned)((2 * H + a * d) * 2);
  const float c2 = scale * kLog2e;
  const int ntq = (S + 127) / 128;                 // causal: query tiles x and ntq-1-x in turn (equal work per block)
  for (int pass = 0; pass < (CAUSAL ? 2 : 1); ++pass) {
  const int qt = pass == 0 ? blk.x : ntq - 1 - blk.x;
  if (pass == 1 && qt == blk.x) break;
  const int q0 = qt * 128 + qsub * 32;
  const int q = q0 + (lane & 31);

  bf16x8 qf[D / 16], dof[D / 16];
  load_row_frags<D>(base, ld, q0, S, qf, d);
  load_row_frags<D>(dO + (int64_t)n * S * H + a * d, H, q0, S, dof, d);
  const int64_t stat = ((int64_t)n * A + a) * S + q;
  const float lse2 = (q < S) ? lse[stat] * kLog2e : 0.f;
  const float dv = (q < S) ? dvec[stat] : 0.f;

  f32x16 dq[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) dq[dt][e] = 0.f;

  const int kv_end = CAUSAL ? min(S, qt * 128 + 128) : S;
  const int ntiles = (kv_end + 127) / 128;
  bf16x8 rk[TL::DIRECT ? 1 : TL::PER_THREAD], rv[TL::DIRECT ? 1 : TL::PER_THREAD];   // register staging (D = 64)
  if constexpr (TL::DIRECT) {
    TL::stage(rs_qkv, k_bytes, (unsigned)ld * 2, 0, Ks(0), d);
    TL::stage(rs_qkv, v_bytes, (unsigned)ld * 2, 0, Vs(0), d);
  } else {
    TL::load_global(base + H, ld, 0, S, rk, d);
    TL::load_global(base + 2 * H, ld, 0, S, rv, d);
    TL::store_lds(Ks(0), rk);
    TL::store_lds(Vs(0), rv);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0): this wavefront's rows have landed
  __syncthreads();

  for (int kt = 0; kt < ntiles; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < ntiles) {                             // the next stage flies meanwhile
      if constexpr (TL::DIRECT) {
        TL::stage(rs_qkv, k_bytes, (unsigned)ld * 2, (kt + 1) * 128, Ks(cur ^ 1), d);
        TL::stage(rs_qkv, v_bytes, (unsigned)ld * 2, (kt + 1) * 128, Vs(cur ^ 1), d);
      } else {
        TL::load_global(base + H, ld, (kt + 1) * 128, S, rk, d);
        TL::load_global(base + 2 * H, ld, (kt + 1) * 128, S, rv, d);
      }
    }
    const int t0 = kt * 128 + kh * 64;                 // this wavefront's 64 keys
    const lds_bf16* Kt = Ks(cur) + kh * 64 * TL::LD;
    const lds_bf16* Vt = Vs(cur) + kh * 64 * TL::LD;
    if (t0 < S && (!CAUSAL || t0 <= q0 + 31)) {
#pragma unroll
      for (int tb = 0; tb < 2; ++tb) {
        f32x16 s, dp;       // S^T and dP^T accumulate in turn: no dependent accumulator between consecutive MFMAs
#pragma unroll
        for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) {
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_rows(Kt, tb * 32, kk * 16), qf[kk], s, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_rows(Vt, tb * 32, kk * 16), dof[kk], dp, 0, 0, 0);
        }
        // (the dQ products of the first key block share a basic block with the second block's scores)
        if (tb == 0) lds_ahead_schedule<D / 8, 1>();
        else lds_ahead_schedule<D / 16, 2, D / 8, 1>();
        const int tb0 = t0 + tb * 32;
        if ((CAUSAL && tb0 + 31 > q0) || tb0 + 32 > S) {      // block touches the diagonal or the ragged end (wave-uniform)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int t = tb0 + 8 * (e >> 2) + 4 * h + (e & 3);
            float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[e], c2, -lse2));
            if (t >= S || (CAUSAL && t > q)) p = 0.f;
            s[e] = p * (dp[e] - dv);              // dS^T
          }
        } else {
#pragma unroll
          for (int e = 0; e < 16; ++e) s[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[e], c2, -lse2)) * (dp[e] - dv);
        }
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
          const bf16x8 df = pack8(s, 8 * jj);
#pragma unroll
          for (int dt = 0; dt < D / 32; ++dt)
            dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_cols(Kt, dt * 32, tb * 32 + 16 * jj), df, dq[dt], 0, 0, 0);
        }
        if (tb == 1) lds_ahead_schedule<D / 16, 2>();
      }
    }
    if constexpr (!TL::DIRECT) {
      if (kt + 1 < ntiles) {
        TL::store_lds(Ks(cur ^ 1), rk);
        TL::store_lds(Vs(cur ^ 1), rv);
      }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                // vmcnt(0)
    __syncthreads();
  }
  // the second half's sums go through LDS ([query block][value][lane], lanes contiguous) and the first half stores
  constexpr int NV = D / 32 * 16;
  LDS_AS float* mrg = (LDS_AS float*)smem_raw + qsub * NV * 64 + lane;
  if (kh == 1) {
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) mrg[(dt * 16 + e) * 64] = dq[dt][e];
  }
  __syncthreads();
  if (kh == 0) {
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) dq[dt][e] += mrg[(dt * 16 + e) * 64];
    if (ROT) store_transposed_unrotated<D>(dq, dqkv + (int64_t)n * S * ld + a * d, ld, q, S, scale, rot, d);
    else store_transposed<D>(dq, dqkv + (int64_t)n * S * ld + a * d, ld, q, S, scale, d);
  }
  __syncthreads();     // the merge area is staged over again by the next pass
  }   // pass
}

// ------------------------------------------------------------------------------------ dK, dV
// A block owns 128 keys (causal: tile x, then its mirror tile) and walks the query tiles that see them.  Eight
// wavefronts: wavefront w takes the 32 keys of group w & 3 and, of every 64-query tile, the 32 queries of half w >> 2,
// so the two wavefronts of a SIMD work on different halves and one's exponentials run under the other's MFMAs.  Each
// half accumulates its own dK and dV; at the end of the pass the second half hands its sums over through LDS.
//
// The block's keys and values stay in LDS for the whole pass: held in registers (64 of them at D = 128) they push the
// kernel past 256 registers, where the accumulators move to the second register file and every score has to be copied
// back for the vector unit.  Query and dO tiles are double-buffered; at D = 128 they come straight from global memory.
template <int D, bool CAUSAL, bool ROT>
__global__ void __launch_bounds__(kThreads8)
attn_dkv_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ dO, const float* __restrict__ lse,
                const float* __restrict__ dvec, bf16* __restrict__ dqkv, int S, int H, int A, float scale,
                const float* __restrict__ rot) {
  typedef Tile<D, TILE, kThreads8> TL;
  typedef Tile<D, 128, kThreads8> TKV;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  lds_bf16* smem = (lds_bf16*)smem_raw;
  auto Qs = [&](int st) { return smem + st * 2 * TL::ELEMS; };
  auto dOs = [&](int st) { return smem + st * 2 * TL::ELEMS + TL::ELEMS; };
  lds_bf16* Ks = smem + 4 * TL::ELEMS;
  lds_bf16* Vs = Ks + TKV::ELEMS;
  LDS_AS float* stats = (LDS_AS float*)(Vs + TKV::ELEMS);   // [2 buffers][lse2 | dvec][64]

  const BlockCoords blk = block_coords();
  const int a = blk.y, n = blk.z;
  const int d = H / A;        // the head's own width: D, or less (a multiple of 8) with the tiles' further columns held at zero
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: tests on a wavefront's rows become real branches
  const int lane = threadIdx.x & 63, h = lane >> 5;
  const int kg = wave & 3, qh = wave >> 2;          // group of 32 keys, half of the query tile
  const int64_t ld = 3 * (int64_t)H;
  const bf16* base = qkv + (int64_t)n * S * ld + a * d;
  const bf16* dObase = dO + (int64_t)n * S * H + a * d;
  const i32x4 rs_qkv = make_rsrc_words(qkv + (int64_t)n * S * ld, (unsigned)(S * ld * 2));
  const i32x4 rs_do = make_rsrc_words(dO + (int64_t)n * S * H, (unsigned)((int64_t)S * H * 2));
  const unsigned col_bytes = (unsigned)(a * d * 2);
  const float* lse_base = lse + ((int64_t)n * A + a) * S;
  const float* dv_base = dvec + ((int64_t)n * A + a) * S;
  const float c2 = scale * kLog2e;
  const int ntk = (S + 127) / 128;                 // causal: key tiles x and ntk-1-x in turn (early key tiles see the most queries)
  for (int pass = 0; pass < (CAUSAL ? 2 : 1); ++pass) {
  const int tt = pass == 0 ? blk.x : ntk - 1 - blk.x;
  if (pass == 1 && tt == blk.x) break;
  const int t0 = tt * 128 + kg * 32;               // this wavefront's 32 keys
  const int t = t0 + (lane & 31);

  if constexpr (TL::DIRECT) {
    TKV::stage(rs_qkv, (unsigned)H * 2 + col_bytes, (unsigned)ld * 2, tt * 128, Ks, d);
    TKV::stage(rs_qkv, (unsigned)H * 4 + col_bytes, (unsigned)ld * 2, tt * 128, Vs, d);
  } else {
    bf16x8 rkv[TKV::PER_THREAD];
    TKV::load_global(base + H, ld, tt * 128, S, rkv, d);
    TKV::store_lds(Ks, rkv);
    TKV::load_global(base + 2 * H, ld, tt * 128, S, rkv, d);
    TKV::store_lds(Vs, rkv);
  }

  f32x16 dk[D / 32], dvv[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) { dk[dt][e] = 0.f; dvv[dt][e] = 0.f; }

  const int first = CAUSAL ? (tt * 128) / TILE : 0;    // first query tile that can see these keys
  const int ntiles = (S + TILE - 1) / TILE;
  float rstat = 0.f;                                   // threads 0..63: lse2, 64..127: dvec
  auto load_stats = [&](int row0) {
    rstat = 0.f;
    if (threadIdx.x < 128) {
      const int r = row0 + (threadIdx.x & 63);
      if (r < S) rstat = threadIdx.x < 64 ? lse_base[r] * kLog2e : dv_base[r];
    }
  };
  bf16x8 rq[TL::DIRECT ? 1 : TL::PER_THREAD], rdo[TL::DIRECT ? 1 : TL::PER_THREAD];   // register staging (D = 64)
  if constexpr (TL::DIRECT) {
    TL::stage(rs_qkv, col_bytes, (unsigned)ld * 2, first * TILE, Qs(0), d);
    TL::stage(rs_do, col_bytes, (unsigned)H * 2, first * TILE, dOs(0), d);
  } else {
    TL::load_global(base, ld, first * TILE, S, rq, d);
    TL::load_global(dObase, H, first * TILE, S, rdo, d);
    TL::store_lds(Qs(0), rq);
    TL::store_lds(dOs(0), rdo);
  }
  load_stats(first * TILE);
  if (threadIdx.x < 128) stats[threadIdx.x] = rstat;
  __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0): this wavefront's rows have landed
  __syncthreads();

  for (int it = first; it < ntiles; ++it) {
    const int cur = (it - first) & 1, qb0 = it * TILE;
    if (it + 1 < ntiles) {                             // the next tile flies into the other stage meanwhile
      if constexpr (TL::DIRECT) {
        TL::stage(rs_qkv, col_bytes, (unsigned)ld * 2, qb0 + TILE, Qs(cur ^ 1), d);
        TL::stage(rs_do, col_bytes, (unsigned)H * 2, qb0 + TILE, dOs(cur ^ 1), d);
      } else {
        TL::load_global(base, ld, qb0 + TILE, S, rq, d);
        TL::load_global(dObase, H, qb0 + TILE, S, rdo, d);
      }
      load_stats(qb0 + TILE);
    }
    const LDS_AS float* st = stats + cur * 128;
    const int q0 = qb0 + qh * 32;                      // this wavefront's 32 queries
    if (!CAUSAL || q0 + 31 >= t0) {
      constexpr int NP = D / 8;                        // products per phase
      // S and dP of the 32 queries x 32 keys
      f32x16 sc, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) { sc[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) {
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_rows(Qs(cur), qh * 32, kk * 16), TKV::frag_rows(Ks, kg * 32, kk * 16), sc, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_rows(dOs(cur), qh * 32, kk * 16), TKV::frag_rows(Vs, kg * 32, kk * 16), dp, 0, 0, 0);
      }
      lds_ahead_schedule<NP, 2>();
      __builtin_amdgcn_sched_barrier(0);
      // P = exp2(S c2 - lse2) and dS = P (dP - dvec) as bf16 operands.  They are not written back into the MFMA results.
      f32x16 pv, dsv;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int r = qh * 32 + 8 * j + 4 * h;         // 4 consecutive query rows
        const f32x4 l4 = *reinterpret_cast<const LDS_AS f32x4*>(st + r);
        const f32x4 d4 = *reinterpret_cast<const LDS_AS f32x4*>(st + 64 + r);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int e = 4 * j + i;
          pv[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[e], c2, -l4[i]));
          dsv[e] = dp[e] - d4[i];
        }
      }
      if ((CAUSAL && t0 + 31 > q0) || q0 + 32 > S) {    // diagonal or ragged end (wave-uniform): one branch around all the masking
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int qq = q0 + 8 * (e >> 2) + 4 * h + (e & 3);
          if (qq >= S || (CAUSAL && t > qq)) pv[e] = 0.f;
        }
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) dsv[e] *= pv[e];
      // dV += P^T dO, dK += dS^T Q
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const bf16x8 pf = pack8(pv, 8 * jj), df = pack8(dsv, 8 * jj);
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt) {
          dvv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_cols(dOs(cur), dt * 32, qh * 32 + 16 * jj), pf, dvv[dt], 0, 0, 0);
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_cols(Qs(cur), dt * 32, qh * 32 + 16 * jj), df, dk[dt], 0, 0, 0);
        }
      }
      lds_ahead_schedule<NP, 2>();
    }
    if constexpr (!TL::DIRECT) {
      if (it + 1 < ntiles) {
        TL::store_lds(Qs(cur ^ 1), rq);
        TL::store_lds(dOs(cur ^ 1), rdo);
      }
    }
    if (it + 1 < ntiles && threadIdx.x < 128) stats[(cur ^ 1) * 128 + threadIdx.x] = rstat;
    __builtin_amdgcn_s_waitcnt(0x0F70);                // vmcnt(0)
    __syncthreads();
  }
  // the second half's sums go through LDS ([key group][value][lane], lanes contiguous) and the first half stores
  constexpr int NV = D / 32 * 16 * 2;
  LDS_AS float* mrg = (LDS_AS float*)smem_raw + kg * NV * 64 + lane;
  if (qh == 1) {
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        mrg[(dt * 16 + e) * 64] = dk[dt][e];
        mrg[(NV / 2 + dt * 16 + e) * 64] = dvv[dt][e];
      }
  }
  __syncthreads();
  if (qh == 0) {
    bf16* out = dqkv + (int64_t)n * S * ld + a * d;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) dvv[dt][e] += mrg[(NV / 2 + dt * 16 + e) * 64];
    store_transposed<D>(dvv, out + 2 * H, ld, t, S, 1.0f, d);
    __builtin_amdgcn_sched_barrier(0);      // dv leaves its registers before dk's merge (and its rotary factors) need theirs
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) dk[dt][e] += mrg[(dt * 16 + e) * 64];
    if (ROT) store_transposed_unrotated<D>(dk, out + H, ld, t, S, scale, rot, d);
    else store_transposed<D>(dk, out + H, ld, t, S, scale, d);
  }
  __syncthreads();     // the merge area is staged over again by the next pass
  }   // pass
}

template <typename K>
int reserve_lds(K kern, size_t bytes) {
  static bool done = false;       // one flag per kernel instantiation
  if (done) return CEPHALO_OK;
  done = true;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
    return fail(CEPHALO_EHIP, "attention: cannot reserve %zu B of LDS", bytes);
  return CEPHALO_OK;
}

template <int D, bool CAUSAL>
int fwd_cfg(const bf16* qkv, bf16* O, float* lse, int m, int S, int H, int A, hipStream_t s) {
  const int nt = (S + 127) / 128;
  dim3 grid(CAUSAL ? (nt + 1) / 2 : nt, A, m);     // causal: a block takes a tile and its mirror image
  if constexpr (CAUSAL) {
    // one paired block per compute unit: eight wavefronts, the staged keys split between two groups
    const size_t lds = 4 * (size_t)Tile<D, 128, kThreads8>::ELEMS * sizeof(bf16);
    if constexpr (Tile<D, 128, kThreads8>::DIRECT) {
      // (tiles staged straight into LDS: the two groups take turns on the matrix core and the vector unit)
      auto kern = attn_fwd_turns_kernel<D, CAUSAL>;
      int rc = reserve_lds(kern, lds);
      if (rc != CEPHALO_OK) return rc;
      kern<<<grid, kThreads8, lds, s>>>(qkv, O, lse, S, H, A, 1.0f / sqrtf((float)(H / A)));
    } else {
      auto kern = attn_fwd8_kernel<D, CAUSAL>;
      int rc = reserve_lds(kern, lds);
      if (rc != CEPHALO_OK) return rc;
      kern<<<grid, kThreads8, lds, s>>>(qkv, O, lse, S, H, A, 1.0f / sqrtf((float)(H / A)));
    }
  } else {
    // uniform tiles: two independent four-wavefront blocks per compute unit run out of phase with each other
    // (measured 12 % faster than the eight-wavefront form, whose wavefronts move in step between barriers)
    const size_t lds = 4 * (size_t)Tile<D>::ELEMS * sizeof(bf16);
    auto kern = attn_fwd_kernel<D, CAUSAL>;
    int rc = reserve_lds(kern, lds);
    if (rc != CEPHALO_OK) return rc;
    kern<<<grid, kThreads, lds, s>>>(qkv, O, lse, S, H, A, 1.0f / sqrtf((float)(H / A)));
  }
  CEPHALO_CHECK_LAUNCH("attn_fwd_mfma");
  return CEPHALO_OK;
}

template <int D, bool CAUSAL, bool ROT>
int bwd_cfg(const bf16* qkv, const bf16* O, const bf16* dO, const float* lse, float* dvec, bf16* dqkv,
            int m, int S, int H, int A, const float* rot, hipStream_t s) {
  const int d = H / A;
  const float scale = 1.0f / sqrtf((float)d);
  const int rows = m * S;
  if (d == D) attn_dvec_kernel<D><<<(rows + 3) / 4, kThreads, 0, s>>>(O, dO, dvec, rows, S, H, A);
  else if (d == 32) attn_dvec_kernel<32><<<(rows + 3) / 4, kThreads, 0, s>>>(O, dO, dvec, rows, S, H, A);
  else attn_dvec_any_kernel<<<(int)(((int64_t)rows * A + kThreads - 1) / kThreads), kThreads, 0, s>>>(O, dO, dvec, rows, S, H, A);
  const int nt = (S + 127) / 128;
  dim3 grid(CAUSAL ? (nt + 1) / 2 : nt, A, m);     // causal: a block takes a tile and its mirror image
  {
    const size_t lds = 4 * (size_t)Tile<D, 128, kThreads8>::ELEMS * sizeof(bf16);   // two stages of 128 keys and values
    auto kern = attn_dq_kernel<D, CAUSAL, ROT>;
    int rc = reserve_lds(kern, lds);
    if (rc != CEPHALO_OK) return rc;
    kern<<<grid, kThreads8, lds, s>>>(qkv, dO, lse, dvec, dqkv, S, H, A, scale, rot);
  }
  {
    // staging (2 stages of Q and dO, the keys, the values, the row statistics) or, at the end, the merge of the halves
    const size_t staging = (4 * (size_t)Tile<D>::ELEMS + 2 * (size_t)Tile<D, 128>::ELEMS) * sizeof(bf16) + 2 * 128 * sizeof(float);
    const size_t merge = (size_t)4 * (D / 32 * 16 * 2) * 64 * sizeof(float);
    const size_t lds = staging > merge ? staging : merge;
    auto kern = attn_dkv_kernel<D, CAUSAL, ROT>;
    int rc = reserve_lds(kern, lds);
    if (rc != CEPHALO_OK) return rc;
    kern<<<grid, kThreads8, lds, s>>>(qkv, dO, lse, dvec, dqkv, S, H, A, scale, rot);
  }
  CEPHALO_CHECK_LAUNCH("attn_bwd_mfma");
  return CEPHALO_OK;
}

template <int D>
int bwd_pick(const bf16* qkv, const bf16* O, const bf16* dO, const float* lse, float* dvec, bf16* dqkv,
             int m, int S, int H, int A, int causal, const float* rot, hipStream_t s) {
  if (rot) return causal ? bwd_cfg<D, true, true>(qkv, O, dO, lse, dvec, dqkv, m, S, H, A, rot, s)
                         : bwd_cfg<D, false, true>(qkv, O, dO, lse, dvec, dqkv, m, S, H, A, rot, s);
  return causal ? bwd_cfg<D, true, false>(qkv, O, dO, lse, dvec, dqkv, m, S, H, A, rot, s)
                : bwd_cfg<D, false, false>(qkv, O, dO, lse, dvec, dqkv, m, S, H, A, rot, s);
}

}  // namespace

int launch_attn_fwd_mfma(const bf16* qkv, bf16* O, float* lse, int m, int S, int H, int A, int causal, hipStream_t s) {
  const int D = A > 0 ? H / A : 0;
  if (H % 8 != 0 || !aligned16(qkv) || !aligned16(O)) return fail(CEPHALO_EINVAL, "attention: rows must be 16-byte aligned");
  if ((int64_t)S * 3 * H * 2 >= (int64_t)1 << 31)
    return fail(CEPHALO_EUNSUPPORTED, "attention: one sample of qkv (%lld bytes) exceeds the 2 GiB a buffer offset reaches", (long long)S * 3 * H * 2);
  // a head narrower than the 64- or 128-wide tile runs on that tile with its further columns held at zero
  if (A <= 0 || H % A != 0 || D % 8 != 0 || D > 128)
    return fail(CEPHALO_EUNSUPPORTED, "attention (matrix-core kernel): head dim %d is not a multiple of 8 up to 128", A > 0 ? D : 0);
  if (D <= 64) return causal ? fwd_cfg<64, true>(qkv, O, lse, m, S, H, A, s) : fwd_cfg<64, false>(qkv, O, lse, m, S, H, A, s);
  return causal ? fwd_cfg<128, true>(qkv, O, lse, m, S, H, A, s) : fwd_cfg<128, false>(qkv, O, lse, m, S, H, A, s);
}

int launch_attn_bwd_mfma(const bf16* qkv, const bf16* O, const bf16* dO, const float* lse, float* dvec, bf16* dqkv,
                         int m, int S, int H, int A, int causal, hipStream_t s, const float* rot) {
  const int D = A > 0 ? H / A : 0;
  if (H % 8 != 0 || !aligned16(qkv) || !aligned16(O) || !aligned16(dO) || !aligned16(dqkv) || !aligned16(rot))
    return fail(CEPHALO_EINVAL, "attention: rows must be 16-byte aligned");
  if ((int64_t)S * 3 * H * 2 >= (int64_t)1 << 31)
    return fail(CEPHALO_EUNSUPPORTED, "attention: one sample of qkv (%lld bytes) exceeds the 2 GiB a buffer offset reaches", (long long)S * 3 * H * 2);
  if (A <= 0 || H % A != 0 || D % 8 != 0 || D > 128)
    return fail(CEPHALO_EUNSUPPORTED, "attention (matrix-core kernel): head dim %d is not a multiple of 8 up to 128", A > 0 ? D : 0);
  if (D <= 64) return bwd_pick<64>(qkv, O, dO, lse, dvec, dqkv, m, S, H, A, causal, rot, s);
  return bwd_pick<128>(qkv, O, dO, lse, dvec, dqkv, m, S, H, A, causal, rot, s);
}

}  // namespace cephalo
