// bf16 GEMM on the gfx950 matrix cores:  C[M,N] = sum_k A(m,k) B(n,k), fp32 accumulate, fused epilogue.
//
// One kernel template covers the contractions of a linear layer; each operand is either k-contiguous or
// row-contiguous (strided along k):
//   forward          Y  = X W^T        both k-contiguous
//   input gradient   dX = dY (W^T)^T   both k-contiguous (the layer keeps a transposed copy of its weights)
//   weight gradient  dW = dY^T X       tokens are k: one operand is transposed beforehand by the caller, the other
//                                      is read row-contiguous
//
// Matrix instruction: v_mfma_f32_16x16x32_bf16.  On this chip a stream of 16x16x32 products sustains an eighth
// more than a stream of 32x32x16 products on the same data (measured with operands held in registers, the same
// 64 x 128 wavefront tile either way: 2.06 against 1.82 PFLOP/s; the chip is power-limited long before its nominal
// 2.5), and the LDS bytes per flop depend on the wavefront tile only, not on the MFMA shape.
//
// Data path.  The tile is as large as the accumulators allow (256 x 256 per block of 8 wavefronts, 64 x 128 per
// wavefront: every byte brought into LDS and every LDS byte read feeds the most MFMAs) and operand slabs of 64
// k-values go from global memory straight into LDS (buffer_load ... lds, 16 bytes per lane) without passing through
// registers.  Those loads write 64 lanes x 16 B = 1 KiB of consecutive LDS per instruction, so rows cannot be padded;
// bank conflicts are avoided by an XOR swizzle of the 16-byte chunk index, applied to the global address each lane
// fetches and again when fragments are read:
//   k-contiguous tile [row][64 k]  (128 B rows):  chunk' = chunk ^ ((row >> 1) & 7)
//   row-contiguous tile [k][rows]:                chunk' = chunk ^ (((k & 3) << 2) | (((k >> 3) & 1) << 1))
// A k-contiguous operand's MFMA fragment (16 rows x 32 k: 8 consecutive k of one row per lane) is one 16-byte LDS
// read.  A row-contiguous operand's fragment is fetched with the transposing LDS read of gfx950
// (ds_read_b64_tr_b16): within each 16-lane group, lane i supplies the address of 4 consecutive rows at one k-row
// and receives 4 k-values of row i; two such reads make a fragment.  Both read patterns are free of bank conflicts
// under the swizzles above (checked with the LDS conflict counters).
// Rows or k-values outside the matrix are never read: their buffer offsets are out of the descriptor's range and the
// hardware returns zeros.
//
// Pipeline: two or three LDS stages; the loads of the following slab(s) are in flight while a slab is multiplied;
// one barrier per slab.  The loads are issued through inline assembly (see load_slab_untracked).
#include "kernels.h"
#include <atomic>
#include <cstdlib>
#include <cstdint>
#include <algorithm>

namespace cephalo {
namespace {

typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
#define LDS_AS __attribute__((address_space(3)))

constexpr int kThreads = 256;
constexpr int BK = 64;    // k-slab
constexpr unsigned kOob = 0x80000000u;   // byte offset beyond any buffer: such a buffer load returns zero

// Buffer descriptor over `bytes` bytes at p: loads at offsets >= bytes return 0 (hardware range check).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
// the same descriptor as four words (base, base high half with stride 0, extent, flags), for inline assembly
typedef int i32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ i32x4 make_rsrc_words(const void* p, unsigned bytes) {
  const uint64_t addr = (uint64_t)(uintptr_t)p;
  return i32x4{(int)(unsigned)addr, (int)(unsigned)((addr >> 32) & 0xffffu), (int)bytes, 0x00020000};
}

// One operand's tile: ROWS matrix rows (m or n) by BK k-values, ROWS*BK*2 bytes of LDS, unpadded.
template <int ROWS, bool KFAST, int NW>
struct OperandTile {
  static constexpr int BYTES = ROWS * BK * 2;
  static constexpr int INSTR = BYTES / 1024;            // direct-to-LDS load instructions per tile (1 KiB each)
  static constexpr int PER_WAVE = INSTR / NW;           // NW wavefronts share the loads
  static constexpr int PITCH = KFAST ? BK * 2 : ROWS * 2;   // bytes per LDS row
  static constexpr int CHUNKS = PITCH / 16;                 // 16-byte chunks per LDS row
  static_assert(INSTR % NW == 0, "tile must split evenly over the wavefronts");
  static_assert(KFAST || ROWS >= 128, "row-contiguous tiles need at least 128 rows");

  // LDS row / chunk slot that lane `lane` of load instruction `j` of this wavefront fills, and the
  // (un-swizzled) chunk of the tile that belongs there
  __device__ static void slot(int j, int& line, int& chunk) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int s = (wave * PER_WAVE + j) * 64 + lane;    // 16-byte slot index within the tile
    line = s / CHUNKS;
    const int cs = s % CHUNKS;
    // (row-contiguous tiles: a half-wavefront of a transposing fragment read covers k-rows k..k+3 and k+8..k+11 at two
    // chunks each; the k bits 0, 1 and 3 spread them over the 16 chunk positions of the 64 banks)
    chunk = KFAST ? (cs ^ ((line >> 1) & 7)) : (cs ^ (((line & 3) << 2) | (((line >> 3) & 1) << 1)));
  }
  // byte offsets into the operand for k-slab 0; rows outside the matrix get the out-of-range mark
  __device__ static void init_offsets(int64_t rs, int64_t cs, int row0, int nrows, int K, unsigned (&off)[PER_WAVE]) {
#pragma unroll
    for (int j = 0; j < PER_WAVE; ++j) {
      int line, chunk;
      slot(j, line, chunk);
      if (KFAST) {      // line = tile row, chunk = 8 k-values
        const int64_t e = (int64_t)(row0 + line) * rs + chunk * 8;
        off[j] = (row0 + line < nrows) ? (unsigned)(e * 2) : kOob;
      } else {          // line = k, chunk = 8 rows
        const int64_t e = (int64_t)line * cs + row0 + chunk * 8;
        off[j] = (row0 + chunk * 8 < nrows) ? (unsigned)(e * 2) : kOob;
      }
    }
    (void)K;
  }
  // Issue the loads of the slab starting at k0 into the LDS tile at `lds` (off[] already points at that slab; rsrc:
  // the four descriptor words).  Written as assembly, behind the compiler's back: it tracks loads that write LDS,
  // cannot tell one stage from another, and makes the next transposing LDS read wait for all of them (a vmcnt(0)
  // right after the loads: their whole latency, once per slab).  The kernel writes out the waits that are needed.
  __device__ static void load_one(i32x4 rsrc, const unsigned (&off)[PER_WAVE], int k0, int K, LDS_AS char* lds, int j) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    unsigned o = off[j];
    if (KFAST) {      // a ragged last slab: chunks past K must read as zero, not as the next row
      int line, chunk;
      slot(j, line, chunk);
      if (k0 + chunk * 8 >= K) o = kOob;
    }
    const unsigned dst = (unsigned)(uintptr_t)(lds + (wave * PER_WAVE + j) * 1024);   // LDS byte address, wave-uniform
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" :: "s"(dst), "v"(o), "s"(rsrc) : "m0");
  }
  __device__ static void load_slab_untracked(i32x4 rsrc, const unsigned (&off)[PER_WAVE], int k0, int K, LDS_AS char* lds) {
#pragma unroll
    for (int j = 0; j < PER_WAVE; ++j) load_one(rsrc, off, k0, K, lds, j);
  }
  __device__ static void advance(unsigned (&off)[PER_WAVE], unsigned slab_bytes) {
#pragma unroll
    for (int j = 0; j < PER_WAVE; ++j) off[j] += slab_bytes;    // the mark stays out of range (extents are < 2^31)
  }

};

// Second half of the bf16/fp32-output epilogue: 32 rows x WTN columns of fp32 results staged row-major in LDS (pitch
// WTN + 4 floats) are read back 8 columns per lane, bias / residual / pre-activation applied, and written as
// coalesced 16-byte accesses.  A lane keeps its 8 columns and walks down the rows in PASSES steps.
//
// Everything here is straight-line code.  What the epilogue reads from memory is fetched for a whole staged block at
// once (`fetch`, into a register set), the bias once per tile; then every row's result is formed, then every row is
// stored.  All accesses go through buffer descriptors over the wavefront's 64 rows, whose range check drops what lies
// past the matrix (rows past M; columns past N get an out-of-range offset), so no row needs a branch.  Written row by
// row as load, use, store under a bounds test, every row waited for its loads behind the previous row's stores: one
// memory round trip per row, 16 in a row per tile, 12 000 to 25 000 clocks of epilogue on a tile whose main loop takes
// 83 000 at K = 2048.  (The compiler counts memory operations in order and gives up at branches.)
template <int EPI, int WTN>
struct StagedRows {
  static constexpr int SP = WTN + 4, LPR = WTN / 8, RPS = 64 / LPR, PASSES = (32 + RPS - 1) / RPS;
  static constexpr bool BIAS = EPI == EPI_BIAS || EPI == EPI_BIAS_GELU || EPI == EPI_BIAS_GELU_DERIV || EPI == EPI_BIAS_RESID;
  // 16-byte vectors a row's 8 columns need from memory
  static constexpr int NX = (EPI == EPI_BIAS_RESID || EPI == EPI_DSWIGLU || EPI == EPI_ROPE) ? 2 : (EPI == EPI_DGELU || EPI == EPI_MUL) ? 1 : 0;
  typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
  typedef f16 f16x8 __attribute__((ext_vector_type(8)));
  struct Set { f32x4 x0[PASSES], x1[PASSES]; };     // (small arrays of their own: one large one stays in scratch memory)
  float b8[8];
  int c, n, r0, ldc, mrow;
  unsigned col_off;                                  // 0, or the out-of-range mark for a lane whose columns lie past N
  __amdgpu_buffer_rsrc_t out16, out32, zed, res;     // C, Cf, Z, R or Rf: the wavefront's rows of each
  unsigned res_es, res_second;                       // residual: bytes per element, offset of its second vector

  // mrow0, ncol0: matrix coordinates of the wavefront tile's corner (64 rows: two staged blocks)
  __device__ __forceinline__ void init(const GemmArgs<bf16>& a, int mrow0, int ncol0, int ldc_) {
    mrow0 = __builtin_amdgcn_readfirstlane(mrow0);       // (the same in every lane: the descriptors must be scalars)
    const int lane = threadIdx.x & 63;
    c = (lane % LPR) * 8;
    n = ncol0 + c;
    r0 = lane / LPR;
    ldc = ldc_;
    mrow = mrow0;
    col_off = n < a.N ? 0u : kOob;
    const int rows = max(0, min(a.M - mrow0, 64));
    const int64_t base = (int64_t)mrow0 * ldc;
    const unsigned elems = (unsigned)rows * (unsigned)ldc;
    out16 = make_rsrc(a.C ? a.C + base : nullptr, a.C ? elems * 2 : 0);
    out32 = make_rsrc(a.Cf ? a.Cf + base : nullptr, a.Cf ? elems * 4 : 0);
    zed = make_rsrc(a.Z ? a.Z + base : nullptr, a.Z ? elems * 2 : 0);       // (bf16 or IEEE half: two bytes either way)
    res_es = a.Rf ? 4 : 2;
    res_second = a.Rf ? 16u : kOob;                                          // (a bf16 residual is one vector)
    const void* rp = a.Rf ? static_cast<const void*>(a.Rf + base) : static_cast<const void*>(a.R ? a.R + base : nullptr);
    res = make_rsrc(rp, (a.Rf || a.R) ? elems * res_es : 0);
#pragma unroll
    for (int t = 0; t < 8; ++t) b8[t] = 0.f;
    if (BIAS && n < a.N && (EPI != EPI_BIAS_RESID || a.bias)) load_vec<bf16>(a.bias + n, b8);     // (no bias: residual only)
  }
  // element offset of this lane's 8 columns in row `r` of staged block `blk`, relative to the wavefront's first row
  __device__ __forceinline__ unsigned elem(int blk, int r) const { return (unsigned)(blk * 32 + r) * (unsigned)ldc + (unsigned)n; }
  __device__ static __forceinline__ f32x4 load16(__amdgpu_buffer_rsrc_t rsrc, unsigned off) {
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, 0));
  }
  __device__ static __forceinline__ void store16(__amdgpu_buffer_rsrc_t rsrc, unsigned off, f32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(i32x4, v), rsrc, (int)off, 0, 0);
  }
  // the memory operands of staged block `blk` (0 or 1), into register set `set`
  __device__ __forceinline__ void fetch(const GemmArgs<bf16>& a, Set& set, int blk) {
    if (NX == 0) return;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      const int r = min(r0 + p * RPS, 31);
      const unsigned e = elem(blk, r);
      if (EPI == EPI_BIAS_RESID) {
        set.x0[p] = load16(res, (e * res_es) | col_off);
        set.x1[p] = load16(res, (e * res_es + res_second) | col_off);
      }
      if (EPI == EPI_DGELU || EPI == EPI_MUL) set.x0[p] = load16(zed, (e * 2) | col_off);
      if (EPI == EPI_DSWIGLU) {
        set.x0[p] = load16(zed, (e * 2) | col_off);
        set.x1[p] = load16(zed, ((e + (unsigned)a.N) * 2) | col_off);
      }
      if (EPI == EPI_ROPE) {       // (a small table: plain loads at a row and column kept inside it)
        const int m = min(mrow + blk * 32 + r, a.M - 1), nr = n < a.rot_cols ? n : 0;
        const f32x4* cs = reinterpret_cast<const f32x4*>(a.rot + ((int64_t)(m % a.rot_S) * (a.rot_d / 2) + (nr % a.rot_d) / 2) * 2);
        set.x0[p] = cs[0];
        set.x1[p] = cs[1];
      }
    }
  }
  template <typename V> __device__ static __forceinline__ void widen(const f32x4& raw, float (&out)[8]) {
    const V v = __builtin_bit_cast(V, raw);
#pragma unroll
    for (int t = 0; t < 8; ++t) out[t] = (float)v[t];
  }
  template <typename V, typename E> __device__ static __forceinline__ f32x4 narrow(const float (&in)[8]) {
    V v;
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] = (E)in[t];
    return __builtin_bit_cast(f32x4, v);
  }
  // staged block `blk`, with the operands of register set `set`
  __device__ __forceinline__ void write(const GemmArgs<bf16>& a, const LDS_AS float* stage, const Set& set, int blk) {
    float out[PASSES][8];
    f32x4 second[PASSES];         // a second output of 8 two-byte values (pre-activation, saved derivative, the up projection's gradient)
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      const int r = min(r0 + p * RPS, 31);
      const f32x4 v0 = *reinterpret_cast<const LDS_AS f32x4*>(stage + r * SP + c);
      const f32x4 v1 = *reinterpret_cast<const LDS_AS f32x4*>(stage + r * SP + c + 4);
      float (&v)[8] = out[p];
#pragma unroll
      for (int t = 0; t < 4; ++t) { v[t] = v0[t]; v[4 + t] = v1[t]; }
      if (BIAS) {
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] += b8[t];
      }
      if (EPI == EPI_BIAS_RESID) {
        if (a.Rf) {
#pragma unroll
          for (int t = 0; t < 4; ++t) { v[t] += set.x0[p][t]; v[4 + t] += set.x1[p][t]; }
        } else {
          float r8[8];
          widen<bf16x8>(set.x0[p], r8);
#pragma unroll
          for (int t = 0; t < 8; ++t) v[t] += r8[t];
        }
      }
      if (EPI == EPI_BIAS_GELU) {
        second[p] = narrow<bf16x8, bf16>(v);
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] = gelu_fast(v[t]);
      }
      if (EPI == EPI_DGELU) {
        float z8[8];
        widen<bf16x8>(set.x0[p], z8);
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] *= gelu_grad_fast(z8[t]);
      }
      if (EPI == EPI_BIAS_GELU_DERIV) {
        float d8[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) gelu_and_grad_fast(v[t], v[t], d8[t]);
        second[p] = narrow<f16x8, f16>(d8);      // a factor, not an operand: IEEE half
      }
      if (EPI == EPI_MUL) {
        float z8[8];
        widen<f16x8>(set.x0[p], z8);
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] *= z8[t];
      }
      if (EPI == EPI_ROPE) {
        if (n < a.rot_cols) {
          const f32x4 r0v = set.x0[p], r1v = set.x1[p];
          const float c4[4] = {r0v[0], r0v[2], r1v[0], r1v[2]}, s4[4] = {r0v[1], r0v[3], r1v[1], r1v[3]};
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const float e = v[2 * t], od = v[2 * t + 1];
            v[2 * t] = e * c4[t] - od * s4[t];
            v[2 * t + 1] = e * s4[t] + od * c4[t];
          }
        }
      }
      if (EPI == EPI_DSWIGLU) {     // two outputs per product: the gate's and the up projection's gradient, N columns apart
        float g8[8], u8[8], du[8];
        widen<bf16x8>(set.x0[p], g8);
        widen<bf16x8>(set.x1[p], u8);
#pragma unroll
        for (int t = 0; t < 8; ++t) swiglu_grad(g8[t], u8[t], v[t], v[t], du[t]);
        second[p] = narrow<bf16x8, bf16>(du);
      }
    }
    if (EPI != EPI_DSWIGLU && a.Cf) {        // fp32 output (residual stream, or a gradient that an element-wise kernel reads next)
#pragma unroll
      for (int p = 0; p < PASSES; ++p) {
        const unsigned e = elem(blk, min(r0 + p * RPS, 31));
        if (EPI == EPI_BIAS_GELU || EPI == EPI_BIAS_GELU_DERIV) store16(zed, (e * 2) | col_off, second[p]);
        store16(out32, (e * 4) | col_off, f32x4{out[p][0], out[p][1], out[p][2], out[p][3]});
        store16(out32, (e * 4 + 16) | col_off, f32x4{out[p][4], out[p][5], out[p][6], out[p][7]});
      }
    } else {
#pragma unroll
      for (int p = 0; p < PASSES; ++p) {
        const unsigned e = elem(blk, min(r0 + p * RPS, 31));
        if (EPI == EPI_BIAS_GELU || EPI == EPI_BIAS_GELU_DERIV) store16(zed, (e * 2) | col_off, second[p]);
        if (EPI == EPI_DSWIGLU) store16(out16, ((e + (unsigned)a.N) * 2) | col_off, second[p]);
        store16(out16, (e * 2) | col_off, narrow<bf16x8, bf16>(out[p]));
      }
    }
  }
};

// s_waitcnt operand that waits for vmcnt(n) only (6-bit counter split over two fields; the other counters at their maxima)
constexpr int vmcnt_only(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }

// The kernel.
//
// Operand fragment (16 rows x 32 k): lane l holds row l%16, k-values 8*(l/16) .. +7 -- one 16-byte LDS read of a
// k-contiguous tile, two transposing reads (4 k-values each) of a row-contiguous one.
// Accumulator of the exchanged product (C^T block): lane l owns row m = l%16 and columns n = 4*(l/16) .. +3.
// A k-slab of 64 is two k-steps.  Register plan per wavefront (tile WTM x WTN, MI = WTM/16, NI = WTN/16): MI*NI*4
// accumulators, the MI row-operand fragments of this k-step and of the next, and NI column-operand fragments that
// are refilled in place: as soon as the MI products of column block j have been issued, its register takes the
// fragment of the next k-step, which is needed a whole k-step later.
//
// L2 prefetch (PF > 0: the distance in slabs).  The blocks of an XCD walk the contracted axis in step, so the slab they
// all ask for next is in no L2 yet and every direct-to-LDS load pays the full memory latency inside a budget of one
// slab period (two stages).  One tile of the XCD's patch therefore touches each 128-byte line of the slab PF slabs
// beyond the one being loaded: a 4-byte direct-to-LDS load per wavefront and slab into a scratch line of LDS that
// nothing reads (a load without a register result, so nothing can be clobbered when it lands).  The loads proper then
// hit L2.  The prefetch is last in issue order, so the waits leave one more operation outstanding.
//
// Three A buffers, two B buffers (A3; NS = 2, no prefetch).  With two whole stages every load of a slab has to be issued
// between the mid-slab barrier (its stage falls free there) and the end of the slab, and the address unit, 16 cycles per
// load, is saturated in that window while it idles in the other half.  A third buffer for A alone still fits (5 x 32 KB
// at 256 x 256): the A tile of slab kt+2 goes into the buffer that slab kt-1 left at the previous barrier and is loaded
// during k-step 0 of slab kt, with a whole slab to land; only the B tile is loaded after the barrier.
template <int BM, int BN, int WGM, int WGN, bool AK, bool BKF, int EPI, int NS, int PF, bool A3 = false>
__global__ void __launch_bounds__(64 * WGM * WGN) gemm_mfma_kernel(GemmArgs<bf16> a, int tiles_m, int tiles_n, int slabs_per_split) {
  constexpr int NW = WGM * WGN;
  typedef OperandTile<BM, AK, NW> TA;
  typedef OperandTile<BN, BKF, NW> TB;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int MI = WTM / 16, NI = WTN / 16;
  constexpr int STAGE = TA::BYTES + TB::BYTES;
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  LDS_AS char* smem = (LDS_AS char*)smem_raw;

  // Tile order.  Blocks are dealt round-robin to the 8 XCDs (each with its own L2), so XCD x runs blocks x, x+8, ...:
  // give it a contiguous run of the tile order, and make that order walk 4-row groups of the tile grid column by
  // column, so that the tiles an XCD works on at the same time form a compact patch sharing A row-panels and B
  // column-panels in its L2.
  const int total = tiles_m * tiles_n;
  const int split = blockIdx.x / total;
  int pid = blockIdx.x % total;
  if (total % 8 == 0) pid = (pid % 8) * (total / 8) + pid / 8;
  constexpr int GROUP = 4;
  const int per_group = GROUP * tiles_n;
  const int g0 = (pid / per_group) * GROUP;
  const int gsz = min(tiles_m - g0, GROUP);
  const int tile_m = g0 + (pid % per_group) % gsz, tile_n = (pid % per_group) / gsz;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = (wave / WGN) * WTM, wn = (wave % WGN) * WTN;

  f32x4 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  const unsigned a_bytes = (unsigned)(2 * (AK ? (int64_t)a.M * a.a_rs : (int64_t)a.K * a.a_cs));
  const unsigned b_bytes = (unsigned)(2 * (BKF ? (int64_t)a.N * a.b_rs : (int64_t)a.K * a.b_cs));
  const i32x4 ra_rsrc = make_rsrc_words(a.A, a_bytes), rb_rsrc = make_rsrc_words(a.B, b_bytes);
  unsigned offa[TA::PER_WAVE], offb[TB::PER_WAVE];
  TA::init_offsets(a.a_rs, a.a_cs, m0, a.M, a.K, offa);
  TB::init_offsets(a.b_rs, a.b_cs, n0, a.N, a.K, offb);
  const unsigned a_step = (unsigned)(2 * BK * a.a_cs), b_step = (unsigned)(2 * BK * a.b_cs);   // bytes per k-slab
  const int slabs = (a.K + BK - 1) / BK;
  const int kb0 = split * slabs_per_split;
  const int nk = min(slabs - kb0, slabs_per_split);
  if (kb0 > 0) {
    TA::advance(offa, (unsigned)kb0 * a_step);
    TB::advance(offb, (unsigned)kb0 * b_step);
  }
  // Fragment addresses (per lane, for block 0 and k-step 0 of the wavefront tile).
  //  k-contiguous tile [row][64 k]: row l%16, chunk l/16; k-step 1 is chunk + 4, under the XOR swizzle the same
  //   address with bit 6 flipped; block b is 16 rows further.
  //  row-contiguous tile [k][rows]: within a group of 16 lanes, lane i addresses 4 consecutive rows (8 bytes) of
  //   k-row 8*(l/16) + i/4 and receives the 4 k-values of row i; a second read 4 k-rows further completes the 8.
  //   The swizzle term of those k-rows is the same for both reads and both k-steps; block b is two chunks further,
  //   which under the XOR is the address with b << 5 flipped (the wavefront's first chunk is a multiple of 8 or 16,
  //   so the block bits are free).
  auto frag_base = [&](bool kfast, int w0, int pitch) {
    if (kfast) return (w0 + (lane & 15)) * pitch + (((lane >> 4) ^ ((lane & 15) >> 1)) << 4);
    const int g = lane >> 4, i = lane & 15;
    const int krow = 8 * g + (i >> 2);
    const int sw = ((krow & 3) << 2) | ((g & 1) << 1);
    return krow * pitch + ((((w0 >> 3) | ((i & 3) >> 1)) ^ sw) << 4) + 8 * (i & 1);
  };
  const int fa0 = frag_base(AK, wm, TA::PITCH), fb0 = frag_base(BKF, wn, TB::PITCH);
  auto frag_a = [&](const LDS_AS char* tile, int blk, int kstep) -> bf16x8 {
    if constexpr (AK) {
      return *reinterpret_cast<const LDS_AS bf16x8*>(tile + (fa0 ^ (kstep << 6)) + blk * 16 * TA::PITCH);
    } else {
      const LDS_AS char* p0 = tile + (fa0 ^ (blk << 5)) + kstep * 32 * TA::PITCH;
      union { struct { s16x4 a, b; } s; bf16x8 v; } u;
      u.s.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(p0));
      u.s.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(p0 + 4 * TA::PITCH));
      return u.v;
    }
  };
  auto frag_b = [&](const LDS_AS char* tile, int blk, int kstep) -> bf16x8 {
    if constexpr (BKF) {
      return *reinterpret_cast<const LDS_AS bf16x8*>(tile + (fb0 ^ (kstep << 6)) + blk * 16 * TB::PITCH);
    } else {
      const LDS_AS char* p0 = tile + (fb0 ^ (blk << 5)) + kstep * 32 * TB::PITCH;
      union { struct { s16x4 a, b; } s; bf16x8 v; } u;
      u.s.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(p0));
      u.s.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(p0 + 4 * TB::PITCH));
      return u.v;
    }
  };
  constexpr int RA = AK ? 1 : 2, RB = BKF ? 1 : 2;       // LDS reads per fragment
  static_assert(AK || WTM % 64 == 0, "block bits of a row-contiguous A tile");
  static_assert(BKF || WTN % 64 == 0, "block bits of a row-contiguous B tile");

  constexpr int LOADS = TA::PER_WAVE + TB::PER_WAVE;
  constexpr int PER_SLAB = LOADS + (PF > 0 ? 1 : 0);      // memory operations a wavefront issues per slab
  constexpr int LAST = PF > 0 ? 1 : 0;                     // ... of which these come after the slab's own loads
  static_assert((NS - 1) * PER_SLAB + LAST < 64, "the outstanding loads must fit the counter");
  // Prefetch bookkeeping.  A panel of R rows has R lines per slab in either layout (k-contiguous: a row's 64 k-values;
  // row-contiguous: 64 k-rows of R / 64 lines each).  pf_k: the k-row within the slab that this lane's line belongs to
  // (0 for k-contiguous panels).
  unsigned pf_off = kOob, pf_step = 0;
  int pf_k = 0, pf_slab = kb0 + NS;
  i32x4 pf_rsrc = ra_rsrc;
  const unsigned pf_lds = (unsigned)(uintptr_t)(smem + NS * STAGE);
  if constexpr (PF > 0) {
    // The 32 tiles an XCD runs at a time are 4 tile rows by 8 tile columns: a row panel of A is wanted by 8 of them, a
    // column panel of B by 4, and one touch per line is enough -- the tile in column c of the patch takes the c-th
    // eighth of its A panel's lines, the tile in row r the r-th quarter of its B panel's.  Wavefront 0 touches A,
    // wavefront 1 touches B, the others issue the same instruction with every lane out of range (the waits count
    // operations).  Tiles that are not in step with their patch only lose the benefit.
    const int wv = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const bool in_a = wv == 0;
    const int lane_ = (int)threadIdx.x & 63;
    const bool kf = in_a ? AK : BKF;
    const int rows = in_a ? BM : BN, row0 = in_a ? m0 : n0, nrows = in_a ? a.M : a.N;
    const int share = in_a ? 8 : 4, part = in_a ? (tile_n & 7) : (tile_m & 3);
    const int lines = rows / share;                        // this tile's share of the panel's lines (<= 64)
    const int64_t rs = in_a ? a.a_rs : a.b_rs, cs = in_a ? a.a_cs : a.b_cs;
    if (wv < 2 && lane_ < lines) {
      const int t = part * lines + lane_;
      if (kf) {
        if (row0 + t < nrows) pf_off = (unsigned)(2 * ((int64_t)(row0 + t) * rs));
      } else {
        const int lpk = rows / 64, seg = t % lpk;
        pf_k = t / lpk;
        if (row0 + seg * 64 < nrows) pf_off = (unsigned)(2 * ((int64_t)pf_k * cs + row0 + seg * 64));
      }
    }
    pf_step = in_a ? a_step : b_step;
    if (!in_a) pf_rsrc = rb_rsrc;
    if (pf_off != kOob) pf_off += (unsigned)pf_slab * pf_step;
  }
  auto prefetch_next = [&]() {            // touch the lines of slab pf_slab, move on to the next slab
    if constexpr (PF > 0) {
      const unsigned o = (pf_slab * BK + pf_k < a.K) ? pf_off : kOob;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds" :: "s"(pf_lds), "v"(o), "s"(pf_rsrc) : "m0");
      if (pf_off != kOob) pf_off += pf_step;
      ++pf_slab;
    }
  };
  auto prefetch_none = [&]() {            // keeps the count of operations per slab
    if constexpr (PF > 0)
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds" :: "s"(pf_lds), "v"(kOob), "s"(pf_rsrc) : "m0");
  };
  static_assert(!A3 || (NS == 2 && PF == 0), "the third A buffer goes with two B buffers and no prefetch");
  // where slab k's tiles live: whole stages [A | B] one after the other, or (A3) three A buffers and then two B buffers
  auto a_tile = [&](int stage3, int stage) { return A3 ? smem + stage3 * TA::BYTES : smem + stage * STAGE; };
  auto b_tile = [&](int stage) { return A3 ? smem + 3 * TA::BYTES + stage * TB::BYTES : smem + stage * STAGE + TA::BYTES; };
#pragma unroll
  for (int p = 0; p < NS; ++p) {
    if (p > 0) { TA::advance(offa, a_step); TB::advance(offb, b_step); }
    TA::load_slab_untracked(ra_rsrc, offa, (kb0 + p) * BK, a.K, a_tile(p, p));
    TB::load_slab_untracked(rb_rsrc, offb, (kb0 + p) * BK, a.K, b_tile(p));
    if (p < PF) prefetch_next(); else prefetch_none();
  }
  __builtin_amdgcn_s_waitcnt(vmcnt_only((NS - 1) * PER_SLAB + LAST));
  __syncthreads();

  bf16x8 fa[2][MI], fb[NI];
#pragma unroll
  for (int i = 0; i < MI; ++i) fa[0][i] = frag_a(a_tile(0, 0), i, 0);
#pragma unroll
  for (int j = 0; j < NI; ++j) fb[j] = frag_b(b_tile(0), j, 0);

  // Row sums of A (GemmArgs::rowsum).  The wavefronts that hold the same rows of A, over the blocks of a tile row and
  // the WGN wavefront columns of each, take the k-slabs in turn.  One accumulator serves the four row fragments:
  // fragment i is multiplied by a left operand whose rows 4i..4i+3 are ones and whose other rows are zero, so that
  // result row 4i + x, column c is the sum of row c of fragment i -- lane l ends up with the sum of the wavefront's row l.
  const int owners = tiles_n * WGN, owner = tile_n * WGN + wave % WGN;
  int next_sum = 0x7fffffff;
  f32x4 rsum = {0.f, 0.f, 0.f, 0.f};
  if constexpr (EPI == EPI_GRAD) {
    static_assert(EPI != EPI_GRAD || MI == 4, "four row fragments share the accumulator");
    if (a.rowsum_part) next_sum = ((owner - kb0) % owners + owners) % owners;
  }
  auto ones_for = [&](int i, int row4) -> bf16x8 {         // row4: (this lane's operand row) / 4
    union { unsigned u[4]; bf16x8 v; } sel;
    const unsigned w = (row4 == i) ? 0x3F803F80u : 0u;      // two bf16 ones
    sel.u[0] = w; sel.u[1] = w; sel.u[2] = w; sel.u[3] = w;
    return sel.v;
  };

  constexpr int JB = 1;                                    // column blocks of k-step 1 multiplied before the barrier
  if constexpr (A3) TA::advance(offa, a_step);             // (the prologue left the offsets at slab 1; A's next load is slab 2)
  int st = 0, st3 = 0;                                     // slab kt's stage; (A3) its A buffer
  for (int kt = 0; kt < nk; ++kt) {
    const int st1 = st + 1 == NS ? 0 : st + 1;
    const int st31 = st3 + 1 == 3 ? 0 : st3 + 1, st32 = st31 + 1 == 3 ? 0 : st31 + 1;
    const LDS_AS char* As = a_tile(st3, st);
    const LDS_AS char* Bs = b_tile(st);
    const LDS_AS char* An = a_tile(st31, st1);
    const LDS_AS char* Bn = b_tile(st1);
    // Wave priority falls as a wavefront moves through a slab (2 after the barrier, 1 during k-step 0, 0 on the way
    // to the barrier).  The two wavefronts of a SIMD compete for its matrix core; left alone the older one wins every
    // time, races ahead and then sits at the barrier while the younger one runs alone and cannot keep the matrix core
    // busy by itself (timestamps showed the older wavefronts idle at the barrier for a third of every slab).  With the
    // priority tied to progress the one that is behind goes first: the slab period dropped by 9 %.
    __builtin_amdgcn_s_setprio(1);
    // k-step 0: its fragments are in registers; fetch those of k-step 1 from the same stage meanwhile
    if constexpr (A3) {
      // pinned: block j's products, its column fragment of k-step 1, a row fragment of k-step 1, and the A tile of slab
      // kt+2, one load after each of the first blocks
      fa[1][0] = frag_a(As, 0, 1);
#pragma unroll
      for (int j = 0; j < NI; ++j) {
#pragma unroll
        for (int i = 0; i < MI; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[0][i], acc[i][j], 0, 0, 0);
        fb[j] = frag_b(Bs, j, 1);
        if (j + 1 < MI) fa[1][j + 1] = frag_a(As, j + 1, 1);
#pragma unroll
        for (int q = j * TA::PER_WAVE / NI; q < (j + 1) * TA::PER_WAVE / NI; ++q)
          TA::load_one(ra_rsrc, offa, (kb0 + kt + 2) * BK, a.K, smem + st32 * TA::BYTES, q);
        __builtin_amdgcn_sched_barrier(0);
      }
      TA::advance(offa, a_step);
    } else {
#pragma unroll
    for (int i = 0; i < MI; ++i) fa[1][i] = frag_a(As, i, 1);
#pragma unroll
    for (int j = 0; j < NI; ++j) {
#pragma unroll
      for (int i = 0; i < MI; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[0][i], acc[i][j], 0, 0, 0);
      fb[j] = frag_b(Bs, j, 1);
    }
    {
      // MI reads first (the row fragments of k-step 1), then one column fragment after every MI products
      __builtin_amdgcn_sched_group_barrier(0x100, RA, 0);
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        __builtin_amdgcn_sched_group_barrier(0x008, MI, 0);
        if (j + 1 < MI) __builtin_amdgcn_sched_group_barrier(0x100, RA + RB, 0);
        else __builtin_amdgcn_sched_group_barrier(0x100, RB, 0);
      }
    }
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(0);
    if constexpr (EPI == EPI_GRAD) {
      if (kt == next_sum) {                                // this wavefront's turn: both k-steps' row fragments are in registers
        next_sum += owners;
        int row4 = (lane & 15) >> 2;
        asm volatile("" : "+v"(row4));                     // (computed here each time: kept across the loop, the four operands cost 16 registers)
#pragma unroll
        for (int i = 0; i < MI; ++i) {
          const bf16x8 sel = ones_for(i, row4);
          rsum = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sel, fa[0][i], rsum, 0, 0, 0);
          rsum = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sel, fa[1][i], rsum, 0, 0, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // k-step 1: after the first JB column blocks every read of this stage has been issued long ago; wait for slab
    // kt+1 (the loads of the NS-2 slabs after it may still fly), barrier, start the loads of slab kt+NS into this
    // stage, and refill the fragment registers from the stage of slab kt+1 as they fall free.
#pragma unroll
    for (int j = 0; j < JB; ++j)
#pragma unroll
      for (int i = 0; i < MI; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[1][i], acc[i][j], 0, 0, 0);
    // (A3: the A tile of slab kt+2, issued during k-step 0 just now, may still fly)
    __builtin_amdgcn_s_waitcnt(vmcnt_only(A3 ? TA::PER_WAVE : (NS - 2) * PER_SLAB + LAST) & 0xF0FF);     // ... and lgkmcnt(0)
    __syncthreads();
    __builtin_amdgcn_s_setprio(2);
    if constexpr (!A3) TA::advance(offa, a_step);
    TB::advance(offb, b_step);
    // From here on the order is pinned: after every column block's products (and the refill of its fragment) come a
    // share of the slab's global loads and one or two of the early fragment reads of slab kt+1.  (The loads are
    // opaque assembly, which the scheduler otherwise bunches together and strands the products behind them.)  The
    // loads are dealt evenly over all the blocks left in the slab, and only one block is multiplied before the barrier:
    // a load instruction keeps the address unit busy for 16 cycles, the 64 of a slab issued within four blocks by all
    // eight wavefronts saturate it and the wavefronts queue at issue (evenly over seven blocks: +2 %).
    constexpr int SLOTS = NI - JB;
    constexpr int EARLY = MI + JB;                         // fragments wanted at the start of the next slab
    constexpr int EPS = (EARLY + SLOTS - 1) / SLOTS;       // early fragments per slot
    constexpr int NOW = A3 ? TB::PER_WAVE : LOADS;         // loads issued after the barrier
    auto issue_load = [&](int q) {
      if constexpr (A3) {
        TB::load_one(rb_rsrc, offb, (kb0 + kt + NS) * BK, a.K, smem + 3 * TA::BYTES + st * TB::BYTES, q);
      } else {
        if (q < TA::PER_WAVE) TA::load_one(ra_rsrc, offa, (kb0 + kt + NS) * BK, a.K, smem + st * STAGE, q);
        else if (q < LOADS) TB::load_one(rb_rsrc, offb, (kb0 + kt + NS) * BK, a.K, smem + st * STAGE + TA::BYTES, q - TA::PER_WAVE);
      }
    };
    auto early_read = [&](int e) {
      if (e < MI) fa[0][e] = frag_a(An, e, 0);
      else if (e < EARLY) fb[e - MI] = frag_b(Bn, e - MI, 0);
    };
#pragma unroll
    for (int j = JB; j < NI; ++j) {
      const int slot = j - JB;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int q = slot * NOW / SLOTS; q < (slot + 1) * NOW / SLOTS; ++q) issue_load(q);
      if (j == NI - 1) prefetch_next();
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int e = 0; e < EPS; ++e) early_read(slot * EPS + e);
#pragma unroll
      for (int i = 0; i < MI; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[1][i], acc[i][j], 0, 0, 0);
      fb[j] = frag_b(Bn, j, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    st = st1;
    st3 = st31;
  }

  __builtin_amdgcn_s_setprio(0);
  // Epilogue
  if (EPI == EPI_GRAD) {
    if (a.rowsum_part) {
      const int m = m0 + wm + lane;
      if (m < a.M) a.rowsum_part[((int64_t)split * owners + owner) * a.M + m] = rsum[0];
    }
    const bool partial = a.splits > 1;
    float* const gbase = partial ? a.part + (int64_t)split * a.M * a.N : a.G;
    const float scale = partial ? 1.0f : a.scale;
    const bool accumulate = !partial && a.accumulate;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int m = m0 + wm + 16 * i + (lane & 15);
      if (m >= a.M) continue;
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        const int n = n0 + wn + 16 * j + 4 * (lane >> 4);
        if (n >= a.N) continue;                           // N is a multiple of 8: the group of 4 is inside or outside
        f32x4* gp = reinterpret_cast<f32x4*>(gbase + (int64_t)m * a.N + n);
        f32x4 v = scale * acc[i][j];
        if (accumulate) v += *gp;
        *gp = v;
      }
    }
    return;
  }
  // Other outputs: each wavefront passes its tile through its own LDS region, 32 rows at a time, to turn the
  // accumulator layout into row-major 16-byte vectors; bias, residual and pre-activation are then read, and the
  // results written, as coalesced 16-byte accesses.
  const int ldc = a.ldc ? a.ldc : a.N;
  constexpr int SP = WTN + 4;
  static_assert(NW * 32 * SP * 4 <= 160 * 1024, "staging regions must fit in LDS");
  LDS_AS float* stage = (LDS_AS float*)(smem + wave * (32 * SP * 4));
  __builtin_amdgcn_s_waitcnt(vmcnt_only(0) & 0xF0FF);     // the last (unused) slab loads and fragment reads are over,
  StagedRows<EPI, WTN> rows;
  rows.init(a, m0 + wm, n0 + wn, ldc);
  typedef typename StagedRows<EPI, WTN>::Set Operands;
  Operands set0, set1;                                    // (named, not indexed: a choice of address keeps them out of registers)
  rows.fetch(a, set0, 0);                                 // (the first block's operands fly across the barrier)
  __syncthreads();                                        // in every wavefront, before the stages are overwritten
  static_assert(MI == 4, "two staged blocks of 32 rows");
  // The second block's operands are asked for before the first block is written where one 16-byte vector per row is
  // all (two register sets); with two vectors per row the accumulators still held leave room for one set only, and the
  // second block's loads follow the first block's stores.
  constexpr bool TWO_SETS = StagedRows<EPI, WTN>::NX < 2;
  auto stage_block = [&](int i2) {
#pragma unroll
    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
      for (int j = 0; j < NI; ++j)
        *reinterpret_cast<LDS_AS f32x4*>(stage + (16 * ii + (lane & 15)) * SP + 16 * j + 4 * (lane >> 4)) = acc[2 * i2 + ii][j];
  };
  if constexpr (TWO_SETS) rows.fetch(a, set1, 1);
  stage_block(0);
  rows.write(a, stage, set0, 0);
  if constexpr (!TWO_SETS) rows.fetch(a, set0, 1);
  stage_block(1);
  rows.write(a, stage, TWO_SETS ? set1 : set0, 1);
}

// G = (accumulate ? G : 0) + scale * (part[0] + part[1] + ... ) in split order, 4 floats per thread
__global__ void __launch_bounds__(256)
splitk_reduce_kernel(const float* __restrict__ part, int splits, int64_t mn4, float* __restrict__ G, float scale, int accumulate) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= mn4) return;
  f32x4 sum = reinterpret_cast<const f32x4*>(part)[i];
  for (int p = 1; p < splits; ++p) sum += reinterpret_cast<const f32x4*>(part)[(int64_t)p * mn4 + i];
  f32x4 out = scale * sum;
  if (accumulate) out += reinterpret_cast<const f32x4*>(G)[i];
  reinterpret_cast<f32x4*>(G)[i] = out;
}

// Launch of one instantiation: LDS reservation (once), the split of the contracted axis, the reduction of the pieces.
template <auto KERN>
int launch_kernel(const GemmArgs<bf16>& a, int BMv, int BNv, int wgn, int threads, size_t lds, hipStream_t s) {
  const int tm = (a.M + BMv - 1) / BMv, tn = (a.N + BNv - 1) / BNv;
  // per instantiation; setting the attribute again with the same value is harmless, so two threads that both find the
  // flag clear may both set it
  static std::atomic<bool> attr_set{false};
  if (!attr_set.load(std::memory_order_acquire)) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(KERN), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return fail(CEPHALO_EHIP, "gemm_mfma: cannot reserve %zu B of LDS", lds);
    attr_set.store(true, std::memory_order_release);
  }
  const int slabs = (a.K + BK - 1) / BK;
  int splits = (a.epi == EPI_GRAD && a.splits > 1 && a.part) ? a.splits : 1;
  int per = (slabs + splits - 1) / splits;
  splits = (slabs + per - 1) / per;                       // every piece holds at least one k-slab
  GemmArgs<bf16> k = a;
  k.splits = splits;
  const bool rowsum = a.epi == EPI_GRAD && a.rowsum;
  const int pieces = splits * tn * wgn;                   // of the row sums: one per split and owner
  if (rowsum && (!a.rowsum_part || a.rowsum_part_bytes < (size_t)pieces * a.M * sizeof(float)))
    return fail(CEPHALO_EWORKSPACE, "gemm_mfma: %zu B for the %d pieces of %d row sums", a.rowsum_part_bytes, pieces, a.M);
  if (!rowsum) k.rowsum_part = nullptr;
  KERN<<<tm * tn * splits, threads, lds, s>>>(k, tm, tn, per);
  CEPHALO_CHECK_LAUNCH("gemm_mfma");
  if (rowsum) {
    const int rc = launch_reduce_partials(a.rowsum_part, pieces, a.M, a.rowsum, a.scale, a.accumulate, nullptr, 0, s);
    if (rc != CEPHALO_OK) return rc;
  }
  if (splits > 1) {
    const int64_t mn4 = (int64_t)a.M * a.N / 4;
    splitk_reduce_kernel<<<(int)((mn4 + 255) / 256), 256, 0, s>>>(a.part, splits, mn4, a.G, a.scale, a.accumulate);
    CEPHALO_CHECK_LAUNCH("splitk_reduce");
  }
  return CEPHALO_OK;
}

template <int BM, int BN, int WGM, int WGN, bool AK, bool BKF, int EPI, int NS = 2>
int launch_cfg(const GemmArgs<bf16>& a, hipStream_t s) {
  // The L2 prefetch pays where both operands are read token-major (the weight gradients: +3..5 % on c5's shapes); the
  // k-contiguous kernels lose 1..6 % with it, so they run without.
  constexpr int PF = (!AK && !BKF) ? 2 : 0;
  // a third buffer for A where it fits beside two whole stages (the 256 x 256 and 256 x 192 tiles)
  constexpr bool A3 = NS == 2 && PF == 0 && (size_t)(3 * BM + 2 * BN) * BK * 2 <= 160 * 1024;
  constexpr size_t stages = A3 ? (size_t)(3 * BM + 2 * BN) * BK * 2 : (size_t)NS * (BM + BN) * BK * 2 + (PF > 0 ? 256 : 0);    // + the prefetches' scratch line
  constexpr size_t staging = (size_t)WGM * WGN * 32 * (BN / WGN + 4) * 4;
  static_assert(stages <= 160 * 1024, "the stages must fit in LDS");
  const size_t lds = std::max<size_t>(stages, EPI == EPI_GRAD ? 0 : staging);
  return launch_kernel<gemm_mfma_kernel<BM, BN, WGM, WGN, AK, BKF, EPI, NS, PF, A3>>(a, BM, BN, WGN, 64 * WGM * WGN, lds, s);
}

thread_local int side_by_side = 1;     // kernels the caller runs at once (GemmSideBySide)

template <bool AK, bool BKF, int EPI>
int launch_tiles(const GemmArgs<bf16>& a, hipStream_t s) {
  // Tile choice: the score of a configuration is the fraction of the last round of blocks that the 256 compute
  // units fill, times the rate its main loop reaches relative to the 256 x 256 tile (measured: bigger tiles
  // move fewer LDS and L2 bytes per MFMA).
  const int nsplit = (EPI == EPI_GRAD && a.splits > 1 && a.part) ? a.splits : 1;
  const double cus = 256.0 / side_by_side;        // compute units this launch can count on
  auto fill = [&](int bm, int bn) {
    const double t = (double)((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn) * nsplit;
    return t / (cus * (double)(int64_t)((t + cus - 1) / cus));
  };
  int cfg = 0;
  // 256 x 128 tiles run three LDS stages (they fit, and long contractions over few tiles gain a quarter from the
  // deeper prefetch; short ones lose nothing).
  if (cfg == 0) {
    double best = fill(256, 256); cfg = 1;
    if (BKF) { const double v = 0.95 * fill(256, 192); if (v > best) { best = v; cfg = 2; } }
    { const double v = 0.83 * fill(256, 128); if (v > best) { best = v; cfg = 3; } }
    { const double v = 0.60 * fill(128, 128); if (v > best) { best = v; cfg = 4; } }
  }
  switch (cfg) {
    case 1: return launch_cfg<256, 256, 4, 2, AK, BKF, EPI>(a, s);
    case 2: if constexpr (BKF) return launch_cfg<256, 192, 4, 2, AK, BKF, EPI>(a, s); else return launch_cfg<256, 256, 4, 2, AK, BKF, EPI>(a, s);
    case 3: return launch_cfg<256, 128, 4, 2, AK, BKF, EPI, 3>(a, s);
    default: return launch_cfg<128, 128, 2, 2, AK, BKF, EPI, 3>(a, s);
  }
}

}  // namespace

int gemm_grad_splits(int M, int N, int K) {
  const double tiles = (double)((M + 255) / 256) * ((N + 255) / 256);
  int best = 1;
  double best_score = 0.0;
  for (int sp : {1, 2, 3, 4, 6, 8}) {
    if (sp > 1 && K / sp < 1024) break;                 // keep each piece's main loop long
    const double t = tiles * sp;
    const double score = t / (256.0 * (double)(int64_t)((t + 255) / 256)) * (1.0 - 0.03 * (sp - 1));   // fill, minus the second pass
    if (score > best_score + 1e-9) { best_score = score; best = sp; }
  }
  return best;
}

namespace {
std::atomic<int64_t> general_count{0};
int general(const GemmArgs<bf16>& a, hipStream_t s) {
  general_count.fetch_add(1, std::memory_order_relaxed);
  return launch_gemm_simple<bf16>(a, s);
}
}  // namespace
int64_t gemm_general_count() { return general_count.load(std::memory_order_relaxed); }
GemmSideBySide::GemmSideBySide(int kernels) : before(side_by_side) { side_by_side = kernels < 1 ? 1 : kernels; }
GemmSideBySide::~GemmSideBySide() { side_by_side = before; }
void GemmSideBySide::now(int kernels) { side_by_side = kernels < 1 ? 1 : kernels; }
int gemm_set_side_by_side(int kernels) { const int was = side_by_side; side_by_side = kernels < 1 ? 1 : kernels; return was; }

size_t gemm_rowsum_part_bytes(int M, int N) {
  // the most splits of gemm_grad_splits, the narrowest tile (128 columns) and its two wavefront columns
  return (size_t)8 * ((N + 127) / 128) * 2 * (size_t)M * sizeof(float);
}

namespace {
// operands and outputs fit the vector loads, buffer descriptors and vector epilogue of the MFMA kernels
bool fits_mfma(const GemmArgs<bf16>& a) {
  const bool ak = a.a_cs == 1, bk = a.b_cs == 1;
  // 16-byte vector loads: pitches are multiples of 8 elements; a contiguous extent that is not a multiple of 8 is
  // accepted when the pitch covers it rounded up (the caller keeps that padding zero: it is read, never stored).
  auto up8 = [](int64_t v) { return (v + 7) / 8 * 8; };
  const bool ok_a = ak ? (a.a_rs % 8 == 0 && a.a_rs >= up8(a.K)) : (a.a_rs == 1 && a.a_cs % 8 == 0 && a.a_cs >= up8(a.M));
  const bool ok_b = bk ? (a.b_rs % 8 == 0 && a.b_rs >= up8(a.K)) : (a.b_rs == 1 && a.b_cs % 8 == 0 && a.b_cs >= up8(a.N));
  const int64_t ext_a = 2 * (ak ? (int64_t)a.M * a.a_rs : (int64_t)a.K * a.a_cs), ext_b = 2 * (bk ? (int64_t)a.N * a.b_rs : (int64_t)a.K * a.b_cs);
  const bool small = ext_a < (int64_t)0x7fffffff && ext_b < (int64_t)0x7fffffff;   // 32-bit buffer extents and offsets
  const int64_t pitch_c = a.ldc ? a.ldc : a.N;
  // (the epilogue addresses a wavefront's 64 rows of the output through a 32-bit buffer extent)
  const bool ok_c = pitch_c % 8 == 0 && pitch_c >= up8(a.N) && pitch_c * 64 * 4 < (int64_t)0x7fffffff && (a.epi != EPI_GRAD || a.N % 8 == 0) && aligned16(a.C) && aligned16(a.R) && aligned16(a.Z) && aligned16(a.bias) && aligned16(a.G) && aligned16(a.Rf) && aligned16(a.Cf);   // vector epilogue
  return ok_a && ok_b && ok_c && small && aligned16(a.A) && aligned16(a.B);
}
}  // namespace

bool gemm_mfma_takes(const GemmArgs<bf16>& a) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0 || !fits_mfma(a)) return false;
  return a.epi == EPI_GRAD;      // (asked for the weight gradients only: every operand layout of those is instantiated)
}

int launch_gemm_mfma(const GemmArgs<bf16>& a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return fail(CEPHALO_EINVAL, "gemm: empty problem %dx%dx%d", a.M, a.N, a.K);
  const bool ak = a.a_cs == 1, bk = a.b_cs == 1;
  if (!fits_mfma(a)) {
    if (a.rowsum) return fail(CEPHALO_EUNSUPPORTED, "gemm: row sums come with the MFMA kernels only");
    return general(a, s);
  }
  // Only the layout/epilogue pairs a linear layer produces are instantiated.
  if (ak && bk) {          // forward: Y = X W^T
    switch (a.epi) {
      case EPI_NONE: return launch_tiles<true, true, EPI_NONE>(a, s);
      case EPI_NONE_HEAD: return launch_tiles<true, true, EPI_NONE_HEAD>(a, s);
      case EPI_ROPE: if (a.rot_cols % 8 == 0 && a.rot_d % 8 == 0 && aligned16(a.rot)) return launch_tiles<true, true, EPI_ROPE>(a, s); break;
      case EPI_BIAS: return launch_tiles<true, true, EPI_BIAS>(a, s);
      case EPI_BIAS_RESID: return launch_tiles<true, true, EPI_BIAS_RESID>(a, s);
      case EPI_BIAS_GELU: return launch_tiles<true, true, EPI_BIAS_GELU>(a, s);
      case EPI_DGELU: return launch_tiles<true, true, EPI_DGELU>(a, s);
      case EPI_BIAS_GELU_DERIV: return launch_tiles<true, true, EPI_BIAS_GELU_DERIV>(a, s);
      case EPI_MUL: return launch_tiles<true, true, EPI_MUL>(a, s);
      case EPI_DSWIGLU: if (a.N % 8 == 0) return launch_tiles<true, true, EPI_DSWIGLU>(a, s); break;
      case EPI_GRAD: return launch_tiles<true, true, EPI_GRAD>(a, s);
    }
  } else if (ak && !bk) {  // dgrad: dX = dY W
    switch (a.epi) {
      case EPI_NONE: return launch_tiles<true, false, EPI_NONE>(a, s);
      case EPI_DGELU: return launch_tiles<true, false, EPI_DGELU>(a, s);
      default: break;
    }
    if (a.epi == EPI_GRAD) return launch_tiles<true, false, EPI_GRAD>(a, s);   // wgrad with dY pre-transposed
  } else if (!ak && !bk) {  // wgrad: dW = dY^T X
    if (a.epi == EPI_GRAD) return launch_tiles<false, false, EPI_GRAD>(a, s);
  } else {                  // wgrad with X pre-transposed
    if (a.epi == EPI_GRAD) return launch_tiles<false, true, EPI_GRAD>(a, s);
  }
  return general(a, s);
}

}  // namespace cephalo
