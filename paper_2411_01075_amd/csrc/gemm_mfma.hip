// bf16 GEMM on the gfx950 matrix cores:  C[M,N] = sum_k A(m,k) B(n,k), fp32 accumulate, fused epilogue.
//
// One kernel template covers the three contractions of a linear layer without any transposed
// copy in HBM:
//   forward   Y  = X W^T      A k-contiguous, B k-contiguous
//   dgrad     dX = dY W       A k-contiguous, B n-contiguous (k strided)
//   wgrad     dW = dY^T X     A m-contiguous, B n-contiguous (both strided along k = tokens)
// A k-contiguous operand is staged in LDS as [row][k] and its MFMA fragment (8 consecutive k of
// one row per lane) is one 16-byte LDS read.  A row-contiguous operand is staged as [k][row] and
// its fragment is fetched with the transposing LDS read of gfx950 (ds_read_b64_tr_b16): within
// each 16-lane group, lane i supplies the address of 4 consecutive rows at k-row (i/4) and
// receives the 4 k-values of row i -- exactly the MFMA operand layout.
//
// Tiling: 256 threads = 4 wavefronts in a 2x2 grid; v_mfma_f32_32x32x16_bf16; k-slab 64;
// global->register->LDS double buffering (next slab's global loads are in flight during the
// current slab's MFMAs; one barrier per slab).
#include "kernels.h"

namespace cephalo {
namespace {

typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
#define LDS_AS __attribute__((address_space(3)))
typedef LDS_AS bf16 lds_bf16;

constexpr int kThreads = 256;
constexpr int BK = 64;    // k-slab
constexpr unsigned kOob = 0x80000000u;   // byte offset beyond any buffer: such a buffer load returns zero

// Buffer descriptor over `bytes` bytes at p: loads at offsets >= bytes return 0 (hardware range check).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}

// One operand's tile: ROWS matrix rows (m or n) by BK k-values.
//   KFAST  : LDS [row][k], row pitch BK+8 elements; the 16 lanes of a 16-byte read phase fall in 16 different
//            16-byte bank groups (pitch 144 B = 9 * 16 B).
//   !KFAST : LDS [k][row], row pitch ROWS+32 elements; the four k-rows a transposing read touches are 64 B apart
//            modulo 256 B, so a 16-lane group covers the banks once.
template <int ROWS, bool KFAST>
struct OperandTile {
  static constexpr int LD = KFAST ? (BK + 8) : (ROWS + 32);      // LDS row pitch, elements
  static constexpr int ELEMS = KFAST ? ROWS * LD : BK * LD;
  static constexpr int VECS = ROWS * BK / 8;                     // 16-byte vectors per tile
  static constexpr int PER_THREAD = VECS / kThreads;
  static_assert(VECS % kThreads == 0, "tile must split evenly over the threads");

  __device__ static void vec_coords(int p, int& row, int& k) {
    const int v = threadIdx.x + kThreads * p;
    if (KFAST) { row = v / (BK / 8); k = (v % (BK / 8)) * 8; }
    else       { k = v / (ROWS / 8); row = (v % (ROWS / 8)) * 8; }
  }
  // byte offsets of this thread's vectors for k-slab 0; rows outside the matrix get the out-of-range mark
  __device__ static void init_offsets(int64_t rs, int64_t cs, int row0, int nrows, unsigned (&off)[PER_THREAD]) {
#pragma unroll
    for (int p = 0; p < PER_THREAD; ++p) {
      int row, k;
      vec_coords(p, row, k);
      const int64_t e = (int64_t)(row0 + row) * rs + (int64_t)k * cs;
      off[p] = (row0 + row < nrows) ? (unsigned)(e * 2) : kOob;
    }
  }
  // global -> registers for the slab starting at k0 (off[] already points at that slab)
  __device__ static void load_global(__amdgpu_buffer_rsrc_t rsrc, const unsigned (&off)[PER_THREAD], int k0, int K,
                                     u32x4 (&reg)[PER_THREAD]) {
#pragma unroll
    for (int p = 0; p < PER_THREAD; ++p) {
      int row, k;
      vec_coords(p, row, k);
      const unsigned o = (k0 + k < K) ? off[p] : kOob;
      reg[p] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, o, 0, 0);
    }
  }
  __device__ static void advance(unsigned (&off)[PER_THREAD], unsigned slab_bytes) {
#pragma unroll
    for (int p = 0; p < PER_THREAD; ++p) off[p] += slab_bytes;    // the mark stays out of range (no wrap below 2^31 steps)
  }
  __device__ static void store_lds(lds_bf16* lds, const u32x4 (&reg)[PER_THREAD]) {
#pragma unroll
    for (int p = 0; p < PER_THREAD; ++p) {
      int row, k;
      vec_coords(p, row, k);
      lds_bf16* dst = KFAST ? (lds + row * LD + k) : (lds + k * LD + row);
      *reinterpret_cast<LDS_AS u32x4*>(dst) = reg[p];
    }
  }
  // MFMA 32x32x16 operand fragment: rows [rb, rb+32), k-values [kk, kk+16) of the tile
  __device__ static bf16x8 fragment(const lds_bf16* lds, int rb, int kk) {
    const int lane = threadIdx.x & 63;
    if (KFAST) {
      return *reinterpret_cast<const LDS_AS bf16x8*>(lds + (rb + (lane & 31)) * LD + kk + (lane >> 5) * 8);
    } else {
      const int g = lane >> 4, i = lane & 15;
      const int r = rb + 16 * (g & 1) + 4 * (i & 3);
      const int k = kk + 8 * (g >> 1) + (i >> 2);
      const lds_bf16* p0 = lds + k * LD + r;
      s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(p0));
      s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(p0 + 4 * LD));
      union { struct { s16x4 a, b; } s; bf16x8 v; } u;
      u.s.a = lo; u.s.b = hi;
      return u.v;
    }
  }
};

template <int BM, int BN, bool AK, bool BKF, int EPI>
__global__ void __launch_bounds__(kThreads) gemm_mfma_kernel(GemmArgs<bf16> a, int tiles_n, int tiles_total) {
  typedef OperandTile<BM, AK> TA;
  typedef OperandTile<BN, BKF> TB;
  constexpr int WTM = BM / 2, WTN = BN / 2;     // wavefront tile (2x2 wavefronts)
  constexpr int MI = WTM / 32, NI = WTN / 32;
  constexpr int STAGE = TA::ELEMS + TB::ELEMS;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  lds_bf16* smem = (lds_bf16*)smem_raw;

  // Blocks are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of tiles so
  // that neighbours in the tile order (which share operand panels) share an L2.
  int pid = blockIdx.x;
  if (tiles_total % 8 == 0) pid = (pid % 8) * (tiles_total / 8) + pid / 8;
  const int tile_m = pid / tiles_n, tile_n = pid % tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = (wave >> 1) * WTM, wn = (wave & 1) * WTN;

  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // operand extents in bytes (dense matrices: the strided pitch times the number of strided steps)
  const unsigned a_bytes = (unsigned)(2 * (AK ? (int64_t)a.M * a.a_rs : (int64_t)a.K * a.a_cs));
  const unsigned b_bytes = (unsigned)(2 * (BKF ? (int64_t)a.N * a.b_rs : (int64_t)a.K * a.b_cs));
  const __amdgpu_buffer_rsrc_t ra_rsrc = make_rsrc(a.A, a_bytes), rb_rsrc = make_rsrc(a.B, b_bytes);
  unsigned offa[TA::PER_THREAD], offb[TB::PER_THREAD];
  TA::init_offsets(a.a_rs, a.a_cs, m0, a.M, offa);
  TB::init_offsets(a.b_rs, a.b_cs, n0, a.N, offb);
  const unsigned a_step = (unsigned)(2 * BK * a.a_cs), b_step = (unsigned)(2 * BK * a.b_cs);

  u32x4 ra[TA::PER_THREAD], rb[TB::PER_THREAD];
  TA::load_global(ra_rsrc, offa, 0, a.K, ra);
  TB::load_global(rb_rsrc, offb, 0, a.K, rb);
  TA::store_lds(smem, ra);
  TB::store_lds(smem + TA::ELEMS, rb);
  __syncthreads();

  const int nk = (a.K + BK - 1) / BK;
  for (int kt = 0; kt < nk; ++kt) {
    const lds_bf16* As = smem + (kt & 1) * STAGE;
    const lds_bf16* Bs = As + TA::ELEMS;
    if (kt + 1 < nk) {
      TA::advance(offa, a_step);
      TB::advance(offb, b_step);
      TA::load_global(ra_rsrc, offa, (kt + 1) * BK, a.K, ra);
      TB::load_global(rb_rsrc, offb, (kt + 1) * BK, a.K, rb);
    }
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      bf16x8 fa[MI], fb[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i) fa[i] = TA::fragment(As, wm + 32 * i, kk);
#pragma unroll
      for (int j = 0; j < NI; ++j) fb[j] = TB::fragment(Bs, wn + 32 * j, kk);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      lds_bf16* An = smem + ((kt + 1) & 1) * STAGE;
      TA::store_lds(An, ra);
      TB::store_lds(An + TA::ELEMS, rb);
    }
    __syncthreads();
  }

  // Epilogue.  Accumulator element e of a 32x32 tile: row 8*(e/4) + 4*(lane/32) + e%4, column lane%32.
#pragma unroll
  for (int i = 0; i < MI; ++i) {
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int n = n0 + wn + 32 * j + (lane & 31);
      if (n >= a.N) continue;
      float bias = 0.f;
      if (EPI == EPI_BIAS || EPI == EPI_BIAS_RESID || EPI == EPI_BIAS_GELU) bias = (float)a.bias[n];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wm + 32 * i + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        if (m >= a.M) continue;
        const int64_t o = (int64_t)m * a.N + n;
        const float v = acc[i][j][e];
        if (EPI == EPI_NONE) a.C[o] = (bf16)v;
        if (EPI == EPI_BIAS) a.C[o] = (bf16)(v + bias);
        if (EPI == EPI_BIAS_RESID) a.C[o] = (bf16)(v + bias + (float)a.R[o]);
        if (EPI == EPI_BIAS_GELU) {
          const float z = v + bias;
          a.Z[o] = (bf16)z;
          a.C[o] = (bf16)gelu_f(z);
        }
        if (EPI == EPI_DGELU) a.C[o] = (bf16)(v * gelu_grad_f((float)a.Z[o]));
        if (EPI == EPI_GRAD) a.G[o] = (a.accumulate ? a.G[o] : 0.f) + a.scale * v;
      }
    }
  }
}

template <int BM, int BN, bool AK, bool BKF, int EPI>
int launch_cfg(const GemmArgs<bf16>& a, hipStream_t s) {
  typedef OperandTile<BM, AK> TA;
  typedef OperandTile<BN, BKF> TB;
  const size_t lds = 2 * (size_t)(TA::ELEMS + TB::ELEMS) * sizeof(bf16);
  const int tm = (a.M + BM - 1) / BM, tn = (a.N + BN - 1) / BN;
  auto kern = gemm_mfma_kernel<BM, BN, AK, BKF, EPI>;
  static bool attr_set = false;   // per instantiation
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return fail(CEPHALO_EHIP, "gemm_mfma: cannot reserve %zu B of LDS", lds);
    attr_set = true;
  }
  kern<<<tm * tn, kThreads, lds, s>>>(a, tn, tm * tn);
  CEPHALO_CHECK_LAUNCH("gemm_mfma");
  return CEPHALO_OK;
}

template <bool AK, bool BKF, int EPI>
int launch_tiles(const GemmArgs<bf16>& a, hipStream_t s) {
  // Largest tile that still yields about one block per compute unit.
  const int64_t t256 = (int64_t)((a.M + 255) / 256) * ((a.N + 127) / 128);
  if (t256 >= 200) return launch_cfg<256, 128, AK, BKF, EPI>(a, s);
  const int64_t t128 = (int64_t)((a.M + 127) / 128) * ((a.N + 127) / 128);
  if (t128 >= 200) return launch_cfg<128, 128, AK, BKF, EPI>(a, s);
  return launch_cfg<128, 64, AK, BKF, EPI>(a, s);
}

}  // namespace

int launch_gemm_mfma(const GemmArgs<bf16>& a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return fail(CEPHALO_EINVAL, "gemm: empty problem %dx%dx%d", a.M, a.N, a.K);
  const bool ak = a.a_cs == 1, bk = a.b_cs == 1;
  // 16-byte vector loads need the contiguous extent and the strided pitch to be multiples of 8 elements.
  const bool ok_a = ak ? (a.K % 8 == 0 && a.a_rs % 8 == 0) : (a.a_rs == 1 && a.M % 8 == 0 && a.a_cs % 8 == 0);
  const bool ok_b = bk ? (a.K % 8 == 0 && a.b_rs % 8 == 0) : (a.b_rs == 1 && a.N % 8 == 0 && a.b_cs % 8 == 0);
  const int64_t ext_a = 2 * (ak ? (int64_t)a.M * a.a_rs : (int64_t)a.K * a.a_cs), ext_b = 2 * (bk ? (int64_t)a.N * a.b_rs : (int64_t)a.K * a.b_cs);
  const bool small = ext_a < (int64_t)0x7fffffff && ext_b < (int64_t)0x7fffffff;   // 32-bit buffer extents and offsets
  if (!ok_a || !ok_b || !small || !aligned16(a.A) || !aligned16(a.B)) return launch_gemm_simple<bf16>(a, s);
  // Only the layout/epilogue pairs a linear layer produces are instantiated.
  if (ak && bk) {          // forward: Y = X W^T
    switch (a.epi) {
      case EPI_NONE: return launch_tiles<true, true, EPI_NONE>(a, s);
      case EPI_BIAS: return launch_tiles<true, true, EPI_BIAS>(a, s);
      case EPI_BIAS_RESID: return launch_tiles<true, true, EPI_BIAS_RESID>(a, s);
      case EPI_BIAS_GELU: return launch_tiles<true, true, EPI_BIAS_GELU>(a, s);
    }
  } else if (ak && !bk) {  // dgrad: dX = dY W
    switch (a.epi) {
      case EPI_NONE: return launch_tiles<true, false, EPI_NONE>(a, s);
      case EPI_DGELU: return launch_tiles<true, false, EPI_DGELU>(a, s);
    }
  } else if (!ak && !bk) {  // wgrad: dW = dY^T X
    if (a.epi == EPI_GRAD) return launch_tiles<false, false, EPI_GRAD>(a, s);
  }
  return launch_gemm_simple<bf16>(a, s);
}

}  // namespace cephalo
