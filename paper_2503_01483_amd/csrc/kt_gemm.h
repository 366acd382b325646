// kt_gemm.h -- MFMA GEMM core for gfx950 shared by every contraction on the path.
//
// One device-side main loop computes a BM x BN tile of  C = A * B^T  where both
// operands are stored with the contraction index contiguous ("NT" form):
//   A [M][lda], B [N][ldb], C[m][n] = sum_k A[m][k] * B[n][k].
// The loss/gradient step only ever needs this form: the rotation is kept
// transposed (R^T rows are output features), activations are token-major for the
// forward passes and feature-major (token-minor) copies feed X^T * G.
//
// Tiling: 64-wide wavefronts, each wave owns WTM x WTN of the tile as a grid of
// 32x32 MFMA blocks (v_mfma_f32_32x32x16_bf16, or 4 x v_mfma_f32_32x32x2_f32 per
// 16-byte fragment on the fp32 path).  In the accumulator layout of these
// instructions a lane owns ONE column n (= lane & 31) and 16 rows
// m = 8*(r/4) + 4*(lane>>5) + (r&3), r = 0..15.  Callers put the index they
// reduce over (the hidden dimension of a token row) on m, so row statistics
// accumulate in registers with no cross-lane traffic until one final shuffle.
//
// LDS: each stage holds BM + BN rows of 128 bytes of K; 16-byte chunks are
// XOR-swizzled with the row so both the 16-byte stores and the MFMA fragment reads
// are bank-conflict free.  Two stages, register prefetch of the next K slab.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx4 __attribute__((ext_vector_type(4)));

constexpr int kRowBytes = 128;  // bytes of K per LDS tile row
constexpr int kChunks = 8;      // 16-byte chunks per row

template <typename T>
struct Mma;

template <>
struct Mma<__bf16> {
  static __device__ __forceinline__ void run(const intx4& a, const intx4& b, floatx16& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};

template <>
struct Mma<float> {
  static __device__ __forceinline__ void run(const intx4& a, const intx4& b, floatx16& c) {
    const floatx4 fa = __builtin_bit_cast(floatx4, a);
    const floatx4 fb = __builtin_bit_cast(floatx4, b);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[0], fb[0], c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[1], fb[1], c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[2], fb[2], c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[3], fb[3], c, 0, 0, 0);
  }
};

// Tile shape: BM x BN per workgroup, WGM x WGN waves.
template <typename T_, int BM_, int BN_, int WGM_, int WGN_>
struct Tile {
  using T = T_;
  static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_;
  static constexpr int NT = WGM * WGN * 64;
  static constexpr int WTM = BM / WGM, WTN = BN / WGN;
  static constexpr int MB = WTM / 32, NB = WTN / 32;
  static constexpr int BK = kRowBytes / (int)sizeof(T);  // elements of K per slab
  static constexpr int A_BYTES = BM * kRowBytes, B_BYTES = BN * kRowBytes;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
  static constexpr int A_LD = BM * kChunks / NT;  // 16-byte loads per thread per slab
  static constexpr int B_LD = BN * kChunks / NT;
  static_assert(BM % (32 * WGM) == 0 && BN % (32 * WGN) == 0, "wave tile must be 32-blocked");
  static_assert((BM * kChunks) % NT == 0 && (BN * kChunks) % NT == 0, "loads must divide evenly");
  static_assert(NT % kChunks == 0, "thread count must be a multiple of 8");
};

__device__ __forceinline__ int lds_off(int row, int chunk) {
  return row * kRowBytes + (((chunk ^ row) & (kChunks - 1)) << 4);
}

// Geometry of one accumulator element, shared by every epilogue.
template <class TL>
struct Frag {
  int lane, half, wm, wn;
  __device__ __forceinline__ Frag() {
    const int wave = threadIdx.x >> 6;
    lane = threadIdx.x & 63;
    half = lane >> 5;
    wm = wave / TL::WGN;
    wn = wave % TL::WGN;
  }
  // row offset inside the workgroup tile of accumulator register r in block mb
  __device__ __forceinline__ int m_of(int mb, int r) const {
    return wm * TL::WTM + mb * 32 + ((r >> 2) << 3) + (half << 2) + (r & 3);
  }
  __device__ __forceinline__ int m_block(int mb) const { return wm * TL::WTM + mb * 32; }
  __device__ __forceinline__ int n_of(int nb) const { return wn * TL::WTN + nb * 32 + (lane & 31); }
};

// Main loop.  Rows of A beyond M (and of B beyond N) are read from the last valid
// row, so every load stays inside the operand; the epilogue masks them out.
// The K range [k0, k0 + k_slabs*BK) must lie inside both operands' rows.
template <class TL>
__device__ __forceinline__ void gemm_mainloop(const typename TL::T* __restrict__ A, int64_t lda,
                                              int M, int m0,
                                              const typename TL::T* __restrict__ B, int64_t ldb,
                                              int N, int n0, int64_t k0, int k_slabs,
                                              floatx16 (&acc)[TL::MB][TL::NB], char* lds) {
  using T = typename TL::T;
  constexpr int EPC = 16 / (int)sizeof(T);  // elements per 16-byte chunk
  const int tid = threadIdx.x;
  const int lrow = tid >> 3;  // row handled by this thread in load pass 0
  const int lchunk = tid & 7;
  constexpr int ROWS_PER_PASS = TL::NT / kChunks;

  const T* ga[TL::A_LD];
  const T* gb[TL::B_LD];
  int sa[TL::A_LD], sb[TL::B_LD];
#pragma unroll
  for (int i = 0; i < TL::A_LD; ++i) {
    const int row = lrow + i * ROWS_PER_PASS;
    int grow = m0 + row;
    grow = grow < M ? grow : M - 1;
    ga[i] = A + (int64_t)grow * lda + k0 + lchunk * EPC;
    sa[i] = lds_off(row, lchunk);
  }
#pragma unroll
  for (int i = 0; i < TL::B_LD; ++i) {
    const int row = lrow + i * ROWS_PER_PASS;
    int grow = n0 + row;
    grow = grow < N ? grow : N - 1;
    gb[i] = B + (int64_t)grow * ldb + k0 + lchunk * EPC;
    sb[i] = TL::A_BYTES + lds_off(row, lchunk);
  }

  const Frag<TL> f;
  // fragment read offsets for K sub-step 0; sub-step s flips chunk bits by (2s)
  int fa[TL::MB], fb[TL::NB];
#pragma unroll
  for (int mb = 0; mb < TL::MB; ++mb) fa[mb] = (f.m_block(mb) + (f.lane & 31)) * kRowBytes;
#pragma unroll
  for (int nb = 0; nb < TL::NB; ++nb)
    fb[nb] = TL::A_BYTES + (f.wn * TL::WTN + nb * 32 + (f.lane & 31)) * kRowBytes;
  const int swz = f.lane & 7;  // row & 7 for every fragment row of this lane

  intx4 ra[TL::A_LD], rb[TL::B_LD];
  auto load_global = [&](int slab) {
    const int64_t ko = (int64_t)slab * TL::BK;
#pragma unroll
    for (int i = 0; i < TL::A_LD; ++i) ra[i] = *reinterpret_cast<const intx4*>(ga[i] + ko);
#pragma unroll
    for (int i = 0; i < TL::B_LD; ++i) rb[i] = *reinterpret_cast<const intx4*>(gb[i] + ko);
  };
  auto store_lds = [&](int stage) {
    char* base = lds + stage * TL::STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < TL::A_LD; ++i) *reinterpret_cast<intx4*>(base + sa[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < TL::B_LD; ++i) *reinterpret_cast<intx4*>(base + sb[i]) = rb[i];
  };
  auto compute = [&](int stage) {
    const char* base = lds + stage * TL::STAGE_BYTES;
#pragma unroll
    for (int s = 0; s < kChunks / 2; ++s) {
      const int coff = (((2 * s + f.half) ^ swz) & (kChunks - 1)) << 4;
      intx4 av[TL::MB], bv[TL::NB];
#pragma unroll
      for (int mb = 0; mb < TL::MB; ++mb) av[mb] = *reinterpret_cast<const intx4*>(base + fa[mb] + coff);
#pragma unroll
      for (int nb = 0; nb < TL::NB; ++nb) bv[nb] = *reinterpret_cast<const intx4*>(base + fb[nb] + coff);
#pragma unroll
      for (int mb = 0; mb < TL::MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < TL::NB; ++nb) Mma<T>::run(av[mb], bv[nb], acc[mb][nb]);
    }
  };

  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int slab = 0; slab < k_slabs; ++slab) {
    const int cur = slab & 1;
    const bool more = slab + 1 < k_slabs;
    if (more) load_global(slab + 1);
    compute(cur);
    if (more) store_lds(cur ^ 1);
    __syncthreads();
  }
}

// Launch description of one batched NT GEMM.
struct GemmShape {
  const void* A;
  const void* B;
  int64_t lda, ldb;
  int64_t batch_stride_a, batch_stride_b;  // elements
  int M, N;
  int tiles_m, tiles_n;
  int split_k;       // number of K splits (>= 1)
  int slabs_total;   // K / BK
  int slabs_per_split;
  int tiles_total;   // tiles_m * tiles_n * split_k
  int grid_padded;   // tiles_total rounded up to a multiple of 8
};

// Workgroup -> tile.  Consecutive workgroup ids land on different XCDs (8 of them,
// each with its own L2), so ids are first regrouped so that each XCD walks a
// contiguous range of tiles, then the range is walked in bands of 4 tile-rows so
// that the ~32 tiles an XCD holds at once share few A and B slabs.
__device__ __forceinline__ bool tile_of_block(const GemmShape& g, int& tm, int& tn, int& ks) {
  const int id = blockIdx.x;
  const int per_xcd = g.grid_padded >> 3;
  int L = (id & 7) * per_xcd + (id >> 3);
  if (L >= g.tiles_total) return false;
  const int per_split = g.tiles_m * g.tiles_n;
  ks = L / per_split;
  L -= ks * per_split;
  constexpr int BAND = 4;
  const int band_tiles = BAND * g.tiles_n;
  const int band = L / band_tiles;
  const int first_m = band * BAND;
  const int rows = (g.tiles_m - first_m) < BAND ? (g.tiles_m - first_m) : BAND;
  const int in_band = L - band * band_tiles;
  tm = first_m + in_band % rows;
  tn = in_band / rows;
  return true;
}

template <class TL, class Epi>
__global__ __launch_bounds__(TL::NT) void gemm_nt_kernel(GemmShape g, Epi epi) {
  extern __shared__ __align__(16) char lds[];
  using T = typename TL::T;
  const int batch = blockIdx.y;
  int tm, tn, ks;
  if (!tile_of_block(g, tm, tn, ks)) return;
  if (epi.skip(batch)) return;
  const int m0 = tm * TL::BM, n0 = tn * TL::BN;
  const int slab0 = ks * g.slabs_per_split;
  int slabs = g.slabs_total - slab0;
  slabs = slabs < g.slabs_per_split ? slabs : g.slabs_per_split;

  floatx16 acc[TL::MB][TL::NB];
#pragma unroll
  for (int mb = 0; mb < TL::MB; ++mb)
#pragma unroll
    for (int nb = 0; nb < TL::NB; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.0f;

  const T* A = static_cast<const T*>(g.A) + (int64_t)batch * g.batch_stride_a;
  const T* B = static_cast<const T*>(g.B) + (int64_t)batch * g.batch_stride_b;
  gemm_mainloop<TL>(A, g.lda, g.M, m0, B, g.ldb, g.N, n0, (int64_t)slab0 * TL::BK, slabs, acc, lds);
  epi(acc, batch, tm, tn, ks, m0, n0);
}

}  // namespace kt
