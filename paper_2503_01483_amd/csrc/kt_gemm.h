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
// XOR-swizzled with the row pair so both the 16-byte stores and the MFMA fragment
// reads are bank-conflict free.  Two stages, register prefetch of the next K slab.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace kt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx4 __attribute__((ext_vector_type(4)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

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

// LDS has 64 banks of 4 bytes: two 128-byte tile rows share one bank window, and a
// 16-byte access is served 16 lanes at a time.  XOR-ing the chunk index with (row >> 1)
// makes 16 consecutive rows at the same logical chunk hit 16 distinct 16-byte slots of
// the 256-byte window (measured: 194 B/clk/CU, against 122 with a plain row & 7 key).
__device__ __forceinline__ int swizzle_key(int row) { return (row >> 1) & (kChunks - 1); }
__device__ __forceinline__ int lds_off(int row, int chunk) {
  return row * kRowBytes + ((chunk ^ swizzle_key(row)) << 4);
}

// Two transposing 8-byte LDS reads (ds_read_b64_tr_b16) -> one MFMA operand: 8 values along K for
// this lane's row, taken from a tile that is stored with K as the ROW index.  In a group of 16
// lanes, lane r supplies the address of 4 consecutive columns of tile row k0 + r/4 starting at
// column c0 + 4*(r%4); lane L of the group receives column c0 + L of rows k0..k0+3.
// `addr_lo` / `addr_hi` are this lane's addresses for rows +0..3 / +4..7.
typedef short shortx4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ intx4 read_tr_operand(const char* lds, int addr_lo, int addr_hi) {
  typedef __attribute__((address_space(3))) shortx4* lds_ptr;
  const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(lds + addr_lo));
  const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(lds + addr_hi));
  typedef short shortx8 __attribute__((ext_vector_type(8)));
  const shortx8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(intx4, v);
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

template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
  (f(std::integral_constant<int, Is>{}), ...);
}
// Calls f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), fully unrolled.
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Wait for this wave's outstanding LDS operations only (vmcnt and expcnt left at their
// maxima), then meet the other waves.  A full __syncthreads() would also drain the
// global loads that are deliberately kept in flight across the barrier.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
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
  int slabs_per_block;             // K blocking of the operand rows (see gemm_mainloop)
  int64_t block_bytes_a, block_bytes_b;
  int k_valid;                     // ATN: rows of A that exist (K may be padded beyond them)
#ifdef KT_PHASE_STAMPS
  int stamp_slot;                  // developer build only: which launch record the stamps go to
#endif
};

#ifdef KT_PHASE_STAMPS
// Developer build (-DKT_PHASE_STAMPS, never the shipped library): wave 0 of every workgroup records the
// shader-clock counter at kernel entry, after the prologue, after the main loop and after the epilogue,
// plus the constant-rate (100 MHz) counter at entry and exit and the hardware id of its CU, so that a
// launch can be broken down into phases and the clock the chip actually held can be read off.
constexpr int kStampSlots = 8, kStampWgs = 16384, kStampWords = 8;
__device__ unsigned long long g_phase_stamps[kStampSlots * kStampWgs * kStampWords];
__device__ __forceinline__ void phase_stamp(const GemmShape& g, int word, bool wall = false) {
  if (threadIdx.x != 0 || g.stamp_slot < 0) return;
  const size_t wg = (size_t)blockIdx.y * gridDim.x + blockIdx.x;
  if (wg >= (size_t)kStampWgs) return;
  unsigned long long* rec = g_phase_stamps + ((size_t)g.stamp_slot * kStampWgs + wg) * kStampWords;
  rec[word] = wall ? __builtin_amdgcn_s_memrealtime() : __builtin_readcyclecounter();
}
#define KT_STAMP(g, word) phase_stamp(g, word)
#define KT_STAMP_WALL(g, word) phase_stamp(g, word, true)
#define KT_STAMP_PARAM , const GemmShape* stamp_g = nullptr
#define KT_STAMP_ARG , &g
#define KT_STAMP_LOOP_START() do { if (stamp_g) phase_stamp(*stamp_g, 1); } while (0)
#else
#define KT_STAMP(g, word)
#define KT_STAMP_WALL(g, word)
#define KT_STAMP_PARAM
#define KT_STAMP_ARG
#define KT_STAMP_LOOP_START()
#endif

// Main loop.  Rows of A beyond M (and of B beyond N) are read from the last valid
// row, so every load stays inside the operand; the epilogue masks them out.
// K is addressed in slabs: slab g of an operand row starts at byte
//   (g / slabs_per_block) * block_bytes + (g % slabs_per_block) * 128
// of the row, which is the plain g * 128 for an ordinary row-major operand
// (slabs_per_block = number of slabs in a row) and lets the token-minor operands of
// dR = X^T G be stored in blocks of a few thousand tokens, so that the 256 rows a tile
// reads at any one time lie within a couple of MiB instead of 256 separate pages.
// The slab range [slab0, slab0 + k_slabs) must lie inside both operands' rows, and
// (BM-1)*lda*sizeof(T) + 128 (same for B) must fit 32 bits (the host checks this).
//
// Schedule.  One K slab = 4 sub-steps of MB*NB MFMA "slots".  Everything that is not
// an MFMA is dealt out over the slots, one or two instructions behind each MFMA, and
// pinned there with sched_barrier, so the matrix pipe never waits for a block of
// memory instructions to issue:
//   sub-steps 0-2: behind the first slots, read the fragments of the next sub-step;
//                  spread over all their slots, write the NEXT slab (registers -> other
//                  LDS stage) one 16-byte chunk at a time, and refill each freed
//                  register with the same chunk of slab+2 from global memory
//   sub-step 3:    barrier (LDS only), then read sub-step 0 of the next slab
// The fragments of sub-step s+1 are therefore on their way a whole sub-step before
// the MFMAs that use them, each global load a whole slab before its LDS store, and
// neither the LDS nor the vector-memory path ever sees a burst (a burst of 16 stores
// per wave made the matrix pipe wait ~1000 cycles per slab).
//
// ATN (bf16, BM = 256): operand A is given with K as its ROW index instead, A[k][lda] with the tile's
// 256 rows m as consecutive columns (the activations X [token][feature] for dR = X^T G: no
// token-minor copy of X is needed).  K is walked in the order the other operand stores it
// (token_position() of the epilogues: position 4a + b of a 128-token group is token a + 32 b).
// A slab is then 64 tile rows of 512 bytes, padded to 576 so that the four consecutive rows a
// transposing read touches lie 64 bytes apart in the bank window; fragments come from
// read_tr_operand.  Rows k >= k_valid are not read (the last valid row is read instead; the other
// operand is zero there).
constexpr int kAtnRowBytes = 576;
constexpr int kAtnStageBytes = 64 * kAtnRowBytes;

template <class TL, bool ATN = false>
__device__ __forceinline__ void gemm_mainloop(const typename TL::T* __restrict__ A, int64_t lda,
                                              int M, int m0,
                                              const typename TL::T* __restrict__ B, int64_t ldb,
                                              int N, int n0, int slab0, int k_slabs,
                                              int slabs_per_block, int64_t block_bytes_a,
                                              int64_t block_bytes_b,
                                              floatx16 (&acc)[TL::MB][TL::NB], char* lds, int k_valid = 0
                                              KT_STAMP_PARAM) {
  using T = typename TL::T;
  static_assert(!ATN || (sizeof(T) == 2 && TL::BM == 256 && TL::NT == 256), "ATN: bf16, 256 tile rows, 4 waves");
  constexpr int A_STAGE = ATN ? kAtnStageBytes : TL::A_BYTES;
  constexpr int EPC = 16 / (int)sizeof(T);  // elements per 16-byte chunk
  constexpr int MB = TL::MB, NB = TL::NB, NMMA = MB * NB, NFRAG = MB + NB;
  constexpr int A_LD = TL::A_LD, B_LD = TL::B_LD, NLD = A_LD + B_LD;
  constexpr int ROWS_PER_PASS = TL::NT / kChunks;
  // LDS layout: [A stage 0][A stage 1][B stage 0][B stage 1]; every stage offset and
  // every per-block row offset below is a compile-time immediate of the ds_ instruction.
  constexpr int B_BASE = 2 * A_STAGE;
  static_assert(kChunks / 2 == 4, "the schedule is written for 4 K sub-steps per slab");
  static_assert(ROWS_PER_PASS % 16 == 0, "swizzle key must not change between load passes");
  static_assert(NFRAG <= NMMA && NLD <= 3 * NMMA, "not enough MFMA slots to hide the memory instructions");

  const int tid = threadIdx.x;
  const int lrow = tid >> 3;  // row handled by this thread in load pass 0
  const int lchunk = tid & 7;

  // global addressing: uniform 64-bit base (advanced per slab) + 32-bit byte offsets
  const char* Ab = reinterpret_cast<const char*>(ATN ? A + m0 : A + (int64_t)m0 * lda);
  const char* Bb = reinterpret_cast<const char*>(B + (int64_t)n0 * ldb);
  // byte offsets of K slab `slab` (relative to slab0) inside a row of A / of B: uniform values
  int64_t ka = 0, kb = 0;
  uint32_t og[NLD];
  // ATN: thread (chunk tid & 31 of the 512-byte row, row group tid >> 5) moves tile rows
  // (tid >> 5) + 8 i of a slab; tile row pr of slab g holds position 64 (g & 1) + pr of 128-token
  // group g >> 1, i.e. token (pr >> 2) + 16 (g & 1) + 32 (pr & 3) of the group.
  const int atn_chunk = tid & 31, atn_rg = tid >> 5;
  auto atn_token = [&](int i) __attribute__((always_inline)) {
    const int pr = atn_rg + 8 * i;
    return (pr >> 2) + 32 * (pr & 3);
  };
  auto locate = [&](int slab) __attribute__((always_inline)) {
    const int g = slab0 + slab;
    const int blk = g / slabs_per_block;
    const int64_t in_blk = (int64_t)(g - blk * slabs_per_block) * kRowBytes;
    kb = blk * block_bytes_b + in_blk;
    if constexpr (ATN) {
      const int grp0 = (g >> 1) * 128, half16 = (g & 1) * 16;  // tile row 0 of this slab is token grp0 + half16
      ka = (int64_t)(grp0 + half16) * lda * (int64_t)sizeof(T);
      if (grp0 + 128 > k_valid) {  // last, partial group: rows past the end read the last valid token
        ka = (int64_t)grp0 * lda * (int64_t)sizeof(T);
        const int last = k_valid - 1 - grp0;  // >= 0: the group starts inside the operand
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
          const int t = half16 + atn_token(i);
          og[i] = (uint32_t)(((int64_t)(t < last ? t : last) * lda + atn_chunk * EPC) * (int64_t)sizeof(T));
        }
      }
    } else {
      ka = blk * block_bytes_a + in_blk;
    }
  };
#pragma unroll
  for (int i = 0; i < A_LD; ++i) {
    if constexpr (ATN) {
      og[i] = (uint32_t)(((int64_t)atn_token(i) * lda + atn_chunk * EPC) * (int64_t)sizeof(T));
    } else {
      int row = lrow + i * ROWS_PER_PASS;
      row = (m0 + row < M) ? row : (M - 1 - m0);
      og[i] = (uint32_t)(((int64_t)row * lda + lchunk * EPC) * (int64_t)sizeof(T));
    }
  }
#pragma unroll
  for (int i = 0; i < B_LD; ++i) {
    int row = lrow + i * ROWS_PER_PASS;
    row = (n0 + row < N) ? row : (N - 1 - n0);
    og[A_LD + i] = (uint32_t)(((int64_t)row * ldb + lchunk * EPC) * (int64_t)sizeof(T));
  }
  const int st_off = lds_off(lrow, lchunk);  // + i*ROWS_PER_PASS*128 per pass (same key)
  const int st_off_atn = atn_rg * kAtnRowBytes + atn_chunk * 16;  // + i * 8 rows per load

  const Frag<TL> f;
  // fragment addresses: one per K sub-step and operand; blocks and stages are immediates
  const int key = swizzle_key(f.lane & 31);
  int fa_s[4], fb_s[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int coff = (((2 * s + f.half) ^ key) & (kChunks - 1)) << 4;
    fa_s[s] = (f.wm * TL::WTM + (f.lane & 31)) * kRowBytes + coff;
    fb_s[s] = B_BASE + (f.wn * TL::WTN + (f.lane & 31)) * kRowBytes + coff;
  }
  // ATN fragments: tile rows 16 s + tr_row (+4), columns (features) wm * WTM + 32 block + tr_col ..
  const int atn_g16 = f.lane >> 4, atn_rr = f.lane & 15;
  const int atn_tr = (8 * (atn_g16 >> 1) + (atn_rr >> 2)) * kAtnRowBytes +
                     (f.wm * TL::WTM + 16 * (atn_g16 & 1) + 4 * (atn_rr & 3)) * 2;

  intx4 rg[NLD];        // one K slab in flight from global memory
  intx4 fr[2][NFRAG];   // MFMA fragments, double buffered: [buf][0..MB) = A, [MB..) = B

  // loads chunk i of the slab last passed to locate()
  auto gload = [&](auto i_c) __attribute__((always_inline)) {
    constexpr int i = decltype(i_c)::value;
    const char* base = i < A_LD ? Ab + ka : Bb + kb;
    rg[i] = *reinterpret_cast<const intx4*>(base + og[i]);
  };
  auto lstore = [&](auto i_c, auto stage_c) __attribute__((always_inline)) {
    constexpr int i = decltype(i_c)::value;
    constexpr int stage = decltype(stage_c)::value;
    if constexpr (ATN && i < A_LD) {
      *reinterpret_cast<intx4*>(lds + st_off_atn + stage * A_STAGE + i * 8 * kAtnRowBytes) = rg[i];
    } else {
      constexpr int off = i < A_LD ? stage * A_STAGE + i * ROWS_PER_PASS * kRowBytes
                                   : B_BASE + stage * TL::B_BYTES + (i - A_LD) * ROWS_PER_PASS * kRowBytes;
      *reinterpret_cast<intx4*>(lds + st_off + off) = rg[i];
    }
  };
  auto fread = [&](auto buf_c, auto i_c, auto stage_c, auto s_c) __attribute__((always_inline)) {
    constexpr int buf = decltype(buf_c)::value, i = decltype(i_c)::value;
    constexpr int stage = decltype(stage_c)::value, s = decltype(s_c)::value;
    if constexpr (ATN && i < MB) {
      constexpr int off = stage * A_STAGE + s * 16 * kAtnRowBytes + i * 64;
      fr[buf][i] = read_tr_operand(lds, atn_tr + off, atn_tr + off + 4 * kAtnRowBytes);
    } else if constexpr (i < MB)
      fr[buf][i] = *reinterpret_cast<const intx4*>(lds + fa_s[s] + stage * A_STAGE + i * 32 * kRowBytes);
    else
      fr[buf][i] = *reinterpret_cast<const intx4*>(lds + fb_s[s] + stage * TL::B_BYTES + (i - MB) * 32 * kRowBytes);
  };
  auto mma = [&](auto buf_c, auto j_c) __attribute__((always_inline)) {
    constexpr int buf = decltype(buf_c)::value, j = decltype(j_c)::value;
    Mma<T>::run(fr[buf][j / NB], fr[buf][MB + j % NB], acc[j / NB][j % NB]);
  };
  using C0 = std::integral_constant<int, 0>;

  // One slab.  PAR: parity of the slab (LDS stage).  The body is the same for every
  // slab, so that the compiler sees one loop and no accumulator-carrying branches: near
  // the end of K the "slab+2" request is clamped to the last slab (a redundant, in-bounds
  // load) and the last slab's LDS store / fragment read move data nobody uses.
  auto one_slab = [&](auto par_c, int slab) __attribute__((always_inline)) {
    constexpr int PAR = decltype(par_c)::value;
    constexpr bool MORE = true, LOAD2 = true;
    using Cur = std::integral_constant<int, PAR>;
    using Nxt = std::integral_constant<int, PAR ^ 1>;
    locate(slab + 2 < k_slabs ? slab + 2 : k_slabs - 1);
    static_for<4 * NMMA>([&](auto g_c) __attribute__((always_inline)) {
      constexpr int g = decltype(g_c)::value;  // slot index inside the slab
      constexpr int s = g / NMMA, j = g % NMMA;
      using Buf = std::integral_constant<int, s & 1>;
      using NBuf = std::integral_constant<int, (s + 1) & 1>;
      if constexpr (g == 3 * NMMA && MORE) lds_barrier();
      mma(Buf{}, std::integral_constant<int, j>{});
      // fragments of the next sub-step: one LDS read behind each of the first slots
      static_for<NFRAG>([&](auto i_c) __attribute__((always_inline)) {
        constexpr int i = decltype(i_c)::value;
        if constexpr (i == j) {
          if constexpr (s < 3) fread(NBuf{}, i_c, Cur{}, std::integral_constant<int, (s + 1) & 3>{});
          else if constexpr (MORE) fread(NBuf{}, i_c, Nxt{}, C0{});
        }
      });
      // next slab: registers -> other LDS stage, spread evenly over the three sub-steps
      // before the barrier; the freed register is refilled at once with slab+2
      static_for<NLD>([&](auto i_c) __attribute__((always_inline)) {
        constexpr int i = decltype(i_c)::value;
        if constexpr (i * 3 * NMMA / NLD == g) {
          if constexpr (MORE) lstore(i_c, Nxt{});
          if constexpr (LOAD2) gload(i_c);
        }
      });
      __builtin_amdgcn_sched_barrier(0);
    });
  };
  using P0 = std::integral_constant<int, 0>;
  using P1 = std::integral_constant<int, 1>;

  // prologue: slab 0 -> LDS stage 0, slab 1 -> registers, first fragments -> buffer 0
  locate(0);
  static_for<NLD>([&](auto i_c) __attribute__((always_inline)) { gload(i_c); });
  static_for<NLD>([&](auto i_c) __attribute__((always_inline)) { lstore(i_c, P0{}); });
  locate(k_slabs > 1 ? 1 : 0);
  static_for<NLD>([&](auto i_c) __attribute__((always_inline)) { gload(i_c); });
  lds_barrier();
  static_for<NFRAG>([&](auto i_c) __attribute__((always_inline)) { fread(P0{}, i_c, P0{}, C0{}); });
  __builtin_amdgcn_sched_barrier(0);
  KT_STAMP_LOOP_START();

  int slab = 0;
  for (; slab + 1 < k_slabs; slab += 2) {
    one_slab(P0{}, slab);
    one_slab(P1{}, slab + 1);
  }
  if (slab < k_slabs) one_slab(P0{}, slab);
}

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

template <class TL, class Epi, bool ATN = false>
__global__ __launch_bounds__(TL::NT) void gemm_nt_kernel(GemmShape g, Epi epi) {
  extern __shared__ __align__(16) char lds[];
  using T = typename TL::T;
  const int batch = blockIdx.y;
  int tm, tn, ks;
  if (!tile_of_block(g, tm, tn, ks)) return;
  if (epi.skip(batch)) return;
  KT_STAMP_WALL(g, 4);
  KT_STAMP(g, 0);
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
  gemm_mainloop<TL, ATN>(A, g.lda, g.M, m0, B, g.ldb, g.N, n0, slab0, slabs, g.slabs_per_block,
                         g.block_bytes_a, g.block_bytes_b, acc, lds, g.k_valid KT_STAMP_ARG);
  KT_STAMP(g, 2);
  epi(acc, batch, tm, tn, ks, m0, n0);
  KT_STAMP(g, 3);
  KT_STAMP_WALL(g, 5);
#ifdef KT_PHASE_STAMPS
  if (threadIdx.x == 0 && g.stamp_slot >= 0) {
    const size_t wg = (size_t)blockIdx.y * gridDim.x + blockIdx.x;
    if (wg < (size_t)kStampWgs)
      g_phase_stamps[((size_t)g.stamp_slot * kStampWgs + wg) * kStampWords + 6] = __builtin_amdgcn_s_getreg((4 << 0) | (0 << 6) | (31 << 11));
  }
#endif
}

}  // namespace kt
