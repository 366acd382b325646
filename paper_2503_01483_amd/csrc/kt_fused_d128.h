// kt_fused_d128.h -- the whole loss + gradient pass for head-dimension rotations
// (d = 128, bf16) in ONE kernel that reads X exactly once.
//
// For many small independent problems (one 128 x 128 rotation per KV head and layer, the
// R2 learner of "Learning the Rotations") the three-GEMM path is bandwidth-bound: it
// reads X three times and writes and re-reads two token-minor copies.  Here a workgroup
// walks token tiles of 128 rows of one problem and, per tile,
//   B. Y = X_tile R            (MFMA; token on the lane, all 128 features of a token in the
//                               registers of one lane pair)
//   C. per-token mean, centred moments (two-pass, fp32), kurtosis, loss term,
//      coefficients           (Eq. 3 and its chain rule; Y is still in registers: no recompute)
//   D. G = dL/dY -> bf16 -> LDS, token-major like the X tile
//   E. dR += X_tile^T G_tile   (MFMA; both operands are read token-minor straight out of the
//                               token-major LDS tiles with ds_read_b64_tr_b16, the gfx950
//                               transposing LDS read)
// and keeps its 128 x 128 share of dR in accumulator registers until its last tile.
// Partial dR and loss sums of the workgroups of a problem are added by fixed-order
// reduction kernels afterwards.
//
// LDS (160 KiB): three X tiles and two G tiles of 32 KiB, rows of 256 bytes (X(i+2) arrives
// while E reads X(i) and B reads X(i+1); stage E of one tile overlaps stages C-D of the next);
// R^T lives in registers.
//  X: 16-byte chunks XOR-swizzled with xkey(row) = 4*(row%4) + (row/4)%4: distinct over 16
//  consecutive rows (conflict-free 16-byte fragment reads of 16 rows at one column), and the
//  4 consecutive tokens a half wave reads transposed fall into 4 different 64-byte bank groups.
//  G: 8-byte units XOR-swizzled with gkey(t) = 8*(t%4) + (t/4)%8: distinct over 32 tokens
//  (conflict-free 8-byte stores from 32 token lanes), same property for the transposed reads.
//  stores from 32 token lanes and conflict-free transposing reads.
#pragma once
#include "kt_aux.h"
#include "kt_gemm.h"

namespace kt {

constexpr int kF128Tile = 128;                  // tokens per tile
constexpr int kF128BufBytes = kF128Tile * 256;  // one X or G tile: 128 rows of 256 bytes
constexpr int kF128GOff = 3 * kF128BufBytes;     // LDS: X[3] | G[2]
constexpr int kF128LdsBytes = 5 * kF128BufBytes;  // 160 KiB

__device__ __forceinline__ int f128_xkey(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
__device__ __forceinline__ int f128_gkey(int t) { return ((t & 3) << 3) | ((t >> 2) & 7); }

// The matrix-core instructions of this kernel are written as inline assembly so that the
// register file of every operand is fixed: R^T fragments and the dR accumulators live in
// accumulation registers (only the matrix core touches them), Y and the LDS fragments in
// vector registers (the vector ALU consumes Y).  Left to the register allocator the 256
// registers of R^T and accumulators get shuffled between the two files every tile.
// The compiler does not know these are matrix instructions: results are read by other
// instruction types only behind mfma_result_fence().
__device__ __forceinline__ void mfma_y_first(floatx16& y, const intx4& rt, const intx4& x) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(y) : "a"(rt), "v"(x));
}
__device__ __forceinline__ void mfma_y(floatx16& y, const intx4& rt, const intx4& x) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(y) : "a"(rt), "v"(x));
}
__device__ __forceinline__ void mfma_dr(floatx16& acc, const intx4& xt, const intx4& gt) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(xt), "v"(gt));
}
// An 8-pass matrix instruction must be 11 issue slots old before another instruction type
// reads its result.
__device__ __forceinline__ void mfma_result_fence(floatx16& a, floatx16& b, floatx16& c, floatx16& d) {
  asm volatile("s_nop 15" : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}
__device__ __forceinline__ void mfma_result_fence_acc(floatx16& a, floatx16& b, floatx16& c, floatx16& d) {
  asm volatile("s_nop 15" : "+a"(a), "+a"(b), "+a"(c), "+a"(d));
}

// 16 bytes per lane from global memory straight into LDS: lane l lands at lds_addr + 16 l
// (lds_addr is wave-uniform).  Written as assembly so that the compiler does not tie later LDS
// reads to these loads with a full wait; the waits are placed by hand (vmcnt).
__device__ __forceinline__ void load_to_lds_16(const void* src, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds_addr)
               : "memory");
}

// grid = (S, batch): S workgroups share the token tiles of one problem.
// dR_part[(wg * batch + b) * 128*128 + k*128 + j], loss_part[b * S + wg].
//
// Software pipeline over the tiles i = 0, 1, ... of a workgroup (one barrier per tile).
// X(i) lives in X buffer i % 3, G(i) in G buffer i & 1.  Iteration i:
//   request X(i+2) (global -> LDS, buffer last read by E(i-1)); wait for X(i+1)
//   B(i+1): Y = X R on the wave's own 32 rows (it moved those rows itself: no barrier)
//   E(i) and C/D(i+1) as ONE instruction stream: one matrix instruction of
//     dR += X(i)^T G(i) every ~20 vector instructions of the statistics / dL/dY arithmetic
//   barrier (G(i+1) complete for every wave; buffers of tile i free)
__global__ __launch_bounds__(256) void fused_d128_kernel(const __bf16* __restrict__ X, int64_t ldx,
                                                         int64_t x_batch_stride,
                                                         const __bf16* __restrict__ RT, int n,
                                                         float kappa_target,
                                                         float* __restrict__ row_kurt,
                                                         double* __restrict__ loss_part,
                                                         float* __restrict__ dR_part, int want_grad) {
  extern __shared__ __align__(16) char lds[];
  constexpr int D = 128, T = kF128Tile, BUF = kF128BufBytes;
  using std::integral_constant;
  const int b = blockIdx.y, S = gridDim.x, wg = blockIdx.x, batch = gridDim.y;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5, l32 = lane & 31;
  const int wm2 = wave >> 1, wn2 = wave & 1;  // dR quadrant of this wave in stage E
  X += (int64_t)b * x_batch_stride;
  RT += (int64_t)b * D * D;
  const int tiles = (n + T - 1) / T;
  const int my_tiles = wg < tiles ? (tiles - wg + S - 1) / S : 0;  // tiles wg, wg+S, ...
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) char*)lds;

  // R^T fragments for all 8 K sub-steps and 4 feature blocks: 128 registers, loaded once
  intx4 rtf[8][4];
#pragma unroll
  for (int s = 0; s < 8; ++s)
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
      rtf[s][mb] = *reinterpret_cast<const intx4*>(RT + (mb * 32 + l32) * D + (2 * s + half) * 8);
      asm volatile("" : "+a"(rtf[s][mb]));
    }

  // X tile movement: a wave owns rows 32*wave .. +31 of the tile and moves them with 8
  // instructions of 4 rows (1 KiB) each.  The 16-byte swizzle is applied on the source side:
  // LDS chunk position (l & 15) of row r receives global chunk (l & 15) ^ xkey(r).
  const int xrow0 = wave * 32 + (lane >> 4);  // tile row of instruction 0; instruction i: + 4 i
  const __bf16* xlane[4];                     // source of instruction i at tile 0: xlane[i & 3] + 4 i ldx
#pragma unroll
  for (int i = 0; i < 4; ++i)
    xlane[i] = X + (int64_t)xrow0 * ldx + (((lane & 15) ^ f128_xkey(4 * i + (lane >> 4))) << 3);
  auto load_tile = [&](int tile, int buf) __attribute__((always_inline)) {
    const unsigned dst = lds_base + buf * BUF + wave * (32 * 256);
    const int64_t tile_off = (int64_t)tile * T * ldx;
    if (tile * T + T <= n) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
        load_to_lds_16(xlane[i & 3] + tile_off + (int64_t)(4 * i) * ldx, dst + i * 1024);
    } else {  // last, partial tile: rows past the end are zero-filled
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (tile * T + xrow0 + 4 * i < n)
          load_to_lds_16(xlane[i & 3] + tile_off + (int64_t)(4 * i) * ldx, dst + i * 1024);
        else
          *reinterpret_cast<intx4*>(lds + buf * BUF + wave * (32 * 256) + i * 1024 + lane * 16) =
              intx4{0, 0, 0, 0};
      }
    }
  };

  floatx16 acc2[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
      for (int r = 0; r < 16; ++r) acc2[i][j][r] = 0.f;
      asm volatile("" : "+a"(acc2[i][j]));
    }
  double loss_acc = 0.0;
  const float inv_d = 1.0f / (float)D;
  const float grad_scale = 4.0f / ((float)n * (float)D);

  // lane constants of the transposing reads (stage E): token row 16 s + tr_tok (+4) of the tile
  const int g16 = lane >> 4, rr = lane & 15;
  const int tr_feat = 16 * (g16 & 1) + 4 * (rr & 3);
  const int tr_tok = 8 * (g16 >> 1) + (rr >> 2);
  int xa_lo[2], xa_hi[2], gb_lo[2][2], gb_hi[2][2];  // G: [parity of s][block]
#pragma unroll
  for (int ib = 0; ib < 2; ++ib) {
    const int u = (wm2 * 64 + ib * 32 + tr_feat) >> 2;  // 8-byte unit inside the X row
    const int sel = (u & 1) << 3, ch = u >> 1, t_hi = tr_tok + 4;
    xa_lo[ib] = tr_tok * 256 + (((ch ^ f128_xkey(tr_tok)) << 4) | sel);
    xa_hi[ib] = t_hi * 256 + (((ch ^ f128_xkey(t_hi)) << 4) | sel);
  }
#pragma unroll
  for (int par = 0; par < 2; ++par)
#pragma unroll
    for (int jb = 0; jb < 2; ++jb) {
      const int u = (wn2 * 64 + jb * 32 + tr_feat) >> 2;
      const int t_lo = 16 * par + tr_tok, t_hi = t_lo + 4;
      const int z_lo = f128_gkey(t_lo), z_hi = f128_gkey(t_hi);
      gb_lo[par][jb] = tr_tok * 256 + ((u ^ z_lo) << 3);
      gb_hi[par][jb] = (tr_tok + 4) * 256 + ((u ^ z_hi) << 3);
    }

  floatx16 acc[4];  // Y^T of the tile in flight: 64 of the 128 features of this lane's token

  // B: Y^T (128 features x this wave's 32 tokens) = R^T X^T from X buffer `buf`
  auto stage_b = [&](int buf) __attribute__((always_inline)) {
    const char* xrow = lds + buf * BUF + (wave * 32 + l32) * 256;
    intx4 xb[2];
    xb[0] = *reinterpret_cast<const intx4*>(xrow + (((0 + half) ^ f128_xkey(l32)) << 4));
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      if (s + 1 < 8)
        xb[(s + 1) & 1] = *reinterpret_cast<const intx4*>(xrow + (((2 * (s + 1) + half) ^ f128_xkey(l32)) << 4));
#pragma unroll
      for (int mb = 0; mb < 4; ++mb) {
        if (s == 0)
          mfma_y_first(acc[mb], rtf[0][mb], xb[0]);
        else
          mfma_y(acc[mb], rtf[s][mb], xb[s & 1]);
      }
    }
    mfma_result_fence(acc[0], acc[1], acc[2], acc[3]);
  };

  // C, D of tile `tile` (statistics of this lane's token, dL/dY -> G buffer gbuf_w) with the 32
  // matrix instructions of E (X buffer xbuf_r, G buffer gbuf_r) dealt between the arithmetic.
  // WITH_CD / WITH_E switch the two halves off for the first and last tile of a workgroup.
  auto stage_cde = [&](auto with_cd_c, auto with_e_c, int tile, int gbuf_w, int xbuf_r,
                       int gbuf_r) __attribute__((always_inline)) {
    constexpr bool WITH_CD = decltype(with_cd_c)::value, WITH_E = decltype(with_e_c)::value;
    const char* xbase = lds + xbuf_r * BUF;
    const char* gbase = lds + kF128GOff + gbuf_r * BUF;
    intx4 fa[2][2], fb[2][2];
    // one operand of K sub-step s (two transposing reads): 0 X block 0, 1 G block 0, 2 G block 1, 3 X block 1
    auto fread_one = [&](auto s_c, auto which_c) __attribute__((always_inline)) {
      constexpr int s = decltype(s_c)::value, which = decltype(which_c)::value;
      if constexpr (which == 0 || which == 3) {
        constexpr int ib = which == 0 ? 0 : 1;
        fa[s & 1][ib] = read_tr_operand(xbase, xa_lo[ib] + s * 16 * 256, xa_hi[ib] + s * 16 * 256);
      } else {
        constexpr int jb = which - 1;
        fb[s & 1][jb] = read_tr_operand(gbase, gb_lo[s & 1][jb] + s * 16 * 256, gb_hi[s & 1][jb] + s * 16 * 256);
      }
    };
    auto fread = [&](auto s_c) __attribute__((always_inline)) {
      static_for<4>([&](auto w_c) __attribute__((always_inline)) { fread_one(s_c, w_c); });
    };
    // matrix instruction k of E: K sub-step k / 4, dR block (k / 2) & 1, k & 1.  The four operands of the next
    // sub-step are read one per instruction slot, BEHIND the slot's matrix instruction and in the order the next
    // sub-step uses them: never more than eight LDS reads are in flight, so the wait in front of a matrix
    // instruction can name exactly the reads it needs (the counter has four bits: with all sixteen reads of a
    // sub-step issued at once, every fourth matrix instruction also waited for reads it did not need).
    auto tick = [&](auto k_c) __attribute__((always_inline)) {
      if constexpr (WITH_E) {
        constexpr int k = decltype(k_c)::value, s = k >> 2, ib = (k >> 1) & 1, jb = k & 1;
        __builtin_amdgcn_sched_barrier(0);
        mfma_dr(acc2[ib][jb], fa[s & 1][ib], fb[s & 1][jb]);
        if constexpr (s + 1 < 8) fread_one(integral_constant<int, s + 1>{}, integral_constant<int, k & 3>{});
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    if constexpr (WITH_E) fread(integral_constant<int, 0>{});
    if constexpr (!WITH_CD) {
      static_for<32>(tick);
    } else {
      const int tok_local = wave * 32 + l32;
      const int token = tile * T + tok_local;
      const bool valid = token < n;
      float s1 = 0.f;
      static_for<4>([&](auto mb_c) __attribute__((always_inline)) {
        constexpr int mb = decltype(mb_c)::value;
#pragma unroll
        for (int r = 0; r < 16; ++r) s1 += acc[mb][r];
        tick(integral_constant<int, mb>{});
      });
      s1 += __shfl_xor(s1, 32);
      const float mu = s1 * inv_d;
      float s2 = 0.f, s3 = 0.f, s4 = 0.f;
      static_for<16>([&](auto g_c) __attribute__((always_inline)) {
        constexpr int g = decltype(g_c)::value, mb = g >> 2, q = g & 3;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float c = acc[mb][4 * q + e] - mu;
          acc[mb][4 * q + e] = c;
          const float c2 = c * c;
          s2 += c2;
          s3 = fmaf(c2, c, s3);
          s4 = fmaf(c2, c2, s4);
        }
        tick(integral_constant<int, 4 + g>{});
      });
      s2 += __shfl_xor(s2, 32);
      s3 += __shfl_xor(s3, 32);
      s4 += __shfl_xor(s4, 32);
      tick(integral_constant<int, 20>{});
      const float m2 = s2 * inv_d, m3 = s3 * inv_d, m4 = s4 * inv_d;
      const bool ok = valid && m2 > 1e-10f * (m2 + mu * mu);  // same rule as finalize_rows_kernel
      // branch-free: a degenerate or out-of-range token gets kappa = 0 and no gradient
      const float m2s = ok ? m2 : 1.f;
      const float inv_m2sq = 1.0f / (m2s * m2s);
      const float kappa = ok ? m4 * inv_m2sq : 0.f;
      float sgn = 1.f, term = kappa;
      if (kappa_target != 0.f) {  // uniform
        const float dk = kappa - kappa_target;
        sgn = (float)((dk > 0.f) - (dk < 0.f));
        term = fabsf(dk);
      }
      const float alpha = ok ? sgn * grad_scale * inv_m2sq : 0.f;
      const float beta = kappa * m2;
      loss_acc += (half == 0 && valid) ? (double)term : 0.0;
      tick(integral_constant<int, 21>{});
      if (want_grad) {
        const int swz = f128_gkey(tok_local);
        char* grow = lds + kF128GOff + gbuf_w * BUF + tok_local * 256;
        static_for<16>([&](auto g_c) __attribute__((always_inline)) {
          constexpr int g = decltype(g_c)::value, mb = g >> 2, q = g & 3;
          typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float c = acc[mb][4 * q + e];
            v[e] = (__bf16)(alpha * fmaf(c, fmaf(c, c, -beta), -m3));
          }
          const int u = mb * 8 + 2 * q + half;  // 8-byte unit: features 4u .. 4u+3
          *reinterpret_cast<bf16x4*>(grow + ((u ^ swz) << 3)) = v;
          constexpr int k0 = 22 + (g * 10) / 16, k1 = 22 + ((g + 1) * 10) / 16;
          if constexpr (k1 > k0) tick(integral_constant<int, k0>{});
        });
      } else {
        static_for<10>([&](auto j_c) __attribute__((always_inline)) {
          tick(integral_constant<int, 22 + decltype(j_c)::value>{});
        });
      }
      if (row_kurt && half == 0 && valid) row_kurt[(int64_t)b * n + token] = kappa;
    }
  };
  using Yes = std::true_type;
  using No = std::false_type;

  if (my_tiles > 0) {
    load_tile(wg, 0);
    if (my_tiles > 1) load_tile(wg + S, 1);
    // vmcnt(8) leaves the 8 newest loads in flight; a partial tile issues fewer than 8
    if (my_tiles > 1 && (wg + S) * T + T <= n)
      __builtin_amdgcn_s_waitcnt(0x0F78);
    else
      __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    asm volatile("" ::: "memory");
    stage_b(0);
    stage_cde(Yes{}, No{}, wg, 0, 0, 0);
    lds_barrier();
    int xcur = 0;
    // advance to tile i+1: request X(i+2), wait for X(i+1), B(i+1); returns the X buffer of i+1
    auto advance = [&](int i) __attribute__((always_inline)) {
      const int xnxt = xcur == 2 ? 0 : xcur + 1, xnn = xnxt == 2 ? 0 : xnxt + 1;
      const int t2 = wg + (i + 2) * S;
      const bool more2 = i + 2 < my_tiles;
      if (more2) load_tile(t2, xnn);  // buffer last read by E(i-1)
      if (more2 && t2 * T + T <= n)
        __builtin_amdgcn_s_waitcnt(0x0F78);  // X(i+1) landed, X(i+2) in flight
      else
        __builtin_amdgcn_s_waitcnt(0x0F70);
      asm volatile("" ::: "memory");
      stage_b(xnxt);
      return xnxt;
    };
    if (want_grad) {
      for (int i = 0; i + 1 < my_tiles; ++i) {
        const int xnxt = advance(i);
        stage_cde(Yes{}, Yes{}, wg + (i + 1) * S, (i + 1) & 1, xcur, i & 1);
        lds_barrier();
        xcur = xnxt;
      }
      stage_cde(No{}, Yes{}, 0, 0, xcur, (my_tiles - 1) & 1);
    } else {
      for (int i = 0; i + 1 < my_tiles; ++i) {
        const int xnxt = advance(i);
        stage_cde(Yes{}, No{}, wg + (i + 1) * S, (i + 1) & 1, xcur, i & 1);
        lds_barrier();
        xcur = xnxt;
      }
    }
  }

  // ---- wrap-up: partial dR and partial loss of this workgroup ----------------------------
  if (want_grad) {
    mfma_result_fence_acc(acc2[0][0], acc2[0][1], acc2[1][0], acc2[1][1]);
    float* out = dR_part + ((int64_t)wg * batch + b) * (D * D);
#pragma unroll
    for (int ib = 0; ib < 2; ++ib)
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int k = wm2 * 64 + ib * 32 + ((r >> 2) << 3) + (half << 2) + (r & 3);
          const int j = wn2 * 64 + jb * 32 + l32;
          out[k * D + j] = acc2[ib][jb][r];
        }
  }
  __syncthreads();
  double* sh = reinterpret_cast<double*>(lds);
  const double total = block_sum_256(loss_acc, sh);
  if (tid == 0) loss_part[(int64_t)b * S + wg] = total;
}

// ---- single-pass rotate + int4 fake-quant for d = 128 (bf16) -------------------------------
// A lane pair holds a whole rotated token row, so the row maximum, the scale, the codes and the
// error sums all come out of ONE pass over X (the generic path parks the rotated rows in an fp32
// staging buffer between the GEMM and a row kernel).
// Every wave is on its own: 32-token tiles, its rows staged through 8 KiB of private LDS (loads of
// the next tile in flight), R^T fragments in accumulation registers, no workgroup barrier.
// Arithmetic identical to the generic path: s = (clip amax) / 7, q = clamp(rint(y (1/s)), -7, 7).
// grid = (waves / 4, batch).
__global__ __launch_bounds__(256) void quant_d128_kernel(const __bf16* __restrict__ X, int64_t ldx,
                                                         int64_t x_batch_stride, const __bf16* __restrict__ RT,
                                                         int n, float clip, const float* __restrict__ scales_in,
                                                         float* __restrict__ scales_out, int8_t* __restrict__ codes,
                                                         float2* __restrict__ err) {
  __shared__ __align__(16) char lds_all[4 * 32 * 256];
  constexpr int D = 128;
  const int b = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int half = lane >> 5, l32 = lane & 31;
  char* lds = lds_all + wave * (32 * 256);
  X += (int64_t)b * x_batch_stride;
  RT += (int64_t)b * D * D;
  const int tiles = (n + 31) / 32;
  const int wave_id = blockIdx.x * 4 + wave, stride = gridDim.x * 4;

  intx4 rtf[8][4];
#pragma unroll
  for (int s = 0; s < 8; ++s)
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
      rtf[s][mb] = *reinterpret_cast<const intx4*>(RT + (mb * 32 + l32) * D + (2 * s + half) * 8);
      asm volatile("" : "+a"(rtf[s][mb]));
    }

  // chunk i of a lane: tile row (lane >> 4) + 4 i, 16-byte column lane & 15
  intx4 nxt[8];
  auto request = [&](int tile) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = tile * 32 + (lane >> 4) + 4 * i;
      intx4 v = {0, 0, 0, 0};
      if (tile < tiles && row < n) v = *reinterpret_cast<const intx4*>(X + (int64_t)row * ldx + (lane & 15) * 8);
      nxt[i] = v;
    }
  };
  request(wave_id);
  for (int tile = wave_id; tile < tiles; tile += stride) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the previous tile's fragment reads are done
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = (lane >> 4) + 4 * i;
      *reinterpret_cast<intx4*>(lds + row * 256 + (((lane & 15) ^ f128_xkey(row)) << 4)) = nxt[i];
    }
    request(tile + stride);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // LDS of one wave executes in order; keep the compiler in order too
    floatx16 acc[4];
    {
      const char* xrow = lds + l32 * 256;
      intx4 xb[2];
      xb[0] = *reinterpret_cast<const intx4*>(xrow + (((0 + half) ^ f128_xkey(l32)) << 4));
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        if (s + 1 < 8)
          xb[(s + 1) & 1] = *reinterpret_cast<const intx4*>(xrow + (((2 * (s + 1) + half) ^ f128_xkey(l32)) << 4));
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
          if (s == 0)
            mfma_y_first(acc[mb], rtf[0][mb], xb[0]);
          else
            mfma_y(acc[mb], rtf[s][mb], xb[s & 1]);
        }
      }
      mfma_result_fence(acc[0], acc[1], acc[2], acc[3]);
    }
    const int token = tile * 32 + l32;
    const bool tv = token < n;
    const int64_t to = (int64_t)b * n + token;
    float s;
    if (scales_in) {
      s = tv ? scales_in[to] : 0.f;
    } else {
      float a = 0.f;
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) a = fmaxf(a, fabsf(acc[mb][r]));
      a = fmaxf(a, __shfl_xor(a, 32));
      s = __fdiv_rn(__fmul_rn(clip, a), 7.0f);
    }
    if (scales_out && tv && half == 0) scales_out[to] = s;
    if (codes || err) {
      const bool live = s > 0.f;
      const float rinv = live ? __fdiv_rn(1.0f, s) : 0.f;
      float e2 = 0.f, y2 = 0.f;
      int8_t* crow = codes + to * D;
#pragma unroll
      for (int mb = 0; mb < 4; ++mb) {
        unsigned pk[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          unsigned pack = 0u;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float y = acc[mb][4 * g + e];
            float q = rintf(__fmul_rn(y, rinv));
            q = fminf(fmaxf(q, -7.f), 7.f);
            if (!live) q = 0.f;
            const float diff = y - q * s;
            e2 = fmaf(diff, diff, e2);
            y2 = fmaf(y, y, y2);
            pack |= ((unsigned)(int)q & 0xffu) << (8 * e);
          }
          pk[g] = pack;
        }
        // A lane owns features 8g + 4 half .. + 3 of the 32-feature block, its partner (lane ^ 32) the other
        // four of each eight: swap two words so that each of the two holds 16 consecutive bytes of the
        // token's row (lower half-wave bytes 0..15 of the block, upper 16..31) and stores them at once.
        const unsigned r0 = (unsigned)__shfl_xor((int)(half ? pk[0] : pk[2]), 32);
        const unsigned r1 = (unsigned)__shfl_xor((int)(half ? pk[1] : pk[3]), 32);
        uintx4 out;
        if (half == 0) out = uintx4{pk[0], r0, pk[1], r1};
        else out = uintx4{r0, pk[2], r1, pk[3]};
        if (codes && tv) *reinterpret_cast<uintx4*>(crow + mb * 32 + 16 * half) = out;
      }
      if (err) {
        e2 += __shfl_xor(e2, 32);
        y2 += __shfl_xor(y2, 32);
        if (half == 0 && tv) err[to] = make_float2(e2, y2);
      }
    }
  }
}

}  // namespace kt
