// kt_fused_d128.h -- the whole loss + gradient pass for head-dimension rotations
// (d = 128, bf16) in ONE kernel that reads X exactly once.
//
// For many small independent problems (one 128 x 128 rotation per KV head and layer, the
// R2 learner of "Learning the Rotations") the three-GEMM path is bandwidth-bound: it
// reads X three times and writes and re-reads two token-minor copies.  Here a workgroup
// walks token tiles of 256 rows of one problem and, per tile,
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
// LDS (160 KiB): R^T 32 KiB | X tile 64 KiB | G tile 64 KiB, rows of 256 bytes.
//  R^T and X: 16-byte chunks XOR-swizzled with (row & 15) -> conflict-free fragment reads.
//  G: 8-byte units XOR-swizzled with swz(t) = 4*(t%8) + (t/8)%4 -> conflict-free 8-byte
//  stores from 32 token lanes and conflict-free transposing reads.
#pragma once
#include "kt_aux.h"

namespace kt {

constexpr int kF128RtOff = 0, kF128XOff = 32768, kF128GOff = 32768 + 65536;
constexpr int kF128LdsBytes = 32768 + 65536 + 65536;

typedef short shortx4 __attribute__((ext_vector_type(4)));

// Two transposing 8-byte LDS reads -> one MFMA operand (8 bf16 along K for this lane's row).
// In a group of 16 lanes, lane r supplies the address of 4 consecutive features of token
// t0 + r/4 starting at feature f0 + 4*(r%4); lane L of the group receives feature f0 + L of
// tokens t0..t0+3.  `addr_lo` / `addr_hi` are this lane's addresses for tokens +0..3 / +4..7.
__device__ __forceinline__ intx4 read_tr_operand(const char* lds, int addr_lo, int addr_hi) {
  typedef __attribute__((address_space(3))) shortx4* lds_ptr;
  const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(lds + addr_lo));
  const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(lds + addr_hi));
  typedef short shortx8 __attribute__((ext_vector_type(8)));
  const shortx8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(intx4, v);
}

// grid = (S, batch): S workgroups share the token tiles of one problem.
// dR_part[(wg * batch + b) * 128*128 + k*128 + j], loss_part[b * S + wg].
__global__ __launch_bounds__(256) void fused_d128_kernel(const __bf16* __restrict__ X, int64_t ldx,
                                                         int64_t x_batch_stride,
                                                         const __bf16* __restrict__ RT, int n,
                                                         float kappa_target,
                                                         float* __restrict__ row_kurt,
                                                         double* __restrict__ loss_part,
                                                         float* __restrict__ dR_part, int want_grad) {
  extern __shared__ __align__(16) char lds[];
  constexpr int D = 128;
  const int b = blockIdx.y, S = gridDim.x, wg = blockIdx.x, batch = gridDim.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, l32 = lane & 31;
  const int wm2 = wave >> 1, wn2 = wave & 1;  // dR quadrant of this wave in stage E
  X += (int64_t)b * x_batch_stride;
  RT += (int64_t)b * D * D;
  const int tiles = (n + 255) / 256;

  // R^T -> LDS (8 chunks of 16 bytes per thread)
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int c = tid + i * 256, row = c >> 4, ch = c & 15;
    const intx4 v = *reinterpret_cast<const intx4*>(RT + row * D + ch * 8);
    *reinterpret_cast<intx4*>(lds + kF128RtOff + row * 256 + ((ch ^ (row & 15)) << 4)) = v;
  }

  intx4 xr[16];  // one X tile in flight: 16 chunks of 16 bytes per thread
  auto gload_tile = [&](int tile) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int c = tid + i * 256, row = c >> 4, ch = c & 15;
      const int token = tile * 256 + row;
      intx4 v = {0, 0, 0, 0};
      if (token < n) v = *reinterpret_cast<const intx4*>(X + (int64_t)token * ldx + ch * 8);
      xr[i] = v;
    }
  };
  auto store_tile = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int c = tid + i * 256, row = c >> 4, ch = c & 15;
      *reinterpret_cast<intx4*>(lds + kF128XOff + row * 256 + ((ch ^ (row & 15)) << 4)) = xr[i];
    }
  };

  floatx16 acc2[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc2[i][j][r] = 0.f;
  double loss_acc = 0.0;
  const float inv_d = 1.0f / (float)D;
  const float grad_scale = 4.0f / ((float)n * (float)D);

  // lane constants of the transposing reads (stage E)
  const int g16 = lane >> 4, rr = lane & 15;
  const int tr_feat = 16 * (g16 & 1) + 4 * (rr & 3);  // + block base: first of 4 features
  const int tr_tok = 8 * (g16 >> 1) + (rr >> 2);      // + 16*s (+4): token row inside the tile

  int tile = wg;
  if (tile < tiles) gload_tile(tile);
  for (; tile < tiles; tile += S) {
    __syncthreads();  // everyone is done with the previous X and G tiles (and R^T is stored)
    store_tile();
    if (tile + S < tiles) gload_tile(tile + S);
    __syncthreads();

    // ---- B: Y^T (features x this wave's 64 tokens) = R^T X_tile^T -------------------
    floatx16 acc[4][2];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.f;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const int coff = ((2 * s + half) ^ (l32 & 15)) << 4;
      intx4 a[4], bb[2];
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
        a[mb] = *reinterpret_cast<const intx4*>(lds + kF128RtOff + (mb * 32 + l32) * 256 + coff);
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
        bb[nb] = *reinterpret_cast<const intx4*>(lds + kF128XOff + (wave * 64 + nb * 32 + l32) * 256 + coff);
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) Mma<__bf16>::run(a[mb], bb[nb], acc[mb][nb]);
    }

    // ---- C, D: per-token statistics and dL/dY ------------------------------------------
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const int tok_local = wave * 64 + nb * 32 + l32;
      const int token = tile * 256 + tok_local;
      const bool valid = token < n;
      float s1 = 0.f;
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s1 += acc[mb][nb][r];
      s1 += __shfl_xor(s1, 32);
      const float mu = s1 * inv_d;
      float s2 = 0.f, s3 = 0.f, s4 = 0.f;
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float c = acc[mb][nb][r] - mu;
          acc[mb][nb][r] = c;
          const float c2 = c * c;
          s2 += c2;
          s3 = fmaf(c2, c, s3);
          s4 = fmaf(c2, c2, s4);
        }
      s2 += __shfl_xor(s2, 32);
      s3 += __shfl_xor(s3, 32);
      s4 += __shfl_xor(s4, 32);
      const float m2 = s2 * inv_d, m3 = s3 * inv_d, m4 = s4 * inv_d;
      const bool ok = valid && m2 > 1e-5f * (m2 + mu * mu);
      float kappa = 0.f, alpha = 0.f, beta = 0.f, term = 0.f;
      if (ok) {
        kappa = m4 / (m2 * m2);
        float sgn = 1.f;
        if (kappa_target != 0.f) {
          const float dk = kappa - kappa_target;
          sgn = (float)((dk > 0.f) - (dk < 0.f));
          term = fabsf(dk);
        } else {
          term = kappa;
        }
        alpha = sgn * grad_scale / (m2 * m2);
        beta = kappa * m2;
      } else if (valid && kappa_target != 0.f) {
        term = fabsf(kappa_target);
      }
      if (half == 0 && valid) {
        loss_acc += (double)term;
        if (row_kurt) row_kurt[(int64_t)b * n + token] = kappa;
      }
      if (want_grad) {
        const int swz = ((tok_local & 7) << 2) | ((tok_local >> 3) & 3);
        char* grow = lds + kF128GOff + tok_local * 256;
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
            bf16x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float c = acc[mb][nb][4 * q + e];
              float g = alpha * fmaf(c, fmaf(c, c, -beta), -m3);
              if (alpha == 0.f) g = 0.f;
              v[e] = (__bf16)g;
            }
            const int u = mb * 8 + 2 * q + half;  // 8-byte unit: features 4u .. 4u+3
            *reinterpret_cast<bf16x4*>(grow + ((u ^ swz) << 3)) = v;
          }
      }
    }
    if (!want_grad) continue;
    __syncthreads();

    // ---- E: dR quadrant += X_tile^T G_tile, K = the tile's 256 tokens -------------------
#pragma unroll 4
    for (int s = 0; s < 16; ++s) {
      const int t_lo = 16 * s + tr_tok, t_hi = t_lo + 4;
      intx4 a[2], bb[2];
#pragma unroll
      for (int ib = 0; ib < 2; ++ib) {
        const int u = (wm2 * 64 + ib * 32 + tr_feat) >> 2;  // 8-byte unit inside the X row
        const int sel = (u & 1) << 3, ch = u >> 1;
        a[ib] = read_tr_operand(lds, kF128XOff + t_lo * 256 + (((ch ^ (t_lo & 15)) << 4) | sel),
                                kF128XOff + t_hi * 256 + (((ch ^ (t_hi & 15)) << 4) | sel));
      }
#pragma unroll
      for (int jb = 0; jb < 2; ++jb) {
        const int u = (wn2 * 64 + jb * 32 + tr_feat) >> 2;
        const int z_lo = ((t_lo & 7) << 2) | ((t_lo >> 3) & 3), z_hi = ((t_hi & 7) << 2) | ((t_hi >> 3) & 3);
        bb[jb] = read_tr_operand(lds, kF128GOff + t_lo * 256 + ((u ^ z_lo) << 3),
                                 kF128GOff + t_hi * 256 + ((u ^ z_hi) << 3));
      }
#pragma unroll
      for (int ib = 0; ib < 2; ++ib)
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) Mma<__bf16>::run(a[ib], bb[jb], acc2[ib][jb]);
    }
  }

  // ---- wrap-up: partial dR and partial loss of this workgroup ----------------------------
  if (want_grad) {
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

}  // namespace kt
