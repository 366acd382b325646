// kt_aux.h -- the small bandwidth-bound kernels around the GEMMs: layout
// preparation, per-token finalisation, fixed-order reductions.
#pragma once
#include "kt_epilogues.h"

namespace kt {

template <typename Tin>
__device__ __forceinline__ float to_float(Tin v) { return (float)v; }

// out[c*ldo + r'] = in[r*ldi + c] for r < rows, c < cols; columns r in [rows, rows_pad)
// of `out` are zero-filled.  r' = r, or, when `permute` is set, the place of token r in the
// permuted, blocked token order of the X^T G operands (ldo = tokens per block, block b of
// all `cols` feature rows starts at b*cols*ldo; rows_pad must then be a multiple of 128).
// 64 x 64 tiles through LDS, 256 threads.
// grid = (ceil(rows_pad/64), ceil(cols/64), batch)
template <typename Tin, typename Tout>
__global__ __launch_bounds__(256) void transpose_kernel(const Tin* __restrict__ in, int64_t ldi,
                                                        int64_t in_batch_stride,
                                                        Tout* __restrict__ out, int64_t ldo,
                                                        int64_t out_batch_stride, int rows,
                                                        int rows_pad, int cols, int permute) {
  __shared__ float tile[64][65];
  const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  in += (int64_t)blockIdx.z * in_batch_stride;
  out += (int64_t)blockIdx.z * out_batch_stride;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int r = r0 + ty + 4 * i, c = c0 + tx;
    float v = 0.f;
    if (r < rows && c < cols) v = to_float(in[(int64_t)r * ldi + c]);
    tile[ty + 4 * i][tx] = v;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int c = c0 + ty + 4 * i, r = r0 + tx;
    if (c < cols && r < rows_pad) {
      int64_t o = (int64_t)c * ldo + r;
      if (permute) {  // token order and token blocks of the X^T G operands; ldo = block length
        const int64_t p = token_position(r), blk = p / ldo;
        o = blk * cols * ldo + (int64_t)c * ldo + (p - blk * ldo);
      }
      out[o] = from_float<Tout>(tile[tx][ty + 4 * i]);
    }
  }
}

// The token-minor, token-permuted, token-blocked copy of X for 2-byte elements, with
// 16-byte global accesses on both sides (layout as described at EpiGrad; ldo = tokens per
// block, a multiple of 128).
// tile = 128 rows (one token group) x 64 cols; each thread moves four 16-byte chunks in
// and four out.  Needs cols % 64 == 0, rows_pad % 128 == 0, ldi % 8 == 0, ldo % 8 == 0.
// grid = (ceil(rows_pad/128), cols/64, batch)
__global__ __launch_bounds__(256) void transpose16_kernel(const uint16_t* __restrict__ in, int64_t ldi,
                                                          int64_t in_batch_stride,
                                                          uint16_t* __restrict__ out, int64_t ldo,
                                                          int64_t out_batch_stride, int rows,
                                                          int rows_pad, int cols) {
  constexpr int PITCH = 33;  // dwords per tile row (64 elements + 1 dword of skew)
  __shared__ uint32_t tile[128 * PITCH];
  const int r0 = blockIdx.x * 128, c0 = blockIdx.y * 64;
  in += (int64_t)blockIdx.z * in_batch_stride;
  // ldo = tokens per block; the 128-token group r0 lies in block r0 / ldo
  out += (int64_t)blockIdx.z * out_batch_stride + (int64_t)(r0 / ldo) * cols * ldo + (r0 % ldo);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = threadIdx.x + i * 256;
    const int row = c >> 3, col8 = c & 7;
    intx4 v = {0, 0, 0, 0};
    if (r0 + row < rows) v = *reinterpret_cast<const intx4*>(in + (int64_t)(r0 + row) * ldi + c0 + col8 * 8);
    uint32_t* t = tile + row * PITCH + col8 * 4;
    t[0] = (uint32_t)v[0]; t[1] = (uint32_t)v[1]; t[2] = (uint32_t)v[2]; t[3] = (uint32_t)v[3];
  }
  __syncthreads();
  const uint16_t* t16 = reinterpret_cast<const uint16_t*>(tile);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = threadIdx.x + i * 256;
    const int f = c >> 4, t8 = c & 15;
    if (r0 + t8 * 8 < rows_pad) {
      uint32_t w[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        // output position p of the group holds token (p & 3) * 32 + (p >> 2)
        const int p = t8 * 8 + 2 * e;
        const uint32_t lo = t16[(((p & 3) << 5) + (p >> 2)) * (2 * PITCH) + f];
        const uint32_t hi = t16[((((p + 1) & 3) << 5) + ((p + 1) >> 2)) * (2 * PITCH) + f];
        w[e] = lo | (hi << 16);
      }
      intx4 v = {(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
      *reinterpret_cast<intx4*>(out + (int64_t)(c0 + f) * ldo + t8 * 8) = v;
    }
  }
}

// Row-major copy with dtype conversion: out[r*ldo + c] = in[r*ldi + c].
template <typename Tin, typename Tout>
__global__ __launch_bounds__(256) void convert_kernel(const Tin* __restrict__ in, int64_t ldi,
                                                      int64_t in_batch_stride,
                                                      Tout* __restrict__ out, int64_t ldo,
                                                      int64_t out_batch_stride, int rows, int cols) {
  in += (int64_t)blockIdx.z * in_batch_stride;
  out += (int64_t)blockIdx.z * out_batch_stride;
  const int64_t total = (int64_t)rows * cols;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int r = (int)(i / cols), c = (int)(i % cols);
    out[(int64_t)r * ldo + c] = from_float<Tout>(to_float(in[(int64_t)r * ldi + c]));
  }
}

__global__ __launch_bounds__(256) void fill_u32_kernel(unsigned* p, int64_t count, unsigned v) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256)
    p[i] = v;
}

__device__ __forceinline__ double block_sum_256(double v, double* sh) {
  const int tid = threadIdx.x;
  sh[tid] = v;
  __syncthreads();
#pragma unroll
  for (int s = 128; s >= 1; s >>= 1) {
    if (tid < s) sh[tid] += sh[tid + s];
    __syncthreads();
  }
  return sh[0];
}

// Moments of one token row from the P partials the forward epilogue wrote ({mean_p, sum c^2, sum c^3,
// sum c^4} about the partial's own mean, d / P features each), merged in fp64 with the shift
// formulas  sum (c + e)^k = sum c^k + k e sum c^(k-1) + ...  (sum c = 0 inside a partial):
// mu = row mean, M[0..2] = sums of (y - mu)^2, ^3, ^4 over the row.
__device__ __forceinline__ void row_central_sums(const floatx4* __restrict__ part, int P, int n, int64_t batch,
                                                 int token, int d, double& mu, double (&M)[3]) {
  const double cnt = (double)d / (double)P;
  double m = 0.0;
  for (int p = 0; p < P; ++p) m += (double)part[((int64_t)batch * P + p) * n + token][0];
  mu = m / (double)P;
  double M2 = 0.0, M3 = 0.0, M4 = 0.0;
  for (int p = 0; p < P; ++p) {
    const floatx4 v = part[((int64_t)batch * P + p) * n + token];
    const double e = (double)v[0] - mu, e2 = e * e;
    M2 += (double)v[1] + cnt * e2;
    M3 += (double)v[2] + 3.0 * e * (double)v[1] + cnt * e2 * e;
    M4 += (double)v[3] + 4.0 * e * (double)v[2] + 6.0 * e2 * (double)v[1] + cnt * e2 * e2;
  }
  M[0] = M2; M[1] = M3; M[2] = M4;
}

// Per token: merge the P partials in fixed order (fp64) into the central moments of
// Eq. 3, then kappa, the loss term and the coefficients the backward epilogue needs.  One thread per token; grid = (ceil(n/256), batch).
__global__ __launch_bounds__(256) void finalize_rows_kernel(const floatx4* __restrict__ part, int P,
                                                            int n, int d, float kappa_target,
                                                            floatx4* __restrict__ coef,
                                                            float* __restrict__ row_kurt,
                                                            double* __restrict__ loss_part) {
  __shared__ double sh[256];
  const int batch = blockIdx.y;
  const int token = blockIdx.x * 256 + threadIdx.x;
  double term = 0.0;
  if (token < n) {
    double mu, M[3];
    row_central_sums(part, P, n, batch, token, d, mu, M);
    const double inv_d = 1.0 / (double)d;
    const double m2 = M[0] * inv_d, m3 = M[1] * inv_d, m4 = M[2] * inv_d;
    const double r2 = m2 + mu * mu;
    // A row counts as having no spread when its variance is below 1e-10 of its mean square (sigma below 1e-5 of the
    // mean): fp32 accumulation leaves about 1e-13 there on a row that is constant in exact arithmetic, and a row
    // with a real spread that small cannot be resolved from fp32 products anyway.  Above the threshold kappa is
    // returned with an error that grows like 1e-6 |mean| / sigma instead of being silently dropped.
    const bool ok = m2 > 1e-10 * r2;  // same rule as the d = 128 kernel
    double kappa = 0.0, alpha = 0.0, beta = 0.0;
    if (ok) {
      kappa = m4 / (m2 * m2);
      double sgn = 1.0;
      if (kappa_target != 0.f) {
        const double dk = kappa - (double)kappa_target;
        sgn = (dk > 0.0) - (dk < 0.0);
        term = fabs(dk);
      } else {
        term = kappa;
      }
      alpha = sgn * 4.0 / ((double)n * (double)d * m2 * m2);
      beta = kappa * m2;
    } else if (kappa_target != 0.f) {
      term = fabs((double)kappa_target);
    }
    floatx4 c = {(float)alpha, (float)mu, (float)beta, (float)m3};
    coef[(int64_t)batch * n + token] = c;
    if (row_kurt) row_kurt[(int64_t)batch * n + token] = (float)kappa;
  }
  const double s = block_sum_256(term, sh);
  if (threadIdx.x == 0) loss_part[(int64_t)batch * gridDim.x + blockIdx.x] = s;
}

// dL/dY (chain rule through the kurtosis of Eq. 3; coefficients from finalize_rows_kernel) from a kept Y:
// GT[i] = grad_value(YT[i], coef of i's token) for every entry of the token-minor
// layout that EpiMomentsKeep / EpiGrad write (rows = features, blocks of tb tokens, tokens permuted inside
// groups of 128: position 4 j + k of a group holds token j + 32 k).  A half wave takes one group of 128
// positions (16 bytes of YT per lane), its four tokens' coefficients stay in registers while it walks
// FEATS feature rows; the four waves of a workgroup take four runs of feature rows of the same two groups.
// grid = (ceil(ldt / 256), ceil(d / (4 FEATS)), batch).  Padding tokens (>= n) get alpha = 0, as in EpiGrad.
template <typename T, int FEATS>
__global__ __launch_bounds__(256) void grad_from_y_kernel(const float* __restrict__ YT,
                                                          const floatx4* __restrict__ coef, T* __restrict__ GT,
                                                          int64_t ldt, int64_t tb, int64_t batch_stride, int n,
                                                          int d) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, batch = blockIdx.z;
  const int64_t group0 = ((int64_t)blockIdx.x * 2 + (lane >> 5)) * 128;
  if (group0 >= ldt) return;  // ldt is a multiple of 128: the second half wave of the last workgroup may have no group
  const int j = lane & 31;
  float alpha[4], mu[4], beta[4], m3[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int64_t token = group0 + j + 32 * k;
    floatx4 c4 = {0.f, 0.f, 0.f, 0.f};
    if (token < n) c4 = coef[(int64_t)batch * n + token];
    alpha[k] = c4[0]; mu[k] = c4[1]; beta[k] = c4[2]; m3[k] = c4[3];
  }
  const int64_t pos0 = group0 + 4 * j;
  const int64_t blk = pos0 / tb;
  const int64_t base = (int64_t)batch * batch_stride + blk * d * tb + (pos0 - blk * tb);
  const int f0 = (blockIdx.y * 4 + wave) * FEATS;
  float4 y[FEATS];
#pragma unroll
  for (int i = 0; i < FEATS; ++i)
    if (f0 + i < d) y[i] = *reinterpret_cast<const float4*>(YT + base + (int64_t)(f0 + i) * tb);
#pragma unroll
  for (int i = 0; i < FEATS; ++i) {
    if (f0 + i < d) {
      typedef T vecT __attribute__((ext_vector_type(4)));
      vecT v;
      v[0] = from_float<T>(grad_value(y[i].x, alpha[0], mu[0], beta[0], m3[0]));
      v[1] = from_float<T>(grad_value(y[i].y, alpha[1], mu[1], beta[1], m3[1]));
      v[2] = from_float<T>(grad_value(y[i].z, alpha[2], mu[2], beta[2], m3[2]));
      v[3] = from_float<T>(grad_value(y[i].w, alpha[3], mu[3], beta[3], m3[3]));
      *reinterpret_cast<vecT*>(GT + base + (int64_t)(f0 + i) * tb) = v;
    }
  }
}

// ---- pooled (paper-literal) loss: kurtosis of ALL entries of RMSNorm(X R) as one sample ------
// Row sums of z^k = (y / rho)^k follow from the row's sums of y^k, so the forward GEMM with the
// moment epilogue is used unchanged.  Stage 1: per token rho and the block partials of the four
// pooled raw sums.  grid = (ceil(n/256), batch).
__device__ __forceinline__ void pooled_row_sums(const floatx4* __restrict__ part, int P, int n, int64_t batch,
                                                int token, int d, double rms_eps, double& inv_rho,
                                                double (&Z)[4]) {
  double mu, M[3];
  row_central_sums(part, P, n, batch, token, d, mu, M);
  // raw sums of y^k over the row, from the central ones (fp64: nothing is lost going back)
  const double dd = (double)d, mu2 = mu * mu;
  const double S1 = dd * mu, S2 = M[0] + dd * mu2, S3 = M[1] + 3.0 * mu * M[0] + dd * mu2 * mu,
               S4 = M[2] + 4.0 * mu * M[1] + 6.0 * mu2 * M[0] + dd * mu2 * mu2;
  const double rho2 = S2 / (double)d + rms_eps;
  inv_rho = rho2 > 0.0 ? 1.0 / sqrt(rho2) : 0.0;  // a row of zeros: z = 0
  const double i2 = inv_rho * inv_rho;
  Z[0] = S1 * inv_rho; Z[1] = S2 * i2; Z[2] = S3 * i2 * inv_rho; Z[3] = S4 * i2 * i2;
}

__global__ __launch_bounds__(256) void pooled_stage1_kernel(const floatx4* __restrict__ part, int P, int n, int d,
                                                            float rms_eps, double* __restrict__ pool_part) {
  __shared__ double sh[256];
  const int batch = blockIdx.y, token = blockIdx.x * 256 + threadIdx.x;
  double Z[4] = {0, 0, 0, 0}, inv_rho;
  if (token < n) pooled_row_sums(part, P, n, batch, token, d, (double)rms_eps, inv_rho, Z);
  for (int k = 0; k < 4; ++k) {
    const double t = block_sum_256(Z[k], sh);
    if (threadIdx.x == 0) pool_part[(((int64_t)batch * gridDim.x + blockIdx.x) << 2) + k] = t;
    __syncthreads();
  }
}

// Stage 2: pooled moments, kappa, loss; gstat[batch] = {mu, m3, beta = kappa m2, A = s 4/(N m2^2)}.
// grid = batch.
__global__ __launch_bounds__(256) void pooled_stage2_kernel(const double* __restrict__ pool_part, int nblocks,
                                                            int n, int d, float kappa_target,
                                                            double* __restrict__ gstat, float* __restrict__ loss,
                                                            float* __restrict__ kappa_out) {
  __shared__ double sh[256];
  const int batch = blockIdx.x;
  double T[4];
  for (int k = 0; k < 4; ++k) {
    double v = 0.0;
    for (int i = threadIdx.x; i < nblocks; i += 256) v += pool_part[(((int64_t)batch * nblocks + i) << 2) + k];
    T[k] = block_sum_256(v, sh);
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double N = (double)n * (double)d;
    const double mu = T[0] / N, r2 = T[1] / N, r3 = T[2] / N, r4 = T[3] / N;
    const double m2 = r2 - mu * mu;
    const double m3 = r3 - 3.0 * mu * r2 + 2.0 * mu * mu * mu;
    const double m4 = r4 - 4.0 * mu * r3 + 6.0 * mu * mu * r2 - 3.0 * mu * mu * mu * mu;
    double kappa = 0.0, A = 0.0, term = 0.0;
    if (m2 > 1e-7 * r2) {
      kappa = m4 / (m2 * m2);
      double sgn = 1.0;
      if (kappa_target != 0.f) {
        const double dk = kappa - (double)kappa_target;
        sgn = (dk > 0.0) - (dk < 0.0);
        term = fabs(dk);
      } else {
        term = kappa;
      }
      A = sgn * 4.0 / (N * m2 * m2);
    } else if (kappa_target != 0.f) {
      term = fabs((double)kappa_target);
    }
    gstat[4 * batch] = mu; gstat[4 * batch + 1] = m3; gstat[4 * batch + 2] = kappa * m2; gstat[4 * batch + 3] = A;
    loss[batch] = (float)term;
    if (kappa_out) kappa_out[batch] = (float)kappa;
  }
}

// Stage 3: per token, the coefficients of the backward epilogue.  With c' = y - rho mu the gradient
// through the RMSNorm, (g - z (z.g)/d) / rho with g = A [c^3 - m3 - beta c], c = z - mu, is again
//   alpha' [ c'^3 - m3' - beta' c' ],  alpha' = A / rho^4,  beta' = (beta + tau) rho^2,
//   m3' = (m3 + tau mu) rho^3,  tau = (1/d) sum_j z [c^3 - m3 - beta c]  (from the row's sums of z^k),
// so the recompute GEMM and its epilogue are the per-row ones.  grid = (ceil(n/256), batch).
__global__ __launch_bounds__(256) void pooled_stage3_kernel(const floatx4* __restrict__ part, int P, int n, int d,
                                                            float rms_eps, const double* __restrict__ gstat,
                                                            floatx4* __restrict__ coef) {
  const int batch = blockIdx.y, token = blockIdx.x * 256 + threadIdx.x;
  if (token >= n) return;
  double Z[4], inv_rho;
  pooled_row_sums(part, P, n, batch, token, d, (double)rms_eps, inv_rho, Z);
  const double mu = gstat[4 * batch], m3 = gstat[4 * batch + 1], beta = gstat[4 * batch + 2], A = gstat[4 * batch + 3];
  floatx4 c = {0.f, 0.f, 0.f, 0.f};
  if (inv_rho > 0.0 && A != 0.0) {
    const double dd = (double)d, mu2 = mu * mu;
    const double C1 = Z[0] - dd * mu;
    const double C2 = Z[1] - 2.0 * mu * Z[0] + dd * mu2;
    const double C3 = Z[2] - 3.0 * mu * Z[1] + 3.0 * mu2 * Z[0] - dd * mu2 * mu;
    const double C4 = Z[3] - 4.0 * mu * Z[2] + 6.0 * mu2 * Z[1] - 4.0 * mu2 * mu * Z[0] + dd * mu2 * mu2;
    const double tau = (C4 + mu * C3 - m3 * Z[0] - beta * (C2 + mu * C1)) / dd;
    const double rho = 1.0 / inv_rho, i2 = inv_rho * inv_rho;
    c[0] = (float)(A * i2 * i2);
    c[1] = (float)(rho * mu);
    c[2] = (float)((beta + tau) * rho * rho);
    c[3] = (float)((m3 + tau * mu) * rho * rho * rho);
  }
  coef[(int64_t)batch * n + token] = c;
}

// loss[batch] = (sum of the block partials, fixed order) / n.  grid = batch blocks.
__global__ __launch_bounds__(256) void finalize_loss_kernel(const double* __restrict__ loss_part,
                                                            int nblocks, int n,
                                                            float* __restrict__ loss) {
  __shared__ double sh[256];
  const int batch = blockIdx.x;
  double v = 0.0;
  for (int i = threadIdx.x; i < nblocks; i += 256) v += loss_part[(int64_t)batch * nblocks + i];
  const double s = block_sum_256(v, sh);
  if (threadIdx.x == 0) loss[batch] = (float)(s / (double)n);
}

// out[i] = sum_s part[s*stride + i], s ascending.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ part,
                                                            int64_t stride, int splits,
                                                            float* __restrict__ out, int64_t count) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) {
    float v = part[i];
    for (int s = 1; s < splits; ++s) v += part[(int64_t)s * stride + i];
    out[i] = v;
  }
}

// fp32 value -> bf16 head and bf16 tail (x ~ hi + lo to about 2^-17 relative).
__device__ __forceinline__ void split_bf16(float x, __bf16& hi, __bf16& lo) {
  hi = (__bf16)x;
  lo = (__bf16)(x - (float)hi);
}

// Three-term bf16 emulation of an fp32 NT GEMM on the bf16 matrix cores:
//   A B^T ~ A_hi B_hi^T + A_hi B_lo^T + A_lo B_hi^T
// written as ONE bf16 GEMM with K tripled: the left operand is stored as [hi | hi | lo]
// (3*cols wide), the right operand as [hi | lo | hi].  `right` selects the layout.
// grid-stride over rows*cols elements; grid.z = batch.
__global__ __launch_bounds__(256) void split3_kernel(const float* __restrict__ in, int rows, int cols,
                                                     __bf16* __restrict__ out, int right) {
  const int64_t total = (int64_t)rows * cols;
  in += (int64_t)blockIdx.z * total;
  out += (int64_t)blockIdx.z * total * 3;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / cols, c = i - r * cols;
    __bf16 hi, lo;
    split_bf16(in[i], hi, lo);
    __bf16* o = out + r * 3 * cols + c;
    o[0] = hi;
    o[cols] = right ? lo : hi;
    o[2 * (int64_t)cols] = right ? hi : lo;
  }
}

// Cayley set-up: from M = dR R^T build  Bm = (lr/2)(M - M^T)  (exactly skew),
// Rt = R^T, Zt0 = Rt, U0 = 2 Rt (Bm and U0 either as fp32 or as split bf16 operands).  32 x 32 tiles; grid = (d/32, d/32, batch).
__global__ __launch_bounds__(256) void cayley_setup_kernel(const float* __restrict__ Mm,
                                                           const float* __restrict__ R, int d,
                                                           float half_lr, float* __restrict__ Bm,
                                                           float* __restrict__ Rt,
                                                           float* __restrict__ Zt,
                                                           float* __restrict__ U0,
                                                           __bf16* __restrict__ Bs,
                                                           __bf16* __restrict__ Us,
                                                           double* __restrict__ sq_part) {
  __shared__ float tm[32][33];
  __shared__ float tr[32][33];
  __shared__ double shsum[256];
  double sq = 0.0;
  const int64_t bo = (int64_t)blockIdx.z * d * d;
  const int i0 = blockIdx.x * 32, j0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  // load the mirrored tile (rows j0.., cols i0..) of M and of R
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int rr = ty + 8 * k;
    tm[rr][tx] = Mm[bo + (int64_t)(j0 + rr) * d + i0 + tx];
    tr[rr][tx] = R[bo + (int64_t)(j0 + rr) * d + i0 + tx];
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int rr = ty + 8 * k;  // row i0+rr, col j0+tx of the outputs
    const int64_t idx = bo + (int64_t)(i0 + rr) * d + j0 + tx;
    const float m_ij = Mm[idx];
    const float m_ji = tm[tx][rr];
    const float b = half_lr * (m_ij - m_ji);
    sq += (double)b * (double)b;
    const float rt = tr[tx][rr];  // R[j0+tx][i0+rr] = Rt[i0+rr][j0+tx]
    Rt[idx] = rt;
    Zt[idx] = rt;
    if (Bs) {  // split operands of the three-term bf16 GEMM: B as [hi|lo|hi], U as [hi|hi|lo]
      const int64_t so = 3 * bo + (int64_t)(i0 + rr) * 3 * d + j0 + tx;
      __bf16 hi, lo;
      split_bf16(b, hi, lo);
      Bs[so] = hi; Bs[so + d] = lo; Bs[so + 2 * d] = hi;
      split_bf16(2.f * rt, hi, lo);
      Us[so] = hi; Us[so + d] = hi; Us[so + 2 * d] = lo;
    } else {
      Bm[idx] = b;
      U0[idx] = 2.f * rt;
    }
  }
  if (sq_part) {  // per-tile sum of Bm^2 (uniform branch), added up in fixed order by the caller's kernel
    const double tot = block_sum_256(sq, shsum);
    if (threadIdx.x == 0)
      sq_part[((int64_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x] = tot;
  }
}

// ---- Cayley Adam: moments and step scalars (the optimiser the paper names; the update rule is
// that of the cited work on Stiefel-manifold optimisation) --------------------------------------
// M <- beta1 M + (1 - beta1) G in place; g2_part[batch][gridDim.x] = block partial sums of G^2.
__global__ __launch_bounds__(256) void adam_moment_kernel(float* __restrict__ M, const float* __restrict__ G,
                                                          int64_t dd, float beta1,
                                                          double* __restrict__ g2_part) {
  __shared__ double sh[256];
  const int64_t bo = (int64_t)blockIdx.y * dd;
  double s = 0.0;
  for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < dd / 4; q += (int64_t)gridDim.x * 256) {
    const floatx4 g = *reinterpret_cast<const floatx4*>(G + bo + 4 * q);
    floatx4 m = *reinterpret_cast<const floatx4*>(M + bo + 4 * q);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      m[e] = beta1 * m[e] + (1.f - beta1) * g[e];
      s += (double)g[e] * (double)g[e];
    }
    *reinterpret_cast<floatx4*>(M + bo + 4 * q) = m;
  }
  const double tot = block_sum_256(s, sh);
  if (threadIdx.x == 0) g2_part[(int64_t)blockIdx.y * gridDim.x + blockIdx.x] = tot;
}

// v <- beta2 v + (1 - beta2) ||G||_F^2;  scal[4b] = r = c1 sqrt(v / c2 + eps) with the bias
// corrections c1 = 1 - beta1^k, c2 = 1 - beta2^k taken by the host in double.  grid = batch.
__global__ __launch_bounds__(256) void adam_scalars1_kernel(const double* __restrict__ g2_part, int nblk,
                                                            float* __restrict__ v, float beta2, double c1,
                                                            double c2, float eps, float* __restrict__ scal) {
  __shared__ double sh[256];
  double s = 0.0;
  for (int i = threadIdx.x; i < nblk; i += 256) s += g2_part[(int64_t)blockIdx.x * nblk + i];
  const double g2 = block_sum_256(s, sh);
  if (threadIdx.x == 0) {
    const double v1 = (double)beta2 * (double)v[blockIdx.x] + (1.0 - (double)beta2) * g2;
    v[blockIdx.x] = (float)v1;
    scal[4 * blockIdx.x] = (float)(c1 * sqrt(v1 / c2 + (double)eps));
  }
}

// From the tile partials of ||S||_F^2 (S = (P - P^T)/2, W = S / r):
// scal[4b+1] = alpha = min(lr, 2 q / (||W|| + eps)), [4b+2] = ||W||_F, [4b+3] = alpha / (2 r), the factor of S
// in the fixed point Y = X - (alpha/2) W (X + Y).  grid = batch.
__global__ __launch_bounds__(256) void adam_scalars2_kernel(const double* __restrict__ sq_part, int ntile,
                                                            float lr, float q, float eps,
                                                            float* __restrict__ scal,
                                                            float* __restrict__ scalars_out) {
  __shared__ double sh[256];
  double s = 0.0;
  for (int i = threadIdx.x; i < ntile; i += 256) s += sq_part[(int64_t)blockIdx.x * ntile + i];
  const double s2 = block_sum_256(s, sh);
  if (threadIdx.x == 0) {
    const float r = scal[4 * blockIdx.x];
    const float wn = (float)(sqrt(s2) / (double)r);
    const float alpha = fminf(lr, 2.f * q / (wn + eps));
    scal[4 * blockIdx.x + 1] = alpha;
    scal[4 * blockIdx.x + 2] = wn;
    scal[4 * blockIdx.x + 3] = alpha / (2.f * r);
    if (scalars_out) {
      scalars_out[3 * blockIdx.x] = r;
      scalars_out[3 * blockIdx.x + 1] = alpha;
      scalars_out[3 * blockIdx.x + 2] = wn;
    }
  }
}

// One fixed-point update from the GEMM product C = U B^T (three-term bf16 path):
//   Zt_new = Rt - C;  delta[it] = max |Zt_new - Zt|;  U_next = Rt + Zt_new as [hi|hi|lo].
// Four consecutive elements per thread (16-byte loads); grid-stride; grid.y = batch.
// Returns at once (handing the delta on) when an earlier iteration has converged.
__global__ __launch_bounds__(256) void cayley_update_kernel(const float* __restrict__ C,
                                                            const float* __restrict__ Rt,
                                                            float* __restrict__ Zt,
                                                            __bf16* __restrict__ Us, int d,
                                                            unsigned* __restrict__ delta, int it,
                                                            int max_iters, float tol,
                                                            const float* __restrict__ bscale) {
  __shared__ unsigned sh[4];
  unsigned* dl = delta + (int64_t)blockIdx.y * max_iters;
  if (it > 0 && cayley_converged(dl, it - 1, tol)) {
    if (blockIdx.x == 0 && threadIdx.x == 0) dl[it] = 0u;  // a zero change: later launches return too
    return;
  }
  const int64_t dd = (int64_t)d * d, bo = (int64_t)blockIdx.y * dd;
  const float bs = bscale ? bscale[4 * blockIdx.y + 3] : 1.f;  // Cayley Adam: factor of S
  unsigned dmax = 0u;
  for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < dd / 4; q += (int64_t)gridDim.x * 256) {
    const int64_t i = q * 4;
    const int64_t m = i / d, n = i - m * d;
    const floatx4 c = *reinterpret_cast<const floatx4*>(C + bo + i);
    const floatx4 rt = *reinterpret_cast<const floatx4*>(Rt + bo + i);
    const floatx4 zo = *reinterpret_cast<const floatx4*>(Zt + bo + i);
    floatx4 z;
    __bf16 hi[4], lo[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      z[e] = rt[e] - bs * c[e];
      dmax = umax(dmax, abs_bits(z[e] - zo[e]));
      split_bf16(rt[e] + z[e], hi[e], lo[e]);
    }
    *reinterpret_cast<floatx4*>(Zt + bo + i) = z;
    __bf16* o = Us + 3 * bo + m * 3 * d + n;
    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
    const bf16x4 vh = {hi[0], hi[1], hi[2], hi[3]}, vl = {lo[0], lo[1], lo[2], lo[3]};
    *reinterpret_cast<bf16x4*>(o) = vh;
    *reinterpret_cast<bf16x4*>(o + d) = vh;
    *reinterpret_cast<bf16x4*>(o + 2 * (int64_t)d) = vl;
  }
  dmax = wave_umax(dmax);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = dmax;
  __syncthreads();
  if (threadIdx.x == 0) atomicMax(&dl[it], umax(umax(sh[0], sh[1]), umax(sh[2], sh[3])));
}

// Cayley wrap-up: R = Zt^T (and its bf16 copy), info = iterations used or -1.  An iteration that did
// not converge is rejected as a whole: R stays as it is and the bf16 copy is taken from it.
__global__ __launch_bounds__(256) void cayley_finish_kernel(const float* __restrict__ Zt, int d,
                                                            float* __restrict__ R,
                                                            __bf16* __restrict__ R_lowp,
                                                            const unsigned* __restrict__ delta,
                                                            int max_iters, float tol,
                                                            int32_t* __restrict__ info) {
  __shared__ float tz[32][33];
  const int64_t bo = (int64_t)blockIdx.z * d * d;
  const int i0 = blockIdx.x * 32, j0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  int used = -1;  // the same scan in every thread: at most max_iters words, all cache hits
  for (int k = 0; k < max_iters; ++k) {
    if (cayley_converged(delta + (int64_t)blockIdx.z * max_iters, k, tol)) { used = k + 1; break; }
  }
  if (used > 0) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int rr = ty + 8 * k;
      tz[rr][tx] = Zt[bo + (int64_t)(j0 + rr) * d + i0 + tx];
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int rr = ty + 8 * k;
    const int64_t idx = bo + (int64_t)(i0 + rr) * d + j0 + tx;
    if (used > 0) {
      const float v = tz[tx][rr];
      R[idx] = v;
      if (R_lowp) R_lowp[idx] = (__bf16)v;
    } else if (R_lowp) {
      R_lowp[idx] = (__bf16)R[idx];
    }
  }
  if (info && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) info[blockIdx.z] = used;
}

// Diagonal of Zt Zt^T - I: | sum_k Zt[m][k]^2 - 1 | summed in fp64, folded into err[batch]
// (bit pattern of a non-negative float) by atomicMax.  grid = (d, batch).
__global__ __launch_bounds__(256) void ortho_diag_kernel(const float* __restrict__ Zt, int d,
                                                         unsigned* __restrict__ err) {
  __shared__ double sh[256];
  const float* row = Zt + ((int64_t)blockIdx.y * d + blockIdx.x) * d;
  double s = 0.0;
  for (int k = threadIdx.x; k < d; k += 256) s += (double)row[k] * (double)row[k];
  s = block_sum_256(s, sh);
  if (threadIdx.x == 0) atomicMax(&err[blockIdx.y], abs_bits((float)(s - 1.0)));
}

// Fake-quant scales: amax over the P partials, s = (clip * amax) / 7 in fp32.
__global__ __launch_bounds__(256) void quant_scale_kernel(const float* __restrict__ part, int P,
                                                          int64_t n_total_per_batch, float clip,
                                                          float* __restrict__ scales_ws,
                                                          float* __restrict__ scales_out) {
  const int batch = blockIdx.y;
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= n_total_per_batch) return;
  float a = 0.f;
  for (int p = 0; p < P; ++p) a = fmaxf(a, part[((int64_t)batch * P + p) * n_total_per_batch + t]);
  const float s = __fdiv_rn(__fmul_rn(clip, a), 7.0f);
  scales_ws[batch * n_total_per_batch + t] = s;
  if (scales_out) scales_out[batch * n_total_per_batch + t] = s;
}

// err[token] = sum over the PN partial pairs, fixed order.
__global__ __launch_bounds__(256) void quant_err_kernel(const float2* __restrict__ part, int PN,
                                                        int64_t n, float2* __restrict__ err) {
  const int batch = blockIdx.y;
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= n) return;
  float e = 0.f, y = 0.f;
  for (int p = 0; p < PN; ++p) {
    const float2 v = part[((int64_t)batch * PN + p) * n + t];
    e += v.x;
    y += v.y;
  }
  err[batch * n + t] = make_float2(e, y);
}

// Fake-quant of token rows of a materialised fp32 Y ([rows][d], contiguous): one wave per row, no
// workgroup barrier.  The row is read once (KEEP: it stays in CH float4 registers per lane, d <= 256 CH)
// or twice (the second read comes out of the caches); amax, s = (clip amax)/7, one reciprocal per row,
// q = clamp(rint(y * (1/s)), -7, 7), four codes per 4-byte store, {sum (y - q s)^2, sum y^2}.
// scales_out / codes / err are indexed from the first row of this launch; any of them may be null.
template <int CH, bool KEEP>
__global__ __launch_bounds__(256) void quant_rows_kernel(const float* __restrict__ Y, int64_t rows, int d,
                                                         float clip, float* __restrict__ scales_out,
                                                         int8_t* __restrict__ codes, float2* __restrict__ err) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const float4* y4 = reinterpret_cast<const float4*>(Y + row * d) + lane;
  const int nch = (d + 255) >> 8;  // chunks of 256 values; d % 128 == 0: the last one may be half
  const int last_lanes = (d & 255) ? 32 : 64;
  float4 v[KEEP ? CH : 1];
  float a = 0.f;
  if (KEEP) {
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      v[c] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (c < nch && (c + 1 < nch || lane < last_lanes)) v[c] = y4[c * 64];
      a = fmaxf(fmaxf(a, fmaxf(fabsf(v[c].x), fabsf(v[c].y))), fmaxf(fabsf(v[c].z), fabsf(v[c].w)));
    }
  } else {
    for (int c = 0; c < nch; ++c)
      if (c + 1 < nch || lane < last_lanes) {
        const float4 t = y4[c * 64];
        a = fmaxf(fmaxf(a, fmaxf(fabsf(t.x), fabsf(t.y))), fmaxf(fabsf(t.z), fabsf(t.w)));
      }
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) a = fmaxf(a, __shfl_xor(a, o));
  const float s = __fdiv_rn(__fmul_rn(clip, a), 7.0f);
  const bool live = s > 0.f;
  const float rinv = live ? __fdiv_rn(1.0f, s) : 0.f;
  float e2 = 0.f, y2 = 0.f;
  unsigned* crow = codes ? reinterpret_cast<unsigned*>(codes + row * d) + lane : nullptr;
  auto quantise = [&](const float4& t, int c) {
    const float y[4] = {t.x, t.y, t.z, t.w};
    unsigned pack = 0u;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float q = rintf(__fmul_rn(y[e], rinv));
      q = fminf(fmaxf(q, -7.f), 7.f);
      if (!live) q = 0.f;
      const float diff = y[e] - q * s;
      e2 = fmaf(diff, diff, e2);
      y2 = fmaf(y[e], y[e], y2);
      pack |= ((unsigned)(int)q & 0xffu) << (8 * e);
    }
    if (crow) crow[c * 64] = pack;
  };
  if (KEEP) {
#pragma unroll
    for (int c = 0; c < CH; ++c)
      if (c < nch && (c + 1 < nch || lane < last_lanes)) quantise(v[c], c);
  } else {
    for (int c = 0; c < nch; ++c)
      if (c + 1 < nch || lane < last_lanes) quantise(y4[c * 64], c);
  }
  if (err) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      e2 += __shfl_xor(e2, o);
      y2 += __shfl_xor(y2, o);
    }
  }
  if (lane == 0) {
    if (scales_out) scales_out[row] = s;
    if (err) err[row] = make_float2(e2, y2);
  }
}

// ---- per-token quantisation-quality figures of a materialised Y = X R ----------------------
// (max-value "success" of "Evaluation ... on Channel Outliers"; Setup: symmetric per-token
// quantisation clipped at a quantile, asymmetric quantisation for KV caches; Background:
// "Uniform Quantization for k-bit Precision".)  One workgroup per token row, the row in LDS.
// Every rounding-critical step is a single IEEE fp32 operation, as in the symmetric fake-quant.
__device__ __forceinline__ float block_fmax_256(float v, float* red4) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red4[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(red4[0], red4[1]), fmaxf(red4[2], red4[3]));
}
// Sum over the 256 threads in a fixed order (xor butterfly inside each wave, then the four wave
// sums left to right): two barriers instead of the nine of the LDS tree.
__device__ __forceinline__ double block_dsum_fast_256(double v, double* red4) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red4[threadIdx.x >> 6] = v;
  __syncthreads();
  return ((red4[0] + red4[1]) + red4[2]) + red4[3];
}
__device__ __forceinline__ unsigned block_umin_256(unsigned v, unsigned* red4) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const unsigned w = (unsigned)__shfl_xor((int)v, o);
    v = w < v ? w : v;
  }
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red4[threadIdx.x >> 6] = v;
  __syncthreads();
  const unsigned a = red4[0] < red4[1] ? red4[0] : red4[1], b = red4[2] < red4[3] ? red4[2] : red4[3];
  return a < b ? a : b;
}

// One WAVE per token row, the row in registers (NV4 float4 per lane: d <= 256 NV4; FULL: d = 256 NV4, no
// bounds tests), no workgroup barrier: the four waves of a workgroup work on four rows independently, all
// loads of a row are in flight at once, and the reductions are wave shuffles.  The quantile needs two order
// statistics of |y|: a radix select on the bit patterns (integer work, bit-exact) in three rounds of 11, 11
// and 9 bits, each a histogram of up to 2048 bins that the wave keeps in LDS (one LDS atomic per value that
// still matches the bits decided so far; in the later rounds whole 256-value pieces are skipped).
// grid = (row workgroups, batch); a wave walks several rows.  Y [batch][n][d] fp32.
// Error sums: the difference y - q s as one fused multiply-add in fp32 (exact before its single rounding),
// squares summed four at a time in fp32 and then in fp64; the asymmetric difference, whose terms cancel
// from the size of the row's range, in fp64 throughout.
// (second launch bound: waves per SIMD the register allocation must leave room for, so that the loads of
// several rows are in flight per SIMD; the row itself takes 4 NV4 registers)
template <typename TX, int NV4, bool FULL>
__global__ __launch_bounds__(256, (NV4 <= 4 ? 4 : NV4 <= 16 ? 3 : 2)) void quant_metrics_row_kernel(const float* __restrict__ Y,
                                                                const TX* __restrict__ X, int64_t ldx,
                                                                int64_t x_batch_stride, int n, int d,
                                                                double quant, float* __restrict__ amax_out,
                                                                float* __restrict__ thr_out,
                                                                float* __restrict__ err_sym,
                                                                float* __restrict__ err_asym,
                                                                unsigned long long* __restrict__ success) {
  __shared__ __align__(16) unsigned hist_all[4][2048];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, batch = blockIdx.y;
  unsigned* hist = hist_all[wave];
  unsigned wins = 0u;  // rows of this wave whose largest magnitude shrank: one atomic per wave, not per row
  constexpr int EPC = 16 / (int)sizeof(TX);             // elements of X per 16 bytes
  constexpr int NXV = (NV4 * (int)sizeof(TX) + 3) / 4;  // 16-byte pieces of the X row per lane: d <= 64 NXV EPC
  typedef TX vecx __attribute__((ext_vector_type(16 / sizeof(TX))));
  // piece c of a row holds values 256 c + 4 lane .. + 3; d is a multiple of 128, so the last piece may be half full
  auto live = [&](int c) __attribute__((always_inline)) { return FULL || 256 * c + 4 * lane < d; };
  // every 16-byte load of a row (Y and X) is requested at once; nothing here waits for them
  auto load_row = [&](float4 (&v)[NV4], vecx (&xv)[NXV], int token) __attribute__((always_inline)) {
    const float4* y4 = reinterpret_cast<const float4*>(Y + ((int64_t)batch * n + token) * d);
    const TX* x = X + (int64_t)batch * x_batch_stride + (int64_t)token * ldx;
#pragma unroll
    for (int c = 0; c < NV4; ++c) {
      v[c] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (live(c)) v[c] = y4[c * 64 + lane];
    }
#pragma unroll
    for (int c = 0; c < NXV; ++c) {
      const int j = (c * 64 + lane) * EPC;
      if (FULL || j < d) xv[c] = *reinterpret_cast<const vecx*>(x + j);
      else {
#pragma unroll
        for (int e = 0; e < EPC; ++e) xv[c][e] = (TX)0.0f;
      }
    }
  };
  // a wave walks rows token, token + 4 gridDim.x, ...; whole waves leave the loop, nothing synchronises across waves
  const int stride = 4 * (int)gridDim.x;
  float4 v[NV4];
  vecx xv[NXV];
#pragma unroll 1
  for (int token = blockIdx.x * 4 + wave; token < n; token += stride) {
  load_row(v, xv, token);
  float ab = 0.f;  // largest magnitude of the unrotated row
#pragma unroll
  for (int c = 0; c < NXV; ++c)
#pragma unroll
    for (int e = 0; e < EPC; ++e) ab = fmaxf(ab, fabsf((float)xv[c][e]));
  float ar = 0.f, mn = 3.0e38f, mx = -3.0e38f;
  double y2 = 0.0;
#pragma unroll
  for (int c = 0; c < NV4; ++c) {
    if (live(c)) {
      const float e4[4] = {v[c].x, v[c].y, v[c].z, v[c].w};
      float y24 = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        ar = fmaxf(ar, fabsf(e4[e]));
        mn = fminf(mn, e4[e]);
        mx = fmaxf(mx, e4[e]);
        y24 = fmaf(e4[e], e4[e], y24);
      }
      y2 += (double)y24;
    }
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    ab = fmaxf(ab, __shfl_xor(ab, o));
    ar = fmaxf(ar, __shfl_xor(ar, o));
    mn = fminf(mn, __shfl_xor(mn, o));
    mx = fmaxf(mx, __shfl_xor(mx, o));
    y2 += __shfl_xor(y2, o);
  }

  float t = ar;
  if (quant < 1.0) {
    const double pos = quant * (double)(d - 1);
    const int k = (int)floor(pos);
    const float frac = (float)(pos - (double)k);
    // a_k = the value of rank k (0-based, ascending) among the |y| bit patterns: radix select in three rounds
    // on bits 30..20, 19..9 and 8..0, each a histogram of up to 2048 bins kept by this wave in LDS.
    auto clear_hist = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int j = 0; j < 8; ++j) *reinterpret_cast<uint4*>(hist + 256 * j + 4 * lane) = make_uint4(0u, 0u, 0u, 0u);
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
    };
    // The bin that holds rank kk: lane l sums bins 32 l .. 32 l + 31 (its eight 16-byte pieces read in an order
    // that depends on the lane number, which spreads them over the banks), a scan over the lanes finds the group,
    // then lane i < 32 takes bin i of that group and a second scan finds the bin.
    // -> bin, cum = entries in lower bins, cnt = entries in the bin; own / c2 / grp / idx stay for next_bin.
    unsigned own = 0u, c2 = 0u;
    int grp = 0, idx = 0;
    auto pick = [&](unsigned kk, unsigned& bin, unsigned& cum, unsigned& cnt) __attribute__((always_inline)) {
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
      own = 0u;
      unsigned hb = (unsigned)lane * 128u + (unsigned)(lane & 7) * 16u;  // byte offset of piece (lane & 7) of this lane
      asm volatile("" : "+v"(hb));  // recomputed here: eight piece addresses kept across the row cost registers
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const uint4 c = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(hist) + (hb ^ (unsigned)(j << 4)));
        own += (c.x + c.y) + (c.z + c.w);
      }
      unsigned incl = own;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const unsigned up = (unsigned)__shfl_up((int)incl, o);
        if (lane >= o) incl += up;
      }
      const unsigned excl = incl - own;
      const unsigned long long hits = __ballot(excl <= kk && kk < incl);  // exactly one lane: the counts sum to > kk
      grp = hits ? __builtin_ctzll(hits) : 0;
      const unsigned base = (unsigned)__shfl((int)excl, grp);
      c2 = lane < 32 ? hist[32 * grp + lane] : 0u;
      unsigned incl2 = c2;
#pragma unroll
      for (int o = 1; o < 32; o <<= 1) {
        const unsigned up = (unsigned)__shfl_up((int)incl2, o);
        if (lane >= o) incl2 += up;
      }
      const unsigned excl2 = base + incl2 - c2;
      const unsigned long long hits2 = __ballot(lane < 32 && excl2 <= kk && kk < excl2 + c2);
      idx = hits2 ? __builtin_ctzll(hits2) : 0;
      bin = (unsigned)(32 * grp + idx);
      cum = (unsigned)__shfl((int)excl2, idx);
      cnt = (unsigned)__shfl((int)c2, idx);
      __builtin_amdgcn_wave_barrier();
    };
    // first non-empty bin above the one pick() returned, 0xffffffff if there is none
    auto next_bin = [&]() __attribute__((always_inline)) -> unsigned {
      const unsigned long long nz = __ballot(lane < 32 && c2 > 0u) & ~((2ull << idx) - 1ull);
      if (nz) return (unsigned)(32 * grp + __builtin_ctzll(nz));
      const unsigned long long g = __ballot(own > 0u) & ~((2ull << grp) - 1ull);
      if (!g) return 0xffffffffu;
      const int g0 = __builtin_ctzll(g);
      const unsigned c3 = lane < 32 ? hist[32 * g0 + lane] : 0u;
      const unsigned long long nz3 = __ballot(c3 > 0u);
      return (unsigned)(32 * g0 + __builtin_ctzll(nz3));
    };
    unsigned kk = (unsigned)k, bin, cum, cnt;
    // first digit, bits 30..20: every value of the row counts
    clear_hist();
#pragma unroll
    for (int c = 0; c < NV4; ++c) {
      if (live(c)) {
        const float e4[4] = {v[c].x, v[c].y, v[c].z, v[c].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) atomicAdd(&hist[(__float_as_uint(e4[e]) & 0x7fffffffu) >> 20], 1u);
      }
    }
    pick(kk, bin, cum, cnt);
    const unsigned p11 = bin;
    kk -= cum;
    // second digit, bits 19..9 of the values whose bits 30..20 equal p11
    clear_hist();
#pragma unroll
    for (int c = 0; c < NV4; ++c) {
      const float e4[4] = {v[c].x, v[c].y, v[c].z, v[c].w};
      unsigned u[4];
      bool m[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        u[e] = __float_as_uint(e4[e]) & 0x7fffffffu;
        m[e] = live(c) && (u[e] >> 20) == p11;
      }
      if (!__any((int)(m[0] | m[1] | m[2] | m[3]))) continue;  // skipped by the whole wave
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (m[e]) atomicAdd(&hist[(u[e] >> 9) & 2047u], 1u);
    }
    pick(kk, bin, cum, cnt);
    const unsigned p22 = (p11 << 11) | bin;
    kk -= cum;
    // third digit, bits 8..0 of the values whose bits 30..9 equal p22; the same pass finds the smallest value
    // beyond that group: u - base wraps to >= 2^31 for every u < base = (p22 + 1) 2^9 <= 2^31
    clear_hist();
    const unsigned base = (p22 + 1u) << 9;
    unsigned above = 0xffffffffu;
#pragma unroll
    for (int c = 0; c < NV4; ++c) {
      const float e4[4] = {v[c].x, v[c].y, v[c].z, v[c].w};
      unsigned u[4];
      bool m[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        u[e] = __float_as_uint(e4[e]) & 0x7fffffffu;
        m[e] = live(c) && (u[e] >> 9) == p22;
        const unsigned w = u[e] - base;
        above = w < above ? w : above;
      }
      if (!__any((int)(m[0] | m[1] | m[2] | m[3]))) continue;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (m[e]) atomicAdd(&hist[u[e] & 511u], 1u);
    }
    pick(kk, bin, cum, cnt);
    kk -= cum;  // rank of a_k among its cnt copies
    const unsigned prefix = (p22 << 9) | bin;
    // a_{k+1} = a_k if another copy of it follows, else the smallest larger value: the next occupied bin of
    // the last histogram, else the smallest value beyond the group
    unsigned nxt = next_bin();
    if (nxt != 0xffffffffu) nxt |= p22 << 9;
    else {
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) {
        const unsigned w = (unsigned)__shfl_xor((int)above, o);
        above = w < above ? w : above;
      }
      if (above < 0x80000000u) nxt = above + base;
    }
    const float ak = __uint_as_float(prefix);
    const float ak1 = (cnt >= kk + 2u || nxt == 0xffffffffu) ? ak : __uint_as_float(nxt);
    float inc = __fmul_rn(frac, __fsub_rn(ak1, ak));
    asm volatile("" : "+v"(inc));  // keep the product rounded: no contraction with the add below
    t = __fadd_rn(ak, inc);
  }
  const float ss = __fdiv_rn(t, 7.0f);
  const float rs = ss > 0.f ? __fdiv_rn(1.0f, ss) : 0.f;
  const float sa = __fdiv_rn(__fsub_rn(mx, mn), 15.0f);
  const float ra = sa > 0.f ? __fdiv_rn(1.0f, sa) : 0.f;
  const double sad = (double)sa, mnd = (double)mn;
  double es = 0.0, ea = 0.0;
#pragma unroll
  for (int c = 0; c < NV4; ++c) {
    if (live(c)) {
      const float e4[4] = {v[c].x, v[c].y, v[c].z, v[c].w};
      float es4 = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float val = e4[e];
        float q = rintf(__fmul_rn(val, rs));
        q = __builtin_amdgcn_fmed3f(q, -7.f, 7.f);
        const float dsym = fmaf(-q, ss, val);
        es4 = fmaf(dsym, dsym, es4);
        float qa = rintf(__fmul_rn(__fsub_rn(val, mn), ra));
        qa = __builtin_amdgcn_fmed3f(qa, 0.f, 15.f);
        const double dasy = (double)val - fma((double)qa, sad, mnd);
        ea = fma(dasy, dasy, ea);
      }
      es += (double)es4;
    }
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    es += __shfl_xor(es, o);
    ea += __shfl_xor(ea, o);
  }
  if (lane == 0) {
    const int64_t o = (int64_t)batch * n + token;
    if (amax_out) { amax_out[2 * o] = ab; amax_out[2 * o + 1] = ar; }
    if (thr_out) thr_out[o] = t;
    if (err_sym) { err_sym[2 * o] = (float)es; err_sym[2 * o + 1] = (float)y2; }
    if (err_asym) { err_asym[2 * o] = (float)ea; err_asym[2 * o + 1] = (float)y2; }
    if (ar < ab) wins += 1u;
  }
  }
  if (lane == 0 && success && wins) atomicAdd(&success[batch], (unsigned long long)wins);
}

// Plain fp32 matrix transpose out[c][r] = in[r][c] (rows x cols -> cols x rows), 32 x 32 tiles
// through LDS; grid = (ceil(cols/32), ceil(rows/32)).
__global__ __launch_bounds__(256) void transpose_f32_kernel(const float* __restrict__ in, int64_t ld_in,
                                                            float* __restrict__ out, int64_t ld_out,
                                                            int rows, int cols) {
  __shared__ float tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int r = r0 + ty + 8 * k, c = c0 + tx;
    tile[ty + 8 * k][tx] = (r < rows && c < cols) ? in[(int64_t)r * ld_in + c] : 0.f;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int c = c0 + ty + 8 * k, r = r0 + tx;
    if (c < cols && r < rows) out[(int64_t)c * ld_out + r] = tile[tx][ty + 8 * k];
  }
}

// ---- quantisation sensitivity (Background: Definition "Quantization Sensitivity", Eq. 1) ----
// Device state of the search: st[0..31] candidate steps, st[32] = lo, st[33] = hi, st[34] = best step,
// st[35] = amax; best MSE in dst[0] (fp64), sentinel -1 before the first round.
// |y| maximum of a flat fp32 array; grid-stride; bit pattern max (order independent).
__global__ __launch_bounds__(256) void sens_amax_kernel(const float* __restrict__ y, int64_t count,
                                                        unsigned* __restrict__ amax_bits) {
  __shared__ unsigned red[4];
  unsigned m = 0u;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256)
    m = umax(m, abs_bits(y[i]));
  m = wave_umax(m);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) atomicMax(amax_bits, umax(umax(red[0], red[1]), umax(red[2], red[3])));
}

// Sum of squared errors of NS candidate steps in one pass over y: part[block][NS] (fp64).
// q = clamp(rint(y (1/s)), -L, L) in fp32, error in fp32 per element, fp64 across elements of a thread
// every 64 elements and across the block.
constexpr int kSensSteps = 32;
// grid = (blocks, kSensSteps / kSensPerBlock): a workgroup evaluates kSensPerBlock of the candidates, which keeps
// it under 128 registers (four waves per SIMD: a single wave issues a vector instruction only every ~5 cycles).
constexpr int kSensPerBlock = 16;
__global__ __launch_bounds__(256) void sens_sweep_kernel(const float* __restrict__ y, int64_t count,
                                                         const float* __restrict__ steps, int ns, float L,
                                                         double* __restrict__ part) {
  __shared__ double sh[4];
  const int j0 = blockIdx.y * kSensPerBlock;
  // candidate steps and reciprocals in registers; fp32 partial sums over 64 elements, then fp64
  float cs[kSensPerBlock], cr[kSensPerBlock];
#pragma unroll
  for (int j = 0; j < kSensPerBlock; ++j) {
    const float s = j0 + j < ns ? steps[j0 + j] : 0.f;
    cs[j] = s;
    cr[j] = s > 0.f ? __fdiv_rn(1.0f, s) : 0.f;
  }
  double acc[kSensPerBlock];
#pragma unroll
  for (int j = 0; j < kSensPerBlock; ++j) acc[j] = 0.0;
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t base = (int64_t)blockIdx.x * 256 + threadIdx.x; base < count; base += 64 * stride) {
    float facc[kSensPerBlock];
#pragma unroll
    for (int j = 0; j < kSensPerBlock; ++j) facc[j] = 0.f;
    const int64_t left = (count - base + stride - 1) / stride;  // elements of this thread from base on
    const int trips = left < 64 ? (int)left : 64;
    const float* yp = y + base;
    float vnext = *yp;  // the next element is requested before the candidates of this one are evaluated
#pragma unroll 1
    for (int k = 0; k < trips; ++k) {
      const float v = vnext;
      yp += stride;
      if (k + 1 < trips) vnext = *yp;
#pragma unroll
      for (int j = 0; j < kSensPerBlock; ++j) {
        float q = rintf(__fmul_rn(v, cr[j]));
        q = __builtin_amdgcn_fmed3f(q, -L, L);  // clamp in one instruction (q is finite)
        const float dlt = v - q * cs[j];
        facc[j] = fmaf(dlt, dlt, facc[j]);
      }
    }
#pragma unroll
    for (int j = 0; j < kSensPerBlock; ++j) acc[j] += (double)facc[j];
  }
#pragma unroll
  for (int j = 0; j < kSensPerBlock; ++j) {
    if (j0 + j < ns) {  // uniform
      const double t = block_dsum_fast_256(acc[j], sh);
      if (threadIdx.x == 0) part[(int64_t)blockIdx.x * kSensSteps + j0 + j] = t;
    }
  }
}

// One block: add the block partials in fixed order, pick the best candidate, write the next grid.
// stage 0..2 as in the search; stage 3: the steps were {best, best (1 + alpha_i)}: write the outputs.
__global__ __launch_bounds__(256) void sens_select_kernel(const double* __restrict__ part, int nblocks, int ns,
                                                          int64_t count, int round, float L, float* __restrict__ st,
                                                          double* __restrict__ dst, const float* __restrict__ alphas,
                                                          int n_alpha, float* __restrict__ out,
                                                          float* __restrict__ gamma) {
  __shared__ double sh[4];
  __shared__ double mse[kSensSteps];
  if (round >= 0) {
    for (int j = 0; j < ns; ++j) {
      double v = 0.0;
      for (int i = threadIdx.x; i < nblocks; i += 256) v += part[(int64_t)i * kSensSteps + j];
      const double t = block_dsum_fast_256(v, sh);
      if (threadIdx.x == 0) mse[j] = t / (double)count;
    }
    __syncthreads();
  }
  if (threadIdx.x != 0) return;
  const float c4[4] = {1.0f, 0.840896415f, 0.707106781f, 0.594603558f};  // 2^(-k/4)
  if (round < 0) {  // first grid: smax 2^(-j/4)
    const float smax = __fdiv_rn(st[35], L);
    for (int j = 0; j < 32; ++j) st[j] = __fmul_rn(smax, ldexpf(c4[j & 3], -(j >> 2)));
    st[32] = st[33] = st[34] = smax;
    dst[0] = -1.0;
    return;
  }
  if (round == 3) {
    out[0] = st[34];
    out[1] = (float)dst[0];
    for (int i = 0; i < n_alpha; ++i) gamma[i] = (float)fabs(mse[i + 1] - mse[0]);
    return;
  }
  int arg = 0;
  for (int j = 1; j < 32; ++j) if (mse[j] < mse[arg]) arg = j;
  float lo = st[32], hi = st[33], best_s = st[34];
  float nlo, nhi;
  if (round == 0) {
    nlo = st[arg + 1 < 32 ? arg + 1 : arg];
    nhi = st[arg > 0 ? arg - 1 : arg];
  } else {
    nlo = arg > 0 ? st[arg - 1] : lo;
    nhi = arg + 1 < 32 ? st[arg + 1] : hi;
  }
  if (dst[0] < 0.0 || mse[arg] < dst[0]) {
    dst[0] = mse[arg]; best_s = st[arg]; lo = nlo; hi = nhi;
  } else {
    const float q1 = __fsub_rn(best_s, lo), q2 = __fsub_rn(hi, best_s);
    float p1 = __fmul_rn(0.25f, q1), p2 = __fmul_rn(0.25f, q2);
    asm volatile("" : "+v"(p1), "+v"(p2));  // keep the products rounded (no contraction)
    lo = __fsub_rn(best_s, p1);
    hi = __fadd_rn(best_s, p2);
  }
  st[32] = lo; st[33] = hi; st[34] = best_s;
  if (round < 2) {
    const float span = __fsub_rn(hi, lo);
    for (int j = 0; j < 32; ++j) {
      float inc = __fmul_rn(span, __fdiv_rn((float)(j + 1), 33.0f));
      asm volatile("" : "+v"(inc));
      st[j] = __fadd_rn(lo, inc);
    }
  } else {  // last: the best step and its perturbed copies
    st[0] = best_s;
    for (int i = 0; i < n_alpha; ++i) st[i + 1] = __fmul_rn(best_s, __fadd_rn(1.0f, alphas[i]));
  }
}

}  // namespace kt
