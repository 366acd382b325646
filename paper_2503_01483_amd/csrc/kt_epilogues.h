// kt_epilogues.h -- what each GEMM on the path does with its accumulator tile.
//
// Every functor is called as epi(acc, batch, tm, tn, ks, m0, n0) once the main
// loop is done; `skip(batch)` lets a launch return early (used by the Cayley
// fixed-point iteration once it has converged).
#pragma once
#include "kt_gemm.h"

namespace kt {

template <typename T>
__device__ __forceinline__ T from_float(float v);
template <>
__device__ __forceinline__ float from_float<float>(float v) { return v; }
template <>
__device__ __forceinline__ __bf16 from_float<__bf16>(float v) { return (__bf16)v; }

struct EpiBase {
  __device__ __forceinline__ bool skip(int) const { return false; }
};

// ---- forward pass: per-token moments of y over the hidden dimension ---------------
// m = output feature (reduced in registers), n = token (one per lane).
// part[(batch*P + p)*n_tokens + token] = {mean_p, sum c^2, sum c^3, sum c^4}, c = y - mean_p, over
// the WTM features wave-row p = tm*WGM + wm owns: the mean first, then sums about it (two passes
// over the registers), so that a row whose mean is large against its spread loses nothing to
// cancellation in fp32; the partials of a row are merged in fp64 (row_central_sums in kt_aux.h).
template <class TL>
struct EpiMoments : EpiBase {
  floatx4* part;
  int n_tokens, d, P;
  __device__ __forceinline__ void operator()(floatx16 (&acc)[TL::MB][TL::NB], int batch, int tm,
                                             int, int, int m0, int n0) const {
    const Frag<TL> f;
    const int p = tm * TL::WGM + f.wm;
    int blocks = 0;
#pragma unroll
    for (int mb = 0; mb < TL::MB; ++mb) blocks += (m0 + f.m_block(mb) < d) ? 1 : 0;
    const float inv_cnt = blocks > 0 ? 1.0f / (float)(32 * blocks) : 0.f;
#pragma unroll
    for (int nb = 0; nb < TL::NB; ++nb) {
      float s1 = 0.f;
#pragma unroll
      for (int mb = 0; mb < TL::MB; ++mb) {
        if (m0 + f.m_block(mb) < d) {
#pragma unroll
          for (int r = 0; r < 16; ++r) s1 += acc[mb][nb][r];
        }
      }
      s1 += __shfl_xor(s1, 32);
      const float mean = s1 * inv_cnt;
      float s2 = 0.f, s3 = 0.f, s4 = 0.f;
#pragma unroll
      for (int mb = 0; mb < TL::MB; ++mb) {
        if (m0 + f.m_block(mb) < d) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float c = acc[mb][nb][r] - mean;
            const float c2 = c * c;
            s2 += c2;
            s3 = fmaf(c2, c, s3);
            s4 = fmaf(c2, c2, s4);
          }
        }
      }
      s2 += __shfl_xor(s2, 32);
      s3 += __shfl_xor(s3, 32);
      s4 += __shfl_xor(s4, 32);
      const int token = n0 + f.n_of(nb);
      if (f.half == 0 && token < n_tokens) {
        floatx4 v = {mean, s2, s3, s4};
        part[((int64_t)batch * P + p) * n_tokens + token] = v;
      }
    }
  }
};

// ---- backward pass: recomputed y -> dL/dy, stored token-minor ---------------------
// coef[token] = {alpha, mu, beta, m3};  g = alpha * (c (c^2 - beta) - m3), c = y - mu.
//
// Layout of GT (and of the token-minor copy of X that meets it in dR = X^T G): rows are
// features, and inside every group of 128 tokens the tokens are PERMUTED,
//     position(t) = (t & 31) * 4 + ((t & 127) >> 5),
// because the contraction over tokens does not care in which order the tokens come as
// long as both operands agree.  In the accumulator layout a lane owns tokens
// t, t+32, t+64, t+96 of a group, so with this order its values for one feature are
// ADJACENT in memory: one 8-byte store per feature instead of four 2-byte ones, and 32
// lanes cover 256 contiguous bytes.  Tokens in [n_tokens, ldt) are written as zero so the
// padded K range contributes nothing; ldt is a multiple of 128.
// Rows are stored in blocks of tb tokens (tb a multiple of 128): position p of feature f
// lives at  (p / tb) * d * tb + f * tb + p % tb  (one block, tb = ldt, is the plain layout).
__host__ __device__ __forceinline__ int64_t token_position(int64_t t) {
  return (t & ~(int64_t)127) + ((t & 31) << 2) + ((t & 127) >> 5);
}

// dL/dy of one entry from the row's coefficients {alpha, mu, beta, m3}; alpha = 0 (padding tokens, rows
// without spread) gives 0 by itself as long as y is finite.  One definition for the recompute epilogue and
// for the kernel that reads a kept Y, so that the two paths round alike.
__device__ __forceinline__ float grad_value(float y, float alpha, float mu, float beta, float m3) {
  const float c = y - mu;
  return alpha * fmaf(c, fmaf(c, c, -beta), -m3);
}

template <class TL>
struct EpiGrad : EpiBase {
  using T = typename TL::T;
  const floatx4* coef;
  T* GT;
  int64_t ldt, tb, batch_stride;
  int n_tokens, d;
  static_assert(TL::BN % 128 == 0 && (TL::WTN == 128 || TL::WTN == 64), "token groups are 128 wide");
  __device__ __forceinline__ void operator()(floatx16 (&acc)[TL::MB][TL::NB], int batch, int,
                                             int, int, int m0, int n0) const {
    typedef T vecT __attribute__((ext_vector_type(TL::NB)));
    const Frag<TL> f;
    const int wave_tok0 = n0 + f.wn * TL::WTN;            // first token of this wave
    const int group0 = wave_tok0 & ~127;                   // its 128-token group
    if (group0 >= ldt) return;
    // lane's tokens: wave_tok0 + nb*32 + (lane & 31); positions are consecutive in nb
    const int64_t pos0 = group0 + ((f.lane & 31) << 2) + ((wave_tok0 & 127) >> 5);
    const int64_t blk = pos0 / tb;
    T* out = GT + (int64_t)batch * batch_stride + blk * d * tb + (pos0 - blk * tb);
    float alpha[TL::NB], mu[TL::NB], beta[TL::NB], m3[TL::NB];
#pragma unroll
    for (int nb = 0; nb < TL::NB; ++nb) {
      const int token = n0 + f.n_of(nb);
      floatx4 c4 = {0.f, 0.f, 0.f, 0.f};  // alpha = 0 zeroes the padding tokens
      if (token < n_tokens) c4 = coef[(int64_t)batch * n_tokens + token];
      alpha[nb] = c4[0]; mu[nb] = c4[1]; beta[nb] = c4[2]; m3[nb] = c4[3];
    }
#pragma unroll
    for (int mb = 0; mb < TL::MB; ++mb) {
      if (m0 + f.m_block(mb) < d) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          vecT v;
#pragma unroll
          for (int nb = 0; nb < TL::NB; ++nb)  // (the accumulators of padding tokens come from re-read valid rows and are finite)
            v[nb] = from_float<T>(grad_value(acc[mb][nb][r], alpha[nb], mu[nb], beta[nb], m3[nb]));
          const int feat = m0 + f.m_of(mb, r);
          *reinterpret_cast<vecT*>(out + (int64_t)feat * tb) = v;
        }
      }
    }
  }
};

// ---- forward pass that also keeps Y = X R ("Learning the Rotations"): the moments of EpiMoments (Eq. 3), and the fp32 accumulators written
// in the layout of GT above (features on the rows, tokens permuted inside groups of 128, blocks of tb
// tokens): one 16-byte store per lane and feature.  grad_from_y_kernel then turns YT into GT entry by
// entry, which replaces the recompute GEMM of the backward pass (same accumulators, same arithmetic: the
// gradient is bit-identical) at the price of n d 4 bytes of scratch, one write and one read of them.
template <class TL>
struct EpiMomentsKeep : EpiBase {
  EpiMoments<TL> mom;
  float* YT;
  int64_t ldt, tb, batch_stride;  // batch_stride in elements of YT
  static_assert(TL::BN % 128 == 0 && (TL::WTN == 128 || TL::WTN == 64), "token groups are 128 wide");
  __device__ __forceinline__ void operator()(floatx16 (&acc)[TL::MB][TL::NB], int batch, int tm,
                                             int tn, int ks, int m0, int n0) const {
    mom(acc, batch, tm, tn, ks, m0, n0);
    typedef float vecF __attribute__((ext_vector_type(TL::NB)));
    const Frag<TL> f;
    const int wave_tok0 = n0 + f.wn * TL::WTN;
    const int group0 = wave_tok0 & ~127;
    if (group0 >= ldt) return;
    const int64_t pos0 = group0 + ((f.lane & 31) << 2) + ((wave_tok0 & 127) >> 5);
    const int64_t blk = pos0 / tb;
    float* out = YT + (int64_t)batch * batch_stride + blk * mom.d * tb + (pos0 - blk * tb);
#pragma unroll
    for (int mb = 0; mb < TL::MB; ++mb) {
      if (m0 + f.m_block(mb) < mom.d) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          vecF v;
#pragma unroll
          for (int nb = 0; nb < TL::NB; ++nb) v[nb] = acc[mb][nb][r];
          *reinterpret_cast<vecF*>(out + (int64_t)(m0 + f.m_of(mb, r)) * tb) = v;
        }
      }
    }
  }
};

// ---- plain fp32 store, optionally into split-K partial slabs ---------------------
// C[ks*split_stride + batch*batch_stride + m*ldc + n]
template <class TL>
struct EpiStore : EpiBase {
  float* C;
  int64_t ldc, batch_stride, split_stride;
  int M, N;
  float alpha = 1.f;  // C = alpha * acc
  // An accumulator block leaves the matrix pipe with one COLUMN per lane (4 consecutive rows in 4 registers), so
  // a direct store is a 4-byte store per lane, 256 of them per wave and tile, and the address path handles
  // each at the same rate as a 16-byte one.  Here every 8 x 32 piece (4 registers of the two wave halves)
  // passes through a 1.1 KiB buffer of the wave's own in LDS and comes back as 16 bytes per lane, 8 lanes
  // to a 128-byte row piece: 64 stores per wave and tile, each of 8 whole 128-byte lines.
  static constexpr int kPieceWords = 8 * 32 + 32;  // rows 4..7 sit 32 words further: the two halves hit different banks
  static constexpr int kPieceBufs = 4;
  static_assert(TL::NT / 64 * kPieceBufs * kPieceWords * 4 <= TL::LDS_BYTES, "piece buffers must fit the operand LDS");
  __device__ __forceinline__ void operator()(floatx16 (&acc)[TL::MB][TL::NB], int batch, int,
                                             int, int ks, int m0, int n0) const {
    const Frag<TL> f;
    float* base = C + (int64_t)ks * split_stride + (int64_t)batch * batch_stride;
    // 16-byte stores need aligned rows and whole groups of 4 columns inside N (uniform over the launch)
    const bool vec = ((reinterpret_cast<uintptr_t>(base) | (uintptr_t)(ldc * 4)) & 15) == 0 && (N & 3) == 0;
    if (!vec) {
#pragma unroll
      for (int mb = 0; mb < TL::MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < TL::NB; ++nb) {
          const int n = n0 + f.n_of(nb);
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int m = m0 + f.m_of(mb, r);
            if (m < M && n < N) base[(int64_t)m * ldc + n] = alpha * acc[mb][nb][r];
          }
        }
      return;
    }
    extern __shared__ __align__(16) char lds_raw[];
    __syncthreads();  // every wave has read its last operand slab: the LDS is free
    float* buf = reinterpret_cast<float*>(lds_raw) + (threadIdx.x >> 6) * (kPieceBufs * kPieceWords);
    const int wofs = f.half * 160 + (f.lane & 31);  // register i of this lane -> row 4 half + i, column lane % 32
    const int rrow = f.lane >> 3, rcol = 4 * (f.lane & 7);
    const int rofs = rrow * 32 + (rrow >> 2) * 32 + rcol;
#pragma unroll
    for (int mb = 0; mb < TL::MB; ++mb)
#pragma unroll
      for (int nb = 0; nb < TL::NB; ++nb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float* b = buf + (((mb * TL::NB + nb) * 4 + g) % kPieceBufs) * kPieceWords;
#pragma unroll
          for (int i = 0; i < 4; ++i) b[wofs + 32 * i] = alpha * acc[mb][nb][4 * g + i];
          // the wave's LDS operations complete in order: no barrier between its own writes and reads
          const float4 v = *reinterpret_cast<const float4*>(b + rofs);
          const int m = m0 + f.m_block(mb) + 8 * g + rrow;
          const int n = n0 + f.wn * TL::WTN + nb * 32 + rcol;
          if (m < M && n < N) *reinterpret_cast<float4*>(base + (int64_t)m * ldc + n) = v;
        }
  }
};

// Max of |x| taken on bit patterns: for non-negative floats the unsigned order is the
// numeric order, +inf sits above every finite value and NaN above +inf, so a NaN
// anywhere survives the reduction instead of being dropped as fmaxf would.
__device__ __forceinline__ unsigned abs_bits(float v) { return __float_as_uint(v) & 0x7fffffffu; }
__device__ __forceinline__ unsigned umax(unsigned a, unsigned b) { return a > b ? a : b; }
__device__ __forceinline__ unsigned wave_umax(unsigned v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = umax(v, (unsigned)__shfl_xor((int)v, o));
  return v;
}

// ---- Cayley fixed point, in transposed space ---------------------------------------
// acc = U_k * B^T.  Zt_new = Rt - acc;  U_{k+1} = Rt + Zt_new;
// delta[it] = max |Zt_new - Zt_old| (bit pattern of a non-negative float, max is
// order independent so the result is deterministic).  The launch for iteration `it`
// returns at once when iteration it-1 already met the tolerance.
// When an iteration counts as converged.  The map is linear, Z_k+1 - Z_k = -B (Z_k - Z_k-1), so the
// changes shrink geometrically with the spectral radius rho of B = (lr/2) A and the iterate just written
// is within d_k rho / (1 - rho) of the fixed point (d_k = max |Z_k - Z_k-1|).  rho is estimated from the
// changes themselves.  Even and odd powers of a skew matrix have different patterns (for a low-rank
// gradient, B^2k is concentrated on a few entries and B^2k+1 is not, or the other way round), so that
// successive maxima alternate between two levels: the ratio over TWO steps, d_k / d_k-2 = rho^2, does not
// see that and is used as soon as three changes are there; with two, the one-step ratio.
//  - first iteration: converged only if the whole step is below the tolerance;
//  - 4 d_k rho / (1 - rho) <= tol (four times the distance bound), rho < 0.95; for rho < 0.2 this
//    accepts an iterate before its own change is below the tolerance and saves the product that would only
//    confirm it, for slow contractions it asks for more than d_k <= tol: what is left of the series then
//    still matters for max |R^T R - I|;
//  - the rounding floor: the change is small (within 64 tolerances) and has stopped shrinking over both of
//    the last two steps (for the three-term bf16 products the floor lies at a few 1e-7 and would never pass
//    a fixed fp32-sized tolerance).
// d1, d0, d00: changes of iterations k, k-1, k-2; nprev: how many of d0, d00 exist (0, 1 or 2).
__device__ __forceinline__ bool cayley_converged_hist(float d1, float d0, float d00, int nprev, float tol) {
  if (nprev == 0) return d1 <= tol;
  if (d1 == 0.f) return true;
  const float rho = nprev >= 2 ? sqrtf(d1 / d00) : d1 / d0;
  if (rho < 0.95f && 4.f * d1 * rho <= tol * (1.f - rho)) return true;
  if (nprev < 2 || !(d1 <= 64.f * tol)) return false;
  return d1 >= 0.9f * d0 && d1 >= 0.8f * d00;
}
__device__ __forceinline__ bool cayley_converged(const unsigned* dl, int k, float tol) {
  return cayley_converged_hist(__uint_as_float(dl[k]), k > 0 ? __uint_as_float(dl[k - 1]) : 0.f,
                               k > 1 ? __uint_as_float(dl[k - 2]) : 0.f, k > 1 ? 2 : k, tol);
}

// Unew is written as fp32, or (Usplit != null) as the [hi | hi | lo] bf16 operand of the
// three-term bf16 GEMM that runs the next iteration.
template <class TL>
struct EpiCayleyIter {
  const float* Rt;
  float* Zt;
  float* Unew;
  __bf16* Usplit;
  unsigned* delta;  // [batch][max_iters]
  int d, it, max_iters;
  float tol;
  const float* bscale = nullptr;  // acc is scaled by bscale[4 * batch + 3] when given (Cayley Adam)
  __device__ __forceinline__ bool skip(int batch) const {
    if (it == 0) return false;
    const unsigned* dl = delta + (int64_t)batch * max_iters;
    if (!cayley_converged(dl, it - 1, tol)) return false;
    // converged earlier: record a zero change so that every later launch returns too
    if (blockIdx.x == 0 && threadIdx.x == 0) delta[(int64_t)batch * max_iters + it] = 0u;
    return true;
  }
  __device__ __forceinline__ void operator()(floatx16 (&acc)[TL::MB][TL::NB], int batch, int,
                                             int, int, int m0, int n0) const {
    const Frag<TL> f;
    const int64_t bo = (int64_t)batch * d * d;
    const float bs = bscale ? bscale[4 * batch + 3] : 1.f;
    unsigned dmax = 0u;
#pragma unroll
    for (int mb = 0; mb < TL::MB; ++mb)
#pragma unroll
      for (int nb = 0; nb < TL::NB; ++nb) {
        const int n = n0 + f.n_of(nb);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = m0 + f.m_of(mb, r);
          if (m < d && n < d) {
            const int64_t idx = bo + (int64_t)m * d + n;
            const float rt = Rt[idx];
            const float z = rt - bs * acc[mb][nb][r];
            dmax = umax(dmax, abs_bits(z - Zt[idx]));
            Zt[idx] = z;
            const float u = rt + z;
            if (Usplit) {
              const int64_t so = 3 * bo + (int64_t)m * 3 * d + n;
              const __bf16 hi = (__bf16)u;
              const __bf16 lo = (__bf16)(u - (float)hi);
              Usplit[so] = hi;
              Usplit[so + d] = hi;
              Usplit[so + 2 * d] = lo;
            } else {
              Unew[idx] = u;
            }
          }
        }
      }
    dmax = wave_umax(dmax);
    if (f.lane == 0) atomicMax(&delta[(int64_t)batch * max_iters + it], dmax);
  }
};

// Plain fp32 store of one Cayley iteration's product (the update runs as a separate
// elementwise kernel); returns at once when an earlier iteration has converged.
template <class TL>
struct EpiCayleyProduct : EpiStore<TL> {
  const unsigned* delta;  // [batch][max_iters]
  int it, max_iters;
  float tol;
  __device__ __forceinline__ bool skip(int batch) const {
    return it > 0 && cayley_converged(delta + (int64_t)batch * max_iters, it - 1, tol);
  }
};

// ---- orthogonality check: max |acc_mn| over m != n -----------------------------------
// The diagonal (sums of squares close to 1, where fp32 accumulation loses ~1e-7 per
// entry) is left to ortho_diag_kernel, which sums in fp64.
template <class TL>
struct EpiOrtho : EpiBase {
  unsigned* err;  // [batch], bit pattern of a non-negative float, zeroed before launch
  int d;
  __device__ __forceinline__ void operator()(floatx16 (&acc)[TL::MB][TL::NB], int batch, int,
                                             int, int, int m0, int n0) const {
    const Frag<TL> f;
    unsigned e = 0u;
#pragma unroll
    for (int mb = 0; mb < TL::MB; ++mb)
#pragma unroll
      for (int nb = 0; nb < TL::NB; ++nb) {
        const int n = n0 + f.n_of(nb);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = m0 + f.m_of(mb, r);
          if (m < d && n < d && m != n) e = umax(e, abs_bits(acc[mb][nb][r]));
        }
      }
    e = wave_umax(e);
    if (f.lane == 0) atomicMax(&err[batch], e);
  }
};

// ---- fake-quant pass A: per-token max |y| -----------------------------------------
// same orientation as EpiMoments; part[(batch*P + p)*n_tokens + token]
template <class TL>
struct EpiAmax : EpiBase {
  float* part;
  int n_tokens, d, P;
  __device__ __forceinline__ void operator()(floatx16 (&acc)[TL::MB][TL::NB], int batch, int tm,
                                             int, int, int m0, int n0) const {
    const Frag<TL> f;
    const int p = tm * TL::WGM + f.wm;
#pragma unroll
    for (int nb = 0; nb < TL::NB; ++nb) {
      float a = 0.f;
#pragma unroll
      for (int mb = 0; mb < TL::MB; ++mb)
        if (m0 + f.m_block(mb) < d) {
#pragma unroll
          for (int r = 0; r < 16; ++r) a = fmaxf(a, fabsf(acc[mb][nb][r]));
        }
      a = fmaxf(a, __shfl_xor(a, 32));
      const int token = n0 + f.n_of(nb);
      if (f.half == 0 && token < n_tokens) part[((int64_t)batch * P + p) * n_tokens + token] = a;
    }
  }
};

// ---- fake-quant pass B: quantise the recomputed y ----------------------------------
// Same orientation as the moment epilogue (token on the lane, features on the registers): the
// scale and its reciprocal are taken once per token, the error sums accumulate in registers and
// meet only the other half-wave, and the codes leave as 16-byte stores (a lane and its partner in
// the other half-wave exchange two packed words first).  q = clamp(rint(y * (1/s)), -7, 7) in fp32;
// pe[(batch*P + p)*n_tokens + token] = {sum (y - q s)^2, sum y^2} over the wave's feature rows.
template <class TL>
struct EpiQuant : EpiBase {
  const float* scales;  // [batch][n_tokens]
  int8_t* codes;        // [batch][n_tokens][d] or null
  float2* err_part;     // or null
  int n_tokens, d, P;
  __device__ __forceinline__ void operator()(floatx16 (&acc)[TL::MB][TL::NB], int batch, int tm,
                                             int, int, int m0, int n0) const {
    const Frag<TL> f;
    const int p = tm * TL::WGM + f.wm;
#pragma unroll
    for (int nb = 0; nb < TL::NB; ++nb) {
      const int token = n0 + f.n_of(nb);
      const bool tv = token < n_tokens;
      const float s = tv ? scales[(int64_t)batch * n_tokens + token] : 0.f;
      const bool live = s > 0.f;
      const float rinv = live ? __fdiv_rn(1.0f, s) : 0.f;
      int8_t* crow = codes + ((int64_t)batch * n_tokens + token) * d;
      float e2 = 0.f, y2 = 0.f;
#pragma unroll
      for (int mb = 0; mb < TL::MB; ++mb) {
        if (m0 + f.m_block(mb) < d) {
          unsigned pk[4];
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            unsigned pack = 0u;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float y = acc[mb][nb][4 * g + e];
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
          // the lane and its partner (lane ^ 32) own alternate groups of four features: two words change
          // hands, then the lower half-wave stores bytes 0..15 of the 32-feature block, the upper 16..31
          const unsigned r0 = (unsigned)__shfl_xor((int)(f.half ? pk[0] : pk[2]), 32);
          const unsigned r1 = (unsigned)__shfl_xor((int)(f.half ? pk[1] : pk[3]), 32);
          uintx4 out;
          if (f.half == 0) out = uintx4{pk[0], r0, pk[1], r1};
          else out = uintx4{r0, pk[2], r1, pk[3]};
          if (codes && tv) *reinterpret_cast<uintx4*>(crow + m0 + f.m_block(mb) + 16 * f.half) = out;
        }
      }
      if (err_part) {
        e2 += __shfl_xor(e2, 32);
        y2 += __shfl_xor(y2, 32);
        if (f.half == 0 && tv) err_part[((int64_t)batch * P + p) * n_tokens + token] = make_float2(e2, y2);
      }
    }
  }
};

}  // namespace kt
