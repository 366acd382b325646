// kt_cayley_d128.h -- the whole Cayley retraction of a 128 x 128 rotation in ONE workgroup.
//
// Head-dimension problems (one rotation per KV head and layer) come in batches of hundreds of
// independent 128 x 128 matrices.  The generic path spends ~35 launches on them, most of them
// returning at once; here one workgroup per problem keeps both GEMM operands in LDS (2 x 64 KiB)
// and R^T / the iterate in registers, and runs
//   M = dR R^T,  B = (lr/2)(M - M^T),  Zt <- Rt - U B^T,  U <- Rt + Zt  (to convergence),
//   R <- Zt^T,   max |R^T R - I|
// without touching HBM in between.  The Cayley Adam variant (ADAM = true) adds, in the same
// launch, the moment updates, the step scalars and the momentum projection M <- S R.
// Same arithmetic (fp32 MFMA, transposed-space fixed point of the Cayley updates the paper names
// in its implementation details), same convergence rule and same outputs as the generic fp32 path.
//
// LDS matrices are [128 rows][128 floats], 16-byte chunks XOR-swizzled with (row & 15) so that the
// 16-byte fragment reads of 16 consecutive rows at one K position are conflict-free.
#pragma once
#include "kt_aux.h"
#include "kt_gemm.h"

namespace kt {

constexpr int kC128MatBytes = 128 * 128 * 4;
constexpr int kC128LdsBytes = 2 * kC128MatBytes + 64 + 256 * 8;  // + max slots + fp64 sum scratch

__device__ __forceinline__ int c128_addr(int row, int col) {
  return row * 512 + ((((col >> 2) ^ (row & 15))) << 4) + ((col & 3) << 2);
}

// acc (this wave's 64 x 64 quadrant) = A B^T with A, B row-major 128 x 128 in LDS
__device__ __forceinline__ void c128_gemm_nt(const char* A, const char* B, floatx16 (&acc)[2][2], int wm,
                                             int wn, int l32, int half) {
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  const int arow0 = wm * 64 + l32, brow0 = wn * 64 + l32;  // (row & 15) is the same for + 32
  const char* ap = A + arow0 * 512;
  const char* bp = B + brow0 * 512;
  const int key = l32 & 15;
#pragma unroll 4
  for (int step = 0; step < 16; ++step) {
    const int off = ((2 * step + half) ^ key) << 4;
    intx4 fa[2], fb[2];
    fa[0] = *reinterpret_cast<const intx4*>(ap + off);
    fa[1] = *reinterpret_cast<const intx4*>(ap + 32 * 512 + off);
    fb[0] = *reinterpret_cast<const intx4*>(bp + off);
    fb[1] = *reinterpret_cast<const intx4*>(bp + 32 * 512 + off);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) Mma<float>::run(fa[i], fb[j], acc[i][j]);
  }
}

// max over the workgroup of a non-negative float's bit pattern (NaN patterns win)
__device__ __forceinline__ unsigned c128_block_umax(unsigned v, unsigned* red, int wave, int lane) {
  v = wave_umax(v);
  if (lane == 0) red[wave] = v;
  __syncthreads();
  return umax(umax(red[0], red[1]), umax(red[2], red[3]));
}

// Hyper-parameters of the Adam variant; c1 = 1 - beta1^k, c2 = 1 - beta2^k from the host.
struct C128Adam {
  float* M;            // [batch][128][128] momentum, in/out
  float* v;            // [batch] second moment, in/out
  float* scalars_out;  // [batch][3] {r, alpha, ||W||_F} or null
  float lr, beta1, beta2, eps, q;
  double c1, c2;
};

// grid = batch, 256 threads, kC128LdsBytes of dynamic LDS.
// SGD: S = half_lr (P - P^T) with P = dR R^T, transform factor 1.
// Adam: S = (P - P^T)/2 with P = M1 R^T, transform factor alpha/(2r), M <- S R.
template <bool ADAM>
__global__ __launch_bounds__(256) void cayley_d128_kernel(float* __restrict__ R, const float* __restrict__ dR,
                                                          __bf16* __restrict__ R_lowp, float half_lr,
                                                          float* __restrict__ ortho_err,
                                                          int32_t* __restrict__ info, int max_iters, float tol,
                                                          C128Adam ad) {
  extern __shared__ __align__(16) char lds[];
  char* bufA = lds;
  char* bufB = lds + kC128MatBytes;
  unsigned* red = reinterpret_cast<unsigned*>(lds + 2 * kC128MatBytes);
  double* dsum = reinterpret_cast<double*>(lds + 2 * kC128MatBytes + 64);
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, l32 = lane & 31, wm = wave >> 1, wn2 = wave & 1;
  float* Rb = R + (int64_t)b * 16384;
  const float* Gb = dR + (int64_t)b * 16384;

  // dR (Adam: M1 = beta1 M + (1 - beta1) dR) -> bufA, R -> bufB
  float* Mb = ADAM ? ad.M + (int64_t)b * 16384 : nullptr;
  double g2 = 0.0;
#pragma unroll 4
  for (int i = 0; i < 16; ++i) {
    const int f = i * 256 + tid, row = f >> 5, ch = f & 31;
    const int off = row * 512 + ((ch ^ (row & 15)) << 4);
    floatx4 g = *reinterpret_cast<const floatx4*>(Gb + row * 128 + ch * 4);
    if constexpr (ADAM) {
      const floatx4 m = *reinterpret_cast<const floatx4*>(Mb + row * 128 + ch * 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        g2 += (double)g[e] * (double)g[e];
        g[e] = ad.beta1 * m[e] + (1.f - ad.beta1) * g[e];
      }
    }
    *reinterpret_cast<floatx4*>(bufA + off) = g;
    *reinterpret_cast<intx4*>(bufB + off) = *reinterpret_cast<const intx4*>(Rb + row * 128 + ch * 4);
  }
  float r_adam = 1.f;
  if constexpr (ADAM) {
    const double tot = block_sum_256(g2, dsum);  // ends with a barrier: the tiles are complete too
    const double v1 = (double)ad.beta2 * (double)ad.v[b] + (1.0 - (double)ad.beta2) * tot;
    r_adam = (float)(ad.c1 * sqrt(v1 / ad.c2 + (double)ad.eps));
    __syncthreads();  // every thread has read v[b]
    if (tid == 0) ad.v[b] = (float)v1;
  } else {
    __syncthreads();
  }

  // element (i, j, r) of this lane: row m, column n of the 128 x 128 result
  auto m_of = [&](int i, int r) { return wm * 64 + i * 32 + ((r >> 2) << 3) + (half << 2) + (r & 3); };
  auto n_of = [&](int j) { return wn2 * 64 + j * 32 + l32; };

  floatx16 acc[2][2];
  c128_gemm_nt(bufA, bufB, acc, wm, wn2, l32, half);  // P = dR R^T (Adam: M1 R^T)
  __syncthreads();
  float rt[2][2][16], zt[2][2][16];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m_of(i, r), n = n_of(j);
        rt[i][j][r] = *reinterpret_cast<const float*>(bufB + c128_addr(n, m));  // Rt[m][n] = R[n][m]
        *reinterpret_cast<float*>(bufA + c128_addr(m, n)) = acc[i][j][r];       // M
      }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m_of(i, r), n = n_of(j);
        acc[i][j][r] = half_lr * (acc[i][j][r] - *reinterpret_cast<const float*>(bufA + c128_addr(n, m)));
      }
  __syncthreads();
  float bs = 1.f;  // factor of S in the fixed point
  if constexpr (ADAM) {
    double s2 = 0.0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s2 += (double)acc[i][j][r] * (double)acc[i][j][r];
    const double tot = block_sum_256(s2, dsum);
    const float wn = (float)(sqrt(tot) / (double)r_adam);
    const float alpha = fminf(ad.lr, 2.f * ad.q / (wn + ad.eps));
    bs = alpha / (2.f * r_adam);
    if (ad.scalars_out && tid == 0) {
      ad.scalars_out[3 * b] = r_adam;
      ad.scalars_out[3 * b + 1] = alpha;
      ad.scalars_out[3 * b + 2] = wn;
    }
    // M <- S R = S (Rt)^T: S -> bufB, Rt -> bufA
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = m_of(i, r), n = n_of(j);
          *reinterpret_cast<float*>(bufB + c128_addr(m, n)) = acc[i][j][r];
          *reinterpret_cast<float*>(bufA + c128_addr(m, n)) = rt[i][j][r];
        }
    __syncthreads();
    floatx16 mp[2][2];
    c128_gemm_nt(bufB, bufA, mp, wm, wn2, l32, half);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) Mb[m_of(i, r) * 128 + n_of(j)] = mp[i][j][r];
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m_of(i, r), n = n_of(j);
        *reinterpret_cast<float*>(bufB + c128_addr(m, n)) = acc[i][j][r];            // B, exactly skew
        *reinterpret_cast<float*>(bufA + c128_addr(m, n)) = 2.f * rt[i][j][r];        // U0 = Rt + Zt0
        zt[i][j][r] = rt[i][j][r];
      }
  __syncthreads();

  // fixed point in transposed space: Zt <- Rt - U B^T, U <- Rt + Zt
  int used = -1;
  float dprev = 0.f, dprev2 = 0.f;
  for (int it = 0; it < max_iters; ++it) {
    c128_gemm_nt(bufA, bufB, acc, wm, wn2, l32, half);
    unsigned dmax = 0u;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float z = rt[i][j][r] - bs * acc[i][j][r];
          dmax = umax(dmax, abs_bits(z - zt[i][j][r]));
          zt[i][j][r] = z;
        }
    dmax = c128_block_umax(dmax, red, wave, lane);  // its barrier also ends every wave's reads of bufA
    const float d1 = __uint_as_float(dmax);
    const bool conv = cayley_converged_hist(d1, dprev, dprev2, it > 1 ? 2 : it, tol);  // same rule as the generic path
    dprev2 = dprev;
    dprev = d1;
    if (conv) {
      used = it + 1;
      break;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          *reinterpret_cast<float*>(bufA + c128_addr(m_of(i, r), n_of(j))) = rt[i][j][r] + zt[i][j][r];
    __syncthreads();
  }

  // Zt -> bufA, then R = Zt^T with coalesced 16-byte stores.  An iteration that did not converge is
  // rejected as a whole: R (and its bf16 copy) come out as they went in.
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        *reinterpret_cast<float*>(bufA + c128_addr(m_of(i, r), n_of(j))) = used < 0 ? rt[i][j][r] : zt[i][j][r];
  __syncthreads();
#pragma unroll 4
  for (int i = 0; i < 16; ++i) {
    const int f = i * 256 + tid, row = f >> 5, c4 = (f & 31) * 4;  // R[row][c4 .. c4+3] = Zt[c4 + e][row]
    floatx4 v;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = *reinterpret_cast<const float*>(bufA + c128_addr(c4 + e, row));
    *reinterpret_cast<floatx4*>(Rb + row * 128 + c4) = v;
    if (R_lowp) {
      typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
      bf16x4 h;
#pragma unroll
      for (int e = 0; e < 4; ++e) h[e] = (__bf16)v[e];
      *reinterpret_cast<bf16x4*>(R_lowp + (int64_t)b * 16384 + row * 128 + c4) = h;
    }
  }
  if (info && tid == 0) info[b] = used;

  if (ortho_err) {  // max |Zt Zt^T - I|: off-diagonal from the fp32 product, diagonal summed in fp64
    c128_gemm_nt(bufA, bufA, acc, wm, wn2, l32, half);
    unsigned e = 0u;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (m_of(i, r) != n_of(j)) e = umax(e, abs_bits(acc[i][j][r]));
    if (tid < 128) {
      double s = 0.0;
      for (int k = 0; k < 128; ++k) {
        const double z = (double)*reinterpret_cast<const float*>(bufA + c128_addr(tid, k));
        s += z * z;
      }
      e = umax(e, abs_bits((float)fabs(s - 1.0)));
    }
    __syncthreads();  // red[] was last read in the iteration loop by every thread before this point
    e = c128_block_umax(e, red, wave, lane);
    if (tid == 0) ortho_err[b] = __uint_as_float(e);
  }
}

}  // namespace kt
