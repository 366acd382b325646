// kt_hadamard.h -- the online rotations of "Placement of the Rotations" (R3, R4, R5: random
// Hadamard matrices applied to activations at run time):  y = (x * signs) H_d / sqrt(d) per token
// row.  hadamard_rows_kernel: H_d the Sylvester-Hadamard matrix, d = 2^k <= 4096.
// hadamard_cross_kernel (end of file): the second factor of H_d = H_m (x) S_{2^k} for the sizes
// m 2^k that are not powers of two (or exceed 4096).
//
// HBM-bound: 2 d element reads + 2 d element writes per row against d log2 d additions.  One WAVE
// owns a chunk of 4096 consecutive elements (4096 / d whole rows) and never meets the other waves:
//   1. coalesced 16-byte global loads (issued one chunk ahead) -> fp32 -> its private LDS
//      region (linear order)
//   2. each lane takes 64 consecutive elements: six butterfly stages in registers
//   3. through LDS again, transposed: each lane now holds the elements 64 apart, i.e. the
//      remaining log2(d) - 6 index bits of a row: the last stages in registers
//   4. through LDS back to linear order -> scale, round, coalesced 16-byte stores
// The LDS region is padded by 4 floats per 64 (index i lives at i + 4 (i >> 6)): the 16-byte
// accesses of steps 1, 2, 4 stay aligned and conflict-free (16 lanes of one cycle land 4 or 8
// floats apart modulo the padding), and the 4-byte transposed accesses of step 3 are consecutive
// across lanes.  LDS instructions of one wave execute in order, so no barrier is needed; the
// compiler is kept from reordering them with memory clobbers.
#pragma once
#include "kt_aux.h"
#include "kt_fused_d128.h"  // read_tr_operand

namespace kt {

constexpr int kHadChunk = 4096;
constexpr int kHadRegion = kHadChunk + 4 * (kHadChunk / 64);  // floats per wave

__device__ __forceinline__ void had_lds_fence() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

template <int N>
__device__ __forceinline__ void had_butterflies(float (&a)[64], int first_stage_bit) {
  // N stages on index bits first_stage_bit .. first_stage_bit + N - 1 of the 64 registers
#pragma unroll
  for (int s = 0; s < N; ++s) {
    const int h = 1 << (first_stage_bit + s);
#pragma unroll
    for (int e = 0; e < 64; ++e) {
      if ((e & h) == 0) {
        const float u = a[e], v = a[e | h];
        a[e] = u + v;
        a[e | h] = u - v;
      }
    }
  }
}

// T = float or __bf16; LOG2D in 7..12.  grid.x workgroups of 4 waves walk the chunks.
// sign_rows > 1: the rows are segments of longer rows (sign_rows segments each) and row r takes its
// signs from signs[(r % sign_rows) * D ...].
template <typename T, int LOG2D>
__global__ __launch_bounds__(256) void hadamard_rows_kernel(const T* __restrict__ X, int64_t ldx,
                                                            T* __restrict__ Y, int64_t ldy,
                                                            const int8_t* __restrict__ signs, int64_t n,
                                                            float scale, int sign_rows) {
  constexpr int D = 1 << LOG2D, ROWS = kHadChunk / D, M = LOG2D - 6, VEC = 16 / (int)sizeof(T);
  constexpr int NLD = kHadChunk / (64 * VEC);  // 16-byte accesses per lane and chunk
  extern __shared__ __align__(16) float lds_all[];  // 4 * kHadRegion floats
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* lds = lds_all + wave * kHadRegion;
  const int64_t chunks = (n + ROWS - 1) / ROWS;
  // the loads of the next chunk are in flight while this one is transformed
  intx4 nxt[NLD];
  auto request = [&](int64_t chunk) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < NLD; ++t) {
      const int i = (t * 64 + lane) * VEC;
      const int64_t row = chunk * ROWS + (i >> LOG2D);
      intx4 r = {0, 0, 0, 0};
      if (chunk < chunks && row < n) r = *reinterpret_cast<const intx4*>(X + row * ldx + (i & (D - 1)));
      nxt[t] = r;
    }
  };
  const int64_t stride = (int64_t)gridDim.x * 4;
  request((int64_t)blockIdx.x * 4 + wave);
  for (int64_t chunk = (int64_t)blockIdx.x * 4 + wave; chunk < chunks; chunk += stride) {
    const int64_t row0 = chunk * ROWS;
    intx4 cur[NLD];
#pragma unroll
    for (int t = 0; t < NLD; ++t) cur[t] = nxt[t];
    request(chunk + stride);
    // 1. registers -> LDS (linear, padded)
#pragma unroll
    for (int t = 0; t < NLD; ++t) {
      const int i = (t * 64 + lane) * VEC;
      const int64_t row = row0 + (i >> LOG2D);
      const int col = i & (D - 1);
      float v[VEC];
      if (row < n) {
        const intx4 raw = cur[t];
        if constexpr (sizeof(T) == 4) {
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = __int_as_float(raw[e]);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {  // bf16 -> fp32: the 16 bits are the high half
            v[2 * e] = __int_as_float(raw[e] << 16);
            v[2 * e + 1] = __int_as_float(raw[e] & 0xffff0000);
          }
        }
        if (signs) {
          const int8_t* sg = signs + col;
          if (sign_rows > 1) sg += (int64_t)((unsigned)row % (unsigned)sign_rows) * D;  // rows < 2^31 here
#pragma unroll
          for (int e = 0; e < VEC; ++e) v[e] *= (float)sg[e];
        }
      } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = 0.f;
      }
      float* dst = lds + i + 4 * (i >> 6);
#pragma unroll
      for (int e = 0; e < VEC; e += 4) *reinterpret_cast<floatx4*>(dst + e) = floatx4{v[e], v[e + 1], v[e + 2], v[e + 3]};
    }
    had_lds_fence();
    // 2. 64 consecutive elements per lane (index bits 0..5)
    float a[64];
#pragma unroll
    for (int g = 0; g < 16; ++g) {
      const floatx4 q = *reinterpret_cast<const floatx4*>(lds + 68 * lane + 4 * g);
      a[4 * g] = q[0]; a[4 * g + 1] = q[1]; a[4 * g + 2] = q[2]; a[4 * g + 3] = q[3];
    }
    had_butterflies<6>(a, 0);
    had_lds_fence();
#pragma unroll
    for (int g = 0; g < 16; ++g)
      *reinterpret_cast<floatx4*>(lds + 68 * lane + 4 * g) = floatx4{a[4 * g], a[4 * g + 1], a[4 * g + 2], a[4 * g + 3]};
    had_lds_fence();
    // 3. elements lane + 64 j: index bits 6.. of the chunk; the low M bits of j belong to the row
#pragma unroll
    for (int j = 0; j < 64; ++j) a[j] = lds[lane + 68 * j];
    had_butterflies<M>(a, 0);
    had_lds_fence();
#pragma unroll
    for (int j = 0; j < 64; ++j) lds[lane + 68 * j] = a[j] * scale;
    had_lds_fence();
    // 4. LDS (linear) -> global
#pragma unroll
    for (int t = 0; t < NLD; ++t) {
      const int i = (t * 64 + lane) * VEC;
      const int64_t row = row0 + (i >> LOG2D);
      const int col = i & (D - 1);
      const float* src = lds + i + 4 * (i >> 6);
      float v[VEC];
#pragma unroll
      for (int e = 0; e < VEC; e += 4) {
        const floatx4 q = *reinterpret_cast<const floatx4*>(src + e);
        v[e] = q[0]; v[e + 1] = q[1]; v[e + 2] = q[2]; v[e + 3] = q[3];
      }
      if (row < n) {
        if constexpr (sizeof(T) == 4) {
          *reinterpret_cast<floatx4*>(Y + row * ldy + col) = floatx4{v[0], v[1], v[2], v[3]};
        } else {
          typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));
          bf16x8v o;
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = (__bf16)v[e];
          *reinterpret_cast<bf16x8v*>(Y + row * ldy + col) = o;
        }
      }
    }
    had_lds_fence();
  }
}

// ---- H_d = H_m (x) S_p2 for d = m p2 --------------------------------------------------------------
// hadamard_rows_kernel has already transformed (and scaled) each of the m segments of p2
// consecutive elements of a row; this kernel mixes the segments, in place:
//   y[a p2 + b] = sum_a' x[a' p2 + b] H_m[a'][a].
// H_m (kind 0: Sylvester; 1: Paley's first construction, q = m - 1; 2: Paley's second, q = m/2 - 1)
// is written into LDS as floats by every workgroup from the quadratic residues of q.  A workgroup
// then walks tiles of 128 columns b of one row: the m x 128 values go through LDS as fp32 (all
// loads before any store, so the transform is in place); a thread owns two columns and four
// outputs a at a time, a wave reads its four H_m columns with one broadcast 16-byte LDS read per a'.
// m is a multiple of 4, p2 a multiple of 128.  LDS: (m*m + 128*CG*m) floats + q bytes.
template <typename T>
__global__ __launch_bounds__(256) void hadamard_cross_kernel(T* __restrict__ Y, int64_t ldy, int64_t n, int m,
                                                             int p2, int kind) {
  extern __shared__ __align__(16) float cross_lds[];
  float* S = cross_lds;
  float* xt = cross_lds + m * m;
  const int quads = m >> 2;
  int CG = quads >= 3 ? 1 : (quads == 2 ? 2 : 4);  // column groups of a tile, see below
  while (CG > 1 && (p2 >> 7) < CG) CG >>= 1;
  unsigned char* isq = reinterpret_cast<unsigned char*>(xt + 128 * CG * m);
  const int tid = threadIdx.x;
  const int h = kind == 2 ? m / 2 : m;  // order of the conference matrix
  const int q = h - 1;
  if (kind != 0) {
    for (int t = tid; t < q; t += 256) isq[t] = 0;
    __syncthreads();
    for (int t = 1 + tid; t < q; t += 256) isq[(t * t) % q] = 1;  // equal values: no race that matters
    __syncthreads();
  }
  for (int idx = tid; idx < m * m; idx += 256) {
    const int i = idx / m, j = idx - i * m;
    float e;
    if (kind == 0) {
      e = (__builtin_popcount(i & j) & 1) ? -1.f : 1.f;
    } else {
      const int u = i % h, v = j % h;
      // conference matrix entry: 0 on the diagonal, border +1 (first column of Paley I: -1),
      // inside the quadratic character of u - v
      float c;
      if (u == v) {
        c = 0.f;
      } else if (u == 0 || v == 0) {
        c = (kind == 1 && v == 0) ? -1.f : 1.f;
      } else {
        int x = (u - v) % q;
        if (x < 0) x += q;
        c = isq[x] ? 1.f : -1.f;
      }
      const float id = u == v ? 1.f : 0.f;
      if (kind == 1) e = c + id;
      else if (i < h && j < h) e = c + id;
      else if (i >= h && j >= h) e = -c - id;
      else e = c - id;
    }
    S[idx] = e;
  }
  __syncthreads();

  // A wave works on 128 columns (two per lane) and four outputs a at a time.  With fewer than four
  // such quads (m < 16) the waves share them out over CG = 2 or 4 column groups of a wider tile.
  const int c2 = tid & 63, g = tid >> 6;
  const int tcols = 128 * CG, ncb = p2 / tcols;
  const int cg = g % CG, q0 = g / CG, qstep = 4 / CG;
  const int64_t tiles = n * ncb;
  for (int64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const int64_t row = tile / ncb;
    const int cb = (int)(tile - row * ncb);
    T* base = Y + row * ldy + (int64_t)cb * tcols + 2 * c2;
    for (int idx = g; idx < m * CG; idx += 4) {
      const int a = idx / CG, k = idx - a * CG;
      float x0, x1;
      if constexpr (sizeof(T) == 4) {
        const float2 v = *reinterpret_cast<const float2*>(base + (int64_t)a * p2 + 128 * k);
        x0 = v.x; x1 = v.y;
      } else {
        const unsigned v = *reinterpret_cast<const unsigned*>(base + (int64_t)a * p2 + 128 * k);
        x0 = __uint_as_float(v << 16); x1 = __uint_as_float(v & 0xffff0000u);
      }
      *reinterpret_cast<float2*>(xt + a * tcols + 128 * k + 2 * c2) = make_float2(x0, x1);
    }
    __syncthreads();
    for (int qd = q0; qd < quads; qd += qstep) {
      float acc[4][2] = {{0.f, 0.f}, {0.f, 0.f}, {0.f, 0.f}, {0.f, 0.f}};
#pragma unroll 4
      for (int a = 0; a < m; ++a) {
        const float2 xv = *reinterpret_cast<const float2*>(xt + a * tcols + 128 * cg + 2 * c2);
        const floatx4 sv = *reinterpret_cast<const floatx4*>(S + a * m + 4 * qd);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[j][0] = fmaf(sv[j], xv.x, acc[j][0]);
          acc[j][1] = fmaf(sv[j], xv.y, acc[j][1]);
        }
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        T* dst = base + (int64_t)(4 * qd + j) * p2 + 128 * cg;
        if constexpr (sizeof(T) == 4) {
          *reinterpret_cast<float2*>(dst) = make_float2(acc[j][0], acc[j][1]);
        } else {
          typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
          bf16x2v o = {(__bf16)acc[j][0], (__bf16)acc[j][1]};
          *reinterpret_cast<bf16x2v*>(dst) = o;
        }
      }
    }
    __syncthreads();
  }
}

// The same factor for bf16 rows on the matrix cores: entries +-1 and bf16 inputs make every product
// exact, the sums run in fp32 as in the vector version.  Per tile of 128 NBW columns of one row
// (NBW = 2^lognb blocks of 32 columns per wave, chosen so that a tile holds about 128 x 128 values):
//   Y_tile^T[c][a] = sum_a' x[a'][c] H_m[a'][a]   =   A (M = c, K = a') times B (K = a', N = a)
// H_m^T sits in LDS as bf16, K-minor, zero-padded to 32-row blocks and 16-wide K steps, and is
// read as ordinary 16-byte fragments (the B operand).  The x tile sits in LDS as loaded (row a' =
// the tile's columns); its fragments (8 consecutive a' of one column per lane, the A operand) come
// from the transposing read ds_read_b64_tr_b16.  Rows a' >= m of the tile are zero and never
// written.  In the accumulators a lane then owns ONE output a and 4 x 4 consecutive columns, so the
// results go to the y tile in LDS with 8-byte stores (rows padded by 16 bytes against bank
// conflicts) and from there to memory as whole row pieces; the loads of the next tile are in
// flight while a tile is worked on.  m NBW <= 128.
// LDS bytes: 32 MB * 32 KS (H) + 16 KS * 256 NBW (x tile) + 32 MB * (256 NBW + 16) (y tile).
__global__ __launch_bounds__(256) void hadamard_cross_mfma_kernel(__bf16* __restrict__ Y, int64_t ldy, int64_t n,
                                                                  int m, int p2, int kind, int lognb) {
  extern __shared__ __align__(16) char cross_raw[];
  const int MB = (m + 31) >> 5, KS = (m + 15) >> 4;
  const int NBW = 1 << lognb, rowb = 256 << lognb, tcols = 128 << lognb;
  const int a_stride = 32 * KS;  // bytes per row of A: 16 KS bf16
  char* A = cross_raw;
  char* xt = A + 32 * MB * a_stride;
  char* yt = xt + 16 * KS * rowb;
  const int rowy = rowb + 16;  // bytes per row of the y tile
  unsigned char* isq = reinterpret_cast<unsigned char*>(yt);  // scratch during set-up only
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, l32 = lane & 31;
  const int h = kind == 2 ? m / 2 : m;
  const int q = h - 1;
  if (kind != 0) {
    for (int t = tid; t < q; t += 256) isq[t] = 0;
    __syncthreads();
    for (int t = 1 + tid; t < q; t += 256) isq[(t * t) % q] = 1;
    __syncthreads();
  }
  // A[a][k] = H_m[k][a] (0 in the padding)
  for (int idx = tid; idx < 32 * MB * 16 * KS; idx += 256) {
    const int a = idx / (16 * KS), k = idx - a * (16 * KS);
    float e = 0.f;
    if (a < m && k < m) {
      const int i = k, j = a;  // entry H_m[i][j]
      if (kind == 0) {
        e = (__builtin_popcount(i & j) & 1) ? -1.f : 1.f;
      } else {
        const int u = i % h, v = j % h;
        float c;
        if (u == v) {
          c = 0.f;
        } else if (u == 0 || v == 0) {
          c = (kind == 1 && v == 0) ? -1.f : 1.f;
        } else {
          int x = (u - v) % q;
          if (x < 0) x += q;
          c = isq[x] ? 1.f : -1.f;
        }
        const float id = u == v ? 1.f : 0.f;
        if (kind == 1) e = c + id;
        else if (i < h && j < h) e = c + id;
        else if (i >= h && j >= h) e = -c - id;
        else e = c - id;
      }
    }
    reinterpret_cast<__bf16*>(A)[idx] = (__bf16)e;
  }
  __syncthreads();  // isq (inside yt) is free again
  for (int i = tid; i < KS * rowb; i += 256) reinterpret_cast<intx4*>(xt)[i] = intx4{0, 0, 0, 0};
  __syncthreads();

  // lane constants of the transposing reads: columns tr_col .. +3 of a 32-column block, row 16 s + tr_row (+4)
  const int g16 = lane >> 4, rr = lane & 15;
  const int tr_col = 16 * (g16 & 1) + 4 * (rr & 3);
  const int tr_row = 8 * (g16 >> 1) + (rr >> 2);
  const int ncb = p2 / tcols;
  const int64_t tiles = n * ncb;
  // tile movement: 16-byte chunk c = tid + 256 i of the tile: row a = c / (16 NBW), chunk c % (16 NBW)
  const int chunk_shift = 4 + lognb, chunk_mask = (16 << lognb) - 1;
  intx4 nxt[8];
  auto request = [&](int64_t tile) __attribute__((always_inline)) {
    const int64_t row = tile / ncb;
    const int cb = (int)(tile - row * ncb);
    const __bf16* src = Y + row * ldy + (int64_t)cb * tcols;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int c = tid + 256 * i, a = c >> chunk_shift;
      if (tile < tiles && a < m) nxt[i] = *reinterpret_cast<const intx4*>(src + (int64_t)a * p2 + (c & chunk_mask) * 8);
    }
  };
  request(blockIdx.x);
  for (int64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const int64_t row = tile / ncb;
    const int cb = (int)(tile - row * ncb);
    __bf16* base = Y + row * ldy + (int64_t)cb * tcols;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int c = tid + 256 * i, a = c >> chunk_shift;
      if (a < m) *reinterpret_cast<intx4*>(xt + a * rowb + (c & chunk_mask) * 16) = nxt[i];
    }
    request(tile + gridDim.x);
    __syncthreads();
    for (int nb = 0; nb < NBW; ++nb) {
      const int col0 = (wave * NBW + nb) * 32;  // this wave's block of 32 columns
      const int tr_lo = tr_row * rowb + (col0 + tr_col) * 2, tr_hi = tr_lo + 4 * rowb;
      floatx16 acc[4];
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mb][r] = 0.f;
      for (int s = 0; s < KS; ++s) {
        const intx4 bf = read_tr_operand(xt, tr_lo + s * 16 * rowb, tr_hi + s * 16 * rowb);
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
          if (mb < MB) {
            const intx4 af = *reinterpret_cast<const intx4*>(A + (32 * mb + l32) * a_stride + (2 * s + half) * 16);
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bf),
                                                              __builtin_bit_cast(bf16x8, af), acc[mb], 0, 0, 0);
          }
      }
      // lane: output a = 32 mb + l32, columns col0 + 8 (r / 4) + 4 half + (r & 3)
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
        if (mb < MB) {
          const int a = 32 * mb + l32;
          if (a < m) {
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
              typedef __bf16 bf16x4v __attribute__((ext_vector_type(4)));
              const bf16x4v o = {(__bf16)acc[mb][4 * rg], (__bf16)acc[mb][4 * rg + 1], (__bf16)acc[mb][4 * rg + 2],
                                 (__bf16)acc[mb][4 * rg + 3]};
              *reinterpret_cast<bf16x4v*>(yt + a * rowy + (col0 + 8 * rg + 4 * half) * 2) = o;
            }
          }
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int c = tid + 256 * i, a = c >> chunk_shift;
      if (a < m)
        *reinterpret_cast<intx4*>(base + (int64_t)a * p2 + (c & chunk_mask) * 8) =
            *reinterpret_cast<const intx4*>(yt + a * rowy + (c & chunk_mask) * 16);
    }
    // the next tile's stores to xt come after every wave has passed the barrier above (its reads of
    // xt are done), its stores to yt after the next barrier (the copy-out above is done)
  }
}

}  // namespace kt
