// kt_hadamard.h -- the online rotations of "Placement of the Rotations" (R3, R4, R5: random
// Hadamard matrices applied to activations at run time):  y = (x * signs) H_d / sqrt(d) per token
// row, H_d the Sylvester-Hadamard matrix, d = 2^k.
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
template <typename T, int LOG2D>
__global__ __launch_bounds__(256) void hadamard_rows_kernel(const T* __restrict__ X, int64_t ldx,
                                                            T* __restrict__ Y, int64_t ldy,
                                                            const int8_t* __restrict__ signs, int64_t n,
                                                            float scale) {
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
#pragma unroll
          for (int e = 0; e < VEC; ++e) v[e] *= (float)signs[col + e];
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

}  // namespace kt
