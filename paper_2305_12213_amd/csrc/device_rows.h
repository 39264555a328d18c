// Device helpers for kernels that walk row-major bf16 tensors [rows][ld] with 16-byte
// accesses: a lane takes 8 neighbouring channels of a row, 8 lanes one 128-byte line, the 256
// threads of a workgroup 32 rows x 64 channels per pass (channel granule = tid & 7, row-lane =
// tid >> 3).
#ifndef DYNB_DEVICE_ROWS_H
#define DYNB_DEVICE_ROWS_H

#include <hip/hip_runtime.h>

namespace dynb {

typedef __bf16 bf16;

__device__ inline void unpack8(const uint4& q, float (&f)[8]) {
  f[0] = __uint_as_float(q.x << 16); f[1] = __uint_as_float(q.x & 0xffff0000u);
  f[2] = __uint_as_float(q.y << 16); f[3] = __uint_as_float(q.y & 0xffff0000u);
  f[4] = __uint_as_float(q.z << 16); f[5] = __uint_as_float(q.z & 0xffff0000u);
  f[6] = __uint_as_float(q.w << 16); f[7] = __uint_as_float(q.w & 0xffff0000u);
}

__device__ inline uint32_t pack2(float a, float b) {      // round to nearest even, both halves
  const bf16 x = (bf16)a, y = (bf16)b;
  return (uint32_t)__builtin_bit_cast(unsigned short, x) |
         ((uint32_t)__builtin_bit_cast(unsigned short, y) << 16);
}

__device__ inline uint4 pack8(const float (&f)[8]) {
  return make_uint4(pack2(f[0], f[1]), pack2(f[2], f[3]), pack2(f[4], f[5]), pack2(f[6], f[7]));
}

__device__ inline uint4 load8(const bf16* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ inline void store8(bf16* p, const uint4& q) { *reinterpret_cast<uint4*>(p) = q; }

// Sums a[0..7] (this lane's 8 channels) over the 32 row-lanes of the workgroup, in a fixed
// order; every thread ends with the totals of its channels.  `red` is workgroup-shared.
__device__ inline void sum_over_rows(float (&a)[8], float (*red)[64]) {
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    a[j] += __shfl_xor(a[j], 8);
    a[j] += __shfl_xor(a[j], 16);
    a[j] += __shfl_xor(a[j], 32);
  }
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, cg = threadIdx.x & 7;
  __syncthreads();
  if (lane < 8) {
#pragma unroll
    for (int j = 0; j < 8; ++j) red[wave][lane * 8 + j] = a[j];
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 8; ++j)
    a[j] = ((red[0][cg * 8 + j] + red[1][cg * 8 + j]) + red[2][cg * 8 + j]) + red[3][cg * 8 + j];
}

}  // namespace dynb

#endif
