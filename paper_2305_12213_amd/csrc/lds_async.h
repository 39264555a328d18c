// Asynchronous global -> LDS copies (gfx950 LDS-direct loads) shared by the convolution kernels.
#ifndef DYNB_LDS_ASYNC_H
#define DYNB_LDS_ASYNC_H

#include <hip/hip_runtime.h>

namespace dynb {

// 64 lanes x 16 bytes: lane l's 16 bytes at `src` land at LDS byte address lds_base + 16 * l
// (lds_base wave-uniform).  No registers are involved; completion is tracked by vmcnt only, in
// issue order, and the kernels wait for it by hand before the barrier that publishes a stage.
// Assembly, so that the compiler does not order later LDS reads of other stages behind it.
__device__ inline void async_copy_1k(const void* src, uint32_t lds_base) {
  const uint32_t base = __builtin_amdgcn_readfirstlane(lds_base);
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(base), "v"(src)
               : "memory", "m0");
}

// The same copy through a buffer resource: lane l's 16 bytes at byte offset `voffset` of the
// buffer.  A lane whose offset lies at or beyond the resource's size gets zeros (the hardware's
// range check), so "rows past a worker's last row read as zero" costs no instruction: the size
// is set to the end of the worker's rows.  Offsets must stay below 2^31 for the lanes that are
// parked out of range at 0x80000000.
typedef int i32x4 __attribute__((ext_vector_type(4)));
__device__ inline i32x4 buffer_resource(const void* base, uint32_t bytes) {
  const uint64_t a = (uint64_t)(uintptr_t)base;
  i32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
  r[1] = __builtin_amdgcn_readfirstlane((int)((uint32_t)(a >> 32) & 0xffffu));   // stride 0
  r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
  r[3] = 0x00020000;                                                             // 32-bit data
  return r;
}
__device__ inline void async_copy_1k_buffer(i32x4 rsrc, uint32_t voffset, uint32_t lds_base) {
  const uint32_t base = __builtin_amdgcn_readfirstlane(lds_base);
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(base), "v"(voffset),
               "s"(rsrc)
               : "memory", "m0");
}

// Address, on the current device, of 16 bytes of zeros: what lanes outside an image or a chunk
// copy instead (a copy cannot be predicated to zero).  Passed to kernels as an argument, which
// stays in scalar registers; nullptr if the lookup fails.
const void* device_zero_granule();

}  // namespace dynb

#endif
