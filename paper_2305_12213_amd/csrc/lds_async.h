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

// Address, on the current device, of 16 bytes of zeros: what lanes outside an image or a chunk
// copy instead (a copy cannot be predicated to zero).  Passed to kernels as an argument, which
// stays in scalar registers; nullptr if the lookup fails.
const void* device_zero_granule();

}  // namespace dynb

#endif
