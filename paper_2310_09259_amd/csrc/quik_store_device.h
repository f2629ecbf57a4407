// A 16-byte global store that is written through the XCD's L2 at device scope.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace quik {

// For data the storing kernel never reads again (the GEMM's output tile, the quantized rows): kept as
// dirty lines they would displace operand panels from the XCD's L2 and be written back in one burst
// when the kernel ends; `sc1` sends them on as they are produced (measured on the LLaMA-7B up-projection
// at 2048 tokens: 2 % of the GEMM's time, 3 % of the quantization kernel's).  Inline asm because the
// compiler has no 16-byte store with a scope; the s_nop covers the wait states a store of more than
// 8 bytes needs before its data registers may be overwritten.  Counts in vmcnt like any store.
__device__ __forceinline__ void store16_through(void* dst, uint4 v) {
    typedef unsigned u4v __attribute__((ext_vector_type(4)));
    const u4v vv = {v.x, v.y, v.z, v.w};
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(dst), "v"(vv) : "memory");
}

}  // namespace quik
