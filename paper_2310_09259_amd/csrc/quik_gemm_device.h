// Device helpers shared by the GEMM kernels (integer MFMA path and FP6 MFMA path).
// Private to the shared library.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "quik_store_device.h"

namespace quik {
namespace gemm_dev {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void* lds_ptr;

constexpr int kThreads = 256;
constexpr int kXcds = 8;
constexpr uint32_t kOob = 0x80000000u;     // byte offset beyond any descriptor range

// Maps the hardware workgroup id (dealt round-robin over the 8 XCDs) to a logical
// tile id such that each XCD works on a contiguous range of logical tiles and so
// re-uses operand panels out of its own L2.
__device__ __forceinline__ int xcd_contiguous_id(int b, int nblk) {
    int x = b % kXcds, local = b / kXcds;
    int q = nblk / kXcds, r = nblk % kXcds;
    int start = (x < r) ? x * (q + 1) : r * (q + 1) + (x - r) * q;
    return start + local;
}

// Raw buffer descriptor over [p, p + bytes): loads beyond the range return zero.
__device__ __forceinline__ v4i make_rsrc(const void* p, size_t bytes) {
    uint32_t n = bytes > 0x7FFFFFFFull ? 0x7FFFFFFFu : (uint32_t)bytes;
    uint64_t q = (uint64_t)(uintptr_t)p;
    v4i r = v4i{(int)(uint32_t)q, (int)(uint32_t)(q >> 32), (int)n, 0x00020000};
    r[0] = __builtin_amdgcn_readfirstlane(r[0]);
    r[1] = __builtin_amdgcn_readfirstlane(r[1]);
    r[2] = __builtin_amdgcn_readfirstlane(r[2]);
    return r;
}

// 16 bytes per lane, global -> LDS at lds_base + lane*16, source = rsrc.base + voff + soff.
// Issued as inline asm so that the compiler's wait-count insertion does not serialise
// it against LDS reads of other stage buffers; completion is tracked by hand (vmcnt).
// Extra vector-memory operations the compiler does not know about can only make its
// own waits more conservative, because the counter retires in order.
__device__ __forceinline__ void dma16(v4i rsrc, uint32_t lds_base, uint32_t voff, uint32_t soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_base), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) { return (uint32_t)(uintptr_t)(lds_ptr)(p); }

// XOR swizzle of the 16-byte slot index inside a stage row of BKB bytes.
template <int BKB> __device__ __forceinline__ int swz(int r) {
    if constexpr (BKB == 64) return (r >> 2) & 3;
    else return (r >> 1) & 7;
}
template <int N> __device__ __forceinline__ void wait_vm() {   // s_waitcnt vmcnt(N) only
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

}  // namespace gemm_dev
}  // namespace quik
