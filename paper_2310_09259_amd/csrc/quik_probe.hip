// Measurement probes: what the int8 matrix pipe and the memory system sustain on the chip the
// library runs on, so that a kernel's rate can be quoted against a measured ceiling as well as
// against the data-sheet one.  Not part of the layer.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "quik_kernels.h"

namespace quik {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Nothing but independent v_mfma_i32_32x32x32_i8 instructions on register-resident operands:
// four accumulators per wave, four waves per workgroup.
__global__ __launch_bounds__(256) void mfma_i8_probe_kernel(int iters, int* sink) {
    v4i a = v4i{(int)threadIdx.x, 1, 2, 3}, b = v4i{4, 5, 6, (int)blockIdx.x};
    v16i c0 = {}, c1 = {}, c2 = {}, c3 = {};
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c3, 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
    if (s == 0x7fffffff) sink[0] = s;     // never true in practice: keeps the loop alive
}

// Plain streaming copy, 16 bytes per lane, grid-stride.
__global__ __launch_bounds__(256) void copy_probe_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                         size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

hipError_t launch_mfma_probe(int workgroups, int iters, int* sink, hipStream_t stream) {
    hipLaunchKernelGGL(mfma_i8_probe_kernel, dim3(workgroups), dim3(256), 0, stream, iters, sink);
    return hipGetLastError();
}

hipError_t launch_copy_probe(const void* src, void* dst, size_t bytes, hipStream_t stream) {
    hipLaunchKernelGGL(copy_probe_kernel, dim3(256 * 16), dim3(256), 0, stream, static_cast<const uint4*>(src),
                       static_cast<uint4*>(dst), bytes / 16);
    return hipGetLastError();
}

}  // namespace quik
