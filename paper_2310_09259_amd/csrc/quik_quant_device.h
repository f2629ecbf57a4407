// Device helpers shared by the fused quantization kernel and the unfused (ablation) kernels.
// Private to the shared library.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace quik {
namespace quant_dev {

constexpr int kBlock = 256;

__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

union Chunk {          // 8 fp16 values = one 128-bit load
    uint4 u;
    __half h[8];
};

// Builds mask[w] (bit b set <=> column 32w+b is an outlier) and pre[w] (number of
// outlier columns below 32w) for w < nwords.  Indices outside [0, K) are ignored.
__device__ inline void build_outlier_map(const int32_t* __restrict__ idx, int n_out, int K, int nwords,
                                  uint32_t* mask, uint32_t* pre, uint32_t* wave_tot) {
    const int tid = threadIdx.x;
    for (int w = tid; w < nwords; w += kBlock) mask[w] = 0u;
    __syncthreads();
    for (int j = tid; j < n_out; j += kBlock) {
        int c = idx[j];
        if (c >= 0 && c < K) atomicOr(&mask[c >> 5], 1u << (c & 31));
    }
    __syncthreads();
    // exclusive scan of popcounts; each thread owns `per` consecutive words
    const int per = (nwords + kBlock - 1) / kBlock;
    const int w0 = tid * per;
    uint32_t local = 0;
    for (int i = 0; i < per; ++i)
        if (w0 + i < nwords) local += __popc(mask[w0 + i]);
    uint32_t incl = local;
    const int lane = tid & 63, wv = tid >> 6;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t n = __shfl_up(incl, o, 64);
        if (lane >= o) incl += n;
    }
    if (lane == 63) wave_tot[wv] = incl;
    __syncthreads();
    uint32_t offs = 0;
    for (int i = 0; i < wv; ++i) offs += wave_tot[i];
    uint32_t run = offs + incl - local;
    for (int i = 0; i < per; ++i)
        if (w0 + i < nwords) {
            pre[w0 + i] = run;
            run += __popc(mask[w0 + i]);
        }
    __syncthreads();
}

// Unsigned code rne((x - mn) * inv) in the low BITS bits of the result (upper bits are
// mantissa garbage; callers mask).
__device__ __forceinline__ uint32_t code_bits(__half h, float mn, float inv) {
    float d = __half2float(h) - mn;
    float u = d * inv;
    float v = u + 12582912.0f;                    // 1.5 * 2^23
    return __float_as_uint(v);
}

}  // namespace quant_dev
}  // namespace quik
