// Device helpers shared by the fused quantization kernel and the unfused (ablation) kernels.
// Private to the shared library.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace quik {
namespace quant_dev {

constexpr int kBlock = 256;

// Wave-wide reductions whose result every lane receives.  Four DPP steps (two quad permutes, the
// half-row and the row mirror) leave each row of 16 lanes holding its row's result; the four row
// results are combined through scalar registers.  No LDS round trips (a butterfly of cross-lane
// shuffles costs six dependent LDS-routed permutes per reduction).
template <typename F>
__device__ __forceinline__ int wave_reduce_bits(int v, F op) {
    v = op(v, __builtin_amdgcn_mov_dpp(v, 0xB1, 0xF, 0xF, true));    // quad_perm [1,0,3,2]
    v = op(v, __builtin_amdgcn_mov_dpp(v, 0x4E, 0xF, 0xF, true));    // quad_perm [2,3,0,1]
    v = op(v, __builtin_amdgcn_mov_dpp(v, 0x141, 0xF, 0xF, true));   // row_half_mirror
    v = op(v, __builtin_amdgcn_mov_dpp(v, 0x140, 0xF, 0xF, true));   // row_mirror
    const int r0 = __builtin_amdgcn_readlane(v, 0), r1 = __builtin_amdgcn_readlane(v, 16);
    const int r2 = __builtin_amdgcn_readlane(v, 32), r3 = __builtin_amdgcn_readlane(v, 48);
    return op(op(r0, r1), op(r2, r3));
}
__device__ __forceinline__ float wave_min(float v) {
    return __int_as_float(wave_reduce_bits(__float_as_int(v), [](int a, int b) {
        return __float_as_int(fminf(__int_as_float(a), __int_as_float(b)));
    }));
}
__device__ __forceinline__ float wave_max(float v) {
    return __int_as_float(wave_reduce_bits(__float_as_int(v), [](int a, int b) {
        return __float_as_int(fmaxf(__int_as_float(a), __int_as_float(b)));
    }));
}
__device__ __forceinline__ int wave_sum(int v) {
    return wave_reduce_bits(v, [](int a, int b) { return a + b; });
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
