// Unfused building blocks of the layer, for the fusion ablation of Section 3.4 of
// arXiv 2310.09259 ("Performance Impact": version 1 = unfused quantization and
// dequantization, version 2 = fused quantization only, version 3 = both fused).
//
// The unfused quantization follows the paper's description of the naive pipeline: one
// read-and-write pass for the outlier part, one for the base part, two read passes for the
// per-token minimum and maximum, one read-and-write pass for the quantization itself.  The
// unfused dequantization reads the INT32 accumulators and the result of the separate outlier
// GEMM back from memory (kept in fp32 so that the output meets the same error bar as the fused
// layer; an fp16 intermediate would add a second rounding).  Each kernel is a plain, coalesced, one-pass kernel: the
// point of the ablation is the extra memory trips and launches, not slow kernels.
// The arithmetic is identical to the fused kernels (bit-exact packed activations).
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "quik_kernels.h"
#include "quik_quant_device.h"

namespace quik {

namespace {

using namespace quant_dev;

// pass A: x_out[t, j] = x[t, idx[j]]
__global__ __launch_bounds__(kBlock) void split_outliers_kernel(const __half* __restrict__ x, int T, int K,
                                                                int ldx, const int32_t* __restrict__ idx,
                                                                int n_out, __half* __restrict__ x_out, int ldo) {
    const long i = (long)blockIdx.x * kBlock + threadIdx.x;
    if (i >= (long)T * n_out) return;
    const int t = (int)(i / n_out), j = (int)(i % n_out);
    const int c = idx[j];
    x_out[(size_t)t * ldo + j] = (c >= 0 && c < K) ? x[(size_t)t * ldx + c] : __ushort_as_half((unsigned short)0);
}

// pass B: x_base[t, rank(k)] = x[t, k] for every base column k (one workgroup per row block)
__global__ __launch_bounds__(kBlock) void split_base_kernel(const __half* __restrict__ x, int T, int K, int ldx,
                                                            const int32_t* __restrict__ idx, int n_out,
                                                            __half* __restrict__ x_base, int ldb) {
    extern __shared__ __align__(16) uint32_t lds[];
    const int nwords = (K + 31) >> 5;
    uint32_t* mask = lds;
    uint32_t* pre = mask + nwords;
    uint32_t* wave_tot = pre + nwords;
    build_outlier_map(idx, n_out, K, nwords, mask, pre, wave_tot);
    const int K_b = K - n_out;
    for (int t = blockIdx.x; t < T; t += gridDim.x)
        for (int k = threadIdx.x; k < K; k += kBlock) {
            const uint32_t word = mask[k >> 5];
            if ((word >> (k & 31)) & 1u) continue;
            const int pos = k - (int)(pre[k >> 5] + __popc(word & ((1u << (k & 31)) - 1u)));
            if (pos < K_b) x_base[(size_t)t * ldb + pos] = x[(size_t)t * ldx + k];
        }
}

// passes C and D: per-row minimum / maximum of x_base (two separate read passes)
template <bool IS_MAX>
__global__ __launch_bounds__(kBlock) void row_extreme_kernel(const __half* __restrict__ x_base, int T, int K_b,
                                                             int ldb, float* __restrict__ out) {
    __shared__ float red[4];
    for (int t = blockIdx.x; t < T; t += gridDim.x) {
        float v = IS_MAX ? -__builtin_inff() : __builtin_inff();
        for (int k = threadIdx.x; k < K_b; k += kBlock) {
            float f = __half2float(x_base[(size_t)t * ldb + k]);
            v = IS_MAX ? fmaxf(v, f) : fminf(v, f);
        }
        v = IS_MAX ? wave_max(v) : wave_min(v);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
        __syncthreads();
        if (threadIdx.x == 0) {
            float r = IS_MAX ? fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]))
                             : fminf(fminf(red[0], red[1]), fminf(red[2], red[3]));
            out[t] = r;
        }
        __syncthreads();
    }
}

// pass E: quantize the contiguous base part; also derives scale / zero from the two extremes
template <int BITS>
__global__ __launch_bounds__(kBlock) void quantize_base_kernel(const __half* __restrict__ x_base, int T, int K_b,
                                                               int ldb, const float* __restrict__ row_min,
                                                               const float* __restrict__ row_max,
                                                               uint8_t* __restrict__ xq, int ldq,
                                                               float* __restrict__ scale, float* __restrict__ zero,
                                                               int32_t* __restrict__ code_sum) {
    __shared__ int red_i[kBlock / 64];
    asm volatile("" ::: "v39");                    // keep the highest allocated register unused
    for (int t = blockIdx.x; t < T; t += gridDim.x) {
        const float mn = row_min[t] + 0.0f;
        const float range = row_max[t] - mn;
        const float s = (range == 0.0f) ? 1.0f : range / (float)((1 << BITS) - 1);
        const float inv = 1.0f / s;
        if (threadIdx.x == 0) { scale[t] = s; zero[t] = mn; }
        uint8_t* dst = xq + (size_t)t * ldq;
        const __half* src = x_base + (size_t)t * ldb;
        if constexpr (BITS == 4) {
            // one byte (two elements) per thread step; K_b is even.  Activation bytes keep element
            // 2p in the high nibble; the signed codes at even positions are summed per row.
            int esum = 0;
            for (int p = threadIdx.x; p < ldq; p += kBlock) {
                uint32_t b = 0;
                if (2 * p < K_b) {
                    uint32_t even = code_bits(src[2 * p], mn, inv) & 0xFu;
                    uint32_t odd = code_bits(src[2 * p + 1], mn, inv) & 0xFu;
                    b = (odd | (even << 4)) ^ 0x88u;
                    esum += (int)even - 8;
                }
                dst[p] = (uint8_t)b;
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) esum += __shfl_xor(esum, o, 64);
            if ((threadIdx.x & 63) == 0) red_i[threadIdx.x >> 6] = esum;
            __syncthreads();
            if (threadIdx.x == 0 && code_sum) {
                int tot = 0;
                for (int w = 0; w < kBlock / 64; ++w) tot += red_i[w];
                code_sum[t] = tot;
            }
            __syncthreads();
        } else {
            for (int p = threadIdx.x; p < ldq; p += kBlock)
                dst[p] = (p < K_b) ? (uint8_t)((code_bits(src[p], mn, inv) & 0xFFu) ^ 0x80u) : (uint8_t)0;
        }
    }
}

// unfused dequantization: y = acc*scale*sW + (zero + halfRange*scale)*wRed (+bias) + resultFP
template <int BITS>
__global__ __launch_bounds__(kBlock) void dequant_add_kernel(const int32_t* __restrict__ acc, int ldacc,
                                                             const float* __restrict__ scale,
                                                             const float* __restrict__ zero,
                                                             const __half* __restrict__ w_scale,
                                                             const float* __restrict__ w_reduced,
                                                             const __half* __restrict__ bias,
                                                             const float* __restrict__ result_fp, int ldr,
                                                             int T, int N, __half* __restrict__ y, int ldy) {
    const long i = (long)blockIdx.x * kBlock + threadIdx.x;
    if (i >= (long)T * N) return;
    const int t = (int)(i / N), n = (int)(i % N);
    const float sa = scale[t];
    const float sh = zero[t] + (float)(1 << (BITS - 1)) * sa;
    const float bv = bias ? __half2float(bias[n]) : 0.0f;
    float v = __builtin_fmaf((float)acc[(size_t)t * ldacc + n], sa * __half2float(w_scale[n]),
                             __builtin_fmaf(sh, w_reduced[n], bv));
    if (result_fp) v += result_fp[(size_t)t * ldr + n];
    y[(size_t)t * ldy + n] = __float2half(v);
}

inline int capped(long n) { return (int)(n < 4096 ? (n < 1 ? 1 : n) : 4096); }

}  // namespace

hipError_t launch_unfused_quantize(const QuantizeArgs& a, void* x_base, int ldb, float* row_min,
                                   float* row_max, hipStream_t stream) {
    const int K_b = a.K - a.n_out;
    if (a.n_out > 0) {
        long n = (long)a.T * a.n_out;
        hipLaunchKernelGGL(split_outliers_kernel, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0,
                           stream, (const __half*)a.x, a.T, a.K, a.ldx, a.idx, a.n_out, (__half*)a.x_out, a.ldo);
    }
    const int nwords = (a.K + 31) >> 5;
    hipLaunchKernelGGL(split_base_kernel, dim3(capped(a.T)), dim3(kBlock), (size_t)nwords * 8 + 16, stream,
                       (const __half*)a.x, a.T, a.K, a.ldx, a.idx, a.n_out, (__half*)x_base, ldb);
    hipLaunchKernelGGL(row_extreme_kernel<false>, dim3(capped(a.T)), dim3(kBlock), 0, stream,
                       (const __half*)x_base, a.T, K_b, ldb, row_min);
    hipLaunchKernelGGL(row_extreme_kernel<true>, dim3(capped(a.T)), dim3(kBlock), 0, stream,
                       (const __half*)x_base, a.T, K_b, ldb, row_max);
    if (a.bits == 4)
        hipLaunchKernelGGL(quantize_base_kernel<4>, dim3(capped(a.T)), dim3(kBlock), 0, stream,
                           (const __half*)x_base, a.T, K_b, ldb, row_min, row_max, (uint8_t*)a.xq, a.ldq,
                           a.scale, a.zero, a.code_sum);
    else
        hipLaunchKernelGGL(quantize_base_kernel<8>, dim3(capped(a.T)), dim3(kBlock), 0, stream,
                           (const __half*)x_base, a.T, K_b, ldb, row_min, row_max, (uint8_t*)a.xq, a.ldq,
                           a.scale, a.zero, a.code_sum);
    return hipGetLastError();
}

hipError_t launch_dequant_add(const GemmArgs& a, const int32_t* acc, int ldacc, const void* result_fp,
                              int ldr, hipStream_t stream) {
    long n = (long)a.T * a.N;
    dim3 grid((unsigned)((n + kBlock - 1) / kBlock));
    if (a.bits == 4)
        hipLaunchKernelGGL(dequant_add_kernel<4>, grid, dim3(kBlock), 0, stream, acc, ldacc, a.scale, a.zero,
                           (const __half*)a.w_scale, a.w_reduced, (const __half*)a.bias,
                           (const float*)result_fp, ldr, a.T, a.N, (__half*)a.y, a.ldy);
    else
        hipLaunchKernelGGL(dequant_add_kernel<8>, grid, dim3(kBlock), 0, stream, acc, ldacc, a.scale, a.zero,
                           (const __half*)a.w_scale, a.w_reduced, (const __half*)a.bias,
                           (const float*)result_fp, ldr, a.T, a.N, (__half*)a.y, a.ldy);
    return hipGetLastError();
}

}  // namespace quik
