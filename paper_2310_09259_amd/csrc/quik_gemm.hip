// Integer GEMM + dequantization epilogue + fp16 outlier GEMM for gfx950
// (Algorithm 1 of arXiv 2310.09259: "INTmatmul", "Dequantization", "FPmatmul" and
// the final add; epilogue fusion as in Section 3.4).
//
// gfx950 has no 4-bit integer MFMA, so packed nibbles travel HBM -> LDS -> VGPR
// still packed and are widened in registers: for a 32-bit word w holding eight
// two's-complement nibbles, (w & 0xF0F0F0F0) and ((w << 4) & 0xF0F0F0F0) are two
// int8x4 vectors holding 16x the odd and 16x the even nibbles.  Doing the same to
// both operands makes every product 256x too large, exactly; the INT32 accumulator
// is shifted right by 8 at the end.  A dot product does not care in which order k
// is visited as long as both operands agree, so the odd/even split needs no
// re-interleaving.  Headroom: K_b * 64 * 256 < 2^31 requires K_b < 131072.
//
// MFMA shape: v_mfma_i32_32x32x32_i8.  First operand = activations (32 token
// rows), second = weights (32 output channels).  Lane l supplies row/column l%32
// and the k-group l/32; it receives output column l%32 and rows
// 8*(r/4) + 4*(l/32) + r%4 in accumulator register r.  The fp16 outlier product
// uses v_mfma_f32_32x32x16_f16, whose accumulator has the same layout, so the
// dequantized tile is simply the C operand of the outlier loop.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "quik_kernels.h"

namespace quik {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

constexpr int kThreads = 256;
constexpr int kXcds = 8;

// Maps the hardware workgroup id (dealt round-robin over the 8 XCDs) to a logical
// tile id such that each XCD works on a contiguous range of logical tiles and so
// re-uses operand panels out of its own L2.
__device__ __forceinline__ int xcd_contiguous_id(int b, int nblk) {
    int x = b % kXcds, local = b / kXcds;
    int q = nblk / kXcds, r = nblk % kXcds;
    int start = (x < r) ? x * (q + 1) : r * (q + 1) + (x - r) * q;
    return start + local;
}

template <int BITS>
__device__ __forceinline__ void widen(const uint4& w, v4i& op0, v4i& op1) {
    if constexpr (BITS == 4) {
        constexpr uint32_t M = 0xF0F0F0F0u;
        op0 = v4i{(int)((w.x << 4) & M), (int)(w.x & M), (int)((w.y << 4) & M), (int)(w.y & M)};
        op1 = v4i{(int)((w.z << 4) & M), (int)(w.z & M), (int)((w.w << 4) & M), (int)(w.w & M)};
    } else {
        op0 = v4i{(int)w.x, (int)w.y, (int)w.z, (int)w.w};
        op1 = op0;
    }
}

// BM x BN output tile per workgroup, WM x WN waves, BKB bytes of every packed row
// per LDS stage.  RAW: write INT32 accumulators instead of running the epilogue.
template <int BITS, int BM, int BN, int WM, int WN, int BKB, bool RAW>
__global__ __launch_bounds__(kThreads) void gemm_kernel(GemmArgs a) {
    static_assert(WM * WN == 4, "four waves per workgroup");
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;   // MFMA tiles per wave
    constexpr int CPR = BKB / 16;                         // 16-byte chunks per row per stage
    constexpr int LDS_STRIDE = BKB + 16;                  // padded row stride (bank spread)
    constexpr int A_CHUNKS = BM * CPR / kThreads, B_CHUNKS = BN * CPR / kThreads;
    static_assert(BM * CPR % kThreads == 0 && BN * CPR % kThreads == 0, "tile/threads mismatch");
    constexpr int KSUB = BKB / 32;                        // 32-byte sub-steps per stage
    constexpr int SHIFT = (BITS == 4) ? 8 : 0;

    __shared__ __align__(16) uint8_t lds_a[2][BM * LDS_STRIDE];
    __shared__ __align__(16) uint8_t lds_b[2][BN * LDS_STRIDE];
    __shared__ float lds_sa[BM];   // scaleAct per tile row
    __shared__ float lds_sh[BM];   // zeroAct + halfRange * scaleAct per tile row

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, g = lane >> 5;

    const int tiles_m = (a.T + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    const int id = xcd_contiguous_id(blockIdx.x, tiles_m * tiles_n);
    const int t0 = (id % tiles_m) * BM, n0 = (id / tiles_m) * BN;

    const uint8_t* __restrict__ gA = static_cast<const uint8_t*>(a.xq);
    const uint8_t* __restrict__ gB = static_cast<const uint8_t*>(a.w_q);
    const int row_bytes = a.K_b * BITS / 8;
    const int nk = (row_bytes + BKB - 1) / BKB;

    if constexpr (!RAW) {
        for (int r = tid; r < BM; r += kThreads) {
            int t = t0 + r;
            float s = (t < a.T) ? a.scale[t] : 0.0f;
            float z = (t < a.T) ? a.zero[t] : 0.0f;
            lds_sa[r] = s;
            lds_sh[r] = z + (float)(1 << (BITS - 1)) * s;
        }
    }

    // global -> register staging of one K stage
    uint4 ga[A_CHUNKS], gb[B_CHUNKS];
    auto load_stage = [&](int kt) {
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            int c = tid + i * kThreads, r = c / CPR, ch = c % CPR;
            int t = min(t0 + r, a.T - 1);
            int off = kt * BKB + ch * 16;
            ga[i] = (off < a.ldq) ? *reinterpret_cast<const uint4*>(gA + (size_t)t * a.ldq + off)
                                  : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) {
            int c = tid + i * kThreads, r = c / CPR, ch = c % CPR;
            int n = min(n0 + r, a.N - 1);
            int off = kt * BKB + ch * 16;
            gb[i] = (off < a.ldw) ? *reinterpret_cast<const uint4*>(gB + (size_t)n * a.ldw + off)
                                  : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            int c = tid + i * kThreads, r = c / CPR, ch = c % CPR;
            *reinterpret_cast<uint4*>(&lds_a[buf][r * LDS_STRIDE + ch * 16]) = ga[i];
        }
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) {
            int c = tid + i * kThreads, r = c / CPR, ch = c % CPR;
            *reinterpret_cast<uint4*>(&lds_b[buf][r * LDS_STRIDE + ch * 16]) = gb[i];
        }
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    load_stage(0);
    store_stage(0);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_stage(kt + 1);
        const uint8_t* pa = &lds_a[buf][(wm * TM * 32 + l32) * LDS_STRIDE + g * 16];
        const uint8_t* pb = &lds_b[buf][(wn * TN * 32 + l32) * LDS_STRIDE + g * 16];
#pragma unroll
        for (int ks = 0; ks < KSUB; ++ks) {
            v4i a0[TM], a1[TM], b0[TN], b1[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                uint4 w = *reinterpret_cast<const uint4*>(pa + i * 32 * LDS_STRIDE + ks * 32);
                widen<BITS>(w, a0[i], a1[i]);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                uint4 w = *reinterpret_cast<const uint4*>(pb + j * 32 * LDS_STRIDE + ks * 32);
                widen<BITS>(w, b0[j], b1[j]);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0[i], b0[j], acc[i][j], 0, 0, 0);
                    if constexpr (BITS == 4)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1[i], b1[j], acc[i][j], 0, 0, 0);
                }
        }
        if (kt + 1 < nk) store_stage(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue
    const int tw = t0 + wm * TM * 32, nw = n0 + wn * TN * 32;
    if constexpr (RAW) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int n = nw + j * 32 + l32;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int t = tw + i * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (t < a.T && n < a.N) a.acc[(size_t)t * a.ldacc + n] = acc[i][j][r] >> SHIFT;
                }
            }
    } else {
        const __half* __restrict__ wsc = static_cast<const __half*>(a.w_scale);
        const __half* __restrict__ bias = static_cast<const __half*>(a.bias);
        v16f cf[TM][TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            int n = min(nw + j * 32 + l32, a.N - 1);
            float sw = __half2float(wsc[n]);
            float wr = a.w_reduced[n];
            float bv = bias ? __half2float(bias[n]) : 0.0f;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int lr = wm * TM * 32 + i * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                    float v = (float)(acc[i][j][r] >> SHIFT);
                    cf[i][j][r] = v * (lds_sa[lr] * sw) + (lds_sh[lr] * wr + bv);
                }
        }
        // fp16 outlier product accumulated on top of the dequantized tile
        const __half* __restrict__ xo = static_cast<const __half*>(a.x_out);
        const __half* __restrict__ wo = static_cast<const __half*>(a.w_out);
        for (int ko = 0; ko < a.n_out; ko += 16) {
            const int kk = ko + g * 8;
            v8h fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                int t = min(tw + i * 32 + l32, a.T - 1);
                uint4 w = (kk < a.n_out) ? *reinterpret_cast<const uint4*>(xo + (size_t)t * a.ldo + kk)
                                         : make_uint4(0, 0, 0, 0);
                fa[i] = __builtin_bit_cast(v8h, w);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int n = min(nw + j * 32 + l32, a.N - 1);
                uint4 w = (kk < a.n_out) ? *reinterpret_cast<const uint4*>(wo + (size_t)n * a.ldwo + kk)
                                         : make_uint4(0, 0, 0, 0);
                fb[j] = __builtin_bit_cast(v8h, w);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    cf[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[i], fb[j], cf[i][j], 0, 0, 0);
        }
        __half* __restrict__ y = static_cast<__half*>(a.y);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int n = nw + j * 32 + l32;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int t = tw + i * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (t < a.T && n < a.N) y[(size_t)t * a.ldy + n] = __float2half(cf[i][j][r]);
                }
            }
    }
}

template <int BITS, int BM, int BN, int WM, int WN, int BKB, bool RAW>
hipError_t launch_cfg(const GemmArgs& a, hipStream_t stream) {
    int tiles = ((a.T + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    hipLaunchKernelGGL((gemm_kernel<BITS, BM, BN, WM, WN, BKB, RAW>), dim3(tiles), dim3(kThreads), 0,
                       stream, a);
    return hipGetLastError();
}

template <int BITS, bool RAW>
hipError_t dispatch(const GemmArgs& a, hipStream_t stream) {
    return launch_cfg<BITS, 128, 128, 2, 2, 64, RAW>(a, stream);
}

// one wave per output channel; lanes stride over the packed row
template <int BITS>
__global__ __launch_bounds__(kThreads) void weight_reduce_kernel(WeightReduceArgs a) {
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (n >= a.N) return;
    const uint8_t* row = static_cast<const uint8_t*>(a.w_q) + (size_t)n * a.ldw;
    const int row_bytes = a.K_b * BITS / 8;
    int s = 0;
    for (int p = lane; p < row_bytes; p += 64) {
        int b = row[p];
        if constexpr (BITS == 4) {
            s += ((b & 0xF) ^ 8) - 8;
            s += ((b >> 4) ^ 8) - 8;
        } else {
            s += (int)(int8_t)b;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0)
        a.w_reduced[n] = __half2float(static_cast<const __half*>(a.w_scale)[n]) * (float)s;
}

}  // namespace

hipError_t launch_gemm(const GemmArgs& a, hipStream_t stream) {
    const bool raw = a.y == nullptr;
    if (a.bits == 4) return raw ? dispatch<4, true>(a, stream) : dispatch<4, false>(a, stream);
    return raw ? dispatch<8, true>(a, stream) : dispatch<8, false>(a, stream);
}

hipError_t launch_weight_reduce(const WeightReduceArgs& a, hipStream_t stream) {
    int blocks = (a.N + 3) / 4;
    if (a.bits == 4)
        hipLaunchKernelGGL(weight_reduce_kernel<4>, dim3(blocks), dim3(kThreads), 0, stream, a);
    else
        hipLaunchKernelGGL(weight_reduce_kernel<8>, dim3(blocks), dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

}  // namespace quik
