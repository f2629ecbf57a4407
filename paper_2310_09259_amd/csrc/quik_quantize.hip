// Fused split + per-token quantization kernel for gfx950 (Algorithm 1, "split" and
// "Quantization"; fusion as in Section 3.4 of arXiv 2310.09259).
//
// One group of TPR threads owns one token row.  The row is read from HBM exactly
// once with 128-bit loads and kept in registers; the three passes of the paper's
// fused kernel (min/max over the non-outlier elements, quantization of the
// non-outliers, moving the outliers) all run from those registers or from cache.
//
// Outlier columns are described by a bitmask over the K columns plus an exclusive
// prefix count per 32-column word, both built once per workgroup in LDS.  A thread
// that holds columns [k0, k0+8) derives from them which of its elements are base
// columns and the position of its first base element in the packed output row.
// Its (at most 8) quantized codes are squeezed into one 32/64-bit value and OR-ed
// into an LDS image of the packed row at an arbitrary bit offset, so the packed
// row leaves the CU as full, aligned 128-bit stores.
//
// Bit exactness: binary32 arithmetic, one IEEE division and one IEEE reciprocal
// per row, a subtract and a multiply per element (never contracted).  Rounding to
// the nearest integer, ties to even, is done by adding 1.5 * 2^23: the sum's unit
// in the last place is 1 there, so the adder's own round-to-nearest-even performs
// the rounding and the low mantissa bits are the integer.  For finite inputs
// (x - min) * (1 / scale) lies in [0, (2^bits - 1) * (1 + 2^-22)], so the clamp of
// the method can never fire and is replaced by a bit mask.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "quik_kernels.h"
#include "quik_quant_device.h"

namespace quik {

namespace {

using namespace quant_dev;

// Removes the element at position p (element width W bits) from the packed value w,
// closing the gap.
template <typename U, int W>
__device__ __forceinline__ U drop_element(U w, int p) {
    const U low = (p == 0) ? U(0) : (~U(0) >> (sizeof(U) * 8 - W * p));
    return (w & low) | ((w >> W) & ~low);
}

// Quantizes one chunk, squeezes its base elements together and ORs them into the LDS
// row image at element position base0.  Elements at positions >= K_b are dropped.
template <int BITS>
__device__ __forceinline__ int emit_chunk(const Chunk& c, uint32_t m8, int base0, int K_b,
                                          float mn, float inv, uint32_t* stage) {
    if constexpr (BITS == 4) {
        uint32_t w = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) w |= (code_bits(c.h[i], mn, inv) & 0xFu) << (4 * i);
        int cnt = 8;
        while (m8) {                               // rare: squeeze out outlier positions, highest first
            int p = 31 - __clz(m8);
            w = drop_element<uint32_t, 4>(w, p);
            m8 &= ~(1u << p);
            --cnt;
        }
        if (base0 >= K_b || cnt == 0) return 0;
        int room = K_b - base0;
        if (room < cnt) cnt = room;
        const uint32_t keep = (cnt < 8) ? ((1u << (4 * cnt)) - 1u) : 0xFFFFFFFFu;
        w &= keep;                                 // unsigned codes 0..15 of the kept elements
        // sum of the codes at even positions of the packed row (nibbles base0-parity, +2, ...)
        const uint32_t sel = (w >> (4 * (base0 & 1))) & 0x0F0F0F0Fu;
        const int even_sum = (int)__builtin_amdgcn_sad_u8(sel, 0u, 0u);
        w = (w ^ 0x88888888u) & keep;              // code - halfRange as two's complement nibbles
        uint32_t bit = (uint32_t)base0 * 4u;
        uint32_t wi = bit >> 5, sh = bit & 31u;
        uint32_t lo = w << sh;
        uint32_t hi = sh ? (w >> (32u - sh)) : 0u;
        if (lo) atomicOr(&stage[wi], lo);
        if (hi) atomicOr(&stage[wi + 1], hi);
        return even_sum;
    } else {
        uint64_t w = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) w |= (uint64_t)(code_bits(c.h[i], mn, inv) & 0xFFu) << (8 * i);
        w ^= 0x8080808080808080ull;
        int cnt = 8;
        while (m8) {
            int p = 31 - __clz(m8);
            w = drop_element<uint64_t, 8>(w, p);
            m8 &= ~(1u << p);
            --cnt;
        }
        if (base0 >= K_b || cnt == 0) return 0;
        int room = K_b - base0;
        if (cnt < 8) w &= (1ull << (8 * cnt)) - 1ull;
        if (room < 8) w &= (1ull << (8 * room)) - 1ull;
        uint32_t bit = (uint32_t)base0 * 8u;
        uint32_t wi = bit >> 5, sh = bit & 31u;
        uint64_t lo64 = w << sh;
        uint32_t p0 = (uint32_t)lo64, p1 = (uint32_t)(lo64 >> 32);
        uint32_t p2 = sh ? (uint32_t)(w >> (64u - sh)) : 0u;
        if (p0) atomicOr(&stage[wi], p0);
        if (p1) atomicOr(&stage[wi + 1], p1);
        if (p2) atomicOr(&stage[wi + 2], p2);
        return 0;
    }
}

// NCH > 0: the row is cached in NCH 128-bit registers per thread (K <= TPR*8*NCH).
// NCH == 0: any K; the second pass re-reads the row (from cache).
template <int BITS, int TPR, int NCH>
__global__ __launch_bounds__(kBlock) void quantize_kernel(
    const __half* __restrict__ x, int T, int K, int ldx, const int32_t* __restrict__ idx, int n_out,
    uint8_t* __restrict__ xq, int ldq, float* __restrict__ scale, float* __restrict__ zero,
    int32_t* __restrict__ code_sum, __half* __restrict__ x_out, int ldo) {
    constexpr int RPB = kBlock / TPR;             // rows per workgroup iteration
    extern __shared__ __align__(16) uint32_t lds[];
    const int nwords = (K + 31) >> 5;
    uint32_t* mask = lds;
    uint32_t* pre = mask + nwords;
    float* red = reinterpret_cast<float*>(pre + nwords);       // [2 * 4] wave partials
    uint32_t* wave_tot = reinterpret_cast<uint32_t*>(red + 8); // [4]
    int* red_i = reinterpret_cast<int*>(wave_tot + 4);         // [4] wave partials of the code sum
    uint32_t* stage_all = reinterpret_cast<uint32_t*>(red_i + 4);   // RPB rows of ldq bytes
    // keep the row images 16-byte aligned
    stage_all = reinterpret_cast<uint32_t*>((reinterpret_cast<uintptr_t>(stage_all) + 15) & ~(uintptr_t)15);

    const int tid = threadIdx.x;
    const int g = tid / TPR, lt = tid % TPR;
    const int K_b = K - n_out;
    const int ldq_words = ldq >> 2;
    uint32_t* stage = stage_all + (size_t)g * ldq_words;
    const int nrowblk = (T + RPB - 1) / RPB;
    const int nch_rt = (K + TPR * 8 - 1) / (TPR * 8);          // chunks per thread (runtime form)

    constexpr int NC = NCH > 0 ? NCH : 1;
    auto load_row = [&](Chunk (&cache)[NC], int rb) {
        const int t = rb * RPB + g;
        const __half* row = x + (size_t)(t < T ? t : 0) * ldx;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            int k0 = (c * TPR + lt) * 8;
            if (t < T && k0 < K) cache[c].u = *reinterpret_cast<const uint4*>(row + k0);
            else cache[c].u = make_uint4(0, 0, 0, 0);
        }
    };

    // All three passes for the row block rb; `cache` holds the row when NCH > 0.
    auto process_row = [&](const Chunk (&cache)[NC], int rb) {
        const int t = rb * RPB + g;
        const bool valid = t < T;
        const __half* row = x + (size_t)(valid ? t : 0) * ldx;

        for (int i = lt; i < ldq_words; i += TPR) stage[i] = 0u;

        // ---- pass 1: min/max over base columns
        float mn = __builtin_inff(), mx = -__builtin_inff();
        auto scan_chunk = [&](const Chunk& c, int k0) {
            uint32_t m8 = (mask[k0 >> 5] >> (k0 & 31)) & 0xFFu;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float f = __half2float(c.h[i]);
                bool keep = !((m8 >> i) & 1u);
                mn = keep ? fminf(mn, f) : mn;
                mx = keep ? fmaxf(mx, f) : mx;
            }
        };
        if constexpr (NCH > 0) {
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                int k0 = (c * TPR + lt) * 8;
                if (valid && k0 < K) scan_chunk(cache[c], k0);
            }
        } else {
            for (int c = 0; c < nch_rt; ++c) {
                int k0 = (c * TPR + lt) * 8;
                if (valid && k0 < K) {
                    Chunk ch;
                    ch.u = *reinterpret_cast<const uint4*>(row + k0);
                    scan_chunk(ch, k0);
                }
            }
        }
        mn = wave_min(mn);
        mx = wave_max(mx);
        if constexpr (TPR > 64) {
            const int wv = tid >> 6;
            if ((tid & 63) == 0) { red[wv] = mn; red[4 + wv] = mx; }
            __syncthreads();
            mn = fminf(fminf(red[0], red[1]), fminf(red[2], red[3]));
            mx = fmaxf(fmaxf(red[4], red[5]), fmaxf(red[6], red[7]));
        } else {
            __syncthreads();                       // row image zeroed by all lanes
        }
        mn = mn + 0.0f;                            // -0 -> +0
        const float range = mx - mn;
        const float s = (range == 0.0f) ? 1.0f : range / (float)((1 << BITS) - 1);
        const float inv = 1.0f / s;
        if (valid && lt == 0) { scale[t] = s; zero[t] = mn; }

        // ---- pass 2: quantize the base elements into the LDS row image
        int esum = 0;                              // unsigned codes at even positions (4-bit only)
        auto quant_chunk = [&](const Chunk& c, int k0) {
            uint32_t word = mask[k0 >> 5];
            uint32_t below = pre[k0 >> 5] + __popc(word & ((1u << (k0 & 31)) - 1u));
            uint32_t m8 = (word >> (k0 & 31)) & 0xFFu;
            esum += emit_chunk<BITS>(c, m8, k0 - (int)below, K_b, mn, inv, stage);
        };
        if constexpr (NCH > 0) {
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                int k0 = (c * TPR + lt) * 8;
                if (valid && k0 < K) quant_chunk(cache[c], k0);
            }
        } else {
            for (int c = 0; c < nch_rt; ++c) {
                int k0 = (c * TPR + lt) * 8;
                if (valid && k0 < K) {
                    Chunk ch;
                    ch.u = *reinterpret_cast<const uint4*>(row + k0);
                    quant_chunk(ch, k0);
                }
            }
        }
        if constexpr (BITS == 4) {
            // sum over even positions of the signed codes (the GEMM's correction term for the
            // cheap operand widening); wave partials are combined after the barrier below
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) esum += __shfl_xor(esum, o, 64);
            if constexpr (TPR > 64) {
                if ((tid & 63) == 0) red_i[tid >> 6] = esum;
            }
        }
        __syncthreads();
        if constexpr (BITS == 4) {
            if constexpr (TPR > 64) esum = red_i[0] + red_i[1] + red_i[2] + red_i[3];
            if (valid && lt == 0 && code_sum) code_sum[t] = esum - 8 * (K_b >> 1);
        }

        // ---- write the packed row (including its zero padding up to ldq); 4-bit rows leave with
        // the two nibbles of every byte swapped: element 2p in the high nibble
        if (valid) {
            uint4* dst = reinterpret_cast<uint4*>(xq + (size_t)t * ldq);
            const uint4* src = reinterpret_cast<const uint4*>(stage);
            for (int i = lt; i < (ldq >> 4); i += TPR) {
                uint4 v = src[i];
                if constexpr (BITS == 4) {
                    auto sw = [](uint32_t w) { return ((w & 0x0F0F0F0Fu) << 4) | ((w >> 4) & 0x0F0F0F0Fu); };
                    v = make_uint4(sw(v.x), sw(v.y), sw(v.z), sw(v.w));
                }
                dst[i] = v;
            }
            // ---- pass 3: move the outlier columns
            for (int j = lt; j < n_out; j += TPR) {
                int c = idx[j];
                __half v = (c >= 0 && c < K) ? row[c] : __ushort_as_half((unsigned short)0);
                x_out[(size_t)t * ldo + j] = v;
            }
        }
        __syncthreads();                           // before the next row clears the image
    };

    if constexpr (NCH > 0) {
        // Row loads do not depend on the outlier map: the first row's loads are issued before
        // the map is built, and from then on the next row is fetched into a second register
        // set while the current one is processed.
        Chunk ca[NC], cb[NC];
        int rb = blockIdx.x;
        if (rb < nrowblk) load_row(ca, rb);
        build_outlier_map(idx, n_out, K, nwords, mask, pre, wave_tot);
        while (rb < nrowblk) {
            int nx = rb + gridDim.x;
            if (nx < nrowblk) load_row(cb, nx);
            process_row(ca, rb);
            rb = nx;
            if (rb >= nrowblk) break;
            nx = rb + gridDim.x;
            if (nx < nrowblk) load_row(ca, nx);
            process_row(cb, rb);
            rb = nx;
        }
    } else {
        build_outlier_map(idx, n_out, K, nwords, mask, pre, wave_tot);
        Chunk none[NC];
        none[0].u = make_uint4(0, 0, 0, 0);
        for (int rb = blockIdx.x; rb < nrowblk; rb += gridDim.x) process_row(none, rb);
    }
}

template <int BITS, int TPR, int NCH>
hipError_t launch(const QuantizeArgs& a, hipStream_t stream) {
    constexpr int RPB = kBlock / TPR;
    const int nwords = (a.K + 31) >> 5;
    size_t lds = (size_t)nwords * 8 + 8 * 4 + 4 * 4 + 4 * 4 + 16 + (size_t)RPB * a.ldq;
    int nrowblk = (a.T + RPB - 1) / RPB;
    // a bounded grid: the outlier map is built once per workgroup and the rows of a workgroup
    // are software-pipelined (next row's loads in flight while the current one is processed)
    int grid = nrowblk < 2048 ? nrowblk : 2048;
    hipLaunchKernelGGL((quantize_kernel<BITS, TPR, NCH>), dim3(grid), dim3(kBlock), lds, stream,
                       (const __half*)a.x, a.T, a.K, a.ldx, a.idx, a.n_out, (uint8_t*)a.xq, a.ldq,
                       a.scale, a.zero, a.code_sum, (__half*)a.x_out, a.ldo);
    return hipGetLastError();
}

template <int BITS>
hipError_t dispatch(const QuantizeArgs& a, hipStream_t stream) {
    const int K = a.K;
    if (K <= 64 * 8 * 1) return launch<BITS, 64, 1>(a, stream);
    if (K <= 64 * 8 * 2) return launch<BITS, 64, 2>(a, stream);
    if (K <= 64 * 8 * 4) return launch<BITS, 64, 4>(a, stream);
    if (K <= 64 * 8 * 8) return launch<BITS, 64, 8>(a, stream);
    if (K <= 256 * 8 * 4) return launch<BITS, 256, 4>(a, stream);
    if (K <= 256 * 8 * 8) return launch<BITS, 256, 8>(a, stream);
    return launch<BITS, 256, 0>(a, stream);
}

}  // namespace

hipError_t launch_quantize(const QuantizeArgs& a, hipStream_t stream) {
    return a.bits == 4 ? dispatch<4>(a, stream) : dispatch<8>(a, stream);
}

}  // namespace quik
