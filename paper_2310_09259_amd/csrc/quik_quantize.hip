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
// holds the same columns [k0, k0+8) of every row it works on, so everything that
// follows from the outlier set alone is computed once per workgroup and kept in
// registers: which of its elements are base columns, where its first base element
// lands in the packed row, the bit masks that squeeze outlier positions out of a
// packed chunk.  Per row and element that leaves: one half->float conversion, the
// subtract, the multiply and the rounding add of the method, and one shift-add that
// packs the code.
//   pass 1: outlier halves are overwritten with a quiet NaN, which the packed fp16
//           minimum/maximum instructions ignore (IEEE minNum/maxNum); fp16 min/max
//           are exact, so this equals the binary32 min/max of the method;
//   pass 2: outlier halves are overwritten with the row minimum (code 0) so that
//           their huge quotients cannot disturb neighbouring codes, then squeezed out.
// The (at most 8) codes of a chunk are OR-ed into an LDS image of the packed row at
// an arbitrary bit offset, so the packed row leaves the CU as full, aligned 128-bit
// stores.  With one wave per row (K <= 4096) nothing in the row loop needs a
// workgroup barrier: a wave's LDS operations execute in order.
//
// Bit exactness: binary32 arithmetic, one IEEE division and one IEEE reciprocal
// per row, a subtract and a multiply per element (never contracted).  Rounding to
// the nearest integer, ties to even, is done by adding 1.5 * 2^23: the sum's unit
// in the last place is 1 there, so the adder's own round-to-nearest-even performs
// the rounding, and the sum's bit pattern is 0x4B400000 + code.  For finite inputs
// (x - min) * (1 / scale) lies in [0, (2^bits - 1) * (1 + 2^-22)], so the clamp of
// the method can never fire; the codes of a chunk are accumulated with shift-adds of
// the whole bit patterns and the constant part is subtracted once.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "quik_kernels.h"
#include "quik_quant_device.h"
#include "quik_store_device.h"
#include "quik_fp6_device.h"
#include "quik_sp24_device.h"

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

// ---- fast path (row cached in registers) -------------------------------------------------

__device__ __forceinline__ uint32_t pk_min_f16(uint32_t a, uint32_t b) {
    uint32_t r;
    asm("v_pk_min_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ uint32_t pk_max_f16(uint32_t a, uint32_t b) {
    uint32_t r;
    asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
// (m & a) | (~m & b)
__device__ __forceinline__ uint32_t bit_select(uint32_t m, uint32_t a, uint32_t b) { return (m & a) | (~m & b); }

constexpr uint32_t kNaN2 = 0x7E007E00u;           // two quiet fp16 NaNs
constexpr uint32_t kMagicBits = 0x4B400000u;      // bit pattern of 1.5 * 2^23

// What a thread knows about one of its chunks from the outlier set alone.
template <int BITS>
struct ChunkPlan {
    uint32_t sel[4];      // per dword: all-ones halves where the element is an outlier (or beyond K)
    uint32_t low[3];      // 4-bit: masks that drop the three highest outlier positions (all-ones = no-op)
    uint32_t keep_lo, keep_hi;   // bits of the squeezed chunk that hold codes
    // bits 0..4: bit offset of the squeezed chunk inside its first word of the row image;
    // bit 5: the chunk starts at an odd packed position; bits 8..15: outlier positions left for
    // the generic loop (8-bit: all of them); bits 16..31: index of that first word
    uint32_t pos;
    __device__ __forceinline__ uint32_t more() const { return (pos >> 8) & 0xFFu; }
};
__device__ __forceinline__ uint32_t pos_shift(uint32_t pos) { return pos & 31u; }
__device__ __forceinline__ uint32_t pos_even_shift(uint32_t pos) { return (pos >> 3) & 4u; }
__device__ __forceinline__ uint32_t pos_more(uint32_t pos) { return (pos >> 8) & 0xFFu; }
__device__ __forceinline__ uint32_t pos_word(uint32_t pos) { return pos >> 16; }

template <int BITS, int TPR>
__device__ __forceinline__ void plan_chunk(ChunkPlan<BITS>& p, int k0, int K, int K_b,
                                           const uint32_t* mask, const uint32_t* pre) {
    uint32_t m8 = 0xFFu;
    int base0 = 0;
    if (k0 < K) {
        const uint32_t word = mask[k0 >> 5];
        m8 = (word >> (k0 & 31)) & 0xFFu;
        base0 = k0 - (int)(pre[k0 >> 5] + __popc(word & ((1u << (k0 & 31)) - 1u)));
    }
    int cnt = 8 - __popc(m8);
    if (base0 >= K_b) cnt = 0;                     // only with a malformed index list
    if (cnt > K_b - base0) cnt = K_b - base0;
    if (cnt <= 0) { cnt = 0; base0 = 0; }          // nothing to emit: park the (zero) write at word 0
    const uint32_t squeeze = cnt ? m8 : 0u;        // an empty chunk is masked away whole: no squeeze
#pragma unroll
    for (int d = 0; d < 4; ++d)
        p.sel[d] = (((m8 >> (2 * d)) & 1u) ? 0x0000FFFFu : 0u) | (((m8 >> (2 * d + 1)) & 1u) ? 0xFFFF0000u : 0u);
    uint32_t rest = squeeze;
    if constexpr (BITS == 4) {
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            if (rest) {
                const int pos = 31 - __clz(rest);
                p.low[j] = pos ? (0xFFFFFFFFu >> (32 - 4 * pos)) : 0u;
                rest &= ~(1u << pos);
            } else {
                p.low[j] = 0xFFFFFFFFu;
            }
        }
    }
    const int bits = cnt * BITS;                   // 0 .. 64
    p.keep_lo = bits >= 32 ? 0xFFFFFFFFu : ((1u << bits) - 1u);
    p.keep_hi = bits >= 64 ? 0xFFFFFFFFu : (bits > 32 ? ((1u << (bits - 32)) - 1u) : 0u);
    const uint32_t bit = (uint32_t)base0 * BITS;
    p.pos = (bit & 31u) | ((base0 & 1) ? 32u : 0u) | (rest << 8) | ((bit >> 5) << 16);
}

// Codes of the eight elements of a chunk whose outlier halves already read as the row minimum.
// 4-bit: nibble i of the result; 8-bit: byte i of (lo, hi).
template <int BITS>
__device__ __forceinline__ void chunk_codes(const uint32_t (&x)[4], float mn, float inv, uint32_t& lo, uint32_t& hi) {
    uint32_t b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const __half h = __ushort_as_half((unsigned short)(x[i >> 1] >> (16 * (i & 1))));
        b[i] = code_bits(h, mn, inv);              // 0x4B400000 + code
    }
    if constexpr (BITS == 4) {
        uint32_t w = b[0];
#pragma unroll
        for (int i = 1; i < 8; ++i) w += b[i] << (4 * i);
        uint32_t c = 0;                            // the eight shifted copies of the constant part
#pragma unroll
        for (int i = 0; i < 8; ++i) c += kMagicBits << (4 * i);
        lo = w - c;
        hi = 0;
    } else {
        uint32_t w0 = b[0], w1 = b[4];
#pragma unroll
        for (int i = 1; i < 4; ++i) { w0 += b[i] << (8 * i); w1 += b[4 + i] << (8 * i); }
        uint32_t c = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) c += kMagicBits << (8 * i);
        lo = w0 - c;
        hi = w1 - c;
    }
}

// K <= TPR * 8 * NCH: the row lives in NCH 128-bit registers per thread.  FMT 1 (4-bit codes only):
// the packed row is written as E3M2 patterns in the panel layout of quik_fp6_device.h (xq is then the
// whole [stage][row][48-byte] buffer, ldq the 48 * stages bytes of one row's LDS image) and no code sum
// is produced.  FMT 2 (4-bit codes only): the packed row leaves in the activation format of the 2:4-sparse
// path (quik_sp24_device.h: [stage][row][32-byte] buffer, ldq = 32 * stages), again without a code sum.
template <int BITS, int TPR, int NCH, int FMT>
__global__ __launch_bounds__(kBlock, (NCH >= 4 ? 2 : 3)) void quantize_rows_kernel(
    const __half* __restrict__ x, int T, int K, int ldx, const int32_t* __restrict__ idx, int n_out,
    uint8_t* __restrict__ xq, int ldq, float* __restrict__ scale, float* __restrict__ zero,
    int32_t* __restrict__ code_sum, __half* __restrict__ x_out, int ldo) {
    constexpr int RPB = kBlock / TPR;             // rows per workgroup iteration
    constexpr bool WAVE_ROW = TPR == 64;          // a row never leaves its wave: no workgroup barriers
    constexpr bool FP6 = FMT == 1, SP24 = FMT == 2;
    extern __shared__ __align__(16) uint32_t lds[];
    // Claim the whole register budget of the launch bounds (512 / waves per SIMD, in units of 8).
    // Measured on MI355X: when this kernel's allocation ended exactly at its highest live register
    // (208 and 96 registers, leaving part of the SIMD's file unallocated), that register now and then
    // read as the work-item id in the second workgroup of a CU; the identical code with a larger
    // allocation never did.  With the budget claimed, the top of the allocation is live only in the
    // instantiation that needs all 256 registers (a wave then owns exactly half the file, like the
    // GEMM kernels, which have shown no such reads).
    if constexpr (NCH >= 4) asm volatile("" ::: "v255");
    else asm volatile("" ::: "v167");
    const int nwords = (K + 31) >> 5;
    uint32_t* mask = lds;
    uint32_t* pre = mask + nwords;
    float* red = reinterpret_cast<float*>(pre + nwords);       // [2 * 4] wave partials
    uint32_t* wave_tot = reinterpret_cast<uint32_t*>(red + 8); // [4]
    int* red_i = reinterpret_cast<int*>(wave_tot + 4);         // [4] wave partials of the code sum
    const int img0 = (2 * nwords + 16 + 3) & ~3;               // first row image, 16-byte aligned (in words)

    const int tid = threadIdx.x;
    const int g = tid / TPR, lt = tid % TPR;
    const int K_b = K - n_out;
    const int ldq_words = ldq >> 2;
    // two images per row group, used by alternate rows: a row may start clearing and filling its
    // image while slower waves still write the previous row's image out (one spare 16 bytes behind
    // every image)
    uint32_t* const stage0 = lds + img0 + g * (ldq_words + 4);
    const int img_stride = RPB * (ldq_words + 4);
    int row_parity = 0;
    const int nrowblk = (T + RPB - 1) / RPB;

    // the outlier columns this thread moves (the first GJ * TPR of them; -1: none)
    constexpr int GJ = 4;
    int cidx[GJ];
#pragma unroll
    for (int q = 0; q < GJ; ++q) {
        const int j = lt + q * TPR;
        const int c = (j < n_out) ? idx[j] : -1;
        cidx[q] = (c >= 0 && c < K) ? c : -1;
    }

    // a row's loads: its chunks and its outlier values, requested together (the outlier values
    // are needed last, so fetching them with the row keeps their latency off the row's tail)
    auto load_row = [&](uint4 (&cache)[NCH], uint32_t (&gv)[GJ], int rb) {
        const int t = rb * RPB + g;
        const __half* row = x + (size_t)(t < T ? t : 0) * ldx;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int k0 = (c * TPR + lt) * 8;
            if (t < T && k0 < K) cache[c] = *reinterpret_cast<const uint4*>(row + k0);
            else cache[c] = make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int q = 0; q < GJ; ++q)
            gv[q] = (t < T && cidx[q] >= 0) ? (uint32_t)__half_as_ushort(row[cidx[q]]) : 0u;
    };

    // second register set for the next row, where the register budget has room for it
    constexpr bool DOUBLE = FP6 ? NCH <= 4 : NCH <= 6;
    uint4 ca[NCH], cb[DOUBLE ? NCH : 1];
    uint32_t gva[GJ], gvb[GJ];                    // one register each: packing two would stall on the load
    int rb = blockIdx.x;
    if (rb < nrowblk) load_row(ca, gva, rb);       // the first loads do not depend on the outlier map
    build_outlier_map(idx, n_out, K, nwords, mask, pre, wave_tot);

    ChunkPlan<BITS> plan[NCH];
    uint32_t any_more = 0;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        plan_chunk<BITS, TPR>(plan[c], (c * TPR + lt) * 8, K, K_b, mask, pre);
        any_more |= plan[c].more();
    }
    // generic squeeze needed by some lane of this wave? (more than three outliers in one 4-bit chunk)
    const bool wave_more = __builtin_amdgcn_ballot_w64(any_more != 0) != 0;

    auto process_row = [&](const uint4 (&cache)[NCH], const uint32_t (&gv)[GJ], int rbk) {
        const int t = rbk * RPB + g;
        const bool valid = t < T;
        const __half* row = x + (size_t)(valid ? t : 0) * ldx;
        uint32_t* const stage = stage0 + row_parity * img_stride;
        row_parity ^= 1;

        for (int i = lt; i < ldq_words; i += TPR) stage[i] = 0u;

        // ---- pass 1: min/max over base columns
        uint32_t mn2 = kNaN2, mx2 = kNaN2;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const uint32_t xw[4] = {cache[c].x, cache[c].y, cache[c].z, cache[c].w};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const uint32_t v = bit_select(plan[c].sel[d], kNaN2, xw[d]);
                mn2 = pk_min_f16(mn2, v);
                mx2 = pk_max_f16(mx2, v);
            }
        }
        float mn = fminf(__half2float(__ushort_as_half((unsigned short)mn2)),
                         __half2float(__ushort_as_half((unsigned short)(mn2 >> 16))));
        float mx = fmaxf(__half2float(__ushort_as_half((unsigned short)mx2)),
                         __half2float(__ushort_as_half((unsigned short)(mx2 >> 16))));
        mn = wave_min(mn);
        mx = wave_max(mx);
        if constexpr (!WAVE_ROW) {
            const int wv = tid >> 6;
            if ((tid & 63) == 0) { red[wv] = mn; red[4 + wv] = mx; }
            __syncthreads();                       // also: row image zeroed by all lanes
            mn = fminf(fminf(red[0], red[1]), fminf(red[2], red[3]));
            mx = fmaxf(fmaxf(red[4], red[5]), fmaxf(red[6], red[7]));
        }
        mn = mn + 0.0f;                            // -0 -> +0
        const float range = mx - mn;
        const float s = (range == 0.0f) ? 1.0f : range / (float)((1 << BITS) - 1);
        const float inv = 1.0f / s;
        if (valid && lt == 0) { scale[t] = s; zero[t] = mn; }
        const uint32_t mnh = __half_as_ushort(__float2half(mn));   // exact: the minimum is an fp16 value
        const uint32_t mnh2 = mnh | (mnh << 16);

        // ---- pass 2: quantize the base elements into the LDS row image
        uint32_t esum = 0;                         // unsigned codes at even positions (4-bit only)
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const ChunkPlan<BITS>& p = plan[c];
            const uint32_t xw[4] = {bit_select(p.sel[0], mnh2, cache[c].x), bit_select(p.sel[1], mnh2, cache[c].y),
                                    bit_select(p.sel[2], mnh2, cache[c].z), bit_select(p.sel[3], mnh2, cache[c].w)};
            uint32_t lo, hi;
            chunk_codes<BITS>(xw, mn, inv, lo, hi);
            // the fields of pos are unpacked per row on purpose (hoisting them out of the row loop
            // would cost three registers per chunk)
            uint32_t pos = p.pos;
            asm volatile("" : "+v"(pos));
            if constexpr (BITS == 4) {
#pragma unroll
                for (int j = 0; j < 3; ++j) lo = bit_select(p.low[j], lo, lo >> 4);
                if (wave_more) {
                    uint32_t m = pos_more(pos);
                    while (m) {
                        const int hp = 31 - __clz(m);
                        lo = drop_element<uint32_t, 4>(lo, hp);
                        m &= ~(1u << hp);
                    }
                }
                lo &= p.keep_lo;
                if constexpr (FP6) {
                    // the kept elements as 6-bit patterns, OR-ed into dwords d, d+1, d+2 of the 192-bit
                    // string of their group of 32 columns (running on into the next group)
                    const uint32_t bits6 = 6u * ((uint32_t)__popc(p.keep_lo) >> 2);
                    const uint64_t v6 = fp6::pack8(lo) & (bits6 >= 48u ? 0xFFFFFFFFFFFFull : ((1ull << bits6) - 1ull));
                    const uint32_t e0 = (pos_word(pos) * 32u + pos_shift(pos)) >> 2;   // first element's position
                    const uint32_t G = e0 >> 5, b0 = 6u * (e0 & 31u), d0 = b0 >> 5, sh = b0 & 31u;
                    const uint64_t vs = v6 << sh;
                    const uint32_t w3[3] = {(uint32_t)vs, (uint32_t)(vs >> 32), sh ? (uint32_t)(v6 >> (64u - sh)) : 0u};
#pragma unroll
                    for (int i = 0; i < 3; ++i) {
                        uint32_t dd = d0 + i, GG = G;
                        if (dd >= 6u) { dd -= 6u; ++GG; }
                        if (w3[i]) atomicOr(&stage[12u * (GG >> 1) + (uint32_t)fp6::block_dword((int)(GG & 1u), (int)dd)], w3[i]);
                    }
                } else {
                    if constexpr (!SP24)
                        esum = __builtin_amdgcn_sad_u8((lo >> pos_even_shift(pos)) & 0x0F0F0F0Fu, 0u, esum);
                    lo = (lo ^ 0x88888888u) & p.keep_lo;      // code - halfRange as two's complement nibbles
                    const uint64_t v = (uint64_t)lo << pos_shift(pos);
                    atomicOr(&stage[pos_word(pos)], (uint32_t)v);
                    atomicOr(&stage[pos_word(pos) + 1], (uint32_t)(v >> 32));
                }
            } else {
                uint64_t w = ((uint64_t)hi << 32) | lo;
                uint32_t m = pos_more(pos);
                while (m) {
                    const int hp = 31 - __clz(m);
                    w = drop_element<uint64_t, 8>(w, hp);
                    m &= ~(1u << hp);
                }
                const uint64_t keep = ((uint64_t)p.keep_hi << 32) | p.keep_lo;
                w = (w ^ 0x8080808080808080ull) & keep;
                const uint32_t sh = pos_shift(pos);
                const uint64_t v = w << sh;
                const uint32_t top = sh ? (uint32_t)(w >> (64u - sh)) : 0u;
                atomicOr(&stage[pos_word(pos)], (uint32_t)v);
                atomicOr(&stage[pos_word(pos) + 1], (uint32_t)(v >> 32));
                atomicOr(&stage[pos_word(pos) + 2], top);
            }
        }
        if constexpr (BITS == 4 && FMT == 0) {
            // sum over even positions of the signed codes (the GEMM's correction term for its
            // single-AND operand widening)
            int es = wave_sum((int)esum);
            if constexpr (!WAVE_ROW) {
                if ((tid & 63) == 0) red_i[tid >> 6] = es;
                __syncthreads();
                es = red_i[0] + red_i[1] + red_i[2] + red_i[3];
            }
            if (valid && lt == 0 && code_sum) code_sum[t] = es - 8 * (K_b >> 1);
        } else if constexpr (!WAVE_ROW) {
            __syncthreads();
        }
        if constexpr (WAVE_ROW) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");

        // ---- write the packed row (including its zero padding up to ldq); 4-bit rows leave with
        // the two nibbles of every byte swapped: element 2p in the high nibble
        if (valid) {
            uint4* dst = reinterpret_cast<uint4*>(xq + (FMT != 0 ? (size_t)0 : (size_t)t * ldq));
            const uint4* src = reinterpret_cast<const uint4*>(stage);
            for (int i = lt; i < (ldq >> 4); i += TPR) {
                uint4 v = src[i];
                if constexpr (FP6) {                   // piece i of the image = piece i % 3 of stage i / 3
                    const int st = i / 3, c = i - 3 * st;
                    store16_through(dst + ((size_t)st * T + t) * 3 + c, v);
                    continue;
                }
                if constexpr (SP24) {                  // piece i of the image = piece i % 2 of stage i / 2
                    v = make_uint4(sp24::act_word(v.x), sp24::act_word(v.y), sp24::act_word(v.z), sp24::act_word(v.w));
                    store16_through(dst + ((size_t)(i >> 1) * T + t) * 2 + (i & 1), v);
                    continue;
                }
                if constexpr (BITS == 4 && FMT == 0) {
                    auto sw = [](uint32_t w) { return ((w & 0x0F0F0F0Fu) << 4) | ((w >> 4) & 0x0F0F0F0Fu); };
                    v = make_uint4(sw(v.x), sw(v.y), sw(v.z), sw(v.w));
                }
                store16_through(dst + i, v);
            }
            // ---- pass 3: move the outlier columns
#pragma unroll
            for (int q = 0; q < GJ; ++q) {
                const int j = lt + q * TPR;
                if (j < n_out) x_out[(size_t)t * ldo + j] = __ushort_as_half((unsigned short)gv[q]);
            }
            for (int j = lt + GJ * TPR; j < n_out; j += TPR) {
                const int c = idx[j];
                x_out[(size_t)t * ldo + j] = (c >= 0 && c < K) ? row[c] : __ushort_as_half((unsigned short)0);
            }
        }
        // no barrier here: the next row works on the other image, and two barriers of that row lie
        // between this write-out and the next clearing of this image
        if constexpr (WAVE_ROW) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    };

    if constexpr (DOUBLE) {
        // The next row is fetched into a second register set while the current one is processed.
        while (rb < nrowblk) {
            int nx = rb + gridDim.x;
            if (nx < nrowblk) load_row(cb, gvb, nx);
            process_row(ca, gva, rb);
            rb = nx;
            if (rb >= nrowblk) break;
            nx = rb + gridDim.x;
            if (nx < nrowblk) load_row(ca, gva, nx);
            process_row(cb, gvb, rb);
            rb = nx;
        }
    } else {
        // Long rows: one register set; other waves of the CU cover the load latency.
        while (rb < nrowblk) {
            process_row(ca, gva, rb);
            rb += gridDim.x;
            if (rb < nrowblk) load_row(ca, gva, rb);
        }
    }
}

// Generic form for any K (used above 16384 columns): the second pass re-reads the row from cache.
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
                store16_through(dst + i, v);
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

template <int BITS, int TPR, int NCH, int FMT>
hipError_t launch(const QuantizeArgs& a, hipStream_t stream) {
    constexpr int RPB = kBlock / TPR;
    const int nwords = (a.K + 31) >> 5;
    int nrowblk = (a.T + RPB - 1) / RPB;
    // a bounded grid: the outlier map and the chunk plans are built once per workgroup, so no more
    // workgroups are launched than the chip keeps resident; each loops over its row blocks (the
    // next row's loads in flight while the current one is processed where registers allow)
    constexpr int kResident = 256 * ((NCH >= 4 || NCH == 0) ? 2 : 3);
    int grid = nrowblk < (NCH > 0 ? kResident : 2048) ? nrowblk : (NCH > 0 ? kResident : 2048);
    if constexpr (NCH > 0) {
        // map + prefix, reduction scratch, then 2 * RPB row images of ldq bytes + 16 spare bytes each
        const size_t img0 = (size_t)((2 * nwords + 16 + 3) & ~3);
        const size_t lds = (img0 + 2 * (size_t)RPB * ((a.ldq >> 2) + 4)) * 4;
        hipLaunchKernelGGL((quantize_rows_kernel<BITS, TPR, NCH, FMT>), dim3(grid), dim3(kBlock), lds, stream,
                           (const __half*)a.x, a.T, a.K, a.ldx, a.idx, a.n_out, (uint8_t*)a.xq, a.ldq,
                           a.scale, a.zero, a.code_sum, (__half*)a.x_out, a.ldo);
    } else if constexpr (FMT != 0) {
        return hipErrorInvalidValue;               // rows beyond 16384 columns: row-major integer formats only
    } else {
        const size_t lds = (size_t)nwords * 8 + 8 * 4 + 4 * 4 + 4 * 4 + 16 + (size_t)RPB * a.ldq;
        hipLaunchKernelGGL((quantize_kernel<BITS, TPR, NCH>), dim3(grid), dim3(kBlock), lds, stream,
                           (const __half*)a.x, a.T, a.K, a.ldx, a.idx, a.n_out, (uint8_t*)a.xq, a.ldq,
                           a.scale, a.zero, a.code_sum, (__half*)a.x_out, a.ldo);
    }
    return hipGetLastError();
}

template <int BITS, int FMT>
hipError_t dispatch(const QuantizeArgs& a, hipStream_t stream) {
    const int K = a.K;
    if (K <= 64 * 8 * 1) return launch<BITS, 64, 1, FMT>(a, stream);
    if (K <= 64 * 8 * 2) return launch<BITS, 64, 2, FMT>(a, stream);
    if (K <= 64 * 8 * 4) return launch<BITS, 64, 4, FMT>(a, stream);
    if (K <= 256 * 8 * 2) return launch<BITS, 256, 2, FMT>(a, stream);
    if (K <= 256 * 8 * 3) return launch<BITS, 256, 3, FMT>(a, stream);
    if (K <= 256 * 8 * 4) return launch<BITS, 256, 4, FMT>(a, stream);
    if (K <= 256 * 8 * 6) return launch<BITS, 256, 6, FMT>(a, stream);
    if (K <= 256 * 8 * 8) return launch<BITS, 256, 8, FMT>(a, stream);
    return launch<BITS, 256, 0, FMT>(a, stream);
}

}  // namespace

hipError_t launch_quantize(const QuantizeArgs& a, hipStream_t stream) {
    if (a.format == 1) return a.bits == 4 ? dispatch<4, 1>(a, stream) : hipErrorInvalidValue;
    if (a.format == 2) return a.bits == 4 ? dispatch<4, 2>(a, stream) : hipErrorInvalidValue;
    if (a.format != 0) return hipErrorInvalidValue;
    return a.bits == 4 ? dispatch<4, 0>(a, stream) : dispatch<8, 0>(a, stream);
}

}  // namespace quik
