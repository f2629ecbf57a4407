// Measurement probes: what the int8 matrix pipe and the memory system sustain on the chip the
// library runs on, so that a kernel's rate can be quoted against a measured ceiling as well as
// against the data-sheet one.  Not part of the layer.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "quik_kernels.h"
#include "quik_gemm_device.h"

namespace quik {

namespace {

using gemm_dev::v4i;
using gemm_dev::v16i;

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

// The instruction mix of the 4-bit GEMM's K loop around the matrix instruction, one ingredient at a time and
// without any data dependence between them: what each kind of instruction costs the matrix pipe in issue
// slots.  Eight waves per workgroup (two per SIMD, as in the GEMM), twelve MFMAs per iteration and wave on
// six accumulators.  MIX bits:
//   1  operands of pseudo-random bytes that change from MFMA to MFMA (four register sets; else one constant
//      set of small values, most bytes zero)
//   2  four vector bit operations per MFMA (the nibble widening's count)
//   4  five 16-byte LDS reads per iteration (the fragment reads' count), waited for at its end
//   8  two global -> LDS copies of 16 bytes per lane per iteration (the operand copies' count), out of a
//      512 KB window of `src` that the CUs of an XCD share (L2-resident)
//  16  a workgroup barrier every fourth iteration (one per K stage)
//  32  (with 1) the changing operands are bytes of the kind the GEMM's nibble widening makes: in one
//      operand's even words and the other's odd words only the high nibble of a byte varies (16 x a signed
//      code), in the remaining words only the low nibble (a code + 8).  The clock the chip holds depends on
//      how many operand bits toggle, so this -- not bit 1 alone -- is the ceiling for the GEMM's own operands.
//  64  (with 1 and 32) the same work on v_mfma_i32_16x16x64_i8, the persistent kernel's instruction: two of
//      them in place of every 32 x 32 x 32 one, and ten 8-byte LDS reads in place of five 16-byte ones.
//      Built for mix 97 (matrix instructions alone) and 127 (the whole K-loop mix).
// clocks[0], clocks[1]: the shader clock counter and the 100 MHz real-time counter over the loop of
// workgroup 0 (their ratio is the clock the chip held under this load).
constexpr int kMixWaves = 8, kMixMfma = 12, kMixAcc = 6;

template <int MIX>
__global__ __launch_bounds__(kMixWaves * 64, 1) void mfma_mix_probe_kernel(int iters, int* sink, const uint8_t* src,
                                                                         uint32_t src_bytes, unsigned long long* clocks) {
    using namespace gemm_dev;
    constexpr bool TOGGLE = MIX & 1, VALU = MIX & 2, LDSR = MIX & 4, COPY = MIX & 8, BARRIER = MIX & 16, NIBBLE = MIX & 32,
                   X16 = MIX & 64;
    constexpr int NL = 5, ND = 2, WINDOW = 512 * 1024;
    asm volatile("" ::: "v255");       // a wave owns half of its SIMD's register file: claim it whole (see build.py)
    __shared__ __align__(1024) uint8_t frag[64 * 1024];
    __shared__ __align__(1024) uint8_t ring[COPY ? 64 * 1024 : 1024];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    for (int i = threadIdx.x; i < 16 * 1024; i += blockDim.x) reinterpret_cast<int*>(frag)[i] = i * 0x9E3779B1u;
    __syncthreads();
    v16i acc[kMixAcc];              // the 16 x 16 form uses them as 4 x kMixAcc blocks of four registers
#pragma unroll
    for (int j = 0; j < kMixAcc; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0;
    v4i a[4], b[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            // constant operands: small values, most bytes zero (as in mfma_i8_probe_kernel); changing
            // operands: pseudo-random bytes, a different set for consecutive instructions
            const uint32_t h = (uint32_t)(lane * 4 + e + 1) * 0x9E3779B1u;
            a[q][e] = TOGGLE ? (int)(h * (2 * q + 3)) : (e == 0 ? lane : e);
            b[q][e] = TOGGLE ? (int)((h ^ 0x5bd1e995u) * (2 * q + 5)) : (e == 3 ? (int)blockIdx.x : 4 + e);
            if constexpr (TOGGLE && NIBBLE) {
                a[q][e] &= (e & 1) ? 0x0F0F0F0F : (int)0xF0F0F0F0u;
                b[q][e] &= (e & 1) ? (int)0xF0F0F0F0u : 0x0F0F0F0F;
            }
        }
    uint32_t x[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) x[q] = (uint32_t)lane * 17u + q;
    // fragment-style LDS addresses: row lane % 32 of 128-byte rows, swizzled 16-byte slot
    const int l = lane & 31, kg = lane >> 5;
    const uint32_t faddr = lds_addr(frag) + (uint32_t)(wave * 4096 + l * 128 + ((kg ^ swz<128>(l)) << 4));
    typedef unsigned u4 __attribute__((ext_vector_type(4)));
    typedef unsigned u2 __attribute__((ext_vector_type(2)));
    u4 rr[NL];
    u2 rh[2 * NL];
#pragma unroll
    for (int q = 0; q < 2 * NL; ++q) rh[q] = u2{0, 0};
#pragma unroll
    for (int q = 0; q < NL; ++q) rr[q] = u4{0, 0, 0, 0};
    const v4i rs = make_rsrc(src, src_bytes);
    const uint32_t ring_base = lds_addr(ring);
    uint32_t gpos = (uint32_t)((blockIdx.x / kXcds / 8) * WINDOW) % (src_bytes - WINDOW + 1);
    const uint32_t gwin = gpos;

    const uint64_t t0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < kMixMfma; ++m) {
            if constexpr (X16) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {        // blocks 2 * (m / kMixAcc) + h of accumulator m % kMixAcc
                    const int q0 = 8 * (m / kMixAcc) + 4 * h;
                    v16i& c = acc[m % kMixAcc];
                    v4i d = v4i{c[q0], c[q0 + 1], c[q0 + 2], c[q0 + 3]};
                    d = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[m % 4], b[(m + m / 4 + h) % 4], d, 0, 0, 0);
                    c[q0] = d[0]; c[q0 + 1] = d[1]; c[q0 + 2] = d[2]; c[q0 + 3] = d[3];
                }
            } else {
                acc[m % kMixAcc] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[m % 4], b[(m + m / 4) % 4], acc[m % kMixAcc], 0, 0, 0);
            }
            if constexpr (VALU) {
#pragma unroll
                for (int v = 0; v < 4; ++v) asm volatile("v_and_b32 %0, 0xf0f0f0f0, %0" : "+v"(x[(m * 4 + v) % 8]));
            }
            if constexpr (LDSR) {
                if constexpr (X16) {
                    if (m < 2 * NL) asm volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(rh[m < 2 * NL ? m : 0]) : "v"(faddr), "n"((m % 16) * 2048 % 32768));
                } else {
                    if (m < NL) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(rr[m]) : "v"(faddr), "n"((m % 8) * 4096 % 32768));
                }
            }
            if constexpr (COPY) {
                if (m < ND) dma16(rs, ring_base + (uint32_t)((((it & 3) * ND + m) * kMixWaves + wave) * 1024) % 65536u,
                                  gpos + (uint32_t)((m * kMixWaves + wave) * 1024 + lane * 16), 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (COPY) {
            gpos += ND * kMixWaves * 1024;
            if (gpos + ND * kMixWaves * 1024 > gwin + WINDOW) gpos = gwin;
        }
        if ((it & 3) == 3) {
            if constexpr (COPY) wait_vm<2 * ND>();          // all but the two youngest iterations' copies have landed
            if constexpr (BARRIER) __builtin_amdgcn_s_barrier();
        }
        if constexpr (LDSR) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int q = 0; q < NL; ++q) asm volatile("" ::"v"(rr[q]));
#pragma unroll
            for (int q = 0; q < 2 * NL; ++q) asm volatile("" ::"v"(rh[q]));
        }
    }
    if constexpr (COPY) wait_vm<0>();
    const uint64_t t1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
    if (clocks != nullptr && blockIdx.x == 0 && threadIdx.x == 0) {
        clocks[0] = t1 - t0;
        clocks[1] = r1 - r0;
    }
    int s = 0;
#pragma unroll
    for (int j = 0; j < kMixAcc; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[j][r];
#pragma unroll
    for (int q = 0; q < 8; ++q) s += (int)x[q];
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

hipError_t launch_mix_probe(int mix, int workgroups, int iters, int* sink, const void* src, size_t src_bytes,
                            unsigned long long* clocks, hipStream_t stream) {
    const uint8_t* s8 = static_cast<const uint8_t*>(src);
    const uint32_t nb = src_bytes > 0x40000000u ? 0x40000000u : (uint32_t)src_bytes;
#define QUIK_MIX_CASE(M) \
    case M: hipLaunchKernelGGL(mfma_mix_probe_kernel<M>, dim3(workgroups), dim3(kMixWaves * 64), 0, stream, iters, sink, s8, nb, clocks); break;
    switch (mix) {
        QUIK_MIX_CASE(0) QUIK_MIX_CASE(1) QUIK_MIX_CASE(2) QUIK_MIX_CASE(3) QUIK_MIX_CASE(4) QUIK_MIX_CASE(5) QUIK_MIX_CASE(6) QUIK_MIX_CASE(7)
        QUIK_MIX_CASE(8) QUIK_MIX_CASE(9) QUIK_MIX_CASE(10) QUIK_MIX_CASE(11) QUIK_MIX_CASE(12) QUIK_MIX_CASE(13) QUIK_MIX_CASE(14) QUIK_MIX_CASE(15)
        QUIK_MIX_CASE(16) QUIK_MIX_CASE(17) QUIK_MIX_CASE(18) QUIK_MIX_CASE(19) QUIK_MIX_CASE(20) QUIK_MIX_CASE(21) QUIK_MIX_CASE(22) QUIK_MIX_CASE(23)
        QUIK_MIX_CASE(24) QUIK_MIX_CASE(25) QUIK_MIX_CASE(26) QUIK_MIX_CASE(27) QUIK_MIX_CASE(28) QUIK_MIX_CASE(29) QUIK_MIX_CASE(30) QUIK_MIX_CASE(31)
        QUIK_MIX_CASE(33) QUIK_MIX_CASE(35) QUIK_MIX_CASE(37) QUIK_MIX_CASE(39) QUIK_MIX_CASE(41) QUIK_MIX_CASE(43) QUIK_MIX_CASE(45) QUIK_MIX_CASE(47)
        QUIK_MIX_CASE(49) QUIK_MIX_CASE(51) QUIK_MIX_CASE(53) QUIK_MIX_CASE(55) QUIK_MIX_CASE(57) QUIK_MIX_CASE(59) QUIK_MIX_CASE(61) QUIK_MIX_CASE(63)
        QUIK_MIX_CASE(97) QUIK_MIX_CASE(127)
        default: return hipErrorInvalidValue;
    }
#undef QUIK_MIX_CASE
    return hipGetLastError();
}

hipError_t launch_copy_probe(const void* src, void* dst, size_t bytes, hipStream_t stream) {
    hipLaunchKernelGGL(copy_probe_kernel, dim3(256 * 16), dim3(256), 0, stream, static_cast<const uint4*>(src),
                       static_cast<uint4*>(dst), bytes / 16);
    return hipGetLastError();
}

}  // namespace quik
