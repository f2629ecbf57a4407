// QUIK-4B linear layer with the integer product computed on the FP6 matrix pipe of gfx950
// (Algorithm 1 of arXiv 2310.09259: "INTmatmul", "Dequantization", "FPmatmul", final add; the
// epilogue fusion of Section 3.4).  The signed 4-bit codes travel as E3M2 patterns (see
// quik_fp6_device.h: exact, and the fp32 accumulators hold the exact integer dot products), so the
// K loop is DMA -> LDS -> registers -> v_mfma_f32_32x32x64_f8f6f4 with no widening work at all, at
// twice the int8 rate of the matrix pipe.
//
// A workgroup of WM x WN waves owns a BM x BN output tile.  A stage is 64 columns = one matrix step = one
// 48-byte block per operand row; the operands are stored stage by stage (quik_fp6_device.h), so the
// tile's rows of a stage are one contiguous run of BM * 48 (BN * 48) bytes that 16-byte-per-lane DMA
// instructions copy global -> LDS as it is.  The K loop needs many bytes in flight per CU (completion is
// in order, so every request waits like the slowest before it), but not as many as the LDS could hold: a
// ring of six stages for the 256 x 192 tile (108 KB in flight) runs 5 % faster than one of seven.  Lane (row l%32, half g = l/32) reads,
// per stage, 16 bytes (dwords 0..3 of its group) and 8 bytes (dwords 4, 5); 48-byte rows need no
// swizzle (twelve dwords per row walk all 64 banks in sixteen rows).  One workgroup barrier per stage;
// right after it the buffer that was read during the previous stage is refilled, the DMA
// instructions spread between the matrix instructions.  The fp16 outlier columns run through the same
// ring as stages of 16 columns (32-byte rows, 32 rows per DMA instruction, pieces exchanged in every
// second group of eight rows), with the dequantized integer part as the C operand of
// v_mfma_f32_32x32x16_f16, whose accumulator layout is the same.  Rows beyond T / N are out of range
// for the per-stage buffer descriptors and arrive as zeros (the E3M2 pattern of 0); columns beyond K_b
// are zero padding.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "quik_kernels.h"
#include "quik_gemm_device.h"
#include "quik_fp6_device.h"

namespace quik {

namespace {

using namespace gemm_dev;

typedef int v8i __attribute__((ext_vector_type(8)));

__device__ __forceinline__ int swz_f(int r) { return (r >> 3) & 1; }   // fp16 stages: 32-byte rows, two pieces

// descriptor r moved forward by `bytes`
__device__ __forceinline__ v4i advance(v4i r, uint32_t bytes) {
    const uint64_t base = (((uint64_t)(uint32_t)r[1]) << 32 | (uint32_t)r[0]) + bytes;
    r[0] = (int)(uint32_t)base;
    r[1] = (int)(uint32_t)(base >> 32);
    return r;
}

// MODE 0: fused epilogue, fp16 output; MODE 1: the integer accumulators as INT32.
template <int BM, int BN, int WM, int WN, int NST, int GM, int MODE>
__global__ __launch_bounds__(WM * WN * 64, (WM * WN == 8) ? 1 : 2) void gemm_fp6_kernel(GemmArgs a) {
    constexpr bool RAW = MODE != 0;
    // claim the whole register budget of the launch bounds, so that the highest allocated register is
    // never a live one (see the note in the row-quantization kernel)
    asm volatile("" ::: "v255");
    constexpr int NWAVES = WM * WN, NT = NWAVES * 64;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32, NF = TM + TN;
    constexpr int A_BYTES = BM * 48, B_BYTES = BN * 48, ST_BYTES = A_BYTES + B_BYTES;
    // DMA instructions of a stage (1 KB each): FP6 stages N_A + N_B over the tile's two runs, fp16 stages
    // BM / 32 and BN / 32.  A wave issues LPS of them per stage: instruction i = wave + NWAVES * slot; one
    // that does not exist is issued empty so that every wave counts the same number.
    constexpr int N_A = BM * 48 / 1024, N_B = BN * 48 / 1024, N_AF = BM / 32, N_BF = BN / 32;
    constexpr int LPS = (N_A + N_B + NWAVES - 1) / NWAVES;
    static_assert(BM % 64 == 0 && BN % 64 == 0 && N_AF + N_BF <= LPS * NWAVES && (BM + BN) * 32 <= ST_BYTES, "geometry");
    static_assert(NST * LPS < 64, "vmcnt range");
    constexpr int DUMMY = NST * ST_BYTES;                 // 1 KB that empty DMA instructions clear

    __shared__ __align__(1024) uint8_t lds[NST * ST_BYTES + 1024];
    __shared__ __align__(16) float lds_sa[BM];
    __shared__ __align__(16) float lds_sh[BM];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave_u = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave_u / WN, wn = wave_u % WN;
    const int l32 = lane & 31, g = lane >> 5;

    const int tiles_m = (a.T + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    const int id = xcd_contiguous_id(blockIdx.x, tiles_m * tiles_n);
    int tile_m, tile_n;
    if constexpr (GM > 0) {
        const int per_group = GM * tiles_n;
        const int grp = id / per_group, rem = id % per_group;
        const int first_m = grp * GM;
        const int gsz = min(GM, tiles_m - first_m);
        tile_m = first_m + rem % gsz;
        tile_n = rem / gsz;
    } else {
        tile_m = id % tiles_m;
        tile_n = id / tiles_m;
    }
    const int t0 = tile_m * BM, n0 = tile_n * BN;

    const int S = fp6::stages(a.K_b);
    const int nk_int = a.fp_only ? 0 : S;
    const int fp_bytes = a.n_out * 2;
    const int nk_fp = RAW ? 0 : (fp_bytes + 31) / 32;
    const int nk = nk_int + nk_fp;
    const int lda_fp = a.ldo * 2, ldb_fp = a.ldwo * 2;
    const int T_ = a.T, N_ = a.N;                         // values, so that nothing takes the address of an argument

    // stage 0 of the tile's rows; stage s lies s * T * 48 (s * N * 48) bytes further on
    const v4i rA = make_rsrc((const uint8_t*)a.xq + (size_t)t0 * 48, (size_t)(a.T - t0) * 48);
    const v4i rB = make_rsrc((const uint8_t*)a.w_q + (size_t)n0 * 48, (size_t)(a.N - n0) * 48);
    const v4i rAf = make_rsrc(a.n_out ? (const uint8_t*)a.x_out + (size_t)t0 * lda_fp : (const uint8_t*)a.xq,
                              a.n_out ? (size_t)(a.T - t0) * lda_fp : 0);
    const v4i rBf = make_rsrc(a.n_out ? (const uint8_t*)a.w_out + (size_t)n0 * ldb_fp : (const uint8_t*)a.xq,
                              a.n_out ? (size_t)(a.N - n0) * ldb_fp : 0);
    const uint32_t lds_base = lds_addr(lds);

    // fp16 stage: 32 rows (lane / 2) x two 16-byte pieces of a 32-byte stage row per instruction
    const int colF = ((lane & 1) ^ ((lane >> 4) & 1)) * 16;
    const uint32_t vo_af = (uint32_t)((lane >> 1) * lda_fp + colF), vo_bf = (uint32_t)((lane >> 1) * ldb_fp + colF);
    // DMA slot j of stage s (int part, fp16 part, or past the end: every lane out of range)
    auto issue_one = [&](int s, int j) __attribute__((always_inline)) {
        const int i = wave_u + NWAVES * j;                      // instruction of the stage (wave-uniform)
        const uint32_t sb = (uint32_t)(s % NST) * ST_BYTES;
        const bool fp = s >= nk_int;
        uint32_t vo = kOob, dst = (uint32_t)DUMMY;
        v4i r;
        if (!fp) {
            // instructions 0 .. N_A-1 copy A's run, N_A .. N_A+N_B-1 B's: piece 64 i' + lane of the run
            const bool isb = i >= N_A;
            const int ii = isb ? i - N_A : i;
            if (i < N_A + N_B) {
                dst = sb + (isb ? A_BYTES : 0) + ii * 1024;
                if (s < nk) vo = (uint32_t)(ii * 1024 + lane * 16);
            }
            r = isb ? advance(rB, (uint32_t)s * (uint32_t)N_ * 48u) : advance(rA, (uint32_t)s * (uint32_t)T_ * 48u);
        } else {
            const bool isb = i >= N_AF;
            const int ii = isb ? i - N_AF : i;
            const int c0 = 32 * (s - nk_int);
            if (i < N_AF + N_BF) {
                dst = sb + (isb ? BM * 32 : 0) + ii * 1024;
                if (s < nk && c0 + colF < fp_bytes)
                    vo = (isb ? vo_bf : vo_af) + (uint32_t)(ii * 32 * (isb ? ldb_fp : lda_fp) + c0);
            }
            r = isb ? rBf : rAf;
        }
        // wave-uniform by construction; say so, the DMA takes them in scalar registers
        r = v4i{__builtin_amdgcn_readfirstlane(r[0]), __builtin_amdgcn_readfirstlane(r[1]),
                __builtin_amdgcn_readfirstlane(r[2]), __builtin_amdgcn_readfirstlane(r[3])};
        dma16(r, (uint32_t)__builtin_amdgcn_readfirstlane((int)(lds_base + dst)), vo, 0);
    };
    // DMA slot j of an FP6 stage that exists (the hot loop's form)
    auto issue_int = [&](int s, int j) __attribute__((always_inline)) {
        const int i = wave_u + NWAVES * j;
        const bool isb = i >= N_A;
        const int ii = isb ? i - N_A : i;
        const bool exists = i < N_A + N_B;
        const uint32_t dst = exists ? (uint32_t)(s % NST) * ST_BYTES + (isb ? A_BYTES : 0) + ii * 1024 : (uint32_t)DUMMY;
        const uint32_t vo = exists ? (uint32_t)(ii * 1024 + lane * 16) : kOob;
        v4i r = isb ? advance(rB, (uint32_t)s * (uint32_t)N_ * 48u) : advance(rA, (uint32_t)s * (uint32_t)T_ * 48u);
        r = v4i{__builtin_amdgcn_readfirstlane(r[0]), __builtin_amdgcn_readfirstlane(r[1]),
                __builtin_amdgcn_readfirstlane(r[2]), __builtin_amdgcn_readfirstlane(r[3])};
        dma16(r, (uint32_t)__builtin_amdgcn_readfirstlane((int)(lds_base + dst)), vo, 0);
    };
    auto issue = [&](int s) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < LPS; ++j) issue_one(s, j);
    };

    // ---- epilogue parameters, requested before the first DMA
    constexpr int RPT = (BM + NT - 1) / NT;
    float p_s[RPT], p_z[RPT];
    float c_sw[TN], c_wr[TN], c_bv[TN];
    if constexpr (!RAW) {
#pragma unroll
        for (int q = 0; q < RPT; ++q) {
            const int t = t0 + tid + q * NT;
            const bool ok = (tid + q * NT < BM) && t < a.T;
            p_s[q] = ok ? a.scale[t] : 0.0f;
            p_z[q] = ok ? a.zero[t] : 0.0f;
        }
        const __half* __restrict__ wsc = static_cast<const __half*>(a.w_scale);
        const __half* __restrict__ bias = static_cast<const __half*>(a.bias);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = min(n0 + wn * TN * 32 + j * 32 + l32, a.N - 1);
            c_sw[j] = __half2float(wsc[n]);
            c_bv[j] = bias ? __half2float(bias[n]) : 0.0f;
            c_wr[j] = a.w_reduced[n];
            if (a.fp_only) { c_sw[j] = 0.0f; c_bv[j] = 0.0f; c_wr[j] = 0.0f; }
        }
    }

#pragma unroll
    for (int s = 0; s < NST; ++s) issue(s);

    if constexpr (!RAW) {
#pragma unroll
        for (int q = 0; q < RPT; ++q) {
            const int r = tid + q * NT;
            if (r < BM) {
                lds_sa[r] = p_s[q];                        // scaleAct
                lds_sh[r] = p_z[q] + 8.0f * p_s[q];        // zeroAct + halfRange * scaleAct
            }
        }
    }

    // LDS read addresses of this lane's row of every fragment.  FP6 stage: piece g of the row's 48-byte
    // block (16 bytes) and 8 bytes at 32 + 8 g; fp16 stage: piece g of a 32-byte row.
    uint32_t rdp[NF], rdf[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        const int r = (f < TM) ? (wm * TM * 32 + f * 32 + l32) : (wn * TN * 32 + (f - TM) * 32 + l32);
        rdp[f] = (f < TM ? 0 : A_BYTES) + r * 48 + 16 * g;
        rdf[f] = (f < TM ? 0 : BM * 32) + r * 32 + ((g ^ swz_f(r)) << 4);
    }
    // two fragment sets: the matrix instructions of one stage run on one set while the LDS reads of the
    // next stage fill the other
    uint4 FP[2][NF];
    uint2 FQ[2][NF];
    auto read_frag = [&](int set, int f, int s) __attribute__((always_inline)) {
        const uint8_t* st = lds + (s % NST) * ST_BYTES;
        FP[set][f] = *reinterpret_cast<const uint4*>(st + rdp[f]);
        FQ[set][f] = *reinterpret_cast<const uint2*>(st + rdp[f] + 32 - 8 * g);     // 32 + 8 g of the block
    };

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // FP6 stage s.  Its successor must have landed for everybody (its fragments are read during this
    // stage); all reads of stage s itself completed before the barrier, so its buffer is refilled with
    // stage s + NST right away, one DMA instruction per matrix instruction.  PLAIN: stage s + NST is an
    // FP6 stage; AHEAD: stage s + 1 is one.
    auto step = [&](int s, int set, bool plain, bool ahead) __attribute__((always_inline)) {
        wait_vm<(NST - 2) * LPS>();
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < TM * TN; ++m) {
            const int i = m / TN, j = m % TN;
            const v8i oa = v8i{(int)FP[set][i].x, (int)FP[set][i].y, (int)FP[set][i].z, (int)FP[set][i].w,
                               (int)FQ[set][i].x, (int)FQ[set][i].y, 0, 0};
            const v8i ob = v8i{(int)FP[set][TM + j].x, (int)FP[set][TM + j].y, (int)FP[set][TM + j].z,
                               (int)FP[set][TM + j].w, (int)FQ[set][TM + j].x, (int)FQ[set][TM + j].y, 0, 0};
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(oa, ob, acc[i][j], 3, 3, 0, 0, 0, 0);
            if (m < LPS) { if (plain) issue_int(s + NST, m); else issue_one(s + NST, m); }
            if (ahead && m < NF) read_frag(set ^ 1, m, s + 1);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    static_assert(TM * TN >= NF && TM * TN >= LPS, "a stage has fewer matrix instructions than reads or copies to place");

    wait_vm<(NST - 1) * LPS>();            // stage 0 landed
    __syncthreads();
    if (nk_int > 0) {
#pragma unroll
        for (int f = 0; f < NF; ++f) read_frag(0, f, 0);
    }

    int s = 0;
    for (; s + 1 + NST < nk_int; s += 2) {
        step(s, 0, true, true);
        step(s + 1, 1, true, true);
    }
    for (; s + 2 < nk_int; s += 2) {
        step(s, 0, false, true);
        step(s + 1, 1, false, true);
    }
    if (s + 2 == nk_int) {
        step(s, 0, false, true);
        step(s + 1, 1, false, false);
        s += 2;
    } else if (s + 1 == nk_int) {
        step(s, 0, false, false);
        s += 1;
    }

    const int tw = t0 + wm * TM * 32, nw = n0 + wn * TN * 32;
    if constexpr (RAW) {
        wait_vm<0>();                      // drain the look-ahead DMA before the wave ends
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = nw + j * 32 + l32;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int t = tw + i * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (t < a.T && n < a.N) a.acc[(size_t)t * a.ldacc + n] = (int)acc[i][j][r];
                }
            }
        return;
    }

    // Dequantization: the accumulators are exact integers already in binary32.
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
            const int lr = wm * TM * 32 + i * 32 + 8 * rq + 4 * g;
            const float4 sa4 = *reinterpret_cast<const float4*>(&lds_sa[lr]);
            const float4 sh4 = *reinterpret_cast<const float4*>(&lds_sh[lr]);
            const float sa_[4] = {sa4.x, sa4.y, sa4.z, sa4.w}, sh_[4] = {sh4.x, sh4.y, sh4.z, sh4.w};
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const int r = rq * 4 + rr;
                    acc[i][j][r] = __builtin_fmaf(acc[i][j][r], sa_[rr] * c_sw[j],
                                                  __builtin_fmaf(sh_[rr], c_wr[j], c_bv[j]));
                }
        }

    // fp16 outlier stages: 16 columns each, one matrix step, same protocol as the FP6 stages (fragments
    // of stage s + 1 are read while the matrix instructions of stage s run; one barrier per stage)
    auto wide_step = [&](int s, int set) __attribute__((always_inline)) {
        wait_vm<(NST - 2) * LPS>();
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        const uint8_t* nxt = lds + ((s + 1) % NST) * ST_BYTES;
#pragma unroll
        for (int m = 0; m < TM * TN; ++m) {
            const int i = m / TN, j = m % TN;
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, FP[set][i]),
                                                               __builtin_bit_cast(v8h, FP[set][TM + j]), acc[i][j], 0, 0, 0);
            if (m < LPS) issue_one(s + NST, m);
            if (m < NF) FP[set ^ 1][m] = *reinterpret_cast<const uint4*>(nxt + rdf[m]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    if (s < nk) {
        wait_vm<(NST - 1) * LPS>();        // first fp16 stage landed
        __syncthreads();
        const uint8_t* st = lds + (s % NST) * ST_BYTES;
#pragma unroll
        for (int f = 0; f < NF; ++f) FP[0][f] = *reinterpret_cast<const uint4*>(st + rdf[f]);
        for (; s + 1 < nk; s += 2) {
            wide_step(s, 0);
            wide_step(s + 1, 1);
        }
        if (s < nk) { wide_step(s, 0); ++s; }
    }

    wait_vm<0>();                          // drain the look-ahead DMA before the wave ends
    __half* __restrict__ y = static_cast<__half*>(a.y);
    // Output through LDS (each wave parks its fp16 tile in its own slice of the dead stage ring and
    // writes whole row segments as 16-byte pieces); needs 16-byte aligned output rows.
    constexpr int WROW = (NWAVES * TM * 32 * (TN * 64 + 16) <= NST * ST_BYTES) ? TN * 64 + 16 : TN * 64;
    constexpr int WBUF = TM * 32 * WROW;
    static_assert(NWAVES * WBUF <= NST * ST_BYTES, "stage ring too small to park the output tile");
    const bool vec_ok = !a.fp_only && ((reinterpret_cast<uintptr_t>(a.y) & 15u) == 0) && (a.ldy % 8 == 0);
    if (vec_ok) {
        __syncthreads();                   // every wave is past its last read of the stage ring
        uint8_t* wbuf = lds + wave_u * WBUF;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = i * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                    *reinterpret_cast<__half*>(wbuf + row * WROW + (j * 32 + l32) * 2) = __float2half(acc[i][j][r]);
                }
        constexpr int CH = TN * 4;                       // 16-byte pieces per row
        constexpr int RPS = 64 / CH;                     // rows per store instruction
        const int prow = lane / CH, pch = lane % CH;
#pragma unroll
        for (int p = 0; p < (TM * 32 + RPS - 1) / RPS; ++p) {
            const int row = p * RPS + prow;
            if (prow >= RPS || row >= TM * 32) continue;
            const uint4 v = *reinterpret_cast<const uint4*>(wbuf + row * WROW + pch * 16);
            const int t = tw + row, n = nw + pch * 8;
            if (t < a.T) {
                __half* dst = y + (size_t)t * a.ldy + n;
                if (n + 8 <= a.N) {
                    store16_through(dst, v);
                } else {
                    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (n + e < a.N)
                            reinterpret_cast<uint16_t*>(dst)[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
                }
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = nw + j * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int t = tw + i * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                if (t < a.T && n < a.N) {
                    if (a.fp_only) reinterpret_cast<float*>(a.y)[(size_t)t * a.ldy + n] = acc[i][j][r];
                    else y[(size_t)t * a.ldy + n] = __float2half(acc[i][j][r]);
                }
            }
        }
}

// Signed 4-bit weights (two per byte, column 2p in the low nibble) -> FP6 panels.  One thread per
// (row, group of 32 columns).  Offline step.
__global__ __launch_bounds__(256) void weight_pack_fp6_kernel(const uint8_t* __restrict__ w_q, int ldw, int N, int K_b,
                                                              uint32_t* __restrict__ w6) {
    const int S = fp6::stages(K_b);
    const int groups = 2 * S;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)N * groups) return;
    const int n = (int)(idx / groups), G = (int)(idx % groups);
    const uint8_t* src = w_q + (size_t)n * ldw + G * 16;
    uint32_t cw[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint32_t v = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int col = G * 32 + i * 8 + b * 2;                 // first column of this byte
            uint32_t byte = (col < K_b) ? src[i * 4 + b] : 0u;      // columns at or beyond K_b: value 0
            if (col + 1 >= K_b) byte &= 0x0Fu;
            v |= byte << (8 * b);
        }
        cw[i] = v ^ 0x88888888u;                                    // two's complement -> unsigned code (value + 8)
    }
    // 32 columns = four 48-bit strings at bits 0, 48, 96, 144
    const uint64_t e0 = fp6::pack8(cw[0]), e1 = fp6::pack8(cw[1]), e2 = fp6::pack8(cw[2]), e3 = fp6::pack8(cw[3]);
    uint32_t d[6];
    d[0] = (uint32_t)e0;
    d[1] = (uint32_t)(e0 >> 32) | (uint32_t)(e1 << 16);
    d[2] = (uint32_t)(e1 >> 16);
    d[3] = (uint32_t)e2;
    d[4] = (uint32_t)(e2 >> 32) | (uint32_t)(e3 << 16);
    d[5] = (uint32_t)(e3 >> 16);
    uint32_t* blk = w6 + ((size_t)(G >> 1) * N + n) * 12;         // the row's 48-byte block of this stage
#pragma unroll
    for (int i = 0; i < 6; ++i) blk[fp6::block_dword(G & 1, i)] = d[i];
}

template <int BM, int BN, int WM, int WN, int NST, int GM, int MODE>
hipError_t launch_cfg(const GemmArgs& a, hipStream_t stream) {
    const int tiles = ((a.T + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    hipLaunchKernelGGL((gemm_fp6_kernel<BM, BN, WM, WN, NST, GM, MODE>), dim3(tiles), dim3(WM * WN * 64), 0, stream, a);
    return hipGetLastError();
}

template <int MODE>
hipError_t dispatch6(const GemmArgs& a, hipStream_t stream) {
    // One workgroup of eight waves per CU, so a launch runs in ceil(tiles / 256) rounds; a 256 x 192 tile
    // takes about 1.4x as long as a 256 x 128 one.  Few tokens or few tiles: 128 x 128 tiles, two
    // workgroups per CU.  Ring depths as measured: six buffers for the 256 x 192 tile (five 1 %, seven, all
    // the LDS holds, 5 % slower), eight for the 256 x 128 tile (six 2 %, seven 6 % slower).
    auto rounds = [&](int bm, int bn) { return (((long)(a.T + bm - 1) / bm) * ((a.N + bn - 1) / bn) + 255) / 256; };
    const long tiles_128 = (long)((a.T + 255) / 256) * ((a.N + 127) / 128);
    if (a.T <= 128 || tiles_128 < 256) return launch_cfg<128, 128, 2, 2, 6, 0, MODE>(a, stream);
    if (1.4 * (double)rounds(256, 192) <= (double)rounds(256, 128)) return launch_cfg<256, 192, 4, 2, 6, 4, MODE>(a, stream);
    return launch_cfg<256, 128, 4, 2, 8, 4, MODE>(a, stream);
}

}  // namespace

hipError_t launch_gemm_fp6(const GemmArgs& a, hipStream_t stream) {
    if (a.T <= 0 || a.N <= 0) return hipSuccess;
    return a.y ? dispatch6<0>(a, stream) : dispatch6<1>(a, stream);
}

hipError_t launch_weight_pack_fp6(const void* w_q, int ldw, int N, int K_b, void* w6, hipStream_t stream) {
    if (N <= 0 || K_b <= 0) return hipSuccess;
    const long total = (long)N * 2 * fp6::stages(K_b);
    hipLaunchKernelGGL(weight_pack_fp6_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       static_cast<const uint8_t*>(w_q), ldw, N, K_b, static_cast<uint32_t*>(w6));
    return hipGetLastError();
}

}  // namespace quik
