// QUIK-4B linear layer with the integer product computed on the FP6 matrix pipe of gfx950
// (Algorithm 1 of arXiv 2310.09259: "INTmatmul", "Dequantization", "FPmatmul", final add; the
// epilogue fusion of Section 3.4).  The signed 4-bit codes travel as E3M2 patterns (see
// quik_fp6_device.h: exact, and the fp32 accumulators hold the exact integer dot products), so the
// K loop is DMA -> LDS -> registers -> v_mfma_f32_32x32x64_f8f6f4 with no widening work at all, at
// twice the int8 rate of the matrix pipe.
//
// A workgroup of WM x WN waves owns a BM x BN output tile.  A stage is 128 columns = one 96-byte block per
// operand row; the operands are stored stage by stage (quik_fp6_device.h), so the tile's rows of a stage
// are one contiguous run of BM * 96 (BN * 96) bytes that 16-byte-per-lane DMA instructions copy global ->
// LDS as it is, whole cache lines per instruction; three stage buffers.  Lane (row l%32, half g = l/32)
// reads, per 64-column step, 16 bytes (dwords 0..3 of its group) and 8 bytes (dwords 4, 5); the 16-byte
// pieces of a block are exchanged pairwise in every second group of eight rows (by the DMA's choice of
// source piece) so that the rows one read instruction touches fall into distinct banks.  The fp16
// outlier columns run through the same ring as stages of 32 columns (64-byte rows, 16 rows per DMA
// instruction), with the dequantized integer part as the C operand of v_mfma_f32_32x32x16_f16, whose
// accumulator layout is the same.  Rows beyond T / N are out of range for the per-stage buffer
// descriptors and arrive as zeros (the E3M2 pattern of 0); columns beyond K_b are zero padding.
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

__device__ __forceinline__ int swz_f(int r) { return (r >> 2) & 3; }   // fp16 stages: 64-byte rows, four pieces
__device__ __forceinline__ int swz_6(int r) { return (r >> 3) & 1; }   // FP6 stages: 96-byte rows, pieces paired

// descriptor r moved forward by `bytes`
__device__ __forceinline__ v4i advance(v4i r, uint32_t bytes) {
    const uint64_t base = (((uint64_t)(uint32_t)r[1]) << 32 | (uint32_t)r[0]) + bytes;
    r[0] = (int)(uint32_t)base;
    r[1] = (int)(uint32_t)(base >> 32);
    return r;
}

// MODE 0: fused epilogue, fp16 output; MODE 1: the integer accumulators as INT32.
template <int BM, int BN, int WM, int WN, int GM, int MODE>
__global__ __launch_bounds__(WM * WN * 64, (WM * WN == 8) ? 1 : 2) void gemm_fp6_kernel(GemmArgs a) {
    constexpr bool RAW = MODE != 0;
    // claim the whole register budget of the launch bounds, so that the highest allocated register is
    // never a live one (see the note in the row-quantization kernel)
    asm volatile("" ::: "v255");
    constexpr int NWAVES = WM * WN, NT = NWAVES * 64;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32, NF = TM + TN;
    constexpr int NST = 3;
    constexpr int A_BYTES = BM * 96, B_BYTES = BN * 96, ST_BYTES = A_BYTES + B_BYTES;
    // DMA instructions of a stage (1 KB each): FP6 stages BM * 96 / 1024 and BN * 96 / 1024, fp16 stages
    // BM / 16 and BN / 16.  Slots of a wave per stage: S_A for A, then S_B for B; instruction
    // i = wave + NWAVES * (slot within its operand); a slot whose i does not exist is issued empty so
    // that every wave counts the same number of DMA instructions.
    constexpr int N_A = BM * 96 / 1024, N_B = BN * 96 / 1024, N_AF = BM / 16, N_BF = BN / 16;
    constexpr int S_A = (N_A + NWAVES - 1) / NWAVES, S_B = (N_B + NWAVES - 1) / NWAVES;
    constexpr int LPS = S_A + S_B;
    static_assert(BM % 32 == 0 && BN % 32 == 0 && N_AF <= S_A * NWAVES && N_BF <= S_B * NWAVES, "slot count");
    static_assert((NST - 1) * LPS < 64, "vmcnt range");
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
    const int nk_fp = RAW ? 0 : (fp_bytes + 63) / 64;
    const int nk = nk_int + nk_fp;
    const int lda_fp = a.ldo * 2, ldb_fp = a.ldwo * 2;
    const int T_ = a.T, N_ = a.N;                         // values, so that nothing takes the address of an argument

    // stage 0 of the tile's rows; stage s lies s * T * 96 (s * N * 96) bytes further on
    const v4i rA = make_rsrc((const uint8_t*)a.xq + (size_t)t0 * 96, (size_t)(a.T - t0) * 96);
    const v4i rB = make_rsrc((const uint8_t*)a.w_q + (size_t)n0 * 96, (size_t)(a.N - n0) * 96);
    const v4i rAf = make_rsrc(a.n_out ? (const uint8_t*)a.x_out + (size_t)t0 * lda_fp : (const uint8_t*)a.xq,
                              a.n_out ? (size_t)(a.T - t0) * lda_fp : 0);
    const v4i rBf = make_rsrc(a.n_out ? (const uint8_t*)a.w_out + (size_t)n0 * ldb_fp : (const uint8_t*)a.xq,
                              a.n_out ? (size_t)(a.N - n0) * ldb_fp : 0);
    const uint32_t lds_base = lds_addr(lds);

    // Per-lane DMA source offsets.  FP6 stage, slot q: lane handles the 16-byte piece p = 64 i + lane of the
    // tile's run, i.e. piece p % 6 of row p / 6, and fetches the piece the swizzle assigns to that place.
    uint32_t vo_a[S_A], vo_b[S_B];
#pragma unroll
    for (int q = 0; q < S_A; ++q) {
        const int pc = 64 * (wave_u + NWAVES * q) + lane, row = pc / 6, c = pc - 6 * row;
        vo_a[q] = (uint32_t)(row * 96 + ((c ^ swz_6(row)) << 4));
    }
#pragma unroll
    for (int q = 0; q < S_B; ++q) {
        const int pc = 64 * (wave_u + NWAVES * q) + lane, row = pc / 6, c = pc - 6 * row;
        vo_b[q] = (uint32_t)(row * 96 + ((c ^ swz_6(row)) << 4));
    }
    // fp16 stage: 16 rows (lane / 4) x four pieces of a 64-byte stage row per instruction
    const int colF = ((lane & 3) ^ ((lane >> 4) & 3)) * 16;
    const uint32_t vo_af = (uint32_t)((lane >> 2) * lda_fp + colF), vo_bf = (uint32_t)((lane >> 2) * ldb_fp + colF);
    // DMA slot j of stage s (int part, fp16 part, or past the end: every lane out of range)
    auto issue_one = [&](int s, int j) __attribute__((always_inline)) {
        const bool isb = j >= S_A;
        const int seq = isb ? j - S_A : j;
        const int i = wave_u + NWAVES * seq;                    // instruction of this operand (wave-uniform)
        const uint32_t sb = (uint32_t)(s % NST) * ST_BYTES;
        const bool fp = s >= nk_int;
        uint32_t vo = kOob;
        bool exists;
        uint32_t dst;
        if (!fp) {
            exists = i < (isb ? N_B : N_A);
            if (s < nk && exists) vo = isb ? vo_b[isb ? seq : 0] : vo_a[isb ? 0 : seq];
            dst = sb + (isb ? A_BYTES : 0) + i * 1024;
        } else {
            exists = i < (isb ? N_BF : N_AF);
            const int c0 = 64 * (s - nk_int);
            if (s < nk && exists && c0 + colF < fp_bytes)
                vo = (isb ? vo_bf : vo_af) + (uint32_t)(i * 16 * (isb ? ldb_fp : lda_fp) + c0);
            dst = sb + (isb ? BM * 64 : 0) + i * 1024;
        }
        dst = lds_base + (exists ? dst : (uint32_t)DUMMY);
        if (fp) dma16(isb ? rBf : rAf, dst, vo, 0);
        else if (isb) dma16(advance(rB, (uint32_t)s * (uint32_t)N_ * 96u), dst, vo, 0);
        else dma16(advance(rA, (uint32_t)s * (uint32_t)T_ * 96u), dst, vo, 0);
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

    // LDS read addresses of this lane's row of every fragment.  FP6 stage: piece 2 ks + g of the row's
    // 96-byte block (16 bytes) and 8 bytes at 64 + 16 g + 8 ks; fp16 stage: piece 2 ks + g of a 64-byte row.
    uint32_t rdp[NF][2], rdq[NF], rdf[NF][2];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        const int r = (f < TM) ? (wm * TM * 32 + f * 32 + l32) : (wn * TN * 32 + (f - TM) * 32 + l32);
        const uint32_t b6 = (f < TM ? 0 : A_BYTES) + r * 96, bf = (f < TM ? 0 : BM * 64) + r * 64;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            rdp[f][ks] = b6 + (((ks * 2 + g) ^ swz_6(r)) << 4);
            rdf[f][ks] = bf + (((ks * 2 + g) ^ swz_f(r)) << 4);
        }
        rdq[f] = b6 + 64 + ((g ^ swz_6(r)) << 4);
    }
    // two fragment sets: the matrix instructions of one 64-column step run on one set while the
    // LDS reads of the next step fill the other
    uint4 FP[2][NF];
    uint2 FQ[2][NF];
    auto read_p = [&](int set, int f, int s, int ks) __attribute__((always_inline)) {
        const uint32_t ad = (s >= nk_int) ? rdf[f][ks] : rdp[f][ks];
        FP[set][f] = *reinterpret_cast<const uint4*>(lds + (s % NST) * ST_BYTES + ad);
    };
    auto read_q = [&](int set, int f, int s, int ks) __attribute__((always_inline)) {
        FQ[set][f] = *reinterpret_cast<const uint2*>(lds + (s % NST) * ST_BYTES + rdq[f] + 8 * ks);
    };

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // Step ks of stage s.  Before its second step a stage's successor must have landed for everybody
    // (its first fragments are read during that step); all reads of stage s itself have completed by
    // then, so its buffer is refilled with stage s + NST right away, one DMA instruction per matrix
    // instruction.
    auto step = [&](int s, int ks, bool wide) __attribute__((always_inline)) {
        if (ks == 1) {
            wait_vm<(NST - 2) * LPS>();
            __syncthreads();
        }
        const int ns = ks ? s + 1 : s, nks = ks ^ 1;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < TM * TN; ++m) {
            const int i = m / TN, j = m % TN;
            if (!wide) {
                const v8i oa = v8i{(int)FP[ks][i].x, (int)FP[ks][i].y, (int)FP[ks][i].z, (int)FP[ks][i].w,
                                   (int)FQ[ks][i].x, (int)FQ[ks][i].y, 0, 0};
                const v8i ob = v8i{(int)FP[ks][TM + j].x, (int)FP[ks][TM + j].y, (int)FP[ks][TM + j].z,
                                   (int)FP[ks][TM + j].w, (int)FQ[ks][TM + j].x, (int)FQ[ks][TM + j].y, 0, 0};
#ifndef QF_NOMFMA
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(oa, ob, acc[i][j], 3, 3, 0, 0, 0, 0);
#else
                asm volatile("" :: "v"(oa), "v"(ob));
#endif
            } else {
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, FP[ks][i]),
                                                                   __builtin_bit_cast(v8h, FP[ks][TM + j]),
                                                                   acc[i][j], 0, 0, 0);
            }
            if (ks == 1) {
                constexpr int PER = (TM * TN >= LPS) ? TM * TN / LPS : 1;
#ifndef QF_NODMA
                if (m % PER == 0 && m / PER < LPS) issue_one(s + NST, m / PER);
#endif
                if constexpr (TM * TN < LPS) {
                    if (m == TM * TN - 1) {
#pragma unroll
                        for (int d = TM * TN; d < LPS; ++d) issue_one(s + NST, d);
                    }
                }
            }
#ifndef QF_NOREAD
            if (m < NF) { read_p(nks, m, ns, nks); read_q(nks, m, ns, nks); }
#endif
            if constexpr (TM * TN < NF) {
                if (m == TM * TN - 1) {
#pragma unroll
                    for (int f = TM * TN; f < NF; ++f) { read_p(nks, f, ns, nks); read_q(nks, f, ns, nks); }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    wait_vm<(NST - 1) * LPS>();            // stage 0 landed
    __syncthreads();
#pragma unroll
    for (int f = 0; f < NF; ++f) { read_p(0, f, 0, 0); read_q(0, f, 0, 0); }

    int s = 0;
    for (; s < nk_int; ++s) {
        step(s, 0, false);
        step(s, 1, false);
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

    // fp16 outlier stages: 32 columns each, two matrix steps of 16 (plane P geometry; the 8 bytes read
    // from the plane Q region are ignored)
    for (; s < nk; ++s) {
        step(s, 0, true);
        step(s, 1, true);
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
                    *reinterpret_cast<uint4*>(dst) = v;
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
    const int groups = 4 * S;
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
    uint32_t* blk = w6 + ((size_t)(G >> 2) * N + n) * 24;         // the row's 96-byte block of this stage
#pragma unroll
    for (int i = 0; i < 6; ++i) blk[fp6::block_dword(G & 3, i)] = d[i];
}

template <int BM, int BN, int WM, int WN, int GM, int MODE>
hipError_t launch_cfg(const GemmArgs& a, hipStream_t stream) {
    const int tiles = ((a.T + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    hipLaunchKernelGGL((gemm_fp6_kernel<BM, BN, WM, WN, GM, MODE>), dim3(tiles), dim3(WM * WN * 64), 0, stream, a);
    return hipGetLastError();
}

template <int MODE>
hipError_t dispatch6(const GemmArgs& a, hipStream_t stream) {
    const long big = (long)((a.T + 255) / 256) * ((a.N + 191) / 192);
    if (a.T > 128 && big >= 128) return launch_cfg<256, 192, 4, 2, 4, MODE>(a, stream);
    return launch_cfg<128, 128, 2, 2, 0, MODE>(a, stream);
}

}  // namespace

hipError_t launch_gemm_fp6(const GemmArgs& a, hipStream_t stream) {
    if (a.T <= 0 || a.N <= 0) return hipSuccess;
    return a.y ? dispatch6<0>(a, stream) : dispatch6<1>(a, stream);
}

hipError_t launch_weight_pack_fp6(const void* w_q, int ldw, int N, int K_b, void* w6, hipStream_t stream) {
    if (N <= 0 || K_b <= 0) return hipSuccess;
    const long total = (long)N * 4 * fp6::stages(K_b);
    hipLaunchKernelGGL(weight_pack_fp6_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       static_cast<const uint8_t*>(w_q), ldw, N, K_b, static_cast<uint32_t*>(w6));
    return hipGetLastError();
}

}  // namespace quik
