// QUIK-4B linear layer for 2:4-sparse weights, the integer product computed by the sparse int8 matrix
// instruction of gfx950 (Algorithm 1 of arXiv 2310.09259: "INTmatmul", "Dequantization", "FPmatmul",
// final add, with the epilogue fusion of Section 3.4; the weight format is the joint INT4 + 2:4 one of
// Section 4.3.2).  v_smfmac_i32_32x32x64_i8 runs at twice the dense int8 rate and accumulates exactly in
// INT32.  Operand formats and the measured register layout of the instruction: quik_sp24_device.h.
//
// The sparse operand is the instruction's first one, so it carries the weights: an accumulator register
// belongs to an output channel and a lane to a token, the transpose of the dense kernels' arrangement.
// Per-token parameters therefore live in registers, per-channel ones in LDS, and a lane converts four
// neighbouring channels of its token at a time.
//
// A workgroup of WM x WN waves owns a BM (tokens) x BN (channels) output tile.  A stage is 64 columns = one
// matrix step: 32 bytes per token row and 32 per weight row, stored stage by stage, so the tile's rows of
// a stage are two contiguous runs that 16-byte-per-lane DMA instructions copy global -> LDS (32 rows per
// instruction, the two 16-byte pieces of a row exchanged in every second group of eight rows, which keeps
// the 16-byte LDS reads free of bank conflicts).  The stage ring takes most of the LDS.  The packed words
// of stage s + 2 are read from LDS (one 16-byte read per fragment) and those of stage s + 1 widened to
// int8 (two or three VALU operations per two operand registers) while the matrix instructions of stage s
// issue; one workgroup barrier per two stages, after which the buffers just read are refilled.  Measured
// on MI355X: LDS read instructions of a wave do not hide behind its matrix instructions (their cost adds
// to the loop time whatever their latency slack), VALU work in these amounts does.  The fp16 outlier
// columns run through the same ring as stages of 16 columns of the same shape, with the dequantized
// integer part as the C operand of v_mfma_f32_32x32x16_f16 (weights first, so the accumulator layout is
// the same).  Rows beyond T / N are out of range for the per-stage buffer descriptors and arrive as
// zeros.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "quik_kernels.h"
#include "quik_gemm_device.h"
#include "quik_sp24_device.h"

namespace quik {

namespace {

using namespace gemm_dev;

typedef int v8i __attribute__((ext_vector_type(8)));

__device__ __forceinline__ int swz_f(int r) { return (r >> 3) & 1; }   // 32-byte rows, two pieces

// descriptor r moved forward by `bytes`
__device__ __forceinline__ v4i advance(v4i r, uint32_t bytes) {
    const uint64_t base = (((uint64_t)(uint32_t)r[1]) << 32 | (uint32_t)r[0]) + bytes;
    r[0] = (int)(uint32_t)base;
    r[1] = (int)(uint32_t)(base >> 32);
    return r;
}

// MODE 0: fused epilogue, fp16 output; MODE 1: the integer accumulators as INT32.
// NST: stage buffers of the ring; KS: stages per workgroup barrier.
template <int BM, int BN, int WM, int WN, int NST, int KS, int GM, int MODE>
__global__ __launch_bounds__(WM * WN * 64, (WM * WN == 8) ? 1 : 2) void gemm_sp24_kernel(GemmArgs a) {
    constexpr bool RAW = MODE != 0;
    // claim the whole register budget of the launch bounds, so that the highest allocated register is
    // never a live one (see the note in the row-quantization kernel)
    asm volatile("" ::: "v255");
    constexpr int NWAVES = WM * WN, NT = NWAVES * 64;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32, NF = TM + TN, SL = TM * TN;
    static_assert(sp24::kActBytes == 32 && sp24::kWgtBytes == 32, "every stage row is 32 bytes");
    // Integer and fp16 stages have the same shape in LDS: BM token rows, then BN channel rows, 32 bytes
    // each.  DMA instructions of a stage (1 KB = 32 rows each): N_A + N_B.  A wave issues LPS per stage:
    // instruction i = wave + NWAVES * slot; one that does not exist is issued empty so that every wave
    // counts the same number.
    constexpr int A_BYTES = BM * 32, B_BYTES = BN * 32, ST_BYTES = A_BYTES + B_BYTES;
    constexpr int N_A = BM / 32, N_B = BN / 32;
    constexpr int LPS = (N_A + N_B + NWAVES - 1) / NWAVES;
    static_assert(BM % 64 == 0 && BN % 64 == 0 && BN <= NT, "geometry");
    static_assert(NST * LPS < 64, "vmcnt range");
    static_assert(NST >= KS + 3, "ring too short");
    // Ring protocol.  The packed words of integer stage s + 2 are read from LDS while the matrix
    // instructions of stage s issue (and widened during stage s + 1), and the workgroup meets at a barrier
    // before every KS-th stage s (s % KS == 0).  At that barrier stages up to s + KS + 1 must have landed
    // (they are read before the next barrier), and stages up to s + 1 are in registers everywhere, so
    // during stage s' of the group its own buffer is refilled with stage s' + NST.  The prologue requests
    // stages 0 .. NST - 1.  (fp16 stages: read one stage ahead, a barrier before every stage.)
    constexpr int AHEAD = NST;
    constexpr int WAIT_BAR = (NST - KS - 2) * LPS;        // requests that may still be in flight at a barrier
    static_assert(SL >= 2 && SL >= LPS && SL >= TM, "a stage has too few matrix instructions to place its reads and copies");
    constexpr int DUMMY = NST * ST_BYTES;                 // 1 KB that empty DMA instructions clear

    __shared__ __align__(1024) uint8_t lds[NST * ST_BYTES + 1024];
    __shared__ __align__(16) float lds_sw[BN];            // scaleWeight / 256
    __shared__ __align__(16) float lds_wr[BN];            // wReduced
    __shared__ __align__(16) float lds_bv[BN];            // bias

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

    const int S = sp24::stages(a.K_b);
    const int nk_int = a.fp_only ? 0 : S;
    const int fp_bytes = a.n_out * 2;
    const int nk_fp = RAW ? 0 : (fp_bytes + 31) / 32;
    const int nk = nk_int + nk_fp;
    const int lda_fp = a.ldo * 2, ldb_fp = a.ldwo * 2;
    const uint32_t strideA = (uint32_t)a.T * sp24::kActBytes;                  // bytes from stage to stage
    const uint32_t strideB = (uint32_t)a.N * sp24::kWgtBytes;

    // stage 0 of the tile's rows
    const v4i rA = make_rsrc((const uint8_t*)a.xq + (size_t)t0 * sp24::kActBytes, (size_t)(a.T - t0) * sp24::kActBytes);
    const v4i rB = make_rsrc((const uint8_t*)a.w_q + (size_t)n0 * sp24::kWgtBytes, (size_t)(a.N - n0) * sp24::kWgtBytes);
    const v4i rAf = make_rsrc(a.n_out ? (const uint8_t*)a.x_out + (size_t)t0 * lda_fp : (const uint8_t*)a.xq,
                              a.n_out ? (size_t)(a.T - t0) * lda_fp : 0);
    const v4i rBf = make_rsrc(a.n_out ? (const uint8_t*)a.w_out + (size_t)n0 * ldb_fp : (const uint8_t*)a.xq,
                              a.n_out ? (size_t)(a.N - n0) * ldb_fp : 0);
    const uint32_t lds_base = lds_addr(lds);

    // 32-byte rows (activation stages and both operands of fp16 stages): an instruction copies 32 rows
    // (lane / 2), two 16-byte pieces each, exchanged in every second group of eight rows
    const int colF = ((lane & 1) ^ ((lane >> 4) & 1)) * 16;
    const uint32_t vo_a = (uint32_t)((lane >> 1) * 32 + colF);
    const uint32_t vo_af = (uint32_t)((lane >> 1) * lda_fp + colF), vo_bf = (uint32_t)((lane >> 1) * ldb_fp + colF);
    // DMA slot j of stage s (int part, fp16 part, or past the end: every lane out of range)
    auto issue_one = [&](int s, int j) __attribute__((always_inline)) {
        const int i = wave_u + NWAVES * j;                      // instruction of the stage (wave-uniform)
        const uint32_t sb = (uint32_t)(s % NST) * ST_BYTES;
        const bool fp = s >= nk_int;
        uint32_t vo = kOob, dst = (uint32_t)DUMMY;
        v4i r;
        if (!fp) {
            const bool isb = i >= N_A;
            const int ii = isb ? i - N_A : i;
            if (i < N_A + N_B) {
                dst = sb + (isb ? A_BYTES : 0) + ii * 1024;
                if (s < nk) vo = (uint32_t)(ii * 1024) + vo_a;
            }
            r = isb ? advance(rB, (uint32_t)s * strideB) : advance(rA, (uint32_t)s * strideA);
        } else {
            const bool isb = i >= N_A;
            const int ii = isb ? i - N_A : i;
            const int c0 = 32 * (s - nk_int);
            if (i < N_A + N_B) {
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
    // DMA slot j of an integer stage that exists (the hot loop's form)
    auto issue_int = [&](int s, int j) __attribute__((always_inline)) {
        const int i = wave_u + NWAVES * j;
        const bool isb = i >= N_A;
        const int ii = isb ? i - N_A : i;
        const bool exists = i < N_A + N_B;
        const uint32_t dst = exists ? (uint32_t)(s % NST) * ST_BYTES + (isb ? A_BYTES : 0) + ii * 1024 : (uint32_t)DUMMY;
        const uint32_t vo = exists ? (uint32_t)(ii * 1024) + vo_a : kOob;
        v4i r = isb ? advance(rB, (uint32_t)s * strideB) : advance(rA, (uint32_t)s * strideA);
        r = v4i{__builtin_amdgcn_readfirstlane(r[0]), __builtin_amdgcn_readfirstlane(r[1]),
                __builtin_amdgcn_readfirstlane(r[2]), __builtin_amdgcn_readfirstlane(r[3])};
        dma16(r, (uint32_t)__builtin_amdgcn_readfirstlane((int)(lds_base + dst)), vo, 0);
    };
    auto issue = [&](int s) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < LPS; ++j) issue_one(s, j);
    };

    // ---- epilogue parameters: per token in registers (a lane owns one token of every token fragment),
    // per channel through LDS.  They are requested before the first DMA, so that their (in-order) return
    // does not sit behind the stage loads, and first touched after the integer stages: an earlier use
    // would make the compiler wait for them and, with them, for every stage load requested since.
    float t_s[TM], t_z[TM];
    float p_wr = 0.0f;
    uint32_t p_sw = 0, p_bv = 0;                           // binary16 patterns
    if constexpr (!RAW) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int t = t0 + wm * TM * 32 + i * 32 + l32;
            t_s[i] = t < a.T ? a.scale[t] : 0.0f;
            t_z[i] = t < a.T ? a.zero[t] : 0.0f;
        }
        const uint16_t* __restrict__ wsc = static_cast<const uint16_t*>(a.w_scale);
        const uint16_t* __restrict__ bias = static_cast<const uint16_t*>(a.bias);
        if (tid < BN && !a.fp_only) {
            const int n = min(n0 + tid, a.N - 1);
            p_sw = wsc[n];
            p_bv = (bias ? bias : wsc)[n];                 // no branch here: a join would wait for the loads
            p_wr = a.w_reduced[n];
        }
    }

#pragma unroll
    for (int s = 0; s < AHEAD; ++s) issue(s);

    // LDS read addresses of this lane's row of every fragment (token fragments first): piece g of the
    // 32-byte row, exchanged as above
    uint32_t rdf[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        const int r = (f < TM) ? (wm * TM * 32 + f * 32 + l32) : (wn * TN * 32 + (f - TM) * 32 + l32);
        rdf[f] = (f < TM ? 0 : BM * 32) + r * 32 + ((g ^ swz_f(r)) << 4);
    }
    // two sets of packed fragments and two sets of widened operands, by stage parity: the matrix
    // instructions of stage s run on one set of operands while the words of stage s + 1 are widened into
    // the other and those of stage s + 2 arrive from LDS
    // (a weight fragment's packed words hold its index word too, which the matrix instruction takes as it
    // is: such a fragment is requested only after the last matrix instruction that uses the old index)
    uint4 RA[2][TM];
    uint4 RW[2][TN];                                       // x, y: values; z: index word
    v8i UA[2][TM];
    v4i UW[2][TN];
    uint4 FP[2][NF];                                       // fp16 stages

    auto read_frag = [&](int set, int f, int s) __attribute__((always_inline)) {
        const uint8_t* st = lds + (s % NST) * ST_BYTES;
        if (f < TM) RA[set][f] = *reinterpret_cast<const uint4*>(st + rdf[f]);
        else RW[set][f - TM] = *reinterpret_cast<const uint4*>(st + rdf[f]);
    };
    auto widen = [&](int set, int f) __attribute__((always_inline)) {
        constexpr uint32_t M = 0xF0F0F0F0u;
        if (f < TM) {
            const uint32_t w[4] = {RA[set][f].x, RA[set][f].y, RA[set][f].z, RA[set][f].w};
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                UA[set][f][2 * m] = (int)(w[m] & M);               // columns 8 m .. 8 m + 3, sixteen-fold
                UA[set][f][2 * m + 1] = (int)((w[m] << 4) & M);    // columns 8 m + 4 .. 8 m + 7
            }
        } else {
            const int j = f - TM;
            UW[set][j] = v4i{(int)((RW[set][j].x << 4) & M), (int)(RW[set][j].x & M), (int)((RW[set][j].y << 4) & M),
                             (int)(RW[set][j].y & M)};
        }
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // Integer stage s, set = s % 2 (BAR: s % KS == 0, the group's barrier comes first).  PLAIN: stage
    // s + NST is an integer stage; NEXT1 / NEXT2: stages s + 1 / s + 2 are.  Stage s + 1's words (they
    // arrived during the previous stage) are widened between the matrix instructions, stage s + 2's are
    // requested one fragment per slot.
    auto step = [&](int s, int set, bool bar, bool plain, bool next1, bool next2) __attribute__((always_inline)) {
        if (bar) {
            wait_vm<WAIT_BAR>();
            __syncthreads();
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < SL; ++m) {
            const int i = m / TN, j = m % TN;
            acc[i][j] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(UW[set][j], UA[set][i], acc[i][j], (int)RW[set][j].z, 0, 0);
            if (m < LPS) { if (plain) issue_int(s + AHEAD, m); else issue_one(s + AHEAD, m); }
            if (next2) {
                if (m < TM) read_frag(set, m, s + 2);
                if (i == TM - 1) read_frag(set, TM + j, s + 2);
            }
            if (next1) {
#pragma unroll
                for (int f = 0; f < NF; ++f)
                    if (f * SL / NF == m) widen(set ^ 1, f);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    wait_vm<(NST - 2) * LPS>();            // stages 0 and 1 landed
    __syncthreads();
    if (nk_int > 0) {
#pragma unroll
        for (int f = 0; f < NF; ++f) read_frag(0, f, 0);
    }
    if (nk_int > 1) {
#pragma unroll
        for (int f = 0; f < NF; ++f) read_frag(1, f, 1);
    }
    if (nk_int > 0) {
#pragma unroll
        for (int f = 0; f < NF; ++f) widen(0, f);
    }

    static_assert(KS == 1 || KS == 2, "the loops below step two stages at a time");
    constexpr bool BAR1 = KS == 1;         // the odd stage of a pair opens a group only if groups are single stages
    int s = 0;
    for (; s + 1 + AHEAD < nk_int; s += 2) {
        step(s, 0, true, true, true, true);
        step(s + 1, 1, BAR1, true, true, true);
    }
    for (; s + 1 < nk_int; s += 2) {
        step(s, 0, true, false, true, s + 2 < nk_int);
        step(s + 1, 1, BAR1, false, s + 2 < nk_int, s + 3 < nk_int);
    }
    if (s < nk_int) {
        step(s, 0, true, false, false, false);
        s += 1;
    }

    // lane: token tw + 32 i + l32; register r of fragment j: channel nw + 32 j + 8 (r / 4) + 4 g + r % 4
    const int tw = t0 + wm * TM * 32, nw = n0 + wn * TN * 32;
    if constexpr (RAW) {
        wait_vm<0>();                      // drain the look-ahead DMA before the wave ends
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int t = tw + i * 32 + l32;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int n = nw + j * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (t < a.T && n < a.N) a.acc[(size_t)t * a.ldacc + n] = acc[i][j][r] >> 8;   // exact: a multiple of 256
                }
            }
        return;
    }

    // Dequantization: the accumulators are 256 times the integer dot products (the factor rides on the
    // weight scale); the conversion to binary32 is exact (at most 24 significant bits).
    if (tid < BN) {
        lds_sw[tid] = __half2float(__ushort_as_half((unsigned short)p_sw)) * (1.0f / 256.0f);   // exact power-of-two factor
        lds_wr[tid] = p_wr;
        lds_bv[tid] = a.bias ? __half2float(__ushort_as_half((unsigned short)p_bv)) : 0.0f;
    }
    float t_h[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) t_h[i] = t_z[i] + 8.0f * t_s[i];     // zeroAct + halfRange * scaleAct
    __syncthreads();
    v16f cf[TM][TN];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
            const int lc = wn * TN * 32 + j * 32 + 8 * rq + 4 * g;
            const float4 sw4 = *reinterpret_cast<const float4*>(&lds_sw[lc]);
            const float4 wr4 = *reinterpret_cast<const float4*>(&lds_wr[lc]);
            const float4 bv4 = *reinterpret_cast<const float4*>(&lds_bv[lc]);
            const float sw_[4] = {sw4.x, sw4.y, sw4.z, sw4.w}, wr_[4] = {wr4.x, wr4.y, wr4.z, wr4.w};
            const float bv_[4] = {bv4.x, bv4.y, bv4.z, bv4.w};
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const int r = rq * 4 + rr;
                    cf[i][j][r] = __builtin_fmaf((float)acc[i][j][r], t_s[i] * sw_[rr],
                                                 __builtin_fmaf(t_h[i], wr_[rr], bv_[rr]));
                }
        }

    // fp16 outlier stages: 16 columns each, one matrix step; stage s + 1 is read while the matrix
    // instructions of stage s issue, and stage s's buffer (read during stage s - 1, before this barrier)
    // is refilled
    auto wide_step = [&](int s, int set) __attribute__((always_inline)) {
        wait_vm<WAIT_BAR>();
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        const uint8_t* nxt = lds + ((s + 1) % NST) * ST_BYTES;
#pragma unroll
        for (int m = 0; m < SL; ++m) {
            const int i = m / TN, j = m % TN;
            cf[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, FP[set][TM + j]),
                                                              __builtin_bit_cast(v8h, FP[set][i]), cf[i][j], 0, 0, 0);
            if (m < LPS) issue_one(s + AHEAD, m);
            if (m < NF) FP[set ^ 1][m] = *reinterpret_cast<const uint4*>(nxt + rdf[m]);
            if (SL < NF && m == SL - 1) {
#pragma unroll
                for (int f = SL; f < NF; ++f) FP[set ^ 1][f] = *reinterpret_cast<const uint4*>(nxt + rdf[f]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    if (s < nk) {
        // the first fp16 stage has landed (at most KS + 1 stages behind the last barrier's stage); the wait
        // and barrier matter only if there was no integer stage
        wait_vm<WAIT_BAR>();
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
    // Output through LDS: each wave parks its fp16 tile (token rows) in its own slice of the dead stage
    // ring, four channels = 8 bytes per lane and write, and stores whole row segments as 16-byte pieces;
    // needs 16-byte aligned output rows.
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
                for (int rq = 0; rq < 4; ++rq) {
                    const __half2 h0 = __floats2half2_rn(cf[i][j][4 * rq], cf[i][j][4 * rq + 1]);
                    const __half2 h1 = __floats2half2_rn(cf[i][j][4 * rq + 2], cf[i][j][4 * rq + 3]);
                    uint2 v;
                    v.x = __builtin_bit_cast(uint32_t, h0);
                    v.y = __builtin_bit_cast(uint32_t, h1);
                    *reinterpret_cast<uint2*>(wbuf + (i * 32 + l32) * WROW + (j * 32 + 8 * rq + 4 * g) * 2) = v;
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
            const int t = tw + i * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int n = nw + j * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                if (t < a.T && n < a.N) {
                    if (a.fp_only) reinterpret_cast<float*>(a.y)[(size_t)t * a.ldy + n] = cf[i][j][r];
                    else y[(size_t)t * a.ldy + n] = __float2half(cf[i][j][r]);
                }
            }
        }
}

// Small-T variant (T <= 32 TM): the layer is bound by streaming the weights, so the point is many bytes in
// flight per CU and many workgroups.  A workgroup owns a 32 TM (tokens) x 32 (channels) output tile and its
// four waves split K: every wave streams its own quarter of the stages (1 KB of weights and TM KB of
// activations each, one DMA instruction per KB) through a private ring, with no workgroup barrier in the
// main loop (a wave waits only for its own DMA).  The four partial INT32 accumulators are summed exactly
// through LDS; wave 0 then dequantizes, adds the fp16 outlier product (every wave takes every fourth
// 16-column step, operands straight from global memory, requested before the weight stream starts) and
// stores.
template <int TM, int NST, int MODE>
__global__ __launch_bounds__(256) void gemm_sp24_skinny(GemmArgs a) {
    constexpr bool RAW = MODE != 0;
    constexpr int BM = 32 * TM, A_BYTES = BM * 32, ST_BYTES = A_BYTES + 1024, RING = NST * ST_BYTES, LPS = TM + 1;
    constexpr int RED_BYTES = 2 * TM * 16 * 64 * 4;        // one wave's INT32 accumulators + fp32 outlier partials
    constexpr int LDS_BYTES = (4 * RING > 3 * RED_BYTES) ? 4 * RING : 3 * RED_BYTES;
    static_assert((NST - 1) * LPS < 64, "vmcnt range");
    __shared__ __align__(1024) uint8_t lds[LDS_BYTES];
    __shared__ float prm_sw[32], prm_wr[32], prm_bv[32];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5;
    const int tiles_m = (a.T + BM - 1) / BM;
    const int t0 = (blockIdx.x % tiles_m) * BM, n0 = (blockIdx.x / tiles_m) * 32;

    const int nk = a.fp_only ? 0 : sp24::stages(a.K_b);
    const int s_begin = (int)((long)nk * wave / 4), s_end = (int)((long)nk * (wave + 1) / 4);   // this wave's stages
    const uint32_t strideA = (uint32_t)a.T * sp24::kActBytes, strideB = (uint32_t)a.N * sp24::kWgtBytes;
    const v4i rA = make_rsrc((const uint8_t*)a.xq + (size_t)t0 * sp24::kActBytes, (size_t)(a.T - t0) * sp24::kActBytes);
    const v4i rB = make_rsrc((const uint8_t*)a.w_q + (size_t)n0 * sp24::kWgtBytes, (size_t)(a.N - n0) * sp24::kWgtBytes);

    uint8_t* ring = lds + wave * RING;
    const uint32_t ring_addr = lds_addr(ring);
    // 32 rows of 32 bytes per instruction, pieces exchanged in every second group of eight rows
    const uint32_t vo = (uint32_t)((lane >> 1) * 32 + (((lane & 1) ^ ((lane >> 4) & 1)) * 16));
    auto issue = [&](int s) __attribute__((always_inline)) {   // stage s of this wave's range (or beyond: nothing is read)
        const uint32_t sb = (uint32_t)((s - s_begin) % NST) * ST_BYTES;
        const bool live = s < s_end;
        v4i ra = advance(rA, (uint32_t)s * strideA), rb = advance(rB, (uint32_t)s * strideB);
        ra = v4i{__builtin_amdgcn_readfirstlane(ra[0]), __builtin_amdgcn_readfirstlane(ra[1]),
                 __builtin_amdgcn_readfirstlane(ra[2]), __builtin_amdgcn_readfirstlane(ra[3])};
        rb = v4i{__builtin_amdgcn_readfirstlane(rb[0]), __builtin_amdgcn_readfirstlane(rb[1]),
                 __builtin_amdgcn_readfirstlane(rb[2]), __builtin_amdgcn_readfirstlane(rb[3])};
#pragma unroll
        for (int i = 0; i < TM; ++i)
            dma16(ra, (uint32_t)__builtin_amdgcn_readfirstlane((int)(ring_addr + sb + i * 1024)), live ? vo + i * 1024 : kOob, 0);
        dma16(rb, (uint32_t)__builtin_amdgcn_readfirstlane((int)(ring_addr + sb + A_BYTES)), live ? vo : kOob, 0);
    };
    const uint32_t rd = (uint32_t)(l32 * 32 + ((g ^ swz_f(l32)) << 4));   // this lane's piece of its row

    // ---- everything the epilogue needs is requested before the weight stream starts
    constexpr int PF = (TM == 1) ? 4 : 2;                  // prefetched outlier steps per wave
    float t_s[TM], t_z[TM];
    uint4 pfa[PF][TM], pfb[PF];
    const int fsteps = (a.n_out + 15) >> 4;                // 16-column steps of the outlier product
    const __half* __restrict__ xo = static_cast<const __half*>(a.x_out);
    const __half* __restrict__ wo = static_cast<const __half*>(a.w_out);
    const int n2 = min(n0 + l32, a.N - 1);
    if constexpr (!RAW) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int t = t0 + i * 32 + l32;
            const bool ok = t < a.T && !a.fp_only;
            t_s[i] = ok ? a.scale[t] : 0.0f;
            t_z[i] = ok ? a.zero[t] : 0.0f;
        }
        if (tid < 32) {
            const int n = min(n0 + tid, a.N - 1);
            const __half* __restrict__ wsc = static_cast<const __half*>(a.w_scale);
            const __half* __restrict__ bias = static_cast<const __half*>(a.bias);
            prm_sw[tid] = a.fp_only ? 0.0f : __half2float(wsc[n]) * (1.0f / 256.0f);   // exact power-of-two factor
            prm_wr[tid] = a.fp_only ? 0.0f : a.w_reduced[n];
            prm_bv[tid] = (bias && !a.fp_only) ? __half2float(bias[n]) : 0.0f;
        }
#pragma unroll
        for (int q = 0; q < PF; ++q) {
            const int kk = (wave + 4 * q) * 16 + g * 8;    // first of this lane's 8 outlier columns
            const bool live = (wave + 4 * q) < fsteps && kk < a.n_out;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int t2 = min(t0 + i * 32 + l32, a.T - 1);
                pfa[q][i] = live ? *reinterpret_cast<const uint4*>(xo + (size_t)t2 * a.ldo + kk) : make_uint4(0, 0, 0, 0);
            }
            pfb[q] = live ? *reinterpret_cast<const uint4*>(wo + (size_t)n2 * a.ldwo + kk) : make_uint4(0, 0, 0, 0);
        }
    }

    v16i acc[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;

#pragma unroll
    for (int s = 0; s < NST - 1; ++s) issue(s_begin + s);
    for (int s = s_begin; s < s_end; ++s) {
        issue(s + NST - 1);
        wait_vm<(NST - 1) * LPS>();                        // stage s has landed (this wave's own loads)
        const uint8_t* st = ring + ((s - s_begin) % NST) * ST_BYTES;
        constexpr uint32_t M = 0xF0F0F0F0u;
        const uint4 ww = *reinterpret_cast<const uint4*>(st + A_BYTES + rd);
        const v4i uw = v4i{(int)((ww.x << 4) & M), (int)(ww.x & M), (int)((ww.y << 4) & M), (int)(ww.y & M)};
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const uint4 wa = *reinterpret_cast<const uint4*>(st + i * 1024 + rd);
            const v8i ua = v8i{(int)(wa.x & M), (int)((wa.x << 4) & M), (int)(wa.y & M), (int)((wa.y << 4) & M),
                               (int)(wa.z & M), (int)((wa.z << 4) & M), (int)(wa.w & M), (int)((wa.w << 4) & M)};
            acc[i] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(uw, ua, acc[i], (int)ww.z, 0, 0);
        }
        // the buffer read here is refilled NST - 1 iterations later by this same wave: the LDS reads above
        // have returned (their data fed the matrix instructions) before that DMA is issued
    }
    wait_vm<0>();

    // ---- this wave's share of the fp16 outlier product (weights first: same accumulator layout)
    v16f cf[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) cf[i][r] = 0.0f;
    if constexpr (!RAW) {
#pragma unroll
        for (int q = 0; q < PF; ++q)
#pragma unroll
            for (int i = 0; i < TM; ++i)
                cf[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, pfb[q]), __builtin_bit_cast(v8h, pfa[q][i]),
                                                               cf[i], 0, 0, 0);
        for (int stp = wave + 4 * PF; stp < fsteps; stp += 4) {     // the outlier columns beyond the prefetched ones
            const int kk = stp * 16 + g * 8;
            const uint4 fb = (kk < a.n_out) ? *reinterpret_cast<const uint4*>(wo + (size_t)n2 * a.ldwo + kk) : make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int t2 = min(t0 + i * 32 + l32, a.T - 1);
                const uint4 fa = (kk < a.n_out) ? *reinterpret_cast<const uint4*>(xo + (size_t)t2 * a.ldo + kk) : make_uint4(0, 0, 0, 0);
                cf[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, fb), __builtin_bit_cast(v8h, fa), cf[i], 0, 0, 0);
            }
        }
    }
    __syncthreads();                                       // rings are dead: reuse LDS for the reduction

    // ---- sum the four partial results: waves 1..3 publish, wave 0 adds (INT32 exactly; the fp32 outlier
    // partials in wave order)
    int* red = reinterpret_cast<int*>(lds);
    float* redf = reinterpret_cast<float*>(lds) + 3 * TM * 16 * 64;
    if (wave > 0) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int slot = (((wave - 1) * TM + i) * 16 + r) * 64 + lane;
                red[slot] = acc[i][r];
                if constexpr (!RAW) redf[slot] = cf[i][r];
            }
    }
    __syncthreads();
    if (wave > 0) return;
    auto add_partial = [&](int w) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int slot = ((w * TM + i) * 16 + r) * 64 + lane;
                acc[i][r] += red[slot];
                if constexpr (!RAW) cf[i][r] += redf[slot];
            }
    };
    if constexpr (TM == 1) {
        // all 96 loads at once: 0.5 us faster than one partial result after the other, at 60 registers
        add_partial(0); add_partial(1); add_partial(2);
    } else {
        // one partial result after the other: hoisting all the loads would halve the occupancy
#pragma unroll 1
        for (int w = 0; w < 3; ++w) add_partial(w);
    }

    // lane: token t0 + 32 i + l32; register r: channel n0 + 8 (r / 4) + 4 g + r % 4
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int t = t0 + i * 32 + l32;
        if constexpr (RAW) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int n = n0 + 8 * (r >> 2) + 4 * g + (r & 3);
                if (t < a.T && n < a.N) a.acc[(size_t)t * a.ldacc + n] = acc[i][r] >> 8;   // exact: a multiple of 256
            }
        } else {
            __half* __restrict__ y = static_cast<__half*>(a.y);
            const float t_h = t_z[i] + 8.0f * t_s[i];      // zeroAct + halfRange * scaleAct
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int c = 8 * (r >> 2) + 4 * g + (r & 3), n = n0 + c;
                const float v = __builtin_fmaf((float)acc[i][r], t_s[i] * prm_sw[c], __builtin_fmaf(t_h, prm_wr[c], prm_bv[c])) + cf[i][r];
                if (t < a.T && n < a.N) {
                    if (a.fp_only) reinterpret_cast<float*>(a.y)[(size_t)t * a.ldy + n] = v;
                    else y[(size_t)t * a.ldy + n] = __float2half(v);
                }
            }
        }
    }
}

// Signed 4-bit weights (two per byte, column 2p in the low nibble) -> the weight format of
// quik_sp24_device.h.  One thread per (row, stage).  A group of four with more than two nonzero values
// is counted in *violations (if not null) and keeps its first two.  Offline step.
__global__ __launch_bounds__(256) void weight_pack_sp24_kernel(const uint8_t* __restrict__ w_q, int ldw, int N, int K_b,
                                                               uint32_t* __restrict__ w24, int* __restrict__ violations) {
    const int S = sp24::stages(K_b);
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)N * S) return;
    const int n = (int)(idx / S), s = (int)(idx % S);
    const uint8_t* src = w_q + (size_t)n * ldw + s * 32;
    uint64_t vals[2] = {0, 0};
    uint32_t ind[2] = {0, 0};
    int bad = 0;
    for (int kappa = 0; kappa < 16; ++kappa) {
        int v[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int col = s * 64 + kappa * 4 + p;
            int nib = 0;
            if (col < K_b) {
                const uint32_t byte = src[(kappa * 4 + p) >> 1];
                nib = (int)((p & 1) ? (byte >> 4) : (byte & 0xFu));
            }
            v[p] = nib;                                   // two's complement nibble; 0 = value 0
        }
        // kept positions: the nonzero ones (at most two count), then the lowest unused ones, ascending
        int keep[2], nk = 0, nz = 0;
#pragma unroll
        for (int p = 0; p < 4; ++p)
            if (v[p] != 0) { if (nk < 2) keep[nk++] = p; ++nz; }
        if (nz > 2) ++bad;
#pragma unroll
        for (int p = 0; p < 4; ++p)
            if (nk < 2 && v[p] == 0) keep[nk++] = p;
        if (keep[0] > keep[1]) { const int tmp = keep[0]; keep[0] = keep[1]; keep[1] = tmp; }
        const int hg = sp24::half_of_group(kappa), q = sp24::pair_of_group(kappa);
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int c = 2 * q + e;
            const int bit = 32 * (c >> 3) + 8 * (c & 3) + 4 * ((c >> 2) & 1);
            vals[hg] |= (uint64_t)(uint32_t)v[keep[e]] << bit;
            ind[hg] |= (uint32_t)keep[e] << (2 * c);
        }
    }
    uint4* blk = reinterpret_cast<uint4*>(w24) + ((size_t)s * N + n) * 2;
    blk[0] = make_uint4((uint32_t)vals[0], (uint32_t)(vals[0] >> 32), ind[0], 0u);
    blk[1] = make_uint4((uint32_t)vals[1], (uint32_t)(vals[1] >> 32), ind[1], 0u);
    if (bad && violations) atomicAdd(violations, bad);
}

template <int BM, int BN, int WM, int WN, int NST, int KS, int GM, int MODE>
hipError_t launch_cfg(const GemmArgs& a, hipStream_t stream) {
    const int tiles = ((a.T + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    hipLaunchKernelGGL((gemm_sp24_kernel<BM, BN, WM, WN, NST, KS, GM, MODE>), dim3(tiles), dim3(WM * WN * 64), 0, stream, a);
    return hipGetLastError();
}

template <int MODE>
hipError_t dispatch24(const GemmArgs& a, hipStream_t stream) {
    // Few tokens: weight streaming dominates.  The K-split kernel, one workgroup per 32 channels and 32 or 64
    // tokens (ring depth at 32 tokens: 4 and 6 measured alike, 8 to 16 up to 15 % slower).
    if (a.T <= 32) {
        hipLaunchKernelGGL((gemm_sp24_skinny<1, 4, MODE>), dim3((a.N + 31) / 32), dim3(256), 0, stream, a);
        return hipGetLastError();
    }
    if (a.T <= 64) {
        hipLaunchKernelGGL((gemm_sp24_skinny<2, 4, MODE>), dim3((a.N + 31) / 32), dim3(256), 0, stream, a);
        return hipGetLastError();
    }
    // One workgroup of eight waves per CU, so a launch runs in ceil(tiles / 256) rounds; a 256 x 192 tile
    // takes about 1.4x as long as a 256 x 128 one.  Few tiles: 128 x 128 tiles, two workgroups per CU.
    // Ring of eight stage buffers everywhere (measured: 6 and 8 run alike, odd counts and
    // deeper rings up to the LDS limit 3 - 7 % slower).
    auto rounds = [&](int bm, int bn) { return (((long)(a.T + bm - 1) / bm) * ((a.N + bn - 1) / bn) + 255) / 256; };
    const long tiles_128 = (long)((a.T + 255) / 256) * ((a.N + 127) / 128);
    // 65 .. 128 tokens: 128 x 64 tiles (twice the workgroups of 128 x 128 tiles: 15 % faster there, slower
    // from 192 tokens on)
    if (a.T <= 128) return launch_cfg<128, 64, 2, 2, 8, 2, 0, MODE>(a, stream);
    if (tiles_128 < 256) return launch_cfg<128, 128, 2, 2, 8, 2, 0, MODE>(a, stream);
    if (1.4 * (double)rounds(256, 192) <= (double)rounds(256, 128)) return launch_cfg<256, 192, 4, 2, 8, 2, 4, MODE>(a, stream);
    return launch_cfg<256, 128, 4, 2, 8, 2, 4, MODE>(a, stream);
}

}  // namespace

hipError_t launch_gemm_sp24(const GemmArgs& a, hipStream_t stream) {
    if (a.T <= 0 || a.N <= 0) return hipSuccess;
    return a.y ? dispatch24<0>(a, stream) : dispatch24<1>(a, stream);
}

hipError_t launch_weight_pack_sp24(const void* w_q, int ldw, int N, int K_b, void* w24, int* violations,
                                   hipStream_t stream) {
    if (N <= 0 || K_b <= 0) return hipSuccess;
    const long total = (long)N * sp24::stages(K_b);
    hipLaunchKernelGGL(weight_pack_sp24_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       static_cast<const uint8_t*>(w_q), ldw, N, K_b, static_cast<uint32_t*>(w24), violations);
    return hipGetLastError();
}

}  // namespace quik
