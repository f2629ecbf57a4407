// Integer GEMM + dequantization epilogue + fp16 outlier GEMM for gfx950
// (Algorithm 1 of arXiv 2310.09259: "INTmatmul", "Dequantization", "FPmatmul" and
// the final add; epilogue fusion as in Section 3.4).
//
// Data path.  gfx950 has no 4-bit integer MFMA, so packed nibbles travel
// HBM -> LDS -> VGPR still packed and are widened to int8 in registers.  A dot
// product does not care in which order k is visited as long as both operands
// agree, so the high and the low nibbles of a packed word simply become two
// different operand registers (no re-interleaving).  Two widenings are used:
//   symmetric:  (w & 0xF0F0F0F0) and ((w << 4) & 0xF0F0F0F0) hold 16x the signed
//     nibbles; done to both operands every product is exactly 256x too large
//     (3 VALU operations per two operand registers).  Used by the raw-accumulator
//     hook when it is given no correction terms.
//   asymmetric: one AND per operand register.  (w & 0xF0F0F0F0) is 16x the signed
//     high nibble; ((w ^ 0x08080808) & 0x0F0F0F0F) is the low nibble plus 8 (an
//     unsigned value 0..15).  Activations keep element 2p in the high nibble,
//     weights in the low nibble, so every product pairs a "16x" register with a
//     "+8" register of the same k: even k gives 16*a*(b+8), odd k gives (a+8)*16*b,
//     and the accumulator holds 16*sum(a*b) + 128*sum_{even k} a + 128*sum_{odd k} b.
//     The two sums are per-token / per-channel integers computed once (by the
//     quantization kernel and by the weight preparation) and subtracted, exactly,
//     in the epilogue.
// Headroom: the raw accumulator stays below 2^31 for K_b < 131072.
//
// MFMA shape: v_mfma_i32_32x32x32_i8.  First operand = activations (32 token
// rows), second = weights (32 output channels).  Lane l supplies row/column l%32
// and the k-group l/32; it receives output column l%32 and rows
// 8*(r/4) + 4*(l/32) + r%4 in accumulator register r.  The fp16 outlier product
// uses v_mfma_f32_32x32x16_f16, whose accumulator has the same layout, so the
// dequantized tile is simply the C operand of the outlier stages.
//
// Mixed widths (4-bit weights under 8-bit activations): see MIXED in gemm_kernel.
//
// Pipeline.  A workgroup of four or eight waves owns a BM x BN output tile.  Operand panels
// are copied global -> LDS without passing through registers (buffer_load ... lds,
// 16 bytes per lane, BKB bytes of every row per stage, NST stage buffers).  Rows
// beyond T / N and bytes beyond the row end are out of range for the buffer
// descriptor and arrive as zeros.  The 16-byte slots of a row are XOR-swizzled so
// that the 32 rows a ds_read_b128 touches fall into distinct banks.  The int4
// stages and the fp16 outlier stages run through the same stage ring.  Inside a
// wave the work is software pipelined three deep and the order is pinned with
// scheduling barriers: while the MFMAs of sub-step q issue, the packed words of
// sub-step q+1 are widened and the LDS reads of sub-step q+2 are in flight.
// One workgroup barrier per stage; right after it the stage buffer it has just
// freed is refilled, the DMA instructions spread between MFMAs.
//
// Epilogue.  Per-row parameters (LDS) and per-column parameters (registers) are
// fetched before the first DMA.  After the int stages the accumulators are
// dequantized in place of the C operand of the fp16 outlier stages; the fp16
// result tile is parked in the dead stage ring and leaves the CU as 16-byte
// pieces, whole row segments per store instruction.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "quik_kernels.h"
#include "quik_gemm_device.h"

namespace quik {

namespace {

using namespace gemm_dev;

// BM x BN output tile per workgroup, WM x WN waves, BKB bytes of every packed row per
// stage, NST stage buffers, GM = m-tiles per group of the tile order (0: plain column sweep).
// MODE 0: fused epilogue (asymmetric widening for 4 bits); MODE 1: write raw INT32 accumulators,
// symmetric widening; MODE 2: raw accumulators, asymmetric widening plus correction terms.
// BITS: activation bits; WBITS: weight bits (equal, or 4-bit weights under 8-bit activations).
template <int BITS, int WBITS, int BM, int BN, int WM, int WN, int BKB, int NST, int OCC, int GM, int MODE>
__global__ __launch_bounds__(WM * WN * 64, OCC) void gemm_kernel(GemmArgs a) {
    constexpr bool RAW = MODE != 0;
    constexpr bool ASYM = (BITS == 4) && (MODE != 1);
    // Every form runs two waves per SIMD (WM * WN * OCC = 8 waves per CU, and the stage buffers leave no room
    // for more workgroups), so each claims the full 256 registers of its share: the top of the allocation is
    // then never a live register (the row-quantization kernel misread such a register on MI355X when its
    // allocation left part of the SIMD's file free).
    static_assert(WM * WN * OCC == 8, "two waves per SIMD");
    asm volatile("" ::: "v255");
    // Mixed layers: a stage still covers BKB activation bytes = BKB k, which is only BKB/2 packed
    // weight bytes.  The weight nibbles are widened to 16x int8 (even / odd k of a word in two
    // registers); the int8 activations are brought into the same k order with two byte permutes
    // per 8 elements.  Accumulators are exactly 16x the integer dot product.
    constexpr bool MIXED = (BITS == 8 && WBITS == 4);
    static_assert(WBITS == BITS || MIXED, "weights: same width as the activations, or 4 under 8");
    constexpr int NWAVES = WM * WN, NT = NWAVES * 64;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int CPR = BKB / 16, RPI = 64 / CPR;
    constexpr int A_INSTR = BM / RPI / NWAVES, B_INSTR = BN / RPI / NWAVES;
    static_assert(A_INSTR >= 1 && B_INSTR >= 1, "tile too small for the wave count");
    constexpr int LPS = A_INSTR + B_INSTR;
    constexpr int KSUB = BKB / 32;
    constexpr int SHIFT = (BITS == 4) ? (ASYM ? 4 : 8) : (MIXED ? 4 : 0);
    constexpr int A_BYTES = BM * BKB, B_BYTES = BN * BKB, ST_BYTES = A_BYTES + B_BYTES;
    // mixed int stages: weight rows of BKW bytes, RPW rows per DMA instruction, WI instructions
    // per wave; the remaining B_INSTR - WI slots of a stage are issued as empty (out-of-range)
    // loads so that every stage counts the same number of DMA instructions
    constexpr int BKW = BKB / 2, CPW = BKW / 16, RPW = 64 / CPW;
    constexpr int WI = MIXED ? BN / RPW / NWAVES : B_INSTR;
    static_assert(!MIXED || (WI >= 1 && BKB == 128), "mixed layers: tile too small for the wave count");
    constexpr int NF = TM + TN;
    constexpr int HALVES = (BITS == 4) ? 2 : 1;          // MFMAs per output tile per sub-step
    constexpr int SLOTS = TM * TN * HALVES;
    constexpr int WORDS = NF * 4;
    // LDS reads run LA sub-steps ahead of their MFMAs (3 and 4 were measured: no faster, so the cost of
    // the fragment reads is their throughput, not their latency)
    constexpr int LA = (2 < KSUB) ? 2 : KSUB - 1;
    constexpr int RD = (KSUB % LA == 0) ? LA : LA + 1;   // raw fragment sets (a divisor of KSUB: static indices)
    constexpr int BAR_KS = KSUB - LA;                    // stage barrier sits before this sub-step
    static_assert(KSUB % 2 == 0 && NST >= 2 && LA >= 1 && KSUB % RD == 0, "raw set index must be static");

    __shared__ __align__(1024) uint8_t lds[NST * ST_BYTES];
    __shared__ __align__(16) float lds_sa[BM];
    __shared__ __align__(16) float lds_sh[BM];
    __shared__ __align__(16) int lds_ct[BM];             // 8 * (per-token correction sum)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int wm = wave_u / WN, wn = wave_u % WN;
    const int l32 = lane & 31, g = lane >> 5;

    const int tiles_m = (a.T + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    const int id = xcd_contiguous_id(blockIdx.x, tiles_m * tiles_n);
    // Tile order inside an XCD's range: GM consecutive m-tiles form a group that is swept along n
    // (m fastest), so the group's activation panels stay in that XCD's L2 while weight panels stream.
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

    const int row_bytes = a.K_b * BITS / 8;
    const int int_bytes = (row_bytes + 15) & ~15;
    const int nk_int = a.fp_only ? 0 : (row_bytes + BKB - 1) / BKB;
    const int fp_bytes = a.n_out * 2;
    const int nk_fp = RAW ? 0 : (fp_bytes + BKB - 1) / BKB;
    const int nk = nk_int + nk_fp;
    const int lda_fp = a.ldo * 2, ldb_fp = a.ldwo * 2;

    const v4i rA = make_rsrc((const uint8_t*)a.xq + (size_t)t0 * a.ldq, (size_t)(a.T - t0) * a.ldq);
    const v4i rB = make_rsrc((const uint8_t*)a.w_q + (size_t)n0 * a.ldw, (size_t)(a.N - n0) * a.ldw);
    const v4i rAf = make_rsrc(a.n_out ? (const uint8_t*)a.x_out + (size_t)t0 * lda_fp : (const uint8_t*)a.xq,
                              a.n_out ? (size_t)(a.T - t0) * lda_fp : 0);
    const v4i rBf = make_rsrc(a.n_out ? (const uint8_t*)a.w_out + (size_t)n0 * ldb_fp : (const uint8_t*)a.xq,
                              a.n_out ? (size_t)(a.N - n0) * ldb_fp : 0);

    const int lrow = lane / CPR, lslot = lane % CPR;
    const uint32_t lds_base = lds_addr(lds);
    uint32_t voA[A_INSTR], voB[B_INSTR];
    int chA[A_INSTR], chB[B_INSTR], rwA[A_INSTR], rwB[B_INSTR];
#pragma unroll
    for (int i = 0; i < A_INSTR; ++i) {
        int row = (wave_u * A_INSTR + i) * RPI + lrow;
        int c = (lslot ^ swz<BKB>(row)) * 16;
        rwA[i] = row; chA[i] = c;
        voA[i] = (uint32_t)(row * a.ldq + c);
    }
#pragma unroll
    for (int i = 0; i < B_INSTR; ++i) {
        int row = (wave_u * B_INSTR + i) * RPI + lrow;
        int c = (lslot ^ swz<BKB>(row)) * 16;
        rwB[i] = row; chB[i] = c;
        voB[i] = (uint32_t)(row * a.ldw + c);
    }
    const uint32_t m0A = lds_base + wave_u * A_INSTR * 1024;
    const uint32_t m0B = lds_base + A_BYTES + wave_u * B_INSTR * 1024;
    // mixed int stages: geometry of the half-width weight rows
    uint32_t voW[WI];
    int chW[WI];
    if constexpr (MIXED) {
#pragma unroll
        for (int i = 0; i < WI; ++i) {
            int row = (wave_u * WI + i) * RPW + lane / CPW;
            int c = ((lane % CPW) ^ swz<BKW>(row)) * 16;
            chW[i] = c;
            voW[i] = (uint32_t)(row * a.ldw + c);
        }
    }
    const uint32_t m0W = lds_base + A_BYTES + wave_u * WI * 1024;
    // where a mixed stage's empty loads land: this wave's 1 KB of the unused half of the B region
    const uint32_t m0D = lds_base + A_BYTES + BN * BKW + wave_u * 1024;
    static_assert(!MIXED || NWAVES * 1024 <= BN * BKW, "no room for the empty loads");

    // DMA instruction d of a full (unguarded) int stage
    auto issue_one = [&](int s, int d) {
        const uint32_t sb = (uint32_t)(s % NST) * ST_BYTES;
        const uint32_t so = (uint32_t)s * BKB;
        if (d < A_INSTR) {
            dma16(rA, m0A + sb + d * 1024, voA[d < A_INSTR ? d : 0], so);
        } else if constexpr (MIXED) {
            const int j = d - A_INSTR;
            if (j < WI) dma16(rB, m0W + sb + j * 1024, voW[j < WI ? j : 0], (uint32_t)s * BKW);
            else dma16(rB, m0D + sb, kOob, 0);
        } else {
            dma16(rB, m0B + sb + (d - A_INSTR) * 1024, voB[d >= A_INSTR ? d - A_INSTR : 0], so);
        }
    };
    // any stage: K tail of the int part, fp16 part, or past the end (all lanes out of range)
    auto issue_any = [&](int s) {
        const uint32_t sb = (uint32_t)(s % NST) * ST_BYTES;
        const bool fp = s >= nk_int;
        const int koff = (fp ? s - nk_int : s) * BKB;
        // integer stages stop at the 16-byte piece that holds a row's last packed byte: what lies beyond may
        // be anything in the weight matrix
        const int lima = s < nk ? (fp ? fp_bytes : int_bytes) : 0;
        const int limb = s < nk ? (fp ? fp_bytes : (MIXED ? (((a.K_b / 2) + 15) & ~15) : int_bytes)) : 0;
        const int lda = fp ? lda_fp : a.ldq, ldb = fp ? ldb_fp : a.ldw;
        const v4i ra_ = fp ? rAf : rA;
        const v4i rb_ = fp ? rBf : rB;
#pragma unroll
        for (int i = 0; i < A_INSTR; ++i) {
            uint32_t vo = (koff + chA[i] < lima) ? (uint32_t)(rwA[i] * lda + koff + chA[i]) : kOob;
            dma16(ra_, m0A + sb + i * 1024, vo, 0);
        }
        if (MIXED && !fp) {
            const int koffw = s * BKW;
#pragma unroll
            for (int i = 0; i < B_INSTR; ++i) {
                uint32_t vo = kOob;
                if (i < WI && koffw + chW[i < WI ? i : 0] < limb) vo = voW[i < WI ? i : 0] + (uint32_t)koffw;
                dma16(rb_, (i < WI ? m0W + i * 1024 : m0D) + sb, vo, 0);
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < B_INSTR; ++i) {
            uint32_t vo = (koff + chB[i] < limb) ? (uint32_t)(rwB[i] * ldb + koff + chB[i]) : kOob;
            dma16(rb_, m0B + sb + i * 1024, vo, 0);
        }
    };

    // ---- epilogue parameters, fetched before the first DMA so that their (in-order) return does
    // not sit behind the stage loads: per token row (to LDS below) and per output column (registers)
    constexpr int RPT = (BM + NT - 1) / NT;              // token rows per thread
    float p_s[RPT], p_z[RPT];
    int p_c[RPT];
    float c_sw[TN], c_wr[TN], c_bv[TN];
    int c_nc[TN];
    if constexpr (!RAW) {
#pragma unroll
        for (int q = 0; q < RPT; ++q) {
            const int t = t0 + tid + q * NT;
            const bool ok = (tid + q * NT < BM) && t < a.T;
            p_s[q] = ok ? a.scale[t] : 0.0f;
            p_z[q] = ok ? a.zero[t] : 0.0f;
            p_c[q] = 0;
            if constexpr (ASYM) p_c[q] = (ok && !a.fp_only) ? a.code_sum[t] : 0;
        }
        const __half* __restrict__ wsc = static_cast<const __half*>(a.w_scale);
        const __half* __restrict__ bias = static_cast<const __half*>(a.bias);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = min(n0 + wn * TN * 32 + j * 32 + l32, a.N - 1);
            c_sw[j] = __half2float(wsc[n]) * (1.0f / (float)(1 << SHIFT));   // exact power-of-two factor
            c_bv[j] = bias ? __half2float(bias[n]) : 0.0f;
            c_wr[j] = a.w_reduced[n];
            c_nc[j] = 0;
            if constexpr (ASYM) c_nc[j] = a.fp_only ? 0 : -128 * a.w_code_sum[n];
            if (a.fp_only) { c_sw[j] = 0.0f; c_bv[j] = 0.0f; c_wr[j] = 0.0f; }
        }
    }

    // ---- prologue: fill every stage buffer
#pragma unroll
    for (int s = 0; s < NST; ++s) issue_any(s);

    if constexpr (!RAW) {
#pragma unroll
        for (int q = 0; q < RPT; ++q) {
            const int r = tid + q * NT;
            if (r < BM) {
                lds_sa[r] = p_s[q];                                          // scaleAct
                lds_sh[r] = p_z[q] + (float)(1 << (BITS - 1)) * p_s[q];      // zeroAct + halfRange * scaleAct
                if constexpr (ASYM) lds_ct[r] = -128 * p_c[q];               // in raw accumulator units
            }
        }
    }

    uint32_t rd[NF][KSUB];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        int r = (f < TM) ? (wm * TM * 32 + f * 32 + l32) : (wn * TN * 32 + (f - TM) * 32 + l32);
        uint32_t base = (f < TM ? 0 : A_BYTES) + r * BKB;
#pragma unroll
        for (int ks = 0; ks < KSUB; ++ks) rd[f][ks] = base + (((ks * 2 + g) ^ swz<BKB>(r)) << 4);
    }

    uint4 R[RD][NF];
    v4i U[2][NF][HALVES];

    // mixed int stages: 8 bytes (16 nibbles = this lane's k-group) of a half-width weight row
    uint32_t rdw[MIXED ? TN : 1][KSUB];
    if constexpr (MIXED) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int r = wn * TN * 32 + j * 32 + l32;
#pragma unroll
            for (int ks = 0; ks < KSUB; ++ks) rdw[j][ks] = A_BYTES + r * BKW + ((ks ^ swz<BKW>(r)) << 4) + g * 8;
        }
    }
    auto read_frag = [&](int set, int f, const uint8_t* stage, int ks) {
        R[set][f] = *reinterpret_cast<const uint4*>(stage + rd[f][ks]);
    };
    // fragment f of sub-step ks of a stage that is an int stage (wide == false) or an fp16 stage
    auto read_any = [&](int set, int f, const uint8_t* stage, int ks, bool wide) {
        if constexpr (MIXED) {
            if (f >= TM && !wide) {
                const uint2 v = *reinterpret_cast<const uint2*>(stage + rdw[f >= TM ? f - TM : 0][ks]);
                R[set][f].x = v.x;
                R[set][f].y = v.y;
                return;
            }
        }
        read_frag(set, f, stage, ks);
    };
    auto widen_word = [&](int set, int rset, int w) {
        const int f = w >> 2, k = w & 3;
        const uint32_t x = (k == 0) ? R[rset][f].x : (k == 1) ? R[rset][f].y : (k == 2) ? R[rset][f].z : R[rset][f].w;
        if constexpr (BITS == 4) {
            // slot 0 of a word pair holds the even k of the word, slot 1 the odd k
            constexpr uint32_t M = 0xF0F0F0F0u;
            const bool act = f < TM;                     // activations: even k in the high nibble
            uint32_t hi, lo;
            if constexpr (ASYM) {
                hi = x & M;                              // 16 * signed high nibble
                lo = (x ^ 0x08080808u) & 0x0F0F0F0Fu;    // low nibble + 8
            } else {
                hi = x & M;
                lo = (x << 4) & M;                       // 16 * signed, both
            }
            U[set][f][k >> 1][(k & 1) * 2] = (int)(act ? hi : lo);
            U[set][f][k >> 1][(k & 1) * 2 + 1] = (int)(act ? lo : hi);
        } else if constexpr (MIXED) {
            if (f < TM) {
                // int8 activations k0..k15 -> [even k of the low 8 | odd | even of the high 8 | odd]
                const uint32_t lo = (k < 2) ? R[rset][f].x : R[rset][f].z, hi = (k < 2) ? R[rset][f].y : R[rset][f].w;
                U[set][f][0][k] = (int)__builtin_amdgcn_perm(hi, lo, (k & 1) ? 0x07050301u : 0x06040200u);
            } else {
                // packed weights: word k/2 holds 8 nibbles; even k (low nibbles) / odd k (high), 16x
                constexpr uint32_t M = 0xF0F0F0F0u;
                const uint32_t wv = (k < 2) ? R[rset][f].x : R[rset][f].y;
                U[set][f][0][k] = (int)((k & 1) ? (wv & M) : ((wv << 4) & M));
            }
        } else {
            U[set][f][0][k] = (int)x;
        }
    };

    // With the single-AND widening and the fused epilogue the accumulators start at
    // -128 * (code_sum[t] + w_code_sum[n]) instead of zero, so that the K loop ends on 16 x the integer dot
    // product (the widening leaves it plus 128 times these sums; two's complement, nothing overflows on the way).
    v16i acc[TM][TN];
    if constexpr (ASYM && !RAW) {
        __syncthreads();                                  // lds_ct is complete (the first stages are in flight)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int4 ct4 = *reinterpret_cast<const int4*>(&lds_ct[wm * TM * 32 + i * 32 + 8 * rq + 4 * g]);
                const int ct_[4] = {ct4.x, ct4.y, ct4.z, ct4.w};
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) acc[i][j][rq * 4 + rr] = ct_[rr] + c_nc[j];
            }
    } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
    }

    // stage barrier of iteration s: stage s+1 has landed for everybody, and nobody reads stage s any more
    auto stage_barrier = [&]() {
        wait_vm<(NST - 2) * LPS>();
        __syncthreads();
    };

    // sub-step ks of stage s.  PLAIN: the DMA into the freed buffer is a full int stage and is spread over
    // the MFMA slots that follow the barrier; otherwise it is issued in one go.
    auto substep = [&](int s, int ks, bool plain) {
        const int par = ks & 1;
        if (ks == BAR_KS) {
            stage_barrier();
            if (!plain) issue_any(s + NST);
        }
        const int ts = (ks + LA < KSUB) ? s : s + 1, tks = (ks + LA) % KSUB;
        const uint8_t* tgt = lds + (ts % NST) * ST_BYTES;
        const int rnext = (ks + 1) % RD, rload = (ks + LA) % RD;   // static: KSUB is a multiple of RD
        const bool wide = ts >= nk_int;                             // the look-ahead reaches the fp16 part
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < SLOTS; ++m) {
            const int h = m / (TM * TN), ij = m % (TM * TN), i = ij / TN, j = ij % TN;
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(U[par][i][h], U[par][TM + j][h], acc[i][j], 0, 0, 0);
            if (plain && ks == BAR_KS) {
                constexpr int PER = (SLOTS >= LPS) ? SLOTS / LPS : 1;
                if (m % PER == 0 && m / PER < LPS) issue_one(s + NST, m / PER);
                if (SLOTS < LPS && m == SLOTS - 1)
                    for (int d = SLOTS; d < LPS; ++d) issue_one(s + NST, d);
            }
#pragma unroll
            for (int w = 0; w < WORDS; ++w)
                if (w * SLOTS / WORDS == m) widen_word(par ^ 1, rnext, w);
            if (m < NF) read_any(rload, m, tgt, tks, wide);
            if (SLOTS < NF && m == SLOTS - 1)
                for (int f = SLOTS; f < NF; ++f) read_any(rload, f, tgt, tks, wide);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    wait_vm<(NST - 1) * LPS>();          // stage 0 landed
    __syncthreads();
#pragma unroll
    for (int q = 0; q < LA; ++q)
#pragma unroll
        for (int f = 0; f < NF; ++f) read_any(q, f, lds, q, nk_int == 0);
#pragma unroll
    for (int w = 0; w < WORDS; ++w) widen_word(0, 0, w);

    int s = 0;
    for (; s + NST < nk_int - 1; ++s) {
#pragma unroll
        for (int ks = 0; ks < KSUB; ++ks) substep(s, ks, true);
    }
    for (; s < nk_int; ++s) {
#pragma unroll
        for (int ks = 0; ks < KSUB; ++ks) substep(s, ks, false);
    }
    // here: R[0 .. LA-1] hold raw sub-steps 0 .. LA-1 of stage nk_int (fp16 data)

    const int tw = t0 + wm * TM * 32, nw = n0 + wn * TN * 32;
    if constexpr (RAW) {
        wait_vm<0>();                      // drain the look-ahead DMA before the wave ends
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int n = nw + j * 32 + l32;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int t = tw + i * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (t < a.T && n < a.N) {
                        int v = acc[i][j][r] >> SHIFT;
                        if constexpr (ASYM) v -= 8 * (a.code_sum[t] + a.w_code_sum[n]);
                        a.acc[(size_t)t * a.ldacc + n] = v;
                    }
                }
            }
        return;
    }
    // Dequantization.  The accumulator is 2^SHIFT times the integer dot product, its conversion to binary32
    // is exact (at most 24 significant bits), and 2^-SHIFT rides on the weight scale.
    v16f cf[TM][TN];
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
                    cf[i][j][r] = __builtin_fmaf((float)acc[i][j][r], sa_[rr] * c_sw[j],
                                                 __builtin_fmaf(sh_[rr], c_wr[j], c_bv[j]));
                }
        }

    for (; s < nk; ++s) {
#pragma unroll
        for (int ks = 0; ks < KSUB; ++ks) {
            if (ks == BAR_KS) { stage_barrier(); issue_any(s + NST); }
            const int ts = (ks + LA < KSUB) ? s : s + 1, tks = (ks + LA) % KSUB;
            const uint8_t* tgt = lds + (ts % NST) * ST_BYTES;
            v8h fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = __builtin_bit_cast(v8h, R[ks % RD][i]);
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[j] = __builtin_bit_cast(v8h, R[ks % RD][TM + j]);
#pragma unroll
            for (int f = 0; f < NF; ++f) read_frag((ks + LA) % RD, f, tgt, tks);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    cf[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[i], fb[j], cf[i][j], 0, 0, 0);
        }
    }

    wait_vm<0>();                          // drain the look-ahead DMA before the wave ends
    __half* __restrict__ y = static_cast<__half*>(a.y);
    // Output through LDS: a lane owns one column of sixteen rows of every 32 x 32 block, so direct
    // stores would be 2 bytes per lane.  Each wave instead parks its fp16 tile in its own slice of
    // the (now dead) stage ring and writes it out as 16-byte pieces, whole 64/128-byte row
    // segments per instruction.  Needs 16-byte aligned output rows; otherwise the direct path below.
    // bytes per parked row: padded against bank conflicts where the ring has the room
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
                    *reinterpret_cast<__half*>(wbuf + row * WROW + (j * 32 + l32) * 2) = __float2half(cf[i][j][r]);
                }
        constexpr int CH = TN * 4;                       // 16-byte pieces per row
        constexpr int RPS = 64 / CH;                     // rows per store instruction (lanes >= RPS * CH idle)
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
            int n = nw + j * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int t = tw + i * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                if (t < a.T && n < a.N) {
                    if (a.fp_only) reinterpret_cast<float*>(a.y)[(size_t)t * a.ldy + n] = cf[i][j][r];
                    else y[(size_t)t * a.ldy + n] = __float2half(cf[i][j][r]);
                }
            }
        }
}

// Small-T variant (T <= 32*TM): the layer is bound by streaming the packed weights, not by the
// matrix cores, so the point is many bytes in flight per CU.  A workgroup owns a (32*TM) x (32*TN)
// output tile and its four waves split K: every wave streams its own quarter of the weight rows
// (and of the activations) through a private global->LDS ring, with no workgroup barrier in the main
// loop (a wave waits only for its own DMA).  The four partial INT32 accumulators are summed exactly
// through LDS; wave 0 then dequantizes, adds the fp16 outlier product (operands read straight from
// global memory: they are tiny) and stores.
template <int BITS, int TM, int TN, int BKB, int NST, int MODE>
__global__ __launch_bounds__(256) void gemm_skinny(GemmArgs a) {
    constexpr bool RAW = MODE != 0;
    constexpr bool ASYM = (BITS == 4) && (MODE != 1);
    constexpr int CPR = BKB / 16, RPI = 64 / CPR;        // 16-byte pieces per stage row, rows per DMA instr
    constexpr int BM = 32 * TM, BN = 32 * TN;
    constexpr int A_INSTR = BM / RPI, B_INSTR = BN / RPI; // per wave (each wave loads its own tiles)
    constexpr int LPS = A_INSTR + B_INSTR;
    constexpr int KSUB = BKB / 32;
    constexpr int SHIFT = (BITS == 4) ? (ASYM ? 4 : 8) : 0;
    constexpr int A_BYTES = BM * BKB, B_BYTES = BN * BKB, ST_BYTES = A_BYTES + B_BYTES;
    constexpr int NF = TM + TN;
    constexpr int HALVES = (BITS == 4) ? 2 : 1;
    constexpr int RING = NST * ST_BYTES;                  // per wave
    constexpr int RED_BYTES = 2 * TM * TN * 16 * 64 * 4;  // one wave's INT32 accumulators + fp32 outlier partials
    constexpr int LDS_BYTES = (4 * RING > 3 * RED_BYTES) ? 4 * RING : 3 * RED_BYTES;
    static_assert((NST - 1) * LPS < 64, "vmcnt range");

    __shared__ __align__(1024) uint8_t lds[LDS_BYTES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5;

    const int tiles_m = (a.T + BM - 1) / BM;
    const int t0 = (blockIdx.x % tiles_m) * BM, n0 = (blockIdx.x / tiles_m) * BN;

    const int row_bytes = a.K_b * BITS / 8;
    const int int_bytes = (row_bytes + 15) & ~15;      // up to the 16-byte piece that holds the last packed byte
    const int nk = a.fp_only ? 0 : (row_bytes + BKB - 1) / BKB;
    // this wave's K range, in stages
    const int s_begin = (int)((long)nk * wave / 4), s_end = (int)((long)nk * (wave + 1) / 4);

    const v4i rA = make_rsrc((const uint8_t*)a.xq + (size_t)t0 * a.ldq, (size_t)(a.T - t0) * a.ldq);
    const v4i rB = make_rsrc((const uint8_t*)a.w_q + (size_t)n0 * a.ldw, (size_t)(a.N - n0) * a.ldw);

    uint8_t* ring = lds + wave * RING;
    const uint32_t ring_addr = lds_addr(ring);
    const int lrow = lane / CPR, lslot = lane % CPR;

    auto issue = [&](int s) {            // stage s of this wave's range (or beyond: all lanes out of range)
        const uint32_t sb = (uint32_t)((s - s_begin) % NST) * ST_BYTES;
        const int koff = s * BKB;
        const bool live = s < s_end;
#pragma unroll
        for (int i = 0; i < A_INSTR; ++i) {
            int row = i * RPI + lrow;
            int c = (lslot ^ swz<BKB>(row)) * 16;
            uint32_t vo = (live && koff + c < int_bytes) ? (uint32_t)(row * a.ldq + koff + c) : kOob;
            dma16(rA, ring_addr + sb + i * 1024, vo, 0);
        }
#pragma unroll
        for (int i = 0; i < B_INSTR; ++i) {
            int row = i * RPI + lrow;
            int c = (lslot ^ swz<BKB>(row)) * 16;
            uint32_t vo = (live && koff + c < int_bytes) ? (uint32_t)(row * a.ldw + koff + c) : kOob;
            dma16(rB, ring_addr + sb + A_BYTES + i * 1024, vo, 0);
        }
    };

    uint32_t rd[NF][KSUB];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        int r = (f < TM) ? (f * 32 + l32) : ((f - TM) * 32 + l32);
        uint32_t base = (f < TM ? 0 : A_BYTES) + r * BKB;
#pragma unroll
        for (int ks = 0; ks < KSUB; ++ks) rd[f][ks] = base + (((ks * 2 + g) ^ swz<BKB>(r)) << 4);
    }

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // ---- everything the epilogue needs is requested before the weight stream starts, so none of it
    // is waited for at the end: per-row parameters (to LDS), per-column parameters and this wave's
    // share of the fp16 outlier operands (registers).  The outlier product is split over the four
    // waves like K: wave w takes every fourth 16-column step.
    constexpr int PF = 4;                                 // prefetched outlier steps per wave (n_out <= 256)
    __shared__ float prm_sa[BM], prm_sh[BM];
    __shared__ int prm_ct[BM];
    float c_sw[TN], c_wr[TN], c_bv[TN];
    int c_nc[TN];
    uint4 pfa[PF][TM], pfb[PF][TN];
    const int fsteps = (a.n_out + 15) >> 4;               // 16-column steps of the outlier product
    if constexpr (!RAW) {
        if (tid < BM) {
            const int t = t0 + tid;
            const bool ok = t < a.T;
            const float sc = ok ? a.scale[t] : 0.0f;
            prm_sa[tid] = sc;
            prm_sh[tid] = (ok ? a.zero[t] : 0.0f) + (float)(1 << (BITS - 1)) * sc;
            int cs = 0;
            if constexpr (ASYM) cs = (ok && !a.fp_only) ? a.code_sum[t] : 0;
            prm_ct[tid] = -(1 << SHIFT) * 8 * cs;
        }
        const __half* __restrict__ wsc = static_cast<const __half*>(a.w_scale);
        const __half* __restrict__ bias = static_cast<const __half*>(a.bias);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = min(n0 + j * 32 + l32, a.N - 1);
            c_sw[j] = __half2float(wsc[n]) * (1.0f / (float)(1 << SHIFT));
            c_wr[j] = a.w_reduced[n];
            c_bv[j] = bias ? __half2float(bias[n]) : 0.0f;
            c_nc[j] = 0;
            if constexpr (ASYM) c_nc[j] = a.fp_only ? 0 : -(1 << SHIFT) * 8 * a.w_code_sum[n];
            if (a.fp_only) { c_sw[j] = 0.0f; c_wr[j] = 0.0f; c_bv[j] = 0.0f; }
        }
        const __half* __restrict__ xo = static_cast<const __half*>(a.x_out);
        const __half* __restrict__ wo = static_cast<const __half*>(a.w_out);
#pragma unroll
        for (int q = 0; q < PF; ++q) {
            const int kk = (wave + 4 * q) * 16 + g * 8;   // first of this lane's 8 outlier columns
            const bool live = (wave + 4 * q) < fsteps && kk < a.n_out;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int t = min(t0 + i * 32 + l32, a.T - 1);
                pfa[q][i] = live ? *reinterpret_cast<const uint4*>(xo + (size_t)t * a.ldo + kk) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = min(n0 + j * 32 + l32, a.N - 1);
                pfb[q][j] = live ? *reinterpret_cast<const uint4*>(wo + (size_t)n * a.ldwo + kk) : make_uint4(0, 0, 0, 0);
            }
        }
    }

#pragma unroll
    for (int s = 0; s < NST - 1; ++s) issue(s_begin + s);

    for (int s = s_begin; s < s_end; ++s) {
        issue(s + NST - 1);
        wait_vm<(NST - 1) * LPS>();                       // stage s has landed (this wave's own loads)
        const uint8_t* st = ring + ((s - s_begin) % NST) * ST_BYTES;
#pragma unroll
        for (int ks = 0; ks < KSUB; ++ks) {
            v4i ua[TM][HALVES], ub[TN][HALVES];
#pragma unroll
            for (int f = 0; f < NF; ++f) {
                const uint4 w = *reinterpret_cast<const uint4*>(st + rd[f][ks]);
                v4i* u = (f < TM) ? ua[f] : ub[f - TM];
                if constexpr (BITS == 4) {
                    // register slots 0/2 hold the even k of a word, slots 1/3 the odd k
                    constexpr uint32_t M = 0xF0F0F0F0u;
                    auto hi = [](uint32_t x) { return (int)(x & M); };
                    auto lo = [](uint32_t x) {
                        return ASYM ? (int)((x ^ 0x08080808u) & 0x0F0F0F0Fu) : (int)((x << 4) & M);
                    };
                    if (f < TM) {                         // activations: even k in the high nibble
                        u[0] = v4i{hi(w.x), lo(w.x), hi(w.y), lo(w.y)};
                        u[1] = v4i{hi(w.z), lo(w.z), hi(w.w), lo(w.w)};
                    } else {                              // weights: even k in the low nibble
                        u[0] = v4i{lo(w.x), hi(w.x), lo(w.y), hi(w.y)};
                        u[1] = v4i{lo(w.z), hi(w.z), lo(w.w), hi(w.w)};
                    }
                } else {
                    u[0] = v4i{(int)w.x, (int)w.y, (int)w.z, (int)w.w};
                }
            }
#pragma unroll
            for (int h = 0; h < HALVES; ++h)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ua[i][h], ub[j][h], acc[i][j], 0, 0, 0);
        }
        // the buffer read here is refilled NST-1 iterations later by this same wave: LDS reads above
        // have returned (their data fed the MFMAs) before that DMA is issued
    }
    wait_vm<0>();

    // ---- this wave's share of the fp16 outlier product, on fresh fp32 accumulators
    v16f cf[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) cf[i][j][r] = 0.0f;
    if constexpr (!RAW) {
#pragma unroll
        for (int q = 0; q < PF; ++q)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    cf[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, pfa[q][i]),
                                                                     __builtin_bit_cast(v8h, pfb[q][j]), cf[i][j], 0, 0, 0);
        // more than 16 * 4 * PF outlier columns: the rest straight from memory
        const __half* __restrict__ xo = static_cast<const __half*>(a.x_out);
        const __half* __restrict__ wo = static_cast<const __half*>(a.w_out);
        for (int st = wave + 4 * PF; st < fsteps; st += 4) {
            const int kk = st * 16 + g * 8;
            v8h fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int t = min(t0 + i * 32 + l32, a.T - 1);
                const uint4 w = (kk < a.n_out) ? *reinterpret_cast<const uint4*>(xo + (size_t)t * a.ldo + kk) : make_uint4(0, 0, 0, 0);
                fa[i] = __builtin_bit_cast(v8h, w);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = min(n0 + j * 32 + l32, a.N - 1);
                const uint4 w = (kk < a.n_out) ? *reinterpret_cast<const uint4*>(wo + (size_t)n * a.ldwo + kk) : make_uint4(0, 0, 0, 0);
                fb[j] = __builtin_bit_cast(v8h, w);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    cf[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[i], fb[j], cf[i][j], 0, 0, 0);
        }
    }
    __syncthreads();                                      // rings are dead: reuse LDS for the reduction

    // ---- sum the four partial results: waves 1..3 publish, wave 0 adds (INT32 exactly; the fp32
    // outlier partials in wave order)
    int* red = reinterpret_cast<int*>(lds);
    float* redf = reinterpret_cast<float*>(lds) + 3 * TM * TN * 16 * 64;
    if (wave > 0) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int slot = (((wave - 1) * TM * TN + i * TN + j) * 16 + r) * 64 + lane;
                    red[slot] = acc[i][j][r];
                    if constexpr (!RAW) redf[slot] = cf[i][j][r];
                }
    }
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int w = 0; w < 3; ++w)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int slot = ((w * TM * TN + i * TN + j) * 16 + r) * 64 + lane;
                    acc[i][j][r] += red[slot];
                    if constexpr (!RAW) cf[i][j][r] += redf[slot];
                }

    if constexpr (RAW) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int n = n0 + j * 32 + l32;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int t = t0 + i * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (t < a.T && n < a.N) {
                        int v = acc[i][j][r] >> SHIFT;
                        if constexpr (ASYM) v -= 8 * (a.code_sum[t] + a.w_code_sum[n]);
                        a.acc[(size_t)t * a.ldacc + n] = v;
                    }
                }
            }
        return;
    } else {
        // ---- epilogue on wave 0: dequantize (as in gemm_kernel), add the outlier product, store
        __half* __restrict__ y = static_cast<__half*>(a.y);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = n0 + j * 32 + l32;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int lr = i * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                    const int t = t0 + lr;
                    int ai = acc[i][j][r];
                    if constexpr (ASYM) ai = ai + prm_ct[lr] + c_nc[j];
                    const float v = __builtin_fmaf((float)ai, prm_sa[lr] * c_sw[j], __builtin_fmaf(prm_sh[lr], c_wr[j], c_bv[j])) +
                                    cf[i][j][r];
                    if (t < a.T && n < a.N) {
                        if (a.fp_only) reinterpret_cast<float*>(a.y)[(size_t)t * a.ldy + n] = v;
                        else y[(size_t)t * a.ldy + n] = __float2half(v);
                    }
                }
            }
    }
}


template <int BITS, int WBITS, int BM, int BN, int WM, int WN, int BKB, int NST, int OCC, int GM, int MODE>
hipError_t launch_cfg(const GemmArgs& a, hipStream_t stream) {
    int tiles = ((a.T + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    hipLaunchKernelGGL((gemm_kernel<BITS, WBITS, BM, BN, WM, WN, BKB, NST, OCC, GM, MODE>), dim3(tiles),
                       dim3(WM * WN * 64), 0, stream, a);
    return hipGetLastError();
}

template <int BITS, int TM, int TN, int BKB, int NST, int MODE>
hipError_t launch_skinny(const GemmArgs& a, hipStream_t stream) {
    int tiles = ((a.T + 32 * TM - 1) / (32 * TM)) * ((a.N + 32 * TN - 1) / (32 * TN));
    hipLaunchKernelGGL((gemm_skinny<BITS, TM, TN, BKB, NST, MODE>), dim3(tiles), dim3(256), 0, stream, a);
    return hipGetLastError();
}

template <int BITS, int WBITS, int MODE>
hipError_t dispatch(const GemmArgs& a, hipStream_t stream) {
    // Few tokens: weight streaming dominates.  Up to 32 tokens the K-split kernel (same operand
    // widths only); up to 128 tokens small tiles with a deeper stage ring so that enough workgroups
    // and bytes are in flight.
    if constexpr (BITS == WBITS) {
        if (a.T <= 32) return launch_skinny<BITS, 1, 1, 128, 2, MODE>(a, stream);
    }
    if (a.T <= 64) return launch_cfg<BITS, WBITS, 64, 64, 2, 2, 128, 4, 2, 0, MODE>(a, stream);
    if (a.T <= 128) return launch_cfg<BITS, WBITS, 128, 64, 2, 2, 128, 2, 2, 0, MODE>(a, stream);
    // 128-byte stage rows (a full cache line per row per stage), two stage buffers.
    // Large problems: 256 x 128 tiles shared by eight waves (one workgroup per CU) move 25 % fewer
    // operand bytes per MFMA through L1/LDS than two independent 128 x 128 workgroups.  They need
    // at least one tile per CU to pay off; otherwise 128 x 128 tiles with two workgroups per CU.
    const long big_tiles = (long)((a.T + 255) / 256) * ((a.N + 127) / 128);
    if (big_tiles < 256) return launch_cfg<BITS, WBITS, 128, 128, 2, 2, 128, 2, 2, 8, MODE>(a, stream);
    if constexpr (BITS == WBITS) {   // every MODE: the accumulator hook runs the tiles of the fused call
        // One workgroup per CU, so a launch runs in ceil(tiles / 256) rounds.  Tiles of 1.5x the area
        // (64 x 96 or 96 x 64 per wave: 17 % fewer LDS fragment reads and widening operations per
        // MFMA, a third fewer per-tile prologues and epilogues) take 1.42x as long per round
        // (measured); they win whenever they save enough rounds.
        auto rounds = [&](int bm, int bn) { return (((long)(a.T + bm - 1) / bm) * ((a.N + bn - 1) / bn) + 255) / 256; };
        const double cost_a = (double)rounds(256, 128);
        const double cost_b = 1.42 * (double)rounds(256, 192);
        const double cost_c = 1.42 * (double)rounds(192, 256);
        if (cost_b < cost_a && cost_b <= cost_c) return launch_cfg<BITS, WBITS, 256, 192, 4, 2, 128, 2, 1, 4, MODE>(a, stream);
        if (cost_c < cost_a) return launch_cfg<BITS, WBITS, 192, 256, 2, 4, 128, 2, 1, 4, MODE>(a, stream);
    }
    // Equal widths run this tile on the 16 x 16 matrix instructions (quik_gemm_tiles16.hip), under which the
    // chip keeps its clock: 2 - 6 % faster here with 4-bit operands, where two waves share every SIMD, 10 %
    // with 8-bit ones (full bytes cost the 32 x 32 form most clock).  The smaller tiles
    // above mostly run one wave per SIMD, which the 16 x 16 form's doubled instruction count slows down
    // (128 tokens of the 13B QKV shape: +7 %), and the larger ones do not fit the register file in that form.
    if constexpr (BITS == WBITS) return launch_gemm_tiles16(a, stream);
    else return launch_cfg<BITS, WBITS, 256, 128, 4, 2, 128, 2, 1, 4, MODE>(a, stream);
}

// one wave per output channel; lanes stride over the packed row
template <int BITS>
__global__ __launch_bounds__(kThreads) void weight_reduce_kernel(WeightReduceArgs a) {
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (n >= a.N) return;
    const uint8_t* row = static_cast<const uint8_t*>(a.w_q) + (size_t)n * a.ldw;
    const int row_bytes = a.K_b * BITS / 8;
    int s = 0, s_odd = 0;                  // all codes; codes at odd positions (high nibbles)
    for (int p = lane; p < row_bytes; p += 64) {
        int b = row[p];
        if constexpr (BITS == 4) {
            int hi = ((b >> 4) ^ 8) - 8;
            s += ((b & 0xF) ^ 8) - 8 + hi;
            s_odd += hi;
        } else {
            s += (int)(int8_t)b;
        }
    }
    if constexpr (BITS == 4) {
        // The GEMM reads a row up to the end of the 16-byte piece that holds its last packed byte.  Against
        // the zero bytes the activations have there, the single-AND widening turns whatever the weight
        // matrix holds in those pad bytes into 128 x (their high nibbles); counting them in the side data
        // makes the epilogue's correction remove exactly that, so pad bytes may hold anything.
        const int padded = min((row_bytes + 15) & ~15, a.ldw);
        for (int p = row_bytes + lane; p < padded; p += 64) s_odd += (((int)row[p] >> 4) ^ 8) - 8;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        s += __shfl_xor(s, o, 64);
        s_odd += __shfl_xor(s_odd, o, 64);
    }
    if (lane == 0) {
        a.w_reduced[n] = __half2float(static_cast<const __half*>(a.w_scale)[n]) * (float)s;
        if (a.w_code_sum) a.w_code_sum[n] = s_odd;
    }
}

}  // namespace

// compute units of the current device (looked up once per device)
static int compute_units() {
    static int cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cached[dev] = n;
    }
    return cached[dev];
}

// Estimated time of the per-tile kernels' launch for a 4-bit [T, N] output on `cus` compute units, in the
// unit of plan_gemm_stream's estimate (one 32-channel block of a 256-row tile through the K loop): the
// rounds and relative round times of dispatch() below.
static double tiles_estimate(int T, int N, int cus) {
    auto rounds = [&](int bm, int bn) { return (double)((((long)(T + bm - 1) / bm) * ((N + bn - 1) / bn) + cus - 1) / cus); };
    const double a = 4.0 * rounds(256, 128), b = 4.0 * 1.42 * rounds(256, 192), c = 4.0 * 1.42 * rounds(192, 256);
    return a < b ? (a < c ? a : c) : (b < c ? b : c);
}

static int g_gemm_path = 0;     // 0: automatic; 1: the persistent kernel wherever it can run; 2: never
void set_gemm_path(int mode) { g_gemm_path = mode; }

// 0: the persistent kernel cannot run this shape; 1: it can and is the automatic choice; 2: it can, but
// the per-tile kernels are estimated to be at least as fast.  Measured on the LLaMA shapes, in the unit of
// tiles_estimate: a block of the persistent kernel costs 0.91 - 0.95 where its tiles are five or six blocks
// wide (its K loop runs on the 16 x 16 x 64 matrix instruction, under which the chip keeps its clock; whole
// rounds of fixed 256 x 192 tiles cost 0.947 per block, so it also wins 4 % where those balance perfectly),
// and 1.04 where the tiles are four blocks wide (a wave then holds two column blocks: more fragment reads
// and widening per MFMA than the per-tile 256 x 128 form) or K is shallow (its longer per-tile epilogue).
int choose_gemm_stream(int T, int N, int K_b, int cus, StreamPlan* plan) {
    if (!plan_gemm_stream(T, N, K_b, cus, plan)) return 0;
    const long tiles = (long)plan->tiles_m * plan->tn;
    const long r = (tiles + cus - 1) / cus;
    const double blocks = (double)(r * plan->base + (r * plan->rem + plan->tn - 1) / plan->tn);
    return (K_b >= 2048 && plan->base >= 5 && 0.94 * blocks <= tiles_estimate(T, N, cus)) ? 1 : 2;
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t stream) {
    if (a.bits == 4 && !a.fp_only && g_gemm_path != 2) {
        StreamPlan plan;
        const int c = choose_gemm_stream(a.T, a.N, a.K_b, compute_units(), &plan);
        if (c == 1 || (c == 2 && g_gemm_path == 1)) return launch_gemm_stream(a, plan, stream);
    }
    return launch_gemm_tiles(a, stream);
}

// one workgroup per output tile (every shape the persistent kernel does not take)
hipError_t launch_gemm_tiles(const GemmArgs& a, hipStream_t stream) {
    const bool raw = a.y == nullptr;
    if (a.bits == 4) {
        if (!raw) return dispatch<4, 4, 0>(a, stream);
        return (a.code_sum && a.w_code_sum) ? dispatch<4, 4, 2>(a, stream) : dispatch<4, 4, 1>(a, stream);
    }
    if (a.w_bits == 4) return raw ? dispatch<8, 4, 1>(a, stream) : dispatch<8, 4, 0>(a, stream);
    return raw ? dispatch<8, 8, 1>(a, stream) : dispatch<8, 8, 0>(a, stream);
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
