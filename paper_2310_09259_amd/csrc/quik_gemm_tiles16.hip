// Per-tile form of the integer GEMM + dequantization epilogue + fp16 outlier GEMM on the
// 16 x 16 matrix instructions (Algorithm 1 of arXiv 2310.09259: "INTmatmul", "Dequantization",
// "FPmatmul" and the final add; epilogue fusion as in Section 3.4).
//
// Same data path, operand formats, widenings, stage ring, tile shapes and epilogue arithmetic as
// gemm_kernel in quik_gemm.hip (see the header of that file; the output is bit-identical), for equal
// operand widths (4 + 4 or 8 + 8 bits).  What differs is the matrix instruction: v_mfma_i32_16x16x64_i8
// for the integer product and v_mfma_f32_16x16x32_f16 for the outlier product.  On MI355X the chip holds
// its full clock under these, where it lowers it under the 32 x 32 forms on the same operand bytes.
//
// Layout.  Lane (l = lane % 16, g = lane / 16) supplies the 16 int8 values of k-group g for token row
// (or channel) l of a 16-row block: 8 packed bytes, bytes 8g .. 8g + 7 of the sub-step's 32 bytes of
// that row, read with ds_read_b64 and widened into the four registers of one operand.  It holds, in the
// four registers of a 16 x 16 accumulator block, channel l of token rows 4g .. 4g + 3.  An fp16 k-step
// is 32 columns (64 bytes of a row): lane (l, g) supplies columns 8g .. 8g + 7, one 16-byte piece; an
// 8-bit integer k-step is 64 bytes of a row likewise, the 16-byte piece being the operand itself.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "quik_kernels.h"
#include "quik_gemm_device.h"

namespace quik {

namespace {

using namespace gemm_dev;

typedef float v4f __attribute__((ext_vector_type(4)));

// BM x BN output tile per workgroup, WM x WN waves, BKB bytes of every packed row per stage, NST stage
// buffers, GM = m-tiles per group of the tile order (0: plain column sweep).
// MODE 0: fused epilogue (single-AND widening + correction); MODE 1: raw INT32 accumulators, symmetric
// widening; MODE 2: raw accumulators, single-AND widening + correction.
template <int BITS, int BM, int BN, int WM, int WN, int BKB, int NST, int OCC, int GM, int MODE>
__global__ __launch_bounds__(WM * WN * 64, OCC) void gemm_tiles16_kernel(GemmArgs a) {
    constexpr bool RAW = MODE != 0;
    constexpr bool ASYM = (BITS == 4) && (MODE != 1);
    // Every form claims the full share of the register file its launch bounds give it (two waves per
    // SIMD: 256 registers), so that the top of the allocation is never a live register: the
    // row-quantization kernel misread such a register on MI355X when its allocation ended below its share.
    asm volatile("" ::: "v255");
    constexpr int NWAVES = WM * WN, NT = NWAVES * 64;
    constexpr int IB = BM / WM / 16, JB = BN / WN / 16;  // 16 x 16 accumulator blocks per wave
    constexpr int CPR = BKB / 16, RPI = 64 / CPR;
    constexpr int A_INSTR = BM / RPI / NWAVES, B_INSTR = BN / RPI / NWAVES;
    static_assert(A_INSTR >= 1 && B_INSTR >= 1, "tile too small for the wave count");
    constexpr int LPS = A_INSTR + B_INSTR;
    constexpr int KSUB = BKB / 32;
    constexpr int SHIFT = (BITS == 4) ? (ASYM ? 4 : 8) : 0;
    constexpr int A_BYTES = BM * BKB, B_BYTES = BN * BKB, ST_BYTES = A_BYTES + B_BYTES;
    constexpr int NF = IB + JB;                          // fragments per sub-step
    constexpr int SLOTS = IB * JB;                       // MFMAs per sub-step
    constexpr int WORDS = NF * 2;                        // packed words per sub-step and lane
    // LDS reads run LA sub-steps ahead of their MFMAs, issued from MFMA slot RO of a sub-step on
    constexpr int LA = 2, RD = 2;
    constexpr int BAR_KS = KSUB - LA;                    // stage barrier sits before this sub-step
    constexpr int RO = 0;
    static_assert(KSUB == 4 && NST >= 2 && BKB == 128, "written for 128-byte stage rows");

    __shared__ __align__(1024) uint8_t lds[NST * ST_BYTES];
    __shared__ __align__(16) float lds_sa[BM];
    __shared__ __align__(16) float lds_sh[BM];
    __shared__ __align__(16) int lds_ct[BM];             // -128 * (per-token correction sum)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int wm = wave_u / WN, wn = wave_u % WN;
    const int l16 = lane & 15, g = lane >> 4;

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

    // DMA instruction d of a full (unguarded) int stage
    auto issue_one = [&](int s, int d) {
        const uint32_t sb = (uint32_t)(s % NST) * ST_BYTES;
        const uint32_t so = (uint32_t)s * BKB;
        if (d < A_INSTR) dma16(rA, m0A + sb + d * 1024, voA[d < A_INSTR ? d : 0], so);
        else dma16(rB, m0B + sb + (d - A_INSTR) * 1024, voB[d >= A_INSTR ? d - A_INSTR : 0], so);
    };
    // any stage: K tail of the int part, fp16 part, or past the end (all lanes out of range)
    auto issue_any = [&](int s) {
        const uint32_t sb = (uint32_t)(s % NST) * ST_BYTES;
        const bool fp = s >= nk_int;
        const int koff = (fp ? s - nk_int : s) * BKB;
        // integer stages stop at the 16-byte piece that holds a row's last packed byte: what lies beyond may
        // be anything in the weight matrix
        const int lim = s < nk ? (fp ? fp_bytes : int_bytes) : 0;
        const int lda = fp ? lda_fp : a.ldq, ldb = fp ? ldb_fp : a.ldw;
        const v4i ra_ = fp ? rAf : rA;
        const v4i rb_ = fp ? rBf : rB;
#pragma unroll
        for (int i = 0; i < A_INSTR; ++i) {
            uint32_t vo = (koff + chA[i] < lim) ? (uint32_t)(rwA[i] * lda + koff + chA[i]) : kOob;
            dma16(ra_, m0A + sb + i * 1024, vo, 0);
        }
#pragma unroll
        for (int i = 0; i < B_INSTR; ++i) {
            uint32_t vo = (koff + chB[i] < lim) ? (uint32_t)(rwB[i] * ldb + koff + chB[i]) : kOob;
            dma16(rb_, m0B + sb + i * 1024, vo, 0);
        }
    };

    // ---- epilogue parameters, fetched before the first DMA so that their (in-order) return does
    // not sit behind the stage loads: per token row (to LDS below) and per output column (registers)
    constexpr int RPT = (BM + NT - 1) / NT;              // token rows per thread
    float p_s[RPT], p_z[RPT];
    int p_c[RPT];
    float c_sw[JB], c_wr[JB], c_bv[JB];
    int c_nc[JB];
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
        for (int j = 0; j < JB; ++j) {
            const int n = min(n0 + wn * JB * 16 + j * 16 + l16, a.N - 1);
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

    // With the single-AND widening and the fused epilogue the accumulators start at
    // -128 * (code_sum[t] + w_code_sum[n]) instead of zero, so that the K loop ends on 16 x the integer dot
    // product (the widening leaves it plus 128 times these sums; two's complement, nothing overflows on the way).
    v4i acc[IB][JB];
    if constexpr (ASYM && !RAW) {
        __syncthreads();                                  // lds_ct is complete (the first stages are in flight)
#pragma unroll
        for (int i = 0; i < IB; ++i) {
            const int4 ct4 = *reinterpret_cast<const int4*>(&lds_ct[wm * IB * 16 + i * 16 + 4 * g]);
            const int ct_[4] = {ct4.x, ct4.y, ct4.z, ct4.w};
#pragma unroll
            for (int j = 0; j < JB; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[i][j][r] = ct_[r] + c_nc[j];
        }
    } else {
#pragma unroll
        for (int i = 0; i < IB; ++i)
#pragma unroll
            for (int j = 0; j < JB; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[i][j][r] = 0;
    }

    // stage barrier of iteration s: stage s+1 has landed for everybody, and nobody reads stage s any more
    auto stage_barrier = [&]() {
        wait_vm<(NST - 2) * LPS>();
        __syncthreads();
    };

    v4i U[2][NF];
    // 16-byte fragments of a 64-byte k-step (an fp16 k-step of 32 columns; an 8-bit integer k-step of 64):
    // row l of 16-row block f, k-step kk of a stage, k-group g
    uint32_t fpo[NF][2];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        int r = (f < IB) ? (wm * IB * 16 + f * 16 + l16) : (wn * JB * 16 + (f - IB) * 16 + l16);
        uint32_t base = (f < IB ? 0 : A_BYTES) + r * BKB;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) fpo[f][kk] = base + (((kk * 4 + g) ^ swz<BKB>(r)) << 4);
    }
    auto read_fp = [&](int kk, int st) {
        const uint8_t* stage = lds + (st % NST) * ST_BYTES;
#pragma unroll
        for (int f = 0; f < NF; ++f) U[kk][f] = *reinterpret_cast<const v4i*>(stage + fpo[f][kk]);
    };

    int s = 0;
    if constexpr (BITS == 4) {
        // fragment addresses inside a stage buffer: row l of 16-row block f, sub-step ks, k-group g
        uint32_t rd[NF][KSUB];
    #pragma unroll
        for (int f = 0; f < NF; ++f) {
            int r = (f < IB) ? (wm * IB * 16 + f * 16 + l16) : (wn * JB * 16 + (f - IB) * 16 + l16);
            uint32_t base = (f < IB ? 0 : A_BYTES) + r * BKB;
    #pragma unroll
            for (int ks = 0; ks < KSUB; ++ks) rd[f][ks] = base + (((ks * 2 + (g >> 1)) ^ swz<BKB>(r)) << 4) + (g & 1) * 8;
        }

        uint2 R[RD][NF];
        auto read_frag = [&](int set, int f, const uint8_t* stage, int ks) {
            R[set][f] = *reinterpret_cast<const uint2*>(stage + rd[f][ks]);
        };
        // word w (fragment w / 2, word w % 2) of raw set `rset`, widened into operand set `set`: slot 0 of a
        // word pair holds the even k of the word, slot 1 the odd k
        auto widen_word = [&](int set, int rset, int w) {
            constexpr uint32_t M = 0xF0F0F0F0u;
            const int f = w >> 1, k = w & 1;
            const bool act = f < IB;                         // activations: even k in the high nibble
            const uint32_t x = k ? R[rset][f].y : R[rset][f].x;
            const uint32_t hi = x & M;                       // 16 * signed high nibble
            const uint32_t lo = ASYM ? ((x ^ 0x08080808u) & 0x0F0F0F0Fu)   // low nibble + 8
                                     : ((x << 4) & M);                     // 16 * signed low nibble
            U[set][f][2 * k] = (int)(act ? hi : lo);
            U[set][f][2 * k + 1] = (int)(act ? lo : hi);
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
            const int rnext = (ks + 1) % RD, rload = (ks + LA) % RD;
            __builtin_amdgcn_sched_barrier(0);
    #pragma unroll
            for (int m = 0; m < SLOTS; ++m) {
                const int j = m / IB, i = m % IB;
                acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(U[par][i], U[par][IB + j], acc[i][j], 0, 0, 0);
                if (plain && ks == BAR_KS) {
                    constexpr int PER = (SLOTS >= LPS) ? SLOTS / LPS : 1;
                    if (m % PER == 0 && m / PER < LPS) issue_one(s + NST, m / PER);
                    if (SLOTS < LPS && m == SLOTS - 1)
                        for (int d = SLOTS; d < LPS; ++d) issue_one(s + NST, d);
                }
    #pragma unroll
                for (int w = 0; w < WORDS; ++w)
                    if (w * SLOTS / WORDS == m) widen_word(par ^ 1, rnext, w);
                if (m >= RO && m - RO < NF) read_frag(rload, m - RO, tgt, tks);
                if (SLOTS - RO < NF && m == SLOTS - 1)
                    for (int f = SLOTS - RO; f < NF; ++f) read_frag(rload, f, tgt, tks);
                __builtin_amdgcn_sched_barrier(0);
            }
        };

        wait_vm<(NST - 1) * LPS>();          // stage 0 landed
        __syncthreads();
    #pragma unroll
        for (int q = 0; q < LA; ++q)
    #pragma unroll
            for (int f = 0; f < NF; ++f) read_frag(q, f, lds, q);
    #pragma unroll
        for (int w = 0; w < WORDS; ++w) widen_word(0, 0, w);

        for (; s + NST < nk_int - 1; ++s) {
    #pragma unroll
            for (int ks = 0; ks < KSUB; ++ks) substep(s, ks, true);
        }
        for (; s < nk_int; ++s) {
    #pragma unroll
            for (int ks = 0; ks < KSUB; ++ks) substep(s, ks, false);
        }
    } else {
        // 8-bit operands go from LDS into the matrix instruction as they are: lane (l, g) supplies bytes
        // 16g .. 16g + 15 of a 64-byte k-step, two k-steps per stage.  The two operand sets hold the stage's
        // two k-steps; a set is refilled with the same k-step of the next stage once its MFMAs are issued.
        // The stage barrier sits after the first k-step's MFMAs: every read of this stage was issued during
        // the stage before, so its buffer is free, and the reads that follow go to the next stage.
        auto int8_mfmas = [&](int kk, int s_, bool copies) {
#pragma unroll
            for (int m = 0; m < SLOTS; ++m) {
                const int j = m / IB, i = m % IB;
                acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(U[kk][i], U[kk][IB + j], acc[i][j], 0, 0, 0);
                if (copies) {
                    constexpr int PER = (SLOTS >= LPS) ? SLOTS / LPS : 1;
                    if (m % PER == 0 && m / PER < LPS) issue_one(s_ + NST, m / PER);
                    if (SLOTS < LPS && m == SLOTS - 1)
                        for (int d = SLOTS; d < LPS; ++d) issue_one(s_ + NST, d);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        auto int8_stage = [&](int s_, bool plain) {
            int8_mfmas(0, s_, false);
            stage_barrier();
            if (!plain) issue_any(s_ + NST);
            read_fp(0, s_ + 1);
            int8_mfmas(1, s_, plain);
            read_fp(1, s_ + 1);
        };
        wait_vm<(NST - 1) * LPS>();          // stage 0 landed
        __syncthreads();
        read_fp(0, 0);
        read_fp(1, 0);
        for (; s + NST < nk_int - 1; ++s) int8_stage(s, true);
        for (; s < nk_int; ++s) int8_stage(s, false);
    }

    const int tw = t0 + wm * IB * 16, nw = n0 + wn * JB * 16;
    if constexpr (RAW) {
        wait_vm<0>();                      // drain the look-ahead DMA before the wave ends
#pragma unroll
        for (int i = 0; i < IB; ++i)
#pragma unroll
            for (int j = 0; j < JB; ++j) {
                int n = nw + j * 16 + l16;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    int t = tw + i * 16 + 4 * g + r;
                    if (t < a.T && n < a.N) {
                        int v = acc[i][j][r] >> SHIFT;
                        if constexpr (ASYM) v -= 8 * (a.code_sum[t] + a.w_code_sum[n]);
                        a.acc[(size_t)t * a.ldacc + n] = v;
                    }
                }
            }
        return;
    }
    // Dequantization.  The accumulator is 2^SHIFT times the integer dot product, its conversion to binary32 is
    // exact (at most 24 significant bits), and 2^-SHIFT rides on the weight scale.
    v4f cf[IB][JB];
#pragma unroll
    for (int i = 0; i < IB; ++i) {
        const int lr = wm * IB * 16 + i * 16 + 4 * g;
        const float4 sa4 = *reinterpret_cast<const float4*>(&lds_sa[lr]);
        const float4 sh4 = *reinterpret_cast<const float4*>(&lds_sh[lr]);
        const float sa_[4] = {sa4.x, sa4.y, sa4.z, sa4.w}, sh_[4] = {sh4.x, sh4.y, sh4.z, sh4.w};
#pragma unroll
        for (int j = 0; j < JB; ++j)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                cf[i][j][rr] = __builtin_fmaf((float)acc[i][j][rr], sa_[rr] * c_sw[j], __builtin_fmaf(sh_[rr], c_wr[j], c_bv[j]));
            }
    }

    // fp16 outlier stages on the dequantized tile: two k-steps of 32 columns per stage.  The two operand
    // sets of the integer phase (free now) hold the stage's two k-steps; a set is refilled with the same
    // k-step of the next stage once its MFMAs are issued.  The stage barrier sits after the first k-step's
    // MFMAs: every read of this stage was issued during the stage before, so its buffer is free, and the
    // reads that follow go to the next stage, which must have landed.
    auto fp_mfmas = [&](int kk) {
#pragma unroll
        for (int m = 0; m < SLOTS; ++m) {
            const int j = m / IB, i = m % IB;
            cf[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, U[kk][i]),
                                                             __builtin_bit_cast(v8h, U[kk][IB + j]), cf[i][j], 0, 0, 0);
        }
    };
    if (BITS == 4 && s < nk) {           // (the 8-bit loop has already read them)
        read_fp(0, s);
        read_fp(1, s);
    }
    for (; s < nk; ++s) {
        fp_mfmas(0);
        stage_barrier();
        issue_any(s + NST);
        if (s + 1 < nk) read_fp(0, s + 1);
        fp_mfmas(1);
        if (s + 1 < nk) read_fp(1, s + 1);
    }

    wait_vm<0>();                          // drain the look-ahead DMA before the wave ends
    __half* __restrict__ y = static_cast<__half*>(a.y);
    // Output through LDS: a lane owns four rows of one column of every 16 x 16 block, so direct stores
    // would be 2 bytes per lane.  Each wave instead parks its fp16 tile in its own slice of the (now dead)
    // stage ring and writes it out as 16-byte pieces, whole row segments per instruction.  Needs 16-byte
    // aligned output rows; otherwise the direct path below.
    // bytes per parked row: padded against bank conflicts where the ring has the room
    constexpr int WROW = (NWAVES * IB * 16 * (JB * 32 + 16) <= NST * ST_BYTES) ? JB * 32 + 16 : JB * 32;
    constexpr int WBUF = IB * 16 * WROW;
    static_assert(NWAVES * WBUF <= NST * ST_BYTES, "stage ring too small to park the output tile");
    const bool vec_ok = !a.fp_only && ((reinterpret_cast<uintptr_t>(a.y) & 15u) == 0) && (a.ldy % 8 == 0);
    if (vec_ok) {
        __syncthreads();                   // every wave is past its last read of the stage ring
        uint8_t* wbuf = lds + wave_u * WBUF;
#pragma unroll
        for (int i = 0; i < IB; ++i)
#pragma unroll
            for (int j = 0; j < JB; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = i * 16 + 4 * g + r;
                    *reinterpret_cast<__half*>(wbuf + row * WROW + (j * 16 + l16) * 2) = __float2half(cf[i][j][r]);
                }
        constexpr int CH = JB * 2;                       // 16-byte pieces per row
        constexpr int RPS = 64 / CH;                     // rows per store instruction (lanes >= RPS * CH idle)
        const int prow = lane / CH, pch = lane % CH;
#pragma unroll
        for (int p = 0; p < (IB * 16 + RPS - 1) / RPS; ++p) {
            const int row = p * RPS + prow;
            if (prow >= RPS || row >= IB * 16) continue;
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
    for (int i = 0; i < IB; ++i)
#pragma unroll
        for (int j = 0; j < JB; ++j) {
            int n = nw + j * 16 + l16;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                int t = tw + i * 16 + 4 * g + r;
                if (t < a.T && n < a.N) {
                    if (a.fp_only) reinterpret_cast<float*>(a.y)[(size_t)t * a.ldy + n] = cf[i][j][r];
                    else y[(size_t)t * a.ldy + n] = __float2half(cf[i][j][r]);
                }
            }
        }
}

template <int BITS, int BM, int BN, int WM, int WN, int BKB, int NST, int OCC, int GM, int MODE>
hipError_t launch_cfg(const GemmArgs& a, hipStream_t stream) {
    int tiles = ((a.T + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    hipLaunchKernelGGL((gemm_tiles16_kernel<BITS, BM, BN, WM, WN, BKB, NST, OCC, GM, MODE>), dim3(tiles),
                       dim3(WM * WN * 64), 0, stream, a);
    return hipGetLastError();
}

}  // namespace

// Equal operand widths, 256 x 128 tiles: eight waves, one workgroup per CU.  (The kernel is written for any
// tile of gemm_kernel's; the smaller ones mostly run one wave per SIMD, which this form's doubled instruction
// count slows down, and 64 x 96 or 96 x 64 per wave do not fit the register file in it.)
hipError_t launch_gemm_tiles16(const GemmArgs& a, hipStream_t stream) {
    const bool raw = a.y == nullptr;
    if (a.bits == 8) {
        if (!raw) return launch_cfg<8, 256, 128, 4, 2, 128, 2, 1, 4, 0>(a, stream);
        return launch_cfg<8, 256, 128, 4, 2, 128, 2, 1, 4, 1>(a, stream);
    }
    if (!raw) return launch_cfg<4, 256, 128, 4, 2, 128, 2, 1, 4, 0>(a, stream);
    if (a.code_sum && a.w_code_sum) return launch_cfg<4, 256, 128, 4, 2, 128, 2, 1, 4, 2>(a, stream);
    return launch_cfg<4, 256, 128, 4, 2, 128, 2, 1, 4, 1>(a, stream);
}

}  // namespace quik
