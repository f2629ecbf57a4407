// Persistent form of the 4-bit integer GEMM + dequantization epilogue + fp16 outlier GEMM for
// large token counts (Algorithm 1 of arXiv 2310.09259: "INTmatmul", "Dequantization", "FPmatmul"
// and the final add; epilogue fusion as in Section 3.4).  Same arithmetic, operand formats and
// widening as gemm_kernel in quik_gemm.hip (see the header of that file); what differs is the matrix
// instruction and how the work is laid over the chip:
//
//  * The integer product runs on v_mfma_i32_16x16x64_i8 and the outlier product on
//    v_mfma_f32_16x16x32_f16 (16 x 16 accumulator blocks: a lane holds four token rows of one channel).
//    On MI355X the chip holds its full clock under these where it lowers it under the 32 x 32 forms on
//    the same operand bytes; the price is twice the matrix instructions and 8-byte instead of 16-byte
//    fragment reads for the same bytes.
//  * One workgroup of eight waves per CU stays resident and walks through a list of output tiles
//    (256 token rows x 128 / 160 / 192 output channels).  The two-slot stage ring keeps running
//    across the tile boundary: while a tile's last two stages are multiplied, the slots they free
//    are already being filled with the first two stages of the workgroup's next tile.  A tile
//    therefore starts its matrix instructions right after the previous tile's stores were issued,
//    instead of after a workgroup launch, a parameter fetch and a first-stage round trip to memory.
//  * Tile widths are chosen per launch so that every CU gets the same number of 32-channel
//    column blocks (+-1): N / 32 blocks are cut into `tn` tiles per token-row panel, `rem` of them
//    one block wider than the others, spread evenly.  (With one fixed 256 x 192 tile the LLaMA-7B
//    up-projection at 2048 tokens is 464 tiles on 256 CUs: two rounds for 1.81 rounds of work.)
//    The two wave columns of the workgroup split a tile's blocks 3 + 3, 3 + 2 or 2 + 2; a wave with
//    two blocks runs a K loop instantiated for two.  Waves w and w + 4 take different wave columns,
//    so the two waves that share a SIMD carry 3 + 2 blocks on a five-block tile.
//  * XCD-aware order: each XCD owns a contiguous range of the tile list (channel panels outermost,
//    all token-row panels of a channel panel adjacent), and its CUs take neighbouring tiles of that
//    range at the same time, so a weight panel is fetched by one XCD only and the activation
//    panels it needs stay in that XCD's L2.
//  * One stage body serves every integer stage of a tile, whatever ring slot it sits in: the two slots
//    of an operand lie 32 KB apart, and the fragment address registers are flipped between them
//    (one XOR each per stage) right before the reads that need the other slot.
//  * The epilogue parameters (per token: scale, zero; per channel: weight scale, wReduced, bias) are
//    copied global -> LDS by the same DMA path as the operands, two stages before they are needed, so
//    they never occupy registers during the K loop.  With them come the code sums (per token, per
//    channel) of the tile that starts next: its accumulators start at -128 times their sum, which is
//    what the single-AND widening adds to 16 x the dot product, so the K loop ends on the latter.
//  * Which tile comes next is computed without run-time divisions: the plan carries the divisors of
//    that walk as multipliers prepared on the host (stream_tile in quik_kernels.h).
//  * The output tile leaves through a small per-wave LDS buffer, sixteen rows at a time, so the
//    stage ring is never needed for it.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include <type_traits>

#include "quik_kernels.h"
#include "quik_gemm_device.h"

namespace quik {

namespace {

using namespace gemm_dev;

template <int V> using ic = std::integral_constant<int, V>;
typedef float v4f __attribute__((ext_vector_type(4)));
#define QUIK_INLINE __attribute__((always_inline))

constexpr int BM = kStreamRows;         // token rows per tile
constexpr int TNX = 3;                  // most 32-channel blocks per wave
constexpr int BNX = 2 * TNX * 32;       // widest tile
constexpr int BKB = 128;                // bytes of every packed row per stage (256 columns)
constexpr int TM = 2;                   // 32-row blocks per wave
constexpr int IB = 2 * TM;              // 16 x 16 accumulator blocks per wave along the token rows
constexpr int NWAVES = 8, NT = NWAVES * 64;
constexpr int CPR = BKB / 16, RPI = 64 / CPR;
constexpr int IROWS = NWAVES * RPI;     // rows between a wave's consecutive copy instructions
constexpr int A_INSTR = BM / IROWS, B_INSTR = BNX / IROWS, LPS = A_INSTR + B_INSTR;
constexpr int KSUB = BKB / 32;
constexpr int A_BYTES = BM * BKB, B_BYTES = BNX * BKB;
// LDS map.  The two ring slots of an operand are SLOT_STRIDE apart (a power of two, so that a fragment
// address switches slots with one XOR); the gaps hold the epilogue parameters:
//   0       weights, slot 0 (24 KB)      24576  parameters (5 KB)
//   32768   weights, slot 1              57344  code sums of the tile that starts next (2 KB)
//   65536   activations, slot 0 (32 KB)  98304  activations, slot 1
//   131072  per-wave output buffers
constexpr int SLOT_STRIDE = 32768;
constexpr int OFF_B = 0, OFF_A = 65536;
static_assert(B_BYTES <= SLOT_STRIDE && A_BYTES <= SLOT_STRIDE, "ring slots overlap");
constexpr int PARK_ROWS = 16, PARK_ROW_BYTES = TNX * 64 + 16, PARK_BYTES = PARK_ROWS * PARK_ROW_BYTES;
constexpr int OFF_PARK = OFF_A + 2 * SLOT_STRIDE;
// parameter area: two per-token arrays of BM words, then three per-channel arrays of 256 words
// (weight scale and bias are fp16: 96 words used)
constexpr int OFF_PRM = B_BYTES;
constexpr int PRM_SCALE = 0, PRM_ZERO = BM * 4;
constexpr int PRM_WSCALE = 2 * BM * 4, PRM_WRED = PRM_WSCALE + 1024, PRM_BIAS = PRM_WRED + 1024;
static_assert(OFF_PRM + PRM_BIAS + 1024 <= SLOT_STRIDE, "parameters do not fit the gap");
// code sums of the next tile's BM token rows and (up to) 256 channels: they are the accumulators' initial value
constexpr int OFF_SUMS = SLOT_STRIDE + B_BYTES, SUMS_CS = 0, SUMS_WCS = BM * 4;
static_assert(OFF_SUMS + SUMS_WCS + 1024 <= OFF_A, "code sums do not fit the gap");
constexpr int SMEM_BYTES = OFF_PARK + NWAVES * PARK_BYTES;
static_assert(SMEM_BYTES <= 160 * 1024, "LDS budget");
static_assert(KSUB == 4, "the stage code below is written for four sub-steps");

// 4 bytes per lane, global -> LDS at lds_base + lane * 4 (see dma16 in quik_gemm_device.h)
__device__ __forceinline__ void dma4(v4i rsrc, uint32_t lds_base, uint32_t voff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                 :
                 : "s"(lds_base), "v"(voff), "s"(rsrc)
                 : "memory", "m0");
}

// MODE 0: fused epilogue (single-AND widening + correction); MODE 1: raw INT32 accumulators, widening
// without side data; MODE 2: raw accumulators, single-AND widening + correction.
template <int MODE>
__global__ __launch_bounds__(NT, 1) void gemm_stream_kernel(GemmArgs a, StreamPlan p) {
    constexpr bool RAW = MODE != 0;
    constexpr bool ASYM = MODE != 1;
    constexpr int SHIFT = ASYM ? 4 : 8;

    // One workgroup per CU owns half of every SIMD's register file: claim all 256 registers, so that the top
    // of the allocation is never a live register (the row-quantization kernel misread such a register on
    // MI355X when its allocation ended below its share of the file).
    asm volatile("" ::: "v255");
    __shared__ __align__(1024) uint8_t smem[SMEM_BYTES];
    uint8_t* const lds = smem;
    const uint8_t* const prm = smem + OFF_PRM;

    const int lane = threadIdx.x & 63;
    const int wave_u = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave_u & 3, wn = wave_u >> 2;
    // Per-lane address registers are set from an opaque copy of the lane id right before the phase that
    // uses them.  Computed once from the lane id, they would stay alive across the register-hungry
    // dequantization and output phases of every tile, be spilled there, and be re-read from scratch
    // memory inside the K loops, where a wait for such a reload is also a wait for the copies.
    auto opaque_lane = [&]() QUIK_INLINE -> int {
        int ln = lane;
        asm volatile("" : "+v"(ln));
        return ln;
    };

    // ---- this workgroup's tiles (stream_tile in quik_kernels.h has the order)
    // k-th tile of this workgroup: first token row, first channel, channels that exist, width in blocks
    // (plain scalars on purpose: a struct selected at run time ends up in scratch memory)
    auto geo = [&](int k, int& t0, int& n0, int& ncols, int& w) QUIK_INLINE -> bool {
        int nt, m, b0;
        if (!stream_tile(p, (int)blockIdx.x, k, &nt, &m)) return false;
        stream_panel(p, nt, &b0, &w);
        t0 = m * BM;
        n0 = b0 * 32;
        ncols = min(w * 32, a.N - n0);
        return true;
    };

    // stages of a tile: integer stages 0 .. nk_int-1, then the fp16 stages; stage v of a tile that starts
    // in ring slot P sits in slot (P + v) & 1
    const int row_bytes = a.K_b / 2;
    const int int_bytes = (row_bytes + 15) & ~15;        // up to the 16-byte piece that holds the last packed byte
    const int nk_int = (row_bytes + BKB - 1) / BKB;
    const int fp_bytes = a.n_out * 2;
    const int nk_fp = RAW ? 0 : (fp_bytes + BKB - 1) / BKB;
    const int nk = nk_int + nk_fp;
    const int lda_fp = a.ldo * 2, ldb_fp = a.ldwo * 2;

    // ---- copy geometry (the same for every tile: offsets are relative to the tile's descriptors).
    // Copy instruction i of a wave moves 16 bytes per lane: rows (i * 8 + wave) * 8 + lane / 8 of the
    // operand panel, 16-byte slot lane % 8 of the row, XOR-swizzled with the row.  With this row order the
    // swizzle term does not depend on i, so one register per operand holds a lane's offset and
    // instruction i adds i * 64 rows.
    const uint32_t lds_base = lds_addr(lds);
    const uint32_t m0A = lds_base + OFF_A + wave_u * 1024;
    const uint32_t m0B = lds_base + OFF_B + wave_u * 1024;
    // One stage's copy: descriptors, per-lane offsets of copy instruction 0 (or out of range), the
    // offset of the stage inside a row and the step between a wave's consecutive copy instructions.
    struct Copy {
        v4i A, B;
        uint32_t va, vb, so, stepA, stepB;
    };
    // stage j (integer, or fp16 if `fp`) of the tile at token row t0, channel n0 with `ncols` channels.  The
    // two descriptors are rebuilt here from the tile's origin (a few scalar operations) rather than kept
    // for every tile and kind.  Lanes whose 16-byte piece lies beyond the row's data (last, partial stage)
    // are pointed out of range and deliver zeros; so are all lanes of a copy that is switched off (`on`
    // false: no next tile -- the slot's content is dead then), which keeps the stage code free of branches.
    auto prep_copy = [&](Copy& r, int t0, int n0, int ncols, bool fp, int j, bool on) QUIK_INLINE {
        const uint32_t ln = (uint32_t)opaque_lane();
        const uint32_t row0 = (uint32_t)wave_u * RPI + ln / CPR, c = ((ln % CPR) ^ (uint32_t)swz<BKB>((int)row0)) * 16;
        const int lda = fp ? lda_fp : a.ldq, ldb = fp ? ldb_fp : a.ldw;
        const uint8_t* pa = static_cast<const uint8_t*>(fp ? a.x_out : a.xq);
        const uint8_t* pb = static_cast<const uint8_t*>(fp ? a.w_out : a.w_q);
        r.A = make_rsrc(pa + (size_t)t0 * lda, (size_t)(a.T - t0) * lda);
        r.B = make_rsrc(pb + (size_t)n0 * ldb, (size_t)ncols * ldb);
        const bool live = on && ((uint32_t)(j * BKB) + c < (uint32_t)(fp ? fp_bytes : int_bytes));
        r.va = live ? row0 * (uint32_t)lda + c : kOob;
        r.vb = live ? row0 * (uint32_t)ldb + c : kOob;
        r.so = (uint32_t)(j * BKB);
        r.stepA = (uint32_t)(IROWS * lda);
        r.stepB = (uint32_t)(IROWS * ldb);
    };
    // copy instruction d (0 .. LPS-1) of that stage into ring slot `slot`
    auto issue_copy = [&](const Copy& r, int slot, int d) QUIK_INLINE {
        const uint32_t so = (uint32_t)slot * SLOT_STRIDE;
        if (d < A_INSTR) dma16(r.A, m0A + so + d * (IROWS * BKB), r.va + (uint32_t)d * r.stepA, r.so);
        else dma16(r.B, m0B + so + (d - A_INSTR) * (IROWS * BKB), r.vb + (uint32_t)(d - A_INSTR) * r.stepB, r.so);
    };
    // the epilogue parameters of a tile, global -> LDS (each wave copies a share)
    auto issue_params = [&](int t0, int n0, int ncols) QUIK_INLINE {
        if constexpr (!RAW) {
            const uint32_t pb = lds_base + OFF_PRM;
            const uint32_t l4 = (uint32_t)opaque_lane() * 4u;
            const size_t rows = (size_t)(a.T - t0), cols = (size_t)ncols;
            if (wave_u < 4) {                              // 64 token rows each
                const uint32_t o = (uint32_t)wave_u * 256u;
                dma4(make_rsrc(a.scale + t0, rows * 4), pb + PRM_SCALE + o, l4 + o);
                dma4(make_rsrc(a.zero + t0, rows * 4), pb + PRM_ZERO + o, l4 + o);
            } else if (wave_u < 7) {                       // 64 channels each
                const uint32_t o = (uint32_t)(wave_u - 4) * 256u;
                dma4(make_rsrc(a.w_reduced + n0, cols * 4), pb + PRM_WRED + o, l4 + o);
            } else {                                       // fp16 arrays: 128 channels per instruction
                const __half* ws = static_cast<const __half*>(a.w_scale) + n0;
                const __half* bs = a.bias ? static_cast<const __half*>(a.bias) + n0 : ws;
                const size_t bb = a.bias ? cols * 2 : 0;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    dma4(make_rsrc(ws, cols * 2), pb + PRM_WSCALE + h * 256, l4 + h * 256);
                    dma4(make_rsrc(bs, bb), pb + PRM_BIAS + h * 256, l4 + h * 256);
                }
            }
        }
    };

    // the code sums of a tile (the one that starts next), global -> LDS; `on` false: no such tile, zeros arrive
    auto issue_sums = [&](int t0, int n0, int ncols, bool on) QUIK_INLINE {
        if constexpr (ASYM) {
            const uint32_t sb = lds_base + OFF_SUMS;
            const uint32_t l4 = (uint32_t)opaque_lane() * 4u;
            if (wave_u < 4) {                              // 64 token rows each
                const uint32_t o = (uint32_t)wave_u * 256u;
                dma4(make_rsrc(a.code_sum + t0, on ? (size_t)(a.T - t0) * 4 : 0), sb + SUMS_CS + o, l4 + o);
            } else if (wave_u < 7) {                       // 64 channels each
                const uint32_t o = (uint32_t)(wave_u - 4) * 256u;
                dma4(make_rsrc(a.w_code_sum + n0, on ? (size_t)ncols * 4 : 0), sb + SUMS_WCS + o, l4 + o);
            }
        }
    };

    // The compiler does not see the DMA's writes to LDS, so it is free to move an ordinary LDS read up to
    // the last barrier; for the reads that start a phase that means registers held across the whole phase
    // before.  tie() makes an address register depend (without any instruction) on a value computed at
    // the end of that phase, which keeps the reads behind it.
    auto tie = [&](uint32_t& addr, uint32_t dep) QUIK_INLINE { asm volatile("" : "+v"(addr) : "v"(dep)); };

    // ---- fragment addresses: one register per operand and sub-step.  The matrix instruction is the
    // 16 x 16 x 64 one: lane (l = lane % 16, g = lane / 16) supplies the 16 int8 values of k-group g for row
    // (or channel) l of a 16-row block, i.e. 8 packed bytes: bytes 8g .. 8g + 7 of the sub-step's 32 bytes
    // of that row.  A register holds the address for the wave's first block; the block is an immediate.
    // Registers 0, 1 point into ring slot `slot`, registers 2, 3 into the other one: a stage flips the
    // register of sub-step q to its own slot right before it reads that sub-step (see int_stage).
    uint32_t rdA[KSUB], rdB[KSUB];
    auto set_rd = [&](int cb0, int slot, uint32_t dep) QUIK_INLINE {
        uint32_t lnu = (uint32_t)lane;
        tie(lnu, dep);
        const int ln = (int)lnu;
        const int l = ln & 15, g = (ln >> 4) & 3;
        const int ra = wm * TM * 32 + l, rb = cb0 * 32 + l;
#pragma unroll
        for (int ks = 0; ks < KSUB; ++ks) {
            const int so = (ks < 2 ? slot : slot ^ 1) * SLOT_STRIDE;
            rdA[ks] = OFF_A + so + ra * BKB + (((ks * 2 + (g >> 1)) ^ swz<BKB>(ra)) << 4) + (g & 1) * 8;
            rdB[ks] = OFF_B + so + rb * BKB + (((ks * 2 + (g >> 1)) ^ swz<BKB>(rb)) << 4) + (g & 1) * 8;
        }
    };
    // first block and block count of this wave in a tile of width w (tiles narrower than four blocks
    // are run as four: the surplus rows of the weight panel arrive as zeros)
    auto wave_cols = [&](int w, int& cb0, int& tna) QUIK_INLINE {
        const int we = max(w, 4);
        cb0 = wn ? (we + 1) / 2 : 0;
        tna = wn ? we / 2 : (we + 1) / 2;
    };

    // Raw fragments of two sub-steps (a fragment: 8 packed bytes per lane = 16 columns of one row of a 16-row
    // block) and two sets of widened operands (a fragment widens to the 16 int8 values one matrix instruction
    // takes from the lane): while the MFMAs of a sub-step read one set, the next sub-step's raw words are
    // widened into the other, a word per MFMA slot, so no MFMA ever waits for an operand made just before it.
    constexpr int NFX = IB + 2 * TNX;
    uint2 R[2][NFX];
    v4i U[2][NFX];
    auto read_frag = [&](int set, int f, int ks) QUIK_INLINE {
        const uint32_t off = (f < IB) ? rdA[ks] + (uint32_t)(f * 16 * BKB) : rdB[ks] + (uint32_t)((f - IB) * 16 * BKB);
        R[set][f] = *reinterpret_cast<const uint2*>(lds + off);
    };
    // word w (fragment w / 2, word w % 2) of raw set `rset`, widened into operand set `set`
    auto widen_word = [&](int set, int rset, int w) QUIK_INLINE {
        constexpr uint32_t M = 0xF0F0F0F0u;
        const int f = w >> 1, k = w & 1;
        const bool act = f < IB;                             // activations: even k in the high nibble
        const uint32_t x = k ? R[rset][f].y : R[rset][f].x;
        uint32_t hi = x & M;                                 // 16 * signed high nibble
        uint32_t lo = ASYM ? ((x ^ 0x08080808u) & 0x0F0F0F0Fu)         // low nibble + 8
                           : ((x << 4) & M);                           // 16 * signed low nibble
        // A use right here: the operands of a stage's third sub-step are first read behind the stage
        // barrier's branches, and without it the compiler sinks their widening out of the MFMA slots of the
        // second sub-step into one burst behind the barrier.
        asm volatile("" : "+v"(hi), "+v"(lo));
        U[set][f][2 * k] = (int)(act ? hi : lo);
        U[set][f][2 * k + 1] = (int)(act ? lo : hi);
    };
    // a tile's first two sub-steps' fragments (its stage 0, in ring slot `slot`), and the operands its
    // first sub-step starts with
    auto first_reads = [&](int cb0, int slot, uint32_t dep) QUIK_INLINE {
        set_rd(cb0, slot, dep);
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int f = 0; f < NFX; ++f) read_frag(q, f, q);
#pragma unroll
        for (int w = 0; w < NFX * 2; ++w) widen_word(0, 0, w);
    };

    int cur_t0 = 0, cur_n0 = 0, cur_nc = 0, cur_w = 0, nxt_t0 = 0, nxt_n0 = 0, nxt_nc = 0, nxt_w = 0;
    if (!geo(0, cur_t0, cur_n0, cur_nc, cur_w)) return;

    // ---- first tile: its first two stages.  `rf` describes the stage copied last and is carried from
    // stage to stage (see prep_refill).
    issue_sums(cur_t0, cur_n0, cur_nc, true);            // (first: the wait for stage 0 below then covers it)
    Copy rf;
    prep_copy(rf, cur_t0, cur_n0, cur_nc, false, 0, true);
#pragma unroll
    for (int d = 0; d < LPS; ++d) issue_copy(rf, 0, d);
    prep_copy(rf, cur_t0, cur_n0, cur_nc, false, 1, true);
#pragma unroll
    for (int d = 0; d < LPS; ++d) issue_copy(rf, 1, d);
    wait_vm<LPS>();                                       // stage 0 has landed
    __syncthreads();
    {
        int cb0, tna;
        wave_cols(cur_w, cb0, tna);
        first_reads(cb0, 0, 0u);
    }

    int P = 0;                                            // ring slot of the current tile's stage 0
    for (int k = 0;; ++k) {
        const bool more = geo(k + 1, nxt_t0, nxt_n0, nxt_nc, nxt_w);
        int cb0, tna, cb0n = 0, tnan = 0;
        wave_cols(cur_w, cb0, tna);
        if (more) wave_cols(nxt_w, cb0n, tnan);

        // What goes into the slot that the barrier of stage v frees: stage v + 2 of this tile, else a stage of
        // the next tile (the ring simply runs on).  Descriptors and lane offsets are rebuilt only where they
        // change -- at the first stage of an operand kind or tile, and at a last, partial stage (lanes beyond
        // the data are masked) -- which is a handful of times per tile; every other stage just moves the
        // offset inside the rows.  (Rebuilding them at every stage costs about a hundred scalar
        // instructions per wave right behind the barrier, where all eight waves would do it at once.)
        auto prep_refill = [&](Copy& r, int v) QUIK_INLINE {
            const int u = v + 2;
            const bool next = u >= nk, fp = !next && u >= nk_int;
            const int j = next ? u - nk : (fp ? u - nk_int : u);
            if (j == 0 || (j + 1) * BKB > (fp ? fp_bytes : int_bytes))
                prep_copy(r, next ? nxt_t0 : cur_t0, next ? nxt_n0 : cur_n0, next ? nxt_nc : cur_nc, fp, j, !next || more);
            else
                r.so = (uint32_t)(j * BKB);
        };

        auto tile = [&](auto tna_c) QUIK_INLINE {
            constexpr int TNA = decltype(tna_c)::value;
            constexpr int JB = 2 * TNA;                               // 16-channel accumulator blocks per wave
            constexpr int NFA = IB + JB;                              // fragments per sub-step
            constexpr int NMF = IB * JB;                              // MFMAs per sub-step
            constexpr int CS = NMF / 8;                               // a copy instruction every CS-th MFMA slot
            static_assert(NMF >= NFA * 2 && 8 >= LPS, "copy, read and widening work is spread over the MFMA slots");

            // The accumulators start at -128 * (code_sum[t] + w_code_sum[n]): the single-AND widening leaves
            // 16 x the integer dot product plus 128 times these sums, so that the K loop ends on 16 x the dot
            // product itself (two's complement, nothing overflows on the way).  The sums were copied to LDS
            // two stages before the previous tile's K loop ended (before the first stage for the first tile).
            v4i acc[IB][JB];
            if constexpr (ASYM) {
                const int lane_i = opaque_lane();
                const int l16i = lane_i & 15, gi = lane_i >> 4;
                const uint8_t* sums = smem + OFF_SUMS;
                int nw[JB];
#pragma unroll
                for (int j = 0; j < JB; ++j)
                    nw[j] = -128 * *reinterpret_cast<const int*>(sums + SUMS_WCS + (cb0 * 32 + j * 16 + l16i) * 4);
#pragma unroll
                for (int i = 0; i < IB; ++i) {
                    const int4 cs = *reinterpret_cast<const int4*>(sums + SUMS_CS + (wm * TM * 32 + i * 16 + 4 * gi) * 4);
                    const int nc[4] = {-128 * cs.x, -128 * cs.y, -128 * cs.z, -128 * cs.w};
#pragma unroll
                    for (int j = 0; j < JB; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[i][j][r] = nc[r] + nw[j];
                }
            } else {
#pragma unroll
                for (int i = 0; i < IB; ++i)
#pragma unroll
                    for (int j = 0; j < JB; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[i][j][r] = 0;
            }

            // One integer stage (stage s of the tile, in ring slot `slot`).  The refill of the slot it frees
            // is spread over the MFMA slots after the barrier.  A sub-step (32 packed bytes of every row) is
            // one 16 x 16 x 64 instruction per accumulator block, issued from one operand set; meanwhile the
            // next sub-step's raw fragments are widened into the other set and the raw registers of this
            // sub-step (widened during the one before) are refilled from LDS with the fragments of the
            // sub-step after the next -- which, in the last two sub-steps, belongs to the next stage in the
            // other slot (after the last integer stage that is an fp16 stage, or the next tile: its
            // fragments are simply not used as integers).
            auto int_stage = [&](int s, int slot) QUIK_INLINE {
#pragma unroll
                for (int ks = 0; ks < KSUB; ++ks) {
                    const int par = ks & 1;                           // raw set of this sub-step; the other holds the next one
                    const int tks = (ks + 2) % KSUB;
                    if (ks == 2) {
                        wait_vm<0>();
                        __syncthreads();          // stage s + 1 has landed for everybody; nobody reads this stage's slot any more
                        prep_refill(rf, s);
                        if (s == nk_int - 2) {
                            issue_params(cur_t0, cur_n0, cur_nc);
                            issue_sums(nxt_t0, nxt_n0, nxt_nc, more);
                        }
                    }
                    // sub-step tks was last read in the other slot
                    rdA[tks] ^= SLOT_STRIDE;
                    rdB[tks] ^= SLOT_STRIDE;
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int hm = 0; hm < NMF; ++hm) {
                        const int j = hm / IB, i = hm % IB;
                        acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(U[par][i], U[par][IB + j], acc[i][j], 0, 0, 0);
                        if (ks == 2 && hm % CS == 0 && hm / CS < LPS) issue_copy(rf, slot, hm / CS);
                        // the next sub-step's operands, a word per MFMA slot
#pragma unroll
                        for (int w = 0; w < NFA * 2; ++w)
                            if (w * NMF / (NFA * 2) == hm) widen_word(par ^ 1, par ^ 1, w);
                        // this sub-step's raw registers were widened during the sub-step before
                        if (hm >= NMF / 3 && hm - NMF / 3 < NFA) read_frag(par, hm - NMF / 3, tks);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            };

            int slot = P;
            for (int s = 0; s < nk_int; ++s) {
                int_stage(s, slot);
                slot ^= 1;
            }
            __builtin_amdgcn_sched_barrier(0);

            // The epilogue's per-lane addresses depend only on the lane, so the compiler would compute them
            // once, before the tile loop, and keep dozens of registers alive through the K loops.  An
            // opaque copy of the lane id per tile keeps that arithmetic here.
            const int lane_e = opaque_lane();
            const int l16e = lane_e & 15, ge = lane_e >> 4;     // accumulator block: channel l16e, token rows 4 ge .. 4 ge + 3
            const int tw = cur_t0 + wm * TM * 32, nw = cur_n0 + cb0 * 32, n_end = cur_n0 + cur_nc;
            uint32_t done = 0;                            // a value from the end of this tile's output
            if constexpr (RAW) {
#pragma unroll
                for (int i = 0; i < IB; ++i)
#pragma unroll
                    for (int j = 0; j < JB; ++j) {
                        const int n = nw + j * 16 + l16e;
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int t = tw + i * 16 + 4 * ge + r;
                            if (t < a.T && n < n_end) {
                                a.acc[(size_t)t * a.ldacc + n] = acc[i][j][r] >> SHIFT;   // exact: a multiple of 2^SHIFT
                            }
                        }
                    }
            } else {
                // Dequantization: the accumulator is 16 x the integer dot product, its conversion to binary32
                // is exact, and 2^-4 rides on the weight scale.
                float c_sw[JB], c_wr[JB], c_bv[JB];
#pragma unroll
                for (int j = 0; j < JB; ++j) {
                    const int col = cb0 * 32 + j * 16 + l16e;         // inside the tile
                    c_sw[j] = __half2float(*reinterpret_cast<const __half*>(prm + PRM_WSCALE + col * 2)) *
                              (1.0f / (float)(1 << SHIFT));           // exact power-of-two factor
                    c_bv[j] = a.bias ? __half2float(*reinterpret_cast<const __half*>(prm + PRM_BIAS + col * 2)) : 0.0f;
                    c_wr[j] = *reinterpret_cast<const float*>(prm + PRM_WRED + col * 4);
                }
                // Per-token parameters of the four rows a lane holds of a 16-row block, read one block ahead of
                // their use; tied to the results of the block before, or the scheduler would hoist all reads
                // to the top.
                uint32_t dq_dep = 0;
                v4f cf[IB][JB];
                float4 sa4[2], z4[2];
                auto load_group = [&](int i) QUIK_INLINE {
                    const int lr = wm * TM * 32 + i * 16 + 4 * ge;
                    uint32_t o = (uint32_t)lr * 4u;
                    tie(o, dq_dep);
                    sa4[i & 1] = *reinterpret_cast<const float4*>(prm + PRM_SCALE + o);
                    z4[i & 1] = *reinterpret_cast<const float4*>(prm + PRM_ZERO + o);
                };
                load_group(0);
#pragma unroll
                for (int i = 0; i < IB; ++i) {
                    const int b = i & 1;
                    if (i + 1 < IB) load_group(i + 1);
                    const float sa_[4] = {sa4[b].x, sa4[b].y, sa4[b].z, sa4[b].w};
                    const float sh_[4] = {z4[b].x + 8.0f * sa4[b].x, z4[b].y + 8.0f * sa4[b].y, z4[b].z + 8.0f * sa4[b].z,
                                          z4[b].w + 8.0f * sa4[b].w};    // zeroAct + halfRange * scaleAct
#pragma unroll
                    for (int j = 0; j < JB; ++j)
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr) {
                            cf[i][j][rr] = __builtin_fmaf((float)acc[i][j][rr], sa_[rr] * c_sw[j],
                                                          __builtin_fmaf(sh_[rr], c_wr[j], c_bv[j]));
                        }
                    dq_dep = __float_as_uint(cf[i][JB - 1][3]);
                }

                // fp16 outlier stages on the dequantized tile (stage nk_int + f of the tile): two k-steps of 32
                // columns (64 bytes of every row) per stage, one 16 x 16 x 32 instruction per accumulator block
                // and k-step; lane (l, g) supplies columns 8g .. 8g + 7 of the k-step, one 16-byte piece.  The
                // two operand sets of the integer phase (free now) hold one k-step each; while one feeds the
                // MFMAs, the other is refilled.
                uint32_t fpA[2], fpB[2];
                {
                    uint32_t lnu = (uint32_t)lane;
                    tie(lnu, dq_dep);
                    const int l = (int)lnu & 15, g = ((int)lnu >> 4) & 3;
                    const int ra = wm * TM * 32 + l, rb = cb0 * 32 + l;
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk) {
                        fpA[kk] = OFF_A + slot * SLOT_STRIDE + ra * BKB + (((kk * 4 + g) ^ swz<BKB>(ra)) << 4);
                        fpB[kk] = OFF_B + slot * SLOT_STRIDE + rb * BKB + (((kk * 4 + g) ^ swz<BKB>(rb)) << 4);
                    }
                }
                auto read_fp_frag = [&](auto kk_c, int f) QUIK_INLINE {
                    constexpr int KK = decltype(kk_c)::value;
                    const uint32_t off = (f < IB) ? fpA[KK] + (uint32_t)(f * 16 * BKB) : fpB[KK] + (uint32_t)((f - IB) * 16 * BKB);
                    U[KK][f] = *reinterpret_cast<const v4i*>(lds + off);
                };
                // k-step KK of a stage: its MFMAs from set KK, and beside them, a fragment per MFMA slot, the
                // reads that refill the other set -- the stage's second k-step during the first, the next
                // stage's first k-step (other slot) during the second, together with the refill copies.
                auto fp_mfmas = [&](auto kk_c, int slot_, bool reads) QUIK_INLINE {
                    constexpr int KK = decltype(kk_c)::value;
#pragma unroll
                    for (int m = 0; m < NMF; ++m) {
                        const int j = m / IB, i = m % IB;
                        cf[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, U[KK][i]),
                                                                         __builtin_bit_cast(v8h, U[KK][IB + j]), cf[i][j], 0, 0, 0);
                        if (KK == 1 && m % CS == 0 && m / CS < LPS) issue_copy(rf, slot_, m / CS);
                        if (m < NFA && reads) read_fp_frag(ic<KK ^ 1>{}, m);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                };
                // The barrier sits between the k-steps: every read of this stage has been issued by then (and is
                // waited for), so its slot is free, and the reads that follow go to the next stage, which must
                // have landed.  LAST: the tile's last stage -- no look-ahead into the next tile, whose waves'
                // column blocks may differ.
                auto fp_stage = [&](auto last_c, int f, int slot_) QUIK_INLINE {
                    constexpr bool LAST = decltype(last_c)::value != 0;
                    fp_mfmas(ic<0>{}, slot_, true);
                    wait_vm<0>();
                    __syncthreads();
                    prep_refill(rf, nk_int + f);
                    __builtin_amdgcn_sched_barrier(0);
                    fp_mfmas(ic<1>{}, slot_, !LAST);
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk) {
                        fpA[kk] ^= SLOT_STRIDE;
                        fpB[kk] ^= SLOT_STRIDE;
                    }
                };
                // the first stage's first k-step (unconditional: a conditional definition would keep the set's
                // registers occupied from the top of the epilogue); from here on set 0 is read in the other slot
#pragma unroll
                for (int f = 0; f < NFA; ++f) read_fp_frag(ic<0>{}, f);
                fpA[0] ^= SLOT_STRIDE;
                fpB[0] ^= SLOT_STRIDE;
                for (int f = 0; f + 1 < nk_fp; ++f) {
                    fp_stage(ic<0>{}, f, slot);
                    slot ^= 1;
                }
                if (nk_fp > 0) fp_stage(ic<1>{}, nk_fp - 1, slot);
                __builtin_amdgcn_sched_barrier(0);

                // Output: a lane owns four rows of one column of every 16 x 16 block, so direct stores would be
                // 2 bytes per lane.  Each wave parks the sixteen rows of a block row of its fp16 tile in its own
                // LDS buffer and writes them out as 16-byte pieces, whole row segments per store
                // instruction.  Needs 16-byte aligned output rows; otherwise the direct path below.
                __half* __restrict__ y = static_cast<__half*>(a.y);
                const bool vec_ok = ((reinterpret_cast<uintptr_t>(a.y) & 15u) == 0) && (a.ldy % 8 == 0);
                if (vec_ok) {
                    uint8_t* wbuf = smem + OFF_PARK + wave_u * PARK_BYTES;
                    constexpr int CH = TNA * 4;                  // 16-byte pieces per row
                    constexpr int RPS = 64 / CH;                 // rows per store instruction
                    const int prow = lane_e / CH, pch = lane_e % CH;
#pragma unroll
                    for (int i = 0; i < IB; ++i) {               // rows 16 i .. 16 i + 15 of the wave's tile
#pragma unroll
                        for (int j = 0; j < JB; ++j)
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const int row = 4 * ge + r;      // inside the 16 rows
                                *reinterpret_cast<__half*>(wbuf + row * PARK_ROW_BYTES + (j * 16 + l16e) * 2) =
                                    __float2half(cf[i][j][r]);
                            }
#pragma unroll
                        for (int q = 0; q < (PARK_ROWS + RPS - 1) / RPS; ++q) {
                            const int row = q * RPS + prow;
                            if (prow < RPS && row < PARK_ROWS) {
                                const uint4 v = *reinterpret_cast<const uint4*>(wbuf + row * PARK_ROW_BYTES + pch * 16);
                                done = v.x;
                                const int t = tw + i * 16 + row, n = nw + pch * 8;
                                if (t < a.T) {
                                    __half* dst = y + (size_t)t * a.ldy + n;
                                    if (n + 8 <= n_end) {
                                        store16_through(dst, v);
                                    } else {
                                        const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                                        for (int e = 0; e < 8; ++e)
                                            if (n + e < n_end)
                                                reinterpret_cast<uint16_t*>(dst)[e] = (uint16_t)(wv[e >> 1] >> (16 * (e & 1)));
                                    }
                                }
                            }
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < IB; ++i)
#pragma unroll
                        for (int j = 0; j < JB; ++j) {
                            const int n = nw + j * 16 + l16e;
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const int t = tw + i * 16 + 4 * ge + r;
                                if (t < a.T && n < n_end) y[(size_t)t * a.ldy + n] = __float2half(cf[i][j][r]);
                            }
                        }
                }
            }
            // The next tile's first fragments (its stage 0 has landed: the barrier of this tile's last
            // stage waited for it), read once this tile's results have left the registers.
            __builtin_amdgcn_sched_barrier(0);
            if (more) first_reads(cb0n, (P + nk) & 1, done);
        };

        if (tna >= 3) tile(ic<3>{});
        else tile(ic<2>{});

        if (!more) break;
        P = (P + nk) & 1;
        cur_t0 = nxt_t0; cur_n0 = nxt_n0; cur_nc = nxt_nc; cur_w = nxt_w;
    }
    wait_vm<0>();
}

}  // namespace

// Tile plan of the persistent kernel for a [T, N] output with K_b base columns on `cus` compute
// units, or false if the shape is better served by the per-tile kernels (too few tiles to give every
// CU one, or too shallow).
bool plan_gemm_stream(int T, int N, int K_b, int cus, StreamPlan* p) {
    if (cus < kXcds || cus % kXcds) return false;
    if (K_b < 4 * 2 * BKB || (N & 1)) return false;     // at least four integer stages; fp16 arrays copied as dwords
    const int tiles_m = (T + BM - 1) / BM;
    const int nb = (N + 31) / 32;                       // 32-channel blocks
    const int tn_min = (nb + 2 * TNX - 1) / (2 * TNX);  // tiles per row panel at full width
    // Candidate tile counts: from full width down to four blocks per tile.  Estimated time of a
    // launch in units of one block's K loop: the busiest CU's blocks (its tiles, each `base` wide plus
    // its share of the wider ones) plus a fixed cost per tile.
    const int tn_max = nb / 4 > tn_min ? nb / 4 : tn_min;
    if ((long)tiles_m * tn_max < cus) return false;     // even the narrowest tiles leave CUs without one
    double best = 1e30;
    int best_tn = tn_min;
    for (int tn = tn_min; tn <= tn_max; ++tn) {
        const int base = nb / tn, rem = nb % tn;
        if (base + (rem ? 1 : 0) > 2 * TNX) continue;
        const long tiles = (long)tiles_m * tn;
        const long r = (tiles + cus - 1) / cus;         // tiles of the busiest CU
        const double blocks = (double)(r * base + (r * rem + tn - 1) / tn);
        // (last term: among equal estimates, the tile count that leaves the fewest CUs one tile short)
        const double cost = blocks + 0.35 * (double)r + 1e-3 * (double)(r * cus - tiles) / (double)cus;
        if (cost < best - 1e-9) { best = cost; best_tn = tn; }
    }
    p->tiles_m = tiles_m;
    p->tn = best_tn;
    p->base = nb / best_tn;
    p->rem = nb % best_tn;
    p->grid = cus;
    return best < 1e29 && finish_stream_plan(p);
}

hipError_t launch_gemm_stream(const GemmArgs& a, const StreamPlan& p, hipStream_t stream) {
    const bool raw = a.y == nullptr;
    if (!raw) hipLaunchKernelGGL(gemm_stream_kernel<0>, dim3(p.grid), dim3(NT), 0, stream, a, p);
    else if (a.code_sum && a.w_code_sum) hipLaunchKernelGGL(gemm_stream_kernel<2>, dim3(p.grid), dim3(NT), 0, stream, a, p);
    else hipLaunchKernelGGL(gemm_stream_kernel<1>, dim3(p.grid), dim3(NT), 0, stream, a, p);
    return hipGetLastError();
}

}  // namespace quik
