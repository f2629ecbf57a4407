// Internal launch interfaces between the C ABI (quik_api.hip) and the kernels.
// Everything here is private to the shared library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace quik {

struct QuantizeArgs {
    const void* x;        // fp16 [T, ldx]
    int T, K, ldx;
    const int32_t* idx;   // [n_out]
    int n_out, bits;
    void* xq;             // packed [T, ldq bytes]
    int ldq;
    float* scale;         // [T]
    float* zero;          // [T]
    void* x_out;          // fp16 [T, ldo]
    int ldo;
    int32_t* code_sum;    // [T] sum of the signed codes at even positions (4-bit; may be null)
    int format;           // 0: row-major packed rows.  1: 4-bit codes written as E3M2 patterns in the panel
                          //    layout (quik_fp6_device.h); xq is then the [stage][T][48-byte] buffer and
                          //    ldq = 48 * stages.  2: 4-bit codes in the activation format of the 2:4-sparse
                          //    path (quik_sp24_device.h); xq is the [stage][T][32-byte] buffer, ldq = 32 * stages
};

struct GemmArgs {
    const void* xq;       // packed [T, ldq bytes]
    int ldq;
    const float* scale;   // [T]
    const float* zero;    // [T]
    const int32_t* code_sum;    // [T] sum of the signed activation codes at even k (4-bit; see quik_gemm.hip)
    const void* x_out;    // fp16 [T, ldo]
    int ldo;
    int T, K_b, n_out, bits;
    const void* w_q;      // packed [N, ldw bytes]
    int ldw;
    const void* w_scale;  // fp16 [N]
    const float* w_reduced;
    const int32_t* w_code_sum;  // [N] sum of the signed weight codes at odd k (4-bit)
    const void* w_out;    // fp16 [N, ldwo]
    int ldwo;
    const void* bias;     // fp16 [N] or null
    int N;
    void* y;              // fp16 [T, ldy]   (epilogue mode)
    int ldy;
    int32_t* acc;         // int32 [T, ldacc] (raw-accumulator mode, y == null)
    int ldacc;
    int fp_only;          // 1: skip the integer part; y is then fp32 [T, ldy] = outlier product only
    int w_bits;           // weight bits if they differ from `bits` (4 under 8-bit activations); 0: same
};

struct WeightReduceArgs {
    const void* w_q;
    int ldw;
    const void* w_scale;
    int N, K_b, bits;
    float* w_reduced;
    int32_t* w_code_sum;  // [N], may be null
};

// Tile plan of the persistent 4-bit GEMM (quik_gemm_stream.hip): every token-row panel of 256 rows is
// cut into `tn` tiles along the output channels, `rem` of them `base + 1` blocks of 32 channels wide
// and the others `base`, spread evenly; `grid` resident workgroups walk through the tiles.
// The fields after `grid` are derived from the first five by finish_stream_plan(): whatever the walk over
// the tiles would have to divide by is prepared on the host (a division of two run-time scalars costs a
// workgroup some three hundred clocks, and the walk needs seventeen of them per tile).
struct StreamPlan {
    int tiles_m, tn, base, rem, grid;
    int per_xcd, tq, tr;                    // workgroups per XCD; tiles per XCD: tq, and one more on the first tr XCDs
    int blocked_mask;                       // bit x: XCD x walks its range in the blocked order (see stream_tile)
    int mpr[2], panels[2], inc[2];          // blocked order, XCDs with tq + 1 tiles [0] / with tq tiles [1]
    unsigned long long mg_tiles_m, mg_tn, mg_mpr[2], mg_panels[2];   // stream_magic() of these divisors
};
constexpr int kStreamRows = 256;       // token rows per tile
constexpr int kStreamXcds = 8;         // workgroup b runs on XCD b % 8
constexpr int kStreamMagicBits = 40;
constexpr int kStreamMagicRange = 1 << 20;   // stream_div is exact for x, d below this

// x / d for 0 <= x, 1 <= d below kStreamMagicRange, with mg = stream_magic(d) = ceil(2^40 / d): mg * d =
// 2^40 + e with e < d, so x * mg / 2^40 exceeds x / d by x * e / (d * 2^40) < x / 2^40 < 1 / d, too little to
// carry the fraction of x / d (at most (d - 1) / d) to the next integer.
inline unsigned long long stream_magic(int d) {
    return d > 0 ? ((1ull << kStreamMagicBits) + (unsigned long long)d - 1) / (unsigned long long)d : 0;
}
__host__ __device__ inline int stream_div(int x, unsigned long long mg) {
    return (int)(((unsigned long long)(unsigned)x * mg) >> kStreamMagicBits);
}

// The k-th tile of workgroup `block`: channel panel nt (of p.tn) and token panel m (of p.tiles_m), or false
// if the workgroup has fewer tiles.  The tile list (channel panels outermost, the token panels of a channel
// panel adjacent) is cut into one contiguous range per XCD.  Plain order inside a range: a round of the
// XCD's workgroups takes consecutive tiles, i.e. a few channel panels with all their token panels, and
// every round streams all activations through the XCD's L2 again.  When the range is a whole number of
// channel panels and of rounds, a round instead takes ALL channel panels of the range with a slice of the
// token panels (the activations pass through the L2 once per launch, the XCD's smaller share of the
// weights once per round); from round to round a workgroup moves on by 1/rounds of the range's channel
// panels, so that it meets the narrower and the wider tiles like in the plain order.
// stream_tile_reference spells this out with plain divisions (host: tests and finish_stream_plan);
// stream_tile is the same function on the plan's prepared values, for host and device.
inline bool stream_range_blocked(const StreamPlan& p, int first, int count, int per_xcd) {
    const int rounds = (count + per_xcd - 1) / per_xcd;
    return rounds > 1 && first % p.tiles_m == 0 && count % p.tiles_m == 0 && count == rounds * per_xcd &&
           p.tiles_m % rounds == 0 && (count / p.tiles_m) % rounds == 0;
}
inline bool stream_tile_reference(const StreamPlan& p, int block, int k, int* nt, int* m) {
    const int xcd = block % kStreamXcds, wg = block / kStreamXcds, per_xcd = p.grid / kStreamXcds;
    const int total = p.tiles_m * p.tn;
    const int tq = total / kStreamXcds, tr = total % kStreamXcds;
    const int first = (xcd < tr) ? xcd * (tq + 1) : tr * (tq + 1) + (xcd - tr) * tq;
    const int count = tq + (xcd < tr ? 1 : 0);
    const int local = wg + k * per_xcd;
    if (k < 0 || local >= count) return false;
    if (stream_range_blocked(p, first, count, per_xcd)) {
        const int rounds = (count + per_xcd - 1) / per_xcd;
        const int m_per_round = p.tiles_m / rounds, panels = count / p.tiles_m;
        *nt = first / p.tiles_m + (wg / m_per_round + k * (panels / rounds)) % panels;
        *m = k * m_per_round + wg % m_per_round;
    } else {
        *nt = (first + local) / p.tiles_m;
        *m = (first + local) % p.tiles_m;
    }
    return true;
}
// fills the derived fields; false if a quantity leaves the range of stream_div
inline bool finish_stream_plan(StreamPlan* p) {
    const int per_xcd = p->grid / kStreamXcds;
    const long total = (long)p->tiles_m * p->tn;
    if (per_xcd < 1 || per_xcd >= kStreamMagicRange || total >= kStreamMagicRange / 2 ||
        (long)p->tn * p->tn >= kStreamMagicRange)
        return false;
    p->per_xcd = per_xcd;
    p->tq = (int)(total / kStreamXcds);
    p->tr = (int)(total % kStreamXcds);
    p->blocked_mask = 0;
    for (int c = 0; c < 2; ++c) { p->mpr[c] = p->panels[c] = p->inc[c] = 1; }
    for (int xcd = 0; xcd < kStreamXcds; ++xcd) {
        const int c = xcd < p->tr ? 0 : 1;
        const int first = c == 0 ? xcd * (p->tq + 1) : p->tr * (p->tq + 1) + (xcd - p->tr) * p->tq;
        const int count = p->tq + (c == 0 ? 1 : 0);
        if (count < 1 || !stream_range_blocked(*p, first, count, per_xcd)) continue;
        const int rounds = (count + per_xcd - 1) / per_xcd;
        p->blocked_mask |= 1 << xcd;
        p->mpr[c] = p->tiles_m / rounds;
        p->panels[c] = count / p->tiles_m;
        p->inc[c] = p->panels[c] / rounds;
    }
    p->mg_tiles_m = stream_magic(p->tiles_m);
    p->mg_tn = stream_magic(p->tn);
    for (int c = 0; c < 2; ++c) { p->mg_mpr[c] = stream_magic(p->mpr[c]); p->mg_panels[c] = stream_magic(p->panels[c]); }
    return true;
}
__host__ __device__ inline bool stream_tile(const StreamPlan& p, int block, int k, int* nt, int* m) {
    const int xcd = block % kStreamXcds, wg = block / kStreamXcds;
    const bool lo = xcd < p.tr;
    const int first = lo ? xcd * (p.tq + 1) : p.tr * (p.tq + 1) + (xcd - p.tr) * p.tq;
    const int count = p.tq + (lo ? 1 : 0);
    const int local = wg + k * p.per_xcd;
    if (k < 0 || local >= count) return false;
    if ((p.blocked_mask >> xcd) & 1) {
        const int mpr = lo ? p.mpr[0] : p.mpr[1], panels = lo ? p.panels[0] : p.panels[1], inc = lo ? p.inc[0] : p.inc[1];
        const int q = stream_div(wg, lo ? p.mg_mpr[0] : p.mg_mpr[1]);
        const int x = q + k * inc;                                     // < 2 * panels
        *nt = stream_div(first, p.mg_tiles_m) + x - stream_div(x, lo ? p.mg_panels[0] : p.mg_panels[1]) * panels;
        *m = k * mpr + wg - q * mpr;
    } else {
        const int idx = first + local, q = stream_div(idx, p.mg_tiles_m);
        *nt = q;
        *m = idx - q * p.tiles_m;
    }
    return true;
}
// first channel block and width (in 32-channel blocks) of channel panel nt
__host__ __device__ inline void stream_panel(const StreamPlan& p, int nt, int* block0, int* width) {
    const int lo = stream_div(nt * p.rem, p.mg_tn), hi = stream_div((nt + 1) * p.rem, p.mg_tn);   // x / p.tn
    *block0 = nt * p.base + lo;
    *width = p.base + hi - lo;
}

hipError_t launch_quantize(const QuantizeArgs& a, hipStream_t stream);
hipError_t launch_gemm(const GemmArgs& a, hipStream_t stream);
hipError_t launch_gemm_tiles(const GemmArgs& a, hipStream_t stream);
// equal operand widths, 256 x 128 tiles: the per-tile kernel on 16 x 16 matrix instructions (quik_gemm_tiles16.hip)
hipError_t launch_gemm_tiles16(const GemmArgs& a, hipStream_t stream);
hipError_t launch_weight_reduce(const WeightReduceArgs& a, hipStream_t stream);
bool plan_gemm_stream(int T, int N, int K_b, int cus, StreamPlan* p);
int choose_gemm_stream(int T, int N, int K_b, int cus, StreamPlan* p);   // 0 cannot, 1 chosen, 2 possible but not chosen
void set_gemm_path(int mode);                                           // test hook: 0 automatic, 1 persistent wherever possible, 2 per-tile
hipError_t launch_gemm_stream(const GemmArgs& a, const StreamPlan& p, hipStream_t stream);
// FP6 path (quik_gemm_fp6.hip): xq / w_q of GemmArgs are panel buffers [stage][row][48 bytes]; ldq / ldw unused
hipError_t launch_gemm_fp6(const GemmArgs& a, hipStream_t stream);
hipError_t launch_weight_pack_fp6(const void* w_q, int ldw, int N, int K_b, void* w6, hipStream_t stream);
// 2:4-sparse path (quik_gemm_sp24.hip): xq = activations [stage][T][32 bytes], w_q = weights
// [stage][N][32 bytes] (quik_sp24_device.h); ldq / ldw unused
hipError_t launch_gemm_sp24(const GemmArgs& a, hipStream_t stream);
hipError_t launch_weight_pack_sp24(const void* w_q, int ldw, int N, int K_b, void* w24, int* violations,
                                   hipStream_t stream);

// measurement probes (quik_probe.hip)
hipError_t launch_mfma_probe(int workgroups, int iters, int* sink, hipStream_t stream);
hipError_t launch_copy_probe(const void* src, void* dst, size_t bytes, hipStream_t stream);
hipError_t launch_mix_probe(int mix, int workgroups, int iters, int* sink, const void* src, size_t src_bytes,
                            unsigned long long* clocks, hipStream_t stream);

// unfused stages (fusion ablation)
hipError_t launch_unfused_quantize(const QuantizeArgs& a, void* x_base, int ldb, float* row_min,
                                   float* row_max, hipStream_t stream);
hipError_t launch_dequant_add(const GemmArgs& a, const int32_t* acc, int ldacc, const void* result_fp,
                              int ldr, hipStream_t stream);

}  // namespace quik
