// C ABI of the library: argument validation and kernel dispatch.  See include/quik.h
// for the contract of every entry point.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>
#include <vector>

#include "quik.h"
#include "quik_kernels.h"

namespace {

constexpr int kMaxK = 32768;
constexpr int kMaxKb = 131072;

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t up256(size_t v) { return (v + 255u) & ~size_t(255); }

struct WorkspaceLayout {
    size_t xq, scale, zero, code_sum, x_out, total;
    int ldq;
};

bool workspace_layout(int T, int K, int n_out, int bits, WorkspaceLayout* w) {
    if (T <= 0 || K <= 0 || n_out < 0 || n_out >= K || (bits != 4 && bits != 8)) return false;
    int ldq = quik_packed_row_bytes(K - n_out, bits);
    if (ldq <= 0) return false;
    w->ldq = ldq;
    w->xq = 0;
    w->scale = up256((size_t)T * ldq);
    w->zero = w->scale + up256((size_t)T * sizeof(float));
    w->code_sum = w->zero + up256((size_t)T * sizeof(float));
    w->x_out = w->code_sum + up256((size_t)T * sizeof(int32_t));
    w->total = w->x_out + up256((size_t)T * (n_out ? n_out : 1) * 2);
    return true;
}

// the side data of the 4-bit path inside the buffers the ABI calls `workspace` and `w_reduced`
inline size_t side_bytes(int T, int bits) { return bits == 4 ? (size_t)T * sizeof(int32_t) : 4; }
inline const int32_t* w_side(const float* w_reduced, int N) {
    return reinterpret_cast<const int32_t*>(w_reduced + N);
}

int check_quantize(const void* x, int T, int K, int ldx, const int32_t* idx, int n_out, int bits,
                   void* xq, int ldq, float* scale, float* zero, void* x_out, int ldo) {
    if (bits != 4 && bits != 8) return QUIK_EINVAL;
    if (T <= 0 || K <= 0 || n_out < 0 || n_out >= K || ldx < K) return QUIK_EINVAL;
    const int K_b = K - n_out;
    if ((K_b * bits) % 8) return QUIK_EINVAL;
    if (ldq < K_b * bits / 8) return QUIK_EINVAL;
    if (n_out > 0 && ldo < n_out) return QUIK_EINVAL;
    if (!x || !xq || !scale || !zero) return QUIK_ENULL;
    if (n_out > 0 && (!idx || !x_out)) return QUIK_ENULL;
    if (K > kMaxK) return QUIK_EUNSUPPORTED;
    if (K % 8 || n_out % 8) return QUIK_EUNSUPPORTED;
    if (ldx % 8 || ldq % 16 || (n_out > 0 && ldo % 8)) return QUIK_EALIGN;
    if (!aligned16(x) || !aligned16(xq) || (n_out > 0 && !aligned16(x_out))) return QUIK_EALIGN;
    if ((reinterpret_cast<uintptr_t>(scale) & 3u) || (reinterpret_cast<uintptr_t>(zero) & 3u))
        return QUIK_EALIGN;
    return QUIK_OK;
}

int check_gemm(const void* xq, int ldq, const void* x_out, int ldo, int T, int K_b, int n_out,
               int bits, const void* w_q, int ldw, const void* w_out, int ldwo, int N, int w_bits = 0) {
    if (bits != 4 && bits != 8) return QUIK_EINVAL;
    if (w_bits == 0) w_bits = bits;
    if (w_bits != bits && !(bits == 8 && w_bits == 4)) return QUIK_EINVAL;
    if (T <= 0 || N <= 0 || K_b <= 0 || n_out < 0) return QUIK_EINVAL;
    if ((K_b * bits) % 8 || (K_b * w_bits) % 8) return QUIK_EINVAL;
    if (ldq < K_b * bits / 8 || ldw < K_b * w_bits / 8) return QUIK_EINVAL;
    if (n_out > 0 && (ldo < n_out || ldwo < n_out)) return QUIK_EINVAL;
    if (!xq || !w_q) return QUIK_ENULL;
    if (n_out > 0 && (!x_out || !w_out)) return QUIK_ENULL;
    if (K_b >= kMaxKb) return QUIK_EUNSUPPORTED;
    if (n_out % 8) return QUIK_EUNSUPPORTED;
    if (ldq % 16 || ldw % 16) return QUIK_EALIGN;
    if (n_out > 0 && (ldo % 8 || ldwo % 8)) return QUIK_EALIGN;
    if (!aligned16(xq) || !aligned16(w_q)) return QUIK_EALIGN;
    if (n_out > 0 && (!aligned16(x_out) || !aligned16(w_out))) return QUIK_EALIGN;
    return QUIK_OK;
}

}  // namespace

extern "C" {

int quik_version(void) { return 1; }

const char* quik_status_string(int status) {
    switch (status) {
        case QUIK_OK: return "QUIK_OK";
        case QUIK_EINVAL: return "QUIK_EINVAL: size or flag out of range";
        case QUIK_ENULL: return "QUIK_ENULL: required pointer is NULL";
        case QUIK_EALIGN: return "QUIK_EALIGN: pointer or leading dimension misaligned";
        case QUIK_EUNSUPPORTED: return "QUIK_EUNSUPPORTED: shape outside the built limits";
        case QUIK_EWORKSPACE: return "QUIK_EWORKSPACE: workspace too small";
        case QUIK_ELAUNCH: return "QUIK_ELAUNCH: HIP launch failed";
        default: return "unknown quik status";
    }
}

int quik_packed_row_bytes(int K_b, int bits) {
    if (K_b <= 0 || (bits != 4 && bits != 8) || K_b >= kMaxKb) return 0;
    if ((K_b * bits) % 8) return 0;
    return ((K_b * bits / 8) + 15) & ~15;
}

size_t quik_workspace_bytes(int T, int K, int N, int n_out, int bits) {
    (void)N;
    WorkspaceLayout w;
    if (!workspace_layout(T, K, n_out, bits, &w)) return 0;
    return w.total;
}

int quik_workspace_regions(int T, int K, int N, int n_out, int bits, size_t* offsets, int* ldq) {
    (void)N;
    WorkspaceLayout w;
    if (!workspace_layout(T, K, n_out, bits, &w)) return QUIK_EINVAL;
    if (!offsets || !ldq) return QUIK_ENULL;
    offsets[0] = w.xq; offsets[1] = w.scale; offsets[2] = w.zero; offsets[3] = w.x_out;
    *ldq = w.ldq;
    return QUIK_OK;
}

int quik_debug_gemm_plan(int T, int N, int K_b, int cus, int* plan) {
    if (T <= 0 || N <= 0 || K_b <= 0 || (K_b & 1) || K_b >= kMaxKb || cus <= 0) return QUIK_EINVAL;
    if (!plan) return QUIK_ENULL;
    quik::StreamPlan p;
    const int c = quik::choose_gemm_stream(T, N, K_b, cus, &p);
    if (c == 0) return 0;
    plan[0] = p.tiles_m; plan[1] = p.tn; plan[2] = p.base; plan[3] = p.rem; plan[4] = p.grid;
    return c;
}

int quik_debug_gemm_tile(int T, int N, int K_b, int cus, int workgroup, int k, int* tile) {
    if (T <= 0 || N <= 0 || K_b <= 0 || (K_b & 1) || K_b >= kMaxKb || cus <= 0 || workgroup < 0 || k < 0) return QUIK_EINVAL;
    if (!tile) return QUIK_ENULL;
    quik::StreamPlan p;
    if (quik::choose_gemm_stream(T, N, K_b, cus, &p) == 0 || workgroup >= p.grid) return QUIK_EINVAL;
    int nt, m, b0, w, nt_ref = -1, m_ref = -1;
    const bool any = quik::stream_tile(p, workgroup, k, &nt, &m);
    // the walk on the plan's prepared divisors against its definition with plain divisions
    if (any != quik::stream_tile_reference(p, workgroup, k, &nt_ref, &m_ref) || (any && (nt != nt_ref || m != m_ref)))
        return QUIK_EUNSUPPORTED;
    if (!any) return 0;
    quik::stream_panel(p, nt, &b0, &w);
    tile[0] = m * quik::kStreamRows;
    tile[1] = b0 * 32;
    tile[2] = (w * 32 < N - b0 * 32) ? w * 32 : N - b0 * 32;
    return 1;
}

int quik_debug_set_gemm_path(int mode) {
    if (mode < 0 || mode > 2) return QUIK_EINVAL;
    quik::set_gemm_path(mode);
    return QUIK_OK;
}

size_t quik_quantize_workspace_bytes(int T, int bits) {
    if (T <= 0 || (bits != 4 && bits != 8)) return 0;
    return side_bytes(T, bits);
}

size_t quik_w_reduced_bytes(int N, int bits) {
    if (N <= 0 || (bits != 4 && bits != 8)) return 0;
    return (size_t)N * (bits == 4 ? 8 : 4);
}

int quik_quantize(const void* x, int T, int K, int ldx, const int32_t* outlier_idx, int n_out,
                  int bits, void* xq, int ldq, float* scale, float* zero, void* x_out, int ldo,
                  void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_quantize(x, T, K, ldx, outlier_idx, n_out, bits, xq, ldq, scale, zero, x_out, ldo);
    if (rc != QUIK_OK) return rc;
    if (reinterpret_cast<uintptr_t>(workspace) & 3u) return QUIK_EALIGN;
    if (workspace && workspace_bytes < side_bytes(T, bits)) return QUIK_EWORKSPACE;
    int32_t* code_sum = bits == 4 ? static_cast<int32_t*>(workspace) : nullptr;
    quik::QuantizeArgs a{x, T, K, ldx, outlier_idx, n_out, bits, xq, ldq, scale, zero, x_out, ldo, code_sum};
    return quik::launch_quantize(a, static_cast<hipStream_t>(stream)) == hipSuccess ? QUIK_OK
                                                                                   : QUIK_ELAUNCH;
}

int quik_weight_reduce(const void* w_q, int ldw, const void* w_scale, int N, int K_b, int bits,
                       float* w_reduced, void* stream) {
    if (bits != 4 && bits != 8) return QUIK_EINVAL;
    if (N <= 0 || K_b <= 0 || (K_b * bits) % 8 || ldw < K_b * bits / 8) return QUIK_EINVAL;
    if (!w_q || !w_scale || !w_reduced) return QUIK_ENULL;
    if (K_b >= kMaxKb) return QUIK_EUNSUPPORTED;
    if (reinterpret_cast<uintptr_t>(w_reduced) & 3u) return QUIK_EALIGN;
    int32_t* w_code_sum = bits == 4 ? reinterpret_cast<int32_t*>(w_reduced + N) : nullptr;
    quik::WeightReduceArgs a{w_q, ldw, w_scale, N, K_b, bits, w_reduced, w_code_sum};
    return quik::launch_weight_reduce(a, static_cast<hipStream_t>(stream)) == hipSuccess
               ? QUIK_OK
               : QUIK_ELAUNCH;
}

int quik_gemm_dequant(const void* xq, int ldq, const float* scale, const float* zero,
                      const void* x_out, int ldo, int T, int K_b, int n_out,
                      int bits, const void* w_q, int ldw, const void* w_scale, const float* w_reduced,
                      const void* w_out, int ldwo, const void* bias, int N,
                      void* y, int ldy, const void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_gemm(xq, ldq, x_out, ldo, T, K_b, n_out, bits, w_q, ldw, w_out, ldwo, N);
    if (rc != QUIK_OK) return rc;
    if (ldy < N) return QUIK_EINVAL;
    if (!scale || !zero || !w_scale || !w_reduced || !y) return QUIK_ENULL;
    if (bits == 4 && !workspace) return QUIK_ENULL;
    if (bits == 4 && (reinterpret_cast<uintptr_t>(workspace) & 3u)) return QUIK_EALIGN;
    if (bits == 4 && workspace_bytes < side_bytes(T, bits)) return QUIK_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(y) & 1u) return QUIK_EALIGN;
    quik::GemmArgs a{};
    a.xq = xq; a.ldq = ldq; a.scale = scale; a.zero = zero; a.x_out = x_out; a.ldo = ldo;
    if (bits == 4) { a.code_sum = static_cast<const int32_t*>(workspace); a.w_code_sum = w_side(w_reduced, N); }
    a.T = T; a.K_b = K_b; a.n_out = n_out; a.bits = bits;
    a.w_q = w_q; a.ldw = ldw; a.w_scale = w_scale; a.w_reduced = w_reduced;
    a.w_out = w_out; a.ldwo = ldwo; a.bias = bias; a.N = N;
    a.y = y; a.ldy = ldy; a.acc = nullptr; a.ldacc = 0;
    return quik::launch_gemm(a, static_cast<hipStream_t>(stream)) == hipSuccess ? QUIK_OK
                                                                               : QUIK_ELAUNCH;
}

int quik_debug_int_gemm(const void* xq, int ldq, const void* w_q, int ldw, int T, int N, int K_b, int bits,
                        int32_t* acc, int ldacc, const void* workspace, size_t workspace_bytes,
                        const float* w_reduced, void* stream) {
    int rc = check_gemm(xq, ldq, nullptr, 0, T, K_b, 0, bits, w_q, ldw, nullptr, 0, N);
    if (rc != QUIK_OK) return rc;
    if (ldacc < N) return QUIK_EINVAL;
    if (!acc) return QUIK_ENULL;
    if ((workspace == nullptr) != (w_reduced == nullptr)) return QUIK_ENULL;   // both or neither
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 3u)) return QUIK_EALIGN;
    if (workspace && workspace_bytes < side_bytes(T, bits)) return QUIK_EWORKSPACE;
    quik::GemmArgs a{};
    if (bits == 4 && workspace) { a.code_sum = static_cast<const int32_t*>(workspace); a.w_code_sum = w_side(w_reduced, N); }
    a.xq = xq; a.ldq = ldq; a.T = T; a.K_b = K_b; a.n_out = 0; a.bits = bits;
    a.w_q = w_q; a.ldw = ldw; a.N = N; a.y = nullptr; a.acc = acc; a.ldacc = ldacc;
    return quik::launch_gemm(a, static_cast<hipStream_t>(stream)) == hipSuccess ? QUIK_OK
                                                                               : QUIK_ELAUNCH;
}

int quik_int_gemm(const void* xq, int ldq, const void* w_q, int ldw, int T, int N, int K_b, int bits,
                  int32_t* acc, int ldacc, const void* workspace, size_t workspace_bytes,
                  const float* w_reduced, void* stream) {
    return quik_debug_int_gemm(xq, ldq, w_q, ldw, T, N, K_b, bits, acc, ldacc, workspace, workspace_bytes,
                               w_reduced, stream);
}

int quik_linear(const void* x, int T, int K, int ldx, const int32_t* outlier_idx, int n_out,
                int bits, const void* w_q, int ldw, const void* w_scale, const float* w_reduced,
                const void* w_out, int ldwo, const void* bias, int N, void* y,
                int ldy, void* workspace, size_t workspace_bytes, void* stream) {
    WorkspaceLayout w;
    if (!workspace_layout(T, K, n_out, bits, &w)) return QUIK_EINVAL;
    if (!workspace) return QUIK_ENULL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return QUIK_EALIGN;
    if (workspace_bytes < w.total) return QUIK_EWORKSPACE;
    uint8_t* base = static_cast<uint8_t*>(workspace);
    void* xq = base + w.xq;
    float* scale = reinterpret_cast<float*>(base + w.scale);
    float* zero = reinterpret_cast<float*>(base + w.zero);
    int32_t* code_sum = reinterpret_cast<int32_t*>(base + w.code_sum);
    void* x_out = base + w.x_out;
    const int K_b = K - n_out;
    // validate both stages before anything is enqueued
    int rc = check_quantize(x, T, K, ldx, outlier_idx, n_out, bits, xq, w.ldq, scale, zero, x_out, n_out);
    if (rc != QUIK_OK) return rc;
    rc = check_gemm(xq, w.ldq, x_out, n_out, T, K_b, n_out, bits, w_q, ldw, w_out, ldwo, N);
    if (rc != QUIK_OK) return rc;
    if (ldy < N) return QUIK_EINVAL;
    if (!w_scale || !w_reduced || !y) return QUIK_ENULL;
    if (reinterpret_cast<uintptr_t>(y) & 1u) return QUIK_EALIGN;
    const size_t side = side_bytes(T, bits);
    rc = quik_quantize(x, T, K, ldx, outlier_idx, n_out, bits, xq, w.ldq, scale, zero, x_out, n_out,
                       code_sum, side, stream);
    if (rc != QUIK_OK) return rc;
    return quik_gemm_dequant(xq, w.ldq, scale, zero, x_out, n_out, T, K_b, n_out, bits, w_q, ldw, w_scale,
                             w_reduced, w_out, ldwo, bias, N, y, ldy, code_sum, side, stream);
}

// ---- quik_linear for callers that cannot allocate: the workspace is a static device array

namespace {
// The intermediate results of one layer (packed activations, scale, zero, side data, outlier
// block).  Every GPU the library runs on holds its own copy of this array, at its own address, until the
// process ends; the name below is only a host-side handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[QUIK_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up once per device).
int scratch_of_current_device(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return QUIK_ELAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return QUIK_ELAUNCH;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return QUIK_OK;
}
}  // namespace

int quik_linear_noalloc(const void* x, int T, int K, int ldx, const int32_t* outlier_idx, int n_out, int bits,
                        const void* w_q, int ldw, const void* w_scale, const float* w_reduced,
                        const void* w_out, int ldwo, const void* bias, int N, void* y, int ldy,
                        void* stream) {
    WorkspaceLayout w;
    if (!workspace_layout(T, K, n_out, bits, &w)) return QUIK_EINVAL;
    if (w.total > (size_t)QUIK_NOALLOC_SCRATCH_BYTES) return QUIK_EWORKSPACE;
    void* ws = nullptr;
    int rc = scratch_of_current_device(&ws);
    if (rc != QUIK_OK) return rc;
    // quik_quantize writes every byte of the regions quik_gemm_dequant reads (the zero tail of the
    // packed rows included), so what an earlier call left in the array does not matter
    return quik_linear(x, T, K, ldx, outlier_idx, n_out, bits, w_q, ldw, w_scale, w_reduced, w_out, ldwo, bias,
                       N, y, ldy, ws, (size_t)QUIK_NOALLOC_SCRATCH_BYTES, stream);
}

// ---- 4-bit weights under 8-bit activations (the W4A8 rows of the paper's precision ablation)

int quik_gemm_dequant_w4a8(const void* xq, int ldq, const float* scale, const float* zero,
                           const void* x_out, int ldo, int T, int K_b, int n_out, const void* w_q,
                           int ldw, const void* w_scale, const float* w_reduced, const void* w_out,
                           int ldwo, const void* bias, int N, void* y, int ldy, void* stream) {
    int rc = check_gemm(xq, ldq, x_out, ldo, T, K_b, n_out, 8, w_q, ldw, w_out, ldwo, N, 4);
    if (rc != QUIK_OK) return rc;
    if (ldy < N) return QUIK_EINVAL;
    if (!scale || !zero || !w_scale || !w_reduced || !y) return QUIK_ENULL;
    if (reinterpret_cast<uintptr_t>(y) & 1u) return QUIK_EALIGN;
    quik::GemmArgs a{};
    a.xq = xq; a.ldq = ldq; a.scale = scale; a.zero = zero; a.x_out = x_out; a.ldo = ldo;
    a.T = T; a.K_b = K_b; a.n_out = n_out; a.bits = 8; a.w_bits = 4;
    a.w_q = w_q; a.ldw = ldw; a.w_scale = w_scale; a.w_reduced = w_reduced;
    a.w_out = w_out; a.ldwo = ldwo; a.bias = bias; a.N = N;
    a.y = y; a.ldy = ldy; a.acc = nullptr; a.ldacc = 0;
    return quik::launch_gemm(a, static_cast<hipStream_t>(stream)) == hipSuccess ? QUIK_OK
                                                                               : QUIK_ELAUNCH;
}

int quik_int_gemm_w4a8(const void* xq, int ldq, const void* w_q, int ldw, int T, int N, int K_b,
                       int32_t* acc, int ldacc, void* stream) {
    int rc = check_gemm(xq, ldq, nullptr, 0, T, K_b, 0, 8, w_q, ldw, nullptr, 0, N, 4);
    if (rc != QUIK_OK) return rc;
    if (ldacc < N) return QUIK_EINVAL;
    if (!acc) return QUIK_ENULL;
    quik::GemmArgs a{};
    a.xq = xq; a.ldq = ldq; a.T = T; a.K_b = K_b; a.n_out = 0; a.bits = 8; a.w_bits = 4;
    a.w_q = w_q; a.ldw = ldw; a.N = N; a.y = nullptr; a.acc = acc; a.ldacc = ldacc;
    return quik::launch_gemm(a, static_cast<hipStream_t>(stream)) == hipSuccess ? QUIK_OK
                                                                               : QUIK_ELAUNCH;
}

int quik_linear_w4a8(const void* x, int T, int K, int ldx, const int32_t* outlier_idx, int n_out,
                     const void* w_q, int ldw, const void* w_scale, const float* w_reduced,
                     const void* w_out, int ldwo, const void* bias, int N, void* y, int ldy,
                     void* workspace, size_t workspace_bytes, void* stream) {
    WorkspaceLayout w;
    if (!workspace_layout(T, K, n_out, 8, &w)) return QUIK_EINVAL;
    if (!workspace) return QUIK_ENULL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return QUIK_EALIGN;
    if (workspace_bytes < w.total) return QUIK_EWORKSPACE;
    uint8_t* base = static_cast<uint8_t*>(workspace);
    void* xq = base + w.xq;
    float* scale = reinterpret_cast<float*>(base + w.scale);
    float* zero = reinterpret_cast<float*>(base + w.zero);
    void* x_out = base + w.x_out;
    const int K_b = K - n_out;
    int rc = check_quantize(x, T, K, ldx, outlier_idx, n_out, 8, xq, w.ldq, scale, zero, x_out, n_out);
    if (rc != QUIK_OK) return rc;
    rc = check_gemm(xq, w.ldq, x_out, n_out, T, K_b, n_out, 8, w_q, ldw, w_out, ldwo, N, 4);
    if (rc != QUIK_OK) return rc;
    if (ldy < N) return QUIK_EINVAL;
    if (!w_scale || !w_reduced || !y) return QUIK_ENULL;
    if (reinterpret_cast<uintptr_t>(y) & 1u) return QUIK_EALIGN;
    rc = quik_quantize(x, T, K, ldx, outlier_idx, n_out, 8, xq, w.ldq, scale, zero, x_out, n_out, nullptr, 0,
                       stream);
    if (rc != QUIK_OK) return rc;
    return quik_gemm_dequant_w4a8(xq, w.ldq, scale, zero, x_out, n_out, T, K_b, n_out, w_q, ldw, w_scale,
                                  w_reduced, w_out, ldwo, bias, N, y, ldy, stream);
}

namespace {
struct AblationLayout {
    WorkspaceLayout base;
    size_t x_base, row_min, row_max, acc, result_fp, total;
    int ldb;
};
bool ablation_layout(int T, int K, int N, int n_out, int bits, AblationLayout* w) {
    if (N <= 0 || !workspace_layout(T, K, n_out, bits, &w->base)) return false;
    const int K_b = K - n_out;
    w->ldb = (K_b + 7) & ~7;
    w->x_base = w->base.total;
    w->row_min = w->x_base + up256((size_t)T * w->ldb * 2);
    w->row_max = w->row_min + up256((size_t)T * sizeof(float));
    w->acc = w->row_max + up256((size_t)T * sizeof(float));
    w->result_fp = w->acc + up256((size_t)T * N * sizeof(int32_t));
    w->total = w->result_fp + up256((size_t)T * N * sizeof(float));
    return true;
}
}  // namespace

size_t quik_ablation_workspace_bytes(int T, int K, int N, int n_out, int bits) {
    AblationLayout w;
    if (!ablation_layout(T, K, N, n_out, bits, &w)) return 0;
    return w.total;
}

int quik_linear_ablation(int version, const void* x, int T, int K, int ldx, const int32_t* outlier_idx,
                         int n_out, int bits, const void* w_q, int ldw, const void* w_scale,
                         const float* w_reduced, const void* w_out, int ldwo,
                         const void* bias, int N, void* y, int ldy, void* workspace,
                         size_t workspace_bytes, void* stream) {
    if (version == 3)
        return quik_linear(x, T, K, ldx, outlier_idx, n_out, bits, w_q, ldw, w_scale, w_reduced,
                           w_out, ldwo, bias, N, y, ldy, workspace, workspace_bytes, stream);
    if (version != 1 && version != 2) return QUIK_EINVAL;
    AblationLayout w;
    if (!ablation_layout(T, K, N, n_out, bits, &w)) return QUIK_EINVAL;
    if (!workspace) return QUIK_ENULL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return QUIK_EALIGN;
    if (workspace_bytes < w.total) return QUIK_EWORKSPACE;
    uint8_t* base = static_cast<uint8_t*>(workspace);
    void* xq = base + w.base.xq;
    float* scale = reinterpret_cast<float*>(base + w.base.scale);
    float* zero = reinterpret_cast<float*>(base + w.base.zero);
    int32_t* code_sum = reinterpret_cast<int32_t*>(base + w.base.code_sum);
    void* x_out = base + w.base.x_out;
    void* x_base = base + w.x_base;
    float* row_min = reinterpret_cast<float*>(base + w.row_min);
    float* row_max = reinterpret_cast<float*>(base + w.row_max);
    int32_t* acc = reinterpret_cast<int32_t*>(base + w.acc);
    void* result_fp = base + w.result_fp;
    const int K_b = K - n_out, ldq = w.base.ldq;
    int rc = check_quantize(x, T, K, ldx, outlier_idx, n_out, bits, xq, ldq, scale, zero, x_out, n_out);
    if (rc != QUIK_OK) return rc;
    rc = check_gemm(xq, ldq, x_out, n_out, T, K_b, n_out, bits, w_q, ldw, w_out, ldwo, N);
    if (rc != QUIK_OK) return rc;
    if (ldy < N) return QUIK_EINVAL;
    if (!w_scale || !w_reduced || !y) return QUIK_ENULL;
    if (reinterpret_cast<uintptr_t>(y) & 1u) return QUIK_EALIGN;
    const int32_t* w_code_sum = bits == 4 ? w_side(w_reduced, N) : nullptr;
    hipStream_t st = static_cast<hipStream_t>(stream);
    quik::QuantizeArgs qa{x, T, K, ldx, outlier_idx, n_out, bits, xq, ldq, scale, zero, x_out, n_out, code_sum};
    if (version == 1) {
        if (quik::launch_unfused_quantize(qa, x_base, w.ldb, row_min, row_max, st) != hipSuccess)
            return QUIK_ELAUNCH;
    } else {
        if (quik::launch_quantize(qa, st) != hipSuccess) return QUIK_ELAUNCH;
    }
    quik::GemmArgs g{};
    g.xq = xq; g.ldq = ldq; g.scale = scale; g.zero = zero; g.x_out = x_out; g.ldo = n_out;
    g.code_sum = code_sum; g.w_code_sum = w_code_sum;
    g.T = T; g.K_b = K_b; g.n_out = n_out; g.bits = bits;
    g.w_q = w_q; g.ldw = ldw; g.w_scale = w_scale; g.w_reduced = w_reduced;
    g.w_out = w_out; g.ldwo = ldwo; g.bias = nullptr; g.N = N;
    // INTmatmul alone: accumulators go to memory
    g.y = nullptr; g.acc = acc; g.ldacc = N; g.n_out = 0;
    if (quik::launch_gemm(g, st) != hipSuccess) return QUIK_ELAUNCH;
    // FPmatmul alone: fp16 result goes to memory
    const void* rfp = nullptr;
    if (n_out > 0) {
        g.n_out = n_out; g.y = result_fp; g.ldy = N; g.acc = nullptr; g.fp_only = 1;
        if (quik::launch_gemm(g, st) != hipSuccess) return QUIK_ELAUNCH;
        rfp = result_fp;
    }
    // Dequantization + final add as a separate elementwise pass
    g.fp_only = 0; g.y = y; g.ldy = ldy; g.bias = bias;
    return quik::launch_dequant_add(g, acc, N, rfp, N, st) == hipSuccess ? QUIK_OK : QUIK_ELAUNCH;
}

// ---- FP6 (E3M2) path of the 4-bit layer -----------------------------------------------------

int quik_fp6_row_bytes(int K_b) {
    if (K_b <= 0 || K_b >= kMaxKb) return 0;
    return 48 * ((K_b + 63) / 64);
}

size_t quik_workspace_bytes_fp6(int T, int K, int N, int n_out) {
    (void)N;
    if (T <= 0 || K <= 0 || n_out < 0 || n_out >= K) return 0;
    const int rb = quik_fp6_row_bytes(K - n_out);
    if (rb <= 0) return 0;
    return up256((size_t)T * rb) + 2 * up256((size_t)T * sizeof(float)) + up256((size_t)T * (n_out ? n_out : 1) * 2);
}

int quik_weight_pack_fp6(const void* w_q, int ldw, int N, int K_b, void* w6, void* stream) {
    if (N <= 0 || K_b <= 0 || K_b % 2 || ldw < K_b / 2) return QUIK_EINVAL;
    if (!w_q || !w6) return QUIK_ENULL;
    if (K_b >= kMaxKb) return QUIK_EUNSUPPORTED;
    if (!aligned16(w6)) return QUIK_EALIGN;
    return quik::launch_weight_pack_fp6(w_q, ldw, N, K_b, w6, static_cast<hipStream_t>(stream)) == hipSuccess
               ? QUIK_OK
               : QUIK_ELAUNCH;
}

int quik_quantize_fp6(const void* x, int T, int K, int ldx, const int32_t* outlier_idx, int n_out, void* xq6,
                      float* scale, float* zero, void* x_out, int ldo, void* stream) {
    // same argument rules as the 4-bit integer form, except for the layout of the packed output
    int rc = check_quantize(x, T, K, ldx, outlier_idx, n_out, 4, xq6, 16 * ((K + 15) / 16), scale, zero, x_out, ldo);
    if (rc != QUIK_OK) return rc;
    if (K > 16384) return QUIK_EUNSUPPORTED;
    quik::QuantizeArgs a{x, T, K, ldx, outlier_idx, n_out, 4, xq6, quik_fp6_row_bytes(K - n_out), scale, zero,
                         x_out, ldo, nullptr, 1};
    return quik::launch_quantize(a, static_cast<hipStream_t>(stream)) == hipSuccess ? QUIK_OK : QUIK_ELAUNCH;
}

namespace {
int check_gemm_fp6(const void* xq6, const void* x_out, int ldo, int T, int K_b, int n_out, const void* w6,
                   const void* w_out, int ldwo, int N) {
    if (T <= 0 || N <= 0 || K_b <= 0 || n_out < 0) return QUIK_EINVAL;
    if (K_b >= kMaxKb) return QUIK_EUNSUPPORTED;
    // a stage of all rows must stay below 4 GB (32-bit offsets inside the copy descriptors)
    if ((uint64_t)quik_fp6_row_bytes(K_b) * (uint64_t)(T > N ? T : N) >= (1ull << 32)) return QUIK_EUNSUPPORTED;
    if (n_out > 0 && (ldo < n_out || ldwo < n_out)) return QUIK_EINVAL;
    if (!xq6 || !w6) return QUIK_ENULL;
    if (n_out > 0 && (!x_out || !w_out)) return QUIK_ENULL;
    if (n_out % 8) return QUIK_EUNSUPPORTED;
    if (n_out > 0 && (ldo % 8 || ldwo % 8)) return QUIK_EALIGN;
    if (!aligned16(xq6) || !aligned16(w6)) return QUIK_EALIGN;
    if (n_out > 0 && (!aligned16(x_out) || !aligned16(w_out))) return QUIK_EALIGN;
    return QUIK_OK;
}
}  // namespace

int quik_gemm_dequant_fp6(const void* xq6, const float* scale, const float* zero, const void* x_out, int ldo, int T,
                          int K_b, int n_out, const void* w6, const void* w_scale, const float* w_reduced,
                          const void* w_out, int ldwo, const void* bias, int N, void* y, int ldy, void* stream) {
    int rc = check_gemm_fp6(xq6, x_out, ldo, T, K_b, n_out, w6, w_out, ldwo, N);
    if (rc != QUIK_OK) return rc;
    if (ldy < N) return QUIK_EINVAL;
    if (!scale || !zero || !w_scale || !w_reduced || !y) return QUIK_ENULL;
    if (reinterpret_cast<uintptr_t>(y) & 1u) return QUIK_EALIGN;
    quik::GemmArgs a{};
    a.xq = xq6; a.scale = scale; a.zero = zero; a.x_out = x_out; a.ldo = ldo;
    a.T = T; a.K_b = K_b; a.n_out = n_out; a.bits = 4;
    a.w_q = w6; a.w_scale = w_scale; a.w_reduced = w_reduced;
    a.w_out = w_out; a.ldwo = ldwo; a.bias = bias; a.N = N;
    a.y = y; a.ldy = ldy; a.acc = nullptr; a.ldacc = 0;
    return quik::launch_gemm_fp6(a, static_cast<hipStream_t>(stream)) == hipSuccess ? QUIK_OK : QUIK_ELAUNCH;
}

int quik_int_gemm_fp6(const void* xq6, const void* w6, int T, int N, int K_b, int32_t* acc, int ldacc,
                      void* stream) {
    int rc = check_gemm_fp6(xq6, nullptr, 0, T, K_b, 0, w6, nullptr, 0, N);
    if (rc != QUIK_OK) return rc;
    if (ldacc < N) return QUIK_EINVAL;
    if (!acc) return QUIK_ENULL;
    quik::GemmArgs a{};
    a.xq = xq6; a.T = T; a.K_b = K_b; a.n_out = 0; a.bits = 4;
    a.w_q = w6; a.N = N; a.y = nullptr; a.acc = acc; a.ldacc = ldacc;
    return quik::launch_gemm_fp6(a, static_cast<hipStream_t>(stream)) == hipSuccess ? QUIK_OK : QUIK_ELAUNCH;
}

int quik_linear_fp6(const void* x, int T, int K, int ldx, const int32_t* outlier_idx, int n_out, const void* w6,
                    const void* w_scale, const float* w_reduced, const void* w_out, int ldwo, const void* bias,
                    int N, void* y, int ldy, void* workspace, size_t workspace_bytes, void* stream) {
    const size_t need = quik_workspace_bytes_fp6(T, K, N, n_out);
    if (need == 0) return QUIK_EINVAL;
    if (!workspace) return QUIK_ENULL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return QUIK_EALIGN;
    if (workspace_bytes < need) return QUIK_EWORKSPACE;
    const int K_b = K - n_out, rb = quik_fp6_row_bytes(K_b);
    uint8_t* base = static_cast<uint8_t*>(workspace);
    void* xq6 = base;
    float* scale = reinterpret_cast<float*>(base + up256((size_t)T * rb));
    float* zero = reinterpret_cast<float*>(reinterpret_cast<uint8_t*>(scale) + up256((size_t)T * sizeof(float)));
    void* x_out = reinterpret_cast<uint8_t*>(zero) + up256((size_t)T * sizeof(float));
    // validate both stages before anything is enqueued
    int rc = check_quantize(x, T, K, ldx, outlier_idx, n_out, 4, xq6, 16 * ((K + 15) / 16), scale, zero, x_out, n_out);
    if (rc != QUIK_OK) return rc;
    if (K > 16384) return QUIK_EUNSUPPORTED;
    rc = check_gemm_fp6(xq6, x_out, n_out, T, K_b, n_out, w6, w_out, ldwo, N);
    if (rc != QUIK_OK) return rc;
    if (ldy < N) return QUIK_EINVAL;
    if (!w_scale || !w_reduced || !y) return QUIK_ENULL;
    if (reinterpret_cast<uintptr_t>(y) & 1u) return QUIK_EALIGN;
    rc = quik_quantize_fp6(x, T, K, ldx, outlier_idx, n_out, xq6, scale, zero, x_out, n_out, stream);
    if (rc != QUIK_OK) return rc;
    return quik_gemm_dequant_fp6(xq6, scale, zero, x_out, n_out, T, K_b, n_out, w6, w_scale, w_reduced, w_out, ldwo,
                                 bias, N, y, ldy, stream);
}

// ---- 2:4-sparse weights on the sparse int8 matrix instruction -----------------------------------

int quik_sp24_act_row_bytes(int K_b) {
    if (K_b <= 0 || K_b >= kMaxKb) return 0;
    return 32 * ((K_b + 63) / 64);
}

size_t quik_sp24_weight_bytes(int N, int K_b) {
    if (N <= 0 || K_b <= 0 || K_b >= kMaxKb) return 0;
    return (size_t)((K_b + 63) / 64) * (size_t)N * 32u;
}

size_t quik_workspace_bytes_sp24(int T, int K, int N, int n_out) {
    (void)N;
    if (T <= 0 || K <= 0 || n_out < 0 || n_out >= K) return 0;
    const int rb = quik_sp24_act_row_bytes(K - n_out);
    if (rb <= 0) return 0;
    return up256((size_t)T * rb) + 2 * up256((size_t)T * sizeof(float)) + up256((size_t)T * (n_out ? n_out : 1) * 2);
}

int quik_weight_pack_sp24(const void* w_q, int ldw, int N, int K_b, void* w24, int32_t* violations, void* stream) {
    if (N <= 0 || K_b <= 0 || K_b % 2 || ldw < K_b / 2) return QUIK_EINVAL;
    if (!w_q || !w24) return QUIK_ENULL;
    if (K_b >= kMaxKb) return QUIK_EUNSUPPORTED;
    if (!aligned16(w24)) return QUIK_EALIGN;
    if (violations && (reinterpret_cast<uintptr_t>(violations) & 3u)) return QUIK_EALIGN;
    return quik::launch_weight_pack_sp24(w_q, ldw, N, K_b, w24, violations, static_cast<hipStream_t>(stream)) ==
                   hipSuccess
               ? QUIK_OK
               : QUIK_ELAUNCH;
}

int quik_quantize_sp24(const void* x, int T, int K, int ldx, const int32_t* outlier_idx, int n_out, void* xq24,
                       float* scale, float* zero, void* x_out, int ldo, void* stream) {
    // same argument rules as the 4-bit integer form, except for the layout of the packed output
    int rc = check_quantize(x, T, K, ldx, outlier_idx, n_out, 4, xq24, 16 * ((K + 15) / 16), scale, zero, x_out, ldo);
    if (rc != QUIK_OK) return rc;
    if (K > 16384) return QUIK_EUNSUPPORTED;
    quik::QuantizeArgs a{x, T, K, ldx, outlier_idx, n_out, 4, xq24, quik_sp24_act_row_bytes(K - n_out), scale, zero,
                         x_out, ldo, nullptr, 2};
    return quik::launch_quantize(a, static_cast<hipStream_t>(stream)) == hipSuccess ? QUIK_OK : QUIK_ELAUNCH;
}

namespace {
int check_gemm_sp24(const void* xq24, const void* x_out, int ldo, int T, int K_b, int n_out, const void* w24,
                    const void* w_out, int ldwo, int N) {
    if (T <= 0 || N <= 0 || K_b <= 0 || n_out < 0) return QUIK_EINVAL;
    if (K_b >= kMaxKb) return QUIK_EUNSUPPORTED;
    // both buffers must stay below 4 GB (32-bit stage offsets inside the copy descriptors)
    if ((uint64_t)quik_sp24_act_row_bytes(K_b) * (uint64_t)T >= (1ull << 32)) return QUIK_EUNSUPPORTED;
    if ((uint64_t)quik_sp24_weight_bytes(N, K_b) >= (1ull << 32)) return QUIK_EUNSUPPORTED;
    if (n_out > 0 && (ldo < n_out || ldwo < n_out)) return QUIK_EINVAL;
    if (!xq24 || !w24) return QUIK_ENULL;
    if (n_out > 0 && (!x_out || !w_out)) return QUIK_ENULL;
    if (n_out % 8) return QUIK_EUNSUPPORTED;
    if (n_out > 0 && (ldo % 8 || ldwo % 8)) return QUIK_EALIGN;
    if (!aligned16(xq24) || !aligned16(w24)) return QUIK_EALIGN;
    if (n_out > 0 && (!aligned16(x_out) || !aligned16(w_out))) return QUIK_EALIGN;
    return QUIK_OK;
}
}  // namespace

int quik_gemm_dequant_sp24(const void* xq24, const float* scale, const float* zero, const void* x_out, int ldo, int T,
                           int K_b, int n_out, const void* w24, const void* w_scale, const float* w_reduced,
                           const void* w_out, int ldwo, const void* bias, int N, void* y, int ldy, void* stream) {
    int rc = check_gemm_sp24(xq24, x_out, ldo, T, K_b, n_out, w24, w_out, ldwo, N);
    if (rc != QUIK_OK) return rc;
    if (ldy < N) return QUIK_EINVAL;
    if (!scale || !zero || !w_scale || !w_reduced || !y) return QUIK_ENULL;
    if (reinterpret_cast<uintptr_t>(y) & 1u) return QUIK_EALIGN;
    quik::GemmArgs a{};
    a.xq = xq24; a.scale = scale; a.zero = zero; a.x_out = x_out; a.ldo = ldo;
    a.T = T; a.K_b = K_b; a.n_out = n_out; a.bits = 4;
    a.w_q = w24; a.w_scale = w_scale; a.w_reduced = w_reduced;
    a.w_out = w_out; a.ldwo = ldwo; a.bias = bias; a.N = N;
    a.y = y; a.ldy = ldy; a.acc = nullptr; a.ldacc = 0;
    return quik::launch_gemm_sp24(a, static_cast<hipStream_t>(stream)) == hipSuccess ? QUIK_OK : QUIK_ELAUNCH;
}

int quik_int_gemm_sp24(const void* xq24, const void* w24, int T, int N, int K_b, int32_t* acc, int ldacc,
                       void* stream) {
    int rc = check_gemm_sp24(xq24, nullptr, 0, T, K_b, 0, w24, nullptr, 0, N);
    if (rc != QUIK_OK) return rc;
    if (ldacc < N) return QUIK_EINVAL;
    if (!acc) return QUIK_ENULL;
    quik::GemmArgs a{};
    a.xq = xq24; a.T = T; a.K_b = K_b; a.n_out = 0; a.bits = 4;
    a.w_q = w24; a.N = N; a.y = nullptr; a.acc = acc; a.ldacc = ldacc;
    return quik::launch_gemm_sp24(a, static_cast<hipStream_t>(stream)) == hipSuccess ? QUIK_OK : QUIK_ELAUNCH;
}

int quik_linear_sp24(const void* x, int T, int K, int ldx, const int32_t* outlier_idx, int n_out, const void* w24,
                     const void* w_scale, const float* w_reduced, const void* w_out, int ldwo, const void* bias,
                     int N, void* y, int ldy, void* workspace, size_t workspace_bytes, void* stream) {
    const size_t need = quik_workspace_bytes_sp24(T, K, N, n_out);
    if (need == 0) return QUIK_EINVAL;
    if (!workspace) return QUIK_ENULL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return QUIK_EALIGN;
    if (workspace_bytes < need) return QUIK_EWORKSPACE;
    const int K_b = K - n_out, rb = quik_sp24_act_row_bytes(K_b);
    uint8_t* base = static_cast<uint8_t*>(workspace);
    void* xq24 = base;
    float* scale = reinterpret_cast<float*>(base + up256((size_t)T * rb));
    float* zero = reinterpret_cast<float*>(reinterpret_cast<uint8_t*>(scale) + up256((size_t)T * sizeof(float)));
    void* x_out = reinterpret_cast<uint8_t*>(zero) + up256((size_t)T * sizeof(float));
    // validate both stages before anything is enqueued
    int rc = check_quantize(x, T, K, ldx, outlier_idx, n_out, 4, xq24, 16 * ((K + 15) / 16), scale, zero, x_out, n_out);
    if (rc != QUIK_OK) return rc;
    if (K > 16384) return QUIK_EUNSUPPORTED;
    rc = check_gemm_sp24(xq24, x_out, n_out, T, K_b, n_out, w24, w_out, ldwo, N);
    if (rc != QUIK_OK) return rc;
    if (ldy < N) return QUIK_EINVAL;
    if (!w_scale || !w_reduced || !y) return QUIK_ENULL;
    if (reinterpret_cast<uintptr_t>(y) & 1u) return QUIK_EALIGN;
    rc = quik_quantize_sp24(x, T, K, ldx, outlier_idx, n_out, xq24, scale, zero, x_out, n_out, stream);
    if (rc != QUIK_OK) return rc;
    return quik_gemm_dequant_sp24(xq24, scale, zero, x_out, n_out, T, K_b, n_out, w24, w_scale, w_reduced, w_out,
                                  ldwo, bias, N, y, ldy, stream);
}

// ---- measurement probes

int quik_debug_mfma_probe(int workgroups, int iters, int32_t* sink, void* stream) {
    if (workgroups <= 0 || iters <= 0) return QUIK_EINVAL;
    if (!sink) return QUIK_ENULL;
    return quik::launch_mfma_probe(workgroups, iters, sink, static_cast<hipStream_t>(stream)) == hipSuccess
               ? QUIK_OK
               : QUIK_ELAUNCH;
}

int quik_debug_mix_probe(int mix, int workgroups, int iters, int32_t* sink, const void* src, size_t src_bytes,
                         unsigned long long* clocks, void* stream) {
    if (mix < 0 || (mix > 63 && mix != 97 && mix != 127) || ((mix & 32) && !(mix & 1)) || workgroups <= 0 || workgroups > 4096 ||
        iters <= 0)
        return QUIK_EINVAL;
    if (!sink) return QUIK_ENULL;
    if (mix & 8) {
        if (!src) return QUIK_ENULL;
        if (src_bytes < (size_t(16) << 20)) return QUIK_EINVAL;
        if (!aligned16(src)) return QUIK_EALIGN;
    }
    return quik::launch_mix_probe(mix, workgroups, iters, sink, src, (mix & 8) ? src_bytes : 0, clocks,
                                  static_cast<hipStream_t>(stream)) == hipSuccess
               ? QUIK_OK
               : QUIK_ELAUNCH;
}

int quik_debug_copy_probe(const void* src, void* dst, size_t bytes, void* stream) {
    if (bytes == 0 || bytes % 16) return QUIK_EINVAL;
    if (!src || !dst) return QUIK_ENULL;
    if (!aligned16(src) || !aligned16(dst)) return QUIK_EALIGN;
    return quik::launch_copy_probe(src, dst, bytes, static_cast<hipStream_t>(stream)) == hipSuccess ? QUIK_OK
                                                                                                   : QUIK_ELAUNCH;
}

int quik_check_outlier_idx_host(const int32_t* idx, int n_out, int K) {
    if (n_out < 0 || K <= 0 || n_out >= K) return QUIK_EINVAL;
    if (n_out > 0 && !idx) return QUIK_ENULL;
    std::vector<bool> seen((size_t)K, false);
    for (int j = 0; j < n_out; ++j) {
        if (idx[j] < 0 || idx[j] >= K || seen[idx[j]]) return QUIK_EINVAL;
        seen[idx[j]] = true;
    }
    return QUIK_OK;
}

}  // extern "C"
