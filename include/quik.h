/*
 * quik.h -- C ABI of the MI355X (gfx950) QUIK hybrid-quantized linear layer.
 *
 * The library computes the forward pass of one QUIK linear layer, "QUIK Matmul"
 * (arXiv 2310.09259, Section 3.3, Algorithm 1), for a batch of T tokens:
 *
 *   1. split the input columns into n_out outlier columns (kept in fp16) and
 *      K_b = K - n_out base columns, and quantize the base part per token,
 *      asymmetrically, to signed `bits`-bit integers in a packed format
 *      (Algorithm 1, "split" and "Quantization");
 *   2. multiply the packed activations with the packed, offline-quantized
 *      weights using integer matrix cores with INT32 accumulation ("INTmatmul");
 *   3. dequantize in the GEMM epilogue with the per-token and per-output-channel
 *      scales and the zero-point correction of Eq. (1) ("Dequantization") and add
 *      the fp16 product of the outlier columns ("FPmatmul", final add).
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller, unless a
 *     parameter is explicitly called "host".  The library never allocates,
 *     frees or keeps a pointer.  `stream` is a hipStream_t passed as void*
 *     (NULL = the default stream).  Calls enqueue work on `stream` and return;
 *     they do not synchronize.
 *   - Matrices are row-major.  Leading dimensions ("ld...") are row strides, in
 *     ELEMENTS for fp16 / int32 matrices and in BYTES for packed integer
 *     matrices.
 *   - Packed integers: bits = 4 stores two two's-complement nibbles per byte.
 *     WEIGHTS keep element 2p in bits 0..3 and element 2p+1 in bits 4..7 of byte
 *     p.  ACTIVATIONS (xq, produced and consumed only inside this library) keep
 *     element 2p in bits 4..7 and element 2p+1 in bits 0..3: with opposite
 *     orders every product pairs a high with a low nibble, which lets the GEMM
 *     widen each operand register with a single AND.  bits = 8 stores one signed
 *     byte per element.  Quantized activations lie in
 *     [-2^(bits-1), 2^(bits-1) - 1], weights likewise.
 *   - Side data (bits = 4 only; an implementation device that the argument
 *     lists do not show): the GEMM widens each packed operand register with a
 *     single AND, which leaves an offset of 8 on the low nibbles.  Two INT32
 *     vectors remove it exactly in the epilogue, so the accumulator that is
 *     dequantized is the exact integer dot product: the sum of a token's signed
 *     codes at EVEN k, which quik_quantize leaves in its `workspace` and
 *     quik_gemm_dequant reads from there, and the sum of a channel's signed
 *     weight codes at ODD k, which quik_weight_reduce appends to `w_reduced`
 *     (entries N .. 2N-1, as INT32 bit patterns).  Callers only carry the two
 *     buffers from the producing call to the consuming one.
 *   - Base columns keep their ascending original order; outlier column j of
 *     x_out and w_out corresponds to input column outlier_idx[j].
 *   - Return value: QUIK_OK (0) or a negative quik_status.  When an error is
 *     returned nothing has been enqueued.  Arguments are validated on the host;
 *     the contents of device buffers (for example the index list) are not, but
 *     no index value can make a kernel access memory outside the buffers
 *     described here: out-of-range or repeated indices only give unspecified
 *     VALUES.
 *   - Limits: bits in {4, 8}; K, ldx multiples of 8; n_out a multiple of 8,
 *     0 <= n_out < K; K_b * bits a multiple of 8; K <= 32768; all input base
 *     pointers 16-byte aligned; ldq, ldw multiples of 16 bytes; ldo, ldwo
 *     multiples of 8 elements; y and ldy are unconstrained (ldy >= N).
 *   - Thread safety: no global mutable state; calls on different streams are
 *     independent.
 */
#ifndef QUIK_H_
#define QUIK_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QUIK_OK = 0,
    QUIK_EINVAL = -1,       /* a size or flag is out of range or inconsistent      */
    QUIK_ENULL = -2,        /* a required pointer is NULL                           */
    QUIK_EALIGN = -3,       /* a pointer or leading dimension is not aligned        */
    QUIK_EUNSUPPORTED = -4, /* valid in the paper's terms, not built here           */
    QUIK_EWORKSPACE = -5,   /* workspace too small                                  */
    QUIK_ELAUNCH = -6       /* the HIP runtime refused a launch                     */
} quik_status;

/* Library version (monotonic integer). */
int quik_version(void);

/* Static, human-readable name of a status code. */
const char *quik_status_string(int status);

/*
 * Canonical row stride in bytes of a packed matrix with K_b elements per row:
 * K_b * bits / 8 rounded up to a multiple of 16.  Returns 0 on invalid input.
 */
int quik_packed_row_bytes(int K_b, int bits);

/*
 * Bytes of device workspace quik_linear needs for a [T, K] input with n_out
 * outlier columns: packed activations [T, quik_packed_row_bytes], per-token
 * scale and zero (fp32 each), the side data of quik_quantize and the fp16
 * outlier block [T, n_out], each region aligned to 256 bytes.  Returns 0 on
 * invalid input.  N is accepted for symmetry and does not change the result.
 */
size_t quik_workspace_bytes(int T, int K, int N, int n_out, int bits);

/*
 * Where quik_linear (and quik_linear_ablation) keep their intermediate results
 * inside `workspace`, for callers that want to look at them (tests, debugging):
 * byte offsets of the packed activations, scale, zero and the outlier block
 * are written to offsets[0..3] (HOST pointer), the row stride of the packed
 * activations to *ldq (HOST pointer).  Returns QUIK_OK or QUIK_EINVAL / QUIK_ENULL.
 */
int quik_workspace_regions(int T, int K, int N, int n_out, int bits, size_t *offsets, int *ldq);

/*
 * Bytes of the `workspace` of quik_quantize / quik_gemm_dequant /
 * quik_debug_int_gemm (4 T for bits = 4, nothing for bits = 8; never 0 for
 * valid input, so that a buffer of this size can always be allocated), and of
 * the `w_reduced` buffer of quik_weight_reduce (8 N for bits = 4, 4 N for
 * bits = 8).  Return 0 on invalid input.
 */
size_t quik_quantize_workspace_bytes(int T, int bits);
size_t quik_w_reduced_bytes(int N, int bits);

/*
 * Fused split + per-token asymmetric quantization (Algorithm 1, "split" and
 * function "Quantization"; fusion as in Section 3.4, "Quantization Fusion").
 *
 * For every token t: zero[t] = min and scale[t] = (max - min) / (2^bits - 1)
 * over the BASE columns only (scale = 1 for a constant row); every base element
 * becomes q = clamp(rne((x - zero) * (1 / scale)), 0, 2^bits - 1) - 2^(bits-1),
 * evaluated in IEEE binary32 with a once-per-token correctly rounded reciprocal,
 * and is stored packed; outlier columns are copied bit for bit to x_out.
 *
 *   x            in   fp16 [T, ldx], ldx >= K
 *   outlier_idx  in   int32 [n_out], unique, in [0, K); may be NULL if n_out = 0
 *   xq           out  packed [T, ldq bytes], ldq >= K_b*bits/8; bytes of each row
 *                     past the packed data up to ldq are written as zero
 *   scale, zero  out  fp32 [T]
 *   x_out        out  fp16 [T, ldo], ldo >= n_out; may be NULL if n_out = 0
 *   workspace    out  device scratch of at least quik_quantize_workspace_bytes(T, bits)
 *                     bytes, 4-byte aligned: receives the side data that
 *                     quik_gemm_dequant needs beside xq (see "Side data").  NULL =
 *                     not wanted (the result can then only feed quik_debug_int_gemm
 *                     without side data).  QUIK_EWORKSPACE if given and too small.
 */
int quik_quantize(const void *x, int T, int K, int ldx,
                  const int32_t *outlier_idx, int n_out, int bits,
                  void *xq, int ldq, float *scale, float *zero,
                  void *x_out, int ldo, void *workspace, size_t workspace_bytes, void *stream);

/*
 * wReduced (Section 3.3, text after Eq. (1)): the static per-output-channel
 * term of the zero-point correction,
 *   w_reduced[n] = float(w_scale[n]) * float(sum_k w_q[n, k]),  k < K_b.
 * Offline preparation, not part of the timed path.
 *
 *   w_q         in   packed [N, ldw bytes]
 *   w_scale     in   fp16 [N]
 *   w_reduced   out  quik_w_reduced_bytes(N, bits) bytes: fp32 [N] = wReduced; for
 *                    bits = 4 followed by N INT32 values of side data (see "Side data")
 */
int quik_weight_reduce(const void *w_q, int ldw, const void *w_scale,
                       int N, int K_b, int bits, float *w_reduced, void *stream);

/*
 * Integer GEMM + dequantization epilogue + outlier GEMM (Algorithm 1,
 * "INTmatmul", function "Dequantization", "FPmatmul" and the final add; the
 * epilogue fusion of Section 3.4):
 *
 *   acc[t,n] = sum_{k<K_b} xq[t,k] * w_q[n,k]                       (INT32, exact)
 *   y[t,n]   = acc * scale[t] * w_scale[n]
 *            + (zero[t] + 2^(bits-1) * scale[t]) * w_reduced[n]
 *            + sum_{j<n_out} x_out[t,j] * w_out[n,j]  (+ bias[n])   -> fp16
 *
 * Floating point is binary32 with fp16 inputs to the outlier product; y is
 * rounded once to fp16.
 *
 *   xq       in  packed [T, ldq bytes]; bytes of a row between K_b*bits/8 and
 *                ldq MUST be zero (quik_quantize writes them so)
 *   scale, zero  in  fp32 [T]
 *   x_out    in  fp16 [T, ldo]        (ignored if n_out = 0, may be NULL)
 *   w_q      in  packed [N, ldw bytes]; pad bytes may hold anything
 *   w_scale  in  fp16 [N]
 *   w_reduced in the buffer quik_weight_reduce wrote for these weights and `bits`
 *   w_out    in  fp16 [N, ldwo]       (ignored if n_out = 0, may be NULL)
 *   bias     in  fp16 [N] or NULL
 *   y        out fp16 [T, ldy], ldy >= N
 *   workspace in the workspace quik_quantize filled together with xq (required for
 *                bits = 4: QUIK_ENULL / QUIK_EWORKSPACE; ignored for bits = 8)
 * K_b must be below 131072 (INT32 headroom of the 4-bit path).
 */
int quik_gemm_dequant(const void *xq, int ldq, const float *scale, const float *zero,
                      const void *x_out, int ldo,
                      int T, int K_b, int n_out, int bits,
                      const void *w_q, int ldw, const void *w_scale, const float *w_reduced,
                      const void *w_out, int ldwo,
                      const void *bias, int N, void *y, int ldy,
                      const void *workspace, size_t workspace_bytes, void *stream);

/*
 * Test hook: the same integer K-loop as quik_gemm_dequant -- same kernel, same
 * tile choice -- writing the exact INT32 accumulators instead of running the
 * epilogue ("INTmatmul" alone).
 *   workspace, w_reduced  in  both given (as for quik_gemm_dequant): the single-AND
 *                operand widening of the fused kernel plus its exact correction from
 *                the side data; both NULL: a widening that needs no side data (one
 *                more shift per register pair).  Giving exactly one of them is
 *                QUIK_ENULL.  Same result either way.  Ignored for bits = 8.
 *   acc  out  int32 [T, ldacc], ldacc >= N
 * quik_int_gemm is the same function under its earlier name.
 */
int quik_debug_int_gemm(const void *xq, int ldq, const void *w_q, int ldw,
                        int T, int N, int K_b, int bits, int32_t *acc, int ldacc,
                        const void *workspace, size_t workspace_bytes, const float *w_reduced,
                        void *stream);
int quik_int_gemm(const void *xq, int ldq, const void *w_q, int ldw,
                  int T, int N, int K_b, int bits, int32_t *acc, int ldacc,
                  const void *workspace, size_t workspace_bytes, const float *w_reduced,
                  void *stream);

/*
 * Test hook (host only, no GPU call): how quik_gemm_dequant and quik_debug_int_gemm
 * lay a 4-bit [T, N] output with K_b base columns over a GPU with `cus` compute
 * units.  Returns 0 if the persistent kernel cannot run the shape (plan untouched);
 * 1 if it can and is the automatic choice; 2 if it can but the per-tile kernels are
 * estimated to be at least as fast and are used.  For 1 and 2 the persistent
 * kernel's tile plan is written to plan[0..4] (HOST pointer): 256-row token panels,
 * tiles per panel, the width of the narrower tiles in 32-channel blocks, the number
 * of tiles one block wider (spread evenly), resident workgroups.
 * QUIK_EINVAL / QUIK_ENULL on invalid input.
 */
int quik_debug_gemm_plan(int T, int N, int K_b, int cus, int *plan);

/*
 * Test hook (host only): the k-th output tile (k = 0, 1, ...) that resident workgroup
 * `workgroup` (0 .. plan[4]-1) of the persistent kernel computes for the shape of
 * quik_debug_gemm_plan: tile[0] = first token row, tile[1] = first output channel,
 * tile[2] = number of channels (HOST pointer; the tile has 256 token rows, fewer at
 * the end of T).  Returns 1, or 0 if the workgroup has fewer than k + 1 tiles (tile
 * untouched), or QUIK_EINVAL (also when the persistent kernel cannot run the shape) /
 * QUIK_ENULL.  The kernel walks its tiles with divisors prepared on the host; the hook
 * evaluates that walk and its definition with plain divisions, and returns
 * QUIK_EUNSUPPORTED should the two ever differ.
 */
int quik_debug_gemm_tile(int T, int N, int K_b, int cus, int workgroup, int k, int *tile);

/*
 * Test hook: which kernel family the 4-bit GEMM entry points use from now on, in
 * this process: 0 = automatic (the default), 1 = the persistent kernel wherever
 * quik_debug_gemm_plan returns 1 or 2, 2 = the per-tile kernels always.  Results
 * are the same either way.  Not synchronised with calls in flight on other
 * threads.  Returns QUIK_OK or QUIK_EINVAL.
 */
int quik_debug_set_gemm_path(int mode);

/*
 * The whole layer: quik_quantize into `workspace`, then quik_gemm_dequant
 * (Algorithm 1, "QUIK Matmul").  Two kernel launches on `stream`.
 *
 *   x            in   fp16 [T, ldx]
 *   outlier_idx  in   int32 [n_out]
 *   w_q, w_scale, w_reduced, w_out, bias: as in quik_gemm_dequant
 *   y            out  fp16 [T, ldy]
 *   workspace    device scratch of at least quik_workspace_bytes(...) bytes,
 *                256-byte aligned; contents after the call: packed activations,
 *                scale, zero, x_out (at the places quik_workspace_regions reports)
 *                and side data
 */
int quik_linear(const void *x, int T, int K, int ldx,
                const int32_t *outlier_idx, int n_out, int bits,
                const void *w_q, int ldw, const void *w_scale, const float *w_reduced,
                const void *w_out, int ldwo, const void *bias, int N,
                void *y, int ldy, void *workspace, size_t workspace_bytes, void *stream);

/*
 * quik_linear for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (without
 * the workspace), same kernels and bit-identical results; the intermediate results live in a
 * static device array of QUIK_NOALLOC_SCRATCH_BYTES that the library holds on every GPU it runs on
 * until the process ends.  The call allocates nothing (no hipMalloc / hipFree, no allocating
 * library routine).  QUIK_EWORKSPACE if quik_workspace_bytes(T, K, N, n_out, bits) exceeds
 * QUIK_NOALLOC_SCRATCH_BYTES (the LLaMA-7B up-projection shape at 2048 tokens needs 5.0 MB;
 * roughly T * (K_b * bits / 8 + 2 * n_out + 12) bytes in general).  All calls on one GPU share
 * that GPU's array: calls that may overlap in time on one GPU (different streams, different host
 * threads) race on it and must be serialized by the caller; calls on different GPUs are
 * independent.  Nothing in the array has to be cleared between calls.
 */
#define QUIK_NOALLOC_SCRATCH_BYTES (8u << 20)
int quik_linear_noalloc(const void *x, int T, int K, int ldx,
                        const int32_t *outlier_idx, int n_out, int bits,
                        const void *w_q, int ldw, const void *w_scale, const float *w_reduced,
                        const void *w_out, int ldwo, const void *bias, int N,
                        void *y, int ldy, void *stream);

/*
 * Fusion ablation of Section 3.4 ("Performance Impact", the kernel versions 1-3): the same layer
 * with its stages left unfused, for measuring what the fusions buy.
 *   version 1: unfused quantization (separate passes: move the outlier part, move the base part,
 *              per-token minimum, per-token maximum, quantize) and unfused dequantization
 *              (INTmatmul writes INT32 accumulators, FPmatmul writes an fp32 matrix, a last
 *              elementwise pass dequantizes and adds them);
 *   version 2: the fused quantization kernel, unfused dequantization;
 *   version 3: quik_linear itself.
 * Arguments as for quik_linear; `workspace` must hold quik_ablation_workspace_bytes(...) bytes
 * (it additionally stages the fp16 base part, the accumulators and the outlier product).
 * Packed activations, scale and zero are bit-identical to quik_quantize's; the output meets the
 * same error bar as quik_linear's (summation order differs).
 */
size_t quik_ablation_workspace_bytes(int T, int K, int N, int n_out, int bits);
int quik_linear_ablation(int version, const void *x, int T, int K, int ldx,
                         const int32_t *outlier_idx, int n_out, int bits,
                         const void *w_q, int ldw, const void *w_scale, const float *w_reduced,
                         const void *w_out, int ldwo,
                         const void *bias, int N,
                         void *y, int ldy, void *workspace, size_t workspace_bytes, void *stream);

/*
 * 4-bit weights under 8-bit activations ("W4A8", the mixed rows of the paper's
 * precision ablation for the down-projection, appendix table "LLaMA-2 perplexity
 * results ... using 256 outliers"): activations are quantized with
 * quik_quantize(bits = 8); the weights are the packed 4-bit matrix (weight nibble
 * order, ldw >= K_b/2) with w_reduced from quik_weight_reduce(bits = 4).  The
 * arithmetic is Algorithm 1 with halfRange = 128 for the activations:
 *   acc[t,n] = sum_k xq8[t,k] * w_q4[n,k]                               (INT32, exact)
 *   y[t,n]   = acc * scale[t] * w_scale[n] + (zero[t] + 128 * scale[t]) * w_reduced[n]
 *            + sum_j x_out[t,j] * w_out[n,j]  (+ bias[n])               -> fp16
 * Other arguments, limits and error behaviour as for quik_gemm_dequant /
 * quik_int_gemm / quik_linear with bits = 8 (the workspace is
 * quik_workspace_bytes(T, K, N, n_out, 8)).  No side data is involved.
 */
int quik_gemm_dequant_w4a8(const void *xq, int ldq, const float *scale, const float *zero,
                           const void *x_out, int ldo, int T, int K_b, int n_out,
                           const void *w_q, int ldw, const void *w_scale, const float *w_reduced,
                           const void *w_out, int ldwo, const void *bias, int N,
                           void *y, int ldy, void *stream);
int quik_int_gemm_w4a8(const void *xq, int ldq, const void *w_q, int ldw,
                       int T, int N, int K_b, int32_t *acc, int ldacc, void *stream);
int quik_linear_w4a8(const void *x, int T, int K, int ldx,
                     const int32_t *outlier_idx, int n_out,
                     const void *w_q, int ldw, const void *w_scale, const float *w_reduced,
                     const void *w_out, int ldwo, const void *bias, int N,
                     void *y, int ldy, void *workspace, size_t workspace_bytes, void *stream);

/*
 * QUIK-4B with the integer product on the FP6 matrix pipe of gfx950 (a higher-rate, still exact,
 * form of Algorithm 1's "INTmatmul" for 4-bit weights and activations; same arithmetic and same
 * results as the bits = 4 entry points above).  The signed codes -8 .. 7 are stored as the 6-bit
 * float format E3M2 (1 sign bit, 3 exponent bits with bias 3, 2 mantissa bits), in which they
 * are exact; products are integers of magnitude <= 64 and a dot product over K_b < 131072
 * columns stays below 2^24, so the fp32 accumulators of the matrix instruction hold the
 * integer results exactly (checked against the INT32 reference by quik_int_gemm_fp6).
 *
 * "FP6 panels": the K_b columns of a matrix with R rows are padded with zeros to
 * S = ceil(K_b / 64) stages of 64 columns and stored stage by stage: stage s of row r is the
 * 48-byte block at byte (s * R + r) * 48 of the buffer (S * R * 48 bytes, 16-byte aligned;
 * quik_fp6_row_bytes(K_b) = 48 S).  A stage holds two groups of 32 columns, g = 0, 1.  A group
 * is a 192-bit little-endian string (column j of the group in bits [6j, 6j+6)) = dwords
 * d0 .. d5; d0 .. d3 of group g sit at byte 16 g of the block, d4, d5 at byte 32 + 8 g.
 *
 *  quik_weight_pack_fp6   offline: packed signed 4-bit weights w_q [N, ldw] (weight nibble
 *                         order of quik.h, ldw >= K_b/2, K_b even) -> FP6 panels w6 (R = N).
 *                         w_scale, w_reduced, w_out stay as for bits = 4 (the side data is not read).
 *  quik_quantize_fp6      quik_quantize(bits = 4) with the packed output as FP6 panels xq6
 *                         (R = T); scale, zero, x_out as there; K <= 16384.
 *  quik_gemm_dequant_fp6  quik_gemm_dequant for FP6 panels.
 *  quik_int_gemm_fp6      acc[t,n] = sum_k q[t,k] * w[n,k] as INT32 (test hook).
 *  quik_linear_fp6        quik_quantize_fp6 + quik_gemm_dequant_fp6 on one stream; workspace of
 *                         quik_workspace_bytes_fp6(T, K, N, n_out) bytes, 256-byte aligned.
 * All pointers are DEVICE pointers (16-byte aligned where the integer forms require it); error
 * behaviour as for the integer forms; additionally QUIK_EUNSUPPORTED if one stage of all rows
 * (max(T, N) * 48 bytes) reaches 4 GB.
 */
int quik_fp6_row_bytes(int K_b);
size_t quik_workspace_bytes_fp6(int T, int K, int N, int n_out);
int quik_weight_pack_fp6(const void *w_q, int ldw, int N, int K_b, void *w6, void *stream);
int quik_quantize_fp6(const void *x, int T, int K, int ldx, const int32_t *outlier_idx, int n_out,
                      void *xq6, float *scale, float *zero, void *x_out, int ldo, void *stream);
int quik_gemm_dequant_fp6(const void *xq6, const float *scale, const float *zero,
                          const void *x_out, int ldo, int T, int K_b, int n_out,
                          const void *w6, const void *w_scale, const float *w_reduced,
                          const void *w_out, int ldwo, const void *bias, int N,
                          void *y, int ldy, void *stream);
int quik_int_gemm_fp6(const void *xq6, const void *w6, int T, int N, int K_b,
                      int32_t *acc, int ldacc, void *stream);
int quik_linear_fp6(const void *x, int T, int K, int ldx, const int32_t *outlier_idx, int n_out,
                    const void *w6, const void *w_scale, const float *w_reduced,
                    const void *w_out, int ldwo, const void *bias, int N,
                    void *y, int ldy, void *workspace, size_t workspace_bytes, void *stream);

/*
 * QUIK-4B for 2:4-sparse weights (the joint INT4 + 2:4 format of Section 4.3, paragraph
 * "Joint INT-4 Quantization and 2:4 Sparsification"; the
 * arithmetic is Algorithm 1 unchanged, with a weight matrix in which at most two of every four
 * consecutive base columns 4i .. 4i+3 are nonzero).  The integer product runs on the sparse int8
 * matrix instruction of gfx950 (twice the dense int8 rate, exact INT32 accumulation); results are
 * those of the bits = 4 entry points for the same matrices.
 *
 * Both operands are stored stage by stage: the K_b columns are padded with zeros to
 * S = ceil(K_b / 64) stages of 64 columns, and the rows of a stage follow each other.
 *   activations xq24: stage s of token t is the 32-byte block at byte (s * T + t) * 32
 *     (S * T * 32 bytes; quik_sp24_act_row_bytes(K_b) = 32 S).  Byte 4 m + p of a block holds the
 *     signed codes (two's complement nibbles) of columns 8 m + p (high nibble) and 8 m + 4 + p
 *     (low nibble) of the stage.
 *   weights w24: stage s of channel n is the 32-byte block at byte (s * N + n) * 32
 *     (quik_sp24_weight_bytes(N, K_b) = S * N * 32 bytes).  A block is two 16-byte records
 *     (halves h = 0, 1): an 8-byte value field, a 4-byte index word, 4 zero bytes.  The group
 *     of four columns kappa (0 .. 15) of the stage belongs to half h = (kappa / 4) % 2, pair
 *     q = 4 (kappa / 8) + kappa % 4; its two kept values are values c = 2 q and 2 q + 1 of the
 *     half: value c is a two's complement nibble in dword c / 8 of the field, byte c % 4, low
 *     nibble if (c / 4) % 2 == 0, else high; bits [2 c, 2 c + 2) of the half's index word give its
 *     position 0 .. 3 in the group.  Kept positions: the nonzero ones, filled up to two with the
 *     lowest unused positions, ascending.
 *
 *  quik_weight_pack_sp24   offline: packed signed 4-bit weights w_q [N, ldw] (weight nibble order
 *                          of quik.h, ldw >= K_b/2, K_b even) -> w24.  `violations` (DEVICE int32,
 *                          may be NULL) is incremented by the number of groups with more than two
 *                          nonzero values (such a group keeps only its first two: clear the counter
 *                          before the call, read it after the stream has finished, and reject the
 *                          matrix unless it is 0).  w_scale, w_reduced, w_out stay as for bits = 4
 *                          (the side data is not read).
 *  quik_quantize_sp24      quik_quantize(bits = 4) with the packed output as xq24; scale, zero,
 *                          x_out as there; K <= 16384.
 *  quik_gemm_dequant_sp24  quik_gemm_dequant for these operands.
 *  quik_int_gemm_sp24      acc[t,n] = sum_k q[t,k] * w[n,k] as INT32 (test hook).
 *  quik_linear_sp24        quik_quantize_sp24 + quik_gemm_dequant_sp24 on one stream; workspace of
 *                          quik_workspace_bytes_sp24(T, K, N, n_out) bytes, 256-byte aligned.
 * All pointers are DEVICE pointers (16-byte aligned where the integer forms require it); error
 * behaviour as for the integer forms; additionally QUIK_EUNSUPPORTED if xq24 or w24 reaches 4 GB.
 */
int quik_sp24_act_row_bytes(int K_b);
size_t quik_sp24_weight_bytes(int N, int K_b);
size_t quik_workspace_bytes_sp24(int T, int K, int N, int n_out);
int quik_weight_pack_sp24(const void *w_q, int ldw, int N, int K_b, void *w24,
                          int32_t *violations, void *stream);
int quik_quantize_sp24(const void *x, int T, int K, int ldx, const int32_t *outlier_idx, int n_out,
                       void *xq24, float *scale, float *zero, void *x_out, int ldo, void *stream);
int quik_gemm_dequant_sp24(const void *xq24, const float *scale, const float *zero,
                           const void *x_out, int ldo, int T, int K_b, int n_out,
                           const void *w24, const void *w_scale, const float *w_reduced,
                           const void *w_out, int ldwo, const void *bias, int N,
                           void *y, int ldy, void *stream);
int quik_int_gemm_sp24(const void *xq24, const void *w24, int T, int N, int K_b,
                       int32_t *acc, int ldacc, void *stream);
int quik_linear_sp24(const void *x, int T, int K, int ldx, const int32_t *outlier_idx, int n_out,
                     const void *w24, const void *w_scale, const float *w_reduced,
                     const void *w_out, int ldwo, const void *bias, int N,
                     void *y, int ldy, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Measurement probes (not part of the layer): what the chip sustains, so that a kernel's rate can
 * be quoted against a measured ceiling beside the data-sheet one.
 *  quik_debug_mfma_probe  `workgroups` workgroups of four waves, each wave issuing 4 * iters
 *                         independent 32x32x32 int8 matrix instructions on register-resident
 *                         operands: 2 * 32 * 32 * 32 * 16 * workgroups * iters integer operations.
 *                         `sink` (DEVICE int32 [1]) is never written in practice.
 *  quik_debug_copy_probe  plain streaming copy of `bytes` (a multiple of 16; both pointers DEVICE,
 *                         16-byte aligned): reads `bytes`, writes `bytes`.
 */
int quik_debug_mfma_probe(int workgroups, int iters, int32_t *sink, void *stream);
int quik_debug_copy_probe(const void *src, void *dst, size_t bytes, void *stream);

/*
 * Measurement probe: the instruction mix of the 4-bit GEMM's K loop around the int8 matrix
 * instruction, one ingredient at a time and free of data dependences, to show what each kind of
 * instruction costs the matrix pipe.  `workgroups` workgroups of eight waves (one per CU on a 256-CU
 * chip with workgroups = 256); every wave issues 12 * iters matrix instructions
 * (2 * 32 * 32 * 32 * 12 * 8 * workgroups * iters integer operations) plus, per bit of `mix`:
 *   1  operands of pseudo-random bytes that change from one matrix instruction to the next (else
 *      constant operands of small values, most bytes zero)
 *   2  four vector bit operations per matrix instruction
 *   4  five 16-byte-per-lane LDS reads per 12 matrix instructions
 *   8  two global -> LDS copies of 16 bytes per lane per 12 matrix instructions, out of `src`
 *      (DEVICE, 16-byte aligned, src_bytes >= 16 MiB; read only)
 *  16  a workgroup barrier per 48 matrix instructions
 *  32  (only together with 1) the changing operands are bytes as the GEMM's nibble widening makes
 *      them: half of the operand words vary in the high nibble of every byte only, the other half
 *      in the low nibble only.  The clock the chip sustains depends on how many operand bits toggle,
 *      so the rates with this bit set are the ceiling for the GEMM's own operands.
 *  64  the same work on the 16 x 16 x 64 int8 matrix instruction (two in place of every 32 x 32 x 32 one,
 *      ten 8-byte LDS reads in place of five 16-byte ones): the persistent kernel's instruction.  Only as
 *      mix = 97 (matrix instructions alone on widened-nibble operands) and mix = 127 (the whole mix).
 * clocks (DEVICE uint64 [2], or NULL): ticks of the s_memtime and of the s_memrealtime counter over
 * the loop of workgroup 0 (for comparing loads with each other).  `sink` as above.
 * QUIK_EINVAL for mix outside 0..63, 97, 127, for bit 32 without bit 1, or bad sizes; QUIK_ENULL, QUIK_EALIGN.
 */
int quik_debug_mix_probe(int mix, int workgroups, int iters, int32_t *sink, const void *src, size_t src_bytes,
                         unsigned long long *clocks, void *stream);

/*
 * Host-side validator for an outlier index list (HOST pointer): returns QUIK_OK
 * if all n_out entries are unique and inside [0, K), QUIK_EINVAL otherwise.
 */
int quik_check_outlier_idx_host(const int32_t *outlier_idx_host, int n_out, int K);

#ifdef __cplusplus
}
#endif
#endif /* QUIK_H_ */
