/*
 * fp6.h - C ABI of the MI355X (gfx950) W6A16 linear-layer library.
 *
 * The library implements the weight-only-quantized linear layer of FP6-LLM
 * (arXiv 2401.14112): Y = dequant(W_fp6) * X with 6-bit e3m2 weights
 * (Section 2.2, Eq. 1: 1 sign, 3 exponent, 2 mantissa bits, bias 3), one fp16
 * scale per output channel (Algorithm 1's "Scales"; Section 3), fp16 activations,
 * weights de-quantized in registers inside the GEMM kernel and never written back
 * to memory (Section 4.1, the unified-kernel design).
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers (hipMalloc'ed or equivalent) and must
 *     be 16-byte aligned.  The caller owns every buffer; the library allocates
 *     and frees nothing and never synchronizes.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     work is enqueued on it; the calls are safe to record into a HIP graph.
 *   - Matrices follow Section 6 of the paper: weights are A = [M][K] (M output
 *     channels, K input features); activations B = [K][N] and outputs C = [M][N]
 *     are column-major, i.e. X is stored [N][K] (K contiguous) and Y is stored
 *     [N][M] (M contiguous) - the natural layout of a linear layer over N tokens.
 *   - Supported shapes: M a multiple of 16, K a multiple of 256, 1 <= N < 2^31
 *     (M < 2^31, K < 2^24: activations are addressed with 32-bit byte offsets; token
 *     counts whose activations exceed 2 GiB are processed as several launches on the
 *     same stream).  Packed weights are addressed with
 *     32-bit offsets: (K/256 + 64) * (M/16) * 3072 must stay below 2^31 (about
 *     2.8e9 weights per matrix, at every width); larger matrices are refused with
 *     FP6_ERR_SHAPE and their size queries return 0 - split them along M.
 *   - Errors are detected on the host before anything is launched and reported
 *     as a status code; nothing is enqueued when a call fails.
 *   - W must be finite (the method has no inf/NaN code); this is not checked.
 */
#ifndef FP6_MI355X_H
#define FP6_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FP6_OK = 0,
    FP6_ERR_NULL = 1,      /* a required pointer is NULL */
    FP6_ERR_SHAPE = 2,     /* M, N, K not positive, M % 16 != 0, K % 256 != 0, or the matrix too large */
    FP6_ERR_WORKSPACE = 3, /* workspace missing or smaller than fp6_linear_workspace_bytes() */
    FP6_ERR_ALIGN = 4,     /* a pointer is not 16-byte aligned */
    FP6_ERR_HIP = 5        /* the HIP runtime refused the launch */
} fp6_status;

/* Human-readable name of a status code (static string). */
const char *fp6_status_str(int status);

/* Version of the packed weight layouts written by the *_quantize_pack calls and read by the
 * *_unpack / *_linear calls.  Store it next to any packed buffer that is saved.  (4: the
 * 3-bit stream moved to tiles of 512 columns; the 6-, 5- and 4-bit streams are those of 3.) */
int fp6_layout_version(void);

/* Bytes of the packed code stream of an M x K matrix: 6 bits per weight, no
 * padding (Section 5.2: 32 x-bit weights occupy x 32-bit words) = 3*M*K/4.
 * Returns 0 for an unsupported shape. */
size_t fp6_packed_bytes(int64_t M, int64_t K);

/*
 * Ahead-of-time weight preparation (Section 5.2, "Ahead-of-time Bit-level
 * Pre-packing"; the quantizer itself is outside the paper and follows the
 * benchmark recipe): for every row m
 *     scale[m] = fp16_rne(max_k |W[m][k]| / 28)
 *     code     = sign bit of W | nearest e3m2 magnitude of |W[m][k]| / scale[m],
 *                ties to the even code, saturating at 28
 * (a row whose scale rounds to 0 gets sign-only codes), and the 6-bit codes are
 * written in the library's gfx950 tile order so that the GEMM reads them as
 * contiguous 16-byte-per-lane loads.
 *   W_f16   in   device, fp16 row-major [M][K]
 *   packed  out  device, fp6_packed_bytes(M, K) bytes, every bit written
 *   scales  out  device, fp16 [M]
 */
fp6_status fp6_quantize_pack(const void *W_f16, int64_t M, int64_t K, void *packed, void *scales_f16,
                             void *stream);

/*
 * De-quantize a packed matrix back to fp16 (the first half of the "dual-kernel"
 * scheme of Section 4.1; a test aid, not the production path):
 *     W_out[m][k] = fp16_rne(e3m2_value(code[m][k]) * scale[m])      (one rounding)
 *   packed  in   device, fp6_packed_bytes(M, K) bytes
 *   scales  in   device, fp16 [M]
 *   W_out   out  device, fp16 row-major [M][K]
 */
fp6_status fp6_unpack(const void *packed, const void *scales_f16, int64_t M, int64_t K, void *W_f16_out,
                      void *stream);

/*
 * Workspace needed by fp6_linear / fp16_linear for this shape (0 when the
 * kernel chosen for it needs none).  The workspace holds split-K partial sums and
 * arrival counters.  It MUST be zero-filled once before its first use
 * (fp6_workspace_init or any device memset); the kernels leave the counters at
 * zero, so it can be reused by later calls without clearing it again.  Two calls
 * that may run concurrently (different streams) need different workspaces.
 */
size_t fp6_linear_workspace_bytes(int64_t M, int64_t N, int64_t K);
size_t fp16_linear_workspace_bytes(int64_t M, int64_t N, int64_t K);

/* Zero-fill a workspace with a kernel on `stream` (graph-capturable). */
fp6_status fp6_workspace_init(void *workspace, size_t workspace_bytes, void *stream);

/*
 * The W6A16 linear layer (Section 6: C = A x B; Sections 4.1, 5.3, 5.4: weights
 * are fetched in packed form, de-quantized to fp16 in registers and fed to the
 * matrix cores in one kernel):
 *     Y[n][m] = fp16_rne( scale[m] * sum_k e3m2_value(code[m][k]) * X[n][k] )
 * accumulated in fp32; the per-row scale is applied once after accumulation.
 *   packed     in   device, written by fp6_quantize_pack for the same (M, K)
 *   scales     in   device, fp16 [M]
 *   X_f16      in   device, fp16 [N][K]
 *   Y_f16      out  device, fp16 [N][M]
 *   workspace  in/out  device, >= fp6_linear_workspace_bytes(M, N, K) bytes, may
 *              be NULL when that is 0
 * Results are deterministic: the same inputs give the same bits on every call.
 */
fp6_status fp6_linear(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M,
                      int64_t N, int64_t K, void *workspace, size_t workspace_bytes, void *stream);

/*
 * fp6_linear for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  The split-K partial sums and arrival
 * counters live in a buffer of FP6_STATIC_SCRATCH_BYTES that is part of the library's device
 * image (each GPU the library runs on holds it until the process ends), so there is no
 * workspace argument and the call allocates nothing: no hipMalloc, no hipFree, no library
 * routine that allocates.  Inputs and outputs are the caller's, as for fp6_linear; the result
 * is bit-identical to fp6_linear's.
 *   - A shape whose split-K state does not fit the buffer is refused with FP6_ERR_WORKSPACE
 *     before anything is enqueued (the 8192 x 22016 layer fits up to N = 512; shapes that need
 *     no split-K always fit).  The check is host arithmetic only.
 *   - The buffer keeps the contents of the last call; each call clears the counters it uses
 *     with a small fill kernel on `stream` first (no memset node, so it can be captured).
 *   - All calls on one GPU share that GPU's buffer: two calls that may overlap on one GPU
 *     (different streams, two threads) race on it.  Serialize them, or give the overlapping
 *     ones fp6_linear with workspaces of their own.
 */
#define FP6_STATIC_SCRATCH_BYTES ((32u << 20) + (64u << 10))
fp6_status fp6_linear_static(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M,
                             int64_t N, int64_t K, void *stream);

/*
 * fp6_linear with the element-wise steps that a decoder block attaches to its
 * projections done in the kernel's last step, on the fp32 sums, before the one
 * rounding to fp16 (Section 7.3 runs whole LLaMA / OPT decoders; this removes the
 * separate kernels, and their trip through memory, between the projections):
 *     z[n][m] = scale[m] * sum_k e3m2_value(code[m][k]) * X[n][k]
 *     z[n][m] += bias[m]                                   if bias_f16 != NULL
 *     gated != 0:  y[n][i] = silu(z[n][2i]) * z[n][2i+1]   (i < M/2; silu(t) = t / (1 + exp(-t)))
 *     gated == 0:  y[n][m] = z[n][m]
 *     y += residual[n][.]                                  if residual_f16 != NULL
 *     Y = fp16_rne(y)
 * For the gated form the caller interleaves the two projections row by row before
 * fp6_quantize_pack: weight row 2i is row i of the gate projection, row 2i+1 is row i
 * of the up projection (M counts both, so Y has M/2 rows).
 *   bias_f16      in   device, fp16 [M] (one per weight row), or NULL
 *   residual_f16  in   device, fp16 [N][Mout], Mout = gated ? M/2 : M, or NULL;
 *                 may be Y_f16 itself (each element is read before it is written)
 *   Y_f16         out  device, fp16 [N][Mout]
 *   everything else as for fp6_linear, including the workspace size
 *   (fp6_linear_workspace_bytes(M, N, K)) and the status codes; bias and residual
 *   must be 16-byte aligned.
 */
fp6_status fp6_linear_fused(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M,
                            int64_t N, int64_t K, const void *bias_f16, const void *residual_f16, int gated,
                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * The library's own W16A16 linear layer, Y[n][m] = fp16_rne(sum_k W[m][k] X[n][k]),
 * built on the same kernel skeleton; it is the in-library baseline that the paper's
 * comparison against an fp16 GEMM (Section 7.1) is re-run against.
 *   W_f16 in device fp16 row-major [M][K]; X, Y, workspace as for fp6_linear
 *   (size from fp16_linear_workspace_bytes).
 */
fp6_status fp16_linear(const void *W_f16, const void *X_f16, void *Y_f16, int64_t M, int64_t N, int64_t K,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * 6-bit weights with group-wise scales (fine-grained quantization): one fp16 scale per
 * row and per group of `group` consecutive columns instead of one per row - the scheme
 * that Section 3 of the paper contrasts with the coarse-grained one, with the scales
 * multiplied into the de-quantized weights before the matrix multiplication as in
 * Algorithm 1.  scales is fp16 [M][K/group], row-major; inside a group the quantizer is
 * that of fp6_quantize_pack (scale = fp16_rne(group max |W| / 28), ...).  The packed
 * stream is the one of fp6_quantize_pack (fp6_packed_bytes).  Only group = 128 is
 * supported (FP6_ERR_SHAPE otherwise).
 *     fp6g_unpack:  W_out[m][k] = fp16_rne(e3m2_value(code) * scale[m][k/group])
 *     fp6g_linear:  Y[n][m] = fp16_rne(sum_k fp16_rne(e3m2_value(code[m][k]) * scale[m][k/group]) * X[n][k]),
 *                   accumulated in fp32 (each weight is rounded to fp16 once before it is used)
 * Workspace: fp6_linear_workspace_bytes(M, N, K).  Everything else as for the fp6_ calls.
 */
fp6_status fp6g_quantize_pack(const void *W_f16, int64_t M, int64_t K, int64_t group, void *packed,
                              void *scales_f16, void *stream);
fp6_status fp6g_unpack(const void *packed, const void *scales_f16, int64_t M, int64_t K, int64_t group,
                       void *W_f16_out, void *stream);
fp6_status fp6g_linear(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M,
                       int64_t N, int64_t K, int64_t group, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same three calls for 5-bit weights (W5A16).  The paper presents its pre-packing
 * and its cast to fp16 as independent of the bit-width (Section 1 names widths from 6
 * down to 3 bits; Sections 5.2 and 5.3).  FP5 is e2m2: code = s e1 e0 m1 m0, Eq. 1 with
 * bias 2^(2-1)-1 = 1, subnormal E = 0 binade, no inf/NaN: magnitudes 0 .25 .5 .75,
 * 1 .. 1.75, 2 .. 3.5, 4 .. 7.  Quantizer: scale[m] = fp16_rne(max_k |W[m][k]| / 7),
 * nearest e2m2 magnitude of |W| / scale, ties to the even code, saturating at 7.
 * The packed stream has fp5_packed_bytes(M, K) = 5*M*K/8 bytes (tiles of 2560 bytes)
 * and is de-quantized in registers with whole-word shifts and masks and the
 * exponent-bias multiply of Eq. 3, the gfx950 having no conversion for this format.
 * Arguments, layouts of W, X, Y, scales, workspace rules, shapes, alignment and error
 * behaviour are those of the fp6_ calls; the workspace size is that of fp6_linear.
 */
size_t fp5_packed_bytes(int64_t M, int64_t K);
size_t fp5_linear_workspace_bytes(int64_t M, int64_t N, int64_t K);
fp6_status fp5_quantize_pack(const void *W_f16, int64_t M, int64_t K, void *packed, void *scales_f16,
                             void *stream);
fp6_status fp5_unpack(const void *packed, const void *scales_f16, int64_t M, int64_t K, void *W_f16_out,
                      void *stream);
fp6_status fp5_linear(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M,
                      int64_t N, int64_t K, void *workspace, size_t workspace_bytes, void *stream);

/*
 * And for 4-bit weights (W4A16): FP4 is e2m1, code = s e1 e0 m0, Eq. 1 with bias 1,
 * subnormal E = 0 binade, no inf/NaN: magnitudes 0 .5 1 1.5 2 3 4 6 (the FP4 element
 * type of the OCP microscaling formats, which the gfx950 converts to fp16 itself).
 * Quantizer: scale[m] = fp16_rne(max_k |W[m][k]| / 6), nearest magnitude, ties to the
 * even code, saturating at 6.  fp4_packed_bytes(M, K) = M*K/2 (tiles of 2048 bytes).
 * Everything else as for the fp6_ calls.
 */
size_t fp4_packed_bytes(int64_t M, int64_t K);
size_t fp4_linear_workspace_bytes(int64_t M, int64_t N, int64_t K);
fp6_status fp4_quantize_pack(const void *W_f16, int64_t M, int64_t K, void *packed, void *scales_f16,
                             void *stream);
fp6_status fp4_unpack(const void *packed, const void *scales_f16, int64_t M, int64_t K, void *W_f16_out,
                      void *stream);
fp6_status fp4_linear(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M,
                      int64_t N, int64_t K, void *workspace, size_t workspace_bytes, void *stream);

/*
 * And for 3-bit weights (W3A16; Section 1 of the paper names 3-bit among the widths
 * the scheme covers): FP3 is read as e2m0, code = s e1 e0, Eq. 1 with bias 1 and no
 * mantissa bits, E = 0 holding only zero, no inf/NaN: magnitudes 0 1 2 4.  Quantizer:
 * scale[m] = fp16_rne(max_k |W[m][k]| / 4), nearest magnitude, ties to the even code,
 * saturating at 4.  The stream is made of tiles of 16 rows x 512 columns, 3072 bytes each
 * (three whole 128-bit pieces per lane; the codes are pre-arranged bit by bit so that the
 * kernel rebuilds four 4-bit words from three stored ones with a handful of AND/shift/OR):
 * fp3_packed_bytes(M, K) = ceil(K/512) * (M/16) * 3072, i.e. 3*M*K/8 when K is a multiple
 * of 512 and half a tile of zero padding per row tile otherwise (written by
 * fp3_quantize_pack).  This layout is the one of fp6_layout_version() >= 4.  Everything
 * else as for the fp6_ calls.
 */
size_t fp3_packed_bytes(int64_t M, int64_t K);
size_t fp3_linear_workspace_bytes(int64_t M, int64_t N, int64_t K);
fp6_status fp3_quantize_pack(const void *W_f16, int64_t M, int64_t K, void *packed, void *scales_f16,
                             void *stream);
fp6_status fp3_unpack(const void *packed, const void *scales_f16, int64_t M, int64_t K, void *W_f16_out,
                      void *stream);
fp6_status fp3_linear(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M,
                      int64_t N, int64_t K, void *workspace, size_t workspace_bytes, void *stream);

/*
 * fp6_linear_fused for the other weight formats: the same steps (bias, silu(gate) * up over
 * interleaved row pairs, residual) after fp5_linear, fp4_linear, fp3_linear and fp6g_linear.
 * Arguments as for fp6_linear_fused (fp6g: scales fp16 [M][K/group], group = 128).
 */
fp6_status fp5_linear_fused(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M,
                            int64_t N, int64_t K, const void *bias_f16, const void *residual_f16, int gated,
                            void *workspace, size_t workspace_bytes, void *stream);
fp6_status fp4_linear_fused(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M,
                            int64_t N, int64_t K, const void *bias_f16, const void *residual_f16, int gated,
                            void *workspace, size_t workspace_bytes, void *stream);
fp6_status fp3_linear_fused(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M,
                            int64_t N, int64_t K, const void *bias_f16, const void *residual_f16, int gated,
                            void *workspace, size_t workspace_bytes, void *stream);
fp6_status fp6g_linear_fused(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M,
                             int64_t N, int64_t K, int64_t group, const void *bias_f16, const void *residual_f16,
                             int gated, void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FP6_MI355X_H */
