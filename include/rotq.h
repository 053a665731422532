/*
 * rotq - online Hadamard rotate-and-quantize for MI355X (gfx950).
 *
 * C ABI of the inference-time hot path of rotation-based W/A/KV quantization
 * (arXiv 2504.13989): every token row is multiplied by a normalised Hadamard
 * matrix (section 2.3.2 Eq. 1 for orders 2^k; section 2.3.3 / Appendix B
 * Algorithm 2 for Paley orders; zero-padding of section 4.2 Eq. 2 when the row is
 * narrower than the order) and then quantized per token with the symmetric uniform
 * quantizer of section 2.1 under a clip ratio (section 3.1).
 *
 * Conventions
 *   - Order n = p * 2^k, where 2^k is the largest power of two for which p is 1 or a
 *     Paley order <= 256: p = q+1 with q prime, q = 3 (mod 4) (Algorithm 2), or
 *     p = 2(q+1) with q prime, q = 1 (mod 4) (Paley II; not in the paper, standard
 *     construction H = C (x) [[1,1],[1,-1]] + I (x) [[1,-1],[-1,-1]]).  Where both
 *     exist for one p the first is used.  n must be a multiple of 8 and at least 32 (packed rows are
 *     whole bytes); where no block of at most 256 exists a Paley block of up to 4096 is taken.  The
 *     fast kernels serve 16-bit rows of the orders rq_next_order returns (2^k >= 32, block <= 256);
 *     every other case (fp32 rows, unaligned rows, other orders) runs on a general kernel that
 *     keeps the row in the 160 KB of LDS, which bounds n: 2^15 for Sylvester orders and 20448 for
 *     block orders; fp32 rows are quantized from an fp64 copy of the row and stop at n = 2^14
 *     (Sylvester) and 9728 (block orders).  A row call on an order beyond what its kernels can hold
 *     returns RQ_ERR_NO_ORDER.
 *   - H_n = H_p (x) H_{2^k}: flat index j = a * 2^k + c (a < p, c < 2^k),
 *     H_n[i, j] = H_p[i / 2^k, j / 2^k] * (-1)^popcount((i % 2^k) & (j % 2^k)).
 *   - Rotated row: y = H_n pad(x) / sqrt(n), pad() appends n - d zeros.
 *   - Quantizer: amax = max_j |y_j|; Delta = clip * amax / (2^b - 1);
 *     code_j = clamp(round_half_even(y_j / Delta), -2^(b-1), 2^(b-1) - 1);
 *     amax == 0 gives Delta = 0 and all-zero codes.  Arithmetic is fp32.
 *   - Packed codes: row r starts at byte r * n * b / 8; element j of the rotated row is
 *     the b-bit field at bits [j*b, (j+1)*b) of the row's little-endian bit stream (stream
 *     bit i = bit i % 8 of byte i / 8), holding the code's low b bits (two's complement).
 *   - scales[r] = Delta of row r, so that y^_j = code_j * scales[r].
 *
 * All functions return RQ_OK (0) or a negative error code; none throws or aborts.
 * Argument errors are detected on the host before any HIP call.  Data values are not
 * validated (NaN / Inf propagate).  The hot-path calls enqueue work on the caller's
 * stream and return without synchronising and without allocating.
 */
#ifndef ROTQ_H
#define ROTQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RQ_OK             0
#define RQ_ERR_ARG       -1   /* bad pointer, size, stride, bit-width, clip, alignment, workspace */
#define RQ_ERR_NO_ORDER  -2   /* n has no supported factorisation p * 2^k, n % 8 != 0, or no kernel can hold a row of n */
#define RQ_ERR_HIP       -3   /* HIP allocation / launch failure, or the handle has no device table */
#define RQ_ERR_NOMEM     -4   /* host allocation failure */
#define RQ_ERR_TOO_LARGE -5   /* rq_quant_error_noalloc: rows * n_clips exceeds the static scratch buffer */

#define RQ_BF16 0             /* X elements are bfloat16 (2 bytes) */
#define RQ_F32  1             /* X elements are float (4 bytes) */
#define RQ_F16  2             /* IEEE half precision (2 bytes): rows of X, and results of rq_rotate / rq_dequantize_rotate */

#define RQ_KIND_SYLVESTER 0
#define RQ_KIND_PALEY1    1
#define RQ_KIND_PALEY2    2

#define RQ_MAX_CLIPS 64
#define RQ_GROUP 128

/* Opaque.  The factorisation and the device tables do not change after rq_hadamard_build, and the
 * row calls take the handle as const: one handle may serve any number of host threads and streams at
 * once.  Two fields are written later, both atomically: the kernel selector of
 * rq_hadamard_set_variant (a test hook; calls already running keep the kernel they chose) and the
 * diagnostic name read by rq_hadamard_last_kernel (the most recent call on any thread). */
typedef struct rq_hadamard rq_hadamard_t;

/*
 * Build the rotation of order n (sections 2.3.2, 2.3.3, Appendix B Algorithm 2): factor
 * n = p * 2^k, build the +-1 block H_p from Legendre symbols in integer arithmetic on the
 * host, and, when a GPU is present, upload the block tables to the current device.
 * Without a GPU the handle is host-only: the info/dense calls work, the hot-path calls
 * return RQ_ERR_HIP.
 * The largest 2^k is taken for which p is 1 or a Paley order of at most 256; where there is none, a
 * large Paley block of at most 4096 is used, up to the whole dimension (section 5.2.2:
 * 1544 = 1543 + 1).
 *   n    [in]  rotation order, multiple of 8 (packed rows are whole bytes)
 *   out  [out] host pointer receiving the handle; owned by the caller, released with
 *              rq_hadamard_free.  Untouched on error.
 * Errors: RQ_ERR_ARG (out NULL, n < 32), RQ_ERR_NO_ORDER (n not a multiple of 8, or no
 * factorisation), RQ_ERR_NOMEM, RQ_ERR_HIP.
 */
int rq_hadamard_build(int n, rq_hadamard_t** out);

/* Release a handle and its device tables (NULL is a no-op).  Work already enqueued that
 * uses the handle must have completed. */
void rq_hadamard_free(rq_hadamard_t* h);

/*
 * Factorisation held by a handle.  Any output pointer may be NULL.
 *   n      order;  p  block order (1 = pure Sylvester);  kind  RQ_KIND_*;
 *   q      the prime of the Paley construction (0 for Sylvester);  log2m  k.
 * Errors: RQ_ERR_ARG (h NULL).
 */
int rq_hadamard_info(const rq_hadamard_t* h, int* n, int* p, int* kind, int* q, int* log2m);

/*
 * Test hook: the dense un-normalised matrix H_n, n*n entries of +-1, row-major, written
 * to HOST memory host_out (caller-owned, n*n bytes).  Refused for n > 8192.
 * Errors: RQ_ERR_ARG.
 */
int rq_hadamard_dense(const rq_hadamard_t* h, int8_t* host_out);

/*
 * Dimension expansion helper (section 4.2): the smallest order n >= d that
 * rq_hadamard_build accepts with 2^k >= 32 and a block of at most 256 (the orders the fast
 * kernels serve).  n_out is a host pointer.
 * Errors: RQ_ERR_ARG (d < 1, n_out NULL), RQ_ERR_NO_ORDER (none below 2^30).
 */
int rq_next_order(int d, int* n_out);

/*
 * Rotate and quantize `rows` token rows (sections 2.1, 2.3, 3.1, 4.2; see Conventions).
 *   h       [in]  handle of order n >= d, with device tables on the current device
 *   X       [in]  DEVICE pointer, rows x d elements of `dtype`, row-major with leading
 *                 dimension ld >= d (in elements); aligned to the element size.  A row of
 *                 width d < n is treated as zero-padded to n.  Not modified.
 *   bits    [in]  3 or 4
 *   clip    [in]  clip ratio in (0, 1]
 *   codes   [out] DEVICE pointer, rows * n * bits / 8 bytes, 4-byte aligned, caller-owned
 *   scales  [out] DEVICE pointer, rows floats, caller-owned
 *   stream  [in]  hipStream_t (NULL = the null stream)
 * rows == 0 is a successful no-op (X, codes and scales may then be NULL).
 * Errors: RQ_ERR_ARG (NULL pointer, rows < 0, d < 1, d > n, ld < d, bits not 3/4, clip not in
 * (0,1] or NaN, misaligned pointer, unknown dtype), RQ_ERR_NO_ORDER (no kernel can hold a row of
 * this order and type, see Conventions), RQ_ERR_HIP.
 */
int rq_rotate_quantize(const rq_hadamard_t* h,
                       const void* X, int dtype, int64_t rows, int d, int64_t ld,
                       int bits, float clip,
                       void* codes, float* scales, void* stream);

/*
 * Rotate, then quantize asymmetrically in groups of RQ_GROUP consecutive rotated values (the
 * KV-cache setting of section 5.1: 3-bit asymmetric quantization with a group size of 128;
 * rotation as in sections 2.3, 4.2).  The paper names the scheme without a formula; per group g
 * of the rotated row y:
 *   lo = clip * min(y_g), hi = clip * max(y_g), Delta = (hi - lo) / (2^b - 1),
 *   code_j = clamp(round_half_even((y_j - lo) / Delta), 0, 2^b - 1),  y^_j = code_j * Delta + lo.
 * A constant group has Delta = 0 and all-zero codes.
 *   h       [in]  handle whose order n is a multiple of RQ_GROUP
 *   codes   [out] DEVICE, rows * n * bits / 8 bytes: unsigned b-bit fields, bitstream layout as
 *                 in rq_rotate_quantize
 *   scales  [out] DEVICE, rows * (n / RQ_GROUP) floats: Delta, row-major [row][group]
 *   mins    [out] DEVICE, rows * (n / RQ_GROUP) floats: lo
 * Other arguments, ownership and the rows == 0 rule as in rq_rotate_quantize.
 * Errors: RQ_ERR_ARG (as rq_rotate_quantize, or n not a multiple of RQ_GROUP), RQ_ERR_NO_ORDER
 * (no kernel can hold a row of this order), RQ_ERR_HIP.
 */
int rq_rotate_quantize_asym(const rq_hadamard_t* h,
                            const void* X, int dtype, int64_t rows, int d, int64_t ld,
                            int bits, float clip,
                            void* codes, float* scales, float* mins, void* stream);

/*
 * Measurement aid (no operation of the paper): a kernel with the memory traffic of
 * rq_rotate_quantize on 16-bit rows of width n and no arithmetic - it reads every row with the same
 * loads and writes n * bits / 8 bytes of codes and one float per row (an xor fold of the input, not
 * a quantization).  Its duration is the practical floor for a rotate_quantize launch of that shape
 * on this chip; bench.py reports it next to the real kernel.
 *   X       [in]  DEVICE, rows x n 16-bit elements, leading dimension ld >= n (a multiple of 8),
 *                 16-byte aligned
 *   n       [in]  a multiple of 512, at most 8192
 *   codes   [out] DEVICE, rows * n * bits / 8 bytes, 4-byte aligned;  scales [out] DEVICE, rows floats
 * Errors: RQ_ERR_ARG, RQ_ERR_HIP.
 */
int rq_stream_reference(const void* X, int64_t rows, int n, int64_t ld, int bits, void* codes,
                        float* scales, void* stream);

/*
 * The per-token symmetric quantizer of section 2.1 (with the clip ratio of section 3.1) on the
 * rows as they are, without a rotation: for activations whose rotation has been fused into the
 * neighbouring weights offline (section 2.2), so that only the quantizer remains online.
 *   X       [in]  DEVICE, rows x d elements of `dtype`, leading dimension ld >= d
 *   d       [in]  row width, a multiple of 32
 *   codes   [out] DEVICE, rows * d * bits / 8 bytes, 4-byte aligned (signed fields, same layout)
 *   scales  [out] DEVICE, rows floats: Delta = clip * max|x| / (2^b - 1)
 * Runs on the current device.  rows == 0 is a successful no-op.
 * Errors: RQ_ERR_ARG, RQ_ERR_HIP.
 */
int rq_quantize(const void* X, int dtype, int64_t rows, int d, int64_t ld,
                int bits, float clip, void* codes, float* scales, void* stream);

/*
 * The asymmetric group quantizer of rq_rotate_quantize_asym on the rows as they are, without a
 * rotation (section 5.1 for a tensor whose rotation is fused into the producing weights, e.g. the
 * value cache): per group of RQ_GROUP consecutive values lo = clip * min, hi = clip * max,
 * Delta = (hi - lo) / (2^b - 1), code = clamp(round((x - lo) / Delta), 0, 2^b - 1).
 *   X       [in]  DEVICE, rows x d elements of `dtype`, leading dimension ld >= d
 *   d       [in]  row width, a multiple of RQ_GROUP
 *   codes   [out] DEVICE, rows * d * bits / 8 bytes, 4-byte aligned (unsigned fields, same bit stream)
 *   scales  [out] DEVICE, rows * d / RQ_GROUP floats: Delta of each group
 *   mins    [out] DEVICE, rows * d / RQ_GROUP floats: lo of each group
 * Runs on the current device.  rows == 0 is a successful no-op.
 * Errors: RQ_ERR_ARG, RQ_ERR_HIP.
 */
int rq_quantize_asym(const void* X, int dtype, int64_t rows, int d, int64_t ld,
                     int bits, float clip, void* codes, float* scales, float* mins, void* stream);

/*
 * Rotation alone with a floating-point result: Y = (H_n pad(x) / sqrt(n))[:d_out] for every row,
 * or with H_n^T when transpose = 1.  Three uses:
 *   - the online rotation of a tensor that is not quantized afterwards (section 2.2: the part of
 *     the rotations that "needs to be done at inference"), e.g. the query heads, which must carry
 *     the same per-head rotation as the keys that go into the quantized cache;
 *   - offline weight fusion (section 4.2, Eq. 2): W' = H_n pad(W) / sqrt(n) is this call on the
 *     rows of W^T (input side) or of W (output side), so that rotate(x) W' = x W;
 *   - the inverse rotation x = H_n^T y / sqrt(n) (H_n^T H_n = n I, section 2.3) with
 *     transpose = 1 and d_out = the un-padded width.
 *   X        [in]  DEVICE, rows x d, leading dimension ld, `dtype` (as rq_rotate_quantize)
 *   Y        [out] DEVICE, rows x d_out elements of out_dtype (RQ_F32, or RQ_BF16 / RQ_F16 rounded
 *                  to nearest even), leading dimension ld_out >= d_out; 1 <= d_out <= n
 * rows == 0 is a successful no-op.
 * Errors: RQ_ERR_ARG, RQ_ERR_NO_ORDER (the row does not fit the kernel's LDS), RQ_ERR_HIP.
 */
int rq_rotate(const rq_hadamard_t* h, const void* X, int dtype, int64_t rows, int d, int64_t ld,
              int transpose, void* Y, int out_dtype, int d_out, int64_t ld_out, void* stream);

/*
 * Dequantize packed codes and rotate back (the inverse of rq_rotate_quantize up to the
 * quantization error): y^ = code * Delta (mins == NULL, signed codes) or code * Delta_g + lo_g
 * (mins != NULL, unsigned codes in groups of RQ_GROUP as written by rq_rotate_quantize_asym),
 * then Y = (H_n^T y^ / sqrt(n))[:d_out] with transpose = 1 (transpose = 0 applies H_n).
 *   codes, scales, mins [in] DEVICE, layouts as the quantizing calls write them
 *   Y                   [out] as in rq_rotate
 * Errors: RQ_ERR_ARG, RQ_ERR_NO_ORDER, RQ_ERR_HIP.
 */
int rq_dequantize_rotate(const rq_hadamard_t* h, const void* codes, const float* scales,
                         const float* mins, int64_t rows, int bits, int transpose,
                         void* Y, int out_dtype, int d_out, int64_t ld_out, void* stream);

/*
 * Dequantize in the rotated, normalised domain (section 2.1: X^ = round(X / Delta) * Delta), no
 * rotation: Y[r, j] = code_j * scales[r] for the signed codes rq_rotate_quantize / rq_quantize write.
 *   h       [in]  handle of the order n the codes were written with (n codes per row)
 *   codes   [in]  DEVICE, rows * n * bits / 8 bytes, 4-byte aligned
 *   scales  [in]  DEVICE, rows floats
 *   Y       [out] DEVICE, rows x n floats, row-major, leading dimension n, 4-byte aligned, caller-owned
 * The product is a single fp32 multiplication.  rows == 0 is a successful no-op.
 * Errors: RQ_ERR_ARG (NULL or misaligned pointer, rows < 0, bits not 3/4), RQ_ERR_HIP.
 */
int rq_dequantize(const rq_hadamard_t* h, const void* codes, const float* scales, int64_t rows, int bits,
                  float* Y, void* stream);

/*
 * The same for the unsigned group codes of rq_rotate_quantize_asym / rq_quantize_asym (section 5.1):
 * Y[r, j] = code_j * scales[r, g] + mins[r, g], g = j / RQ_GROUP, one fused multiply-add.
 *   scales, mins [in] DEVICE, rows * (n / RQ_GROUP) floats each
 * Errors: RQ_ERR_ARG (as rq_dequantize, or n not a multiple of RQ_GROUP), RQ_ERR_HIP.
 */
int rq_dequantize_asym(const rq_hadamard_t* h, const void* codes, const float* scales, const float* mins,
                       int64_t rows, int bits, float* Y, void* stream);

/*
 * Lemma "Expanding limit" (section 4.2): the largest number of added dimensions d for which a
 * product over n + d dimensions at bits_reduced bits costs no more bit operations than the
 * product over n dimensions at `bits` bits: (n + d) * bits_reduced <= n * bits, i.e.
 * floor(n (bits - bits_reduced) / bits_reduced).  Host-only; d_max is a HOST pointer.
 * Errors: RQ_ERR_ARG (n < 1, bits_reduced < 1, bits_reduced > bits, bits > 64, NULL).
 */
int rq_expand_limit(int n, int bits, int bits_reduced, int64_t* d_max);

/* Bytes of device workspace rq_quant_error needs for (rows, n_clips); 0 on bad arguments. */
size_t rq_quant_error_workspace(int64_t rows, int n_clips);

/*
 * Quantization error of the rotated rows for several clip ratios in one pass (the
 * objective a clip-ratio search evaluates repeatedly; sections 3.1, 4.1):
 *   mse[k] = (1 / (rows * n)) * sum over rows, j of (code_j * Delta_k - y_j)^2,
 * with y, Delta_k = clips[k] * amax / (2^b - 1) and code_j as in rq_rotate_quantize.
 *   clips     [in]  HOST pointer, n_clips floats in (0, 1]; read before the call returns
 *   n_clips   [in]  1 .. RQ_MAX_CLIPS
 *   mse       [out] DEVICE pointer, n_clips floats, caller-owned
 *   workspace [in]  DEVICE pointer, at least rq_quant_error_workspace(rows, n_clips) bytes,
 *                   8-byte aligned, caller-owned; contents are scratch
 * Other arguments as in rq_rotate_quantize.  rows == 0 writes zeros to mse (X may then be NULL).
 * The result is deterministic (fixed reduction order).
 * Errors: RQ_ERR_ARG (as above, n_clips out of range, a clip not in (0,1], workspace too small
 * or misaligned), RQ_ERR_NO_ORDER (as rq_rotate_quantize), RQ_ERR_HIP.
 */
int rq_quant_error(const rq_hadamard_t* h,
                   const void* X, int dtype, int64_t rows, int d, int64_t ld, int bits,
                   const float* clips, int n_clips,
                   float* mse, void* workspace, size_t workspace_bytes, void* stream);

/*
 * rq_quant_error with the asymmetric group quantizer of rq_rotate_quantize_asym (sections 4.1, 5.1:
 * the objective of a clip search on the KV cache): mse[k] = (1 / (rows * n)) * sum of
 * (code * Delta_g + lo_g - y)^2 at clip ratio clips[k].  The order n must be a multiple of RQ_GROUP.
 * Arguments, workspace size (rq_quant_error_workspace) and errors as rq_quant_error.
 */
int rq_quant_error_asym(const rq_hadamard_t* h,
                        const void* X, int dtype, int64_t rows, int d, int64_t ld, int bits,
                        const float* clips, int n_clips,
                        float* mse, void* workspace, size_t workspace_bytes, void* stream);

/*
 * For callers that cannot allocate device memory - code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc: rq_quant_error without a workspace argument.  The per-row
 * partial sums go to a static device array of RQ_NOALLOC_SCRATCH_BYTES that every GPU the library runs
 * on holds until the process ends (its address on the handle's device is taken when the handle is
 * built).  The call allocates nothing and frees nothing; same kernels and same results as
 * rq_quant_error.
 *   limit: rq_quant_error_workspace(rows, n_clips) <= RQ_NOALLOC_SCRATCH_BYTES, i.e.
 *          rows * n_clips <= 524288 (e.g. 8192 rows x 64 clip ratios); beyond it RQ_ERR_TOO_LARGE.
 * All calls on one GPU share the array: calls that may overlap in time on that GPU (different
 * streams, or different host threads) race on it and must be ordered by the caller.  The handle's
 * device must be the current device.
 * Other arguments and errors as rq_quant_error.
 */
#define RQ_NOALLOC_SCRATCH_BYTES (4u << 20)
int rq_quant_error_noalloc(const rq_hadamard_t* h,
                           const void* X, int dtype, int64_t rows, int d, int64_t ld, int bits,
                           const float* clips, int n_clips, float* mse, void* stream);

/* Bytes of device workspace rq_gbs_search needs for `rows` rows; 0 on bad arguments. */
size_t rq_gbs_workspace(int64_t rows);

/*
 * Clip-ratio search for one projection: the inner loop of the Gradual Binary Search
 * (section 4.1, Algorithm 1) with f(clip) = rq_quant_error of X at that single clip ratio as
 * the objective (the paper's objective, perplexity of a model, is not available here).
 * a = 0, b = 1, m = 1/2; iterations alternate the probes (a + m)/2 and (b + m)/2; a probe with
 * f(x) < f(m) becomes the new middle and the far bracket end moves to the old middle, otherwise
 * the bracket end on the probe's side moves to the probe; stops when b - a <= eps or after
 * max_evals evaluations of f.  The probes and their values are those of that loop taken one at a
 * time; they are evaluated ahead in batches (one rq_quant_error launch covers every probe the next
 * few steps can ask for, whatever the comparisons give), each batch followed by a synchronisation of
 * `stream`: a calibration call, not a hot-path call.  The values of a batch come back through 256
 * bytes of pinned host memory that the library allocates at the first search of a host thread on a
 * device and keeps until the process ends (copied back on `stream` instead where that allocation
 * fails); nothing else is allocated.
 *   eps          [in]  bracket width to stop at, > 0
 *   max_evals    [in]  1 .. 256
 *   workspace    [in]  DEVICE, >= rq_gbs_workspace(rows) bytes, 8-byte aligned, scratch
 *   clip_out     [out] HOST, the final middle m
 *   mse_out      [out] HOST, f(m)
 *   trace_clips  [out] HOST, max_evals floats or NULL: the probes in evaluation order
 *   trace_mse    [out] HOST, max_evals floats or NULL: f at those probes
 *   n_evals      [out] HOST or NULL: number of evaluations made
 * X, dtype, rows (>= 1), d, ld, bits as in rq_rotate_quantize.
 * Errors: RQ_ERR_ARG, RQ_ERR_NO_ORDER, RQ_ERR_HIP.
 */
int rq_gbs_search(const rq_hadamard_t* h, const void* X, int dtype, int64_t rows, int d, int64_t ld,
                  int bits, float eps, int max_evals, void* workspace, size_t workspace_bytes,
                  void* stream, float* clip_out, float* mse_out, float* trace_clips,
                  float* trace_mse, int* n_evals);

/* rq_gbs_search with rq_quant_error_asym as the objective (n a multiple of RQ_GROUP). */
int rq_gbs_search_asym(const rq_hadamard_t* h, const void* X, int dtype, int64_t rows, int d, int64_t ld,
                       int bits, float eps, int max_evals, void* workspace, size_t workspace_bytes,
                       void* stream, float* clip_out, float* mse_out, float* trace_clips,
                       float* trace_mse, int* n_evals);

/*
 * Select the kernel family for subsequent hot-path calls on this handle (testing /
 * measurement): 0 = automatic (fastest available), 1 = the general LDS kernel; for long
 * power-of-two rows 2 = one wave per row at any row count, 3 / 4 = a row split over 2 / 4 waves
 * at any row count (automatic picks by the number of rows).
 * Errors: RQ_ERR_ARG.
 */
int rq_hadamard_set_variant(rq_hadamard_t* h, int variant);

/* Name of the kernel family the last hot-path call on this handle used ("" if none). */
const char* rq_hadamard_last_kernel(const rq_hadamard_t* h);

/* Static description of an error code. */
const char* rq_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* ROTQ_H */
