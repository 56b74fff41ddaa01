/*
 * ptq4vm.h - C ABI of the MI355X (gfx950) quantized-linear library for PTQ4VM
 * ("Post-Training Quantization for Visual Mamba", arXiv 2412.20386).
 *
 * The library runs the paper's W8A8 linear layer with Per-Token Static (PTS) activation
 * quantization (Sec. 5.1) and SmoothQuant-style smoothing (Sec. 2.4), i.e. the four stages of
 * the paper's acceleration kernel (App. B.1: activation smoothing, quantization, INT GEMM,
 * dequantization) as two fused launches, plus the offline weight preparation and an FP16
 * linear used as the comparison baseline of the paper's latency table.
 *
 * Conventions shared by every entry point
 *   - Storage is token-major: activations X[B*L, K], weights W[N, K] (same as a framework's
 *     linear.weight and as the paper's W-bar in R^{Dout x Din}), outputs Y[B*L, N]; all
 *     row-major, leading dimensions (ld*) counted in ELEMENTS and >= the row width.  Row r
 *     belongs to token position t = r mod L.  The paper writes activations as Din x L
 *     (token = column); this is the transpose, so diag(Delta_X) scales rows of Y and
 *     diag(Delta_W) scales its columns.
 *   - Every pointer is DEVICE memory owned by the caller.  The library allocates nothing,
 *     keeps no state between calls and never synchronises: work is enqueued on `stream`
 *     (a hipStream_t passed as void*, NULL = the default stream) and the call returns at once.
 *     Inputs are only read; outputs must not overlap inputs.  fp16 buffers are passed as
 *     void* (IEEE binary16).  A matrix buffer must span rows * ld elements (the last row's
 *     padding up to its pitch included): vector loads may touch the padding of a row.
 *   - Alignment: base pointers of fp16 and int8 matrices must be 16-byte aligned, float
 *     vectors 4-byte aligned (else PTQ4VM_ERR_ALIGN).  Rows need not be 16-byte multiples
 *     (K = 12 with ld = 12, N = 44 with ld = 44 are valid); rows whose byte pitch is a multiple
 *     of 16 take the fastest loads and stores.
 *   - Return value: PTQ4VM_OK (0) or a negative ptq4vm_status.  All argument checks run on the
 *     host before any launch.  A problem with zero rows or zero output columns is PTQ4VM_OK and
 *     launches nothing.  Device-side values (steps <= 0, NaN scales) are the caller's
 *     responsibility and are not inspected on the hot path; ptq4vm_validate_scales checks them on
 *     request.
 */
#ifndef PTQ4VM_H
#define PTQ4VM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PTQ4VM_OK = 0,
    PTQ4VM_ERR_NULL = -1,   /* a required pointer is NULL */
    PTQ4VM_ERR_SHAPE = -2,  /* a size is negative, zero where it must not be, or too large */
    PTQ4VM_ERR_STRIDE = -3, /* a leading dimension is smaller than the row width */
    PTQ4VM_ERR_ALIGN = -4,  /* a base pointer is not aligned as stated above */
    PTQ4VM_ERR_HIP = -5,    /* the HIP runtime refused a launch; see ptq4vm_last_hip_error() */
    PTQ4VM_ERR_VALUE = -6   /* ptq4vm_validate_scales found a scale that is not a finite number > 0 */
} ptq4vm_status;

/* Largest K for which sum_k (+-127)(+-127) is guaranteed to fit int32: floor((2^31-1)/127^2). */
#define PTQ4VM_MAX_K 133143

/*
 * Offline weight preparation: fold the smoothing vector into the weight (Eq. (smooth),
 * Sec. 2.4: Y = (W diag(s)) (diag(s)^-1 X)), then quantize each OUTPUT channel symmetrically to
 * 8 bits (Sec. 2.3, Delta_W = max|W| / (2^(b-1) - 1), codes clipped to [-127, 127]; Sec. 5.1:
 * Delta_W is per output channel).
 *   w_f16 [N, ldw]  fp16 in   unsmoothed weight
 *   m     [K]       f32  in   smoothing vector s of the paper, every entry > 0
 *   wq    [N, ldwq] int8 out  wq[o,k] = clip(rne(W'[o,k] / s_w[o]), -127, 127), W' = f32(W)*m[k]
 *   s_w   [N]       f32  out  max_k |W'[o,k]| / 127, or 1 for an all-zero row
 *   inv_m [K]       f32  out  1 / m[k] (correctly rounded), what the activation side multiplies by
 * All arithmetic is fp32 with IEEE division; rounding is to nearest, ties to even.
 * Errors: NULL pointer, N < 0 or K <= 0, ld* < K, misaligned w_f16 / wq.
 */
int ptq4vm_fold_smoothing(const void *w_f16, const float *m, int8_t *wq, float *s_w, float *inv_m,
                          int64_t N, int64_t K, int64_t ldw, int64_t ldwq, void *stream);

/*
 * Per-Token Static activation quantizer (Sec. 5.1) with the activation-smoothing multiply
 * fused in front (App. B.1 "Activation smoothing" + "Quantization"):
 *   xq[r,k] = clip(rne((f32(x[r,k]) * inv_m[k]) * (1 / s_tok[r mod L])), -127, 127)
 * evaluated in fp32 in exactly this order, 1/s_tok correctly rounded, ties to even; the zero
 * offset is omitted as in the paper's PTS equation.  NaN quantizes to 0, +-Inf to +-127.
 *   x_f16 [B*L, ldx]  fp16 in
 *   inv_m [K]         f32  in   may be NULL (no smoothing, all ones)
 *   s_tok [L]         f32  in   static step per token position (Delta_X in R^{1 x L}), > 0
 *   xq    [B*L, ldxq] int8 out
 * Errors: NULL x_f16 / s_tok / xq, B < 0 or L <= 0 or K <= 0, ld* < K, misaligned x_f16 / xq.
 */
int ptq4vm_quantize_pts(const void *x_f16, const float *inv_m, const float *s_tok, int8_t *xq,
                        int64_t B, int64_t L, int64_t K, int64_t ldx, int64_t ldxq, void *stream);

/*
 * Per-token dynamic activation quantizer: the comparison scheme of Sec. 4 and of the "Per-token
 * dynamic" rows of the latency table (Sec. 6.4, Computation Acceleration).  The step of every token row is computed online
 * from the row itself, after smoothing (fp32, in this order):
 *   v[k] = f32(x[r,k]) * inv_m[k];  s_row[r] = max_k |v[k]| / 127  (1 for an all-zero row; NaNs
 *   do not take part in the maximum);  xq[r,k] = clip(rne(v[k] * (1 / s_row[r])), -127, 127).
 * The linear that follows is ptq4vm_w8a8_linear(..., s_tok = s_row, B = 1, L = M).
 *   x_f16 [M, ldx] fp16 in;  inv_m [K] f32 in, may be NULL;  xq [M, ldxq] int8 out;  s_row [M] f32 out
 * Errors: NULL x_f16 / xq / s_row, M < 0, K <= 0, ld* < K, misaligned x_f16 / xq (16 bytes).
 */
int ptq4vm_quantize_dynamic(const void *x_f16, const float *inv_m, int8_t *xq, float *s_row, int64_t M,
                            int64_t K, int64_t ldx, int64_t ldxq, void *stream);

/*
 * W8A8 linear: integer GEMM and fused dequantization (PTS equation of Sec. 5.1,
 * Y ~= diag(Delta_W) (W-bar X-bar) diag(Delta_X); App. B.1 "INT GEMM" + "Dequantization"):
 *   acc[r,o] = sum_k xq[r,k] * wq[o,k]                                   (exact, int32)
 *   y[r,o]   = fp16( f32(acc[r,o]) * (s_tok[r mod L] * s_w[o]) + f32(bias[o]) )   (fp32)
 * The step-size outer product is never materialised.
 *   xq       [B*L, ldxq] int8 in
 *   wq       [N, ldwq]   int8 in
 *   s_tok    [L]         f32  in
 *   s_w      [N]         f32  in
 *   bias_f16 [N]         fp16 in   may be NULL
 *   y_f16    [B*L, ldy]  fp16 out
 *   acc_out  [B*L, N]    int32 out, dense; may be NULL.  Exists so that the exact accumulators
 *                        can be compared with a reference; leave NULL when timing.
 * Errors: NULL xq / wq / s_tok / s_w / y_f16, B < 0, N < 0, L <= 0, K <= 0, K > PTQ4VM_MAX_K,
 * ld* too small, misaligned xq / wq / y_f16 (y_f16 needs only 2-byte alignment; 16 is faster).
 */
int ptq4vm_w8a8_linear(const int8_t *xq, const int8_t *wq, const float *s_tok, const float *s_w,
                       const void *bias_f16, void *y_f16, int32_t *acc_out, int64_t B, int64_t L,
                       int64_t K, int64_t N, int64_t ldxq, int64_t ldwq, int64_t ldy, void *stream);

/*
 * PTS with a per-token zero offset.  Sec. 5.1 gives every token position a zero offset next to its
 * step size and then leaves the offset out of its equation; the offset form is the activation quantizer
 * of Sec. 2.3, clip(round(X / Delta) + eps, 0, 2^b - 1), here with the code range shifted by 128
 * so that codes are int8 (z_tok = eps - 128):
 *   xq[r,k] = clip(rne((f32(x[r,k]) * inv_m[k]) * (1 / s_tok[t])) + z_tok[t], -128, 127),  t = r mod L
 *   x-hat   = s_tok[t] * (xq - z_tok[t])
 *   y[r,o]  = fp16( f32(acc[r,o] - z_tok[t] * rowsum[o]) * (s_tok[t] * s_w[o]) + f32(bias[o]) ),
 *             acc = sum_k xq[r,k] wq[o,k],  rowsum[o] = sum_k wq[o,k]
 * ptq4vm_weight_rowsum prepares rowsum once per weight (offline, like the fold).
 * Arguments as in ptq4vm_quantize_pts / ptq4vm_w8a8_linear, plus z_tok [L] int32 in (values in
 * [-128, 127]) and rowsum [N] int32.  acc_out receives the raw accumulators (before the correction).
 * K <= PTQ4VM_MAX_K_OFFSET keeps acc - z * rowsum inside int32 and |rowsum| <= 128 K inside 24 signed
 * bits: the kernels form z * rowsum with a 24-bit multiply, so z_tok outside [-128, 127] or a rowsum
 * that is not the weight's row sum gives undefined results (not checked).  Runs on the same tiled,
 * persistent and short-reduction kernels as ptq4vm_w8a8_linear.
 */
#define PTQ4VM_MAX_K_OFFSET 65536
int ptq4vm_quantize_pts_offset(const void *x_f16, const float *inv_m, const float *s_tok, const int32_t *z_tok,
                               int8_t *xq, int64_t B, int64_t L, int64_t K, int64_t ldx, int64_t ldxq, void *stream);
int ptq4vm_weight_rowsum(const int8_t *wq, int32_t *rowsum, int64_t N, int64_t K, int64_t ldwq, void *stream);
int ptq4vm_w8a8_linear_offset(const int8_t *xq, const int8_t *wq, const float *s_tok, const int32_t *z_tok,
                              const int32_t *rowsum, const float *s_w, const void *bias_f16, void *y_f16,
                              int32_t *acc_out, int64_t B, int64_t L, int64_t K, int64_t N, int64_t ldxq,
                              int64_t ldwq, int64_t ldy, void *stream);

/*
 * W4A4: the precision of the paper's latency table (Sec. 6.4, Computation Acceleration).  Codes are clipped to +-7
 * (Sec. 2.3, +-(2^(b-1) - 1) with b = 4) and packed two per byte, the even reduction index in the
 * low nibble, the odd one in the high nibble, two's complement (the packing of App. B.1).  K must be
 * even; packed matrices are [rows, K / 2] bytes with pitches ldwq / ldxq in bytes.
 *   ptq4vm_fold_smoothing_w4  as ptq4vm_fold_smoothing with s_w = max|W'| / 7
 *   ptq4vm_quantize_pts_a4    as ptq4vm_quantize_pts with the +-7 clip (s_tok calibrated for 4 bits)
 *   ptq4vm_w4a4_linear        as ptq4vm_w8a8_linear on packed operands; acc_out holds sum_k xq wq
 * gfx950 has no int4 MFMA: packed operands are expanded in registers to int8 right before the
 * int8 MFMA, so the gain over W8A8 is in bytes moved, not in MFMA rate.  The linear runs on the
 * tiled, persistent (128-row tiles) and short-reduction kernels of ptq4vm_w8a8_linear.  Errors as
 * for the 8-bit entry points, plus odd K -> PTQ4VM_ERR_SHAPE and K > PTQ4VM_MAX_K_W4 ->
 * PTQ4VM_ERR_SHAPE: the kernels multiply codes scaled by 16, so the int32 accumulator holds 256 times
 * the sum, and with the nibble -8 accepted on input (the quantizers never emit it) |256 acc| can reach
 * 2^14 K, which must stay below 2^31.
 */
#define PTQ4VM_MAX_K_W4 131071
int ptq4vm_fold_smoothing_w4(const void *w_f16, const float *m, uint8_t *wq4, float *s_w, float *inv_m,
                             int64_t N, int64_t K, int64_t ldw, int64_t ldwq, void *stream);
int ptq4vm_quantize_pts_a4(const void *x_f16, const float *inv_m, const float *s_tok, uint8_t *xq4, int64_t B,
                           int64_t L, int64_t K, int64_t ldx, int64_t ldxq, void *stream);
int ptq4vm_w4a4_linear(const uint8_t *xq4, const uint8_t *wq4, const float *s_tok, const float *s_w,
                       const void *bias_f16, void *y_f16, int32_t *acc_out, int64_t B, int64_t L, int64_t K,
                       int64_t N, int64_t ldxq, int64_t ldwq, int64_t ldy, void *stream);

/*
 * W4A4 on the FP6 matrix path.  The same 4-bit codes (clip +-7, Sec. 2.3; the precision of the latency table,
 * Sec. 6.4) stored as FP6 "E2M3" numbers (1 sign, 2 exponent, 3 mantissa bits, exponent bias 1), a format that
 * holds every integer -7..7 exactly and that gfx950's v_mfma_f32_16x16x128_f8f6f4 multiplies at twice the
 * int8 MFMA rate.  Products and partial sums are integers below 2^24 for K <= PTQ4VM_MAX_K_E2M3, so the fp32
 * accumulators hold sum_k xq wq of App. B.1 "INT GEMM" exactly and the outputs equal those of
 * ptq4vm_w4a4_linear on the same codes.
 * Container (xq6, wq6) of a matrix of R rows: a row of K codes is zero padded to PTQ4VM_E2M3_BLOCKS(K) blocks of
 * 128 codes, each block 96 bytes.  In a block, group g = 0..3 holds codes 32 g .. 32 g + 31 as a 192-bit
 * little-endian string, code j of the group at bits [6 j, 6 j + 6); the string's first 16 bytes sit at block
 * offset 16 g, its last 8 bytes at block offset 64 + 8 g.  Storage is block-major: block b of row r starts at
 * byte b * pitch + 96 r, where the plane pitch (ldxq / ldwq, in bytes) is at least 96 R and a multiple of 16 -
 * what a tile of the linear reads per block, and what the quantizer writes per 16 rows, is one contiguous span.
 * The pattern of an integer v is its E2M3 encoding with zero written as 0 (never as "-0"); patterns of padding
 * codes must be 0, and patterns that are not one of these 15 give undefined results in the linear (not checked).
 *   ptq4vm_fold_smoothing_w4_e2m3  as ptq4vm_fold_smoothing_w4, codes to wq6 (R = N)
 *   ptq4vm_quantize_pts_a4_e2m3    as ptq4vm_quantize_pts_a4, codes to xq6 (R = B*L)
 *   ptq4vm_w4a4_linear_e2m3        as ptq4vm_w4a4_linear on these containers; acc_out holds sum_k xq wq (int32)
 * xq6 / wq6 are 16-byte aligned; any K >= 1 (odd K too).  Errors as for the 4-bit entry points, with
 * K > PTQ4VM_MAX_K_E2M3 -> PTQ4VM_ERR_SHAPE and a plane pitch below 96 R or not a multiple of 16 -> PTQ4VM_ERR_STRIDE.
 * The linear runs on a persistent 256 x 256-tile kernel (K a multiple of 128 and >= 256, N a multiple of 8,
 * 16-byte aligned y rows, enough tiles to fill the device) or on a small tiled kernel (every other shape).
 */
#define PTQ4VM_E2M3_BLOCKS(K) ((((int64_t)(K)) + 127) / 128)
#define PTQ4VM_MAX_K_E2M3 262144
int ptq4vm_fold_smoothing_w4_e2m3(const void *w_f16, const float *m, uint8_t *wq6, float *s_w, float *inv_m,
                                  int64_t N, int64_t K, int64_t ldw, int64_t ldwq, void *stream);
int ptq4vm_quantize_pts_a4_e2m3(const void *x_f16, const float *inv_m, const float *s_tok, uint8_t *xq6, int64_t B,
                                int64_t L, int64_t K, int64_t ldx, int64_t ldxq, void *stream);
int ptq4vm_w4a4_linear_e2m3(const uint8_t *xq6, const uint8_t *wq6, const float *s_tok, const float *s_w,
                            const void *bias_f16, void *y_f16, int32_t *acc_out, int64_t B, int64_t L, int64_t K,
                            int64_t N, int64_t ldxq, int64_t ldwq, int64_t ldy, void *stream);

/*
 * Fused activation quantizer + W8A8 linear: the stages "Activation smoothing", "Quantization",
 * "INT GEMM" and "Dequantization" of App. B.1 in one launch (PTS equation of Sec. 5.1).
 * Computes exactly, bit for bit, what ptq4vm_quantize_pts followed by ptq4vm_w8a8_linear
 * compute; the int8 codes stay on chip.  Worth using over many rows when the output is narrow
 * (N <= 128 over >= 4096 rows, e.g. x_proj: every activation element is read and quantized once)
 * or the reduction short (K <= 128 over >= 16384 rows, e.g. dt_proj); for wide outputs a tiled GEMM
 * would re-quantize each element once per tile column and below ~2000 rows only that tiled kernel
 * applies: the two separate calls are faster there, but every shape is accepted.
 *   x_f16    [B*L, ldx]  fp16 in
 *   inv_m    [K]         f32  in   may be NULL (no smoothing)
 *   s_tok    [L]         f32  in
 *   wq       [N, ldwq]   int8 in
 *   s_w      [N]         f32  in
 *   bias_f16 [N]         fp16 in   may be NULL
 *   y_f16    [B*L, ldy]  fp16 out
 *   acc_out  [B*L, N]    int32 out, dense; may be NULL (parity aid, leave NULL when timing)
 *   xq_out   [B*L, ldxq] int8 out; may be NULL (parity aid: the codes the GEMM consumed)
 * Errors: NULL x_f16 / s_tok / wq / s_w / y_f16, B < 0, N < 0, L <= 0, K <= 0, K > PTQ4VM_MAX_K,
 * ld* too small, misaligned x_f16 / wq (16 bytes) or y_f16 (2 bytes).
 */
int ptq4vm_w8a8_linear_fused(const void *x_f16, const float *inv_m, const float *s_tok, const int8_t *wq,
                             const float *s_w, const void *bias_f16, void *y_f16, int32_t *acc_out,
                             int8_t *xq_out, int64_t B, int64_t L, int64_t K, int64_t N, int64_t ldx,
                             int64_t ldwq, int64_t ldy, int64_t ldxq, void *stream);

/*
 * Fused activation quantizer + W4A4 linear: ptq4vm_quantize_pts_a4 followed by ptq4vm_w4a4_linear in one launch
 * (the four stages of App. B.1 at the precision of the latency table, Sec. 6.4); the 4-bit codes stay on chip.  Same
 * codes and accumulators as the two calls, bit for bit.  Arguments as ptq4vm_w8a8_linear_fused, except
 *   wq4      [N, ldwq]   packed 4-bit codes in (two per byte, even index in the low nibble; ldwq in bytes >= K / 2)
 *   s_tok    [L]         the 4-bit steps
 *   xq_out   [B*L, ldxq] int8 out; may be NULL (parity aid: the 4-bit codes the GEMM consumed, ONE per byte)
 * Runs on the weight-resident kernel (N <= 128, K a multiple of 64, >= 2048 rows, 16-byte aligned rows of x and
 * wq4) and on the row-streaming kernel (K <= 128, >= 1024 rows): the shapes where fusing pays (x_proj, dt_proj).
 * Every other shape returns PTQ4VM_ERR_SHAPE - call ptq4vm_quantize_pts_a4 and ptq4vm_w4a4_linear there.
 * Errors otherwise as ptq4vm_w4a4_linear / ptq4vm_w8a8_linear_fused (odd K, K > PTQ4VM_MAX_K_W4 -> PTQ4VM_ERR_SHAPE).
 */
int ptq4vm_w4a4_linear_fused(const void *x_f16, const float *inv_m, const float *s_tok, const uint8_t *wq4,
                             const float *s_w, const void *bias_f16, void *y_f16, int32_t *acc_out,
                             int8_t *xq_out, int64_t B, int64_t L, int64_t K, int64_t N, int64_t ldx,
                             int64_t ldwq, int64_t ldy, int64_t ldxq, void *stream);

/*
 * Fused zero-offset form: ptq4vm_quantize_pts_offset followed by ptq4vm_w8a8_linear_offset in one launch (Sec. 5.1: a
 * zero offset per token position next to its step; the quantizer of Sec. 2.3 in the loader of the linear).  Same codes,
 * accumulators and outputs as the two calls, bit for bit.  Arguments as ptq4vm_w8a8_linear_fused plus z_tok [L] int32
 * and rowsum [N] int32 as in ptq4vm_w8a8_linear_offset; acc_out receives the raw accumulators (before the correction),
 * xq_out the codes with the offset in them.
 * Runs on the weight-resident kernel (N <= 128, K a multiple of 64, >= 2048 rows, 16-byte aligned rows of x and wq)
 * and on the row-streaming kernel (K <= 128, >= 1024 rows): the shapes where fusing pays (x_proj, dt_proj).  Every
 * other shape returns PTQ4VM_ERR_SHAPE - call the two entry points there.
 * Errors otherwise as ptq4vm_w8a8_linear_fused, with NULL z_tok / rowsum -> PTQ4VM_ERR_NULL and
 * K > PTQ4VM_MAX_K_OFFSET -> PTQ4VM_ERR_SHAPE.
 */
int ptq4vm_w8a8_linear_offset_fused(const void *x_f16, const float *inv_m, const float *s_tok, const int32_t *z_tok,
                                    const int8_t *wq, const int32_t *rowsum, const float *s_w, const void *bias_f16,
                                    void *y_f16, int32_t *acc_out, int8_t *xq_out, int64_t B, int64_t L, int64_t K,
                                    int64_t N, int64_t ldx, int64_t ldwq, int64_t ldy, int64_t ldxq, void *stream);

/*
 * Debug validator of the device-resident scale vectors (Sec. 5.1: per-token steps Delta_X and
 * per-output-channel steps Delta_W; Sec. 2.4: smoothing vector s).  An entry is bad unless it is a
 * finite number > 0 (zero, negative, +-Inf and NaN are bad).  The hot path never looks at these
 * values; call this once after calibration / loading a checkpoint.
 *   s_tok [L], m [K] (the smoothing vector or its reciprocal inv_m), s_w [N]   f32 in; a vector of
 *                    length 0 is skipped and its pointer may then be NULL
 *   bad_counts [3]   int32 out (device): bad entries found in s_tok, m, s_w
 *   workspace        device scratch, 16-byte aligned, at least
 *                    PTQ4VM_VALIDATE_WORKSPACE_BYTES(L, K, N) bytes; contents need no initialisation
 *                    and are undefined afterwards (per-workgroup partial counts)
 * UNLIKE EVERY OTHER ENTRY POINT THIS ONE SYNCHRONISES: it enqueues two small kernels and a 12-byte
 * device-to-host copy on `stream`, waits for the stream and returns PTQ4VM_OK when all counts are zero,
 * PTQ4VM_ERR_VALUE otherwise (bad_counts tells which vector).  Not usable under stream capture.
 * Errors: NULL bad_counts / workspace / a non-empty vector, negative length, more than
 * PTQ4VM_VALIDATE_MAX_ELEMS entries in total, workspace too small, misalignment.
 */
#define PTQ4VM_VALIDATE_BLOCK 4096 /* entries per workgroup = per 16-byte workspace slot */
#define PTQ4VM_VALIDATE_MAX_ELEMS ((int64_t)1 << 31)
#define PTQ4VM_VALIDATE_WORKSPACE_BYTES(L, K, N) \
    (16 * ((((int64_t)(L) + (int64_t)(K) + (int64_t)(N)) + PTQ4VM_VALIDATE_BLOCK - 1) / PTQ4VM_VALIDATE_BLOCK + 1))
int ptq4vm_validate_scales(const float *s_tok, int64_t L, const float *m, int64_t K, const float *s_w, int64_t N,
                           int32_t *bad_counts, void *workspace, int64_t workspace_bytes, void *stream);

/*
 * ptq4vm_validate_scales for callers that can neither allocate device memory nor synchronise: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same vectors and
 * the same bad_counts [3] (device) as above, but
 *   - the per-workgroup partial counts live in a device array of the library itself
 *     (16 * (PTQ4VM_VALIDATE_STATIC_MAX_ELEMS / PTQ4VM_VALIDATE_BLOCK + 1) = 65552 bytes, which
 *     every GPU the library runs on holds until the process ends), so L + K + N may not exceed
 *     PTQ4VM_VALIDATE_STATIC_MAX_ELEMS (else PTQ4VM_ERR_SHAPE, nothing is launched);
 *   - the call only enqueues its two kernels on `stream` and returns PTQ4VM_OK: the counts are in
 *     bad_counts once the stream has reached that point, and PTQ4VM_ERR_VALUE is never returned.
 * No hipMalloc / hipFree, no copy, no synchronisation; nothing in the array has to be zero (every
 * slot that is read was written by the same call).  All calls on one GPU share that GPU's array:
 * calls that may overlap (different streams, several threads) race; order them on one stream.
 * The first call on a device looks the array's address up (hipGetSymbolAddress).
 * Errors: as ptq4vm_validate_scales without the workspace ones; PTQ4VM_ERR_HIP if the lookup fails.
 */
#define PTQ4VM_VALIDATE_STATIC_MAX_ELEMS ((int64_t)1 << 24)
int ptq4vm_validate_scales_static(const float *s_tok, int64_t L, const float *m, int64_t K, const float *s_w,
                                  int64_t N, int32_t *bad_counts, void *stream);

/*
 * Unquantized comparison linear (the "FP16" column of the paper's latency table, Sec. 6.4):
 *   y[r,o] = fp16( sum_k x[r,k] * w[o,k]  (fp32 accumulation)  + bias[o] )
 *   x_f16 [M, ldx], w_f16 [N, ldw], bias_f16 [N] or NULL, y_f16 [M, ldy]
 * Errors as for ptq4vm_w8a8_linear.
 */
int ptq4vm_f16_linear(const void *x_f16, const void *w_f16, const void *bias_f16, void *y_f16,
                      int64_t M, int64_t K, int64_t N, int64_t ldx, int64_t ldw, int64_t ldy,
                      void *stream);

/* Static, never freed. */
const char *ptq4vm_status_string(int status);
/* Thread-local text of the last HIP error that produced PTQ4VM_ERR_HIP on this thread. */
const char *ptq4vm_last_hip_error(void);
/* major * 10000 + minor * 100 + patch */
int ptq4vm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PTQ4VM_H */
