/*
 * libconvrot - ConvLinear4bit forward path for AMD MI355X (gfx950).
 *
 * C ABI.  The path is the one layer the ConvRot paper (arXiv 2512.03673, Sec. 4.3) calls
 * ConvLinear4bit:  Y = X W^T  computed as
 *
 *   X' = R_g(X)                      group-wise regular-Hadamard rotation        (Sec. 4.2, Eq. 11-13)
 *   q_x, s_x = Q4(X') per token      symmetric 4-bit codes, one scale per row    (Eq. 1, Sec. 5.2)
 *   acc = q_x q_w^T                  integer GEMM on the codes                   (Sec. 4.3)
 *   Y = bf16(acc * s_x[m] * s_w[n])  dequantisation                              (Sec. 4.3, suppl. Sec. B)
 *
 * with (q_w, s_w) = Q4(R_g(W)) prepared once, offline, per output channel (Eq. 12-13, Sec. 5.2).
 * R_g applies H_g / sqrt(g) to every length-g block of every row, H_g being the Kronecker power
 * of the order-4 regular Hadamard matrix of Thm 3.3 / Eq. 9; g (the paper's N_0) is 4, 16, 64,
 * 256 or 1024.
 *
 * Conventions for every entry point
 *   - Pointers named in the comments as DEVICE are device (HBM) pointers; everything else is
 *     passed by value.  All matrices are row-major and contiguous.  bf16 is the raw 16-bit
 *     pattern.  `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Calls are asynchronous on `stream`; they allocate and free nothing.  The caller owns every
 *     buffer, including the workspace, for the duration of the work.  The library keeps no state
 *     between calls except what convrot_init / convlinear4bit_forward_noalloc describe below (the
 *     per-device address of one static device array, looked up once); every other call depends on
 *     its arguments only and may be the first call of a process, also under stream capture.
 *   - Inputs are never written.  Outputs must not alias inputs.
 *   - Return value: CONVROT_OK (0) or a negative convrot_status.  Arguments are validated on
 *     the host before any launch: on an argument error nothing is launched and no output byte
 *     is written.  The library never throws or aborts.
 *   - Shapes: M, N >= 0 (M == 0 or N == 0 is a valid no-op, and a matrix with no rows may be
 *     passed as NULL), 0 < K <= CONVROT_MAX_K,
 *     K % 32 == 0 and K % g == 0 (the paper defines no padding for a ragged last block).
 *     bf16 and int32 matrices must be 16-byte aligned, code matrices 256-byte aligned, scale
 *     pointers 4-byte aligned.
 *
 * Codes.  A 4-bit code is an integer in [-7, 7] (-8 is never produced).  In memory it is the FP6
 * (E2M3: 1 sign, 2 exponent, 3 mantissa bits, bias 1) number of that value, six bits, the operand
 * format of the CDNA4 matrix instruction the GEMM runs on (every such integer is an E2M3 number;
 * products and their sums up to K = 65536 stay below 2^24, so the fp32 accumulation is exact and
 * the GEMM is the integer GEMM, bit for bit).  A code matrix of `rows` x K codes is laid out as
 *
 *   unit    16 consecutive codes of a row = 96 bits (3 little-endian dwords); code e of the unit
 *           sits at bit 6 * (2 * (e % 8) + e / 8)
 *   chunk   an even unit followed by the odd unit after it = 32 codes = 24 bytes:
 *           "A part" = its first 16 bytes, "B part" = its last 8
 *   block   32 rows x 128 codes (4 chunks per row) = 3 KB:
 *             A part of chunk c of row r  at  r * 64 + ((c ^ (((r >> 1) ^ (r >> 3)) & 3)) * 16)
 *             B part                      at  2048 + r * 32 + ((c ^ ((r >> 3) & 3)) * 8)
 *   matrix  block (R, S) - rows 32 R .., codes 128 S .. - at (R * ceil(K / 128) + S) * 3072
 *
 * i.e. ceil(rows / 32) * ceil(K / 128) * 3072 bytes (convrot_packed_bytes).  The codes of the last
 * block of a row past K are written as zeros by the producing call (a caller that fills a code
 * matrix itself must zero that K padding too).  The rows past `rows` of the last row block are never
 * written; the GEMM does load them along with the rest of the 3 KB block, but their products only
 * reach accumulators of rows that are not stored (every six-bit pattern is a finite number and rows
 * are independent), so their contents do not matter and need no initialisation.  (8-bit variant: one int8 in [-127, 127] per code, K bytes per row, stored
 * as 1 KB panels of 16 rows x 64 bytes, the K-panels of the same 16 rows adjacent: byte b of row r
 * at ((r / 16) * KP + b / 64) * 1024 + (r % 16) * 64 + b % 64, KP = ceil(K / 64), same padding
 * rules; convrot_packed_bytes8.)  Both layouts exist so that the GEMM's loads are whole contiguous
 * kilobytes; they are a contract between the producing calls (convrot_prepare_weight,
 * convrot_rotquant_act) and the GEMM calls of the same library version.
 *
 * Quantiser (both operands): a = max_k |x'[k]| over the rotated row, s = a / 7 in fp32 (s = 1
 * when a == 0), q = clamp(round_half_even(x' / s), -7, 7).
 *
 * Values.  X and W must be finite.  A NaN or an infinity leaves the scale and the codes of its own
 * row undefined (as any absmax quantiser does) and, because 64 units of 16 elements are rotated in
 * one matrix instruction, may do the same to the other rows of the same block of 32 rows (16 in the
 * 8-bit variant); rows of other blocks are not affected.
 */
#ifndef CONVROT_H
#define CONVROT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CONVROT_VERSION 500          /* major*10000 + minor*100 + patch */
#define CONVROT_MAX_K 65536          /* longest row the single-pass rotate+quantise kernel holds on chip */

typedef enum convrot_status {
    CONVROT_OK = 0,
    CONVROT_ERR_NULL = -1,       /* a required pointer is NULL                                     */
    CONVROT_ERR_SHAPE = -2,      /* M or N < 0, K <= 0, K > CONVROT_MAX_K, K % 32 != 0, K % g != 0 */
    CONVROT_ERR_GROUP = -3,      /* g not in {4, 16, 64, 256, 1024}                                */
    CONVROT_ERR_ALIGN = -4,      /* a pointer is not aligned as required                           */
    CONVROT_ERR_WORKSPACE = -5,  /* workspace_bytes < convrot_workspace_bytes(M, K)                */
    CONVROT_ERR_HIP = -6         /* a launch failed; the HIP error is left for hipGetLastError()   */
} convrot_status;

/* Host.  Static string for a status code ("unknown status" for anything else). */
const char *convrot_status_string(int status);

/* Host.  CONVROT_VERSION of the loaded library. */
int convrot_version(void);

/* Host.  Static string naming the compiler the library was built with (the kernels rely on details of its code
 * generation, so measurements should carry it), e.g. "clang 22.0.0git (...), HIP 7.2.26015". */
const char *convrot_build_info(void);

/*
 * Host.  Set-up of convlinear4bit_forward_noalloc for the calling thread's current device: looks up the
 * device address of that call's static workspace (which loads the library's device code onto the device if
 * no kernel of it has run there yet).  Idempotent, thread-safe, allocates nothing itself: the array is part of
 * the library's device code and stays resident on a device from the moment that code is loaded until the
 * process ends.  Optional - convlinear4bit_forward_noalloc does the same on its first call on a device - but
 * that first call, or this one, must be made outside stream capture.  No other entry point needs it.
 * CONVROT_ERR_HIP when there is no usable device.
 */
int convrot_init(void);

/* Host.  X rows per block tile that both GEMM kernels use for an [M, N] output: 192 (tile 192 x 192) or
 * 256 (tile 256 x 128); 0 when M or N < 0.  The result of the GEMM does not depend on it; the query
 * exists so that tests and tuning runs can tell which kernel configuration a shape exercises. */
int convrot_gemm_tile_rows(int64_t M, int64_t N);

/* Host.  Bytes of a 4-bit code matrix with `rows` rows of K codes in the layout above
 * (ceil(rows / 32) * ceil(K / 128) * 3 KB: 0.75 byte per code).  0 on bad input. */
size_t convrot_packed_bytes(int64_t rows, int64_t K);

/* Host.  Bytes of workspace convlinear4bit_forward needs for an [M, K] activation: the code matrix
 * (convrot_packed_bytes(M, K)) followed by M fp32 scales (rounded up to 256).  0 on bad input. */
size_t convrot_workspace_bytes(int64_t M, int64_t K);

/*
 * Offline weight preparation (Eq. 12-13, Sec. 5.2 "per-channel"): W' = R_g(W); for each output
 * channel n, s_w[n] = max_k |W'[n,k]| / 7 and q_w[n,:] = Q4(W'[n,:]); packed.
 *   W_bf16   DEVICE in   [N, K] bf16
 *   Wq       DEVICE out  convrot_packed_bytes(N, K) bytes: 4-bit codes [N, K], layout above
 *   w_scale  DEVICE out  [N] fp32
 */
int convrot_prepare_weight(const void *W_bf16, int64_t N, int64_t K, int group,
                           void *Wq, float *w_scale, void *stream);

/*
 * Online activation path (Sec. 4.2 + Eq. 1, Sec. 5.2 "per-token"): X' = R_g(X), per-token scale,
 * 4-bit codes, packed - one pass over X.
 *   X_bf16   DEVICE in   [M, K] bf16
 *   Xq       DEVICE out  convrot_packed_bytes(M, K) bytes: 4-bit codes [M, K], layout above
 *   x_scale  DEVICE out  [M] fp32
 */
int convrot_rotquant_act(const void *X_bf16, int64_t M, int64_t K, int group,
                         void *Xq, float *x_scale, void *stream);

/*
 * W4A4 GEMM with the dequantisation fused (Sec. 4.3; suppl. Sec. B lists them as two stages):
 * Y[m,n] = bf16( (sum_k q_x[m,k] q_w[n,k]) * x_scale[m] * w_scale[n] + bias[n] ), the sum exact.
 *   Xq, Wq            DEVICE in   4-bit codes [M, K], [N, K], layout above
 *   x_scale, w_scale  DEVICE in   [M], [N] fp32
 *   bias_bf16         DEVICE in   [N] bf16, or NULL for none.  Eq. 10 of the paper has no bias; the
 *                                 linear layers it replaces carry one, added here in fp32 before the
 *                                 single rounding to bf16.  2-byte aligned.
 *   Y_bf16            DEVICE out  [M, N] bf16
 */
int convrot_w4a4_gemm_dequant(const void *Xq, const float *x_scale, const void *Wq, const float *w_scale,
                              const void *bias_bf16, int64_t M, int64_t N, int64_t K, void *Y_bf16,
                              void *stream);

/*
 * The whole ConvLinear4bit forward (Sec. 4.3): convrot_rotquant_act into the workspace, then
 * convrot_w4a4_gemm_dequant, on one stream.
 *   X_bf16     DEVICE in   [M, K] bf16
 *   Wq         DEVICE in   codes [N, K] from convrot_prepare_weight (same `group`)
 *   w_scale    DEVICE in   [N]
 *   bias_bf16  DEVICE in   [N] bf16 or NULL, as above
 *   Y_bf16     DEVICE out  [M, N] bf16
 *   workspace  DEVICE scratch, 256-byte aligned, at least convrot_workspace_bytes(M, K) bytes;
 *              holds the activation codes and scales after the call.
 */
int convlinear4bit_forward(const void *X_bf16, const void *Wq, const float *w_scale, const void *bias_bf16,
                           int64_t M, int64_t N, int64_t K, int group, void *Y_bf16,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * convlinear4bit_forward for callers that cannot allocate device memory at all and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and bit-identical output; the activation codes and scales go to a static device
 * array of CONVROT_NOALLOC_WORKSPACE_BYTES (64 MiB) inside the library instead of a caller's workspace, and
 * the call (like every call of this library) invokes no hipMalloc / hipFree and no allocating routine.
 *   - Limit: convrot_workspace_bytes(M, K) <= CONVROT_NOALLOC_WORKSPACE_BYTES, i.e. about M * K <= 89e6 codes
 *     (4608 x 15360, the widest FLUX layer at 1024 x 1024 pixels, needs 53 MB); CONVROT_ERR_WORKSPACE beyond
 *     it, with nothing launched.
 *   - The array belongs to the device: every call on one GPU uses the same memory and finds the previous
 *     call's contents there (nothing needs clearing: each call overwrites all it reads).  Calls whose work
 *     overlaps in time on one GPU - different streams, or graph replays running concurrently - race on it;
 *     serialise them or use convlinear4bit_forward with separate workspaces.
 *   - The device used is the calling thread's current device, which must be the device of `stream`.  The
 *     array's address is looked up on the first call on a device (or by convrot_init); make that first
 *     call, or convrot_init, outside stream capture.
 */
#define CONVROT_NOALLOC_WORKSPACE_BYTES (64u << 20)
int convlinear4bit_forward_noalloc(const void *X_bf16, const void *Wq, const float *w_scale, const void *bias_bf16,
                                   int64_t M, int64_t N, int64_t K, int group, void *Y_bf16, void *stream);

/*
 * Gate / debug export, not a hot-path call: the raw integer accumulators of the GEMM stage
 * (Sec. 4.3), acc[m,n] = sum_k q_x[m,k] q_w[n,k], so that the GEMM can be checked bit for bit.
 *   acc  DEVICE out  [M, N] int32
 */
int convrot_w4a4_gemm_i32(const void *Xq, const void *Wq, int64_t M, int64_t N, int64_t K,
                          int32_t *acc, void *stream);

/*
 * Gate / debug export, not a hot-path call: the codes of a 4-bit code matrix as plain integers, so that
 * what convrot_prepare_weight and convrot_rotquant_act produced can be compared code by code
 * (Eq. 1) without knowing the layout.
 *   Xq     DEVICE in   4-bit codes [rows, K], layout above
 *   codes  DEVICE out  [rows, K] int8, row-major, each in [-7, 7]; 16-byte aligned
 */
int convrot_unpack_codes(const void *Xq, int64_t rows, int64_t K, int8_t *codes, void *stream);

/*
 * Diagnostic, not a hot-path call: the paper's outlier-amplitude metric max |X H| (Sec. 4.2; Table 5-1
 * and Fig. 3-2 report it on FLUX activations), per row, for three choices of the group-wise rotation:
 *   kind 0 (CONVROT_ROT_NONE)      no rotation: max_k |X[m,k]|
 *   kind 1 (CONVROT_ROT_REGULAR)   the layer's regular Hadamard rotation: max_k |R_g(X)[m,k]| (= 7 x_scale[m])
 *   kind 2 (CONVROT_ROT_SYLVESTER) the Sylvester Hadamard matrix of order g instead, normalised alike -
 *                                  the comparison the paper draws (its first column of ones adds up a
 *                                  one-signed row: Sec. 3.2)
 *   X_bf16      DEVICE in   [M, K] bf16
 *   row_absmax  DEVICE out  [M] fp32
 * CONVROT_ERR_GROUP for a `kind` outside 0..2 as for a bad `group`.
 */
#define CONVROT_ROT_NONE 0
#define CONVROT_ROT_REGULAR 1
#define CONVROT_ROT_SYLVESTER 2
int convrot_rotated_absmax(const void *X_bf16, int64_t M, int64_t K, int group, int kind,
                           float *row_absmax, void *stream);

/*
 * ---- W8A8 variant of the layer (the paper's W8A8 rows, Sec. 5, Tables 5-2 and 5-4, and the ~20 % of
 * layers its mixed-precision mode keeps at 8 bits): the same rotation, the same symmetric quantiser
 * with 127 levels (s = a / 127, q in [-127, 127]), int8 codes stored one per byte in the panel layout.
 * Everything said above about pointers, streams, errors and shapes holds.
 */

/* Host.  Bytes of an 8-bit code matrix [rows, K] in the panel layout (ceil(rows / 16) * ceil(K / 64) KB). */
size_t convrot_packed_bytes8(int64_t rows, int64_t K);

/* Host.  Workspace of convlinear8bit_forward: convrot_packed_bytes8(M, K) + M fp32 scales (rounded up to 256). */
size_t convrot_workspace_bytes8(int64_t M, int64_t K);

/* As convrot_prepare_weight / convrot_rotquant_act, 8-bit: Wq, Xq are int8 codes [rows, K], panel layout. */
int convrot_prepare_weight8(const void *W_bf16, int64_t N, int64_t K, int group,
                            void *Wq, float *w_scale, void *stream);
int convrot_rotquant_act8(const void *X_bf16, int64_t M, int64_t K, int group,
                          void *Xq, float *x_scale, void *stream);

/* As convrot_w4a4_gemm_dequant on int8 codes [M, K], [N, K], panel layout. */
int convrot_w8a8_gemm_dequant(const void *Xq, const float *x_scale, const void *Wq, const float *w_scale,
                              const void *bias_bf16, int64_t M, int64_t N, int64_t K, void *Y_bf16,
                              void *stream);

/* As convlinear4bit_forward with 8-bit codes; workspace of convrot_workspace_bytes8(M, K) bytes. */
int convlinear8bit_forward(const void *X_bf16, const void *Wq, const float *w_scale, const void *bias_bf16,
                           int64_t M, int64_t N, int64_t K, int group, void *Y_bf16,
                           void *workspace, size_t workspace_bytes, void *stream);

/* Gate / debug export: raw int32 accumulators of the 8-bit GEMM. */
int convrot_w8a8_gemm_i32(const void *Xq, const void *Wq, int64_t M, int64_t N, int64_t K,
                          int32_t *acc, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CONVROT_H */
