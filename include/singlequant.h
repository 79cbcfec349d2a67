/*
 * singlequant.h -- C ABI of the MI355X (gfx950) W4A4 inference hot path of
 * SingleQuant (arxiv 2511.22316).
 *
 * The path of one quantized linear layer, Y ~= X W, is (Sec. 4.2, Eq. 1):
 *
 *     X' = X R,  R = G_1 G_2 ... G_P (R1 (x) R2)         online rotation
 *     (Qx, sx) = int4 codes and per-token steps of X'      Sec. 3.2 quantizer
 *     Y = dequant( Qx Qw^T ),  Qw = int4 codes of W^T R    offline-rotated weights
 *
 * Conventions common to every entry point
 *   - "device" pointers are HIP device memory on the current device; "host"
 *     pointers are ordinary host memory that is read before the call returns.
 *   - The caller owns every buffer.  No entry point allocates, frees or
 *     synchronises; all work is enqueued on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and the call returns at once.
 *   - Arguments are validated on the host first.  On any error nothing is
 *     enqueued and the code of the first failing check is returned.
 *   - Token rows are row-major; channel k of a token is viewed as entry
 *     (p, q) of an n1 x n2 matrix with k = p*n2 + q (row-major vectorisation,
 *     Sec. 4.2 "Kronecker Product").
 *   - int4 codes are two's-complement nibbles in [-8, 7], two per byte, the
 *     LOW nibble holding the EVEN channel.
 *   - NaN or Inf in X gives undefined codes (not checked).
 */
#ifndef SINGLEQUANT_H
#define SINGLEQUANT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SQ_OK = 0,
    SQ_ERR_NULL = 1,     /* a required pointer is NULL                                  */
    SQ_ERR_SHAPE = 2,    /* K != n1*n2, K odd, a size <= 0 where > 0 is required, P < 0,
                            a leading dimension shorter than its row, or a size beyond
                            the limits below                                            */
    SQ_ERR_INDEX = 3,    /* a Givens index outside [0, K) or i == j                     */
    SQ_ERR_ALIGN = 4,    /* a pointer or leading dimension breaks the stated alignment  */
    SQ_ERR_LAUNCH = 5,   /* the HIP runtime refused the launch                          */
    SQ_ERR_TIMEOUT = 6   /* sq_decode_layer_status only: a workgroup gave up its wait   */
} sq_status;

/* Limits (SQ_ERR_SHAPE beyond them): n1 <= 128, n2 <= 256 and n2 a multiple
 * of 8, K = n1*n2 <= 16384, P <= 64, at most 2^30 rows per call of the row
 * kernels (2^24 tokens for the GEMM), K a multiple of 32 and at most
 * SQ_GEMM_MAX_K for the GEMM. */
#define SQ_MAX_N1 128
#define SQ_MAX_N2 256
#define SQ_MAX_K 16384
#define SQ_MAX_GIVENS 64
#define SQ_MAX_ROWS (1 << 30)
#define SQ_DECODE_MAX_TOKENS 32
#define SQ_GEMM_MAX_K 131040

/*
 * sq_rotate_quantize -- online rotation fused with per-token 4-bit quantization.
 *
 * For every token row x of X (fp16, read as exact reals):
 *   1. Givens list (Sec. 4.1; ART, Sec. 4.2), in order p = 0 .. P-1, on the
 *      K-channel index space:  (x_i, x_j) <- (x_i cos t + x_j sin t,
 *                                             x_j cos t - x_i sin t)
 *      i.e. x <- x G(i_p, j_p; t_p) with the 2x2 block of Lemma 1 (App. A.3).
 *      Pairs may share channels; the order is part of the definition.
 *   2. Kronecker rotation (Eq. 18):  x' = rvec(R1^T X_mat R2),  X_mat the
 *      n1 x n2 view of x;  R1, R2 are passed un-transposed.
 *   3. Quantizer of Sec. 3.2 with a per-token step:  s = max_k |x'_k| / 7
 *      (s = 1 for an all-zero row), code_k = clamp(floor(x'_k / s + 1/2), -8, 7).
 * Arithmetic is fp32 or better; x' is never written to memory unless
 * xrot_dbg is given.
 *
 *   X          device, fp16 [T, ldx]; rows 16-byte aligned (ldx % 8 == 0)
 *   T, K, ldx  tokens, channels (= n1*n2, even), leading dimension >= K
 *   giv_i/j    host, int32 [P]; giv_theta host, float [P] (radians); P may be 0
 *              and then the three pointers may be NULL
 *   R1, R2     device, fp16 [n1,n1] and [n2,n2], row-major, 16-byte aligned
 *   Q          device out, uint8 [T, K/2], 16-byte aligned
 *   scales     device out, float [T]
 *   xrot_dbg   device out float [T, K], or NULL.  For parity checks only: it
 *              triples the HBM traffic.
 * T == 0 is legal and enqueues nothing.
 */
sq_status sq_rotate_quantize(const void *X, int64_t T, int32_t K, int64_t ldx,
                             const int32_t *giv_i, const int32_t *giv_j,
                             const float *giv_theta, int32_t P,
                             const void *R1, int32_t n1,
                             const void *R2, int32_t n2,
                             uint8_t *Q, float *scales, float *xrot_dbg,
                             void *stream);

/*
 * sq_prepare_rotation / sq_rotate_quantize_prepared -- the same operation as
 * sq_rotate_quantize (Eq. 18 after the Givens list of Sec. 4.1 / 4.2, then the
 * quantizer of Sec. 3.2) for a caller that keeps a layer's R1 and R2 for many
 * calls.  R1 and R2 are constants of the layer (Sec. 4.2 builds them once from
 * calibration data), so their rearrangement into the order in which the matrix
 * cores take them as operands is moved out of the online call: with it there,
 * every wave of every launch gathers the two matrices row by row, about 2.5 us
 * of a launch that takes 11 us at T = 2048, K = 4096.
 *
 * sq_prepared_rotation_bytes   size of the prepared form, a multiple of 256;
 *              0 if (n1, n2) is not a shape sq_rotate_quantize accepts.
 * sq_prepare_rotation          writes it (two small kernels on `stream`).
 *   R1, R2     device, fp16 [n1,n1] and [n2,n2], row-major, 16-byte aligned
 *   prepared   device out, sq_prepared_rotation_bytes(n1, n2) bytes, 16-byte
 *              aligned, owned by the caller; opaque (copies of R1 and R2 and,
 *              for the shapes the matrix-core kernel covers, its operand
 *              fragments); valid for this library build only
 * sq_rotate_quantize_prepared  all other arguments, limits, results and error
 *              codes as sq_rotate_quantize; the results are identical bit for
 *              bit to those of sq_rotate_quantize with the R1, R2 the prepared
 *              form was written from.  The Givens list is not part of the
 *              prepared form and is passed on every call as before.
 */
int64_t sq_prepared_rotation_bytes(int32_t n1, int32_t n2);
sq_status sq_prepare_rotation(const void *R1, int32_t n1, const void *R2, int32_t n2,
                              void *prepared, void *stream);
sq_status sq_rotate_quantize_prepared(const void *X, int64_t T, int32_t K, int64_t ldx,
                                      const int32_t *giv_i, const int32_t *giv_j,
                                      const float *giv_theta, int32_t P,
                                      const void *prepared, int32_t n1, int32_t n2,
                                      uint8_t *Q, float *scales, float *xrot_dbg,
                                      void *stream);

/*
 * sq_w4a4_gemm -- int4 x int4 GEMM with dequantizing epilogue (Eq. 1 evaluated
 * on the codes; the weight operand is Flat(W~_R) = W^T R of Sec. 4.2, one
 * K-contiguous row per output channel).
 *
 *   acc[t, n] = sum_k Qx[t, k] * Qw[n, k]          exact, int32
 *   Y[t, n]   = fp16( float(acc[t, n]) * sx[t] * sw[n] )
 *
 *   Qx, sx   device, uint8 [T, K/2] and float [T]  (what sq_rotate_quantize wrote)
 *   Qw, sw   device, uint8 [N, K/2] and float [N]  (per-output-channel codes / steps)
 *   Y        device out, fp16 [T, ldy], ldy >= N
 *   acc_dbg  device out int32 [T, N], or NULL (parity checks only)
 * Requires K % 32 == 0, K <= SQ_GEMM_MAX_K = 131040 (the kernels accumulate
 * 256 * acc in int32, and 256 * 64 * K must stay below 2^31 when every product
 * is (-8)(-8): at K = 131072 it would be 2^31 exactly), Qx, Qw 16-byte
 * aligned.  T == 0 or N == 0 is legal and enqueues nothing.
 */
sq_status sq_w4a4_gemm(const uint8_t *Qx, const float *sx, int64_t T, int32_t K,
                       const uint8_t *Qw, const float *sw, int32_t N,
                       void *Y, int64_t ldy, int32_t *acc_dbg, void *stream);

/*
 * sq_tile_weights_decode / sq_w4a4_gemm_decode -- sq_w4a4_gemm for at most
 * SQ_DECODE_MAX_TOKENS tokens on a second copy of the weight codes, laid out
 * so that the one pass over the weights that decoding is (Sec. 5.4 "Inference
 * Efficiency") reads consecutive bytes: 24.0 instead of 27.0 us per launch at
 * T = 8, K = 8192, N = 28672.  Same operation, same accumulators, same Y bit
 * for bit as sq_w4a4_gemm on the canonical codes.  The canonical layout stays
 * the interchange format (what sq_prepare_weights writes and every other call
 * reads); this copy is made from it once per layer.
 *
 * Layout (the paper fixes none beyond one row per output channel, Sec. 4.2):
 * channels in blocks of 32 (the last block padded with zero codes), K in
 * slices of 256 codes, i.e. 128 bytes of a row.  Block b, slice S is one piece
 * of 4096 bytes at byte offset (b * (K / 256) + S) * 4096; inside a piece, the
 * 16-byte unit number 64 c + 32 g + r (c in 0..3, g in 0..1, r in 0..31) holds
 * bytes 64 g + 16 c .. + 15 of that slice of channel 32 b + r.
 *
 * sq_decode_weights_bytes   size of the copy: ceil(N / 32) * 32 * K / 2; 0 if
 *                           K is not a positive multiple of 256 within
 *                           SQ_GEMM_MAX_K or N < 0.  Host only.
 * sq_tile_weights_decode    Qw device, uint8 [N, K/2], 16-byte aligned;
 *                           Qw_tiled device out, sq_decode_weights_bytes(K, N)
 *                           bytes, 16-byte aligned.  K % 256 == 0.
 * sq_w4a4_gemm_decode       arguments, limits and errors as sq_w4a4_gemm, with
 *                           Qw_tiled in place of Qw; T <= SQ_DECODE_MAX_TOKENS
 *                           and K % 256 == 0, else SQ_ERR_SHAPE.
 * T == 0 or N == 0 is legal and enqueues nothing.
 */
int64_t sq_decode_weights_bytes(int32_t K, int32_t N);
sq_status sq_tile_weights_decode(const uint8_t *Qw, int32_t K, int32_t N,
                                 uint8_t *Qw_tiled, void *stream);
sq_status sq_w4a4_gemm_decode(const uint8_t *Qx, const float *sx, int64_t T, int32_t K,
                              const uint8_t *Qw_tiled, const float *sw, int32_t N,
                              void *Y, int64_t ldy, int32_t *acc_dbg, void *stream);

/*
 * sq_rotate_fp16 / sq_w4a16_gemm -- the weight-only setting (W4A16) of the
 * paper's appendix (paragraph "Weight-only Quantization" and its table): Eq. 1,
 * X W = (X R)(R^T W), with only the weight operand quantized.  The weight codes
 * and steps are the ones sq_prepare_weights writes (or sq_rotate_quantize on
 * the rows of W^T); the activations stay 16-bit.  Reading (the paper gives
 * perplexities only): the online rotation is the same as in the W4A4 path and
 * its result is kept in fp16.
 *
 * sq_rotate_fp16   steps 1 and 2 of sq_rotate_quantize (Givens list, then the
 *   Kronecker rotation of Eq. 18) with fp32-or-better arithmetic, each entry of
 *   the rotated row then rounded once to fp16 (nearest even; beyond the fp16
 *   range the result is infinite).  No quantizer.
 *     X, T, K, ldx, giv_*, P, R1, n1, R2, n2   as sq_rotate_quantize
 *     Xrot   device out, fp16 [T, ldo], 16-byte aligned, ldo >= K, ldo % 8 == 0
 *
 * sq_w4a16_gemm    Y[t, n] = fp16( sw[n] * sum_k X[t, k] * Qw[n, k] ), products
 *   exact, sums in fp32 on the matrix cores.
 *     X        device, fp16 [T, ldx] (what sq_rotate_fp16 wrote); rows 16-byte
 *              aligned (ldx % 8 == 0), ldx >= K
 *     Qw, sw   device, uint8 [N, K/2] (16-byte aligned) and float [N]
 *     Y        device out, fp16 [T, ldy], ldy >= N
 *   Requires K % 64 == 0, K <= 131072.  T == 0 or N == 0 is legal and enqueues
 *   nothing.
 * Three-bit weights (W3A16, the other column of that table): codes written by
 * sq_prepare_weights_variant with bits = 3 lie in [-4, 3] and are legal input
 * here as they are (one nibble each); sq_pack_w3 / sq_w3a16_gemm below keep
 * them in three bits each.
 */
sq_status sq_rotate_fp16(const void *X, int64_t T, int32_t K, int64_t ldx,
                         const int32_t *giv_i, const int32_t *giv_j,
                         const float *giv_theta, int32_t P,
                         const void *R1, int32_t n1, const void *R2, int32_t n2,
                         void *Xrot, int64_t ldo, void *stream);
sq_status sq_w4a16_gemm(const void *X, int64_t T, int32_t K, int64_t ldx,
                        const uint8_t *Qw, const float *sw, int32_t N,
                        void *Y, int64_t ldy, void *stream);

/*
 * sq_pack_w3 / sq_w3a16_gemm -- W3A16 of the same table with the weight codes
 * stored in three bits each, 3K/8 bytes per output channel.  The paper gives
 * no storage format; this one is the library's, chosen so that eight codes
 * become one dword of nibbles in two to four instructions:
 *   - a row of K codes takes 24 bytes per 64 codes, read as six little-endian
 *     32-bit words w[0..5];
 *   - code k = 64 g + 32 h + 8 m + i  (h in 0..1, m in 0..3, i in 0..7) is
 *     stored as u = code + 4 in 0..7;
 *   - the two low bits of u are bits 4i + 2 (m % 2) and the next one of word
 *     w[3h + m / 2] of group g; the high bit of u is bit 4i + m of w[3h + 2].
 *
 * sq_pack_w3      nibble codes -> 3-bit storage (offline, once per layer).
 *     Qw    device, uint8 [N, K/2], 16-byte aligned, every code in [-4, 3]
 *           (the low three bits of code + 4 are kept of any other)
 *     Qw3   device out, uint8 [N, 3K/8], 8-byte aligned
 *   Requires K % 64 == 0, K <= 131072.
 *
 * sq_w3a16_gemm   Y[t, n] = fp16( sw[n] * sum_k X[t, k] * Qw3[n, k] ), as
 *   sq_w4a16_gemm.  The kernel is the decode-shaped one (one pass over the
 *   weights per 16 tokens, which is where the smaller storage pays); for many
 *   tokens keep the codes as nibbles and call sq_w4a16_gemm.
 *     X, sw, Y as sq_w4a16_gemm; Qw3 device, 8-byte aligned
 *   Requires K % 256 == 0, K <= 131072, T <= SQ_W3A16_MAX_ROWS.
 * T == 0 or N == 0 is legal and enqueues nothing.
 */
#define SQ_W3A16_MAX_ROWS (16 * 65535)
sq_status sq_pack_w3(const uint8_t *Qw, int32_t K, int32_t N, uint8_t *Qw3, void *stream);
sq_status sq_w3a16_gemm(const void *X, int64_t T, int32_t K, int64_t ldx,
                        const uint8_t *Qw3, const float *sw, int32_t N,
                        void *Y, int64_t ldy, void *stream);

/*
 * sq_decode_layer -- sq_rotate_quantize_prepared followed by sq_w4a4_gemm in one
 * launch, for at most SQ_DECODE_MAX_TOKENS tokens (decoding, Sec. 5.4 "Inference
 * Efficiency",
 * where the layer is one pass over the weights and the rotation of a few tokens
 * is pure latency in front of it).  Same operation, same results bit for bit
 * as the two calls: the first workgroups rotate and quantize one token group
 * each into `workspace`, every workgroup then multiplies its block of output
 * channels once all groups are done.
 *
 *   X, T, K, ldx, giv_*, P, prepared, n1, n2   as sq_rotate_quantize_prepared;
 *              (n1, n2) one of 16x32, 32x32, 32x64, 64x64, 64x128, else
 *              SQ_ERR_SHAPE (use the two calls)
 *   Qw, sw, N, Y, ldy                          as sq_w4a4_gemm; K % 256 == 0
 *   workspace  device, sq_decode_layer_workspace_bytes(T, K) bytes, 256-byte
 *              aligned, owned by the caller.  Its first 16 bytes are counters:
 *              they must be zero before the first call (one hipMemsetAsync by
 *              the caller, once) and every call leaves them zero again, so the
 *              same workspace serves call after call on one stream without
 *              further clearing.  Calls that may overlap need a workspace each.
 *              Bytes 12..15 are an error word: a workgroup that waited about a
 *              second for the rotated tokens gives up, leaves its outputs
 *              unwritten and sets the word to 1; it stays 0 otherwise.  (The
 *              workgroups with the lowest indices rotate the tokens and the
 *              others wait for them; the bound is what a dispatch order other
 *              than lowest-index-first would run into.)
 * The only benefit of this entry point is one host call per layer instead of
 * two.  It saves no GPU time: on one MI355X the single launch takes slightly
 * longer than the two launches it replaces (35.4 us against 32.9 us at T = 8,
 * K = 8192, N = 28672), because the multiplying workgroups wait for the
 * rotating ones across the chip and then read the codes with agent-coherent
 * loads (the writers release their stores at agent scope; the readers' loads
 * bypass their own caches, so that no stale line can be returned and nothing
 * has to be invalidated).  Use it where the host's launch path is the bound
 * (a handful of tokens on small layers), otherwise use the two calls.
 * Needs at least as many blocks of 32 (N < 16384) or 64 output channels as there
 * are token groups (N >= 32 T is always enough), else SQ_ERR_SHAPE.
 */
int64_t sq_decode_layer_workspace_bytes(int64_t T, int32_t K);
sq_status sq_decode_layer(const void *X, int64_t T, int32_t K, int64_t ldx,
                          const int32_t *giv_i, const int32_t *giv_j,
                          const float *giv_theta, int32_t P,
                          const void *prepared, int32_t n1, int32_t n2,
                          const uint8_t *Qw, const float *sw, int32_t N,
                          void *Y, int64_t ldy, void *workspace, void *stream);

/*
 * sq_decode_layer_status -- has any sq_decode_layer call on this workspace given
 * up a wait (see the error word above)?  The one call of this library that
 * waits: it blocks until `stream` has finished all work enqueued so far, copies
 * the error word to the host and, if it was set, clears it.
 *   workspace  the workspace of the calls in question, or NULL for the array
 *              inside the library that sq_decode_layer_static uses (on the
 *              current device)
 * Returns SQ_OK (no call gave up: every Y was written), SQ_ERR_TIMEOUT (at
 * least one workgroup of at least one call since the last check left its part
 * of Y unwritten) or SQ_ERR_LAUNCH (the runtime refused the wait or the copy).
 * Not capturable in a HIP graph.
 */
sq_status sq_decode_layer_status(void *workspace, void *stream);

/*
 * sq_decode_layer_static -- sq_decode_layer for callers that cannot allocate
 * device memory or have nowhere to keep a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments without `workspace`, same limits, same error codes, same results
 * bit for bit.  The counters, steps and codes live in a device array inside the
 * library instead, sized for the largest call the entry point accepts
 * (SQ_DECODE_MAX_TOKENS tokens of SQ_MAX_K channels: 512 + 32 * 8192 = 262656
 * bytes; larger T or K is SQ_ERR_SHAPE as in sq_decode_layer).  Every GPU the
 * library runs on holds its own copy from the first call on it until the
 * process ends.  The call allocates and frees nothing; its first call on a
 * device looks the array's address up (hipGetSymbolAddress), which fails with
 * SQ_ERR_LAUNCH if the runtime refuses.
 * All calls on one GPU share that array, which keeps the last call's codes:
 * calls that may overlap on one GPU (two streams, two threads) race, and
 * must use sq_decode_layer with a workspace each.  The counters start at zero
 * when the library is loaded and every call leaves them zero, as with a
 * caller's workspace; the error word of a workgroup that gave up waiting
 * stays set until sq_decode_layer_status(NULL, stream) reads and clears it.
 */
sq_status sq_decode_layer_static(const void *X, int64_t T, int32_t K, int64_t ldx,
                                 const int32_t *giv_i, const int32_t *giv_j,
                                 const float *giv_theta, int32_t P,
                                 const void *prepared, int32_t n1, int32_t n2,
                                 const uint8_t *Qw, const float *sw, int32_t N,
                                 void *Y, int64_t ldy, void *stream);

/*
 * sq_prepare_weights -- offline weight path of Sec. 4.2: the rotation that is
 * applied to the activations online is folded into the weights,
 * W~ = R^T W with R = G_1 ... G_P (R1 (x) R2), stored as Flat(W~_R) = W^T R, one
 * K-contiguous row per output channel, and quantized per output channel with
 * the quantizer of Sec. 3.2 (round to nearest, step = row maximum / 7).
 * Row n of W^T goes through exactly the steps sq_rotate_quantize applies to a
 * token row, so (X R)(R^T W) = X W holds up to the two quantizations.
 *
 *   W          device, fp16 [K, ldw], W[k, n] = weight from input channel k to
 *              output channel n (the layout of y = x W); ldw >= N
 *   workspace  device, N * K fp16 values, 16-byte aligned: receives W^T.
 *              Caller-owned; may be released once the stream has passed the call.
 *   Qw, sw     device out, uint8 [N, K/2] (16-byte aligned) and float [N]:
 *              the weight operand of sq_w4a4_gemm
 * Givens list, R1, R2 as in sq_rotate_quantize; the same shape limits apply.
 * N == 0 is legal and enqueues nothing.
 */
sq_status sq_prepare_weights(const void *W, int32_t K, int32_t N, int64_t ldw,
                             const int32_t *giv_i, const int32_t *giv_j,
                             const float *giv_theta, int32_t P,
                             const void *R1, int32_t n1,
                             const void *R2, int32_t n2,
                             void *workspace, uint8_t *Qw, float *sw,
                             void *stream);

/*
 * sq_rotate_quantize_variant / sq_prepare_weights_variant -- the same two calls
 * with the quantizer of Sec. 3.2 taken at `bits` bits and with a clipping ratio:
 *
 *   step = clip_ratio * max|x'| / (2^(bits-1) - 1)      (1 for an all-zero row)
 *   code = clamp( floor(x' / step + 1/2), -2^(bits-1), 2^(bits-1) - 1 )
 *
 * bits = 3 is the W3A16 column of the weight-only table in the appendix.
 * clip_ratio is a reading: the paper names learnable clipping thresholds in
 * its comparison with FlatQuant and does not define the operation; here the
 * threshold is a fixed fraction of the row maximum, chosen by the caller, and
 * entries beyond it take the end levels.  Codes are written as two's-complement
 * nibbles whatever `bits` is, so every GEMM of this library takes them.
 *
 *   bits        2, 3 or 4, else SQ_ERR_SHAPE
 *   clip_ratio  in (0, 1], else SQ_ERR_SHAPE
 * All other arguments, limits and errors as sq_rotate_quantize /
 * sq_prepare_weights, which are these calls with bits = 4, clip_ratio = 1.
 */
sq_status sq_rotate_quantize_variant(const void *X, int64_t T, int32_t K, int64_t ldx,
                                     const int32_t *giv_i, const int32_t *giv_j,
                                     const float *giv_theta, int32_t P,
                                     const void *R1, int32_t n1,
                                     const void *R2, int32_t n2,
                                     int32_t bits, float clip_ratio,
                                     uint8_t *Q, float *scales, float *xrot_dbg,
                                     void *stream);
sq_status sq_prepare_weights_variant(const void *W, int32_t K, int32_t N, int64_t ldw,
                                     const int32_t *giv_i, const int32_t *giv_j,
                                     const float *giv_theta, int32_t P,
                                     const void *R1, int32_t n1,
                                     const void *R2, int32_t n2,
                                     int32_t bits, float clip_ratio,
                                     void *workspace, uint8_t *Qw, float *sw,
                                     void *stream);

/*
 * sq_kron_factor -- Kronecker dimension factorization (Alg. 1): n2 is the power
 * of two dividing n that lies closest to sqrt(n) (of two equally close ones the
 * smaller), n1 = n / n2.  Host only; n >= 1.
 */
sq_status sq_kron_factor(int32_t n, int32_t *n1, int32_t *n2);

/*
 * sq_build_rotation -- the closed-form construction of the rotation from one
 * batch of calibration activations (Sec. 4.2; no gradients, no iterations).
 * What is computed, in this order (the points the paper leaves open are marked
 * "reading"):
 *   1. Calibration vector c: the row of X with the largest |entry|, the lowest
 *      such row among equals (reading).
 *   2. ART, P steps ("Alignment Rotation Transformation"; several steps as in
 *      the paper's study of the number of ART steps): i = channel of largest
 *      |c|, j = channel of smallest |c| other than i (lowest channel among
 *      equals), theta = atan2(c_j, c_i) - pi/4 (Lemma 1), after which c_i and
 *      c_j both hold sqrt(c_i^2 + c_j^2) / sqrt(2).  The pairs index the
 *      K-channel space and are returned as the Givens list sq_rotate_quantize
 *      takes; they are not folded into a Kronecker factor (reading).
 *   3. URT ("Uniformity Rotation Transformation") for each side, from a vector
 *      V: uniform target U = template q_k = (2k - n - 1)/n handed out by the
 *      rank order of V (ascending, lower index first among equals) and scaled
 *      to ||V||; R_map, R'_map = n - 1 plane rotations each that take V and U
 *      to ||V|| e_1, entry k being zeroed in the plane (k-1, k), k = n-1 .. 1
 *      (reading: the paper leaves the chain open); R^U = R_map R'_map^T, so
 *      that V R^U = U.  Side vectors (reading): with C the n1 x n2 view of c
 *      after step 2, V1 = row means of C, V2 = column means of C.
 *   4. Composition ("The Overall SingleQuant Method"): R1 = R^U(V1),
 *      R2 = H R^U(V2 H), H the normalised Sylvester Hadamard matrix.  Reading:
 *      the paper prints the left factor transposed, for matrices acting on
 *      column vectors; with rows acted on as in Eq. 18 (R1 enters as R1^T) the
 *      factor that sends the columns of C to their uniform target is R^U
 *      itself.
 * Index decisions (steps 1, 2 and the rank order of step 3) are taken on fp64
 * values.  Several ART steps make near-ties by themselves (a massive entry a
 * rotated against a tiny entry b leaves a (1 + b^2/2a^2) / sqrt(2) in both
 * channels, so the halves of two outliers can agree to 15 digits or more);
 * which of two channels that close counts as the larger is not defined beyond
 * fp64 rounding.  Matrices are fp32, rounded to fp16 at the end.
 *
 *   X          device, fp16 [T, ldx], T >= 1; rows 16-byte aligned (ldx % 8 == 0)
 *   n1, n2     2 <= n1 <= 128; n2 a power of two, 8 <= n2 <= 256; K = n1*n2 <= 16384
 *   P          0 .. 64 ART steps
 *   giv_i/j    device out, int32 [P]; giv_theta device out, float [P].  Copy them
 *              to the host (after the stream has passed this call) to hand them
 *              to sq_rotate_quantize / sq_prepare_weights.  May be NULL if P == 0.
 *   R1, R2     device out, fp16 [n1,n1] and [n2,n2], row-major
 *   workspace  device, sq_build_rotation_workspace_bytes(T, n1, n2) bytes, 16-byte
 *              aligned, caller-owned; free to reuse once the stream has passed
 *              the call
 */
sq_status sq_build_rotation(const void *X, int64_t T, int32_t K, int64_t ldx,
                            int32_t n1, int32_t n2, int32_t P,
                            int32_t *giv_i, int32_t *giv_j, float *giv_theta,
                            void *R1, void *R2, void *workspace, void *stream);

/* Bytes of workspace sq_build_rotation needs; 0 if a size is out of range. */
int64_t sq_build_rotation_workspace_bytes(int64_t T, int32_t n1, int32_t n2);

/* Static, human-readable name of a status code. */
const char *sq_status_string(sq_status status);

/* ---- Debug and test aids ------------------------------------------------------
 * Not needed in normal use and not part of the method: switches that force a
 * launch variant the library would not pick by itself (so that tests and tuning
 * runs can reach every variant), and a view of the host-side launch plan.  The
 * library reads no environment variables.
 *
 * sq_debug_set_option   process-wide; takes effect from the next call on.
 *                       value 0 always means "the library decides".
 *                       SQ_ERR_SHAPE for an unknown option.
 */
typedef enum {
    SQ_DEBUG_GEMM_LAUNCH_SHAPE = 0,     /* 1 + case number of sq_w4a4_gemm's dispatcher; shapes the
                                           case does not fit fall back to the normal choice      */
    SQ_DEBUG_ROTQ_RING = 1,             /* 2 or 3: LDS tiles per token slot of the rotate kernel     */
    SQ_DEBUG_ROTQ_R1_IN_REGISTERS = 2,  /* 1: never keep R1's operand fragments in LDS              */
    SQ_DEBUG_ROTQ_PLAIN_KERNEL = 3,     /* 1: every shape takes the plain-FMA rotate kernel         */
    SQ_DEBUG_DECODE_SPIN_LIMIT = 4,     /* polls after which a waiting workgroup of sq_decode_layer
                                           gives up (default 2^20, about a second)                */
    SQ_DEBUG_W4A16_LAUNCH_SHAPE = 5,    /* sq_w4a16_gemm: the tile kernel with 128 x 256 tiles and
                                           loading waves (1) or 256 x 256 tiles (2), whatever T     */
    SQ_DEBUG_OPTION_COUNT = 6
} sq_debug_option;
sq_status sq_debug_set_option(sq_debug_option option, int32_t value);

/*
 * sq_debug_rotq_plan -- how the host regroups a Givens list (Sec. 4.1 / 4.2;
 * list order is part of the definition) for the matrix-core rotate kernel:
 * touched channels get slots, distinct values of channel % n2 get q-slots, and
 * pair p goes to level 1 + the latest level of an earlier pair sharing a
 * channel with it, so that the pairs of a level are disjoint and level order
 * equals list order.  Host only.  Every out array has room for
 * 2 * SQ_MAX_GIVENS entries (pair_* are indexed by list position).  Returns the
 * number of levels, or -1 if P is out of range or the list cannot be planned.
 */
int32_t sq_debug_rotq_plan(const int32_t *giv_i, const int32_t *giv_j, int32_t P, int32_t n2,
                           int32_t *n_slots, int32_t *n_qslots, int32_t *slot_chan,
                           int32_t *slot_qslot, int32_t *qslot_q, int32_t *pair_slot_i,
                           int32_t *pair_slot_j, int32_t *pair_level);

#ifdef __cplusplus
}
#endif
#endif /* SINGLEQUANT_H */
