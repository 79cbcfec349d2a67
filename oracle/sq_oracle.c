/*
 * CPU oracle for the SingleQuant W4A4 inference hot path (arxiv 2511.22316).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a plain, slow, fp64
 * restatement of what the paper defines, written so that it can be checked
 * against the paper by eye.  Only the tests, the smoke check and the
 * "cpu_baseline" leg of the benchmark may call it.  It shares no code, no
 * header, no table and no constant with the HIP library.
 *
 * What each function follows:
 *   sqo_givens_apply      Sec. 4.1 (Givens rotation, row-vector convention
 *                         x G(i,j;theta)) and the action formula in the proof
 *                         of Lemma 1 (App. A.3):
 *                         V G(theta) = (a cos + b sin, b cos - a sin).
 *   sqo_art_angle         Lemma 1: theta* = atan2(b, a) - pi/4.
 *   sqo_kron_apply        Eq. 18: V (R1 (x) R2) = rvec(R1^T V_mat R2), V_mat
 *                         the row-major n1 x n2 view of V.
 *   sqo_kron_apply_dense  the definition R = R1 (x) R2 multiplied out entry by
 *                         entry (tiny sizes only; the pin for sqo_kron_apply).
 *   sqo_rotate            Sec. 4.2: Givens list first (ART), then the Kronecker
 *                         rotation, per token row.
 *   sqo_quantize_rows     the rounding quantizer of Sec. 3.2,
 *                         Q_D(z) = D floor(z/D + 1/2), with a per-row step
 *                         D = max|z| / 7 and codes clamped to [-8, 7].
 *   sqo_quantize_rows_variant  the same quantizer Q_D of Sec. 3.2 with b bits
 *                         (the W3A16 column of the weight-only table in the
 *                         appendix) and a clipping ratio (the clipping
 *                         thresholds named in the comparison with FlatQuant,
 *                         read as a fixed fraction of the row maximum):
 *                         D = ratio max|z| / (2^(b-1) - 1), codes clamped to
 *                         [-2^(b-1), 2^(b-1) - 1].
 *   sqo_pack_w3 / sqo_unpack_w3  storage of 3-bit codes in three bits each.  The
 *                         paper does not give a storage format; the one used
 *                         is stated at the function.
 *   sqo_tile_weights_decode  the library's second weight layout (a permutation
 *                         of the bytes; no arithmetic), from its statement.
 *   sqo_gemm              Eq. 1 / Eq. (xw): (XR)(R^T W) evaluated on the integer
 *                         codes, then scaled back: y = acc * s_x * s_w.
 *   sqo_kron_factor       Alg. 1 (Kronecker dimension factorization).
 *
 * Parity pins (tests/test_oracle_*.py): Lemma 1's closed form and a brute
 * force over theta; explicit dense kron(R1,R2) from numpy; norm and inner
 * product preservation; XW = (XR)(R^T W); hand-worked rounding ties;
 * brute-force integer GEMM; fp16 conversion against IEEE binary16 tables;
 * the variant quantizer against sqo_quantize_rows at b = 4, ratio 1, against
 * hand-worked rows at b = 3 and at ratio 1/2, and against its error bound;
 * the 3-bit storage against bytes worked out by hand from the format; the
 * decode layout against hand-worked positions and as a bijection.
 * No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- fp16 --- */

/* IEEE binary16 bits -> double (exact). */
double sqo_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int mant = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)mant, -24);              /* subnormal or zero */
    } else if (expo == 31) {
        v = mant ? NAN : INFINITY;
    } else {
        v = ldexp((double)(mant + 1024), expo - 25);
    }
    return sign ? -v : v;
}

/* double -> IEEE binary16 bits, round to nearest, ties to even. */
uint16_t sqo_double_to_half(double x)
{
    uint16_t sign = (uint16_t)(signbit(x) ? 0x8000 : 0);
    double a = fabs(x);
    if (isnan(x)) return (uint16_t)(sign | 0x7e00);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00);   /* rounds to inf */
    if (a < ldexp(1.0, -14)) {
        /* subnormal range: spacing 2^-24; nearbyint is ties-to-even in the
           default rounding mode; a result of 1024 is the smallest normal. */
        double q = nearbyint(ldexp(a, 24));
        return (uint16_t)(sign | (uint16_t)q);
    }
    int e;
    double m = frexp(a, &e);                /* a = m 2^e, m in [0.5, 1) */
    double q = nearbyint(ldexp(m, 11));     /* 11 significant bits: [1024, 2048] */
    int expo = e - 1 + 15;
    if (q == 2048.0) { q = 1024.0; expo += 1; }
    if (expo >= 31) return (uint16_t)(sign | 0x7c00);
    return (uint16_t)(sign | (uint16_t)(expo << 10) | ((uint16_t)q - 1024));
}

/* --------------------------------------------------------- Sec. 4.1 ------ */

/* Lemma 1: the angle that equalises the pair (a, b). */
double sqo_art_angle(double a, double b)
{
    return atan2(b, a) - M_PI / 4.0;
}

/* x <- x G(i,j;theta): only coordinates i and j change (App. A.3). */
void sqo_givens_apply(double *row, int64_t i, int64_t j, double theta)
{
    double a = row[i], b = row[j];
    double c = cos(theta), s = sin(theta);
    row[i] = a * c + b * s;
    row[j] = b * c - a * s;
}

/* --------------------------------------------------------- Eq. 18 -------- */

/* out = rvec(R1^T V_mat R2).  R1 is n1 x n1, R2 is n2 x n2, both row-major and
   NOT transposed by the caller.  tmp holds n1*n2 doubles. */
void sqo_kron_apply(const double *row, const double *R1, int n1,
                    const double *R2, int n2, double *out, double *tmp)
{
    /* tmp = V_mat R2 */
    for (int p = 0; p < n1; ++p)
        for (int qo = 0; qo < n2; ++qo) {
            double acc = 0.0;
            for (int q = 0; q < n2; ++q)
                acc += row[(int64_t)p * n2 + q] * R2[(int64_t)q * n2 + qo];
            tmp[(int64_t)p * n2 + qo] = acc;
        }
    /* out = R1^T tmp */
    for (int po = 0; po < n1; ++po)
        for (int qo = 0; qo < n2; ++qo) {
            double acc = 0.0;
            for (int p = 0; p < n1; ++p)
                acc += R1[(int64_t)p * n1 + po] * tmp[(int64_t)p * n2 + qo];
            out[(int64_t)po * n2 + qo] = acc;
        }
}

/* The definition, multiplied out: out[k'] = sum_k row[k] (R1 (x) R2)[k, k'],
   (R1 (x) R2)[(p,q),(p',q')] = R1[p,p'] R2[q,q'].  O(K^2): tiny sizes only. */
void sqo_kron_apply_dense(const double *row, const double *R1, int n1,
                          const double *R2, int n2, double *out)
{
    for (int po = 0; po < n1; ++po)
        for (int qo = 0; qo < n2; ++qo) {
            double acc = 0.0;
            for (int p = 0; p < n1; ++p)
                for (int q = 0; q < n2; ++q)
                    acc += row[(int64_t)p * n2 + q] *
                           (R1[(int64_t)p * n1 + po] * R2[(int64_t)q * n2 + qo]);
            out[(int64_t)po * n2 + qo] = acc;
        }
}

/* --------------------------------------------------------- Sec. 4.2 ------ */

/* Rotate T rows.  X: fp16 bits [T, ldx]; Givens list applied in order
   p = 0..P-1 on the K-channel index space; then the Kronecker rotation with
   fp64 factors.  Xrot: [T, K] doubles.  Returns 0, or -1 on a bad argument. */
int sqo_rotate(const uint16_t *X, int64_t T, int K, int64_t ldx,
               const int32_t *giv_i, const int32_t *giv_j,
               const double *giv_theta, int P,
               const double *R1, int n1, const double *R2, int n2,
               double *Xrot)
{
    if (K != n1 * n2 || ldx < K || T < 0 || P < 0) return -1;
    for (int p = 0; p < P; ++p)
        if (giv_i[p] < 0 || giv_i[p] >= K || giv_j[p] < 0 || giv_j[p] >= K ||
            giv_i[p] == giv_j[p])
            return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *row = (double *)malloc(sizeof(double) * (size_t)K);
        double *tmp = (double *)malloc(sizeof(double) * (size_t)K);
        if (!row || !tmp) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(static)
            for (int64_t t = 0; t < T; ++t) {
                for (int k = 0; k < K; ++k)
                    row[k] = sqo_half_to_double(X[t * ldx + k]);
                for (int p = 0; p < P; ++p)
                    sqo_givens_apply(row, giv_i[p], giv_j[p], giv_theta[p]);
                sqo_kron_apply(row, R1, n1, R2, n2, Xrot + t * (int64_t)K, tmp);
            }
        }
        free(row);
        free(tmp);
    }
    return fail ? -1 : 0;
}

/* --------------------------------------------------------- Sec. 3.2 ------ */

static uint8_t nibble(int q) { return (uint8_t)(q & 0xf); }

/* Per-row symmetric 4-bit quantization.  Step D = max|z|/7 rounded to fp32
   (D = 1 for an all-zero row); code = clamp(floor(z/D + 1/2), -8, 7) decided
   in fp64.  Q: [T, K/2], low nibble = even channel, two's complement. */
int sqo_quantize_rows(const double *Xrot, int64_t T, int K,
                      uint8_t *Q, float *scales)
{
    if (K <= 0 || (K & 1)) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const double *z = Xrot + t * (int64_t)K;
        double amax = 0.0;
        for (int k = 0; k < K; ++k) {
            double a = fabs(z[k]);
            if (a > amax) amax = a;
        }
        float D = (amax == 0.0) ? 1.0f : (float)(amax / 7.0);
        scales[t] = D;
        for (int k = 0; k < K; k += 2) {
            int q[2];
            for (int u = 0; u < 2; ++u) {
                double c = floor(z[k + u] / (double)D + 0.5);
                if (c < -8.0) c = -8.0;
                if (c > 7.0) c = 7.0;
                q[u] = (int)c;
            }
            Q[t * (int64_t)(K / 2) + k / 2] =
                (uint8_t)(nibble(q[0]) | (nibble(q[1]) << 4));
        }
    }
    return 0;
}

/* The same quantizer with every step taken in fp32, for rows that are already
   fp32 (the precision a GPU kernel decides its codes in). */
int sqo_quantize_rows_f32(const float *Xrot, int64_t T, int K,
                          uint8_t *Q, float *scales)
{
    if (K <= 0 || (K & 1)) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const float *z = Xrot + t * (int64_t)K;
        float amax = 0.0f;
        for (int k = 0; k < K; ++k) {
            float a = fabsf(z[k]);
            if (a > amax) amax = a;
        }
        float D = (amax == 0.0f) ? 1.0f : amax / 7.0f;
        scales[t] = D;
        for (int k = 0; k < K; k += 2) {
            int q[2];
            for (int u = 0; u < 2; ++u) {
                float c = floorf(z[k + u] / D + 0.5f);
                if (c < -8.0f) c = -8.0f;
                if (c > 7.0f) c = 7.0f;
                q[u] = (int)c;
            }
            Q[t * (int64_t)(K / 2) + k / 2] =
                (uint8_t)(nibble(q[0]) | (nibble(q[1]) << 4));
        }
    }
    return 0;
}

/* The quantizer with b bits and a clipping ratio.  Levels: the integers
   -2^(b-1) .. 2^(b-1) - 1 (Sec. 3.2 rounds to the grid D Z; b bits keep that
   many of its points around zero).  Step D = ratio max|z| / (2^(b-1) - 1),
   evaluated in fp64 and rounded to fp32 (D = 1 for an all-zero row);
   code = clamp(floor(z/D + 1/2), -2^(b-1), 2^(b-1) - 1) decided in fp64.
   With b = 4 and ratio = 1 this is sqo_quantize_rows.  Codes are stored as
   two's-complement nibbles whatever b is.  2 <= bits <= 4, 0 < ratio <= 1. */
int sqo_quantize_rows_variant(const double *Xrot, int64_t T, int K, int bits,
                              double ratio, uint8_t *Q, float *scales)
{
    if (K <= 0 || (K & 1) || bits < 2 || bits > 4) return -1;
    if (!(ratio > 0.0) || ratio > 1.0) return -1;
    const double top = (double)((1 << (bits - 1)) - 1);
    const double bottom = -(double)(1 << (bits - 1));
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const double *z = Xrot + t * (int64_t)K;
        double amax = 0.0;
        for (int k = 0; k < K; ++k) {
            double a = fabs(z[k]);
            if (a > amax) amax = a;
        }
        float D = (amax == 0.0) ? 1.0f : (float)(ratio * amax / top);
        scales[t] = D;
        for (int k = 0; k < K; k += 2) {
            int q[2];
            for (int u = 0; u < 2; ++u) {
                double c = floor(z[k + u] / (double)D + 0.5);
                if (c < bottom) c = bottom;
                if (c > top) c = top;
                q[u] = (int)c;
            }
            Q[t * (int64_t)(K / 2) + k / 2] =
                (uint8_t)(nibble(q[0]) | (nibble(q[1]) << 4));
        }
    }
    return 0;
}

/* Signed value of nibble number k of a packed row. */
static int code_at(const uint8_t *rowq, int k)
{
    int v = (rowq[k >> 1] >> ((k & 1) * 4)) & 0xf;
    return v >= 8 ? v - 16 : v;
}

/* Unpack [T, K/2] bytes into [T, K] int8 codes. */
void sqo_unpack_codes(const uint8_t *Q, int64_t T, int K, int8_t *codes)
{
    for (int64_t t = 0; t < T; ++t)
        for (int k = 0; k < K; ++k)
            codes[t * (int64_t)K + k] = (int8_t)code_at(Q + t * (int64_t)(K / 2), k);
}

/* ------------------------------------------ 3-bit storage (W3A16) --------- */

/* Where code number k of a row lives in the 3-bit storage.  The paper gives no
   format; this one is the library's (stated in its header) and is written
   out here from that statement, not from the library's code:
     - a row of K codes (K a multiple of 64) takes 3K/8 bytes: 24 bytes for
       every 64 codes, read as six little-endian 32-bit words w[0..5];
     - code k = 64 g + 32 h + 8 m + i  (h in 0..1, m in 0..3, i in 0..7) is
       stored as u = code + 4 in 0..7;
     - the two low bits of u are bits 4i + 2 (m % 2) and the next one of word
       w[3h + m / 2] of group g;
     - the high bit of u is bit 4i + m of word w[3h + 2] of group g. */
static void w3_place(int k, int64_t *word_lo, int *bit_lo, int64_t *word_hi, int *bit_hi)
{
    int g = k / 64, h = (k / 32) % 2, m = (k / 8) % 4, i = k % 8;
    *word_lo = 6 * (int64_t)g + 3 * h + m / 2;
    *bit_lo = 4 * i + 2 * (m % 2);
    *word_hi = 6 * (int64_t)g + 3 * h + 2;
    *bit_hi = 4 * i + m;
}

static void w3_set_bit(uint8_t *row, int64_t word, int bit)
{
    row[4 * word + bit / 8] |= (uint8_t)(1u << (bit % 8));     /* little endian */
}

static int w3_get_bit(const uint8_t *row, int64_t word, int bit)
{
    return (row[4 * word + bit / 8] >> (bit % 8)) & 1;
}

/* Q: [N, K/2] nibble codes, every code in [-4, 3] (else -2 is returned);
   Q3: [N, 3K/8] bytes. */
int sqo_pack_w3(const uint8_t *Q, int64_t N, int K, uint8_t *Q3)
{
    if (K <= 0 || (K % 64)) return -1;
    memset(Q3, 0, (size_t)N * (size_t)(3 * K / 8));
    for (int64_t n = 0; n < N; ++n) {
        uint8_t *row = Q3 + n * (int64_t)(3 * K / 8);
        for (int k = 0; k < K; ++k) {
            int c = code_at(Q + n * (int64_t)(K / 2), k);
            if (c < -4 || c > 3) return -2;
            int u = c + 4, bl, bh;
            int64_t wl, wh;
            w3_place(k, &wl, &bl, &wh, &bh);
            if (u & 1) w3_set_bit(row, wl, bl);
            if (u & 2) w3_set_bit(row, wl, bl + 1);
            if (u & 4) w3_set_bit(row, wh, bh);
        }
    }
    return 0;
}

/* Back to nibble codes: Q3 [N, 3K/8] -> Q [N, K/2]. */
int sqo_unpack_w3(const uint8_t *Q3, int64_t N, int K, uint8_t *Q)
{
    if (K <= 0 || (K % 64)) return -1;
    memset(Q, 0, (size_t)N * (size_t)(K / 2));
    for (int64_t n = 0; n < N; ++n) {
        const uint8_t *row = Q3 + n * (int64_t)(3 * K / 8);
        for (int k = 0; k < K; ++k) {
            int bl, bh;
            int64_t wl, wh;
            w3_place(k, &wl, &bl, &wh, &bh);
            int u = w3_get_bit(row, wl, bl) | (w3_get_bit(row, wl, bl + 1) << 1) |
                    (w3_get_bit(row, wh, bh) << 2);
            Q[n * (int64_t)(K / 2) + k / 2] |= (uint8_t)(nibble(u - 4) << ((k & 1) * 4));
        }
    }
    return 0;
}

/* ------------------------------- weight layout for few tokens (decode) ---- */

/* The library's second layout of the weight codes, for its decode-shaped
   GEMM (the paper fixes no layout beyond "one row per output channel",
   Sec. 4.2).  Written out here from the statement in the library's header:
     - channels in blocks of 32 (the last block padded with zero bytes), K in
       slices of 256 codes, i.e. 128 bytes of a row;
     - block b, slice S is one piece of 4096 bytes at byte offset
       (b (K/256) + S) 4096;
     - inside a piece, the 16-byte unit number 64 c + 32 g + r (c in 0..3,
       g in 0..1, r in 0..31) holds bytes 64 g + 16 c .. + 15 of that slice of
       channel 32 b + r.
   Q: [N, K/2]; Qt: ceil(N/32) * 32 * K/2 bytes.  inverse != 0: Qt -> Q. */
int sqo_tile_weights_decode(const uint8_t *Q, int64_t N, int K, uint8_t *Qt, int inverse)
{
    if (K <= 0 || (K % 256) || N < 0) return -1;
    const int64_t Kb = K / 2, slices = K / 256, blocks = (N + 31) / 32;
    if (!inverse) memset(Qt, 0, (size_t)(blocks * 32 * Kb));
    for (int64_t n = 0; n < N; ++n) {
        const int64_t b = n / 32, r = n % 32;
        for (int64_t j = 0; j < Kb; ++j) {
            const int64_t S = j / 128, w = j % 128, g = w / 64, c = (w % 64) / 16, e = w % 16;
            const int64_t at = (b * slices + S) * 4096 + (64 * c + 32 * g + r) * 16 + e;
            if (inverse) ((uint8_t *)Q)[n * Kb + j] = Qt[at];
            else Qt[at] = Q[n * Kb + j];
        }
    }
    return 0;
}

/* ---------------------------------------------------- Eq. 1 on the codes -- */

/* acc[t,n] = sum_k qx[t,k] qw[n,k] (exact, int64, checked to fit int32);
   Y[t,n] = fp16(acc * sx[t] * sw[n]) with one rounding from fp64.
   Qw is [N, K/2]: one K-contiguous row per output channel, i.e. the rows of
   Flat(W~_R) = W^T R (Sec. 4.2).  acc may be NULL.  Returns 0, -1 bad
   argument, -2 accumulator outside int32. */
int sqo_gemm(const uint8_t *Qx, const float *sx, int64_t T, int K,
             const uint8_t *Qw, const float *sw, int N,
             uint16_t *Y, int64_t ldy, int32_t *acc)
{
    if (K <= 0 || (K & 1) || T < 0 || N < 0 || ldy < N) return -1;
    int overflow = 0;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const uint8_t *qx = Qx + t * (int64_t)(K / 2);
        for (int n = 0; n < N; ++n) {
            const uint8_t *qw = Qw + (int64_t)n * (K / 2);
            int64_t a = 0;
            for (int k = 0; k < K; ++k)
                a += (int64_t)code_at(qx, k) * (int64_t)code_at(qw, k);
            if (a > INT32_MAX || a < INT32_MIN) {
#pragma omp atomic write
                overflow = 1;
            }
            if (acc) acc[t * (int64_t)N + n] = (int32_t)a;
            Y[t * ldy + n] =
                sqo_double_to_half((double)a * (double)sx[t] * (double)sw[n]);
        }
    }
    return overflow ? -2 : 0;
}

/* One output element of the GEMM (for sampled checks at full size). */
int64_t sqo_gemm_acc_at(const uint8_t *Qx, const uint8_t *Qw, int K,
                        int64_t t, int64_t n)
{
    const uint8_t *qx = Qx + t * (int64_t)(K / 2);
    const uint8_t *qw = Qw + n * (int64_t)(K / 2);
    int64_t a = 0;
    for (int k = 0; k < K; ++k)
        a += (int64_t)code_at(qx, k) * (int64_t)code_at(qw, k);
    return a;
}

/* ------------------------------- weight-only variant (W4A16, Table B.3) ---- */

/* Round T rows of K doubles to fp16 (nearest even): the 16-bit activations of
   the weight-only setting are the rotated rows X R of Eq. 1 kept in fp16. */
void sqo_round_rows_to_half(const double *Xrot, int64_t T, int K,
                            uint16_t *Xh, int64_t ldo)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t)
        for (int k = 0; k < K; ++k)
            Xh[t * ldo + k] = sqo_double_to_half(Xrot[t * (int64_t)K + k]);
}

/* Y[t,n] = fp16( sw[n] * sum_k x[t,k] qw[n,k] ): Eq. 1 with only the weight
   operand quantized (4-bit codes and per-output-channel steps, Sec. 3.2),
   the activations fp16 values read as exact reals; sums in fp64, one rounding
   to fp16 at the end.  abs_sum (may be NULL) receives sw[n] * sum_k |x qw|,
   the size that bounds the error of any other summation order. */
int sqo_gemm_w4a16(const uint16_t *Xh, int64_t T, int K, int64_t ldx,
                   const uint8_t *Qw, const float *sw, int N,
                   uint16_t *Y, int64_t ldy, double *abs_sum)
{
    if (K <= 0 || (K & 1) || T < 0 || N < 0 || ldy < N || ldx < K) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int n = 0; n < N; ++n) {
            const uint8_t *qw = Qw + (int64_t)n * (K / 2);
            double a = 0.0, m = 0.0;
            for (int k = 0; k < K; ++k) {
                double term = sqo_half_to_double(Xh[t * ldx + k]) * (double)code_at(qw, k);
                a += term;
                m += fabs(term);
            }
            Y[t * ldy + n] = sqo_double_to_half(a * (double)sw[n]);
            if (abs_sum) abs_sum[t * (int64_t)N + n] = m * (double)sw[n];
        }
    }
    return 0;
}

/* --------------------------------------------------------- Alg. 1 -------- */

/* n2 = the power of two dividing n that is closest to sqrt(n) (first found
   wins ties, scanning upwards), n1 = n / n2. */
void sqo_kron_factor(int64_t n, int64_t *n1, int64_t *n2)
{
    double root = sqrt((double)n);
    int64_t best = 1;
    for (int64_t a = 1; a <= n; a *= 2) {
        if (n % a != 0) continue;
        if (fabs((double)a - root) < fabs((double)best - root)) best = a;
    }
    *n2 = best;
    *n1 = n / best;
}

int sqo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
