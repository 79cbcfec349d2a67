// sq_w4a16_gemm: fp16 activations times 4-bit weight codes on the fp16 matrix cores of gfx950, with
// the per-output-channel step applied in the epilogue -- the weight-only setting of the paper's
// appendix (weight-only quantization table): Eq. 1 with only the weight operand quantized, the
// weight operand being Flat(W~_R) = W^T R of Sec. 4.2, one K-contiguous row of codes per channel.
//
//   Y[t, n] = fp16( sw[n] * sum_k X[t, k] * Qw[n, k] )        fp32 accumulation
//
// Codes are widened to fp16 in registers: with x = dword ^ 0x88888888 every nibble holds code + 8,
// "(x >> 4j) & 0x000F000F | 0x64006400" is the pair of halves (1024 + code_j + 8, 1024 + code_{j+4} + 8),
// and one packed subtraction of 1032 leaves the codes themselves, exactly.  A dword therefore
// yields its eight codes in the order 0 4 1 5 2 6 3 7; the activations of a 16-byte chunk are put
// into the same order, which a dot product does not see.  Both happen once per element, on the way
// into LDS (every tile row is read by two waves afterwards): the loop over a tile is then LDS reads
// and MFMAs only.
#include "sq_common.h"

namespace sq {

namespace {

constexpr int kBM = 128, kBN = 128, kBK = 64;      // block tile and codes per K tile
constexpr int kXRow = kBK * 2, kWRow = kBK / 2;    // bytes of a tile row in memory: activations, weight codes

// halves 0..7 of a chunk -> order 0 4 1 5 2 6 3 7 (dword d holds halves 2d, 2d+1)
__device__ __forceinline__ uint4 interleave_halves(const uint4 v)
{
    uint4 r;
    r.x = __builtin_amdgcn_perm(v.z, v.x, 0x05040100u);      // (x0, x4)
    r.y = __builtin_amdgcn_perm(v.z, v.x, 0x07060302u);      // (x1, x5)
    r.z = __builtin_amdgcn_perm(v.w, v.y, 0x05040100u);      // (x2, x6)
    r.w = __builtin_amdgcn_perm(v.w, v.y, 0x07060302u);      // (x3, x7)
    return r;
}

// eight codes of a dword as fp16, in the order 0 4 1 5 2 6 3 7
__device__ __forceinline__ v8h widen_codes_f16(uint32_t w)
{
    const uint32_t x = w ^ 0x88888888u;
    const v2h bias = {(_Float16)1032.f, (_Float16)1032.f};
    v2h p[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        p[j] = __builtin_bit_cast(v2h, ((x >> (4 * j)) & 0x000F000Fu) | 0x64006400u) - bias;
    return v8h{p[0][0], p[0][1], p[1][0], p[1][1], p[2][0], p[2][1], p[3][0], p[3][1]};
}

// Block tile 128 x 128, four waves of 64 x 64 (2 x 2 fragments of 32 x 32), K walked in tiles of 64
// codes.  Tiles travel global -> registers -> LDS (activations reordered, codes widened to fp16 on
// the way), the next tile's loads in flight while this one is multiplied; two LDS buffers, one
// barrier per tile.  Both operands sit in LDS as rows of eight 16-byte chunks (eight fp16 values
// each), chunk c of row r at slot r * 8 + (c ^ (r & 7)).  Within a K tile lane half g takes codes
// 32g .. 32g + 31 and step s the eight codes 32g + 8s ..: chunk 4g + s of its row, for both operands.
__global__ __launch_bounds__(256, 2) void w4a16_gemm_kernel(
    const __half *__restrict__ X, int64_t ldx, int T, int K, const uint8_t *__restrict__ Qw,
    const float *__restrict__ sw, int N, __half *__restrict__ Y, int64_t ldy, int tiles_m, int tiles_n)
{
    __shared__ uint4 xs[2][kBM * 8];               // activations
    __shared__ uint4 ws[2][kBN * 8];               // weight codes as fp16

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int l32 = lane & 31, g = lane >> 5, wm = wave >> 1, wn = wave & 1;
    // XCD-contiguous tile ids, column-major inside groups of 8 row tiles: the tiles resident on one
    // XCD share a few row and column panels in its L2
    int bm, bn;
    {
        const int id = xcd_contiguous_id(blockIdx.x, tiles_m * tiles_n);
        constexpr int GM = 8;
        const int group = id / (GM * tiles_n), gm = min(GM, tiles_m - group * GM);
        const int in_group = id - group * GM * tiles_n;
        bm = group * GM + in_group % gm;
        bn = in_group / gm;
    }
    const int row0 = bm * kBM, col0 = bn * kBN, Kb = K / 2;

    // this thread's share of a tile: four activation chunks, one weight chunk (rows past the ends
    // are clamped: their products are never stored)
    const __half *x_src[4];
    int x_slot[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int c = tid + 256 * u, r = c >> 3, ch = c & 7;
        x_src[u] = X + (int64_t)min(row0 + r, T - 1) * ldx + ch * 8;
        x_slot[u] = r * 8 + (ch ^ (r & 7));
    }
    const uint8_t *w_src = Qw + (int64_t)min(col0 + (tid >> 1), N - 1) * Kb + (tid & 1) * 16;
    // the 32 codes of this thread's weight chunk become chunks 4 (tid & 1) .. + 3 of row tid >> 1
    int w_slot[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) w_slot[u] = (tid >> 1) * 8 + ((4 * (tid & 1) + u) ^ ((tid >> 1) & 7));

    v16f acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    uint4 xr[4], wr;
    auto fetch = [&](int kt) {
#pragma unroll
        for (int u = 0; u < 4; ++u) xr[u] = *reinterpret_cast<const uint4 *>(x_src[u] + kt * kBK);
        wr = *reinterpret_cast<const uint4 *>(w_src + kt * kWRow);
    };
    auto park = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 4; ++u) xs[buf][x_slot[u]] = interleave_halves(xr[u]);
        const uint32_t wd[4] = {wr.x, wr.y, wr.z, wr.w};
#pragma unroll
        for (int u = 0; u < 4; ++u) ws[buf][w_slot[u]] = __builtin_bit_cast(uint4, widen_codes_f16(wd[u]));
    };

    const int ktiles = K / kBK;
    fetch(0);
    park(0);
    __syncthreads();
    for (int kt = 0; kt < ktiles; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < ktiles) fetch(kt + 1);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            v8h a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int r = wm * 64 + 32 * i + l32;
                a[i] = __builtin_bit_cast(v8h, xs[buf][r * 8 + ((4 * g + s) ^ (r & 7))]);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int r = wn * 64 + 32 * j + l32;
                b[j] = __builtin_bit_cast(v8h, ws[buf][r * 8 + ((4 * g + s) ^ (r & 7))]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < ktiles) park(buf ^ 1);
        __syncthreads();
    }

    // 32 x 32 accumulator layout: lane holds channel l32, register e holds token 8 (e / 4) + 4 g + e % 4
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int n = col0 + wn * 64 + 32 * j + l32;
        if (n >= N) continue;
        const float step = sw[n];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int t = row0 + wm * 64 + 32 * i + 8 * (e / 4) + 4 * g + (e % 4);
                if (t < T) Y[(int64_t)t * ldy + n] = __float2half_rn(acc[i][j][e] * step);
            }
    }
}

// Decode-shaped kernel (T <= 32, K % 256 == 0): the product is one pass over the weight codes,
// 117 MB for 8 tokens at K = 8192, N = 28672, and the tile kernel above would walk K in 224
// workgroups one tile at a time.  Here a workgroup owns 16 NS output channels and one block of 16
// tokens (v_mfma_f32_16x16x32_f16: lane = token or channel l % 16, its quarter q = l / 16 of the
// 32 contraction indices of a step); its NW waves split K in slices of 256 codes dealt round-robin
// and add their partial sums through LDS at the end.  Both operands go global -> registers, the
// next slice in flight while this one is multiplied.  Per slice a lane reads the 64 codes
// [64 q, 64 q + 64) of its channel rows (two 16-byte loads each, so that the four quarters of a
// wave consume whole 128-byte lines) and the same 64 activations of its token (128 contiguous
// bytes); dword d of chunk c, widened, is the operand of step (c, d), against the activations
// 32 c + 8 d .. + 7 of the lane's 64, put into the order 0 4 1 5 2 6 3 7 the widening produces.
template <int NS, int NW>
__global__ __launch_bounds__(NW *kWave) void w4a16_gemm_skinny_kernel(
    const __half *__restrict__ X, int64_t ldx, int T, int K, const uint8_t *__restrict__ Qw,
    const float *__restrict__ sw, int N, __half *__restrict__ Y, int64_t ldy)
{
    constexpr int BN = 16 * NS;
    static_assert(NW * NS * 4 * kWave * 4 <= 64 * 1024, "partial sums must fit in static LDS");
    __shared__ float red[NW][NS][4][kWave];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int l16 = lane & 15, q = lane >> 4;
    const int col0 = blockIdx.x * BN, t0 = blockIdx.y * 16, Kb = K / 2;

    // rows past the ends are clamped: their products are never stored
    const __half *a_ptr = X + (int64_t)min(t0 + l16, T - 1) * ldx + q * 64;
    const uint8_t *b_ptr[NS];
#pragma unroll
    for (int j = 0; j < NS; ++j) b_ptr[j] = Qw + (int64_t)min(col0 + 16 * j + l16, N - 1) * Kb + q * 32;

    v4f acc[NS];
#pragma unroll
    for (int j = 0; j < NS; ++j) acc[j] = v4f{0.f, 0.f, 0.f, 0.f};

    uint4 ra[2][8], rb[2][NS][2];
    const int slices = K / 256;
#define SQ_W16_FETCH(BUF, S)                                                                         \
    do {                                                                                             \
        _Pragma("unroll") for (int j = 0; j < NS; ++j)                                               \
            _Pragma("unroll") for (int c = 0; c < 2; ++c)                                            \
                rb[BUF][j][c] = *reinterpret_cast<const uint4 *>(b_ptr[j] + (S) * 128 + 16 * c);     \
        _Pragma("unroll") for (int u = 0; u < 8; ++u)                                                \
            ra[BUF][u] = *reinterpret_cast<const uint4 *>(a_ptr + (S) * 256 + 8 * u);                \
    } while (0)
#define SQ_W16_MULTIPLY(BUF)                                                                         \
    do {                                                                                             \
        _Pragma("unroll") for (int c = 0; c < 2; ++c)                                                \
            _Pragma("unroll") for (int d = 0; d < 4; ++d) {                                          \
                const v8h a = __builtin_bit_cast(v8h, interleave_halves(ra[BUF][4 * c + d]));        \
                _Pragma("unroll") for (int j = 0; j < NS; ++j) {                                     \
                    const uint4 w4 = rb[BUF][j][c];                                                  \
                    const uint32_t w = d == 0 ? w4.x : d == 1 ? w4.y : d == 2 ? w4.z : w4.w;         \
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, widen_codes_f16(w), acc[j], 0, 0, 0); \
                }                                                                                    \
            }                                                                                        \
    } while (0)

    // wave w takes slices w, w + NW, w + 2 NW, ...; two register sets alternate
    int S = wave;
    if (S < slices) SQ_W16_FETCH(0, S);
    while (S < slices) {
        if (S + NW < slices) SQ_W16_FETCH(1, S + NW);
        SQ_W16_MULTIPLY(0);
        S += NW;
        if (S >= slices) break;
        if (S + NW < slices) SQ_W16_FETCH(0, S + NW);
        SQ_W16_MULTIPLY(1);
        S += NW;
    }
#undef SQ_W16_FETCH
#undef SQ_W16_MULTIPLY

#pragma unroll
    for (int j = 0; j < NS; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wave][j][r][lane] = acc[j][r];
    __syncthreads();
    // 16 x 16 accumulator layout: lane holds channel l % 16, register r holds token 4 (l / 16) + r
    for (int idx = tid; idx < NS * 4 * kWave; idx += NW * kWave) {
        const int ln = idx & (kWave - 1), r = (idx >> 6) & 3, j = idx >> 8;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) sum += red[w][j][r][ln];
        const int t = t0 + 4 * (ln >> 4) + r, n = col0 + 16 * j + (ln & 15);
        if (t < T && n < N) Y[(int64_t)t * ldy + n] = __float2half_rn(sum * sw[n]);
    }
}

template <int NS, int NW>
sq_status launch_w4a16_skinny(const __half *X, int64_t ldx, int T, int K, const uint8_t *Qw, const float *sw, int N,
                              __half *Y, int64_t ldy, hipStream_t st)
{
    hipLaunchKernelGGL((w4a16_gemm_skinny_kernel<NS, NW>), dim3((unsigned)((N + 16 * NS - 1) / (16 * NS)), (unsigned)((T + 15) / 16)),
                       dim3(NW * kWave), 0, st, X, ldx, T, K, Qw, sw, N, Y, ldy);
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

}  // namespace

}  // namespace sq

extern "C" sq_status sq_w4a16_gemm(const void *X, int64_t T, int32_t K, int64_t ldx, const uint8_t *Qw,
                                   const float *sw, int32_t N, void *Y, int64_t ldy, void *stream)
{
    if (T < 0 || N < 0 || K <= 0 || (K % sq::kBK) != 0 || K > 131072) return SQ_ERR_SHAPE;
    if (T > (1 << 24) || ldx < K || ldy < N) return SQ_ERR_SHAPE;
    if (T == 0 || N == 0) return SQ_OK;
    if (!X || !Qw || !sw || !Y) return SQ_ERR_NULL;
    if (((uintptr_t)X & 15) || (ldx % 8) != 0 || ((uintptr_t)Qw & 15) || ((uintptr_t)Y & 1) || ((uintptr_t)sw & 3))
        return SQ_ERR_ALIGN;
    // At most 32 tokens: one pass over the weights (two token blocks above 16 tokens read them twice,
    // the second time mostly out of the caches; beyond that the tile kernel is the better choice).
    // Launch shapes as in the W4A4 decode-shaped kernel: about eight waves on every CU.
    if (T <= 32 && (K % 256) == 0) {
        const hipStream_t st = static_cast<hipStream_t>(stream);
        const __half *Xh = static_cast<const __half *>(X);
        __half *Yh = static_cast<__half *>(Y);
        if (N >= 64 * 384) return sq::launch_w4a16_skinny<4, 4>(Xh, ldx, (int)T, K, Qw, sw, N, Yh, ldy, st);
        return sq::launch_w4a16_skinny<2, 8>(Xh, ldx, (int)T, K, Qw, sw, N, Yh, ldy, st);
    }
    const int tiles_m = (int)((T + sq::kBM - 1) / sq::kBM), tiles_n = (N + sq::kBN - 1) / sq::kBN;
    hipLaunchKernelGGL(sq::w4a16_gemm_kernel, dim3((unsigned)(tiles_m * tiles_n)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const __half *>(X), ldx, (int)T, K, Qw, sw, N,
                       static_cast<__half *>(Y), ldy, tiles_m, tiles_n);
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}
