// sq_w4a4_gemm: int4 x int4 GEMM on the int8 matrix cores of gfx950 with a dequantizing epilogue
// (Eq. 1 of the paper evaluated on the 4-bit codes; the weight operand is Flat(W~_R) = W^T R of
// Sec. 4.2, one K-contiguous row per output channel).
//
//   acc[t, n] = sum_k Qx[t, k] Qw[n, k]   (int32, exact)      Y[t, n] = fp16(acc * sx[t] * sw[n])
//
// Nibbles are widened to int8 in registers as (code << 4): "w & 0xF0F0F0F0" yields the odd codes
// of a dword times 16 with their sign in place, "(w << 4) & 0xF0F0F0F0" the even ones.  Both
// operands carry the factor 16, so the int32 accumulator holds 256 * acc exactly
// (64 * K * 256 < 2^31 for K <= 131072) and the epilogue shifts it out.  The split into even and
// odd codes permutes the contraction index the same way on both operands, which a dot product
// does not see.
#include "sq_common.h"

namespace sq {

// LDS tile of one operand: ROWS rows of BKB bytes (2*BKB codes), stored as 16-byte chunks.
// Chunk c of row r sits at chunk slot r*CPR + (c ^ swz(r)): 8 consecutive rows then touch 8
// different 16-byte bank groups both for the row-major writes and for the MFMA-fragment reads.
template <int BKB>
__device__ __forceinline__ int lds_chunk_slot(int row, int chunk)
{
    constexpr int CPR = BKB / 16;
    static_assert(CPR == 4 || CPR == 8, "tile row must be 64 or 128 bytes");
    const int swz = (CPR == 8) ? (row & 7) : ((row >> 1) & 3);
    return row * CPR + (chunk ^ swz);
}

__device__ __forceinline__ void widen_chunk(const uint4 w, v4i &first, v4i &second)
{
    const uint32_t m = 0xF0F0F0F0u;
    first = v4i{(int)((w.x << 4) & m), (int)(w.x & m), (int)((w.y << 4) & m), (int)(w.y & m)};
    second = v4i{(int)((w.z << 4) & m), (int)(w.z & m), (int)((w.w << 4) & m), (int)(w.w & m)};
}

// Block tile (WM*FM*32) x (WN*FN*32), WM*WN waves, each wave FM x FN fragments of 32x32.
// K is walked in tiles of 2*BKB codes: global -> registers (prefetch of the next tile while the
// current one is multiplied) -> LDS (still packed) -> registers -> widen -> MFMA.
template <int WM, int WN, int FM, int FN, int BKB>
__global__ __launch_bounds__(WM *WN *kWave) void w4a4_gemm_kernel(
    const uint8_t *__restrict__ Qx, const float *__restrict__ sx, int T, int Kb,
    const uint8_t *__restrict__ Qw, const float *__restrict__ sw, int N, __half *__restrict__ Y,
    int64_t ldy, int32_t *__restrict__ acc_dbg, int tiles_m, int tiles_n)
{
    constexpr int NT = WM * WN * kWave;
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
    constexpr int CPR = BKB / 16;
    constexpr int A_CHUNKS = BM * CPR, B_CHUNKS = BN * CPR;
    constexpr int A_PER = A_CHUNKS / NT, B_PER = B_CHUNKS / NT;
    static_assert(A_CHUNKS % NT == 0 && B_CHUNKS % NT == 0, "tile must split evenly over threads");

    __shared__ uint4 sA[A_CHUNKS];
    __shared__ uint4 sB[B_CHUNKS];

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int wm = wave / WN, wn = wave % WN;

    // XCD-contiguous ids, then groups of 8 row-tiles walked column by column: the 32 tiles that
    // are resident on one XCD share a few row panels and a few column panels in its L2.
    const int id = xcd_contiguous_id(blockIdx.x, tiles_m * tiles_n);
    constexpr int GM = 8;
    const int group = id / (GM * tiles_n);
    const int gm = min(GM, tiles_m - group * GM);
    const int in_group = id - group * GM * tiles_n;
    const int bm = group * GM + in_group % gm, bn = in_group / gm;

    const int row0 = bm * BM, col0 = bn * BN;

    // global-load assignment: chunk g*NT + tid of the tile -> (row, chunk-in-row)
    const uint8_t *a_src[A_PER];
    const uint8_t *b_src[B_PER];
    int a_slot[A_PER], b_slot[B_PER], a_off[A_PER], b_off[B_PER];
#pragma unroll
    for (int g = 0; g < A_PER; ++g) {
        const int c = g * NT + tid, r = c / CPR, ch = c % CPR;
        a_src[g] = Qx + (int64_t)min(row0 + r, T - 1) * Kb + ch * 16;   // clamped: rows past T are never stored
        a_slot[g] = lds_chunk_slot<BKB>(r, ch);
        a_off[g] = ch * 16;
    }
#pragma unroll
    for (int g = 0; g < B_PER; ++g) {
        const int c = g * NT + tid, r = c / CPR, ch = c % CPR;
        b_src[g] = Qw + (int64_t)min(col0 + r, N - 1) * Kb + ch * 16;
        b_slot[g] = lds_chunk_slot<BKB>(r, ch);
        b_off[g] = ch * 16;
    }

    v16i acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    uint4 ra[A_PER], rb[B_PER];
    const int ktiles = (Kb + BKB - 1) / BKB;
    auto fetch = [&](int kt) {
        const int kb0 = kt * BKB;
#pragma unroll
        for (int g = 0; g < A_PER; ++g)
            ra[g] = (kb0 + a_off[g] < Kb) ? *reinterpret_cast<const uint4 *>(a_src[g] + kb0) : uint4{0, 0, 0, 0};
#pragma unroll
        for (int g = 0; g < B_PER; ++g)
            rb[g] = (kb0 + b_off[g] < Kb) ? *reinterpret_cast<const uint4 *>(b_src[g] + kb0) : uint4{0, 0, 0, 0};
    };

    fetch(0);
    const int frow = lane & 31, fhalf = lane >> 5;
    for (int kt = 0; kt < ktiles; ++kt) {
        __syncthreads();     // everyone is done reading the previous tile
#pragma unroll
        for (int g = 0; g < A_PER; ++g) sA[a_slot[g]] = ra[g];
#pragma unroll
        for (int g = 0; g < B_PER; ++g) sB[b_slot[g]] = rb[g];
        __syncthreads();
        if (kt + 1 < ktiles) fetch(kt + 1);

#pragma unroll
        for (int s = 0; s < CPR / 2; ++s) {
            const int ch = 2 * s + fhalf;
            v4i af[FM][2], bf[FN][2];
#pragma unroll
            for (int i = 0; i < FM; ++i)
                widen_chunk(sA[lds_chunk_slot<BKB>((wm * FM + i) * 32 + frow, ch)], af[i][0], af[i][1]);
#pragma unroll
            for (int j = 0; j < FN; ++j)
                widen_chunk(sB[lds_chunk_slot<BKB>((wn * FN + j) * 32 + frow, ch)], bf[j][0], bf[j][1]);
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i][u], bf[j][u], acc[i][j], 0, 0, 0);
        }
    }

    // epilogue.  32x32 accumulator layout: lane holds column (lane % 32); register e holds row
    // 8 * (e / 4) + 4 * (lane / 32) + e % 4.
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int n = col0 + (wn * FN + j) * 32 + frow;
        if (n >= N) continue;
        const float swn = sw[n];
#pragma unroll
        for (int i = 0; i < FM; ++i) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int t = row0 + (wm * FM + i) * 32 + 8 * (e / 4) + 4 * fhalf + (e % 4);
                if (t >= T) continue;
                const int a = acc[i][j][e] >> 8;
                Y[(int64_t)t * ldy + n] = __float2half_rn((float)a * sx[t] * swn);
                if (acc_dbg != nullptr) acc_dbg[(int64_t)t * N + n] = a;
            }
        }
    }
}

template <int WM, int WN, int FM, int FN, int BKB>
static sq_status launch_gemm(const uint8_t *Qx, const float *sx, int T, int K, const uint8_t *Qw,
                             const float *sw, int N, __half *Y, int64_t ldy, int32_t *acc_dbg,
                             hipStream_t st)
{
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
    const int tiles_m = (T + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    hipLaunchKernelGGL((w4a4_gemm_kernel<WM, WN, FM, FN, BKB>), dim3((unsigned)(tiles_m * tiles_n)),
                       dim3(WM * WN * kWave), 0, st, Qx, sx, T, K / 2, Qw, sw, N, Y, ldy, acc_dbg,
                       tiles_m, tiles_n);
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

}  // namespace sq

extern "C" sq_status sq_w4a4_gemm(const uint8_t *Qx, const float *sx, int64_t T, int32_t K,
                                  const uint8_t *Qw, const float *sw, int32_t N, void *Y,
                                  int64_t ldy, int32_t *acc_dbg, void *stream)
{
    if (T < 0 || N < 0 || K <= 0 || (K % 32) != 0 || K > 131072) return SQ_ERR_SHAPE;
    if (T > (1 << 24) || ldy < N) return SQ_ERR_SHAPE;
    if (T == 0 || N == 0) return SQ_OK;
    if (!Qx || !sx || !Qw || !sw || !Y) return SQ_ERR_NULL;
    if (((uintptr_t)Qx & 15) || ((uintptr_t)Qw & 15) || ((uintptr_t)Y & 1) ||
        ((uintptr_t)sx & 3) || ((uintptr_t)sw & 3) || ((uintptr_t)acc_dbg & 3))
        return SQ_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return sq::launch_gemm<2, 2, 2, 4, 128>(Qx, sx, (int)T, K, Qw, sw, N, static_cast<__half *>(Y),
                                            ldy, acc_dbg, st);
}
