// sq_prepare_weights: offline weight path (Sec. 4.2).  W [K, N] is transposed into the caller's
// workspace, then every row of W^T (one output channel) takes the same path as a token row:
// Givens list, Kronecker rotation, per-row int4 quantizer (sq_rotate_quantize).
#include "sq_common.h"

namespace sq {

// 64 x 64 tile through LDS.  Tiles that lie inside the matrix move in 8-byte accesses on both
// sides (four halves along n in, four halves along k out) when the pointers and leading dimensions
// allow it (vec); edge tiles and unaligned matrices go element by element with bounds checks.
// The LDS row stride of 66 halves keeps both the row-wise writes and the column-wise reads spread
// over the banks.
__global__ __launch_bounds__(256) void transpose_fp16_kernel(const __half *__restrict__ W, int K, int N,
                                                             int64_t ldw, __half *__restrict__ Wt, int vec)
{
    constexpr int TILE = 64, LD = TILE + 2;
    __shared__ __half tile[TILE * LD];
    const int k0 = blockIdx.y * TILE, n0 = blockIdx.x * TILE;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;       // 16 x 16 threads, 4 elements each
    const bool fast = vec && k0 + TILE <= K && n0 + TILE <= N;    // the same for the whole block
    if (fast) {
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int kl = ty + 16 * pass;
            const uint2 v = *reinterpret_cast<const uint2 *>(W + (int64_t)(k0 + kl) * ldw + n0 + 4 * tx);
            uint32_t *dst = reinterpret_cast<uint32_t *>(tile + kl * LD + 4 * tx);      // 4-byte aligned: LD, 4 tx even
            dst[0] = v.x;
            dst[1] = v.y;
        }
    } else {
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int k = k0 + ty + 16 * pass, n = n0 + 4 * tx;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                tile[(ty + 16 * pass) * LD + 4 * tx + e] =
                    (k < K && n + e < N) ? W[(int64_t)k * ldw + n + e] : __float2half(0.f);
        }
    }
    __syncthreads();
    const uint16_t *t16 = reinterpret_cast<const uint16_t *>(tile);
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
        const int nl = ty + 16 * pass, n = n0 + nl, k = k0 + 4 * tx;
        if (fast) {
            const uint32_t lo = t16[(4 * tx) * LD + nl] | ((uint32_t)t16[(4 * tx + 1) * LD + nl] << 16);
            const uint32_t hi = t16[(4 * tx + 2) * LD + nl] | ((uint32_t)t16[(4 * tx + 3) * LD + nl] << 16);
            *reinterpret_cast<uint2 *>(Wt + (int64_t)n * K + k) = uint2{lo, hi};
        } else if (n < N) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (k + e < K) Wt[(int64_t)n * K + k + e] = tile[(4 * tx + e) * LD + nl];
        }
    }
}

}  // namespace sq

extern "C" sq_status sq_prepare_weights_variant(const void *W, int32_t K, int32_t N, int64_t ldw,
                                                const int32_t *giv_i, const int32_t *giv_j,
                                                const float *giv_theta, int32_t P, const void *R1,
                                                int32_t n1, const void *R2, int32_t n2, int32_t bits,
                                                float clip_ratio, void *workspace, uint8_t *Qw,
                                                float *sw, void *stream)
{
    if (N < 0 || K <= 0 || ldw < N) return SQ_ERR_SHAPE;
    if (N > 0 && (!W || !workspace)) return SQ_ERR_NULL;
    if (((uintptr_t)W & 1) || ((uintptr_t)workspace & 15)) return SQ_ERR_ALIGN;
    // every other check (shape limits, Givens indices, R1/R2/Qw/sw pointers) is the row kernel's;
    // run it on an empty batch first so that nothing is enqueued when an argument is bad
    const sq_status pre = sq_rotate_quantize_variant(workspace, 0, K, K, giv_i, giv_j, giv_theta, P, R1, n1, R2, n2,
                                                     bits, clip_ratio, Qw, sw, nullptr, stream);
    if (pre != SQ_OK) return pre;
    if (N == 0) return SQ_OK;
    if (!Qw || !sw) return SQ_ERR_NULL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(sq::transpose_fp16_kernel, dim3((unsigned)((N + 63) / 64), (unsigned)((K + 63) / 64)),
                       dim3(256), 0, st, static_cast<const __half *>(W), K, N, ldw,
                       static_cast<__half *>(workspace),
                       (((uintptr_t)W & 7) == 0 && (ldw % 4) == 0 && (K % 4) == 0) ? 1 : 0);
    if (hipGetLastError() != hipSuccess) return SQ_ERR_LAUNCH;
    return sq_rotate_quantize_variant(workspace, N, K, K, giv_i, giv_j, giv_theta, P, R1, n1, R2, n2, bits,
                                      clip_ratio, Qw, sw, nullptr, stream);
}

extern "C" sq_status sq_prepare_weights(const void *W, int32_t K, int32_t N, int64_t ldw,
                                        const int32_t *giv_i, const int32_t *giv_j,
                                        const float *giv_theta, int32_t P, const void *R1, int32_t n1,
                                        const void *R2, int32_t n2, void *workspace, uint8_t *Qw,
                                        float *sw, void *stream)
{
    return sq_prepare_weights_variant(W, K, N, ldw, giv_i, giv_j, giv_theta, P, R1, n1, R2, n2, 4, 1.0f,
                                      workspace, Qw, sw, stream);
}
