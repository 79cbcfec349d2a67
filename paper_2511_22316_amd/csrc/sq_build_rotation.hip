// sq_build_rotation: the closed-form construction of the rotation from calibration activations
// (Sec. 4.2: ART with the angle of Lemma 1, URT, the Hadamard factor, the composition of "The
// Overall SingleQuant Method"), and sq_kron_factor (Alg. 1).
//
// One pass over the calibration activations finds the calibration row (HBM-bound, the only part
// that touches more than a few hundred KB); everything after it is small and runs in a handful
// of tiny launches:
//   row_absmax_kernel     max |x| of every token row
//   art_urt_kernel        one workgroup: calibration row, P ART steps, the vectors of the two URTs,
//                         their uniform targets, and the four chains of plane rotations
//   rmap_kernel           the four maps to e_1 as dense matrices, row by row in closed form
//   urt_product_kernel    R^U = R_map R'_map^T for both sides (side 1 is R1)
//   hadamard_left_kernel  R2 = H R^U_2
//
// Wherever floating point decides an index -- the ART channels and the rank order of the URT --
// the deciding values are computed in fp32 with one rounding per operation, in index order: every
// such product and sum passes through an opaque register, so the compiler can neither fuse a
// multiply with an add nor reorder a sum (square root and division are the correctly rounded ones
// hipcc uses by default).
#include "sq_common.h"

#include <math.h>

namespace sq {

namespace {

constexpr int kBuildThreads = 1024;
constexpr int kBuildWaves = kBuildThreads / kWave;
constexpr int kMaxSide = 256;                 // n1 <= 128, n2 <= 256
constexpr int kBuildSmallBytes = 2 * kBuildWaves * 8 + 5 * kMaxSide * 4;

// workspace, in floats
struct BuildWorkspace {
    float *rowmax;      // [T]
    float *chain;       // [side 0..1][vector V, U][cos, sin][kMaxSide]
    float *rmap[4];     // side 1: V, U (n1 x n1 each); side 2: V, U (n2 x n2 each)
    float *ru2;         // n2 x n2
};

__host__ int64_t build_workspace_floats(int64_t T, int n1, int n2)
{
    const int64_t t_pad = (T + 63) / 64 * 64;
    return t_pad + 8 * kMaxSide + 2 * (int64_t)n1 * n1 + 3 * (int64_t)n2 * n2;
}

__host__ BuildWorkspace carve_workspace(void *workspace, int64_t T, int n1, int n2)
{
    BuildWorkspace w;
    float *p = static_cast<float *>(workspace);
    w.rowmax = p;
    p += (T + 63) / 64 * 64;
    w.chain = p;
    p += 8 * kMaxSide;
    w.rmap[0] = p;
    p += (int64_t)n1 * n1;
    w.rmap[1] = p;
    p += (int64_t)n1 * n1;
    w.rmap[2] = p;
    p += (int64_t)n2 * n2;
    w.rmap[3] = p;
    p += (int64_t)n2 * n2;
    w.ru2 = p;
    return w;
}

typedef unsigned short v2us __attribute__((ext_vector_type(2)));

// fp32 product / sum rounded once, to nearest: the empty statement hides the value from the
// optimiser, so it is a result in a register before anything else uses it
__device__ __forceinline__ float rn_mul(float a, float b)
{
    float r = a * b;
    asm volatile("" : "+v"(r));
    return r;
}
__device__ __forceinline__ float rn_add(float a, float b)
{
    float r = a + b;
    asm volatile("" : "+v"(r));
    return r;
}
__device__ __forceinline__ uint64_t larger(uint64_t a, uint64_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint64_t smaller(uint64_t a, uint64_t b) { return a < b ? a : b; }

// max |x| per token row.  One wave per row; a lane reads 16 bytes at a time, four loads in
// flight.  |fp16| bit patterns order like unsigned integers, so the maximum is taken on the
// masked 16-bit patterns, two per instruction, and converted once at the end.
__global__ __launch_bounds__(256) void row_absmax_kernel(const __half *__restrict__ X, int64_t ldx, int T, int K,
                                                         float *__restrict__ rowmax)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int chunks = K / 8;
    for (int t = blockIdx.x * 4 + wave; t < T; t += gridDim.x * 4) {
        const uint4 *row = reinterpret_cast<const uint4 *>(X + (int64_t)t * ldx);
        v2us m = {0, 0};
        for (int c0 = 0; c0 < chunks; c0 += 4 * kWave) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + u * kWave + lane;
                v[u] = (c < chunks) ? row[c] : uint4{0, 0, 0, 0};
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    m = __builtin_elementwise_max(m, __builtin_bit_cast(v2us, w[e] & 0x7FFF7FFFu));
            }
        }
        const unsigned short top = m[0] > m[1] ? m[0] : m[1];
        const float f = wave_max(__half2float(__ushort_as_half(top)));
        if (lane == 0) rowmax[t] = f;
    }
}

__device__ __forceinline__ uint64_t shfl_xor_u64(uint64_t v, int mask)
{
    const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)v, mask, kWave);
    const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(v >> 32), mask, kWave);
    return ((uint64_t)hi << 32) | lo;
}

// largest (or smallest) key of the workgroup, returned in every thread; `slots` holds one key
// per wave and must not be rewritten before every thread has passed a later barrier
template <bool LARGEST>
__device__ __forceinline__ uint64_t block_select(uint64_t key, uint64_t *slots)
{
#pragma unroll
    for (int off = kWave / 2; off >= 1; off >>= 1) {
        const uint64_t o = shfl_xor_u64(key, off);
        key = LARGEST ? (o > key ? o : key) : (o < key ? o : key);
    }
    if ((threadIdx.x & (kWave - 1)) == 0) slots[threadIdx.x / kWave] = key;
    __syncthreads();
    uint64_t best = slots[0];
#pragma unroll
    for (int w = 1; w < kBuildWaves; ++w) {
        const uint64_t o = slots[w];
        best = LARGEST ? (o > best ? o : best) : (o < best ? o : best);
    }
    return best;
}

// Givens chain that takes `vec` (n entries) to ||vec|| e_1: entry k is zeroed by a rotation in the
// plane (k - 1, k), k = n - 1 down to 1; (cos, sin) of step k go to cs[k] and cs[kMaxSide + k].
__device__ void chain_to_e1(const float *vec, int n, float *cs)
{
    double carry = vec[n - 1];
    for (int k = n - 1; k >= 1; --k) {
        const double x = vec[k - 1], h = sqrt(x * x + carry * carry);
        const double co = (h == 0.0) ? 1.0 : x / h, si = (h == 0.0) ? 0.0 : carry / h;
        cs[k] = (float)co;
        cs[kMaxSide + k] = (float)si;
        carry = h;
    }
}

// One workgroup.  All of its LDS is dynamic (kBuildSmallBytes + 4K bytes): the reduction slots,
// the small vectors, then the calibration vector.
__global__ __launch_bounds__(kBuildThreads) void art_urt_kernel(
    const __half *__restrict__ X, int64_t ldx, int T, int K, int n1, int n2, int P, float inv_sqrt_n2,
    const float *__restrict__ rowmax, int32_t *__restrict__ giv_i, int32_t *__restrict__ giv_j,
    float *__restrict__ giv_theta, float *__restrict__ chain)
{
    extern __shared__ uint64_t build_lds[];
    uint64_t *slot_a = build_lds, *slot_b = build_lds + kBuildWaves;
    float(*vec)[kMaxSide] = reinterpret_cast<float(*)[kMaxSide]>(build_lds + 2 * kBuildWaves);   // V1 | V2 H
    float *v2 = vec[2];
    float(*target)[kMaxSide] = reinterpret_cast<float(*)[kMaxSide]>(vec[3]);                     // U1 | U2
    float *cvec = vec[5];
    const int tid = threadIdx.x;

    // calibration row: the largest row maximum, lowest row among equals
    uint64_t key = 0;
    for (int t = tid; t < T; t += kBuildThreads)
        key = larger(key, ((uint64_t)__float_as_uint(rowmax[t]) << 32) | (0xFFFFFFFFu - (uint32_t)t));
    const int t_star = (int)(0xFFFFFFFFu - (uint32_t)block_select<true>(key, slot_a));
    for (int k = tid; k < K; k += kBuildThreads) cvec[k] = __half2float(X[(int64_t)t_star * ldx + k]);
    __syncthreads();

    // ART (Sec. 4.2; several steps as in the "ART steps" study): largest against smallest
    // magnitude, angle of Lemma 1, after which both channels hold r / sqrt(2)
    for (int p = 0; p < P; ++p) {
        uint64_t hi = 0;
        for (int k = tid; k < K; k += kBuildThreads)
            hi = larger(hi, ((uint64_t)__float_as_uint(fabsf(cvec[k])) << 32) | (0xFFFFFFFFu - (uint32_t)k));
        const int i = (int)(0xFFFFFFFFu - (uint32_t)block_select<true>(hi, slot_a));
        uint64_t lo = ~0ull;
        for (int k = tid; k < K; k += kBuildThreads)
            if (k != i) lo = smaller(lo, ((uint64_t)__float_as_uint(fabsf(cvec[k])) << 32) | (uint32_t)k);
        const int j = (int)(uint32_t)block_select<false>(lo, slot_b);
        if (tid == 0) {
            const float a = cvec[i], b = cvec[j];
            const float r = sqrtf(rn_add(rn_mul(a, a), rn_mul(b, b)));
            const float e = rn_mul(r, 0.70710678118654752440f);
            giv_i[p] = i;
            giv_j[p] = j;
            giv_theta[p] = (float)(atan2((double)b, (double)a) - 0.78539816339744830962);
            cvec[i] = e;
            cvec[j] = e;
        }
        __syncthreads();
    }

    // vectors of the two URTs: means of the n1 x n2 view over the other dimension, added in index
    // order; the second one goes through the Hadamard matrix first, because H acts first in R2
    if (tid < n1) {
        float s = 0.f;
        for (int q = 0; q < n2; ++q) s = rn_add(s, cvec[tid * n2 + q]);
        vec[0][tid] = s / (float)n2;
    }
    if (tid >= 512 && tid - 512 < n2) {
        const int q = tid - 512;
        float s = 0.f;
        for (int pp = 0; pp < n1; ++pp) s = rn_add(s, cvec[pp * n2 + q]);
        v2[q] = s / (float)n1;
    }
    __syncthreads();
    if (tid < n2) {
        float s = 0.f;
        for (int a = 0; a < n2; ++a) s = rn_add(s, (__popc(a & tid) & 1) ? -v2[a] : v2[a]);
        vec[1][tid] = rn_mul(s, inv_sqrt_n2);
    }
    __syncthreads();

    // uniform targets (Sec. 4.2 URT): template q_k = (2k - n - 1)/n by rank (ties: lower index
    // first), scaled to the norm of the vector; ||q||^2 = (n^2 - 1)/(3n)
    {
        const int side = tid >= 512, k = tid - 512 * side, n = side ? n2 : n1;
        if (k < n) {
            const float *v = vec[side];
            const float mine = v[k];
            int rank = 0;
            double norm2 = 0.0;
            for (int m = 0; m < n; ++m) {
                const float o = v[m];
                rank += (o < mine) || (o == mine && m < k);
                norm2 += (double)o * (double)o;
            }
            const double qnorm2 = ((double)n * n - 1.0) / (3.0 * n);
            target[side][k] = (float)(sqrt(norm2 / qnorm2) * (2.0 * (rank + 1) - n - 1.0) / n);
        }
    }
    __syncthreads();

    // the four chains, one thread each, in four different waves
    if ((tid & (kWave - 1)) == 0 && tid < 4 * kWave) {
        const int which = tid / kWave, side = which >> 1, is_target = which & 1;
        chain_to_e1(is_target ? target[side] : vec[side], side ? n2 : n1, chain + which * 2 * kMaxSide);
    }
}

// Row r of the product of the chain (step n-1 first): nothing right of column r + 1; the entry
// that starts as 1 in column r is carried leftwards, multiplied by sin at every step.
__global__ __launch_bounds__(kMaxSide) void rmap_kernel(const float *__restrict__ chain, int n1, int n2,
                                                       float *m0, float *m1, float *m2, float *m3)
{
    const int which = blockIdx.x, n = (which >> 1) ? n2 : n1, r = threadIdx.x;
    float *M = which == 0 ? m0 : which == 1 ? m1 : which == 2 ? m2 : m3;
    const float *co = chain + which * 2 * kMaxSide, *si = co + kMaxSide;
    if (r >= n) return;
    float *row = M + (int64_t)r * n;
    for (int k = r + 2; k < n; ++k) row[k] = 0.f;
    float carry = 1.f;
    if (r + 1 < n) {
        row[r + 1] = -si[r + 1];
        carry = co[r + 1];
    }
    for (int k = r; k >= 1; --k) {
        row[k] = carry * co[k];
        carry *= si[k];
    }
    row[0] = carry;
}

// R^U = R_map R'_map^T (Sec. 4.2 URT).  blockIdx.y = side; side 1 leaves as fp16 R1, side 2 stays
// fp32 for the Hadamard factor.
__global__ __launch_bounds__(256) void urt_product_kernel(const float *__restrict__ a1, const float *__restrict__ b1,
                                                          const float *__restrict__ a2, const float *__restrict__ b2,
                                                          int n1, int n2, __half *__restrict__ R1,
                                                          float *__restrict__ ru2)
{
    const int side = blockIdx.y, n = side ? n2 : n1;
    const float *A = side ? a2 : a1, *B = side ? b2 : b1;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= n * n) return;
    const int r = idx / n, b = idx % n;
    float s = 0.f;
    for (int k = 0; k < n; ++k) s += A[r * n + k] * B[b * n + k];
    if (side) ru2[idx] = s;
    else R1[idx] = __float2half_rn(s);
}

// R2 = H R^U_2 with the normalised Sylvester Hadamard matrix, H[a][m] = (-1)^popcount(a & m) / sqrt n
__global__ __launch_bounds__(256) void hadamard_left_kernel(const float *__restrict__ ru2, int n2, float inv_sqrt_n2,
                                                            __half *__restrict__ R2)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= n2 * n2) return;
    const int a = idx / n2, b = idx % n2;
    float s = 0.f;
    for (int m = 0; m < n2; ++m) {
        const float x = ru2[m * n2 + b];
        s += (__popc(a & m) & 1) ? -x : x;
    }
    R2[idx] = __float2half_rn(s * inv_sqrt_n2);
}

bool build_shape_ok(int64_t T, int32_t K, int32_t n1, int32_t n2, int32_t P)
{
    if (T < 1 || T > 0x7FFFFFFF || K <= 0 || P < 0 || P > SQ_MAX_GIVENS) return false;
    if (n1 < 2 || n1 > SQ_MAX_N1 || n2 < 8 || n2 > SQ_MAX_N2 || (n2 & (n2 - 1)) != 0) return false;
    return (int64_t)n1 * n2 == K && K <= SQ_MAX_K;
}

}  // namespace

}  // namespace sq

extern "C" sq_status sq_kron_factor(int32_t n, int32_t *n1, int32_t *n2)
{
    if (!n1 || !n2) return SQ_ERR_NULL;
    if (n < 1) return SQ_ERR_SHAPE;
    // Alg. 1: the power of two dividing n that is closest to sqrt(n); the earlier (smaller) one
    // of two equally close candidates stays
    const double root = sqrt((double)n);
    int64_t best = 1;
    for (int64_t a = 1; a <= n; a *= 2) {
        if (n % a != 0) continue;
        if (fabs((double)a - root) < fabs((double)best - root)) best = a;
    }
    *n2 = (int32_t)best;
    *n1 = (int32_t)(n / best);
    return SQ_OK;
}

extern "C" int64_t sq_build_rotation_workspace_bytes(int64_t T, int32_t n1, int32_t n2)
{
    if (T < 1 || n1 < 1 || n2 < 1 || n1 > SQ_MAX_N1 || n2 > SQ_MAX_N2) return 0;
    return 4 * sq::build_workspace_floats(T, n1, n2);
}

extern "C" sq_status sq_build_rotation(const void *X, int64_t T, int32_t K, int64_t ldx, int32_t n1, int32_t n2,
                                       int32_t P, int32_t *giv_i, int32_t *giv_j, float *giv_theta, void *R1,
                                       void *R2, void *workspace, void *stream)
{
    if (!X || !R1 || !R2 || !workspace) return SQ_ERR_NULL;
    if (P > 0 && (!giv_i || !giv_j || !giv_theta)) return SQ_ERR_NULL;
    if (!sq::build_shape_ok(T, K, n1, n2, P) || ldx < K) return SQ_ERR_SHAPE;
    if ((ldx % 8) != 0 || ((uintptr_t)X & 15) || ((uintptr_t)R1 & 1) || ((uintptr_t)R2 & 1) ||
        ((uintptr_t)workspace & 15) || ((uintptr_t)giv_i & 3) || ((uintptr_t)giv_j & 3) || ((uintptr_t)giv_theta & 3))
        return SQ_ERR_ALIGN;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const sq::BuildWorkspace w = sq::carve_workspace(workspace, T, n1, n2);
    const float inv_sqrt_n2 = (float)(1.0 / sqrt((double)n2));
    const __half *Xh = static_cast<const __half *>(X);

    const int64_t row_groups = (T + 3) / 4;
    hipLaunchKernelGGL(sq::row_absmax_kernel, dim3((unsigned)(row_groups < 4096 ? row_groups : 4096)), dim3(256), 0,
                       st, Xh, ldx, (int)T, K, w.rowmax);
    auto art = sq::art_urt_kernel;
    const size_t lds = sq::kBuildSmallBytes + (size_t)K * sizeof(float);      // 69.4 KiB at the largest K
    if (!sq::allow_large_lds(reinterpret_cast<const void *>(art))) return SQ_ERR_LAUNCH;
    hipLaunchKernelGGL(art, dim3(1), dim3(sq::kBuildThreads), lds, st, Xh, ldx, (int)T, K, n1, n2, P, inv_sqrt_n2,
                       w.rowmax, giv_i, giv_j, giv_theta, w.chain);
    hipLaunchKernelGGL(sq::rmap_kernel, dim3(4), dim3(sq::kMaxSide), 0, st, w.chain, n1, n2, w.rmap[0], w.rmap[1],
                       w.rmap[2], w.rmap[3]);
    const int big = n1 > n2 ? n1 : n2;
    hipLaunchKernelGGL(sq::urt_product_kernel, dim3((unsigned)((big * big + 255) / 256), 2), dim3(256), 0, st,
                       w.rmap[0], w.rmap[1], w.rmap[2], w.rmap[3], n1, n2, static_cast<__half *>(R1), w.ru2);
    hipLaunchKernelGGL(sq::hadamard_left_kernel, dim3((unsigned)((n2 * n2 + 255) / 256)), dim3(256), 0, st, w.ru2,
                       n2, inv_sqrt_n2, static_cast<__half *>(R2));
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}
