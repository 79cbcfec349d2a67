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
//   rmap_kernel           the four maps to e_1 as dense matrices, entry by entry in closed form
//   urt_product_kernel    R^U = R_map R'_map^T for both sides (side 1 is R1)
//   hadamard_left_kernel  R2 = H R^U_2
//
// Wherever floating point decides an index -- the ART channels and the rank order of the URT --
// the deciding values (the calibration vector as the ART steps rewrite it, the means, the Hadamard
// image) are kept and compared in fp64: the paper defines these choices over the reals, and at
// fp64 only values that agree to about fifteen digits could be ordered differently from that.
// The matrices that follow the decisions are fp32.
#include "sq_common.h"

#include <math.h>

namespace sq {

namespace {

constexpr int kBuildThreads = 1024;
constexpr int kBuildWaves = kBuildThreads / kWave;
constexpr int kMaxSide = 256;                 // n1 <= 128, n2 <= 256
static_assert(kBuildThreads == 4 * kMaxSide, "one thread per step of each of the four chains");
static_assert(SQ_MAX_N1 <= kMaxSide && SQ_MAX_N2 <= kMaxSide && SQ_MAX_GIVENS <= kBuildThreads, "limits");
// reduction slots (two sets of three words per wave), five small fp64 vectors, the ART pairs
constexpr int kBuildSmallBytes = 6 * kBuildWaves * 4 + 5 * kMaxSide * 8 + 2 * SQ_MAX_GIVENS * 8;
static_assert(kBuildSmallBytes % 8 == 0, "the fp64 vectors behind the slots are 8-byte aligned");

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

// Largest (or smallest) 32-bit unsigned value of the wave, in every lane.  DPP steps as in
// wave_max; lanes a step does not write keep the identity of the operation.
template <bool LARGEST>
__device__ __forceinline__ uint32_t wave_extreme(uint32_t v)
{
    constexpr int kIdentity = LARGEST ? 0 : -1;
#define SQ_DPP_STEP(ctrl, row_mask)                                                                  \
    do {                                                                                             \
        const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(kIdentity, (int)v, ctrl, row_mask, 0xF, false); \
        v = LARGEST ? (o > v ? o : v) : (o < v ? o : v);                                             \
    } while (0)
    SQ_DPP_STEP(0xB1, 0xF);     // quad_perm [1,0,3,2]
    SQ_DPP_STEP(0x4E, 0xF);     // quad_perm [2,3,0,1]
    SQ_DPP_STEP(0x141, 0xF);    // row_half_mirror
    SQ_DPP_STEP(0x140, 0xF);    // row_mirror: every lane holds the result of its row of 16
    SQ_DPP_STEP(0x142, 0xA);    // row_bcast:15 into rows 1 and 3
    SQ_DPP_STEP(0x143, 0xC);    // row_bcast:31 into rows 2 and 3: lane 63 holds the wave's result
#undef SQ_DPP_STEP
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// Index of the largest (or smallest) 64-bit key (hi, lo) in the workgroup, the lowest index among
// equal keys; every thread passes the best (key, index) of its own elements and gets the result.
// Magnitudes of finite fp64 (and fp32) values order like their bit patterns read as unsigned
// integers.  `slots` ([3][kBuildWaves] words) must not be rewritten before every thread has passed
// a later barrier.
template <bool LARGEST>
__device__ __forceinline__ uint32_t wave_arg(uint32_t hi, uint32_t lo, uint32_t idx, uint32_t &best_hi,
                                             uint32_t &best_lo)
{
    constexpr uint32_t kNone = LARGEST ? 0u : 0xFFFFFFFFu;
    best_hi = wave_extreme<LARGEST>(hi);
    best_lo = wave_extreme<LARGEST>(hi == best_hi ? lo : kNone);
    return wave_extreme<false>((hi == best_hi && lo == best_lo) ? idx : 0xFFFFFFFFu);
}

template <bool LARGEST>
__device__ __forceinline__ uint32_t block_arg(uint32_t hi, uint32_t lo, uint32_t idx, uint32_t *slots)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    constexpr uint32_t kNone = LARGEST ? 0u : 0xFFFFFFFFu;
    uint32_t bh, bl;
    const uint32_t who = wave_arg<LARGEST>(hi, lo, idx, bh, bl);
    if (lane == 0) {
        slots[wave] = bh;
        slots[kBuildWaves + wave] = bl;
        slots[2 * kBuildWaves + wave] = who;
    }
    __syncthreads();
    // every wave combines the per-wave results on its own; a wave whose threads had no element
    // passes index 0xFFFFFFFF and never wins against one that had
    const bool in = lane < kBuildWaves;
    const uint32_t i2 = in ? slots[2 * kBuildWaves + lane] : 0xFFFFFFFFu;
    const bool has = i2 != 0xFFFFFFFFu;
    return wave_arg<LARGEST>(has ? slots[lane] : kNone, has ? slots[kBuildWaves + lane] : kNone, i2, bh, bl);
}

__device__ __forceinline__ void magnitude_key(double v, uint32_t &hi, uint32_t &lo)
{
    const uint64_t bits = (uint64_t)__double_as_longlong(fabs(v));
    hi = (uint32_t)(bits >> 32);
    lo = (uint32_t)bits;
}

// Step k of the Givens chain that takes `vec` (n entries) to ||vec|| e_1: entry k is zeroed by a
// rotation in the plane (k - 1, k), k = n - 1 down to 1.  When step k acts, entry k holds the norm
// of the original entries k .. n-1, so with S_k the sum of their squares
//   cos_k = v_{k-1} / sqrt(S_{k-1}),   sin_k = sqrt(S_k / S_{k-1})     (cos = 1, sin = 0 if S_{k-1} = 0;
//   sin_{n-1} = v_{n-1} / sqrt(S_{n-2}), because the last entry enters with its sign)
// and the steps can be computed independently of one another.  Stored at cs[k], cs[kMaxSide + k].
__device__ __forceinline__ void chain_step(const double *vec, int n, int k, float *cs)
{
    double tail = 0.0;
    for (int m = n - 1; m >= k; --m) tail += vec[m] * vec[m];
    const double x = vec[k - 1], all = tail + x * x;
    cs[k] = (all == 0.0) ? 1.f : (float)(x / sqrt(all));
    // the first step (k = n-1) meets the last entry itself, sign included; later ones meet a norm
    cs[kMaxSide + k] = (all == 0.0) ? 0.f : (float)(k == n - 1 ? vec[k] / sqrt(all) : sqrt(tail / all));
}

// One workgroup.  All of its LDS is dynamic (kBuildSmallBytes + 8K bytes): the reduction slots,
// the small vectors, then the calibration vector, in fp64.
__global__ __launch_bounds__(kBuildThreads) void art_urt_kernel(
    const __half *__restrict__ X, int64_t ldx, int T, int K, int n1, int n2, int P, double inv_sqrt_n2,
    const float *__restrict__ rowmax, int32_t *__restrict__ giv_i, int32_t *__restrict__ giv_j,
    float *__restrict__ giv_theta, float *__restrict__ chain)
{
    extern __shared__ uint32_t build_lds[];
    uint32_t *slots_a = build_lds, *slots_b = build_lds + 3 * kBuildWaves;
    double(*vec)[kMaxSide] = reinterpret_cast<double(*)[kMaxSide]>(build_lds + 6 * kBuildWaves);   // V1 | V2 H
    double *v2 = vec[2];
    double(*target)[kMaxSide] = reinterpret_cast<double(*)[kMaxSide]>(vec[3]);                     // U1 | U2
    double *pair_a = vec[5], *pair_b = pair_a + SQ_MAX_GIVENS;     // (c_i, c_j) each ART angle is made for
    double *cvec = pair_b + SQ_MAX_GIVENS;
    const int tid = threadIdx.x;

    // calibration row: the largest row maximum, lowest row among equals
    uint32_t top = 0, top_at = 0xFFFFFFFFu;
    for (int t = tid; t < T; t += kBuildThreads) {
        const uint32_t m = __float_as_uint(rowmax[t]);
        if (m > top || top_at == 0xFFFFFFFFu) top = m, top_at = (uint32_t)t;      // t ascends: ties keep the lower row
    }
    const int t_star = (int)block_arg<true>(top, 0u, top_at, slots_a);
    for (int k = tid; k < K; k += kBuildThreads) cvec[k] = (double)__half2float(X[(int64_t)t_star * ldx + k]);
    __syncthreads();

    // ART (Sec. 4.2; several steps as in the "ART steps" study): largest against smallest
    // magnitude, angle of Lemma 1, after which both channels hold r / sqrt(2)
    for (int p = 0; p < P; ++p) {
        // k ascends within a thread, so strict comparisons keep the lower channel among equals
        uint32_t hi_h = 0, hi_l = 0, hi_at = 0xFFFFFFFFu;
        for (int k = tid; k < K; k += kBuildThreads) {
            uint32_t h, l;
            magnitude_key(cvec[k], h, l);
            if (hi_at == 0xFFFFFFFFu || h > hi_h || (h == hi_h && l > hi_l)) hi_h = h, hi_l = l, hi_at = (uint32_t)k;
        }
        const int i = (int)block_arg<true>(hi_h, hi_l, hi_at, slots_a);
        uint32_t lo_h = 0xFFFFFFFFu, lo_l = 0xFFFFFFFFu, lo_at = 0xFFFFFFFFu;
        for (int k = tid; k < K; k += kBuildThreads) {
            uint32_t h, l;
            magnitude_key(cvec[k], h, l);
            if (k != i && (lo_at == 0xFFFFFFFFu || h < lo_h || (h == lo_h && l < lo_l)))
                lo_h = h, lo_l = l, lo_at = (uint32_t)k;
        }
        const int j = (int)block_arg<false>(lo_h, lo_l, lo_at, slots_b);
        if (tid == 0) {
            const double a = cvec[i], b = cvec[j];
            const double e = sqrt(a * a + b * b) * 0.70710678118654752440;
            giv_i[p] = i;
            giv_j[p] = j;
            pair_a[p] = a;
            pair_b[p] = b;
            cvec[i] = e;
            cvec[j] = e;
        }
        __syncthreads();
    }

    // vectors of the two URTs: means of the n1 x n2 view over the other dimension; the second one
    // goes through the Hadamard matrix first, because H acts first in R2
    if (tid < n1) {
        double s = 0.0;
        for (int q = 0; q < n2; ++q) s += cvec[tid * n2 + q];
        vec[0][tid] = s / (double)n2;
    }
    if (tid >= 512 && tid - 512 < n2) {
        const int q = tid - 512;
        double s = 0.0;
        for (int pp = 0; pp < n1; ++pp) s += cvec[pp * n2 + q];
        v2[q] = s / (double)n1;
    }
    __syncthreads();
    if (tid < n2) {
        double s = 0.0;
        for (int a = 0; a < n2; ++a) s += (__popc(a & tid) & 1) ? -v2[a] : v2[a];
        vec[1][tid] = s * inv_sqrt_n2;
    }
    __syncthreads();

    // uniform targets (Sec. 4.2 URT): template q_k = (2k - n - 1)/n by rank (ties: lower index
    // first), scaled to the norm of the vector; ||q||^2 = (n^2 - 1)/(3n)
    {
        const int side = tid >= 512, k = tid - 512 * side, n = side ? n2 : n1;
        if (k < n) {
            const double *v = vec[side];
            const double mine = v[k];
            int rank = 0;
            double norm2 = 0.0;
            for (int m = 0; m < n; ++m) {
                const double o = v[m];
                rank += (o < mine) || (o == mine && m < k);
                norm2 += o * o;
            }
            const double qnorm2 = ((double)n * n - 1.0) / (3.0 * n);
            target[side][k] = sqrt(norm2 / qnorm2) * (2.0 * (rank + 1) - n - 1.0) / n;
        }
    }
    __syncthreads();

    // the four chains: thread (which, k) computes step k of chain `which`
    {
        const int which = tid / kMaxSide, k = tid % kMaxSide, side = which >> 1, is_target = which & 1;
        const int n = side ? n2 : n1;
        if (k >= 1 && k < n) chain_step(is_target ? target[side] : vec[side], n, k, chain + which * 2 * kMaxSide);
    }

    // the angles of Lemma 1, one thread per ART step
    if (tid < P) giv_theta[tid] = (float)(atan2(pair_b[tid], pair_a[tid]) - 0.78539816339744830962);
}

// Entry (r, k) of the product of a chain (step n-1 first).  Row r starts as e_r; step r+1 leaves
// (cos, -sin) in columns r and r+1, and every later step k <= r multiplies what is carried in
// column k by sin_k on its way to column k-1 and leaves carry * cos_k behind.  Nothing ever
// reaches a column right of r+1.  blockIdx.y = which of the four matrices.
__global__ __launch_bounds__(256) void rmap_kernel(const float *__restrict__ chain, int n1, int n2,
                                                   float *m0, float *m1, float *m2, float *m3)
{
    const int which = blockIdx.y, n = (which >> 1) ? n2 : n1;
    float *M = which == 0 ? m0 : which == 1 ? m1 : which == 2 ? m2 : m3;
    const float *co = chain + which * 2 * kMaxSide, *si = co + kMaxSide;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= n * n) return;
    const int r = idx / n, k = idx % n;
    float v = 0.f;
    if (k == r + 1) {
        v = -si[k];
    } else if (k <= r) {
        v = (r + 1 < n) ? co[r + 1] : 1.f;
        for (int m = r; m > k; --m) v *= si[m];
        if (k >= 1) v *= co[k];
    }
    M[idx] = v;
}

// R^U = R_map R'_map^T (Sec. 4.2 URT), 16 x 16 output tile per workgroup, operands staged through
// LDS.  blockIdx.z = side; side 1 leaves as fp16 R1, side 2 stays fp32 for the Hadamard factor.
__global__ __launch_bounds__(256) void urt_product_kernel(const float *__restrict__ a1, const float *__restrict__ b1,
                                                          const float *__restrict__ a2, const float *__restrict__ b2,
                                                          int n1, int n2, __half *__restrict__ R1,
                                                          float *__restrict__ ru2)
{
    __shared__ float ta[16][17], tb[16][17];
    const int side = blockIdx.z, n = side ? n2 : n1;
    const float *A = side ? a2 : a1, *B = side ? b2 : b1;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int r0 = blockIdx.y * 16, c0 = blockIdx.x * 16;
    if (r0 >= n || c0 >= n) return;                      // whole workgroup: the grid is sized for the larger side
    float s = 0.f;
    for (int k0 = 0; k0 < n; k0 += 16) {
        ta[ty][tx] = (r0 + ty < n && k0 + tx < n) ? A[(r0 + ty) * n + k0 + tx] : 0.f;
        tb[ty][tx] = (c0 + ty < n && k0 + tx < n) ? B[(c0 + ty) * n + k0 + tx] : 0.f;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) s += ta[ty][k] * tb[tx][k];
        __syncthreads();
    }
    const int r = r0 + ty, c = c0 + tx;
    if (r < n && c < n) {
        if (side) ru2[r * n + c] = s;
        else R1[r * n + c] = __float2half_rn(s);
    }
}

// R2 = H R^U_2 with the normalised Sylvester Hadamard matrix, H[a][m] = (-1)^popcount(a & m) / sqrt n;
// same tiling (n2 is a power of two >= 8; partial tiles are masked)
__global__ __launch_bounds__(256) void hadamard_left_kernel(const float *__restrict__ ru2, int n2, float inv_sqrt_n2,
                                                            __half *__restrict__ R2)
{
    __shared__ float tm[16][17];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int a = blockIdx.y * 16 + ty, b0 = blockIdx.x * 16;
    float s = 0.f;
    for (int m0 = 0; m0 < n2; m0 += 16) {
        tm[ty][tx] = (m0 + ty < n2 && b0 + tx < n2) ? ru2[(m0 + ty) * n2 + b0 + tx] : 0.f;
        __syncthreads();
#pragma unroll
        for (int m = 0; m < 16; ++m) s += (__popc(a & (m0 + m)) & 1) ? -tm[m][tx] : tm[m][tx];
        __syncthreads();
    }
    if (a < n2 && b0 + tx < n2) R2[a * n2 + b0 + tx] = __float2half_rn(s * inv_sqrt_n2);
}

bool build_shape_ok(int64_t T, int32_t K, int32_t n1, int32_t n2, int32_t P)
{
    if (T < 1 || T > SQ_MAX_ROWS || K <= 0 || P < 0 || P > SQ_MAX_GIVENS) return false;
    if (n1 < 2 || n1 > SQ_MAX_N1 || n2 < 8 || n2 > SQ_MAX_N2 || (n2 & (n2 - 1)) != 0) return false;
    return (int64_t)n1 * n2 == K && K <= SQ_MAX_K;
}

}  // namespace

}  // namespace sq

extern "C" sq_status sq_kron_factor(int32_t n, int32_t *n1, int32_t *n2)
{
    if (!n1 || !n2) return SQ_ERR_NULL;
    if (n < 1) return SQ_ERR_SHAPE;
    // Alg. 1 asks for the power of two dividing n nearest to sqrt(n).  Distances to sqrt(n) shrink
    // while a^2 <= n and grow afterwards, so only two candidates matter: the largest divisor `below`
    // with below^2 <= n, and its double if that divides n as well.  2 below - sqrt(n) < sqrt(n) - below
    // is 3 below < 2 sqrt(n), i.e. 9 below^2 < 4 n, in integers; equality keeps the smaller one.
    const int64_t m = n;
    int64_t below = 1;
    while (m % (2 * below) == 0 && 4 * below * below <= m) below *= 2;
    const bool above_divides = m % (2 * below) == 0;
    const int64_t best = (above_divides && 9 * below * below < 4 * m) ? 2 * below : below;
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
    const double inv_sqrt_n2 = 1.0 / sqrt((double)n2);
    const __half *Xh = static_cast<const __half *>(X);

    const int64_t row_groups = (T + 3) / 4;
    hipLaunchKernelGGL(sq::row_absmax_kernel, dim3((unsigned)(row_groups < 4096 ? row_groups : 4096)), dim3(256), 0,
                       st, Xh, ldx, (int)T, K, w.rowmax);
    auto art = sq::art_urt_kernel;
    const size_t lds = sq::kBuildSmallBytes + (size_t)K * sizeof(double);     // 139.4 KiB at the largest K
    if (!sq::allow_large_lds(reinterpret_cast<const void *>(art))) return SQ_ERR_LAUNCH;
    hipLaunchKernelGGL(art, dim3(1), dim3(sq::kBuildThreads), lds, st, Xh, ldx, (int)T, K, n1, n2, P, inv_sqrt_n2,
                       w.rowmax, giv_i, giv_j, giv_theta, w.chain);
    const int big = n1 > n2 ? n1 : n2;
    hipLaunchKernelGGL(sq::rmap_kernel, dim3((unsigned)((big * big + 255) / 256), 4), dim3(256), 0, st, w.chain, n1,
                       n2, w.rmap[0], w.rmap[1], w.rmap[2], w.rmap[3]);
    const unsigned tiles = (unsigned)((big + 15) / 16), tiles2 = (unsigned)((n2 + 15) / 16);
    hipLaunchKernelGGL(sq::urt_product_kernel, dim3(tiles, tiles, 2), dim3(256), 0, st, w.rmap[0], w.rmap[1],
                       w.rmap[2], w.rmap[3], n1, n2, static_cast<__half *>(R1), w.ru2);
    hipLaunchKernelGGL(sq::hadamard_left_kernel, dim3(tiles2, tiles2), dim3(256), 0, st, w.ru2, n2, (float)inv_sqrt_n2,
                       static_cast<__half *>(R2));
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}
