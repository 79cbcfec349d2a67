// Matrix-core kernel of sq_rotate_quantize (Sec. 4.1-4.2, Eq. 18; quantizer of Sec. 3.2).
//
// Per token, with X_mat the n1 x n2 row-major view of the (Givens-rotated) row:
//   stage A   Z = X_mat R2                 fp16 x fp16 MFMA, fp32 accumulate: products are exact
//   stage B   Y^T = Z^T R1                 Z split as hi + lo (two fp16 halves, ~21 bits), two MFMA
//                                          passes; computes rvec(R1^T X_mat R2) transposed
//   quantize  s = max|Y| / 7, codes = floor(Y / s + 1/2), two nibbles per byte
//
// One wave owns 32 columns q' of one token through both stages: the 32x32 accumulator layout of
// stage A (lane = column, registers = rows p) is, register for register, the operand layout stage
// B needs for its contraction over p, so Z never leaves the registers.  R2 and R1 are held in
// registers as MFMA operands for the life of the workgroup, which walks over many tokens (for
// three 32-row blocks the fragments of R1, which every wave needs alike, are kept once in LDS
// instead, so that the registers allow a second workgroup on the CU).
//
// Token rows stream from HBM straight into a ring of LDS tiles (global_load_lds): three tiles, two
// rows ahead of the one being multiplied, with two workgroups per CU; or two tiles where that
// makes room for one more workgroup per CU.
// The loop is rotated so that the MFMAs of stage A of the NEXT token are issued between the VALU
// instructions that quantize the current one, and the hi/lo split of the next stage-B step
// between the MFMAs of the current step.
//
// Givens list (ART): the touched channels (at most 2P) are rotated in fp32 on a small LDS array,
// level by level (pairs of one level share no channel, so lanes work in parallel while the list
// order is kept).  A rotated value v goes back as hi = fp16(v) into the token tile and
// lo = fp16(v - hi) into a small side tile; stage A contracts the side tile against the matching
// rows of R2 in a few extra MFMA steps, so the fp16 rounding of hi is repaired to ~21 bits.
// The first wave of a token does this for the next token.
#include "sq_rotq_body.h"

namespace sq {

// values of the launch chain's `prepared` argument beyond 0 (R1, R2 as they are) and 1 (prepared
// fragments): the fp16-output kernel, and the quantizer with a clipping ratio (R1, R2 as they are)
constexpr int kRotqFp16Out = 2;
constexpr int kRotqClip = 3;

// QS_MAX: repair steps of 16 q-slots each the kernel holds rotation rows for (4 or 8).
// PREPARED: R1 and R2 point at the operand fragments written by rotation_fragments_kernel.
template <int N1, int N2, int OCC, int QS_MAX, int NSX_, bool R1LDS, bool PREPARED, bool CLIP = false>
__global__ __launch_bounds__(256, OCC) void rotate_quantize_mfma_kernel(
    const __half *__restrict__ X, int64_t ldx, int T, RotqPlan plan,
    const __half *__restrict__ R1, const __half *__restrict__ R2, uint8_t *__restrict__ Q,
    float *__restrict__ scales, float *__restrict__ xrot, int sides)
{
    extern __shared__ uint4 smem_u4[];
    rotate_quantize_mfma_body<N1, N2, QS_MAX, NSX_, R1LDS, PREPARED, false, CLIP>(X, ldx, T, plan, R1, R2, Q, scales, xrot,
                                                                                 (int)blockIdx.x, (int)gridDim.x,
                                                                                 smem_u4, sides);
}

// The same rotation without the quantizer: the rotated rows leave as fp16 (the 16-bit activations
// of the weight-only setting).  Built for R1, R2 as they are only.
template <int N1, int N2, int OCC, int QS_MAX, int NSX_, bool R1LDS>
__global__ __launch_bounds__(256, OCC) void rotate_fp16_mfma_kernel(
    const __half *__restrict__ X, int64_t ldx, int T, RotqPlan plan, const __half *__restrict__ R1,
    const __half *__restrict__ R2, __half *__restrict__ xout, int64_t ldo, int sides)
{
    extern __shared__ uint4 smem_u4[];
    rotate_quantize_mfma_body<N1, N2, QS_MAX, NSX_, R1LDS, false, true>(X, ldx, T, plan, R1, R2, nullptr, nullptr,
                                                                        nullptr, (int)blockIdx.x, (int)gridDim.x,
                                                                        smem_u4, sides, xout, ldo);
}

// OCC: workgroups per CU the registers allow (512 per lane and SIMD, one wave of each workgroup
// per SIMD); the LDS the list needs may allow fewer.
template <int N1, int N2, int QS_MAX, int NSX, int OCC, bool R1LDS = false>
static sq_status launch_rotq_mfma_ring(const __half *X, int64_t ldx, int T, const RotqPlan &plan,
                                       const __half *R1, const __half *R2, uint8_t *Q, float *scales,
                                       float *xrot, hipStream_t st, int prepared, __half *xout, int64_t ldo)
{
    using S = RotqShape<N1, N2, NSX, R1LDS>;
    const int qsteps = (plan.n_qslots + 15) / 16;
    const int sides = S::side_tiles(qsteps, OCC);
    const int lds = S::lds_bytes(qsteps, sides);
    if (lds > kMaxDynamicLds) return SQ_ERR_SHAPE;
    const int groups = (T + S::TPP - 1) / S::TPP;
    const int by_lds = (160 * 1024) / lds;
    const int per_cu = by_lds < OCC ? by_lds : OCC;                       // workgroups a CU holds
    const int resident = 256 * per_cu;
    const int grid = groups < resident ? groups : resident;
    if (prepared == kRotqFp16Out) {
        auto kernel = rotate_fp16_mfma_kernel<N1, N2, OCC, QS_MAX, NSX, R1LDS>;
        if (!allow_large_lds(reinterpret_cast<const void *>(kernel))) return SQ_ERR_LAUNCH;
        hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), lds, st, X, ldx, T, plan, R1, R2, xout, ldo, sides);
        return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
    }
    auto kernel = prepared == kRotqClip ? rotate_quantize_mfma_kernel<N1, N2, OCC, QS_MAX, NSX, R1LDS, false, true>
                  : prepared            ? rotate_quantize_mfma_kernel<N1, N2, OCC, QS_MAX, NSX, R1LDS, true>
                                        : rotate_quantize_mfma_kernel<N1, N2, OCC, QS_MAX, NSX, R1LDS, false>;
    if (!allow_large_lds(reinterpret_cast<const void *>(kernel))) return SQ_ERR_LAUNCH;
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), lds, st, X, ldx, T, plan, R1, R2, Q, scales, xrot, sides);
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

template <int N1, int N2, int QS_MAX>
static sq_status launch_rotq_mfma_qs(const __half *X, int64_t ldx, int T, const RotqPlan &plan,
                                     const __half *R1, const __half *R2, uint8_t *Q, float *scales,
                                     float *xrot, hipStream_t st, int prepared, __half *xout, int64_t ldo)
{
    constexpr int MB = (N1 + 31) / 32;
    if constexpr (N1 == 64 && N2 == 64) {
        // 168 registers: three workgroups fit a CU if the ring has two tiles.  Measured faster than
        // the ring of three at two workgroups per CU from 4096 tokens on (4 % there, 12 % at 32768),
        // 3 % slower below.  The debug option SQ_DEBUG_ROTQ_RING (2 or 3) forces one of them.
        const int forced = debug_option(SQ_DEBUG_ROTQ_RING);
        // With prepared operands the prologue is shorter and the third workgroup pays earlier: in a
        // stream of such launches T = 2048 10.0 -> 9.6 us, 3072 14.3 -> 12.6, 4096 16.7 -> 14.1.  At
        // 2048 the layer (this launch behind a GEMM) was 0.35 us slower with it, so it starts at 3072.
        const bool ring2 = forced == 2 || (forced != 3 && T >= (prepared == 1 ? 3072 : 4096));
        if (ring2) return launch_rotq_mfma_ring<N1, N2, QS_MAX, 2, 3>(X, ldx, T, plan, R1, R2, Q, scales, xrot, st, prepared, xout, ldo);
    }
    if constexpr (MB == 3 && QS_MAX == 4) {       // more than 64 q-slots never leave room for two workgroups
        // With R1 in registers three row blocks need more than 256 of them: one workgroup per CU.
        // With the shared copy in LDS and a ring of two tiles, two fit if the list's side tiles are
        // small enough.  The debug option SQ_DEBUG_ROTQ_R1_IN_REGISTERS forces the register variant.
        using S2 = RotqShape<N1, N2, 2, true>;
        const bool force_reg = debug_option(SQ_DEBUG_ROTQ_R1_IN_REGISTERS) != 0;
        if (!force_reg && 2 * S2::lds_bytes((plan.n_qslots + 15) / 16, 1) <= 160 * 1024)
            return launch_rotq_mfma_ring<N1, N2, QS_MAX, 2, 2, true>(X, ldx, T, plan, R1, R2, Q, scales, xrot, st, prepared, xout, ldo);
    }
    return launch_rotq_mfma_ring<N1, N2, QS_MAX, 3, (MB <= 2) ? 2 : 1>(X, ldx, T, plan, R1, R2, Q, scales, xrot, st, prepared, xout, ldo);
}

// A list touches at most min(2P, n2) distinct columns q: more than 64 only if n2 is 128.
template <int N1, int N2>
static sq_status launch_rotq_mfma(const __half *X, int64_t ldx, int T, const RotqPlan &plan,
                                  const __half *R1, const __half *R2, uint8_t *Q, float *scales,
                                  float *xrot, hipStream_t st, int prepared, __half *xout, int64_t ldo)
{
    if constexpr (N2 > 64) {
        if (plan.n_qslots > 64)
            return launch_rotq_mfma_qs<N1, N2, 8>(X, ldx, T, plan, R1, R2, Q, scales, xrot, st, prepared, xout, ldo);
    }
    return launch_rotq_mfma_qs<N1, N2, 4>(X, ldx, T, plan, R1, R2, Q, scales, xrot, st, prepared, xout, ldo);
}

// The operand fragments of R2 (stage A) and R1 (stage B) exactly as the kernel above holds them,
// written lane by lane so that a wave fetches each with one contiguous 1 KB load:
//   f2[(cb KSA + ks) 64 + lane][e] = R2[16 ks + 8 g + e][32 cb + l32]
//   f1[(nb KSB + ks) 64 + lane][e] = R1[16 ks + 8 (e / 4) + 4 g + e % 4][32 nb + l32]   (0 outside R1)
// with l32 = lane % 32, g = lane / 32, KSA = n2 / 16, KSB = 2 ceil(n1 / 32).
__global__ __launch_bounds__(256) void rotation_fragments_kernel(const __half *__restrict__ R1, int n1,
                                                                  const __half *__restrict__ R2, int n2,
                                                                  v8h *__restrict__ f1, v8h *__restrict__ f2)
{
    const int ksa = n2 / 16, ncb = n2 / 32, mb = (n1 + 31) / 32, ksb = 2 * mb;
    const int first = blockIdx.x * blockDim.x + threadIdx.x, step = gridDim.x * blockDim.x;
    for (int u = first; u < ncb * ksa * kWave; u += step) {
        const int lane = u % kWave, ks = (u / kWave) % ksa, cb = u / (kWave * ksa);
        const int l32 = lane & 31, g = lane >> 5;
        v8h v;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (_Float16)__half2float(R2[(16 * ks + 8 * g + e) * n2 + 32 * cb + l32]);
        f2[u] = v;
    }
    for (int u = first; u < mb * ksb * kWave; u += step) {
        const int lane = u % kWave, ks = (u / kWave) % ksb, nb = u / (kWave * ksb);
        const int l32 = lane & 31, g = lane >> 5, col = 32 * nb + l32;
        v8h v;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int row = 16 * ks + 8 * (e / 4) + 4 * g + e % 4;
            v[e] = (row < n1 && col < n1) ? (_Float16)__half2float(R1[row * n1 + col]) : (_Float16)0.f;
        }
        f1[u] = v;
    }
}

bool rotq_mfma_covers(int n1, int n2)
{
    static const int shapes[][2] = {{16, 32}, {32, 32}, {32, 64}, {64, 64}, {80, 64}, {64, 128},
                                    {128, 64}, {86, 128}, {108, 128}, {112, 128}, {128, 128}};
    for (const auto &sh : shapes)
        if (sh[0] == n1 && sh[1] == n2) return true;
    return false;
}

size_t rotq_fragment_bytes_r1(int n1) { const int mb = (n1 + 31) / 32; return (size_t)mb * 2 * mb * kWave * 16; }
size_t rotq_fragment_bytes_r2(int n2) { return (size_t)(n2 / 32) * (n2 / 16) * kWave * 16; }

sq_status rotq_write_fragments(const __half *R1, int n1, const __half *R2, int n2, void *f1, void *f2,
                               hipStream_t st)
{
    const size_t b1 = rotq_fragment_bytes_r1(n1), b2 = rotq_fragment_bytes_r2(n2);
    const int units = (int)((b1 > b2 ? b1 : b2) / 16);
    hipLaunchKernelGGL(rotation_fragments_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, st, R1, n1,
                       R2, n2, static_cast<v8h *>(f1), static_cast<v8h *>(f2));
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

// Picks the instantiation for (n1, n2); returns false if this kernel does not cover the shape.
// prepared: R1 and R2 point at the fragments written by rotq_write_fragments.
static bool rotq_mfma_dispatch_mode(const __half *X, int64_t ldx, int T, int n1, int n2, const RotqPlan &plan,
                                    const __half *R1, const __half *R2, uint8_t *Q, float *scales, float *xrot,
                                    hipStream_t st, sq_status *status, int prepared, __half *xout, int64_t ldo)
{
#define SQ_ROTQ_CASE(N1, N2)                                                                         \
    if (n1 == N1 && n2 == N2) {                                                                      \
        *status = launch_rotq_mfma<N1, N2>(X, ldx, T, plan, R1, R2, Q, scales, xrot, st, prepared, xout, ldo);            \
        return true;                                                                                 \
    }
    SQ_ROTQ_CASE(16, 32)     // K = 512
    SQ_ROTQ_CASE(32, 32)     // 1024
    SQ_ROTQ_CASE(32, 64)     // 2048
    SQ_ROTQ_CASE(64, 64)     // 4096
    SQ_ROTQ_CASE(80, 64)     // 5120
    SQ_ROTQ_CASE(64, 128)    // 8192
    SQ_ROTQ_CASE(128, 64)    // 8192, the split Alg. 1 picks
    SQ_ROTQ_CASE(86, 128)    // 11008
    SQ_ROTQ_CASE(108, 128)   // 13824
    SQ_ROTQ_CASE(112, 128)   // 14336
    SQ_ROTQ_CASE(128, 128)   // 16384
#undef SQ_ROTQ_CASE
    return false;
}

bool rotq_mfma_dispatch(const __half *X, int64_t ldx, int T, int n1, int n2, const RotqPlan &plan,
                        const __half *R1, const __half *R2, uint8_t *Q, float *scales, float *xrot,
                        hipStream_t st, sq_status *status, bool prepared)
{
    // a clipping ratio below one comes with R1, R2 as they are only (sq_rotate_quantize_variant)
    const int mode = plan.clip < 1.0f ? kRotqClip : prepared ? 1 : 0;
    if (plan.clip < 1.0f && prepared) {
        *status = SQ_ERR_SHAPE;
        return true;
    }
    return rotq_mfma_dispatch_mode(X, ldx, T, n1, n2, plan, R1, R2, Q, scales, xrot, st, status, mode, nullptr, 0);
}

bool rotq_mfma_dispatch_f16(const __half *X, int64_t ldx, int T, int n1, int n2, const RotqPlan &plan,
                            const __half *R1, const __half *R2, __half *xout, int64_t ldo, hipStream_t st,
                            sq_status *status)
{
    return rotq_mfma_dispatch_mode(X, ldx, T, n1, n2, plan, R1, R2, nullptr, nullptr, nullptr, st, status,
                                   kRotqFp16Out, xout, ldo);
}

}  // namespace sq
