// sq_rotate_quantize: online rotation (Givens list, then Kronecker product, Sec. 4.1-4.2, Eq. 18)
// fused with the per-token 4-bit rounding quantizer of Sec. 3.2.  gfx950 only.
#include "sq_common.h"
#include "sq_rotq_plan.h"

#include <math.h>
#include <string.h>

namespace sq {

// ------------------------------------------------------------------------------------------
// Generic kernel: any (n1, n2) with n2 % 8 == 0.  One workgroup per token, the token row and
// the intermediate V_mat R2 live in LDS as fp32, contractions are plain fp32 FMAs.
//   stage 0  x <- x G_1 ... G_P                 (one lane, in list order: pairs may overlap)
//   stage A  Z = X_mat R2                       (n1 x n2) (n2 x n2)
//   stage B  Y = R1^T Z                         (n1 x n1)^T (n1 x n2)
//   stage Q  s = max|Y| / 7, codes = floor(Y / s + 1/2), two nibbles per byte (in general
//            s = max|Y| / (q_top / clip) and codes clamped to [-q_top - 1, q_top])
// ------------------------------------------------------------------------------------------
constexpr int kGenThreads = 256;

__global__ __launch_bounds__(kGenThreads) void rotate_quantize_generic_kernel(
    const __half *__restrict__ X, int64_t ldx, int K, int n1, int n2, GivensList giv,
    const __half *__restrict__ R1, const __half *__restrict__ R2, uint8_t *__restrict__ Q,
    float *__restrict__ scales, float *__restrict__ xrot, __half *__restrict__ xout, int64_t ldo,
    float q_top, float q_div)
{
    extern __shared__ float smem[];
    float *xs = smem;          // [K]  token row, then reused for Y
    float *zs = smem + K;      // [K]  Z = X_mat R2
    __shared__ float red[kGenThreads / kWave];

    const int tid = threadIdx.x;
    const int64_t t = blockIdx.x;
    const __half *xrow = X + t * ldx;

    for (int c = tid; c < K / 8; c += kGenThreads) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(xrow + c * 8);
        const __half *h = reinterpret_cast<const __half *>(&raw);
#pragma unroll
        for (int u = 0; u < 8; ++u) xs[c * 8 + u] = __half2float(h[u]);
    }
    __syncthreads();

    if (tid == 0) {
        for (int p = 0; p < giv.count; ++p) {
            const float a = xs[giv.i[p]], b = xs[giv.j[p]];
            xs[giv.i[p]] = a * giv.c[p] + b * giv.s[p];
            xs[giv.j[p]] = b * giv.c[p] - a * giv.s[p];
        }
    }
    __syncthreads();

    // stage A: each thread makes 4 consecutive output columns of one row of Z
    const int n2q = n2 / 4;
    for (int o = tid; o < n1 * n2q; o += kGenThreads) {
        const int p = o / n2q, q0 = (o % n2q) * 4;
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        const float *xr = xs + p * n2;
        for (int q = 0; q < n2; ++q) {
            const float xv = xr[q];
            const uint2 raw = *reinterpret_cast<const uint2 *>(R2 + (int64_t)q * n2 + q0);
            const __half *h = reinterpret_cast<const __half *>(&raw);
            a0 = fmaf(xv, __half2float(h[0]), a0);
            a1 = fmaf(xv, __half2float(h[1]), a1);
            a2 = fmaf(xv, __half2float(h[2]), a2);
            a3 = fmaf(xv, __half2float(h[3]), a3);
        }
        float *zr = zs + p * n2 + q0;
        zr[0] = a0; zr[1] = a1; zr[2] = a2; zr[3] = a3;
    }
    __syncthreads();

    // stage B: Y[p', q'] = sum_p R1[p, p'] Z[p, q'];  written over xs
    float amax = 0.f;
    for (int o = tid; o < n1 * n2q; o += kGenThreads) {
        const int po = o / n2q, q0 = (o % n2q) * 4;
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        for (int p = 0; p < n1; ++p) {
            const float r = __half2float(R1[(int64_t)p * n1 + po]);
            const float *zr = zs + p * n2 + q0;
            a0 = fmaf(r, zr[0], a0);
            a1 = fmaf(r, zr[1], a1);
            a2 = fmaf(r, zr[2], a2);
            a3 = fmaf(r, zr[3], a3);
        }
        float *yr = xs + po * n2 + q0;
        yr[0] = a0; yr[1] = a1; yr[2] = a2; yr[3] = a3;
        amax = fmaxf(amax, fmaxf(fmaxf(fabsf(a0), fabsf(a1)), fmaxf(fabsf(a2), fabsf(a3))));
    }
    amax = wave_max(amax);
    if ((tid & (kWave - 1)) == 0) red[tid / kWave] = amax;
    __syncthreads();
    if (xout != nullptr) {       // weight-only setting: the rotated row leaves as fp16, no quantizer
        __half *orow = xout + t * ldo;
        for (int k = tid; k < K; k += kGenThreads) orow[k] = __float2half_rn(xs[k]);
        return;
    }
    amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));

    const float step = (amax == 0.f) ? 1.0f : amax / q_div;             // q_div = q_top / clip; 7: max|Y| / 7
    if (tid == 0) scales[t] = step;

    uint32_t *qrow = reinterpret_cast<uint32_t *>(Q + t * (int64_t)(K / 2));
    for (int c = tid; c < K / 8; c += kGenThreads) {
        uint32_t word = 0;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            float v = floorf(xs[c * 8 + u] / step + 0.5f);
            v = fminf(fmaxf(v, -q_top - 1.0f), q_top);
            word |= (static_cast<uint32_t>(static_cast<int>(v)) & 0xFu) << (4 * u);
        }
        qrow[c] = word;
    }
    if (xrot != nullptr) {
        float *orow = xrot + t * (int64_t)K;
        for (int k = tid; k < K; k += kGenThreads) orow[k] = xs[k];
    }
}

// Regroup the Givens list into levels of mutually disjoint pairs (see RotqPlan).  Returns false
// if the list touches more distinct values of channel % n2 than the matrix-core kernel repairs.
static bool build_rotq_plan(const GivensList &giv, int n2, RotqPlan &plan)
{
    memset(&plan, 0, sizeof(plan));
    int slot_level[kRotqMaxSlots];
    int pair_level[SQ_MAX_GIVENS], pair_si[SQ_MAX_GIVENS], pair_sj[SQ_MAX_GIVENS];
    auto slot_of = [&](int ch) {
        for (int s = 0; s < plan.n_slots; ++s)
            if (plan.chan[s] == ch) return s;
        const int s = plan.n_slots++;
        plan.chan[s] = (uint16_t)ch;
        slot_level[s] = 0;
        const int q = ch % n2;
        int qs = 0;
        while (qs < plan.n_qslots && plan.qlist[qs] != q) ++qs;
        if (qs == plan.n_qslots) {
            if (plan.n_qslots == kRotqMaxQSlots) return -1;
            plan.qlist[plan.n_qslots++] = (uint16_t)q;
        }
        plan.qslot[s] = (uint8_t)qs;
        return s;
    };
    int levels = 0;
    for (int p = 0; p < giv.count; ++p) {
        const int si = slot_of(giv.i[p]), sj = slot_of(giv.j[p]);
        if (si < 0 || sj < 0) return false;
        const int lv = 1 + (slot_level[si] > slot_level[sj] ? slot_level[si] : slot_level[sj]);
        slot_level[si] = slot_level[sj] = lv;
        pair_level[p] = lv - 1;
        pair_si[p] = si;
        pair_sj[p] = sj;
        if (lv > levels) levels = lv;
    }
    plan.n_levels = levels;
    plan.q_top = 7.0f;                        // four bits, no clipping, unless a call says otherwise
    plan.clip = 1.0f;
    plan.q_div = 7.0f;
    memset(plan.pair_level, 0xFF, sizeof(plan.pair_level));
    int pos = 0;
    for (int lv = 0; lv < levels; ++lv) {          // stable: list order is kept inside a level
        plan.level_begin[lv] = (uint8_t)pos;
        for (int p = 0; p < giv.count; ++p)
            if (pair_level[p] == lv) {
                plan.pair_i[pos] = (uint8_t)pair_si[p];
                plan.pair_j[pos] = (uint8_t)pair_sj[p];
                plan.pair_level[pos] = (uint8_t)lv;
                plan.c[pos] = giv.c[p];
                plan.s[pos] = giv.s[p];
                ++pos;
            }
    }
    plan.level_begin[levels] = (uint8_t)pos;
    return true;
}

}  // namespace sq

// The launch plan the matrix-core kernel would get for a Givens list, flattened into int32 arrays
// so that host-only tests can check the regrouping (declared in the debug section of
// singlequant.h).  Returns the number of levels, or -1 if the list cannot be planned.
extern "C" int32_t sq_debug_rotq_plan(const int32_t *giv_i, const int32_t *giv_j, int32_t P, int32_t n2,
                                         int32_t *n_slots, int32_t *n_qslots, int32_t *slot_chan,
                                         int32_t *slot_qslot, int32_t *qslot_q, int32_t *pair_slot_i,
                                         int32_t *pair_slot_j, int32_t *pair_level)
{
    if (P < 0 || P > SQ_MAX_GIVENS || n2 <= 0) return -1;
    sq::GivensList giv;
    giv.count = P;
    for (int p = 0; p < P; ++p) {
        giv.i[p] = giv_i[p];
        giv.j[p] = giv_j[p];
        giv.c[p] = (float)p;              // tags that let the test recover the list position of a sorted pair
        giv.s[p] = 0.f;
    }
    sq::RotqPlan plan;
    if (!sq::build_rotq_plan(giv, n2, plan)) return -1;
    *n_slots = plan.n_slots;
    *n_qslots = plan.n_qslots;
    for (int s = 0; s < plan.n_slots; ++s) {
        slot_chan[s] = plan.chan[s];
        slot_qslot[s] = plan.qslot[s];
    }
    for (int q = 0; q < plan.n_qslots; ++q) qslot_q[q] = plan.qlist[q];
    for (int k = 0; k < P; ++k) {         // sorted position k holds list position (int)c[k]
        const int p = (int)plan.c[k];
        pair_slot_i[p] = plan.pair_i[k];
        pair_slot_j[p] = plan.pair_j[k];
        pair_level[p] = plan.pair_level[k];
    }
    return plan.n_levels;
}

namespace sq {

// Layout of a prepared rotation: copies of R1 and R2 (each padded to 256 bytes), then, for the
// shapes the matrix-core kernel covers, its operand fragments of R1 and of R2.
struct PreparedLayout {
    size_t off_r1, off_r2, off_f1, off_f2, bytes;
    bool fragments;
};

static PreparedLayout prepared_layout(int n1, int n2)
{
    auto pad = [](size_t b) { return (b + 255) / 256 * 256; };
    PreparedLayout l;
    l.off_r1 = 0;
    l.off_r2 = pad((size_t)n1 * n1 * 2);
    l.off_f1 = l.off_r2 + pad((size_t)n2 * n2 * 2);
    l.fragments = rotq_mfma_covers(n1, n2);
    l.off_f2 = l.off_f1 + (l.fragments ? rotq_fragment_bytes_r1(n1) : 0);
    l.bytes = l.off_f2 + (l.fragments ? rotq_fragment_bytes_r2(n2) : 0);
    return l;
}

__global__ __launch_bounds__(256) void copy_halves_kernel(const __half *__restrict__ a, int na, __half *__restrict__ da,
                                                         const __half *__restrict__ b, int nb, __half *__restrict__ db)
{
    const int first = blockIdx.x * blockDim.x + threadIdx.x, step = gridDim.x * blockDim.x;
    for (int i = first; i < na; i += step) da[i] = a[i];
    for (int i = first; i < nb; i += step) db[i] = b[i];
}

static bool rotation_shape_ok(int64_t K, int32_t n1, int32_t n2)
{
    if (K <= 0 || n1 <= 0 || n2 <= 0) return false;
    if (n1 > SQ_MAX_N1 || n2 > SQ_MAX_N2) return false;
    return (int64_t)n1 * n2 == K && (n2 % 8) == 0 && K <= SQ_MAX_K;
}

}  // namespace sq

extern "C" int64_t sq_prepared_rotation_bytes(int32_t n1, int32_t n2)
{
    if (!sq::rotation_shape_ok((int64_t)n1 * n2, n1, n2)) return 0;
    return (int64_t)sq::prepared_layout(n1, n2).bytes;
}

extern "C" sq_status sq_prepare_rotation(const void *R1, int32_t n1, const void *R2, int32_t n2,
                                         void *prepared, void *stream)
{
    if (!sq::rotation_shape_ok((int64_t)n1 * n2, n1, n2)) return SQ_ERR_SHAPE;
    if (!R1 || !R2 || !prepared) return SQ_ERR_NULL;
    if (((uintptr_t)R1 & 15) || ((uintptr_t)R2 & 15) || ((uintptr_t)prepared & 15)) return SQ_ERR_ALIGN;
    const sq::PreparedLayout l = sq::prepared_layout(n1, n2);
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *base = static_cast<char *>(prepared);
    const __half *r1 = static_cast<const __half *>(R1), *r2 = static_cast<const __half *>(R2);
    const int most = n1 * n1 > n2 * n2 ? n1 * n1 : n2 * n2;
    hipLaunchKernelGGL(sq::copy_halves_kernel, dim3((unsigned)((most + 255) / 256)), dim3(256), 0, st, r1, n1 * n1,
                       reinterpret_cast<__half *>(base + l.off_r1), r2, n2 * n2,
                       reinterpret_cast<__half *>(base + l.off_r2));
    if (hipGetLastError() != hipSuccess) return SQ_ERR_LAUNCH;
    if (!l.fragments) return SQ_OK;
    return sq::rotq_write_fragments(r1, n1, r2, n2, base + l.off_f1, base + l.off_f2, st);
}

namespace sq {

// The list as the kernels take it (cos / sin, and the regrouping into levels) is kept from the
// last call of this thread and reused when the same list comes again, which is what a layer
// called once per forward pass sends.  The caller has checked P and the pointers.
struct ListCache {
    int32_t count = -1, channels = 0, cols = 0;
    int32_t i[SQ_MAX_GIVENS], j[SQ_MAX_GIVENS];
    float theta[SQ_MAX_GIVENS];
    GivensList giv;
    RotqPlan plan;
    bool plan_ok = false;
};

static sq_status cached_list(const int32_t *giv_i, const int32_t *giv_j, const float *giv_theta, int32_t P,
                             int32_t K, int32_t n2, const ListCache **out)
{
    static thread_local ListCache prep;
    const bool same = prep.count == P && prep.channels == K && prep.cols == n2 &&
                      (P == 0 || (memcmp(prep.i, giv_i, sizeof(int32_t) * P) == 0 &&
                                  memcmp(prep.j, giv_j, sizeof(int32_t) * P) == 0 &&
                                  memcmp(prep.theta, giv_theta, sizeof(float) * P) == 0));
    if (!same) {
        prep.count = -1;                     // stays invalid if a check below fails
        GivensList &g = prep.giv;
        g.count = P;
        for (int p = 0; p < P; ++p) {
            if (giv_i[p] < 0 || giv_i[p] >= K || giv_j[p] < 0 || giv_j[p] >= K || giv_i[p] == giv_j[p])
                return SQ_ERR_INDEX;
            g.i[p] = giv_i[p];
            g.j[p] = giv_j[p];
            g.c[p] = (float)cos((double)giv_theta[p]);
            g.s[p] = (float)sin((double)giv_theta[p]);
        }
        prep.plan_ok = build_rotq_plan(g, n2, prep.plan);
        if (P > 0) {
            memcpy(prep.i, giv_i, sizeof(int32_t) * P);
            memcpy(prep.j, giv_j, sizeof(int32_t) * P);
            memcpy(prep.theta, giv_theta, sizeof(float) * P);
        }
        prep.channels = K;
        prep.cols = n2;
        prep.count = P;
    }
    *out = &prep;
    return SQ_OK;
}

}  // namespace sq

// fragments: null, or the two fragment blocks of a prepared rotation (then R1 / R2 are its copies)
static sq_status rotate_quantize_any(const void *X, int64_t T, int32_t K, int64_t ldx,
                                     const int32_t *giv_i, const int32_t *giv_j,
                                     const float *giv_theta, int32_t P, const void *R1,
                                     int32_t n1, const void *R2, int32_t n2, uint8_t *Q,
                                     float *scales, float *xrot_dbg, void *stream, const void *frag1,
                                     const void *frag2, void *xout = nullptr, int64_t ldo = 0,
                                     int32_t bits = 4, float clip_ratio = 1.0f)
{
    if (bits < 2 || bits > 4 || !(clip_ratio > 0.0f) || clip_ratio > 1.0f) return SQ_ERR_SHAPE;
    const float q_top = (float)((1 << (bits - 1)) - 1);
    const bool f16out = ldo != 0;        // sq_rotate_fp16: Q and scales are unused, xout [T, ldo] is written
    if (T < 0 || K <= 0 || n1 <= 0 || n2 <= 0 || P < 0) return SQ_ERR_SHAPE;
    if (n1 > SQ_MAX_N1 || n2 > SQ_MAX_N2 || P > SQ_MAX_GIVENS) return SQ_ERR_SHAPE;
    if ((int64_t)n1 * n2 != K || (n2 % 8) != 0 || K > SQ_MAX_K || ldx < K) return SQ_ERR_SHAPE;
    if (T > SQ_MAX_ROWS) return SQ_ERR_SHAPE;
    if (P > 0 && (!giv_i || !giv_j || !giv_theta)) return SQ_ERR_NULL;
    if (!R1 || !R2) return SQ_ERR_NULL;
    if (f16out && ldo < K) return SQ_ERR_SHAPE;
    if (T > 0 && (!X || (f16out ? !xout : (!Q || !scales)))) return SQ_ERR_NULL;
    const sq::ListCache *cache = nullptr;
    const sq_status list_status = sq::cached_list(giv_i, giv_j, giv_theta, P, K, n2, &cache);
    if (list_status != SQ_OK) return list_status;
    const sq::ListCache &prep = *cache;
    const sq::GivensList &giv = prep.giv;
    if ((ldx % 8) != 0 || ((uintptr_t)X & 15) || ((uintptr_t)Q & 15) || ((uintptr_t)R1 & 15) ||
        ((uintptr_t)R2 & 15) || ((uintptr_t)scales & 3) || ((uintptr_t)xrot_dbg & 3))
        return SQ_ERR_ALIGN;
    if (f16out && (((uintptr_t)xout & 15) || (ldo % 8) != 0)) return SQ_ERR_ALIGN;
    if (T == 0) return SQ_OK;

    hipStream_t st = static_cast<hipStream_t>(stream);
    // matrix-core kernel for the shapes it covers (n2 in {32, 64, 128}, n1 <= 128); the plain-FMA
    // kernel takes every other shape.  The debug option SQ_DEBUG_ROTQ_PLAIN_KERNEL forces the latter.
    const bool force_generic = sq::debug_option(SQ_DEBUG_ROTQ_PLAIN_KERNEL) != 0;
    if (!force_generic && prep.plan_ok) {
        sq_status status = SQ_OK;
        const bool prepared = frag1 != nullptr;
        const bool plain_quantizer = bits == 4 && clip_ratio == 1.0f;
        sq::RotqPlan variant;                     // the cached plan with this call's quantizer
        if (!plain_quantizer) {
            variant = prep.plan;
            variant.q_top = q_top;
            variant.clip = clip_ratio;
            variant.q_div = q_top / clip_ratio;
        }
        const sq::RotqPlan &plan = plain_quantizer ? prep.plan : variant;
        if (f16out) {
            if (sq::rotq_mfma_dispatch_f16(static_cast<const __half *>(X), ldx, (int)T, n1, n2, plan,
                                           static_cast<const __half *>(R1), static_cast<const __half *>(R2),
                                           static_cast<__half *>(xout), ldo, st, &status))
                return status;
        } else if (sq::rotq_mfma_dispatch(static_cast<const __half *>(X), ldx, (int)T, n1, n2, plan,
                                   static_cast<const __half *>(prepared ? frag1 : R1),
                                   static_cast<const __half *>(prepared ? frag2 : R2), Q, scales, xrot_dbg, st,
                                   &status, prepared))
            return status;
    }
    const size_t lds = sizeof(float) * 2 * (size_t)K;
    if (!sq::allow_large_lds(reinterpret_cast<const void *>(sq::rotate_quantize_generic_kernel)))
        return SQ_ERR_LAUNCH;
    hipLaunchKernelGGL(sq::rotate_quantize_generic_kernel, dim3((unsigned)T), dim3(sq::kGenThreads),
                       lds, st, static_cast<const __half *>(X), ldx, K, n1, n2, giv,
                       static_cast<const __half *>(R1), static_cast<const __half *>(R2), Q, scales,
                       xrot_dbg, static_cast<__half *>(xout), ldo, q_top, q_top / clip_ratio);
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

extern "C" sq_status sq_rotate_fp16(const void *X, int64_t T, int32_t K, int64_t ldx,
                                    const int32_t *giv_i, const int32_t *giv_j, const float *giv_theta,
                                    int32_t P, const void *R1, int32_t n1, const void *R2, int32_t n2,
                                    void *Xrot, int64_t ldo, void *stream)
{
    if (ldo <= 0) return SQ_ERR_SHAPE;
    return rotate_quantize_any(X, T, K, ldx, giv_i, giv_j, giv_theta, P, R1, n1, R2, n2, nullptr, nullptr, nullptr,
                               stream, nullptr, nullptr, Xrot, ldo);
}

extern "C" sq_status sq_rotate_quantize(const void *X, int64_t T, int32_t K, int64_t ldx,
                                        const int32_t *giv_i, const int32_t *giv_j,
                                        const float *giv_theta, int32_t P, const void *R1,
                                        int32_t n1, const void *R2, int32_t n2, uint8_t *Q,
                                        float *scales, float *xrot_dbg, void *stream)
{
    return rotate_quantize_any(X, T, K, ldx, giv_i, giv_j, giv_theta, P, R1, n1, R2, n2, Q, scales, xrot_dbg,
                               stream, nullptr, nullptr);
}

extern "C" sq_status sq_rotate_quantize_variant(const void *X, int64_t T, int32_t K, int64_t ldx,
                                                const int32_t *giv_i, const int32_t *giv_j,
                                                const float *giv_theta, int32_t P, const void *R1,
                                                int32_t n1, const void *R2, int32_t n2, int32_t bits,
                                                float clip_ratio, uint8_t *Q, float *scales,
                                                float *xrot_dbg, void *stream)
{
    return rotate_quantize_any(X, T, K, ldx, giv_i, giv_j, giv_theta, P, R1, n1, R2, n2, Q, scales, xrot_dbg,
                               stream, nullptr, nullptr, nullptr, 0, bits, clip_ratio);
}

extern "C" sq_status sq_rotate_quantize_prepared(const void *X, int64_t T, int32_t K, int64_t ldx,
                                                 const int32_t *giv_i, const int32_t *giv_j,
                                                 const float *giv_theta, int32_t P, const void *prepared,
                                                 int32_t n1, int32_t n2, uint8_t *Q, float *scales,
                                                 float *xrot_dbg, void *stream)
{
    if (!sq::rotation_shape_ok(K, n1, n2)) return SQ_ERR_SHAPE;
    if (!prepared) return SQ_ERR_NULL;
    if ((uintptr_t)prepared & 15) return SQ_ERR_ALIGN;
    const sq::PreparedLayout l = sq::prepared_layout(n1, n2);
    const char *base = static_cast<const char *>(prepared);
    return rotate_quantize_any(X, T, K, ldx, giv_i, giv_j, giv_theta, P, base + l.off_r1, n1, base + l.off_r2, n2,
                               Q, scales, xrot_dbg, stream, l.fragments ? base + l.off_f1 : nullptr,
                               l.fragments ? base + l.off_f2 : nullptr);
}

extern "C" int64_t sq_decode_layer_workspace_bytes(int64_t T, int32_t K)
{
    if (T < 0 || T > SQ_DECODE_MAX_TOKENS || K <= 0 || K > SQ_MAX_K || (K % 2) != 0) return 0;
    return 512 + T * (int64_t)(K / 2);       // counters, steps, codes
}

// ---- workspace of sq_decode_layer_static ----------------------------------------------------------
// Counters, steps and codes of the largest legal call (SQ_DECODE_MAX_TOKENS tokens of SQ_MAX_K
// channels) in device memory that belongs to the loaded code object: 256.5 KiB per GPU, there
// from the moment the library is loaded on that GPU until the process ends, zero-filled by the
// loader (which is the state the counters must start from).
namespace sq {
constexpr size_t kStaticDecodeBytes = 512 + (size_t)SQ_DECODE_MAX_TOKENS * (SQ_MAX_K / 2);
}
static __device__ __align__(256) unsigned char sq_decode_scratch[sq::kStaticDecodeBytes];

namespace sq {

// Device address of sq_decode_scratch on the current device.  The array's name is only a handle
// on the host: every GPU holds its own copy at its own address, looked up once per device.
static void *decode_scratch_address()
{
    constexpr int kMaxDevices = 64;
    static std::mutex guard;
    static void *address[kMaxDevices] = {};
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(guard);
    if (address[device] == nullptr) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(sq_decode_scratch)) != hipSuccess) return nullptr;
        address[device] = p;
    }
    return address[device];
}

}  // namespace sq

// Validation and launch shared by sq_decode_layer and sq_decode_layer_static.  `workspace` is
// device memory (counters, steps, codes: sq_decode_layer_workspace_bytes of it), or null for the
// array inside the library, whose address is looked up once every check has passed.
static sq_status decode_layer_any(const void *X, int64_t T, int32_t K, int64_t ldx, const int32_t *giv_i,
                                  const int32_t *giv_j, const float *giv_theta, int32_t P, const void *prepared,
                                  int32_t n1, int32_t n2, const uint8_t *Qw, const float *sw, int32_t N, void *Y,
                                  int64_t ldy, void *workspace, bool use_static, void *stream)
{
    if (T < 0 || T > SQ_DECODE_MAX_TOKENS || N < 0 || P < 0 || P > SQ_MAX_GIVENS) return SQ_ERR_SHAPE;
    if (!sq::rotation_shape_ok(K, n1, n2) || ldx < K || ldy < N) return SQ_ERR_SHAPE;
    if (!sq::decode_layer_covers(n1, n2)) return SQ_ERR_SHAPE;
    if (P > 0 && (!giv_i || !giv_j || !giv_theta)) return SQ_ERR_NULL;
    if (!prepared) return SQ_ERR_NULL;
    if (T > 0 && N > 0 && (!X || !Qw || !sw || !Y || (!use_static && !workspace))) return SQ_ERR_NULL;
    const sq::ListCache *cache = nullptr;
    const sq_status list_status = sq::cached_list(giv_i, giv_j, giv_theta, P, K, n2, &cache);
    if (list_status != SQ_OK) return list_status;
    if (!cache->plan_ok) return SQ_ERR_SHAPE;
    if ((ldx % 8) != 0 || ((uintptr_t)X & 15) || ((uintptr_t)prepared & 15) || ((uintptr_t)Qw & 15) ||
        ((uintptr_t)sw & 3) || ((uintptr_t)Y & 1) || (!use_static && ((uintptr_t)workspace & 255)))
        return SQ_ERR_ALIGN;
    if (T == 0 || N == 0) return SQ_OK;
    if (use_static) {
        // every size that got here fits: T <= SQ_DECODE_MAX_TOKENS and K <= SQ_MAX_K were checked
        static_assert(512 + SQ_DECODE_MAX_TOKENS * (SQ_MAX_K / 2) <= sq::kStaticDecodeBytes, "largest call fits");
        workspace = sq::decode_scratch_address();
        if (!workspace) return SQ_ERR_LAUNCH;
    }
    const sq::PreparedLayout l = sq::prepared_layout(n1, n2);
    const char *base = static_cast<const char *>(prepared);
    char *ws = static_cast<char *>(workspace);
    return sq::decode_layer_dispatch(static_cast<const __half *>(X), ldx, (int)T, n1, n2, cache->plan,
                                     reinterpret_cast<const __half *>(base + l.off_f1),
                                     reinterpret_cast<const __half *>(base + l.off_f2),
                                     reinterpret_cast<uint8_t *>(ws + 512), reinterpret_cast<float *>(ws + 256),
                                     reinterpret_cast<int *>(ws), Qw, sw, N, static_cast<__half *>(Y), ldy,
                                     static_cast<hipStream_t>(stream));
}

extern "C" sq_status sq_decode_layer(const void *X, int64_t T, int32_t K, int64_t ldx,
                                     const int32_t *giv_i, const int32_t *giv_j, const float *giv_theta,
                                     int32_t P, const void *prepared, int32_t n1, int32_t n2,
                                     const uint8_t *Qw, const float *sw, int32_t N, void *Y, int64_t ldy,
                                     void *workspace, void *stream)
{
    return decode_layer_any(X, T, K, ldx, giv_i, giv_j, giv_theta, P, prepared, n1, n2, Qw, sw, N, Y, ldy, workspace,
                            false, stream);
}

extern "C" sq_status sq_decode_layer_static(const void *X, int64_t T, int32_t K, int64_t ldx,
                                            const int32_t *giv_i, const int32_t *giv_j,
                                            const float *giv_theta, int32_t P, const void *prepared,
                                            int32_t n1, int32_t n2, const uint8_t *Qw, const float *sw,
                                            int32_t N, void *Y, int64_t ldy, void *stream)
{
    return decode_layer_any(X, T, K, ldx, giv_i, giv_j, giv_theta, P, prepared, n1, n2, Qw, sw, N, Y, ldy, nullptr,
                            true, stream);
}

extern "C" sq_status sq_decode_layer_status(void *workspace, void *stream)
{
    if (((uintptr_t)workspace & 255) != 0) return SQ_ERR_ALIGN;
    char *ws = static_cast<char *>(workspace ? workspace : sq::decode_scratch_address());
    if (!ws) return SQ_ERR_LAUNCH;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (hipStreamSynchronize(st) != hipSuccess) return SQ_ERR_LAUNCH;
    int32_t word = 0;
    if (hipMemcpy(&word, ws + 12, sizeof(word), hipMemcpyDeviceToHost) != hipSuccess) return SQ_ERR_LAUNCH;
    if (word == 0) return SQ_OK;
    word = 0;
    if (hipMemcpy(ws + 12, &word, sizeof(word), hipMemcpyHostToDevice) != hipSuccess) return SQ_ERR_LAUNCH;
    return SQ_ERR_TIMEOUT;
}
