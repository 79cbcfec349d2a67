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
// registers as MFMA operands for the life of the workgroup, which walks over many tokens.
//
// Givens list (ART): the touched channels (at most 2P) are rotated in fp32 on a small LDS array,
// level by level (pairs of one level share no channel, so lanes work in parallel while the list
// order is kept).  A rotated value v goes back as hi = fp16(v) into the token tile and
// lo = fp16(v - hi) into a small side tile; stage A contracts the side tile against the matching
// rows of R2 in a few extra MFMA steps, so the fp16 rounding of hi is repaired to ~21 bits.
#include "sq_common.h"
#include "sq_rotq_plan.h"

namespace sq {

namespace {

__device__ __forceinline__ void dma_16(const void *gptr, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(gptr), "s"(lds_addr)
                 : "memory", "m0");
}

__device__ __forceinline__ void wait_all_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// swizzle of a tile row with CPR 16-byte chunks: 8 consecutive rows land on 8 different
// 16-byte bank groups for the column-of-rows access pattern of MFMA operand reads
template <int CPR>
__device__ __forceinline__ int swz(int row)
{
    return (CPR >= 8) ? (row & 7) : ((row >> 1) & 3);
}

}  // namespace

template <int N1P, int N2>
struct RotqShape {
    static constexpr int MB = N1P / 32;           // 32-row blocks of X_mat / Z (rows p)
    static constexpr int NCB = N2 / 32;           // 32-column blocks (columns q'): waves per token
    static constexpr int TPP = 4 / NCB;           // tokens per workgroup pass
    static constexpr int KSA = N2 / 16;           // MFMA steps of stage A (contraction over q)
    static constexpr int KSB = N1P / 16;          // MFMA steps of stage B (contraction over p)
    static constexpr int CPRX = N2 / 8;           // 16-byte chunks per tile row
    static constexpr int TILE_BYTES = N1P * N2 * 2;
    static constexpr int LO_ROW_BYTES = kRotqMaxQSlots * 2;           // 64 q-slots of fp16
    static constexpr int LO_BYTES = N1P * LO_ROW_BYTES;
    static constexpr int OUT_BYTES = N1P * N2 / 2;
    // LDS map (bytes)
    static constexpr int OFF_X = 0;                                   // [TPP][2][TILE]
    static constexpr int OFF_LO = OFF_X + TPP * 2 * TILE_BYTES;       // [TPP][LO]
    static constexpr int OFF_GV = OFF_LO + TPP * LO_BYTES;            // [TPP][128] float
    static constexpr int OFF_RED = OFF_GV + TPP * kRotqMaxSlots * 4;  // [TPP][4] float
    static constexpr int OFF_OUT = OFF_RED + TPP * 4 * 4;             // [TPP][OUT]
    static constexpr int WORK_BYTES = OFF_OUT + TPP * OUT_BYTES;
    // the prologue stages R2 and then R1 at the start of LDS
    static constexpr int PRO_BYTES = (N2 * N2 > N1P * N1P ? N2 * N2 : N1P * N1P) * 2;
    static constexpr int LDS_BYTES = WORK_BYTES > PRO_BYTES ? WORK_BYTES : PRO_BYTES;
    static_assert(N2 == 32 || N2 == 64 || N2 == 128, "one to four waves per token");
    static_assert(N1P % 32 == 0 && N1P <= 96, "rows padded to a multiple of 32");
};

template <int N1P, int N2>
__global__ __launch_bounds__(256, 2) void rotate_quantize_mfma_kernel(
    const __half *__restrict__ X, int64_t ldx, int T, int n1, RotqPlan plan,
    const __half *__restrict__ R1, const __half *__restrict__ R2, uint8_t *__restrict__ Q,
    float *__restrict__ scales, float *__restrict__ xrot)
{
    using S = RotqShape<N1P, N2>;
    constexpr int MB = S::MB, NCB = S::NCB, TPP = S::TPP, KSA = S::KSA, KSB = S::KSB, CPRX = S::CPRX;
    constexpr int QS_STEPS = kRotqMaxQSlots / 16;
    extern __shared__ uint4 smem_u4[];
    char *lds = reinterpret_cast<char *>(smem_u4);
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4 *)smem_u4;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tok_slot = wave / NCB, cb = wave % NCB;        // which token of the pass, which columns
    const int l32 = lane & 31, g = lane >> 5;
    const int K = n1 * N2;
    const int row_chunks = n1 * CPRX;                        // 16-byte chunks of one token row

    // ---- prologue: R2 and R1 as MFMA operands in registers ---------------------------------
    // R2 (stage A, operand B): lane holds column q' = 32cb + l32, step ks, element e <-> row
    // q = 16ks + 8g + e.  Staged through LDS so that the global reads are coalesced.
    v8h r2f[KSA], r2x[QS_STEPS], r1f[MB][KSB];
    {
        __half *tmp = reinterpret_cast<__half *>(lds);
        for (int c = tid; c < N2 * N2 / 8; c += 256)
            reinterpret_cast<uint4 *>(tmp)[c] = reinterpret_cast<const uint4 *>(R2)[c];
        __syncthreads();
        const int qo = 32 * cb + l32;
#pragma unroll
        for (int ks = 0; ks < KSA; ++ks)
#pragma unroll
            for (int e = 0; e < 8; ++e) r2f[ks][e] = (_Float16)tmp[(16 * ks + 8 * g + e) * N2 + qo];
        // rows of R2 that pair with the q-slots of the Givens side tile
#pragma unroll
        for (int x = 0; x < QS_STEPS; ++x)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int qs = 16 * x + 8 * g + e;
                r2x[x][e] = (qs < plan.n_qslots) ? (_Float16)tmp[plan.qlist[qs] * N2 + qo] : (_Float16)0.f;
            }
        __syncthreads();
        // R1 (stage B, operand B): lane holds column p' = 32nb + l32; step ks, element e <-> row
        // p = 16ks + 8(e/4) + 4g + e%4, which is where stage A leaves row p of Z in this lane.
        for (int c = tid; c < n1 * n1; c += 256) tmp[c] = R1[c];
        __syncthreads();
#pragma unroll
        for (int nb = 0; nb < MB; ++nb)
#pragma unroll
            for (int ks = 0; ks < KSB; ++ks)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int p = 16 * ks + 8 * (e / 4) + 4 * g + (e % 4), po = 32 * nb + l32;
                    r1f[nb][ks][e] = (p < n1 && po < n1) ? (_Float16)tmp[p * n1 + po] : (_Float16)0.f;
                }
        __syncthreads();
        // tiles start as zeros: padding rows (p >= n1) and unused side-tile slots stay zero
        for (int c = tid; c < S::OFF_GV / 16; c += 256) smem_u4[c] = uint4{0, 0, 0, 0};
        __syncthreads();
    }

    // ---- token loop ---------------------------------------------------------------------
    const int groups = (T + TPP - 1) / TPP;
    auto issue_group = [&](int grp, int buf) {
        // all four waves share the loads of the TPP token rows of the group
        const int loads_per_tok = (row_chunks + 63) / 64;
        for (int li = wave; li < TPP * loads_per_tok; li += 4) {
            const int ts = li / loads_per_tok, part = li % loads_per_tok;
            const int t = grp * TPP + ts;
            const int slot = part * 64 + lane;
            if (t < T && slot < row_chunks) {
                const int row = slot / CPRX, pc = slot % CPRX;
                const __half *src = X + (int64_t)t * ldx + row * N2 + ((pc ^ swz<CPRX>(row)) * 8);
                const uint32_t dst = lds_base + S::OFF_X + (ts * 2 + buf) * S::TILE_BYTES + part * 1024;
                dma_16(src, __builtin_amdgcn_readfirstlane(dst));
            }
        }
    };

    int buf = 0;
    if ((int)blockIdx.x < groups) issue_group(blockIdx.x, 0);
    for (int grp = blockIdx.x; grp < groups; grp += gridDim.x, buf ^= 1) {
        const int t = grp * TPP + tok_slot;
        const bool live = t < T;
        wait_all_loads();
        __syncthreads();                       // tiles of this group are in LDS; outputs of the last one are out
        if (grp + (int)gridDim.x < groups) issue_group(grp + gridDim.x, buf ^ 1);

        char *xt = lds + S::OFF_X + (tok_slot * 2 + buf) * S::TILE_BYTES;
        char *lo_t = lds + S::OFF_LO + tok_slot * S::LO_BYTES;

        // ---- Givens list on the touched channels (first wave of the token) -----------------
        if (cb == 0 && plan.n_slots > 0) {
            float *gv = reinterpret_cast<float *>(lds + S::OFF_GV) + tok_slot * kRotqMaxSlots;
            auto tile_half = [&](int ch) -> __half * {
                const int p = ch / N2, q = ch % N2;
                return reinterpret_cast<__half *>(xt + (p * CPRX + ((q >> 3) ^ swz<CPRX>(p))) * 16 + (q & 7) * 2);
            };
            for (int s = lane; s < plan.n_slots; s += 64) gv[s] = __half2float(*tile_half(plan.chan[s]));
            for (int lv = 0; lv < plan.n_levels; ++lv) {
                __builtin_amdgcn_wave_barrier();     // LDS traffic of one wave stays in program order
                const int pi = plan.level_begin[lv] + lane;
                if (pi < plan.level_begin[lv + 1]) {
                    const int si = plan.pair_i[pi], sj = plan.pair_j[pi];
                    const float a = gv[si], b = gv[sj], c = plan.c[pi], sn = plan.s[pi];
                    gv[si] = a * c + b * sn;
                    gv[sj] = b * c - a * sn;
                }
            }
            for (int s = lane; s < plan.n_slots; s += 64) {
                const float v = gv[s];
                const __half hi = __float2half_rn(v);
                const int ch = plan.chan[s], p = ch / N2, qs = plan.qslot[s];
                *tile_half(ch) = hi;
                *reinterpret_cast<__half *>(lo_t + (p * 8 + ((qs >> 3) ^ (p & 7))) * 16 + (qs & 7) * 2) =
                    __float2half_rn(v - __half2float(hi));
            }
        }
        __syncthreads();

        // ---- stage A: Z = X_mat R2 (+ side tile x matching rows of R2) ---------------------
        v16f accz[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
            for (int e = 0; e < 16; ++e) accz[mb][e] = 0.f;
            const int row = 32 * mb + l32;
#pragma unroll
            for (int ks = 0; ks < KSA; ++ks) {
                const v8h a = *reinterpret_cast<const v8h *>(xt + (row * CPRX + ((2 * ks + g) ^ swz<CPRX>(row))) * 16);
                accz[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, r2f[ks], accz[mb], 0, 0, 0);
            }
#pragma unroll
            for (int x = 0; x < QS_STEPS; ++x) {
                if (16 * x < plan.n_qslots) {
                    const v8h a = *reinterpret_cast<const v8h *>(lo_t + (row * 8 + ((2 * x + g) ^ (row & 7))) * 16);
                    accz[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, r2x[x], accz[mb], 0, 0, 0);
                }
            }
        }

        // ---- power-of-two prescale of this wave's columns so that hi/lo fit fp16 -------------
        // Stage B contracts over rows p within a column, so a per-wave factor commutes with it.
        float zmax = 0.f;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int e = 0; e < 16; e += 2) zmax = fmaxf(zmax, fmaxf(fabsf(accz[mb][e]), fabsf(accz[mb][e + 1])));
        zmax = wave_max(zmax);
        float fz = 1.0f, fz_inv = 1.0f;          // Z * fz in [2^13, 2^14) at its largest entry
        if (!(zmax >= 1.0f && zmax < 16384.0f) && zmax > 0.f) {
            const int ez = (int)((__float_as_uint(zmax) >> 23) & 0xFF) - 127;
            const int sh = max(-100, min(100, 13 - ez));
            fz = __uint_as_float((uint32_t)(127 + sh) << 23);
            fz_inv = __uint_as_float((uint32_t)(127 - sh) << 23);
        }

        // ---- stage B: Y^T = Z^T R1, Z = hi + lo -------------------------------------------
        v16f accy[MB];
#pragma unroll
        for (int nb = 0; nb < MB; ++nb)
#pragma unroll
            for (int e = 0; e < 16; ++e) accy[nb][e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KSB; ++ks) {
            const int mb = ks >> 1, r0 = 8 * (ks & 1);
            v8h zh, zl;
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const float z0 = accz[mb][r0 + e] * fz, z1 = accz[mb][r0 + e + 1] * fz;
                const auto h = __builtin_amdgcn_cvt_pkrtz(z0, z1);
                const auto l = __builtin_amdgcn_cvt_pkrtz(z0 - (float)h[0], z1 - (float)h[1]);
                zh[e] = (_Float16)h[0]; zh[e + 1] = (_Float16)h[1];
                zl[e] = (_Float16)l[0]; zl[e + 1] = (_Float16)l[1];
            }
#pragma unroll
            for (int nb = 0; nb < MB; ++nb) {
                accy[nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(zh, r1f[nb][ks], accy[nb], 0, 0, 0);
                accy[nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(zl, r1f[nb][ks], accy[nb], 0, 0, 0);
            }
        }

        // ---- per-token step -----------------------------------------------------------------
        float amax = 0.f;
#pragma unroll
        for (int nb = 0; nb < MB; ++nb)
#pragma unroll
            for (int e = 0; e < 16; e += 2) amax = fmaxf(amax, fmaxf(fabsf(accy[nb][e]), fabsf(accy[nb][e + 1])));
        amax = wave_max(amax) * fz_inv;        // padded rows and columns of Y are exact zeros
        float *red = reinterpret_cast<float *>(lds + S::OFF_RED) + tok_slot * 4;
        if (lane == 0) red[cb] = amax;
        __syncthreads();
        amax = red[0];
#pragma unroll
        for (int w = 1; w < NCB; ++w) amax = fmaxf(amax, red[w]);
        const float step = (amax == 0.f) ? 1.0f : amax / 7.0f;
        const float inv = fz_inv / step;       // codes = Y / step with Y = accy * fz_inv
        if (live && cb == 0 && lane == 0) scales[t] = step;

        // ---- codes -> LDS staging: lane holds column p' = 32nb + l32 of Y^T and, per register
        // group r/4, four consecutive q' = 32cb + 8(r/4) + 4g + (0..3): two bytes of the row
        char *outq = lds + S::OFF_OUT + tok_slot * S::OUT_BYTES;
#pragma unroll
        for (int nb = 0; nb < MB; ++nb) {
            const int po = 32 * nb + l32;
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                uint32_t w = 0;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    // floor(v + 1/2) + 8 = trunc(v + 8.5) for v in [-8, 7.5); two's-complement nibble = that ^ 8
                    const uint32_t c = (uint32_t)fmaf(accy[nb][4 * rg + u], inv, 8.5f);
                    w |= c << (4 * u);
                }
                if (po < n1)
                    *reinterpret_cast<uint16_t *>(outq + po * (N2 / 2) + 16 * cb + 4 * rg + 2 * g) =
                        (uint16_t)(w ^ 0x8888u);
            }
        }
        if (xrot != nullptr && live) {
#pragma unroll
            for (int nb = 0; nb < MB; ++nb) {
                const int po = 32 * nb + l32;
                if (po < n1) {
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        xrot[(int64_t)t * K + po * N2 + 32 * cb + 8 * (e / 4) + 4 * g + (e % 4)] =
                            accy[nb][e] * fz_inv;
                }
            }
        }
        __syncthreads();

        // ---- coalesced copy-out of the TPP code rows ----------------------------------------
        const int row_out_chunks = K / 32;       // 16-byte chunks of one code row
        for (int c = tid; c < TPP * row_out_chunks; c += 256) {
            const int ts = c / row_out_chunks, cc = c % row_out_chunks;
            const int tt = grp * TPP + ts;
            if (tt < T)
                reinterpret_cast<uint4 *>(Q + (int64_t)tt * (K / 2))[cc] =
                    *reinterpret_cast<const uint4 *>(lds + S::OFF_OUT + ts * S::OUT_BYTES + cc * 16);
        }
    }
    wait_all_loads();
}

template <int N1P, int N2>
static sq_status launch_rotq_mfma(const __half *X, int64_t ldx, int T, int n1, const RotqPlan &plan,
                                  const __half *R1, const __half *R2, uint8_t *Q, float *scales,
                                  float *xrot, hipStream_t st)
{
    using S = RotqShape<N1P, N2>;
    static_assert(S::LDS_BYTES <= 80 * 1024, "two workgroups per CU");
    auto kernel = rotate_quantize_mfma_kernel<N1P, N2>;
    if (!allow_large_lds(reinterpret_cast<const void *>(kernel))) return SQ_ERR_LAUNCH;
    const int groups = (T + S::TPP - 1) / S::TPP;
    const int grid = groups < 512 ? groups : 512;           // two workgroups on each of 256 CUs
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), S::LDS_BYTES, st, X, ldx, T, n1, plan, R1,
                       R2, Q, scales, xrot);
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

// Picks the instantiation for (n1, n2); returns false if this kernel does not cover the shape.
bool rotq_mfma_dispatch(const __half *X, int64_t ldx, int T, int n1, int n2, const RotqPlan &plan,
                        const __half *R1, const __half *R2, uint8_t *Q, float *scales, float *xrot,
                        hipStream_t st, sq_status *status)
{
    if (n1 % 2 != 0 && ((n1 * n2) % 32) != 0) return false;
    if (((int64_t)n1 * n2) % 32 != 0) return false;          // copy-out works in 16-byte chunks
#define SQ_ROTQ_CASE(N1P, N2)                                                                        \
    if (n2 == N2 && n1 <= N1P && n1 > N1P - 32) {                                                    \
        *status = launch_rotq_mfma<N1P, N2>(X, ldx, T, n1, plan, R1, R2, Q, scales, xrot, st);       \
        return true;                                                                                 \
    }
    SQ_ROTQ_CASE(32, 32)
    SQ_ROTQ_CASE(64, 32)
    SQ_ROTQ_CASE(32, 64)
    SQ_ROTQ_CASE(64, 64)
    SQ_ROTQ_CASE(96, 64)
    SQ_ROTQ_CASE(32, 128)
    SQ_ROTQ_CASE(64, 128)
    SQ_ROTQ_CASE(96, 128)
#undef SQ_ROTQ_CASE
    return false;
}

}  // namespace sq
