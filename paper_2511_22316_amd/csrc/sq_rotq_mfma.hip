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
// Token rows stream from HBM straight into a ring of three LDS tiles (global_load_lds), two rows
// ahead of the one being multiplied; two workgroups share a CU, so four rows per CU are in flight.
//
// Givens list (ART): the touched channels (at most 2P) are rotated in fp32 on a small LDS array,
// level by level (pairs of one level share no channel, so lanes work in parallel while the list
// order is kept).  A rotated value v goes back as hi = fp16(v) into the token tile and
// lo = fp16(v - hi) into a small side tile; stage A contracts the side tile against the matching
// rows of R2 in a few extra MFMA steps, so the fp16 rounding of hi is repaired to ~21 bits.
// The first wave of a token does this for the NEXT token while the other waves finish the
// current one.
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

template <int N>
__device__ __forceinline__ void wait_loads_le()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// swizzle of a tile row with CPR 16-byte chunks: 8 consecutive rows land on 8 different
// 16-byte bank groups for the column-of-rows access pattern of MFMA operand reads
template <int CPR>
__device__ __forceinline__ int swz(int row)
{
    return (CPR >= 8) ? (row & 7) : ((row >> 1) & 3);
}

typedef uint32_t v4u __attribute__((ext_vector_type(4)));

// (z0, z1) -> hi = their fp16 truncations packed in one dword, lo = fp16 of the exact remainders
// z - hi (the mixed-precision FMA reads the fp16 half directly, and the difference is exact)
__device__ __forceinline__ void split_pair(float z0, float z1, uint32_t &hi, uint32_t &lo)
{
    hi = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(z0, z1));
    float r0, r1;
    asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel_hi:[1,0,0]" : "=v"(r0) : "v"(hi), "v"(z0));
    asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r1) : "v"(hi), "v"(z1));
    lo = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(r0, r1));
}

}  // namespace

template <int N1, int N2>
struct RotqShape {
    static constexpr int N1P = (N1 + 31) / 32 * 32;   // rows padded to the MFMA block
    static constexpr int MB = N1P / 32;           // 32-row blocks of X_mat / Z (rows p)
    static constexpr int NCB = N2 / 32;           // 32-column blocks (columns q'): waves per token
    static constexpr int TPP = 4 / NCB;           // tokens per workgroup pass
    static constexpr int KSA = N2 / 16;           // MFMA steps of stage A (contraction over q)
    static constexpr int KSB = N1P / 16;          // MFMA steps of stage B (contraction over p)
    static constexpr int CPRX = N2 / 8;           // 16-byte chunks per tile row
    static constexpr int ROW_CHUNKS = N1 * CPRX;  // 16-byte chunks of one token row
    static constexpr int LPT = (ROW_CHUNKS + 63) / 64;    // wave-wide loads per token row
    static constexpr int NSX = 3;                 // ring of token tiles
    static constexpr int TILE_BYTES = N1P * N2 * 2;
    static constexpr int LO_ROW_BYTES = kRotqMaxQSlots * 2;           // 64 q-slots of fp16
    static constexpr int LO_BYTES = N1P * LO_ROW_BYTES;
    static constexpr int OUT_UNITS = N2 / 4;      // 2-byte units (4 codes) per output row p'
    static constexpr int OUT_BYTES = OUT_UNITS * N1P * 2;             // staged as [unit][p']
    // LDS map (bytes)
    static constexpr int OFF_X = 0;                                   // [TPP][NSX][TILE]
    static constexpr int OFF_LO = OFF_X + TPP * NSX * TILE_BYTES;     // [TPP][2][LO]
    static constexpr int OFF_ZERO_END = OFF_LO + TPP * 2 * LO_BYTES;
    static constexpr int OFF_GV = OFF_ZERO_END;                       // [TPP][128] float
    static constexpr int OFF_RED = OFF_GV + TPP * kRotqMaxSlots * 4;  // [TPP][4] float
    static constexpr int OFF_OUT = OFF_RED + TPP * 4 * 4;             // [TPP][OUT]
    static constexpr int WORK_BYTES = OFF_OUT + TPP * OUT_BYTES;
    // the prologue stages R2 and then R1 at the start of LDS
    static constexpr int PRO_BYTES = (N2 * N2 > N1 * N1 ? N2 * N2 : N1 * N1) * 2;
    static constexpr int LDS_BYTES = WORK_BYTES > PRO_BYTES ? WORK_BYTES : PRO_BYTES;
    static constexpr int OCC = (2 * LDS_BYTES <= 158 * 1024) ? 2 : 1;   // workgroups per CU
    static_assert(N2 == 32 || N2 == 64 || N2 == 128, "one to four waves per token");
    static_assert(N1P <= 96, "at most three row blocks");
    static_assert(2 * LPT < 64, "outstanding loads must fit the vmcnt counter");
    static_assert(PRO_BYTES <= OFF_ZERO_END, "prologue staging lies inside the tile ring");
};

template <int N1, int N2>
__global__ __launch_bounds__(256, (RotqShape<N1, N2>::OCC)) void rotate_quantize_mfma_kernel(
    const __half *__restrict__ X, int64_t ldx, int T, RotqPlan plan,
    const __half *__restrict__ R1, const __half *__restrict__ R2, uint8_t *__restrict__ Q,
    float *__restrict__ scales, float *__restrict__ xrot)
{
    using S = RotqShape<N1, N2>;
    constexpr int N1P = S::N1P, MB = S::MB, NCB = S::NCB, TPP = S::TPP, KSA = S::KSA, KSB = S::KSB;
    constexpr int CPRX = S::CPRX, LPT = S::LPT, NSX = S::NSX, K = N1 * N2;
    constexpr int QS_STEPS = kRotqMaxQSlots / 16;
    extern __shared__ uint4 smem_u4[];
    char *lds = reinterpret_cast<char *>(smem_u4);
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4 *)smem_u4;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tok_slot = wave / NCB, cb = wave % NCB;        // which token of the pass, which columns
    const int l32 = lane & 31, g = lane >> 5;
    const bool lead = (cb == 0);                             // this wave loads and Givens-rotates its token

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
        for (int c = tid; c < N1 * N1; c += 256) tmp[c] = R1[c];
        __syncthreads();
#pragma unroll
        for (int nb = 0; nb < MB; ++nb)
#pragma unroll
            for (int ks = 0; ks < KSB; ++ks)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int p = 16 * ks + 8 * (e / 4) + 4 * g + (e % 4), po = 32 * nb + l32;
                    r1f[nb][ks][e] = (p < N1 && po < N1) ? (_Float16)tmp[p * N1 + po] : (_Float16)0.f;
                }
        __syncthreads();
        // tiles start as zeros: padding rows (p >= N1) and unused side-tile slots stay zero
        for (int c = tid; c < S::OFF_ZERO_END / 16; c += 256) smem_u4[c] = uint4{0, 0, 0, 0};
        __syncthreads();
    }

    // lane l owns pair l of the level-sorted Givens list: its slots, angle and level
    int my_level = -1, my_si = 0, my_sj = 0;
    float my_c = 1.f, my_s = 0.f;
    {
        const int n_pairs = plan.level_begin[plan.n_levels];
        if (lane < n_pairs) {
            my_si = plan.pair_i[lane];
            my_sj = plan.pair_j[lane];
            my_c = plan.c[lane];
            my_s = plan.s[lane];
            for (int lv = 0; lv < plan.n_levels; ++lv)
                if (lane >= plan.level_begin[lv]) my_level = lv;
        }
    }
    // per-lane gather / scatter addresses of the touched channels (two slots per lane)
    int gs_tile[2], gs_lo[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int s = lane + 64 * u;
        gs_tile[u] = -1;
        gs_lo[u] = 0;
        if (s < plan.n_slots) {
            const int ch = plan.chan[s], p = ch / N2, q = ch % N2, qs = plan.qslot[s];
            gs_tile[u] = (p * CPRX + ((q >> 3) ^ swz<CPRX>(p))) * 16 + (q & 7) * 2;
            gs_lo[u] = (p * 8 + ((qs >> 3) ^ (p & 7))) * 16 + (qs & 7) * 2;
        }
    }

    // LDS byte offsets of this lane's operand chunks inside a tile (row block 0): the swizzle
    // only touches the low bits of the chunk index, so four offsets cover every step
    constexpr int NJ = KSA < 4 ? KSA : 4;
    int a_off[NJ], lo_off[QS_STEPS];
#pragma unroll
    for (int j = 0; j < NJ; ++j) a_off[j] = (l32 * CPRX + ((2 * j + g) ^ swz<CPRX>(l32))) * 16;
#pragma unroll
    for (int x = 0; x < QS_STEPS; ++x) lo_off[x] = (l32 * 8 + ((2 * x + g) ^ (l32 & 7))) * 16;

    const int groups = (T + TPP - 1) / TPP;
    const int stride = gridDim.x;
    // does this wave's token exist in group grp (the last group may be partial)?
    auto has_row = [&](int grp) { return (int64_t)grp * TPP + tok_slot < T; };
    // lead wave: all loads of its token row of group `grp` into ring slot `slot`
    auto issue_row = [&](int grp, int slot) {
        if (has_row(grp)) {
            const __half *row = X + ((int64_t)grp * TPP + tok_slot) * ldx;
            const uint32_t dst0 = lds_base + S::OFF_X + (tok_slot * NSX + slot) * S::TILE_BYTES;
#pragma unroll
            for (int part = 0; part < LPT; ++part) {
                const int c = part * 64 + lane;
                if (c < S::ROW_CHUNKS) {
                    const int r = c / CPRX, pc = c % CPRX;
                    dma_16(row + r * N2 + ((pc ^ swz<CPRX>(r)) * 8),
                           __builtin_amdgcn_readfirstlane(dst0 + part * 1024));
                }
            }
        }
    };
    // lead wave: Givens list on the tile in ring slot `slot`, side tile `lo_sel`
    auto givens = [&](int slot, int lo_sel) {
        if (plan.n_slots == 0) return;
        char *xt = lds + S::OFF_X + (tok_slot * NSX + slot) * S::TILE_BYTES;
        char *lo_t = lds + S::OFF_LO + (tok_slot * 2 + lo_sel) * S::LO_BYTES;
        float *gv = reinterpret_cast<float *>(lds + S::OFF_GV) + tok_slot * kRotqMaxSlots;
#pragma unroll
        for (int u = 0; u < 2; ++u)
            if (gs_tile[u] >= 0) gv[lane + 64 * u] = __half2float(*reinterpret_cast<const __half *>(xt + gs_tile[u]));
        for (int lv = 0; lv < plan.n_levels; ++lv) {
            __builtin_amdgcn_wave_barrier();     // LDS traffic of one wave stays in program order
            if (my_level == lv) {                // lane l owns pair l of the level-sorted list
                const float a = gv[my_si], b = gv[my_sj];
                gv[my_si] = a * my_c + b * my_s;
                gv[my_sj] = b * my_c - a * my_s;
            }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < 2; ++u)
            if (gs_tile[u] >= 0) {
                const float v = gv[lane + 64 * u];
                const __half hi = __float2half_rn(v);
                *reinterpret_cast<__half *>(xt + gs_tile[u]) = hi;
                *reinterpret_cast<__half *>(lo_t + gs_lo[u]) = __float2half_rn(v - __half2float(hi));
            }
    };

    // ---- pipeline prologue: three rows in flight, first one rotated -------------------------
    const int g0 = blockIdx.x;
    if (lead) {
        issue_row(g0, 0);
        issue_row(g0 + stride, 1);
        issue_row(g0 + 2 * stride, 2);
        if (has_row(g0 + 2 * stride)) wait_loads_le<2 * LPT>();
        else if (has_row(g0 + stride)) wait_loads_le<LPT>();
        else wait_loads_le<0>();
        givens(0, 0);
    }
    __syncthreads();

    int slot = 0, it = 0;
    for (int grp = g0; grp < groups; grp += stride, ++it) {
        const int t = grp * TPP + tok_slot;
        const bool live = t < T;
        const int slot1 = (slot + 1 == NSX) ? 0 : slot + 1;
        const char *xt = lds + S::OFF_X + (tok_slot * NSX + slot) * S::TILE_BYTES;
        const char *lo_t = lds + S::OFF_LO + (tok_slot * 2 + (it & 1)) * S::LO_BYTES;

        // ---- stage A: Z = X_mat R2 (+ side tile x matching rows of R2) ---------------------
        v16f accz[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
            for (int e = 0; e < 16; ++e) accz[mb][e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KSA; ++ks) {
                const v8h a = *reinterpret_cast<const v8h *>(xt + a_off[ks % 4] + (ks / 4) * 128 + mb * (32 * CPRX * 16));
                accz[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, r2f[ks], accz[mb], 0, 0, 0);
            }
#pragma unroll
            for (int x = 0; x < QS_STEPS; ++x) {
                if (16 * x < plan.n_qslots) {
                    const v8h a = *reinterpret_cast<const v8h *>(lo_t + lo_off[x] + mb * (32 * 8 * 16));
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
        const bool rescale = !(zmax >= 1.0f && zmax < 16384.0f) && zmax > 0.f;
        if (rescale) {
            const int ez = (int)((__float_as_uint(zmax) >> 23) & 0xFF) - 127;
            const int sh = max(-100, min(100, 13 - ez));
            fz = __uint_as_float((uint32_t)(127 + sh) << 23);
            fz_inv = __uint_as_float((uint32_t)(127 - sh) << 23);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int e = 0; e < 16; ++e) accz[mb][e] *= fz;
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
            v4u zhu, zlu;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                uint32_t hi, lo;
                split_pair(accz[mb][r0 + 2 * e], accz[mb][r0 + 2 * e + 1], hi, lo);
                zhu[e] = hi;
                zlu[e] = lo;
            }
            const v8h zh = __builtin_bit_cast(v8h, zhu), zl = __builtin_bit_cast(v8h, zlu);
#pragma unroll
            for (int nb = 0; nb < MB; ++nb) {
                accy[nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(zh, r1f[nb][ks], accy[nb], 0, 0, 0);
                accy[nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(zl, r1f[nb][ks], accy[nb], 0, 0, 0);
            }
        }

        // ---- per-token step: wave maximum now, token maximum after the barrier --------------
        float amax = 0.f;
#pragma unroll
        for (int nb = 0; nb < MB; ++nb)
#pragma unroll
            for (int e = 0; e < 16; e += 2) amax = fmaxf(amax, fmaxf(fabsf(accy[nb][e]), fabsf(accy[nb][e + 1])));
        amax = wave_max(amax) * fz_inv;        // padded rows and columns of Y are exact zeros
        float *red = reinterpret_cast<float *>(lds + S::OFF_RED) + tok_slot * 4;
        if (lane == 0) red[cb] = amax;

        // ---- lead wave: the next row has landed (rows complete in order; only the row after it
        // may still be in flight) -> rotate its touched channels while the others catch up
        if (lead) {
            if (has_row(grp + 2 * stride)) wait_loads_le<LPT>();
            else wait_loads_le<0>();
            if (has_row(grp + stride)) givens(slot1, (it + 1) & 1);
        }
        __syncthreads();     // B2: maxima visible; tile `slot` is no longer read; next tile rotated
        if (lead) issue_row(grp + 3 * stride, slot);

        amax = red[0];
#pragma unroll
        for (int w = 1; w < NCB; ++w) amax = fmaxf(amax, red[w]);
        const float step = (amax == 0.f) ? 1.0f : amax / 7.0f;
        const float inv = fz_inv / step;       // codes = Y / step with Y = accy * fz_inv
        if (live && lead && lane == 0) scales[t] = step;

        // ---- codes -> LDS staging.  A lane holds column p' = 32nb + l32 of Y^T and, per register
        // group rg, four consecutive q' = 32cb + 8rg + 4g + (0..3): one 2-byte unit of the row.
        // Staged as [unit][p'] so that the 32 lanes of a store hit 32 consecutive halfwords.
        uint16_t *outq = reinterpret_cast<uint16_t *>(lds + S::OFF_OUT + tok_slot * S::OUT_BYTES);
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
                outq[(8 * cb + 2 * rg + g) * N1P + po] = (uint16_t)(w ^ 0x8888u);
            }
        }
        if (xrot != nullptr && live) {
#pragma unroll
            for (int nb = 0; nb < MB; ++nb) {
                const int po = 32 * nb + l32;
                if (po < N1) {
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        xrot[(int64_t)t * K + po * N2 + 32 * cb + 8 * (e / 4) + 4 * g + (e % 4)] =
                            accy[nb][e] * fz_inv;
                }
            }
        }
        __syncthreads();     // B3: staged codes complete

        // ---- copy-out: 16 bytes (8 units of one row p') per lane, coalesced along the row -----
        constexpr int ROW_OUT_CHUNKS = K / 32;      // 16-byte chunks of one code row
        constexpr int CH_PER_P = S::OUT_UNITS / 8;  // chunks per row p'
        for (int c = tid; c < TPP * ROW_OUT_CHUNKS; c += 256) {
            const int ts = c / ROW_OUT_CHUNKS, cc = c % ROW_OUT_CHUNKS;
            const int tt = grp * TPP + ts;
            const int po = cc / CH_PER_P, u0 = (cc % CH_PER_P) * 8;
            const uint16_t *src = reinterpret_cast<const uint16_t *>(lds + S::OFF_OUT + ts * S::OUT_BYTES) + u0 * N1P + po;
            uint4 v;
            v.x = src[0] | ((uint32_t)src[N1P] << 16);
            v.y = src[2 * N1P] | ((uint32_t)src[3 * N1P] << 16);
            v.z = src[4 * N1P] | ((uint32_t)src[5 * N1P] << 16);
            v.w = src[6 * N1P] | ((uint32_t)src[7 * N1P] << 16);
            if (tt < T) reinterpret_cast<uint4 *>(Q + (int64_t)tt * (K / 2))[cc] = v;
        }
        slot = slot1;
    }
    wait_loads_le<0>();
}

template <int N1, int N2>
static sq_status launch_rotq_mfma(const __half *X, int64_t ldx, int T, const RotqPlan &plan,
                                  const __half *R1, const __half *R2, uint8_t *Q, float *scales,
                                  float *xrot, hipStream_t st)
{
    using S = RotqShape<N1, N2>;
    auto kernel = rotate_quantize_mfma_kernel<N1, N2>;
    if (!allow_large_lds(reinterpret_cast<const void *>(kernel))) return SQ_ERR_LAUNCH;
    const int groups = (T + S::TPP - 1) / S::TPP;
    const int resident = 256 * S::OCC;                      // workgroups the chip holds at once
    const int grid = groups < resident ? groups : resident;
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), S::LDS_BYTES, st, X, ldx, T, plan, R1, R2, Q,
                       scales, xrot);
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

// Picks the instantiation for (n1, n2); returns false if this kernel does not cover the shape.
bool rotq_mfma_dispatch(const __half *X, int64_t ldx, int T, int n1, int n2, const RotqPlan &plan,
                        const __half *R1, const __half *R2, uint8_t *Q, float *scales, float *xrot,
                        hipStream_t st, sq_status *status)
{
#define SQ_ROTQ_CASE(N1, N2)                                                                         \
    if (n1 == N1 && n2 == N2) {                                                                      \
        *status = launch_rotq_mfma<N1, N2>(X, ldx, T, plan, R1, R2, Q, scales, xrot, st);            \
        return true;                                                                                 \
    }
    SQ_ROTQ_CASE(16, 32)     // K = 512
    SQ_ROTQ_CASE(32, 32)     // 1024
    SQ_ROTQ_CASE(32, 64)     // 2048
    SQ_ROTQ_CASE(64, 64)     // 4096
    SQ_ROTQ_CASE(80, 64)     // 5120
    SQ_ROTQ_CASE(64, 128)    // 8192
    SQ_ROTQ_CASE(86, 128)    // 11008
#undef SQ_ROTQ_CASE
    return false;
}

}  // namespace sq
