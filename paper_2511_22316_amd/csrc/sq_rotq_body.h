// Body of the matrix-core rotate + quantize kernel (see sq_rotq_mfma.hip for the description of the
// method) as a device function, so that a kernel which does more than this step can run it too.
#pragma once

#include "sq_common.h"
#include "sq_rotq_plan.h"

#include <type_traits>

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

// max(m, |a[0]|, ..., |a[15]|), as four independent chains of two steps each (one long chain of
// dependent maxima costs a wave its issue latency sixteen times over)
__device__ __forceinline__ float max_abs16(const v16f &a, float m)
{
    float c[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        c[k] = fmaxf(fabsf(a[4 * k]), fmaxf(fabsf(a[4 * k + 1]), fabsf(a[4 * k + 2])));
        c[k] = fmaxf(c[k], fabsf(a[4 * k + 3]));
    }
    return fmaxf(fmaxf(m, c[0]), fmaxf(fmaxf(c[1], c[2]), c[3]));
}

}  // namespace

// NSX_: token tiles per ring (3: two rows ahead of the one being multiplied; 2: one row ahead,
// with less LDS so that a third workgroup fits a CU)
// R1LDS_: the stage-B operand fragments of R1 live in LDS, one copy shared by the four waves,
// instead of in every wave's registers (frees 8 MB^2 registers per lane)
template <int N1, int N2, int NSX_, bool R1LDS_ = false>
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
    static constexpr int NSX = NSX_;              // ring of token tiles
    static constexpr int TILE_BYTES = N1P * N2 * 2;
    static constexpr int LO_STEP_BYTES = N1P * 32;        // side tile: [step][row p][16 fp16]
    static constexpr int OFF_X = 0;                                   // [TPP][NSX][TILE]
    static constexpr int OFF_R1F = TPP * NSX * TILE_BYTES;            // [MB][KSB][64 lanes][16 bytes]
    // R1's fragments pass through LDS whenever one wave per column block can build them for all
    // (up to four column blocks): to stay there (R1LDS_) or to be copied into every wave's registers
    static constexpr bool R1_SHARED = R1LDS_ || MB <= 2;
    static constexpr int R1F_BYTES = R1_SHARED ? MB * KSB * 1024 : 0;
    static constexpr int OFF_LO = OFF_R1F + R1F_BYTES;                // [TPP][side tiles][qsteps][LO_STEP]
    // after the side tiles (runtime size): [TPP][128] float, [2][TPP][4] float
    static constexpr int TAIL_BYTES = TPP * (kRotqMaxSlots * 4 + 32);
    // sides: side tiles per token slot, 2 (they alternate from token to token, one barrier per
    // token) or 1 (less LDS, a second barrier per token)
    static constexpr int lds_bytes(int qsteps, int sides)
    {
        return OFF_LO + TPP * sides * qsteps * LO_STEP_BYTES + TAIL_BYTES;
    }
    // two side tiles per token slot unless they would cost a workgroup its place on the CU (occ:
    // workgroups per CU that the registers allow) or do not fit at all
    static constexpr int side_tiles(int qsteps, int occ)
    {
        const int l1 = lds_bytes(qsteps, 1), l2 = lds_bytes(qsteps, 2);
        const int per_cu_1 = (160 * 1024) / l1 < occ ? (160 * 1024) / l1 : occ;
        const int per_cu_2 = (160 * 1024) / l2 < occ ? (160 * 1024) / l2 : occ;
        return (l2 <= kMaxDynamicLds && per_cu_2 >= per_cu_1) ? 2 : 1;
    }
    static_assert(N2 == 32 || N2 == 64 || N2 == 128, "one to four waves per token");
    static_assert(NSX == 2 || NSX == 3, "ring of two or three tiles");
    static_assert(N1P <= 128, "at most four row blocks");
    // two rows are in flight at most; at 64 outstanding loads the counter is full and the issue
    // of the last one simply waits
    static_assert(2 * LPT <= 64, "outstanding loads must fit the vmcnt counter");
};

// QS_MAX: repair steps of 16 q-slots each the kernel holds rotation rows for (4 or 8).
// PREPARED: R1 and R2 point at the operand fragments written by rotation_fragments_kernel.
// F16OUT: no quantizer; the rotated row leaves as fp16 (round to nearest even) in xout [T, ldo]
// (the 16-bit activations of the weight-only setting), and Q, scales, xrot are not touched.
// g0, stride: the workgroup takes token groups g0, g0 + stride, ... (a kernel of its own passes its
// block index and grid size); smem_u4: the workgroup's dynamic LDS, RotqShape::lds_bytes() of it;
// sides: side tiles per token slot (RotqShape::side_tiles).
// CLIP: the quantizer has a clipping ratio below one (plan.clip): entries beyond the end levels
// are clamped to them.  Without it nothing can lie beyond them and the clamp is not compiled in.
template <int N1, int N2, int QS_MAX, int NSX_, bool R1LDS, bool PREPARED, bool F16OUT = false, bool CLIP = false>
__device__ __forceinline__ void rotate_quantize_mfma_body(
    const __half *__restrict__ X, int64_t ldx, int T, const RotqPlan &plan,
    const __half *__restrict__ R1, const __half *__restrict__ R2, uint8_t *__restrict__ Q,
    float *__restrict__ scales, float *__restrict__ xrot, const int g0, const int stride, uint4 *smem_u4,
    const int sides, __half *__restrict__ xout = nullptr, int64_t ldo = 0)
{
    using S = RotqShape<N1, N2, NSX_, R1LDS>;
    constexpr bool prepared = PREPARED;
    constexpr int N1P = S::N1P, MB = S::MB, NCB = S::NCB, TPP = S::TPP, KSA = S::KSA, KSB = S::KSB;
    constexpr int CPRX = S::CPRX, LPT = S::LPT, NSX = S::NSX, K = N1 * N2;
    static_assert(QS_MAX == 4 || QS_MAX == 8, "64 or 128 q-slots");
    char *lds = reinterpret_cast<char *>(smem_u4);
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4 *)smem_u4;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tok_slot = wave / NCB, cb = wave % NCB;        // which token of the pass, which columns
    const int l32 = lane & 31, g = lane >> 5;
    // The waves of a token take turns as the owner of its rows: the owner of row r (the r-th row this
    // workgroup handles for the token slot) requests it from memory and later applies the Givens
    // list to it.  A fixed owner would have about twice the work of the others -- the row requests
    // cost a wave some tens of ns each to issue, the list several LDS round trips -- and, being
    // wave 0 of every workgroup, would share one SIMD with the owners of the CU's other workgroups
    // while the other three SIMDs wait at the barrier.
    auto owns = [&](int r) { return cb == r % NCB; };
    const bool lead = owns(0);                               // owner of the first row: the prologue's extra work

    // Every scalar argument the kernel will need is fetched here, in one batch.  Left to the
    // compiler, each is loaded in front of its first use, and the prologue waits for five scalar
    // memory round trips one after the other (two of them in front of the first loads of R1 / R2).
    const int n_slots = plan.n_slots, n_levels = plan.n_levels, n_qslots = plan.n_qslots;
    asm volatile("" ::"s"(X), "s"(ldx), "s"(T), "s"(n_slots), "s"(n_levels), "s"(n_qslots), "s"(R1), "s"(R2),
                 "s"(Q), "s"(scales), "s"(xrot), "s"(stride));

    const int qsteps = (n_qslots + 15) / 16;                 // extra MFMA steps that repair the Givens rounding
    const int lo_bytes = qsteps * S::LO_STEP_BYTES;          // one side tile; every token slot has two
    const int off_gv = S::OFF_LO + TPP * sides * lo_bytes;
    const int side_mask = sides - 1;                         // 1: the two tiles alternate, 0: one tile
    const int off_red = off_gv + TPP * kRotqMaxSlots * 4;    // [2][TPP][4] floats

    const int groups = (T + TPP - 1) / TPP;
    // does this wave's token exist in group grp (the last group may be partial)?
    auto has_row = [&](int grp) { return (int64_t)grp * TPP + tok_slot < T; };
    // a row's owner: all loads of its token row of group `grp` into ring slot `slot`
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

    // ---- prologue -------------------------------------------------------------------------
    // Memory latencies are overlapped in this order: the first token row leaves for LDS, then the
    // plan entries of this lane and the rotation blocks are requested, and only when those have
    // been consumed do rows two and three follow (loads complete in order, so anything issued
    // before the blocks would have to land before them).
    if (lead) issue_row(g0, 0);

    // This lane's plan entries are requested now and used after the rotation blocks are built.
    // Lane l owns pair l of the level-sorted Givens list (its slots, angle and level) and two of
    // the touched channels (slots l and l + 64) for the gather / scatter around the list.
    // The first Givens pass below relies on these loads being issued after the row request above
    // (loads complete in order, so the row has landed once they have).  Their index therefore
    // carries a zero that exists only after that request: volatile statements keep their order,
    // and the loads cannot move ahead of a value they depend on.
    int after_row_request;
    asm volatile("v_mov_b32 %0, 0" : "=v"(after_row_request));
    const int pl = lane + after_row_request;
    const int my_level_raw = plan.pair_level[pl];
    const int my_si = plan.pair_i[pl], my_sj = plan.pair_j[pl];
    const float my_c = plan.c[pl], my_s = plan.s[pl];
    const int my_chan[2] = {plan.chan[pl], plan.chan[pl + 64]};
    const int my_qslot[2] = {plan.qslot[pl], plan.qslot[pl + 64]};

    // R2 (stage A, operand B): lane holds column q' = 32cb + l32, step ks, element e <-> row
    // q = 16ks + 8g + e.  R1 (stage B, operand B): lane holds column p' = 32nb + l32; step ks,
    // element e <-> row p = 16ks + 8(e/4) + 4g + e%4, which is where stage A leaves row p of Z in
    // this lane.
    //
    // Both are columns of a row-major matrix, which a lane cannot fetch with wide loads.  The
    // matrix cores transpose instead: a 32x32 block of R is loaded as operand A (lane = row,
    // eight consecutive columns = 16 contiguous bytes) and multiplied by slices of the identity,
    // which is exact; the product arrives in the accumulator layout (lane = column, registers =
    // rows 8(e/4) + 4g + e%4).  That is the row order stage B wants.  Stage A wants rows 8g + e
    // per step, which is the same order with bits 2 and 3 of the row swapped, so the lanes of
    // operand A fetch their rows in that swapped order.
    // declared here, filled in once the plan entries have arrived
    int my_level = -1, gs_tile[2] = {-1, -1}, gs_lo[2] = {0, 0};

    // a row's owner: Givens list on the tile in ring slot `slot`; fills side tile `side` (0 / 1: the two
    // alternate from token to token, so that the list of the token after next can be applied while
    // stage A of the next one may still be reading its side tile)
    auto givens = [&](int slot, int side) {
        if (n_slots == 0) return;
        char *xt = lds + S::OFF_X + (tok_slot * NSX + slot) * S::TILE_BYTES;
        char *lo_t = lds + S::OFF_LO + (tok_slot * sides + (side & side_mask)) * lo_bytes;
        float *gv = reinterpret_cast<float *>(lds + off_gv) + tok_slot * kRotqMaxSlots;
#pragma unroll
        for (int u = 0; u < 2; ++u)
            if (gs_tile[u] >= 0) gv[lane + 64 * u] = __half2float(*reinterpret_cast<const __half *>(xt + gs_tile[u]));
        for (int lv = 0; lv < n_levels; ++lv) {
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

    v8h r2f[KSA], r2x[QS_MAX], r1f[R1LDS ? 1 : MB][R1LDS ? 1 : KSB];
    static_assert(!R1LDS || MB <= 4, "one wave per column block of R1 builds the shared fragments");
    // The fragments of R1 are the same for every wave.  Fetched by each wave for itself they are
    // two thirds of all the prologue's loads (64 x 64 at 2048 tokens: 10.2 us with them, 8.9 us when
    // a timing-only build fetched one fragment instead of eight), so wave nb fetches (and, from a
    // row-major R1, transposes) column block nb alone and hands it to the others through LDS: to
    // stay there (R1LDS) or, with at most two row blocks, to be copied into every wave's registers.
    constexpr bool R1_SHARED = S::R1_SHARED;
    {
        v8h sel[2];                       // identity slices: B[k][n] = (16kk + k == n), k = 8g + e
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int e = 0; e < 8; ++e) sel[kk][e] = (16 * kk + 8 * g + e == l32) ? (_Float16)1.f : (_Float16)0.f;
        // All loads are unconditional (clamped addresses, zeros selected afterwards) and the code
        // is free of branches, so the requests leave together and one memory round trip covers
        // them all.
        // Elements BASE + 8g .. +7 of a row of NC columns as a 16-byte load.  A chunk that reaches
        // past the end of the row is fetched from NC-8 and shifted down; the elements behind the
        // end are zero.
        auto chunk = [&](const __half *row, auto base_c, auto nc_c) {
            constexpr int BASE = decltype(base_c)::value, NC = decltype(nc_c)::value;
            static_assert(NC >= 8, "a row holds at least one chunk");
            constexpr int COL0 = BASE < NC - 8 ? BASE : NC - 8, COL1 = BASE + 8 < NC - 8 ? BASE + 8 : NC - 8;
            constexpr int OVER0 = BASE - COL0 > 8 ? 8 : BASE - COL0;           // elements to shift out
            constexpr int OVER1 = BASE + 8 - COL1 > 8 ? 8 : BASE + 8 - COL1;
            const int col = g ? COL1 : COL0;
            const v8h v = *reinterpret_cast<const v8h *>(__builtin_assume_aligned(row + col, 4));
            if constexpr (OVER0 == 0 && OVER1 == 0) {
                return v;
            } else {
                v8h lo_g, hi_g;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    lo_g[e] = (e + OVER0 < 8) ? v[(e + OVER0) & 7] : (_Float16)0.f;
                    hi_g[e] = (e + OVER1 < 8) ? v[(e + OVER1) & 7] : (_Float16)0.f;
                }
                return g ? hi_g : lo_g;
            }
        };
        auto zero_unless = [&](bool keep, const v8h v) {
            const v4u w = __builtin_bit_cast(v4u, v);
            const v4u z = {keep ? w[0] : 0u, keep ? w[1] : 0u, keep ? w[2] : 0u, keep ? w[3] : 0u};
            return __builtin_bit_cast(v8h, z);
        };
        // 32 rows x 32 columns -> accumulator layout
        auto block_t = [&](const v8h a0, const v8h a1) {
            v16f c;
#pragma unroll
            for (int e = 0; e < 16; ++e) c[e] = 0.f;
            c = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, sel[0], c, 0, 0, 0);
            return __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, sel[1], c, 0, 0, 0);
        };
        auto to_frag = [&](const v16f &c, int s) {      // registers 8s .. 8s+7, exact in fp16
            v4u w;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                w[e] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(c[8 * s + 2 * e], c[8 * s + 2 * e + 1]));
            return __builtin_bit_cast(v8h, w);
        };
        const int lsw = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
        const __half *r2col = R2 + 32 * cb;
        using C0 = std::integral_constant<int, 0>;
        using C16 = std::integral_constant<int, 16>;
        using CN2 = std::integral_constant<int, N2>;
        using CN1 = std::integral_constant<int, N1>;
        // Up to three row blocks, all of R1 is requested at once.  With four, that would not fit
        // the registers: the blocks of column block nb + 1 are requested while those of nb are
        // transposed, in two alternating sets.
        constexpr int RAW1_SETS = R1_SHARED ? 1 : (MB <= 3 ? MB : 2);
        v8h raw2[N2 / 32][2], raw1[RAW1_SETS][MB][2];
        auto load_raw1 = [&](int nb, v8h (&dst)[MB][2]) {
#pragma unroll
            for (int blk = 0; blk < MB; ++blk) {
                const __half *row = R1 + min(32 * blk + l32, N1 - 1) * N1;
                if (nb == 0) {
                    dst[blk][0] = chunk(row, std::integral_constant<int, 0>{}, CN1{});
                    dst[blk][1] = chunk(row, std::integral_constant<int, 16>{}, CN1{});
                } else if (nb == 1) {
                    dst[blk][0] = chunk(row, std::integral_constant<int, 32>{}, CN1{});
                    dst[blk][1] = chunk(row, std::integral_constant<int, 48>{}, CN1{});
                } else if (nb == 2) {
                    dst[blk][0] = chunk(row, std::integral_constant<int, 64>{}, CN1{});
                    dst[blk][1] = chunk(row, std::integral_constant<int, 80>{}, CN1{});
                } else {
                    dst[blk][0] = chunk(row, std::integral_constant<int, 96>{}, CN1{});
                    dst[blk][1] = chunk(row, std::integral_constant<int, 112>{}, CN1{});
                }
            }
        };
        int qrow[QS_MAX / 2];             // row of R2 that q-slot 32xb + lsw repairs, -1 behind the end
#pragma unroll
        for (int xb = 0; xb < QS_MAX / 2; ++xb) qrow[xb] = plan.qlist[32 * xb + lsw];
        // shared fragments: wave nb fetches (and later transposes) column block nb of R1
        const int wave_s = __builtin_amdgcn_readfirstlane(wave);
        if constexpr (prepared) {
            // R1 and R2 point at the operand fragments themselves, stored lane by lane (see
            // rotation_fragments_kernel): 16 contiguous bytes per lane, whole lines per wave.  Row
            // gathers like the ones below cost a wave about 80 ns of issue time each.
            const v8h *f2 = reinterpret_cast<const v8h *>(R2) + (cb * KSA) * kWave + lane;
#pragma unroll
            for (int ks = 0; ks < KSA; ++ks) r2f[ks] = f2[ks * kWave];
            const v8h *f1 = reinterpret_cast<const v8h *>(R1) + lane;
            if constexpr (R1_SHARED) {
                if (wave_s < MB) {
#pragma unroll
                    for (int blk = 0; blk < MB; ++blk) {
                        raw1[0][blk][0] = f1[(wave_s * KSB + 2 * blk) * kWave];
                        raw1[0][blk][1] = f1[(wave_s * KSB + 2 * blk + 1) * kWave];
                    }
                }
            } else {
#pragma unroll
                for (int nb = 0; nb < MB; ++nb)
#pragma unroll
                    for (int ks = 0; ks < KSB; ++ks) r1f[nb][ks] = f1[(nb * KSB + ks) * kWave];
            }
        } else {
#pragma unroll
            for (int blk = 0; blk < N2 / 32; ++blk) {
                raw2[blk][0] = chunk(r2col + (32 * blk + lsw) * N2, C0{}, CN2{});
                raw2[blk][1] = chunk(r2col + (32 * blk + lsw) * N2, C16{}, CN2{});
            }
            if constexpr (R1_SHARED) {
                if (wave_s < MB) load_raw1(wave_s, raw1[0]);
            } else {
#pragma unroll
                for (int nb = 0; nb < (MB <= 3 ? MB : 1); ++nb) load_raw1(nb, raw1[nb]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);              // every request is out before the first use
        // While those requests are in flight: zeros where nothing is ever loaded, then the lead wave
        // rotates the first row.  Row one was requested before the plan entries and loads complete in
        // order, so it has landed once the entries are here.  The barrier is the bare instruction:
        // the fence of __syncthreads would wait for every load above.  (Zeros: padding rows p >= N1
        // of every ring tile, and the side tiles.)
        if (N1P > N1) {
            constexpr int PAD_CHUNKS = (N1P - N1) * CPRX;
            for (int c = tid; c < TPP * NSX * PAD_CHUNKS; c += 256) {
                const int tile = c / PAD_CHUNKS, r = c % PAD_CHUNKS;
                *reinterpret_cast<uint4 *>(lds + S::OFF_X + tile * S::TILE_BYTES + (N1 * CPRX + r) * 16) = uint4{0, 0, 0, 0};
            }
        }
        for (int c = tid; c < TPP * sides * lo_bytes / 16; c += 256)
            *reinterpret_cast<uint4 *>(lds + S::OFF_LO + c * 16) = uint4{0, 0, 0, 0};

        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        my_level = (my_level_raw == 0xFF) ? -1 : my_level_raw;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int p = my_chan[u] / N2, q = my_chan[u] % N2, qs = my_qslot[u];
            gs_tile[u] = (lane + 64 * u < n_slots) ? (p * CPRX + ((q >> 3) ^ swz<CPRX>(p))) * 16 + (q & 7) * 2 : -1;
            gs_lo[u] = (qs >> 4) * S::LO_STEP_BYTES + p * 32 + (qs & 15) * 2;
        }
        if (lead) givens(0, 0);
        if constexpr (!prepared) {
#pragma unroll
            for (int blk = 0; blk < N2 / 32; ++blk) {
                const v16f c = block_t(raw2[blk][0], raw2[blk][1]);
                r2f[2 * blk] = to_frag(c, 0);
                r2f[2 * blk + 1] = to_frag(c, 1);
            }
        }
        if constexpr (R1_SHARED) {
            // visible to the other waves after the barrier that precedes the first stage A
            if (wave_s < MB) {
                v8h *dst = reinterpret_cast<v8h *>(lds + S::OFF_R1F) + (wave_s * KSB) * kWave + lane;
#pragma unroll
                for (int blk = 0; blk < MB; ++blk) {
                    if constexpr (prepared) {
                        dst[(2 * blk) * kWave] = raw1[0][blk][0];
                        dst[(2 * blk + 1) * kWave] = raw1[0][blk][1];
                    } else {
                        const bool keep = 32 * blk + l32 < N1;
                        const v16f c = block_t(zero_unless(keep, raw1[0][blk][0]), zero_unless(keep, raw1[0][blk][1]));
                        dst[(2 * blk) * kWave] = to_frag(c, 0);
                        dst[(2 * blk + 1) * kWave] = to_frag(c, 1);
                    }
                }
            }
        } else if constexpr (!prepared) {
#pragma unroll
            for (int nb = 0; nb < MB; ++nb) {
                constexpr bool ALTERNATE = MB > 3;
                const int set = ALTERNATE ? (nb & 1) : nb;
                if (ALTERNATE && nb + 1 < MB) load_raw1(nb + 1, raw1[(nb + 1) & 1]);
#pragma unroll
                for (int blk = 0; blk < MB; ++blk) {
                    const bool keep = 32 * blk + l32 < N1;
                    const v16f c = block_t(zero_unless(keep, raw1[set][blk][0]), zero_unless(keep, raw1[set][blk][1]));
                    r1f[nb][2 * blk] = to_frag(c, 0);
                    r1f[nb][2 * blk + 1] = to_frag(c, 1);
                }
            }
        }
        // The rows of R2 that repair the Givens rounding (one per q-slot) are picked out of the
        // blocks just built, again on the matrix cores and again exactly: operand A holds a single
        // 1 per row, at column qlist[slot], and operand B is R2 as stage A uses it.  This saves
        // a second trip to memory behind the plan entries.
#pragma unroll
        for (int xb = 0; xb < QS_MAX / 2; ++xb) {
            if (32 * xb < n_qslots) {
                const int q = (32 * xb + lsw < n_qslots) ? qrow[xb] : -1;
                v16f c;
#pragma unroll
                for (int e = 0; e < 16; ++e) c[e] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KSA; ++ks) {
                    const int d = q - 16 * ks - 8 * g;          // element of this lane's eight that is 1
                    const uint32_t one = ((uint32_t)d < 8u) ? (0x3C00u << (16 * (d & 1))) : 0u;
                    const v4u a = {(d >> 1) == 0 ? one : 0u, (d >> 1) == 1 ? one : 0u,
                                   (d >> 1) == 2 ? one : 0u, (d >> 1) == 3 ? one : 0u};
                    c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), r2f[ks], c, 0, 0, 0);
                }
                r2x[2 * xb] = to_frag(c, 0);
                r2x[2 * xb + 1] = to_frag(c, 1);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) r2x[2 * xb][e] = r2x[2 * xb + 1][e] = (_Float16)0.f;
            }
        }
    }

    if (owns(1)) issue_row(g0 + stride, 1);
    if (NSX == 3 && owns(2)) issue_row(g0 + 2 * stride, 2);

    // LDS byte offsets of this lane's operand chunks inside a tile (row block 0): the swizzle
    // only touches the low bits of the chunk index, so four offsets cover every step
    constexpr int NJ = KSA < 4 ? KSA : 4;
    int a_off[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) a_off[j] = (l32 * CPRX + ((2 * j + g) ^ swz<CPRX>(l32))) * 16;
    const int lo_off = (l32 * 2 + g) * 16;

    // stage A of the token in ring slot `slot` (and its side tile); after MFMA m, `between(m)` is
    // issued (quantization units of the previous token, or nothing)
    v16f accz[MB], accy[MB];
    constexpr int NMA = MB * KSA;
    auto stage_a = [&](int slot, int side, auto between) {
        const char *xt = lds + S::OFF_X + (tok_slot * NSX + slot) * S::TILE_BYTES;
        auto a_at = [&](int m) {
            const int mb = m / KSA, ks = m % KSA;
            return *reinterpret_cast<const v8h *>(xt + a_off[ks % 4] + (ks / 4) * 128 + mb * (32 * CPRX * 16));
        };
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int e = 0; e < 16; ++e) accz[mb][e] = 0.f;
        v8h a0 = a_at(0), a1 = a_at(NMA > 1 ? 1 : 0);
#pragma unroll
        for (int m = 0; m < NMA; ++m) {
            // operand reads run two MFMAs ahead (four ahead measured 2-4 % slower on every shape)
            const v8h a2 = a_at(m + 2 < NMA ? m + 2 : NMA - 1);
            accz[m / KSA] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, r2f[m % KSA], accz[m / KSA], 0, 0, 0);
            between(m);
            __builtin_amdgcn_sched_barrier(0);
            a0 = a1;
            a1 = a2;
        }
        const char *lo_t = lds + S::OFF_LO + (tok_slot * sides + (side & side_mask)) * lo_bytes;
#pragma unroll
        for (int x = 0; x < QS_MAX; ++x) {
            if (x < qsteps) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    const v8h a = *reinterpret_cast<const v8h *>(lo_t + x * S::LO_STEP_BYTES + mb * 1024 + lo_off);
                    accz[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, r2x[x], accz[mb], 0, 0, 0);
                }
            }
        }
    };

    // ---- pipeline prologue: first row rotated, its stage A done -------------------------------
    __syncthreads();                       // first row rotated; the fragments of R1 are in LDS
    if constexpr (R1_SHARED && !R1LDS) {
        const v8h *r1s0 = reinterpret_cast<const v8h *>(lds + S::OFF_R1F) + lane;
#pragma unroll
        for (int nb = 0; nb < MB; ++nb)
#pragma unroll
            for (int ks = 0; ks < KSB; ++ks) r1f[nb][ks] = r1s0[(nb * KSB + ks) * kWave];
    }
    stage_a(0, 0, [](int) {});
    if (sides == 1) __syncthreads();       // the one side tile is rewritten in the first iteration

    // Barriers per token: one (B2), behind which the token maximum, the rotated next tile and its
    // side tile are visible.  Nothing else is shared between waves: codes leave from registers, and
    // what a wave writes ahead of B2 of one iteration (its maximum, the owner's side tile) goes
    // into the copy that nobody can still be reading, because the two copies alternate from token
    // to token and every wave has passed the previous B2 since the last use.  With a ring of two
    // tiles a second barrier per token (B3) protects the tile that is refilled right behind it,
    // and with a single side tile per token slot (very long lists on the largest shapes) the
    // side tile that the next list overwrites.
    int slot = 0, par = 0;                 // ring slot and parity (side tile, maxima) of the current token
    int it = 0;                            // rows of this token slot done so far: the current row's number
    for (int grp = g0; grp < groups; grp += stride, ++it) {
        const int t = grp * TPP + tok_slot;
        const bool live = t < T;
        const int slot1 = (slot + 1 == NSX) ? 0 : slot + 1;
        // ring of two: the tile of this token went through stage A an iteration ago (every wave
        // has passed the barrier that ended it), so the row after next can start now
        if (NSX == 2 && owns(it + 2)) issue_row(grp + 2 * stride, slot);

        // ---- power-of-two prescale of this wave's columns so that hi/lo fit fp16 -------------
        // Stage B contracts over rows p within a column, so a per-wave factor commutes with it.
        float zmax = 0.f;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) zmax = max_abs16(accz[mb], zmax);
        zmax = wave_max(zmax);
        float fz_inv = 1.0f;                     // Z * fz in [2^13, 2^14) at its largest entry
        if (!(zmax >= 1.0f && zmax < 16384.0f) && zmax > 0.f) {
            const int ez = (int)((__float_as_uint(zmax) >> 23) & 0xFF) - 127;
            const int sh = max(-100, min(100, 13 - ez));
            const float fz = __uint_as_float((uint32_t)(127 + sh) << 23);
            fz_inv = __uint_as_float((uint32_t)(127 - sh) << 23);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int e = 0; e < 16; ++e) accz[mb][e] *= fz;
        }

        // ---- stage B: Y^T = Z^T R1, Z = hi + lo; the split of step ks+1 is issued between the
        // MFMAs of step ks -----------------------------------------------------------------
#pragma unroll
        for (int nb = 0; nb < MB; ++nb)
#pragma unroll
            for (int e = 0; e < 16; ++e) accy[nb][e] = 0.f;
        v4u zh, zl, zh_n, zl_n;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint32_t hi, lo;
            split_pair(accz[0][2 * e], accz[0][2 * e + 1], hi, lo);
            zh[e] = hi;
            zl[e] = lo;
        }
        // shared fragments of R1: those of step ks + 1 are read while step ks is multiplied
        const v8h *r1s = reinterpret_cast<const v8h *>(lds + S::OFF_R1F) + lane;
        v8h rb[R1LDS ? MB : 1], rb_n[R1LDS ? MB : 1];
        if constexpr (R1LDS) {
#pragma unroll
            for (int nb = 0; nb < MB; ++nb) rb[nb] = r1s[(nb * KSB) * kWave];
        }
#pragma unroll
        for (int ks = 0; ks < KSB; ++ks) {
            const v8h zhv = __builtin_bit_cast(v8h, zh), zlv = __builtin_bit_cast(v8h, zl);
            constexpr int NMB = 2 * MB;          // MFMAs of this step
#pragma unroll
            for (int j = 0; j < (NMB > 4 ? NMB : 4); ++j) {
                if constexpr (R1LDS) {
                    if (j < NMB && (j & 1) == 0 && ks + 1 < KSB) rb_n[j / 2] = r1s[((j / 2) * KSB + ks + 1) * kWave];
                    if (j < NMB)
                        accy[j / 2] = __builtin_amdgcn_mfma_f32_32x32x16_f16((j & 1) ? zlv : zhv, rb[j / 2], accy[j / 2], 0, 0, 0);
                } else {
                    if (j < NMB)
                        accy[j / 2] = __builtin_amdgcn_mfma_f32_32x32x16_f16((j & 1) ? zlv : zhv, r1f[j / 2][ks], accy[j / 2], 0, 0, 0);
                }
                if (ks + 1 < KSB) {
                    // pairs of the next step: 4 pairs spread over the MFMAs (all after the last if fewer)
                    const int per = (4 + NMB - 1) / NMB;
#pragma unroll
                    for (int e = j * per; e < (j + 1) * per && e < 4; ++e) {
                        if (j < NMB || true) {
                            const int ks1 = ks + 1, mb1 = ks1 >> 1, r1 = 8 * (ks1 & 1);
                            uint32_t hi, lo;
                            split_pair(accz[mb1][r1 + 2 * e], accz[mb1][r1 + 2 * e + 1], hi, lo);
                            zh_n[e] = hi;
                            zl_n[e] = lo;
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            zh = zh_n;
            zl = zl_n;
            if constexpr (R1LDS) {
#pragma unroll
                for (int nb = 0; nb < MB; ++nb) rb[nb] = rb_n[nb];
            }
        }

        // ---- per-token step: wave maximum now, token maximum after the barrier --------------
        float amax = 0.f;
        float *red = reinterpret_cast<float *>(lds + off_red) + (par * TPP + tok_slot) * 4;
        if constexpr (!F16OUT) {
#pragma unroll
            for (int nb = 0; nb < MB; ++nb) amax = max_abs16(accy[nb], amax);
            amax = wave_max(amax) * fz_inv;    // padded rows and columns of Y are exact zeros
            if (lane == 0) red[cb] = amax;
        }

        // ---- owner of the next row: the row has landed -> rotate its touched channels.  With one
        // wave per token the owner also requested the row after it, which may still be in flight
        // (rows complete in order); with turns, every other request of this wave is older.
        if (owns(it + 1)) {
            if (NCB == 1 && has_row(grp + 2 * stride)) wait_loads_le<LPT>();
            else wait_loads_le<0>();
            if (has_row(grp + stride)) givens(slot1, par ^ 1);
        }
        __syncthreads();     // B2: maxima visible; next tile and its side tile rotated
        // stage A of this token ran an iteration ago, so its ring slot is free for the row after next
        if (NSX == 3 && owns(it + 3)) issue_row(grp + 3 * stride, slot);

        float inv = fz_inv;                    // F16OUT: Y = accy * fz_inv
        if constexpr (!F16OUT) {
            amax = red[0];
#pragma unroll
            for (int w = 1; w < NCB; ++w) amax = fmaxf(amax, red[w]);
            const float step = (amax == 0.f) ? 1.0f : amax / plan.q_div;      // q_div = 7: max|Y| / 7
            inv = fz_inv / step;               // codes = Y / step with Y = accy * fz_inv
            if (live && cb == 0 && lane == 0) scales[t] = step;
        }
        if (!F16OUT && xrot != nullptr && live) {
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

        if constexpr (!F16OUT && CLIP) {
            // With a clipping ratio below one, entries beyond the end levels are pulled back to
            // values that round to those levels (-q_top - 1 and q_top), so that the conversion
            // below keeps its range; without clipping |Y / step| <= q_top and nothing need be done.
            const float unit = 1.0f / inv;           // the accumulator value of one step
            const float lo = -(plan.q_top + 1.0f) * unit, hi = (plan.q_top + 0.25f) * unit;
#pragma unroll
            for (int nb = 0; nb < MB; ++nb)
#pragma unroll
                for (int e = 0; e < 16; ++e) accy[nb][e] = fminf(fmaxf(accy[nb][e], lo), hi);
        }

        // ---- codes of this token, issued between the stage-A MFMAs of the next one ------------
        // A lane holds column p' = 32nb + l32 of Y^T and, per register group rg, four consecutive
        // q' = 32cb + 8rg + 4g + (0..3): one 2-byte unit of the code row; the eight units (rg, g) of
        // a row p' are 16 contiguous bytes of Q.  The two half-waves trade units (one cross-half
        // swap per pair) so that lanes g = 0 end up with the eight bytes of rg = 0, 1 and lanes
        // g = 1 with those of rg = 2, 3, and the wave stores 32 row pieces of 16 bytes with one
        // 8-byte store per lane, straight from registers.
        constexpr int NU = 4 * MB;               // quantization units of 4 codes
        uint32_t unit[4];                        // the four units of the row block being quantized
        auto quant_unit = [&](int u) {
            const int nb = u / 4, rg = u % 4;
            if constexpr (F16OUT) {
                // four consecutive q' of row p' = 32nb + l32 as one 8-byte store
                const int po = 32 * nb + l32;
                const v2h lo2 = {(_Float16)(accy[nb][4 * rg] * inv), (_Float16)(accy[nb][4 * rg + 1] * inv)};
                const v2h hi2 = {(_Float16)(accy[nb][4 * rg + 2] * inv), (_Float16)(accy[nb][4 * rg + 3] * inv)};
                if (live && po < N1)
                    *reinterpret_cast<uint2 *>(xout + (int64_t)t * ldo + po * N2 + 32 * cb + 8 * rg + 4 * g) =
                        uint2{__builtin_bit_cast(uint32_t, lo2), __builtin_bit_cast(uint32_t, hi2)};
                return;
            }
            uint32_t w = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                // floor(v + 1/2) + 8 = trunc(v + 8.5) for v in [-8, 7.5); two's-complement nibble = that ^ 8
                const uint32_t c = (uint32_t)fmaf(accy[nb][4 * rg + k], inv, 8.5f);
                w |= c << (4 * k);
            }
            unit[rg] = w;
            if (rg == 3) {
                // swap(a, b): result 0 = (a of lanes 0..31, b of lanes 0..31), result 1 = (a of lanes
                // 32..63, b of lanes 32..63).  With a = unit rg, b = unit rg + 2: lanes g = 0 get both
                // halves (g = 0 low, g = 1 high) of unit rg, lanes g = 1 those of unit rg + 2.
                typedef uint32_t v2u __attribute__((ext_vector_type(2)));
                const v2u s02 = __builtin_amdgcn_permlane32_swap(unit[0], unit[2], false, false);
                const v2u s13 = __builtin_amdgcn_permlane32_swap(unit[1], unit[3], false, false);
                const uint32_t d0 = (s02[0] | (s02[1] << 16)) ^ 0x88888888u;     // rg = 0 (g = 0) or 2 (g = 1)
                const uint32_t d1 = (s13[0] | (s13[1] << 16)) ^ 0x88888888u;     // rg = 1 (g = 0) or 3 (g = 1)
                const int po = 32 * nb + l32;
                if (live && po < N1)
                    *reinterpret_cast<uint2 *>(Q + (int64_t)t * (K / 2) + po * (N2 / 2) + 16 * cb + 8 * g) = uint2{d0, d1};
            }
        };
        stage_a(slot1, par ^ 1, [&](int m) {
            // NU units spread over the NMA MFMAs
#pragma unroll
            for (int u = 0; u < NU; ++u)
                if (u * NMA / NU == m) quant_unit(u);
        });
        if (NSX == 2 || sides == 1) __syncthreads();     // B3: every wave is done with the tile / side tile rewritten next
        slot = slot1;
        par ^= 1;
    }
    wait_loads_le<0>();
}

}  // namespace sq
