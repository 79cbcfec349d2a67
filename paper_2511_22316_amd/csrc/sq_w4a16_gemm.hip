// sq_w4a16_gemm: fp16 activations times 4-bit weight codes on the fp16 matrix cores of gfx950, with
// the per-output-channel step applied in the epilogue -- the weight-only setting of the paper's
// appendix (weight-only quantization table): Eq. 1 with only the weight operand quantized, the
// weight operand being Flat(W~_R) = W^T R of Sec. 4.2, one K-contiguous row of codes per channel.
//
//   Y[t, n] = fp16( sw[n] * sum_k X[t, k] * Qw[n, k] )        fp32 accumulation
//
// Three kernels: a tile kernel for many tokens (w4a16_gemm_ring_kernel) and two decode-shaped ones,
// for at most 32 tokens (w4a16_gemm_skinny_kernel) and for at most 16 whose rows fit in LDS
// (w4a16_gemm_xlds_kernel).  All widen the codes to fp16 in registers, exactly, with the
// magic-number form described at the two widening functions below.
// sq_pack_w3 / sq_w3a16_gemm (W3A16 of the same table) live here too: the decode-shaped kernels
// with the codes in three bits each, expanded to nibbles in registers (w3_nibbles).
#include "sq_common.h"

#include <type_traits>

namespace sq {

namespace {

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

// eight codes of a dword as fp16, in the order 0 4 1 5 2 6 3 7.  With x = dword ^ 0x88888888 every
// nibble holds u = code + 8.  "x & 0x000F000F | 0x64006400" is the pair of halves (1024 + u_0,
// 1024 + u_4), and one packed subtraction of 1032 leaves the codes; "x & 0x00F000F0 | 0x64006400"
// is (1024 + 16 u_1, 1024 + 16 u_5), and one packed multiply-add with 1/16 and -72 leaves those
// codes, exactly (every intermediate is a small multiple of 1/16).  The upper two nibble pairs
// take the same two forms on x >> 8.  Ten instructions per dword; the and-or is written as the
// one three-operand instruction it is (its constants must come from registers in that form, which
// the compiler avoids by emitting two instructions).
// The other operand's 16-byte chunks are put into the same order (interleave_halves), which a dot
// product does not see.
// PLUS4: the nibbles already hold code + 4 (the 3-bit storage expanded by w3_nibbles below), so
// there is nothing to flip and the offsets are 1028 and 68.
template <bool PLUS4 = false>
__device__ __forceinline__ v8h widen_codes_f16(uint32_t w, uint32_t magic_vgpr)
{
    const uint32_t x = PLUS4 ? w : (w ^ 0x88888888u);
    const _Float16 off = PLUS4 ? (_Float16)-1028.f : (_Float16)-1032.f;
    const _Float16 off16 = PLUS4 ? (_Float16)-68.f : (_Float16)-72.f;
    const v2h sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f};
    const v2h bias = {off, off}, bias16 = {off16, off16};
    const uint32_t x8 = x >> 8;
    uint32_t h0, h1, h2, h3;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(h0) : "v"(x), "s"(0x000F000Fu), "v"(magic_vgpr));
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(h1) : "v"(x), "s"(0x00F000F0u), "v"(magic_vgpr));
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(h2) : "v"(x8), "s"(0x000F000Fu), "v"(magic_vgpr));
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(h3) : "v"(x8), "s"(0x00F000F0u), "v"(magic_vgpr));
    const v2h p0 = __builtin_bit_cast(v2h, h0) + bias;
    const v2h p1 = __builtin_bit_cast(v2h, h1) * sixteenth + bias16;
    const v2h p2 = __builtin_bit_cast(v2h, h2) + bias;
    const v2h p3 = __builtin_bit_cast(v2h, h3) * sixteenth + bias16;
    return v8h{p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
}

// 3-bit storage (sq_pack_w3): 32 codes are three dwords a0, a1, h.  Codes 8m .. 8m + 7 have their
// two low bits (of code + 4) at bits 4i + 2 (m % 2) of a[m / 2] and their high bit at bit 4i + m of
// h.  Returned: the dword whose nibble i holds code_{8m + i} + 4, i.e. the 4-bit layout the
// widening above takes.  Two to four instructions per eight codes.
template <int M>
__device__ __forceinline__ uint32_t w3_nibbles(uint32_t a0, uint32_t a1, uint32_t h)
{
    const uint32_t a = M < 2 ? a0 : a1;
    const uint32_t low = ((M & 1) ? (a >> 2) : a) & 0x33333333u;
    const uint32_t high = M == 0 ? (h << 2) : M == 1 ? (h << 1) : M == 2 ? h : (h >> 1);
    return low | (high & 0x44444444u);
}

// eight codes of a dword as fp16, in their own order.  Byte m of the dword (with every nibble
// holding code + 8) is copied into both halves of a dword; "& 0x00F0000F | 0x64006400" leaves
// 1024 + (code_2m + 8) in the low half and 1024 + 16 (code_2m+1 + 8) in the high half, and one
// packed multiply-add with (1, 1/16) and (-1032, -72) the two codes, exactly.  Thirteen
// instructions per dword: the and-or is written as the one three-operand instruction it is (its
// constants must come from registers in that form, which the compiler avoids by emitting two).
__device__ __forceinline__ v8h widen_codes_f16_in_order(uint32_t w, uint32_t magic_vgpr)
{
    const uint32_t x = w ^ 0x88888888u;
    const v2h scale = {(_Float16)1.f, (_Float16)0.0625f}, bias = {(_Float16)-1032.f, (_Float16)-72.f};
    v2h p[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const uint32_t sel = 0x0C000C00u | (uint32_t)m | ((uint32_t)m << 16);
        uint32_t h;
        asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(h) : "v"(__builtin_amdgcn_perm(0u, x, sel)), "s"(0x00F0000Fu), "v"(magic_vgpr));
        p[m] = __builtin_bit_cast(v2h, h) * scale + bias;
    }
    return v8h{p[0][0], p[0][1], p[1][0], p[1][1], p[2][0], p[2][1], p[3][0], p[3][1]};
}

__device__ __forceinline__ void dma_16_if(const void *gptr, uint32_t lds_addr, int a, int b)
{
    // 16 bytes per lane, global memory -> LDS at lds_addr + 16 lane, issued only if a < b (both
    // wave-uniform); the branch lives inside the assembly so that the loop body stays one block
    asm volatile("s_cmp_lt_i32 %2, %3\n\t"
                 "s_cbranch_scc0 .Lsq16_skip_%=\n\t"
                 "s_mov_b32 m0, %1\n\t"
                 "s_nop 0\n\t"
                 "global_load_lds_dwordx4 %0, off\n"
                 ".Lsq16_skip_%=:"
                 :
                 : "v"(gptr), "s"(lds_addr), "s"(a), "s"(b)
                 : "memory", "m0", "scc");
}

// Wait for a tile of the ring.  Behind it at most one more tile is in flight, if rem >= 1 (L loads
// per loading wave and tile, and loads complete in order): then L loads may stay outstanding, else
// none.  After that the wave's own LDS reads are drained and the waves meet.
template <int L>
__device__ __forceinline__ void wait_tile_then_barrier(int rem)
{
    static_assert(L > 0 && L < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%1)\n\t"
                 "s_cmp_ge_i32 %0, 1\n\t"
                 "s_cbranch_scc1 .Lsq16_landed_%=\n\t"
                 "s_waitcnt vmcnt(0)\n"
                 ".Lsq16_landed_%=:\n\t"
                 "s_waitcnt lgkmcnt(0)\n\t"
                 "s_barrier"
                 :
                 : "s"(rem), "n"(L)
                 : "memory", "scc");
}

// Tile kernel for many tokens.  Block tile (WM FM 32) tokens x (WN FN 32) channels, WM x WN waves
// of FM x FN fragments of 32 x 32; K walked in tiles of 64.  Both operands travel global -> LDS
// without passing registers (16 bytes per lane), through a ring of three stages, two tiles ahead,
// completion tracked by hand: activations as they are (rows of 128 bytes, the 16-byte chunks of a
// row XOR-swizzled by (row / 2) % 8), weight codes packed (rows of 32 bytes).  A wave widens the codes
// of its own channels in registers, in order, so the activations need no reordering; one dword
// makes the operand of FM MFMAs, which is why a wave's tile is tall (FM = 4: 128 tokens x 64
// channels, 13 VALU instructions per 4 MFMAs) rather than wide.  Within a K tile lane half g takes
// elements 32g .. 32g + 31 and step s the eight elements 32g + 8s ..: chunk 4g + s of an
// activation row, dword s of chunk g of a code row.
// The weights are the first MFMA operand, so the 32 x 32 accumulator has the token in the lane and
// the channel in the register: register e holds channel 8 (e / 4) + 4 (lane / 32) + e % 4, four
// runs of four consecutive channels.  Two runs are traded between the half-waves (one cross-half
// swap per dword) and every lane stores 16 contiguous bytes of a row of Y.
// BK: elements of K per tile (a tile row of activations is 2 BK bytes, of codes BK / 2); 64 is what
// is built (128 was measured: 2 % faster at 2048 tokens, 10 % slower at 8192, and its 256-byte rows
// would want another swizzle).
// LW > 0: LW more waves that only request the tiles and wait for them; the multiplying waves then
// issue no memory instruction inside the loop and meet the others at the barrier of each tile.
template <int WM, int WN, int FM, int FN, int OCC, int BK, int LW>
__global__ __launch_bounds__((WM * WN + LW) * kWave, OCC) void w4a16_gemm_ring_kernel(
    const __half *__restrict__ X, int64_t ldx, int T, int K, const uint8_t *__restrict__ Qw,
    const float *__restrict__ sw, int N, __half *__restrict__ Y, int64_t ldy, int tiles_m, int tiles_n,
    int vec_store)
{
    static_assert(BK == 64, "tiles of 64 elements of K");
    constexpr int NW = WM * WN, NS = 3, STEPS = BK / 16;     // waves; ring stages; MFMA steps per K tile
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
    constexpr int A_ROW = 2 * BK, B_ROW = BK / 2;            // bytes of a tile row
    constexpr int A_CPR = A_ROW / 16, B_CPR = B_ROW / 16;    // 16-byte chunks per row
    constexpr int A_RPL = 64 / A_CPR, B_RPL = 64 / B_CPR;    // rows filled by one wave-wide load
    constexpr int A_BYTES = BM * A_ROW, B_BYTES = BN * B_ROW, STAGE = A_BYTES + B_BYTES;
    constexpr int NL = LW > 0 ? LW : NW;                     // waves that share the loads of a tile
    constexpr int A_LOADS = BM / A_RPL / NL, B_LOADS = BN / B_RPL / NL;       // wave-wide loads per loading wave and tile
    constexpr int LOADS = A_LOADS + B_LOADS;
    static_assert((BM / A_RPL) % NL == 0 && (BN / B_RPL) % NL == 0, "loads must split evenly over the waves");
    extern __shared__ uint4 ring[];

    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const bool loader = LW > 0 && tid / kWave >= NW;
    const int wave = loader ? tid / kWave - NW : tid / kWave;    // a loading wave counts from 0 again
    const int l32 = lane & 31, g = lane >> 5;
    const int wm = wave / WN, wn = wave % WN;
    int bm, bn;
    {
        const int id = xcd_contiguous_id(blockIdx.x, tiles_m * tiles_n);
        constexpr int GM = 8;
        const int group = id / (GM * tiles_n), gm = min(GM, tiles_m - group * GM);
        const int in_group = id - group * GM * tiles_n;
        bm = group * GM + in_group % gm;
        bn = in_group / gm;
    }
    const int row0 = bm * BM, col0 = bn * BN, Kb = K / 2;

    // global -> LDS.  One wave-wide load fills 64 consecutive chunk slots: A_RPL rows of activations
    // (lane l lands in row l / A_CPR, physical chunk l % A_CPR, which holds the logical chunk
    // (l % A_CPR) ^ ((row / 2) % 8): sixteen consecutive rows, two per 256 bytes of the 64 banks, then
    // keep the same logical chunk in sixteen different bank groups) or B_RPL rows of codes.  Rows past the ends are clamped: their
    // products are never stored.
    const __half *a_src[A_LOADS];
    const uint8_t *b_src[B_LOADS];
#pragma unroll
    for (int u = 0; u < A_LOADS; ++u) {
        const int r = A_RPL * (wave + NL * u) + lane / A_CPR;
        a_src[u] = X + (int64_t)min(row0 + r, T - 1) * ldx + (((lane % A_CPR) ^ ((r >> 1) & 7)) * 8);
    }
#pragma unroll
    for (int u = 0; u < B_LOADS; ++u) {
        const int r = B_RPL * (wave + NL * u) + lane / B_CPR;
        b_src[u] = Qw + (int64_t)min(col0 + r, N - 1) * Kb + (lane % B_CPR) * 16;
    }
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4 *)ring;
    const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
    auto issue_tile = [&](int kt, int stage, int limit) {
        const uint32_t sa = lds_base + (uint32_t)stage * STAGE;
#pragma unroll
        for (int u = 0; u < A_LOADS; ++u) dma_16_if(a_src[u] + kt * BK, sa + (wave_u + NL * u) * 1024, kt, limit);
#pragma unroll
        for (int u = 0; u < B_LOADS; ++u)
            dma_16_if(b_src[u] + kt * (BK / 2), sa + A_BYTES + (wave_u + NL * u) * 1024, kt, limit);
    };

    v16f acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // LDS byte offsets of this lane's fragment chunks inside a stage: lane half g takes the elements
    // [g BK / 2, (g + 1) BK / 2) of a K tile, step s the eight elements 8 s .. of those
    int a_off[STEPS];
#pragma unroll
    for (int s = 0; s < STEPS; ++s)
        a_off[s] = (wm * FM * 32 + l32) * A_ROW + (((STEPS * g + s) ^ ((l32 >> 1) & 7)) * 16);
    const int b_off = A_BYTES + (wn * FN * 32 + l32) * B_ROW + g * (STEPS * 4);
    const char *lds = reinterpret_cast<const char *>(ring);

    uint32_t magic;                                    // 1024.0 in both halves, held in a vector register
    asm volatile("v_mov_b32 %0, 0x64006400" : "=v"(magic));
    const int ktiles = K / BK;
    if (LW == 0 || loader) {
        issue_tile(0, 0, ktiles);
        issue_tile(1, 1, ktiles);
    }
    int stage = 0;
    if constexpr (LW > 0) {
        if (loader) {
            // a loading wave: the waits and requests of the loop below and nothing else; it meets the
            // multiplying waves at each of the ktiles barriers of the kernel
            for (int kt = 0; kt < ktiles; ++kt) {
                wait_tile_then_barrier<LOADS>(ktiles - 1 - kt);
                issue_tile(kt + 2, stage == 0 ? 2 : stage - 1, ktiles);
                stage = stage == 2 ? 0 : stage + 1;
            }
            return;
        }
    }
    for (int kt = 0; kt < ktiles; ++kt) {
        // Tile kt has landed once only the loads of tile kt + 1 (if it exists) are outstanding.
        // Behind the barrier every wave's share of it is in LDS and nobody reads tile kt - 1 any
        // more, so that stage takes tile kt + 2.
        if constexpr (LW == 0) {
            wait_tile_then_barrier<LOADS>(ktiles - 1 - kt);
            issue_tile(kt + 2, stage == 0 ? 2 : stage - 1, ktiles);
        } else {
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        }
        const char *st = lds + stage * STAGE;
        uint32_t rb[FN][STEPS];                        // one dword of codes per step
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int c = 0; c < STEPS / 4; ++c) {
                const uint4 v = *reinterpret_cast<const uint4 *>(st + b_off + j * (32 * B_ROW) + 16 * c);
                rb[j][4 * c] = v.x, rb[j][4 * c + 1] = v.y, rb[j][4 * c + 2] = v.z, rb[j][4 * c + 3] = v.w;
            }
        v8h a[2][FM];
#pragma unroll
        for (int i = 0; i < FM; ++i) a[0][i] = *reinterpret_cast<const v8h *>(st + a_off[0] + i * (32 * A_ROW));
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            if (s + 1 < STEPS) {
#pragma unroll
                for (int i = 0; i < FM; ++i)
                    a[(s + 1) & 1][i] = *reinterpret_cast<const v8h *>(st + a_off[s + 1] + i * (32 * A_ROW));
            }
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const v8h b = widen_codes_f16_in_order(rb[j][s], magic);
#pragma unroll
                for (int i = 0; i < FM; ++i)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(b, a[s & 1][i], acc[i][j], 0, 0, 0);
            }
        }
        stage = stage == 2 ? 0 : stage + 1;
    }

    typedef uint32_t v2u __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int nf = col0 + (wn * FN + j) * 32;            // first channel of the fragment
        float swq[4][4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int r = 0; r < 4; ++r) swq[q][r] = sw[min(nf + 8 * q + 4 * g + r, N - 1)];
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const int t = row0 + (wm * FM + i) * 32 + l32;
            uint32_t run[4][2];                              // run q: channels 8q + 4g .. + 3 as two dwords
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const v2h pair = {(_Float16)__float2half_rn(acc[i][j][4 * q + 2 * h] * swq[q][2 * h]),
                                      (_Float16)__float2half_rn(acc[i][j][4 * q + 2 * h + 1] * swq[q][2 * h + 1])};
                    run[q][h] = __builtin_bit_cast(uint32_t, pair);
                }
#pragma unroll
            for (int q = 0; q < 4; q += 2) {
                // swap(a, b): result 0 = (a of lanes 0..31, b of lanes 0..31), result 1 = (a of lanes
                // 32..63, b of lanes 32..63).  With a = run q, b = run q + 1: the lower half-wave gets
                // both halves of run q (channels 8q .. 8q + 7), the upper one those of run q + 1.
                const v2u s0 = __builtin_amdgcn_permlane32_swap(run[q][0], run[q + 1][0], false, false);
                const v2u s1 = __builtin_amdgcn_permlane32_swap(run[q][1], run[q + 1][1], false, false);
                const uint32_t w[4] = {s0[0], s1[0], s0[1], s1[1]};
                const int n0 = nf + 8 * (q + g);
                if (t >= T || n0 >= N) continue;
                __half *dst = Y + (int64_t)t * ldy + n0;
                if (vec_store && n0 + 8 <= N) {
                    *reinterpret_cast<uint4 *>(dst) = uint4{w[0], w[1], w[2], w[3]};
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e)              // register-only: no addressable copy of the chunk
                        if (n0 + e < N) reinterpret_cast<uint16_t *>(dst)[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
                }
            }
        }
    }
}

template <int WM, int WN, int FM, int FN, int OCC, int BK, int LW = 0>
sq_status launch_w4a16_ring(const __half *X, int64_t ldx, int T, int K, const uint8_t *Qw, const float *sw, int N,
                            __half *Y, int64_t ldy, hipStream_t st)
{
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
    constexpr size_t lds = (size_t)3 * (BM * 2 * BK + BN * BK / 2);
    static_assert(lds <= (size_t)kMaxDynamicLds, "ring does not fit in LDS");
    auto kernel = w4a16_gemm_ring_kernel<WM, WN, FM, FN, OCC, BK, LW>;
    if ((K % BK) != 0) return SQ_ERR_SHAPE;
    if (!allow_large_lds(reinterpret_cast<const void *>(kernel))) return SQ_ERR_LAUNCH;
    const int tiles_m = (T + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int vec_store = (((uintptr_t)Y & 15) == 0 && (ldy % 8) == 0) ? 1 : 0;
    hipLaunchKernelGGL(kernel, dim3((unsigned)(tiles_m * tiles_n)), dim3((WM * WN + LW) * kWave), lds, st, X, ldx, T, K, Qw,
                       sw, N, Y, ldy, tiles_m, tiles_n, vec_store);
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
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
// W3: the codes come in the 3-bit storage, 24 bytes per lane and slice instead of 32.
template <int NS, int NW, bool W3 = false>
__global__ __launch_bounds__(NW *kWave) void w4a16_gemm_skinny_kernel(
    const __half *__restrict__ X, int64_t ldx, int T, int K, const uint8_t *__restrict__ Qw,
    const float *__restrict__ sw, int N, __half *__restrict__ Y, int64_t ldy)
{
    constexpr int BN = 16 * NS;
    static_assert(NW * NS * 4 * kWave * 4 <= 64 * 1024, "partial sums must fit in static LDS");
    __shared__ float red[NW][NS][4][kWave];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int l16 = lane & 15, q = lane >> 4;
    const int col0 = blockIdx.x * BN, t0 = blockIdx.y * 16;
    const int Kb = W3 ? 3 * (K / 8) : K / 2;                 // bytes of a row of codes
    constexpr int LANE_BYTES = W3 ? 24 : 32;                 // 64 codes
    constexpr int NLD = W3 ? 3 : 2;                          // loads per lane, channel block and slice
    typedef typename std::conditional<W3, uint2, uint4>::type CodeLoad;

    // rows past the ends are clamped: their products are never stored
    const __half *a_ptr = X + (int64_t)min(t0 + l16, T - 1) * ldx + q * 64;
    const uint8_t *b_ptr[NS];
#pragma unroll
    for (int j = 0; j < NS; ++j) b_ptr[j] = Qw + (int64_t)min(col0 + 16 * j + l16, N - 1) * Kb + q * LANE_BYTES;

    v4f acc[NS];
#pragma unroll
    for (int j = 0; j < NS; ++j) acc[j] = v4f{0.f, 0.f, 0.f, 0.f};

    uint4 ra[2][8];
    CodeLoad rb[2][NS][NLD];
    const int slices = K / 256;
#define SQ_W16_FETCH(BUF, S)                                                                         \
    do {                                                                                             \
        _Pragma("unroll") for (int j = 0; j < NS; ++j)                                               \
            _Pragma("unroll") for (int c = 0; c < NLD; ++c)                                          \
                rb[BUF][j][c] = *reinterpret_cast<const CodeLoad *>(b_ptr[j] + (S) * (4 * LANE_BYTES) + \
                                                                    (int)sizeof(CodeLoad) * c);     \
        _Pragma("unroll") for (int u = 0; u < 8; ++u)                                                \
            ra[BUF][u] = *reinterpret_cast<const uint4 *>(a_ptr + (S) * 256 + 8 * u);                \
    } while (0)
#define SQ_W16_MULTIPLY(BUF)                                                                         \
    do {                                                                                             \
        _Pragma("unroll") for (int c = 0; c < 2; ++c)                                                \
            _Pragma("unroll") for (int d = 0; d < 4; ++d) {                                          \
                const v8h a = __builtin_bit_cast(v8h, interleave_halves(ra[BUF][4 * c + d]));        \
                _Pragma("unroll") for (int j = 0; j < NS; ++j)                                       \
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, codes_of(rb[BUF][j], c, d), acc[j], 0, 0, 0); \
            }                                                                                        \
    } while (0)

    // codes 32c + 8d .. + 7 of the lane's 64 as fp16, in the order interleave_halves gives the tokens
    uint32_t magic;                                    // 1024.0 in both halves, held in a vector register
    asm volatile("v_mov_b32 %0, 0x64006400" : "=v"(magic));
    auto codes_of = [magic](const CodeLoad(&r)[NLD], int c, int d) -> v8h {
        if constexpr (W3) {
            // six dwords: (a0, a1, h) of codes 0 .. 31, then of codes 32 .. 63
            const uint32_t w[6] = {r[0].x, r[0].y, r[1].x, r[1].y, r[2].x, r[2].y};
            const uint32_t a0 = w[3 * c], a1 = w[3 * c + 1], h = w[3 * c + 2];
            const uint32_t n = d == 0 ? w3_nibbles<0>(a0, a1, h) : d == 1 ? w3_nibbles<1>(a0, a1, h)
                             : d == 2 ? w3_nibbles<2>(a0, a1, h) : w3_nibbles<3>(a0, a1, h);
            return widen_codes_f16<true>(n, magic);
        } else {
            const uint4 w4 = r[c];
            return widen_codes_f16(d == 0 ? w4.x : d == 1 ? w4.y : d == 2 ? w4.z : w4.w, magic);
        }
    };
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

template <int NS, int NW, bool W3 = false>
sq_status launch_w4a16_skinny(const __half *X, int64_t ldx, int T, int K, const uint8_t *Qw, const float *sw, int N,
                              __half *Y, int64_t ldy, hipStream_t st)
{
    hipLaunchKernelGGL((w4a16_gemm_skinny_kernel<NS, NW, W3>), dim3((unsigned)((N + 16 * NS - 1) / (16 * NS)), (unsigned)((T + 15) / 16)),
                       dim3(NW * kWave), 0, st, X, ldx, T, K, Qw, sw, N, Y, ldy);
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

// ---- at most 16 tokens whose rows fit in LDS, many channels ---------------------------------
// In the kernel above every workgroup fetches the token rows again for each slice (twice the
// bytes of its weight codes when 16-bit rows meet 4-bit codes), and the fewer channels a workgroup
// owns the more of that traffic there is.  Here a workgroup of eight waves copies the rows into
// LDS once (each 16-byte chunk already in the order the widened codes take) and every wave then
// works alone: it owns blocks of 16 channels over the whole of K, slice after slice, with the
// codes of the next D slices in flight in a ring of registers and the token chunks of the next
// slice read from LDS while this one is multiplied.  No wave waits for another after the copy:
// no partial sums, no barriers.
// One workgroup per CU (the rows take most of the LDS); block b belongs to workgroup b % grid,
// wave (b / grid) % 8.
constexpr int kXldsRowPad = 16;        // bytes; sixteen rows then start in sixteen different 16-byte bank groups
constexpr int kXldsWaves = 8;
// 16-byte chunks of the rows per thread, at most
constexpr int kXldsChunks = (kMaxDynamicLds / 16 + kXldsWaves * kWave - 1) / (kXldsWaves * kWave);

template <bool W3, int D>
__global__ __launch_bounds__(kXldsWaves *kWave) void w4a16_gemm_xlds_kernel(
    const __half *__restrict__ X, int64_t ldx, int T, int K, const uint8_t *__restrict__ Qw,
    const float *__restrict__ sw, int N, __half *__restrict__ Y, int64_t ldy)
{
    static_assert(D % 2 == 0, "the token chunks alternate between two register sets");
    constexpr int NT = kXldsWaves * kWave;
    extern __shared__ uint4 xlds_u4[];
    char *xs = reinterpret_cast<char *>(xlds_u4);
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int l16 = lane & 15, q = lane >> 4;
    const int stride = 2 * K + kXldsRowPad;
    const int Kb = W3 ? 3 * (K / 8) : K / 2;                 // bytes of a row of codes
    constexpr int NLD = W3 ? 3 : 2;                          // loads per lane and slice
    typedef typename std::conditional<W3, uint2, uint4>::type CodeLoad;
    const int slices = K / 256, nblocks = (N + 15) / 16;
    const int first = blockIdx.x + gridDim.x * wave, step = gridDim.x * kXldsWaves;
    const int my_blocks = first < nblocks ? (nblocks - first + step - 1) / step : 0;

    // A lane holds the channel l16 of a block and a quarter q of a slice, codes 64 q .. 64 q + 63:
    // bytes 32q .. 32q + 31 of the slice's 128, or, in the 3-bit storage, bytes 24q .. 24q + 23
    // of its 96.  (Reading 64 contiguous bytes of a row per load instruction instead, or even
    // 1 KB contiguous per instruction from a re-tiled copy, changed nothing: 32.8 / 32.0 us.)
    // The loads of a round of D slices are issued D slices ahead, into the registers the round
    // has just consumed; slices % D == 0 (the launcher sees to it), so a round never straddles two
    // blocks and the loop body has no branch: the compiler's count of outstanding loads stays
    // exact.  Behind the last round of the last block that same round is requested once more.
    CodeLoad rb[D][NLD];
    auto row_of = [&](int bi) { return Qw + (int64_t)min(16 * (int64_t)(first + bi * step) + l16, (int64_t)N - 1) * Kb; };
    auto issue = [&](CodeLoad(&r)[NLD], const uint8_t *row, int S) {
        if constexpr (W3) {
#pragma unroll
            for (int c = 0; c < 3; ++c) r[c] = *reinterpret_cast<const uint2 *>(row + S * 96 + 24 * q + 8 * c);
        } else {
#pragma unroll
            for (int c = 0; c < 2; ++c) r[c] = *reinterpret_cast<const uint4 *>(row + S * 128 + 32 * q + 16 * c);
        }
    };

    // The token rows are requested first, 16-byte chunk by chunk (at most kXldsChunks per thread:
    // what fits in LDS), then the first D slices of codes; loads complete in order, so the rows
    // can be written to LDS while the codes are still on their way.  All requests are
    // unconditional (clamped), which keeps the compiler's count of outstanding loads exact.
    const int chunks_per_row = K / 8, chunks = T * chunks_per_row;
    {
        uint4 xv[kXldsChunks];
#pragma unroll
        for (int u = 0; u < kXldsChunks; ++u) {
            const int j = min(tid + NT * u, chunks - 1);
            xv[u] = *reinterpret_cast<const uint4 *>(X + (int64_t)(j / chunks_per_row) * ldx + 8 * (j % chunks_per_row));
        }
        const uint8_t *row0 = row_of(0);             // a wave without blocks requests (and drops) a valid row
#pragma unroll
        for (int i = 0; i < D; ++i) issue(rb[i], row0, i);
#pragma unroll
        for (int u = 0; u < kXldsChunks; ++u) {
            const int j = tid + NT * u;
            if (j < chunks)
                *reinterpret_cast<uint4 *>(xs + (j / chunks_per_row) * stride + 16 * (j % chunks_per_row)) =
                    interleave_halves(xv[u]);
        }
    }
    __syncthreads();

    uint32_t magic;                                    // 1024.0 in both halves, held in a vector register
    asm volatile("v_mov_b32 %0, 0x64006400" : "=v"(magic));
    // this lane's token row (rows past T repeat the last one: their products are never stored)
    // and the offset of its first chunk inside a slice.  Chunk j of the lane's eight per slice:
    // codes 64 q + 8 j .. + 7 of the slice.
    const char *xa = xs + min(l16, T - 1) * stride + 128 * q;
    auto read_tokens = [&](v8h(&a)[8], int S) {
        const char *xi = xa + S * 512;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            a[j] = *reinterpret_cast<const v8h *>(xi + 16 * j);
    };
    v4f acc0, acc1;
    auto multiply = [&](const CodeLoad(&r)[NLD], const v8h(&a)[8]) {
        if constexpr (W3) {
            // (a0, a1, h) of codes 0 .. 31 and of codes 32 .. 63 of the lane's 64
            const uint32_t w[6] = {r[0].x, r[0].y, r[1].x, r[1].y, r[2].x, r[2].y};
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t a0 = w[3 * h], a1 = w[3 * h + 1], hb = w[3 * h + 2];
                const uint32_t nib[4] = {w3_nibbles<0>(a0, a1, hb), w3_nibbles<1>(a0, a1, hb),
                                         w3_nibbles<2>(a0, a1, hb), w3_nibbles<3>(a0, a1, hb)};
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    v4f &acc = (m & 1) ? acc1 : acc0;
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[4 * h + m], widen_codes_f16<true>(nib[m], magic), acc, 0, 0, 0);
                }
            }
        } else {
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const uint32_t w[4] = {r[c].x, r[c].y, r[c].z, r[c].w};
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    v4f &acc = (d & 1) ? acc1 : acc0;
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[4 * c + d], widen_codes_f16(w[d], magic), acc, 0, 0, 0);
                }
            }
        }
    };
    v8h ta[2][8];                                      // token chunks of this slice and of the next
    read_tokens(ta[0], 0);
    for (int bi = 0; bi < my_blocks; ++bi) {
        const int n = 16 * (first + bi * step) + l16;
        const float step_n = sw[min(n, N - 1)];
        const uint8_t *row = row_of(bi);
        const uint8_t *row_after = row_of(bi + 1 < my_blocks ? bi + 1 : bi);
        acc0 = v4f{0.f, 0.f, 0.f, 0.f};
        acc1 = v4f{0.f, 0.f, 0.f, 0.f};
        for (int S0 = 0; S0 < slices; S0 += D) {
            const bool wrap = S0 + D >= slices;            // the round D slices ahead opens the next block
            const uint8_t *row_n = wrap ? row_after : row;
            const int S_n = wrap ? (bi + 1 < my_blocks ? 0 : S0) : S0 + D;
#pragma unroll
            for (int i = 0; i < D; ++i) {
                // the slice after this one: behind the last slice of a block comes slice 0 again
                // (the token rows are the same for every block)
                read_tokens(ta[(i + 1) & 1], (i + 1 == D && wrap) ? 0 : S0 + i + 1);
                multiply(rb[i], ta[i & 1]);
                issue(rb[i], row_n, S_n + i);
                // keep the requests here, one slice behind another: collected at the end of the
                // round (where the scheduler puts them) they would all be waited for at once
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // 16 x 16 accumulator layout: lane holds channel l16, register r holds token 4 q + r
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const int t = 4 * q + r4;
            if (t < T && n < N) Y[(int64_t)t * ldy + n] = __float2half_rn((acc0[r4] + acc1[r4]) * step_n);
        }
    }
}

// T <= 16, K % 1024 == 0 (rounds of at least four slices), the rows fit: T (2K + 16) bytes of LDS.
template <bool W3>
sq_status launch_w4a16_xlds(const __half *X, int64_t ldx, int T, int K, const uint8_t *Qw, const float *sw, int N,
                            __half *Y, int64_t ldy, hipStream_t st)
{
    const int nblocks = (N + 15) / 16;
    const int grid = nblocks < 256 ? nblocks : 256;
    const size_t lds = (size_t)T * (2 * K + kXldsRowPad);
    // eight slices in flight per wave where the slices of a row come in eights (K % 2048 == 0), else four
    if ((K / 256) % 8 == 0) {
        auto kernel = w4a16_gemm_xlds_kernel<W3, 8>;
        if (!allow_large_lds(reinterpret_cast<const void *>(kernel))) return SQ_ERR_LAUNCH;
        hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(kXldsWaves * kWave), lds, st, X, ldx, T, K, Qw, sw, N, Y, ldy);
    } else {
        auto kernel = w4a16_gemm_xlds_kernel<W3, 4>;
        if (!allow_large_lds(reinterpret_cast<const void *>(kernel))) return SQ_ERR_LAUNCH;
        hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(kXldsWaves * kWave), lds, st, X, ldx, T, K, Qw, sw, N, Y, ldy);
    }
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

// does the kernel above take the shape?  Enough blocks of 16 channels that every CU gets several waves
inline bool w4a16_xlds_covers(int64_t T, int K, int N)
{
    return T <= 16 && (K % 1024) == 0 && T * (int64_t)(2 * K + kXldsRowPad) <= kMaxDynamicLds && N >= 16 * 256 * 4;
}

// Nibble codes [N, K/2] (two's complement, every code in [-4, 3]) -> 3-bit storage [N, 3K/8].
// One thread per 32 codes: 16 bytes in, 12 bytes out.  (nibble ^ 4) & 7 is code + 4.
__global__ __launch_bounds__(256) void pack_w3_kernel(const uint8_t *__restrict__ Qw, int64_t units,
                                                      uint32_t *__restrict__ Qw3)
{
    const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= units) return;
    const uint4 v = *reinterpret_cast<const uint4 *>(Qw + 16 * u);
    const uint32_t x0 = v.x ^ 0x44444444u, x1 = v.y ^ 0x44444444u, x2 = v.z ^ 0x44444444u, x3 = v.w ^ 0x44444444u;
    const uint32_t lo = 0x33333333u, hi = 0x44444444u;
    Qw3[3 * u + 0] = (x0 & lo) | ((x1 & lo) << 2);
    Qw3[3 * u + 1] = (x2 & lo) | ((x3 & lo) << 2);
    Qw3[3 * u + 2] = ((x0 & hi) >> 2) | ((x1 & hi) >> 1) | (x2 & hi) | ((x3 & hi) << 1);
}

}  // namespace

}  // namespace sq

extern "C" sq_status sq_pack_w3(const uint8_t *Qw, int32_t K, int32_t N, uint8_t *Qw3, void *stream)
{
    if (N < 0 || K <= 0 || (K % 64) != 0 || K > 131072) return SQ_ERR_SHAPE;
    if (N == 0) return SQ_OK;
    if (!Qw || !Qw3) return SQ_ERR_NULL;
    if (((uintptr_t)Qw & 15) || ((uintptr_t)Qw3 & 7)) return SQ_ERR_ALIGN;
    const int64_t units = (int64_t)N * (K / 32);
    hipLaunchKernelGGL(sq::pack_w3_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), Qw, units, reinterpret_cast<uint32_t *>(Qw3));
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

extern "C" sq_status sq_w3a16_gemm(const void *X, int64_t T, int32_t K, int64_t ldx, const uint8_t *Qw3,
                                   const float *sw, int32_t N, void *Y, int64_t ldy, void *stream)
{
    if (T < 0 || N < 0 || K <= 0 || (K % 256) != 0 || K > 131072) return SQ_ERR_SHAPE;
    if (T > SQ_W3A16_MAX_ROWS || ldx < K || ldy < N) return SQ_ERR_SHAPE;       // 16 tokens per grid row
    if (T == 0 || N == 0) return SQ_OK;
    if (!X || !Qw3 || !sw || !Y) return SQ_ERR_NULL;
    if (((uintptr_t)X & 15) || (ldx % 8) != 0 || ((uintptr_t)Qw3 & 7) || ((uintptr_t)Y & 1) || ((uintptr_t)sw & 3))
        return SQ_ERR_ALIGN;
    const hipStream_t s0 = static_cast<hipStream_t>(stream);
    const __half *X0 = static_cast<const __half *>(X);
    if (sq::w4a16_xlds_covers(T, K, N))
        return sq::launch_w4a16_xlds<true>(X0, ldx, (int)T, K, Qw3, sw, N, static_cast<__half *>(Y), ldy, s0);
    if (N >= 64 * 384) return sq::launch_w4a16_skinny<4, 4, true>(X0, ldx, (int)T, K, Qw3, sw, N, static_cast<__half *>(Y), ldy, s0);
    return sq::launch_w4a16_skinny<2, 8, true>(X0, ldx, (int)T, K, Qw3, sw, N, static_cast<__half *>(Y), ldy, s0);
}

extern "C" sq_status sq_w4a16_gemm(const void *X, int64_t T, int32_t K, int64_t ldx, const uint8_t *Qw,
                                   const float *sw, int32_t N, void *Y, int64_t ldy, void *stream)
{
    if (T < 0 || N < 0 || K <= 0 || (K % 64) != 0 || K > 131072) return SQ_ERR_SHAPE;
    if (T > (1 << 24) || ldx < K || ldy < N) return SQ_ERR_SHAPE;
    if (T == 0 || N == 0) return SQ_OK;
    if (!X || !Qw || !sw || !Y) return SQ_ERR_NULL;
    if (((uintptr_t)X & 15) || (ldx % 8) != 0 || ((uintptr_t)Qw & 15) || ((uintptr_t)Y & 1) || ((uintptr_t)sw & 3))
        return SQ_ERR_ALIGN;
    // At most 32 tokens: one pass over the weights (two token blocks above 16 tokens read them twice,
    // the second time mostly out of the caches; beyond that the tile kernel is the better choice).
    // Launch shapes as in the W4A4 decode-shaped kernel: about eight waves on every CU.
    if (T <= 32 && (K % 256) == 0 && sq::debug_option(SQ_DEBUG_W4A16_LAUNCH_SHAPE) == 0) {
        const hipStream_t s0 = static_cast<hipStream_t>(stream);
        const __half *X0 = static_cast<const __half *>(X);
        if (sq::w4a16_xlds_covers(T, K, N))
            return sq::launch_w4a16_xlds<false>(X0, ldx, (int)T, K, Qw, sw, N, static_cast<__half *>(Y), ldy, s0);
        if (N >= 64 * 384) return sq::launch_w4a16_skinny<4, 4>(X0, ldx, (int)T, K, Qw, sw, N, static_cast<__half *>(Y), ldy, s0);
        return sq::launch_w4a16_skinny<2, 8>(X0, ldx, (int)T, K, Qw, sw, N, static_cast<__half *>(Y), ldy, s0);
    }
    // Many tokens: 256 x 256 tiles (eight waves) when there are enough of them to fill the CUs, else
    // 128 x 256 tiles (four multiplying waves and four loading waves: with the loads in the multiplying
    // waves this tile took 69.1 instead of 67.2 us on 2048 x 4096 x 4096 and 177 instead of 165 us at
    // K = 11008).
    const hipStream_t st = static_cast<hipStream_t>(stream);
    const __half *Xh = static_cast<const __half *>(X);
    __half *Yh = static_cast<__half *>(Y);
    const int shape = sq::debug_option(SQ_DEBUG_W4A16_LAUNCH_SHAPE);
    const int64_t tiles_large = ((T + 255) / 256) * ((N + 255) / 256);
    if (shape == 2 || (shape != 1 && tiles_large >= 192))
        return sq::launch_w4a16_ring<2, 4, 4, 2, 1, 64>(Xh, ldx, (int)T, K, Qw, sw, N, Yh, ldy, st);
    return sq::launch_w4a16_ring<1, 4, 4, 2, 1, 64, 4>(Xh, ldx, (int)T, K, Qw, sw, N, Yh, ldy, st);
}
