// sq_w4a16_gemm: fp16 activations times 4-bit weight codes on the fp16 matrix cores of gfx950, with
// the per-output-channel step applied in the epilogue -- the weight-only setting of the paper's
// appendix (weight-only quantization table): Eq. 1 with only the weight operand quantized, the
// weight operand being Flat(W~_R) = W^T R of Sec. 4.2, one K-contiguous row of codes per channel.
//
//   Y[t, n] = fp16( sw[n] * sum_k X[t, k] * Qw[n, k] )        fp32 accumulation
//
// Two kernels: a tile kernel for many tokens (w4a16_gemm_ring_kernel) and a decode-shaped one for
// at most 32 (w4a16_gemm_skinny_kernel).  Both widen the codes to fp16 in registers, exactly, with
// the magic-number form described at the two widening functions below.
#include "sq_common.h"

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

// eight codes of a dword as fp16, in the order 0 4 1 5 2 6 3 7: with x = dword ^ 0x88888888 every
// nibble holds code + 8, "(x >> 4j) & 0x000F000F | 0x64006400" is the pair of halves
// (1024 + code_j + 8, 1024 + code_{j+4} + 8), and one packed subtraction of 1032 leaves the codes.
// The other operand's 16-byte chunks are put into the same order (interleave_halves), which a dot
// product does not see.
__device__ __forceinline__ v8h widen_codes_f16(uint32_t w)
{
    const uint32_t x = w ^ 0x88888888u;
    const v2h bias = {(_Float16)1032.f, (_Float16)1032.f};
    v2h p[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        p[j] = __builtin_bit_cast(v2h, ((x >> (4 * j)) & 0x000F000Fu) | 0x64006400u) - bias;
    return v8h{p[0][0], p[0][1], p[1][0], p[1][1], p[2][0], p[2][1], p[3][0], p[3][1]};
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
template <int NS, int NW>
__global__ __launch_bounds__(NW *kWave) void w4a16_gemm_skinny_kernel(
    const __half *__restrict__ X, int64_t ldx, int T, int K, const uint8_t *__restrict__ Qw,
    const float *__restrict__ sw, int N, __half *__restrict__ Y, int64_t ldy)
{
    constexpr int BN = 16 * NS;
    static_assert(NW * NS * 4 * kWave * 4 <= 64 * 1024, "partial sums must fit in static LDS");
    __shared__ float red[NW][NS][4][kWave];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int l16 = lane & 15, q = lane >> 4;
    const int col0 = blockIdx.x * BN, t0 = blockIdx.y * 16, Kb = K / 2;

    // rows past the ends are clamped: their products are never stored
    const __half *a_ptr = X + (int64_t)min(t0 + l16, T - 1) * ldx + q * 64;
    const uint8_t *b_ptr[NS];
#pragma unroll
    for (int j = 0; j < NS; ++j) b_ptr[j] = Qw + (int64_t)min(col0 + 16 * j + l16, N - 1) * Kb + q * 32;

    v4f acc[NS];
#pragma unroll
    for (int j = 0; j < NS; ++j) acc[j] = v4f{0.f, 0.f, 0.f, 0.f};

    uint4 ra[2][8], rb[2][NS][2];
    const int slices = K / 256;
#define SQ_W16_FETCH(BUF, S)                                                                         \
    do {                                                                                             \
        _Pragma("unroll") for (int j = 0; j < NS; ++j)                                               \
            _Pragma("unroll") for (int c = 0; c < 2; ++c)                                            \
                rb[BUF][j][c] = *reinterpret_cast<const uint4 *>(b_ptr[j] + (S) * 128 + 16 * c);     \
        _Pragma("unroll") for (int u = 0; u < 8; ++u)                                                \
            ra[BUF][u] = *reinterpret_cast<const uint4 *>(a_ptr + (S) * 256 + 8 * u);                \
    } while (0)
#define SQ_W16_MULTIPLY(BUF)                                                                         \
    do {                                                                                             \
        _Pragma("unroll") for (int c = 0; c < 2; ++c)                                                \
            _Pragma("unroll") for (int d = 0; d < 4; ++d) {                                          \
                const v8h a = __builtin_bit_cast(v8h, interleave_halves(ra[BUF][4 * c + d]));        \
                _Pragma("unroll") for (int j = 0; j < NS; ++j) {                                     \
                    const uint4 w4 = rb[BUF][j][c];                                                  \
                    const uint32_t w = d == 0 ? w4.x : d == 1 ? w4.y : d == 2 ? w4.z : w4.w;         \
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, widen_codes_f16(w), acc[j], 0, 0, 0); \
                }                                                                                    \
            }                                                                                        \
    } while (0)

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

template <int NS, int NW>
sq_status launch_w4a16_skinny(const __half *X, int64_t ldx, int T, int K, const uint8_t *Qw, const float *sw, int N,
                              __half *Y, int64_t ldy, hipStream_t st)
{
    hipLaunchKernelGGL((w4a16_gemm_skinny_kernel<NS, NW>), dim3((unsigned)((N + 16 * NS - 1) / (16 * NS)), (unsigned)((T + 15) / 16)),
                       dim3(NW * kWave), 0, st, X, ldx, T, K, Qw, sw, N, Y, ldy);
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

}  // namespace

}  // namespace sq

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
