// sq_w4a16_gemm: fp16 activations times 4-bit weight codes on the fp16 matrix cores of gfx950, with
// the per-output-channel step applied in the epilogue -- the weight-only setting of the paper's
// appendix (weight-only quantization table): Eq. 1 with only the weight operand quantized, the
// weight operand being Flat(W~_R) = W^T R of Sec. 4.2, one K-contiguous row of codes per channel.
//
//   Y[t, n] = fp16( sw[n] * sum_k X[t, k] * Qw[n, k] )        fp32 accumulation
//
// Codes are widened to fp16 in registers: with x = dword ^ 0x88888888 every nibble holds code + 8,
// "(x >> 4j) & 0x000F000F | 0x64006400" is the pair of halves (1024 + code_j + 8, 1024 + code_{j+4} + 8),
// and one packed subtraction of 1032 leaves the codes themselves, exactly.  A dword therefore
// yields its eight codes in the order 0 4 1 5 2 6 3 7; the activations of a 16-byte chunk are put
// into the same order, which a dot product does not see.  Both happen once per element, on the way
// into LDS (every tile row is read by two waves afterwards): the loop over a tile is then LDS reads
// and MFMAs only.
#include "sq_common.h"

namespace sq {

namespace {

constexpr int kBM = 128, kBN = 128, kBK = 64;      // block tile and codes per K tile
constexpr int kXRow = kBK * 2, kWRow = kBK / 2;    // bytes of a tile row in memory: activations, weight codes

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

// eight codes of a dword as fp16, in the order 0 4 1 5 2 6 3 7
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

// Block tile 128 x 128, four waves of 64 x 64 (2 x 2 fragments of 32 x 32), K walked in tiles of 64
// codes.  Tiles travel global -> registers -> LDS (activations reordered, codes widened to fp16 on
// the way), the next tile's loads in flight while this one is multiplied; two LDS buffers, one
// barrier per tile.  Both operands sit in LDS as rows of eight 16-byte chunks (eight fp16 values
// each), chunk c of row r at slot r * 8 + (c ^ (r & 7)).  Within a K tile lane half g takes codes
// 32g .. 32g + 31 and step s the eight codes 32g + 8s ..: chunk 4g + s of its row, for both operands.
__global__ __launch_bounds__(256, 2) void w4a16_gemm_kernel(
    const __half *__restrict__ X, int64_t ldx, int T, int K, const uint8_t *__restrict__ Qw,
    const float *__restrict__ sw, int N, __half *__restrict__ Y, int64_t ldy, int tiles_m, int tiles_n)
{
    __shared__ uint4 xs[2][kBM * 8];               // activations
    __shared__ uint4 ws[2][kBN * 8];               // weight codes as fp16

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int l32 = lane & 31, g = lane >> 5, wm = wave >> 1, wn = wave & 1;
    // XCD-contiguous tile ids, column-major inside groups of 8 row tiles: the tiles resident on one
    // XCD share a few row and column panels in its L2
    int bm, bn;
    {
        const int id = xcd_contiguous_id(blockIdx.x, tiles_m * tiles_n);
        constexpr int GM = 8;
        const int group = id / (GM * tiles_n), gm = min(GM, tiles_m - group * GM);
        const int in_group = id - group * GM * tiles_n;
        bm = group * GM + in_group % gm;
        bn = in_group / gm;
    }
    const int row0 = bm * kBM, col0 = bn * kBN, Kb = K / 2;

    // this thread's share of a tile: four activation chunks, one weight chunk (rows past the ends
    // are clamped: their products are never stored)
    const __half *x_src[4];
    int x_slot[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int c = tid + 256 * u, r = c >> 3, ch = c & 7;
        x_src[u] = X + (int64_t)min(row0 + r, T - 1) * ldx + ch * 8;
        x_slot[u] = r * 8 + (ch ^ (r & 7));
    }
    const uint8_t *w_src = Qw + (int64_t)min(col0 + (tid >> 1), N - 1) * Kb + (tid & 1) * 16;
    // the 32 codes of this thread's weight chunk become chunks 4 (tid & 1) .. + 3 of row tid >> 1
    int w_slot[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) w_slot[u] = (tid >> 1) * 8 + ((4 * (tid & 1) + u) ^ ((tid >> 1) & 7));

    v16f acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    uint4 xr[4], wr;
    auto fetch = [&](int kt) {
#pragma unroll
        for (int u = 0; u < 4; ++u) xr[u] = *reinterpret_cast<const uint4 *>(x_src[u] + kt * kBK);
        wr = *reinterpret_cast<const uint4 *>(w_src + kt * kWRow);
    };
    auto park = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 4; ++u) xs[buf][x_slot[u]] = interleave_halves(xr[u]);
        const uint32_t wd[4] = {wr.x, wr.y, wr.z, wr.w};
#pragma unroll
        for (int u = 0; u < 4; ++u) ws[buf][w_slot[u]] = __builtin_bit_cast(uint4, widen_codes_f16(wd[u]));
    };

    const int ktiles = K / kBK;
    fetch(0);
    park(0);
    __syncthreads();
    for (int kt = 0; kt < ktiles; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < ktiles) fetch(kt + 1);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            v8h a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int r = wm * 64 + 32 * i + l32;
                a[i] = __builtin_bit_cast(v8h, xs[buf][r * 8 + ((4 * g + s) ^ (r & 7))]);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int r = wn * 64 + 32 * j + l32;
                b[j] = __builtin_bit_cast(v8h, ws[buf][r * 8 + ((4 * g + s) ^ (r & 7))]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < ktiles) park(buf ^ 1);
        __syncthreads();
    }

    // 32 x 32 accumulator layout: lane holds channel l32, register e holds token 8 (e / 4) + 4 g + e % 4
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int n = col0 + wn * 64 + 32 * j + l32;
        if (n >= N) continue;
        const float step = sw[n];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int t = row0 + wm * 64 + 32 * i + 8 * (e / 4) + 4 * g + (e % 4);
                if (t < T) Y[(int64_t)t * ldy + n] = __float2half_rn(acc[i][j][e] * step);
            }
    }
}

// eight codes of a dword as fp16, in their own order.  Byte m of the dword (with every nibble
// holding code + 8) is copied into both halves of a dword; "& 0x00F0000F | 0x64006400" leaves
// 1024 + (code_2m + 8) in the low half and 1024 + 16 (code_2m+1 + 8) in the high half, and one
// packed multiply-add with (1, 1/16) and (-1032, -72) the two codes, exactly.
__device__ __forceinline__ v8h widen_codes_f16_in_order(uint32_t w)
{
    const uint32_t x = w ^ 0x88888888u;
    const v2h scale = {(_Float16)1.f, (_Float16)0.0625f}, bias = {(_Float16)-1032.f, (_Float16)-72.f};
    v2h p[4];
    p[0] = __builtin_bit_cast(v2h, (__builtin_amdgcn_perm(0u, x, 0x0C000C00u) & 0x00F0000Fu) | 0x64006400u) * scale + bias;
    p[1] = __builtin_bit_cast(v2h, (__builtin_amdgcn_perm(0u, x, 0x0C010C01u) & 0x00F0000Fu) | 0x64006400u) * scale + bias;
    p[2] = __builtin_bit_cast(v2h, (__builtin_amdgcn_perm(0u, x, 0x0C020C02u) & 0x00F0000Fu) | 0x64006400u) * scale + bias;
    p[3] = __builtin_bit_cast(v2h, (__builtin_amdgcn_perm(0u, x, 0x0C030C03u) & 0x00F0000Fu) | 0x64006400u) * scale + bias;
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

// the tile that must have landed is followed by `rem` more tiles in flight at most one of which
// may still be outstanding (L loads per wave and tile, in order); then the waves meet
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
// row XOR-swizzled by row % 8), weight codes packed (rows of 32 bytes).  A wave widens the codes
// of its own channels in registers, in order, so the activations need no reordering; one dword
// makes the operand of FM MFMAs, which is why a wave's tile is tall (FM = 4: 128 tokens x 64
// channels, 13 VALU instructions per 4 MFMAs) rather than wide.  Within a K tile lane half g takes
// elements 32g .. 32g + 31 and step s the eight elements 32g + 8s ..: chunk 4g + s of an
// activation row, dword s of chunk g of a code row.
// The weights are the first MFMA operand, so the 32 x 32 accumulator has the token in the lane and
// the channel in the register: register e holds channel 8 (e / 4) + 4 (lane / 32) + e % 4, four
// runs of four consecutive channels.  Two runs are traded between the half-waves (one cross-half
// swap per dword) and every lane stores 16 contiguous bytes of a row of Y.
template <int WM, int WN, int FM, int FN, int OCC>
__global__ __launch_bounds__(WM *WN *kWave, OCC) void w4a16_gemm_ring_kernel(
    const __half *__restrict__ X, int64_t ldx, int T, int K, const uint8_t *__restrict__ Qw,
    const float *__restrict__ sw, int N, __half *__restrict__ Y, int64_t ldy, int tiles_m, int tiles_n,
    int vec_store)
{
    constexpr int NW = WM * WN, NS = 3;
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
    constexpr int A_ROW = 128, B_ROW = 32;                   // bytes of a tile row
    constexpr int A_BYTES = BM * A_ROW, B_BYTES = BN * B_ROW, STAGE = A_BYTES + B_BYTES;
    constexpr int A_LOADS = BM / 8 / NW, B_LOADS = BN / 32 / NW;       // wave-wide loads per wave and tile
    constexpr int LOADS = A_LOADS + B_LOADS;
    static_assert((BM / 8) % NW == 0 && (BN / 32) % NW == 0, "loads must split evenly over the waves");
    extern __shared__ uint4 ring[];

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int l32 = lane & 31, g = lane >> 5, wm = wave / WN, wn = wave % WN;
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

    // global -> LDS.  Activations: one wave-wide load fills 8 rows x 8 chunks; lane l lands in row
    // l / 8, physical chunk l % 8, which holds the logical chunk (l % 8) ^ (row % 8).  Codes: 32 rows
    // x 2 chunks.  Rows past the ends are clamped: their products are never stored.
    const __half *a_src[A_LOADS];
    const uint8_t *b_src[B_LOADS];
#pragma unroll
    for (int u = 0; u < A_LOADS; ++u) {
        const int r = 8 * (wave + NW * u) + lane / 8;
        a_src[u] = X + (int64_t)min(row0 + r, T - 1) * ldx + (((lane & 7) ^ (r & 7)) * 8);
    }
#pragma unroll
    for (int u = 0; u < B_LOADS; ++u) {
        const int r = 32 * (wave + NW * u) + lane / 2;
        b_src[u] = Qw + (int64_t)min(col0 + r, N - 1) * Kb + (lane & 1) * 16;
    }
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4 *)ring;
    const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
    auto issue_tile = [&](int kt, int stage, int limit) {
        const uint32_t sa = lds_base + (uint32_t)stage * STAGE;
#pragma unroll
        for (int u = 0; u < A_LOADS; ++u) dma_16_if(a_src[u] + kt * 64, sa + (wave_u + NW * u) * 1024, kt, limit);
#pragma unroll
        for (int u = 0; u < B_LOADS; ++u)
            dma_16_if(b_src[u] + kt * 32, sa + A_BYTES + (wave_u + NW * u) * 1024, kt, limit);
    };

    v16f acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // LDS byte offsets of this lane's fragment chunks inside a stage
    int a_off[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) a_off[s] = (wm * FM * 32 + l32) * A_ROW + (((4 * g + s) ^ (l32 & 7)) * 16);
    const int b_off = A_BYTES + (wn * FN * 32 + l32) * B_ROW + g * 16;
    const char *lds = reinterpret_cast<const char *>(ring);

    const int ktiles = K / 64;
    issue_tile(0, 0, ktiles);
    issue_tile(1, 1, ktiles);
    int stage = 0;
    for (int kt = 0; kt < ktiles; ++kt) {
        // Tile kt has landed once only the loads of tile kt + 1 (if it exists) are outstanding.
        // Behind the barrier every wave's share of it is in LDS and nobody reads tile kt - 1 any
        // more, so that stage takes tile kt + 2.
        wait_tile_then_barrier<LOADS>(ktiles - 1 - kt);
        issue_tile(kt + 2, stage == 0 ? 2 : stage - 1, ktiles);
        const char *st = lds + stage * STAGE;
        uint4 rb[FN];
#pragma unroll
        for (int j = 0; j < FN; ++j) rb[j] = *reinterpret_cast<const uint4 *>(st + b_off + j * (32 * B_ROW));
        v8h a[2][FM];
#pragma unroll
        for (int i = 0; i < FM; ++i) a[0][i] = *reinterpret_cast<const v8h *>(st + a_off[0] + i * (32 * A_ROW));
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (s + 1 < 4) {
#pragma unroll
                for (int i = 0; i < FM; ++i)
                    a[(s + 1) & 1][i] = *reinterpret_cast<const v8h *>(st + a_off[s + 1] + i * (32 * A_ROW));
            }
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const uint32_t w = s == 0 ? rb[j].x : s == 1 ? rb[j].y : s == 2 ? rb[j].z : rb[j].w;
                const v8h b = widen_codes_f16_in_order(w);
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

template <int WM, int WN, int FM, int FN, int OCC>
sq_status launch_w4a16_ring(const __half *X, int64_t ldx, int T, int K, const uint8_t *Qw, const float *sw, int N,
                            __half *Y, int64_t ldy, hipStream_t st)
{
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
    constexpr size_t lds = (size_t)3 * (BM * 128 + BN * 32);
    static_assert(lds <= (size_t)kMaxDynamicLds, "ring does not fit in LDS");
    auto kernel = w4a16_gemm_ring_kernel<WM, WN, FM, FN, OCC>;
    if (!allow_large_lds(reinterpret_cast<const void *>(kernel))) return SQ_ERR_LAUNCH;
    const int tiles_m = (T + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int vec_store = (((uintptr_t)Y & 15) == 0 && (ldy % 8) == 0) ? 1 : 0;
    hipLaunchKernelGGL(kernel, dim3((unsigned)(tiles_m * tiles_n)), dim3(WM * WN * kWave), lds, st, X, ldx, T, K, Qw, sw,
                       N, Y, ldy, tiles_m, tiles_n, vec_store);
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
    if (T < 0 || N < 0 || K <= 0 || (K % sq::kBK) != 0 || K > 131072) return SQ_ERR_SHAPE;
    if (T > (1 << 24) || ldx < K || ldy < N) return SQ_ERR_SHAPE;
    if (T == 0 || N == 0) return SQ_OK;
    if (!X || !Qw || !sw || !Y) return SQ_ERR_NULL;
    if (((uintptr_t)X & 15) || (ldx % 8) != 0 || ((uintptr_t)Qw & 15) || ((uintptr_t)Y & 1) || ((uintptr_t)sw & 3))
        return SQ_ERR_ALIGN;
    // At most 32 tokens: one pass over the weights (two token blocks above 16 tokens read them twice,
    // the second time mostly out of the caches; beyond that the tile kernel is the better choice).
    // Launch shapes as in the W4A4 decode-shaped kernel: about eight waves on every CU.
    if (T <= 32 && (K % 256) == 0 && sq::debug_option(SQ_DEBUG_W4A16_LAUNCH_SHAPE) == 0) {
        const hipStream_t st = static_cast<hipStream_t>(stream);
        const __half *Xh = static_cast<const __half *>(X);
        __half *Yh = static_cast<__half *>(Y);
        if (N >= 64 * 384) return sq::launch_w4a16_skinny<4, 4>(Xh, ldx, (int)T, K, Qw, sw, N, Yh, ldy, st);
        return sq::launch_w4a16_skinny<2, 8>(Xh, ldx, (int)T, K, Qw, sw, N, Yh, ldy, st);
    }
    {
        const hipStream_t st = static_cast<hipStream_t>(stream);
        const __half *Xh = static_cast<const __half *>(X);
        __half *Yh = static_cast<__half *>(Y);
        const int shape = sq::debug_option(SQ_DEBUG_W4A16_LAUNCH_SHAPE);
        const int64_t tiles_large = ((T + 255) / 256) * ((N + 255) / 256);
        if (shape == 3 || (shape == 0 && tiles_large >= 192))
            return sq::launch_w4a16_ring<2, 4, 4, 2, 1>(Xh, ldx, (int)T, K, Qw, sw, N, Yh, ldy, st);
        if (shape == 2 || shape == 0)
            return sq::launch_w4a16_ring<1, 4, 4, 2, 2>(Xh, ldx, (int)T, K, Qw, sw, N, Yh, ldy, st);
    }
    const int tiles_m = (int)((T + sq::kBM - 1) / sq::kBM), tiles_n = (N + sq::kBN - 1) / sq::kBN;
    hipLaunchKernelGGL(sq::w4a16_gemm_kernel, dim3((unsigned)(tiles_m * tiles_n)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const __half *>(X), ldx, (int)T, K, Qw, sw, N,
                       static_cast<__half *>(Y), ldy, tiles_m, tiles_n);
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}
