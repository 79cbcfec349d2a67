// sq_w4a4_gemm: int4 x int4 GEMM on the int8 matrix cores of gfx950 with a dequantizing epilogue
// (Eq. 1 of the paper evaluated on the 4-bit codes; the weight operand is Flat(W~_R) = W^T R of
// Sec. 4.2, one K-contiguous row per output channel).
//
//   acc[t, n] = sum_k Qx[t, k] Qw[n, k]   (int32, exact)      Y[t, n] = fp16(acc * sx[t] * sw[n])
//
// Nibbles are widened to int8 in registers as (code << 4): "w & 0xF0F0F0F0" yields the odd codes
// of a dword times 16 with their sign in place, "(w << 4) & 0xF0F0F0F0" the even ones.  Both
// operands carry the factor 16, so the int32 accumulator holds 256 * acc exactly
// (64 * K * 256 < 2^31 for K <= 131040, the limit of the entry point) and the epilogue shifts it
// out.  The split into even and odd codes permutes the contraction index the same way on both
// operands, which a dot product does not see.
#include "sq_common.h"


namespace sq {

// LDS tile of one operand: rows of BKB bytes (2*BKB codes), stored as 16-byte chunks.
// Chunk c of row r sits at chunk slot r*CPR + (c ^ swz(r)).  The LDS of this part serves a
// 16-byte read of sixteen lanes per cycle from 64 banks (256 bytes): with swz(r) = (r / 2) % 8 for
// rows of 128 bytes (two rows per 256 bytes) and (r / 4) % 4 for rows of 64 bytes, the sixteen
// consecutive rows that read the same logical chunk land in sixteen different 16-byte bank groups
// (SQ_LDS_BANK_CONFLICT reads 0 for the kernel; with swz(r) = r % 8, which would be right for 32
// banks, it read 46 % of the LDS-active cycles -- at no difference in time: LDS is a third busy).
template <int BKB>
__device__ __forceinline__ int lds_chunk_slot(int row, int chunk)
{
    constexpr int CPR = BKB / 16;
    static_assert(CPR == 4 || CPR == 8, "tile row must be 64 or 128 bytes");
    const int swz = (CPR == 8) ? ((row >> 1) & 7) : ((row >> 2) & 3);
    return row * CPR + (chunk ^ swz);
}

__device__ __forceinline__ void widen_chunk(const uint4 w, v4i &first, v4i &second)
{
    const uint32_t m = 0xF0F0F0F0u;
    first = v4i{(int)((w.x << 4) & m), (int)(w.x & m), (int)((w.y << 4) & m), (int)(w.y & m)};
    second = v4i{(int)((w.z << 4) & m), (int)(w.z & m), (int)((w.w << 4) & m), (int)(w.w & m)};
}

// 16 bytes per lane from global memory straight into LDS at lds_addr + lane * 16 (lds_addr is
// wave-uniform).  Issued from inline assembly so that the compiler does not serialise later LDS
// reads of *other* stages behind it; completion is tracked by hand with wait_vmcnt below.
__device__ __forceinline__ void load_to_lds_16(const void *gptr, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(gptr), "s"(lds_addr)
                 : "memory", "m0");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// s_barrier without the memory fence of __syncthreads (which would wait for every outstanding
// global -> LDS load).  The wave's own LDS reads are drained first.
__device__ __forceinline__ void block_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// The same load, issued only if a < b (both wave-uniform).  The branch lives inside the assembly
// so that the surrounding loop body stays one basic block for the instruction scheduler.
__device__ __forceinline__ void load_to_lds_16_if(const void *gptr, uint32_t lds_addr, int a, int b)
{
    asm volatile("s_cmp_lt_i32 %2, %3\n\t"
                 "s_cbranch_scc0 .Lsq_skip_load_%=\n\t"
                 "s_mov_b32 m0, %1\n\t"
                 "s_nop 0\n\t"
                 "global_load_lds_dwordx4 %0, off\n"
                 ".Lsq_skip_load_%=:"
                 :
                 : "v"(gptr), "s"(lds_addr), "s"(a), "s"(b)
                 : "memory", "m0", "scc");
}

// Ring of NS stages, L loads per wave and tile, `rem` tiles exist beyond the one that must have
// landed (rem may be negative).  Loads complete in order, so that tile is in LDS once at most
// min(rem, NS - 2) * L loads are outstanding: wait for the largest count first and step down only
// in the last turns.  Then the LDS reads are drained and the waves meet at the barrier.
template <int L, int NS>
__device__ __forceinline__ void wait_tile_and_barrier(int rem)
{
    constexpr int D = NS - 2;
    static_assert(D >= 1 && D <= 4 && D * L < 64, "vmcnt is a 6-bit counter; at most four levels");
    constexpr int d0 = D, d1 = D > 1 ? D - 1 : 0, d2 = D > 2 ? D - 2 : 0, d3 = D > 3 ? D - 3 : 0;
    asm volatile("s_waitcnt vmcnt(%1)\n\t"
                 "s_cmp_ge_i32 %0, %2\n\t"
                 "s_cbranch_scc1 .Lsq_landed_%=\n\t"
                 "s_waitcnt vmcnt(%3)\n\t"
                 "s_cmp_ge_i32 %0, %4\n\t"
                 "s_cbranch_scc1 .Lsq_landed_%=\n\t"
                 "s_waitcnt vmcnt(%5)\n\t"
                 "s_cmp_ge_i32 %0, %6\n\t"
                 "s_cbranch_scc1 .Lsq_landed_%=\n\t"
                 "s_waitcnt vmcnt(%7)\n\t"
                 "s_cmp_ge_i32 %0, %8\n\t"
                 "s_cbranch_scc1 .Lsq_landed_%=\n\t"
                 "s_waitcnt vmcnt(0)\n"
                 ".Lsq_landed_%=:\n\t"
                 "s_waitcnt lgkmcnt(0)\n\t"
                 "s_barrier"
                 :
                 : "s"(rem), "n"(d0 * L), "n"(d0), "n"(d1 * L), "n"(d1), "n"(d2 * L), "n"(d2), "n"(d3 * L), "n"(d3)
                 : "memory", "scc");
}

// XCD-contiguous ids, then groups of 8 row-tiles walked column by column: the tiles resident on
// one XCD at a time share a few row panels and a few column panels in its L2.
__device__ __forceinline__ void tile_of_workgroup(int tiles_m, int tiles_n, int &bm, int &bn)
{
    const int id = xcd_contiguous_id(blockIdx.x, tiles_m * tiles_n);
    constexpr int GM = 8;
    const int group = id / (GM * tiles_n);
    const int gm = min(GM, tiles_m - group * GM);
    const int in_group = id - group * GM * tiles_n;
    bm = group * GM + in_group % gm;
    bn = in_group / gm;
}

// Epilogue of one wave.  32x32 accumulator layout: lane holds column (lane % 32); register e
// holds row 8 * (e / 4) + 4 * (lane / 32) + e % 4.
template <int FM, int FN>
__device__ __forceinline__ void store_tile(const v16i (&acc)[FM][FN], int row_base, int col_base,
                                           int lane, const float *__restrict__ sx,
                                           const float *__restrict__ sw, int T, int N,
                                           __half *__restrict__ Y, int64_t ldy,
                                           int32_t *__restrict__ acc_dbg)
{
    const int frow = lane & 31, fhalf = lane >> 5;
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int n = col_base + j * 32 + frow;
        if (n >= N) continue;
        const float swn = sw[n];
#pragma unroll
        for (int i = 0; i < FM; ++i) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int t = row_base + i * 32 + 8 * (e / 4) + 4 * fhalf + (e % 4);
                if (t >= T) continue;
                const int a = acc[i][j][e] >> 8;
                Y[(int64_t)t * ldy + n] = __float2half_rn((float)a * sx[t] * swn);
                if (acc_dbg != nullptr) acc_dbg[(int64_t)t * N + n] = a;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Main kernel (K % (2*BKB) == 0).  Block tile (WM*FM*32) x (WN*FN*32), WM x WN waves, each FM x FN
// fragments of 32x32.  K is walked in tiles of 2*BKB codes (BKB bytes per row).  Tiles go from
// global memory straight into LDS (global_load_lds, 16 bytes per lane, no register staging)
// through a ring of NS stages, NS - 1 tiles ahead of the one being multiplied (three stages in
// every launch shape: deeper rings measured no faster, for large tiles or small).  The epilogue
// stages the fp16 tile in LDS and writes it out in full 16-byte, row-contiguous stores.
// ------------------------------------------------------------------------------------------
// KG = 2: two groups of WM x WN waves share the block tile and split K in halves (group g walks
// bytes [g Kb/2, (g+1) Kb/2) of every row); the second group's accumulators are added to the
// first's through LDS before the epilogue.  For tiles so small that the time is the walk over K.
// LW > 0: LW more waves that do nothing but move the tiles (global -> LDS, the waits for them) while
// the WM x WN others never issue a memory instruction inside the loop.  A global -> LDS load holds
// the wave that issues it for some tens of ns, in which it issues no MFMA either; with the loads
// of a 128 x 256 tile spread over the eight multiplying waves that was a tenth of the kernel (a
// timing-only build without the weights' loads: 28.3 against 31.5 us with them cache-hot).  The
// loading waves cost registers (every wave of a workgroup gets the same allocation), so this form
// needs at most 168 of them per wave: three waves per SIMD.
template <int WM, int WN, int FM, int FN, int BKB, int OCC, int KG, int NS, int LW>
__global__ __launch_bounds__((KG * WM * WN + LW) * kWave, OCC) void w4a4_gemm_kernel(
    const uint8_t *__restrict__ Qx, const float *__restrict__ sx, int T, int Kb,
    const uint8_t *__restrict__ Qw, const float *__restrict__ sw, int N, __half *__restrict__ Y,
    int64_t ldy, int32_t *__restrict__ acc_dbg, int tiles_m, int tiles_n, int vec_store)
{
    static_assert(NS >= 3 && NS <= 6, "ring of three to six stages");
    static_assert(KG == 1 || KG == 2, "one or two K groups");
    static_assert(LW == 0 || KG == 1, "loading waves: one K group");
    constexpr int NW = WM * WN;                                // NW: multiplying waves of one K group
    constexpr int NTC = KG * NW * kWave, NT = NTC + LW * kWave;  // multiplying threads; all threads
    constexpr int NL = LW > 0 ? LW : NW;                       // waves that share the loads of a tile
    constexpr bool SELF_LOAD = LW == 0;                        // the multiplying waves load for themselves
    constexpr int CPR = BKB / 16;                 // 16-byte chunks per tile row
    constexpr int STEPS = CPR / 2;                // steps of 64 codes per tile
    constexpr int RPL = kWave / CPR;              // tile rows filled by one wave-wide load
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
    constexpr int A_SLOTS = BM * CPR, B_SLOTS = BN * CPR, STAGE_SLOTS = A_SLOTS + B_SLOTS;
    constexpr int A_LOADS = BM / RPL / NL, B_LOADS = BN / RPL / NL;   // loads per loading wave per tile
    constexpr int LOADS = A_LOADS + B_LOADS;
    static_assert((BM / RPL) % NL == 0 && (BN / RPL) % NL == 0, "loads must split evenly over waves");
    static_assert(STEPS == 2 || STEPS == 4, "tile rows of 64 or 128 bytes");

    extern __shared__ uint4 smem[];

    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    // K group and wave within it; a loading wave (index NW and up) counts from 0 again
    const bool loader = LW > 0 && tid / kWave >= NW;
    const int kg = LW > 0 ? 0 : (tid / kWave) / NW, wave = (tid / kWave) % NW;
    const int wm = wave / WN, wn = wave % WN;
    if constexpr (KG == 2) {                 // this group's half of K
        Kb /= 2;
        Qx += kg * Kb;
        Qw += kg * Kb;
    }
    const int row_bytes = KG * Kb;           // distance between rows in memory
    int bm, bn;
    tile_of_workgroup(tiles_m, tiles_n, bm, bn);
    const int row0 = bm * BM, col0 = bn * BN;

    // Global -> LDS.  One wave-wide load fills 64 consecutive chunk slots = RPL rows x CPR chunks;
    // lane l lands in slot base + l, i.e. row l/CPR, physical chunk l%CPR, which holds the logical
    // chunk (l%CPR) ^ swizzle(row).  Wave w issues the loads for row groups w, w+NW, w+2NW, ...
    const int lrow = lane / CPR;
    // (the swizzle has a period of 16 rows, and every load of a wave starts a multiple of 16 rows from its first)
    static_assert((RPL * NL) % 16 == 0, "loads of one wave must start at the same row modulo 16");
    const int lrow16 = (RPL * wave + lrow) & 15;
    const int lchunk = (lane % CPR) ^ (CPR == 8 ? ((lrow16 >> 1) & 7) : ((lrow16 >> 2) & 3));
    const uint8_t *a_src[A_LOADS];
    const uint8_t *b_src[B_LOADS];
#pragma unroll
    for (int g = 0; g < A_LOADS; ++g)   // rows past the end are clamped: their products are never stored
        a_src[g] = Qx + (int64_t)min(row0 + RPL * (wave + NL * g) + lrow, T - 1) * row_bytes + lchunk * 16;
#pragma unroll
    for (int g = 0; g < B_LOADS; ++g)
        b_src[g] = Qw + (int64_t)min(col0 + RPL * (wave + NL * g) + lrow, N - 1) * row_bytes + lchunk * 16;

    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4 *)smem;
    const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t group_byte = __builtin_amdgcn_readfirstlane(kg) * (STAGE_SLOTS * 16);   // this group's part of a stage
    // loads of tile kt into ring stage `stage`, issued only if kt < limit
    auto issue_tile = [&](int kt, int stage, int limit) {
        const uint32_t sa = lds_base + (uint32_t)stage * (KG * STAGE_SLOTS * 16) + group_byte + wave_u * 1024;
        const uint32_t sb = sa + A_SLOTS * 16;
        const int kb0 = kt * BKB;
#pragma unroll
        for (int g = 0; g < A_LOADS; ++g) load_to_lds_16_if(a_src[g] + kb0, sa + g * NL * 1024, kt, limit);
#pragma unroll
        for (int g = 0; g < B_LOADS; ++g) load_to_lds_16_if(b_src[g] + kb0, sb + g * NL * 1024, kt, limit);
    };
    // one of those loads: index 0 .. A_LOADS-1 the tokens' part, then the weights' part
    auto issue_one = [&](int idx, int kt, int stage, int limit) {
        const uint32_t sa = lds_base + (uint32_t)stage * (KG * STAGE_SLOTS * 16) + group_byte + wave_u * 1024;
        const int kb0 = kt * BKB;
        if (idx < A_LOADS) load_to_lds_16_if(a_src[idx] + kb0, sa + idx * NL * 1024, kt, limit);
        else load_to_lds_16_if(b_src[idx - A_LOADS] + kb0, sa + A_SLOTS * 16 + (idx - A_LOADS) * NL * 1024, kt, limit);
    };

    v16i acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    const int ktiles = Kb / BKB;
    const int frow = lane & 31, fhalf = lane >> 5;

    // LDS byte offsets of this lane's fragment chunks inside a stage, per step s (the step picks
    // logical chunk 2s + fhalf; the swizzle depends on row % 8 = frow % 8 for every fragment).
    constexpr int STAGE_BYTES = KG * STAGE_SLOTS * 16, FRAG_BYTES = 32 * BKB;
    int a_off[STEPS], b_off[STEPS];
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
        a_off[s] = kg * (STAGE_SLOTS * 16) + lds_chunk_slot<BKB>(wm * FM * 32 + frow, 2 * s + fhalf) * 16;
        b_off[s] = kg * (STAGE_SLOTS * 16) + A_SLOTS * 16 + lds_chunk_slot<BKB>(wn * FN * 32 + frow, 2 * s + fhalf) * 16;
    }
    const char *lds = reinterpret_cast<const char *>(smem);

    // Software pipeline over the steps (one step = 64 codes of K = two MFMAs per fragment pair):
    //   raw        chunks of step s+1, read from LDS during step s-1
    //   frag[1-C]  widened operands of step s+1, made from raw during step s
    //   frag[C]    widened operands of step s, fed to the MFMAs of step s
    // so every step interleaves its MFMAs with the widening VALU work of the next step and the
    // LDS reads of the step after that.
    uint4 raw[FM + FN];
    v4i frag[2][FM + FN][2];

    auto read_step = [&](int stage_byte, int s) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
            raw[i] = *reinterpret_cast<const uint4 *>(lds + stage_byte + a_off[s] + i * FRAG_BYTES);
#pragma unroll
        for (int j = 0; j < FN; ++j)
            raw[FM + j] = *reinterpret_cast<const uint4 *>(lds + stage_byte + b_off[s] + j * FRAG_BYTES);
    };
    // One step, written in the order it should issue: each MFMA on frag[C] is followed by the
    // widening of a few dwords of raw into frag[1-C] (three VALU ops per dword), and a chunk of
    // raw is refilled from (stage_byte, s_read) as soon as its last dword has been widened.
    // The scheduling barriers keep the compiler from regrouping the units.
    constexpr int NMFMA = 2 * FM * FN, NDW = 4 * (FM + FN);
    // DPART: -1, or which half of the loads of the tile three ahead this step issues (0 / 1): a
    // global -> LDS load costs the wave some tens of ns to issue, and six of them in a row right
    // behind the barrier, in all eight waves at once, leave the matrix cores idle; spread over the
    // MFMAs of the two steps that follow the barrier they do not.
    constexpr int DMA_FIRST_HALF = (LOADS + 1) / 2;
#define SQ_GEMM_STEP(C, stage_byte, s_read, DPART)                                                   \
    do {                                                                                             \
        constexpr int dn = (DPART) < 0 ? 0 : ((DPART) == 0 ? DMA_FIRST_HALF : LOADS - DMA_FIRST_HALF); \
        constexpr int dbase = (DPART) == 1 ? DMA_FIRST_HALF : 0;                                     \
        static_assert(dn <= NMFMA, "at most one load behind each MFMA");                             \
        _Pragma("unroll") for (int m = 0; m < NMFMA; ++m) {                                          \
            const int u = m / (FM * FN), i = (m / FN) % FM, j = m % FN;                              \
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(frag[C][i][u], frag[C][FM + j][u],     \
                                                              acc[i][j], 0, 0, 0);                   \
            _Pragma("unroll") for (int d = m * NDW / NMFMA; d < (m + 1) * NDW / NMFMA; ++d) {        \
                const int c = d >> 2, w = d & 3;                                                     \
                const uint32_t x = (w == 0) ? raw[c].x : (w == 1) ? raw[c].y : (w == 2) ? raw[c].z : raw[c].w; \
                frag[1 - (C)][c][w >> 1][2 * (w & 1)] = (int)((x << 4) & 0xF0F0F0F0u);               \
                frag[1 - (C)][c][w >> 1][2 * (w & 1) + 1] = (int)(x & 0xF0F0F0F0u);                  \
                if (w == 3) {                                                                        \
                    const int off = (c < FM) ? a_off[s_read] + c * FRAG_BYTES                        \
                                             : b_off[s_read] + (c - FM) * FRAG_BYTES;                \
                    raw[c] = *reinterpret_cast<const uint4 *>(lds + (stage_byte) + off);             \
                }                                                                                    \
            }                                                                                        \
            _Pragma("unroll") for (int q = 0; q < dn; ++q)                                           \
                if (m == q * NMFMA / (dn > 0 ? dn : 1)) issue_one(dbase + q, kt + NS, st_cur, ktiles); \
            __builtin_amdgcn_sched_barrier(0);                                                       \
        }                                                                                            \
    } while (0)
    // Between two tiles.  Loads complete in order, so tile kt+1 has landed once only the loads of
    // tile kt+2 (if it exists) are outstanding.  After the barrier every wave's share of tile kt+1
    // is in LDS and nobody reads tile kt any more (all its reads were issued, and the barrier
    // drains them), so its stage can take tile kt+3.
#define SQ_GEMM_TURN()                                                                               \
    do {                                                                                             \
        if constexpr (SELF_LOAD) wait_tile_and_barrier<LOADS, NS>(ktiles - kt - 2);                  \
        else block_barrier();                                                                        \
    } while (0)

    // prologue: tiles 0 and 1 in flight, wait for tile 0, start tile 2, first fragments ready
    if (SELF_LOAD || loader) {
#pragma unroll
        for (int t = 0; t < NS - 1; ++t) issue_tile(t, t, ktiles);
    }
    // While the first tiles are on their way, the block's dequantization steps are parked in LDS
    // behind the ring and the staged output tile, so that the epilogue does not wait on global
    // memory: sx * 2^-8 for the BM tokens (the accumulators carry a factor 256), then sw for the
    // BN output channels; 0 past the edges.
    constexpr int SCALE_BYTE = (NS * STAGE_BYTES > BM * (BN * 2 + 16)) ? NS * STAGE_BYTES : BM * (BN * 2 + 16);
    float *scale_lds = reinterpret_cast<float *>(reinterpret_cast<char *>(smem) + SCALE_BYTE);
    for (int r = tid; r < BM + BN; r += NT) {
        float v;
        if (r < BM) v = (row0 + r < T) ? sx[row0 + r] * 0.00390625f : 0.f;
        else v = (col0 + r - BM < N) ? sw[col0 + r - BM] : 0.f;
        scale_lds[r] = v;
    }

    if constexpr (!SELF_LOAD) {
        if (loader) {
            // A loading wave: the waits and requests of the multiplying waves' loop, nothing else.  It
            // meets them at every barrier of the kernel, the epilogue's two included.
            wait_tile_and_barrier<LOADS, NS>(ktiles - 1);
            issue_tile(NS - 1, NS - 1, ktiles);
            int st = 0;
            for (int kt = 0; kt < ktiles; ++kt) {
                wait_tile_and_barrier<LOADS, NS>(ktiles - kt - 2);
                issue_tile(kt + NS, st, ktiles);
                st = (st + 1 == NS) ? 0 : st + 1;
            }
            block_barrier();
            __syncthreads();
            return;
        }
        block_barrier();                   // tile 0 has landed (the loading waves waited for it)
    } else {
        wait_tile_and_barrier<LOADS, NS>(ktiles - 1);
        issue_tile(NS - 1, NS - 1, ktiles);
    }
    read_step(0, 0);
#pragma unroll
    for (int c = 0; c < FM + FN; ++c) widen_chunk(raw[c], frag[0][c][0], frag[0][c][1]);
    read_step(0, 1);

    int st_cur = 0;                 // ring stage of tile kt
    for (int kt = 0; kt < ktiles; ++kt) {
        const int st_next = (st_cur + 1 == NS) ? 0 : st_cur + 1;
        const int cur_byte = st_cur * STAGE_BYTES, next_byte = st_next * STAGE_BYTES;
        // the LDS reads run two steps ahead of the MFMAs, so the last two steps of a tile already
        // read the next tile (for the very last tile they read a stale stage; never used)
        if constexpr (STEPS == 4) {
            SQ_GEMM_STEP(0, cur_byte, 2, -1);
            SQ_GEMM_STEP(1, cur_byte, 3, -1);
            SQ_GEMM_TURN();
            SQ_GEMM_STEP(0, next_byte, 0, SELF_LOAD ? 0 : -1);
            SQ_GEMM_STEP(1, next_byte, 1, SELF_LOAD ? 1 : -1);
        } else {
            SQ_GEMM_TURN();
            SQ_GEMM_STEP(0, next_byte, 0, SELF_LOAD ? 0 : -1);
            SQ_GEMM_STEP(1, next_byte, 1, SELF_LOAD ? 1 : -1);
        }
        st_cur = st_next;
    }
#undef SQ_GEMM_STEP
#undef SQ_GEMM_TURN

    // ---- epilogue ------------------------------------------------------------------------
    // 32x32 accumulator layout: lane holds column (lane % 32); register e holds row
    // 8 * (e / 4) + 4 * (lane / 32) + e % 4, i.e. four runs of four consecutive tokens.
    constexpr int YS = BN * 2 + 16;      // LDS row stride of the staged fp16 tile, bytes
    static_assert(BM * YS <= kMaxDynamicLds, "staged output tile must fit in LDS");
    wait_vmcnt<0>();
    block_barrier();                     // the ring is dead: reuse it for the output tile
    char *ys = reinterpret_cast<char *>(smem);
    if constexpr (KG == 2) {
        // partial sums of the second group, parked behind where the output tile will be staged
        constexpr int PART_BYTE = (BM * YS + 15) / 16 * 16;
        static_assert(PART_BYTE + NW * FM * FN * 16 * kWave * 4 <= NS * STAGE_BYTES, "partial sums must fit in the dead ring");
        int *part = reinterpret_cast<int *>(ys + PART_BYTE) + wave * (FM * FN * 16 * kWave) + lane;
        if (kg == 1) {
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) part[((i * FN + j) * 16 + e) * kWave] = acc[i][j][e];
        }
        block_barrier();
        if (kg == 0) {
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[i][j][e] += part[((i * FN + j) * 16 + e) * kWave];
        }
    }
    if (kg == 0) {
    float swn[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j) swn[j] = scale_lds[BM + (wn * FN + j) * 32 + frow];
#pragma unroll
    for (int i = 0; i < FM; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int tl0 = (wm * FM + i) * 32 + 8 * q + 4 * fhalf;
            const float4 s4 = *reinterpret_cast<const float4 *>(scale_lds + tl0);
            const float sxt[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
            for (int r = 0; r < 4; ++r) {
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    const int nl = (wn * FN + j) * 32 + frow;
                    *reinterpret_cast<__half *>(ys + (tl0 + r) * YS + nl * 2) =
                        __float2half_rn((float)acc[i][j][4 * q + r] * sxt[r] * swn[j]);
                }
            }
        }
    }
    if (acc_dbg != nullptr) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int t = row0 + (wm * FM + i) * 32 + 8 * (e / 4) + 4 * fhalf + (e % 4);
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    const int n = col0 + (wn * FN + j) * 32 + frow;
                    if (t < T && n < N) acc_dbg[(int64_t)t * N + n] = acc[i][j][e] >> 8;
                }
            }
    }
    }   // kg == 0
    __syncthreads();
    constexpr int CPRY = BN / 8;         // 16-byte chunks per output row
    constexpr int ROUNDS = BM * CPRY / NTC, BATCH = (ROUNDS % 4 == 0) ? 4 : (ROUNDS % 2 == 0) ? 2 : 1;
    static_assert((BM * CPRY) % NTC == 0, "every multiplying thread copies the same number of chunks");
    for (int r0 = 0; r0 < ROUNDS; r0 += BATCH) {       // up to four LDS reads in flight, then their stores
        uint4 v[BATCH];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int idx = (r0 + u) * NTC + tid;
            v[u] = *reinterpret_cast<const uint4 *>(ys + (idx / CPRY) * YS + (idx % CPRY) * 16);
        }
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int idx = (r0 + u) * NTC + tid;
            const int t = row0 + idx / CPRY, n0 = col0 + (idx % CPRY) * 8;
            if (t >= T || n0 >= N) continue;
            __half *dst = Y + (int64_t)t * ldy + n0;
            if (vec_store && n0 + 8 <= N) {
                *reinterpret_cast<uint4 *>(dst) = v[u];
            } else {
                const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int e = 0; e < 8; ++e)          // register-only: no addressable copy of the chunk
                    if (n0 + e < N) reinterpret_cast<uint16_t *>(dst)[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Skinny kernel (T <= 32*FM <= 64, K % 256 == 0): the decode-shaped product, bound by the one
// pass over the weights.  A workgroup owns 32*FN output channels and all tokens; its NW waves
// split K between them (256-code slices dealt round-robin) and add their partial accumulators
// through LDS at the end.  The weights go straight from global memory to registers: a lane reads
// 64 contiguous bytes of its row per slice as four 16-byte loads, so each wave-wide group of four
// loads consumes whole 128-byte lines, and the loads of the next slice are in flight while this
// one is multiplied.
// The tokens' codes are the same for every workgroup and come out of L2, but loaded like the
// weights they are a third of all vector-memory instructions (2.2 of 27.5 us at T = 8, K = 8192,
// N = 28672).  ALDS: when all T rows fit, each workgroup copies them into LDS once (global -> LDS,
// behind the request for its first weight slice) and the waves read their operand chunks from
// there; rows are padded by 16 bytes so that the rows a wave reads together fall into different
// banks.
// ------------------------------------------------------------------------------------------
constexpr int kSkinnyRowPad = 16;      // bytes between the token rows in LDS beyond their length

// TILED: Qw is the decode layout written by sq_tile_weights_decode (blocks of 32 channels, slices
// of 256 codes, each block-slice one contiguous 4 KB piece in the order the lanes load it), so that
// every load instruction of a wave reads 1 KB of consecutive bytes and a slice 4 KB: the same
// kernel on the same bytes took 24.0 instead of 27.0 us (T = 8, K = 8192, N = 28672).
template <int FM, int FN, int NW, bool ALDS, bool TILED = false>
__global__ __launch_bounds__(NW *kWave) void w4a4_gemm_skinny_kernel(
    const uint8_t *__restrict__ Qx, const float *__restrict__ sx, int T, int Kb,
    const uint8_t *__restrict__ Qw, const float *__restrict__ sw, int N, __half *__restrict__ Y,
    int64_t ldy, int32_t *__restrict__ acc_dbg)
{
    constexpr int BN = 32 * FN, SLICE = 128;        // bytes of a row per slice (256 codes)
    static_assert(NW * FM * FN * 16 * kWave * 4 <= 64 * 1024, "partial sums must fit in LDS");
    static_assert(!ALDS || FM == 1, "token rows in LDS: one token block");
    // ALDS: the dynamic LDS holds the token rows during the loop and the partial sums after it
    __shared__ int red_static[ALDS ? 1 : NW][FM][FN][16][kWave];
    extern __shared__ uint4 dyn[];
    int(*red)[FM][FN][16][kWave] = ALDS ? reinterpret_cast<int(*)[FM][FN][16][kWave]>(dyn) : red_static;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int l32 = lane & 31, g = lane >> 5;
    const int col0 = blockIdx.x * BN;

    // rows past the ends are clamped: their products are never stored
    const uint8_t *a_ptr[FM];
    const uint8_t *b_ptr[FN];
#pragma unroll
    for (int i = 0; i < FM; ++i) a_ptr[i] = Qx + (int64_t)min(32 * i + l32, T - 1) * Kb + g * 64;
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        if constexpr (TILED)     // the lane's 16-byte unit of load 0 of slice 0 of its block (blocks past the end: the last)
            b_ptr[j] = Qw + (int64_t)min((int)blockIdx.x * FN + j, (N + 31) / 32 - 1) * 32 * Kb + (32 * g + l32) * 16;
        else
            b_ptr[j] = Qw + (int64_t)min(col0 + 32 * j + l32, N - 1) * Kb + g * 64;
    }

    v16i acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    uint4 ra[ALDS ? 1 : 2][FM][4], rb[2][FN][4];
    const int slices = Kb / SLICE;
    const int a_stride = Kb + kSkinnyRowPad;
    const char *a_lds = reinterpret_cast<const char *>(dyn) + min(l32, T - 1) * a_stride + g * 64;
#define SQ_SKINNY_FETCH(BUF, S)                                                                      \
    do {                                                                                             \
        const int off_ = (S) * SLICE;                                                                \
        _Pragma("unroll") for (int j = 0; j < FN; ++j)                                               \
            _Pragma("unroll") for (int c = 0; c < 4; ++c)                                            \
                rb[BUF][j][c] = *reinterpret_cast<const uint4 *>(b_ptr[j] + (TILED ? (S) * 4096 + 1024 * c : off_ + 16 * c)); \
        if constexpr (!ALDS) {                                                                       \
            _Pragma("unroll") for (int i = 0; i < FM; ++i)                                           \
                _Pragma("unroll") for (int c = 0; c < 4; ++c)                                        \
                    ra[BUF][i][c] = *reinterpret_cast<const uint4 *>(a_ptr[i] + off_ + 16 * c);      \
        }                                                                                            \
    } while (0)
#define SQ_SKINNY_MULTIPLY(BUF, S)                                                                   \
    do {                                                                                             \
        if constexpr (ALDS) {                                                                        \
            _Pragma("unroll") for (int c = 0; c < 4; ++c)                                            \
                ra[0][0][c] = *reinterpret_cast<const uint4 *>(a_lds + (S) * SLICE + 16 * c);        \
        }                                                                                            \
        _Pragma("unroll") for (int c = 0; c < 4; ++c) {                                              \
            v4i b0[FN], b1[FN];                                                                      \
            _Pragma("unroll") for (int j = 0; j < FN; ++j) widen_chunk(rb[BUF][j][c], b0[j], b1[j]); \
            _Pragma("unroll") for (int i = 0; i < FM; ++i) {                                         \
                v4i a0, a1;                                                                          \
                widen_chunk(ra[ALDS ? 0 : BUF][i][c], a0, a1);                                       \
                _Pragma("unroll") for (int j = 0; j < FN; ++j) {                                     \
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b0[j], acc[i][j], 0, 0, 0); \
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1[j], acc[i][j], 0, 0, 0); \
                }                                                                                    \
            }                                                                                        \
        }                                                                                            \
    } while (0)

    // wave w takes slices w, w+NW, w+2NW, ...; two register sets alternate
    int S = wave;
    if (S < slices) SQ_SKINNY_FETCH(0, S);
    if constexpr (ALDS) {
        // token rows -> LDS, 1 KB per wave-wide load, behind the first weight request (which has
        // the longer way to go); visible to every wave after the barrier
        const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4 *)dyn;
        const int parts = (Kb + 1023) / 1024;
        for (int idx = wave; idx < T * parts; idx += NW) {
            const int row = idx / parts, part = idx - row * parts;
            if (part * 1024 + lane * 16 < Kb)
                load_to_lds_16(Qx + (int64_t)row * Kb + part * 1024 + lane * 16,
                               __builtin_amdgcn_readfirstlane(lds_base + row * a_stride + part * 1024));
        }
        wait_vmcnt<0>();
        __syncthreads();
    }
    while (S < slices) {
        if (S + NW < slices) SQ_SKINNY_FETCH(1, S + NW);
        SQ_SKINNY_MULTIPLY(0, S);
        S += NW;
        if (S >= slices) break;
        if (S + NW < slices) SQ_SKINNY_FETCH(0, S + NW);
        SQ_SKINNY_MULTIPLY(1, S);
        S += NW;
    }
#undef SQ_SKINNY_FETCH
#undef SQ_SKINNY_MULTIPLY

    if constexpr (ALDS) __syncthreads();        // every wave is done with the token rows: the sums take their place
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) red[wave][i][j][e][lane] = acc[i][j][e];
    __syncthreads();
    // accumulator layout: lane holds channel (lane % 32); register e holds token
    // 8 * (e / 4) + 4 * (lane / 32) + e % 4.  The sums carry the factor 256 of the widening.
    for (int idx = tid; idx < FM * FN * 16 * kWave; idx += NW * kWave) {
        const int ln = idx & (kWave - 1), e = (idx >> 6) & 15, j = (idx >> 10) % FN, i = (idx >> 10) / FN;
        int sum = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) sum += red[w][i][j][e][ln];
        const int t = 32 * i + 8 * (e / 4) + 4 * (ln >> 5) + (e % 4), n = col0 + 32 * j + (ln & 31);
        if (t < T && n < N) {
            Y[(int64_t)t * ldy + n] = __float2half_rn((float)sum * (sx[t] * 0.00390625f) * sw[n]);
            if (acc_dbg != nullptr) acc_dbg[(int64_t)t * N + n] = sum >> 8;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Generic kernel: any K % 32 == 0 (zero-fills the last partial K tile).  Tiles are staged through
// registers; used only for shapes the main kernel does not take.
// ------------------------------------------------------------------------------------------
template <int FM, int FN, int BKB>
__global__ __launch_bounds__(256) void w4a4_gemm_generic_kernel(
    const uint8_t *__restrict__ Qx, const float *__restrict__ sx, int T, int Kb,
    const uint8_t *__restrict__ Qw, const float *__restrict__ sw, int N, __half *__restrict__ Y,
    int64_t ldy, int32_t *__restrict__ acc_dbg, int tiles_m, int tiles_n)
{
    constexpr int NT = 256;
    constexpr int BM = 64 * FM, BN = 64 * FN;
    constexpr int CPR = BKB / 16;
    constexpr int A_CHUNKS = BM * CPR, B_CHUNKS = BN * CPR;
    constexpr int A_PER = A_CHUNKS / NT, B_PER = B_CHUNKS / NT;
    static_assert(A_CHUNKS % NT == 0 && B_CHUNKS % NT == 0, "tile must split evenly over threads");

    __shared__ uint4 sA[A_CHUNKS];
    __shared__ uint4 sB[B_CHUNKS];

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int wm = wave >> 1, wn = wave & 1;
    int bm, bn;
    tile_of_workgroup(tiles_m, tiles_n, bm, bn);
    const int row0 = bm * BM, col0 = bn * BN;

    const uint8_t *a_src[A_PER];
    const uint8_t *b_src[B_PER];
    int a_slot[A_PER], b_slot[B_PER], a_off[A_PER], b_off[B_PER];
#pragma unroll
    for (int g = 0; g < A_PER; ++g) {
        const int c = g * NT + tid, r = c / CPR, ch = c % CPR;
        a_src[g] = Qx + (int64_t)min(row0 + r, T - 1) * Kb + ch * 16;   // clamped: rows past T are never stored
        a_slot[g] = lds_chunk_slot<BKB>(r, ch);
        a_off[g] = ch * 16;
    }
#pragma unroll
    for (int g = 0; g < B_PER; ++g) {
        const int c = g * NT + tid, r = c / CPR, ch = c % CPR;
        b_src[g] = Qw + (int64_t)min(col0 + r, N - 1) * Kb + ch * 16;
        b_slot[g] = lds_chunk_slot<BKB>(r, ch);
        b_off[g] = ch * 16;
    }

    v16i acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    uint4 ra[A_PER], rb[B_PER];
    const int ktiles = (Kb + BKB - 1) / BKB;
    auto fetch = [&](int kt) {
        const int kb0 = kt * BKB;
#pragma unroll
        for (int g = 0; g < A_PER; ++g)
            ra[g] = (kb0 + a_off[g] < Kb) ? *reinterpret_cast<const uint4 *>(a_src[g] + kb0) : uint4{0, 0, 0, 0};
#pragma unroll
        for (int g = 0; g < B_PER; ++g)
            rb[g] = (kb0 + b_off[g] < Kb) ? *reinterpret_cast<const uint4 *>(b_src[g] + kb0) : uint4{0, 0, 0, 0};
    };

    fetch(0);
    const int frow = lane & 31, fhalf = lane >> 5;
    for (int kt = 0; kt < ktiles; ++kt) {
        __syncthreads();     // everyone is done reading the previous tile
#pragma unroll
        for (int g = 0; g < A_PER; ++g) sA[a_slot[g]] = ra[g];
#pragma unroll
        for (int g = 0; g < B_PER; ++g) sB[b_slot[g]] = rb[g];
        __syncthreads();
        if (kt + 1 < ktiles) fetch(kt + 1);

#pragma unroll
        for (int s = 0; s < CPR / 2; ++s) {
            const int ch = 2 * s + fhalf;
            v4i af[FM][2], bf[FN][2];
#pragma unroll
            for (int i = 0; i < FM; ++i)
                widen_chunk(sA[lds_chunk_slot<BKB>((wm * FM + i) * 32 + frow, ch)], af[i][0], af[i][1]);
#pragma unroll
            for (int j = 0; j < FN; ++j)
                widen_chunk(sB[lds_chunk_slot<BKB>((wn * FN + j) * 32 + frow, ch)], bf[j][0], bf[j][1]);
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i][u], bf[j][u], acc[i][j], 0, 0, 0);
        }
    }

    store_tile<FM, FN>(acc, row0 + wm * FM * 32, col0 + wn * FN * 32, lane, sx, sw, T, N, Y, ldy, acc_dbg);
}

template <int WM, int WN, int FM, int FN, int BKB, int OCC, int KG = 1, int NS = 3, int LW = 0>
static sq_status launch_main(const uint8_t *Qx, const float *sx, int T, int K, const uint8_t *Qw,
                             const float *sw, int N, __half *Y, int64_t ldy, int32_t *acc_dbg,
                             hipStream_t st)
{
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
    constexpr size_t ring = (size_t)NS * KG * (BM + BN) * BKB, out_tile = (size_t)BM * (BN * 2 + 16);
    // the epilogue reuses the ring for the output tile; the scales sit behind both
    constexpr size_t lds = (ring > out_tile ? ring : out_tile) + (size_t)(BM + BN) * 4;
    static_assert(lds <= (size_t)kMaxDynamicLds, "ring does not fit in LDS");
    auto kernel = w4a4_gemm_kernel<WM, WN, FM, FN, BKB, OCC, KG, NS, LW>;
    if ((K / 2) % (KG * BKB) != 0) return SQ_ERR_SHAPE;      // every K group walks whole tiles
    if (!allow_large_lds(reinterpret_cast<const void *>(kernel))) return SQ_ERR_LAUNCH;
    const int tiles_m = (T + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int vec_store = (((uintptr_t)Y & 15) == 0 && (ldy % 8) == 0) ? 1 : 0;
    hipLaunchKernelGGL(kernel, dim3((unsigned)(tiles_m * tiles_n)), dim3((KG * WM * WN + LW) * kWave), lds, st, Qx,
                       sx, T, K / 2, Qw, sw, N, Y, ldy, acc_dbg, tiles_m, tiles_n, vec_store);
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

template <int FM, int FN, int NW, bool TILED = false>
static sq_status launch_skinny(const uint8_t *Qx, const float *sx, int T, int K, const uint8_t *Qw,
                               const float *sw, int N, __half *Y, int64_t ldy, int32_t *acc_dbg,
                               hipStream_t st)
{
    const dim3 grid((unsigned)((N + 32 * FN - 1) / (32 * FN))), block(NW * kWave);
    // token rows in LDS where they fit 64 KB (and two workgroups a CU)
    const size_t rows_bytes = (size_t)T * (K / 2 + kSkinnyRowPad), sums_bytes = (size_t)NW * FM * FN * 16 * kWave * 4;
    // (sixteen waves have two slices each at K = 8192: the wait for the rows costs them more than it saves)
    if constexpr (FM == 1 && NW <= 8) {
        if (rows_bytes <= 64 * 1024) {
            hipLaunchKernelGGL((w4a4_gemm_skinny_kernel<FM, FN, NW, true, TILED>), grid, block,
                               rows_bytes > sums_bytes ? rows_bytes : sums_bytes, st, Qx, sx, T, K / 2, Qw, sw, N, Y,
                               ldy, acc_dbg);
            return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
        }
    }
    hipLaunchKernelGGL((w4a4_gemm_skinny_kernel<FM, FN, NW, false, TILED>), grid, block, 0, st, Qx, sx, T, K / 2, Qw, sw, N,
                       Y, ldy, acc_dbg);
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

static sq_status launch_generic(const uint8_t *Qx, const float *sx, int T, int K, const uint8_t *Qw,
                                const float *sw, int N, __half *Y, int64_t ldy, int32_t *acc_dbg,
                                hipStream_t st)
{
    constexpr int FM = 2, FN = 2, BM = 64 * FM, BN = 64 * FN;
    const int tiles_m = (T + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    hipLaunchKernelGGL((w4a4_gemm_generic_kernel<FM, FN, 64>), dim3((unsigned)(tiles_m * tiles_n)),
                       dim3(256), 0, st, Qx, sx, T, K / 2, Qw, sw, N, Y, ldy, acc_dbg, tiles_m, tiles_n);
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

// Canonical weight codes [N, K/2] -> decode layout.  One thread per 16-byte unit of the output:
// unit 64 c + 32 g + r of piece (b, S) holds bytes 64 g + 16 c .. + 15 of slice S of channel
// 32 b + r (zeros for channels past N).
__global__ __launch_bounds__(256) void tile_weights_decode_kernel(const uint8_t *__restrict__ Qw, int Kb, int N,
                                                                  int64_t units, uint4 *__restrict__ Qt)
{
    const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= units) return;
    const int slices = Kb / 128;
    const int64_t piece = o / 256;
    const int u = (int)(o % 256), c = u / 64, g = (u / 32) % 2, r = u % 32;
    const int64_t b = piece / slices, S = piece % slices, n = 32 * b + r;
    uint4 v = {0u, 0u, 0u, 0u};
    if (n < N) v = *reinterpret_cast<const uint4 *>(Qw + n * Kb + S * 128 + 64 * g + 16 * c);
    Qt[o] = v;
}

}  // namespace sq

extern "C" int64_t sq_decode_weights_bytes(int32_t K, int32_t N)
{
    if (K <= 0 || (K % 256) != 0 || K > SQ_GEMM_MAX_K || N < 0) return 0;
    return ((int64_t)N + 31) / 32 * 32 * (K / 2);
}

extern "C" sq_status sq_tile_weights_decode(const uint8_t *Qw, int32_t K, int32_t N, uint8_t *Qw_tiled, void *stream)
{
    if (N < 0 || K <= 0 || (K % 256) != 0 || K > SQ_GEMM_MAX_K) return SQ_ERR_SHAPE;
    if (N == 0) return SQ_OK;
    if (!Qw || !Qw_tiled) return SQ_ERR_NULL;
    if (((uintptr_t)Qw & 15) || ((uintptr_t)Qw_tiled & 15)) return SQ_ERR_ALIGN;
    const int64_t units = sq_decode_weights_bytes(K, N) / 16;
    hipLaunchKernelGGL(sq::tile_weights_decode_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), Qw, K / 2, N, units, reinterpret_cast<uint4 *>(Qw_tiled));
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

extern "C" sq_status sq_w4a4_gemm_decode(const uint8_t *Qx, const float *sx, int64_t T, int32_t K,
                                         const uint8_t *Qw_tiled, const float *sw, int32_t N, void *Y,
                                         int64_t ldy, int32_t *acc_dbg, void *stream)
{
    if (T < 0 || T > SQ_DECODE_MAX_TOKENS || N < 0 || K <= 0 || (K % 256) != 0 || K > SQ_GEMM_MAX_K) return SQ_ERR_SHAPE;
    if (ldy < N) return SQ_ERR_SHAPE;
    if (T == 0 || N == 0) return SQ_OK;
    if (!Qx || !sx || !Qw_tiled || !sw || !Y) return SQ_ERR_NULL;
    if (((uintptr_t)Qx & 15) || ((uintptr_t)Qw_tiled & 15) || ((uintptr_t)Y & 1) ||
        ((uintptr_t)sx & 3) || ((uintptr_t)sw & 3) || ((uintptr_t)acc_dbg & 3))
        return SQ_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    __half *Yh = static_cast<__half *>(Y);
    const int Ti = (int)T;
    // the launch shapes sq_w4a4_gemm gives the decode-shaped kernel (see there)
    const bool rows_fit_lds = (int64_t)Ti * (K / 2 + sq::kSkinnyRowPad) <= 64 * 1024;
    if (N >= 64 * 384 && !rows_fit_lds) return sq::launch_skinny<1, 2, 4, true>(Qx, sx, Ti, K, Qw_tiled, sw, N, Yh, ldy, acc_dbg, st);
    if (N >= 10240) return sq::launch_skinny<1, 1, 8, true>(Qx, sx, Ti, K, Qw_tiled, sw, N, Yh, ldy, acc_dbg, st);
    return sq::launch_skinny<1, 1, 16, true>(Qx, sx, Ti, K, Qw_tiled, sw, N, Yh, ldy, acc_dbg, st);
}

extern "C" sq_status sq_w4a4_gemm(const uint8_t *Qx, const float *sx, int64_t T, int32_t K,
                                  const uint8_t *Qw, const float *sw, int32_t N, void *Y,
                                  int64_t ldy, int32_t *acc_dbg, void *stream)
{
    if (T < 0 || N < 0 || K <= 0 || (K % 32) != 0 || K > SQ_GEMM_MAX_K) return SQ_ERR_SHAPE;
    if (T > (1 << 24) || ldy < N) return SQ_ERR_SHAPE;
    if (T == 0 || N == 0) return SQ_OK;
    if (!Qx || !sx || !Qw || !sw || !Y) return SQ_ERR_NULL;
    if (((uintptr_t)Qx & 15) || ((uintptr_t)Qw & 15) || ((uintptr_t)Y & 1) ||
        ((uintptr_t)sx & 3) || ((uintptr_t)sw & 3) || ((uintptr_t)acc_dbg & 3))
        return SQ_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    __half *Yh = static_cast<__half *>(Y);
    if ((K % 256) != 0) return sq::launch_generic(Qx, sx, (int)T, K, Qw, sw, N, Yh, ldy, acc_dbg, st);
    // Kernel choice, from few tokens to many.  The two large tile shapes run eight waves per CU
    // (two per SIMD): the VALU work of widening nibbles issues nearly twice as fast from two waves
    // as from one.  256x256 tiles (64x128 per wave: fewer VALU ops per MFMA) or 128x256 tiles,
    // whichever needs less time for its rounds over the CUs.  The debug option SQ_DEBUG_GEMM_LAUNCH_SHAPE (case number
    // below plus one) overrides the choice.
    const int forced = sq::debug_option(SQ_DEBUG_GEMM_LAUNCH_SHAPE) - 1;
    const int Ti = (int)T;
    int choice = forced;
    // At most 64 tokens: one pass over the weights by the decode-shaped kernel; its launch shape
    // (token blocks, channels per workgroup, K split) keeps about eight waves on every CU.
    // From 33 tokens on (17 with very many channels) and 10240 channels on, 64x64 / 64x128 tiles of
    // the tile kernel are faster than its token blocks (T = 64, K = 8192, N = 28672: 48.7 -> 32.2 us).
    // With at most 256 tiles (one per CU) the tile kernel's two-K-group form is faster still: eight
    // waves per CU, each walking half of K (T = 64, K = N = 8192: 18.3 -> 16.7 us; T = 64, K = 8192,
    // N = 28672: 31.2 -> 28.9 us).  It needs K % 512 == 0.
    const bool two_k_groups = (K % 512) == 0;
    if (choice < 0 && Ti > 32 && Ti <= 64 && N >= 8192 && N <= 64 * 256 && two_k_groups) choice = 14;
    // The same two tile forms win below 33 tokens as well where their tiles number 192 .. 256 (nearly one
    // per CU) and K is long: with 24576 .. 32768 channels and K >= 8192 the 64x128 tiles with two K groups
    // take 25.5 - 26.3 us for 1 .. 32 tokens at N = 28672 (the decode-shaped kernel 27.2 - 28.6 us up to 16
    // tokens, 64x64 tiles 29.6 - 32.0 us from 17 on; at K = 4096 all are within 0.5 us); with 10240 .. 16384
    // channels and 17 .. 32 tokens the 64x64 tiles with two K groups (T = 32, K = 4096, N = 14336: 10.7 -> 10.0 us).
    if (choice < 0 && Ti <= 32 && N >= 64 * 384 && N <= 128 * 256 && two_k_groups && K >= 8192) choice = 15;
    if (choice < 0 && Ti > 16 && Ti <= 32 && N >= 10240 && N <= 64 * 256 && two_k_groups) choice = 14;
    if (choice < 0 && Ti <= 64 && N >= 10240 && (Ti > 32 || (Ti > 16 && N >= 64 * 384))) {
        choice = (N >= 64 * 384 && Ti > 32) ? 11 : 10;
        if (choice == 11 && N <= 128 * 256 && two_k_groups) choice = 15;
    }
    // (with the token rows in LDS -- they fit up to 64 KB -- eight waves on 32 channels beat four waves on 64:
    // T = 8, K = 8192, N = 28672 27.1 against 27.4 us, and 27.6 us for the latter without the rows in LDS)
    const bool rows_fit_lds = (int64_t)Ti * (K / 2 + sq::kSkinnyRowPad) <= 64 * 1024;
    if (choice < 0 && Ti <= 32) choice = (N >= 64 * 384 && !rows_fit_lds) ? 8 : (N >= 10240 ? 9 : 7);
    if (choice < 0 && Ti <= 64) choice = 13;
    // Few tokens times few output channels: even 128x128 tiles would be too few for 256 CUs, and the
    // time is one workgroup's walk over K.  64x64 tiles (four times as many workgroups) up to 64
    // tiles of 128x128, 64x128 tiles up to 128.  (T = 128, K = N = 4096: 19.9 -> 14.6 us.)
    if (choice < 0) {
        const int64_t n128 = (int64_t)((Ti + 127) / 128) * ((N + 127) / 128);
        if (n128 <= 64) choice = two_k_groups ? 14 : 10;          // T = 200, K = N = 4096: 13.3 -> 11.6 us
        else if (n128 <= 128) choice = two_k_groups ? 15 : 11;    // T = 384, K = N = 4096: 16.8 -> 15.5 us
    }
    // Up to a few hundred tokens 128x256 tiles would leave CUs idle: 128x128 tiles (four waves).
    if (choice < 0) {
        const int64_t wide = (int64_t)((Ti + 127) / 128) * ((N + 255) / 256);
        if (wide <= 128) choice = (2 * wide <= 256) ? 5 : 2;
    }
    // 128x256 or 256x256 tiles: one workgroup per CU either way, so the time goes with the number
    // of rounds of 256 tiles; a 256x256 tile takes about 1.8 times as long as a 128x256 one (twice
    // the work at a slightly better rate).  Measured with random codes on shapes from 1024 x 11008
    // to 8192 x 28672.
    if (choice < 0) {
        const int64_t n_small = (int64_t)((Ti + 127) / 128) * ((N + 255) / 256);
        const int64_t n_large = (int64_t)((Ti + 255) / 256) * ((N + 255) / 256);
        const int64_t rounds_small = (n_small + 255) / 256, rounds_large = (n_large + 255) / 256;
        // (the 128x256 tile with four loading waves.  Case 16, eight multiplying waves of 64x64: attn_proj
        // 32.0 -> 31.5 us, mlp_down 74.5 -> 73.4 us against case 1, the same tile with the loads in the
        // multiplying waves.  Case 17, four multiplying waves of 64x128 -- half the widening per MFMA, and
        // the four loading waves keep eight waves on the CU: attn_proj 31.0 -> 30.7 us, mlp_down 72.2 -> 68.8 us
        // against case 16 for the GEMM alone; without loading waves that wave shape, case 0, is slower than
        // both.  Behind the rotate kernel, as a layer, attn_proj is 0.3 us slower with it (41.5 -> 41.8 us) and
        // mlp_down 2.2 us faster (98.6 -> 96.4 us): its gain grows with the number of K tiles, 16 against 43
        // here, and turns positive at about 20 of them.)
        choice = (20 * rounds_small > 37 * rounds_large) ? 4 : (K >= 6144 ? 17 : 16);
    }
    switch (choice) {
        case 0: return sq::launch_main<2, 2, 2, 4, 128, 1>(Qx, sx, Ti, K, Qw, sw, N, Yh, ldy, acc_dbg, st);
        case 2: return sq::launch_main<2, 2, 2, 2, 64, 2>(Qx, sx, Ti, K, Qw, sw, N, Yh, ldy, acc_dbg, st);
        case 3: return sq::launch_main<2, 2, 4, 4, 64, 1>(Qx, sx, Ti, K, Qw, sw, N, Yh, ldy, acc_dbg, st);
        case 4: return sq::launch_main<4, 2, 2, 4, 64, 1>(Qx, sx, Ti, K, Qw, sw, N, Yh, ldy, acc_dbg, st);
        case 5: return sq::launch_main<2, 2, 2, 2, 128, 1>(Qx, sx, Ti, K, Qw, sw, N, Yh, ldy, acc_dbg, st);
        case 6: return sq::launch_main<2, 4, 2, 2, 64, 1>(Qx, sx, Ti, K, Qw, sw, N, Yh, ldy, acc_dbg, st);
        case 10: return sq::launch_main<2, 2, 1, 1, 128, 2>(Qx, sx, Ti, K, Qw, sw, N, Yh, ldy, acc_dbg, st);
        case 11: return sq::launch_main<2, 2, 1, 2, 128, 2>(Qx, sx, Ti, K, Qw, sw, N, Yh, ldy, acc_dbg, st);
        case 16: return sq::launch_main<2, 4, 2, 2, 128, 1, 1, 3, 4>(Qx, sx, Ti, K, Qw, sw, N, Yh, ldy, acc_dbg, st);
        case 17: return sq::launch_main<2, 2, 2, 4, 128, 1, 1, 3, 4>(Qx, sx, Ti, K, Qw, sw, N, Yh, ldy, acc_dbg, st);
        case 14: if (K % 512 == 0) return sq::launch_main<2, 2, 1, 1, 128, 1, 2>(Qx, sx, Ti, K, Qw, sw, N, Yh, ldy, acc_dbg, st); break;
        case 15: if (K % 512 == 0) return sq::launch_main<2, 2, 1, 2, 128, 1, 2>(Qx, sx, Ti, K, Qw, sw, N, Yh, ldy, acc_dbg, st); break;
        case 7: if (Ti <= 32) return sq::launch_skinny<1, 1, 16>(Qx, sx, Ti, K, Qw, sw, N, Yh, ldy, acc_dbg, st); break;
        case 8: if (Ti <= 32) return sq::launch_skinny<1, 2, 4>(Qx, sx, Ti, K, Qw, sw, N, Yh, ldy, acc_dbg, st); break;
        case 9: if (Ti <= 32) return sq::launch_skinny<1, 1, 8>(Qx, sx, Ti, K, Qw, sw, N, Yh, ldy, acc_dbg, st); break;
        case 13: if (Ti <= 64) return sq::launch_skinny<2, 1, 8>(Qx, sx, Ti, K, Qw, sw, N, Yh, ldy, acc_dbg, st); break;
        default: break;
    }
    return sq::launch_main<2, 4, 2, 2, 128, 1>(Qx, sx, Ti, K, Qw, sw, N, Yh, ldy, acc_dbg, st);
}
