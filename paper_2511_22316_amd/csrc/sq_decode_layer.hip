// sq_decode_layer: the whole layer in one launch for a few tokens (decode).
//
// With T <= 32 tokens the layer is one pass over the weights (HBM-bound) behind a rotation that is
// pure latency: a handful of workgroups rotate and quantize one or two tokens each while the rest
// of the chip waits for the next launch.  Here both steps share a launch:
//   * blocks 0 .. groups-1 run the rotate + quantize body on token group `block`, publish codes
//     and steps in the caller's workspace (release: their XCD's L2 is written back) and count
//     themselves done;
//   * every block then takes the output channels [block BN, (block + 1) BN): the weights of its
//     first K slice are requested, it waits until all groups are done, reads the codes and runs
//     the decode-shaped GEMM loop (K split over the four waves, partial sums added through LDS);
//   * the last block clears the counters for the next launch once every block is past its wait.
// The waits are bounded: a block that has polled for about a second skips its channels and raises
// the error word instead.  That bound is also what stands behind the one assumption made here,
// that the blocks with the lowest indices are not dispatched after the others (every block of a
// decode-sized launch is resident at once anyway: two per CU, 512 on the chip).
// Device-wide atomics and cache maintenance are expensive on this part (eight L2s): a ticket per
// block instead of the block index cost 7 us and an exit count with acquire-release ordering 16 us
// of a 34 us layer, and even a single acquire load per block behind the last poll (one cache
// invalidation per block) 1.7 us.  What is left: one release per rotating block (its stores are
// written back before its count becomes visible), relaxed polls, reads of the codes and steps by
// agent-scope coherent loads behind the poll and the block barrier (they go to the point where the
// written-back data is, so no invalidation is needed), and one relaxed add per block that nobody
// waits for.
// The launch ramp of a second kernel, the drain between the two and the first weight latency are
// what is saved; the codes still go through memory (32 KB for 8 tokens of 8192 channels).
#include "sq_rotq_body.h"

#include "singlequant.h"


namespace sq {

namespace {

__device__ __forceinline__ void widen_codes(const uint4 w, v4i &first, v4i &second)
{
    const uint32_t m = 0xF0F0F0F0u;
    first = v4i{(int)((w.x << 4) & m), (int)(w.x & m), (int)((w.y << 4) & m), (int)(w.y & m)};
    second = v4i{(int)((w.z << 4) & m), (int)(w.z & m), (int)((w.w << 4) & m), (int)(w.w & m)};
}

// counters in the workspace: [0] token groups done, [1] workgroups past their wait, [3] error word
// (a wait gave up)
template <int N1, int N2, int QS_MAX, int FN>
__global__ __launch_bounds__(256, 2) void decode_layer_kernel(
    const __half *__restrict__ X, int64_t ldx, int T, RotqPlan plan, const __half *__restrict__ F1,
    const __half *__restrict__ F2, uint8_t *Qx, float *sx, int *__restrict__ ctr,
    const uint8_t *__restrict__ Qw, const float *__restrict__ sw, int N, __half *__restrict__ Y, int64_t ldy,
    int lds_main, int spin_limit, int sides)
{
    using S = RotqShape<N1, N2, 3, false>;
    constexpr int Kb = N1 * N2 / 2, NW = 4, BN = 32 * FN, SLICE = 128;
    static_assert(Kb % SLICE == 0, "whole slices of 256 codes");
    extern __shared__ uint4 smem_u4[];
    int *note = reinterpret_cast<int *>(reinterpret_cast<char *>(smem_u4) + lds_main);   // [0] gave up
    const int tid = threadIdx.x;

    const int block = blockIdx.x;
    const int groups = (T + S::TPP - 1) / S::TPP;

    if (block < groups) {
        rotate_quantize_mfma_body<N1, N2, QS_MAX, 3, false, true>(X, ldx, T, plan, F1, F2, Qx, sx, nullptr, block,
                                                                  groups, smem_u4, sides);
        // Every wave has waited for its own stores (the body ends on vmcnt(0)); behind the barrier one
        // release writes this XCD's L2 back before the count can be seen.
        __syncthreads();
        if (tid == 0) __hip_atomic_fetch_add(&ctr[0], 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }

    // ---- decode-shaped GEMM on channels [col0, col0 + BN) ----------------------------------------
    const int lane = tid & (kWave - 1), wave = tid / kWave, l32 = lane & 31, g = lane >> 5;
    const int col0 = block * BN;
    // The codes and steps were written by other workgroups of this launch, on other XCDs.  They
    // are read with agent-scope coherent loads (the sc1 form, which is what a relaxed agent-scope
    // atomic load compiles to, here 16 bytes wide through a buffer descriptor): such a load
    // cannot be served by a stale line of this XCD's caches, so nothing has to be invalidated.
    constexpr int kAgentCoherent = 16;                                    // cache-policy bit sc1
    const __amdgpu_buffer_rsrc_t qx_rsrc = __builtin_amdgcn_make_buffer_rsrc(Qx, 0, T * Kb, 0x00020000);
    const int a_off = min(l32, T - 1) * Kb + g * 64;                      // rows past the end: never stored
    const uint8_t *b_ptr[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j) b_ptr[j] = Qw + (int64_t)min(col0 + 32 * j + l32, N - 1) * Kb + g * 64;

    v16i acc[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0;

    uint4 ra[2][4], rb[2][FN][4];
    constexpr int slices = Kb / SLICE;
#define SQ_DECODE_FETCH_B(BUF, SL)                                                                   \
    do {                                                                                             \
        _Pragma("unroll") for (int j = 0; j < FN; ++j)                                               \
            _Pragma("unroll") for (int c = 0; c < 4; ++c)                                            \
                rb[BUF][j][c] = *reinterpret_cast<const uint4 *>(b_ptr[j] + (SL) * SLICE + 16 * c);  \
    } while (0)
#define SQ_DECODE_FETCH_A(BUF, SL)                                                                   \
    do {                                                                                             \
        _Pragma("unroll") for (int c = 0; c < 4; ++c)                                                \
            ra[BUF][c] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(            \
                qx_rsrc, a_off + (SL) * SLICE + 16 * c, 0, kAgentCoherent));                        \
    } while (0)
#define SQ_DECODE_MULTIPLY(BUF)                                                                      \
    do {                                                                                             \
        _Pragma("unroll") for (int c = 0; c < 4; ++c) {                                              \
            v4i a0, a1;                                                                              \
            widen_codes(ra[BUF][c], a0, a1);                                                         \
            _Pragma("unroll") for (int j = 0; j < FN; ++j) {                                         \
                v4i b0, b1;                                                                          \
                widen_codes(rb[BUF][j][c], b0, b1);                                                  \
                acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b0, acc[j], 0, 0, 0);             \
                acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1, acc[j], 0, 0, 0);             \
            }                                                                                        \
        }                                                                                            \
    } while (0)

    // Wave w takes slices w, w+NW, ...; the weights of its first slice leave before the wait.  A block
    // that does not rotate holds them back for about 1.5 us, so that the first loads of the rotating
    // blocks (token rows, list, fragments) do not queue behind 14 MB of weights.
    int sl = wave;
    if (block >= groups) __builtin_amdgcn_s_sleep(60);
    if (sl < slices) SQ_DECODE_FETCH_B(0, sl);

    if (tid == 0) {
        int spins = 0, gave_up = 0;
        while (__hip_atomic_load(&ctr[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < groups) {
            if (++spins > spin_limit) {
                gave_up = 1;
                __hip_atomic_store(&ctr[3], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(8);
        }
        note[0] = gave_up;
    }
    __syncthreads();
    const bool gave_up = note[0] != 0;

    if (!gave_up && sl < slices) SQ_DECODE_FETCH_A(0, sl);
    // This block no longer looks at the count.  No value comes back and the add is queued behind the
    // loads just issued, so nothing waits for it; the loads behind it are not needed for a while.
    if (tid == 0) __hip_atomic_fetch_add(&ctr[1], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (!gave_up) {
        while (sl < slices) {
            if (sl + NW < slices) {
                SQ_DECODE_FETCH_B(1, sl + NW);
                SQ_DECODE_FETCH_A(1, sl + NW);
            }
            SQ_DECODE_MULTIPLY(0);
            sl += NW;
            if (sl >= slices) break;
            if (sl + NW < slices) {
                SQ_DECODE_FETCH_B(0, sl + NW);
                SQ_DECODE_FETCH_A(0, sl + NW);
            }
            SQ_DECODE_MULTIPLY(1);
            sl += NW;
        }

        // partial sums of the four waves through LDS (the rotation's tiles are dead by now)
        int *red = reinterpret_cast<int *>(smem_u4);         // [NW][FN][16][64]
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) red[((wave * FN + j) * 16 + e) * kWave + lane] = acc[j][e];
        __syncthreads();
        // accumulator layout: lane holds channel (lane % 32); register e holds token
        // 8 * (e / 4) + 4 * (lane / 32) + e % 4.  The sums carry the factor 256 of the widening.
        for (int idx = tid; idx < FN * 16 * kWave; idx += NW * kWave) {
            const int ln = idx & (kWave - 1), e = (idx >> 6) & 15, j = idx >> 10;
            int sum = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) sum += red[((w * FN + j) * 16 + e) * kWave + ln];
            const int t = 8 * (e / 4) + 4 * (ln >> 5) + (e % 4), n = col0 + 32 * j + (ln & 31);
            if (t < T && n < N) {
                const float sxt = __hip_atomic_load(&sx[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                Y[(int64_t)t * ldy + n] = __float2half_rn((float)sum * (sxt * 0.00390625f) * sw[n]);
            }
        }
    }
#undef SQ_DECODE_FETCH_A
#undef SQ_DECODE_FETCH_B
#undef SQ_DECODE_MULTIPLY

    // The last block makes the counters ready for the next launch, once every workgroup is past its
    // wait (they all were long ago when this block has finished its channels; the wait is bounded
    // like the other one).
    if (block == (int)gridDim.x - 1 && tid == 0) {
        int spins = 0;
        while (__hip_atomic_load(&ctr[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < (int)gridDim.x) {
            if (++spins > spin_limit) {
                __hip_atomic_store(&ctr[3], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(8);
        }
        __hip_atomic_store(&ctr[0], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&ctr[1], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <int N1, int N2, int QS_MAX, int FN>
sq_status launch_decode_layer(const __half *X, int64_t ldx, int T, const RotqPlan &plan, const __half *F1,
                              const __half *F2, uint8_t *Qx, float *sx, int *ctr, const uint8_t *Qw,
                              const float *sw, int N, __half *Y, int64_t ldy, hipStream_t st)
{
    using S = RotqShape<N1, N2, 3, false>;
    constexpr int BN = 32 * FN;
    // the rotation's tiles, then the partial sums
    const int qsteps = (plan.n_qslots + 15) / 16, sides = S::side_tiles(qsteps, 2);
    const int rot_lds = S::lds_bytes(qsteps, sides), red_lds = 4 * FN * 16 * kWave * 4;
    const int lds_main = ((rot_lds > red_lds ? rot_lds : red_lds) + 15) / 16 * 16;
    const int lds = lds_main + 16;
    if (lds > kMaxDynamicLds) return SQ_ERR_SHAPE;
    auto kernel = decode_layer_kernel<N1, N2, QS_MAX, FN>;
    if (!allow_large_lds(reinterpret_cast<const void *>(kernel))) return SQ_ERR_LAUNCH;
    const int tiles = (N + BN - 1) / BN, groups = (T + S::TPP - 1) / S::TPP;
    // every token group needs a block
    if (tiles < groups) return SQ_ERR_SHAPE;
    // about a second of polling before a workgroup gives up; the debug option SQ_DEBUG_DECODE_SPIN_LIMIT
    // sets another bound (test aid: the give-up path with a workspace whose "done" counter can never
    // be reached)
    const int option = debug_option(SQ_DEBUG_DECODE_SPIN_LIMIT);
    const int spin_limit = option > 0 ? option : (1 << 20);
    hipLaunchKernelGGL(kernel, dim3((unsigned)tiles), dim3(256), lds, st, X, ldx, T, plan, F1, F2, Qx, sx, ctr, Qw, sw,
                       N, Y, ldy, lds_main, spin_limit, sides);
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

}  // namespace

bool decode_layer_covers(int n1, int n2)
{
    return (n1 == 16 && n2 == 32) || (n1 == 32 && n2 == 32) || (n1 == 32 && n2 == 64) || (n1 == 64 && n2 == 64) ||
           (n1 == 64 && n2 == 128);
}

sq_status decode_layer_dispatch(const __half *X, int64_t ldx, int T, int n1, int n2, const RotqPlan &plan,
                                const __half *F1, const __half *F2, uint8_t *Qx, float *sx, int *ctr,
                                const uint8_t *Qw, const float *sw, int N, __half *Y, int64_t ldy, hipStream_t st)
{
    // two channel blocks per wave from 16384 channels on (then there are at least 256 workgroups)
    const bool wide = N >= 16384;
#define SQ_DECODE_CASE(N1, N2, QS)                                                                   \
    if (n1 == N1 && n2 == N2 && plan.n_qslots <= 16 * QS)                                            \
        return wide ? launch_decode_layer<N1, N2, QS, 2>(X, ldx, T, plan, F1, F2, Qx, sx, ctr, Qw, sw, N, Y, ldy, st) \
                    : launch_decode_layer<N1, N2, QS, 1>(X, ldx, T, plan, F1, F2, Qx, sx, ctr, Qw, sw, N, Y, ldy, st);
    SQ_DECODE_CASE(16, 32, 4)
    SQ_DECODE_CASE(32, 32, 4)
    SQ_DECODE_CASE(32, 64, 4)
    SQ_DECODE_CASE(64, 64, 4)
    SQ_DECODE_CASE(64, 128, 4)
    SQ_DECODE_CASE(64, 128, 8)
#undef SQ_DECODE_CASE
    return SQ_ERR_SHAPE;
}

}  // namespace sq
