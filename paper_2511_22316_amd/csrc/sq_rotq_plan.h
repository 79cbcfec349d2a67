// Launch-time plan for the Givens list (ART pairs, Sec. 4.1-4.2) of sq_rotate_quantize: it travels
// by value in the kernel-argument block.
#pragma once

#include <stdint.h>

#include "singlequant.h"

namespace sq {

constexpr int kRotqMaxSlots = 2 * SQ_MAX_GIVENS;   // distinct channels a list can touch
constexpr int kRotqMaxQSlots = 128;                // distinct q = channel % n2 the MFMA kernel repairs

// The list is regrouped into levels: a pair goes one level after the latest earlier pair that
// shares a channel with it.  Pairs of one level touch disjoint channels, and every dependency
// points to an earlier level, so applying level after level equals applying the list in order.
struct RotqPlan {
    int32_t n_slots;                          // touched channels
    int32_t n_levels;
    int32_t n_qslots;                         // distinct values of channel % n2 among them
    uint16_t chan[kRotqMaxSlots];             // slot -> channel
    uint8_t qslot[kRotqMaxSlots];             // slot -> index into qlist
    uint16_t qlist[kRotqMaxQSlots];           // q-slot -> q
    uint8_t level_begin[SQ_MAX_GIVENS + 1];   // pairs [level_begin[l], level_begin[l+1]) form level l
    uint8_t pair_i[SQ_MAX_GIVENS];            // slots of the pair, in level order
    uint8_t pair_j[SQ_MAX_GIVENS];
    uint8_t pair_level[SQ_MAX_GIVENS];        // level of the pair, 0xFF behind the end of the list
    float c[SQ_MAX_GIVENS];                   // cos, sin of the pair's angle
    float s[SQ_MAX_GIVENS];
    // the quantizer of Sec. 3.2: largest level 2^(bits-1) - 1 (7 for four bits) and the fraction
    // of the row maximum that maps to it (1 = no clipping).  Per call, not part of the list.
    float q_top;
    float clip;
    float q_div;                              // q_top / clip: the step is the row maximum divided by this
};

}  // namespace sq

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

namespace sq {

// Matrix-core kernel (sq_rotq_mfma.hip).  Returns false if it does not cover (n1, n2); otherwise
// launches on `st` and stores the launch status.
// prepared: R1 and R2 point at the operand fragments written by rotq_write_fragments, not at the
// matrices.
bool rotq_mfma_dispatch(const __half *X, int64_t ldx, int T, int n1, int n2, const RotqPlan &plan,
                        const __half *R1, const __half *R2, uint8_t *Q, float *scales, float *xrot,
                        hipStream_t st, sq_status *status, bool prepared = false);

// The same rotation with fp16 output and no quantizer (R1, R2 as they are).
bool rotq_mfma_dispatch_f16(const __half *X, int64_t ldx, int T, int n1, int n2, const RotqPlan &plan,
                            const __half *R1, const __half *R2, __half *xout, int64_t ldo, hipStream_t st,
                            sq_status *status);

// Shapes the matrix-core kernel covers, and its operand fragments of R1 / R2 in the order the
// lanes hold them (sizes in bytes; both multiples of 1024).
bool rotq_mfma_covers(int n1, int n2);
size_t rotq_fragment_bytes_r1(int n1);
size_t rotq_fragment_bytes_r2(int n2);
sq_status rotq_write_fragments(const __half *R1, int n1, const __half *R2, int n2, void *f1, void *f2,
                               hipStream_t st);

// The layer in one launch for a few tokens (sq_decode_layer.hip): shapes it is built for, and
// the launch.  F1 / F2: operand fragments of a prepared rotation; Qx / sx / ctr: the caller's
// workspace (codes, steps, four counters that are zero between launches).
bool decode_layer_covers(int n1, int n2);
sq_status decode_layer_dispatch(const __half *X, int64_t ldx, int T, int n1, int n2, const RotqPlan &plan,
                                const __half *F1, const __half *F2, uint8_t *Qx, float *sx, int *ctr,
                                const uint8_t *Qw, const float *sw, int N, __half *Y, int64_t ldy, hipStream_t st);

}  // namespace sq
