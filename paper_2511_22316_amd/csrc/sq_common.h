// Internal helpers shared by the HIP translation units of libsinglequant (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include <mutex>
#include <utility>
#include <vector>

#include "singlequant.h"

namespace sq {

constexpr int kWave = 64;       // CDNA wavefront
constexpr int kNumXcd = 8;      // MI355X: 8 XCDs, workgroups are dealt to them round-robin

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));

// Givens list as it travels in the kernel-argument block: cos/sin evaluated in double on the
// host and rounded once to fp32 (Sec. 4.1; action formula of App. A.3).
struct GivensList {
    int32_t count;
    int32_t i[SQ_MAX_GIVENS];
    int32_t j[SQ_MAX_GIVENS];
    float c[SQ_MAX_GIVENS];
    float s[SQ_MAX_GIVENS];
};

// Current value of a debug option of singlequant.h (0 = the library decides).
int32_t debug_option(sq_debug_option option);

// Workgroup id -> logical work item such that each XCD (which owns one L2) receives a contiguous
// range of logical ids.  Hardware deals workgroup i to XCD i % 8.
__device__ __forceinline__ int xcd_contiguous_id(int wg, int nwg)
{
    const int q = nwg / kNumXcd, r = nwg % kNumXcd;
    const int xcd = wg % kNumXcd, local = wg / kNumXcd;
    return xcd * q + (xcd < r ? xcd : r) + local;
}

// Maximum of a non-negative value over the 64 lanes, returned in every lane.  Cross-lane steps
// use DPP modifiers (register-file speed) rather than LDS permutes.
__device__ __forceinline__ float wave_max(float v)
{
#define SQ_DPP_MAX(ctrl, row_mask)                                                                   \
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(                              \
                     0, __builtin_bit_cast(int, v), ctrl, row_mask, 0xF, false)))
    SQ_DPP_MAX(0xB1, 0xF);     // quad_perm [1,0,3,2]
    SQ_DPP_MAX(0x4E, 0xF);     // quad_perm [2,3,0,1]
    SQ_DPP_MAX(0x141, 0xF);    // row_half_mirror
    SQ_DPP_MAX(0x140, 0xF);    // row_mirror: every lane holds the maximum of its row of 16
    SQ_DPP_MAX(0x142, 0xA);    // row_bcast:15 into rows 1 and 3
    SQ_DPP_MAX(0x143, 0xC);    // row_bcast:31 into rows 2 and 3: lane 63 holds the wave maximum
#undef SQ_DPP_MAX
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// gfx950 has 160 KiB of LDS per workgroup; HIP needs an opt-in above 64 KiB of dynamic LDS.
constexpr int kMaxDynamicLds = 160 * 1024 - 1024;

// Opt a kernel in to large dynamic LDS, once per (kernel, device); later calls only look the pair
// up.  Host side, thread-safe.
inline bool allow_large_lds(const void *kernel)
{
    static std::mutex guard;
    static std::vector<std::pair<const void *, int>> done;
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return false;
    std::lock_guard<std::mutex> lock(guard);
    for (const auto &d : done)
        if (d.first == kernel && d.second == device) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDynamicLds) != hipSuccess)
        return false;
    done.emplace_back(kernel, device);
    return true;
}

}  // namespace sq
