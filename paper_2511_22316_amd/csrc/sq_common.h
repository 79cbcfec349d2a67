// Internal helpers shared by the HIP translation units of libsinglequant (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

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

// Workgroup id -> logical work item such that each XCD (which owns one L2) receives a contiguous
// range of logical ids.  Hardware deals workgroup i to XCD i % 8.
__device__ __forceinline__ int xcd_contiguous_id(int wg, int nwg)
{
    const int q = nwg / kNumXcd, r = nwg % kNumXcd;
    const int xcd = wg % kNumXcd, local = wg / kNumXcd;
    return xcd * q + (xcd < r ? xcd : r) + local;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

// gfx950 has 160 KiB of LDS per workgroup; HIP needs an opt-in above 64 KiB of dynamic LDS.
constexpr int kMaxDynamicLds = 160 * 1024 - 1024;

// Opt a kernel in to large dynamic LDS, once per (kernel, device).  Host side.
inline bool allow_large_lds(const void *kernel)
{
    return hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDynamicLds) ==
           hipSuccess;
}

}  // namespace sq
