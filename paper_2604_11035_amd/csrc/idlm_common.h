// Shared host/device helpers of the ISD hot-path library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <float.h>
#include "../../include/idlm.h"
#include "../../include/idlm_debug.h"

#define IDLM_WAVE 64

namespace idlm {

constexpr float kLog2e = 1.4426950408889634f;

// Sums of exponentials are kept as z = sum 2^(l*log2e - r) against a reference exponent r that
// is the rounded fp32 product m*log2e of the slice's maximum m (0 for a slice that has only seen
// -inf, whose terms are then all exactly 0).  Contraction into fma is switched off where r is
// formed so that the same m always gives the same r.
__device__ __forceinline__ float ref_log2(float m)
{
#pragma clang fp contract(off)
    return (m == -INFINITY) ? 0.f : m * kLog2e;
}

// 2^x through the hardware instruction (inputs here are <= 0 or small; no denormal fix-ups).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Factor that re-expresses a sum kept against maximum m_old against the reference r_new >=
// ref_log2(m_old); an empty slice (m_old = -inf, z = 0) contributes nothing.
__device__ __forceinline__ float rescale_factor(float m_old, float r_new)
{
#pragma clang fp contract(off)
    return (m_old == -INFINITY) ? 0.f : fast_exp2(m_old * kLog2e - r_new);
}

__device__ __forceinline__ int wave_id() { return __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); }

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline int launch_status() { return hipGetLastError() == hipSuccess ? IDLM_OK : IDLM_ERR_LAUNCH; }

}  // namespace idlm
