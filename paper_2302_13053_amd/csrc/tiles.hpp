// Pieces shared by the MFMA kernels (dense transform and weight gradient).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kTileK = 16;    // K extent of one LDS tile

// Four consecutive floats starting at base[off], fetched without a branch: an
// element that is not wanted (or would be out of range) is fetched from base[0]
// instead; zero4 later replaces it by zero.  Keeping the replacement out of the
// load lets all loads of a K step stay in flight behind the MFMAs of the
// previous step.
//   VEC: the four are one aligned 16-byte load and are wanted all or none
template <bool VEC>
__device__ __forceinline__ void load4(const float* __restrict__ base, int64_t off, int wanted, float (&r)[4])
{
    if constexpr (VEC) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(base + (wanted >= 4 ? off : 0));
        r[0] = t.x; r[1] = t.y; r[2] = t.z; r[3] = t.w;
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) r[q] = base[q < wanted ? off + q : 0];
    }
}

template <bool VEC>
__device__ __forceinline__ void zero4(int wanted, float (&r)[4])
{
#pragma unroll
    for (int q = 0; q < 4; ++q) r[q] = (VEC ? wanted >= 4 : q < wanted) ? r[q] : 0.0f;
}

