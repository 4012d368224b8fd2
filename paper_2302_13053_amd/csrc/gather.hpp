// Device helpers shared by the gather kernels (aggregation forward and backward):
// row loads/stores of VEC floats per lane, wave reductions and lane broadcasts.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kLightWaves = 4;   // independent rows per workgroup in the light kernels
constexpr int kHeavyWaves = 8;   // cooperating waves per row in the heavy kernels
constexpr int kUnroll = 4;       // neighbours fetched per unrolled step

template <int VEC>
__device__ __forceinline__ void load_row(const float* p, float (&v)[VEC])
{
    if constexpr (VEC == 4) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else if constexpr (VEC == 2) {
        const f32x2 t = *reinterpret_cast<const f32x2*>(p);
        v[0] = t.x; v[1] = t.y;
    } else {
        v[0] = *p;
    }
}

// vec_ok: p allows one VEC-wide store; half_ok (VEC == 4 only): p is 8-byte aligned, two 8-byte stores — the
// aggregate half of a concatenated row of odd half-width (602 columns) starts 8 bytes into a 16-byte piece,
// and four scalar stores per lane cost six times the L2 write requests of one wide store
template <int VEC>
__device__ __forceinline__ void store_row(float* p, const float (&v)[VEC], int valid, bool vec_ok, bool half_ok = false)
{
    if constexpr (VEC == 4) {
        if (!vec_ok && half_ok && valid >= 4) {
            *reinterpret_cast<f32x2*>(p) = f32x2{v[0], v[1]};
            *reinterpret_cast<f32x2*>(p + 2) = f32x2{v[2], v[3]};
            return;
        }
    }
    if (vec_ok && valid >= VEC) {
        if constexpr (VEC == 4) {
            f32x4 t = {v[0], v[1], v[2], v[3]};
            *reinterpret_cast<f32x4*>(p) = t;
        } else if constexpr (VEC == 2) {
            f32x2 t = {v[0], v[1]};
            *reinterpret_cast<f32x2*>(p) = t;
        } else {
            *p = v[0];
        }
    } else {
#pragma unroll
        for (int k = 0; k < VEC; ++k)
            if (k < valid) p[k] = v[k];
    }
}

// data that is read once per pass (indices, row bookkeeping, running sums) is fetched with a
// non-temporal hint so that it does not push the reused feature rows out of L2
template <typename T>
__device__ __forceinline__ T ldg_stream(const T* p) { return __builtin_nontemporal_load(p); }

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) x = fmaxf(x, __shfl_xor(x, m, 64));
    return x;
}

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) x += __shfl_xor(x, m, 64);
    return x;
}

__device__ __forceinline__ int bcast_i(int x, int lane) { return __builtin_amdgcn_readlane(x, lane); }
__device__ __forceinline__ float bcast_f(float x, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), lane));
}

// sum over aligned groups of G neighbouring lanes (G a power of two): up to 16 lanes with DPP moves inside
// a row of 16, beyond that with cross-row shuffles
template <int G>
__device__ __forceinline__ float group_sum(float x)
{
    // butterfly over the G lanes of a head; every lane ends with the group's sum
    if constexpr (G >= 2) x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
    if constexpr (G >= 4) x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
    if constexpr (G >= 8) x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xF, 0xF, true));  // row_half_mirror
    if constexpr (G >= 16) x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x140, 0xF, 0xF, true)); // row_mirror
    if constexpr (G >= 32) x += __shfl_xor(x, 16, 64);
    if constexpr (G >= 64) x += __shfl_xor(x, 32, 64);
    return x;
}

// pick s[h] for a per-lane head index from per-head wave-uniform values
template <int HP>
__device__ __forceinline__ float select_head(const float (&s)[HP], int h)
{
    float r = s[0];
#pragma unroll
    for (int i = 1; i < HP; ++i) r = (h == i) ? s[i] : r;
    return r;
}

}  // namespace
