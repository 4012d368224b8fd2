// Aggregation over a feature table kept in 16-bit storage (bfloat16 or IEEE half).
//
// The aggregation is bound by the bytes it gathers (one row of Z per CSR entry),
// so a table stored in 16 bits moves half of them.  This is a variant outside
// the fp32 results: the stored value is the float32 value rounded to nearest
// even in the target format (retexo_store_rows), every sum is still accumulated
// in float32 and the output is float32.  Against the same rounded table the
// result obeys the same 1e-5 bound as the fp32 path; against the unrounded
// table the difference is the rounding of the storage format.
//
// Kernels (each decodes 16-byte loads of eight elements per lane):
//   * whole rows per wave, for sum / mean / gcn_sym / max        (any shape; scalar loads when unaligned)
//   * 64-column slabs, one row per 8-lane group, walked source range by source range so that the
//     slab of the current range stays in L2 (dense graphs; same plan split as the fp32 path)
//   * edge softmax, whole rows per wave, software-pipelined with per-edge weights in LDS
#include "common.hpp"
#include "gather.hpp"

namespace {

enum { FMT_BF16 = RETEXO_STORE_BF16, FMT_FP16 = RETEXO_STORE_FP16 };

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));    // sixteen bytes of stored elements, kept as integers
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int FMT>
__device__ __forceinline__ float decode1(uint16_t x)
{
    if constexpr (FMT == FMT_BF16) {
        return __uint_as_float((uint32_t)x << 16);
    } else {
        _Float16 h;
        __builtin_memcpy(&h, &x, 2);
        return (float)h;
    }
}

// eight stored elements (16 bytes) -> floats
template <int FMT>
__device__ __forceinline__ void decode8(const u32x4& raw, float (&v)[8])
{
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if constexpr (FMT == FMT_BF16) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        } else {
            v[2 * i] = decode1<FMT>((uint16_t)(w[i] & 0xffffu));
            v[2 * i + 1] = decode1<FMT>((uint16_t)(w[i] >> 16));
        }
    }
}

template <int FMT>
__device__ __forceinline__ uint16_t encode1(float x)
{
    if constexpr (FMT == FMT_BF16) {
        const uint32_t b = __float_as_uint(x);
        if (x != x) return (uint16_t)((b >> 16) | 0x0040u);                   // NaN stays NaN (quiet)
        return (uint16_t)((b + 0x7fffu + ((b >> 16) & 1u)) >> 16);            // nearest, ties to even
    } else {
        const _Float16 h = (_Float16)x;                                       // hardware conversion: nearest even
        uint16_t r;
        __builtin_memcpy(&r, &h, 2);
        return r;
    }
}

template <int FMT>
__global__ __launch_bounds__(256) void store_rows_kernel(int64_t N, int64_t F, const float* __restrict__ src,
                                                          int64_t lds, uint16_t* __restrict__ dst, int64_t ldd)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= N * F) return;
    const int64_t r = i / F, c = i % F;
    dst[r * ldd + c] = encode1<FMT>(src[r * lds + c]);
}

// row loads of E stored elements per lane (E = 8: one 16-byte load; 4: one 8-byte load; 1: one 2-byte load)
template <int FMT, int E>
__device__ __forceinline__ void load_stored(const uint16_t* p, float (&v)[E])
{
    if constexpr (E == 8) {
        const u32x4 raw = *reinterpret_cast<const u32x4*>(p);
        decode8<FMT>(raw, v);
    } else if constexpr (E == 4) {
        const u32x2 raw = *reinterpret_cast<const u32x2*>(p);
        const uint32_t w[2] = {raw.x, raw.y};
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if constexpr (FMT == FMT_BF16) {
                v[2 * i] = __uint_as_float(w[i] << 16);
                v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
            } else {
                v[2 * i] = decode1<FMT>((uint16_t)(w[i] & 0xffffu));
                v[2 * i + 1] = decode1<FMT>((uint16_t)(w[i] >> 16));
            }
        }
    } else {
        v[0] = decode1<FMT>(*p);
    }
}

// vec_ok: 16-byte stores; half_ok: p is at least 8-byte aligned (the aggregate half of a concatenated row of odd
// half-width): 8-byte stores instead of one per element
template <int E>
__device__ __forceinline__ void store_floats(float* p, const float (&v)[E], int valid, bool vec_ok, bool half_ok = false)
{
    if (E % 2 == 0 && !vec_ok && half_ok && valid >= E) {
#pragma unroll
        for (int k = 0; k < E; k += 2) *reinterpret_cast<f32x2*>(p + k) = f32x2{v[k], v[k + 1 < E ? k + 1 : k]};
        return;
    }
    if (E == 8 && vec_ok && valid >= 8) {
        const f32x4 a = {v[0], v[1], v[2], v[3]}, b = {v[E > 4 ? 4 : 0], v[E > 5 ? 5 : 0], v[E > 6 ? 6 : 0], v[E > 7 ? 7 : 0]};
        *reinterpret_cast<f32x4*>(p) = a;
        *reinterpret_cast<f32x4*>(p + 4) = b;
    } else if (E == 4 && vec_ok && valid >= 4) {
        const f32x4 a = {v[0], v[E > 1 ? 1 : 0], v[E > 2 ? 2 : 0], v[E > 3 ? 3 : 0]};
        *reinterpret_cast<f32x4*>(p) = a;
    } else {
#pragma unroll
        for (int k = 0; k < E; ++k)
            if (k < valid) p[k] = v[k];
    }
}

struct StoredArgs {
    const int64_t* row_ptr;
    const int32_t* col_idx;
    const int32_t* order;
    const int32_t* deg;
    const float* dinv;
    const float* wsrc;       // per-source weights (gcn_sym: dinv) or NULL
    const uint16_t* Z;
    int64_t ldz;             // in elements
    float* out;
    int64_t ldo;
    int64_t ocol;
    const float* el;
    const float* er;
    int64_t row_begin, row_count;
    int64_t F;
    int nslab;
    int scale;               // 0 sum, 1 mean, 2 gcn
    int heads, Dh;
    float slope;
    int copy_self;
    int out_vec;             // aggregate half of out allows 16-byte stores
    int out_half;            // ... or at least 8-byte stores
    int self_vec;
    const int32_t* part_ptr;
    int64_t n_rows;
    int part_lo, part_hi;
    int first, last;
};

// ---------------------------------------------------------------------------
// sum / mean / gcn_sym / max, whole rows: one wave per (row, slab of 64*E*NC columns)
// ---------------------------------------------------------------------------
template <int FMT, int E, int NC, int NW, bool MAXOP>
__global__ __launch_bounds__(64 * (NW == 1 ? kLightWaves : NW)) void stored_linear_kernel(StoredArgs a)
{
    constexpr int U = E == 8 ? 2 : kUnroll;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t items = a.row_count * a.nslab;
    const int64_t item = (NW == 1) ? (int64_t)blockIdx.x * kLightWaves + wave : (int64_t)blockIdx.x;
    if (item >= items) return;
    const int64_t slot = item / a.nslab;
    const int slab = (int)(item % a.nslab);
    const int v = __builtin_amdgcn_readfirstlane(a.order[a.row_begin + slot]);
    const int lo = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v]);
    const int hi = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v + 1]);

    const int64_t col0 = (int64_t)slab * (64 * E * NC) + lane * E;
    bool act[NC];
    int64_t colsafe[NC];
    float acc[NC][E];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int64_t col = col0 + c * 64 * E;
        act[c] = col < a.F;
        colsafe[c] = act[c] ? col : 0;        // lanes past the row width gather column 0 (never stored)
#pragma unroll
        for (int k = 0; k < E; ++k) acc[c][k] = MAXOP ? -INFINITY : 0.0f;
    }
    const bool weighted = a.wsrc != nullptr;

    for (int base = lo + 64 * (NW == 1 ? 0 : wave); base < hi; base += 64 * NW) {
        const int e = base + lane;
        const bool valid = e < hi;
        int my_u = valid ? a.col_idx[e] : 0;
        my_u = valid ? my_u : bcast_i(my_u, 0);
        const float my_w = weighted ? (valid ? a.wsrc[my_u] : 0.0f) : (valid ? 1.0f : 0.0f);
        const int cnt = min(64, hi - base);
        for (int j = 0; j < cnt; j += U) {
            float z[U][NC][E], w[U];
#pragma unroll
            for (int t = 0; t < U; ++t) {
                const int jj = (j + t) & 63;                        // past the tile: a repeat with weight zero
                const uint16_t* zr = a.Z + (int64_t)bcast_i(my_u, jj) * a.ldz;
                w[t] = j + t < cnt ? bcast_f(my_w, jj) : 0.0f;
#pragma unroll
                for (int c = 0; c < NC; ++c) load_stored<FMT, E>(zr + colsafe[c], z[t][c]);
            }
#pragma unroll
            for (int t = 0; t < U; ++t)
#pragma unroll
                for (int c = 0; c < NC; ++c)
#pragma unroll
                    for (int k = 0; k < E; ++k) {
                        if constexpr (MAXOP) acc[c][k] = j + t < cnt ? fmaxf(acc[c][k], z[t][c][k]) : acc[c][k];
                        else acc[c][k] = fmaf(w[t], z[t][c][k], acc[c][k]);
                    }
        }
    }

    if constexpr (NW > 1) {
        __shared__ float red[NW][NC * E][64];
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int k = 0; k < E; ++k) red[wave][c * E + k][lane] = acc[c][k];
        __syncthreads();
        if (wave != 0) return;
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int k = 0; k < E; ++k) {
                float s = red[0][c * E + k][lane];
#pragma unroll
                for (int w = 1; w < NW; ++w) s = MAXOP ? fmaxf(s, red[w][c * E + k][lane]) : s + red[w][c * E + k][lane];
                acc[c][k] = s;
            }
    }

    const int d = hi - lo;
    float* orow = a.out + (int64_t)v * a.ldo;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        if (!act[c]) continue;
        const int64_t col = col0 + c * 64 * E;
        const int valid = (int)min((int64_t)E, a.F - col);
        float r[E];
#pragma unroll
        for (int k = 0; k < E; ++k) {
            float x = acc[c][k];
            if (MAXOP) x = d > 0 ? x : 0.0f;
            else if (a.scale == 1) x = d > 0 ? x / (float)d : 0.0f;
            else if (a.scale == 2) x = x * a.dinv[v];
            r[k] = x;
        }
        store_floats<E>(orow + a.ocol + col, r, valid, a.out_vec != 0, a.out_half != 0);
        if (a.copy_self) {
            float zs[E];
            load_stored<FMT, E>(a.Z + (int64_t)v * a.ldz + col, zs);
            store_floats<E>(orow + col, zs, valid, a.self_vec != 0);
        }
    }
}

// ---------------------------------------------------------------------------
// sum / mean / gcn_sym on 64-column slabs: one row per 8-lane group, eight elements per lane, so a
// gathered row-slab is one 128-byte line.  Launched once per group of source-id ranges: the running
// sum is kept in `out` between launches.  Branch-free inner loop: lanes past the end of a row gather
// the row's first neighbour with weight zero.
// ---------------------------------------------------------------------------
template <int FMT, bool WEIGHTED>
__global__ __launch_bounds__(64 * kLightWaves) void stored_rowgroup_kernel(StoredArgs a)
{
    constexpr int LPG = 8, G = 64 / LPG, U = 8;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t bundles = (a.row_count + G - 1) / G;
    const int64_t item = (int64_t)blockIdx.x * kLightWaves + wave;
    if (item >= bundles * a.nslab) return;
    const int slab = (int)(item / bundles);                 // slab-major: neighbouring waves share a slab
    const int64_t bundle = item % bundles;

    const int li = lane % LPG, g = lane / LPG;
    const int64_t slot = bundle * G + g;
    const bool has_row = slot < a.row_count;
    int v = 0, lo = 0, hi = 0;
    if (has_row) {
        v = a.order[a.row_begin + slot];
        if (a.part_ptr) {
            lo = a.part_ptr[(int64_t)a.part_lo * a.n_rows + a.row_begin + slot];
            hi = a.part_ptr[(int64_t)a.part_hi * a.n_rows + a.row_begin + slot];
        } else {
            lo = (int)a.row_ptr[v];
            hi = (int)a.row_ptr[v + 1];
        }
    }
    const int len = hi - lo;
    int maxlen = len, minlen = len;
#pragma unroll
    for (int m = LPG; m < 64; m <<= 1) {
        maxlen = max(maxlen, __shfl_xor(maxlen, m, 64));
        minlen = min(minlen, __shfl_xor(minlen, m, 64));
    }
    maxlen = __builtin_amdgcn_readfirstlane(maxlen);
    minlen = __builtin_amdgcn_readfirstlane(minlen);

    const int64_t col = (int64_t)slab * 64 + li * 8;
    const bool act = col < a.F;
    const bool writer = act && has_row;
    const int valid = (int)min((int64_t)8, a.F - col);
    const int64_t gcol = act ? col : 0;
    const char* zbase = reinterpret_cast<const char*>(a.Z);
    const uint32_t colbytes = (uint32_t)(gcol * 2);
    const uint32_t rowbytes = (uint32_t)(a.ldz * 2);
    float* orow = a.out + (int64_t)v * a.ldo;

    float acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = 0.0f;
    if (!a.first && writer) {
        if (a.out_vec && valid >= 8) {
            const f32x4 p0 = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(orow + a.ocol + col));
            const f32x4 p1 = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(orow + a.ocol + col + 4));
            acc[0] = p0.x; acc[1] = p0.y; acc[2] = p0.z; acc[3] = p0.w;
            acc[4] = p1.x; acc[5] = p1.y; acc[6] = p1.z; acc[7] = p1.w;
        } else if (a.out_half && valid >= 8) {
#pragma unroll
            for (int k = 0; k < 8; k += 2) {
                const f32x2 t = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(orow + a.ocol + col + k));
                acc[k] = t.x;
                acc[k + 1] = t.y;
            }
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (k < valid) acc[k] = orow[a.ocol + col + k];
        }
    }

    const int gaddr = (lane - li) * 4;          // ds_bpermute byte address of this group's lane 0
    // Neighbour ids: every lane of a group fetches eight consecutive ids at a time, so a group reads col_idx in
    // whole cache lines (64 entries) a block ahead of its use; entry e of a block sits in component e % 8 of the
    // group's lane e / 8.  Past the end of a row: id 0 with weight zero.
    constexpr int IPL = 8, BLOCK = IPL * LPG;
    typedef int i32x4u __attribute__((ext_vector_type(4), aligned(4)));      // 4-byte aligned 16-byte load
    int nxt_u[IPL];
    float nxt_w[IPL];
    auto fetch_ids = [&](int first) {
        const int nb = first + IPL * li;
        if (nb + IPL <= len) {
#pragma unroll
            for (int k = 0; k < IPL; k += 4) {
                const i32x4u t = *reinterpret_cast<const i32x4u*>(a.col_idx + lo + nb + k);
                nxt_u[k] = t.x; nxt_u[k + 1] = t.y; nxt_u[k + 2] = t.z; nxt_u[k + 3] = t.w;
            }
        } else {
#pragma unroll
            for (int k = 0; k < IPL; ++k) nxt_u[k] = nb + k < len ? a.col_idx[lo + nb + k] : 0;
        }
#pragma unroll
        for (int k = 0; k < IPL; ++k) nxt_w[k] = nb + k < len ? (WEIGHTED ? a.wsrc[nxt_u[k]] : 1.0f) : 0.0f;
    };
    fetch_ids(0);
    for (int s0 = 0; s0 < maxlen; s0 += BLOCK) {
        uint32_t my_off[IPL];
        float my_w[IPL];
#pragma unroll
        for (int k = 0; k < IPL; ++k) {
            my_off[k] = (uint32_t)nxt_u[k] * rowbytes;
            my_w[k] = nxt_w[k];
        }
        fetch_ids(s0 + BLOCK);
#pragma unroll
        for (int q = 0; q < IPL; ++q) {
            const int c0 = s0 + q * LPG;
            if (c0 >= maxlen) break;                     // (uniform)
            const bool full = c0 + LPG <= minlen;        // every group still has LPG entries: nothing to mask
#pragma unroll
            for (int i0 = 0; i0 < LPG; i0 += U) {
                u32x4 raw[U];
                float w[U];
#pragma unroll
                for (int t = 0; t < U; ++t) {
                    const int e = q * LPG + i0 + t;
                    const uint32_t off =
                        (uint32_t)__builtin_amdgcn_ds_bpermute(gaddr + 4 * (e / IPL), (int)my_off[e % IPL]) + colbytes;
                    raw[t] = *reinterpret_cast<const u32x4*>(zbase + off);
                    w[t] = __int_as_float(__builtin_amdgcn_ds_bpermute(gaddr + 4 * (e / IPL), __float_as_int(my_w[e % IPL])));
                }
                if (!full) {
                    // entries past the end of this group's row gathered row 0: clear their bits (both formats
                    // decode zero bits to +0), so that nothing of an unrelated row can reach the sum
#pragma unroll
                    for (int t = 0; t < U; ++t) {
                        const uint32_t keep = c0 + i0 + t < len ? 0xffffffffu : 0u;
                        raw[t].x &= keep;
                        raw[t].y &= keep;
                        raw[t].z &= keep;
                        raw[t].w &= keep;
                    }
                }
#pragma unroll
                for (int t = 0; t < U; ++t) {
                    float z[8];
                    decode8<FMT>(raw[t], z);
#pragma unroll
                    for (int k = 0; k < 8; ++k) acc[k] = fmaf(w[t], z[k], acc[k]);
                }
            }
        }
    }
    if (!writer) return;
    const int d = (a.last && a.scale == 1) ? a.deg[v] : 0;      // only the mean's last range needs it
    float r[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float x = acc[k];
        if (a.last) {
            if (a.scale == 1) x = d > 0 ? x / (float)d : 0.0f;
            else if (a.scale == 2) x = x * a.dinv[v];
        }
        r[k] = x;
    }
    store_floats<8>(orow + a.ocol + col, r, valid, a.out_vec != 0, a.out_half != 0);
    if (a.copy_self && a.first) {
        float zs[8];
        load_stored<FMT, 8>(a.Z + (int64_t)v * a.ldz + col, zs);
        store_floats<8>(orow + col, zs, valid, a.self_vec != 0);
    }
}

// ---------------------------------------------------------------------------
// The same slabs for long rows: a workgroup of eight waves per (row, slab).  A wave reads 64
// consecutive entries of the row at a time; each of its eight 8-lane groups gathers the eight entries
// its own lanes hold.  Partial sums are combined across the groups of a wave by shuffles and across
// waves through LDS, in a fixed order.
// ---------------------------------------------------------------------------
template <int FMT, bool WEIGHTED>
__global__ __launch_bounds__(64 * kHeavyWaves) void stored_grouped_kernel(StoredArgs a)
{
    constexpr int LPG = 8, U = 8;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t item = blockIdx.x;                        // slab-major
    const int slab = (int)(item / a.row_count);
    const int64_t slot = item % a.row_count;
    const int v = a.order[a.row_begin + slot];
    int lo, hi;
    if (a.part_ptr) {
        lo = a.part_ptr[(int64_t)a.part_lo * a.n_rows + a.row_begin + slot];
        hi = a.part_ptr[(int64_t)a.part_hi * a.n_rows + a.row_begin + slot];
    } else {
        lo = (int)a.row_ptr[v];
        hi = (int)a.row_ptr[v + 1];
    }
    const int li = lane % LPG;
    const int64_t col = (int64_t)slab * 64 + li * 8;
    const bool act = col < a.F;
    const int valid = (int)min((int64_t)8, a.F - col);
    const char* zbase = reinterpret_cast<const char*>(a.Z);
    const uint32_t colbytes = (uint32_t)((act ? col : 0) * 2);
    const uint32_t rowbytes = (uint32_t)(a.ldz * 2);
    const int gaddr = (lane - li) * 4;

    float acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = 0.0f;
    for (int base = lo + 64 * wave; base < hi; base += 64 * kHeavyWaves) {
        const int e = base + lane;
        const bool ok = e < hi;
        const int my_u = ok ? a.col_idx[e] : 0;
        const float my_w = ok ? (WEIGHTED ? a.wsrc[my_u] : 1.0f) : 0.0f;
        const uint32_t my_off = (uint32_t)my_u * rowbytes;
        const bool full = base + 64 <= hi;
        u32x4 raw[U];
        float w[U];
#pragma unroll
        for (int t = 0; t < U; ++t) {
            const uint32_t off = (uint32_t)__builtin_amdgcn_ds_bpermute(gaddr + 4 * t, (int)my_off) + colbytes;
            raw[t] = *reinterpret_cast<const u32x4*>(zbase + off);
            w[t] = __int_as_float(__builtin_amdgcn_ds_bpermute(gaddr + 4 * t, __float_as_int(my_w)));
        }
        if (!full) {
#pragma unroll
            for (int t = 0; t < U; ++t) {
                const uint32_t keep = base + (lane - li) + t < hi ? 0xffffffffu : 0u;
                raw[t].x &= keep;
                raw[t].y &= keep;
                raw[t].z &= keep;
                raw[t].w &= keep;
            }
        }
#pragma unroll
        for (int t = 0; t < U; ++t) {
            float z[8];
            decode8<FMT>(raw[t], z);
#pragma unroll
            for (int k = 0; k < 8; ++k) acc[k] = fmaf(w[t], z[k], acc[k]);
        }
    }
    // the eight groups of a wave, then the eight waves
#pragma unroll
    for (int m = LPG; m < 64; m <<= 1)
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] += __shfl_xor(acc[k], m, 64);
    __shared__ float red[kHeavyWaves][LPG][8];
    if (lane < LPG) {
#pragma unroll
        for (int k = 0; k < 8; ++k) red[wave][lane][k] = acc[k];
    }
    __syncthreads();
    if (wave != 0 || lane >= LPG || !act) return;
    float* orow = a.out + (int64_t)v * a.ldo;
    float r[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float x = red[0][lane][k];
#pragma unroll
        for (int w = 1; w < kHeavyWaves; ++w) x += red[w][lane][k];
        if (!a.first && k < valid) x += orow[a.ocol + col + k];
        if (a.last) {
            const int d = (a.last && a.scale == 1) ? a.deg[v] : 0;      // only the mean's last range needs it
            if (a.scale == 1) x = d > 0 ? x / (float)d : 0.0f;
            else if (a.scale == 2) x = x * a.dinv[v];
        }
        r[k] = x;
    }
    store_floats<8>(orow + a.ocol + col, r, valid, a.out_vec != 0, a.out_half != 0);
    if (a.copy_self && a.first) {
        float zs[8];
        load_stored<FMT, 8>(a.Z + (int64_t)v * a.ldz + col, zs);
        store_floats<8>(orow + col, zs, valid, a.self_vec != 0);
    }
}

// ---------------------------------------------------------------------------
// attention scores from a stored table (one wave per node)
// ---------------------------------------------------------------------------
template <int FMT, int HP>
__global__ __launch_bounds__(256) void stored_scores_kernel(
    int64_t N, int64_t F, int Dh, const uint16_t* __restrict__ Z, int64_t ldz,
    const float* __restrict__ a_src, const float* __restrict__ a_dst, float* __restrict__ el, float* __restrict__ er)
{
    const int lane = threadIdx.x & 63;
    const int64_t v = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= N) return;
    float ps[HP], pd[HP];
#pragma unroll
    for (int h = 0; h < HP; ++h) { ps[h] = 0.0f; pd[h] = 0.0f; }
    for (int64_t c = lane; c < F; c += 64) {
        const float z = decode1<FMT>(Z[v * ldz + c]);
        const int h = (int)(c / Dh);
        const float s = z * a_src[c], t = z * a_dst[c];
#pragma unroll
        for (int i = 0; i < HP; ++i) {
            ps[i] += (h == i) ? s : 0.0f;
            pd[i] += (h == i) ? t : 0.0f;
        }
    }
#pragma unroll
    for (int h = 0; h < HP; ++h) {
        const float s = wave_sum(ps[h]), t = wave_sum(pd[h]);
        if (lane == 0) { el[v * HP + h] = s; er[v * HP + h] = t; }
    }
}

// The same scores with 8-byte loads: 16 lanes per node (four nodes per wave), each lane walks the row in steps
// of 64 columns, four stored elements at a time, all pieces of a row of up to 256 columns requested before the
// first is used; the per-head partial sums are reduced over the 16 lanes of a node.
// Needs 8-byte aligned rows, 16-byte aligned attention vectors and F % 4 == 0.
template <int FMT, int HP>
__global__ __launch_bounds__(256) void stored_scores_vec_kernel(
    int64_t N, int64_t F, int Dh, const uint16_t* __restrict__ Z, int64_t ldz,
    const float* __restrict__ a_src, const float* __restrict__ a_dst, float* __restrict__ el, float* __restrict__ er)
{
    const int li = threadIdx.x & 15;
    const int64_t v = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const bool have = v < N;
    const int64_t vv = have ? v : N - 1;                 // idle groups repeat the last node (nothing stored)
    const bool whole = Dh % 4 == 0;
    float ps[HP], pd[HP];
#pragma unroll
    for (int h = 0; h < HP; ++h) { ps[h] = 0.0f; pd[h] = 0.0f; }
    for (int64_t c0 = li * 4; c0 < F; c0 += 256) {
        float zq[4][4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int64_t c = c0 + 64 * q;
            if (c < F) load_stored<FMT, 4>(Z + vv * ldz + c, zq[q]);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int64_t c = c0 + 64 * q;
            if (c >= F) break;
            const f32x4 as = *reinterpret_cast<const f32x4*>(a_src + c);
            const f32x4 ad = *reinterpret_cast<const f32x4*>(a_dst + c);
            const float sa[4] = {as.x, as.y, as.z, as.w}, da[4] = {ad.x, ad.y, ad.z, ad.w};
            if (whole) {
                const int h = (int)c / Dh;
                const float s = ((zq[q][0] * sa[0] + zq[q][1] * sa[1]) + zq[q][2] * sa[2]) + zq[q][3] * sa[3];
                const float t = ((zq[q][0] * da[0] + zq[q][1] * da[1]) + zq[q][2] * da[2]) + zq[q][3] * da[3];
#pragma unroll
                for (int i = 0; i < HP; ++i) {
                    ps[i] += (h == i) ? s : 0.0f;
                    pd[i] += (h == i) ? t : 0.0f;
                }
                continue;
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int h = ((int)c + k) / Dh;
                const float s = zq[q][k] * sa[k], t = zq[q][k] * da[k];
#pragma unroll
                for (int i = 0; i < HP; ++i) {
                    ps[i] += (h == i) ? s : 0.0f;
                    pd[i] += (h == i) ? t : 0.0f;
                }
            }
        }
    }
#pragma unroll
    for (int h = 0; h < HP; ++h) {
#pragma unroll
        for (int m = 8; m >= 1; m >>= 1) {
            ps[h] += __shfl_xor(ps[h], m, 64);
            pd[h] += __shfl_xor(pd[h], m, 64);
        }
    }
    if (have && li == 0) {
#pragma unroll
        for (int h = 0; h < HP; ++h) { el[v * HP + h] = ps[h]; er[v * HP + h] = pd[h]; }
    }
}

// ---------------------------------------------------------------------------
// edge softmax over a stored table: whole rows per wave, online softmax at tile granularity, per-edge
// weights through wave-private LDS, next batch of rows requested before the current one is consumed.
//   HU: every lane's E columns lie inside one head (Dh % E == 0)
// ---------------------------------------------------------------------------
template <int FMT, int E, int NC, int NW, int HP, bool HU>
__global__ __launch_bounds__(64 * (NW == 1 ? kLightWaves : NW)) void stored_gat_kernel(StoredArgs a)
{
    constexpr int WAVES = NW == 1 ? kLightWaves : NW;
    constexpr int U = E * NC >= 16 ? 2 : 4;
    constexpr int Q = HU ? 1 : E;
    __shared__ float wl[WAVES][HP][64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t items = a.row_count * a.nslab;
    const int64_t item = (NW == 1) ? (int64_t)blockIdx.x * kLightWaves + wave : (int64_t)blockIdx.x;
    if (item >= items) return;
    const int64_t slot = item / a.nslab;
    const int slab = (int)(item % a.nslab);
    const int v = __builtin_amdgcn_readfirstlane(a.order[a.row_begin + slot]);
    const int lo = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v]);
    const int hi = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v + 1]);

    const int64_t col0 = (int64_t)slab * (64 * E * NC) + lane * E;
    bool act[NC];
    int64_t colsafe[NC];
    int hc[NC][Q];
    float acc[NC][E];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int64_t col = col0 + c * 64 * E;
        act[c] = col < a.F;
        colsafe[c] = act[c] ? col : 0;
#pragma unroll
        for (int k = 0; k < Q; ++k) hc[c][k] = min((int)((col + k) / a.Dh), a.heads - 1);
#pragma unroll
        for (int k = 0; k < E; ++k) acc[c][k] = 0.0f;
    }
    float* myw = &wl[wave][0][0];

    float m[HP], s[HP], erv[HP];
#pragma unroll
    for (int h = 0; h < HP; ++h) {
        m[h] = -INFINITY;
        s[h] = 0.0f;
        erv[h] = a.er[(int64_t)v * HP + h];
    }

    const int first = lo + 64 * (NW == 1 ? 0 : wave);
    for (int base = first; base < hi; base += 64 * NW) {
        const int e = base + lane;
        const bool valid = e < hi;
        const int cnt = min(64, hi - base);
        int my_u = valid ? a.col_idx[e] : 0;
        my_u = valid ? my_u : bcast_i(my_u, 0);

        float zq[U][NC][E];
#pragma unroll
        for (int t = 0; t < U; ++t) {
            const uint16_t* zr = a.Z + (int64_t)bcast_i(my_u, t) * a.ldz;
#pragma unroll
            for (int c = 0; c < NC; ++c) load_stored<FMT, E>(zr + colsafe[c], zq[t][c]);
        }
        float elu[HP], scale[HP];
        if constexpr (HP == 4) {
            const f32x4 t = *reinterpret_cast<const f32x4*>(a.el + (int64_t)my_u * 4);
            elu[0] = t.x; elu[1] = t.y; elu[2] = t.z; elu[3] = t.w;
        } else {
#pragma unroll
            for (int h = 0; h < HP; ++h) elu[h] = a.el[(int64_t)my_u * HP + h];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // earlier reads of wl are done
#pragma unroll
        for (int h = 0; h < HP; ++h) {
            const float x = elu[h] + erv[h];
            const float sc = valid ? (x > 0.0f ? x : a.slope * x) : -INFINITY;
            const float mn = fmaxf(m[h], wave_max(sc));
            scale[h] = expf(m[h] - mn);
            const float pe = valid ? expf(sc - mn) : 0.0f;
            s[h] = s[h] * scale[h] + wave_sum(pe);
            m[h] = mn;
            myw[h * 64 + lane] = pe;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if (base != first) {
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int k = 0; k < E; ++k) acc[c][k] *= select_head<HP>(scale, hc[c][HU ? 0 : k]);
        }

        for (int j = 0; j < cnt; j += U) {
            float zn[U][NC][E];
            const bool more = j + U < cnt;
            if (more) {
#pragma unroll
                for (int t = 0; t < U; ++t) {
                    const uint16_t* zr = a.Z + (int64_t)bcast_i(my_u, (j + U + t) & 63) * a.ldz;
#pragma unroll
                    for (int c = 0; c < NC; ++c) load_stored<FMT, E>(zr + colsafe[c], zn[t][c]);
                }
            }
#pragma unroll
            for (int t = 0; t < U; ++t)
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    if constexpr (HU) {
                        const float w = myw[hc[c][0] * 64 + j + t];
#pragma unroll
                        for (int k = 0; k < E; ++k) acc[c][k] = fmaf(w, zq[t][c][k], acc[c][k]);
                    } else {
#pragma unroll
                        for (int k = 0; k < E; ++k) acc[c][k] = fmaf(myw[hc[c][k] * 64 + j + t], zq[t][c][k], acc[c][k]);
                    }
                }
            if (more) {
#pragma unroll
                for (int t = 0; t < U; ++t)
#pragma unroll
                    for (int c = 0; c < NC; ++c)
#pragma unroll
                        for (int k = 0; k < E; ++k) zq[t][c][k] = zn[t][c][k];
            }
        }
    }

    if constexpr (NW > 1) {
        __shared__ float red[NW][NC * E][64];
        __shared__ float mred[NW][HP], sred[NW][HP];
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int k = 0; k < E; ++k) red[wave][c * E + k][lane] = acc[c][k];
        if (lane == 0) {
#pragma unroll
            for (int h = 0; h < HP; ++h) { mred[wave][h] = m[h]; sred[wave][h] = s[h]; }
        }
        __syncthreads();
        if (wave != 0) return;
        float f[NW][HP];
#pragma unroll
        for (int h = 0; h < HP; ++h) {
            float mm = mred[0][h];
#pragma unroll
            for (int w = 1; w < NW; ++w) mm = fmaxf(mm, mred[w][h]);
            float ss = 0.0f;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                f[w][h] = (mred[w][h] == -INFINITY) ? 0.0f : expf(mred[w][h] - mm);
                ss += sred[w][h] * f[w][h];
            }
            s[h] = ss;
        }
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int k = 0; k < E; ++k) {
                float t = 0.0f;
#pragma unroll
                for (int w = 0; w < NW; ++w) t += red[w][c * E + k][lane] * select_head<HP>(f[w], hc[c][HU ? 0 : k]);
                acc[c][k] = t;
            }
    }

    float* orow = a.out + (int64_t)v * a.ldo;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        if (!act[c]) continue;
        const int64_t col = col0 + c * 64 * E;
        const int valid = (int)min((int64_t)E, a.F - col);
        float r[E];
#pragma unroll
        for (int k = 0; k < E; ++k) {
            const float den = select_head<HP>(s, hc[c][HU ? 0 : k]);
            r[k] = den > 0.0f ? acc[c][k] / den : 0.0f;
        }
        store_floats<E>(orow + a.ocol + col, r, valid, a.out_vec != 0, a.out_half != 0);
        if (a.copy_self) {
            float zs[E];
            load_stored<FMT, E>(a.Z + (int64_t)v * a.ldz + col, zs);
            store_floats<E>(orow + col, zs, valid, a.self_vec != 0);
        }
    }
}

// ---------------------------------------------------------------------------
// gat_softmax over a stored table for rows of ordinary length when the row fits one wave at four
// elements per lane (F <= 256) and a head is a power-of-two group of lanes: the source score of an
// entry is computed from the gathered (decoded) row itself instead of being read from the score
// table, which costs a cache line per entry — a fifth of the traffic when a row is only 512 bytes.
// Same scheme as the fp32 kernel of that name: per-lane dot product with a_src, sum over the head's
// lanes, online softmax over batches of four entries, scores in units of log2(e).
// ---------------------------------------------------------------------------
template <int FMT, int G>
__global__ __launch_bounds__(64 * kLightWaves) void stored_gat_flash_kernel(StoredArgs a, const float* __restrict__ attn_src,
                                                                            int er_stride)
{
    constexpr int U = 4, E = 4;
    constexpr float kLog2e = 1.4426950408889634f;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t slot = (int64_t)blockIdx.x * kLightWaves + wave;
    if (slot >= a.row_count) return;
    const int v = __builtin_amdgcn_readfirstlane(a.order[a.row_begin + slot]);
    const int lo = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v]);
    const int hi = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v + 1]);

    const int64_t col = lane * E;
    const bool act = col < a.F;
    const int64_t colsafe = act ? col : 0;            // idle lanes read the row start (weight vector zero, never stored)
    const int h = min((int)(col / a.Dh), a.heads - 1);
    float as[E] = {0.0f, 0.0f, 0.0f, 0.0f};
    float erv = 0.0f;
    if (act) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(attn_src + col);
        as[0] = t.x * kLog2e; as[1] = t.y * kLog2e; as[2] = t.z * kLog2e; as[3] = t.w * kLog2e;
        erv = a.er[(int64_t)v * er_stride + h] * kLog2e;
    }

    float m = -INFINITY, s = 0.0f;
    float acc[E] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int base = lo; base < hi; base += 64) {
        const int e = base + lane;
        const bool valid = e < hi;
        const int cnt = min(64, hi - base);
        int my_u = valid ? a.col_idx[e] : 0;
        my_u = valid ? my_u : bcast_i(my_u, 0);

        float zq[U][E];
#pragma unroll
        for (int t = 0; t < U; ++t) load_stored<FMT, E>(a.Z + (int64_t)bcast_i(my_u, t) * a.ldz + colsafe, zq[t]);

        for (int j = 0; j < cnt; j += U) {
            float zn[U][E];
            const bool more = j + U < cnt;
            if (more) {
#pragma unroll
                for (int t = 0; t < U; ++t)
                    load_stored<FMT, E>(a.Z + (int64_t)bcast_i(my_u, (j + U + t) & 63) * a.ldz + colsafe, zn[t]);
            }
            float sc[U];
#pragma unroll
            for (int t = 0; t < U; ++t) {
                float d = as[0] * zq[t][0];
                d = fmaf(as[1], zq[t][1], d);
                d = fmaf(as[2], zq[t][2], d);
                d = fmaf(as[3], zq[t][3], d);
                const float x = group_sum<G>(d) + erv;
                sc[t] = (j + t < cnt) ? (x > 0.0f ? x : a.slope * x) : -INFINITY;
            }
            float mn = m;
#pragma unroll
            for (int t = 0; t < U; ++t) mn = fmaxf(mn, sc[t]);      // finite: entry j of the tile is real
            const float scale = __builtin_amdgcn_exp2f(m - mn);
            float pw[U], ps = 0.0f;
#pragma unroll
            for (int t = 0; t < U; ++t) { pw[t] = __builtin_amdgcn_exp2f(sc[t] - mn); ps += pw[t]; }
            s = s * scale + ps;
#pragma unroll
            for (int k = 0; k < E; ++k) acc[k] *= scale;
#pragma unroll
            for (int t = 0; t < U; ++t)
#pragma unroll
                for (int k = 0; k < E; ++k) acc[k] = fmaf(pw[t], zq[t][k], acc[k]);
            m = mn;
            if (more) {
#pragma unroll
                for (int t = 0; t < U; ++t)
#pragma unroll
                    for (int k = 0; k < E; ++k) zq[t][k] = zn[t][k];
            }
        }
    }

    if (!act) return;
    float* orow = a.out + (int64_t)v * a.ldo;
    float r[E];
#pragma unroll
    for (int k = 0; k < E; ++k) r[k] = s > 0.0f ? acc[k] / s : 0.0f;
    store_floats<E>(orow + a.ocol + col, r, E, a.out_vec != 0, a.out_half != 0);
    if (a.copy_self) {
        float zs[E];
        load_stored<FMT, E>(a.Z + (int64_t)v * a.ldz + col, zs);
        store_floats<E>(orow + col, zs, E, a.self_vec != 0);
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
template <typename K, typename KH>
void launch_pair(K light, KH heavy, const StoredArgs& base, int64_t n_heavy, int64_t N, hipStream_t stream)
{
    if (n_heavy > 0) {
        StoredArgs a = base;
        a.row_begin = 0;
        a.row_count = n_heavy;
        heavy<<<dim3((unsigned)(n_heavy * a.nslab)), dim3(64 * kHeavyWaves), 0, stream>>>(a);
    }
    if (N > n_heavy) {
        StoredArgs a = base;
        a.row_begin = n_heavy;
        a.row_count = N - n_heavy;
        const int64_t blocks = (a.row_count * a.nslab + kLightWaves - 1) / kLightWaves;
        light<<<dim3((unsigned)blocks), dim3(64 * kLightWaves), 0, stream>>>(a);
    }
}

template <int FMT, int E, bool MAXOP>
void dispatch_linear(int nc, const StoredArgs& a, int64_t nh, int64_t N, hipStream_t s)
{
    if (nc == 1) launch_pair(stored_linear_kernel<FMT, E, 1, 1, MAXOP>, stored_linear_kernel<FMT, E, 1, kHeavyWaves, MAXOP>, a, nh, N, s);
    else launch_pair(stored_linear_kernel<FMT, E, 2, 1, MAXOP>, stored_linear_kernel<FMT, E, 2, kHeavyWaves, MAXOP>, a, nh, N, s);
}

template <int FMT, int E, int HP, bool HU>
void dispatch_gat(int nc, const StoredArgs& a, int64_t nh, int64_t N, hipStream_t s)
{
    if (nc == 1) launch_pair(stored_gat_kernel<FMT, E, 1, 1, HP, HU>, stored_gat_kernel<FMT, E, 1, kHeavyWaves, HP, HU>, a, nh, N, s);
    else launch_pair(stored_gat_kernel<FMT, E, 2, 1, HP, HU>, stored_gat_kernel<FMT, E, 2, kHeavyWaves, HP, HU>, a, nh, N, s);
}

bool aligned_rows(const void* p, int64_t ld_elems, int bytes_per_elem)
{
    return ((uintptr_t)p % 16) == 0 && (ld_elems * bytes_per_elem) % 16 == 0;
}

template <int FMT>
int launch_stored(const StoredCall& c, hipStream_t stream)
{
    const retexo_plan* p = c.plan;
    const int64_t N = p->N, F = c.F;
    const AggOptions& opt = agg_options();
    const bool gat = c.mode == RETEXO_GAT_SOFTMAX;
    const uint16_t* Z = (const uint16_t*)c.Z;

    // 16-byte loads of eight elements need aligned rows padded to whole vectors; rows of at most 256
    // columns use 8-byte loads of four elements so that all 64 lanes of a wave carry a share of the row
    const bool wide = aligned_rows(Z, c.ldz, 2) && align_up(F, 8) <= c.ldz && opt.max_vec >= 4;
    const int E = wide ? (F <= 256 ? 4 : 8) : 1;

    StoredArgs a;
    a.row_ptr = p->row_ptr;
    a.col_idx = p->col_idx;
    a.order = p->order;
    a.deg = p->deg;
    a.dinv = p->dinv;
    a.wsrc = c.mode == RETEXO_GCN_SYM ? p->dinv : nullptr;
    a.Z = Z;
    a.ldz = c.ldz;
    a.out = c.out;
    a.ldo = c.ldo;
    a.ocol = c.self_concat ? F : 0;
    a.el = nullptr;
    a.er = nullptr;
    a.row_begin = 0;
    a.row_count = 0;
    a.F = F;
    a.scale = c.mode == RETEXO_MEAN ? 1 : c.mode == RETEXO_GCN_SYM ? 2 : 0;
    a.heads = c.heads;
    a.Dh = gat ? (int)(F / c.heads) : (int)F;
    a.slope = c.slope;
    a.copy_self = (c.self_concat && c.copy_self) ? 1 : 0;
    a.out_vec = aligned_rows(c.out + a.ocol, c.ldo, 4) ? 1 : 0;
    a.out_half = ((uintptr_t)(c.out + a.ocol) % 8 == 0 && c.ldo % 2 == 0) ? 1 : 0;
    a.self_vec = aligned_rows(c.out, c.ldo, 4) ? 1 : 0;
    a.part_ptr = nullptr;
    a.n_rows = N;
    a.part_lo = 0;
    a.part_hi = 0;
    a.first = 1;
    a.last = 1;

    int64_t n_heavy = 0;
    for (int i = 0; i < 8; ++i)
        if (kPlanThresholds[i] >= opt.heavy_degree) { n_heavy = p->rows_at_least[i]; break; }

    const int max_nc = 2;
    int nc = (int)((F + 64 * E - 1) / (64 * E));
    nc = nc < 1 ? 1 : nc > max_nc ? max_nc : nc;
    const int64_t slab_w = 64 * (int64_t)E * nc;
    a.nslab = (int)((F + slab_w - 1) / slab_w);

    // dense graphs whose table exceeds L2 although a 64-column slab of one source range fits: narrow slabs
    const bool off32 = (N * c.ldz + F) * 2 < (1ll << 32) && !opt.wide_offsets;
    const bool linear_sum = c.mode == RETEXO_SUM || c.mode == RETEXO_MEAN || c.mode == RETEXO_GCN_SYM;
    bool narrow = linear_sum && wide && off32 && (p->part_ptr || (p->nnz >= 32 * N && N * c.ldz * 2 > (4ll << 20)));
    if (opt.slab_cols > 64) narrow = false;
    if (opt.slab_cols == 64 && linear_sum && wide && off32) narrow = true;
    if (narrow) {
        a.nslab = (int)((F + 63) / 64);
        int parts = (int)opt.parts;
        if (parts < 0) {
            parts = 1;
            while (parts < kMaxParts && N * 128 > (int64_t)parts * (8ll << 20)) parts *= 2;
        }
        if (!p->part_ptr || (parts != 2 && parts != 4 && parts != 8 && parts != 16)) parts = 1;
        if (parts > 1) a.part_ptr = p->part_ptr;
        // rows whose share of one range is long get a workgroup each
        int64_t n_long = 0;
        for (int i = 0; i < 8; ++i)
            if (kPlanThresholds[i] >= opt.narrow_heavy * parts || kPlanThresholds[i] >= 16384) {
                n_long = p->rows_at_least[i];
                break;
            }
        const int64_t bundles = (N - n_long + 7) / 8;
        const int64_t blocks = (bundles * a.nslab + kLightWaves - 1) / kLightWaves;
        for (int k = 0; k < parts; ++k) {
            a.part_lo = k * (kMaxParts / parts);
            a.part_hi = (k + 1) * (kMaxParts / parts);
            a.first = k == 0;
            a.last = k == parts - 1;
            if (n_long > 0) {
                a.row_begin = 0;
                a.row_count = n_long;
                const dim3 grid((unsigned)(n_long * a.nslab));
                if (a.wsrc) stored_grouped_kernel<FMT, true><<<grid, dim3(64 * kHeavyWaves), 0, stream>>>(a);
                else stored_grouped_kernel<FMT, false><<<grid, dim3(64 * kHeavyWaves), 0, stream>>>(a);
            }
            if (N > n_long) {
                a.row_begin = n_long;
                a.row_count = N - n_long;
                if (a.wsrc) stored_rowgroup_kernel<FMT, true><<<dim3((unsigned)blocks), dim3(64 * kLightWaves), 0, stream>>>(a);
                else stored_rowgroup_kernel<FMT, false><<<dim3((unsigned)blocks), dim3(64 * kLightWaves), 0, stream>>>(a);
            }
        }
    } else if (!gat) {
        const bool maxop = c.mode == RETEXO_MAX;
        if (E == 8)      { if (maxop) dispatch_linear<FMT, 8, true>(nc, a, n_heavy, N, stream); else dispatch_linear<FMT, 8, false>(nc, a, n_heavy, N, stream); }
        else if (E == 4) { if (maxop) dispatch_linear<FMT, 4, true>(nc, a, n_heavy, N, stream); else dispatch_linear<FMT, 4, false>(nc, a, n_heavy, N, stream); }
        else             { if (maxop) dispatch_linear<FMT, 1, true>(nc, a, n_heavy, N, stream); else dispatch_linear<FMT, 1, false>(nc, a, n_heavy, N, stream); }
    } else {
        const int hp = heads_padded(c.heads);
        const GatWorkspace w = gat_workspace(N, F, c.heads, false);
        float* el = (float*)((char*)c.workspace + w.el);
        float* er = (float*)((char*)c.workspace + w.er);
        a.el = el;
        a.er = er;
        const bool vec_scores = F % 4 == 0 && c.ldz % 4 == 0 && (uintptr_t)Z % 8 == 0 && F < (1ll << 30) &&
                                (uintptr_t)c.attn_src % 16 == 0 && (uintptr_t)c.attn_dst % 16 == 0 && opt.max_vec >= 4;
        if (vec_scores) {
            const unsigned gv = (unsigned)((N + 15) / 16);
            if (hp == 4) stored_scores_vec_kernel<FMT, 4><<<dim3(gv), dim3(256), 0, stream>>>(N, F, a.Dh, Z, c.ldz, c.attn_src, c.attn_dst, el, er);
            else stored_scores_vec_kernel<FMT, 8><<<dim3(gv), dim3(256), 0, stream>>>(N, F, a.Dh, Z, c.ldz, c.attn_src, c.attn_dst, el, er);
        } else {
            const unsigned gb = (unsigned)((N + 3) / 4);
            if (hp == 4) stored_scores_kernel<FMT, 4><<<dim3(gb), dim3(256), 0, stream>>>(N, F, a.Dh, Z, c.ldz, c.attn_src, c.attn_dst, el, er);
            else stored_scores_kernel<FMT, 8><<<dim3(gb), dim3(256), 0, stream>>>(N, F, a.Dh, Z, c.ldz, c.attn_src, c.attn_dst, el, er);
        }
        const bool hu = (a.Dh % E) == 0;
        // rows of ordinary length compute the source scores from the gathered rows (see the kernel)
        const int g = a.Dh / 4;
        const bool flash = E == 4 && opt.gat_flash && a.Dh % 4 == 0 && g <= 64 && (g & (g - 1)) == 0 &&
                           (uintptr_t)c.attn_src % 16 == 0;
        int64_t n_table = N;          // rows [0, n_table) of the schedule go through the table kernels
        if (flash && N > n_heavy) {
            StoredArgs f = a;
            f.nslab = 1;
            f.row_begin = n_heavy;
            f.row_count = N - n_heavy;
            const dim3 grid((unsigned)((f.row_count + kLightWaves - 1) / kLightWaves)), block(64 * kLightWaves);
            switch (g) {
                case 1:  stored_gat_flash_kernel<FMT, 1><<<grid, block, 0, stream>>>(f, c.attn_src, hp); break;
                case 2:  stored_gat_flash_kernel<FMT, 2><<<grid, block, 0, stream>>>(f, c.attn_src, hp); break;
                case 4:  stored_gat_flash_kernel<FMT, 4><<<grid, block, 0, stream>>>(f, c.attn_src, hp); break;
                case 8:  stored_gat_flash_kernel<FMT, 8><<<grid, block, 0, stream>>>(f, c.attn_src, hp); break;
                case 16: stored_gat_flash_kernel<FMT, 16><<<grid, block, 0, stream>>>(f, c.attn_src, hp); break;
                case 32: stored_gat_flash_kernel<FMT, 32><<<grid, block, 0, stream>>>(f, c.attn_src, hp); break;
                default: stored_gat_flash_kernel<FMT, 64><<<grid, block, 0, stream>>>(f, c.attn_src, hp); break;
            }
            n_table = n_heavy;
        }
        if (n_table == 0) {
            // nothing left for the table kernels
        } else if (E == 8) {
            if (hp == 4) { if (hu) dispatch_gat<FMT, 8, 4, true>(nc, a, n_heavy, N, stream); else dispatch_gat<FMT, 8, 4, false>(nc, a, n_heavy, N, stream); }
            else         { if (hu) dispatch_gat<FMT, 8, 8, true>(nc, a, n_heavy, N, stream); else dispatch_gat<FMT, 8, 8, false>(nc, a, n_heavy, N, stream); }
        } else if (E == 4) {
            if (hp == 4) { if (hu) dispatch_gat<FMT, 4, 4, true>(nc, a, n_heavy, n_table, stream); else dispatch_gat<FMT, 4, 4, false>(nc, a, n_heavy, n_table, stream); }
            else         { if (hu) dispatch_gat<FMT, 4, 8, true>(nc, a, n_heavy, n_table, stream); else dispatch_gat<FMT, 4, 8, false>(nc, a, n_heavy, n_table, stream); }
        } else {
            if (hp == 4) dispatch_gat<FMT, 1, 4, true>(nc, a, n_heavy, N, stream);
            else dispatch_gat<FMT, 1, 8, true>(nc, a, n_heavy, N, stream);
        }
    }
    if (hipGetLastError() != hipSuccess) return RETEXO_E_HIP;
    return RETEXO_OK;
}

}  // namespace

int launch_store_rows(int storage, int64_t N, int64_t F, const float* src, int64_t lds, void* dst, int64_t ldd,
                      hipStream_t stream)
{
    if (N == 0 || F == 0) return RETEXO_OK;
    const dim3 grid((unsigned)((N * F + 255) / 256));
    if (storage == RETEXO_STORE_BF16)
        store_rows_kernel<FMT_BF16><<<grid, dim3(256), 0, stream>>>(N, F, src, lds, (uint16_t*)dst, ldd);
    else
        store_rows_kernel<FMT_FP16><<<grid, dim3(256), 0, stream>>>(N, F, src, lds, (uint16_t*)dst, ldd);
    if (hipGetLastError() != hipSuccess) return RETEXO_E_HIP;
    return RETEXO_OK;
}

int launch_aggregate_stored(const StoredCall& c, hipStream_t stream)
{
    if (c.plan->N == 0 || c.F == 0) return RETEXO_OK;
    return c.storage == RETEXO_STORE_BF16 ? launch_stored<FMT_BF16>(c, stream) : launch_stored<FMT_FP16>(c, stream);
}
