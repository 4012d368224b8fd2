// Neighbourhood aggregation over a CSR graph: the AGGR / COMBINE of Eq. 1 in
// the forms of the paper's three model families (GraphSAGE mean with
// self-concatenation, GCN symmetric normalisation, GAT edge softmax).
//
// The work is a sparse-times-dense product whose cost is the gather of one
// F-float row of Z per CSR entry: 4 bytes and one FMA per (edge, feature).
// It is bound by memory, not arithmetic, so the design is about the gather:
//
//  * One wavefront owns one (row, column-slab) pair.  Its 64 lanes each own
//    VEC consecutive columns (VEC = 4/2/1 floats depending on alignment) in
//    each of NC chunks, so one neighbour is fetched by NC fully coalesced
//    wave-wide loads of 64*VEC*4 bytes.
//  * Neighbour ids are read 64 at a time (one coalesced load), then broadcast
//    one by one with v_readlane, which leaves the id in a scalar register and
//    turns the row address into scalar arithmetic.  The broadcast loop is
//    unrolled so that several neighbours' loads are in flight per wave.
//  * Rows are scheduled longest first (plan order).  Rows at or above a degree
//    threshold get a whole workgroup: its waves take interleaved 64-edge tiles
//    and combine their partial sums through LDS in a fixed order.  Every
//    output element is written by exactly one wave and nothing is accumulated
//    with atomics, so results are bitwise reproducible.
//  * Edge softmax: per 64-edge tile the scores are computed one edge per lane,
//    the tile maximum and the sum of exponentials are wave reductions, and the
//    running (max, sum, accumulator) triple is rescaled once per tile (online
//    softmax at tile granularity) — one exp per edge and head instead of one
//    per edge and lane.
#include "common.hpp"

namespace {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kLightWaves = 4;   // independent rows per workgroup in the light kernel
constexpr int kHeavyWaves = 8;   // cooperating waves per row in the heavy kernel
constexpr int kUnroll = 4;       // neighbours fetched per unrolled step

enum { SCALE_SUM = 0, SCALE_MEAN = 1, SCALE_GCN = 2 };

struct AggArgs {
    const int64_t* row_ptr;
    const int32_t* col_idx;
    const int32_t* order;
    const int32_t* deg;
    const float* dinv;
    const float* Z;
    int64_t ldz;
    float* out;
    int64_t ldo;
    int64_t ocol;          // first output column of the aggregate
    const float* el;       // [N, HP]  <a_src, z_u>   (edge softmax only)
    const float* er;       // [N, HP]  <a_dst, z_v>
    int64_t row_begin;     // range of plan order handled by this launch
    int64_t row_count;
    int64_t F;
    int nslab;
    int slab_major;
    int scale;             // SCALE_*
    int heads;
    int Dh;
    float slope;
    int copy_self;         // also write z_v into out[:, 0:F]
    int out_vec;           // aggregate slot of out is aligned for VEC-wide stores
    int self_vec;          // self slot of out is aligned for VEC-wide stores
};

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

template <int VEC>
__device__ __forceinline__ void store_row(float* p, const float (&v)[VEC], int valid, bool vec_ok)
{
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

// pick s[h] for a per-lane head index from per-head wave-uniform values
template <int HP>
__device__ __forceinline__ float select_head(const float (&s)[HP], int h)
{
    float r = s[0];
#pragma unroll
    for (int i = 1; i < HP; ++i) r = (h == i) ? s[i] : r;
    return r;
}

// ---------------------------------------------------------------------------
// sum / mean / gcn_sym
//   NW == 1: kLightWaves independent (row, slab) items per workgroup
//   NW  > 1: the NW waves of a workgroup share one (row, slab) item
// ---------------------------------------------------------------------------
template <int VEC, int NC, int NW>
__global__ __launch_bounds__(64 * (NW == 1 ? kLightWaves : NW)) void agg_linear_kernel(AggArgs a)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t items = a.row_count * a.nslab;
    const int64_t item = (NW == 1) ? (int64_t)blockIdx.x * kLightWaves + wave : (int64_t)blockIdx.x;
    if (item >= items) return;        // NW > 1: uniform over the workgroup
    int64_t slot;
    int slab;
    if (a.slab_major) { slab = (int)(item / a.row_count); slot = item % a.row_count; }
    else              { slot = item / a.nslab; slab = (int)(item % a.nslab); }
    const int v = __builtin_amdgcn_readfirstlane(a.order[a.row_begin + slot]);
    const int lo = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v]);
    const int hi = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v + 1]);

    const int64_t col0 = (int64_t)slab * (64 * VEC * NC) + lane * VEC;
    bool act[NC];
    float acc[NC][VEC];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        act[c] = col0 + c * 64 * VEC < a.F;
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc[c][k] = 0.0f;
    }
    const float* zl = a.Z + col0;
    const bool weighted = a.scale == SCALE_GCN;

    for (int base = lo + 64 * (NW == 1 ? 0 : wave); base < hi; base += 64 * NW) {
        const int e = base + lane;
        const int my_u = e < hi ? a.col_idx[e] : 0;
        const float my_w = weighted ? (e < hi ? a.dinv[my_u] : 0.0f) : 1.0f;
        const int cnt = min(64, hi - base);
        int j = 0;
        for (; j + kUnroll <= cnt; j += kUnroll) {
            float z[kUnroll][NC][VEC];
            float w[kUnroll];
#pragma unroll
            for (int t = 0; t < kUnroll; ++t) {
                const int u = bcast_i(my_u, j + t);
                w[t] = bcast_f(my_w, j + t);
                const float* zr = zl + (int64_t)u * a.ldz;
#pragma unroll
                for (int c = 0; c < NC; ++c)
                    if (act[c]) load_row<VEC>(zr + c * 64 * VEC, z[t][c]);
            }
#pragma unroll
            for (int t = 0; t < kUnroll; ++t)
#pragma unroll
                for (int c = 0; c < NC; ++c)
                    if (act[c]) {
#pragma unroll
                        for (int k = 0; k < VEC; ++k) acc[c][k] = fmaf(w[t], z[t][c][k], acc[c][k]);
                    }
        }
        for (; j < cnt; ++j) {
            const int u = bcast_i(my_u, j);
            const float w = bcast_f(my_w, j);
            const float* zr = zl + (int64_t)u * a.ldz;
#pragma unroll
            for (int c = 0; c < NC; ++c)
                if (act[c]) {
                    float z[VEC];
                    load_row<VEC>(zr + c * 64 * VEC, z);
#pragma unroll
                    for (int k = 0; k < VEC; ++k) acc[c][k] = fmaf(w, z[k], acc[c][k]);
                }
        }
    }

    if constexpr (NW > 1) {
        __shared__ float red[NW][NC * VEC][64];
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int k = 0; k < VEC; ++k) red[wave][c * VEC + k][lane] = acc[c][k];
        __syncthreads();
        if (wave != 0) return;
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                float s = red[0][c * VEC + k][lane];
#pragma unroll
                for (int w = 1; w < NW; ++w) s += red[w][c * VEC + k][lane];
                acc[c][k] = s;
            }
    }

    const int d = hi - lo;
    float* orow = a.out + (int64_t)v * a.ldo;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        if (!act[c]) continue;
        const int64_t col = col0 + c * 64 * VEC;
        const int valid = (int)min((int64_t)VEC, a.F - col);
        float r[VEC];
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            float x = acc[c][k];
            if (a.scale == SCALE_MEAN) x = d > 0 ? x / (float)d : 0.0f;
            else if (a.scale == SCALE_GCN) x = x * a.dinv[v];
            r[k] = x;
        }
        store_row<VEC>(orow + a.ocol + col, r, valid, a.out_vec != 0);
        if (a.copy_self) {
            float zs[VEC];
            load_row<VEC>(a.Z + (int64_t)v * a.ldz + col, zs);
            store_row<VEC>(orow + col, zs, valid, a.self_vec != 0);
        }
    }
}

// ---------------------------------------------------------------------------
// attention scores  el[v,h] = <a_src[h], z_v,h>,  er[v,h] = <a_dst[h], z_v,h>
// one wave per node; padded heads (h >= heads) get 0
// ---------------------------------------------------------------------------
template <int HP>
__global__ __launch_bounds__(256) void gat_scores_kernel(
    int64_t N, int64_t F, int heads, int Dh, const float* __restrict__ Z, int64_t ldz,
    const float* __restrict__ a_src, const float* __restrict__ a_dst,
    float* __restrict__ el, float* __restrict__ er)
{
    const int lane = threadIdx.x & 63;
    const int64_t v = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= N) return;
    float ps[HP], pd[HP];
#pragma unroll
    for (int h = 0; h < HP; ++h) { ps[h] = 0.0f; pd[h] = 0.0f; }
    for (int64_t c = lane; c < F; c += 64) {
        const float z = Z[v * ldz + c];
        const int h = (int)(c / Dh);
        const float s = z * a_src[c], t = z * a_dst[c];   // a_* are [heads, Dh] = flat [F]
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

// ---------------------------------------------------------------------------
// gat_softmax.  HU: every lane's VEC columns lie inside one head (Dh % VEC == 0)
// ---------------------------------------------------------------------------
template <int VEC, int NC, int NW, int HP, bool HU>
__global__ __launch_bounds__(64 * (NW == 1 ? kLightWaves : NW)) void agg_gat_kernel(AggArgs a)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t items = a.row_count * a.nslab;
    const int64_t item = (NW == 1) ? (int64_t)blockIdx.x * kLightWaves + wave : (int64_t)blockIdx.x;
    if (item >= items) return;
    int64_t slot;
    int slab;
    if (a.slab_major) { slab = (int)(item / a.row_count); slot = item % a.row_count; }
    else              { slot = item / a.nslab; slab = (int)(item % a.nslab); }
    const int v = __builtin_amdgcn_readfirstlane(a.order[a.row_begin + slot]);
    const int lo = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v]);
    const int hi = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v + 1]);

    const int64_t col0 = (int64_t)slab * (64 * VEC * NC) + lane * VEC;
    bool act[NC];
    int hc[NC][HU ? 1 : VEC];      // head of each owned column (clamped for padding columns)
    float acc[NC][VEC];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int64_t col = col0 + c * 64 * VEC;
        act[c] = col < a.F;
#pragma unroll
        for (int k = 0; k < (HU ? 1 : VEC); ++k) hc[c][k] = min((int)((col + k) / a.Dh), a.heads - 1);
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc[c][k] = 0.0f;
    }
    const float* zl = a.Z + col0;

    float m[HP], s[HP], erv[HP];
#pragma unroll
    for (int h = 0; h < HP; ++h) {
        m[h] = -INFINITY;
        s[h] = 0.0f;
        erv[h] = a.er[(int64_t)v * HP + h];
    }

    for (int base = lo + 64 * (NW == 1 ? 0 : wave); base < hi; base += 64 * NW) {
        const int e = base + lane;
        const bool valid = e < hi;
        const int my_u = valid ? a.col_idx[e] : 0;
        const int cnt = min(64, hi - base);
        float p[HP], scale[HP];
        {
            float elu[HP];
            if constexpr (HP == 4) {
                const f32x4 t = *reinterpret_cast<const f32x4*>(a.el + (int64_t)my_u * 4);
                elu[0] = t.x; elu[1] = t.y; elu[2] = t.z; elu[3] = t.w;
            } else {
#pragma unroll
                for (int h = 0; h < HP; ++h) elu[h] = a.el[(int64_t)my_u * HP + h];
            }
#pragma unroll
            for (int h = 0; h < HP; ++h) {
                const float x = elu[h] + erv[h];
                const float sc = valid ? (x > 0.0f ? x : a.slope * x) : -INFINITY;
                const float mn = fmaxf(m[h], wave_max(sc));      // finite: the tile has an edge
                scale[h] = expf(m[h] - mn);                      // exp(-inf) = 0 on the first tile
                p[h] = valid ? expf(sc - mn) : 0.0f;
                s[h] = s[h] * scale[h] + wave_sum(p[h]);
                m[h] = mn;
            }
        }
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int k = 0; k < VEC; ++k) acc[c][k] *= select_head<HP>(scale, hc[c][HU ? 0 : k]);

        int j = 0;
        for (; j + kUnroll <= cnt; j += kUnroll) {
            float z[kUnroll][NC][VEC];
            float w[kUnroll][HP];
#pragma unroll
            for (int t = 0; t < kUnroll; ++t) {
                const int u = bcast_i(my_u, j + t);
#pragma unroll
                for (int h = 0; h < HP; ++h) w[t][h] = bcast_f(p[h], j + t);
                const float* zr = zl + (int64_t)u * a.ldz;
#pragma unroll
                for (int c = 0; c < NC; ++c)
                    if (act[c]) load_row<VEC>(zr + c * 64 * VEC, z[t][c]);
            }
#pragma unroll
            for (int t = 0; t < kUnroll; ++t)
#pragma unroll
                for (int c = 0; c < NC; ++c)
                    if (act[c]) {
#pragma unroll
                        for (int k = 0; k < VEC; ++k)
                            acc[c][k] = fmaf(select_head<HP>(w[t], hc[c][HU ? 0 : k]), z[t][c][k], acc[c][k]);
                    }
        }
        for (; j < cnt; ++j) {
            const int u = bcast_i(my_u, j);
            float w[HP];
#pragma unroll
            for (int h = 0; h < HP; ++h) w[h] = bcast_f(p[h], j);
            const float* zr = zl + (int64_t)u * a.ldz;
#pragma unroll
            for (int c = 0; c < NC; ++c)
                if (act[c]) {
                    float z[VEC];
                    load_row<VEC>(zr + c * 64 * VEC, z);
#pragma unroll
                    for (int k = 0; k < VEC; ++k)
                        acc[c][k] = fmaf(select_head<HP>(w, hc[c][HU ? 0 : k]), z[k], acc[c][k]);
                }
        }
    }

    if constexpr (NW > 1) {
        // merge the waves' (max, sum, accumulator) triples in wave order
        __shared__ float red[NW][NC * VEC][64];
        __shared__ float mred[NW][HP], sred[NW][HP];
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int k = 0; k < VEC; ++k) red[wave][c * VEC + k][lane] = acc[c][k];
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
                // a wave that saw no tile has max -inf and contributes nothing
                f[w][h] = (mred[w][h] == -INFINITY) ? 0.0f : expf(mred[w][h] - mm);
                ss += sred[w][h] * f[w][h];
            }
            s[h] = ss;
        }
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                float t = 0.0f;
#pragma unroll
                for (int w = 0; w < NW; ++w)
                    t += red[w][c * VEC + k][lane] * select_head<HP>(f[w], hc[c][HU ? 0 : k]);
                acc[c][k] = t;
            }
    }

    float* orow = a.out + (int64_t)v * a.ldo;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        if (!act[c]) continue;
        const int64_t col = col0 + c * 64 * VEC;
        const int valid = (int)min((int64_t)VEC, a.F - col);
        float r[VEC];
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            const float den = select_head<HP>(s, hc[c][HU ? 0 : k]);
            r[k] = den > 0.0f ? acc[c][k] / den : 0.0f;
        }
        store_row<VEC>(orow + a.ocol + col, r, valid, a.out_vec != 0);
        if (a.copy_self) {
            float zs[VEC];
            load_row<VEC>(a.Z + (int64_t)v * a.ldz + col, zs);
            store_row<VEC>(orow + col, zs, valid, a.self_vec != 0);
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
template <int VEC, int NC>
void launch_linear_pair(const AggArgs& base, int64_t n_heavy, int64_t N, hipStream_t stream)
{
    if (n_heavy > 0) {
        AggArgs a = base;
        a.row_begin = 0;
        a.row_count = n_heavy;
        const int64_t blocks = n_heavy * a.nslab;
        agg_linear_kernel<VEC, NC, kHeavyWaves><<<dim3((unsigned)blocks), dim3(64 * kHeavyWaves), 0, stream>>>(a);
    }
    if (N > n_heavy) {
        AggArgs a = base;
        a.row_begin = n_heavy;
        a.row_count = N - n_heavy;
        const int64_t blocks = (a.row_count * a.nslab + kLightWaves - 1) / kLightWaves;
        agg_linear_kernel<VEC, NC, 1><<<dim3((unsigned)blocks), dim3(64 * kLightWaves), 0, stream>>>(a);
    }
}

template <int VEC, int NC, int HP, bool HU>
void launch_gat_pair(const AggArgs& base, int64_t n_heavy, int64_t N, hipStream_t stream)
{
    if (n_heavy > 0) {
        AggArgs a = base;
        a.row_begin = 0;
        a.row_count = n_heavy;
        const int64_t blocks = n_heavy * a.nslab;
        agg_gat_kernel<VEC, NC, kHeavyWaves, HP, HU><<<dim3((unsigned)blocks), dim3(64 * kHeavyWaves), 0, stream>>>(a);
    }
    if (N > n_heavy) {
        AggArgs a = base;
        a.row_begin = n_heavy;
        a.row_count = N - n_heavy;
        const int64_t blocks = (a.row_count * a.nslab + kLightWaves - 1) / kLightWaves;
        agg_gat_kernel<VEC, NC, 1, HP, HU><<<dim3((unsigned)blocks), dim3(64 * kLightWaves), 0, stream>>>(a);
    }
}

template <int VEC>
void dispatch_linear(int nc, const AggArgs& a, int64_t nh, int64_t N, hipStream_t s)
{
    if (nc == 1) launch_linear_pair<VEC, 1>(a, nh, N, s);
    else if (nc == 2) launch_linear_pair<VEC, 2>(a, nh, N, s);
    else launch_linear_pair<VEC, 3>(a, nh, N, s);
}

template <int VEC, int HP, bool HU>
void dispatch_gat_nc(int nc, const AggArgs& a, int64_t nh, int64_t N, hipStream_t s)
{
    if (nc == 1) launch_gat_pair<VEC, 1, HP, HU>(a, nh, N, s);
    else launch_gat_pair<VEC, 2, HP, HU>(a, nh, N, s);
}

bool aligned_for(const void* p, int64_t ld, int vec)
{
    return ((uintptr_t)p % (uintptr_t)(4 * vec)) == 0 && ld % vec == 0;
}

}  // namespace

AggOptions& agg_options()
{
    static AggOptions o;
    return o;
}

int64_t aggregate_workspace_bytes(int64_t N, int mode, int heads)
{
    if (mode != RETEXO_GAT_SOFTMAX) return 0;
    return 2 * align_up((N > 0 ? N : 1) * heads_padded(heads) * (int64_t)sizeof(float), 256);
}

int launch_aggregate(const AggCall& c, hipStream_t stream)
{
    const retexo_plan* p = c.plan;
    const int64_t N = p->N;
    if (N == 0 || c.F == 0) return RETEXO_OK;
    const AggOptions& opt = agg_options();
    const bool gat = c.mode == RETEXO_GAT_SOFTMAX;

    // widest gather the layout of Z allows; a partial last vector may read
    // padding columns of the same row, so the padded width must fit in ldz
    int vec = 1;
    if (aligned_for(c.Z, c.ldz, 4) && align_up(c.F, 4) <= c.ldz) vec = 4;
    else if (aligned_for(c.Z, c.ldz, 2) && align_up(c.F, 2) <= c.ldz) vec = 2;
    if (gat && vec == 2) vec = 1;
    const int max_nc = gat ? 2 : 3;
    int nc;
    if (opt.slab_cols > 0) nc = (int)((opt.slab_cols + 64 * vec - 1) / (64 * vec));
    else nc = (int)((c.F + 64 * vec - 1) / (64 * vec));
    nc = nc < 1 ? 1 : nc > max_nc ? max_nc : nc;
    const int64_t slab_w = 64 * (int64_t)vec * nc;

    AggArgs a;
    a.row_ptr = p->row_ptr;
    a.col_idx = p->col_idx;
    a.order = p->order;
    a.deg = p->deg;
    a.dinv = p->dinv;
    a.Z = c.Z;
    a.ldz = c.ldz;
    a.out = c.out;
    a.ldo = c.ldo;
    a.ocol = c.self_concat ? c.F : 0;
    a.el = nullptr;
    a.er = nullptr;
    a.row_begin = 0;
    a.row_count = 0;
    a.F = c.F;
    a.nslab = (int)((c.F + slab_w - 1) / slab_w);
    a.slab_major = opt.slab_major < 0 ? 1 : (int)opt.slab_major;
    a.scale = c.mode == RETEXO_MEAN ? SCALE_MEAN : c.mode == RETEXO_GCN_SYM ? SCALE_GCN : SCALE_SUM;
    a.heads = c.heads;
    a.Dh = gat ? (int)(c.F / c.heads) : (int)c.F;
    a.slope = c.slope;
    a.copy_self = (c.self_concat && c.copy_self) ? 1 : 0;
    a.out_vec = aligned_for(c.out + a.ocol, c.ldo, vec) ? 1 : 0;
    a.self_vec = aligned_for(c.out, c.ldo, vec) ? 1 : 0;

    // rows at or above the heavy threshold (rounded up to a tabulated one)
    int64_t n_heavy = 0;
    for (int i = 0; i < 8; ++i)
        if (kPlanThresholds[i] >= opt.heavy_degree) { n_heavy = p->rows_at_least[i]; break; }

    if (!gat) {
        if (vec == 4) dispatch_linear<4>(nc, a, n_heavy, N, stream);
        else if (vec == 2) dispatch_linear<2>(nc, a, n_heavy, N, stream);
        else dispatch_linear<1>(nc, a, n_heavy, N, stream);
    } else {
        const int hp = heads_padded(c.heads);
        float* el = (float*)c.workspace;
        float* er = (float*)((char*)c.workspace + align_up(N * heads_padded(c.heads) * (int64_t)sizeof(float), 256));
        a.el = el;
        a.er = er;
        const unsigned gb = (unsigned)((N + 3) / 4);
        if (hp == 4)
            gat_scores_kernel<4><<<dim3(gb), dim3(256), 0, stream>>>(N, c.F, c.heads, a.Dh, c.Z, c.ldz,
                                                                     c.attn_src, c.attn_dst, el, er);
        else
            gat_scores_kernel<8><<<dim3(gb), dim3(256), 0, stream>>>(N, c.F, c.heads, a.Dh, c.Z, c.ldz,
                                                                     c.attn_src, c.attn_dst, el, er);
        const bool hu = (a.Dh % vec) == 0;
        if (vec == 4) {
            if (hp == 4) { if (hu) dispatch_gat_nc<4, 4, true>(nc, a, n_heavy, N, stream); else dispatch_gat_nc<4, 4, false>(nc, a, n_heavy, N, stream); }
            else         { if (hu) dispatch_gat_nc<4, 8, true>(nc, a, n_heavy, N, stream); else dispatch_gat_nc<4, 8, false>(nc, a, n_heavy, N, stream); }
        } else {
            if (hp == 4) dispatch_gat_nc<1, 4, true>(nc, a, n_heavy, N, stream);
            else         dispatch_gat_nc<1, 8, true>(nc, a, n_heavy, N, stream);
        }
    }
    if (hipGetLastError() != hipSuccess) return RETEXO_E_HIP;
    return RETEXO_OK;
}
