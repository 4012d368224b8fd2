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
#include <type_traits>

#include "common.hpp"
#include "gather.hpp"

namespace {


enum { SCALE_SUM = 0, SCALE_MEAN = 1, SCALE_GCN = 2 };

struct AggArgs {
    const int64_t* row_ptr;
    const int32_t* col_idx;
    const int32_t* order;
    const int32_t* deg;
    const float* dinv;
    const float* wsrc;     // per-source weight of every gathered row, or NULL (all 1)
    const float* Z;
    int64_t ldz;
    float* out;
    int64_t ldo;
    int64_t ocol;          // first output column of the aggregate
    const float* el;       // <a_src, z_u> of node u, head h at el[u * el_stride + h]   (edge softmax only)
    int64_t el_stride;     // HP for the table in the workspace; ldz when the scores sit in Z's padding columns
    const float* er;       // [N, HP]  <a_dst, z_v>, or NULL:
    const float* er_from;  // a_dst [heads, Dh]; the kernel forms <a_dst, z_v> from row v itself (pipelined kernel, one slab)
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
    int out_half;          // ... or at least for 8-byte stores (float4 gathers only)
    int self_vec;          // self slot of out is aligned for VEC-wide stores
    // source-range walk (grouped kernel only): this launch covers the entries of each row whose
    // column lies in ranges [part_lo, part_hi) of the plan's split; NULL = whole rows
    const int32_t* part_ptr;
    int64_t n_rows;        // N (row pitch of part_ptr)
    int part_lo, part_hi;
    int first;             // first range of the walk: start from zero, write the self copy
    int last;              // last range: apply the mean / gcn scaling
    // edge softmax, kept for the backward pass (TRAIN kernels only):
    f32x4* save_stats;     // [N, HP] {row maximum, 1/sum, share of the sum with p > 0, share with p <= 0}
    float* save_pos;       // [N, ld_pos] the part of the aggregate that comes from entries with p > 0
    float* save_neg;       // [N, ld_pos] ... and from entries with p <= 0 (the aggregate is their sum)
    int64_t ld_pos;
};

// ---------------------------------------------------------------------------
// sum / mean / gcn_sym, and (MAXOP) the element-wise maximum
//   NW == 1: kLightWaves independent (row, slab) items per workgroup
//   NW  > 1: the NW waves of a workgroup share one (row, slab) item
// ---------------------------------------------------------------------------
template <int VEC, int NC, int NW, bool MAXOP>
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
        for (int k = 0; k < VEC; ++k) acc[c][k] = MAXOP ? -INFINITY : 0.0f;
    }
    const float* zl = a.Z + col0;
    const bool weighted = a.wsrc != nullptr;

    for (int base = lo + 64 * (NW == 1 ? 0 : wave); base < hi; base += 64 * NW) {
        const int e = base + lane;
        const int my_u = e < hi ? a.col_idx[e] : 0;
        const float my_w = weighted ? (e < hi ? a.wsrc[my_u] : 0.0f) : 1.0f;
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
                        for (int k = 0; k < VEC; ++k)
                            acc[c][k] = MAXOP ? fmaxf(acc[c][k], z[t][c][k]) : fmaf(w[t], z[t][c][k], acc[c][k]);
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
                    for (int k = 0; k < VEC; ++k) acc[c][k] = MAXOP ? fmaxf(acc[c][k], z[k]) : fmaf(w, z[k], acc[c][k]);
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
                for (int w = 1; w < NW; ++w) s = MAXOP ? fmaxf(s, red[w][c * VEC + k][lane]) : s + red[w][c * VEC + k][lane];
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
            if (MAXOP) x = d > 0 ? x : 0.0f;                     // empty neighbourhood: zero
            else if (a.scale == SCALE_MEAN) x = d > 0 ? x / (float)d : 0.0f;
            else if (a.scale == SCALE_GCN) x = x * a.dinv[v];
            r[k] = x;
        }
        store_row<VEC>(orow + a.ocol + col, r, valid, a.out_vec != 0, a.out_half != 0);
        if (a.copy_self) {
            float zs[VEC];
            load_row<VEC>(a.Z + (int64_t)v * a.ldz + col, zs);
            store_row<VEC>(orow + col, zs, valid, a.self_vec != 0);
        }
    }
}

// ---------------------------------------------------------------------------
// sum / mean / gcn_sym with narrow column slabs ("grouped gather").
//
// When one column slab of the whole table (N rows x SW columns) is small
// enough to stay in the last-level caches, walking the graph once per slab
// turns most gathers into cache hits instead of HBM reads.  A slab is
// SW = 4*LPG columns wide; a wave splits into G = 64/LPG groups of LPG lanes,
// each lane owning one float4 of the slab, and every wave-wide load fetches the
// slab of G different neighbours (G x SW x 4 = 1 KiB per instruction, as in the
// full-row kernel).  Neighbour ids are loaded 64 at a time and handed to the
// groups with a wave shuffle; the groups' partial sums are combined with
// xor-shuffles when the row is done.  Same ownership rules as above: one wave
// (or one workgroup for long rows) writes an output element, in a fixed order.
// ---------------------------------------------------------------------------
// One 64-edge tile of the grouped gather.  Each lane holds the byte offset of
// one neighbour's row (and its gcn weight); step t hands entry t*G + g to group
// g with a wave shuffle.  All loads of a batch of up to 8 steps are issued
// before their FMAs, and nothing in the batch branches: lanes past the end of
// a partial tile fetch a valid address (offset 0) and have the loaded values
// replaced by zero; lanes past the row width fetch the last valid vector of
// the slab and simply never store.
//   OFF32: every row offset fits 32 bits, so the gather is base + 32-bit offset
template <int LPG, bool FULL, bool WEIGHTED, bool OFF32>
__device__ __forceinline__ void grouped_tile(const char* zbase, uint32_t colbytes, int64_t rowbytes,
                                             uint32_t my_off, int my_u, float my_w, int cnt, int g,
                                             float (&acc)[4])
{
    constexpr int G = 64 / LPG;
    constexpr int STEPS = 64 / G;
    constexpr int U = STEPS < 8 ? STEPS : 8;
#pragma unroll
    for (int t0 = 0; t0 < STEPS; t0 += U) {
        if (!FULL && t0 * G >= cnt) break;
        f32x4 z[U];
        float w[U];
#pragma unroll
        for (int t = 0; t < U; ++t) {
            const int j = (t0 + t) * G + g;
            if constexpr (OFF32) {
                const uint32_t off = (uint32_t)__shfl((int)my_off, j, 64) + colbytes;
                z[t] = *reinterpret_cast<const f32x4*>(zbase + off);
            } else {
                const int u = __shfl(my_u, j, 64);
                z[t] = *reinterpret_cast<const f32x4*>(zbase + (int64_t)u * rowbytes + colbytes);
            }
            if constexpr (WEIGHTED) w[t] = __shfl(my_w, j, 64);
            if constexpr (!FULL) {
                const bool ok = j < cnt;
                z[t].x = ok ? z[t].x : 0.0f;
                z[t].y = ok ? z[t].y : 0.0f;
                z[t].z = ok ? z[t].z : 0.0f;
                z[t].w = ok ? z[t].w : 0.0f;
            }
        }
#pragma unroll
        for (int t = 0; t < U; ++t) {
            if constexpr (WEIGHTED) {
                acc[0] = fmaf(w[t], z[t].x, acc[0]);
                acc[1] = fmaf(w[t], z[t].y, acc[1]);
                acc[2] = fmaf(w[t], z[t].z, acc[2]);
                acc[3] = fmaf(w[t], z[t].w, acc[3]);
            } else {
                acc[0] += z[t].x;
                acc[1] += z[t].y;
                acc[2] += z[t].z;
                acc[3] += z[t].w;
            }
        }
    }
}

// Long rows of the narrow-slab scheme: the NW waves of a workgroup share one
// (row, slab) item, take interleaved 64-edge tiles and combine through LDS.
template <int LPG, int NW, bool WEIGHTED, bool OFF32>
__global__ __launch_bounds__(64 * NW) void agg_grouped_kernel(AggArgs a)
{
    constexpr int SW = 4 * LPG;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t items = a.row_count * a.nslab;
    const int64_t item = (int64_t)blockIdx.x;
    if (item >= items) return;        // uniform over the workgroup
    int64_t slot;
    int slab;
    if (a.slab_major) { slab = (int)(item / a.row_count); slot = item % a.row_count; }
    else              { slot = item / a.nslab; slab = (int)(item % a.nslab); }
    const int v = __builtin_amdgcn_readfirstlane(a.order[a.row_begin + slot]);
    int lo, hi;
    if (a.part_ptr) {
        lo = __builtin_amdgcn_readfirstlane(a.part_ptr[(int64_t)a.part_lo * a.n_rows + a.row_begin + slot]);
        hi = __builtin_amdgcn_readfirstlane(a.part_ptr[(int64_t)a.part_hi * a.n_rows + a.row_begin + slot]);
    } else {
        lo = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v]);
        hi = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v + 1]);
    }

    const int li = lane % LPG, g = lane / LPG;
    const int64_t col = (int64_t)slab * SW + li * 4;
    const bool act = col < a.F;
    const bool writer = act && g == 0 && wave == 0;
    const int valid = (int)min((int64_t)4, a.F - col);
    // lanes past the row width gather the slab's last valid vector instead (never stored)
    const int64_t gcol = act ? col : ((a.F - 1) / 4) * 4;
    const char* zbase = reinterpret_cast<const char*>(a.Z);
    const uint32_t colbytes = (uint32_t)(gcol * 4);
    const int64_t rowbytes = a.ldz * 4;
    float* orow = a.out + (int64_t)v * a.ldo;

    // running sum over the source ranges walked so far (written by the previous launch)
    float prev[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (!a.first && writer) {
        if ((a.out_vec || a.out_half) && valid >= 4) {
            const f32x2 t0 = *reinterpret_cast<const f32x2*>(orow + a.ocol + col);
            const f32x2 t1 = *reinterpret_cast<const f32x2*>(orow + a.ocol + col + 2);
            prev[0] = t0.x; prev[1] = t0.y; prev[2] = t1.x; prev[3] = t1.y;
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (k < valid) prev[k] = orow[a.ocol + col + k];
        }
    }

    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    // the ids (and weights) of a wave's next tile are requested before the current tile's rows
    int nxt_u = lo + 64 * wave + lane < hi ? a.col_idx[lo + 64 * wave + lane] : 0;
    float nxt_w = WEIGHTED ? (lo + 64 * wave + lane < hi ? a.wsrc[nxt_u] : 0.0f) : 1.0f;
    for (int base = lo + 64 * wave; base < hi; base += 64 * NW) {
        const int my_u = nxt_u;
        const float my_w = nxt_w;
        {
            const int en = base + 64 * NW + lane;
            nxt_u = en < hi ? a.col_idx[en] : 0;
            nxt_w = WEIGHTED ? (en < hi ? a.wsrc[nxt_u] : 0.0f) : 1.0f;
        }
        const int cnt = min(64, hi - base);
        const uint32_t my_off = OFF32 ? (uint32_t)my_u * (uint32_t)rowbytes : 0u;
        if (cnt == 64)
            grouped_tile<LPG, true, WEIGHTED, OFF32>(zbase, colbytes, rowbytes, my_off, my_u, my_w, cnt, g, acc);
        else
            grouped_tile<LPG, false, WEIGHTED, OFF32>(zbase, colbytes, rowbytes, my_off, my_u, my_w, cnt, g, acc);
    }
    // combine the lane groups, then the waves (in wave order)
#pragma unroll
    for (int m = LPG; m < 64; m <<= 1)
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[k] += __shfl_xor(acc[k], m, 64);
    __shared__ float red[NW][4][LPG];
    if (g == 0) {
#pragma unroll
        for (int k = 0; k < 4; ++k) red[wave][k][li] = acc[k];
    }
    __syncthreads();
    if (!writer) return;
    const int d = (a.last && a.scale == SCALE_MEAN) ? a.deg[v] : 0;      // only the mean's last range needs it
    float out_v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float x = red[0][k][li];
#pragma unroll
        for (int w = 1; w < NW; ++w) x += red[w][k][li];
        x += prev[k];
        if (a.last) {
            if (a.scale == SCALE_MEAN) x = d > 0 ? x / (float)d : 0.0f;
            else if (a.scale == SCALE_GCN) x = x * a.dinv[v];
        }
        out_v[k] = x;
    }
    store_row<4>(orow + a.ocol + col, out_v, valid, a.out_vec != 0, a.out_half != 0);
    if (a.copy_self && a.first) {
        float zs[4];
        load_row<4>(a.Z + (int64_t)v * a.ldz + col, zs);
        store_row<4>(orow + col, zs, valid, a.self_vec != 0);
    }
}

// ---------------------------------------------------------------------------
// Narrow slabs, ordinary rows: one ROW per lane group.
//
// The G = 64/LPG lane groups of a wave take G consecutive rows of the schedule
// (similar lengths, since the schedule is sorted by degree) and walk their
// neighbour lists in lock step: every wave-wide load fetches the slab of one
// neighbour for each of the G rows.  No cross-group reduction is needed, the
// running-sum read, the scaling and the store are one wave-wide operation for
// G rows, and the per-row bookkeeping is shared — which is what matters once a
// row's share of one source range is only a few dozen entries long.
// Neighbour ids are fetched 8 LPG at a time per group (eight per lane: whole
// cache lines of col_idx, a block ahead) and handed round inside the group
// with ds_bpermute.
// ---------------------------------------------------------------------------
template <int LPG, bool WEIGHTED, bool OFF32>
__global__ __launch_bounds__(64 * kLightWaves) void agg_rowgroup_kernel(AggArgs a)
{
    constexpr int G = 64 / LPG;
    constexpr int SW = 4 * LPG;
    constexpr int U = LPG < 8 ? LPG : 8;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t bundles = (a.row_count + G - 1) / G;
    const int64_t items = bundles * a.nslab;
    const int64_t item = (int64_t)blockIdx.x * kLightWaves + wave;
    if (item >= items) return;
    int64_t bundle;
    int slab;
    if (a.slab_major) { slab = (int)(item / bundles); bundle = item % bundles; }
    else              { bundle = item / a.nslab; slab = (int)(item % a.nslab); }

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

    const int64_t col = (int64_t)slab * SW + li * 4;
    const bool act = col < a.F;
    const bool writer = act && has_row;
    const int valid = (int)min((int64_t)4, a.F - col);
    const int64_t gcol = act ? col : ((a.F - 1) / 4) * 4;
    const char* zbase = reinterpret_cast<const char*>(a.Z);
    const uint32_t colbytes = (uint32_t)(gcol * 4);
    const int64_t rowbytes = a.ldz * 4;
    float* orow = a.out + (int64_t)v * a.ldo;

    float prev[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (!a.first && writer) {
        if (a.out_vec && valid >= 4) {
            const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(orow + a.ocol + col));
            prev[0] = t.x; prev[1] = t.y; prev[2] = t.z; prev[3] = t.w;
        } else if (a.out_half && valid >= 4) {
            const f32x2 t0 = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(orow + a.ocol + col));
            const f32x2 t1 = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(orow + a.ocol + col + 2));
            prev[0] = t0.x; prev[1] = t0.y; prev[2] = t1.x; prev[3] = t1.y;
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (k < valid) prev[k] = orow[a.ocol + col + k];
        }
    }

    const int gaddr = (lane - li) * 4;      // ds_bpermute byte address of this group's lane 0
    // Neighbour ids: every lane of a group fetches eight consecutive ids at a time, so a group reads col_idx in
    // whole cache lines (8 LPG entries: two lines for LPG = 8; measured: 4 per lane 1.4 % slower, 16 per lane
    // 0.6 % slower) instead of one 32-byte piece per LPG entries — the id loads were one L2 request in nine of a
    // kernel that is bound by L2 requests.  Entry e of such a block sits in component e % 8 of the group's
    // lane e / 8.
    constexpr int IPL = 8;
    constexpr int BLOCK = IPL * LPG;
    typedef int i32x4u __attribute__((ext_vector_type(4), aligned(4)));      // 4-byte aligned 16-byte load
    int nxt_u[IPL];
    float nxt_w[IPL];
    auto fetch_ids = [&](int first) {       // entries first + 4 li .. + 3 of this group's row; past its end: id 0
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
        if constexpr (WEIGHTED) {
#pragma unroll
            for (int k = 0; k < IPL; ++k) nxt_w[k] = nb + k < len ? a.wsrc[nxt_u[k]] : 0.0f;
        }
    };
    fetch_ids(0);
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int s0 = 0; s0 < maxlen; s0 += BLOCK) {
        int my_u[IPL];
        float my_w[IPL];
        uint32_t my_off[IPL];
#pragma unroll
        for (int k = 0; k < IPL; ++k) {
            my_u[k] = nxt_u[k];
            my_w[k] = WEIGHTED ? nxt_w[k] : 0.0f;
            my_off[k] = OFF32 ? (uint32_t)my_u[k] * (uint32_t)rowbytes : 0u;
        }
        fetch_ids(s0 + BLOCK);              // the next block, a whole block ahead of its use
        // steps of U entries; the gathers of step st + 1 are issued before those of step st are added up, so a
        // wave has up to 2 U row pieces in flight (two register sets, picked by the parity of the unrolled step)
        constexpr int T = BLOCK / U;
        f32x4 z[2][U];
        float w[2][U];
        // e0: first entry of the step in the block, c0: the same counted from the start of the row's share.  Lanes
        // whose group has no such entry (a shorter row of the bundle, or columns past the row width) issue no
        // load at all: the kernel keeps the address units busy 96 % of its time, and a sixth of the gathers of a
        // bundle are such fillers.
        auto issue = [&](int e0, int c0, f32x4 (&zz)[U], float (&ww)[U]) {
            const bool all = act && c0 + U <= minlen && has_row;       // no filler in this step for this lane
#pragma unroll
            for (int t = 0; t < U; ++t) {
                const int e = e0 + t;              // entry of the block: lane e / IPL, component e % IPL
                const bool ok = all || (act && c0 + t < len);
                const char* src;
                if constexpr (OFF32) {
                    const uint32_t off =
                        (uint32_t)__builtin_amdgcn_ds_bpermute(gaddr + 4 * (e / IPL), (int)my_off[e % IPL]) + colbytes;
                    src = zbase + off;
                } else {
                    const int u = __builtin_amdgcn_ds_bpermute(gaddr + 4 * (e / IPL), my_u[e % IPL]);
                    src = zbase + (int64_t)u * rowbytes + colbytes;
                }
                zz[t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
                if (ok) zz[t] = *reinterpret_cast<const f32x4*>(src);
                if constexpr (WEIGHTED)
                    ww[t] = __int_as_float(__builtin_amdgcn_ds_bpermute(gaddr + 4 * (e / IPL), __float_as_int(my_w[e % IPL])));
            }
        };
        issue(0, s0, z[0], w[0]);
#pragma unroll
        for (int st = 0; st < T; ++st) {
            const int c0 = s0 + st * U;
            if (c0 >= maxlen) break;                   // (uniform)
            if (st + 1 < T && c0 + U < maxlen) issue((st + 1) * U, c0 + U, z[(st + 1) & 1], w[(st + 1) & 1]);
            f32x4 (&zc)[U] = z[st & 1];
            float (&wc)[U] = w[st & 1];
#pragma unroll
            for (int t = 0; t < U; ++t) {
                if constexpr (WEIGHTED) {
                    acc[0] = fmaf(wc[t], zc[t].x, acc[0]);
                    acc[1] = fmaf(wc[t], zc[t].y, acc[1]);
                    acc[2] = fmaf(wc[t], zc[t].z, acc[2]);
                    acc[3] = fmaf(wc[t], zc[t].w, acc[3]);
                } else {
                    acc[0] += zc[t].x;
                    acc[1] += zc[t].y;
                    acc[2] += zc[t].z;
                    acc[3] += zc[t].w;
                }
            }
        }
    }
    if (!writer) return;
    const int d = (a.last && a.scale == SCALE_MEAN) ? a.deg[v] : 0;      // only the mean's last range needs it
    float out_v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float x = acc[k] + prev[k];
        if (a.last) {
            if (a.scale == SCALE_MEAN) x = d > 0 ? x / (float)d : 0.0f;
            else if (a.scale == SCALE_GCN) x = x * a.dinv[v];
        }
        out_v[k] = x;
    }
    if (a.out_vec && valid >= 4) {
        f32x4 t = {out_v[0], out_v[1], out_v[2], out_v[3]};
        __builtin_nontemporal_store(t, reinterpret_cast<f32x4*>(orow + a.ocol + col));
    } else if (a.out_half && valid >= 4) {
        __builtin_nontemporal_store(f32x2{out_v[0], out_v[1]}, reinterpret_cast<f32x2*>(orow + a.ocol + col));
        __builtin_nontemporal_store(f32x2{out_v[2], out_v[3]}, reinterpret_cast<f32x2*>(orow + a.ocol + col + 2));
    } else {
        store_row<4>(orow + a.ocol + col, out_v, valid, false);
    }
    if (a.copy_self && a.first) {
        float zs[4];
        load_row<4>(a.Z + (int64_t)v * a.ldz + col, zs);
        store_row<4>(orow + col, zs, valid, a.self_vec != 0);
    }
}

// ---------------------------------------------------------------------------
// attention scores  el[v,h] = <a_src[h], z_v,h>,  er[v,h] = <a_dst[h], z_v,h>
// one wave per node; padded heads (h >= heads) get 0
// ---------------------------------------------------------------------------
template <int HP>
__global__ __launch_bounds__(256) void gat_scores_kernel(
    int64_t N, int64_t F, int heads, int Dh, const float* Z, int64_t ldz,
    const float* __restrict__ a_src, const float* __restrict__ a_dst,
    float* el, int64_t el_stride, float* __restrict__ er)
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
        if (lane == 0) { el[v * el_stride + h] = s; er[v * HP + h] = t; }
    }
}

// The same scores with 16-byte loads: 16 lanes per node (four nodes per wave), each lane walks the row
// in float4 steps of 64 columns; the per-head partial sums are reduced over the 16 lanes of a node.
// Needs 16-byte aligned rows and F % 4 == 0.
template <int HP>
__global__ __launch_bounds__(256) void gat_scores_vec_kernel(
    int64_t N, int64_t F, int heads, int Dh, const float* Z, int64_t ldz,
    const float* __restrict__ a_src, const float* __restrict__ a_dst,
    float* el, int64_t el_stride, float* __restrict__ er)
{
    const int li = threadIdx.x & 15;
    const int64_t v = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const bool have = v < N;
    const int64_t vv = have ? v : N - 1;                 // idle groups repeat the last node (nothing stored)
    float ps[HP], pd[HP];
#pragma unroll
    for (int h = 0; h < HP; ++h) { ps[h] = 0.0f; pd[h] = 0.0f; }
    const bool whole = Dh % 4 == 0;
    // four row pieces are requested before the first is used (a row of up to 256 columns is one batch)
    for (int64_t c0 = li * 4; c0 < F; c0 += 256) {
        f32x4 zq[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int64_t c = c0 + 64 * q;
            zq[q] = c < F ? *reinterpret_cast<const f32x4*>(Z + vv * ldz + c) : f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int64_t c = c0 + 64 * q;
            if (c >= F) break;
            const f32x4 z = zq[q];
            const f32x4 as = *reinterpret_cast<const f32x4*>(a_src + c);
            const f32x4 ad = *reinterpret_cast<const f32x4*>(a_dst + c);
            const float zs[4] = {z.x, z.y, z.z, z.w}, sa[4] = {as.x, as.y, as.z, as.w}, da[4] = {ad.x, ad.y, ad.z, ad.w};
            if (whole) {
                // the four columns lie in one head: one head index and one add per head for the piece
                const int h = (int)c / Dh;
                const float s = ((zs[0] * sa[0] + zs[1] * sa[1]) + zs[2] * sa[2]) + zs[3] * sa[3];
                const float t = ((zs[0] * da[0] + zs[1] * da[1]) + zs[2] * da[2]) + zs[3] * da[3];
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
                const float s = zs[k] * sa[k], t = zs[k] * da[k];
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
        for (int h = 0; h < HP; ++h) { el[v * el_stride + h] = ps[h]; er[v * HP + h] = pd[h]; }
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
                const f32x4 t = *reinterpret_cast<const f32x4*>(a.el + (int64_t)my_u * a.el_stride);
                elu[0] = t.x; elu[1] = t.y; elu[2] = t.z; elu[3] = t.w;
            } else {
#pragma unroll
                for (int h = 0; h < HP; ++h) elu[h] = a.el[(int64_t)my_u * a.el_stride + h];
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
        store_row<VEC>(orow + a.ocol + col, r, valid, a.out_vec != 0, a.out_half != 0);
        if (a.copy_self) {
            float zs[VEC];
            load_row<VEC>(a.Z + (int64_t)v * a.ldz + col, zs);
            store_row<VEC>(orow + col, zs, valid, a.self_vec != 0);
        }
    }
}

// ---------------------------------------------------------------------------
// gat_softmax, float4 gathers with 32-bit row offsets, software-pipelined.
//
// Same arithmetic as agg_gat_kernel, arranged so that memory latency and the
// score arithmetic overlap: as soon as a tile's neighbour ids are known the
// first batch of feature rows is requested, and the scores, wave reductions and
// exponentials of the tile are computed while those rows are in flight.  The
// per-edge, per-head weights go through a wave-private LDS array, so that a
// lane picks up the weight of its own head with one ds_read whose address is
// an immediate offset (no readlane + select chain per neighbour).  Lanes past
// the end of a tile carry the tile's first neighbour with weight zero, so every
// gather address is valid and nothing in the loop branches per lane.
// ---------------------------------------------------------------------------
template <int NC, int NW, int HP, bool HU, bool TRAIN>
__global__ __launch_bounds__(64 * (NW == 1 ? kLightWaves : NW)) void agg_gat_fast_kernel(AggArgs a)
{
    constexpr int WAVES = NW == 1 ? kLightWaves : NW;
    constexpr int U = 4;
    // TRAIN: the aggregate is accumulated in two parts, entries with a non-positive score (acc) and
    // with a positive score (accp), each with its own weight per edge (zero for the other kind); the
    // backward pass needs the two parts separately, each accurate relative to its own size
    constexpr int WSETS = TRAIN ? 2 : 1;
    __shared__ float wl[WAVES][WSETS][HP][64];
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

    const int64_t col0 = (int64_t)slab * (256 * NC) + lane * 4;
    bool act[NC];
    uint32_t colbytes[NC];
    int hc[NC][HU ? 1 : 4];
    float acc[NC][4], accp[TRAIN ? NC : 1][4];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int64_t col = col0 + c * 256;
        act[c] = col < a.F;
        // lanes past the row width gather the last valid vector instead (never stored)
        colbytes[c] = (uint32_t)((act[c] ? col : ((a.F - 1) / 4) * 4) * 4);
#pragma unroll
        for (int k = 0; k < (HU ? 1 : 4); ++k) hc[c][k] = min((int)((col + k) / a.Dh), a.heads - 1);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            acc[c][k] = 0.0f;
            if constexpr (TRAIN) accp[c][k] = 0.0f;
        }
    }
    const char* zbase = reinterpret_cast<const char*>(a.Z);
    const uint32_t rowbytes = (uint32_t)(a.ldz * 4);
    float* myw = &wl[wave][0][0][0];
    float* mywp = &wl[wave][WSETS - 1][0][0];

    // sp, sn: the parts of s from entries with a positive / non-positive score (kept apart so that a
    // share that is structurally zero comes out as an exact zero)
    float m[HP], s[HP], sp[TRAIN ? HP : 1], sn[TRAIN ? HP : 1], erv[HP];
#pragma unroll
    for (int h = 0; h < HP; ++h) {
        m[h] = -INFINITY;
        s[h] = 0.0f;
        if constexpr (TRAIN) { sp[h] = 0.0f; sn[h] = 0.0f; }
        erv[h] = a.er ? a.er[(int64_t)v * HP + h] : 0.0f;
    }
    // no table of destination scores: this row's come from the row itself.  The row is requested here and
    // used in the first tile, behind that tile's gathers, so that its latency is not one more step of the chain.
    f32x4 zself[NC];
    if (!a.er) {
#pragma unroll
        for (int c = 0; c < NC; ++c)
            zself[c] = *reinterpret_cast<const f32x4*>(zbase + (uint32_t)v * rowbytes + colbytes[c]);
    }
    const int base0 = lo + 64 * (NW == 1 ? 0 : wave);

    for (int base = lo + 64 * (NW == 1 ? 0 : wave); base < hi; base += 64 * NW) {
        const int e = base + lane;
        const bool valid = e < hi;
        const int cnt = min(64, hi - base);
        int my_u = valid ? a.col_idx[e] : 0;
        my_u = valid ? my_u : bcast_i(my_u, 0);          // lane 0 is always valid
        const int my_off = (int)((uint32_t)my_u * rowbytes);

        // first batch of rows is requested before the scores are computed
        f32x4 zq[U][NC];
#pragma unroll
        for (int t = 0; t < U; ++t) {
            const uint32_t off = (uint32_t)bcast_i(my_off, t);
#pragma unroll
            for (int c = 0; c < NC; ++c)
                zq[t][c] = *reinterpret_cast<const f32x4*>(zbase + off + colbytes[c]);
        }

        float elu[HP];
        if constexpr (HP == 4) {
            const f32x4 t = *reinterpret_cast<const f32x4*>(a.el + (int64_t)my_u * a.el_stride);
            elu[0] = t.x; elu[1] = t.y; elu[2] = t.z; elu[3] = t.w;
        } else {
#pragma unroll
            for (int h = 0; h < HP; ++h) elu[h] = a.el[(int64_t)my_u * a.el_stride + h];
        }
        if (!a.er && base == base0) {          // (uniform)
            float pd[HP];
#pragma unroll
            for (int h = 0; h < HP; ++h) pd[h] = 0.0f;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                if (!act[c]) continue;
                const f32x4 ad = *reinterpret_cast<const f32x4*>(a.er_from + col0 + c * 256);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float t = zself[c][k] * ad[k];
                    const int hk = hc[c][HU ? 0 : k];
#pragma unroll
                    for (int h = 0; h < HP; ++h) pd[h] += hk == h ? t : 0.0f;
                }
            }
#pragma unroll
            for (int h = 0; h < HP; ++h) erv[h] = wave_sum(pd[h]);
        }
        float scale[HP];
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
            if constexpr (TRAIN) {
                const float pp = x > 0.0f ? pe : 0.0f, pn = x > 0.0f ? 0.0f : pe;
                sp[h] = sp[h] * scale[h] + wave_sum(pp);
                sn[h] = sn[h] * scale[h] + wave_sum(pn);
                myw[h * 64 + lane] = pn;
                mywp[h * 64 + lane] = pp;
            } else {
                myw[h * 64 + lane] = pe;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if (base != lo + 64 * (NW == 1 ? 0 : wave)) {
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float f = select_head<HP>(scale, hc[c][HU ? 0 : k]);
                    acc[c][k] *= f;
                    if constexpr (TRAIN) accp[c][k] *= f;
                }
        }

        for (int j = 0; j < cnt; j += U) {
            // request the next batch, then consume the current one
            f32x4 zn[U][NC];
            const bool more = j + U < cnt;
            if (more) {
#pragma unroll
                for (int t = 0; t < U; ++t) {
                    const uint32_t off = (uint32_t)bcast_i(my_off, (j + U + t) & 63);
#pragma unroll
                    for (int c = 0; c < NC; ++c)
                        zn[t][c] = *reinterpret_cast<const f32x4*>(zbase + off + colbytes[c]);
                }
            }
#pragma unroll
            for (int t = 0; t < U; ++t) {
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    if constexpr (HU) {
                        const float w = myw[hc[c][0] * 64 + j + t];
                        acc[c][0] = fmaf(w, zq[t][c].x, acc[c][0]);
                        acc[c][1] = fmaf(w, zq[t][c].y, acc[c][1]);
                        acc[c][2] = fmaf(w, zq[t][c].z, acc[c][2]);
                        acc[c][3] = fmaf(w, zq[t][c].w, acc[c][3]);
                        if constexpr (TRAIN) {
                            const float wq = mywp[hc[c][0] * 64 + j + t];
                            accp[c][0] = fmaf(wq, zq[t][c].x, accp[c][0]);
                            accp[c][1] = fmaf(wq, zq[t][c].y, accp[c][1]);
                            accp[c][2] = fmaf(wq, zq[t][c].z, accp[c][2]);
                            accp[c][3] = fmaf(wq, zq[t][c].w, accp[c][3]);
                        }
                    } else {
                        acc[c][0] = fmaf(myw[hc[c][0] * 64 + j + t], zq[t][c].x, acc[c][0]);
                        acc[c][1] = fmaf(myw[hc[c][1] * 64 + j + t], zq[t][c].y, acc[c][1]);
                        acc[c][2] = fmaf(myw[hc[c][2] * 64 + j + t], zq[t][c].z, acc[c][2]);
                        acc[c][3] = fmaf(myw[hc[c][3] * 64 + j + t], zq[t][c].w, acc[c][3]);
                        if constexpr (TRAIN) {
                            accp[c][0] = fmaf(mywp[hc[c][0] * 64 + j + t], zq[t][c].x, accp[c][0]);
                            accp[c][1] = fmaf(mywp[hc[c][1] * 64 + j + t], zq[t][c].y, accp[c][1]);
                            accp[c][2] = fmaf(mywp[hc[c][2] * 64 + j + t], zq[t][c].z, accp[c][2]);
                            accp[c][3] = fmaf(mywp[hc[c][3] * 64 + j + t], zq[t][c].w, accp[c][3]);
                        }
                    }
                }
            }
            if (more) {
#pragma unroll
                for (int t = 0; t < U; ++t)
#pragma unroll
                    for (int c = 0; c < NC; ++c) zq[t][c] = zn[t][c];
            }
        }
    }

    if constexpr (NW > 1) {
        __shared__ float red[NW][NC * 4 * WSETS][64];
        __shared__ float mred[NW][HP], sred[NW][HP], spred[NW][HP], snred[NW][HP];
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                red[wave][c * 4 + k][lane] = acc[c][k];
                if constexpr (TRAIN) red[wave][NC * 4 + c * 4 + k][lane] = accp[c][k];
            }
        if (lane == 0) {
#pragma unroll
            for (int h = 0; h < HP; ++h) {
                mred[wave][h] = m[h];
                sred[wave][h] = s[h];
                if constexpr (TRAIN) { spred[wave][h] = sp[h]; snred[wave][h] = sn[h]; }
            }
        }
        __syncthreads();
        if (wave != 0) return;
        float f[NW][HP];
#pragma unroll
        for (int h = 0; h < HP; ++h) {
            float mm = mred[0][h];
#pragma unroll
            for (int w = 1; w < NW; ++w) mm = fmaxf(mm, mred[w][h]);
            float ss = 0.0f, pp = 0.0f, nn = 0.0f;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                f[w][h] = (mred[w][h] == -INFINITY) ? 0.0f : expf(mred[w][h] - mm);
                ss += sred[w][h] * f[w][h];
                if constexpr (TRAIN) { pp += spred[w][h] * f[w][h]; nn += snred[w][h] * f[w][h]; }
            }
            s[h] = ss;
            m[h] = mm;
            if constexpr (TRAIN) { sp[h] = pp; sn[h] = nn; }
        }
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float t = 0.0f, tp = 0.0f;
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    const float fw = select_head<HP>(f[w], hc[c][HU ? 0 : k]);
                    t += red[w][c * 4 + k][lane] * fw;
                    if constexpr (TRAIN) tp += red[w][NC * 4 + c * 4 + k][lane] * fw;
                }
                acc[c][k] = t;
                if constexpr (TRAIN) accp[c][k] = tp;
            }
    }

    float* orow = a.out + (int64_t)v * a.ldo;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        if (!act[c]) continue;
        const int64_t col = col0 + c * 256;
        const int valid = (int)min((int64_t)4, a.F - col);
        float r[4];
        if constexpr (TRAIN) {
            float rp[4], rn[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float den = select_head<HP>(s, hc[c][HU ? 0 : k]);
                r[k] = den > 0.0f ? (acc[c][k] + accp[c][k]) / den : 0.0f;
                rp[k] = den > 0.0f ? accp[c][k] / den : 0.0f;
                rn[k] = den > 0.0f ? acc[c][k] / den : 0.0f;
            }
            store_row<4>(a.save_pos + (int64_t)v * a.ld_pos + col, rp, valid, true);
            store_row<4>(a.save_neg + (int64_t)v * a.ld_pos + col, rn, valid, true);
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float den = select_head<HP>(s, hc[c][HU ? 0 : k]);
                r[k] = den > 0.0f ? acc[c][k] / den : 0.0f;
            }
        }
        store_row<4>(orow + a.ocol + col, r, valid, a.out_vec != 0, a.out_half != 0);
        if (a.copy_self) {
            float zs[4];
            load_row<4>(a.Z + (int64_t)v * a.ldz + col, zs);
            store_row<4>(orow + col, zs, valid, a.self_vec != 0);
        }
    }
    if constexpr (TRAIN) {
        if (lane == 0 && slab == 0) {
#pragma unroll
            for (int h = 0; h < HP; ++h) {
                const bool any = s[h] > 0.0f;
                const float rs = any ? 1.0f / s[h] : 0.0f;
                const f32x4 t = {any ? m[h] : 0.0f, rs, sp[h] * rs, sn[h] * rs};
                a.save_stats[(int64_t)v * HP + h] = t;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
template <int VEC, int NC, bool MAXOP>
void launch_linear_pair(const AggArgs& base, int64_t n_heavy, int64_t N, hipStream_t stream)
{
    if (n_heavy > 0) {
        AggArgs a = base;
        a.row_begin = 0;
        a.row_count = n_heavy;
        const int64_t blocks = n_heavy * a.nslab;
        agg_linear_kernel<VEC, NC, kHeavyWaves, MAXOP><<<dim3((unsigned)blocks), dim3(64 * kHeavyWaves), 0, stream>>>(a);
    }
    if (N > n_heavy) {
        AggArgs a = base;
        a.row_begin = n_heavy;
        a.row_count = N - n_heavy;
        const int64_t blocks = (a.row_count * a.nslab + kLightWaves - 1) / kLightWaves;
        agg_linear_kernel<VEC, NC, 1, MAXOP><<<dim3((unsigned)blocks), dim3(64 * kLightWaves), 0, stream>>>(a);
    }
}

template <int LPG, bool WEIGHTED, bool OFF32>
void launch_grouped_pair(const AggArgs& base, int64_t n_heavy, int64_t N, hipStream_t stream)
{
    if (n_heavy > 0) {
        AggArgs a = base;
        a.row_begin = 0;
        a.row_count = n_heavy;
        const int64_t blocks = n_heavy * a.nslab;
        agg_grouped_kernel<LPG, kHeavyWaves, WEIGHTED, OFF32>
            <<<dim3((unsigned)blocks), dim3(64 * kHeavyWaves), 0, stream>>>(a);
    }
    if (N > n_heavy) {
        AggArgs a = base;
        a.row_begin = n_heavy;
        a.row_count = N - n_heavy;
        const int64_t bundles = (a.row_count + (64 / LPG) - 1) / (64 / LPG);
        const int64_t blocks = (bundles * a.nslab + kLightWaves - 1) / kLightWaves;
        agg_rowgroup_kernel<LPG, WEIGHTED, OFF32>
            <<<dim3((unsigned)blocks), dim3(64 * kLightWaves), 0, stream>>>(a);
    }
}

template <int LPG>
void dispatch_grouped(const AggArgs& a, int64_t n_heavy, int64_t N, bool weighted, bool off32, hipStream_t s)
{
    if (weighted) {
        if (off32) launch_grouped_pair<LPG, true, true>(a, n_heavy, N, s);
        else launch_grouped_pair<LPG, true, false>(a, n_heavy, N, s);
    } else {
        if (off32) launch_grouped_pair<LPG, false, true>(a, n_heavy, N, s);
        else launch_grouped_pair<LPG, false, false>(a, n_heavy, N, s);
    }
}

// ---------------------------------------------------------------------------
// gat_softmax for rows of ordinary length when the whole row fits one wave
// (F <= 256, four floats per lane) and a head is a power-of-two group of lanes:
// the score of an entry is computed from the gathered source row itself.
//
// The kernels above fetch el[u] = <a_src, z_u> from a table, one 16-byte read
// per entry, which on a graph whose table misses L2 costs a whole extra cache
// line per entry next to the eight lines of the row.  Here every lane
// multiplies its four floats of z_u with its four floats of a_src, the lanes of
// a head add up over the group with DPP moves, and the softmax runs online over
// batches of four entries (running maximum m, sum s and weighted row acc per
// lane, all three rescaled when the maximum moves).  Scores are kept in units
// of log2(e) (LeakyReLU commutes with a positive factor) so that every
// exponential is one v_exp_f32.  The destination's own score <a_dst, z_v> is formed
// the same way from row v when `attn_dst` is given (the plain forward: no score
// kernel runs at all); with attn_dst == NULL it is read from the table (save mode).
// NW > 1: the waves of a workgroup share one long row, take interleaved 64-entry
// tiles and merge their (m, s, acc) triples through LDS in wave order.
// ---------------------------------------------------------------------------
// TRAIN (save mode): the aggregate is accumulated in two parts, entries with a positive score (accp) and the
// others (acc), with the sums of their weights (sp, sn), and the row statistics are kept for the backward
// pass; scores then stay in natural units, because the stored row maximum is used as such.
template <int G, bool TRAIN, int NW>
__global__ __launch_bounds__(64 * (NW == 1 ? kLightWaves : NW)) void agg_gat_flash_kernel(
    AggArgs a, const float* __restrict__ attn_src, const float* __restrict__ attn_dst, int er_stride)
{
    static_assert(!(TRAIN && NW > 1), "save mode keeps the long rows on the table kernel");
    constexpr int U = 4;      // entries per batch of the online softmax (2 and 8 measure the same: the kernel waits for memory)
    constexpr float kLog2e = 1.4426950408889634f;
    constexpr float kIn = TRAIN ? 1.0f : kLog2e;       // factor on the scores as they are formed
    constexpr float kEx = TRAIN ? kLog2e : 1.0f;       // factor inside the exponentials
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t slot = NW == 1 ? (int64_t)blockIdx.x * kLightWaves + wave : (int64_t)blockIdx.x;
    if (slot >= a.row_count) return;          // NW > 1: uniform over the workgroup
    const int v = __builtin_amdgcn_readfirstlane(a.order[a.row_begin + slot]);
    const int lo = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v]);
    const int hi = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v + 1]);

    const int64_t col = lane * 4;
    const bool act = col < a.F;
    // lanes past the row width gather the last valid vector instead (never stored, weight vector zero)
    const uint32_t colbytes = (uint32_t)((act ? col : ((a.F - 1) / 4) * 4) * 4);
    const int h = min((int)(col / a.Dh), a.heads - 1);
    f32x4 as = {0.0f, 0.0f, 0.0f, 0.0f};
    float erv = 0.0f;
    const char* zbase = reinterpret_cast<const char*>(a.Z);
    const uint32_t rowbytes = (uint32_t)(a.ldz * 4);
    if (act) {
        as = *reinterpret_cast<const f32x4*>(attn_src + col);        // [heads, Dh] is F contiguous floats
        as.x *= kIn; as.y *= kIn; as.z *= kIn; as.w *= kIn;
        if (!attn_dst) erv = a.er[(int64_t)v * er_stride + h] * kIn;
    }
    if (attn_dst) {
        // (uniform branch) every lane takes part in the sums; lanes past the row width add zero
        f32x4 ad = {0.0f, 0.0f, 0.0f, 0.0f};
        if (act) ad = *reinterpret_cast<const f32x4*>(attn_dst + col);
        const f32x4 zv = *reinterpret_cast<const f32x4*>(zbase + (uint32_t)v * rowbytes + colbytes);
        float d = (ad.x * kIn) * zv.x;
        d = fmaf(ad.y * kIn, zv.y, d);
        d = fmaf(ad.z * kIn, zv.z, d);
        d = fmaf(ad.w * kIn, zv.w, d);
        erv = group_sum<G>(d);
    }

    float m = -INFINITY, s = 0.0f, sp = 0.0f, sn = 0.0f;
    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f}, accp = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int base = lo + (NW == 1 ? 0 : 64 * wave); base < hi; base += 64 * NW) {
        const int e = base + lane;
        const bool valid = e < hi;
        const int cnt = min(64, hi - base);
        int my_u = valid ? a.col_idx[e] : 0;
        my_u = valid ? my_u : bcast_i(my_u, 0);          // lane 0 is always valid
        const int my_off = (int)((uint32_t)my_u * rowbytes);

        f32x4 zq[U];
#pragma unroll
        for (int t = 0; t < U; ++t)
            zq[t] = *reinterpret_cast<const f32x4*>(zbase + (uint32_t)bcast_i(my_off, t) + colbytes);

        for (int j = 0; j < cnt; j += U) {
            // request the next batch, then consume the current one
            f32x4 zn[U];
            const bool more = j + U < cnt;
            if (more) {
#pragma unroll
                for (int t = 0; t < U; ++t)
                    zn[t] = *reinterpret_cast<const f32x4*>(zbase + (uint32_t)bcast_i(my_off, (j + U + t) & 63) + colbytes);
            }
            float x[U], sc[U];
#pragma unroll
            for (int t = 0; t < U; ++t) {
                float d = as.x * zq[t].x;
                d = fmaf(as.y, zq[t].y, d);
                d = fmaf(as.z, zq[t].z, d);
                d = fmaf(as.w, zq[t].w, d);
                x[t] = group_sum<G>(d) + erv;
                sc[t] = (j + t < cnt) ? (x[t] > 0.0f ? x[t] : a.slope * x[t]) : -INFINITY;   // entries past the tile weigh nothing
            }
            float mn = m;
#pragma unroll
            for (int t = 0; t < U; ++t) mn = fmaxf(mn, sc[t]);                           // finite: entry j of the tile is real
            const float scale = __builtin_amdgcn_exp2f((m - mn) * kEx);
            float pw[U];
#pragma unroll
            for (int t = 0; t < U; ++t) pw[t] = __builtin_amdgcn_exp2f((sc[t] - mn) * kEx);
            float ps = 0.0f;
#pragma unroll
            for (int t = 0; t < U; ++t) ps += pw[t];
            s = s * scale + ps;
            acc.x *= scale; acc.y *= scale; acc.z *= scale; acc.w *= scale;
            if constexpr (TRAIN) {
                float pps = 0.0f, pns = 0.0f;
                accp.x *= scale; accp.y *= scale; accp.z *= scale; accp.w *= scale;
#pragma unroll
                for (int t = 0; t < U; ++t) {
                    const float pp = x[t] > 0.0f ? pw[t] : 0.0f, pn = x[t] > 0.0f ? 0.0f : pw[t];
                    pps += pp;
                    pns += pn;
                    accp.x = fmaf(pp, zq[t].x, accp.x);
                    accp.y = fmaf(pp, zq[t].y, accp.y);
                    accp.z = fmaf(pp, zq[t].z, accp.z);
                    accp.w = fmaf(pp, zq[t].w, accp.w);
                    acc.x = fmaf(pn, zq[t].x, acc.x);
                    acc.y = fmaf(pn, zq[t].y, acc.y);
                    acc.z = fmaf(pn, zq[t].z, acc.z);
                    acc.w = fmaf(pn, zq[t].w, acc.w);
                }
                sp = sp * scale + pps;
                sn = sn * scale + pns;
            } else {
#pragma unroll
                for (int t = 0; t < U; ++t) {
                    acc.x = fmaf(pw[t], zq[t].x, acc.x);
                    acc.y = fmaf(pw[t], zq[t].y, acc.y);
                    acc.z = fmaf(pw[t], zq[t].z, acc.z);
                    acc.w = fmaf(pw[t], zq[t].w, acc.w);
                }
            }
            m = mn;
            if (more) {
#pragma unroll
                for (int t = 0; t < U; ++t) zq[t] = zn[t];
            }
        }
    }

    if constexpr (NW > 1) {
        // merge the waves' running triples, in wave order
        __shared__ float red[NW][6][64];
        red[wave][0][lane] = m;
        red[wave][1][lane] = s;
        red[wave][2][lane] = acc.x;
        red[wave][3][lane] = acc.y;
        red[wave][4][lane] = acc.z;
        red[wave][5][lane] = acc.w;
        __syncthreads();
        if (wave != 0) return;
        float mm = red[0][0][lane];
#pragma unroll
        for (int w = 1; w < NW; ++w) mm = fmaxf(mm, red[w][0][lane]);
        s = 0.0f;
        acc = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float mw = red[w][0][lane];
            // a wave that saw no entry has m = -inf and weighs nothing
            const float f = mw == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f((mw - mm) * kEx);
            s = fmaf(red[w][1][lane], f, s);
            acc.x = fmaf(red[w][2][lane], f, acc.x);
            acc.y = fmaf(red[w][3][lane], f, acc.y);
            acc.z = fmaf(red[w][4][lane], f, acc.z);
            acc.w = fmaf(red[w][5][lane], f, acc.w);
        }
        m = mm;
    }

    if constexpr (TRAIN) {
        // statistics: one lane per head; the padded heads carry no columns and look like a uniform softmax
        if (act && (lane % G) == 0 && col < (int64_t)a.heads * a.Dh) {
            const bool any = s > 0.0f;
            const float rs = any ? 1.0f / s : 0.0f;
            a.save_stats[(int64_t)v * er_stride + h] = f32x4{any ? m : 0.0f, rs, sp * rs, sn * rs};
        }
        if (lane == 0) {
            const bool any = hi > lo;
            const f32x4 t = {0.0f, any ? 1.0f / (float)(hi - lo) : 0.0f, 0.0f, any ? 1.0f : 0.0f};
            for (int k = a.heads; k < er_stride; ++k) a.save_stats[(int64_t)v * er_stride + k] = t;
        }
    }
    if (!act) return;
    float* orow = a.out + (int64_t)v * a.ldo;
    float r[4];
    if constexpr (TRAIN) {
        float rp[4], rn[4];
        const float ap[4] = {accp.x, accp.y, accp.z, accp.w}, an[4] = {acc.x, acc.y, acc.z, acc.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            r[k] = s > 0.0f ? (an[k] + ap[k]) / s : 0.0f;
            rp[k] = s > 0.0f ? ap[k] / s : 0.0f;
            rn[k] = s > 0.0f ? an[k] / s : 0.0f;
        }
        store_row<4>(a.save_pos + (int64_t)v * a.ld_pos + col, rp, 4, true);
        store_row<4>(a.save_neg + (int64_t)v * a.ld_pos + col, rn, 4, true);
    } else {
        r[0] = s > 0.0f ? acc.x / s : 0.0f;
        r[1] = s > 0.0f ? acc.y / s : 0.0f;
        r[2] = s > 0.0f ? acc.z / s : 0.0f;
        r[3] = s > 0.0f ? acc.w / s : 0.0f;
    }
    store_row<4>(orow + a.ocol + col, r, 4, a.out_vec != 0, a.out_half != 0);
    if (a.copy_self) {
        float zs[4];
        load_row<4>(a.Z + (int64_t)v * a.ldz + col, zs);
        store_row<4>(orow + col, zs, 4, a.self_vec != 0);
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

template <int NC, int HP, bool HU, bool TRAIN>
void launch_gat_fast_pair(const AggArgs& base, int64_t n_heavy, int64_t N, hipStream_t stream)
{
    if (n_heavy > 0) {
        AggArgs a = base;
        a.row_begin = 0;
        a.row_count = n_heavy;
        const int64_t blocks = n_heavy * a.nslab;
        agg_gat_fast_kernel<NC, kHeavyWaves, HP, HU, TRAIN><<<dim3((unsigned)blocks), dim3(64 * kHeavyWaves), 0, stream>>>(a);
    }
    if (N > n_heavy) {
        AggArgs a = base;
        a.row_begin = n_heavy;
        a.row_count = N - n_heavy;
        const int64_t blocks = (a.row_count * a.nslab + kLightWaves - 1) / kLightWaves;
        agg_gat_fast_kernel<NC, 1, HP, HU, TRAIN><<<dim3((unsigned)blocks), dim3(64 * kLightWaves), 0, stream>>>(a);
    }
}

template <int HP, bool HU>
void dispatch_gat_fast(int nc, bool train, const AggArgs& a, int64_t nh, int64_t N, hipStream_t s)
{
    if (train) {
        if (nc == 1) launch_gat_fast_pair<1, HP, HU, true>(a, nh, N, s);
        else launch_gat_fast_pair<2, HP, HU, true>(a, nh, N, s);
    } else {
        if (nc == 1) launch_gat_fast_pair<1, HP, HU, false>(a, nh, N, s);
        else launch_gat_fast_pair<2, HP, HU, false>(a, nh, N, s);
    }
}

template <int VEC, bool MAXOP>
void dispatch_linear_nc(int nc, const AggArgs& a, int64_t nh, int64_t N, hipStream_t s)
{
    if (nc == 1) launch_linear_pair<VEC, 1, MAXOP>(a, nh, N, s);
    else if (nc == 2) launch_linear_pair<VEC, 2, MAXOP>(a, nh, N, s);
    else launch_linear_pair<VEC, 3, MAXOP>(a, nh, N, s);
}

template <int VEC>
void dispatch_linear(int nc, bool maxop, const AggArgs& a, int64_t nh, int64_t N, hipStream_t s)
{
    if (maxop) dispatch_linear_nc<VEC, true>(nc, a, nh, N, s);
    else dispatch_linear_nc<VEC, false>(nc, a, nh, N, s);
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

GatWorkspace gat_workspace(int64_t N, int64_t F, int heads, bool save)
{
    const int64_t n = N > 0 ? N : 1, hp = heads_padded(heads);
    GatWorkspace w;
    int64_t off = 0;
    w.el = off; off += align_up(n * hp * (int64_t)sizeof(float), 256);
    w.er = off; off += align_up(n * hp * (int64_t)sizeof(float), 256);
    w.ld_pos = align_up(F > 0 ? F : 1, 32);
    w.stats = off; if (save) off += align_up(n * hp * 16, 256);
    w.pos = off;   if (save) off += align_up(n * w.ld_pos * (int64_t)sizeof(float), 256);
    w.neg = off;   if (save) off += align_up(n * w.ld_pos * (int64_t)sizeof(float), 256);
    w.total = off;
    return w;
}

int64_t aggregate_workspace_bytes(int64_t N, int mode, int heads, int64_t F, bool save)
{
    if (mode != RETEXO_GAT_SOFTMAX) return 0;
    return gat_workspace(N, F, heads, save).total;
}

void launch_gat_scores(int64_t N, int64_t F, int heads, const float* Z, int64_t ldz,
                       const float* a_src, const float* a_dst, float* el, float* er, hipStream_t stream,
                       int64_t el_stride)
{
    const int Dh = (int)(F / heads);
    if (el_stride == 0) el_stride = heads_padded(heads);
    if (F % 4 == 0 && aligned_for(Z, ldz, 4) && aligned_for(a_src, 4, 4) && aligned_for(a_dst, 4, 4) && agg_options().max_vec >= 4) {
        const unsigned gv = (unsigned)((N + 15) / 16);
        if (heads_padded(heads) == 4)
            gat_scores_vec_kernel<4><<<dim3(gv), dim3(256), 0, stream>>>(N, F, heads, Dh, Z, ldz, a_src, a_dst, el, el_stride, er);
        else
            gat_scores_vec_kernel<8><<<dim3(gv), dim3(256), 0, stream>>>(N, F, heads, Dh, Z, ldz, a_src, a_dst, el, el_stride, er);
        return;
    }
    const unsigned gb = (unsigned)((N + 3) / 4);
    if (heads_padded(heads) == 4)
        gat_scores_kernel<4><<<dim3(gb), dim3(256), 0, stream>>>(N, F, heads, Dh, Z, ldz, a_src, a_dst, el, el_stride, er);
    else
        gat_scores_kernel<8><<<dim3(gb), dim3(256), 0, stream>>>(N, F, heads, Dh, Z, ldz, a_src, a_dst, el, el_stride, er);
}

namespace {

// widest gather the layout of Z allows; a partial last vector may read
// padding columns of the same row, so the padded width must fit in ldz
int gather_vec(const AggCall& c)
{
    int vec = 1;
    if (aligned_for(c.Z, c.ldz, 4) && align_up(c.F, 4) <= c.ldz) vec = 4;
    else if (aligned_for(c.Z, c.ldz, 2) && align_up(c.F, 2) <= c.ldz) vec = 2;
    if (vec > agg_options().max_vec) vec = agg_options().max_vec >= 2 ? 2 : 1;
    if (c.mode == RETEXO_GAT_SOFTMAX && vec == 2) vec = 1;
    return vec;
}

// Which edge-softmax kernels a call takes.
struct GatRoute {
    int vec;
    bool off32;     // every byte offset into Z fits 32 bits
    bool flash;     // rows of ordinary length: source scores from the gathered rows themselves
    bool in_rows;   // source scores kept in the unused columns of Z's own rows
};
GatRoute gat_route(const AggCall& c)
{
    const AggOptions& opt = agg_options();
    const int64_t N = c.plan->N;
    GatRoute r;
    r.vec = gather_vec(c);
    r.off32 = (N * c.ldz + c.F) * 4 < (1ll << 32) && !opt.wide_offsets;
    const int hp = heads_padded(c.heads);
    const int64_t Dh = c.F / c.heads;
    const int64_t g = Dh / 4;
    // rows of ordinary length compute the source scores from the gathered rows themselves when a head is
    // a power-of-two group of four-float lanes; the long rows keep the table of scores
    r.flash = r.vec == 4 && r.off32 && opt.gat_fast && opt.gat_flash && c.F <= 256 &&
              Dh % 4 == 0 && g <= 64 && (g & (g - 1)) == 0 && aligned_for(c.attn_src, 4, 4);
    // Otherwise, when Z is the library's own buffer and its rows have unused columns behind F, the source
    // scores of a node are kept there: the gather of a row then brings them along in the row's last cache
    // line, instead of one more line per entry from a table elsewhere.
    r.in_rows = c.z_padding_free && !r.flash && r.vec == 4 && r.off32 && opt.gat_fast && opt.gat_in_rows &&
                c.F % 4 == 0 && c.ldz - c.F >= hp && c.F % 32 != 0 && (c.F % 32) + hp <= 32;
    return r;
}

// One wave per row of W (and one for b): copy the row and append its products with the heads of a_src.
__global__ __launch_bounds__(256) void gat_fold_kernel(int D_in, int F, int heads, int Dh, int hp,
                                                       const float* __restrict__ W, const float* __restrict__ b,
                                                       const float* __restrict__ a_src,
                                                       float* __restrict__ W2, float* __restrict__ b2)
{
    const int lane = threadIdx.x & 63;
    const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (k > D_in) return;
    const float* src = k < D_in ? W + (int64_t)k * F : b;        // b == NULL: a zero bias
    float* dst = k < D_in ? W2 + (int64_t)k * (F + hp) : b2;
    float ps[8];
#pragma unroll
    for (int h = 0; h < 8; ++h) ps[h] = 0.0f;
    for (int j = lane; j < F; j += 64) {
        const float x = src ? src[j] : 0.0f;
        dst[j] = x;
        const float t = x * a_src[j];
        const int hj = j / Dh;
#pragma unroll
        for (int h = 0; h < 8; ++h) ps[h] += hj == h ? t : 0.0f;
    }
#pragma unroll
    for (int h = 0; h < 8; ++h) {
        const float sum = wave_sum(ps[h]);
        if (lane == 0 && h < hp) dst[F + h] = h < heads ? sum : 0.0f;
    }
}

}  // namespace

bool gat_fold_plan(const AggCall& c, int64_t D_in, int64_t avail_bytes)
{
    if (c.mode != RETEXO_GAT_SOFTMAX || c.save || !agg_options().gat_fold) return false;
    const GatRoute r = gat_route(c);
    const int64_t wide = c.F + heads_padded(c.heads);
    // the pipelined kernel forms the destination scores from whole rows: one slab (two float4 per lane at most)
    return r.in_rows && c.F <= 512 && agg_options().slab_cols == 0 && aligned_for(c.attn_dst, 4, 4) &&
           (D_in + 1) * wide * (int64_t)sizeof(float) <= avail_bytes;
}

void launch_gat_fold(int64_t D_in, int64_t F, int heads, const float* W, const float* b, const float* a_src,
                     float* W2, float* b2, hipStream_t stream)
{
    gat_fold_kernel<<<dim3((unsigned)((D_in + 1 + 3) / 4)), dim3(256), 0, stream>>>(
        (int)D_in, (int)F, heads, (int)(F / heads), heads_padded(heads), W, b, a_src, W2, b2);
}

int launch_aggregate(const AggCall& c, hipStream_t stream)
{
    const retexo_plan* p = c.plan;
    const int64_t N = p->N;
    if (N == 0 || c.F == 0) return RETEXO_OK;
    const AggOptions& opt = agg_options();
    const bool gat = c.mode == RETEXO_GAT_SOFTMAX;

    const int vec = gather_vec(c);
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
    a.wsrc = c.mode == RETEXO_GCN_SYM ? p->dinv : nullptr;
    a.Z = c.Z;
    a.ldz = c.ldz;
    a.out = c.out;
    a.ldo = c.ldo;
    a.ocol = c.self_concat ? c.F : 0;
    a.el = nullptr;
    a.el_stride = 0;
    a.er = nullptr;
    a.er_from = nullptr;
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
    a.out_half = (vec == 4 && aligned_for(c.out + a.ocol, c.ldo, 2)) ? 1 : 0;
    a.self_vec = aligned_for(c.out, c.ldo, vec) ? 1 : 0;
    a.part_ptr = nullptr;
    a.n_rows = N;
    a.part_lo = 0;
    a.part_hi = 0;
    a.first = 1;
    a.last = 1;
    a.save_stats = nullptr;
    a.save_pos = nullptr;
    a.save_neg = nullptr;
    a.ld_pos = 0;

    // rows at or above the heavy threshold (rounded up to a tabulated one)
    int64_t n_heavy = 0;
    for (int i = 0; i < 8; ++i)
        if (kPlanThresholds[i] >= opt.heavy_degree) { n_heavy = p->rows_at_least[i]; break; }

    // narrow slabs (32/64/128 columns) use the grouped gather; they need float4 gathers
    // (the maximum is only implemented on whole rows)
    int64_t narrow = (!gat && vec == 4 && c.mode != RETEXO_MAX) ? opt.slab_cols : -1;
    // default for graphs the plan split by source range (dense, table larger than L2): one
    // 128-byte line per row and slab, ranges sized so that a range's slab stays in L2
    // ... and for dense graphs whose table does not fit L2 although one slab of it does
    if (narrow == 0 && (p->part_ptr || (p->nnz >= 32 * N && N * c.ldz * 4 > (4ll << 20)))) narrow = 32;
    if (narrow == 32 || narrow == 64 || narrow == 128) {
        a.nslab = (int)((c.F + narrow - 1) / narrow);
        a.slab_major = opt.slab_major < 0 ? 1 : (int)opt.slab_major;
        int parts = (int)opt.parts;
        if (parts < 0) {
            parts = 1;
            while (parts < kMaxParts && N * narrow * 4 > (int64_t)parts * (8ll << 20)) parts *= 2;
        }
        if (!p->part_ptr || (parts != 2 && parts != 4 && parts != 8 && parts != 16)) parts = 1;
        {
            // long-row class by the length of a row's share of one range
            const int64_t want = opt.narrow_heavy * parts;
            n_heavy = 0;
            for (int i = 0; i < 8; ++i)
                if (kPlanThresholds[i] >= want || kPlanThresholds[i] >= 16384) {
                    n_heavy = p->rows_at_least[i];
                    break;
                }
            if (parts > 1) a.part_ptr = p->part_ptr;
        }
        for (int k = 0; k < parts; ++k) {
            a.part_lo = k * (kMaxParts / parts);
            a.part_hi = (k + 1) * (kMaxParts / parts);
            a.first = k == 0;
            a.last = k == parts - 1;
            const bool wtd = a.wsrc != nullptr;
            const bool off32 = (N * c.ldz + c.F) * 4 < (1ll << 32) && !opt.wide_offsets;
            if (narrow == 32) dispatch_grouped<8>(a, n_heavy, N, wtd, off32, stream);
            else if (narrow == 64) dispatch_grouped<16>(a, n_heavy, N, wtd, off32, stream);
            else dispatch_grouped<32>(a, n_heavy, N, wtd, off32, stream);
        }
    } else if (!gat) {
        const bool maxop = c.mode == RETEXO_MAX;
        if (vec == 4) dispatch_linear<4>(nc, maxop, a, n_heavy, N, stream);
        else if (vec == 2) dispatch_linear<2>(nc, maxop, a, n_heavy, N, stream);
        else dispatch_linear<1>(nc, maxop, a, n_heavy, N, stream);
    } else {
        const int hp = heads_padded(c.heads);
        float* el = (float*)c.workspace;
        float* er = (float*)((char*)c.workspace + gat_workspace(N, c.F, c.heads, false).er);
        const bool hu = (a.Dh % vec) == 0;
        const GatRoute route = gat_route(c);
        const bool off32 = route.off32, flash = route.flash, in_rows = route.in_rows;
        const int g = a.Dh / 4;
        if (c.el_ready && !(in_rows && !c.save && a.nslab == 1)) return RETEXO_E_FLAGS;   // the round asked gat_fold_plan
        a.el_stride = in_rows ? c.ldz : hp;
        if (in_rows) el = const_cast<float*>(c.Z) + c.F;
        a.el = el;
        a.er = er;
        // the plain forward over rows whose scores all come from the gathered rows needs no table
        const bool no_table = flash && !c.save && N > n_heavy && aligned_for(c.attn_dst, 4, 4);
        // only the pipelined kernel keeps the backward's statistics: decided before anything is launched,
        // so that the error leaves the workspace and the output untouched
        if (c.save && !(vec == 4 && off32 && opt.gat_fast)) return RETEXO_E_FLAGS;
        if (c.el_ready) {
            // the transform wrote the source scores; every row forms its own destination scores
            a.er = nullptr;
            a.er_from = c.attn_dst;
        } else if (!no_table) {
            launch_gat_scores(N, c.F, c.heads, c.Z, c.ldz, c.attn_src, c.attn_dst, el, er, stream, a.el_stride);
        }
        if (c.save) {
            const GatWorkspace w = gat_workspace(N, c.F, c.heads, true);
            a.save_stats = (f32x4*)((char*)c.workspace + w.stats);
            a.save_pos = (float*)((char*)c.workspace + w.pos);
            a.save_neg = (float*)((char*)c.workspace + w.neg);
            a.ld_pos = w.ld_pos;
        }
        int64_t n_table = N;          // rows [0, n_table) of the schedule go through the table kernels
        if (flash && N > n_heavy) {
            AggArgs f = a;
            f.nslab = 1;
            f.row_begin = n_heavy;
            f.row_count = N - n_heavy;
            const dim3 grid((unsigned)((f.row_count + kLightWaves - 1) / kLightWaves)), block(64 * kLightWaves);
            auto go = [&](auto gtag) {
                constexpr int GG = decltype(gtag)::value;
                if (c.save) {
                    agg_gat_flash_kernel<GG, true, 1><<<grid, block, 0, stream>>>(f, c.attn_src, nullptr, hp);
                } else if (no_table) {
                    agg_gat_flash_kernel<GG, false, 1><<<grid, block, 0, stream>>>(f, c.attn_src, c.attn_dst, hp);
                    if (n_heavy > 0) {
                        AggArgs fh = f;
                        fh.row_begin = 0;
                        fh.row_count = n_heavy;
                        agg_gat_flash_kernel<GG, false, kHeavyWaves>
                            <<<dim3((unsigned)n_heavy), dim3(64 * kHeavyWaves), 0, stream>>>(fh, c.attn_src, c.attn_dst, hp);
                    }
                } else {
                    agg_gat_flash_kernel<GG, false, 1><<<grid, block, 0, stream>>>(f, c.attn_src, nullptr, hp);
                }
            };
            switch (g) {
                case 1:  go(std::integral_constant<int, 1>{}); break;
                case 2:  go(std::integral_constant<int, 2>{}); break;
                case 4:  go(std::integral_constant<int, 4>{}); break;
                case 8:  go(std::integral_constant<int, 8>{}); break;
                case 16: go(std::integral_constant<int, 16>{}); break;
                case 32: go(std::integral_constant<int, 32>{}); break;
                default: go(std::integral_constant<int, 64>{}); break;
            }
            n_table = no_table ? 0 : n_heavy;
        }
        if (n_table == 0) {
            // nothing left for the table kernels
        } else if (vec == 4 && off32 && opt.gat_fast) {
            if (hp == 4) { if (hu) dispatch_gat_fast<4, true>(nc, c.save, a, n_heavy, n_table, stream); else dispatch_gat_fast<4, false>(nc, c.save, a, n_heavy, n_table, stream); }
            else         { if (hu) dispatch_gat_fast<8, true>(nc, c.save, a, n_heavy, n_table, stream); else dispatch_gat_fast<8, false>(nc, c.save, a, n_heavy, n_table, stream); }
        } else if (vec == 4) {
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
