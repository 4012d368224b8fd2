// Backward of the neighbourhood aggregation: given G = dL/d(out) it produces
// dL/dZ and, for the edge softmax, dL/da_src and dL/da_dst.  It is what a
// worker needs to train, without any message passing, a layer whose AGGR has
// trainable parameters (the gloss under Eq. 1 allows AGGR to have them; GAT's
// attention vectors are such parameters) with the aggregation inside the
// local training loop of the section "Lazy Message Passing".
//
// The graph is undirected, so the CSR is structurally symmetric: the entries
// (v,u) that point at a node u are found by walking u's own row, and the
// transposed product needs no transposed copy of the graph.
//
//  * sum, gcn_sym: the operator is symmetric, the backward is the forward
//    applied to G.  mean: out_v = (1/deg v) sum_u z_u transposes into
//    dZ_u = sum_v G_v / deg v: the rows of G are scaled once into the workspace
//    (one streaming pass) and then summed like any other table.
//  * edge softmax (per head, p_vu = el_u + er_v, e = LeakyReLU(p), alpha = softmax_u e):
//        dZ_u = sum_v alpha_vu G_v  +  a_src * dsrc_u  +  a_dst * ddst_u
//        dsrc_u = sum_v t_vu (<G_v, z_u> - c_v)        t_vu = alpha_vu * LeakyReLU'(p_vu)
//        ddst_v = sum_u t_vu (<G_v, z_u> - c_v)        c_v  = sum_u alpha_vu <G_v, z_u>
//               = (1 - slope) (A+ P- - A- P+)          A+-, P+-: sums of alpha <G_v, z_u> and of alpha
//                 over the entries with positive / non-positive p  (exactly zero when a row has
//                 one neighbour or scores of one sign, where the first form leaves rounding noise)
//        da_src = sum_u dsrc_u z_u,   da_dst = sum_v ddst_v z_v
//    Two gather passes with the structure of the forward kernel (one wave per
//    row, lanes own columns, neighbour ids broadcast from a 64-entry tile):
//      "dst" pass, row v, gathers Z rows: softmax statistics (max, sum), c_v and ddst_v;
//      "src" pass, row u, gathers G rows:  the alpha-weighted sum, dsrc_u, and the output row.
//    The per-edge inner products <G_v, z_u> are never reduced across lanes edge
//    by edge: each lane accumulates weight * (its own columns' share of the
//    product) and the lanes of a head are summed once per row.
//    Nothing is accumulated with atomics; every sum has a fixed order.
#include "common.hpp"
#include "gather.hpp"

namespace {

struct BwdArgs {
    const int64_t* row_ptr;
    const int32_t* col_idx;
    const int32_t* order;
    const float* Z;        // forward input
    int64_t ldz;
    const float* G;        // gradient of the aggregate (first column of that half)
    const float* Gself;    // gradient of the self half, or NULL
    int64_t ldg;
    float* dZ;
    int64_t lddz;
    const float* a_src;    // [F]
    const float* a_dst;
    const float* el;       // [N, HP]
    const float* er;
    f32x4* nbr;            // [N, HP]  {er_v, max_v, 1/sum_v, c_v}
    float* ddst;           // [N, HP]
    float* dsrc;           // [N, HP]
    int64_t row_begin;
    int64_t row_count;
    int64_t F;
    int heads;
    int Dh;
    float slope;
};

// sum over the lanes of a wave of the per-lane values that belong to head h
template <int NC, int Q>
__device__ __forceinline__ float head_total(const float (&q)[NC][Q], const int (&hc)[NC][Q], int h)
{
    float x = 0.0f;
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int k = 0; k < Q; ++k) x += (hc[c][k] == h) ? q[c][k] : 0.0f;
    return wave_sum(x);
}

// ---------------------------------------------------------------------------
// "dst" pass: row v, gathers z_u for u in N(v).  Writes nbr[v,h] and ddst[v,h].
//   HU: every lane's VEC columns lie inside one head (Dh % VEC == 0)
// ---------------------------------------------------------------------------
template <int VEC, int NC, int NW, int HP, bool HU>
__global__ __launch_bounds__(64 * (NW == 1 ? kLightWaves : NW)) void gat_bwd_dst_kernel(BwdArgs a)
{
    constexpr int WAVES = NW == 1 ? kLightWaves : NW;
    constexpr int U = NC * VEC >= 16 ? 2 : kUnroll;   // rows in flight per batch (fewer when a row fills many registers)
    constexpr int Q = HU ? 1 : VEC;
    __shared__ float wl[WAVES][2][HP][64];     // per edge of the tile: exp(e - max) where p > 0 / where p <= 0 (else 0)
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t item = (NW == 1) ? (int64_t)blockIdx.x * kLightWaves + wave : (int64_t)blockIdx.x;
    if (item >= a.row_count) return;          // NW > 1: uniform over the workgroup
    const int v = __builtin_amdgcn_readfirstlane(a.order[a.row_begin + item]);
    const int lo = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v]);
    const int hi = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v + 1]);

    int64_t colsafe[NC];
    int hc[NC][Q];
    float g[NC][VEC], qp[NC][Q], qn[NC][Q];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int64_t col = (int64_t)lane * VEC + c * 64 * VEC;
        const bool act = col < a.F;
        colsafe[c] = act ? col : 0;           // lanes past the row width gather column 0 with a zero multiplier
        load_row<VEC>(a.G + (int64_t)v * a.ldg + colsafe[c], g[c]);
#pragma unroll
        for (int k = 0; k < VEC; ++k) g[c][k] = act ? g[c][k] : 0.0f;
#pragma unroll
        for (int k = 0; k < Q; ++k) {
            hc[c][k] = min((int)((col + k) / a.Dh), a.heads - 1);
            qp[c][k] = 0.0f;
            qn[c][k] = 0.0f;
        }
    }
    float* wp = &wl[wave][0][0][0];
    float* wt = &wl[wave][1][0][0];

    float m[HP], s[HP], sn[HP], erv[HP];     // running max; sums of exp over entries with p > 0 (s) and p <= 0 (sn)
#pragma unroll
    for (int h = 0; h < HP; ++h) {
        m[h] = -INFINITY;
        s[h] = 0.0f;
        sn[h] = 0.0f;
        erv[h] = a.er[(int64_t)v * HP + h];
    }

    const int first = lo + 64 * (NW == 1 ? 0 : wave);
    for (int base = first; base < hi; base += 64 * NW) {
        const int e = base + lane;
        const bool valid = e < hi;
        const int cnt = min(64, hi - base);
        int my_u = valid ? a.col_idx[e] : 0;
        my_u = valid ? my_u : bcast_i(my_u, 0);          // lane 0 is always valid

        float zq[U][NC][VEC];
#pragma unroll
        for (int t = 0; t < U; ++t) {
            const float* zr = a.Z + (int64_t)bcast_i(my_u, t) * a.ldz;
#pragma unroll
            for (int c = 0; c < NC; ++c) load_row<VEC>(zr + colsafe[c], zq[t][c]);
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
            scale[h] = expf(m[h] - mn);                          // exp(-inf) = 0 on the first tile
            const float pe = valid ? expf(sc - mn) : 0.0f;
            const float pp = x > 0.0f ? pe : 0.0f;
            const float pn = x > 0.0f ? 0.0f : pe;
            s[h] = s[h] * scale[h] + wave_sum(pp);               // s: positive part, sn: the rest
            sn[h] = sn[h] * scale[h] + wave_sum(pn);
            m[h] = mn;
            wp[h * 64 + lane] = pp;
            wt[h * 64 + lane] = pn;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if (base != first) {
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int k = 0; k < Q; ++k) {
                    const float f = select_head<HP>(scale, hc[c][k]);
                    qp[c][k] *= f;
                    qn[c][k] *= f;
                }
        }

        for (int j = 0; j < cnt; j += U) {
            float zn[U][NC][VEC];
            const bool more = j + U < cnt;
            if (more) {
#pragma unroll
                for (int t = 0; t < U; ++t) {
                    const float* zr = a.Z + (int64_t)bcast_i(my_u, (j + U + t) & 63) * a.ldz;
#pragma unroll
                    for (int c = 0; c < NC; ++c) load_row<VEC>(zr + colsafe[c], zn[t][c]);
                }
            }
#pragma unroll
            for (int t = 0; t < U; ++t)
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    if constexpr (HU) {
                        float pd = 0.0f;
#pragma unroll
                        for (int k = 0; k < VEC; ++k) pd = fmaf(g[c][k], zq[t][c][k], pd);
                        qp[c][0] = fmaf(wp[hc[c][0] * 64 + j + t], pd, qp[c][0]);
                        qn[c][0] = fmaf(wt[hc[c][0] * 64 + j + t], pd, qn[c][0]);
                    } else {
#pragma unroll
                        for (int k = 0; k < VEC; ++k) {
                            const float pd = g[c][k] * zq[t][c][k];
                            qp[c][k] = fmaf(wp[hc[c][k] * 64 + j + t], pd, qp[c][k]);
                            qn[c][k] = fmaf(wt[hc[c][k] * 64 + j + t], pd, qn[c][k]);
                        }
                    }
                }
            if (more) {
#pragma unroll
                for (int t = 0; t < U; ++t)
#pragma unroll
                    for (int c = 0; c < NC; ++c)
#pragma unroll
                        for (int k = 0; k < VEC; ++k) zq[t][c][k] = zn[t][c][k];
            }
        }
    }

    float QP[HP], QN[HP];
#pragma unroll
    for (int h = 0; h < HP; ++h) {
        QP[h] = head_total<NC, Q>(qp, hc, h);
        QN[h] = head_total<NC, Q>(qn, hc, h);
    }

    if constexpr (NW > 1) {
        // merge the waves' (max, sums) in wave order, rescaled to the common maximum
        __shared__ float red[5][NW][HP];
        if (lane == 0) {
#pragma unroll
            for (int h = 0; h < HP; ++h) {
                red[0][wave][h] = m[h];
                red[1][wave][h] = s[h];
                red[2][wave][h] = sn[h];
                red[3][wave][h] = QP[h];
                red[4][wave][h] = QN[h];
            }
        }
        __syncthreads();
        if (wave != 0) return;
#pragma unroll
        for (int h = 0; h < HP; ++h) {
            float mm = red[0][0][h];
#pragma unroll
            for (int w = 1; w < NW; ++w) mm = fmaxf(mm, red[0][w][h]);
            float ss = 0.0f, tt = 0.0f, aa = 0.0f, bb = 0.0f;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                // a wave that saw no tile has max -inf and contributes nothing
                const float f = (red[0][w][h] == -INFINITY) ? 0.0f : expf(red[0][w][h] - mm);
                ss += red[1][w][h] * f;
                tt += red[2][w][h] * f;
                aa += red[3][w][h] * f;
                bb += red[4][w][h] * f;
            }
            m[h] = mm; s[h] = ss; sn[h] = tt; QP[h] = aa; QN[h] = bb;
        }
    }

    if (lane == 0) {
#pragma unroll
        for (int h = 0; h < HP; ++h) {
            const float sum = s[h] + sn[h];
            const bool any = sum > 0.0f;
            const float rs = any ? 1.0f / sum : 0.0f;
            const float ap = QP[h] * rs, an = QN[h] * rs;        // A+, A-
            const f32x4 t = {erv[h], any ? m[h] : 0.0f, rs, ap + an};
            a.nbr[(int64_t)v * HP + h] = t;
            a.ddst[(int64_t)v * HP + h] = (1.0f - a.slope) * (ap * (sn[h] * rs) - an * (s[h] * rs));
        }
    }
}

// ---------------------------------------------------------------------------
// "dst" pass for rows of ordinary length when the row fits one wave at four floats per lane
// (F <= 256) and a head is a power-of-two group of G lanes: the source score of an entry is
// computed from the gathered row z_u itself (dot product with a_src over the head's lanes)
// instead of being read from the score table, which costs a cache line per entry.  Same
// quantities as gat_bwd_dst_kernel, kept per lane (equal over the lanes of a head) and updated
// online over batches of four entries: running maximum m, sums of exp over entries with a
// positive score (s) and the others (sn), and the lane's share of sum exp * <g_v, z_u>, again
// split by the sign of the score (qp, qn).
// ---------------------------------------------------------------------------
template <int G>
__global__ __launch_bounds__(64 * kLightWaves) void gat_bwd_dst_flash_kernel(BwdArgs a, int hp)
{
    constexpr int U = 4;
    constexpr float kLog2e = 1.4426950408889634f;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t item = (int64_t)blockIdx.x * kLightWaves + wave;
    if (item >= a.row_count) return;
    const int v = __builtin_amdgcn_readfirstlane(a.order[a.row_begin + item]);
    const int lo = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v]);
    const int hi = __builtin_amdgcn_readfirstlane((int)a.row_ptr[v + 1]);

    const int64_t col = (int64_t)lane * 4;
    const bool act = col < a.F;
    const int64_t colsafe = act ? col : 0;    // lanes past the row width gather column 0 with zero multipliers
    const int h = min((int)(col / a.Dh), a.heads - 1);
    float g[4] = {0.0f, 0.0f, 0.0f, 0.0f}, as[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    float erv = 0.0f;
    if (act) {
        load_row<4>(a.G + (int64_t)v * a.ldg + col, g);
        load_row<4>(a.a_src + col, as);
        erv = a.er[(int64_t)v * hp + h];
    }

    float m = -INFINITY, s = 0.0f, sn = 0.0f, qp = 0.0f, qn = 0.0f;
    for (int base = lo; base < hi; base += 64) {
        const int e = base + lane;
        const bool valid = e < hi;
        const int cnt = min(64, hi - base);
        int my_u = valid ? a.col_idx[e] : 0;
        my_u = valid ? my_u : bcast_i(my_u, 0);          // lane 0 is always valid

        float zq[U][4];
#pragma unroll
        for (int t = 0; t < U; ++t) load_row<4>(a.Z + (int64_t)bcast_i(my_u, t) * a.ldz + colsafe, zq[t]);

        for (int j = 0; j < cnt; j += U) {
            float zn[U][4];
            const bool more = j + U < cnt;
            if (more) {
#pragma unroll
                for (int t = 0; t < U; ++t)
                    load_row<4>(a.Z + (int64_t)bcast_i(my_u, (j + U + t) & 63) * a.ldz + colsafe, zn[t]);
            }
            float x[U], sc[U], pd[U];
#pragma unroll
            for (int t = 0; t < U; ++t) {
                float d = as[0] * zq[t][0];
                d = fmaf(as[1], zq[t][1], d);
                d = fmaf(as[2], zq[t][2], d);
                d = fmaf(as[3], zq[t][3], d);
                x[t] = group_sum<G>(d) + erv;
                sc[t] = (j + t < cnt) ? (x[t] > 0.0f ? x[t] : a.slope * x[t]) : -INFINITY;
                float q = g[0] * zq[t][0];
                q = fmaf(g[1], zq[t][1], q);
                q = fmaf(g[2], zq[t][2], q);
                q = fmaf(g[3], zq[t][3], q);
                pd[t] = q;
            }
            float mn = m;
#pragma unroll
            for (int t = 0; t < U; ++t) mn = fmaxf(mn, sc[t]);      // finite: entry j of the tile is real
            const float scale = __builtin_amdgcn_exp2f((m - mn) * kLog2e);   // 0 on the first batch
            float sp_b = 0.0f, sn_b = 0.0f, qp_b = 0.0f, qn_b = 0.0f;
#pragma unroll
            for (int t = 0; t < U; ++t) {
                const float pe = __builtin_amdgcn_exp2f((sc[t] - mn) * kLog2e);   // 0 past the tile
                const float pp = x[t] > 0.0f ? pe : 0.0f;
                const float pn = x[t] > 0.0f ? 0.0f : pe;
                sp_b += pp;
                sn_b += pn;
                qp_b = fmaf(pp, pd[t], qp_b);
                qn_b = fmaf(pn, pd[t], qn_b);
            }
            s = s * scale + sp_b;
            sn = sn * scale + sn_b;
            qp = qp * scale + qp_b;
            qn = qn * scale + qn_b;
            m = mn;
            if (more) {
#pragma unroll
                for (int t = 0; t < U; ++t)
#pragma unroll
                    for (int k = 0; k < 4; ++k) zq[t][k] = zn[t][k];
            }
        }
    }

    const float QP = group_sum<G>(qp), QN = group_sum<G>(qn);
    if (act && (lane % G) == 0 && col < (int64_t)a.heads * a.Dh) {
        const float sum = s + sn;
        const bool any = sum > 0.0f;
        const float rs = any ? 1.0f / sum : 0.0f;
        const float ap = QP * rs, an = QN * rs;              // A+, A-
        const f32x4 t = {erv, any ? m : 0.0f, rs, ap + an};
        a.nbr[(int64_t)v * hp + h] = t;
        a.ddst[(int64_t)v * hp + h] = (1.0f - a.slope) * (ap * (sn * rs) - an * (s * rs));
    }
    if (lane == 0) {
        // padded heads carry no columns: neutral entries
        for (int k = a.heads; k < hp; ++k) {
            a.nbr[(int64_t)v * hp + k] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            a.ddst[(int64_t)v * hp + k] = 0.0f;
        }
    }
}

// ---------------------------------------------------------------------------
// "src" pass: row u, gathers G_v for v in N(u) (the entries (v,u) by symmetry).
// Writes dZ[u,:] and dsrc[u,h].
// ---------------------------------------------------------------------------
template <int VEC, int NC, int NW, int HP, bool HU>
__global__ __launch_bounds__(64 * (NW == 1 ? kLightWaves : NW)) void gat_bwd_src_kernel(BwdArgs a)
{
    constexpr int WAVES = NW == 1 ? kLightWaves : NW;
    constexpr int U = NC * VEC >= 16 ? 2 : kUnroll;   // rows in flight per batch (fewer when a row fills many registers)
    constexpr int Q = HU ? 1 : VEC;
    __shared__ float wl[WAVES][2][HP][64];     // per edge of the tile: alpha_vu and alpha_vu * LeakyReLU'
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t item = (NW == 1) ? (int64_t)blockIdx.x * kLightWaves + wave : (int64_t)blockIdx.x;
    if (item >= a.row_count) return;
    const int u = __builtin_amdgcn_readfirstlane(a.order[a.row_begin + item]);
    const int lo = __builtin_amdgcn_readfirstlane((int)a.row_ptr[u]);
    const int hi = __builtin_amdgcn_readfirstlane((int)a.row_ptr[u + 1]);

    bool act[NC];
    int64_t colsafe[NC];
    int hc[NC][Q];
    float zo[NC][VEC], acc[NC][VEC], q[NC][Q];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int64_t col = (int64_t)lane * VEC + c * 64 * VEC;
        act[c] = col < a.F;
        colsafe[c] = act[c] ? col : 0;
        load_row<VEC>(a.Z + (int64_t)u * a.ldz + colsafe[c], zo[c]);
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            zo[c][k] = act[c] ? zo[c][k] : 0.0f;
            acc[c][k] = 0.0f;
        }
#pragma unroll
        for (int k = 0; k < Q; ++k) {
            hc[c][k] = min((int)((col + k) / a.Dh), a.heads - 1);
            q[c][k] = 0.0f;
        }
    }
    float* wp = &wl[wave][0][0][0];
    float* wt = &wl[wave][1][0][0];

    float elu[HP], tc[HP];
#pragma unroll
    for (int h = 0; h < HP; ++h) {
        elu[h] = a.el[(int64_t)u * HP + h];
        tc[h] = 0.0f;
    }

    for (int base = lo + 64 * (NW == 1 ? 0 : wave); base < hi; base += 64 * NW) {
        const int e = base + lane;
        const bool valid = e < hi;
        const int cnt = min(64, hi - base);
        int my_v = valid ? a.col_idx[e] : 0;
        my_v = valid ? my_v : bcast_i(my_v, 0);

        float gq[U][NC][VEC];
#pragma unroll
        for (int t = 0; t < U; ++t) {
            const float* gr = a.G + (int64_t)bcast_i(my_v, t) * a.ldg;
#pragma unroll
            for (int c = 0; c < NC; ++c) load_row<VEC>(gr + colsafe[c], gq[t][c]);
        }

        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
#pragma unroll
        for (int h = 0; h < HP; ++h) {
            const f32x4 nb = a.nbr[(int64_t)my_v * HP + h];
            const float x = elu[h] + nb.x;
            const float sc = x > 0.0f ? x : a.slope * x;
            const float al = valid ? expf(sc - nb.y) * nb.z : 0.0f;   // sc <= nb.y: row v's maximum covers this entry
            const float t = x > 0.0f ? al : a.slope * al;
            tc[h] = fmaf(t, nb.w, tc[h]);
            wp[h * 64 + lane] = al;
            wt[h * 64 + lane] = t;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        for (int j = 0; j < cnt; j += U) {
            float gn[U][NC][VEC];
            const bool more = j + U < cnt;
            if (more) {
#pragma unroll
                for (int t = 0; t < U; ++t) {
                    const float* gr = a.G + (int64_t)bcast_i(my_v, (j + U + t) & 63) * a.ldg;
#pragma unroll
                    for (int c = 0; c < NC; ++c) load_row<VEC>(gr + colsafe[c], gn[t][c]);
                }
            }
#pragma unroll
            for (int t = 0; t < U; ++t)
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    if constexpr (HU) {
                        const float wa = wp[hc[c][0] * 64 + j + t];
                        float pd = 0.0f;
#pragma unroll
                        for (int k = 0; k < VEC; ++k) {
                            acc[c][k] = fmaf(wa, gq[t][c][k], acc[c][k]);
                            pd = fmaf(gq[t][c][k], zo[c][k], pd);
                        }
                        q[c][0] = fmaf(wt[hc[c][0] * 64 + j + t], pd, q[c][0]);
                    } else {
#pragma unroll
                        for (int k = 0; k < VEC; ++k) {
                            acc[c][k] = fmaf(wp[hc[c][k] * 64 + j + t], gq[t][c][k], acc[c][k]);
                            q[c][k] = fmaf(wt[hc[c][k] * 64 + j + t], gq[t][c][k] * zo[c][k], q[c][k]);
                        }
                    }
                }
            if (more) {
#pragma unroll
                for (int t = 0; t < U; ++t)
#pragma unroll
                    for (int c = 0; c < NC; ++c)
#pragma unroll
                        for (int k = 0; k < VEC; ++k) gq[t][c][k] = gn[t][c][k];
            }
        }
    }

    float ds[HP];
#pragma unroll
    for (int h = 0; h < HP; ++h) ds[h] = head_total<NC, Q>(q, hc, h) - wave_sum(tc[h]);

    if constexpr (NW > 1) {
        __shared__ float red[NW][NC * VEC][64];
        __shared__ float dred[NW][HP];
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int k = 0; k < VEC; ++k) red[wave][c * VEC + k][lane] = acc[c][k];
        if (lane == 0) {
#pragma unroll
            for (int h = 0; h < HP; ++h) dred[wave][h] = ds[h];
        }
        __syncthreads();
        if (wave != 0) return;
#pragma unroll
        for (int h = 0; h < HP; ++h) {
            float t = dred[0][h];
#pragma unroll
            for (int w = 1; w < NW; ++w) t += dred[w][h];
            ds[h] = t;
        }
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                float t = red[0][c * VEC + k][lane];
#pragma unroll
                for (int w = 1; w < NW; ++w) t += red[w][c * VEC + k][lane];
                acc[c][k] = t;
            }
    }

    float dd[HP];
#pragma unroll
    for (int h = 0; h < HP; ++h) dd[h] = a.ddst[(int64_t)u * HP + h];
    if (lane == 0) {
#pragma unroll
        for (int h = 0; h < HP; ++h) a.dsrc[(int64_t)u * HP + h] = ds[h];
    }
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        if (!act[c]) continue;
        const int64_t col = colsafe[c];
        float as[VEC], ad[VEC], gs[VEC], r[VEC];
        load_row<VEC>(a.a_src + col, as);
        load_row<VEC>(a.a_dst + col, ad);
        if (a.Gself) load_row<VEC>(a.Gself + (int64_t)u * a.ldg + col, gs);
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            const int h = hc[c][HU ? 0 : k];
            r[k] = acc[c][k] + as[k] * select_head<HP>(ds, h) + ad[k] * select_head<HP>(dd, h);
            if (a.Gself) r[k] += gs[k];
        }
        store_row<VEC>(a.dZ + (int64_t)u * a.lddz + col, r, VEC, true);
    }
}

// ---------------------------------------------------------------------------
// What the "dst" pass produces, from what a forward pass in save mode left behind instead of a
// second gather over Z:  A+- = <G_v, out+-_v> (out+, out-: the parts of the aggregate from entries
// with a positive / non-positive score),  c_v = A+ + A-,  P+-: the saved shares of the softmax sum.
// One wave per node.
// ---------------------------------------------------------------------------
template <int HP>
__global__ __launch_bounds__(256) void gat_bwd_from_saved_kernel(
    int64_t N, int64_t F, int heads, int Dh, float slope, const float* __restrict__ G, int64_t ldg,
    const float* __restrict__ pos, const float* __restrict__ neg, int64_t ldp,
    const f32x4* __restrict__ stats, const float* __restrict__ er, f32x4* __restrict__ nbr,
    float* __restrict__ ddst)
{
    const int lane = threadIdx.x & 63;
    const int64_t v = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= N) return;
    float pp[HP], pn[HP];
#pragma unroll
    for (int h = 0; h < HP; ++h) { pp[h] = 0.0f; pn[h] = 0.0f; }
    for (int64_t c = lane; c < F; c += 64) {
        const float g = G[v * ldg + c];
        const int h = (int)(c / Dh);
        const float x = g * pos[v * ldp + c], y = g * neg[v * ldp + c];
#pragma unroll
        for (int i = 0; i < HP; ++i) {
            pp[i] += (h == i) ? x : 0.0f;
            pn[i] += (h == i) ? y : 0.0f;
        }
    }
#pragma unroll
    for (int h = 0; h < HP; ++h) {
        const float ap = wave_sum(pp[h]), an = wave_sum(pn[h]);
        if (lane == 0) {
            const f32x4 st = stats[v * HP + h];           // {max, 1/sum, P+, P-}
            const f32x4 t = {er[v * HP + h], st.x, st.y, ap + an};
            nbr[v * HP + h] = t;
            ddst[v * HP + h] = h < heads ? (1.0f - slope) * (ap * st.w - an * st.z) : 0.0f;
        }
    }
}

// The same with 16-byte loads: 16 lanes per node (four nodes per wave), the three rows of a node read in float4
// steps of 64 columns, a row of up to 256 columns requested before any of it is used, per-head partial sums
// reduced over the 16 lanes.  Needs 16-byte aligned rows of G and F % 4 == 0 (the kept rows are aligned).
template <int HP>
__global__ __launch_bounds__(256) void gat_bwd_from_saved_vec_kernel(
    int64_t N, int64_t F, int heads, int Dh, float slope, const float* __restrict__ G, int64_t ldg,
    const float* __restrict__ pos, const float* __restrict__ neg, int64_t ldp,
    const f32x4* __restrict__ stats, const float* __restrict__ er, f32x4* __restrict__ nbr,
    float* __restrict__ ddst)
{
    const int li = threadIdx.x & 15;
    const int64_t v = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const bool have = v < N;
    const int64_t vv = have ? v : N - 1;                 // idle groups repeat the last node (nothing stored)
    const bool whole = Dh % 4 == 0;
    float pp[HP], pn[HP];
#pragma unroll
    for (int h = 0; h < HP; ++h) { pp[h] = 0.0f; pn[h] = 0.0f; }
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int64_t c0 = li * 4; c0 < F; c0 += 256) {
        f32x4 gq[4], pq[4], nq[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int64_t c = c0 + 64 * q;
            const bool in = c < F;
            gq[q] = in ? *reinterpret_cast<const f32x4*>(G + vv * ldg + c) : zero;
            pq[q] = in ? *reinterpret_cast<const f32x4*>(pos + vv * ldp + c) : zero;
            nq[q] = in ? *reinterpret_cast<const f32x4*>(neg + vv * ldp + c) : zero;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int64_t c = c0 + 64 * q;
            if (c >= F) break;
            const float g[4] = {gq[q].x, gq[q].y, gq[q].z, gq[q].w};
            const float p[4] = {pq[q].x, pq[q].y, pq[q].z, pq[q].w};
            const float n[4] = {nq[q].x, nq[q].y, nq[q].z, nq[q].w};
            if (whole) {
                const int h = (int)c / Dh;
                const float x = ((g[0] * p[0] + g[1] * p[1]) + g[2] * p[2]) + g[3] * p[3];
                const float y = ((g[0] * n[0] + g[1] * n[1]) + g[2] * n[2]) + g[3] * n[3];
#pragma unroll
                for (int i = 0; i < HP; ++i) {
                    pp[i] += (h == i) ? x : 0.0f;
                    pn[i] += (h == i) ? y : 0.0f;
                }
                continue;
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int h = ((int)c + k) / Dh;
                const float x = g[k] * p[k], y = g[k] * n[k];
#pragma unroll
                for (int i = 0; i < HP; ++i) {
                    pp[i] += (h == i) ? x : 0.0f;
                    pn[i] += (h == i) ? y : 0.0f;
                }
            }
        }
    }
#pragma unroll
    for (int h = 0; h < HP; ++h) {
#pragma unroll
        for (int m = 8; m >= 1; m >>= 1) {
            pp[h] += __shfl_xor(pp[h], m, 64);
            pn[h] += __shfl_xor(pn[h], m, 64);
        }
    }
    if (have && li == 0) {
#pragma unroll
        for (int h = 0; h < HP; ++h) {
            const f32x4 st = stats[v * HP + h];           // {max, 1/sum, P+, P-}
            const f32x4 t = {er[v * HP + h], st.x, st.y, pp[h] + pn[h]};
            nbr[v * HP + h] = t;
            ddst[v * HP + h] = h < heads ? (1.0f - slope) * (pp[h] * st.w - pn[h] * st.z) : 0.0f;
        }
    }
}

// ---------------------------------------------------------------------------
// da_src[c] = sum_u dsrc[u, head(c)] Z[u, c],  da_dst[c] = sum_v ddst[v, head(c)] Z[v, c]
// stage 1: each workgroup sums a contiguous range of rows, one thread per column
// stage 2: the partial rows are added in index order
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gat_bwd_param_partial_kernel(
    int64_t N, int64_t F, int Dh, int heads, int HP, const float* __restrict__ Z, int64_t ldz,
    const float* __restrict__ dsrc, const float* __restrict__ ddst, int64_t rows_per_block,
    float* __restrict__ partial)
{
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r1 = min(N, r0 + rows_per_block);
    for (int64_t col = threadIdx.x; col < F; col += 256) {
        const int h = min((int)(col / Dh), heads - 1);
        float ss = 0.0f, sd = 0.0f;
        for (int64_t r = r0; r < r1; ++r) {
            const float z = Z[r * ldz + col];
            ss = fmaf(dsrc[r * HP + h], z, ss);
            sd = fmaf(ddst[r * HP + h], z, sd);
        }
        partial[((int64_t)blockIdx.x * 2 + 0) * F + col] = ss;
        partial[((int64_t)blockIdx.x * 2 + 1) * F + col] = sd;
    }
}

// A workgroup of 16 waves owns 64 columns: every wave adds a sixteenth of the blocks' partial sums with four
// running sums (four loads in flight), and the 64 sums of a column are combined in a fixed order.
__global__ __launch_bounds__(1024) void gat_bwd_param_final_kernel(
    int64_t nblk, int64_t F, const float* __restrict__ partial, float* __restrict__ da_src,
    float* __restrict__ da_dst)
{
    __shared__ float sh[2][16][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t col = (int64_t)blockIdx.x * 64 + lane;
    float ss = 0.0f, sd = 0.0f;
    if (col < F) {
        const int64_t per = (nblk + 15) / 16;
        const int64_t b0 = wave * per, b1 = min(nblk, b0 + per);
        float qs[4] = {0.0f, 0.0f, 0.0f, 0.0f}, qd[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        int64_t b = b0;
        for (; b + 4 <= b1; b += 4) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                qs[k] += partial[((b + k) * 2 + 0) * F + col];
                qd[k] += partial[((b + k) * 2 + 1) * F + col];
            }
        }
        for (int k = 0; b < b1; ++b, ++k) {
            qs[k] += partial[(b * 2 + 0) * F + col];
            qd[k] += partial[(b * 2 + 1) * F + col];
        }
        ss = (qs[0] + qs[1]) + (qs[2] + qs[3]);
        sd = (qd[0] + qd[1]) + (qd[2] + qd[3]);
    }
    sh[0][wave][lane] = ss;
    sh[1][wave][lane] = sd;
    __syncthreads();
    if (wave == 0 && col < F) {
        float ts = 0.0f, td = 0.0f;
#pragma unroll
        for (int w = 0; w < 16; ++w) { ts += sh[0][w][lane]; td += sh[1][w][lane]; }
        da_src[col] = ts;
        da_dst[col] = td;
    }
}

// S[v, :] = G[v, :] / deg v (zero for an empty row): the mean's backward sums these rows.
// One thread per four columns; S has a row pitch that is a multiple of four floats.
__global__ __launch_bounds__(256) void scale_rows_by_degree_kernel(
    int64_t N, int64_t F, const float* __restrict__ G, int64_t ldg, const int32_t* __restrict__ deg,
    float* __restrict__ S, int64_t lds)
{
    const int64_t quads = (F + 3) / 4;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= N * quads) return;
    const int64_t v = i / quads, c0 = (i % quads) * 4;
    const int d = deg[v];
    const float r = d > 0 ? 1.0f / (float)d : 0.0f;
#pragma unroll
    for (int k = 0; k < 4; ++k)
        if (c0 + k < F) S[v * lds + c0 + k] = G[v * ldg + c0 + k] * r;
}

// dZ[:, 0:F] += Gself[:, 0:F]
__global__ __launch_bounds__(256) void add_rows_kernel(int64_t N, int64_t F, const float* __restrict__ Gs,
                                                        int64_t ldg, float* __restrict__ dZ, int64_t lddz)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= N * F) return;
    const int64_t r = i / F, c = i % F;
    dZ[r * lddz + c] += Gs[r * ldg + c];
}

bool aligned4(const void* p, int64_t ld) { return ((uintptr_t)p % 16) == 0 && ld % 4 == 0; }

template <int G>
void launch_dst_flash(const BwdArgs& a, int hp, unsigned blocks, hipStream_t stream)
{
    gat_bwd_dst_flash_kernel<G><<<dim3(blocks), dim3(64 * kLightWaves), 0, stream>>>(a, hp);
}

// first_pass 0: the "dst" pass then the "src" pass; 1: the "src" pass alone (statistics already in place).
// flash_g > 0: ordinary rows of the "dst" pass compute the source scores from the gathered rows, flash_g
// lanes per head.
template <int VEC, int NC, int HP, bool HU>
void launch_passes(const BwdArgs& base, int first_pass, int64_t n_heavy, int64_t N, hipStream_t stream, int flash_g = 0)
{
    for (int pass = first_pass; pass < 2; ++pass) {
        if (n_heavy > 0) {
            BwdArgs a = base;
            a.row_begin = 0;
            a.row_count = n_heavy;
            if (pass == 0)
                gat_bwd_dst_kernel<VEC, NC, kHeavyWaves, HP, HU><<<dim3((unsigned)n_heavy), dim3(64 * kHeavyWaves), 0, stream>>>(a);
            else
                gat_bwd_src_kernel<VEC, NC, kHeavyWaves, HP, HU><<<dim3((unsigned)n_heavy), dim3(64 * kHeavyWaves), 0, stream>>>(a);
        }
        if (N > n_heavy) {
            BwdArgs a = base;
            a.row_begin = n_heavy;
            a.row_count = N - n_heavy;
            const unsigned blocks = (unsigned)((a.row_count + kLightWaves - 1) / kLightWaves);
            if (pass == 0 && flash_g > 0) {
                switch (flash_g) {
                    case 1:  launch_dst_flash<1>(a, HP, blocks, stream); break;
                    case 2:  launch_dst_flash<2>(a, HP, blocks, stream); break;
                    case 4:  launch_dst_flash<4>(a, HP, blocks, stream); break;
                    case 8:  launch_dst_flash<8>(a, HP, blocks, stream); break;
                    case 16: launch_dst_flash<16>(a, HP, blocks, stream); break;
                    case 32: launch_dst_flash<32>(a, HP, blocks, stream); break;
                    default: launch_dst_flash<64>(a, HP, blocks, stream); break;
                }
            } else if (pass == 0)
                gat_bwd_dst_kernel<VEC, NC, 1, HP, HU><<<dim3(blocks), dim3(64 * kLightWaves), 0, stream>>>(a);
            else
                gat_bwd_src_kernel<VEC, NC, 1, HP, HU><<<dim3(blocks), dim3(64 * kLightWaves), 0, stream>>>(a);
        }
    }
}

template <int VEC, int HP, bool HU>
void dispatch_nc(int nc, const BwdArgs& a, int fp, int64_t nh, int64_t N, hipStream_t s, int flash_g = 0)
{
    if (nc == 1) launch_passes<VEC, 1, HP, HU>(a, fp, nh, N, s, flash_g);
    else if (nc == 2) launch_passes<VEC, 2, HP, HU>(a, fp, nh, N, s);
    else launch_passes<VEC, 4, HP, HU>(a, fp, nh, N, s);
}

template <int HP>
void dispatch_wide(int nc, const BwdArgs& a, int fp, int64_t nh, int64_t N, hipStream_t s)
{
    // unaligned tables: scalar gathers, up to 16 chunks of 64 columns
    if (nc <= 4) launch_passes<1, 4, HP, true>(a, fp, nh, N, s);
    else if (nc <= 8) launch_passes<1, 8, HP, true>(a, fp, nh, N, s);
    else launch_passes<1, 16, HP, true>(a, fp, nh, N, s);
}

constexpr int64_t kParamBlocks = 2048;

int64_t param_blocks(int64_t N) { return N <= 0 ? 1 : (N + 255) / 256 < kParamBlocks ? (N + 255) / 256 : kParamBlocks; }

struct SoftmaxWorkspace {
    int64_t el, er, nbr, ddst, dsrc, partial, total;
};

SoftmaxWorkspace softmax_workspace(int64_t N, int64_t F, int heads)
{
    const int64_t n = N > 0 ? N : 1, hp = heads_padded(heads);
    SoftmaxWorkspace w;
    int64_t off = 0;
    const int64_t per = align_up(n * hp * (int64_t)sizeof(float), 256);
    w.el = off; off += per;
    w.er = off; off += per;
    w.ddst = off; off += per;
    w.dsrc = off; off += per;
    w.nbr = off; off += align_up(n * hp * 16, 256);
    w.partial = off; off += align_up(param_blocks(N) * 2 * (F > 0 ? F : 1) * (int64_t)sizeof(float), 256);
    w.total = off;
    return w;
}

// row pitch (floats) of the scaled copy of G the mean's backward keeps in the workspace: 128-byte rows
int64_t scaled_pitch(int64_t F) { return align_up(F > 0 ? F : 1, 32); }

}  // namespace

int64_t aggregate_backward_workspace_bytes(int64_t N, int mode, int64_t F, int heads)
{
    if (mode == RETEXO_GAT_SOFTMAX) return softmax_workspace(N, F, heads).total;
    if (mode == RETEXO_MEAN) return align_up((N > 0 ? N : 1) * scaled_pitch(F) * (int64_t)sizeof(float), 256);
    return 0;
}

int launch_aggregate_backward(const AggBackwardCall& c, hipStream_t stream)
{
    const retexo_plan* p = c.plan;
    const int64_t N = p->N, F = c.F;
    if (N == 0 || F == 0) return RETEXO_OK;
    const float* Ga = c.G + (c.self_concat ? F : 0);

    if (c.mode != RETEXO_GAT_SOFTMAX) {
        // the transposed operator is a forward aggregation of G over the (symmetric) graph
        AggCall f;
        f.plan = p;
        f.mode = c.mode == RETEXO_MEAN ? RETEXO_SUM : c.mode;
        f.F = F;
        f.heads = 1;
        f.Z = Ga;
        f.ldz = c.ldg;
        f.attn_src = nullptr;
        f.attn_dst = nullptr;
        f.slope = 0.0f;
        f.self_concat = false;
        f.copy_self = false;
        f.out = c.dZ;
        f.ldo = c.lddz;
        f.workspace = nullptr;
        if (c.mode == RETEXO_MEAN) {
            float* S = (float*)c.workspace;
            const int64_t lds = scaled_pitch(F), threads = N * ((F + 3) / 4);
            scale_rows_by_degree_kernel<<<dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream>>>(
                N, F, Ga, c.ldg, p->deg, S, lds);
            f.Z = S;
            f.ldz = lds;
        }
        if (int s = launch_aggregate(f, stream)) return s;
        if (c.self_concat)
            add_rows_kernel<<<dim3((unsigned)((N * F + 255) / 256)), dim3(256), 0, stream>>>(N, F, c.G, c.ldg, c.dZ, c.lddz);
        if (hipGetLastError() != hipSuccess) return RETEXO_E_HIP;
        return RETEXO_OK;
    }

    const int hp = heads_padded(c.heads);
    const SoftmaxWorkspace w = softmax_workspace(N, F, c.heads);
    char* ws = (char*)c.workspace;
    BwdArgs a;
    a.row_ptr = p->row_ptr;
    a.col_idx = p->col_idx;
    a.order = p->order;
    a.Z = c.Z;
    a.ldz = c.ldz;
    a.G = Ga;
    a.Gself = c.self_concat ? c.G : nullptr;
    a.ldg = c.ldg;
    a.dZ = c.dZ;
    a.lddz = c.lddz;
    a.a_src = c.attn_src;
    a.a_dst = c.attn_dst;
    a.el = (float*)(ws + w.el);
    a.er = (float*)(ws + w.er);
    a.nbr = (f32x4*)(ws + w.nbr);
    a.ddst = (float*)(ws + w.ddst);
    a.dsrc = (float*)(ws + w.dsrc);
    a.row_begin = 0;
    a.row_count = 0;
    a.F = F;
    a.heads = c.heads;
    a.Dh = (int)(F / c.heads);
    a.slope = c.slope;

    int first_pass = 0;
    if (c.saved) {
        // the forward pass left scores, softmax statistics and the positive-score part of the aggregate
        const GatWorkspace fw = gat_workspace(N, F, c.heads, true);
        const char* sv = (const char*)c.saved;
        a.el = (const float*)(sv + fw.el);
        a.er = (const float*)(sv + fw.er);
        const unsigned gb = (unsigned)((N + 3) / 4);
        const bool vec_rows = F % 4 == 0 && F < (1ll << 30) && c.ldg % 4 == 0 && (uintptr_t)Ga % 16 == 0 &&
                              fw.ld_pos % 4 == 0 && (uintptr_t)sv % 16 == 0 && agg_options().max_vec >= 4;
        if (vec_rows && hp == 4)
            gat_bwd_from_saved_vec_kernel<4><<<dim3((unsigned)((N + 15) / 16)), dim3(256), 0, stream>>>(
                N, F, c.heads, a.Dh, c.slope, Ga, c.ldg, (const float*)(sv + fw.pos), (const float*)(sv + fw.neg),
                fw.ld_pos, (const f32x4*)(sv + fw.stats), a.er, a.nbr, a.ddst);
        else if (vec_rows)
            gat_bwd_from_saved_vec_kernel<8><<<dim3((unsigned)((N + 15) / 16)), dim3(256), 0, stream>>>(
                N, F, c.heads, a.Dh, c.slope, Ga, c.ldg, (const float*)(sv + fw.pos), (const float*)(sv + fw.neg),
                fw.ld_pos, (const f32x4*)(sv + fw.stats), a.er, a.nbr, a.ddst);
        else if (hp == 4)
            gat_bwd_from_saved_kernel<4><<<dim3(gb), dim3(256), 0, stream>>>(
                N, F, c.heads, a.Dh, c.slope, Ga, c.ldg, (const float*)(sv + fw.pos), (const float*)(sv + fw.neg),
                fw.ld_pos, (const f32x4*)(sv + fw.stats), a.er, a.nbr, a.ddst);
        else
            gat_bwd_from_saved_kernel<8><<<dim3(gb), dim3(256), 0, stream>>>(
                N, F, c.heads, a.Dh, c.slope, Ga, c.ldg, (const float*)(sv + fw.pos), (const float*)(sv + fw.neg),
                fw.ld_pos, (const f32x4*)(sv + fw.stats), a.er, a.nbr, a.ddst);
        first_pass = 1;
    } else {
        launch_gat_scores(N, F, c.heads, c.Z, c.ldz, c.attn_src, c.attn_dst, (float*)(ws + w.el), (float*)(ws + w.er), stream);
    }

    int64_t n_heavy = 0;
    const AggOptions& opt = agg_options();
    for (int i = 0; i < 8; ++i)
        if (kPlanThresholds[i] >= opt.heavy_degree) { n_heavy = p->rows_at_least[i]; break; }

    // 16-byte gathers need every table aligned, rows padded to whole vectors and F a multiple of 4
    // (the inner products must not see padding columns)
    const bool v4 = F % 4 == 0 && aligned4(c.Z, c.ldz) && aligned4(Ga, c.ldg) && aligned4(c.dZ, c.lddz) &&
                    aligned4(c.attn_src, 4) && aligned4(c.attn_dst, 4) && (!c.self_concat || aligned4(c.G, c.ldg)) &&
                    opt.max_vec >= 4;
    if (v4) {
        const int nc = (int)((F + 255) / 256);
        const bool hu = a.Dh % 4 == 0;
        // ordinary rows of the "dst" pass: source scores from the gathered rows when a head is a power-of-two
        // group of four-float lanes (see the kernel)
        const int g = a.Dh / 4;
        const int flash_g = (opt.gat_flash && nc == 1 && hu && g <= 64 && (g & (g - 1)) == 0) ? g : 0;
        if (hp == 4) { if (hu) dispatch_nc<4, 4, true>(nc, a, first_pass, n_heavy, N, stream, flash_g); else dispatch_nc<4, 4, false>(nc, a, first_pass, n_heavy, N, stream); }
        else         { if (hu) dispatch_nc<4, 8, true>(nc, a, first_pass, n_heavy, N, stream, flash_g); else dispatch_nc<4, 8, false>(nc, a, first_pass, n_heavy, N, stream); }
    } else {
        const int nc = (int)((F + 63) / 64);
        if (hp == 4) dispatch_wide<4>(nc, a, first_pass, n_heavy, N, stream);
        else dispatch_wide<8>(nc, a, first_pass, n_heavy, N, stream);
    }

    const int64_t nblk = param_blocks(N);
    const int64_t rows_per_block = (N + nblk - 1) / nblk;
    float* partial = (float*)(ws + w.partial);
    gat_bwd_param_partial_kernel<<<dim3((unsigned)nblk), dim3(256), 0, stream>>>(
        N, F, a.Dh, c.heads, hp, c.Z, c.ldz, a.dsrc, a.ddst, rows_per_block, partial);
    gat_bwd_param_final_kernel<<<dim3((unsigned)((F + 63) / 64)), dim3(1024), 0, stream>>>(
        nblk, F, partial, c.d_attn_src, c.d_attn_dst);
    if (hipGetLastError() != hipSuccess) return RETEXO_E_HIP;
    return RETEXO_OK;
}
