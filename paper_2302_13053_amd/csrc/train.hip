// Local training of one layer: the work a worker does between two message
// passing rounds (section "Lazy Message Passing").  A layer f (fully connected
// + ReLU, Eq. 1) is trained by itself on its fixed aggregated inputs X with a
// temporary linear classification layer C on top (the appendix sizes C as
// H_m x H_K) and softmax cross-entropy over the labelled nodes; the last layer
// is the classification function itself (H == 0 here).
//
//      A      = ReLU(X W1 + b1)          transform kernel (fp32 MFMA)
//      logits = A Wc + bc                transform kernel
//      dL     = (softmax(logits) - onehot(label)) / n_labelled, 0 for unlabelled nodes
//      gWc    = A^T dL,  gbc = colsum(dL)
//      dA     = (dL Wc^T) where A > 0    transform kernel with Wc^T and a ReLU mask
//      gW1    = X^T dA,  gb1 = colsum(dA)
//
// The two weight gradients are "TN" products whose contraction runs over the
// nodes (hundreds of thousands), with a small output.  wgrad_kernel splits the
// node range over many workgroups, each producing a partial [M, Nq] tile with
// the same fp32 MFMA tile loop as the transform (both operands are already
// k-major in memory, so their tiles are plain 16-byte copies into LDS), and a
// second kernel adds the partials in a fixed order: deterministic, and more
// accurate than one long fp32 accumulation.
#include "common.hpp"
#include "tiles.hpp"

namespace {

constexpr int BK = kTileK;
constexpr int kThreads = 256;

// ---------------------------------------------------------------------------
// part[z][m][n] = sum over k in chunk z of P[k][m] * Q[k][n]
// ---------------------------------------------------------------------------

// Partial tile of one wave -> part[z]: accumulator element r of lane l is row 8*(r/4) + 4*(l/32) + r%4,
// column l%32 of its 32 x 32 tile.
template <int TM, int TN>
__device__ __forceinline__ void write_partial(const f32x16 (&acc)[TM][TN], int M, int Nq, int row_base, int col_base,
                                              int lane, float* __restrict__ out)
{
    const int lrow = lane & 31, lk = lane >> 5;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = col_base + j * 32 + lrow;
        if (col >= Nq) continue;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row0 = row_base + i * 32 + 4 * lk;
            float* p = out + (int64_t)row0 * Nq + col;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ro = 8 * (r / 4) + (r % 4);
                if (row0 + ro < M) p[(int64_t)ro * Nq] = acc[i][j][r];
            }
        }
    }
}

// Aligned operands (rows of P and Q are 16-byte multiples at 16-byte aligned addresses, M >= 4, Nq >= 4):
// the software-pipelined K loop shared with the dense transform.  Columns past M / Nq are clamped to the
// last four (their products land in partials that are never stored); only a partial last K tile of a
// chunk takes a checked, zero-filling fetch.
template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(256, 2) void wgrad_pipe_kernel(
    int64_t K, int M, int Nq, const float* __restrict__ P, int64_t ldp,
    const float* __restrict__ Q, int64_t ldq, int64_t k_chunk, float* __restrict__ part)
{
    static_assert(WGM * WGN == 4, "four waves per workgroup");
    constexpr int TM = BM / (32 * WGM);
    constexpr int TN = BN / (32 * WGN);
    constexpr int LDA = BM + 4;
    constexpr int LDB = BN + 4;
    constexpr int A_F4 = BM * BK / 4 / 256;
    constexpr int B_F4 = (BN * BK / 4 + 255) / 256;
    constexpr bool B_PART = BN * BK / 4 % 256 != 0;
    static_assert(A_F4 >= 1 && BM * BK / 4 % 256 == 0, "tile shape");

    __shared__ float As[2][BK][LDA];
    __shared__ float Bs[2][BK][LDB];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int m0 = blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;
    const int64_t k_begin = (int64_t)blockIdx.z * k_chunk;
    const int64_t k_end = min(K, k_begin + k_chunk);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int nk = k_end > k_begin ? (int)((k_end - k_begin + BK - 1) / BK) : 0;
    if (nk > 0) {
        const int k_tail = (int)((k_end - k_begin) % BK);      // > 0: the chunk's last tile is partial
        const float* pa[A_F4];
        const float* pb[B_F4];
        int ka[A_F4], kb[B_F4];                                // row of the thread's piece inside a tile
#pragma unroll
        for (int i = 0; i < A_F4; ++i) {
            const int id = tid + i * 256;
            const int kk = id / (BM / 4), m4 = id % (BM / 4);
            int m = m0 + m4 * 4;
            m = m < M - 4 ? m : M - 4;
            pa[i] = P + (k_begin + kk) * ldp + m;
            ka[i] = kk;
        }
#pragma unroll
        for (int i = 0; i < B_F4; ++i) {
            const int id = tid + i * 256;
            const int kk = (id / (BN / 4)) % BK, n4 = id % (BN / 4);
            int n = n0 + n4 * 4;
            n = n < Nq - 4 ? n : Nq - 4;
            pb[i] = Q + (k_begin + kk) * ldq + n;
            kb[i] = kk;
        }
        const int64_t step_a = (int64_t)BK * ldp, step_b = (int64_t)BK * ldq;
        f32x4 ra[A_F4], rb[B_F4];

        auto fetch_a = [&](int kt) {
            if (k_tail && kt == nk - 1) {
#pragma unroll
                for (int i = 0; i < A_F4; ++i) {
                    const bool in = ka[i] < k_tail;
                    const f32x4 t = *reinterpret_cast<const f32x4*>(in ? pa[i] : P);
                    ra[i] = in ? t : f32x4{0.f, 0.f, 0.f, 0.f};
                }
            } else {
#pragma unroll
                for (int i = 0; i < A_F4; ++i) ra[i] = *reinterpret_cast<const f32x4*>(pa[i]);
            }
#pragma unroll
            for (int i = 0; i < A_F4; ++i) pa[i] += step_a;
        };
        auto fetch_b = [&](int kt) {
            if (k_tail && kt == nk - 1) {
#pragma unroll
                for (int i = 0; i < B_F4; ++i) {
                    const bool in = kb[i] < k_tail;
                    const f32x4 t = *reinterpret_cast<const f32x4*>(in ? pb[i] : Q);
                    rb[i] = in ? t : f32x4{0.f, 0.f, 0.f, 0.f};
                }
            } else {
#pragma unroll
                for (int i = 0; i < B_F4; ++i) rb[i] = *reinterpret_cast<const f32x4*>(pb[i]);
            }
#pragma unroll
            for (int i = 0; i < B_F4; ++i) pb[i] += step_b;
        };
        auto put_a = [&](int buf, int i) {
            const int id = tid + i * 256;
            const int kk = id / (BM / 4), m4 = id % (BM / 4);
            *reinterpret_cast<f32x4*>(&As[buf][kk][m4 * 4]) = ra[i];
        };
        auto put_b = [&](int buf, int i) {
            const int id = tid + i * 256;
            if (B_PART && id >= BN * BK / 4) return;
            const int kk = id / (BN / 4), n4 = id % (BN / 4);
            *reinterpret_cast<f32x4*>(&Bs[buf][kk][n4 * 4]) = rb[i];
        };

        fetch_a(0);
        fetch_b(0);
#pragma unroll
        for (int i = 0; i < A_F4; ++i) put_a(0, i);
#pragma unroll
        for (int i = 0; i < B_F4; ++i) put_b(0, i);
        if (nk > 1) { fetch_a(1); fetch_b(1); }
        __syncthreads();

        auto put = [&](int buf, int third) {
            if (third == 0) {
#pragma unroll
                for (int x = 0; x < A_F4; ++x) put_a(buf, x);
            } else if (third == 1) {
                put_b(buf, 0);
            } else {
#pragma unroll
                for (int x = 1; x < B_F4; ++x) put_b(buf, x);
            }
        };
        auto fetch = [&](int kt, int half) {
            if (half == 0) fetch_a(kt);
            else fetch_b(kt);
        };
        mfma_k_loop<TM, TN, LDA, LDB>(acc, As, Bs, nk, wm * TM * 32, wn * TN * 32, lane, put, fetch);
    }
    write_partial<TM, TN>(acc, M, Nq, m0 + wm * TM * 32, n0 + wn * TN * 32, lane, part + (int64_t)blockIdx.z * M * Nq);
}

// Any shape: every element fetched under its own check.
template <int BM, int BN, int WGM, int WGN, bool PV, bool QV>
__global__ __launch_bounds__(256, 2) void wgrad_kernel(
    int64_t K, int M, int Nq, const float* __restrict__ P, int64_t ldp,
    const float* __restrict__ Q, int64_t ldq, int64_t k_chunk, float* __restrict__ part)
{
    static_assert(WGM * WGN == 4, "four waves per workgroup");
    constexpr int TM = BM / (32 * WGM);
    constexpr int TN = BN / (32 * WGN);
    constexpr int LDA = BM + 4;
    constexpr int LDB = BN + 4;
    constexpr int A_F4 = (BM * BK / 4 + 255) / 256;
    constexpr int B_F4 = (BN * BK / 4 + 255) / 256;

    __shared__ float As[2][BK][LDA];
    __shared__ float Bs[2][BK][LDB];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int m0 = blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;
    const int64_t k_begin = (int64_t)blockIdx.z * k_chunk;
    const int64_t k_end = min(K, k_begin + k_chunk);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    float ra[A_F4][4], rb[B_F4][4];
    int wa[A_F4], wb[B_F4];

    auto load_tiles = [&](int kt) {
#pragma unroll
        for (int i = 0; i < A_F4; ++i) {
            const int id = tid + i * 256;
            if (BM * BK / 4 % 256 != 0 && id >= BM * BK / 4) continue;
            const int kk = id / (BM / 4), m4 = id % (BM / 4);
            const int64_t k = k_begin + (int64_t)kt * BK + kk;
            const int m = m0 + m4 * 4;
            wa[i] = k < k_end ? M - m : 0;
            load4<PV>(P, k * ldp + m, wa[i], ra[i]);
        }
#pragma unroll
        for (int i = 0; i < B_F4; ++i) {
            const int id = tid + i * 256;
            if (BN * BK / 4 % 256 != 0 && id >= BN * BK / 4) continue;
            const int kk = id / (BN / 4), n4 = id % (BN / 4);
            const int64_t k = k_begin + (int64_t)kt * BK + kk;
            const int n = n0 + n4 * 4;
            wb[i] = k < k_end ? Nq - n : 0;
            load4<QV>(Q, k * ldq + n, wb[i], rb[i]);
        }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_F4; ++i) {
            const int id = tid + i * 256;
            if (BM * BK / 4 % 256 != 0 && id >= BM * BK / 4) continue;
            const int kk = id / (BM / 4), m4 = id % (BM / 4);
            zero4<PV>(wa[i], ra[i]);
            f32x4 t = {ra[i][0], ra[i][1], ra[i][2], ra[i][3]};
            *reinterpret_cast<f32x4*>(&As[buf][kk][m4 * 4]) = t;
        }
#pragma unroll
        for (int i = 0; i < B_F4; ++i) {
            const int id = tid + i * 256;
            if (BN * BK / 4 % 256 != 0 && id >= BN * BK / 4) continue;
            const int kk = id / (BN / 4), n4 = id % (BN / 4);
            zero4<QV>(wb[i], rb[i]);
            f32x4 t = {rb[i][0], rb[i][1], rb[i][2], rb[i][3]};
            *reinterpret_cast<f32x4*>(&Bs[buf][kk][n4 * 4]) = t;
        }
    };

    const int lrow = lane & 31, lk = lane >> 5;
    const int nk = (int)((k_end - k_begin + BK - 1) / BK);
    if (nk > 0) {
        load_tiles(0);
        store_tiles(0);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_tiles(kt + 1);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            float af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = As[buf][kk + lk][wm * TM * 32 + i * 32 + lrow];
#pragma unroll
            for (int j = 0; j < TN; ++j) bf[j] = Bs[buf][kk + lk][wn * TN * 32 + j * 32 + lrow];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_tiles(buf ^ 1);
        __syncthreads();
    }

    write_partial<TM, TN>(acc, M, Nq, m0 + wm * TM * 32, n0 + wn * TN * 32, lane, part + (int64_t)blockIdx.z * M * Nq);
}

// out[m][n] = sum_z part[z][m][n] for n < n_keep (partials are Nq wide).  A workgroup owns 64 outputs; its four
// waves each add a quarter of the z range with four running sums (z mod 4), and the sixteen sums of an output
// are combined in a fixed order: the result does not depend on the launch, and with few outputs and hundreds of
// partials (a classifier's gradient) the additions no longer wait for one load at a time.
__global__ __launch_bounds__(kThreads) void reduce_partials(
    int S, int M, int Nq, int n_keep, const float* __restrict__ part, float* __restrict__ out)
{
    __shared__ float sh[kThreads / 64][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * 64 + lane;
    const bool live = i < (int64_t)M * n_keep;
    float s = 0.0f;
    if (live) {
        const int m = (int)(i / n_keep), n = (int)(i % n_keep);
        const int per = (S + 3) / 4;
        const int z0 = wave * per, z1 = min(S, z0 + per);
        const float* p = part + (int64_t)m * Nq + n;
        const int64_t pitch = (int64_t)M * Nq;
        float q[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        int z = z0;
        for (; z + 4 <= z1; z += 4) {
#pragma unroll
            for (int k = 0; k < 4; ++k) q[k] += p[(int64_t)(z + k) * pitch];
        }
        for (int k = 0; z < z1; ++z, ++k) q[k] += p[(int64_t)z * pitch];
        s = (q[0] + q[1]) + (q[2] + q[3]);
    }
    sh[wave][lane] = s;
    __syncthreads();
    if (wave == 0 && live) out[i] = (sh[0][lane] + sh[1][lane]) + (sh[2][lane] + sh[3][lane]);
}

struct TrainHeader {
    int32_t n_labelled;
    int32_t pad[3];
};

__global__ __launch_bounds__(kThreads) void count_labelled(int64_t N, const int32_t* __restrict__ labels,
                                                           TrainHeader* hdr)
{
    __shared__ int sh[kThreads / 64];
    int cnt = 0;
    for (int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x; v < N; v += (int64_t)gridDim.x * kThreads)
        cnt += labels[v] >= 0;
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) cnt += __shfl_xor(cnt, m, 64);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
        for (int w = 0; w < kThreads / 64; ++w) t += sh[w];
        if (t) atomicAdd(&hdr->n_labelled, t);       // integer: the total does not depend on the order
    }
}

__device__ __forceinline__ float wmax(float x)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) x = fmaxf(x, __shfl_xor(x, m, 64));
    return x;
}
__device__ __forceinline__ float wsum(float x)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) x += __shfl_xor(x, m, 64);
    return x;
}

constexpr int kXentRows = 64;     // nodes per workgroup of the loss kernel (16 per wave)

// One wave per node at a time.  L[v, 0:C] holds the logits on entry and d loss / d logits on
// exit (zero for unlabelled nodes and in the padding columns C..ld).  Per-workgroup loss sums
// go to loss_part[blockIdx.x] (unscaled).
__global__ __launch_bounds__(kThreads) void softmax_xent_kernel(
    int64_t N, int C, float* __restrict__ L, int64_t ld, const int32_t* __restrict__ labels,
    const TrainHeader* hdr, float* __restrict__ loss_part)
{
    __shared__ float wl[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nl = hdr->n_labelled;
    float loss = 0.0f;
    for (int r = wave; r < kXentRows; r += 4) {
        const int64_t v = (int64_t)blockIdx.x * kXentRows + r;
        if (v >= N) break;
        float* row = L + v * ld;
        const int y = labels[v];
        const float scale = (y >= 0 && nl > 0) ? 1.0f / (float)nl : 0.0f;
        float m = -INFINITY;
        for (int j = lane; j < C; j += 64) m = fmaxf(m, row[j]);
        m = wmax(m);
        // s: the softmax denominator; so: its part from the classes other than the label.  The label's
        // gradient p_y - 1 is formed as -so / s: for a confidently classified node p_y is close to one and
        // the subtraction would leave only a few correct digits of what is then the whole gradient.
        float s = 0.0f, so = 0.0f;
        for (int j = lane; j < C; j += 64) {
            const float e = expf(row[j] - m);
            s += e;
            so += j == y ? 0.0f : e;
        }
        s = wsum(s);
        so = wsum(so);
        const float rest = so / s;                 // 1 - p_y
        if (y >= 0 && y < C) loss += rest <= 0.5f ? -log1pf(-rest) : -(row[y] - m - logf(s));
        for (int j = lane; j < ld; j += 64) {
            float g = 0.0f;
            if (j < C) g = (j == y ? -rest : expf(row[j] - m) / s) * scale;
            row[j] = g;
        }
    }
    if (lane == 0) wl[wave] = loss;
    __syncthreads();
    if (threadIdx.x == 0) loss_part[blockIdx.x] = (wl[0] + wl[1]) + (wl[2] + wl[3]);
}

// loss = (sum of the partial sums, pairwise in a fixed order) / n_labelled
__global__ __launch_bounds__(kThreads) void loss_reduce_kernel(int64_t n_part, const float* __restrict__ part,
                                                               const TrainHeader* hdr, float* __restrict__ loss)
{
    __shared__ float sh[kThreads];
    float s = 0.0f;
    for (int64_t i = threadIdx.x; i < n_part; i += kThreads) s += part[i];
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int w = kThreads / 2; w >= 1; w >>= 1) {
        if ((int)threadIdx.x < w) sh[threadIdx.x] += sh[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = hdr->n_labelled > 0 ? sh[0] / (float)hdr->n_labelled : 0.0f;
}

// Column sums in two deterministic stages.  Stage 1: a workgroup takes kColRows rows; its four
// waves stride the rows, lanes stride the columns, every wave keeps four running sums (four loads in
// flight) that are combined in a fixed order, and the waves are added in order through LDS.
// Stage 2: one workgroup per column adds the stage-1 results with a fixed tree.
constexpr int kColRows = 128;

__global__ __launch_bounds__(kThreads) void colsum_stage1(int64_t N, int C, const float* __restrict__ D, int64_t ld,
                                                          float* __restrict__ part)
{
    __shared__ float sh[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t r0 = (int64_t)blockIdx.x * kColRows, r1 = min(N, r0 + kColRows);
    for (int c0 = 0; c0 < C; c0 += 64) {
        const int c = c0 + lane;
        float s = 0.0f;
        if (c < C) {
            float q[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            int64_t r = r0 + wave;
            for (; r + 12 < r1; r += 16) {
#pragma unroll
                for (int k = 0; k < 4; ++k) q[k] += D[(r + 4 * k) * ld + c];
            }
            for (int k = 0; r < r1; r += 4, ++k) q[k] += D[r * ld + c];
            s = (q[0] + q[1]) + (q[2] + q[3]);
        }
        sh[wave][lane] = s;
        __syncthreads();
        if (wave == 0 && c < C)
            part[(int64_t)blockIdx.x * C + c] = (sh[0][lane] + sh[1][lane]) + (sh[2][lane] + sh[3][lane]);
        __syncthreads();
    }
}
__global__ __launch_bounds__(kThreads) void colsum_stage2(int B, int C, const float* __restrict__ part,
                                                          float* __restrict__ out)
{
    __shared__ float sh[kThreads];
    const int c = blockIdx.x;
    float s = 0.0f;
    for (int b = threadIdx.x; b < B; b += kThreads) s += part[(int64_t)b * C + c];
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int w = kThreads / 2; w >= 1; w >>= 1) {
        if ((int)threadIdx.x < w) sh[threadIdx.x] += sh[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[c] = sh[0];
}

// out [Cp, R] = scale * transpose of in [R, Cn], rows Cn..Cp of out zero
__global__ __launch_bounds__(kThreads) void transpose_kernel(int R, int Cn, int Cp, const float* __restrict__ in,
                                                             float* __restrict__ out, float scale)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= (int64_t)R * Cp) return;
    const int c = (int)(i / R), r = (int)(i % R);
    out[i] = c < Cn ? scale * in[(int64_t)r * Cn + c] : 0.0f;
}

// ---------------------------------------------------------------------------
// Dropout on the hidden units (the appendix on hyper-parameters trains with dropout; it is taken on the
// layer's output, in front of the temporary classifier).  The mask is not stored: unit j of node v is
// dropped in draw number `draw` of stream `seed` when word j % 4 of the Philox-4x32-10 block
//      counter = (v, j / 4, draw low, draw high),  key = (seed low, seed high)
// (Salmon, Moraes, Dror, Shaw, SC 2011) is below floor(p * 2^32), so any caller can re-draw it.
// Kept units are scaled by 1 / (1 - p).  The backward pass needs no second draw: a unit of the stored
// activations is positive exactly when it was active and kept.
// ---------------------------------------------------------------------------
struct PhiloxWords { uint32_t w0, w1, w2, w3; };

__device__ __forceinline__ PhiloxWords philox_4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                      uint32_t k0, uint32_t k1)
{
    constexpr uint32_t kMulA = 0xD2511F53u, kMulB = 0xCD9E8D57u;      // multipliers of words 0 and 2
    constexpr uint32_t kKeyA = 0x9E3779B9u, kKeyB = 0xBB67AE85u;      // key increments per round
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hiA = __umulhi(kMulA, c0), loA = kMulA * c0;
        const uint32_t hiB = __umulhi(kMulB, c2), loB = kMulB * c2;
        c0 = hiB ^ c1 ^ k0;
        c2 = hiA ^ c3 ^ k1;
        c1 = loB;
        c3 = loA;
        k0 += kKeyA;
        k1 += kKeyB;
    }
    return {c0, c1, c2, c3};
}

__global__ __launch_bounds__(kThreads) void dropout_kernel(int64_t N, int H, float* __restrict__ A, int64_t ld,
                                                           uint32_t threshold, float scale, uint32_t seed_lo,
                                                           uint32_t seed_hi, uint32_t draw_lo, uint32_t draw_hi)
{
    const int Q = (H + 3) / 4;
    const int64_t total = N * Q;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (int64_t)gridDim.x * kThreads) {
        const int64_t v = i / Q;
        const int q = (int)(i % Q);
        const PhiloxWords w = philox_4x32_10((uint32_t)v, (uint32_t)q, draw_lo, draw_hi, seed_lo, seed_hi);
        float* p = A + v * ld + 4 * q;
        if (4 * q + 3 < H) {
            // rows of the workspace start on 128-byte lines
            f32x4 x = *reinterpret_cast<const f32x4*>(p);
            x.x = w.w0 >= threshold ? x.x * scale : 0.0f;
            x.y = w.w1 >= threshold ? x.y * scale : 0.0f;
            x.z = w.w2 >= threshold ? x.z * scale : 0.0f;
            x.w = w.w3 >= threshold ? x.w * scale : 0.0f;
            *reinterpret_cast<f32x4*>(p) = x;
        } else {
            const uint32_t ws[4] = {w.w0, w.w1, w.w2, w.w3};
            for (int k = 0; k < 4 && 4 * q + k < H; ++k) p[k] = ws[k] >= threshold ? p[k] * scale : 0.0f;
        }
    }
}

__global__ __launch_bounds__(kThreads) void sgd_kernel(int64_t n, float* __restrict__ p, const float* __restrict__ g,
                                                       float lr)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) p[i] = p[i] - lr * g[i];
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct Split { int S; int64_t k_chunk; };

Split choose_split(int64_t K, int64_t M, int64_t Nq, int bn)
{
    const int64_t tiles = ((M + 127) / 128) * ((Nq + bn - 1) / bn);
    // the widest tile runs two workgroups per CU: at most 1024 workgroups are exactly two rounds of the 512
    // slots (one more workgroup would add a third round for it alone)
    int64_t S = 1024 / tiles;
    const int64_t max_s = (K + 255) / 256;                  // at least 256 nodes per chunk
    if (S > max_s) S = max_s;
    if (S < 1) S = 1;
    int64_t chunk = (K + S - 1) / S;
    chunk = (chunk + BK - 1) / BK * BK;
    S = (K + chunk - 1) / chunk;
    if (S < 1) S = 1;
    return {(int)S, chunk};
}

int bn_for(int64_t Nq) { return Nq <= 32 ? 32 : Nq <= 64 ? 64 : Nq <= 128 ? 128 : 256; }

template <int BN, int WGM, int WGN>
void launch_wgrad_bn(int64_t K, int64_t M, int64_t Nq, const float* P, int64_t ldp, const float* Q, int64_t ldq,
                     Split sp, float* part, hipStream_t stream)
{
    const bool pv = (uintptr_t)P % 16 == 0 && ldp % 4 == 0 && M % 4 == 0;
    const bool qv = (uintptr_t)Q % 16 == 0 && ldq % 4 == 0 && Nq % 4 == 0;
    dim3 grid((unsigned)((M + 127) / 128), (unsigned)((Nq + BN - 1) / BN), (unsigned)sp.S);
    if (pv && qv && M >= 4 && Nq >= 4)
        wgrad_pipe_kernel<128, BN, WGM, WGN><<<grid, dim3(256), 0, stream>>>(K, (int)M, (int)Nq, P, ldp, Q, ldq, sp.k_chunk, part);
    else if (pv && qv)
        wgrad_kernel<128, BN, WGM, WGN, true, true><<<grid, dim3(256), 0, stream>>>(K, (int)M, (int)Nq, P, ldp, Q, ldq, sp.k_chunk, part);
    else if (pv)
        wgrad_kernel<128, BN, WGM, WGN, true, false><<<grid, dim3(256), 0, stream>>>(K, (int)M, (int)Nq, P, ldp, Q, ldq, sp.k_chunk, part);
    else if (qv)
        wgrad_kernel<128, BN, WGM, WGN, false, true><<<grid, dim3(256), 0, stream>>>(K, (int)M, (int)Nq, P, ldp, Q, ldq, sp.k_chunk, part);
    else
        wgrad_kernel<128, BN, WGM, WGN, false, false><<<grid, dim3(256), 0, stream>>>(K, (int)M, (int)Nq, P, ldp, Q, ldq, sp.k_chunk, part);
}

// out[M][n_keep] = P^T Q, Q being Nq (>= n_keep) columns wide
void wgrad(int64_t K, int64_t M, int64_t Nq, int64_t n_keep, const float* P, int64_t ldp, const float* Q,
           int64_t ldq, float* part, float* out, hipStream_t stream)
{
    const int bn = bn_for(Nq);
    const Split sp = choose_split(K, M, Nq, bn);
    if (bn == 32) launch_wgrad_bn<32, 4, 1>(K, M, Nq, P, ldp, Q, ldq, sp, part, stream);
    else if (bn == 64) launch_wgrad_bn<64, 4, 1>(K, M, Nq, P, ldp, Q, ldq, sp, part, stream);
    else if (bn == 128) launch_wgrad_bn<128, 2, 2>(K, M, Nq, P, ldp, Q, ldq, sp, part, stream);
    else launch_wgrad_bn<256, 2, 2>(K, M, Nq, P, ldp, Q, ldq, sp, part, stream);
    const int64_t total = M * n_keep;
    reduce_partials<<<dim3((unsigned)((total + 63) / 64)), dim3(kThreads), 0, stream>>>(
        sp.S, (int)M, (int)Nq, (int)n_keep, part, out);
}

void colsum(int64_t N, int64_t C, const float* D, int64_t ld, float* part, float* out, hipStream_t stream)
{
    const int B = (int)((N + kColRows - 1) / kColRows);
    colsum_stage1<<<dim3((unsigned)B), dim3(kThreads), 0, stream>>>(N, (int)C, D, ld, part);
    colsum_stage2<<<dim3((unsigned)C), dim3(kThreads), 0, stream>>>(B, (int)C, part, out);
}

struct TrainLayout {
    int64_t ldh, ldc;
    int64_t hdr, A, L, dA, WcT, W1T, part, colpart, losspart, total;
};

int64_t partial_floats(int64_t K, int64_t M, int64_t Nq)
{
    const Split sp = choose_split(K, M, Nq, bn_for(Nq));
    return (int64_t)sp.S * M * Nq;
}

TrainLayout make_layout(int64_t N, int64_t D_in, int64_t H, int64_t C)
{
    TrainLayout t;
    const int64_t n1 = N > 0 ? N : 1;
    t.ldh = align_up(H > 0 ? H : 1, 32);
    t.ldc = align_up(C > 0 ? C : 1, 32);
    int64_t off = 0;
    auto take = [&](int64_t floats) { const int64_t at = off; off += align_up(floats * 4, 256); return at; };
    t.hdr = off; off += 256;
    t.A = take(H > 0 ? n1 * t.ldh : 0);
    t.L = take(n1 * t.ldc);
    t.dA = take(H > 0 ? n1 * t.ldh : 0);
    t.WcT = take(H > 0 ? t.ldc * H : 0);
    t.W1T = take((H > 0 ? H : t.ldc) * D_in);            // transposed first-layer weights (input gradient)
    int64_t pf = 0;
    if (H > 0) {
        pf = partial_floats(N, D_in, t.ldh);
        const int64_t p2 = partial_floats(N, H, t.ldc);
        if (p2 > pf) pf = p2;
    } else {
        pf = partial_floats(N, D_in, t.ldc);
    }
    t.part = take(pf);
    const int64_t widest = t.ldh > t.ldc ? t.ldh : t.ldc;
    t.colpart = take(((n1 + kColRows - 1) / kColRows) * widest);
    t.losspart = take((n1 + kXentRows - 1) / kXentRows);
    t.total = off;
    return t;
}

int check_sizes(int64_t N, int64_t D_in, int64_t H, int64_t C)
{
    if (N < 0 || D_in < 1 || H < 0 || C < 1) return RETEXO_E_SIZE;
    if (N >= (1ll << 31) || D_in >= (1 << 20) || H >= (1 << 20) || C >= (1 << 20)) return RETEXO_E_SIZE;
    return RETEXO_OK;
}

}  // namespace

extern "C" int64_t retexo_train_workspace_bytes(int64_t N, int64_t D_in, int64_t H, int64_t C)
{
    if (int s = check_sizes(N, D_in, H, C)) return s;
    return make_layout(N, D_in, H, C).total;
}

namespace {
int layer_grad_impl(int64_t N, int64_t D_in, int64_t H, int64_t C,
                    const float* d_X, int64_t ldx, const int32_t* d_labels,
                    const float* d_W1, const float* d_b1, const float* d_Wc, const float* d_bc,
                    float* d_gW1, float* d_gb1, float* d_gWc, float* d_gbc, float* d_loss,
                    float* d_gX, int64_t ldgx, float p_drop, uint64_t seed, uint64_t draw,
                    void* d_workspace, int64_t workspace_bytes, void* stream_)
{
    if (int s = check_sizes(N, D_in, H, C)) return s;
    if (!(p_drop >= 0.0f && p_drop < 1.0f)) return RETEXO_E_SIZE;
    if (p_drop > 0.0f && H == 0) return RETEXO_E_SIZE;        // there is no hidden unit to drop
    const float keep_scale = p_drop > 0.0f ? 1.0f / (1.0f - p_drop) : 1.0f;
    if (ldx < D_in) return RETEXO_E_LD;
    if (d_gX && ldgx < D_in) return RETEXO_E_LD;
    if (d_gX && N > 0 && d_X &&
        !((const char*)d_gX + (size_t)((N - 1) * ldgx + D_in) * 4 <= (const char*)d_X ||
          (const char*)d_X + (size_t)((N - 1) * ldx + D_in) * 4 <= (const char*)d_gX))
        return RETEXO_E_ALIAS;
    if (!d_W1 || !d_b1 || !d_gW1 || !d_gb1 || !d_loss) return RETEXO_E_NULL;
    if (N > 0 && (!d_X || !d_labels)) return RETEXO_E_NULL;
    if (H > 0 && (!d_Wc || !d_bc || !d_gWc || !d_gbc)) return RETEXO_E_NULL;
    const TrainLayout t = make_layout(N, D_in, H, C);
    if (!d_workspace || workspace_bytes < t.total || ((uintptr_t)d_workspace & 255)) return RETEXO_E_WORKSPACE;

    hipStream_t stream = (hipStream_t)stream_;
    char* ws = (char*)d_workspace;
    TrainHeader* hdr = (TrainHeader*)(ws + t.hdr);
    float* A = (float*)(ws + t.A);
    float* L = (float*)(ws + t.L);
    float* dA = (float*)(ws + t.dA);
    float* WcT = (float*)(ws + t.WcT);
    float* W1T = (float*)(ws + t.W1T);
    float* part = (float*)(ws + t.part);
    float* colpart = (float*)(ws + t.colpart);
    float* losspart = (float*)(ws + t.losspart);
    const int64_t W1cols = H > 0 ? H : C;

    if (N == 0) {
        // nothing to learn from: zero loss and gradients
        if (launch_zero(d_gW1, (size_t)(D_in * W1cols) * 4, stream)) return RETEXO_E_HIP;
        if (launch_zero(d_gb1, (size_t)W1cols * 4, stream)) return RETEXO_E_HIP;
        if (H > 0) {
            if (launch_zero(d_gWc, (size_t)(H * C) * 4, stream)) return RETEXO_E_HIP;
            if (launch_zero(d_gbc, (size_t)C * 4, stream)) return RETEXO_E_HIP;
        }
        if (launch_zero(d_loss, 4, stream)) return RETEXO_E_HIP;
        return RETEXO_OK;
    }

    if (launch_zero(hdr, sizeof(TrainHeader), stream)) return RETEXO_E_HIP;
    count_labelled<<<dim3((unsigned)min((int64_t)1024, (N + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream>>>(N, d_labels, hdr);

    // forward
    const float* feat = d_X;        // input of the classifier product
    int64_t ldfeat = ldx, dfeat = D_in;
    if (H > 0) {
        if (int e = launch_transform(N, D_in, H, d_X, ldx, d_W1, d_b1, true, A, t.ldh, stream)) return e;
        if (p_drop > 0.0f) {
            const uint32_t threshold = (uint32_t)((double)p_drop * 4294967296.0);
            const int64_t quads = N * ((H + 3) / 4);
            const int64_t blocks = (quads + kThreads - 1) / kThreads;
            dropout_kernel<<<dim3((unsigned)(blocks < (1 << 20) ? blocks : (1 << 20))), dim3(kThreads), 0, stream>>>(
                N, (int)H, A, t.ldh, threshold, keep_scale, (uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)draw,
                (uint32_t)(draw >> 32));
        }
        feat = A; ldfeat = t.ldh; dfeat = H;
    }
    if (int e = launch_transform(N, dfeat, C, feat, ldfeat, H > 0 ? d_Wc : d_W1, H > 0 ? d_bc : d_b1, false,
                                 L, t.ldc, stream))
        return e;

    // loss and d loss / d logits (in place, padding columns zeroed)
    const unsigned nb = (unsigned)((N + kXentRows - 1) / kXentRows);
    softmax_xent_kernel<<<dim3(nb), dim3(kThreads), 0, stream>>>(N, (int)C, L, t.ldc, d_labels, hdr, losspart);
    loss_reduce_kernel<<<dim3(1), dim3(kThreads), 0, stream>>>((int64_t)nb, losspart, hdr, d_loss);

    // classifier (or only) layer: weight and bias gradients
    float* gW_top = H > 0 ? d_gWc : d_gW1;
    float* gb_top = H > 0 ? d_gbc : d_gb1;
    wgrad(N, dfeat, t.ldc, C, feat, ldfeat, L, t.ldc, part, gW_top, stream);
    colsum(N, C, L, t.ldc, colpart, gb_top, stream);

    if (H > 0) {
        // back through the classifier, the dropout (its scale rides on the transposed classifier, its mask is
        // part of "A > 0") and the ReLU, then the layer's own gradients
        // (the contraction runs over the padded width of dL: its padding columns and the padding rows
        // of the transposed classifier are zero, and a multiple of four keeps the loads 16 bytes wide)
        const int64_t tot = H * t.ldc;
        transpose_kernel<<<dim3((unsigned)((tot + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream>>>(
            (int)H, (int)C, (int)t.ldc, d_Wc, WcT, keep_scale);
        if (int e = launch_transform(N, t.ldc, H, L, t.ldc, WcT, nullptr, false, dA, t.ldh, stream, A, t.ldh)) return e;
        // (padding columns of dA only produce partial columns that reduce_partials never reads)
        wgrad(N, D_in, t.ldh, H, d_X, ldx, dA, t.ldh, part, d_gW1, stream);
        colsum(N, H, dA, t.ldh, colpart, d_gb1, stream);
        if (d_gX) {
            // dL/dX = dA W1^T, contracted over exactly H columns (dA's padding columns are not written)
            const int64_t tot1 = H * D_in;
            transpose_kernel<<<dim3((unsigned)((tot1 + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream>>>(
                (int)D_in, (int)H, (int)H, d_W1, W1T, 1.0f);
            if (int e = launch_transform(N, H, D_in, dA, t.ldh, W1T, nullptr, false, d_gX, ldgx, stream)) return e;
        }
    } else if (d_gX) {
        // dL/dX = dL W1^T over the padded width of dL (its padding columns and the padding rows of W1^T are zero)
        const int64_t tot1 = t.ldc * D_in;
        transpose_kernel<<<dim3((unsigned)((tot1 + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream>>>(
            (int)D_in, (int)C, (int)t.ldc, d_W1, W1T, 1.0f);
        if (int e = launch_transform(N, t.ldc, D_in, L, t.ldc, W1T, nullptr, false, d_gX, ldgx, stream)) return e;
    }
    if (hipGetLastError() != hipSuccess) return RETEXO_E_HIP;
    return RETEXO_OK;
}
}  // namespace

extern "C" int retexo_layer_grad_x(int64_t N, int64_t D_in, int64_t H, int64_t C,
                                   const float* d_X, int64_t ldx, const int32_t* d_labels,
                                   const float* d_W1, const float* d_b1, const float* d_Wc, const float* d_bc,
                                   float* d_gW1, float* d_gb1, float* d_gWc, float* d_gbc, float* d_loss,
                                   float* d_gX, int64_t ldgx,
                                   void* d_workspace, int64_t workspace_bytes, void* stream)
{
    return layer_grad_impl(N, D_in, H, C, d_X, ldx, d_labels, d_W1, d_b1, d_Wc, d_bc, d_gW1, d_gb1, d_gWc, d_gbc,
                           d_loss, d_gX, ldgx, 0.0f, 0, 0, d_workspace, workspace_bytes, stream);
}

extern "C" int retexo_layer_grad_dropout(int64_t N, int64_t D_in, int64_t H, int64_t C,
                                         const float* d_X, int64_t ldx, const int32_t* d_labels,
                                         const float* d_W1, const float* d_b1, const float* d_Wc, const float* d_bc,
                                         float* d_gW1, float* d_gb1, float* d_gWc, float* d_gbc, float* d_loss,
                                         float* d_gX, int64_t ldgx, float p_drop, uint64_t seed, uint64_t draw,
                                         void* d_workspace, int64_t workspace_bytes, void* stream)
{
    return layer_grad_impl(N, D_in, H, C, d_X, ldx, d_labels, d_W1, d_b1, d_Wc, d_bc, d_gW1, d_gb1, d_gWc, d_gbc,
                           d_loss, d_gX, ldgx, p_drop, seed, draw, d_workspace, workspace_bytes, stream);
}

extern "C" int retexo_layer_grad(int64_t N, int64_t D_in, int64_t H, int64_t C,
                                 const float* d_X, int64_t ldx, const int32_t* d_labels,
                                 const float* d_W1, const float* d_b1, const float* d_Wc, const float* d_bc,
                                 float* d_gW1, float* d_gb1, float* d_gWc, float* d_gbc, float* d_loss,
                                 void* d_workspace, int64_t workspace_bytes, void* stream)
{
    return retexo_layer_grad_x(N, D_in, H, C, d_X, ldx, d_labels, d_W1, d_b1, d_Wc, d_bc, d_gW1, d_gb1, d_gWc,
                               d_gbc, d_loss, nullptr, 0, d_workspace, workspace_bytes, stream);
}

namespace {
struct TbLayout { int64_t part, colpart, total; };
TbLayout tb_layout(int64_t N, int64_t D_in, int64_t D_out)
{
    TbLayout t;
    const int64_t n1 = N > 0 ? N : 1;
    int64_t off = 0;
    auto take = [&](int64_t floats) { const int64_t at = off; off += align_up(floats * 4, 256); return at; };
    t.part = take(partial_floats(n1, D_in, D_out));
    t.colpart = take(((n1 + kColRows - 1) / kColRows) * D_out);
    t.total = off;
    return t;
}
}  // namespace

extern "C" int64_t retexo_transform_backward_workspace_bytes(int64_t N, int64_t D_in, int64_t D_out)
{
    if (int s = check_sizes(N, D_in, 0, D_out)) return s;
    return tb_layout(N, D_in, D_out).total;
}

extern "C" int retexo_transform_backward(int64_t N, int64_t D_in, int64_t D_out,
                                         const float* d_H, int64_t ldh, const float* d_dZ, int64_t lddz,
                                         float* d_gW, float* d_gb,
                                         void* d_workspace, int64_t workspace_bytes, void* stream_)
{
    if (int s = check_sizes(N, D_in, 0, D_out)) return s;
    if (ldh < D_in || lddz < D_out) return RETEXO_E_LD;
    if (!d_gW) return RETEXO_E_NULL;
    if (N > 0 && (!d_H || !d_dZ)) return RETEXO_E_NULL;
    const TbLayout t = tb_layout(N, D_in, D_out);
    if (!d_workspace || workspace_bytes < t.total || ((uintptr_t)d_workspace & 255)) return RETEXO_E_WORKSPACE;
    hipStream_t stream = (hipStream_t)stream_;
    if (N == 0) {
        if (launch_zero(d_gW, (size_t)(D_in * D_out) * 4, stream)) return RETEXO_E_HIP;
        if (d_gb) if (launch_zero(d_gb, (size_t)D_out * 4, stream)) return RETEXO_E_HIP;
        return RETEXO_OK;
    }
    char* ws = (char*)d_workspace;
    wgrad(N, D_in, D_out, D_out, d_H, ldh, d_dZ, lddz, (float*)(ws + t.part), d_gW, stream);
    if (d_gb) colsum(N, D_out, d_dZ, lddz, (float*)(ws + t.colpart), d_gb, stream);
    if (hipGetLastError() != hipSuccess) return RETEXO_E_HIP;
    return RETEXO_OK;
}

extern "C" int retexo_sgd_update(int64_t n, float* d_param, const float* d_grad, float lr, void* stream)
{
    if (n < 0) return RETEXO_E_SIZE;
    if (n == 0) return RETEXO_OK;
    if (!d_param || !d_grad) return RETEXO_E_NULL;
    sgd_kernel<<<dim3((unsigned)((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, (hipStream_t)stream>>>(
        n, d_param, d_grad, lr);
    if (hipGetLastError() != hipSuccess) return RETEXO_E_HIP;
    return RETEXO_OK;
}
