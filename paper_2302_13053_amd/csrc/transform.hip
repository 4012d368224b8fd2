// Dense transform Z = act(H W + b): the fully connected layer (+ ReLU) that is
// the f of Eq. 1, evaluated for every node once a layer has been trained.
//
// This is the one dense contraction on the path, so it runs on the matrix
// cores in full fp32 (v_mfma_f32_32x32x2_f32: a 32x32 output tile, two k per
// instruction, fp32 multiply and accumulate) — reduced-precision matrix
// formats would not meet the 1e-5 bound.
//
// Tiling.  A workgroup of 4 waves owns a BM x BN output tile with BN >= D_out
// whenever D_out <= 256, so H — by far the larger operand — is read from HBM
// exactly once.  The K loop moves BK = 16 columns of H and rows of W per step
// through LDS, both stored k-major so that the MFMA operand of lane l
// (row l%32, k = l/32) is a conflict-free consecutive read.
//
// Schedule.  One wave keeps a matrix core busy only if nothing else in its
// instruction stream takes longer than one MFMA (64 cycles), so all staging
// work is cut into pieces of that size and placed between the MFMAs of the
// wave that does it: the operand reads of the next k-step after the first MFMA
// of a step, then one slice per step of "write the next tile to the other LDS
// buffer" and "fetch the tile after that into registers".  Global loads
// therefore have a whole K step of MFMAs (4096 cycles) to arrive, and the one
// barrier per K step sits between the last two k-steps, whose operands are
// already in registers.  Sources are clamped instead of checked (rows past the
// end repeat the last row, columns past D_out repeat the last four), so the
// loop carries no selects; only a partial last K tile takes a checked form
// (and the k-steps of it that hold nothing but zero fill are skipped: D_in =
// 100 issues 50 k-steps, not 56).  Bias and ReLU are applied to the
// accumulators on the way out: through this wave's piece of the dead tiles in
// LDS and from there as 16-byte pieces of rows where the output allows it,
// otherwise through one pointer per 32x32 tile that walks down the rows.
//
// W rows that are not multiples of 16 bytes (41, 47, 7 output columns) keep
// this kernel and fetch W, the small operand, element by element; H rows that
// cannot be fetched as aligned 16-byte pieces take the simple kernel below it
// (same arithmetic, same order, checked scalar loads).  Matrices of few rows
// take the few-rows kernel at the end (K split over the waves of a workgroup).
#include "common.hpp"
#include "tiles.hpp"

#include <type_traits>

namespace {

constexpr int BK = kTileK;

// Bias, ReLU, optional mask and store of the accumulators of one wave.
// Accumulator element r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32 of its tile.
// Only the last row block of the matrix checks rows.
template <int TM, int TN, bool MASKED>
__device__ __forceinline__ void write_out(const f32x16 (&acc)[TM][TN], const float (&bv)[TN], int64_t N, int D_out,
                                          int64_t row_base, int col_base, int lane, int relu,
                                          float* __restrict__ Z, int64_t ldz, const float* __restrict__ mask, int64_t ldm,
                                          bool whole_block)
{
    const int lrow = lane & 31, lk = lane >> 5;
    auto run = [&](auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = col_base + j * 32 + lrow;
            if (col >= D_out) continue;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int64_t row0 = row_base + i * 32 + 4 * lk;
                float* p = Z + row0 * ldz + col;
                float mv[16];
                if constexpr (MASKED) {
                    // backward of a ReLU layer: the value passes only where the forward activation was positive
                    const float* pm = mask + row0 * ldm + col;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int ro = 8 * (r / 4) + (r % 4);
                        mv[r] = (FULL || row0 + ro < N) ? pm[ro * ldm] : 0.0f;
                    }
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int ro = 8 * (r / 4) + (r % 4);
                    float x = acc[i][j][r] + bv[j];
                    if (relu) x = fmaxf(x, 0.0f);
                    if constexpr (MASKED) x = mv[r] > 0.0f ? x : 0.0f;
                    if (FULL || row0 + ro < N) p[ro * ldz] = x;
                }
            }
        }
    };
    if (whole_block) run(std::true_type{});
    else run(std::false_type{});
}

// The same epilogue for outputs whose rows allow 16-byte stores (Z and the mask 16-byte aligned, ldz, ldm and
// D_out multiples of four): each 32 x CW block of results goes through this wave's own piece of LDS (T, 32 rows
// of CW + 4 floats; the K loop's tiles are dead by then) and leaves as whole 16-byte pieces of rows, four times
// fewer store instructions, each covering full cache lines.  Same values as write_out.
template <int TM, int TN, int CW, bool MASKED>
__device__ __forceinline__ void write_out_rows(const f32x16 (&acc)[TM][TN], const float (&bv)[TN], int64_t N, int D_out,
                                               int64_t row_base, int col_base, int lane, int relu,
                                               float* __restrict__ Z, int64_t ldz, const float* __restrict__ mask, int64_t ldm,
                                               float* __restrict__ T)
{
    constexpr int P = CW + 4;            // LDS pitch: rows stay 16-byte aligned, column reads spread over the banks
    constexpr int JT = CW / 32;          // accumulator tiles per pass
    constexpr int LPR = CW / 4;          // lanes that cover one row of the pass
    constexpr int RPI = 64 / LPR;        // rows per store instruction
    static_assert(TN % JT == 0, "passes cover whole tiles");
    const int lrow = lane & 31, lk = lane >> 5;
    const int c4 = (lane % LPR) * 4, rsub = lane / LPR;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j0 = 0; j0 < TN; j0 += JT) {
#pragma unroll
            for (int jj = 0; jj < JT; ++jj)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int ro = 8 * (r / 4) + (r % 4) + 4 * lk;
                    float x = acc[i][j0 + jj][r] + bv[j0 + jj];
                    if (relu) x = fmaxf(x, 0.0f);
                    T[ro * P + jj * 32 + lrow] = x;
                }
            const int col = col_base + j0 * 32 + c4;
#pragma unroll
            for (int s = 0; s < 32 / RPI; ++s) {
                const int rr = s * RPI + rsub;
                f32x4 v = *reinterpret_cast<const f32x4*>(&T[rr * P + c4]);
                const int64_t row = row_base + i * 32 + rr;
                if (row < N && col < D_out) {
                    if constexpr (MASKED) {
                        const f32x4 m = *reinterpret_cast<const f32x4*>(mask + row * ldm + col);
#pragma unroll
                        for (int q = 0; q < 4; ++q) v[q] = m[q] > 0.0f ? v[q] : 0.0f;
                    }
                    *reinterpret_cast<f32x4*>(Z + row * ldz + col) = v;
                }
            }
        }
    }
}

// Aligned shapes: H rows are multiples of 16 bytes at 16-byte aligned addresses.  WVEC: so are the rows of W
// (D_out % 4 == 0, D_out >= 4); otherwise W — the small operand, resident in L2 — is fetched element by element
// (same tiles, same order of arithmetic), which lets classifier-width outputs (41, 47, 7 columns) use this kernel
// and its two-tiles-ahead prefetch of H instead of the simple kernel below.
// ZVEC: the output (and the mask) allow 16-byte stores, see write_out_rows.
template <int BM, int BN, int WGM, int WGN, bool MASKED, bool WVEC = true, bool ZVEC = false>
__global__ __launch_bounds__(256, 2) void transform_kernel(
    int64_t N, int D_in, int D_out, const float* __restrict__ H, int64_t ldh,
    const float* __restrict__ W, const float* __restrict__ bias, int relu,
    float* __restrict__ Z, int64_t ldz, const float* __restrict__ mask, int64_t ldm)
{
    static_assert(WGM * WGN == 4, "four waves per workgroup");
    constexpr int TM = BM / (32 * WGM);
    constexpr int TN = BN / (32 * WGN);
    constexpr int LDA = BM + 2;
    constexpr int LDB = BN + 4;
    constexpr int A_F4 = BM * BK / 4 / 256;
    constexpr int B_F4 = (BN * BK / 4 + 255) / 256;
    constexpr bool B_PART = BN * BK / 4 % 256 != 0;
    static_assert(A_F4 >= 1, "tile shape");
    // row-wise epilogue: 64 columns per pass where the tiles leave room for four waves' 32 x 68 blocks, else 32
    constexpr int CW = (TN % 2 == 0 && 2 * BK * (LDA + LDB) >= 4 * 32 * 68) ? 64 : 32;
    static_assert(2 * BK * (LDA + LDB) >= 4 * 32 * (CW + 4), "the epilogue's blocks fit in the tiles' memory");

    __shared__ __align__(16) float lds[2 * BK * (LDA + LDB)];
    float (*As)[BK][LDA] = reinterpret_cast<float (*)[BK][LDA]>(lds);
    float (*Bs)[BK][LDB] = reinterpret_cast<float (*)[BK][LDB]>(lds + 2 * BK * LDA);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;
    const int lrow = lane & 31;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // per-thread source pointers; rows past the end and columns past D_out are clamped to the
    // last valid ones (their products land in outputs that are never stored)
    const float* pa[A_F4];
    const float* pb[B_F4];
    int ka[A_F4], kb[B_F4];                   // k offset of the thread's element inside a tile
#pragma unroll
    for (int i = 0; i < A_F4; ++i) {
        const int id = tid + i * 256;
        const int r = id / 4, k4 = id % 4;
        int64_t row = m0 + r;
        row = row < N ? row : N - 1;
        pa[i] = H + row * ldh + k4 * 4;
        ka[i] = k4 * 4;
    }
    int cb[B_F4][4];                          // !WVEC: column offsets of the four elements from pb (clamped to the last column)
#pragma unroll
    for (int i = 0; i < B_F4; ++i) {
        const int id = tid + i * 256;
        const int kk = (id / (BN / 4)) % BK, n4 = id % (BN / 4);
        int n = n0 + n4 * 4;
        if constexpr (WVEC) {
            n = n < D_out - 4 ? n : D_out - 4;
            pb[i] = W + (int64_t)kk * D_out + n;
        } else {
            pb[i] = W + (int64_t)kk * D_out;
#pragma unroll
            for (int q = 0; q < 4; ++q) cb[i][q] = n + q < D_out ? n + q : D_out - 1;
        }
        kb[i] = kk;
    }
    const int64_t step_b = (int64_t)BK * D_out;

    f32x4 ra[A_F4], rb[B_F4];
    const int nk = (D_in + BK - 1) / BK;
    const int k_tail = D_in % BK;             // > 0: the last tile is partly outside the matrix

    // fetch tile kt into the staging registers; the partial last tile takes the checked form
    auto fetch_a = [&](int kt) {
        if (k_tail && kt == nk - 1) {
#pragma unroll
            for (int i = 0; i < A_F4; ++i) {
                const bool in = ka[i] < k_tail;
                const f32x4 t = *reinterpret_cast<const f32x4*>(in ? pa[i] : H);
                ra[i] = in ? t : f32x4{0.f, 0.f, 0.f, 0.f};
            }
        } else {
#pragma unroll
            for (int i = 0; i < A_F4; ++i) ra[i] = *reinterpret_cast<const f32x4*>(pa[i]);
        }
#pragma unroll
        for (int i = 0; i < A_F4; ++i) pa[i] += BK;
    };
    auto fetch_b = [&](int kt) {
        if constexpr (!WVEC) {
            const bool tail = k_tail && kt == nk - 1;
#pragma unroll
            for (int i = 0; i < B_F4; ++i) {
                const bool in = !tail || kb[i] < k_tail;
                const float* row = in ? pb[i] : W;
                f32x4 t;
#pragma unroll
                for (int q = 0; q < 4; ++q) t[q] = row[cb[i][q]];
                rb[i] = in ? t : f32x4{0.f, 0.f, 0.f, 0.f};
            }
        } else if (k_tail && kt == nk - 1) {
#pragma unroll
            for (int i = 0; i < B_F4; ++i) {
                const bool in = kb[i] < k_tail;
                const f32x4 t = *reinterpret_cast<const f32x4*>(in ? pb[i] : W);
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
        const int r = id / 4, k4 = id % 4;
#pragma unroll
        for (int q = 0; q < 4; ++q) As[buf][k4 * 4 + q][r] = ra[i][q];
    };
    auto put_b = [&](int buf, int i) {
        const int id = tid + i * 256;
        if (B_PART && id >= BN * BK / 4) return;
        const int kk = id / (BN / 4), n4 = id % (BN / 4);
        *reinterpret_cast<f32x4*>(&Bs[buf][kk][n4 * 4]) = rb[i];
    };

    float bv[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * TN * 32 + j * 32 + lrow;
        bv[j] = (bias && col < D_out) ? bias[col] : 0.0f;
    }

    // prologue: tile 0 -> LDS, tile 1 -> staging registers
    fetch_a(0);
    fetch_b(0);
#pragma unroll
    for (int i = 0; i < A_F4; ++i) put_a(0, i);
#pragma unroll
    for (int i = 0; i < B_F4; ++i) put_b(0, i);
    if (nk > 1) { fetch_a(1); fetch_b(1); }
    __syncthreads();

    // thirds of "staged tile -> LDS": the A pieces, the first B piece, the other B pieces
    auto put = [&](int buf, int third) {
        if (third == 0) {
            put_a(buf, 0);
            if (A_F4 > 1) put_a(buf, 1);
        } else if (third == 1) {
#pragma unroll
            for (int x = 2; x < A_F4; ++x) put_a(buf, x);
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
    mfma_k_loop<TM, TN, LDA, LDB>(acc, As, Bs, nk, wm * TM * 32, wn * TN * 32, lane, put, fetch,
                                  k_tail ? (k_tail + 1) / 2 : BK / 2);

    if constexpr (ZVEC) {
        __syncthreads();                      // every wave is done with the last tile
        write_out_rows<TM, TN, CW, MASKED>(acc, bv, N, D_out, m0 + wm * TM * 32, n0 + wn * TN * 32, lane, relu, Z, ldz,
                                           mask, ldm, lds + wave * 32 * (CW + 4));
    } else {
        write_out<TM, TN, MASKED>(acc, bv, N, D_out, m0 + wm * TM * 32, n0 + wn * TN * 32, lane, relu, Z, ldz, mask, ldm,
                                  m0 + BM <= N);
    }
}

// Any shape: every element is fetched under its own check (HV / WV: the rows of H / W still allow 16-byte
// loads), the next K step's loads are issued before this step's MFMAs and written to the other LDS
// buffer after them.
template <int BM, int BN, int WGM, int WGN, bool HV, bool WV, bool MASKED>
__global__ __launch_bounds__(256, 2) void transform_generic_kernel(
    int64_t N, int D_in, int D_out, const float* __restrict__ H, int64_t ldh,
    const float* __restrict__ W, const float* __restrict__ bias, int relu,
    float* __restrict__ Z, int64_t ldz, const float* __restrict__ mask, int64_t ldm)
{
    static_assert(WGM * WGN == 4, "four waves per workgroup");
    constexpr int TM = BM / (32 * WGM);      // 32x32 MFMA tiles per wave along M
    constexpr int TN = BN / (32 * WGN);      // and along N
    constexpr int LDA = BM + 2;              // LDS row pitches (floats): see the A-tile mapping below
    constexpr int LDB = BN + 4;
    constexpr int A_F4 = BM * BK / 4 / 256;  // float4 loads per thread per step
    constexpr int B_F4 = (BN * BK / 4 + 255) / 256;
    static_assert(A_F4 >= 1, "tile too small");

    __shared__ float As[2][BK][LDA];
    __shared__ float Bs[2][BK][LDB];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    float ra[A_F4][4], rb[B_F4][4];
    int wa[A_F4], wb[B_F4];                  // how many of the four are real (see load4)

    // A tile: thread -> (row = id / 4, k4 = id % 4): four lanes read the 64 contiguous bytes of
    // a row, and with a row pitch of BM + 2 floats the transposing LDS writes of each half-wave
    // (4 k-rows x 8 rows) fall into 32 different banks
    auto load_a = [&](int kt) {
#pragma unroll
        for (int i = 0; i < A_F4; ++i) {
            const int id = tid + i * 256;
            const int r = id / 4, k4 = id % 4;
            const int64_t row = m0 + r;
            const int k = kt * BK + k4 * 4;
            wa[i] = row < N ? D_in - k : 0;                   // may be <= 0 or > 4
            load4<HV>(H, row * ldh + k, wa[i], ra[i]);
        }
    };
    // B tile: thread -> (k = id / (BN/4), n4 = id % (BN/4))
    auto load_b = [&](int kt) {
#pragma unroll
        for (int i = 0; i < B_F4; ++i) {
            const int id = tid + i * 256;
            if (BN * BK / 4 % 256 != 0 && id >= BN * BK / 4) continue;
            const int kk = id / (BN / 4), n4 = id % (BN / 4);
            const int k = kt * BK + kk;
            const int n = n0 + n4 * 4;
            wb[i] = k < D_in ? D_out - n : 0;
            load4<WV>(W, (int64_t)k * D_out + n, wb[i], rb[i]);
        }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_F4; ++i) {
            const int id = tid + i * 256;
            const int r = id / 4, k4 = id % 4;
            zero4<HV>(wa[i], ra[i]);
#pragma unroll
            for (int q = 0; q < 4; ++q) As[buf][k4 * 4 + q][r] = ra[i][q];
        }
#pragma unroll
        for (int i = 0; i < B_F4; ++i) {
            const int id = tid + i * 256;
            if (BN * BK / 4 % 256 != 0 && id >= BN * BK / 4) continue;
            const int kk = id / (BN / 4), n4 = id % (BN / 4);
            zero4<WV>(wb[i], rb[i]);
            f32x4 t = {rb[i][0], rb[i][1], rb[i][2], rb[i][3]};
            *reinterpret_cast<f32x4*>(&Bs[buf][kk][n4 * 4]) = t;
        }
    };

    const int lrow = lane & 31, lk = lane >> 5;
    // bias of this lane's output columns, fetched up front so that the stores at the end wait for nothing
    float bv[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * TN * 32 + j * 32 + lrow;
        bv[j] = (bias && col < D_out) ? bias[col] : 0.0f;
    }

    const int nk = (D_in + BK - 1) / BK;
    load_a(0);
    load_b(0);
    store_tiles(0);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) { load_a(kt + 1); load_b(kt + 1); }
        // operand fragments are double-buffered in registers: the LDS reads of k-step s+1 are issued
        // before the MFMAs of k-step s
        float af[2][TM], bf[2][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) af[0][i] = As[buf][lk][wm * TM * 32 + i * 32 + lrow];
#pragma unroll
        for (int j = 0; j < TN; ++j) bf[0][j] = Bs[buf][lk][wn * TN * 32 + j * 32 + lrow];
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            const int cur = (kk >> 1) & 1;
            if (kk + 2 < BK) {
#pragma unroll
                for (int i = 0; i < TM; ++i) af[cur ^ 1][i] = As[buf][kk + 2 + lk][wm * TM * 32 + i * 32 + lrow];
#pragma unroll
                for (int j = 0; j < TN; ++j) bf[cur ^ 1][j] = Bs[buf][kk + 2 + lk][wn * TN * 32 + j * 32 + lrow];
            }
            RETEXO_SCHED_FENCE();                    // keep those reads ahead of this step's MFMAs
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[cur][i], bf[cur][j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_tiles(buf ^ 1);
        __syncthreads();
    }

    write_out<TM, TN, MASKED>(acc, bv, N, D_out, m0 + wm * TM * 32, n0 + wn * TN * 32, lane, relu, Z, ldz, mask, ldm,
                              m0 + BM <= N);
}

// Few rows: a matrix with so few 128-row blocks that they would leave most compute units idle (a citation
// graph's 2,708 x 2,866 features give 22) is cut into 32-row blocks, and the K extent of each block is cut
// over the eight waves of its workgroup.  A wave needs no LDS and no barrier in its loop: per group of 8 k it
// fetches its operands straight into the MFMA layout — lane l holds k = 4 (l / 32) .. + 3 of row l % 32, so
// MFMA q of the group pairs k = q (lower half-wave) with k = 4 + q (upper half-wave) — four groups at a time,
// the next four in flight behind the MFMAs.  The eight partial tiles are then added in a fixed order (wave w + wave w + 4 in registers, then
// ((0 + 1) + 2) + 3 through LDS), so the result is reproducible; it differs from the block kernels' only in
// the order of the fp32 additions.
template <int TN, bool HV, bool MASKED>
__global__ __launch_bounds__(512) void transform_few_rows_kernel(
    int64_t N, int D_in, int D_out, const float* __restrict__ H, int64_t ldh,
    const float* __restrict__ W, const float* __restrict__ bias, int relu,
    float* __restrict__ Z, int64_t ldz, const float* __restrict__ mask, int64_t ldm)
{
    constexpr int BN = TN * 32, NW = 8;
    __shared__ float part[NW / 2][32][BN];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lk = lane >> 5;
    const int64_t m0 = (int64_t)blockIdx.x * 32;
    const int n0 = blockIdx.y * BN;

    const int groups = (D_in + 7) / 8;
    const int per = (groups + NW - 1) / NW;
    const int g0 = wave * per;
    const int g1 = g0 + per < groups ? g0 + per : groups;

    int64_t row = m0 + lrow;
    row = row < N ? row : N - 1;                 // rows past the end repeat the last one; never stored
    const float* hp = H + row * ldh;
    int col[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int c = n0 + j * 32 + lrow;
        col[j] = c < D_out ? c : D_out - 1;
    }

    f32x16 acc[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;

    // operands of U groups at a time, the next U in flight behind this batch's MFMAs (a wave's loop is a chain
    // of memory latencies; the batch is what keeps enough bytes in flight)
    constexpr int U = 4;
    float a[2][U][4], b[2][U][TN][4];
    auto wanted_of = [&](int g) {                // how many of this lane's four k of group g are data
        const int left = g < g1 ? D_in - (g * 8 + lk * 4) : 0;
        return left < 0 ? 0 : (left < 4 ? left : 4);
    };
    auto fetch = [&](int gb, int slot) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = (gb + u) * 8 + lk * 4;
            const int wanted = wanted_of(gb + u);
            load4<HV>(hp, k, wanted, a[slot][u]);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float* wr = W + (int64_t)(q < wanted ? k + q : 0) * D_out;
#pragma unroll
                for (int j = 0; j < TN; ++j) b[slot][u][j][q] = wr[col[j]];
            }
        }
    };
    auto zero = [&](int gb, int slot) {          // what is not data was fetched from k = 0: replace it
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int wanted = wanted_of(gb + u);
            zero4<HV>(wanted, a[slot][u]);
#pragma unroll
            for (int j = 0; j < TN; ++j) zero4<false>(wanted, b[slot][u][j]);
        }
    };

    auto batch = [&](int gb, auto slot_tag) {    // slot as a type: register arrays want constant indices
        constexpr int cur = decltype(slot_tag)::value;
        if (gb + U < g1) fetch(gb + U, cur ^ 1);
        RETEXO_SCHED_FENCE();
        zero(gb, cur);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][u][q], b[cur][u][j][q], acc[j], 0, 0, 0);
    };
    if (g0 < g1) fetch(g0, 0);
    for (int gb = g0; gb < g1; gb += 2 * U) {
        batch(gb, std::integral_constant<int, 0>{});
        if (gb + U < g1) batch(gb + U, std::integral_constant<int, 1>{});
    }

    // accumulator element r of lane l: row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32 of its tile
    auto put = [&](int slot) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) part[slot][8 * (r / 4) + 4 * lk + (r % 4)][j * 32 + lrow] = acc[j][r];
    };
    if (wave >= NW / 2) put(wave - NW / 2);
    __syncthreads();
    if (wave < NW / 2) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][r] += part[wave][8 * (r / 4) + 4 * lk + (r % 4)][j * 32 + lrow];
    }
    __syncthreads();
    if (wave < NW / 2) put(wave);
    __syncthreads();

    for (int e = tid; e < 32 * BN; e += 512) {
        const int r = e / BN, c = e % BN;
        const int64_t orow = m0 + r;
        const int ocol = n0 + c;
        if (orow >= N || ocol >= D_out) continue;
        float x = ((part[0][r][c] + part[1][r][c]) + part[2][r][c]) + part[3][r][c];
        x += bias ? bias[ocol] : 0.0f;
        if (relu) x = fmaxf(x, 0.0f);
        if constexpr (MASKED) x = mask[orow * ldm + ocol] > 0.0f ? x : 0.0f;
        Z[orow * ldz + ocol] = x;
    }
}

// D_in == 0: the product is empty and every row is act(b); H and W are not touched (they may be NULL)
__global__ void bias_rows_kernel(int64_t N, int D_out, const float* __restrict__ bias, int relu,
                                 float* __restrict__ Z, int64_t ldz, const float* __restrict__ mask, int64_t ldm)
{
    const int64_t total = N * D_out;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = e / D_out;
        const int col = (int)(e % D_out);
        float x = bias ? bias[col] : 0.0f;
        if (relu) x = fmaxf(x, 0.0f);
        if (mask) x = mask[row * ldm + col] > 0.0f ? x : 0.0f;
        Z[row * ldz + col] = x;
    }
}

template <int BM, int BN, int WGM, int WGN, bool MASKED>
void launch(int64_t N, int64_t D_in, int64_t D_out, const float* H, int64_t ldh, const float* W,
            const float* b, bool relu, float* Z, int64_t ldz, const float* mask, int64_t ldm,
            hipStream_t stream)
{
    // 16-byte loads need aligned rows and widths that are multiples of four floats
    const bool hv = (uintptr_t)H % 16 == 0 && ldh % 4 == 0 && D_in % 4 == 0;
    const bool wv = (uintptr_t)W % 16 == 0 && D_out % 4 == 0;
    dim3 grid((unsigned)((N + BM - 1) / BM), (unsigned)((D_out + BN - 1) / BN));
    const int r = relu ? 1 : 0;
    const bool zv = (uintptr_t)Z % 16 == 0 && ldz % 4 == 0 && D_out % 4 == 0 &&
                    (!MASKED || ((uintptr_t)mask % 16 == 0 && ldm % 4 == 0));
    if (hv && wv && zv)
        transform_kernel<BM, BN, WGM, WGN, MASKED, true, true><<<grid, dim3(256), 0, stream>>>(N, (int)D_in, (int)D_out, H, ldh, W, b, r, Z, ldz, mask, ldm);
    else if (hv && wv)
        transform_kernel<BM, BN, WGM, WGN, MASKED><<<grid, dim3(256), 0, stream>>>(N, (int)D_in, (int)D_out, H, ldh, W, b, r, Z, ldz, mask, ldm);
    else if (hv)
        transform_kernel<BM, BN, WGM, WGN, MASKED, false><<<grid, dim3(256), 0, stream>>>(N, (int)D_in, (int)D_out, H, ldh, W, b, r, Z, ldz, mask, ldm);
    else if (wv)
        transform_generic_kernel<BM, BN, WGM, WGN, false, true, MASKED><<<grid, dim3(256), 0, stream>>>(N, (int)D_in, (int)D_out, H, ldh, W, b, r, Z, ldz, mask, ldm);
    else
        transform_generic_kernel<BM, BN, WGM, WGN, false, false, MASKED><<<grid, dim3(256), 0, stream>>>(N, (int)D_in, (int)D_out, H, ldh, W, b, r, Z, ldz, mask, ldm);
}

template <bool MASKED>
void launch_few_rows(int64_t N, int64_t D_in, int64_t D_out, const float* H, int64_t ldh, const float* W,
                     const float* b, bool relu, float* Z, int64_t ldz, const float* mask, int64_t ldm,
                     hipStream_t stream)
{
    const bool hv = (uintptr_t)H % 16 == 0 && ldh % 4 == 0 && D_in % 4 == 0;
    const int r = relu ? 1 : 0;
    const unsigned gx = (unsigned)((N + 31) / 32);
    // 32-column tiles when 64-column ones would not give every compute unit a workgroup
    if (D_out <= 32 || (int64_t)gx * ((D_out + 63) / 64) < 256) {
        dim3 grid(gx, (unsigned)((D_out + 31) / 32));
        if (hv) transform_few_rows_kernel<1, true, MASKED><<<grid, dim3(512), 0, stream>>>(N, (int)D_in, (int)D_out, H, ldh, W, b, r, Z, ldz, mask, ldm);
        else    transform_few_rows_kernel<1, false, MASKED><<<grid, dim3(512), 0, stream>>>(N, (int)D_in, (int)D_out, H, ldh, W, b, r, Z, ldz, mask, ldm);
    } else {
        dim3 grid(gx, (unsigned)((D_out + 63) / 64));
        if (hv) transform_few_rows_kernel<2, true, MASKED><<<grid, dim3(512), 0, stream>>>(N, (int)D_in, (int)D_out, H, ldh, W, b, r, Z, ldz, mask, ldm);
        else    transform_few_rows_kernel<2, false, MASKED><<<grid, dim3(512), 0, stream>>>(N, (int)D_in, (int)D_out, H, ldh, W, b, r, Z, ldz, mask, ldm);
    }
}

// Fewer 128-row blocks (times the column blocks) than the "transform_few_blocks" setting, 128 unless changed:
// the few-rows kernel.  The choice depends on the shape only, never on alignment, so one shape always takes
// one order of additions.

template <bool MASKED>
void launch_by_width(int64_t N, int64_t D_in, int64_t D_out, const float* H, int64_t ldh, const float* W,
                     const float* b, bool relu, float* Z, int64_t ldz, const float* mask, int64_t ldm,
                     hipStream_t stream)
{
    const int64_t bn = D_out <= 32 ? 32 : D_out <= 64 ? 64 : D_out <= 128 ? 128 : D_out <= 192 ? 192 : 256;
    if ((N + 127) / 128 * ((D_out + bn - 1) / bn) < agg_options().few_blocks) {
        launch_few_rows<MASKED>(N, D_in, D_out, H, ldh, W, b, relu, Z, ldz, mask, ldm, stream);
        return;
    }
    if (D_out <= 32)       launch<128, 32, 4, 1, MASKED>(N, D_in, D_out, H, ldh, W, b, relu, Z, ldz, mask, ldm, stream);
    else if (D_out <= 64)  launch<128, 64, 4, 1, MASKED>(N, D_in, D_out, H, ldh, W, b, relu, Z, ldz, mask, ldm, stream);
    else if (D_out <= 128) launch<128, 128, 2, 2, MASKED>(N, D_in, D_out, H, ldh, W, b, relu, Z, ldz, mask, ldm, stream);
    else if (D_out <= 192) launch<128, 192, 2, 2, MASKED>(N, D_in, D_out, H, ldh, W, b, relu, Z, ldz, mask, ldm, stream);
    else                   launch<128, 256, 2, 2, MASKED>(N, D_in, D_out, H, ldh, W, b, relu, Z, ldz, mask, ldm, stream);
}

}  // namespace

int launch_transform(int64_t N, int64_t D_in, int64_t D_out, const float* H, int64_t ldh,
                     const float* W, const float* b, bool relu, float* Z, int64_t ldz,
                     hipStream_t stream, const float* mask, int64_t ldm)
{
    if (N == 0 || D_out == 0) return RETEXO_OK;
    if (D_in == 0) {
        const int64_t blocks = (N * D_out + 255) / 256;
        bias_rows_kernel<<<dim3((unsigned)(blocks < 65536 ? blocks : 65536)), dim3(256), 0, stream>>>(
            N, (int)D_out, b, relu ? 1 : 0, Z, ldz, mask, ldm);
        return hipGetLastError() != hipSuccess ? RETEXO_E_HIP : RETEXO_OK;
    }
    if (mask) launch_by_width<true>(N, D_in, D_out, H, ldh, W, b, relu, Z, ldz, mask, ldm, stream);
    else      launch_by_width<false>(N, D_in, D_out, H, ldh, W, b, relu, Z, ldz, mask, ldm, stream);
    if (hipGetLastError() != hipSuccess) return RETEXO_E_HIP;
    return RETEXO_OK;
}
