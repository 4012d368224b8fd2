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
// (row l%32, k = l/32) is a conflict-free consecutive read.  The next step's
// global loads are issued into registers before the current step's MFMAs and
// written to the other LDS buffer afterwards (one barrier per step).
// Bias and ReLU are applied to the accumulators before the store.
#include "common.hpp"
#include "tiles.hpp"

namespace {

constexpr int BK = kTileK;

template <int BM, int BN, int WGM, int WGN, bool HV, bool WV>
__global__ __launch_bounds__(256, 2) void transform_kernel(
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
        // before the MFMAs of k-step s, so their latency hides behind matrix work
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
            __builtin_amdgcn_sched_barrier(0);       // keep those reads ahead of this step's MFMAs
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[cur][i], bf[cur][j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_tiles(buf ^ 1);
        __syncthreads();
    }

    // accumulator element r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32 of its tile
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * TN * 32 + j * 32 + lrow;
        if (col >= D_out) continue;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + wm * TM * 32 + i * 32 + 8 * (r / 4) + 4 * lk + (r % 4);
                if (row < N) {
                    float x = acc[i][j][r] + bv[j];
                    if (relu) x = fmaxf(x, 0.0f);
                    // backward of a ReLU layer: pass the value only where the forward activation was positive
                    if (mask) x = mask[row * ldm + col] > 0.0f ? x : 0.0f;
                    Z[row * ldz + col] = x;
                }
            }
        }
    }
}

template <int BM, int BN, int WGM, int WGN>
void launch(int64_t N, int64_t D_in, int64_t D_out, const float* H, int64_t ldh, const float* W,
            const float* b, bool relu, float* Z, int64_t ldz, const float* mask, int64_t ldm,
            hipStream_t stream)
{
    // 16-byte loads need aligned rows and widths that are multiples of four floats
    const bool hv = (uintptr_t)H % 16 == 0 && ldh % 4 == 0 && D_in % 4 == 0;
    const bool wv = (uintptr_t)W % 16 == 0 && D_out % 4 == 0;
    dim3 grid((unsigned)((N + BM - 1) / BM), (unsigned)((D_out + BN - 1) / BN));
    const int r = relu ? 1 : 0;
    if (hv && wv)
        transform_kernel<BM, BN, WGM, WGN, true, true><<<grid, dim3(256), 0, stream>>>(N, (int)D_in, (int)D_out, H, ldh, W, b, r, Z, ldz, mask, ldm);
    else if (hv)
        transform_kernel<BM, BN, WGM, WGN, true, false><<<grid, dim3(256), 0, stream>>>(N, (int)D_in, (int)D_out, H, ldh, W, b, r, Z, ldz, mask, ldm);
    else if (wv)
        transform_kernel<BM, BN, WGM, WGN, false, true><<<grid, dim3(256), 0, stream>>>(N, (int)D_in, (int)D_out, H, ldh, W, b, r, Z, ldz, mask, ldm);
    else
        transform_kernel<BM, BN, WGM, WGN, false, false><<<grid, dim3(256), 0, stream>>>(N, (int)D_in, (int)D_out, H, ldh, W, b, r, Z, ldz, mask, ldm);
}

}  // namespace

int launch_transform(int64_t N, int64_t D_in, int64_t D_out, const float* H, int64_t ldh,
                     const float* W, const float* b, bool relu, float* Z, int64_t ldz,
                     hipStream_t stream, const float* mask, int64_t ldm)
{
    if (N == 0 || D_out == 0) return RETEXO_OK;
    if (D_out <= 32)       launch<128, 32, 4, 1>(N, D_in, D_out, H, ldh, W, b, relu, Z, ldz, mask, ldm, stream);
    else if (D_out <= 64)  launch<128, 64, 4, 1>(N, D_in, D_out, H, ldh, W, b, relu, Z, ldz, mask, ldm, stream);
    else if (D_out <= 128) launch<128, 128, 2, 2>(N, D_in, D_out, H, ldh, W, b, relu, Z, ldz, mask, ldm, stream);
    else                   launch<128, 256, 2, 2>(N, D_in, D_out, H, ldh, W, b, relu, Z, ldz, mask, ldm, stream);
    if (hipGetLastError() != hipSuccess) return RETEXO_E_HIP;
    return RETEXO_OK;
}
