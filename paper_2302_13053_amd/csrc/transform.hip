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

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BK = 16;

template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(256) void transform_kernel(
    int64_t N, int D_in, int D_out, const float* __restrict__ H, int64_t ldh,
    const float* __restrict__ W, const float* __restrict__ bias, int relu,
    float* __restrict__ Z, int64_t ldz, int h_vec, int w_vec)
{
    static_assert(WGM * WGN == 4, "four waves per workgroup");
    constexpr int TM = BM / (32 * WGM);      // 32x32 MFMA tiles per wave along M
    constexpr int TN = BN / (32 * WGN);      // and along N
    constexpr int LDA = BM + 4;              // LDS row pitches (floats)
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

    // A tile: thread -> (row = id % BM, k4 = id / BM); rows vary fastest so that
    // the transposing LDS writes of a wave hit consecutive banks
    auto load_a = [&](int kt) {
#pragma unroll
        for (int i = 0; i < A_F4; ++i) {
            const int id = tid + i * 256;
            const int r = id % BM, k4 = id / BM;
            const int64_t row = m0 + r;
            const int k = kt * BK + k4 * 4;
            if (row < N && h_vec && k + 3 < D_in) {
                const f32x4 t = *reinterpret_cast<const f32x4*>(H + row * ldh + k);
                ra[i][0] = t.x; ra[i][1] = t.y; ra[i][2] = t.z; ra[i][3] = t.w;
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    ra[i][q] = (row < N && k + q < D_in) ? H[row * ldh + k + q] : 0.0f;
            }
        }
    };
    // B tile: thread -> (k = id / (BN/4), n4 = id % (BN/4))
    auto load_b = [&](int kt) {
#pragma unroll
        for (int i = 0; i < B_F4; ++i) {
            const int id = tid + i * 256;
            const int kk = id / (BN / 4), n4 = id % (BN / 4);
            const int k = kt * BK + kk;
            const int n = n0 + n4 * 4;
            if (BN * BK / 4 % 256 != 0 && id >= BN * BK / 4) continue;
            if (k < D_in && w_vec && n + 3 < D_out) {
                const f32x4 t = *reinterpret_cast<const f32x4*>(W + (int64_t)k * D_out + n);
                rb[i][0] = t.x; rb[i][1] = t.y; rb[i][2] = t.z; rb[i][3] = t.w;
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    rb[i][q] = (k < D_in && n + q < D_out) ? W[(int64_t)k * D_out + n + q] : 0.0f;
            }
        }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_F4; ++i) {
            const int id = tid + i * 256;
            const int r = id % BM, k4 = id / BM;
#pragma unroll
            for (int q = 0; q < 4; ++q) As[buf][k4 * 4 + q][r] = ra[i][q];
        }
#pragma unroll
        for (int i = 0; i < B_F4; ++i) {
            const int id = tid + i * 256;
            if (BN * BK / 4 % 256 != 0 && id >= BN * BK / 4) continue;
            const int kk = id / (BN / 4), n4 = id % (BN / 4);
            f32x4 t = {rb[i][0], rb[i][1], rb[i][2], rb[i][3]};
            *reinterpret_cast<f32x4*>(&Bs[buf][kk][n4 * 4]) = t;
        }
    };

    const int nk = (D_in + BK - 1) / BK;
    load_a(0);
    load_b(0);
    store_tiles(0);
    __syncthreads();

    const int lrow = lane & 31, lk = lane >> 5;
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) { load_a(kt + 1); load_b(kt + 1); }
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

    // accumulator element r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32 of its tile
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * TN * 32 + j * 32 + lrow;
        if (col >= D_out) continue;
        const float bv = bias ? bias[col] : 0.0f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + wm * TM * 32 + i * 32 + 8 * (r / 4) + 4 * lk + (r % 4);
                if (row < N) {
                    float x = acc[i][j][r] + bv;
                    if (relu) x = fmaxf(x, 0.0f);
                    Z[row * ldz + col] = x;
                }
            }
        }
    }
}

template <int BM, int BN, int WGM, int WGN>
void launch(int64_t N, int64_t D_in, int64_t D_out, const float* H, int64_t ldh, const float* W,
            const float* b, bool relu, float* Z, int64_t ldz, hipStream_t stream)
{
    const int h_vec = ((uintptr_t)H % 16 == 0 && ldh % 4 == 0) ? 1 : 0;
    const int w_vec = ((uintptr_t)W % 16 == 0 && D_out % 4 == 0) ? 1 : 0;
    dim3 grid((unsigned)((N + BM - 1) / BM), (unsigned)((D_out + BN - 1) / BN));
    transform_kernel<BM, BN, WGM, WGN><<<grid, dim3(256), 0, stream>>>(
        N, (int)D_in, (int)D_out, H, ldh, W, b, relu ? 1 : 0, Z, ldz, h_vec, w_vec);
}

}  // namespace

int launch_transform(int64_t N, int64_t D_in, int64_t D_out, const float* H, int64_t ldh,
                     const float* W, const float* b, bool relu, float* Z, int64_t ldz,
                     hipStream_t stream)
{
    if (N == 0 || D_out == 0) return RETEXO_OK;
    if (D_out <= 32)       launch<128, 32, 4, 1>(N, D_in, D_out, H, ldh, W, b, relu, Z, ldz, stream);
    else if (D_out <= 64)  launch<128, 64, 4, 1>(N, D_in, D_out, H, ldh, W, b, relu, Z, ldz, stream);
    else if (D_out <= 128) launch<128, 128, 2, 2>(N, D_in, D_out, H, ldh, W, b, relu, Z, ldz, stream);
    else                   launch<128, 256, 2, 2>(N, D_in, D_out, H, ldh, W, b, relu, Z, ldz, stream);
    if (hipGetLastError() != hipSuccess) return RETEXO_E_HIP;
    return RETEXO_OK;
}
