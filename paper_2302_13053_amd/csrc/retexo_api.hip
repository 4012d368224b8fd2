// C entry points of the embed-and-aggregate library: argument checking and the
// sequencing of one lazy message-passing round (transform, then aggregation,
// on one stream).  All checks that need no device access run first, so an
// argument error leaves every output untouched.
#include <string.h>

#include "common.hpp"
#include "tiles.hpp"

namespace {

bool overlaps(const void* a, int64_t a_bytes, const void* b, int64_t b_bytes)
{
    const uintptr_t a0 = (uintptr_t)a, a1 = a0 + (uintptr_t)a_bytes;
    const uintptr_t b0 = (uintptr_t)b, b1 = b0 + (uintptr_t)b_bytes;
    return a0 < b1 && b0 < a1;
}

int64_t extent_bytes(int64_t rows, int64_t ld, int64_t width)
{
    if (rows <= 0) return 0;
    return ((rows - 1) * ld + width) * (int64_t)sizeof(float);
}

int check_mode(int mode, int64_t F, int heads)
{
    if (mode < RETEXO_MEAN || mode > RETEXO_MAX) return RETEXO_E_MODE;
    if (heads < 1 || heads > kMaxHeads) return RETEXO_E_HEADS;
    if (mode == RETEXO_GAT_SOFTMAX && F % heads != 0) return RETEXO_E_HEADS;
    return RETEXO_OK;
}

// bytes of Z held in the workspace by retexo_round (0 when Z lives in `out`)
int64_t round_z_bytes(int64_t N, int64_t D_out, bool have_w, bool concat, int64_t* ldz_out)
{
    const int64_t ldz = align_up(D_out > 0 ? D_out : 1, 32);   // 128-byte rows
    if (ldz_out) *ldz_out = ldz;
    if (!have_w || concat) return 0;
    return align_up((N > 0 ? N : 1) * ldz * (int64_t)sizeof(float), 256);
}

int check_transform_args(int64_t N, int64_t D_in, int64_t D_out, const float* H, int64_t ldh,
                         const float* W, unsigned flags, const float* Z, int64_t ldz)
{
    if (N < 0 || D_in < 0 || D_out < 0) return RETEXO_E_SIZE;
    if (D_in >= (1ll << 31) || D_out >= (1ll << 31)) return RETEXO_E_SIZE;
    if (flags & ~(unsigned)RETEXO_F_RELU) return RETEXO_E_FLAGS;
    if (N > 0 && D_out > 0 && !Z) return RETEXO_E_NULL;
    if (N > 0 && D_in > 0 && (!H || (D_out > 0 && !W))) return RETEXO_E_NULL;
    if (ldh < D_in || ldz < D_out) return RETEXO_E_LD;
    return RETEXO_OK;
}

}  // namespace

extern "C" const char* retexo_status_string(int s)
{
    switch (s) {
        case RETEXO_OK: return "ok";
        case RETEXO_E_NULL: return "required pointer is NULL";
        case RETEXO_E_SIZE: return "negative or inconsistent size";
        case RETEXO_E_LD: return "leading dimension smaller than row width";
        case RETEXO_E_MODE: return "unknown aggregation mode";
        case RETEXO_E_FLAGS: return "unknown or inapplicable flag";
        case RETEXO_E_HEADS: return "bad head count";
        case RETEXO_E_CSR: return "node id out of range or malformed CSR";
        case RETEXO_E_WORKSPACE: return "workspace missing, misaligned or too small";
        case RETEXO_E_ALIAS: return "output overlaps an input";
        case RETEXO_E_HIP: return "HIP runtime call failed";
        case RETEXO_E_CAPACITY: return "output capacity too small";
        case RETEXO_E_PARTITION: return "worker id out of range";
        default: return "unknown status";
    }
}

extern "C" int retexo_set_option(const char* name, int64_t value)
{
    if (!name) return RETEXO_E_NULL;
    AggOptions& o = agg_options();
    if (!strcmp(name, "agg_slab_cols")) { o.slab_cols = value; return RETEXO_OK; }
    if (!strcmp(name, "agg_slab_major")) { o.slab_major = value; return RETEXO_OK; }
    if (!strcmp(name, "agg_heavy_degree")) { o.heavy_degree = value; return RETEXO_OK; }
    if (!strcmp(name, "agg_max_vec")) { o.max_vec = value; return RETEXO_OK; }
    if (!strcmp(name, "agg_parts")) { o.parts = value; return RETEXO_OK; }
    if (!strcmp(name, "agg_gat_fast")) { o.gat_fast = value; return RETEXO_OK; }
    if (!strcmp(name, "agg_gat_flash")) { o.gat_flash = value; return RETEXO_OK; }
    if (!strcmp(name, "agg_gat_fold")) { o.gat_fold = value; return RETEXO_OK; }
    if (!strcmp(name, "agg_gat_in_rows")) { o.gat_in_rows = value; return RETEXO_OK; }
    if (!strcmp(name, "agg_wide_offsets")) { o.wide_offsets = value; return RETEXO_OK; }
    if (!strcmp(name, "agg_narrow_heavy")) { o.narrow_heavy = value; return RETEXO_OK; }
    if (!strcmp(name, "transform_few_blocks")) { if (value < 0) return RETEXO_E_SIZE; o.few_blocks = value; return RETEXO_OK; }
    if (!strcmp(name, "csr_sorted_keys")) { o.csr_sorted_keys = value; return RETEXO_OK; }
    return RETEXO_E_FLAGS;
}

extern "C" int64_t retexo_workspace_bytes(const retexo_plan* plan, int64_t D_out, int mode, int heads,
                                          unsigned flags)
{
    if (!plan) return RETEXO_E_NULL;
    if (D_out < 0) return RETEXO_E_SIZE;
    if (int s = check_mode(mode, D_out, heads)) return s;
    if (flags & ~(unsigned)(RETEXO_F_RELU | RETEXO_F_SELF_CONCAT | RETEXO_F_SAVE)) return RETEXO_E_FLAGS;
    const bool save = (flags & RETEXO_F_SAVE) != 0;
    if (save && mode != RETEXO_GAT_SOFTMAX) return RETEXO_E_FLAGS;
    // retexo_aggregate in save mode: exactly its own layout (the backward call looks into it)
    if (save) return aggregate_workspace_bytes(plan->N, mode, heads, D_out, true);
    // sized for retexo_round with a weight matrix; retexo_aggregate needs only the second term
    return round_z_bytes(plan->N, D_out, true, (flags & RETEXO_F_SELF_CONCAT) != 0, nullptr) +
           aggregate_workspace_bytes(plan->N, mode, heads);
}

extern "C" int retexo_transform(int64_t N, int64_t D_in, int64_t D_out,
                                const float* d_H, int64_t ldh, const float* d_W, const float* d_b,
                                unsigned flags, float* d_Z, int64_t ldz, void* stream)
{
    if (int s = check_transform_args(N, D_in, D_out, d_H, ldh, d_W, flags, d_Z, ldz)) return s;
    if (N > 0 && D_in > 0 && D_out > 0 &&
        overlaps(d_H, extent_bytes(N, ldh, D_in), d_Z, extent_bytes(N, ldz, D_out)))
        return RETEXO_E_ALIAS;
    return launch_transform(N, D_in, D_out, d_H, ldh, d_W, d_b, (flags & RETEXO_F_RELU) != 0, d_Z, ldz,
                            (hipStream_t)stream);
}

extern "C" int retexo_aggregate(const retexo_plan* plan, int mode, int64_t F, int heads,
                                const float* d_Z, int64_t ldz,
                                const float* d_attn_src, const float* d_attn_dst, float negative_slope,
                                unsigned flags, float* d_out, int64_t ldo,
                                void* d_workspace, int64_t workspace_bytes, void* stream)
{
    if (!plan) return RETEXO_E_NULL;
    if (F < 0 || F >= (1ll << 30)) return RETEXO_E_SIZE;
    if (int s = check_mode(mode, F, heads)) return s;
    if (flags & ~(unsigned)(RETEXO_F_SELF_CONCAT | RETEXO_F_SAVE)) return RETEXO_E_FLAGS;
    const bool concat = (flags & RETEXO_F_SELF_CONCAT) != 0;
    const bool save = (flags & RETEXO_F_SAVE) != 0;
    if (save && mode != RETEXO_GAT_SOFTMAX) return RETEXO_E_FLAGS;
    const int64_t N = plan->N, ow = concat ? 2 * F : F;
    if (N > 0 && F > 0 && (!d_Z || !d_out)) return RETEXO_E_NULL;
    if (mode == RETEXO_GAT_SOFTMAX && N > 0 && F > 0 && (!d_attn_src || !d_attn_dst)) return RETEXO_E_NULL;
    if (ldz < F || ldo < ow) return RETEXO_E_LD;
    const bool in_place = concat && (const float*)d_out == d_Z && ldz == ldo;
    if (!in_place && N > 0 && F > 0 &&
        overlaps(d_Z, extent_bytes(N, ldz, F), d_out, extent_bytes(N, ldo, ow)))
        return RETEXO_E_ALIAS;
    const int64_t need = aggregate_workspace_bytes(N, mode, heads, F, save);
    if (need > 0 && (!d_workspace || workspace_bytes < need || ((uintptr_t)d_workspace & 255)))
        return RETEXO_E_WORKSPACE;

    AggCall c;
    c.plan = plan; c.mode = mode; c.F = F; c.heads = heads; c.Z = d_Z; c.ldz = ldz;
    c.attn_src = d_attn_src; c.attn_dst = d_attn_dst; c.slope = negative_slope;
    c.self_concat = concat; c.copy_self = !in_place; c.out = d_out; c.ldo = ldo;
    c.workspace = d_workspace;
    c.save = save;
    return launch_aggregate(c, (hipStream_t)stream);
}

// Network data volumes of the communication-efficiency analysis (host arithmetic only).
// Appendix "Communication-efficiency Analysis": n workers, B boundary nodes per worker, R training
// rounds, feature size H0, intermediate sizes summing to sum_H, added classifier sizes summing to
// sum_C, model size M (all sizes in one unit, e.g. bytes).
extern "C" int retexo_data_volumes(double n, double B, double R, double H0, double sum_H, double sum_C, double M,
                                   double* out4)
{
    if (!out4) return RETEXO_E_NULL;
    if (!(n >= 0.0) || !(B >= 0.0) || !(R > 0.0) || !(H0 >= 0.0) || !(sum_H >= 0.0) || !(sum_C >= 0.0) || !(M > 0.0))
        return RETEXO_E_SIZE;
    out4[0] = 2.0 * n * R * B * (sum_H + sum_H) + 2.0 * n * B * H0;     // standard, local training
    out4[1] = 2.0 * n * B * sum_H + 2.0 * n * B * H0;                   // lazy, local training
    out4[2] = n * R * M + n * R * M;                                    // standard, gradient aggregation
    out4[3] = 2.0 * n * R * M + 2.0 * n * R * sum_C;                    // lazy, gradient aggregation
    return RETEXO_OK;
}

// gamma of Eq. 2: total standard volume over total lazy volume (independent of n)
extern "C" double retexo_gamma(double B, double R, double H0, double sum_H, double sum_C, double M)
{
    double v[4];
    if (retexo_data_volumes(1.0, B, R, H0, sum_H, sum_C, M, v) != RETEXO_OK) return -1.0;
    return (v[0] + v[2]) / (v[1] + v[3]);
}

extern "C" int64_t retexo_aggregate_backward_workspace_bytes(const retexo_plan* plan, int mode, int64_t F, int heads)
{
    if (!plan) return RETEXO_E_NULL;
    if (F < 0 || F >= (1ll << 30)) return RETEXO_E_SIZE;
    if (int s = check_mode(mode, F, heads)) return s;
    if (mode == RETEXO_MAX) return RETEXO_E_MODE;
    if (mode == RETEXO_GAT_SOFTMAX && F > kMaxBackwardSoftmaxWidth) return RETEXO_E_SIZE;
    return aggregate_backward_workspace_bytes(plan->N, mode, F, heads);
}

namespace {
int aggregate_backward_checked(const retexo_plan* plan, int mode, int64_t F, int heads,
                               const float* d_Z, int64_t ldz,
                               const float* d_attn_src, const float* d_attn_dst, float negative_slope,
                               unsigned flags, const float* d_G, int64_t ldg,
                               const void* d_saved, int64_t saved_bytes,
                               float* d_dZ, int64_t lddz, float* d_dattn_src, float* d_dattn_dst,
                               void* d_workspace, int64_t workspace_bytes, void* stream)
{
    if (!plan) return RETEXO_E_NULL;
    if (F < 0 || F >= (1ll << 30)) return RETEXO_E_SIZE;
    if (int s = check_mode(mode, F, heads)) return s;
    if (mode == RETEXO_MAX) return RETEXO_E_MODE;
    if (flags & ~(unsigned)RETEXO_F_SELF_CONCAT) return RETEXO_E_FLAGS;
    const bool gat = mode == RETEXO_GAT_SOFTMAX;
    if (gat && F > kMaxBackwardSoftmaxWidth) return RETEXO_E_SIZE;
    const bool concat = (flags & RETEXO_F_SELF_CONCAT) != 0;
    const int64_t N = plan->N, gw = concat ? 2 * F : F;
    const bool work = N > 0 && F > 0;
    if (work && (!d_G || !d_dZ)) return RETEXO_E_NULL;
    if (gat && work && (!d_Z || !d_attn_src || !d_attn_dst || !d_dattn_src || !d_dattn_dst)) return RETEXO_E_NULL;
    if (ldg < gw || lddz < F || (gat && ldz < F)) return RETEXO_E_LD;
    if (work) {
        if (overlaps(d_G, extent_bytes(N, ldg, gw), d_dZ, extent_bytes(N, lddz, F))) return RETEXO_E_ALIAS;
        if (gat && overlaps(d_Z, extent_bytes(N, ldz, F), d_dZ, extent_bytes(N, lddz, F))) return RETEXO_E_ALIAS;
    }
    const int64_t need = aggregate_backward_workspace_bytes(N, mode, F, heads);
    if (need > 0 && (!d_workspace || workspace_bytes < need || ((uintptr_t)d_workspace & 255)))
        return RETEXO_E_WORKSPACE;
    if (gat && !work && d_dattn_src && d_dattn_dst && F > 0) {
        // no nodes: the parameter gradients are zero
        if (launch_zero(d_dattn_src, (size_t)F * sizeof(float), (hipStream_t)stream) != RETEXO_OK ||
            launch_zero(d_dattn_dst, (size_t)F * sizeof(float), (hipStream_t)stream) != RETEXO_OK)
            return RETEXO_E_HIP;
        return RETEXO_OK;
    }

    AggBackwardCall c;
    c.plan = plan; c.mode = mode; c.F = F; c.heads = heads; c.Z = d_Z; c.ldz = ldz;
    c.attn_src = d_attn_src; c.attn_dst = d_attn_dst; c.slope = negative_slope;
    c.self_concat = concat; c.G = d_G; c.ldg = ldg; c.dZ = d_dZ; c.lddz = lddz;
    c.d_attn_src = d_dattn_src; c.d_attn_dst = d_dattn_dst; c.workspace = d_workspace;
    if (d_saved) {
        if (!gat) return RETEXO_E_MODE;
        if (saved_bytes < aggregate_workspace_bytes(N, mode, heads, F, true) || ((uintptr_t)d_saved & 255))
            return RETEXO_E_WORKSPACE;
        c.saved = d_saved;
    }
    return launch_aggregate_backward(c, (hipStream_t)stream);
}
}  // namespace

extern "C" int retexo_aggregate_backward(const retexo_plan* plan, int mode, int64_t F, int heads,
                                         const float* d_Z, int64_t ldz,
                                         const float* d_attn_src, const float* d_attn_dst, float negative_slope,
                                         unsigned flags, const float* d_G, int64_t ldg,
                                         float* d_dZ, int64_t lddz, float* d_dattn_src, float* d_dattn_dst,
                                         void* d_workspace, int64_t workspace_bytes, void* stream)
{
    return aggregate_backward_checked(plan, mode, F, heads, d_Z, ldz, d_attn_src, d_attn_dst, negative_slope, flags,
                                      d_G, ldg, nullptr, 0, d_dZ, lddz, d_dattn_src, d_dattn_dst,
                                      d_workspace, workspace_bytes, stream);
}

extern "C" int retexo_aggregate_backward_saved(const retexo_plan* plan, int mode, int64_t F, int heads,
                                               const float* d_Z, int64_t ldz,
                                               const float* d_attn_src, const float* d_attn_dst, float negative_slope,
                                               unsigned flags, const float* d_G, int64_t ldg,
                                               const void* d_saved, int64_t saved_bytes,
                                               float* d_dZ, int64_t lddz, float* d_dattn_src, float* d_dattn_dst,
                                               void* d_workspace, int64_t workspace_bytes, void* stream)
{
    if (!d_saved) return RETEXO_E_NULL;
    return aggregate_backward_checked(plan, mode, F, heads, d_Z, ldz, d_attn_src, d_attn_dst, negative_slope, flags,
                                      d_G, ldg, d_saved, saved_bytes, d_dZ, lddz, d_dattn_src,
                                      d_dattn_dst, d_workspace, workspace_bytes, stream);
}

extern "C" int retexo_store_rows(int storage, int64_t N, int64_t F, const float* d_src, int64_t lds,
                                 void* d_dst, int64_t ldd, void* stream)
{
    if (storage != RETEXO_STORE_BF16 && storage != RETEXO_STORE_FP16) return RETEXO_E_MODE;
    if (N < 0 || F < 0) return RETEXO_E_SIZE;
    if (N > 0 && F > 0 && (!d_src || !d_dst)) return RETEXO_E_NULL;
    if (lds < F || ldd < F) return RETEXO_E_LD;
    if (N > 0 && F > 0 && overlaps(d_src, extent_bytes(N, lds, F), d_dst, (size_t)((N - 1) * ldd + F) * 2))
        return RETEXO_E_ALIAS;
    return launch_store_rows(storage, N, F, d_src, lds, d_dst, ldd, (hipStream_t)stream);
}

extern "C" int retexo_aggregate_stored(const retexo_plan* plan, int mode, int storage, int64_t F, int heads,
                                       const void* d_Z, int64_t ldz,
                                       const float* d_attn_src, const float* d_attn_dst, float negative_slope,
                                       unsigned flags, float* d_out, int64_t ldo,
                                       void* d_workspace, int64_t workspace_bytes, void* stream)
{
    if (!plan) return RETEXO_E_NULL;
    if (storage != RETEXO_STORE_BF16 && storage != RETEXO_STORE_FP16) return RETEXO_E_MODE;
    if (F < 0 || F >= (1ll << 30)) return RETEXO_E_SIZE;
    if (int s = check_mode(mode, F, heads)) return s;
    if (flags & ~(unsigned)RETEXO_F_SELF_CONCAT) return RETEXO_E_FLAGS;
    const bool concat = (flags & RETEXO_F_SELF_CONCAT) != 0;
    const int64_t N = plan->N, ow = concat ? 2 * F : F;
    if (N > 0 && F > 0 && (!d_Z || !d_out)) return RETEXO_E_NULL;
    if (mode == RETEXO_GAT_SOFTMAX && N > 0 && F > 0 && (!d_attn_src || !d_attn_dst)) return RETEXO_E_NULL;
    if (ldz < F || ldo < ow) return RETEXO_E_LD;
    if (N > 0 && F > 0 && overlaps(d_Z, (size_t)((N - 1) * ldz + F) * 2, d_out, extent_bytes(N, ldo, ow)))
        return RETEXO_E_ALIAS;
    const int64_t need = aggregate_workspace_bytes(N, mode, heads);
    if (need > 0 && (!d_workspace || workspace_bytes < need || ((uintptr_t)d_workspace & 255)))
        return RETEXO_E_WORKSPACE;
    StoredCall c;
    c.plan = plan; c.mode = mode; c.storage = storage; c.F = F; c.heads = heads; c.Z = d_Z; c.ldz = ldz;
    c.attn_src = d_attn_src; c.attn_dst = d_attn_dst; c.slope = negative_slope;
    c.self_concat = concat; c.copy_self = true; c.out = d_out; c.ldo = ldo; c.workspace = d_workspace;
    return launch_aggregate_stored(c, (hipStream_t)stream);
}

namespace {
__global__ __launch_bounds__(256) void zero_words_kernel(uint32_t* __restrict__ p, size_t words)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < words) p[i] = 0u;
}
}  // namespace

int launch_zero(void* p, size_t bytes, hipStream_t stream)
{
    const size_t words = bytes / 4;
    if (words == 0) return RETEXO_OK;
    zero_words_kernel<<<dim3((unsigned)((words + 255) / 256)), dim3(256), 0, stream>>>((uint32_t*)p, words);
    return hipGetLastError() == hipSuccess ? RETEXO_OK : RETEXO_E_HIP;
}

namespace {
// out[v, c] = (1 / heads) * sum_h in[v, h * C + c]; heads added in index order.
// Rows of up to 1,024 input columns: a workgroup stages kRowsPerBlock whole rows in LDS with the widest loads
// the layout allows (a row is one contiguous piece of memory whatever C is: 4 x 47 columns are 47 float4), then
// every thread adds the heads of its output elements from LDS and the outputs leave as consecutive addresses.
constexpr int kHeadMeanMaxWidth = 1024;
template <bool VEC>
__global__ __launch_bounds__(256) void head_mean_kernel(int64_t N, int heads, int C, int rows_per_block,
                                                         const float* __restrict__ in, int64_t ldi,
                                                         float* __restrict__ out, int64_t ldo)
{
    __shared__ __align__(16) float stage[4 * kHeadMeanMaxWidth];
    const int W = heads * C;                      // input columns of a row
    const int pitch = VEC ? (W + 3) / 4 * 4 : W;  // floats per staged row (VEC: whole float4, ldi covers them)
    const int64_t v0 = (int64_t)blockIdx.x * rows_per_block;
    const int rows = (int)(N - v0 < rows_per_block ? N - v0 : rows_per_block);
    if constexpr (VEC) {
        const int per_row = pitch / 4;
        for (int i = threadIdx.x; i < rows * per_row; i += 256) {
            const int r = i / per_row, q = i % per_row;
            *reinterpret_cast<f32x4*>(&stage[r * pitch + 4 * q]) =
                *reinterpret_cast<const f32x4*>(in + (v0 + r) * ldi + 4 * q);
        }
    } else {
        for (int i = threadIdx.x; i < rows * W; i += 256) {
            const int r = i / W, q = i % W;
            stage[r * pitch + q] = in[(v0 + r) * ldi + q];
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < rows * C; i += 256) {
        const int r = i / C, c = i % C;
        float sum = 0.0f;
        for (int h = 0; h < heads; ++h) sum += stage[r * pitch + h * C + c];
        out[(v0 + r) * ldo + c] = sum / (float)heads;
    }
}

// wider rows: one thread per element
__global__ __launch_bounds__(256) void head_mean_wide_kernel(int64_t N, int heads, int64_t C, const float* __restrict__ in,
                                                              int64_t ldi, float* __restrict__ out, int64_t ldo)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= N * C) return;
    const int64_t v = i / C, c = i % C;
    float s = 0.0f;
    for (int h = 0; h < heads; ++h) s += in[v * ldi + h * C + c];
    out[v * ldo + c] = s / (float)heads;
}
}  // namespace

extern "C" int retexo_head_mean(int64_t N, int heads, int64_t C, const float* d_in, int64_t ldi,
                                float* d_out, int64_t ldo, void* stream)
{
    if (N < 0 || C < 0 || N * C >= (1ll << 40)) return RETEXO_E_SIZE;
    if (heads < 1 || heads > kMaxHeads) return RETEXO_E_HEADS;
    if (ldi < heads * C || ldo < C) return RETEXO_E_LD;
    if (N == 0 || C == 0) return RETEXO_OK;
    if (!d_in || !d_out) return RETEXO_E_NULL;
    if (overlaps(d_in, extent_bytes(N, ldi, heads * C), d_out, extent_bytes(N, ldo, C))) return RETEXO_E_ALIAS;
    if (heads * C <= kHeadMeanMaxWidth) {
        const int W = (int)(heads * C);
        const bool vec = (uintptr_t)d_in % 16 == 0 && ldi % 4 == 0 && (W + 3) / 4 * 4 <= ldi;
        const int pitch = vec ? (W + 3) / 4 * 4 : W;
        const int rows_per_block = 4 * kHeadMeanMaxWidth / pitch;          // at least 4
        const unsigned grid = (unsigned)((N + rows_per_block - 1) / rows_per_block);
        if (vec) head_mean_kernel<true><<<dim3(grid), dim3(256), 0, (hipStream_t)stream>>>(
                     N, heads, (int)C, rows_per_block, d_in, ldi, d_out, ldo);
        else     head_mean_kernel<false><<<dim3(grid), dim3(256), 0, (hipStream_t)stream>>>(
                     N, heads, (int)C, rows_per_block, d_in, ldi, d_out, ldo);
    } else {
        head_mean_wide_kernel<<<dim3((unsigned)((N * C + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>(
            N, heads, C, d_in, ldi, d_out, ldo);
    }
    if (hipGetLastError() != hipSuccess) return RETEXO_E_HIP;
    return RETEXO_OK;
}

extern "C" int retexo_round(const retexo_plan* plan, int mode, int64_t D_in, int64_t D_out, int heads,
                            const float* d_H, int64_t ldh, const float* d_W, const float* d_b,
                            const float* d_attn_src, const float* d_attn_dst, float negative_slope,
                            unsigned flags, float* d_out, int64_t ldo,
                            void* d_workspace, int64_t workspace_bytes, void* stream)
{
    if (!plan) return RETEXO_E_NULL;
    if (D_in < 0 || D_in >= (1ll << 31) || D_out < 0 || D_out >= (1ll << 30)) return RETEXO_E_SIZE;
    if (int s = check_mode(mode, D_out, heads)) return s;
    if (flags & ~(unsigned)(RETEXO_F_RELU | RETEXO_F_SELF_CONCAT)) return RETEXO_E_FLAGS;
    const bool concat = (flags & RETEXO_F_SELF_CONCAT) != 0;
    const bool have_w = d_W != nullptr;
    const int64_t N = plan->N, ow = concat ? 2 * D_out : D_out;
    if (!have_w) {
        if (D_out != D_in) return RETEXO_E_SIZE;
        if (d_b) return RETEXO_E_FLAGS;
        if (flags & RETEXO_F_RELU) return RETEXO_E_FLAGS;
    }
    if (N > 0 && D_out > 0 && (!d_out || (D_in > 0 && !d_H))) return RETEXO_E_NULL;
    if (mode == RETEXO_GAT_SOFTMAX && N > 0 && D_out > 0 && (!d_attn_src || !d_attn_dst)) return RETEXO_E_NULL;
    if (ldh < D_in || ldo < ow) return RETEXO_E_LD;
    if (N > 0 && D_out > 0 && D_in > 0 &&
        overlaps(d_H, extent_bytes(N, ldh, D_in), d_out, extent_bytes(N, ldo, ow)))
        return RETEXO_E_ALIAS;

    int64_t ldz_ws = 0;
    const int64_t z_bytes = round_z_bytes(N, D_out, have_w, concat, &ldz_ws);
    const int64_t need = z_bytes + aggregate_workspace_bytes(N, mode, heads);
    if (need > 0 && (!d_workspace || workspace_bytes < need || ((uintptr_t)d_workspace & 255)))
        return RETEXO_E_WORKSPACE;
    if (need > 0 && N > 0 && D_out > 0 &&
        (overlaps(d_workspace, need, d_out, extent_bytes(N, ldo, ow)) ||
         (D_in > 0 && overlaps(d_workspace, need, d_H, extent_bytes(N, ldh, D_in)))))
        return RETEXO_E_ALIAS;

    hipStream_t s = (hipStream_t)stream;
    AggCall c;
    c.plan = plan; c.mode = mode; c.F = D_out; c.heads = heads;
    c.attn_src = d_attn_src; c.attn_dst = d_attn_dst; c.slope = negative_slope;
    c.self_concat = concat; c.out = d_out; c.ldo = ldo;
    c.workspace = (char*)d_workspace + z_bytes;
    if (!have_w) {
        // identity transform: the first round aggregates the raw features
        c.Z = d_H; c.ldz = ldh; c.copy_self = true;
    } else if (concat) {
        // Z is produced straight into out's first D_out columns and gathered from there
        if (int e = launch_transform(N, D_in, D_out, d_H, ldh, d_W, d_b, (flags & RETEXO_F_RELU) != 0,
                                     d_out, ldo, s))
            return e;
        c.Z = d_out; c.ldz = ldo; c.copy_self = false;
    } else {
        float* Zws = (float*)d_workspace;
        c.Z = Zws; c.ldz = ldz_ws; c.copy_self = false;
        c.z_padding_free = true;
        const int64_t agg_bytes = need - z_bytes;
        if (mode == RETEXO_GAT_SOFTMAX && N > 0 && D_out > 0 && D_in > 0 && !(flags & RETEXO_F_RELU) &&
            gat_fold_plan(c, D_in, agg_bytes)) {
            // the source scores leave the transform as heads_padded more columns of Z (the score tables' space
            // is free then and holds the widened operands)
            const int64_t wide = D_out + heads_padded(heads);
            float* W2 = (float*)c.workspace;
            float* b2 = W2 + D_in * wide;
            launch_gat_fold(D_in, D_out, heads, d_W, d_b, d_attn_src, W2, b2, s);
            if (int e = launch_transform(N, D_in, wide, d_H, ldh, W2, b2, false, Zws, ldz_ws, s)) return e;
            c.el_ready = true;
        } else if (int e = launch_transform(N, D_in, D_out, d_H, ldh, d_W, d_b, (flags & RETEXO_F_RELU) != 0,
                                            Zws, ldz_ws, s)) {
            return e;
        }
    }
    return launch_aggregate(c, s);
}
