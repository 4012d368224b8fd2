// Per-graph plan: degrees, GCN normalisers and the degree-ordered row schedule.
//
// deg[v] is the CSR row length.  dinv[v] = 1/sqrt(deg v) is what the
// symmetric normalisation D^-1/2 (A+I) D^-1/2 multiplies with on both sides; it
// is computed as a correctly rounded fp32 sqrt followed by a correctly rounded
// fp32 divide (never the hardware rsqrt approximation) so that it can be
// compared bit for bit with a CPU computation.
//
// Power-law graphs have a few very long rows.  The aggregation kernels give
// one wavefront to an ordinary row and a whole workgroup to a long one, and
// start the long rows first, so the plan keeps the row ids sorted by
// decreasing degree (stable: equal degrees stay in id order) and the number of
// rows at or above a few degree thresholds.
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>

#include <new>

#include "common.hpp"

namespace {

constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void degree_kernel(
    int64_t N, int64_t nnz, const int64_t* __restrict__ row_ptr, int32_t* __restrict__ deg,
    float* __restrict__ dinv, uint32_t* __restrict__ sort_key, int32_t* __restrict__ ids,
    uint32_t* bad)
{
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (v >= N) return;
    const int64_t lo = row_ptr[v], hi = row_ptr[v + 1];
    int64_t d = hi - lo;
    if (d < 0 || d > 0x7fffffff || (v == 0 && lo != 0) || (v == N - 1 && hi != nnz)) { atomicOr(bad, 1u); d = 0; }
    deg[v] = (int32_t)d;
    dinv[v] = d > 0 ? 1.0f / sqrtf((float)d) : 0.0f;
    sort_key[v] = (uint32_t)d;
    ids[v] = (int32_t)v;
}

__global__ __launch_bounds__(kThreads) void check_columns(
    int64_t nnz, int64_t N, const int32_t* __restrict__ col_idx, uint32_t* bad)
{
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e >= nnz) return;
    const int32_t c = col_idx[e];
    if (c < 0 || c >= N) atomicOr(bad, 1u);
}

// part_ptr[k][s] = first position in row order[s] whose column is >= k * span (columns ascend in a row).
// Sixteen lanes per row, four rows per wave: lane k finds its boundary by bisection over the row (a dozen
// dependent loads that mostly hit the row's few cache lines in L2; walking every column of every row instead
// kept the vector units busy for 0.25 ms on the Reddit-shaped graph).  A prefix maximum over the sixteen
// positions then makes them a monotone chain from row start to row end whatever the order of the columns, so
// every entry lies in exactly one range even for a caller's CSR with unsorted rows (there the cut points are
// arbitrary, which costs locality, not correctness).
__global__ __launch_bounds__(kThreads) void split_rows_kernel(
    int64_t N, int64_t nnz, int64_t span, const int64_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
    const int32_t* __restrict__ order, int32_t* __restrict__ part_ptr)
{
    static_assert(kMaxParts == 16, "one lane per boundary, four rows per wave");
    const int k = threadIdx.x & 15;
    const int64_t s = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 4;
    bool have = s < N;
    int64_t begin = 0, end = 0;
    if (have) {
        const int64_t v = order[s];
        begin = row_ptr[v];
        end = row_ptr[v + 1];
        // this runs before the host has seen the verdict on row_ptr: a row that does not lie inside
        // col_idx is left alone (such a CSR is rejected and the plan never used)
        if (begin < 0 || end > nnz || begin > end) { have = false; begin = end = 0; }
    }
    const int64_t target = (int64_t)k * span;
    int64_t lo = begin, hi = end;
    while (lo < hi) {
        const int64_t mid = lo + ((hi - lo) >> 1);
        if ((int64_t)col_idx[mid] < target) lo = mid + 1;
        else hi = mid;
    }
    int p = (int)lo;                           // the split exists only for graphs of fewer than 2^31 entries
#pragma unroll
    for (int d = 1; d < 16; d <<= 1) {
        const int o = __shfl_up(p, d, 16);
        if (k >= d) p = max(p, o);
    }
    if (have) {
        part_ptr[(int64_t)k * N + s] = p;
        if (k == 15) part_ptr[(int64_t)kMaxParts * N + s] = (int32_t)end;
    }
}

// counts[i] = number of rows with degree >= thresholds[i]; keys are sorted descending
struct Thresholds { int t[8]; };

__global__ void count_at_least(int64_t N, const uint32_t* __restrict__ keys_desc, Thresholds th,
                               int64_t* counts)
{
    const int i = threadIdx.x;
    if (i >= 8) return;
    const uint32_t t = (uint32_t)th.t[i];
    int64_t lo = 0, hi = N;                 // first index with key < t
    while (lo < hi) {
        const int64_t mid = lo + ((hi - lo) >> 1);
        if (keys_desc[mid] >= t) lo = mid + 1; else hi = mid;
    }
    counts[i] = lo;
    if (i == 0) counts[8] = N > 0 ? (int64_t)keys_desc[0] : 0;   // max degree
}

struct Readback {
    int64_t counts[9];
    int64_t nnz;
    uint32_t bad;
    uint32_t pad;
};

}  // namespace

namespace {

struct PlanLayout {
    bool split;
    int64_t o_deg, o_dinv, o_order, o_part, keep_bytes;            // what the plan keeps
    int64_t s_kin, s_kout, s_ids, s_rb, s_tmp, scratch_bytes;      // what only its construction needs
    size_t sort_bytes;
};

int plan_layout(int64_t N, int64_t nnz, unsigned flags, PlanLayout& L)
{
    const int64_t n1 = N > 0 ? N : 1;
    // Dense-enough graphs whose feature table cannot stay in L2 get the row split that lets
    // the aggregation walk one source-id range at a time.
    L.split = N > 0 && nnz > 0 &&
              ((flags & RETEXO_F_SPLIT_ROWS) ||
               (nnz >= 64 * N && N * 128 > (4ll << 20) && N * 128 <= kMaxParts * (8ll << 20)));
    L.o_deg = 0;
    L.o_dinv = align_up(4 * n1, 256);
    L.o_order = 2 * L.o_dinv;
    L.o_part = 3 * L.o_dinv;
    L.keep_bytes = L.o_part + (L.split ? align_up(4 * N * (kMaxParts + 1), 256) : 0);
    L.sort_bytes = 0;
    if (N > 0 &&
        rocprim::radix_sort_pairs_desc(nullptr, L.sort_bytes, (uint32_t*)nullptr, (uint32_t*)nullptr,
                                       (int32_t*)nullptr, (int32_t*)nullptr, (size_t)N, 0u, 32u,
                                       (hipStream_t)0) != hipSuccess)
        return RETEXO_E_HIP;
    // scratch: keys_in, keys_out, ids_in, readback block, sort temp
    L.s_kin = 0;
    L.s_kout = align_up(4 * n1, 256);
    L.s_ids = 2 * L.s_kout;
    L.s_rb = 3 * L.s_kout;
    L.s_tmp = L.s_rb + 256;
    L.scratch_bytes = L.s_tmp + align_up((int64_t)L.sort_bytes, 256) + 256;
    return RETEXO_OK;
}

// Everything after the sizes are known: the kernels, the one read-back, the host fields.  `keep` and `scratch`
// are device memory of L.keep_bytes and L.scratch_bytes.
int plan_fill(retexo_plan* p, const PlanLayout& L, unsigned flags, void* keep, void* scratch, hipStream_t stream)
{
    const int64_t N = p->N, nnz = p->nnz;
    p->deg = (int32_t*)((char*)keep + L.o_deg);
    p->dinv = (float*)((char*)keep + L.o_dinv);
    p->order = (int32_t*)((char*)keep + L.o_order);
    char* sc = (char*)scratch;
    uint32_t* kin = (uint32_t*)(sc + L.s_kin);
    uint32_t* kout = (uint32_t*)(sc + L.s_kout);
    int32_t* ids = (int32_t*)(sc + L.s_ids);
    Readback* rb = (Readback*)(sc + L.s_rb);

    RETEXO_HIP_TRY(hipMemsetAsync(rb, 0, sizeof(Readback), stream));
    if (N > 0) {
        degree_kernel<<<dim3((unsigned)((N + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream>>>(
            N, nnz, p->row_ptr, p->deg, p->dinv, kin, ids, &rb->bad);
        size_t sort_bytes = L.sort_bytes;
        RETEXO_HIP_TRY(rocprim::radix_sort_pairs_desc(sc + L.s_tmp, sort_bytes, kin, kout, ids, p->order, (size_t)N,
                                                      0u, 32u, stream));
        Thresholds th;
        for (int i = 0; i < 8; ++i) th.t[i] = kPlanThresholds[i];
        count_at_least<<<dim3(1), dim3(64), 0, stream>>>(N, kout, th, rb->counts);
    }
    if (L.split) {
        // needs only the schedule order, so it runs before the host looks at the counts
        p->part_ptr = (int32_t*)((char*)keep + L.o_part);
        p->part_span = (N + kMaxParts - 1) / kMaxParts;
        const int64_t rows_per_block = kThreads / 16;
        split_rows_kernel<<<dim3((unsigned)((N + rows_per_block - 1) / rows_per_block)), dim3(kThreads), 0, stream>>>(
            N, nnz, p->part_span, p->row_ptr, p->col_idx, p->order, p->part_ptr);
    }
    if ((flags & RETEXO_F_VALIDATE) && nnz > 0)
        check_columns<<<dim3((unsigned)((nnz + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream>>>(
            nnz, N, p->col_idx, &rb->bad);
    RETEXO_HIP_TRY(hipGetLastError());
    Readback h;
    RETEXO_HIP_TRY(hipMemcpyAsync(&h, rb, sizeof(h), hipMemcpyDeviceToHost, stream));
    RETEXO_HIP_TRY(hipStreamSynchronize(stream));
    if (h.bad) return RETEXO_E_CSR;
    for (int i = 0; i < 8; ++i) p->rows_at_least[i] = h.counts[i];
    p->max_degree = (int32_t)h.counts[8];
    return RETEXO_OK;
}

}  // namespace

extern "C" int retexo_plan_create(retexo_plan** out, int64_t N, const int64_t* d_row_ptr,
                                  const int32_t* d_col_idx, unsigned flags, void* stream_)
{
    if (!out) return RETEXO_E_NULL;
    *out = nullptr;
    if (N < 0 || N >= (1ll << 31)) return RETEXO_E_SIZE;
    if (flags & ~(unsigned)(RETEXO_F_VALIDATE | RETEXO_F_SPLIT_ROWS)) return RETEXO_E_FLAGS;
    if (!d_row_ptr) return RETEXO_E_NULL;
    hipStream_t stream = (hipStream_t)stream_;

    retexo_plan* p = new (std::nothrow) retexo_plan();
    if (!p) return RETEXO_E_HIP;
    p->N = N;
    p->row_ptr = d_row_ptr;
    p->col_idx = d_col_idx;
    auto fail = [&](int code) { retexo_plan_destroy(p); return code; };

    // The entry count decides whether the row split is built, so it is fetched first; everything the plan
    // keeps then comes from one allocation (device allocations cost tens of microseconds each).
    int64_t nnz = 0;
    if (hipMemcpyAsync(&nnz, d_row_ptr + N, sizeof(int64_t), hipMemcpyDeviceToHost, stream) != hipSuccess)
        return fail(RETEXO_E_HIP);
    if (hipStreamSynchronize(stream) != hipSuccess) return fail(RETEXO_E_HIP);
    if (nnz < 0) return fail(RETEXO_E_CSR);
    if (nnz >= (1ll << 31)) return fail(RETEXO_E_SIZE);
    if (nnz > 0 && !d_col_idx) return fail(RETEXO_E_NULL);
    p->nnz = nnz;
    PlanLayout L;
    if (int e = plan_layout(N, nnz, flags, L)) return fail(e);
    if (hipMalloc(&p->block, (size_t)L.keep_bytes) != hipSuccess) return fail(RETEXO_E_HIP);
    if (hipMalloc(&p->build_scratch, (size_t)L.scratch_bytes) != hipSuccess) return fail(RETEXO_E_HIP);
    if (int e = plan_fill(p, L, flags, p->block, p->build_scratch, stream)) return fail(e);
    (void)hipFree(p->build_scratch);
    p->build_scratch = nullptr;
    *out = p;
    return RETEXO_OK;
}

extern "C" int64_t retexo_plan_workspace_bytes(int64_t N, int64_t nnz, unsigned flags)
{
    if (N < 0 || N >= (1ll << 31) || nnz < 0 || nnz >= (1ll << 31)) return RETEXO_E_SIZE;
    if (flags & ~(unsigned)(RETEXO_F_VALIDATE | RETEXO_F_SPLIT_ROWS)) return RETEXO_E_FLAGS;
    PlanLayout L;
    if (int e = plan_layout(N, nnz, flags, L)) return e;
    return L.keep_bytes + L.scratch_bytes;
}

extern "C" int retexo_plan_create_in(retexo_plan** out, int64_t N, int64_t nnz, const int64_t* d_row_ptr,
                                     const int32_t* d_col_idx, unsigned flags,
                                     void* d_workspace, int64_t workspace_bytes, void* stream_)
{
    if (!out) return RETEXO_E_NULL;
    *out = nullptr;
    if (N < 0 || N >= (1ll << 31) || nnz < 0 || nnz >= (1ll << 31)) return RETEXO_E_SIZE;
    if (flags & ~(unsigned)(RETEXO_F_VALIDATE | RETEXO_F_SPLIT_ROWS)) return RETEXO_E_FLAGS;
    if (!d_row_ptr || (nnz > 0 && !d_col_idx)) return RETEXO_E_NULL;
    PlanLayout L;
    if (int e = plan_layout(N, nnz, flags, L)) return e;
    if (!d_workspace || ((uintptr_t)d_workspace & 255) != 0 || workspace_bytes < L.keep_bytes + L.scratch_bytes)
        return RETEXO_E_WORKSPACE;
    retexo_plan* p = new (std::nothrow) retexo_plan();
    if (!p) return RETEXO_E_HIP;
    p->N = N;
    p->nnz = nnz;
    p->row_ptr = d_row_ptr;
    p->col_idx = d_col_idx;
    // the plan's arrays live in the caller's workspace: nothing to free but the host structure
    if (int e = plan_fill(p, L, flags, d_workspace, (char*)d_workspace + L.keep_bytes, (hipStream_t)stream_)) {
        delete p;
        return e;
    }
    *out = p;
    return RETEXO_OK;
}

extern "C" int retexo_plan_destroy(retexo_plan* p)
{
    if (!p) return RETEXO_OK;
    if (p->block) (void)hipFree(p->block);       // deg, dinv, order and part_ptr live in it
    if (p->build_scratch) (void)hipFree(p->build_scratch);
    delete p;
    return RETEXO_OK;
}

extern "C" int64_t retexo_plan_num_nodes(const retexo_plan* p) { return p ? p->N : RETEXO_E_NULL; }
extern "C" int64_t retexo_plan_nnz(const retexo_plan* p) { return p ? p->nnz : RETEXO_E_NULL; }
extern "C" int32_t retexo_plan_max_degree(const retexo_plan* p) { return p ? p->max_degree : RETEXO_E_NULL; }
extern "C" const int32_t* retexo_plan_deg(const retexo_plan* p) { return p ? p->deg : nullptr; }
extern "C" const float* retexo_plan_dinv(const retexo_plan* p) { return p ? p->dinv : nullptr; }

namespace {
// dst[i] = src[i] for i < n words; the exports are kernels (not copy nodes) so that a caller may record them
// into a HIP graph like every other stream-ordered entry point
__global__ __launch_bounds__(kThreads) void copy_words_kernel(int64_t n, const uint32_t* __restrict__ src,
                                                              uint32_t* __restrict__ dst)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

int copy_words(int64_t n, const void* src, void* dst, hipStream_t stream)
{
    if (n <= 0) return RETEXO_OK;
    copy_words_kernel<<<dim3((unsigned)((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream>>>(
        n, (const uint32_t*)src, (uint32_t*)dst);
    return hipGetLastError() == hipSuccess ? RETEXO_OK : RETEXO_E_HIP;
}
}  // namespace

extern "C" int retexo_plan_export(const retexo_plan* p, int32_t* d_deg, float* d_dinv, int32_t* d_order,
                                  void* stream_)
{
    if (!p) return RETEXO_E_NULL;
    hipStream_t stream = (hipStream_t)stream_;
    const int64_t n = p->N;
    if (n == 0) return RETEXO_OK;
    if (d_deg) if (int e = copy_words(n, p->deg, d_deg, stream)) return e;
    if (d_dinv) if (int e = copy_words(n, p->dinv, d_dinv, stream)) return e;
    if (d_order) if (int e = copy_words(n, p->order, d_order, stream)) return e;
    return RETEXO_OK;
}

static_assert(kMaxParts == RETEXO_SPLIT_PARTS, "the header states the number of source-id ranges");

extern "C" int64_t retexo_plan_export_split(const retexo_plan* p, int32_t* d_pos, void* stream_)
{
    if (!p) return RETEXO_E_NULL;
    if (!p->part_ptr) return 0;
    if (d_pos)
        if (int e = copy_words(p->N * (kMaxParts + 1), p->part_ptr, d_pos, (hipStream_t)stream_)) return e;
    return p->part_span;
}
