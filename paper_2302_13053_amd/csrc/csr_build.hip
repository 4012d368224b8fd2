// CSR construction on the device from raw undirected pairs.
//
// The paper's graphs are undirected (section "Edge-partitioned Distributed
// Setup"), so each pair {u,v} becomes the two directed entries (u,v), (v,u).
// Construction is integer-only and its result is a unique function of the pair
// set: rows in id order, columns strictly ascending, no repeats, no (v,v)
// entries except the single one per node requested by add_self_loops.
//
// Method: every directed entry is packed into one 64-bit key
// (row << cbits | col, cbits = bits needed for N-1), the keys are radix-sorted
// (rocPRIM device sort over only the significant bits), an exclusive scan over
// "first key of a run of equal keys" flags (computed on the fly from the sorted
// keys) gives each kept entry its position in col_idx, and row_ptr[r] is the scan value at the first
// key whose row is >= r (binary search).  A pair with u == v becomes the key
// (u, u), which is exactly the self-loop entry: it is kept (once) when
// self-loops are requested and never flagged otherwise, so no sentinel value
// and no extra key bit is needed: the sort covers exactly 2*cbits bits.
#include <cstring>
#include <iterator>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_scan.hpp>
#include <rocprim/iterator/counting_iterator.hpp>
#include <rocprim/iterator/transform_iterator.hpp>

#include "common.hpp"
#include "csr_bucket.hpp"

namespace {

struct CsrHeader {          // lives at the start of the workspace
    uint32_t bad_id;        // set to 1 if any id is outside [0, N)
    uint32_t pad;
    int64_t nnz;
};

constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void pairs_to_keys(
    int64_t n_pairs, const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
    int64_t N, int add_self_loops, int cbits, uint64_t* __restrict__ keys, CsrHeader* hdr)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n_pairs) {
        const int32_t u = src[i], v = dst[i];
        uint64_t k0 = 0, k1 = 0;
        if (u < 0 || u >= N || v < 0 || v >= N) {
            atomicOr(&hdr->bad_id, 1u);
        } else {
            k0 = ((uint64_t)u << cbits) | (uint64_t)v;
            k1 = ((uint64_t)v << cbits) | (uint64_t)u;
        }
        keys[2 * i] = k0;
        keys[2 * i + 1] = k1;
    } else if (add_self_loops && i < n_pairs + N) {
        const uint64_t v = (uint64_t)(i - n_pairs);
        keys[2 * n_pairs + (i - n_pairs)] = (v << cbits) | v;
    }
}

// 1 for the first key of every run of equal keys, except diagonal keys when no self-loops are wanted
struct FirstOfRun {
    const uint64_t* keys;
    int cbits;
    int keep_diagonal;
    __device__ uint32_t operator()(int64_t i) const
    {
        const uint64_t k = keys[i];
        const bool diagonal = (k >> cbits) == (k & ((1ull << cbits) - 1));
        return ((keep_diagonal || !diagonal) && (i == 0 || keys[i - 1] != k)) ? 1u : 0u;
    }
};

__global__ void total_kept(int64_t M, FirstOfRun flag, const uint32_t* __restrict__ pos, CsrHeader* hdr)
{
    if (threadIdx.x == 0 && blockIdx.x == 0)
        hdr->nnz = (M == 0) ? 0 : (int64_t)pos[M - 1] + (int64_t)flag(M - 1);
}

__global__ __launch_bounds__(kThreads) void scatter_columns(
    int64_t M, FirstOfRun flag, const uint32_t* __restrict__ pos, int32_t* __restrict__ col_idx)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= M || !flag(i)) return;
    col_idx[pos[i]] = (int32_t)(flag.keys[i] & ((1ull << flag.cbits) - 1));
}

__global__ __launch_bounds__(kThreads) void row_offsets(
    int64_t N, int64_t M, const uint64_t* __restrict__ keys, const uint32_t* __restrict__ pos,
    int cbits, const CsrHeader* hdr, int64_t* __restrict__ row_ptr)
{
    const int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (r > N) return;
    const uint64_t want = (uint64_t)r << cbits;   // smallest possible key of row r
    int64_t lo = 0, hi = M;                       // first index with keys[idx] >= want
    while (lo < hi) {
        const int64_t mid = lo + ((hi - lo) >> 1);
        if (keys[mid] < want) lo = mid + 1; else hi = mid;
    }
    row_ptr[r] = (lo < M) ? (int64_t)pos[lo] : hdr->nnz;
}

// ---------------------------------------------------------------------------
// One-pass finish (used when col_idx can hold every key, so nothing can overflow): the exclusive scan
// writes through an iterator whose assignment is the rest of the construction.  For key i with scan
// value pos: a kept key stores its column at col_idx[pos]; the first key of a row stores pos as that
// row's offset; the last key stores the total.  Rows without keys are filled in afterwards.
// Nothing is written when an id was out of range.
// ---------------------------------------------------------------------------
struct EmitCtx {
    const uint64_t* keys;
    int cbits;
    int keep_diagonal;
    int64_t M;
    int32_t* col_idx;
    int64_t* row_ptr;
    CsrHeader* hdr;
};

struct EmitProxy {
    EmitCtx c;
    int64_t i;
    __device__ const EmitProxy& operator=(uint32_t pos) const
    {
        if (c.hdr->bad_id) return *this;
        const uint64_t mask = (1ull << c.cbits) - 1;
        const uint64_t k = c.keys[i];
        const bool first = i == 0;
        const uint64_t prev = first ? 0 : c.keys[i - 1];
        const uint64_t row = k >> c.cbits, col = k & mask;
        const bool kept = (c.keep_diagonal || row != col) && (first || prev != k);
        if (kept) c.col_idx[pos] = (int32_t)col;
        if (first || (prev >> c.cbits) != row) c.row_ptr[row] = (int64_t)pos;
        if (i == c.M - 1) c.hdr->nnz = (int64_t)pos + (kept ? 1 : 0);
        return *this;
    }
};

class EmitIterator {
public:
    using iterator_category = std::random_access_iterator_tag;
    using value_type = uint32_t;
    using difference_type = std::ptrdiff_t;
    using pointer = void;
    using reference = EmitProxy;

    __host__ __device__ EmitIterator(const EmitCtx& c, int64_t i = 0) : c_(c), i_(i) {}
    __host__ __device__ EmitProxy operator*() const { return EmitProxy{c_, i_}; }
    __host__ __device__ EmitProxy operator[](difference_type d) const { return EmitProxy{c_, i_ + d}; }
    __host__ __device__ EmitIterator operator+(difference_type d) const { return EmitIterator(c_, i_ + d); }
    __host__ __device__ EmitIterator operator-(difference_type d) const { return EmitIterator(c_, i_ - d); }
    __host__ __device__ difference_type operator-(const EmitIterator& o) const { return i_ - o.i_; }
    __host__ __device__ EmitIterator& operator+=(difference_type d) { i_ += d; return *this; }
    __host__ __device__ EmitIterator& operator-=(difference_type d) { i_ -= d; return *this; }
    __host__ __device__ EmitIterator& operator++() { ++i_; return *this; }
    __host__ __device__ EmitIterator operator++(int) { EmitIterator t = *this; ++i_; return t; }
    __host__ __device__ bool operator==(const EmitIterator& o) const { return i_ == o.i_; }
    __host__ __device__ bool operator!=(const EmitIterator& o) const { return i_ != o.i_; }
    __host__ __device__ bool operator<(const EmitIterator& o) const { return i_ < o.i_; }

private:
    EmitCtx c_;
    int64_t i_;
};

// every row offset starts as "not set"
__global__ __launch_bounds__(kThreads) void unset_rows(int64_t N, const CsrHeader* hdr, int64_t* __restrict__ row_ptr)
{
    const int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (r > N || hdr->bad_id) return;
    row_ptr[r] = -1;
}

// rows without keys take the offset of the next row that has some (or nnz); row_ptr[N] = nnz
__global__ __launch_bounds__(kThreads) void fill_rows(int64_t N, int64_t M, const uint64_t* __restrict__ keys, int cbits,
                                                      const CsrHeader* hdr, int64_t* row_ptr)
{
    const int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (r > N || hdr->bad_id) return;
    if (r == N) { row_ptr[N] = hdr->nnz; return; }
    if (row_ptr[r] != -1) return;
    const uint64_t want = (uint64_t)r << cbits;
    int64_t lo = 0, hi = M;                       // first index with keys[idx] >= want: a later row's first key
    while (lo < hi) {
        const int64_t mid = lo + ((hi - lo) >> 1);
        if (keys[mid] < want) lo = mid + 1; else hi = mid;
    }
    // that row has keys, so its offset was set by the scan and is not touched here
    row_ptr[r] = lo < M ? row_ptr[(int64_t)(keys[lo] >> cbits)] : hdr->nnz;
}

int column_bits(int64_t N)
{
    int b = 1;
    while ((1ll << b) < N) ++b;
    return b;
}

struct Layout {
    int64_t M, header, keys_a, keys_b, sort_tmp, scan_tmp, total;
    size_t sort_bytes, scan_bytes;
};

int make_layout(int64_t n_pairs, int64_t N, int add_self_loops, Layout& L)
{
    L.M = 2 * n_pairs + (add_self_loops ? N : 0);
    const int cbits = column_bits(N);
    size_t sb = 0, cb = 0;
    if (L.M > 0) {
        if (rocprim::radix_sort_keys(nullptr, sb, (uint64_t*)nullptr, (uint64_t*)nullptr, (size_t)L.M, 0u,
                                     (unsigned)(2 * cbits), (hipStream_t)0) != hipSuccess)
            return RETEXO_E_HIP;
        auto flags_it = rocprim::make_transform_iterator(rocprim::make_counting_iterator<int64_t>(0),
                                                         FirstOfRun{nullptr, cbits, 0});
        if (rocprim::exclusive_scan(nullptr, cb, flags_it, (uint32_t*)nullptr, 0u, (size_t)L.M,
                                    rocprim::plus<uint32_t>(), (hipStream_t)0) != hipSuccess)
            return RETEXO_E_HIP;
    }
    L.sort_bytes = sb;
    L.scan_bytes = cb;
    int64_t off = 0;
    L.header = off;   off += 256;
    L.keys_a = off;   off += align_up(8 * L.M, 256);
    L.keys_b = off;   off += align_up(8 * L.M, 256);
    L.sort_tmp = off; off += align_up((int64_t)sb, 256);
    L.scan_tmp = off; off += align_up((int64_t)cb, 256);
    L.total = off + 256;
    return RETEXO_OK;
}

int check_sizes(int64_t n_pairs, int64_t N)
{
    if (n_pairs < 0 || N < 0) return RETEXO_E_SIZE;
    if (N >= (1ll << 31) || 2 * n_pairs + N >= (1ll << 31)) return RETEXO_E_SIZE;
    return RETEXO_OK;
}

}  // namespace

extern "C" int64_t retexo_csr_workspace_bytes(int64_t n_pairs, int64_t N, int add_self_loops)
{
    if (int s = check_sizes(n_pairs, N)) return s;
    Layout L;
    if (int s = make_layout(n_pairs, N, add_self_loops, L)) return s;
    // enough for either construction (which one runs depends on the size and on the "csr_sorted_keys" knob)
    const int64_t bucketed = csr_bucketed_workspace_bytes(n_pairs, N, add_self_loops);
    return bucketed > L.total ? bucketed : L.total;
}

extern "C" int retexo_csr_from_coo(int64_t n_pairs, const int32_t* d_src, const int32_t* d_dst,
                                   int64_t N, int add_self_loops,
                                   int64_t* d_row_ptr, int32_t* d_col_idx, int64_t col_capacity,
                                   int64_t* h_nnz, void* d_workspace, int64_t workspace_bytes,
                                   void* stream_)
{
    if (int s = check_sizes(n_pairs, N)) return s;
    if (col_capacity < 0) return RETEXO_E_SIZE;
    if (!d_row_ptr) return RETEXO_E_NULL;
    if (n_pairs > 0 && (!d_src || !d_dst)) return RETEXO_E_NULL;
    if (!d_workspace) return RETEXO_E_WORKSPACE;
    if (((uintptr_t)d_workspace & 255) != 0) return RETEXO_E_WORKSPACE;
    Layout L;
    if (int s = make_layout(n_pairs, N, add_self_loops, L)) return s;
    if (workspace_bytes < L.total) return RETEXO_E_WORKSPACE;
    if (L.M > 0 && !d_col_idx && col_capacity > 0) return RETEXO_E_NULL;

    hipStream_t stream = (hipStream_t)stream_;
    // Graphs of up to 2^23 nodes take the bucketing construction (csr_bucket.hip); larger ones, and every graph
    // when the "csr_sorted_keys" knob is set, the sorted-key construction below.  Same result, bit for bit.
    const int64_t bucketed = agg_options().csr_sorted_keys ? -1 : csr_bucketed_workspace_bytes(n_pairs, N, add_self_loops);
    if (bucketed >= 0) {
        if (workspace_bytes < bucketed) return RETEXO_E_WORKSPACE;
        return csr_build_bucketed(n_pairs, d_src, d_dst, N, add_self_loops, d_row_ptr, d_col_idx, col_capacity,
                                  h_nnz, d_workspace, stream);
    }
    char* ws = (char*)d_workspace;
    CsrHeader* hdr = (CsrHeader*)(ws + L.header);
    uint64_t* keys_a = (uint64_t*)(ws + L.keys_a);
    uint64_t* keys_b = (uint64_t*)(ws + L.keys_b);
    // after the sort keys_a is free and holds the scan of the first-of-run flags
    uint32_t* pos = (uint32_t*)keys_a;
    const int cbits = column_bits(N);
    const int64_t M = L.M;

    const FirstOfRun flag{keys_b, cbits, add_self_loops ? 1 : 0};
    // col_idx can hold every key: no count is needed before the columns are written
    const bool one_pass = M > 0 && col_capacity >= M;
    RETEXO_HIP_TRY(hipMemsetAsync(hdr, 0, sizeof(CsrHeader), stream));
    if (M > 0) {
        const int64_t work = n_pairs + (add_self_loops ? N : 0);
        pairs_to_keys<<<dim3((unsigned)((work + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream>>>(
            n_pairs, d_src, d_dst, N, add_self_loops, cbits, keys_a, hdr);
        size_t sb = L.sort_bytes;
        RETEXO_HIP_TRY(rocprim::radix_sort_keys(ws + L.sort_tmp, sb, keys_a, keys_b, (size_t)M, 0u,
                                                (unsigned)(2 * cbits), stream));
        size_t cb = L.scan_bytes;
        auto flags_it = rocprim::make_transform_iterator(rocprim::make_counting_iterator<int64_t>(0), flag);
        if (one_pass) {
            const unsigned gr = (unsigned)((N + 1 + kThreads - 1) / kThreads);
            unset_rows<<<dim3(gr), dim3(kThreads), 0, stream>>>(N, hdr, d_row_ptr);
            const EmitCtx ctx{keys_b, cbits, add_self_loops ? 1 : 0, M, d_col_idx, d_row_ptr, hdr};
            RETEXO_HIP_TRY(rocprim::exclusive_scan(ws + L.scan_tmp, cb, flags_it, EmitIterator(ctx), 0u, (size_t)M,
                                                   rocprim::plus<uint32_t>(), stream));
            fill_rows<<<dim3(gr), dim3(kThreads), 0, stream>>>(N, M, keys_b, cbits, hdr, d_row_ptr);
        } else {
            RETEXO_HIP_TRY(rocprim::exclusive_scan(ws + L.scan_tmp, cb, flags_it, pos, 0u, (size_t)M,
                                                   rocprim::plus<uint32_t>(), stream));
            total_kept<<<dim3(1), dim3(64), 0, stream>>>(M, flag, pos, hdr);
        }
    }
    RETEXO_HIP_TRY(hipGetLastError());
    CsrHeader h;
    RETEXO_HIP_TRY(hipMemcpyAsync(&h, hdr, sizeof(h), hipMemcpyDeviceToHost, stream));
    RETEXO_HIP_TRY(hipStreamSynchronize(stream));
    if (h.bad_id) return RETEXO_E_CSR;
    if (h_nnz) *h_nnz = h.nnz;
    if (one_pass) return RETEXO_OK;                 // everything is written, and the stream is idle
    if (h.nnz > col_capacity) return RETEXO_E_CAPACITY;

    if (M > 0) {
        const unsigned gm = (unsigned)((M + kThreads - 1) / kThreads);
        scatter_columns<<<dim3(gm), dim3(kThreads), 0, stream>>>(M, flag, pos, d_col_idx);
    }
    row_offsets<<<dim3((unsigned)((N + 1 + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream>>>(
        N, M, keys_b, pos, cbits, hdr, d_row_ptr);
    RETEXO_HIP_TRY(hipGetLastError());
    RETEXO_HIP_TRY(hipStreamSynchronize(stream));   // the workspace may be reused by the caller
    return RETEXO_OK;
}
