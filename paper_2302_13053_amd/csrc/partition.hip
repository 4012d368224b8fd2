// One worker's share of an edge-partitioned graph, and the pack / unpack of
// boundary rows around a message-passing round.
//
// Section "Edge-partitioned Distributed Setup": worker i holds its inner nodes
// V_i, the edges that touch an inner node and, as boundary nodes, the other
// endpoints of those edges; before a round it receives the boundary nodes'
// current representations from their owners (the embedding exchange of the
// implementation section).  Given the global CSR and a node -> worker map this
// file derives, on the device and with integer arithmetic only:
//
//   local numbering   [ inner nodes, ascending global id | boundary nodes, ascending global id ]
//   local CSR         an inner node's row = its global row renumbered, columns ascending;
//                     a boundary node's row is empty
//   global degrees    of all local nodes (gcn_sym normalises a boundary node by its true degree)
//   send / receive    per peer q: the inner nodes q needs / the boundary nodes q owns, as local
//   lists             ids ascending in global id, so that the list one worker packs and the list
//                     its peer unpacks line up element by element
//
// Both halves of the numbering are monotone in the global id, so a renumbered
// row is its inner entries (ascending) followed by its boundary entries
// (ascending): a stable two-way split inside each row, no per-row sort.
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_reduce.hpp>
#include <rocprim/device/device_scan.hpp>
#include <rocprim/iterator/counting_iterator.hpp>
#include <rocprim/iterator/transform_iterator.hpp>

#include "common.hpp"

namespace {

constexpr int kThreads = 256;
constexpr int kMaxWorkers = 64;       // one bit per worker in a 64-bit mask

struct ShareHeader {                  // start of the workspace; copied to the host
    uint32_t bad_part;                // a partition id outside [0, n_parts)
    uint32_t pad;
    int64_t n_inner, n_halo, nnz_local, n_send;
    int64_t send_off[kMaxWorkers + 1];
    int64_t recv_off[kMaxWorkers + 1];
};

__device__ __forceinline__ uint64_t wave_or(uint64_t x)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)x, m, 64), hi = __shfl_xor((uint32_t)(x >> 32), m, 64);
        x |= ((uint64_t)hi << 32) | lo;
    }
    return x;
}

// one wave per global row: an inner row marks the foreign endpoints of its entries as boundary
// nodes and collects the set of workers it touches
__global__ __launch_bounds__(kThreads) void mark_kernel(
    int64_t N, const int64_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
    const int32_t* __restrict__ part, int n_parts, int p, uint32_t* __restrict__ halo_flag,
    uint64_t* __restrict__ mask, ShareHeader* hdr)
{
    const int lane = threadIdx.x & 63;
    const int64_t v = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (v >= N) return;
    const int pv = part[v];
    if (pv < 0 || pv >= n_parts) {
        if (lane == 0) atomicOr(&hdr->bad_part, 1u);
        if (lane == 0) mask[v] = 0;
        return;
    }
    uint64_t m = 0;
    if (pv == p) {
        const int64_t lo = row_ptr[v], hi = row_ptr[v + 1];
        for (int64_t e = lo + lane; e < hi; e += 64) {
            const int32_t u = col_idx[e];
            const int q = part[u];
            if (q < 0 || q >= n_parts) continue;          // reported by u's own wave
            if (q != p) {
                halo_flag[u] = 1u;                        // every writer stores the same value
                m |= 1ull << q;
            }
        }
        m = wave_or(m);
    }
    if (lane == 0) mask[v] = m;
}

struct IsInner {
    const int32_t* part;
    int p;
    __device__ uint32_t operator()(int64_t v) const { return part[v] == p ? 1u : 0u; }
};
struct InnerRowLength {
    const int32_t* part;
    const int64_t* row_ptr;
    int p;
    __device__ int64_t operator()(int64_t v) const { return part[v] == p ? row_ptr[v + 1] - row_ptr[v] : 0; }
};
struct PeerCount {
    const uint64_t* mask;
    __device__ uint32_t operator()(int64_t v) const { return (uint32_t)__popcll(mask[v]); }
};
struct LocalRowLength {               // row length of local node i (0 for boundary nodes and for i == n_local)
    const int32_t* local_ids;
    const int64_t* row_ptr;
    int64_t n_inner;
    __device__ int64_t operator()(int64_t i) const
    {
        if (i >= n_inner) return 0;
        const int64_t v = local_ids[i];
        return row_ptr[v + 1] - row_ptr[v];
    }
};

// totals of the three exclusive scans (last scan value + last element), N >= 1
__global__ void totals_kernel(int64_t N, const int32_t* __restrict__ part, int p,
                              const uint32_t* __restrict__ rank_in, const uint32_t* __restrict__ halo_flag,
                              const uint32_t* __restrict__ rank_halo, const uint32_t* __restrict__ key_off,
                              const uint64_t* __restrict__ mask, ShareHeader* hdr)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    hdr->n_inner = (int64_t)rank_in[N - 1] + (part[N - 1] == p ? 1 : 0);
    hdr->n_halo = (int64_t)rank_halo[N - 1] + (int64_t)halo_flag[N - 1];
    hdr->n_send = (int64_t)key_off[N - 1] + __popcll(mask[N - 1]);
}

// local numbering, global ids and degrees of the local nodes, and (for inner nodes) the offset
// of their (peer, node) keys
__global__ __launch_bounds__(kThreads) void number_kernel(
    int64_t N, const int64_t* __restrict__ row_ptr, const int32_t* __restrict__ part, int p,
    const uint32_t* __restrict__ rank_in, const uint32_t* __restrict__ halo_flag,
    const uint32_t* __restrict__ rank_halo, int64_t n_inner, int32_t* __restrict__ to_local,
    int32_t* __restrict__ local_ids, int32_t* __restrict__ global_deg)
{
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (v >= N) return;
    int64_t l = -1;
    if (part[v] == p) l = rank_in[v];
    else if (halo_flag[v]) l = n_inner + rank_halo[v];
    to_local[v] = (int32_t)l;
    if (l >= 0) {
        local_ids[l] = (int32_t)v;
        global_deg[l] = (int32_t)(row_ptr[v + 1] - row_ptr[v]);
    }
}

// one wave per inner local row: renumber the global row; inner entries first, then boundary
// entries, each group in its original (ascending) order
__global__ __launch_bounds__(kThreads) void columns_kernel(
    int64_t n_inner, const int32_t* __restrict__ local_ids, const int64_t* __restrict__ row_ptr,
    const int32_t* __restrict__ col_idx, const int32_t* __restrict__ to_local,
    const int64_t* __restrict__ local_row_ptr, int32_t* __restrict__ local_col)
{
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (i >= n_inner) return;
    const int64_t v = local_ids[i];
    const int64_t lo = row_ptr[v], hi = row_ptr[v + 1], base = local_row_ptr[i];
    const uint64_t below = (1ull << lane) - 1;
    int64_t inner_total = 0;
    for (int64_t e0 = lo; e0 < hi; e0 += 64) {
        const int64_t e = e0 + lane;
        const bool in = e < hi && to_local[col_idx[e]] < n_inner;
        inner_total += __popcll(__ballot(in));
    }
    int64_t done_in = 0, done_out = 0;
    for (int64_t e0 = lo; e0 < hi; e0 += 64) {
        const int64_t e = e0 + lane;
        const bool valid = e < hi;
        const int32_t l = valid ? to_local[col_idx[e]] : 0;
        const bool in = valid && l < n_inner;
        const bool out = valid && !in;
        const uint64_t bin = __ballot(in), bout = __ballot(out);
        if (in) local_col[base + done_in + __popcll(bin & below)] = l;
        if (out) local_col[base + inner_total + done_out + __popcll(bout & below)] = l;
        done_in += __popcll(bin);
        done_out += __popcll(bout);
    }
}

// keys (kind, peer, local id): kind 0 = send (one key per (inner node, peer it touches)),
// kind 1 = receive (one key per boundary node, peer = its owner)
__global__ __launch_bounds__(kThreads) void keys_kernel(
    int64_t n_inner, int64_t n_halo, const int32_t* __restrict__ local_ids,
    const int32_t* __restrict__ part, const uint64_t* __restrict__ mask,
    const uint32_t* __restrict__ key_off, int64_t n_send, uint64_t* __restrict__ keys)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n_inner) {
        const int64_t v = local_ids[i];
        uint64_t m = mask[v];
        int64_t k = key_off[v];
        while (m) {
            const int q = __ffsll((unsigned long long)m) - 1;
            m &= m - 1;
            keys[k++] = ((uint64_t)q << 32) | (uint64_t)i;
        }
    } else if (i < n_inner + n_halo) {
        const int q = part[local_ids[i]];
        keys[n_send + (i - n_inner)] = (1ull << 40) | ((uint64_t)q << 32) | (uint64_t)i;
    }
}

__global__ __launch_bounds__(kThreads) void lists_kernel(
    int64_t n_send, int64_t n_halo, const uint64_t* __restrict__ keys, int n_parts,
    int32_t* __restrict__ send_ids, int32_t* __restrict__ recv_ids, ShareHeader* hdr)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n_send) send_ids[i] = (int32_t)(keys[i] & 0xffffffffu);
    else if (i < n_send + n_halo) recv_ids[i - n_send] = (int32_t)(keys[i] & 0xffffffffu);
    // offsets: first key of each (kind, peer) group, by binary search
    if (i <= 2 * (int64_t)n_parts + 1) {
        const int kind = i > n_parts ? 1 : 0;
        const int q = (int)(kind ? i - n_parts - 1 : i);
        const uint64_t want = ((uint64_t)kind << 40) | ((uint64_t)q << 32);
        int64_t lo = 0, hi = n_send + n_halo;
        while (lo < hi) {
            const int64_t mid = (lo + hi) / 2;
            if (keys[mid] < want) lo = mid + 1; else hi = mid;
        }
        if (kind) hdr->recv_off[q] = lo - n_send;
        else hdr->send_off[q] = lo;
    }
}

// rows of a table <-> a dense buffer; one thread per VEC floats
template <int VEC, bool SCATTER>
__global__ __launch_bounds__(kThreads) void rows_kernel(
    int64_t n, const int32_t* __restrict__ ids, int64_t table_rows, int64_t F,
    const float* __restrict__ src, int64_t lds, float* __restrict__ dst, int64_t ldd)
{
    const int64_t chunks = (F + VEC - 1) / VEC;
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (t >= n * chunks) return;
    const int64_t i = t / chunks, c = (t % chunks) * VEC;
    const int64_t r = ids[i];
    if (r < 0 || r >= table_rows) return;                 // ids outside the table are ignored
    const float* s = SCATTER ? src + i * lds + c : src + r * lds + c;
    float* d = SCATTER ? dst + r * ldd + c : dst + i * ldd + c;
    if constexpr (VEC == 4) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        if (c + 4 <= F) {
            *reinterpret_cast<f4*>(d) = *reinterpret_cast<const f4*>(s);
        } else {                                          // ragged last vector of a row
            for (int k = 0; k < (int)(F - c); ++k) d[k] = s[k];
        }
    } else {
        *d = *s;
    }
}

__global__ __launch_bounds__(kThreads) void set_degrees_kernel(int64_t N, const int32_t* __restrict__ d_in,
                                                               int32_t* __restrict__ deg, float* __restrict__ dinv)
{
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (v >= N) return;
    const int32_t d = d_in[v];
    deg[v] = d;
    dinv[v] = d > 0 ? 1.0f / sqrtf((float)d) : 0.0f;
}

struct Layout {
    int64_t header, mask, halo_flag, rank_in, rank_halo, key_off, to_local, keys_a, keys_b, tmp, total;
    size_t tmp_bytes;
};

int make_layout(int64_t N, int64_t send_capacity, Layout& L)
{
    const int64_t n = N > 0 ? N : 1, K = send_capacity + n;
    size_t a = 0, b = 0, c = 0, d = 0;
    auto it32 = rocprim::make_transform_iterator(rocprim::make_counting_iterator<int64_t>(0), IsInner{nullptr, 0});
    auto it64 = rocprim::make_transform_iterator(rocprim::make_counting_iterator<int64_t>(0),
                                                 InnerRowLength{nullptr, nullptr, 0});
    if (rocprim::exclusive_scan(nullptr, a, it32, (uint32_t*)nullptr, 0u, (size_t)n, rocprim::plus<uint32_t>(),
                                (hipStream_t)0) != hipSuccess) return RETEXO_E_HIP;
    if (rocprim::exclusive_scan(nullptr, b, it64, (int64_t*)nullptr, (int64_t)0, (size_t)(n + 1),
                                rocprim::plus<int64_t>(), (hipStream_t)0) != hipSuccess) return RETEXO_E_HIP;
    if (rocprim::reduce(nullptr, c, it64, (int64_t*)nullptr, (int64_t)0, (size_t)n, rocprim::plus<int64_t>(),
                        (hipStream_t)0) != hipSuccess) return RETEXO_E_HIP;
    if (rocprim::radix_sort_keys(nullptr, d, (uint64_t*)nullptr, (uint64_t*)nullptr, (size_t)K, 0u, 41u,
                                 (hipStream_t)0) != hipSuccess) return RETEXO_E_HIP;
    L.tmp_bytes = a > b ? a : b;
    if (c > L.tmp_bytes) L.tmp_bytes = c;
    if (d > L.tmp_bytes) L.tmp_bytes = d;
    int64_t off = 0;
    L.header = off;    off += align_up((int64_t)sizeof(ShareHeader), 256);
    L.mask = off;      off += align_up(8 * n, 256);
    L.halo_flag = off; off += align_up(4 * n, 256);
    L.rank_in = off;   off += align_up(4 * n, 256);
    L.rank_halo = off; off += align_up(4 * n, 256);
    L.key_off = off;   off += align_up(4 * n, 256);
    L.to_local = off;  off += align_up(4 * n, 256);
    L.keys_a = off;    off += align_up(8 * K, 256);
    L.keys_b = off;    off += align_up(8 * K, 256);
    L.tmp = off;       off += align_up((int64_t)L.tmp_bytes, 256);
    L.total = off;
    return RETEXO_OK;
}

template <bool SCATTER>
int launch_rows(int64_t n, const int32_t* ids, int64_t table_rows, int64_t F, const float* src, int64_t lds,
                float* dst, int64_t ldd, hipStream_t stream)
{
    if (n == 0 || F == 0) return RETEXO_OK;
    const bool v4 = lds % 4 == 0 && ldd % 4 == 0 && (uintptr_t)src % 16 == 0 && (uintptr_t)dst % 16 == 0;
    const int64_t threads = n * (v4 ? (F + 3) / 4 : F);
    const dim3 grid((unsigned)((threads + kThreads - 1) / kThreads));
    if (v4) rows_kernel<4, SCATTER><<<grid, dim3(kThreads), 0, stream>>>(n, ids, table_rows, F, src, lds, dst, ldd);
    else rows_kernel<1, SCATTER><<<grid, dim3(kThreads), 0, stream>>>(n, ids, table_rows, F, src, lds, dst, ldd);
    if (hipGetLastError() != hipSuccess) return RETEXO_E_HIP;
    return RETEXO_OK;
}

}  // namespace

extern "C" int64_t retexo_partition_workspace_bytes(int64_t N, int n_parts, int64_t send_capacity)
{
    if (N < 0 || N >= (1ll << 31) || send_capacity < 0 || send_capacity >= (1ll << 31)) return RETEXO_E_SIZE;
    if (n_parts < 1 || n_parts > kMaxWorkers) return RETEXO_E_SIZE;
    if (N * (int64_t)(n_parts - 1) >= (1ll << 31)) return RETEXO_E_SIZE;     // 32-bit offsets of the send keys
    Layout L;
    if (int s = make_layout(N, send_capacity, L)) return s;
    return L.total;
}

extern "C" int retexo_partition_share(int64_t N, const int64_t* d_row_ptr, const int32_t* d_col_idx,
                                      const int32_t* d_part, int n_parts, int part,
                                      int64_t local_capacity, int64_t col_capacity, int64_t send_capacity,
                                      int32_t* d_local_ids, int64_t* d_local_row_ptr, int32_t* d_local_col_idx,
                                      int32_t* d_global_deg, int32_t* d_send_ids, int32_t* d_recv_ids,
                                      int64_t* h_sizes, int64_t* h_send_offsets, int64_t* h_recv_offsets,
                                      void* d_workspace, int64_t workspace_bytes, void* stream_)
{
    if (N < 0 || N >= (1ll << 31)) return RETEXO_E_SIZE;
    if (n_parts < 1 || n_parts > kMaxWorkers || part < 0 || part >= n_parts) return RETEXO_E_SIZE;
    if (N * (int64_t)(n_parts - 1) >= (1ll << 31)) return RETEXO_E_SIZE;     // 32-bit offsets of the send keys
    if (local_capacity < 0 || col_capacity < 0 || send_capacity < 0 || send_capacity >= (1ll << 31)) return RETEXO_E_SIZE;
    if (!h_sizes) return RETEXO_E_NULL;
    if (N > 0 && (!d_row_ptr || !d_part)) return RETEXO_E_NULL;
    Layout L;
    if (int s = make_layout(N, send_capacity, L)) return s;
    if (!d_workspace || ((uintptr_t)d_workspace & 255) || workspace_bytes < L.total) return RETEXO_E_WORKSPACE;

    hipStream_t stream = (hipStream_t)stream_;
    char* ws = (char*)d_workspace;
    ShareHeader* hdr = (ShareHeader*)(ws + L.header);
    uint64_t* mask = (uint64_t*)(ws + L.mask);
    uint32_t* halo_flag = (uint32_t*)(ws + L.halo_flag);
    uint32_t* rank_in = (uint32_t*)(ws + L.rank_in);
    uint32_t* rank_halo = (uint32_t*)(ws + L.rank_halo);
    uint32_t* key_off = (uint32_t*)(ws + L.key_off);
    int32_t* to_local = (int32_t*)(ws + L.to_local);
    uint64_t* keys_a = (uint64_t*)(ws + L.keys_a);
    uint64_t* keys_b = (uint64_t*)(ws + L.keys_b);
    void* tmp = ws + L.tmp;

    RETEXO_HIP_TRY(hipMemsetAsync(hdr, 0, sizeof(ShareHeader), stream));
    if (N > 0) {
        RETEXO_HIP_TRY(hipMemsetAsync(halo_flag, 0, (size_t)N * 4, stream));
        const int rows_per_block = kThreads / 64;
        mark_kernel<<<dim3((unsigned)((N + rows_per_block - 1) / rows_per_block)), dim3(kThreads), 0, stream>>>(
            N, d_row_ptr, d_col_idx, d_part, n_parts, part, halo_flag, mask, hdr);
        auto count = rocprim::make_counting_iterator<int64_t>(0);
        size_t tb = L.tmp_bytes;
        RETEXO_HIP_TRY(rocprim::exclusive_scan(tmp, tb, rocprim::make_transform_iterator(count, IsInner{d_part, part}),
                                               rank_in, 0u, (size_t)N, rocprim::plus<uint32_t>(), stream));
        tb = L.tmp_bytes;
        RETEXO_HIP_TRY(rocprim::exclusive_scan(tmp, tb, halo_flag, rank_halo, 0u, (size_t)N,
                                               rocprim::plus<uint32_t>(), stream));
        tb = L.tmp_bytes;
        RETEXO_HIP_TRY(rocprim::exclusive_scan(tmp, tb, rocprim::make_transform_iterator(count, PeerCount{mask}),
                                               key_off, 0u, (size_t)N, rocprim::plus<uint32_t>(), stream));
        tb = L.tmp_bytes;
        RETEXO_HIP_TRY(rocprim::reduce(tmp, tb, rocprim::make_transform_iterator(count, InnerRowLength{d_part, d_row_ptr, part}),
                                       &hdr->nnz_local, (int64_t)0, (size_t)N, rocprim::plus<int64_t>(), stream));
        totals_kernel<<<dim3(1), dim3(64), 0, stream>>>(N, d_part, part, rank_in, halo_flag, rank_halo, key_off, mask, hdr);
    }
    ShareHeader h;
    RETEXO_HIP_TRY(hipMemcpyAsync(&h, hdr, sizeof(h), hipMemcpyDeviceToHost, stream));
    RETEXO_HIP_TRY(hipStreamSynchronize(stream));
    if (h.bad_part) return RETEXO_E_PARTITION;
    h_sizes[0] = h.n_inner;
    h_sizes[1] = h.n_halo;
    h_sizes[2] = h.nnz_local;
    h_sizes[3] = h.n_send;
    const int64_t n_local = h.n_inner + h.n_halo;
    // a missing row-pointer array counts as no capacity at all: the size query of an empty share
    if (!d_local_row_ptr || n_local > local_capacity || h.nnz_local > col_capacity || h.n_send > send_capacity)
        return RETEXO_E_CAPACITY;
    if (!h_send_offsets || !h_recv_offsets) return RETEXO_E_NULL;
    if (n_local > 0 && (!d_local_ids || !d_global_deg)) return RETEXO_E_NULL;
    if (h.nnz_local > 0 && !d_local_col_idx) return RETEXO_E_NULL;
    if ((h.n_send > 0 && !d_send_ids) || (h.n_halo > 0 && !d_recv_ids)) return RETEXO_E_NULL;

    if (N > 0) {
        number_kernel<<<dim3((unsigned)((N + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream>>>(
            N, d_row_ptr, d_part, part, rank_in, halo_flag, rank_halo, h.n_inner, to_local, d_local_ids, d_global_deg);
    }
    {
        auto len = rocprim::make_transform_iterator(rocprim::make_counting_iterator<int64_t>(0),
                                                    LocalRowLength{d_local_ids, d_row_ptr, h.n_inner});
        size_t tb = L.tmp_bytes;
        RETEXO_HIP_TRY(rocprim::exclusive_scan(tmp, tb, len, d_local_row_ptr, (int64_t)0, (size_t)(n_local + 1),
                                               rocprim::plus<int64_t>(), stream));
    }
    if (h.n_inner > 0) {
        const int rows_per_block = kThreads / 64;
        columns_kernel<<<dim3((unsigned)((h.n_inner + rows_per_block - 1) / rows_per_block)), dim3(kThreads), 0, stream>>>(
            h.n_inner, d_local_ids, d_row_ptr, d_col_idx, to_local, d_local_row_ptr, d_local_col_idx);
    }
    const int64_t K = h.n_send + h.n_halo;
    if (K > 0) {
        keys_kernel<<<dim3((unsigned)((n_local + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream>>>(
            h.n_inner, h.n_halo, d_local_ids, d_part, mask, key_off, h.n_send, keys_a);
        size_t tb = L.tmp_bytes;
        RETEXO_HIP_TRY(rocprim::radix_sort_keys(tmp, tb, keys_a, keys_b, (size_t)K, 0u, 41u, stream));
    }
    {
        const int64_t work = K > 2 * (int64_t)n_parts + 2 ? K : 2 * (int64_t)n_parts + 2;
        lists_kernel<<<dim3((unsigned)((work + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream>>>(
            h.n_send, h.n_halo, keys_b, n_parts, d_send_ids, d_recv_ids, hdr);
    }
    RETEXO_HIP_TRY(hipGetLastError());
    RETEXO_HIP_TRY(hipMemcpyAsync(&h, hdr, sizeof(h), hipMemcpyDeviceToHost, stream));
    RETEXO_HIP_TRY(hipStreamSynchronize(stream));
    for (int q = 0; q <= n_parts; ++q) {
        h_send_offsets[q] = h.send_off[q];
        h_recv_offsets[q] = h.recv_off[q];
    }
    return RETEXO_OK;
}

extern "C" int retexo_halo_pack(int64_t n, const int32_t* d_ids, int64_t table_rows, int64_t F,
                                const float* d_H, int64_t ldh, float* d_buf, int64_t ldb, void* stream)
{
    if (n < 0 || F < 0 || table_rows < 0) return RETEXO_E_SIZE;
    if (n > 0 && F > 0 && (!d_ids || !d_H || !d_buf)) return RETEXO_E_NULL;
    if (ldh < F || ldb < F) return RETEXO_E_LD;
    return launch_rows<false>(n, d_ids, table_rows, F, d_H, ldh, d_buf, ldb, (hipStream_t)stream);
}

extern "C" int retexo_halo_unpack(int64_t n, const int32_t* d_ids, int64_t table_rows, int64_t F,
                                  const float* d_buf, int64_t ldb, float* d_H, int64_t ldh, void* stream)
{
    if (n < 0 || F < 0 || table_rows < 0) return RETEXO_E_SIZE;
    if (n > 0 && F > 0 && (!d_ids || !d_H || !d_buf)) return RETEXO_E_NULL;
    if (ldh < F || ldb < F) return RETEXO_E_LD;
    return launch_rows<true>(n, d_ids, table_rows, F, d_buf, ldb, d_H, ldh, (hipStream_t)stream);
}

extern "C" int retexo_plan_set_degrees(retexo_plan* plan, const int32_t* d_deg, void* stream)
{
    if (!plan) return RETEXO_E_NULL;
    if (plan->N > 0 && !d_deg) return RETEXO_E_NULL;
    if (plan->N == 0) return RETEXO_OK;
    set_degrees_kernel<<<dim3((unsigned)((plan->N + kThreads - 1) / kThreads)), dim3(kThreads), 0, (hipStream_t)stream>>>(
        plan->N, d_deg, plan->deg, plan->dinv);
    if (hipGetLastError() != hipSuccess) return RETEXO_E_HIP;
    return RETEXO_OK;
}
