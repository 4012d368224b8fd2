// CSR construction from raw undirected pairs by bucketing (the fast path of retexo_csr_from_coo).
//
// The paper's graphs are undirected (section "Edge-partitioned Distributed Setup"): each pair {u,v}
// becomes the entries (u,v) and (v,u), repeats are kept once, self pairs are dropped, and
// add_self_loops appends one entry (v,v) per node.  The result — rows in id order, columns
// ascending and unique — is a function of the pair set alone, so any order of evaluation gives
// the same bits.  That freedom is what this file uses: instead of sorting 64-bit (row, col) keys
// with a general radix sort (five to six passes over 16 bytes per entry), the entries are first
// moved into buckets of consecutive rows that fit the local data share, and each bucket is then
// sorted and cleaned there, by one workgroup, without touching memory in between.
//
//   hist     every workgroup counts its share of the entries per row range ("bin", 2^s rows) in LDS
//   colsum   adds the workgroups' counts
//   plan     one workgroup: prefix sums over the bins, buckets = runs of bins of about kTarget
//            entries (never more than kRowSpan rows), groups = runs of 256 buckets
//   part1    entries -> their group   (skipped when there is only one group)
//   part2    entries -> their bucket, packed as (row - first row of the bucket) << cbits | col
//            (both moves stage a tile in LDS ordered by destination, reserve the destination ranges
//             with one atomic per destination and tile, and write runs)
//   sort     one workgroup per bucket: entries counted per row, every row given a number of column
//            bins proportional to its length (so that a bin holds 4 to 8 entries whatever the
//            degree), LDS counting split into those bins, rank by comparison inside a bin,
//            drop repeats, count the kept entries per row;
//            a bucket that does not fit LDS is worked through in key ranges, the ranges split
//            until each fits (a single long row, a clustered row range, many repeats: all end)
//   total    one workgroup: prefix sums over the buckets' entry counts -> nnz
//   emit     one workgroup per bucket: row offsets of its rows, columns to their final place
//            (nothing is written when an id was out of range or the capacity is too small)
//
// Integer arithmetic only.  The order in which atomics hand out positions inside a bucket is
// arbitrary, but the sorted, repeat-free result is not, so the output is bitwise reproducible.
#include "common.hpp"
#include "csr_bucket.hpp"

namespace {

constexpr int kThreads = 1024;           // hist, plan, part1, part2, sort, total
constexpr int kWaves = kThreads / 64;
constexpr int kMaxBins = 32768;          // row ranges the histogram distinguishes
constexpr int kMaxHistBlocks = 256;
constexpr int kItemsPerTile = 4096;      // pairs per part1 tile (two entries each)
constexpr int kTileEntries = 8192;       // entries per part2 tile
constexpr int kGroupBuckets = 256;       // buckets per group
constexpr int kMaxGroups = 1024;
constexpr int kMaxBuckets = kGroupBuckets * kMaxGroups;
constexpr int kBucketMax = 10240;        // entries a bucket can hold in LDS (10 per thread)
constexpr int kTarget = kBucketMax / 2;  // entries a bucket is filled to
constexpr int kRowSpan = 1024;           // rows per bucket at most (one per thread of the sort)
constexpr int kSortBins = kBucketMax / 4 + kRowSpan;   // bins of the LDS split: a row of c entries gets < max(1, c/4)
constexpr int kStack = 400;              // key ranges waiting in an oversized bucket (6 levels x 63 + 1)

struct BucketHeader {       // start of the workspace
    uint32_t bad_id;        // an id was outside [0, N)
    uint32_t overflow;      // nnz exceeds the capacity of col_idx
    int64_t nnz;
    uint32_t n_buckets;
    uint32_t n_groups;
    uint32_t part2_tiles;
    uint32_t internal;      // a construction invariant failed (never expected)
};


// exclusive prefix sum over the workgroup (NW waves); `total` is the sum over all threads.
// sc: 2 * NW + 1 words of LDS scratch, free again when the call returns.
template <int NW>
__device__ __forceinline__ uint32_t block_scan_excl(uint32_t v, uint32_t* sc, uint32_t& total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t t = __shfl_up(incl, d, 64);
        if (lane >= d) incl += t;
    }
    if (lane == 63) sc[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        const uint32_t w = lane < NW ? sc[lane] : 0u;
        uint32_t wi = w;
#pragma unroll
        for (int d = 1; d < NW; d <<= 1) {
            const uint32_t t = __shfl_up(wi, d, 64);
            if (lane >= d) wi += t;
        }
        if (lane < NW) sc[NW + lane] = wi - w;
        if (lane == NW - 1) sc[2 * NW] = wi;
    }
    __syncthreads();
    const uint32_t excl = incl - v + sc[NW + wave];
    total = sc[2 * NW];
    __syncthreads();
    return excl;
}

// largest g in [0, n) with table[g] <= x (table ascending, table[0] <= x)
__device__ __forceinline__ int find_segment(const uint32_t* table, int n, uint32_t x)
{
    int lo = 0, hi = n;
    while (lo + 1 < hi) {
        const int mid = (lo + hi) >> 1;
        if (table[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// arr[idx] += 1 for every lane with `active` set.  When all of them name the same element (a long row, a
// clustered range) the wave adds their number once instead of queueing up on one LDS address.
// Call with the whole wave (the loop around it must be uniform per wave).
__device__ __forceinline__ void lds_count(uint32_t* arr, uint32_t idx, bool active)
{
    const uint64_t act = __ballot(active);
    if (!act) return;
    const int lane = threadIdx.x & 63;
    const int leader = __ffsll((unsigned long long)act) - 1;
    const uint32_t first = __shfl(idx, leader, 64);
    const uint64_t same = __ballot(active && idx == first);
    if (same == act) {
        if (lane == leader) atomicAdd(&arr[first], (uint32_t)__popcll(act));
    } else if (active) {
        atomicAdd(&arr[idx], 1u);
    }
}

// item i of the input: pair i for i < n_pairs, afterwards the self-loop of node i - n_pairs.
// Returns the number of entries it yields (0, 1 or 2) as (r0,c0), (r1,c1).
__device__ __forceinline__ int item_entries(int64_t i, int64_t n_pairs, const int32_t* __restrict__ src,
                                            const int32_t* __restrict__ dst, int64_t N, bool& bad,
                                            uint32_t& r0, uint32_t& c0, uint32_t& r1, uint32_t& c1)
{
    if (i < n_pairs) {
        const uint32_t u = (uint32_t)src[i], v = (uint32_t)dst[i];
        if (u >= (uint64_t)N || v >= (uint64_t)N) { bad = true; return 0; }
        if (u == v) return 0;                       // self pairs are dropped; self-loops come from the items below
        r0 = u; c0 = v; r1 = v; c1 = u;
        return 2;
    }
    r0 = c0 = (uint32_t)(i - n_pairs);
    return 1;
}

// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void hist_kernel(
    int64_t n_pairs, const int32_t* __restrict__ src, const int32_t* __restrict__ dst, int64_t N, int64_t n_items,
    int64_t items_per_block, int s, int nbins, uint32_t* __restrict__ counts, BucketHeader* hdr)
{
    __shared__ uint32_t hist[kMaxBins];
    for (int i = threadIdx.x; i < nbins; i += kThreads) hist[i] = 0u;
    __syncthreads();
    const int64_t begin = (int64_t)blockIdx.x * items_per_block;
    const int64_t end = begin + items_per_block < n_items ? begin + items_per_block : n_items;
    bool bad = false;
    for (int64_t i = begin + threadIdx.x; i < end; i += kThreads) {
        uint32_t r0, c0, r1, c1;
        const int k = item_entries(i, n_pairs, src, dst, N, bad, r0, c0, r1, c1);
        if (k >= 1) atomicAdd(&hist[r0 >> s], 1u);
        if (k == 2) atomicAdd(&hist[r1 >> s], 1u);
    }
    if (bad) atomicOr(&hdr->bad_id, 1u);
    __syncthreads();
    uint32_t* mine = counts + (size_t)blockIdx.x * nbins;
    for (int i = threadIdx.x; i < nbins; i += kThreads) mine[i] = hist[i];
}

// bin_count[b] += the counts of this block's slice of the histogram blocks (bin_count starts at zero)
constexpr int kColsumSlices = 8;
__global__ __launch_bounds__(256) void colsum_kernel(int nblocks, int nbins, const uint32_t* __restrict__ counts,
                                                     uint32_t* bin_count)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= nbins) return;
    const int per = (nblocks + kColsumSlices - 1) / kColsumSlices;
    const int w0 = blockIdx.y * per, w1 = w0 + per < nblocks ? w0 + per : nblocks;
    uint32_t s = 0;
    for (int w = w0; w < w1; ++w) s += counts[(size_t)w * nbins + b];
    if (s) atomicAdd(&bin_count[b], s);
}

struct PlanArrays {
    uint32_t* bin_off;        // [nbins + 1] entries before each bin
    uint32_t* bucket_bin0;    // [n_buckets + 1] first bin of each bucket
    uint32_t* bucket_off;     // [n_buckets + 1] entries before each bucket
    uint32_t* bucket_cursor;  // [n_buckets] part2's write positions
    uint32_t* group_bin0;     // [n_groups + 1]
    uint32_t* group_off;      // [n_groups + 1]
    uint32_t* group_cursor;   // [n_groups] part1's write positions
    uint32_t* group_tile0;    // [n_groups + 1] first part2 tile of each group
    uint16_t* coarse_group;   // [kMaxBins / 16] per block of 16 bins: group of its first bin | (bin offset inside the
                              // block at which the next group starts, 16 = none) << 10
};

// A bin starts a bucket when the entries before it cross a multiple of kTarget, when it is the
// first bin of a window of `span_bins` bins (so that a bucket never holds more than kRowSpan rows
// and its rows pack into 32 - cbits bits), or when it or its predecessor is a bin of at least
// kTarget entries (large bins stand alone).
__device__ __forceinline__ bool starts_bucket(int bin, uint32_t off, uint32_t prev_off, uint32_t cnt, uint32_t prev_cnt,
                                              int span_bins)
{
    return bin == 0 || off / kTarget != prev_off / kTarget || bin % span_bins == 0 || cnt >= (uint32_t)kTarget ||
           prev_cnt >= (uint32_t)kTarget;
}

__global__ __launch_bounds__(kThreads) void plan_kernel(int nbins, int span_bins, const uint32_t* __restrict__ bin_count,
                                                        PlanArrays a, uint32_t bucket_capacity, BucketHeader* hdr)
{
    __shared__ uint32_t cnts[kMaxBins];            // the bin counts, read three times
    __shared__ uint32_t sc[2 * kWaves + 1];
    if (hdr->bad_id) return;
    for (int b = threadIdx.x; b < nbins; b += kThreads) cnts[b] = bin_count[b];
    __syncthreads();
    const int per = (nbins + kThreads - 1) / kThreads;
    const int b0 = threadIdx.x * per < nbins ? threadIdx.x * per : nbins, b1 = b0 + per < nbins ? b0 + per : nbins;
    uint32_t sum = 0;
    for (int b = b0; b < b1; ++b) sum += cnts[b];
    uint32_t total;
    uint32_t off = block_scan_excl<kWaves>(sum, sc, total);
    uint32_t starts = 0;
    {
        uint32_t o = off;
        for (int b = b0; b < b1; ++b) {
            const uint32_t cnt = cnts[b], pc = b > 0 ? cnts[b - 1] : 0u;
            a.bin_off[b] = o;
            starts += starts_bucket(b, o, o - pc, cnt, pc, span_bins) ? 1u : 0u;
            o += cnt;
        }
    }
    if (threadIdx.x == 0) a.bin_off[nbins] = total;
    uint32_t n_buckets;
    uint32_t id = block_scan_excl<kWaves>(starts, sc, n_buckets);
    if (n_buckets > bucket_capacity) {             // cannot happen: the host sized the arrays for the worst case
        if (threadIdx.x == 0) { hdr->internal = 1u; hdr->n_buckets = 0u; hdr->n_groups = 0u; hdr->part2_tiles = 0u; }
        return;
    }
    {
        uint32_t o = off;
        for (int b = b0; b < b1; ++b) {
            const uint32_t cnt = cnts[b], pc = b > 0 ? cnts[b - 1] : 0u;
            if (starts_bucket(b, o, o - pc, cnt, pc, span_bins)) {
                a.bucket_bin0[id] = (uint32_t)b;
                a.bucket_off[id] = o;
                a.bucket_cursor[id] = o;
                ++id;
            }
            o += cnt;
        }
    }
    const uint32_t n_groups = (n_buckets + kGroupBuckets - 1) / kGroupBuckets;
    if (threadIdx.x == 0) {
        a.bucket_bin0[n_buckets] = (uint32_t)nbins;
        a.bucket_off[n_buckets] = total;
        hdr->n_buckets = n_buckets;
        hdr->n_groups = n_groups;
    }
    __syncthreads();                               // the bucket arrays are complete
    // one group per thread (n_groups <= kMaxGroups = kThreads)
    const uint32_t g = threadIdx.x;
    uint32_t tiles = 0;
    if (g < n_groups) {
        const uint32_t first = g * kGroupBuckets;
        const uint32_t last = first + kGroupBuckets < n_buckets ? first + kGroupBuckets : n_buckets;
        const uint32_t lo = a.bucket_off[first], hi = a.bucket_off[last];
        a.group_bin0[g] = a.bucket_bin0[first];
        a.group_off[g] = lo;
        a.group_cursor[g] = lo;
        tiles = (hi - lo + kTileEntries - 1) / kTileEntries;
    }
    uint32_t n_tiles;
    const uint32_t t0 = block_scan_excl<kWaves>(tiles, sc, n_tiles);
    if (g < n_groups) a.group_tile0[g] = t0;
    if (threadIdx.x == 0) {
        a.group_bin0[n_groups] = (uint32_t)nbins;
        a.group_off[n_groups] = total;
        a.group_tile0[n_groups] = n_tiles;
        hdr->part2_tiles = n_tiles;
    }
    __syncthreads();                               // the group arrays are complete
    // A group other than the last holds 256 buckets, i.e. at least 256 bins, so a block of 16 bins meets at most
    // one group boundary.
    for (int c = threadIdx.x; c < kMaxBins / 16; c += kThreads) {
        const uint32_t first_bin = (uint32_t)c << 4;
        uint32_t g = n_groups - 1, at = 16;
        if (first_bin < (uint32_t)nbins) {
            g = (uint32_t)find_segment(a.group_bin0, (int)n_groups, first_bin);
            if (g + 1 < n_groups && a.group_bin0[g + 1] - first_bin < 16u) at = a.group_bin0[g + 1] - first_bin;
        }
        a.coarse_group[c] = (uint16_t)(g | (at << 10));
    }
}

// ---------------------------------------------------------------------------
// part1: the entries of one tile of items go to their groups as (row, col) pairs.
__global__ __launch_bounds__(kThreads) void part1_kernel(
    int64_t n_pairs, const int32_t* __restrict__ src, const int32_t* __restrict__ dst, int64_t N, int64_t n_items, int s,
    const uint16_t* __restrict__ coarse_group, uint32_t* group_cursor, uint32_t* __restrict__ rows_out,
    uint32_t* __restrict__ cols_out, const BucketHeader* hdr)
{
    constexpr int IPT = kItemsPerTile / kThreads;          // items per thread
    __shared__ uint32_t toff[kMaxGroups + 1];
    __shared__ uint32_t base[kMaxGroups];
    __shared__ uint32_t srow[2 * kItemsPerTile], scol[2 * kItemsPerTile];
    __shared__ uint32_t sc[2 * kWaves + 1];
    __shared__ uint16_t coarse[kMaxBins / 16];
    if (hdr->bad_id || hdr->internal) return;
    const int G = (int)hdr->n_groups;
    for (int i = threadIdx.x; i <= G; i += kThreads) toff[i] = 0u;
    for (int c = threadIdx.x; c < kMaxBins / 16; c += kThreads) coarse[c] = coarse_group[c];
    __syncthreads();
    // the group of a bin: that of its block's first bin, or the next one from the recorded offset on
    auto group_of = [&](uint32_t bin) {
        const uint32_t e = coarse[bin >> 4];
        return (int)((e & 0x3ffu) + ((bin & 15u) >= (e >> 10) ? 1u : 0u));
    };

    // slot 2k / 2k+1: the entries of the thread's k-th item; group kNone marks an unused slot
    constexpr uint32_t kNone = 0xffffffffu;
    uint32_t er[2 * IPT], ec[2 * IPT], erank[2 * IPT], eg[2 * IPT];
    bool bad = false;
#pragma unroll
    for (int k = 0; k < IPT; ++k) {
        const int64_t i = (int64_t)blockIdx.x * kItemsPerTile + k * kThreads + threadIdx.x;
        uint32_t r0 = 0, c0 = 0, r1 = 0, c1 = 0;
        const int cnt = i < n_items ? item_entries(i, n_pairs, src, dst, N, bad, r0, c0, r1, c1) : 0;
        er[2 * k] = r0; ec[2 * k] = c0; er[2 * k + 1] = r1; ec[2 * k + 1] = c1;
        eg[2 * k] = eg[2 * k + 1] = kNone;
        erank[2 * k] = erank[2 * k + 1] = 0u;
        if (cnt >= 1) {
            const int g = group_of(r0 >> s);
            eg[2 * k] = (uint32_t)g;
            erank[2 * k] = atomicAdd(&toff[g], 1u);
        }
        if (cnt == 2) {
            const int g = group_of(r1 >> s);
            eg[2 * k + 1] = (uint32_t)g;
            erank[2 * k + 1] = atomicAdd(&toff[g], 1u);
        }
    }
    __syncthreads();
    // counts -> offsets inside the tile; one reservation per group that received something
    const uint32_t mine = (int)threadIdx.x < G ? toff[threadIdx.x] : 0u;
    uint32_t total;
    const uint32_t excl = block_scan_excl<kWaves>(mine, sc, total);
    if ((int)threadIdx.x < G) {
        toff[threadIdx.x] = excl;
        base[threadIdx.x] = mine ? atomicAdd(&group_cursor[threadIdx.x], mine) : 0u;
    }
    if (threadIdx.x == 0) toff[G] = total;
    __syncthreads();
    // ids are below 2^23, so the nine high bits of a staged row and the high bit of a staged column are free:
    // they carry the entry's group (below 1024) to the write loop
#pragma unroll
    for (int k = 0; k < 2 * IPT; ++k)
        if (eg[k] != kNone) {
            const uint32_t p = toff[eg[k]] + erank[k];
            srow[p] = er[k] | ((eg[k] & 0x1ffu) << 23);
            scol[p] = ec[k] | ((eg[k] >> 9) << 23);
        }
    __syncthreads();
    for (uint32_t j = threadIdx.x; j < total; j += kThreads) {
        const uint32_t r = srow[j], c = scol[j];
        const uint32_t g = (r >> 23) | ((c >> 23) << 9);
        const uint32_t d = base[g] + (j - toff[g]);
        rows_out[d] = r & 0x7fffffu;
        cols_out[d] = c & 0x7fffffu;
    }
}

// part2: the entries of one tile go to their buckets, packed.  FROM_PAIRS: there is a single group and the
// tile is a tile of input items; otherwise the tile is a piece of one group's (row, col) run.
template <bool FROM_PAIRS>
__global__ __launch_bounds__(kThreads) void part2_kernel(
    int64_t n_pairs, const int32_t* __restrict__ src, const int32_t* __restrict__ dst, int64_t N, int64_t n_items, int s,
    int cbits, const uint32_t* __restrict__ rows_in, const uint32_t* __restrict__ cols_in,
    const uint32_t* __restrict__ group_off, const uint32_t* __restrict__ group_tile0,
    const uint32_t* __restrict__ bucket_bin0, uint32_t* bucket_cursor, uint32_t* __restrict__ packed_out,
    const BucketHeader* hdr)
{
    constexpr int EPT = kTileEntries / kThreads;           // entries per thread
    __shared__ uint32_t bb0[kGroupBuckets + 1];
    __shared__ uint32_t toff[kGroupBuckets + 1];
    __shared__ uint32_t base[kGroupBuckets];
    __shared__ uint32_t stage[kTileEntries];
    __shared__ uint8_t stage_lb[kTileEntries];             // local bucket of each staged entry
    __shared__ uint32_t sc[2 * kWaves + 1];
    if (hdr->bad_id || hdr->internal) return;
    const uint32_t n_buckets = hdr->n_buckets;
    uint32_t g = 0, e_begin = 0, e_end = 0;
    if constexpr (!FROM_PAIRS) {
        if (blockIdx.x >= hdr->part2_tiles) return;
        g = (uint32_t)find_segment(group_tile0, (int)hdr->n_groups, blockIdx.x);
        // groups without entries have no tiles and repeat a tile index: the largest g with tile0[g] <= tile holds it
        e_begin = group_off[g] + (blockIdx.x - group_tile0[g]) * kTileEntries;
        e_end = e_begin + kTileEntries < group_off[g + 1] ? e_begin + kTileEntries : group_off[g + 1];
    }
    const uint32_t first = g * kGroupBuckets;
    const int nb = (int)(first + kGroupBuckets < n_buckets ? kGroupBuckets : n_buckets - first);
    for (int i = threadIdx.x; i <= nb; i += kThreads) { bb0[i] = bucket_bin0[first + i]; toff[i] = 0u; }
    __syncthreads();
    // the group's bins -> local bucket, looked up directly when the group spans few enough bins
    constexpr int kDirect = 4096;
    __shared__ uint8_t bin_lb[kDirect];
    const uint32_t bin_first = bb0[0], bin_span = bb0[nb] - bb0[0];
    const bool direct = bin_span <= (uint32_t)kDirect;
    if (direct) {
        for (uint32_t i = threadIdx.x; i < bin_span; i += kThreads)
            bin_lb[i] = (uint8_t)find_segment(bb0, nb, bin_first + i);
        __syncthreads();
    }

    // slot k: one entry (FROM_PAIRS: slots 2k / 2k+1 are the entries of the thread's k-th item); bucket kNone = unused
    constexpr uint32_t kNone = 0xffffffffu;
    uint32_t ev[EPT], erank[EPT], eb[EPT];
    bool bad = false;
    auto take = [&](uint32_t r, uint32_t c, uint32_t& v, uint32_t& lb_out, uint32_t& rank) {
        const int lb = direct ? (int)bin_lb[(r >> s) - bin_first] : find_segment(bb0, nb, r >> s);
        v = ((r - (bb0[lb] << s)) << cbits) | c;
        lb_out = (uint32_t)lb;
        rank = atomicAdd(&toff[lb], 1u);
    };
#pragma unroll
    for (int k = 0; k < EPT; ++k) { ev[k] = 0u; erank[k] = 0u; eb[k] = kNone; }
    if constexpr (FROM_PAIRS) {
#pragma unroll
        for (int k = 0; k < EPT / 2; ++k) {
            const int64_t i = (int64_t)blockIdx.x * kItemsPerTile + k * kThreads + threadIdx.x;
            uint32_t r0 = 0, c0 = 0, r1 = 0, c1 = 0;
            const int cnt = i < n_items ? item_entries(i, n_pairs, src, dst, N, bad, r0, c0, r1, c1) : 0;
            if (cnt >= 1) take(r0, c0, ev[2 * k], eb[2 * k], erank[2 * k]);
            if (cnt == 2) take(r1, c1, ev[2 * k + 1], eb[2 * k + 1], erank[2 * k + 1]);
        }
    } else {
#pragma unroll
        for (int k = 0; k < EPT; ++k) {
            const uint32_t e = e_begin + k * kThreads + threadIdx.x;
            if (e < e_end) take(rows_in[e], cols_in[e], ev[k], eb[k], erank[k]);
        }
    }
    __syncthreads();
    const uint32_t mine = (int)threadIdx.x < nb ? toff[threadIdx.x] : 0u;
    uint32_t total;
    const uint32_t excl = block_scan_excl<kWaves>(mine, sc, total);
    if ((int)threadIdx.x < nb) {
        toff[threadIdx.x] = excl;
        base[threadIdx.x] = mine ? atomicAdd(&bucket_cursor[first + threadIdx.x], mine) : 0u;
    }
    if (threadIdx.x == 0) toff[nb] = total;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < EPT; ++k)
        if (eb[k] != kNone) {
            const uint32_t p = toff[eb[k]] + erank[k];
            stage[p] = ev[k];
            stage_lb[p] = (uint8_t)eb[k];
        }
    __syncthreads();
    for (uint32_t j = threadIdx.x; j < total; j += kThreads) {
        const uint32_t lb = stage_lb[j];
        packed_out[base[lb] + (j - toff[lb])] = stage[j];
    }
}

// ---------------------------------------------------------------------------
// sort: LDS state of one bucket
constexpr int kSortThreads = 1024;       // threads of the sort kernel (512 with twice the keys per thread measured 15 % slower)
constexpr int kSortWaves = kSortThreads / 64;
constexpr int kSortKeys = kBucketMax / kSortThreads;     // keys per thread
constexpr int kSortRows = kRowSpan / kSortThreads;       // rows per thread
constexpr uint32_t kMerged = 255u;       // "bits" of a key range that was put together from small pieces (never split)
struct SortShared {
    uint32_t keys[kBucketMax + 4];       // (the rank loop looks at four keys at a time)
    uint32_t bins[kSortBins + 1];
    uint32_t rowraw[kRowSpan];           // entries per row in the keys being sorted (sizes the row's bins)
    uint32_t rowcnt[kRowSpan];           // entries kept per row so far
    uint32_t rowmeta[kRowSpan];          // first bin of the row | (column shift of its bins << 16)
    uint32_t stk_lo[kStack], stk_hi[kStack], stk_bits[kStack], stk_cnt[kStack];
    uint32_t sc[2 * kSortWaves + 1];
    uint32_t n, sp;
};

// Sort the n <= kBucketMax keys in sh.keys, drop repeats, append the columns to out[out_cursor ...) and add
// the kept entries to the per-row counts.  Returns the number of kept keys (uniform over the workgroup).
// On entry all threads have passed a barrier after the last write to sh.keys; on return sh.keys is free.
// Kept out of line on purpose.  The kernel runs two workgroups per CU (64 registers per lane); as a called
// function this body gets a register allocation of its own and the caller's few live values cross the call
// through scratch memory (about 1.7 GB each way per construction, visible in the byte counters).  Inlined under
// the same cap it spills 13 registers inside its loops and the kernel is 7 % slower; inlined without the cap
// (one workgroup per CU) 30 % slower.
__device__ __noinline__ uint32_t sort_and_emit(SortShared& sh, uint32_t n, int nrows, int cbits,
                                                  uint32_t* __restrict__ out, uint32_t out_cursor)
{
    const int tid = threadIdx.x;
    const uint32_t cmask = (1u << cbits) - 1u;
    for (int i = tid; i < nrows; i += kSortThreads) sh.rowraw[i] = 0u;
    for (int i = tid; i <= kSortBins; i += kSortThreads) sh.bins[i] = 0u;
    __syncthreads();
    uint32_t k[kSortKeys], r[kSortKeys];
#pragma unroll
    for (int j = 0; j < kSortKeys; ++j) {                      // every lane runs every step (lds_count needs whole waves)
        const uint32_t i = tid + j * kSortThreads;
        const bool have = i < n;
        k[j] = have ? sh.keys[i] : 0u;
        lds_count(sh.rowraw, k[j] >> cbits, have);
    }
    __syncthreads();
    // a row of c entries gets 2^lg bins, 2^lg = the power of two at or above c, over 8 (at least one):
    // between c/8 and c/4 bins, so that a bin holds 4 to 8 entries when the columns are spread evenly
    {
        uint32_t lg[kSortRows], nsub = 0;
#pragma unroll
        for (int j = 0; j < kSortRows; ++j) {
            const int row = tid * kSortRows + j;
            lg[j] = 0u;
            if (row < nrows) {
                const uint32_t c = sh.rowraw[row];
                lg[j] = c <= 8u ? 0u : (uint32_t)(32 - __clz(c - 1u)) - 3u;
                lg[j] = lg[j] > (uint32_t)cbits ? (uint32_t)cbits : lg[j];
                nsub += 1u << lg[j];
            }
        }
        uint32_t nbins_total;                                  // <= kSortBins
        uint32_t first = block_scan_excl<kSortWaves>(nsub, sh.sc, nbins_total);
#pragma unroll
        for (int j = 0; j < kSortRows; ++j) {
            const int row = tid * kSortRows + j;
            if (row < nrows) {
                sh.rowmeta[row] = first | (((uint32_t)cbits - lg[j]) << 16);
                first += 1u << lg[j];
            }
        }
    }
    __syncthreads();
    // counting split; the atomic's old value is the rank inside the bin
    uint32_t bin[kSortKeys];
#pragma unroll
    for (int j = 0; j < kSortKeys; ++j) {
        const uint32_t i = tid + j * kSortThreads;
        if (i < n) {
            const uint32_t meta = sh.rowmeta[k[j] >> cbits];
            bin[j] = (meta & 0xffffu) + ((k[j] & cmask) >> (meta >> 16));
            r[j] = atomicAdd(&sh.bins[bin[j]], 1u);
        }
    }
    __syncthreads();
    {
        constexpr int BPT = (kSortBins + kSortThreads - 1) / kSortThreads;
        uint32_t c[BPT], sum = 0;
#pragma unroll
        for (int j = 0; j < BPT; ++j) {
            const int b = tid * BPT + j;
            c[j] = b < kSortBins ? sh.bins[b] : 0u;
            sum += c[j];
        }
        uint32_t total;
        uint32_t o = block_scan_excl<kSortWaves>(sum, sh.sc, total);
#pragma unroll
        for (int j = 0; j < BPT; ++j) {
            const int b = tid * BPT + j;
            if (b < kSortBins) sh.bins[b] = o;
            o += c[j];
        }
        if (tid == 0) sh.bins[kSortBins] = total;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kSortKeys; ++j) {
        const uint32_t i = tid + j * kSortThreads;
        if (i < n) sh.keys[sh.bins[bin[j]] + r[j]] = k[j];
    }
    __syncthreads();
    // rank inside the bin by comparison (a bin holds a few keys); equal keys keep their order of position
    uint32_t fp[kSortKeys];
#pragma unroll
    for (int j = 0; j < kSortKeys; ++j) {
        const uint32_t p = tid + j * kSortThreads;
        if (p < n) {
            const uint32_t key = sh.keys[p];
            const uint32_t meta = sh.rowmeta[key >> cbits];
            const uint32_t d = (meta & 0xffffu) + ((key & cmask) >> (meta >> 16));
            const uint32_t q0 = sh.bins[d], q1 = sh.bins[d + 1];
            uint32_t below = 0;
            for (uint32_t q = q0; q < q1; q += 4) {          // four independent reads per step (the array is padded)
                const uint32_t o0 = sh.keys[q], o1 = sh.keys[q + 1], o2 = sh.keys[q + 2], o3 = sh.keys[q + 3];
                below += (o0 < key || (o0 == key && q < p)) ? 1u : 0u;
                below += (q + 1 < q1 && (o1 < key || (o1 == key && q + 1 < p))) ? 1u : 0u;
                below += (q + 2 < q1 && (o2 < key || (o2 == key && q + 2 < p))) ? 1u : 0u;
                below += (q + 3 < q1 && (o3 < key || (o3 == key && q + 3 < p))) ? 1u : 0u;
            }
            k[j] = key;
            fp[j] = q0 + below;
        }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kSortKeys; ++j)
        if (tid + j * kSortThreads < n) sh.keys[fp[j]] = k[j];
    __syncthreads();
    // keep the first key of every run of equal keys: each thread takes a contiguous piece, reads what it keeps
    // into registers, and after the prefix sum writes it back compacted; rows are counted run by run
    const uint32_t per = (n + kSortThreads - 1) / kSortThreads;          // <= kSortKeys
    const uint32_t p0 = tid * per < n ? tid * per : n;
    const uint32_t p1 = p0 + per < n ? p0 + per : n;
    uint32_t kept = 0, keep_mask = 0;
    {
        uint32_t prev = p0 > 0 ? sh.keys[p0 - 1] : 0u;
        uint32_t cur_row = 0xffffffffu, run = 0;
#pragma unroll
        for (int j = 0; j < kSortKeys; ++j) {
            const uint32_t p = p0 + j;
            if (p < p1) {
                const uint32_t key = sh.keys[p];
                k[j] = key;
                if (p == 0 || key != prev) {
                    keep_mask |= 1u << j;
                    ++kept;
                    const uint32_t row = key >> cbits;
                    if (row != cur_row) {
                        if (run) atomicAdd(&sh.rowcnt[cur_row], run);
                        cur_row = row;
                        run = 0;
                    }
                    ++run;
                }
                prev = key;
            }
        }
        if (run) atomicAdd(&sh.rowcnt[cur_row], run);
    }
    uint32_t total;
    const uint32_t excl = block_scan_excl<kSortWaves>(kept, sh.sc, total);  // its barriers separate the reads from the writes
#pragma unroll
    for (int j = 0; j < kSortKeys; ++j)
        if (keep_mask & (1u << j)) sh.keys[excl + (uint32_t)__popc(keep_mask & ((1u << j) - 1u))] = k[j];
    __syncthreads();
    for (uint32_t i = tid; i < total; i += kSortThreads) out[out_cursor + i] = sh.keys[i] & cmask;
    __syncthreads();
    return total;
}

__global__ __launch_bounds__(kSortThreads, 8) void sort_kernel(
    BucketHeader* hdr, const uint32_t* __restrict__ bucket_off, const uint32_t* __restrict__ bucket_bin0,
    const uint32_t* __restrict__ packed, uint32_t* __restrict__ cols_tmp, int32_t* __restrict__ row_unique,
    uint32_t* __restrict__ bucket_total, int cbits, int s, int64_t N)
{
    __shared__ SortShared sh;
    if (hdr->bad_id || hdr->internal) return;
    const uint32_t b = blockIdx.x;
    if (b >= hdr->n_buckets) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const uint32_t e0 = bucket_off[b], E = bucket_off[b + 1] - e0;
    const int64_t row0 = (int64_t)bucket_bin0[b] << s;
    int64_t row1 = (int64_t)bucket_bin0[b + 1] << s;
    row1 = row1 < N ? row1 : N;
    const int nrows = (int)(row1 - row0);                    // <= kRowSpan
    for (int i = tid; i < nrows; i += kSortThreads) sh.rowcnt[i] = 0u;
    const uint32_t* in = packed + e0;
    uint32_t* out = cols_tmp + e0;
    uint32_t out_cursor = 0;

    // A bucket that fits is loaded and sorted in one go.  One that does not is worked through in key ranges
    // [lo, hi], lowest first: a range that fits is gathered and sorted; one that does not is an aligned block
    // of 2^bits keys, which is counted in 64 pieces by its next key bits; neighbouring pieces are put together
    // into ranges that fit, and a piece that still does not fit is split again (or is a single repeated key).
    // Each level removes 6 key bits, so the stack stays below kStack.
    const bool fits = E <= (uint32_t)kBucketMax;
    if (fits) {
        uint32_t v[kSortKeys];
#pragma unroll
        for (int j = 0; j < kSortKeys; ++j) {                // all loads in flight before the first is used
            const uint32_t i = tid + j * kSortThreads;
            v[j] = i < E ? in[i] : 0u;
        }
#pragma unroll
        for (int j = 0; j < kSortKeys; ++j) {
            const uint32_t i = tid + j * kSortThreads;
            if (i < E) sh.keys[i] = v[j];
        }
        if (tid == 0) sh.sp = 0u;
    } else if (tid == 0) {
        // the walk starts at the bits the bucket's keys really use (its rows, then the columns): a bucket of
        // eight hot rows would otherwise spend three counting passes on key bits that are all zero
        const uint32_t kb = (uint32_t)cbits + (nrows > 1 ? 32u - (uint32_t)__clz((uint32_t)(nrows - 1)) : 0u);
        sh.stk_lo[0] = 0u;
        sh.stk_hi[0] = kb >= 32u ? 0xffffffffu : (1u << kb) - 1u;
        sh.stk_bits[0] = kb >= 32u ? 32u : kb;
        sh.stk_cnt[0] = E;
        sh.sp = 1u;
    }
    __syncthreads();
    for (bool first = true;; first = false) {
        uint32_t n;
        if (fits) {
            if (!first || E == 0) break;
            n = E;
        } else {
            const uint32_t sp = sh.sp;
            if (sp == 0) break;
            const uint32_t lo = sh.stk_lo[sp - 1], hi = sh.stk_hi[sp - 1], bits = sh.stk_bits[sp - 1],
                           cnt = sh.stk_cnt[sp - 1];
            __syncthreads();
            if (tid == 0) { sh.sp = sp - 1; sh.n = 0u; }
            __syncthreads();
            if (cnt > (uint32_t)kBucketMax && bits == 0u) {
                // more than a bucketful of one and the same key: it is kept once
                if (tid == 0) {
                    out[out_cursor] = lo & ((1u << cbits) - 1u);
                    atomicAdd(&sh.rowcnt[lo >> cbits], 1u);
                }
                out_cursor += 1;
                __syncthreads();
                continue;
            }
            if (cnt > (uint32_t)kBucketMax) {
                const uint32_t cb = bits > 6u ? bits - 6u : 0u;
                const int nchild = 1 << (bits - cb);
                if (tid < 64) sh.bins[tid] = 0u;
                __syncthreads();
                for (uint32_t i0 = (uint32_t)(tid - lane); i0 < E; i0 += kSortThreads) {  // uniform per wave
                    const uint32_t i = i0 + lane;
                    const uint32_t key = i < E ? in[i] : 0u;
                    const bool match = i < E && key >= lo && key <= hi;
                    lds_count(sh.bins, match ? (key - lo) >> cb : 0u, match);
                }
                __syncthreads();
                if (tid == 0) {
                    // highest keys first, so that the lowest range is on top of the stack
                    uint32_t top = sh.sp;
                    auto push = [&](int c0, int c1, uint32_t b_, uint32_t n_) {      // pieces c0..c1
                        if (top >= (uint32_t)kStack) { hdr->internal = 1u; return; }  // cannot happen (6 levels x 64)
                        sh.stk_lo[top] = lo + ((uint32_t)c0 << cb);
                        sh.stk_hi[top] = c1 == nchild - 1 ? hi : lo + ((uint32_t)(c1 + 1) << cb) - 1u;
                        sh.stk_bits[top] = b_;
                        sh.stk_cnt[top] = n_;
                        ++top;
                    };
                    int ch = nchild - 1;
                    while (ch >= 0) {
                        if (sh.bins[ch] > (uint32_t)kBucketMax) { push(ch, ch, cb, sh.bins[ch]); --ch; continue; }
                        const int c1 = ch;
                        uint32_t sum = 0;
                        while (ch >= 0 && sum + sh.bins[ch] <= (uint32_t)kBucketMax) { sum += sh.bins[ch]; --ch; }
                        if (sum) push(ch + 1, c1, kMerged, sum);
                    }
                    sh.sp = top;
                }
                __syncthreads();
                continue;
            }
            // the range fits: gather its keys
            for (uint32_t i0 = (uint32_t)(tid - lane); i0 < E; i0 += kSortThreads) {      // uniform per wave
                const uint32_t i = i0 + lane;
                const uint32_t key = i < E ? in[i] : 0u;
                const bool match = i < E && key >= lo && key <= hi;
                const uint64_t mask = __ballot(match);
                if (mask) {
                    const int leader = __ffsll((unsigned long long)mask) - 1;
                    uint32_t at = 0;
                    if (lane == leader) at = atomicAdd(&sh.n, (uint32_t)__popcll(mask));
                    at = __shfl(at, leader, 64);
                    if (match) sh.keys[at + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull))] = key;
                }
            }
            __syncthreads();
            n = sh.n;                                          // == cnt
        }
        out_cursor += sort_and_emit(sh, n, nrows, cbits, out, out_cursor);
    }
    __syncthreads();
    for (int i = tid; i < nrows; i += kSortThreads) row_unique[row0 + i] = (int32_t)sh.rowcnt[i];
    if (tid == 0) bucket_total[b] = out_cursor;
}

__global__ __launch_bounds__(kThreads) void total_kernel(BucketHeader* hdr, const uint32_t* __restrict__ bucket_total,
                                                         uint32_t* __restrict__ bucket_out, int64_t col_capacity)
{
    __shared__ uint32_t sc[2 * kWaves + 1];
    if (hdr->bad_id || hdr->internal) return;
    const uint32_t n = hdr->n_buckets;
    const uint32_t per = (n + kThreads - 1) / kThreads;
    const uint32_t b0 = threadIdx.x * per < n ? threadIdx.x * per : n;
    const uint32_t b1 = b0 + per < n ? b0 + per : n;
    uint32_t s = 0;
    for (uint32_t b = b0; b < b1; ++b) s += bucket_total[b];
    uint32_t total;
    uint32_t o = block_scan_excl<kWaves>(s, sc, total);
    for (uint32_t b = b0; b < b1; ++b) { bucket_out[b] = o; o += bucket_total[b]; }
    if (threadIdx.x == 0) {
        bucket_out[n] = total;
        hdr->nnz = (int64_t)total;
        hdr->overflow = (int64_t)total > col_capacity ? 1u : 0u;
    }
}

__global__ __launch_bounds__(256) void emit_kernel(
    const BucketHeader* hdr, const uint32_t* __restrict__ bucket_off, const uint32_t* __restrict__ bucket_bin0,
    const uint32_t* __restrict__ bucket_out, const uint32_t* __restrict__ cols_tmp, const int32_t* __restrict__ row_unique,
    int s, int64_t N, int64_t* __restrict__ row_ptr, int32_t* __restrict__ col_idx)
{
    constexpr int RPT = kRowSpan / 256;                      // rows per thread
    __shared__ uint32_t sc[2 * 4 + 1];
    if (hdr->bad_id || hdr->internal || hdr->overflow) return;
    const uint32_t b = blockIdx.x, n = hdr->n_buckets;
    if (b >= n) return;
    const int64_t row0 = (int64_t)bucket_bin0[b] << s;
    int64_t row1 = (int64_t)bucket_bin0[b + 1] << s;
    row1 = row1 < N ? row1 : N;
    const int nrows = (int)(row1 - row0);
    const uint32_t out0 = bucket_out[b], count = bucket_out[b + 1] - out0;
    uint32_t c[RPT], sum = 0;
#pragma unroll
    for (int j = 0; j < RPT; ++j) {
        const int i = threadIdx.x * RPT + j;
        c[j] = i < nrows ? (uint32_t)row_unique[row0 + i] : 0u;
        sum += c[j];
    }
    uint32_t total;
    uint32_t o = out0 + block_scan_excl<4>(sum, sc, total);
#pragma unroll
    for (int j = 0; j < RPT; ++j) {
        const int i = threadIdx.x * RPT + j;
        if (i < nrows) row_ptr[row0 + i] = (int64_t)o;
        o += c[j];
    }
    if (b == n - 1 && threadIdx.x == 0) row_ptr[N] = hdr->nnz;
    const uint32_t* from = cols_tmp + bucket_off[b];
    for (uint32_t i = threadIdx.x; i < count; i += 256) col_idx[out0 + i] = (int32_t)from[i];
}

int column_bits(int64_t N)
{
    int b = 1;
    while ((1ll << b) < N) ++b;
    return b;
}

static_assert(sizeof(BucketHeader) <= 256, "the header has 256 bytes of the workspace");

struct BucketLayout {
    int cbits, s, nbins, span_bins, hist_blocks;
    int64_t M, n_items, items_per_block, bucket_bound;
    bool two_level;
    int64_t header, counts, bin_count, bin_off, bucket_bin0, bucket_off, bucket_cursor, bucket_total, bucket_out,
        group_bin0, group_off, group_cursor, group_tile0, coarse_group, buf_a, buf_b, buf_c, row_unique, total;
};

bool make_bucket_layout(int64_t n_pairs, int64_t N, int add_self_loops, BucketLayout& L)
{
    if (N < 1) return false;
    L.cbits = column_bits(N);
    if (L.cbits > 23) return false;                          // rows of a bucket must pack into 32 - cbits bits
    L.M = 2 * n_pairs + (add_self_loops ? N : 0);
    L.n_items = n_pairs + (add_self_loops ? N : 0);
    L.s = L.cbits > 15 ? L.cbits - 15 : 0;
    L.nbins = (int)((N + (1ll << L.s) - 1) >> L.s);          // <= kMaxBins
    const int64_t span_rows = (1ll << (32 - L.cbits)) < kRowSpan ? (1ll << (32 - L.cbits)) : kRowSpan;
    L.span_bins = (int)(span_rows >> L.s);
    if (L.span_bins < 1 || L.nbins > kMaxBins) return false;
    // worst case of starts_bucket: one start per kTarget entries, two per large bin, one per row window
    L.bucket_bound = 3 * (L.M / kTarget) + L.nbins / L.span_bins + 4;
    if (L.bucket_bound > kMaxBuckets) return false;
    L.two_level = L.bucket_bound > kGroupBuckets;
    int64_t hb = (L.n_items + 16383) / 16384;
    L.hist_blocks = (int)(hb < 1 ? 1 : hb > kMaxHistBlocks ? kMaxHistBlocks : hb);
    L.items_per_block = align_up((L.n_items + L.hist_blocks - 1) / L.hist_blocks, kThreads);
    if (L.items_per_block < kThreads) L.items_per_block = kThreads;
    int64_t off = 0;
    auto take = [&](int64_t bytes) { const int64_t at = off; off += align_up(bytes > 0 ? bytes : 4, 256); return at; };
    const int64_t m = L.M > 0 ? L.M : 1;
    L.header = take(256);
    L.bin_count = take(4ll * L.nbins);                       // (zeroed together with the header)
    L.counts = take(4ll * L.hist_blocks * L.nbins);
    L.bin_off = take(4ll * (L.nbins + 1));
    L.bucket_bin0 = take(4 * (L.bucket_bound + 1));
    L.bucket_off = take(4 * (L.bucket_bound + 1));
    L.bucket_cursor = take(4 * L.bucket_bound);
    L.bucket_total = take(4 * L.bucket_bound);
    L.bucket_out = take(4 * (L.bucket_bound + 1));
    L.group_bin0 = take(4 * (kMaxGroups + 1));
    L.group_off = take(4 * (kMaxGroups + 1));
    L.group_cursor = take(4 * kMaxGroups);
    L.group_tile0 = take(4 * (kMaxGroups + 1));
    L.coarse_group = take(2 * (kMaxBins / 16));
    L.buf_a = take(4 * m);                                   // part1: rows; later the sorted columns of the buckets
    L.buf_b = L.two_level ? take(4 * m) : off;               // part1: columns
    L.buf_c = take(4 * m);                                   // part2: packed entries
    L.row_unique = take(4 * N);
    L.total = off + 256;
    return true;
}

}  // namespace

int64_t csr_bucketed_workspace_bytes(int64_t n_pairs, int64_t N, int add_self_loops)
{
    BucketLayout L;
    if (!make_bucket_layout(n_pairs, N, add_self_loops, L)) return -1;
    return L.total;
}

int csr_build_bucketed(int64_t n_pairs, const int32_t* d_src, const int32_t* d_dst, int64_t N, int add_self_loops,
                       int64_t* d_row_ptr, int32_t* d_col_idx, int64_t col_capacity, int64_t* h_nnz,
                       void* d_workspace, hipStream_t stream)
{
    BucketLayout L;
    if (!make_bucket_layout(n_pairs, N, add_self_loops, L)) return RETEXO_E_SIZE;
    char* ws = (char*)d_workspace;
    BucketHeader* hdr = (BucketHeader*)(ws + L.header);
    auto u32 = [&](int64_t at) { return (uint32_t*)(ws + at); };
    PlanArrays pa{u32(L.bin_off), u32(L.bucket_bin0), u32(L.bucket_off), u32(L.bucket_cursor),
                  u32(L.group_bin0), u32(L.group_off), u32(L.group_cursor), u32(L.group_tile0),
                  (uint16_t*)(ws + L.coarse_group)};

    RETEXO_HIP_TRY(hipMemsetAsync(hdr, 0, (size_t)(L.counts - L.header), stream));      // header and bin counts
    hist_kernel<<<dim3((unsigned)L.hist_blocks), dim3(kThreads), 0, stream>>>(
        n_pairs, d_src, d_dst, N, L.n_items, L.items_per_block, L.s, L.nbins, u32(L.counts), hdr);
    colsum_kernel<<<dim3((unsigned)((L.nbins + 255) / 256), kColsumSlices), dim3(256), 0, stream>>>(
        L.hist_blocks, L.nbins, u32(L.counts), u32(L.bin_count));
    plan_kernel<<<dim3(1), dim3(kThreads), 0, stream>>>(L.nbins, L.span_bins, u32(L.bin_count), pa,
                                                        (uint32_t)L.bucket_bound, hdr);
    const unsigned item_tiles = (unsigned)((L.n_items + kItemsPerTile - 1) / kItemsPerTile);
    if (L.M > 0) {
        if (L.two_level) {
            part1_kernel<<<dim3(item_tiles), dim3(kThreads), 0, stream>>>(
                n_pairs, d_src, d_dst, N, L.n_items, L.s, pa.coarse_group, pa.group_cursor, u32(L.buf_a), u32(L.buf_b), hdr);
            const unsigned tiles = (unsigned)((L.M + kTileEntries - 1) / kTileEntries + kMaxGroups);
            part2_kernel<false><<<dim3(tiles), dim3(kThreads), 0, stream>>>(
                n_pairs, d_src, d_dst, N, L.n_items, L.s, L.cbits, u32(L.buf_a), u32(L.buf_b), pa.group_off,
                pa.group_tile0, pa.bucket_bin0, pa.bucket_cursor, u32(L.buf_c), hdr);
        } else {
            part2_kernel<true><<<dim3(item_tiles), dim3(kThreads), 0, stream>>>(
                n_pairs, d_src, d_dst, N, L.n_items, L.s, L.cbits, nullptr, nullptr, pa.group_off,
                pa.group_tile0, pa.bucket_bin0, pa.bucket_cursor, u32(L.buf_c), hdr);
        }
    }
    sort_kernel<<<dim3((unsigned)L.bucket_bound), dim3(kSortThreads), 0, stream>>>(
        hdr, pa.bucket_off, pa.bucket_bin0, u32(L.buf_c), u32(L.buf_a), (int32_t*)(ws + L.row_unique),
        u32(L.bucket_total), L.cbits, L.s, N);
    total_kernel<<<dim3(1), dim3(kThreads), 0, stream>>>(hdr, u32(L.bucket_total), u32(L.bucket_out), col_capacity);
    emit_kernel<<<dim3((unsigned)L.bucket_bound), dim3(256), 0, stream>>>(
        hdr, pa.bucket_off, pa.bucket_bin0, u32(L.bucket_out), u32(L.buf_a), (const int32_t*)(ws + L.row_unique),
        L.s, N, d_row_ptr, d_col_idx);
    RETEXO_HIP_TRY(hipGetLastError());
    BucketHeader h;
    RETEXO_HIP_TRY(hipMemcpyAsync(&h, hdr, sizeof(h), hipMemcpyDeviceToHost, stream));
    RETEXO_HIP_TRY(hipStreamSynchronize(stream));
    if (h.bad_id) return RETEXO_E_CSR;
    if (h.internal) return RETEXO_E_HIP;
    if (h_nnz) *h_nnz = h.nnz;
    if (h.overflow) return RETEXO_E_CAPACITY;
    return RETEXO_OK;
}
