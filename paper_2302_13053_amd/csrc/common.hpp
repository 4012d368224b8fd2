// Shared declarations of the gfx950 embed-and-aggregate library (internal).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "retexo.h"

#define RETEXO_HIP_TRY(expr)                         \
    do {                                             \
        hipError_t _e = (expr);                      \
        if (_e != hipSuccess) return RETEXO_E_HIP;   \
    } while (0)

constexpr int kWave = 64;          // CDNA wavefront width
constexpr int kMaxHeads = 8;       // attention heads supported by the edge-softmax kernel
constexpr int kMaxParts = 16;      // source-id ranges a row can be split into

// Per-graph data.  deg/dinv/order are device arrays owned by the plan; the CSR
// arrays are borrowed from the caller.
struct retexo_plan {
    int64_t N = 0;
    int64_t nnz = 0;
    const int64_t* row_ptr = nullptr;
    const int32_t* col_idx = nullptr;
    int32_t* deg = nullptr;       // [N]
    float* dinv = nullptr;        // [N]
    int32_t* order = nullptr;     // [N] row ids, longest rows first (ties: ascending id)
    // [kMaxParts + 1][N] CSR positions splitting every row by source-id range, stored in
    // SCHEDULE order (index = position in `order`, not row id) so that the rows a wave works
    // on read neighbouring entries: the entries of row order[s] with column in
    // [k*part_span, (k+1)*part_span) are col_idx[part_ptr[k*N + s] .. part_ptr[(k+1)*N + s]).
    // NULL when not built.
    int32_t* part_ptr = nullptr;
    int64_t part_span = 0;
    int32_t max_degree = 0;
    // number of rows with deg >= threshold[i], thresholds fixed in plan.hip
    int64_t rows_at_least[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    void* block = nullptr;          // the one device allocation behind deg, dinv, order, part_ptr
    void* build_scratch = nullptr;
};

constexpr int kPlanThresholds[8] = {1, 256, 512, 1024, 2048, 4096, 8192, 16384};

struct AggOptions {
    int64_t slab_cols = 0;      // 0 = auto
    int64_t slab_major = -1;    // -1 = auto
    int64_t heavy_degree = 2048;
    int64_t max_vec = 4;        // cap on floats per lane per gather (experiments)
    int64_t gat_fast = 1;       // pipelined edge-softmax kernel (0: the plain one)
    int64_t gat_flash = 1;      // ordinary rows: source scores from the gathered rows (0: from the table)
    int64_t gat_fold = 1;       // retexo_round: source scores as extra output columns of a linear transform (0: score kernel)
    int64_t gat_in_rows = 1;    // retexo_round: source scores in the unused columns of its own Z rows (0: table)
    int64_t wide_offsets = 0;   // 1: use the 64-bit row-offset code paths even when 32 bits would do (tests)
    int64_t narrow_heavy = 1024;  // narrow slabs: rows whose share of one source range is at least this long get a workgroup
    int64_t parts = -1;         // source-id ranges per aggregation: -1 auto, 1 = off, 2/4/8/16
    int64_t few_blocks = 128;   // dense transform: fewer 128-row blocks (times column blocks) than this take the few-rows kernel; 0 = never
    int64_t csr_sorted_keys = 0;  // 1: retexo_csr_from_coo always takes the sorted-key construction (tests)
};
AggOptions& agg_options();

// Zero `bytes` (a multiple of 4) at `p` with a small kernel.  The stream-ordered entry points use this
// instead of memset nodes so that a caller can record them into a HIP graph.
int launch_zero(void* p, size_t bytes, hipStream_t stream);

// internal launchers (no argument validation; the C entry points did it)
int launch_transform(int64_t N, int64_t D_in, int64_t D_out, const float* H, int64_t ldh,
                     const float* W, const float* b, bool relu, float* Z, int64_t ldz,
                     hipStream_t stream, const float* mask = nullptr, int64_t ldm = 0);

struct AggCall {
    const retexo_plan* plan;
    int mode;
    int64_t F;
    int heads;
    const float* Z;
    int64_t ldz;
    const float* attn_src;
    const float* attn_dst;
    float slope;
    bool self_concat;
    bool copy_self;       // false when Z already sits in out's first F columns
    float* out;
    int64_t ldo;
    void* workspace;
    bool save = false;    // edge softmax: keep the backward's statistics in the workspace
    bool z_padding_free = false;   // Z is the library's own buffer: columns [F, ldz) of its rows may be written
    bool el_ready = false;         // ... and columns [F, F + heads_padded) already hold <a_src, z_v> (see gat_fold_plan)
};
int launch_aggregate(const AggCall& c, hipStream_t stream);
// Edge softmax inside a round whose transform is linear: <a_src, z_v> = h_v (W a_src) + <b, a_src> is one more
// output column per head of the same product, so the transform can write the source scores behind the F
// columns of its own rows at no cost and no score kernel has to read Z again.  gat_fold_plan says whether the
// aggregation of `c` (Z, ldz, z_padding_free set as the round will set them) would use scores kept there and
// `avail_bytes` of scratch hold the widened operands; launch_gat_fold then writes W2 = [W | W A] as
// [D_in, F + heads_padded] and b2 = [b | b A] right behind it.  The caller runs the transform with W2, b2 and
// F + heads_padded output columns and sets c.el_ready.
bool gat_fold_plan(const AggCall& c, int64_t D_in, int64_t avail_bytes);
void launch_gat_fold(int64_t D_in, int64_t F, int heads, const float* W, const float* b, const float* a_src,
                     float* W2, float* b2, hipStream_t stream);
// edge-softmax workspace: scores, then (save) the row statistics and the aggregate split by the sign of the score
struct GatWorkspace { int64_t el, er, stats, pos, neg, total, ld_pos; };
GatWorkspace gat_workspace(int64_t N, int64_t F, int heads, bool save);
int64_t aggregate_workspace_bytes(int64_t N, int mode, int heads, int64_t F = 0, bool save = false);
// el[v,h] = <a_src[h], z_v,h>, er[v,h] = <a_dst[h], z_v,h>, both [N, heads_padded(heads)]
// (el_stride: floats between the el entries of consecutive nodes; 0 = heads_padded(heads), the dense table)
void launch_gat_scores(int64_t N, int64_t F, int heads, const float* Z, int64_t ldz,
                       const float* a_src, const float* a_dst, float* el, float* er, hipStream_t stream,
                       int64_t el_stride = 0);

// Aggregation over a table in 16-bit storage (see retexo_aggregate_stored)
struct StoredCall {
    const retexo_plan* plan;
    int mode;
    int storage;           // RETEXO_STORE_*
    int64_t F;
    int heads;
    const void* Z;         // [N, ldz] 16-bit elements
    int64_t ldz;           // in elements
    const float* attn_src;
    const float* attn_dst;
    float slope;
    bool self_concat;
    bool copy_self;
    float* out;
    int64_t ldo;
    void* workspace;
};
int launch_aggregate_stored(const StoredCall& c, hipStream_t stream);
int launch_store_rows(int storage, int64_t N, int64_t F, const float* src, int64_t lds, void* dst, int64_t ldd,
                      hipStream_t stream);

// Backward of the aggregation (see retexo_aggregate_backward)
struct AggBackwardCall {
    const retexo_plan* plan;
    int mode;
    int64_t F;
    int heads;
    const float* Z;        // forward input (edge softmax only)
    int64_t ldz;
    const float* attn_src;
    const float* attn_dst;
    float slope;
    bool self_concat;      // G is [N, 2F]: gradient of the self half, then of the aggregate
    const float* G;
    int64_t ldg;
    float* dZ;
    int64_t lddz;
    float* d_attn_src;
    float* d_attn_dst;
    void* workspace;
    // edge softmax after a forward pass in save mode: that pass's workspace (else NULL)
    const void* saved = nullptr;
};
int launch_aggregate_backward(const AggBackwardCall& c, hipStream_t stream);
int64_t aggregate_backward_workspace_bytes(int64_t N, int mode, int64_t F, int heads);
constexpr int64_t kMaxBackwardSoftmaxWidth = 1024;   // heads * Dh the edge-softmax backward handles

// per-node score arrays are padded to 4 or 8 heads (padded heads hold zeros and are never selected)
static inline int heads_padded(int heads) { return heads <= 4 ? 4 : 8; }
static inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
