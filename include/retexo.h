/*
 * retexo.h — C ABI of the MI355X (gfx950) embed-and-aggregate library.
 *
 * The library computes the local, single-device half of one lazy
 * message-passing round (paper: section "Lazy Message Passing"): a trained
 * layer is frozen, evaluated for every node as a dense transform, and the
 * result is aggregated over the graph to become the next layer's input.
 * One round is therefore
 *        Z   = act(H W + b)                       (f of Eq. 1; identity for round 0)
 *        out = COMBINE(Z, AGGR_{u in N(v)} Z_u)   (Eq. 1; COMBINE = concatenation)
 *
 * Conventions for every entry point
 *   - Pointers named d_* are DEVICE pointers owned by the caller; h_* are host
 *     pointers.  The library never frees or keeps them, except that a plan
 *     BORROWS the CSR arrays it was created from (they must outlive it).
 *   - Matrices are fp32, row-major, with a leading dimension (ld*, in floats)
 *     that may exceed the logical width; padding columns are never written
 *     and their contents never reach an output.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     retexo_transform / retexo_aggregate / retexo_round only enqueue work:
 *     they do not allocate, free or synchronise.  retexo_csr_from_coo and
 *     retexo_plan_create synchronise the stream once; retexo_plan_create also
 *     allocates the plan's own small arrays.
 *   - Every entry point documented as "Enqueues on `stream`" only launches kernels there: no
 *     allocation, no host synchronisation, no memset or copy nodes.  A caller may therefore record
 *     a sequence of them (a round, a training step) into a HIP graph by stream capture and
 *     replay it; retexo_csr_from_coo, retexo_plan_create and retexo_partition_share synchronise
 *     and cannot be captured.
 *   - Return value 0 (RETEXO_OK) or a negative retexo_status.  Argument errors
 *     are detected before any kernel is launched, so no output byte has been
 *     written when one is returned.
 *   - Results are bitwise reproducible from call to call for the same plan:
 *     every output row is owned by one workgroup and no floating-point atomics
 *     are used.
 */
#ifndef RETEXO_H
#define RETEXO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct retexo_plan retexo_plan;

/* AGGR of Eq. 1 in the forms of the paper's three model families
 * (evaluation set-up: GCN, GraphSAGE, GAT). deg(v) is the CSR row length. */
typedef enum {
    RETEXO_MEAN = 0,        /* (1/deg v) sum_u z_u            — GraphSAGE mean       */
    RETEXO_SUM = 1,         /* sum_u z_u                                             */
    RETEXO_GCN_SYM = 2,     /* sum_u z_u / sqrt(deg v deg u)  — GCN; pass a CSR that
                               already holds one self-loop per node                  */
    RETEXO_GAT_SOFTMAX = 3, /* sum_u softmax_u(LeakyReLU(<a_src,z_u>+<a_dst,z_v>)) z_u,
                               independently for each of `heads` column blocks — GAT */
    RETEXO_MAX = 4          /* element-wise max_u z_u — the max-pooling AGGR the gloss under
                               Eq. 1 names for GraphSAGE (its pooling network is the round's
                               transform); exact in any order, so results are bit-exact     */
} retexo_mode;

enum {
    RETEXO_F_RELU = 1,         /* transform: act = ReLU (Eq. 1's f)                   */
    RETEXO_F_SELF_CONCAT = 2,  /* aggregate: out row = [ z_v | aggregate ], 2F wide   */
    RETEXO_F_VALIDATE = 4,     /* plan_create: check the CSR on the device first      */
    RETEXO_F_SAVE = 16,        /* aggregate (GAT_SOFTMAX): keep what the backward pass can
                                  reuse in the workspace (retexo_aggregate_backward_saved) */
    RETEXO_F_SPLIT_ROWS = 8    /* plan_create: always build the per-row source-range split
                                  (by default only for dense graphs too large for L2)  */
};

typedef enum {
    RETEXO_OK = 0,
    RETEXO_E_NULL = -1,       /* a required pointer is NULL                           */
    RETEXO_E_SIZE = -2,       /* negative or inconsistent size                        */
    RETEXO_E_LD = -3,         /* a leading dimension is smaller than the row width    */
    RETEXO_E_MODE = -4,       /* unknown aggregation mode                             */
    RETEXO_E_FLAGS = -5,      /* unknown or inapplicable flag bit                     */
    RETEXO_E_HEADS = -6,      /* heads < 1, heads > 8, or heads does not divide F     */
    RETEXO_E_CSR = -7,        /* node id out of range / malformed CSR                 */
    RETEXO_E_WORKSPACE = -8,  /* workspace missing or too small                       */
    RETEXO_E_ALIAS = -9,      /* output overlaps an input                             */
    RETEXO_E_HIP = -10,       /* a HIP runtime call failed                            */
    RETEXO_E_CAPACITY = -11,  /* an output array's capacity is too small              */
    RETEXO_E_PARTITION = -12  /* a node's worker id is outside [0, n_parts)           */
} retexo_status;

const char* retexo_status_string(int status);

/* ---------------------------------------------------------------------------
 * Graph construction (paper: "The graphs are undirected", section
 * "Edge-partitioned Distributed Setup").
 *
 * Builds the CSR of the undirected simple graph given by n_pairs raw pairs
 * (d_src[i], d_dst[i]): each pair with u != v yields entries (u,v) and (v,u);
 * pairs with u == v are dropped; with add_self_loops != 0 exactly one entry
 * (v,v) is added per node; repeated entries are kept once; columns ascend
 * within a row.  The result is a unique function of the pair SET.
 *
 *   d_row_ptr   [N+1] int64, written; d_row_ptr[N] = nnz
 *   d_col_idx   [col_capacity] int32, first nnz entries written
 *   h_nnz       host, optional: receives nnz
 *   d_workspace at least retexo_csr_workspace_bytes(...) bytes, 256-aligned
 * Synchronises `stream`.  Errors: RETEXO_E_CSR if any id is outside [0,N)
 * (nothing written), RETEXO_E_CAPACITY if nnz > col_capacity (nothing written;
 * *h_nnz still reports the required size), RETEXO_E_WORKSPACE, RETEXO_E_SIZE
 * (N < 0, n_pairs < 0, N >= 2^31 or 2*n_pairs + N >= 2^31).
 */
int64_t retexo_csr_workspace_bytes(int64_t n_pairs, int64_t N, int add_self_loops);
int retexo_csr_from_coo(int64_t n_pairs, const int32_t* d_src, const int32_t* d_dst,
                        int64_t N, int add_self_loops,
                        int64_t* d_row_ptr, int32_t* d_col_idx, int64_t col_capacity,
                        int64_t* h_nnz, void* d_workspace, int64_t workspace_bytes,
                        void* stream);

/* ---------------------------------------------------------------------------
 * Plan: per-graph data reused by every round — deg[v] = row length,
 * dinv[v] = 1/sqrt(deg v) (correctly rounded fp32 sqrt then divide; 0 for an
 * empty row), and the degree-ordered row schedule used for load balancing.
 * The plan borrows d_row_ptr / d_col_idx.  Synchronises `stream`.
 * With RETEXO_F_VALIDATE the CSR is checked first (row_ptr[0] == 0,
 * non-decreasing, col_idx within [0,N)); a malformed CSR gives RETEXO_E_CSR
 * and no plan.
 */
int retexo_plan_create(retexo_plan** out, int64_t N, const int64_t* d_row_ptr,
                       const int32_t* d_col_idx, unsigned flags, void* stream);
/* The same plan without any allocation and with one synchronisation instead of two, for callers that
 * build a plan per step: the caller states the entry count (retexo_csr_from_coo reports it) and supplies
 * the memory.  The plan's device arrays then live in d_workspace (retexo_plan_workspace_bytes(N, nnz, flags)
 * bytes, 256-aligned), which must stay untouched until retexo_plan_destroy; destroying such a plan frees
 * only its host structure.  RETEXO_E_CSR also when d_row_ptr[N] != nnz.  Synchronises `stream` once. */
int64_t retexo_plan_workspace_bytes(int64_t N, int64_t nnz, unsigned flags);
int retexo_plan_create_in(retexo_plan** out, int64_t N, int64_t nnz, const int64_t* d_row_ptr,
                          const int32_t* d_col_idx, unsigned flags,
                          void* d_workspace, int64_t workspace_bytes, void* stream);
int retexo_plan_destroy(retexo_plan* plan);
int64_t retexo_plan_num_nodes(const retexo_plan* plan);
int64_t retexo_plan_nnz(const retexo_plan* plan);
int32_t retexo_plan_max_degree(const retexo_plan* plan);
const int32_t* retexo_plan_deg(const retexo_plan* plan);   /* device, [N] */
const float* retexo_plan_dinv(const retexo_plan* plan);    /* device, [N] */
/* Copies the plan's arrays into caller-owned device buffers (any may be NULL):
 * d_deg int32[N], d_dinv float[N], d_order int32[N] (row ids, longest row first,
 * equal lengths in ascending id order).  Enqueued on `stream`. */
int retexo_plan_export(const retexo_plan* plan, int32_t* d_deg, float* d_dinv, int32_t* d_order,
                       void* stream);
/* The row split by source-id range that plans of dense graphs carry (built when the feature table of the
 * graph cannot stay in L2 but a range of it can, or on request with RETEXO_F_SPLIT_ROWS): the entries of
 * row order[s] whose column lies in [k*span, (k+1)*span) are col_idx[pos[k*N + s] .. pos[(k+1)*N + s]),
 * k < RETEXO_SPLIT_PARTS, s = position in the schedule order.  Returns the span (> 0), 0 when the plan
 * has no split, < 0 on error; with d_pos != NULL the int32 [(RETEXO_SPLIT_PARTS + 1) * N] positions are
 * copied there (enqueued on `stream`).  Columns of a row are expected in ascending order, as
 * retexo_csr_from_coo writes them; for any other order the positions still cut every row into
 * consecutive pieces, so aggregation results stay correct and only the locality is lost. */
#define RETEXO_SPLIT_PARTS 16
int64_t retexo_plan_export_split(const retexo_plan* plan, int32_t* d_pos, void* stream);

/* Bytes of workspace retexo_aggregate (D_in == 0) or retexo_round needs for
 * rows of width D_out; < 0 is a retexo_status. */
int64_t retexo_workspace_bytes(const retexo_plan* plan, int64_t D_out, int mode, int heads,
                               unsigned flags);

/* ---------------------------------------------------------------------------
 * Dense transform, the f of Eq. 1 (fully connected layer + optional ReLU):
 *     Z[i, j] = act( sum_k H[i, k] W[k, j] + b[j] ),   i < N, j < D_out
 *   d_H [N, ldh], first D_in columns used;  d_W [D_in, D_out] row-major, dense;
 *   d_b [D_out] or NULL;  d_Z [N, ldz], first D_out columns written.
 * fp32 inputs, fp32 matrix-core accumulation.  flags: RETEXO_F_RELU only.
 * Z must not overlap H.  N == 0 is a no-op; D_in == 0 gives Z[i, j] = act(b[j]) and reads neither H nor W
 * (both may then be NULL).
 */
int retexo_transform(int64_t N, int64_t D_in, int64_t D_out,
                     const float* d_H, int64_t ldh, const float* d_W, const float* d_b,
                     unsigned flags, float* d_Z, int64_t ldz, void* stream);

/* ---------------------------------------------------------------------------
 * Neighbourhood aggregation, the AGGR (and COMBINE) of Eq. 1, over the plan's
 * CSR.  d_Z [N, ldz], first F columns used.  Output row v is
 *     without RETEXO_F_SELF_CONCAT:  [ aggregate_v ]          (F floats)
 *     with    RETEXO_F_SELF_CONCAT:  [ z_v | aggregate_v ]    (2F floats)
 * An empty row aggregates to zeros in every mode.
 * RETEXO_GAT_SOFTMAX: F = heads * Dh; d_attn_src / d_attn_dst are [heads, Dh];
 * negative_slope is the LeakyReLU slope.  Other modes ignore those arguments
 * (heads must still be >= 1).
 * d_out must not overlap d_Z, with one exception: under RETEXO_F_SELF_CONCAT,
 * d_Z == d_out and ldz == ldo means "z_v already sits in the first F columns
 * of out"; then only the aggregate half is written.
 * d_workspace: retexo_workspace_bytes(plan, F, mode, heads, flags) bytes,
 * 256-aligned (may be NULL when that is 0).
 */
int retexo_aggregate(const retexo_plan* plan, int mode, int64_t F, int heads,
                     const float* d_Z, int64_t ldz,
                     const float* d_attn_src, const float* d_attn_dst, float negative_slope,
                     unsigned flags, float* d_out, int64_t ldo,
                     void* d_workspace, int64_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * retexo_aggregate for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results
 * and errors as retexo_aggregate, except that there is no workspace argument: the
 * aggregation's workspace (the per-node attention scores of RETEXO_GAT_SOFTMAX; the other
 * modes need none) is a fixed device array of RETEXO_NOALLOC_SCRATCH_BYTES inside the
 * library, which every GPU the library runs on holds until the process ends.
 *   - RETEXO_E_WORKSPACE if retexo_workspace_bytes(plan, F, mode, heads, 0) for a bare
 *     aggregation exceeds that size (RETEXO_GAT_SOFTMAX: more than 1,048,576 nodes with
 *     up to 4 heads, or 524,288 with 5 to 8); nothing is written.
 *   - RETEXO_F_SAVE is rejected (RETEXO_E_FLAGS): save mode hands its workspace to the
 *     backward call and needs a buffer the caller owns.
 *   - The call allocates nothing, frees nothing and does not synchronise; it only launches
 *     kernels on `stream`.  The device that is current at the call must be the plan's.
 *   - All calls on one GPU share the one array: two calls that overlap in time on the same
 *     GPU (different streams or host threads) race on it.  Calls on one stream are ordered
 *     and safe.  The array keeps the previous call's contents; nothing in it needs clearing,
 *     every entry a call reads was written by that call first.
 */
#define RETEXO_NOALLOC_SCRATCH_BYTES 33554432
int retexo_aggregate_noalloc(const retexo_plan* plan, int mode, int64_t F, int heads,
                             const float* d_Z, int64_t ldz,
                             const float* d_attn_src, const float* d_attn_dst, float negative_slope,
                             unsigned flags, float* d_out, int64_t ldo, void* stream);

/* ---------------------------------------------------------------------------
 * Backward of retexo_aggregate: the gradient of a scalar loss with respect to
 * the aggregation's inputs, given d_G = dL/d(out).  This is what training a
 * layer needs when its AGGR has trainable parameters (the gloss under Eq. 1
 * allows that; GAT's attention vectors are such parameters) and the
 * aggregation therefore sits inside the local training loop of the section
 * "Lazy Message Passing" — no message passing is involved, the inputs Z of
 * the node's neighbours were received once and stay fixed.
 *   d_G   [N, ldg]: F columns, or 2F under RETEXO_F_SELF_CONCAT (gradient of
 *         the self half first, then of the aggregate half)
 *   d_dZ  [N, lddz]: first F columns written: dL/dZ
 *   RETEXO_GAT_SOFTMAX additionally reads d_Z (the forward input), d_attn_src,
 *   d_attn_dst, negative_slope and writes d_dattn_src, d_dattn_dst ([heads, Dh],
 *   summed over the whole graph in a fixed order); F = heads * Dh <= 1024.
 *   The other modes ignore those arguments (heads >= 1).  RETEXO_MAX has no
 *   backward here (RETEXO_E_MODE).
 * PRECONDITION: the plan's CSR is structurally symmetric (u in N(v) <=> v in
 * N(u)), as retexo_csr_from_coo always builds it for the paper's undirected
 * graphs; the transposed product walks a node's own row to find the entries
 * that point at it.  A plan made from foreign, asymmetric arrays gives wrong
 * gradients (not an error).
 * d_dZ must not overlap d_G or d_Z.  d_workspace:
 * retexo_aggregate_backward_workspace_bytes(plan, mode, F, heads) bytes,
 * 256-aligned (may be NULL when that is 0).  Enqueues on `stream`; no
 * allocation, no synchronisation, no atomics (bitwise reproducible).
 */
int64_t retexo_aggregate_backward_workspace_bytes(const retexo_plan* plan, int mode, int64_t F, int heads);

/* The edge-softmax backward after a forward pass in save mode, one gather pass instead of two.
 * In a training loop the forward runs anyway: retexo_aggregate(..., flags | RETEXO_F_SAVE, ...)
 * with a workspace of retexo_workspace_bytes(plan, F, RETEXO_GAT_SOFTMAX, heads, flags |
 * RETEXO_F_SAVE) bytes additionally leaves there the attention scores, each row's softmax
 * statistics and the aggregate split into the parts that come from entries with a positive
 * and with a non-positive score (the forward output is their sum, so in save mode it can
 * differ from the plain forward's in the last bit).
 * Pass that untouched workspace as d_saved (saved_bytes = its size); everything else as in
 * retexo_aggregate_backward, same results within the same bound.  d_Z, the attention vectors
 * and negative_slope must be those of the forward call.
 * Save mode needs 16-byte aligned rows of d_Z (ldz % 4 == 0, aligned base) and a table below
 * 4 GiB; otherwise retexo_aggregate returns RETEXO_E_FLAGS and the caller uses the plain
 * backward. */
int retexo_aggregate_backward_saved(const retexo_plan* plan, int mode, int64_t F, int heads,
                                    const float* d_Z, int64_t ldz,
                                    const float* d_attn_src, const float* d_attn_dst, float negative_slope,
                                    unsigned flags, const float* d_G, int64_t ldg,
                                    const void* d_saved, int64_t saved_bytes,
                                    float* d_dZ, int64_t lddz, float* d_dattn_src, float* d_dattn_dst,
                                    void* d_workspace, int64_t workspace_bytes, void* stream);
int retexo_aggregate_backward(const retexo_plan* plan, int mode, int64_t F, int heads,
                              const float* d_Z, int64_t ldz,
                              const float* d_attn_src, const float* d_attn_dst, float negative_slope,
                              unsigned flags, const float* d_G, int64_t ldg,
                              float* d_dZ, int64_t lddz, float* d_dattn_src, float* d_dattn_dst,
                              void* d_workspace, int64_t workspace_bytes, void* stream);

/* Mean over attention heads: d_out[v, c] = (1 / heads) * sum_h d_in[v, h * C + c] for c < C.
 * The last attention round of a classifier has width heads * classes and its heads are averaged,
 * not concatenated (the standard form of the cited attention network; the paper does not say).
 * d_in [N, ldi] with ldi >= heads * C, d_out [N, ldo]; must not overlap.  Enqueues on `stream`. */
int retexo_head_mean(int64_t N, int heads, int64_t C, const float* d_in, int64_t ldi,
                     float* d_out, int64_t ldo, void* stream);

/* ---------------------------------------------------------------------------
 * One whole round: retexo_transform followed by retexo_aggregate on the same
 * stream, Z being kept in the workspace (or directly in out's first D_out
 * columns under RETEXO_F_SELF_CONCAT).  d_W == NULL means the identity
 * transform (the first round aggregates the raw features); then D_out must
 * equal D_in, d_b must be NULL and RETEXO_F_RELU is rejected.
 * flags: RETEXO_F_RELU (applies to the transform) | RETEXO_F_SELF_CONCAT.
 * d_workspace: retexo_workspace_bytes(plan, D_out, mode, heads, flags) bytes.
 */
int retexo_round(const retexo_plan* plan, int mode, int64_t D_in, int64_t D_out, int heads,
                 const float* d_H, int64_t ldh, const float* d_W, const float* d_b,
                 const float* d_attn_src, const float* d_attn_dst, float negative_slope,
                 unsigned flags, float* d_out, int64_t ldo,
                 void* d_workspace, int64_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * Local training of one layer (section "Lazy Message Passing": every layer is
 * trained by itself on its fixed aggregated inputs, with a temporary
 * classification layer on top that is discarded afterwards; the last layer is
 * the classification function itself).  This is the worker's share of one
 * training round: loss and parameter gradients over its labelled nodes.
 *
 *     A      = ReLU(X W1 + b1)        X [N, ldx] first D_in columns, W1 [D_in, H], b1 [H]
 *     logits = A Wc + bc              Wc [H, C], bc [C]
 *     loss   = mean over nodes with label >= 0 of -log softmax(logits)[label]
 * H == 0 selects the last layer: logits = X W1 + b1 with W1 [D_in, C], b1 [C];
 * d_Wc, d_bc, d_gWc, d_gbc are then ignored.
 *   d_labels [N] int32: class in [0, C) or any negative value for "not a training node"
 *   d_gW1, d_gb1, d_gWc, d_gbc: gradients, same shapes as the parameters, dense, written
 *   d_loss: one float, written
 *   d_workspace: retexo_train_workspace_bytes(N, D_in, H, C) bytes, 256-aligned
 * Enqueues on `stream`; no allocation, no synchronisation.  With no labelled
 * node the loss and all gradients are zero.  Weight gradients are summed over
 * node chunks in a fixed order (no atomics): bitwise reproducible.
 * retexo_sgd_update applies  param <- param - lr * grad  to n floats (the
 * plain SGD step; averaging gradients across workers is the caller's business).
 */
int64_t retexo_train_workspace_bytes(int64_t N, int64_t D_in, int64_t H, int64_t C);
int retexo_layer_grad(int64_t N, int64_t D_in, int64_t H, int64_t C,
                      const float* d_X, int64_t ldx, const int32_t* d_labels,
                      const float* d_W1, const float* d_b1, const float* d_Wc, const float* d_bc,
                      float* d_gW1, float* d_gb1, float* d_gWc, float* d_gbc, float* d_loss,
                      void* d_workspace, int64_t workspace_bytes, void* stream);
int retexo_sgd_update(int64_t n, float* d_param, const float* d_grad, float lr, void* stream);

/* retexo_layer_grad that also returns the gradient with respect to the layer's input,
 * d_gX [N, ldgx] (first D_in columns; zero rows for nodes that are not training nodes), when
 * d_gX is not NULL.  This is what flows back into an aggregation with trainable parameters
 * that produced X: d_gX is the d_G of retexo_aggregate_backward.  d_gX must not overlap d_X.
 * Same workspace as retexo_layer_grad. */
int retexo_layer_grad_x(int64_t N, int64_t D_in, int64_t H, int64_t C,
                        const float* d_X, int64_t ldx, const int32_t* d_labels,
                        const float* d_W1, const float* d_b1, const float* d_Wc, const float* d_bc,
                        float* d_gW1, float* d_gb1, float* d_gWc, float* d_gbc, float* d_loss,
                        float* d_gX, int64_t ldgx,
                        void* d_workspace, int64_t workspace_bytes, void* stream);

/* retexo_layer_grad_x with dropout on the hidden units (appendix on hyper-parameters: the layers are
 * trained with dropout 0.3 or 0.5; the paper does not say where it sits, here it acts on the layer's
 * output A in front of the temporary classifier):
 *     A_vj = keep_vj ? ReLU(X W1 + b1)_vj / (1 - p_drop) : 0
 * and the gradients are those of the loss under this mask.  The mask is not an argument: unit j of node v
 * is dropped when word j % 4 of the Philox-4x32-10 block with
 *     counter = (v, j / 4, low 32 bits of draw, high 32 bits of draw),  key = (low, high 32 bits of seed)
 * is below floor(p_drop * 2^32), so a caller that needs the mask (or the other workers' masks) can draw
 * it again.  `seed` names the stream, `draw` the training step; calls with the same pair use the same mask
 * (both travel by value: a HIP graph that recorded this call replays the mask it recorded).
 *   p_drop in [0, 1); 0 is exactly retexo_layer_grad_x.  RETEXO_E_SIZE if p_drop is outside that range
 *   (or not a number), or positive with H == 0 (the last layer has no hidden units).
 *   d_gX may be NULL.  Same workspace and behaviour as retexo_layer_grad otherwise. */
int retexo_layer_grad_dropout(int64_t N, int64_t D_in, int64_t H, int64_t C,
                              const float* d_X, int64_t ldx, const int32_t* d_labels,
                              const float* d_W1, const float* d_b1, const float* d_Wc, const float* d_bc,
                              float* d_gW1, float* d_gb1, float* d_gWc, float* d_gbc, float* d_loss,
                              float* d_gX, int64_t ldgx, float p_drop, uint64_t seed, uint64_t draw,
                              void* d_workspace, int64_t workspace_bytes, void* stream);

/* Parameter gradients of the dense transform Z = H W + b (the transform in front of an
 * aggregation, trained through retexo_aggregate_backward, which supplies d_dZ = dL/dZ):
 *     gW[k, j] = sum_v H[v, k] dZ[v, j]   (d_gW [D_in, D_out], dense)
 *     gb[j]    = sum_v dZ[v, j]           (d_gb [D_out], or NULL to skip)
 * Summed over node chunks in a fixed order (no atomics).  d_workspace:
 * retexo_transform_backward_workspace_bytes(N, D_in, D_out) bytes, 256-aligned.  Enqueues on `stream`. */
int64_t retexo_transform_backward_workspace_bytes(int64_t N, int64_t D_in, int64_t D_out);
int retexo_transform_backward(int64_t N, int64_t D_in, int64_t D_out,
                              const float* d_H, int64_t ldh, const float* d_dZ, int64_t lddz,
                              float* d_gW, float* d_gb,
                              void* d_workspace, int64_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * Variant: the gathered table kept in 16-bit storage.  The aggregation is bound by the bytes it
 * gathers, so a table in bfloat16 or IEEE half moves half of them.  Outside the fp32 results:
 * the stored value is the float32 value rounded to nearest even in the target format; sums are
 * still accumulated in float32, the output is float32.
 *   retexo_store_rows: d_dst[i, j] = round(d_src[i, j]) for j < F; d_dst is [N, ldd] 16-bit
 *     elements (ldd in elements).  NaN stays NaN, overflow rounds to infinity, fp16 keeps subnormals.
 *   retexo_aggregate_stored: retexo_aggregate with d_Z a stored table ([N, ldz] elements, ldz in
 *     elements); all five modes; under RETEXO_F_SELF_CONCAT the self half is the stored value
 *     widened to float32 (there is no in-place form).  16-byte aligned rows with
 *     ldz >= F rounded up to 8 take 16-byte gathers, anything else two-byte gathers.
 *     Workspace: retexo_workspace_bytes(plan, F, mode, heads, flags).
 */
typedef enum {
    RETEXO_STORE_BF16 = 1,
    RETEXO_STORE_FP16 = 2
} retexo_storage;
int retexo_store_rows(int storage, int64_t N, int64_t F, const float* d_src, int64_t lds,
                      void* d_dst, int64_t ldd, void* stream);
int retexo_aggregate_stored(const retexo_plan* plan, int mode, int storage, int64_t F, int heads,
                            const void* d_Z, int64_t ldz,
                            const float* d_attn_src, const float* d_attn_dst, float negative_slope,
                            unsigned flags, float* d_out, int64_t ldo,
                            void* d_workspace, int64_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * One worker's share of an edge-partitioned graph (section "Edge-partitioned
 * Distributed Setup": worker i holds its inner nodes V_i, the edges touching
 * an inner node and, as boundary nodes, their other endpoints) and the pack /
 * unpack of boundary rows around a round (the embedding exchange between peers
 * of the implementation section; the transport itself is not part of this
 * library).  Input: the global CSR (as retexo_csr_from_coo builds it: columns
 * ascending) and d_part [N], the worker that owns each node, values in
 * [0, n_parts), n_parts <= 64, N * (n_parts - 1) < 2^31.  Output for worker `part`:
 *   local numbering [ inner nodes, ascending global id | boundary nodes, ascending global id ]
 *   d_local_ids      [n_local]     global id of each local node, n_local = n_inner + n_halo
 *   d_local_row_ptr  [n_local + 1] int64; an inner node's row is its global row renumbered,
 *   d_local_col_idx  [nnz_local]   columns ascending; boundary rows are empty
 *   d_global_deg     [n_local]     global row length of each local node (for retexo_plan_set_degrees)
 *   d_send_ids [n_send], h_send_offsets [n_parts + 1]: local ids of the inner nodes peer q needs,
 *                    entries h_send_offsets[q] .. h_send_offsets[q+1]
 *   d_recv_ids [n_halo], h_recv_offsets [n_parts + 1]: local ids of the boundary nodes peer q owns
 *   Both lists are ascending in global id, so what worker p packs for q and what q unpacks
 *   from p line up element by element.
 *   h_sizes [4] (host): n_inner, n_halo, nnz_local, n_send — always written (unless an argument
 *   error is returned); if a capacity (local_capacity for the n_local-sized arrays,
 *   col_capacity, send_capacity) is too small, or d_local_row_ptr is NULL, the call returns
 *   RETEXO_E_CAPACITY with nothing else written: a first call with zero capacities and NULL
 *   outputs is a size query.
 * d_workspace: retexo_partition_workspace_bytes(N, n_parts, send_capacity) bytes, 256-aligned.
 * Synchronises `stream`.  Integer arithmetic only; the result is a unique function of the input.
 * Errors: RETEXO_E_PARTITION (a worker id out of range), RETEXO_E_CAPACITY, RETEXO_E_SIZE,
 * RETEXO_E_NULL, RETEXO_E_WORKSPACE, RETEXO_E_HIP.
 */
int64_t retexo_partition_workspace_bytes(int64_t n_nodes, int n_parts, int64_t send_capacity);
int retexo_partition_share(int64_t n_nodes, const int64_t* d_row_ptr, const int32_t* d_col_idx,
                           const int32_t* d_part, int n_parts, int part,
                           int64_t local_capacity, int64_t col_capacity, int64_t send_capacity,
                           int32_t* d_local_ids, int64_t* d_local_row_ptr, int32_t* d_local_col_idx,
                           int32_t* d_global_deg, int32_t* d_send_ids, int32_t* d_recv_ids,
                           int64_t* h_sizes, int64_t* h_send_offsets, int64_t* h_recv_offsets,
                           void* d_workspace, int64_t workspace_bytes, void* stream);

/* d_buf[i, 0:F] = d_H[d_ids[i], 0:F] for i < n (gather the rows a peer needs into a dense send
 * buffer) and the reverse, d_H[d_ids[i], 0:F] = d_buf[i, 0:F] (scatter received rows into the
 * boundary part of the table).  table_rows = rows of d_H; an id outside [0, table_rows) is
 * skipped.  For unpack the ids must be distinct.  Buffers must not overlap.  Enqueues on `stream`. */
int retexo_halo_pack(int64_t n, const int32_t* d_ids, int64_t table_rows, int64_t F,
                     const float* d_H, int64_t ldh, float* d_buf, int64_t ldb, void* stream);
int retexo_halo_unpack(int64_t n, const int32_t* d_ids, int64_t table_rows, int64_t F,
                       const float* d_buf, int64_t ldb, float* d_H, int64_t ldh, void* stream);

/* Replace the degrees a plan uses for scaling (mean: 1/deg; gcn_sym: dinv = 1/sqrt(deg), the
 * correctly rounded fp32 sqrt and divide) by d_deg [N].  For a worker's local graph, whose
 * boundary rows are empty: pass the d_global_deg of retexo_partition_share so that gcn_sym
 * normalises boundary neighbours by their true degree.  The schedule keeps following the
 * actual row lengths.  Enqueues on `stream`. */
int retexo_plan_set_degrees(retexo_plan* plan, const int32_t* d_deg, void* stream);

/* ---------------------------------------------------------------------------
 * The communication-efficiency analysis as host arithmetic (no GPU involved): the network data
 * volumes of the appendix "Communication-efficiency Analysis" and their ratio gamma, Eq. 2.
 * n workers, B boundary nodes per worker (retexo_partition_share reports a worker's n_halo),
 * R training rounds, H0 feature size, sum_H = H_1 + .. + H_{K-1}, sum_C = C_1 + .. + C_{K-1}
 * (added classifier layers), M model size; sizes in one common unit.
 * retexo_data_volumes writes out4 = { standard local training, lazy local training,
 * standard gradient aggregation, lazy gradient aggregation }; RETEXO_E_SIZE unless
 * n, B, H0, sum_H, sum_C >= 0 and R, M > 0.  retexo_gamma returns (out4[0] + out4[2]) /
 * (out4[1] + out4[3]), which is Eq. 2, or -1 for invalid arguments.
 */
int retexo_data_volumes(double n, double B, double R, double H0, double sum_H, double sum_C, double M,
                        double* out4);
double retexo_gamma(double B, double R, double H0, double sum_H, double sum_C, double M);

/* ---------------------------------------------------------------------------
 * Tuning knobs for experiments and tests (defaults are chosen per shape).  They are ONE set of
 * values per process, read by every launch: set them from a single thread while no other thread
 * is inside the library, and restore the default afterwards.  Production callers never need them.
 * name: "agg_slab_cols" (0 = auto), "agg_slab_major" (-1 auto / 0 / 1),
 *       "agg_heavy_degree" (rows at least this long get a whole workgroup),
 *       "agg_parts" (source-id ranges walked one after the other: -1 auto, 1 off, 2/4/8/16),
 *       "agg_narrow_heavy" (narrow slabs: rows whose share of ONE source range is at least this
 *       long get a whole workgroup; default 1024),
 *       "agg_max_vec" (cap on floats per lane per gather),
 *       "agg_gat_fast" (0: plain edge-softmax kernel), "agg_gat_flash" (0: ordinary rows read the
 *       source scores from the table instead of computing them from the gathered rows),
 *       "agg_gat_in_rows" (0: retexo_round keeps the source scores in the table even when the unused
 *       columns of its own Z rows could hold them),
 *       "agg_gat_fold" (0: retexo_round never lets its transform write those scores, as one more
 *       output column per head of a linear transform, and always runs the score kernel),
 *       "agg_wide_offsets" (1: 64-bit row offsets even for tables below 4 GiB; these four exist
 *       so that tests reach every code path),
 *       "csr_sorted_keys" (1: retexo_csr_from_coo uses its general sorted-key construction, which
 *       otherwise only graphs of more than 2^23 nodes take, instead of the bucketing one),
 *       "transform_few_blocks" (retexo_transform and the transforms inside retexo_round: a matrix
 *       with fewer 128-row blocks, times column blocks, than this takes the kernel that splits K
 *       over the waves of 32-row workgroups; default 128, 0 = never; RETEXO_E_SIZE if negative).
 * Returns RETEXO_E_FLAGS for an unknown name.
 */
int retexo_set_option(const char* name, int64_t value);

#ifdef __cplusplus
}
#endif
#endif /* RETEXO_H */
