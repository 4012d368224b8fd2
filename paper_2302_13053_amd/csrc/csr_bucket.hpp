// Internal interface of the bucketing CSR construction (see csr_bucket.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// Workspace the bucketing construction needs, or -1 when it does not apply to this size
// (more than 2^23 nodes, or more entries than its two bucket levels hold): the caller then
// uses the general sorted-key construction.
int64_t csr_bucketed_workspace_bytes(int64_t n_pairs, int64_t N, int add_self_loops);

// Same contract as retexo_csr_from_coo (arguments already checked, workspace large enough and
// 256-aligned).  Synchronises `stream` once.
int csr_build_bucketed(int64_t n_pairs, const int32_t* d_src, const int32_t* d_dst, int64_t N, int add_self_loops,
                       int64_t* d_row_ptr, int32_t* d_col_idx, int64_t col_capacity, int64_t* h_nnz,
                       void* d_workspace, hipStream_t stream);
