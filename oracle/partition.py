"""CPU oracle for one worker's share of an edge-partitioned graph (test infrastructure).

Section "Edge-partitioned Distributed Setup": the nodes are split over N workers; worker i holds its
inner nodes V_i, the edges that touch an inner node, and — as boundary (halo) nodes — the other
endpoints of those edges.  Before a message-passing round each worker receives the current
representation of its boundary nodes from the workers that own them (`sync_embeddings` in the
section on implementation).  This module writes that bookkeeping out in plain numpy:

  * local numbering  [ inner nodes, ascending global id | boundary nodes, ascending global id ]
  * local CSR: one row per local node; an inner node's row is its global row with the columns
    renumbered (ascending local id), a boundary node's row is empty
  * the global degree of every local node (gcn_sym needs a boundary node's true degree)
  * per peer q: the local ids of the inner nodes q needs (send list) and of the boundary nodes
    q owns (receive list), both ascending in global id so that the two sides line up

Nothing here is shared with, or derived from, the GPU library.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np


@dataclass
class Share:
    n_inner: int
    n_halo: int
    local_ids: np.ndarray          # int32 [n_inner + n_halo]  global id of every local node
    row_ptr: np.ndarray            # int64 [n_local + 1]
    col_idx: np.ndarray            # int32 [nnz_local]         local ids
    global_deg: np.ndarray         # int32 [n_local]
    send_ids: List[np.ndarray]     # per peer: int32 local ids (inner) to send
    recv_ids: List[np.ndarray]     # per peer: int32 local ids (boundary) to receive into


def share(row_ptr, col_idx, part, n_parts: int, p: int) -> Share:
    row_ptr = np.asarray(row_ptr, np.int64)
    col_idx = np.asarray(col_idx, np.int64)
    part = np.asarray(part, np.int64)
    n = row_ptr.size - 1
    deg = np.diff(row_ptr)
    inner = np.flatnonzero(part == p)
    # entries of inner rows
    rows_of_entry = np.repeat(np.arange(n), deg)
    mine = part[rows_of_entry] == p
    cols = col_idx[mine]
    halo = np.setdiff1d(np.unique(cols), inner)              # ascending
    local_ids = np.concatenate([inner, halo])
    to_local = np.full(n, -1, np.int64)
    to_local[local_ids] = np.arange(local_ids.size)
    n_local = local_ids.size
    lrp = np.zeros(n_local + 1, np.int64)
    lrp[1:inner.size + 1] = np.cumsum(deg[inner])
    lrp[inner.size + 1:] = lrp[inner.size]
    # entries of inner rows, renumbered, ordered by (row, local column); inner rows appear in
    # ascending global id, which is also their local order
    lcols = to_local[cols]
    lci = lcols[np.lexsort((lcols, rows_of_entry[mine]))].astype(np.int32)
    send, recv = [], []
    for q in range(n_parts):
        if q == p:
            send.append(np.empty(0, np.int32))
            recv.append(np.empty(0, np.int32))
            continue
        touches_q = np.zeros(n, bool)
        touches_q[rows_of_entry[mine & (part[col_idx] == q)]] = True      # inner rows with a neighbour in V_q
        send.append(to_local[np.flatnonzero(touches_q)].astype(np.int32))
        recv.append(to_local[halo[part[halo] == q]].astype(np.int32))
    return Share(int(inner.size), int(halo.size), local_ids.astype(np.int32), lrp, lci,
                 deg[local_ids].astype(np.int32), send, recv)
