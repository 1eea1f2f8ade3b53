"""Plain fp64 CPU oracle of the retrieval branch's nearest-neighbour search (paper App. C: the retrieval database,
C.1 its construction, C.2 its performance).

TEST INFRASTRUCTURE ONLY, like the rest of this package.

What the paper states: every timestep of the training trajectories is stored as an L2-normalised
4352-dim visual embedding together with its payload (the action that followed); at inference the
current observation's embedding queries the database by cosine similarity and the Top-K entries'
actions become draft candidates (Sec. 4.2: Top-K instead of Top-1).  The paper searches an HNSW graph
(approximate); the exact search written here is what that approximates.

Readings (listed in the design notes):
Q1  stored vectors are bf16-valued (both sides use exactly those values); queries are fp32.
Q2  the similarity of L2-normalised vectors is their dot product; the database side is not
    re-normalised after rounding to bf16.
Q3  order: higher similarity first; equal similarities by lower database index.
"""
from typing import Tuple

import numpy as np

from .heisd_oracle import widen_bf16


def similarity_scores(db_bits: np.ndarray, queries: np.ndarray, chunk: int = 16384) -> np.ndarray:
    """scores[b][i] = <db[i], queries[b]> in fp64.  db_bits: bf16 bit patterns u16 [N, d]."""
    q = np.asarray(queries, np.float64)
    N = db_bits.shape[0]
    out = np.empty((q.shape[0], N))
    for s in range(0, N, chunk):
        out[:, s:s + chunk] = q @ widen_bf16(db_bits[s:s + chunk]).T
    return out


def top_k(scores: np.ndarray, K: int) -> Tuple[np.ndarray, np.ndarray]:
    """Indices and scores of the K largest entries of one score row, reading Q3."""
    K = min(K, len(scores))
    order = sorted(range(len(scores)), key=lambda i: (-scores[i], i)) if len(scores) <= 4096 else None
    if order is None:
        # same order without a Python-level sort of every element: candidates above the K-th value, then exact
        kth = np.partition(scores, len(scores) - K)[len(scores) - K]
        cand = np.flatnonzero(scores >= kth)
        order = sorted(cand.tolist(), key=lambda i: (-scores[i], i))
    idx = np.asarray(order[:K], np.int64)
    return idx, scores[idx]


def retrieve(db_bits: np.ndarray, queries: np.ndarray, K: int, payload: np.ndarray = None):
    """Top-K entries per query: (indices [B, K], scores [B, K], payload rows [B, K, ...] or None)."""
    sc = similarity_scores(db_bits, queries)
    idx = np.zeros((sc.shape[0], min(K, sc.shape[1])), np.int64)
    val = np.zeros(idx.shape)
    for b in range(sc.shape[0]):
        idx[b], val[b] = top_k(sc[b], K)
    return idx, val, (None if payload is None else np.asarray(payload)[idx])
