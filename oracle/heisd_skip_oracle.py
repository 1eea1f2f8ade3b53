"""Plain fp64 CPU oracle of the verify-skip DECISION (paper Sec. 4.1, Alg. 1).

TEST INFRASTRUCTURE ONLY, like the rest of this package.

What the paper states: the input features of the final (`lm_head`) layer are captured while a draft
is verified; on the historical trajectories the feature similarity S of every pair of trajectory
points is computed and "the minimum acceptable similarity" min_S with "its corresponding point
distance" O_dist are collected (offline stage of Alg. 1: for every point i and distance d, if
min_S > S(Feat_i, Feat_{i+d}) > T then min_S, O_dist <- S, d); on a new task these two numbers decide
which trajectory points are so similar that their verification is skipped; after every task they are
nudged up or down by the task's success signal.

Readings where the paper is silent or garbled (listed in the design notes):

S1  the feature of a trajectory point is the final-norm hidden state (the LM head's input) of one row
    of that point's verify forward; by default the last row.
S2  S is the cosine similarity.
S3  offline stage: min_S starts at +infinity (the printed start value 0 could never be undercut by a
    similarity above a boundary T >= 0); d runs over 1 .. n-i; a tie keeps the pair found first in
    loop order (i ascending, then d ascending).  No pair above T: min_S = +infinity, O_dist = 0.
S4  online decision for a point that lies `dist` points after the last verified point: skip iff
    dist <= O_dist and S(feature of the verified point before the last, feature of the last verified
    point) >= min_S.  (Features exist only for verified points, so the rule can only look back.)
S5  the adaptive update of min_S and O_dist from task feedback is scalar host logic whose step sizes
    the paper does not give; it is not part of this path.
"""
from typing import Sequence, Tuple

import numpy as np


def final_features(model, x_last: np.ndarray) -> np.ndarray:
    """S1: RMSNorm of the residual stream after the last layer with the final gain (fp64)."""
    from .heisd_oracle import rmsnorm
    return rmsnorm(np.asarray(x_last, np.float64), model.weights["final_norm"], model.rms_eps)


def cosine(a: np.ndarray, b: np.ndarray) -> float:
    """S2: <a, b> / (|a| |b|); 0 if either vector is all zero."""
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    na, nb = np.sqrt(np.dot(a, a)), np.sqrt(np.dot(b, b))
    if na == 0.0 or nb == 0.0:
        return 0.0
    return float(np.dot(a, b) / (na * nb))


def similarity_matrix(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """S[i][j] = cosine(a[i], b[j])."""
    return np.array([[cosine(x, y) for y in b] for x in a])


def offline_stage(feats: np.ndarray, T: float) -> Tuple[float, int]:
    """Alg. 1, offline stage, reading S3: the smallest similarity above T over all pairs of trajectory
    points (i, i+d) and the distance d at which it occurs."""
    n = len(feats)
    min_s, o_dist = np.inf, 0
    for i in range(n - 1):
        for d in range(1, n - i):
            s = cosine(feats[i], feats[i + d])
            if min_s > s > T:
                min_s, o_dist = s, d
    return float(min_s), int(o_dist)


def skip_decision(feat_prev: np.ndarray, feat_last: np.ndarray, dist: Sequence[int], min_s: float,
                  o_dist: int, similarities=None) -> np.ndarray:
    """Reading S4, per episode.  `similarities` overrides the computed S (to judge a decision on
    similarities computed elsewhere)."""
    B = len(dist)
    out = np.zeros(B, np.uint8)
    for b in range(B):
        s = cosine(feat_prev[b], feat_last[b]) if similarities is None else float(similarities[b])
        out[b] = 1 if (int(dist[b]) <= o_dist and s >= min_s) else 0
    return out
