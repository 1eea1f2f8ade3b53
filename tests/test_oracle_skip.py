"""Pins of the verify-skip decision oracle (paper Sec. 4.1, Alg. 1): closed forms of the similarity,
a hand-worked offline stage, a vectorised second formulation, the decision's truth table."""
import numpy as np
import pytest

import oracle
from oracle import cosine, similarity_matrix, offline_stage, skip_decision
from test_oracle_forward import float_model


def test_cosine_closed_forms():
    e = np.eye(4)
    assert cosine(e[0], e[0]) == 1.0 and cosine(e[0], e[1]) == 0.0 and cosine(e[0], -e[0]) == -1.0
    assert cosine(e[0], np.zeros(4)) == 0.0
    a = np.array([3.0, 4.0, 0.0, 0.0])
    b = np.array([4.0, 3.0, 0.0, 0.0])
    assert abs(cosine(a, b) - 24.0 / 25.0) < 1e-15                    # 3-4-5 triangle
    assert abs(cosine(5 * a, 0.1 * b) - 24.0 / 25.0) < 1e-15          # scale invariant
    ang = 0.3
    assert abs(cosine([1, 0], [np.cos(ang), np.sin(ang)]) - np.cos(ang)) < 1e-15
    rng = np.random.default_rng(0)
    x, y = rng.normal(size=(5, 33)), rng.normal(size=(7, 33))
    ref = (x / np.linalg.norm(x, axis=1, keepdims=True)) @ (y / np.linalg.norm(y, axis=1, keepdims=True)).T
    assert np.allclose(similarity_matrix(x, y), ref, rtol=0, atol=1e-14)


def test_offline_stage_hand_worked():
    """Points on the unit circle at angles 0, 10, 25, 70 degrees: pair similarities are the cosines of
    10, 25, 70 / 15, 60 / 45 degrees.  Above T = 0.6 lie cos10, cos25, cos15, cos45 = 0.7071 (pairs
    (0,1), (0,2), (1,2), (2,3)); the smallest is cos45 at distance 1.  With T = 0.75: cos25 = 0.9063 at
    distance 2.  With T = 0.99: nothing qualifies."""
    deg = np.deg2rad([0.0, 10.0, 25.0, 70.0])
    f = np.stack([np.cos(deg), np.sin(deg)], axis=1)
    s, d = offline_stage(f, 0.6)
    assert abs(s - np.cos(np.deg2rad(45.0))) < 1e-15 and d == 1
    s, d = offline_stage(f, 0.75)
    assert abs(s - np.cos(np.deg2rad(25.0))) < 1e-15 and d == 2
    assert offline_stage(f, 0.99) == (np.inf, 0)
    assert offline_stage(f[:1], 0.0) == (np.inf, 0)


def test_offline_stage_against_vectorised_formulation():
    rng = np.random.default_rng(4)
    for trial in range(50):
        n, dim = int(rng.integers(2, 12)), int(rng.integers(2, 9))
        f = rng.normal(size=(n, dim)) + 2.0
        T = float(rng.uniform(0.0, 0.9))
        S = similarity_matrix(f, f)
        iu = [(S[i, j], i, j - i) for i in range(n) for j in range(i + 1, n) if S[i, j] > T]
        if iu:
            s_ref, _, d_ref = min(iu)            # smallest similarity, then smallest i, then smallest d
            assert offline_stage(f, T) == (s_ref, d_ref)
        else:
            assert offline_stage(f, T) == (np.inf, 0)


def test_tie_keeps_the_first_pair_in_loop_order():
    f = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 0.0], [0.0, 1.0]])        # S = 1 at distance 2 for (0,2), (1,3)
    assert offline_stage(f, 0.5) == (1.0, 2)
    g = np.array([[1.0, 1.0], [1.0, 0.0], [0.0, 1.0]])                    # S(0,1) = S(0,2) = 0.7071, S(1,2) = 0
    s, d = offline_stage(g, 0.1)
    assert abs(s - np.sqrt(0.5)) < 1e-15 and d == 1


def test_decision_truth_table():
    a = np.array([[1.0, 0.0], [1.0, 0.0], [1.0, 0.0], [1.0, 0.0]])
    b = np.array([[1.0, 0.0], [1.0, 1.0], [1.0, 0.0], [0.0, 1.0]])
    # similarities 1, 0.7071, 1, 0; distances 1, 1, 3, 1; min_S 0.7, O_dist 2
    assert skip_decision(a, b, [1, 1, 3, 1], 0.7, 2).tolist() == [1, 1, 0, 0]
    assert skip_decision(a, b, [1, 1, 3, 1], np.inf, 0).tolist() == [0, 0, 0, 0]       # nothing learnt: never skip
    assert skip_decision(a, b, [2, 2, 2, 2], -1.0, 2).tolist() == [1, 1, 1, 1]
    assert skip_decision(a, b, [1, 1, 1, 1], 0.7, 2, similarities=[0.0, 0.0, 0.7, 0.69]).tolist() == [0, 0, 1, 0]


def test_features_are_the_lm_head_input():
    m = float_model(1, 8, 2, 4, 12, n_bins=4, seed=3)
    rng = np.random.default_rng(1)
    x = rng.normal(size=(1, 3, 8))
    out = oracle.forward_block(m, x, [0])
    # logits = W_lm[bins] . feat: the features are what the head multiplies
    w = m.weights["lm_head"][m.bin_base:m.bin_base + m.n_bins]
    assert np.allclose(out["feat"][0] @ w.T, out["logits"][0], rtol=0, atol=1e-12)
    # zero-layer closed form: feat = RMSNorm(x) * gain
    m0 = float_model(1, 8, 2, 4, 12, n_bins=4, seed=3)
    for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
        m0.weights[k] = [np.zeros_like(m0.weights[k][0])]
    f0 = oracle.forward_block(m0, x, [0])["feat"]
    assert np.allclose(f0, oracle.final_features(m0, x), rtol=0, atol=1e-14)
    assert np.allclose(oracle.final_features(m0, x), x / np.sqrt((x * x).mean(-1, keepdims=True) + m0.rms_eps)
                       * m0.weights["final_norm"], rtol=0, atol=1e-14)
