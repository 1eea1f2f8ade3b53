"""Pins of the retrieval oracle (paper App. C: C.1 database construction, C.2 performance - cosine Top-K
over L2-normalised embeddings)."""
import numpy as np

import oracle
import synth


def _bf16(a):
    return synth.f32_to_bf16_bits(np.asarray(a, np.float32))


def test_orthonormal_database_returns_the_query_components():
    d = 16
    db = _bf16(np.eye(d))                                    # exactly representable
    q = np.linspace(-1.0, 2.0, d)[None, :]
    sc = oracle.similarity_scores(db, q)
    assert np.array_equal(sc, q)
    idx, val, _ = oracle.retrieve(db, q, 3)
    assert idx[0].tolist() == [15, 14, 13] and np.array_equal(val[0], q[0, [15, 14, 13]])


def test_a_stored_vector_finds_itself_and_payload_follows():
    rng = np.random.default_rng(0)
    v = rng.normal(size=(200, 64))
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    db = _bf16(v)
    stored = synth.bf16_bits_to_f32(db).astype(np.float64)
    payload = np.arange(200 * 7).reshape(200, 7)
    q = stored[[17, 130]]
    idx, val, pay = oracle.retrieve(db, q, 5, payload)
    assert idx[:, 0].tolist() == [17, 130]
    assert np.allclose(val[:, 0], (stored[[17, 130]] ** 2).sum(1), rtol=0, atol=1e-15)     # |v|^2, close to 1
    assert np.array_equal(pay[:, 0], payload[[17, 130]])
    assert np.all(np.diff(val, axis=1) <= 0)


def test_against_scalar_loops_and_stable_argsort():
    rng = np.random.default_rng(1)
    for _ in range(20):
        N, d, B, K = int(rng.integers(1, 40)), int(rng.integers(1, 9)), int(rng.integers(1, 4)), int(rng.integers(1, 12))
        db = _bf16(rng.integers(-2, 3, (N, d)) * 0.5)                                        # many exact ties
        q = rng.integers(-2, 3, (B, d)).astype(np.float64)
        w = synth.bf16_bits_to_f32(db).astype(np.float64)
        idx, val, _ = oracle.retrieve(db, q, K)
        for b in range(B):
            sc = [sum(w[i][c] * q[b][c] for c in range(d)) for i in range(N)]
            order = np.argsort(-np.array(sc), kind="stable")[:K]                              # ties: lower index first
            assert idx[b].tolist() == order.tolist() and np.array_equal(val[b], np.array(sc)[order])


def test_large_row_takes_the_partition_route_with_the_same_order():
    rng = np.random.default_rng(2)
    sc = np.round(rng.normal(size=10000), 2)                                                  # ties guaranteed
    idx, val = oracle.top_k(sc, 25)
    ref = np.argsort(-sc, kind="stable")[:25]
    assert idx.tolist() == ref.tolist() and np.array_equal(val, sc[ref])
