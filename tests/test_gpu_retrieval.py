"""heisd_retrieve_topk through the C ABI against the oracle's exact search (paper App. C: C.1 database
construction, C.2 performance - cosine Top-K over L2-normalised embeddings; Sec. 4.2: Top-K instead of
Top-1), on seeded synthetic databases."""
import time

import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

SCORE_TOL = 1e-5      # fp32 sums of d products of unit-vector components against fp64; measured ~1e-7


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def gpu_retrieve(db, q, K, payload=None):
    import paper_2603_17573_amd as P
    dev = "cuda:0"
    N, d = db.shape
    B = q.shape[0]
    t_db = torch.from_numpy(db.view(np.int16)).to(dev)
    t_q = torch.from_numpy(np.ascontiguousarray(q, np.float32)).to(dev)
    nbytes = P.heisd_retrieve_workspace_bytes(N, B, K)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    idx = torch.full((B, K), -9, dtype=torch.int32, device=dev)
    val = torch.zeros((B, K), device=dev)
    t_pay = out_pay = None
    if payload is not None:
        t_pay = torch.from_numpy(np.ascontiguousarray(payload, np.int32)).to(dev)
        out_pay = torch.full((B, K, payload.shape[1]), -9, dtype=torch.int32, device=dev)
    rc = P.heisd_retrieve_topk(t_db.data_ptr(), N, d, t_q.data_ptr(), B, K,
                               None if t_pay is None else t_pay.data_ptr(), 0 if payload is None else payload.shape[1],
                               idx.data_ptr(), val.data_ptr(), None if out_pay is None else out_pay.data_ptr(),
                               ws.data_ptr(), nbytes, None)
    assert rc == 0, P.heisd_last_error(None)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), val.cpu().numpy(), (None if out_pay is None else out_pay.cpu().numpy())


def check_against_oracle(db, q, K, payload, idx, val, pay):
    N = db.shape[0]
    sc = oracle.similarity_scores(db, q)
    exact_rows = 0
    for b in range(q.shape[0]):
        ridx, rval = oracle.top_k(sc[b], K + 1)
        n = min(K, N)
        assert np.all(idx[b, n:] == -1) and np.all(np.isneginf(val[b, n:]))
        got_i, got_v = idx[b, :n], val[b, :n].astype(np.float64)
        assert len(set(got_i.tolist())) == n and got_i.min() >= 0 and got_i.max() < N
        assert np.abs(got_v - sc[b][got_i]).max() <= SCORE_TOL            # each score is that entry's similarity
        assert np.abs(got_v - rval[:n]).max() <= SCORE_TOL                # and the k-th best value is right
        assert np.all(np.diff(got_v) <= 0)
        same = got_v[1:] == got_v[:-1]
        assert np.all(got_i[1:][same] > got_i[:-1][same])                 # equal similarities: lower index first
        gaps = np.abs(np.diff(rval))                                      # neighbours in the oracle's order
        for k in range(n):
            clear = (k == 0 or gaps[k - 1] > 2 * SCORE_TOL) and (k >= len(gaps) or gaps[k] > 2 * SCORE_TOL)
            if clear:
                assert got_i[k] == ridx[k]
        exact_rows += int(np.array_equal(got_i, ridx[:n]))
        if payload is not None:
            assert np.array_equal(pay[b, :n], payload[got_i]) and np.all(pay[b, n:] == -1)
    return exact_rows


@pytest.mark.parametrize("N,d,B,K", [(1000, 64, 1, 8), (4097, 256, 3, 1), (2049, 4352, 5, 16), (300, 128, 8, 64),
                                     (5, 64, 2, 8), (1, 4, 1, 1), (6001, 100, 4, 7)])
def test_small_databases(N, d, B, K):
    _need_gpu()
    db, payload = synth.make_retrieval_db(N, d, seed=N + d)
    q = synth.make_retrieval_queries(db, B, noise=0.5, seed=K)
    idx, val, pay = gpu_retrieve(db, q, K, payload)
    exact = check_against_oracle(db, q, K, payload, idx, val, pay)
    print("N=%d d=%d B=%d K=%d: %d of %d index rows identical to the oracle's" % (N, d, B, K, exact, B), flush=True)
    assert idx[0, 0] == 13 % N                                            # the stored vector the query was made from


def test_duplicate_entries_come_in_index_order():
    _need_gpu()
    db, _ = synth.make_retrieval_db(500, 64, seed=3)
    db[100] = db[7]
    db[333] = db[7]
    q = synth.bf16_bits_to_f32(db[[7]]).astype(np.float32)
    idx, val, _ = gpu_retrieve(db, q, 4)
    assert idx[0, :3].tolist() == [7, 100, 333] and val[0, 0] == val[0, 1] == val[0, 2]
    check_against_oracle(db, q, 4, None, idx, val, None)


def test_paper_sized_database():
    """273,465 entries of 4352 dimensions (2.4 GB in bf16), two queries, Top-8."""
    _need_gpu()
    t0 = time.time()
    db, payload = synth.make_retrieval_db(273465, 4352, seed=1)
    q = synth.make_retrieval_queries(db, 2, noise=0.7, seed=2)
    print("database drawn in %.1f s" % (time.time() - t0), flush=True)
    idx, val, pay = gpu_retrieve(db, q, 8, payload)
    t0 = time.time()
    exact = check_against_oracle(db, q, 8, payload, idx, val, pay)
    print("oracle search in %.1f s; %d of 2 index rows identical; top scores %s" % (time.time() - t0, exact,
                                                                                  np.round(val[:, :3], 4).tolist()), flush=True)
    assert idx[:, 0].tolist() == [13, 7932]


def test_argument_errors():
    import paper_2603_17573_amd as P
    _need_gpu()
    B_ = P.binding
    x = torch.zeros(4096, dtype=torch.int16, device="cuda:0")
    q = torch.zeros(64, device="cuda:0")
    o = torch.zeros(64, dtype=torch.int32, device="cuda:0")
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")

    def call(db=x.data_ptr(), N=64, d=64, K=8, wsb=1 << 20, pay=None, tp=None):
        return P.heisd_retrieve_topk(db, N, d, q.data_ptr(), 1, K, pay, 7, o.data_ptr(), q.data_ptr(), tp, ws.data_ptr(), wsb, None)

    assert call(db=None) == B_.HEISD_EINVAL and call(K=65) == B_.HEISD_EINVAL and call(K=0) == B_.HEISD_EINVAL
    assert call(d=62) == B_.HEISD_EINVAL and call(N=0) == B_.HEISD_EINVAL
    assert call(pay=o.data_ptr()) == B_.HEISD_EINVAL                      # payload without an output for it
    assert call(wsb=16) == B_.HEISD_ENOMEM
    assert P.heisd_retrieve_workspace_bytes(0, 1, 8) == 0 and P.heisd_retrieve_workspace_bytes(100, 1, 65) == 0
    assert call() == B_.HEISD_OK
    torch.cuda.synchronize()
