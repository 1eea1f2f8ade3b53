"""The verify-skip decision kernels (paper Sec. 4.1, Alg. 1) through the C ABI against the oracle:
exported final-layer features, cosine similarities, the offline stage and the per-episode decision."""
import numpy as np
import pytest

import oracle
import synth
from helpers import oracle_model, oracle_prefix_cache

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

MID = synth.ModelShape(n_layers=3, d_model=512, n_heads=4, head_dim=128, d_ffn=1376, vocab=2048)
S_TOL = 3e-6          # fp32 sums of d products against fp64: |dS| <= ~d * 2^-24 * |terms|; measured ~1e-7


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def _dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    return (t.to(dtype) if dtype else t).to("cuda:0")


def trajectory_features(n, d, step, seed):
    """n trajectory points whose features drift like a random walk: nearby points are similar."""
    rng = np.random.default_rng(seed)
    f = np.zeros((n, d), np.float32)
    f[0] = rng.normal(size=d)
    for i in range(1, n):
        f[i] = f[i - 1] + step * rng.normal(size=d)
    return f


@pytest.mark.parametrize("n,m,d", [(37, 21, 512), (5, 300, 4096), (1, 1, 4)])
def test_similarity_matrix(n, m, d):
    import paper_2603_17573_amd as P
    _need_gpu()
    rng = np.random.default_rng(n * m)
    a, b = rng.normal(size=(n, d)).astype(np.float32), (rng.normal(size=(m, d)) + 0.5).astype(np.float32)
    if n > 2:
        a[2] = 0.0                                   # an all-zero vector: similarity 0 by definition
    S = torch.full((n, m), -7.0, device="cuda:0")
    assert P.heisd_feature_similarity(_dev(a).data_ptr(), _dev(b).data_ptr(), n, m, d, S.data_ptr(), None) == 0
    torch.cuda.synchronize()
    ref = oracle.similarity_matrix(a, b)
    assert np.abs(S.cpu().numpy() - ref).max() <= S_TOL


@pytest.mark.parametrize("n,d,step,T", [(60, 512, 0.25, 0.5), (300, 4096, 0.1, 0.8), (40, 256, 0.3, 0.97), (1, 64, 0.1, 0.5),
                                        (30, 128, 0.2, 2.0)])
def test_offline_stage(n, d, step, T):
    import paper_2603_17573_amd as P
    _need_gpu()
    f = trajectory_features(n, d, step, seed=n + d)
    S = torch.zeros((n, n), device="cuda:0")
    work = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    min_s = torch.zeros(1, device="cuda:0")
    o_dist = torch.full((1,), -5, dtype=torch.int32, device="cuda:0")
    assert P.heisd_skip_offline(_dev(f).data_ptr(), n, d, T, S.data_ptr(), work.data_ptr(), min_s.data_ptr(),
                                o_dist.data_ptr(), None) == 0
    torch.cuda.synchronize()
    Sg, ms, od = S.cpu().numpy(), float(min_s.cpu()[0]), int(o_dist.cpu()[0])
    Sr = oracle.similarity_matrix(f, f)
    assert np.abs(Sg - Sr).max() <= S_TOL
    # the reduction itself: exact given the GPU's own similarities (the algorithm's loops, literally)
    best, dist = np.inf, 0
    for i in range(n - 1):
        for dd in range(1, n - i):
            if best > Sg[i, i + dd] > np.float32(T):
                best, dist = Sg[i, i + dd], dd
    assert (ms, od) == (float(best), dist)
    # against the oracle: the same pair wherever fp32 rounding cannot change the outcome
    s_ref, d_ref = oracle.offline_stage(f, T)
    cand = np.sort(np.array([Sr[i, j] for i in range(n) for j in range(i + 1, n) if Sr[i, j] > T]))
    near_T = any(abs(Sr[i, j] - T) <= S_TOL for i in range(n) for j in range(i + 1, n))
    if len(cand) == 0:
        assert near_T or ((ms, od) == (np.inf, 0) and (s_ref, d_ref) == (np.inf, 0))
    else:
        assert abs(ms - s_ref) <= S_TOL or near_T
        if not near_T and (len(cand) == 1 or cand[1] - cand[0] > 2 * S_TOL):
            assert od == d_ref
    print("offline n=%d d=%d T=%g: min_S %.6f O_dist %d (oracle %.6f %d)" % (n, d, T, ms, od, s_ref, d_ref), flush=True)


def test_decision_and_its_mask_in_the_verify_step():
    import paper_2603_17573_amd as P
    from gpu_harness import run_gpu_step
    _need_gpu()
    B, d = 6, 512
    rng = np.random.default_rng(5)
    prev = rng.normal(size=(B, d)).astype(np.float32)
    last = (prev + np.array([0.05, 0.3, 0.05, 2.0, 0.8, 0.0])[:, None] * rng.normal(size=(B, d))).astype(np.float32)
    dist = np.array([1, 1, 4, 1, 2, 2], np.int32)
    min_s, o_dist = 0.85, 2
    skip = torch.full((B,), 9, dtype=torch.uint8, device="cuda:0")
    sim = torch.zeros(B, device="cuda:0")
    assert P.heisd_skip_decide(_dev(prev).data_ptr(), _dev(last).data_ptr(), _dev(dist).data_ptr(), B, d,
                               _dev(np.array([min_s], np.float32)).data_ptr(), _dev(np.array([o_dist], np.int32)).data_ptr(),
                               skip.data_ptr(), sim.data_ptr(), None) == 0
    torch.cuda.synchronize()
    sg, mask = sim.cpu().numpy(), skip.cpu().numpy()
    sr = np.array([oracle.cosine(prev[b], last[b]) for b in range(B)])
    assert np.abs(sg - sr).max() <= S_TOL
    assert np.array_equal(mask, oracle.skip_decision(prev, last, dist, np.float32(min_s), o_dist, similarities=sg))
    clear = np.abs(sr - min_s) > S_TOL
    assert np.array_equal(mask[clear], oracle.skip_decision(prev, last, dist, min_s, o_dist)[clear])
    assert mask.tolist() == [1, 1, 0, 0, 0, 1]            # similar & near; similar & near; too far; dissimilar; dissimilar; identical
    # the mask drives the verify step: skipped episodes keep their whole draft
    wl = synth.Workload("skipmask", MID, 0, 12, MID.bin_base, batch=B, K=7, seed=3)
    weights = synth.make_weights(wl.shape, wl.seed)
    k0, v0, f0 = zip(*[synth.make_prefix_kv_direct(wl, e, 20) for e in range(B)])
    drafts = (wl.shape.bin_base + synth.make_drafts_uniform(wl)).astype(np.int32)
    got = run_gpu_step(wl.shape, weights, np.stack(k0, axis=1), np.stack(v0, axis=1), [12] * B, list(f0), drafts,
                       oracle.AcceptRule(0, 0), mask)
    assert np.all(got["accepted_len"][mask == 1] == 7) and np.all(got["next_token"][mask == 1] == -1)
    assert np.all(got["next_token"][mask == 0] >= wl.shape.bin_base)


@pytest.mark.parametrize("path,B,K", [(0, 1, 7), (4, 3, 7), (1, 2, 5)])
def test_exported_features_are_the_lm_head_input(path, B, K):
    """After a verify step: the features of chosen rows against the oracle's final-norm hidden state."""
    from paper_2603_17573_amd import DeviceModel, Verifier, heisd_verify_set_path, heisd_export_features
    from gpu_harness import accept_desc_of, _bits_to_dev
    _need_gpu()
    wl = synth.Workload("feat", MID, 10, 9, MID.bin_base, batch=B, K=K, seed=21 + B)
    sh = wl.shape
    weights = synth.make_weights(sh, wl.seed)
    om = oracle_model(sh, weights)
    cap = wl.prefix_len + K
    kb, vb, plen, first = oracle_prefix_cache(om, wl, cap)
    drafts = (sh.bin_base + synth.make_drafts_uniform(wl)).astype(np.int32)
    rule = oracle.AcceptRule(2, 6)
    ref = oracle.verify_step(om, kb, vb, plen, first, drafts, rule)
    ver = Verifier(DeviceModel(sh, weights), B, K, cap)
    assert heisd_verify_set_path(ver.ctx, path) == 0
    kc, vc = _bits_to_dev(kb, "cuda:0"), _bits_to_dev(vb, "cuda:0")
    ver.step(kc, vc, _dev(plen), _dev(first), _dev(drafts), accept_desc_of(rule))
    feat = torch.zeros((B, sh.d_model), device="cuda:0")
    for rows in (None, np.arange(B, dtype=np.int32) % K):
        r_dev = None if rows is None else _dev(rows)
        assert heisd_export_features(ver.ctx, None if rows is None else r_dev.data_ptr(), K, B, feat.data_ptr(), None) == 0
        torch.cuda.synchronize()
        want = np.stack([ref["feat"][b, K - 1 if rows is None else rows[b]] for b in range(B)])
        err = np.abs(feat.cpu().numpy() - want).max() / np.abs(want).max()
        print("features path %d rows %s: max error %.3g of the largest feature" % (path, rows, err), flush=True)
        assert err <= 1e-4
        assert np.allclose(oracle.final_features(om, want * 0 + 1.0), np.ones_like(want) / np.sqrt(1 + sh.rms_eps))
    ver.close()


def test_argument_errors():
    import paper_2603_17573_amd as P
    _need_gpu()
    f = torch.zeros((4, 64), device="cuda:0")
    S = torch.zeros((4, 4), device="cuda:0")
    B_ = P.binding
    assert P.heisd_feature_similarity(None, f.data_ptr(), 4, 4, 64, S.data_ptr(), None) == B_.HEISD_EINVAL
    assert P.heisd_feature_similarity(f.data_ptr(), f.data_ptr(), 4, 4, 63, S.data_ptr(), None) == B_.HEISD_EINVAL
    assert P.heisd_feature_similarity(f.data_ptr(), f.data_ptr(), 0, 4, 64, S.data_ptr(), None) == B_.HEISD_EINVAL
    assert P.heisd_feature_similarity(f.data_ptr() + 4, f.data_ptr(), 3, 4, 64, S.data_ptr(), None) == B_.HEISD_EINVAL
    assert P.heisd_skip_offline(f.data_ptr(), 4, 64, 0.5, None, None, S.data_ptr(), S.data_ptr(), None) == B_.HEISD_EINVAL
    assert P.heisd_skip_decide(f.data_ptr(), f.data_ptr(), None, 4, 64, S.data_ptr(), S.data_ptr(), S.data_ptr(), None,
                               None) == B_.HEISD_EINVAL
