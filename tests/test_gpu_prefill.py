"""heisd_prefill_chunk through the C ABI against the oracle: chunked prefill of a vision+text prefix
(App. A.1: visual tokens as embeddings, the prompt as token ids) and the autoregressive decode step
(Eq. 2-1; Sec. 4.2: what the method falls back to when every candidate is rejected)."""
import numpy as np
import pytest

import oracle
import synth
from helpers import oracle_model, oracle_chunked_prefill, prefix_embeddings

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

MID = synth.ModelShape(n_layers=3, d_model=512, n_heads=4, head_dim=128, d_ffn=1376, vocab=2048)
SMALL64 = synth.ModelShape(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=1024)
LOGIT_TOL = 3e-2


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def _kv_tolerance_ok(after_bits, ref, name):
    """Rows written by the GPU against the oracle's fp64 rows: half a bf16 ulp + arithmetic error."""
    L = ref.shape[0]
    a = synth.bf16_bits_to_f32(after_bits).astype(np.float64)
    scale = np.abs(ref).reshape(L, -1).max(axis=1)
    e = np.abs(a - ref) - np.abs(ref) * 2.0 ** -8
    rel = e.reshape(L, -1).max(axis=1) / scale
    assert np.all(rel <= 5e-5 + 2e-5 * np.arange(L)), "%s rows off: %s" % (name, np.array2string(rel, precision=5))
    return float(rel.max())


def chunk_inputs(wl, episodes, p, n, dev="cuda:0"):
    """Rows p .. p+n-1 of the episodes' prefixes as the call takes them: embeddings inside the visual
    part, token ids inside the text part."""
    inputs = [synth.make_prefix_inputs(wl, e) for e in episodes]
    if p + n <= wl.n_visual:
        x = np.stack([emb[p:p + n] for emb, _ in inputs]).astype(np.float32)
        return {"x_rows": torch.from_numpy(x).to(dev)}
    if p >= wl.n_visual:
        ids = np.stack([t[p - wl.n_visual:p - wl.n_visual + n] for _, t in inputs]).astype(np.int32)
        return {"token_ids": torch.from_numpy(ids).to(dev)}
    # the chunk straddles the boundary: both inputs, id -1 marks a row that takes its embedding; the
    # embedding rows of the looked-up tokens are NaN (they must not be read)
    nv = wl.n_visual - p
    x = np.full((len(inputs), n, wl.shape.d_model), np.nan, np.float32)
    ids = np.full((len(inputs), n), -1, np.int32)
    for i, (emb, t) in enumerate(inputs):
        x[i, :nv] = emb[p:]
        ids[i, nv:] = t[:n - nv]
    return {"x_rows": torch.from_numpy(x).to(dev), "token_ids": torch.from_numpy(ids).to(dev)}


def gpu_chunked_prefill(ver, wl, episodes, chunks, cap, dev="cuda:0"):
    """The whole prefix on the GPU, every chunk on top of the GPU's own earlier rows."""
    B = len(episodes)
    kc, vc = ver.new_cache(B)
    plen = torch.zeros(B, dtype=torch.int32, device=dev)
    p, out = 0, None
    for n in chunks:
        out = ver.prefill_chunk(kc, vc, plen, want_logits=True, **chunk_inputs(wl, episodes, p, n, dev))
        p += n
        plen += n
    torch.cuda.synchronize()
    return kc, vc, {k: v.cpu().numpy() for k, v in out.items()}


def check_logits(got_logits, got_bin, ref_logits, ref_bin):
    rng_ = ref_logits.max() - ref_logits.min()
    err = np.abs(np.asarray(got_logits, np.float64) - ref_logits).max() / rng_
    assert err <= LOGIT_TOL, "logit error %.3g of the row range" % err
    srt = np.sort(ref_logits)
    if (srt[-1] - srt[-2]) / rng_ > LOGIT_TOL:
        assert got_bin == ref_bin
    return float(err)


def check_chunks_in_isolation(ver, wl, episodes, refs, cap, dev="cuda:0"):
    """Every chunk on the GPU on top of the ORACLE's bf16 cache of the earlier chunks (the same bytes on
    both sides, as in the verify-step tests): new rows to the cache bar, everything else untouched."""
    from gpu_harness import _bits_to_dev, _dev_to_bits
    worst = 0.0
    n_chunks = len(refs[0][2])
    for c in range(n_chunks):
        p, n = refs[0][2][c]["p"], refs[0][2][c]["n"]
        k0 = np.concatenate([r[2][c]["k_before"] for r in refs], axis=1)
        v0 = np.concatenate([r[2][c]["v_before"] for r in refs], axis=1)
        kc, vc = _bits_to_dev(k0, dev), _bits_to_dev(v0, dev)
        plen = torch.full((len(episodes),), p, dtype=torch.int32, device=dev)
        out = ver.prefill_chunk(kc, vc, plen, want_logits=True, **chunk_inputs(wl, episodes, p, n, dev))
        torch.cuda.synchronize()
        kg, vg = _dev_to_bits(kc), _dev_to_bits(vc)
        gl, gb = out["last_logits"].cpu().numpy(), out["next_bin"].cpu().numpy()
        for i in range(len(episodes)):
            rec = refs[i][2][c]
            for got, before, new, nm in ((kg, k0, rec["k_new"], "k"), (vg, v0, rec["v_new"], "v")):
                assert np.array_equal(got[:, i, :, :p], before[:, i, :, :p]), "earlier %s rows modified" % nm
                assert np.array_equal(got[:, i, :, p + n:], before[:, i, :, p + n:]), "later %s rows modified" % nm
                worst = max(worst, _kv_tolerance_ok(got[:, i, :, p:p + n], new, nm))
            check_logits(gl[i], gb[i], rec["logits"], rec["next_bin"])
    return worst


def run_prefill_case(wl, chunks, path=0, n_episodes=None):
    from paper_2603_17573_amd import DeviceModel, Verifier, heisd_verify_set_path
    _need_gpu()
    sh = wl.shape
    weights = synth.make_weights(sh, wl.seed)
    om = oracle_model(sh, weights)
    P = wl.prefix_len
    assert sum(chunks) == P
    episodes = list(range(n_episodes or wl.batch))
    cap = P + 5
    ver = Verifier(DeviceModel(sh, weights), len(episodes), max(chunks), cap)
    assert heisd_verify_set_path(ver.ctx, path) == 0
    xs = [prefix_embeddings(om, wl, e) for e in episodes]
    refs = [oracle_chunked_prefill(om, x, chunks, cap) for x in xs]
    worst = check_chunks_in_isolation(ver, wl, episodes, refs, cap)
    # end to end on the GPU's own cache: a cache element that rounds the other way than the oracle's (rare:
    # the values agree to ~1e-6) perturbs later chunks, so only the outcome is held to the bar here
    kc, vc, out = gpu_chunked_prefill(ver, wl, episodes, chunks, cap)
    for i, x in enumerate(xs):
        last = refs[i][2][-1]
        check_logits(out["last_logits"][i], out["next_bin"][i], last["logits"], last["next_bin"])
        # chunking is faithful: the unchunked fp64 prefill gives the same last-row logits within the bar
        full = oracle.prefill(om, x[None])
        rng_ = last["logits"].max() - last["logits"].min()
        assert np.abs(full["logits_last"][0] - last["logits"]).max() / rng_ <= LOGIT_TOL
    ver.close()
    print(wl.name, "chunks", chunks, "path", path, "worst new-row error", worst, flush=True)


@pytest.mark.parametrize("path", [0, 1, 4])
@pytest.mark.parametrize("chunks", [[64], [7, 30, 27]])
def test_c0_prefix_in_chunks(path, chunks):
    run_prefill_case(synth.WORKLOADS["C0"], chunks, path=path)


def test_visual_rows_as_embeddings_then_text_ids_two_episodes():
    wl = synth.Workload("pf_mid", MID, 30, 11, MID.bin_base, batch=2, K=7, seed=41)
    run_prefill_case(wl, [30, 11])
    run_prefill_case(wl, [16, 14, 11])


@pytest.mark.parametrize("path", [0, 1, 4])
def test_visual_and_text_rows_in_one_chunk(path):
    """Both inputs in one call: the rows with token id -1 take their embeddings, the others are looked
    up (their embedding rows are NaN in the test).  The whole prefix as one chunk, and a split that
    leaves the boundary inside the second chunk."""
    wl = synth.Workload("pf_mixed", MID, 30, 11, MID.bin_base, batch=2, K=7, seed=53)
    run_prefill_case(wl, [41], path=path)
    run_prefill_case(wl, [20, 21], path=path)


def test_chunk_of_256_rows():
    wl = synth.Workload("pf_256", SMALL64, 256, 20, SMALL64.bin_base, batch=1, K=7, seed=43)
    run_prefill_case(wl, [256, 20])


def test_whole_prefix_of_276_rows_as_one_chunk():
    """The paper's prefix shape (256 visual + 20 prompt rows) in a single call: more than 256 rows per
    episode, embeddings and token ids mixed."""
    wl = synth.Workload("pf_276", SMALL64, 256, 20, SMALL64.bin_base, batch=1, K=7, seed=44)
    run_prefill_case(wl, [276])


def test_autoregressive_decode_steps():
    """n_rows = 1: seven decode steps after a prefill, three episodes at once (M = 3: the <= 8-row
    kernels) and one episode on the record kernels; each step is fed the ORACLE's greedy token so that
    the two sides stay on the same sequence."""
    from paper_2603_17573_amd import DeviceModel, Verifier, heisd_verify_set_path
    _need_gpu()
    wl = synth.Workload("ar", SMALL64, 6, 13, SMALL64.bin_base, batch=3, K=7, seed=47)
    sh = wl.shape
    weights = synth.make_weights(sh, wl.seed)
    om = oracle_model(sh, weights)
    P, cap = wl.prefix_len, wl.prefix_len + 9
    for path, eps in ((0, [0, 1, 2]), (4, [1])):
        ver = Verifier(DeviceModel(sh, weights), len(eps), max(wl.n_visual, wl.n_text), cap)
        assert heisd_verify_set_path(ver.ctx, path) == 0
        plen = torch.full((len(eps),), P, dtype=torch.int32, device="cuda")
        refs = [oracle_chunked_prefill(om, prefix_embeddings(om, wl, e), [wl.n_visual, wl.n_text], cap) for e in eps]
        kbs = [r[0] for r in refs]
        vbs = [r[1] for r in refs]
        cur = [r[2][-1]["next_bin"] for r in refs]
        # both sides decode on the oracle's cache bytes
        from gpu_harness import _bits_to_dev
        kc = _bits_to_dev(np.concatenate(kbs, axis=1), "cuda:0")
        vc = _bits_to_dev(np.concatenate(vbs, axis=1), "cuda:0")
        for step in range(7):
            ids = torch.tensor([[sh.bin_base + c] for c in cur], dtype=torch.int32, device="cuda")
            got = ver.prefill_chunk(kc, vc, plen, token_ids=ids, want_logits=True)
            torch.cuda.synchronize()
            gl, gb = got["last_logits"].cpu().numpy().astype(np.float64), got["next_bin"].cpu().numpy()
            for i in range(len(eps)):
                o = oracle.forward_block(om, oracle.embed(om, np.array([[sh.bin_base + cur[i]]])), [P + step],
                                         kbs[i], vbs[i])
                kbs[i][:, 0, :, P + step] = synth.f32_to_bf16_bits(o["k_new"][:, 0, :, 0].astype(np.float32))
                vbs[i][:, 0, :, P + step] = synth.f32_to_bf16_bits(o["v_new"][:, 0, :, 0].astype(np.float32))
                lo = o["logits"][0, 0]
                rng_ = lo.max() - lo.min()
                assert np.abs(gl[i] - lo).max() / rng_ <= LOGIT_TOL
                srt = np.sort(lo)
                nb = int(oracle.argmax_bins(lo))
                if (srt[-1] - srt[-2]) / rng_ > LOGIT_TOL:
                    assert gb[i] == nb
                cur[i] = nb
            plen += 1
        ver.close()


def test_prefill_argument_errors():
    from paper_2603_17573_amd import DeviceModel, Verifier, binding as B
    _need_gpu()
    wl = synth.Workload("pf_err", SMALL64, 0, 8, 1024, batch=2, K=7, seed=1)
    ver = Verifier(DeviceModel(wl.shape, synth.make_weights(wl.shape, 1)), max_batch=2, max_k=16, kv_capacity=40)
    kc, vc = ver.new_cache(2)
    z = torch.zeros(2, dtype=torch.int32, device="cuda")
    ids = torch.zeros((2, 16), dtype=torch.int32, device="cuda")
    x = torch.zeros((2, 16, 256), dtype=torch.float32, device="cuda")
    nb = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    kv = B.heisd_kv_desc(kc.data_ptr(), vc.data_ptr(), z.data_ptr(), None)

    def call(tok=ids.data_ptr(), rows=None, n=16, batch=2, out=nb.data_ptr()):
        return B.heisd_prefill_chunk(ver.ctx, kv, tok, rows, n, batch, out, None, None)

    assert call(tok=None) == B.HEISD_EINVAL                     # neither input
    assert call(n=17) == B.HEISD_EINVAL and call(n=0) == B.HEISD_EINVAL and call(batch=3) == B.HEISD_EINVAL
    assert call(out=None) == B.HEISD_EINVAL
    assert B.heisd_verify_set_path(ver.ctx, B.HEISD_PATH_FAST) == 0
    assert call() == B.HEISD_EUNSUPPORTED                       # 32 rows on the <= 8-row kernels
    assert B.heisd_verify_set_path(ver.ctx, B.HEISD_PATH_AUTO) == 0
    torch.cuda.synchronize()
    assert nb.tolist() == [-7, -7]
    assert call() == B.HEISD_OK and call(tok=None, rows=x.data_ptr()) == B.HEISD_OK
    assert call(rows=x.data_ptr()) == B.HEISD_OK                # both inputs: ids >= 0 are looked up
    torch.cuda.synchronize()
    assert all(0 <= v < 256 for v in nb.tolist())
    ver.close()
