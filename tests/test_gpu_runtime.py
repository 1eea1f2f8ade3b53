"""Properties of the library's run-time behaviour on the GPU, beyond what one step computes (paper Sec. 2.2: one
verification pass per step): a step captured in a HIP graph replays to the bits of the eager call; the caller's
projection matrices are never read once released; the bounded waits inside the kernels give up cleanly and the
next step is unaffected; a context without a slot of uncached barrier flags still runs the persistent kernel.

A captured step: the kernels exchange data through device memory that the launches themselves prepare (flags,
counters, epoch-tagged row scales whose epochs are kernel arguments and therefore frozen at capture), so a
replay must not depend on what the previous replay left behind.  The graph is replayed several times with
different drafts, with eager work and synchronisations of the program's own between the replays, and each
replay is compared with the eager result for the same drafts."""
import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

MID = synth.ModelShape(n_layers=3, d_model=512, n_heads=4, head_dim=128, d_ffn=1376, vocab=2048)


@pytest.mark.parametrize("B,K", [(1, 7), (2, 7), (6, 7)])
def test_graph_replays_give_the_bits_of_the_eager_step(B, K):
    """7 rows (the <= 8-row kernels, one launch per phase under capture), 14 rows (register-B GEMMs) and
    42 rows (LDS-shared B, split reductions): the row scales of the last two are handed over inside
    their launches."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2603_17573_amd as P
    from gpu_harness import _bits_to_dev, accept_desc_of
    wl = synth.Workload("graph_%dx%d" % (B, K), MID, 30, 11, MID.bin_base, batch=B, K=K, draft=("geometric", 0.5), seed=B + 40)
    weights = synth.make_weights(MID, wl.seed)
    cap = wl.prefix_len + K + 1
    k0, v0, f0 = zip(*[synth.make_prefix_kv_direct(wl, e, cap) for e in range(B)])
    kb, vb = np.stack(k0, axis=1), np.stack(v0, axis=1)
    dev = "cuda:0"
    dm = P.DeviceModel(MID, weights)
    ver = P.Verifier(dm, B, K, cap)
    acc = accept_desc_of(oracle.AcceptRule(2, 6))
    kc, vc = _bits_to_dev(kb, dev), _bits_to_dev(vb, dev)
    plen = torch.full((B,), wl.prefix_len, dtype=torch.int32, device=dev)
    first = torch.from_numpy(np.asarray(f0, np.int32)).to(dev)
    rng = np.random.default_rng(7)
    draft_sets = [torch.from_numpy((MID.bin_base + rng.integers(0, MID.n_bins, size=(B, K))).astype(np.int32)).to(dev)
                  for _ in range(2)]
    drafts = draft_sets[0].clone()

    def snapshot(out):
        torch.cuda.synchronize()
        assert P.heisd_verify_check(ver.ctx) == 0
        return {k: v.cpu().numpy().copy() for k, v in out.items()}

    eager = []
    for d in draft_sets:
        drafts.copy_(d)
        eager.append(snapshot(ver.step(kc, vc, plen, first, drafts, acc, None)))
    assert not np.array_equal(eager[0]["bin_logits"], eager[1]["bin_logits"])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        out = ver.step(kc, vc, plen, first, drafts, acc, None)       # allocates the outputs outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ver.step(kc, vc, plen, first, drafts, acc, None, out=out)
    for which in (0, 1, 1, 0, 1):
        drafts.copy_(draft_sets[which])
        scratch = torch.randn(256, 256, device=dev) @ torch.randn(256, 256, device=dev)      # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot(out)
        for k in got:
            assert np.array_equal(got[k], eager[which][k], equal_nan=True), (k, which)
        del scratch
    ver.close()


@pytest.mark.parametrize("B,K,path", [(1, 7, 0), (1, 7, 2), (2, 7, 0), (6, 7, 4)])
def test_released_projection_matrices_are_never_read(B, K, path):
    """After heisd_verify_release_projections the caller's wq .. w_down and lm_head may be freed: here their
    memory is overwritten with NaN patterns instead, and the step still gives the bits it gave before; the
    generic path, which reads them in place, can no longer be selected."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2603_17573_amd as P
    from gpu_harness import _bits_to_dev, accept_desc_of
    wl = synth.Workload("rel_%dx%d" % (B, K), MID, 30, 11, MID.bin_base, batch=B, K=K, draft=("geometric", 0.5), seed=B + 60)
    weights = synth.make_weights(MID, wl.seed)
    cap = wl.prefix_len + K
    k0, v0, f0 = zip(*[synth.make_prefix_kv_direct(wl, e, cap) for e in range(B)])
    kb, vb = np.stack(k0, axis=1), np.stack(v0, axis=1)
    dev = "cuda:0"
    dm = P.DeviceModel(MID, weights)
    ver = P.Verifier(dm, B, K, cap)
    assert P.heisd_verify_set_path(ver.ctx, path) == 0
    acc = accept_desc_of(oracle.AcceptRule(2, 6))
    plen = torch.full((B,), wl.prefix_len, dtype=torch.int32, device=dev)
    first = torch.from_numpy(np.asarray(f0, np.int32)).to(dev)
    drafts = torch.from_numpy((MID.bin_base + synth.make_drafts_uniform(wl)).astype(np.int32)).to(dev)

    def run():
        kc, vc = _bits_to_dev(kb, dev), _bits_to_dev(vb, dev)
        out = ver.step(kc, vc, plen, first, drafts, acc, None)
        torch.cuda.synchronize()
        assert P.heisd_verify_check(ver.ctx) == 0
        return {k: v.cpu().numpy().copy() for k, v in out.items()}

    before = run()
    assert P.heisd_verify_set_path(ver.ctx, P.HEISD_PATH_GENERIC) == 0
    assert P.heisd_verify_release_projections(ver.ctx) == P.HEISD_EUNSUPPORTED      # the selected path reads them
    assert P.heisd_verify_set_path(ver.ctx, path) == 0
    assert P.heisd_verify_release_projections(ver.ctx) == 0
    assert P.heisd_verify_set_path(ver.ctx, P.HEISD_PATH_GENERIC) == P.HEISD_EUNSUPPORTED
    for name in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
        for w in dm.t[name]:
            w.view(torch.int16).fill_(0x7FC1)                  # a NaN in every bf16
    dm.t["lm_head"].view(torch.int16).fill_(0x7FC1)
    torch.cuda.synchronize()
    after = run()
    for k in before:
        assert np.array_equal(before[k], after[k], equal_nan=True), k
    assert np.all(np.isfinite(after["bin_logits"]))
    ver.close()


@pytest.mark.parametrize("B,K,path", [(1, 7, 3), (6, 7, 4)])
def test_waits_inside_the_kernels_give_up_and_the_next_step_is_unaffected(B, K, path):
    """The bounded waits inside the kernels - the grid barriers of the persistent kernel (path 3), the row scales
    handed over inside a launch on the path for more than 8 rows (path 4) - are made to give up from the host
    (one poll per barrier; scales never produced and eight polls for each): every kernel runs to its end,
    heisd_verify_check reports EHIP, and with the defaults restored the next step gives the bits of the step
    before."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2603_17573_amd as P
    from gpu_harness import _bits_to_dev, accept_desc_of
    wl = synth.Workload("giveup_%dx%d" % (B, K), MID, 30, 11, MID.bin_base, batch=B, K=K, draft=("geometric", 0.5), seed=B + 80)
    weights = synth.make_weights(MID, wl.seed)
    cap = wl.prefix_len + K
    k0, v0, f0 = zip(*[synth.make_prefix_kv_direct(wl, e, cap) for e in range(B)])
    kb, vb = np.stack(k0, axis=1), np.stack(v0, axis=1)
    dev = "cuda:0"
    dm = P.DeviceModel(MID, weights)
    ver = P.Verifier(dm, B, K, cap)
    assert P.heisd_verify_set_path(ver.ctx, path) == 0
    acc = accept_desc_of(oracle.AcceptRule(2, 6))
    plen = torch.full((B,), wl.prefix_len, dtype=torch.int32, device=dev)
    first = torch.from_numpy(np.asarray(f0, np.int32)).to(dev)
    drafts = torch.from_numpy((MID.bin_base + synth.make_drafts_uniform(wl)).astype(np.int32)).to(dev)

    def run():
        kc, vc = _bits_to_dev(kb, dev), _bits_to_dev(vb, dev)
        out = ver.step(kc, vc, plen, first, drafts, acc, None)
        torch.cuda.synchronize()
        return {k: v.cpu().numpy().copy() for k, v in out.items()}

    before = run()
    assert P.heisd_verify_check(ver.ctx) == 0
    assert P.heisd_debug_set_wait_limits(ver.ctx, 1, 8, 1) == 0
    run()
    assert P.heisd_verify_check(ver.ctx) == P.HEISD_EHIP
    assert P.heisd_verify_check(ver.ctx) == 0                      # the word is cleared by the check that reports it
    assert P.heisd_debug_set_wait_limits(ver.ctx, 0, 0, 0) == 0
    after = run()
    assert P.heisd_verify_check(ver.ctx) == 0
    for k in before:
        assert np.array_equal(before[k], after[k], equal_nan=True), k
    ver.close()


def test_context_without_a_slot_of_uncached_flags_still_runs_the_persistent_kernel():
    """The persistent kernel's barrier flags live in a slot of a small per-device pool of uncached memory (32 slots);
    a context that gets none keeps its flags in the workspace.  40 contexts alive at once: the last ones are
    without a slot, and their persistent-kernel steps give the bits of the first context's."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2603_17573_amd as P
    from gpu_harness import _bits_to_dev, accept_desc_of
    sh = synth.ModelShape(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=1024)
    B, K = 1, 7
    wl = synth.Workload("slots", sh, 20, 9, sh.bin_base, batch=B, K=K, draft=("geometric", 0.5), seed=91)
    weights = synth.make_weights(sh, wl.seed)
    cap = wl.prefix_len + K
    k0, v0, f0 = zip(*[synth.make_prefix_kv_direct(wl, e, cap) for e in range(B)])
    kb, vb = np.stack(k0, axis=1), np.stack(v0, axis=1)
    dev = "cuda:0"
    dm = P.DeviceModel(sh, weights)
    vers = [P.Verifier(dm, B, K, cap) for _ in range(40)]
    acc = accept_desc_of(oracle.AcceptRule(2, 6))
    plen = torch.full((B,), wl.prefix_len, dtype=torch.int32, device=dev)
    first = torch.from_numpy(np.asarray(f0, np.int32)).to(dev)
    drafts = torch.from_numpy((sh.bin_base + synth.make_drafts_uniform(wl)).astype(np.int32)).to(dev)
    outs = []
    for ver in (vers[0], vers[35], vers[39]):
        assert P.heisd_verify_set_path(ver.ctx, P.HEISD_PATH_PERSIST) == 0
        kc, vc = _bits_to_dev(kb, dev), _bits_to_dev(vb, dev)
        out = ver.step(kc, vc, plen, first, drafts, acc, None)
        torch.cuda.synchronize()
        assert P.heisd_verify_check(ver.ctx) == 0
        outs.append({k: v.cpu().numpy().copy() for k, v in out.items()})
    for o in outs[1:]:
        for k in outs[0]:
            assert np.array_equal(outs[0][k], o[k], equal_nan=True), k
    for ver in vers:
        ver.close()
    again = P.Verifier(dm, B, K, cap)                   # the slots are back in the pool
    assert P.heisd_verify_set_path(again.ctx, P.HEISD_PATH_PERSIST) == 0
    kc, vc = _bits_to_dev(kb, dev), _bits_to_dev(vb, dev)
    out = again.step(kc, vc, plen, first, drafts, acc, None)
    torch.cuda.synchronize()
    assert P.heisd_verify_check(again.ctx) == 0
    for k in outs[0]:
        assert np.array_equal(outs[0][k], out[k].cpu().numpy(), equal_nan=True), k
    again.close()
