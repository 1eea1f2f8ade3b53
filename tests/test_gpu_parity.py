"""Parity of the HIP path (through the C ABI) with the CPU oracle on the same seeded inputs:
element by element at sizes the oracle finishes in seconds, spanning several tiles, ragged
tails, every row-block width of the GEMM and both head sizes."""
import numpy as np
import pytest

import oracle
import synth
from helpers import oracle_model, oracle_prefix_cache, teacher_forced_drafts

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


MID = synth.ModelShape(n_layers=3, d_model=512, n_heads=4, head_dim=128, d_ffn=1376, vocab=2048)
SMALL64 = synth.ModelShape(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=1024)


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def run_case(wl, plen_override=None, skip=None, rule=None, drafts_mode="auto", check_cache=True, path=0,
             max_batch=None):
    from gpu_harness import run_gpu_step, compare_with_oracle
    _need_gpu()
    sh = wl.shape
    weights = synth.make_weights(sh, wl.seed)
    om = oracle_model(sh, weights)
    cap = wl.prefix_len + wl.K + 3                        # capacity is not a multiple of anything
    kb, vb, plen, first = oracle_prefix_cache(om, wl, cap)
    if plen_override is not None:
        plen = np.asarray(plen_override, np.int32)
    rule = rule or oracle.AcceptRule(wl.tau_tok, wl.tau_seq)
    if wl.draft[0] == "geometric":
        off = synth.make_offsets_geometric(wl, wl.draft[1])
        bins = teacher_forced_drafts(om, wl, kb, vb, plen, first, off)
    else:
        bins = synth.make_drafts_uniform(wl)
    drafts = (sh.bin_base + bins).astype(np.int32)
    ref = oracle.verify_step(om, kb, vb, plen, first, drafts, rule, skip)
    got = run_gpu_step(sh, weights, kb, vb, plen, first, drafts, rule, skip, path=path, max_batch=max_batch)
    stats = compare_with_oracle(got, ref, drafts, rule, sh, kb, vb, plen, skip)
    print(wl.name, "path", path, stats, "accepted", got["accepted_len"].tolist())
    return got, ref, stats


@pytest.mark.parametrize("path", [0, 1, 2, 3, 4])
def test_c0_tiny_config(path):
    """C0 through the automatic choice, both any-M paths, the <=8-row kernels and the persistent kernel
    (FFN width 688 = 21.5 k-steps: exercises the clamped tail of the reduction)."""
    got, ref, stats = run_case(synth.WORKLOADS["C0"], path=path)
    assert stats["max_logit_err_over_range"] < 3e-2


@pytest.mark.parametrize("path", [1, 2, 3, 4])
@pytest.mark.parametrize("shape_name,B,K,skip", [("mid", 1, 7, None), ("mid", 2, 4, [0, 1]), ("mid", 1, 8, None),
                                                 ("s64", 2, 3, None), ("s64", 1, 5, None)])
def test_small_row_counts_on_both_paths(path, shape_name, B, K, skip):
    """M <= 8 rows (one or two episodes) on a multi-tile shape, forced through each kernel path."""
    shape = MID if shape_name == "mid" else SMALL64
    wl = synth.Workload("%s_%dx%d" % (shape_name, B, K), shape, 30, 11, shape.bin_base, batch=B, K=K,
                        draft=("geometric", 0.5), seed=B * 7 + K)
    run_case(wl, skip=None if skip is None else np.array(skip, np.uint8), path=path,
             plen_override=[41, 17][:B] if B > 1 else None)


LONGF = synth.ModelShape(n_layers=2, d_model=512, n_heads=4, head_dim=128, d_ffn=4416, vocab=2048)


@pytest.mark.parametrize("path", [2, 3])
@pytest.mark.parametrize("B,K", [(1, 7), (2, 4)])
def test_long_reduction_streams_its_activations(path, B, K):
    """FFN width 4416 (138 k-steps, more than the 128 a workgroup's waves keep resident): the down
    projection of the <=8-row kernels streams its activation fragments through a second ring, with a
    ragged last round (18 steps per wave, the last wave 12)."""
    wl = synth.Workload("longf_%dx%d" % (B, K), LONGF, 20, 9, LONGF.bin_base, batch=B, K=K,
                        draft=("geometric", 0.5), seed=B * 5 + K)
    run_case(wl, path=path)


def test_persistent_kernel_gives_the_bits_of_one_launch_per_phase():
    """The persistent kernel runs the phase bodies of the <= 8-row kernels in the same order of additions: logits,
    bins, accepted lengths and appended cache rows are equal bit for bit (two episodes with different prefix
    lengths, K = 4)."""
    from gpu_harness import run_gpu_step
    _need_gpu()
    wl = synth.Workload("mid_bits", MID, 30, 11, MID.bin_base, batch=2, K=4, draft=("geometric", 0.5), seed=5)
    weights = synth.make_weights(MID, wl.seed)
    cap = 48
    k0, v0, f0 = zip(*[synth.make_prefix_kv_direct(wl, e, cap) for e in range(2)])
    kb, vb = np.stack(k0, axis=1), np.stack(v0, axis=1)
    drafts = (MID.bin_base + synth.make_drafts_uniform(wl)).astype(np.int32)
    rule = oracle.AcceptRule(2, 6)
    outs = [run_gpu_step(MID, weights, kb, vb, [41, 33], list(f0), drafts, rule, None, path=p) for p in (2, 3, 0)]
    for k in outs[0]:
        assert np.array_equal(outs[0][k], outs[1][k], equal_nan=True), k
        assert np.array_equal(outs[0][k], outs[2][k], equal_nan=True), k


@pytest.mark.parametrize("mode", [1, 2, 3, 4, 5])
def test_persistent_kernel_handover_modes_agree(mode):
    """What the persistent kernel requests across its grid barriers changes when weights arrive, never
    what is computed: every mode gives the bits of the default mode (two episodes, one skipped, so that
    attention units without work hand over too)."""
    import torch
    import paper_2603_17573_amd as P
    from gpu_harness import _bits_to_dev, _dev_to_bits, accept_desc_of
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    wl = synth.Workload("mid_ho", MID, 30, 11, MID.bin_base, batch=2, K=4, draft=("geometric", 0.5), seed=3)
    weights = synth.make_weights(MID, wl.seed)
    om = oracle_model(MID, weights)
    cap = wl.prefix_len + wl.K
    kb, vb, plen, first = oracle_prefix_cache(om, wl, cap)
    drafts = (MID.bin_base + synth.make_drafts_uniform(wl)).astype(np.int32)
    dm = P.DeviceModel(MID, weights)
    ver = P.Verifier(dm, 2, 4, cap)
    assert P.heisd_verify_set_path(ver.ctx, 3) == 0
    dev = "cuda:0"
    skip = torch.tensor([0, 1], dtype=torch.uint8, device=dev)
    outs = []
    for m in (0, mode):
        assert P.heisd_verify_set_handover(ver.ctx, m) == 0
        kc, vc = _bits_to_dev(kb, dev), _bits_to_dev(vb, dev)
        out = ver.step(kc, vc, torch.from_numpy(plen).to(dev), torch.from_numpy(first).to(dev),
                       torch.from_numpy(drafts).to(dev), accept_desc_of(oracle.AcceptRule(2, 6)), skip)
        torch.cuda.synchronize()
        assert P.heisd_verify_check(ver.ctx) == 0
        outs.append(({k: v.cpu().numpy().copy() for k, v in out.items()}, _dev_to_bits(kc), _dev_to_bits(vc)))
    for k in outs[0][0]:
        assert np.array_equal(outs[0][0][k], outs[1][0][k], equal_nan=True), k
    assert np.array_equal(outs[0][1], outs[1][1]) and np.array_equal(outs[0][2], outs[1][2])
    assert P.heisd_verify_set_handover(ver.ctx, 7) == P.HEISD_EINVAL
    ver.close()


@pytest.mark.parametrize("path,B,K", [(0, 2, 4), (3, 2, 4), (4, 3, 7), (1, 3, 7)])
def test_episode_that_does_not_fit_its_cache_is_left_out(path, B, K):
    """prefix_len + K > kv_capacity for one episode (the host cannot see it): that episode's cache is
    untouched and its outputs say so, the other episodes still match the oracle, and
    heisd_verify_check reports the episode."""
    import torch
    import paper_2603_17573_amd as P
    from gpu_harness import _bits_to_dev, _dev_to_bits, accept_desc_of, compare_with_oracle
    _need_gpu()
    wl = synth.Workload("mid_ovf", MID, 20, 9, MID.bin_base, batch=B, K=K, seed=17 + B)
    weights = synth.make_weights(MID, wl.seed)
    om = oracle_model(MID, weights)
    cap = wl.prefix_len + K
    kb, vb, plen, first = oracle_prefix_cache(om, wl, cap)
    plen_bad = plen.copy()
    plen_bad[B - 1] = cap - K + 1                         # one row too many
    drafts = (MID.bin_base + synth.make_drafts_uniform(wl)).astype(np.int32)
    rule = oracle.AcceptRule(2, 6)
    good = [b for b in range(B) if b != B - 1]
    ref = oracle.verify_step(om, kb[:, good], vb[:, good], plen[good], first[good], drafts[good], rule)
    dm = P.DeviceModel(MID, weights)
    ver = P.Verifier(dm, B, K, cap)
    assert P.heisd_verify_set_path(ver.ctx, path) == 0
    dev = "cuda:0"
    kc, vc = _bits_to_dev(kb, dev), _bits_to_dev(vb, dev)
    out = ver.step(kc, vc, torch.from_numpy(plen_bad).to(dev), torch.from_numpy(first).to(dev),
                   torch.from_numpy(drafts).to(dev), accept_desc_of(rule))
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in out.items()}
    got["k_cache"], got["v_cache"] = _dev_to_bits(kc), _dev_to_bits(vc)
    assert got["accepted_len"][B - 1] == -1 and got["next_token"][B - 1] == -1
    assert np.all(got["target_bins"][B - 1] == -1) and np.all(np.isnan(got["bin_logits"][B - 1]))
    assert np.array_equal(got["k_cache"][:, B - 1], kb[:, B - 1]) and np.array_equal(got["v_cache"][:, B - 1], vb[:, B - 1])
    compare_with_oracle(got, ref, drafts, rule, MID, kb, vb, plen, None, episodes=good)
    assert P.heisd_verify_check(ver.ctx) == P.HEISD_EINVAL and "did not fit" in P.heisd_last_error(ver.ctx)
    assert P.heisd_verify_check(ver.ctx) == 0             # the word is cleared by the check
    # the same context still serves a step that fits
    kc, vc = _bits_to_dev(kb, dev), _bits_to_dev(vb, dev)
    out = ver.step(kc, vc, torch.from_numpy(plen).to(dev), torch.from_numpy(first).to(dev),
                   torch.from_numpy(drafts).to(dev), accept_desc_of(rule))
    torch.cuda.synchronize()
    assert int(out["accepted_len"].cpu()[B - 1]) >= 0 and P.heisd_verify_check(ver.ctx) == 0
    ver.close()


def test_mid_hd128_ragged_prefixes_geometric_drafts():
    wl = synth.Workload("mid_b3", MID, 50, 20, MID.bin_base, batch=3, K=7, draft=("geometric", 0.5), seed=11)
    got, ref, stats = run_case(wl, plen_override=[70, 33, 64])
    assert len(set(got["accepted_len"].tolist())) >= 1


def test_hd64_two_row_blocks_with_skips_k14():
    wl = synth.Workload("s64_b5k14", SMALL64, 0, 40, 1024, batch=5, K=14, skip_p=0.4,
                        draft=("geometric", 0.6), seed=5)
    skip = np.array([0, 1, 0, 0, 1], np.uint8)            # M = 70 rows: one 64-row block and a tail of 6
    run_case(wl, skip=skip)


@pytest.mark.parametrize("path", [1, 4])
@pytest.mark.parametrize("B,K", [(3, 4), (2, 10), (5, 7), (1, 1), (9, 7)])
def test_row_block_widths(B, K, path):
    """M = 12, 20, 35, 1, 63: the 16-, 32- and 64-row variants of the first any-M path and the 2-, 4-, 7-
    and 8-column-tile variants of the record path, a single row, and K not a multiple of the
    8-query attention block."""
    wl = synth.Workload("w%dx%d" % (B, K), SMALL64, 8, 17, SMALL64.bin_base, batch=B, K=K, seed=B * 31 + K)
    run_case(wl, rule=oracle.AcceptRule(15, 30), path=path)


@pytest.mark.parametrize("shape_name,B,K", [("s64", 10, 7), ("mid", 19, 7), ("s64", 24, 11), ("s64", 40, 13)])
def test_wave_arrangements_of_the_record_path(shape_name, B, K):
    """M = 70, 133, 264, 520 rows: 2, 4 and 8 wave groups across the rows (reduction split 4, 2, 1
    ways), and more than 64 column tiles, where the weights are streamed twice."""
    shape = MID if shape_name == "mid" else SMALL64
    wl = synth.Workload("%s_%dx%d" % (shape_name, B, K), shape, 4, 9, shape.bin_base, batch=B, K=K,
                        draft=("geometric", 0.5), seed=B + K)
    run_case(wl, path=4)


SPLIT = synth.ModelShape(n_layers=2, d_model=1024, n_heads=8, head_dim=128, d_ffn=2816, vocab=2048)


@pytest.mark.parametrize("B,K", [(12, 9), (25, 8)])
def test_split_reductions(B, K):
    """108 and 200 rows (one ragged block of column tiles; two blocks, the second ragged) on a shape
    whose O-proj and down have few weight tiles (64) and long enough reductions (32 and 88 k-steps)
    that the dispatcher cuts them into 4 and 2 runs: every run's sums go through memory and a second
    launch adds them and applies the residual epilogue."""
    wl = synth.Workload("split_%dx%d" % (B, K), SPLIT, 4, 11, SPLIT.bin_base, batch=B, K=K,
                        draft=("geometric", 0.5), seed=3 * B + K)
    run_case(wl)


@pytest.mark.parametrize("B,K", [(17, 1), (3, 8), (3, 11), (5, 8), (8, 8), (5, 13), (9, 8), (16, 8), (43, 3), (17, 8)])
def test_row_counts_at_the_dispatch_boundaries(B, K):
    """17, 24, 33, 40, 64, 65, 72, 128, 129 and 136 rows on the shape whose reductions get split: the row
    counts on either side of the points where the launcher changes kernel or wave arrangement (6 x 1 wide
    kernel from 17 and 33 rows, 3 x 2 from 65, a second block of column tiles from 129), with full and
    ragged last column tiles."""
    wl = synth.Workload("edge_%dx%d" % (B, K), SPLIT, 3, 7, SPLIT.bin_base, batch=B, K=K,
                        draft=("geometric", 0.5), seed=5 * B + K)
    run_case(wl)


def test_context_sized_for_more_rows_than_the_call_uses():
    """A context initialised for 12 episodes verifies 3 (the record stride is that of the context,
    the column-tile count that of the call), on the automatic path and on the <=8-row path."""
    wl = synth.Workload("wide_ctx", SMALL64, 6, 13, SMALL64.bin_base, batch=3, K=7, draft=("geometric", 0.5), seed=77)
    run_case(wl, max_batch=12)
    wl1 = synth.Workload("wide_ctx1", SMALL64, 6, 13, SMALL64.bin_base, batch=1, K=7, draft=("geometric", 0.5), seed=78)
    run_case(wl1, max_batch=12)
    run_case(wl1, max_batch=12, path=4)


def test_strict_and_token_mode_rules_on_device():
    wl = synth.Workload("rules", SMALL64, 0, 24, 1024, batch=6, K=7, draft=("geometric", 0.7), seed=3)
    for rule in (oracle.AcceptRule(0, 0), oracle.AcceptRule(1, 2),
                 oracle.AcceptRule(0, 0, group_sizes=(1,), exact_group_mask=0),
                 oracle.AcceptRule(2, 3, mode=1)):
        run_case(wl, rule=rule, check_cache=False)


def test_idempotent_and_deterministic():
    from gpu_harness import run_gpu_step
    _need_gpu()
    wl = synth.Workload("idem", SMALL64, 0, 30, 1024, batch=2, K=7, seed=9)
    weights = synth.make_weights(wl.shape, wl.seed)
    kb, vb, first = [], [], []
    cap = 40
    k0, v0, f0 = zip(*[synth.make_prefix_kv_direct(wl, e, cap) for e in range(2)])
    kb = np.stack(k0, axis=1)
    vb = np.stack(v0, axis=1)
    drafts = (wl.shape.bin_base + synth.make_drafts_uniform(wl)).astype(np.int32)
    rule = oracle.AcceptRule(2, 6)
    a = run_gpu_step(wl.shape, weights, kb, vb, [30, 30], list(f0), drafts, rule, None, repeat=1)
    b = run_gpu_step(wl.shape, weights, kb, vb, [30, 30], list(f0), drafts, rule, None, repeat=3)
    for k in a:
        assert np.array_equal(a[k], b[k], equal_nan=True), k


@pytest.mark.parametrize("B,K", [(6, 7), (25, 8)])
def test_split_reductions_are_deterministic(B, K):
    """42 and 200 rows on the shape whose reductions are split: the runs' sums are added in the order of the
    runs, whichever workgroup finishes first, so a step repeated on the same inputs gives the same bits."""
    from gpu_harness import run_gpu_step
    _need_gpu()
    wl = synth.Workload("idem_split", SPLIT, 0, 30, SPLIT.bin_base, batch=B, K=K, seed=19)
    weights = synth.make_weights(wl.shape, wl.seed)
    cap = 30 + K + 2
    k0, v0, f0 = zip(*[synth.make_prefix_kv_direct(wl, e, cap) for e in range(B)])
    kb, vb = np.stack(k0, axis=1), np.stack(v0, axis=1)
    drafts = (wl.shape.bin_base + synth.make_drafts_uniform(wl)).astype(np.int32)
    rule = oracle.AcceptRule(2, 6)
    a = run_gpu_step(wl.shape, weights, kb, vb, [30] * B, list(f0), drafts, rule, None, repeat=1)
    b = run_gpu_step(wl.shape, weights, kb, vb, [30] * B, list(f0), drafts, rule, None, repeat=4)
    for k in a:
        assert np.array_equal(a[k], b[k], equal_nan=True), k


@pytest.mark.parametrize("B,K", [(10, 7), (25, 8), (9, 8), (7, 7)])
def test_single_bf16_activations(B, K):
    """The opt-in activation format (one bf16 per value instead of a bf16 head and tail) on the shape whose
    reductions are split: 70 rows (blocks of 8 column tiles, six waves across the weight tiles), 200 rows (3 x 2
    waves, 13 column tiles of 16 rows, a ragged last one), 72 rows and 49 rows (gate/up on the kernel for up to 64 rows); against the oracle to the logit bar (the
    cache rows are then bf16-accurate activations away from the oracle's, so they are not compared).  The format
    takes effect (the logits differ from the split form's), and a step below 33 rows keeps the split form (same bits)."""
    from gpu_harness import run_gpu_step, compare_with_oracle
    import paper_2603_17573_amd as P
    _need_gpu()
    wl = synth.Workload("act_bf16", SPLIT, 0, 30, SPLIT.bin_base, batch=B, K=K, seed=23)
    weights = synth.make_weights(wl.shape, wl.seed)
    om = oracle_model(SPLIT, weights)
    cap = 30 + K + 2
    k0, v0, f0 = zip(*[synth.make_prefix_kv_direct(wl, e, cap) for e in range(B)])
    kb, vb = np.stack(k0, axis=1), np.stack(v0, axis=1)
    plen, first = np.full(B, 30, np.int32), np.array(f0, np.int32)
    drafts = (SPLIT.bin_base + synth.make_drafts_uniform(wl)).astype(np.int32)
    rule = oracle.AcceptRule(2, 6)
    ref = oracle.verify_step(om, kb, vb, plen, first, drafts, rule)
    split = run_gpu_step(SPLIT, weights, kb, vb, plen, first, drafts, rule, None)
    single = run_gpu_step(SPLIT, weights, kb, vb, plen, first, drafts, rule, None, act=P.HEISD_ACT_BF16)
    s0 = compare_with_oracle(split, ref, drafts, rule, SPLIT)
    s1 = compare_with_oracle(single, ref, drafts, rule, SPLIT)
    print("rows %d: split %s, single bf16 %s" % (B * K, s0, s1), flush=True)
    assert s1["max_logit_err_over_range"] > 4 * s0["max_logit_err_over_range"]
    small = run_gpu_step(SPLIT, weights, kb[:, :4], vb[:, :4], plen[:4], first[:4], drafts[:4], rule, None, act=P.HEISD_ACT_BF16)
    small0 = run_gpu_step(SPLIT, weights, kb[:, :4], vb[:, :4], plen[:4], first[:4], drafts[:4], rule, None)
    assert np.array_equal(small["bin_logits"], small0["bin_logits"])


def test_step_argument_errors_enqueue_nothing():
    from paper_2603_17573_amd import DeviceModel, Verifier, make_accept_desc, binding as B
    _need_gpu()
    wl = synth.Workload("err", SMALL64, 0, 8, 1024, batch=2, K=7, seed=1)
    dm = DeviceModel(wl.shape, synth.make_weights(wl.shape, 1))
    ver = Verifier(dm, max_batch=2, max_k=7, kv_capacity=20)
    kc, vc = ver.new_cache(2)
    z = torch.zeros(2, dtype=torch.int32, device="cuda")
    dr = torch.full((2, 7), wl.shape.bin_base, dtype=torch.int32, device="cuda")
    acc = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    nxt = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    kv = B.heisd_kv_desc(kc.data_ptr(), vc.data_ptr(), z.data_ptr(), z.data_ptr())
    ok = make_accept_desc(2, 6)

    def call(K=7, batch=2, accept=ok, kvd=kv, drafts=dr.data_ptr(), out=acc.data_ptr()):
        return B.heisd_verify_step(ver.ctx, kvd, drafts, K, batch, accept, None, out, nxt.data_ptr(), None, None, None)

    assert call(K=8) == B.HEISD_EINVAL and "K=8" in B.heisd_last_error(ver.ctx)
    assert call(batch=3) == B.HEISD_EINVAL
    assert call(K=0) == B.HEISD_EINVAL
    assert call(drafts=None) == B.HEISD_EINVAL
    assert call(out=None) == B.HEISD_EINVAL
    assert call(kvd=B.heisd_kv_desc(0, vc.data_ptr(), z.data_ptr(), z.data_ptr())) == B.HEISD_EINVAL
    assert call(accept=make_accept_desc(2, 6, group_sizes=(3, 0, 1))) == B.HEISD_EINVAL
    assert call(accept=make_accept_desc(-1, 6)) == B.HEISD_EINVAL
    assert call(accept=make_accept_desc(2, 6, mode=2)) == B.HEISD_EINVAL
    torch.cuda.synchronize()
    assert acc.tolist() == [-7, -7] and nxt.tolist() == [-7, -7]      # nothing ran
    assert call() == B.HEISD_OK and B.heisd_last_error(ver.ctx) == ""
    torch.cuda.synchronize()
    assert all(v in (0, 3, 6, 7) for v in acc.tolist())
    ver.close()


@pytest.mark.parametrize("path", [0, 4])
def test_largest_kv_capacity(path):
    """kv_capacity 4096 (the largest the library takes) with a prefix that fills it: the attention
    kernels' LDS score rows are at their longest."""
    from gpu_harness import run_gpu_step, compare_with_oracle
    _need_gpu()
    cap, K = 4096, 7
    wl = synth.Workload("cap4096", SMALL64, 0, cap - K, SMALL64.bin_base, batch=2, K=K, seed=61)
    sh = wl.shape
    weights = synth.make_weights(sh, wl.seed)
    om = oracle_model(sh, weights)
    k0, v0, f0 = zip(*[synth.make_prefix_kv_direct(wl, e, cap) for e in range(2)])
    kb, vb = np.stack(k0, axis=1), np.stack(v0, axis=1)
    plen, first = np.array([cap - K, 1234], np.int32), np.array(f0, np.int32)
    drafts = (sh.bin_base + synth.make_drafts_uniform(wl)).astype(np.int32)
    rule = oracle.AcceptRule(2, 6)
    ref = oracle.verify_step(om, kb, vb, plen, first, drafts, rule)
    got = run_gpu_step(sh, weights, kb, vb, plen, first, drafts, rule, None, path=path)
    stats = compare_with_oracle(got, ref, drafts, rule, sh, kb, vb, plen, None)
    print("cap 4096 path", path, stats, flush=True)
