"""Parity at the full 7B shape, in the launch configuration bench.py times.  The prefix K/V of
these cases is drawn directly by the generator (a CPU prefill of 7B-shaped prefixes is minutes
per episode); the oracle receives the same bf16 bytes."""
import time

import numpy as np
import pytest

import oracle
import synth
from helpers import oracle_model, direct_prefix_cache, teacher_forced_drafts

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def big():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_17573_amd import DeviceModel
    sh = synth.LLAMA7B
    t0 = time.time()
    weights = synth.make_weights(sh, 0)
    print("generated 7B-shaped weights in %.1f s" % (time.time() - t0), flush=True)
    dm = DeviceModel(sh, weights)
    return sh, weights, oracle_model(sh, weights), dm


def test_c1_full_size_uniform_drafts(big):
    from gpu_harness import run_gpu_step, compare_with_oracle
    sh, weights, om, dm = big
    wl = synth.WORKLOADS["C1"]
    cap = wl.prefix_len + wl.K
    kb, vb, plen, first = direct_prefix_cache(wl, cap)
    drafts = (sh.bin_base + synth.make_drafts_uniform(wl)).astype(np.int32)
    rule = oracle.AcceptRule(wl.tau_tok, wl.tau_seq)
    t0 = time.time()
    ref = oracle.verify_step(om, kb, vb, plen, first, drafts, rule)
    print("oracle C1 verify %.1f s" % (time.time() - t0), flush=True)
    got = run_gpu_step(sh, weights, kb, vb, plen, first, drafts, rule, None, model=dm)
    stats = compare_with_oracle(got, ref, drafts, rule, sh, kb, vb, plen, None)
    print("C1", stats, got["accepted_len"].tolist(), flush=True)


def test_c2_full_size_batch8_teacher_forced_drafts(big):
    from gpu_harness import run_gpu_step, compare_with_oracle
    sh, weights, om, dm = big
    wl = synth.WORKLOADS["C2"]
    cap = wl.prefix_len + wl.K
    kb, vb, plen, first = direct_prefix_cache(wl, cap)
    off = synth.make_offsets_geometric(wl, wl.draft[1])
    t0 = time.time()
    bins = teacher_forced_drafts(om, wl, kb, vb, plen, first, off)
    print("teacher-forced drafts %.1f s" % (time.time() - t0), flush=True)
    drafts = (sh.bin_base + bins).astype(np.int32)
    rule = oracle.AcceptRule(wl.tau_tok, wl.tau_seq)
    ref = oracle.verify_step(om, kb, vb, plen, first, drafts, rule)
    got = run_gpu_step(sh, weights, kb, vb, plen, first, drafts, rule, None, model=dm)
    stats = compare_with_oracle(got, ref, drafts, rule, sh, kb, vb, plen, None)
    print("C2", stats, got["accepted_len"].tolist(), ref["accepted_len"].tolist(), flush=True)
    assert len(set(ref["accepted_len"].tolist())) > 1          # acceptance lengths vary over the batch
