"""Pins of the oracle's acceptance rule (Sec. 4.2) and skip handling (Sec. 4.1 / 6.2):
hand-worked examples, exhaustive brute force against a literal transcription,
special cases with a textbook answer, and monotonicity invariants."""
import itertools
import os

import numpy as np
import pytest

from oracle import AcceptRule, accept_block
from brute.plain_decoder import accept_literal

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "accept_examples.txt")


def load_examples():
    out = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, tt, ts, skip, d, v, n, nxt = [p.strip() for p in line.split(";")]
            out.append((name, int(tt), int(ts), int(skip), [int(x) for x in d.split()],
                        [int(x) for x in v.split()], int(n), int(nxt)))
    return out


EXAMPLES = load_examples()


@pytest.mark.parametrize("ex", EXAMPLES, ids=[e[0] for e in EXAMPLES])
def test_hand_worked_examples(ex):
    name, tt, ts, skip, d, v, n_exp, next_exp = ex
    if skip:
        # A skipped episode never reaches accept_block: the line goes through the whole verify step
        # on a small seeded model, whatever its targets would have been (Sec. 4.1 / Sec. 6.2).
        import oracle
        import synth
        from helpers import oracle_model
        sh = synth.ModelShape(1, 16, 2, 8, 24, 300)
        m = oracle_model(sh, synth.make_weights(sh, seed=3))
        kv = [[np.zeros((2, 0, 8))]]
        out = oracle.verify_step(m, kv, kv, [0], [v[0]], sh.bin_base + np.array([d]),
                                 AcceptRule(tok_threshold=tt, seq_budget=ts), skip_mask=[1])
        assert int(out["accepted_len"][0]) == n_exp == len(d) and int(out["next_token"][0]) == next_exp == -1
        assert np.all(out["target_bins"][0] == -1)
        return
    n, nb = accept_block(d, v, AcceptRule(tok_threshold=tt, seq_budget=ts))
    assert (n, nb) == (n_exp, next_exp)


@pytest.mark.parametrize("tau", [(2, 4), (2, 6), (1, 3), (0, 0), (3, 5)])
def test_exhaustive_small_biases(tau):
    """All 4^7 bias patterns in {0..3}^7, both signs alternating, against the literal transcription."""
    v = [100, 90, 80, 70, 60, 50, 1, 33]
    for pat in itertools.product(range(4), repeat=7):
        d = [v[j] + (pat[j] if j % 2 == 0 else -pat[j]) for j in range(7)]
        got = accept_block(d, v, AcceptRule(tok_threshold=tau[0], seq_budget=tau[1]))
        assert got == accept_literal(d, v, tau[0], tau[1]), (pat, tau)
        assert got[0] in (0, 3, 6, 7)


def test_strict_rule_is_longest_matching_prefix():
    """Eq. 2-2: with single-token groups and zero tolerance the rule is textbook greedy
    speculative decoding: accept up to the first draft that differs from the target."""
    rng = np.random.default_rng(0)
    rule = AcceptRule(0, 0, group_sizes=(1,), exact_group_mask=0)
    for _ in range(500):
        K = int(rng.integers(1, 15))
        v = rng.integers(0, 256, K + 1)
        d = v[:K].copy()
        flips = rng.random(K) < 0.2
        d[flips] = (d[flips] + rng.integers(1, 256, flips.sum())) % 256
        first_bad = next((j for j in range(K) if d[j] != v[j]), K)
        assert accept_block(d, v, rule) == (first_bad, int(v[first_bad]))


def test_identical_drafts_accept_everything_and_wide_thresholds_leave_gripper():
    rng = np.random.default_rng(1)
    for K in (1, 3, 6, 7, 9, 14, 21):
        v = rng.integers(0, 256, K + 1)
        assert accept_block(v[:K], v, AcceptRule(0, 0)) == (K, int(v[K]))
        d = rng.integers(0, 256, K)
        n, _ = accept_block(d, v, AcceptRule(255, 765))
        grip = [j for j in range(K) if j % 7 == 6 and d[j] != v[j]]
        assert n == (grip[0] if grip else K)


def test_monotone_in_thresholds_and_bias():
    rng = np.random.default_rng(2)
    for _ in range(300):
        v = rng.integers(20, 236, 15)
        d = v[:14] + rng.integers(-4, 5, 14)
        prev = -1
        for t in range(0, 6):
            n, _ = accept_block(d, v, AcceptRule(t, 3 * t))
            assert n >= prev and n in (0, 3, 6, 7, 10, 13, 14)
            prev = n
        n0, _ = accept_block(d, v, AcceptRule(2, 4))
        j = int(rng.integers(0, 14))
        d2 = d.copy()
        d2[j] += 1 if d2[j] >= v[j] else -1                 # grow one bias
        n1, _ = accept_block(d2, v, AcceptRule(2, 4))
        assert n1 <= n0


def test_out_of_range_draft_rejects_its_group_and_token_mode():
    v = [10, 20, 30, 40, 50, 60, 1, 99]
    assert accept_block([10, 20, 30, 40, 300, 60, 1], v, AcceptRule(255, 765)) == (3, 40)
    assert accept_block([-1, 20, 30, 40, 50, 60, 1], v, AcceptRule(255, 765)) == (0, 10)
    # token-granular variant: stops inside a group, with a running budget over the block
    r1 = AcceptRule(2, 3, mode=1)
    assert accept_block([11, 21, 30, 40, 52, 60, 1], v, r1) == (4, 50)       # 1+1+0+0 then +2 > 3
    assert accept_block([10, 20, 30, 40, 50, 60, 0], v, r1) == (6, 1)        # gripper exact
    assert accept_block([10, 23, 30, 40, 50, 60, 1], v, r1) == (1, 20)       # token over threshold
