"""Pins of the tree-verification oracle (paper Sec. 4.2: Top-K retrieval, sequence-wise draft tree,
chains verified from the root with the relaxed rule): hand-worked trees and selections, closed-form
node counts, an independently written recursive selection and a single masked forward on tiny
shapes, the reduction to the linear verify step, and monotonicity invariants."""
import os

import numpy as np
import pytest

import oracle
from oracle import AcceptRule, accept_block
from oracle.heisd_tree_oracle import (accept_tree, build_sequence_tree, first_chain, tree_chains,
                                      verify_tree_step)
from brute.plain_tree import accept_tree_recursive, masked_tree_logits
from test_oracle_forward import as_lists, float_model

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                yield [p.strip() for p in line.split(";")]


def _ints(s):
    return [int(x) for x in s.split()]


BUILD = [(r[0], int(r[1]), [_ints(c) for c in r[2].split("|")], _ints(r[3]), _ints(r[4]))
         for r in _rows("tree_build_examples.txt")]
ACCEPT = [(r[0], int(r[1]), int(r[2]), _ints(r[3]), _ints(r[4]), int(r[5]), _ints(r[6]), int(r[7]), _ints(r[8]),
           int(r[9])) for r in _rows("tree_accept_examples.txt")]


# ---- building the tree -------------------------------------------------------------------------

@pytest.mark.parametrize("ex", BUILD, ids=[e[0] for e in BUILD])
def test_hand_laid_out_trees(ex):
    _, cap, cands, bins, parent = ex
    tok, par = build_sequence_tree(np.array(cands), AcceptRule(), cap)
    assert tok.tolist() == bins and par.tolist() == parent


def _random_candidates(rng, R, K=7, alphabet=3):
    return rng.integers(0, alphabet, (R, K))


@pytest.mark.parametrize("R", [1, 2, 3, 4, 6])
def test_node_counts_closed_form(R):
    """R candidates whose sequences all differ: R position nodes, each followed by all R rotation
    sequences, each of those by the one gripper of its own candidate: 3R + 3R^2 + R^2 tokens."""
    cands = np.arange(R * 7).reshape(R, 7) + 1
    tok, par = build_sequence_tree(cands, AcceptRule(), 10 ** 6)
    assert len(tok) == 3 * R + 3 * R * R + R * R
    assert len(tree_chains(par)) == R * R
    same = np.tile(np.arange(7), (R, 1))
    tok, par = build_sequence_tree(same, AcceptRule(), 10 ** 6)
    assert tok.tolist() == list(range(7)) and par.tolist() == [-1, 0, 1, 2, 3, 4, 5]


def test_tree_properties_on_random_candidates():
    rng = np.random.default_rng(3)
    rule = AcceptRule()
    for _ in range(200):
        R, K = int(rng.integers(1, 6)), int(rng.choice([7, 14, 5]))
        cands = _random_candidates(rng, R, K, alphabet=int(rng.integers(2, 5)))
        cap = int(rng.choice([10 ** 6, 40]))
        tok, par = build_sequence_tree(cands, rule, cap)
        assert len(tok) <= cap and np.all(par < np.arange(len(par))) and np.all(par >= -1)
        chains = [[int(tok[t]) for t in c] for c in tree_chains(par)]
        if cap > 10 ** 5:
            for c in cands.tolist():                                  # every retrieved draft is a chain
                assert c in chains
            assert all(len(c) == K for c in chains)
        assert len({tuple(c) for c in chains}) == len(chains)         # merged siblings: no chain twice
        for c in chains:                                              # sequences come from candidates;
            j = 0                                                     # the gripper never changes candidate
            for (s, e, g) in [(0, 3, 0), (3, 6, 1), (6, 7, 2), (7, 10, 0), (10, 13, 1), (13, 14, 2)]:
                if s >= len(c):
                    break
                seg = c[s:min(e, K)]
                if len(seg) < min(e, K) - s:
                    break
                owners = [r for r in range(R) if cands[r, s:min(e, K)].tolist() == seg]
                assert owners
                if g == 2:
                    prev = c[s - 3:s]
                    assert any(cands[r, s - 3:s].tolist() == prev for r in owners)
        # preorder: a token's parent is the previous token or an earlier branching point
        assert first_chain(par) == (tree_chains(par)[0] if len(par) else [])


# ---- choosing the chain ------------------------------------------------------------------------

@pytest.mark.parametrize("ex", ACCEPT, ids=[e[0] for e in ACCEPT])
def test_hand_worked_selections(ex):
    _, tt, ts, bins, parent, fp, pred, n, path, nxt = ex
    rule = AcceptRule(tok_threshold=tt, seq_budget=ts)
    assert accept_tree(bins, parent, fp, pred, rule) == (n, path, nxt)
    assert accept_tree_recursive(bins, parent, fp, pred, tt, ts)[0::2] == (n, nxt)


def _random_tree(rng, T, branch=0.35):
    parent = []
    for t in range(T):
        if t == 0 or rng.random() < 0.15:
            parent.append(-1)
        elif rng.random() < branch:
            parent.append(int(rng.integers(0, t)))
        else:
            parent.append(t - 1)
    return parent


@pytest.mark.parametrize("tau", [(2, 6), (0, 0), (1, 2), (15, 30)])
def test_selection_against_recursive_formulation(tau):
    rng = np.random.default_rng(tau[0] * 100 + tau[1])
    rule = AcceptRule(tok_threshold=tau[0], seq_budget=tau[1])
    for _ in range(600):
        T = int(rng.integers(1, 24))
        parent = _random_tree(rng, T)
        spread = max(1, tau[0] + 1)
        pred = rng.integers(100, 100 + spread + 1, T).tolist()
        fp = int(rng.integers(100, 100 + spread + 1))
        bins = []
        for t in range(T):
            base = fp if parent[t] < 0 else pred[parent[t]]
            bins.append(int(base + rng.integers(-spread, spread + 1) * (rng.random() < 0.5)))
        got = accept_tree(bins, parent, fp, pred, rule)
        ref = accept_tree_recursive(bins, parent, fp, pred, tau[0], tau[1])
        assert got == (ref[0], ref[1], ref[2]), (parent, bins, pred, fp)
        assert got[0] == len(got[1])
        for a, b in zip(got[1][1:], got[1][:-1]):
            assert parent[a] == b
        if got[0]:
            assert parent[got[1][0]] == -1


def test_single_chain_is_the_linear_rule_and_siblings_never_hurt():
    rng = np.random.default_rng(9)
    rule = AcceptRule(2, 6)
    for _ in range(300):
        K = int(rng.integers(1, 15))
        v = rng.integers(50, 56, K + 1).tolist()
        d = (np.array(v[:K]) + rng.integers(-1, 2, K) * (rng.random(K) < 0.4)).tolist()
        chain_parent = list(range(-1, K - 1))
        n, path, nxt = accept_tree(d, chain_parent, v[0], v[1:], rule)
        assert (n, nxt) == accept_block(d, v, rule) and path == list(range(n))
        # a second chain hanging under the root can only lengthen the result
        K2 = int(rng.integers(1, 8))
        d2 = rng.integers(50, 56, K2).tolist()
        p2 = [-1] + list(range(K, K + K2 - 1))
        pred2 = rng.integers(50, 56, K2).tolist()
        n2, _, _ = accept_tree(d + d2, chain_parent + p2, v[0], v[1:] + pred2, rule)
        assert n2 >= n


def test_padding_tokens_are_in_no_chain():
    parent = [-1, 0, -2, 1, 7, -2]          # tokens 2 and 5 are padding; token 4 points forward
    assert tree_chains(parent) == [[0, 1, 3]]
    assert first_chain(parent) == [0, 1, 3]
    assert first_chain([-2, -1]) == []


# ---- the whole step ----------------------------------------------------------------------------

def _tiny_case(seed, P=4):
    m = float_model(2, 16, 2, 8, 24, n_bins=8, seed=seed, vocab=20)
    rng = np.random.default_rng(seed + 1)
    x_pre = rng.normal(0, 1, (1, P, 16))
    pre = oracle.forward_block(m, x_pre, [0])
    kv_k = [[pre["k_new"][l, 0]] for l in range(2)]
    kv_v = [[pre["v_new"][l, 0]] for l in range(2)]
    fp = int(oracle.argmax_bins(pre["logits"][0, -1]))
    return m, x_pre, kv_k, kv_v, fp


def test_one_chain_tree_is_the_linear_verify_step():
    m, _, kv_k, kv_v, fp = _tiny_case(21)
    rule = AcceptRule(3, 6)
    toks = m.bin_base + np.array([[1, 4, 2, 7, 0, 3, 5]])
    lin = oracle.verify_step(m, kv_k, kv_v, [4], [fp], toks, rule)
    tree = verify_tree_step(m, kv_k, kv_v, [4], [fp], toks, np.array([[-1, 0, 1, 2, 3, 4, 5]]), rule)
    assert tree["accepted_len"][0] == lin["accepted_len"][0] and tree["next_token"][0] == lin["next_token"][0]
    assert np.array_equal(tree["target_bins"], lin["target_bins"])
    assert np.array_equal(tree["bin_logits"], lin["bin_logits"]) and np.array_equal(tree["k_new"], lin["k_new"])
    assert tree["accepted_path"][0, :tree["accepted_len"][0]].tolist() == list(range(tree["accepted_len"][0]))


@pytest.mark.parametrize("seed", [2, 5, 8])
def test_step_against_single_masked_forward(seed):
    """Per-token logits of the chain-by-chain definition equal ONE forward over all tree tokens with an
    ancestor mask and depth positions (scalar second implementation), and the selection built on them
    equals the recursive formulation."""
    m, x_pre, kv_k, kv_v, fp = _tiny_case(seed)
    rng = np.random.default_rng(seed)
    cands = rng.integers(0, m.n_bins, (3, 7))
    cands[1, :3] = cands[0, :3]
    rule = AcceptRule(3, 7)
    tok, par = build_sequence_tree(m.bin_base + cands, rule, 64)
    out = verify_tree_step(m, kv_k, kv_v, [4], [fp], tok[None], par[None], rule)
    W, shape = as_lists(m)
    x_tree = oracle.embed(m, tok)
    ref = np.array(masked_tree_logits(W, shape, x_pre[0].tolist(), x_tree.tolist(), par.tolist()))
    assert np.allclose(out["bin_logits"][0], ref, rtol=0, atol=1e-9)
    pred = np.argmax(ref, axis=-1)
    assert np.array_equal(out["target_bins"][0, 1:], pred)
    n, path, nxt = accept_tree_recursive((tok - m.bin_base).tolist(), par.tolist(), fp, pred.tolist(), 3, 7)
    assert out["accepted_len"][0] == n and out["next_token"][0] == m.bin_base + nxt
    assert out["accepted_path"][0, :n].tolist() == path and np.all(out["accepted_path"][0, n:] == -1)


def test_teacher_forced_candidate_is_fully_accepted_and_skip_takes_first_chain():
    m, _, kv_k, kv_v, fp = _tiny_case(33)
    rule = AcceptRule(0, 0)
    # candidate 1 = the target's own greedy continuation (Eq. 2-1), candidate 0 = something else
    good, cur, k_ext, v_ext, plen = [], fp, [kv_k[l][0] for l in range(2)], [kv_v[l][0] for l in range(2)], 4
    for _ in range(7):
        good.append(cur)
        o = oracle.forward_block(m, oracle.embed(m, np.array([[m.bin_base + cur]])), [plen],
                                 [[k_ext[l]] for l in range(2)], [[v_ext[l]] for l in range(2)])
        for l in range(2):
            k_ext[l] = np.concatenate([k_ext[l], o["k_new"][l, 0]], axis=1)
            v_ext[l] = np.concatenate([v_ext[l], o["v_new"][l, 0]], axis=1)
        plen += 1
        cur = int(oracle.argmax_bins(o["logits"][0, 0]))
    bad = [(g + 1) % m.n_bins for g in good]
    tok, par = build_sequence_tree(m.bin_base + np.array([bad, good]), rule, 64)
    out = verify_tree_step(m, kv_k, kv_v, [4], [fp], tok[None], par[None], rule)
    n = int(out["accepted_len"][0])
    assert n == 7 and (tok[out["accepted_path"][0, :7]] - m.bin_base).tolist() == good
    assert out["next_token"][0] == m.bin_base + cur
    sk = verify_tree_step(m, kv_k, kv_v, [4], [fp], tok[None], par[None], rule, skip_mask=[1])
    assert sk["accepted_len"][0] == 7 and sk["next_token"][0] == -1
    assert (tok[sk["accepted_path"][0, :7]] - m.bin_base).tolist() == bad
    assert np.all(sk["target_bins"] == -1) and np.all(np.isnan(sk["bin_logits"]))
