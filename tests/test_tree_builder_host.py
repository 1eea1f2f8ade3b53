"""The library's host-side tree builder (plain CPU code behind the C ABI) against the oracle's and
against the hand-laid-out trees.  Paper Sec. 4.2: the draft tree is built sequence by sequence from
the Top-K retrieval results; sequences of different results may follow each other, except the gripper."""
import numpy as np
import pytest

import oracle
from oracle import AcceptRule
from test_oracle_tree import BUILD


@pytest.fixture(scope="module")
def pkg():
    import os
    from paper_2603_17573_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build(force=False)
    import paper_2603_17573_amd as P
    return P


def _desc(P, rule):
    return P.make_accept_desc(rule.tok_threshold, rule.seq_budget, rule.group_sizes, rule.exact_group_mask, rule.mode)


@pytest.mark.parametrize("ex", BUILD, ids=[e[0] for e in BUILD])
def test_hand_laid_out_trees(pkg, ex):
    _, cap, cands, bins, parent = ex
    tok, par = pkg.build_sequence_tree(np.array(cands), _desc(pkg, AcceptRule()), cap)
    assert tok.tolist() == bins and par.tolist() == parent


def test_random_candidates_match_the_oracle(pkg):
    rng = np.random.default_rng(12)
    for trial in range(300):
        R, K = int(rng.integers(1, 9)), int(rng.choice([7, 14, 5, 1]))
        sizes = [(3, 3, 1), (2, 1), (1,), (4, 3)][trial % 4]
        rule = AcceptRule(2, 6, group_sizes=sizes, exact_group_mask=int(rng.integers(0, 1 << len(sizes))))
        cands = rng.integers(0, int(rng.integers(2, 5)), (R, K))
        cap = int(rng.choice([256, 40, 7, 1]))
        t_ref, p_ref = oracle.build_sequence_tree(cands, rule, cap)
        tok, par = pkg.build_sequence_tree(cands, _desc(pkg, rule), cap)
        assert tok.tolist() == t_ref.tolist() and par.tolist() == p_ref.tolist(), (cands.tolist(), sizes, cap)


def test_rejects_bad_arguments(pkg):
    B = pkg.binding
    acc = pkg.make_accept_desc()
    buf = np.zeros(8, np.int32)
    assert B.heisd_build_sequence_tree(None, 1, 7, acc, 8, buf.ctypes.data, buf.ctypes.data)[0] == B.HEISD_EINVAL
    assert B.heisd_build_sequence_tree(buf.ctypes.data, 0, 7, acc, 8, buf.ctypes.data, buf.ctypes.data)[0] == B.HEISD_EINVAL
    assert B.heisd_build_sequence_tree(buf.ctypes.data, 65, 7, acc, 8, buf.ctypes.data, buf.ctypes.data)[0] == B.HEISD_EINVAL
    assert B.heisd_build_sequence_tree(buf.ctypes.data, 1, 7, acc, 0, buf.ctypes.data, buf.ctypes.data)[0] == B.HEISD_EINVAL
