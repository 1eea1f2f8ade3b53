"""Do the oracle's pins bite?  Each case plants ONE plausible mistake in a copy of the oracle's source (a
wrong sign, a dropped scale, a shifted mask, transposed operands, an exclusive threshold ...), swaps the
copy's functions in for the oracle's, and requires that at least one of the pin tests of
test_oracle_forward.py / test_oracle_accept.py fails.  A mutation that every pin lets through would mean
that part of the oracle is not pinned.  CPU only; the planted mistakes live in this file."""
import inspect
import sys
import types

import pytest

import oracle
import oracle.heisd_oracle as ho
import test_oracle_accept as t_acc
import test_oracle_forward as t_fwd

SRC = inspect.getsource(ho)

# (what is planted, text of the oracle's source, its replacement)
MUTATIONS = [
    ("rotation runs the other way",
     "np.concatenate([a * c - b * s, b * c + a * s], axis=-1)", "np.concatenate([a * c + b * s, b * c - a * s], axis=-1)"),
    ("rotary frequencies fall twice as fast",
     "** (-2.0 * np.arange(half, dtype=np.float64) / hd)", "** (-4.0 * np.arange(half, dtype=np.float64) / hd)"),
    ("scores are not divided by sqrt(head_dim)",
     's = np.einsum("thd,hrd->htr", q, k_all) / np.sqrt(float(hd))', 's = np.einsum("thd,hrd->htr", q, k_all)'),
    ("a query does not see its own row",
     "s = np.where(r <= p0 + t, s, -np.inf)", "s = np.where((r < p0 + t) | (r == 0), s, -np.inf)"),
    ("a query sees the whole block",
     "s = np.where(r <= p0 + t, s, -np.inf)", "s = np.where(r <= p0 + T, s, -np.inf)"),
    ("keys and values change places",
     "o[b] = attention_block(qb, k_all, v_all, p0)", "o[b] = attention_block(qb, v_all, k_all, p0)"),
    ("keys are not rotated",
     "kb = rope(k[b], pos, m.rope_base)", "kb = k[b]"),
    ("eps is added outside the root",
     "return x / np.sqrt(ms + eps) * np.asarray(g, dtype=np.float64)",
     "return x / (np.sqrt(ms) + eps) * np.asarray(g, dtype=np.float64)"),
    ("the norm's gain is dropped",
     "return x / np.sqrt(ms + eps) * np.asarray(g, dtype=np.float64)", "return x / np.sqrt(ms + eps)"),
    ("SiLU has the wrong sign in the exponent",
     "return z / (1.0 + np.exp(-z))", "return z / (1.0 + np.exp(z))"),
    ("gate and up change places",
     'a = silu(m.linear(h, "w_gate", l)) * m.linear(h, "w_up", l)', 'a = silu(m.linear(h, "w_up", l)) * m.linear(h, "w_gate", l)'),
    ("the FFN's residual is dropped",
     'x = x + m.linear(a, "w_down", l)', 'x = m.linear(a, "w_down", l)'),
    ("the attention's residual is dropped",
     'x = x + m.linear(o.reshape(B, T, d), "wo", l)', 'x = m.linear(o.reshape(B, T, d), "wo", l)'),
    ("the final norm is skipped",
     'feat = rmsnorm(x, m.weights["final_norm"], m.rms_eps)', "feat = x"),
    ("ties in the greedy choice go to the highest bin",
     "return np.argmax(lg, axis=-1).astype(np.int32)     # numpy returns the first maximum",
     "return (lg.shape[-1] - 1 - np.argmax(lg[..., ::-1], axis=-1)).astype(np.int32)"),
    ("the token threshold is exclusive",
     "ok = all(bj <= rule.tok_threshold for bj in grp) and sum(grp) <= rule.seq_budget",
     "ok = all(bj < rule.tok_threshold for bj in grp) and sum(grp) <= rule.seq_budget"),
    ("the sequence budget is exclusive",
     "ok = all(bj <= rule.tok_threshold for bj in grp) and sum(grp) <= rule.seq_budget",
     "ok = all(bj <= rule.tok_threshold for bj in grp) and sum(grp) < rule.seq_budget"),
    ("the sequence budget bounds the mean bias, not the sum",
     "ok = all(bj <= rule.tok_threshold for bj in grp) and sum(grp) <= rule.seq_budget",
     "ok = all(bj <= rule.tok_threshold for bj in grp) and sum(grp) / len(grp) <= rule.seq_budget"),
    ("the gripper is judged like the other sequences",
     "ok = all(bj == 0 for bj in grp)", "ok = all(bj <= rule.tok_threshold for bj in grp)"),
    ("a rejected sequence does not block the later ones",
     "            if not ok:\n                break\n            n = e", "            if ok:\n                n = e"),
    ("the next token is the target's bin one position late",
     "return n, int(target_bins[n])", "return n, int(target_bins[min(n + 1, K)])"),
    ("a skipped episode accepts nothing",
     "accepted = np.full(B, K, dtype=np.int32)", "accepted = np.zeros(B, dtype=np.int32)"),
]

NAMES = ("embed", "rmsnorm", "rope", "silu", "attention_block", "forward_block", "prefill", "bin_logits",
         "argmax_bins", "accept_block", "verify_step")


def _pins():
    """The pin tests as plain calls (parametrised ones once per parameter)."""
    calls = []
    for cfg in t_fwd.test_against_second_plain_implementation.pytestmark[0].args[1]:
        calls.append(lambda cfg=cfg: t_fwd.test_against_second_plain_implementation(cfg))
    calls += [t_fwd.test_block_equals_sequential_equals_uncached,
              t_fwd.test_zero_layers_reduce_to_one_gemv_and_constructed_shift,
              t_fwd.test_skip_rows_bypass_verification,
              t_fwd.test_rmsnorm_rope_attention_argmax_closed_forms]
    for ex in t_acc.EXAMPLES:
        calls.append(lambda ex=ex: t_acc.test_hand_worked_examples(ex))
    calls += [t_acc.test_strict_rule_is_longest_matching_prefix,
              t_acc.test_identical_drafts_accept_everything_and_wide_thresholds_leave_gripper,
              t_acc.test_monotone_in_thresholds_and_bias,
              t_acc.test_out_of_range_draft_rejects_its_group_and_token_mode,
              lambda: t_acc.test_exhaustive_small_biases((2, 4))]
    return calls


def _swap(mod):
    """Put mod's functions where the pins look the oracle's up; returns what to restore."""
    saved = []
    for name in NAMES:
        orig = getattr(ho, name)
        for holder in (oracle, ho, t_acc, t_fwd, sys.modules.get("helpers")):
            if holder is not None and getattr(holder, name, None) is orig:
                saved.append((holder, name, orig))
                setattr(holder, name, getattr(mod, name))
    return saved


def test_unmutated_copy_passes_every_pin():
    mod = types.ModuleType("oracle_copy")
    mod.__dict__["__file__"] = ho.__file__
    exec(compile(SRC, "oracle_copy", "exec"), mod.__dict__)
    saved = _swap(mod)
    try:
        for call in _pins():
            call()
    finally:
        for holder, name, orig in saved:
            setattr(holder, name, orig)


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_a_pin(what, old, new):
    assert SRC.count(old) == 1, "the oracle's source no longer holds this line: update the mutation"
    mod = types.ModuleType("oracle_mutant")
    mod.__dict__["__file__"] = ho.__file__
    exec(compile(SRC.replace(old, new), "oracle_mutant", "exec"), mod.__dict__)
    saved = _swap(mod)
    caught = 0
    try:
        for call in _pins():
            try:
                call()
            except pytest.skip.Exception:
                continue
            except Exception:            # an assertion of the pin, or an error the mistake provokes inside it
                caught += 1
                break
    finally:
        for holder, name, orig in saved:
            setattr(holder, name, orig)
    assert caught, "no pin noticed: %s" % what
