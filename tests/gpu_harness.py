"""Runs the HIP path through the C ABI binding and compares it with oracle results.
Shared by the GPU tests, smoke() and nothing else."""
import numpy as np
import torch

import oracle
import synth
from paper_2603_17573_amd import DeviceModel, Verifier, make_accept_desc

LOGIT_TOL = 3e-2      # max |delta logit| / (oracle row range), the bar the benchmark spec sets


def accept_desc_of(rule: oracle.AcceptRule):
    return make_accept_desc(rule.tok_threshold, rule.seq_budget, rule.group_sizes, rule.exact_group_mask,
                            rule.mode)


def _bits_to_dev(bits, device):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def _dev_to_bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def run_gpu_step(shape, weights, kb, vb, plen, first, drafts, rule, skip, device="cuda:0",
                 model=None, max_batch=None, max_k=None, repeat=1, path=0, act=0):
    """One heisd_verify_step on the GPU.  kb/vb: bf16 bits [L][B][H][cap][hd].  Returns numpy outputs
    plus the caches after the step."""
    dm = model or DeviceModel(shape, weights, device)
    B, K = drafts.shape
    cap = kb.shape[3]
    ver = Verifier(dm, max_batch or B, max_k or K, cap)
    from paper_2603_17573_amd import heisd_verify_set_path
    assert heisd_verify_set_path(ver.ctx, path) == 0
    if act:
        from paper_2603_17573_amd import heisd_verify_set_activations
        assert heisd_verify_set_activations(ver.ctx, act) == 0
    kc, vc = _bits_to_dev(kb, device), _bits_to_dev(vb, device)
    t_plen = torch.from_numpy(np.asarray(plen, np.int32)).to(device)
    t_first = torch.from_numpy(np.asarray(first, np.int32)).to(device)
    t_drafts = torch.from_numpy(np.ascontiguousarray(drafts, dtype=np.int32)).to(device)
    t_skip = None if skip is None else torch.from_numpy(np.asarray(skip, np.uint8)).to(device)
    out = None
    for _ in range(repeat):
        out = ver.step(kc, vc, t_plen, t_first, t_drafts, accept_desc_of(rule), t_skip, out=out)
    torch.cuda.synchronize()
    from paper_2603_17573_amd import heisd_verify_check
    assert heisd_verify_check(ver.ctx) == 0, "device error word set"
    res = {k: v.cpu().numpy() for k, v in out.items()}
    res["k_cache"], res["v_cache"] = _dev_to_bits(kc), _dev_to_bits(vc)
    ver.close()
    return res


def compare_with_oracle(got, ref, drafts, rule, shape, kb0=None, vb0=None, plen=None, skip=None,
                        episodes=None):
    """Element-by-element parity of one step.  `episodes` maps oracle rows to GPU rows when the
    oracle only ran a sample of the batch.  Returns a dict of measured statistics."""
    B, K = drafts.shape
    eps = list(range(B)) if episodes is None else list(episodes)
    skip = np.zeros(B, bool) if skip is None else np.asarray(skip).astype(bool)
    worst, exempt, rows, mism_exempt = 0.0, 0, 0, 0
    for i, b in enumerate(eps):
        if skip[b]:
            assert got["accepted_len"][b] == K and got["next_token"][b] == -1
            assert np.all(got["target_bins"][b] == -1)
            assert np.all(np.isnan(got["bin_logits"][b]))
            assert ref["accepted_len"][i] == K and ref["next_token"][i] == -1
            continue
        lo = ref["bin_logits"][i]                       # [K, n_bins] fp64
        lg = got["bin_logits"][b].astype(np.float64)
        assert np.all(np.isfinite(lg))
        rng_ = lo.max(axis=-1) - lo.min(axis=-1)
        err = np.abs(lg - lo).max(axis=-1) / rng_
        worst = max(worst, float(err.max()))
        assert err.max() <= LOGIT_TOL, "logit error %.3g of the row range" % err.max()
        srt = np.sort(lo, axis=-1)
        margin = (srt[:, -1] - srt[:, -2]) / rng_
        decided = margin > LOGIT_TOL                      # rows whose argmax the tolerance cannot flip
        tb_ref, tb_got = ref["target_bins"][i], got["target_bins"][b]
        assert tb_got[0] == tb_ref[0]
        assert np.array_equal(tb_got[1:][decided], tb_ref[1:][decided]), "argmax differs on a decided row"
        rows += K
        exempt += int((~decided).sum())
        mism_exempt += int((tb_got[1:] != tb_ref[1:]).sum())
        if decided.all():
            assert got["accepted_len"][b] == ref["accepted_len"][i]
            assert got["next_token"][b] == ref["next_token"][i]
        # the acceptance logic itself: bit-exact given the GPU's own argmax
        n, nb = oracle.accept_block(np.asarray(drafts[b]) - shape.bin_base, tb_got, rule, shape.n_bins)
        assert got["accepted_len"][b] == n and got["next_token"][b] == shape.bin_base + nb
    stats = {"max_logit_err_over_range": worst, "rows": rows, "undecided_rows": exempt,
             "argmax_mismatches": mism_exempt}
    if kb0 is not None:
        stats.update(compare_cache(got, ref, kb0, vb0, plen, skip, K, eps))
    return stats


def compare_cache(got, ref, kb0, vb0, plen, skip, K, eps):
    """Appended rows equal the oracle's new keys/values up to one bf16 rounding plus the arithmetic
    error of the layers below them; every other row of the cache is untouched.

    Tolerance per element of layer l: |r| * 2^-8 (half a bf16 ulp, with slack for a value that
    rounds across a binade) + (5e-5 + 2e-5 * l) * max|r|: fp32 accumulation and 16-bit split
    activations, compounding with depth."""
    worst = 0.0
    per_layer = []
    for name, c0, new in (("k_cache", kb0, ref["k_new"]), ("v_cache", vb0, ref["v_new"])):
        after = got[name]
        L = after.shape[0]
        lay_err = np.zeros(L)
        for i, b in enumerate(eps):
            if skip[b]:
                assert np.array_equal(after[:, b], c0[:, b]), "%s of a skipped episode modified" % name
                continue
            p = int(plen[b])
            assert np.array_equal(after[:, b, :, :p], c0[:, b, :, :p]) and \
                np.array_equal(after[:, b, :, p + K:], c0[:, b, :, p + K:]), \
                "%s modified outside the appended rows" % name
            a = synth.bf16_bits_to_f32(after[:, b, :, p:p + K, :]).astype(np.float64)
            r = new[:, i]                                 # [L, H, K, hd]
            scale = np.abs(r).reshape(L, -1).max(axis=1)
            e = np.abs(a - r) - np.abs(r) * 2.0 ** -8
            rel = e.reshape(L, -1).max(axis=1) / scale
            lay_err = np.maximum(lay_err, rel)
        per_layer.append(lay_err)
        tol = 5e-5 + 2e-5 * np.arange(L)
        assert np.all(lay_err <= tol), "appended %s rows off; excess error per layer / scale: %s" % (
            name, np.array2string(lay_err, precision=5))
        worst = max(worst, float(lay_err.max()))
    return {"max_kv_excess_err_over_scale": worst,
            "kv_err_first_last_layer": [float(per_layer[0][0]), float(per_layer[0][-1])]}


# ---- tree verification -------------------------------------------------------------------------

def run_gpu_tree_step(shape, weights, kb, vb, plen, first, tokens, parent, rule, skip, device="cuda:0",
                      model=None, max_batch=None, max_k=None, repeat=1, path=0):
    """One heisd_verify_tree_step on the GPU.  tokens, parent: i32 [B][T].  Returns numpy outputs plus
    the caches after the step."""
    dm = model or DeviceModel(shape, weights, device)
    B, T = tokens.shape
    cap = kb.shape[3]
    ver = Verifier(dm, max_batch or B, max_k or T, cap)
    from paper_2603_17573_amd import heisd_verify_set_path, heisd_verify_check
    assert heisd_verify_set_path(ver.ctx, path) == 0
    kc, vc = _bits_to_dev(kb, device), _bits_to_dev(vb, device)
    t_plen = torch.from_numpy(np.asarray(plen, np.int32)).to(device)
    t_first = torch.from_numpy(np.asarray(first, np.int32)).to(device)
    t_tok = torch.from_numpy(np.ascontiguousarray(tokens, dtype=np.int32)).to(device)
    t_par = torch.from_numpy(np.ascontiguousarray(parent, dtype=np.int32)).to(device)
    t_skip = None if skip is None else torch.from_numpy(np.asarray(skip, np.uint8)).to(device)
    out = None
    for _ in range(repeat):
        out = ver.tree_step(kc, vc, t_plen, t_first, t_tok, t_par, accept_desc_of(rule), t_skip, out=out)
    torch.cuda.synchronize()
    assert heisd_verify_check(ver.ctx) == 0, "device error word set"
    res = {k: v.cpu().numpy() for k, v in out.items()}
    res["k_cache"], res["v_cache"] = _dev_to_bits(kc), _dev_to_bits(vc)
    ver.close()
    return res


def compare_tree_with_oracle(got, ref, tokens, parent, rule, shape, kb0, vb0, plen, first, skip=None,
                             episodes=None):
    """Parity of one tree step.  ref: oracle.verify_tree_step on the episodes listed (all by default)."""
    B, T = tokens.shape
    eps = list(range(B)) if episodes is None else list(episodes)
    skip = np.zeros(B, bool) if skip is None else np.asarray(skip).astype(bool)
    worst, rows, exempt, mism, worst_kv = 0.0, 0, 0, 0, 0.0
    L = got["k_cache"].shape[0]
    for i, b in enumerate(eps):
        p = int(plen[b])
        n_got = int(got["accepted_len"][b])
        path_got = got["accepted_path"][b]
        if skip[b]:
            chain = oracle.first_chain(parent[b])
            assert n_got == len(chain) == ref["accepted_len"][i] and got["next_token"][b] == -1
            assert path_got[:n_got].tolist() == chain and np.all(path_got[n_got:] == -1)
            assert np.all(got["target_bins"][b] == -1) and np.all(np.isnan(got["bin_logits"][b]))
            for name, c0 in (("k_cache", kb0), ("v_cache", vb0)):
                assert np.array_equal(got[name][:, b], c0[:, b]), "%s of a skipped episode modified" % name
            continue
        in_tree = ref["target_bins"][i, 1:] >= 0
        lo = ref["bin_logits"][i][in_tree]
        lg = got["bin_logits"][b].astype(np.float64)[in_tree]
        assert np.all(np.isfinite(got["bin_logits"][b]))
        rng_ = lo.max(axis=-1) - lo.min(axis=-1)
        err = np.abs(lg - lo).max(axis=-1) / rng_
        worst = max(worst, float(err.max()))
        assert err.max() <= LOGIT_TOL, "logit error %.3g of the row range" % err.max()
        srt = np.sort(lo, axis=-1)
        decided = (srt[:, -1] - srt[:, -2]) / rng_ > LOGIT_TOL
        tb_ref, tb_got = ref["target_bins"][i], got["target_bins"][b]
        assert tb_got[0] == tb_ref[0] == first[b]
        assert np.all(tb_got[1:][~in_tree] == -1)
        assert np.array_equal(tb_got[1:][in_tree][decided], tb_ref[1:][in_tree][decided]), "argmax differs on a decided row"
        rows += int(in_tree.sum())
        exempt += int((~decided).sum())
        mism += int((tb_got[1:] != tb_ref[1:]).sum())
        if decided.all():
            assert n_got == ref["accepted_len"][i] and got["next_token"][b] == ref["next_token"][i]
            assert np.array_equal(path_got, ref["accepted_path"][i])
        # chain selection: bit-exact given the GPU's own greedy bins
        n, pth, nb = oracle.accept_tree(np.asarray(tokens[b]) - shape.bin_base, parent[b], int(first[b]), tb_got[1:],
                                        rule, shape.n_bins)
        assert n_got == n and got["next_token"][b] == shape.bin_base + nb
        assert path_got[:n].tolist() == pth and np.all(path_got[n:] == -1)
        # the cache: prefix and rows past the tree untouched; rows p .. p+n-1 hold the accepted tokens
        for name, c0, new in (("k_cache", kb0, ref["k_new"]), ("v_cache", vb0, ref["v_new"])):
            after = got[name]
            assert np.array_equal(after[:, b, :, :p], c0[:, b, :, :p]) and \
                np.array_equal(after[:, b, :, p + T:], c0[:, b, :, p + T:]), "%s modified outside the tree rows" % name
            if n == 0:
                continue
            a = synth.bf16_bits_to_f32(after[:, b, :, p:p + n, :]).astype(np.float64)
            r = new[:, i][:, :, pth, :]                       # [L, H, n, hd]
            scale = np.abs(new[:, i][:, :, in_tree, :]).reshape(L, -1).max(axis=1)
            e = np.abs(a - r) - np.abs(r) * 2.0 ** -8
            rel = e.reshape(L, -1).max(axis=1) / scale
            tol = 5e-5 + 2e-5 * np.arange(L)
            assert np.all(rel <= tol), "accepted %s rows off; excess error per layer / scale: %s" % (
                name, np.array2string(rel, precision=5))
            worst_kv = max(worst_kv, float(rel.max()))
    return {"max_logit_err_over_range": worst, "rows": rows, "undecided_rows": exempt, "argmax_mismatches": mism,
            "max_kv_excess_err_over_scale": worst_kv}
