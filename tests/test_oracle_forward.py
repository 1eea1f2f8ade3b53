"""Pins of the oracle's decoder forward: a second plain implementation on tiny shapes,
the equivalence of block / sequential / uncached evaluation that Eq. 2-1 and Eq. 2-2
imply, and closed forms."""
import numpy as np
import pytest

import oracle
import synth
from brute.plain_decoder import full_sequence_logits
from helpers import oracle_model, oracle_prefix_cache


def float_model(L, d, H, hd, F, n_bins, seed, scale=0.6, vocab=None):
    """Small model with float (not bf16) weights large enough that attention and the
    nonlinearity matter."""
    rng = np.random.default_rng(seed)
    vocab = vocab or (n_bins + 10)
    w = {"tok_emb": rng.normal(0, 1.0, (vocab, d)), "lm_head": rng.normal(0, scale, (vocab, d)),
         "final_norm": rng.uniform(0.5, 1.5, d)}
    for nm, (o, i) in {"wq": (H * hd, d), "wk": (H * hd, d), "wv": (H * hd, d), "wo": (d, H * hd),
                       "w_gate": (F, d), "w_up": (F, d), "w_down": (d, F)}.items():
        w[nm] = [rng.normal(0, scale, (o, i)) for _ in range(L)]
    w["attn_norm"] = [rng.uniform(0.5, 1.5, d) for _ in range(L)]
    w["ffn_norm"] = [rng.uniform(0.5, 1.5, d) for _ in range(L)]
    return oracle.OracleModel(L, d, H, hd, F, vocab, w, n_bins=n_bins, rms_eps=1e-5, rope_base=100.0)


def as_lists(m):
    W = {k: [a.tolist() for a in m.weights[k]] for k in
         ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "attn_norm", "ffn_norm")}
    W["final_norm"] = m.weights["final_norm"].tolist()
    W["lm_bins"] = m.weights["lm_head"][m.bin_base:m.bin_base + m.n_bins].tolist()
    shape = dict(n_layers=m.n_layers, n_heads=m.n_heads, head_dim=m.head_dim, rms_eps=m.rms_eps,
                 rope_base=m.rope_base)
    return W, shape


@pytest.mark.parametrize("cfg", [(1, 8, 2, 4, 12, 3, 2), (2, 12, 3, 4, 10, 4, 3), (2, 8, 1, 8, 6, 1, 4)])
def test_against_second_plain_implementation(cfg):
    L, d, H, hd, F, P, K = cfg
    m = float_model(L, d, H, hd, F, n_bins=6, seed=sum(cfg))
    rng = np.random.default_rng(11)
    x = rng.normal(0, 1, (P + K, d))
    W, shape = as_lists(m)
    ref_logits, ref_feat = full_sequence_logits(W, shape, x.tolist())
    ref_logits, ref_feat = np.array(ref_logits), np.array(ref_feat)
    # (a) the oracle over the whole sequence at once
    full = oracle.forward_block(m, x[None], [0])
    assert np.allclose(full["logits"][0], ref_logits, rtol=0, atol=1e-10)
    assert np.allclose(full["feat"][0], ref_feat, rtol=0, atol=1e-10)
    # (b) prefix first, then the K-token block against the earlier rows (the verify forward)
    pre = oracle.forward_block(m, x[None, :P], [0])
    kv_k = [[pre["k_new"][l, 0]] for l in range(L)]
    kv_v = [[pre["v_new"][l, 0]] for l in range(L)]
    blk = oracle.forward_block(m, x[None, P:], [P], kv_k, kv_v)
    assert np.allclose(blk["logits"][0], ref_logits[P:], rtol=0, atol=1e-10)
    assert np.array_equal(oracle.argmax_bins(blk["logits"][0]), np.argmax(ref_logits[P:], axis=-1))


def test_block_equals_sequential_equals_uncached():
    """Verification evaluates in one pass what autoregressive decoding (Eq. 2-1) computes token by token."""
    m = float_model(2, 32, 4, 8, 48, n_bins=16, seed=5)
    rng = np.random.default_rng(6)
    B, P, K = 3, 5, 7
    plen = [5, 3, 4]
    x_pre = rng.normal(0, 1, (B, P, 32))
    x_new = rng.normal(0, 1, (B, K, 32))
    kv_k = [[None] * B for _ in range(2)]
    kv_v = [[None] * B for _ in range(2)]
    unc = []
    for b in range(B):
        pre = oracle.forward_block(m, x_pre[b:b + 1, :plen[b]], [0])
        for l in range(2):
            kv_k[l][b], kv_v[l][b] = pre["k_new"][l, 0], pre["v_new"][l, 0]
        unc.append(oracle.forward_block(m, np.concatenate([x_pre[b, :plen[b]], x_new[b]])[None], [0])
                   ["logits"][0, plen[b]:])
    blk = oracle.forward_block(m, x_new, plen, kv_k, kv_v)
    for b in range(B):
        assert np.allclose(blk["logits"][b], unc[b], rtol=0, atol=1e-9)
    # sequential single-token decode with a growing cache
    kk = [[kv_k[l][b] for b in range(B)] for l in range(2)]
    vv = [[kv_v[l][b] for b in range(B)] for l in range(2)]
    cur = list(plen)
    for j in range(K):
        st = oracle.forward_block(m, x_new[:, j:j + 1], cur, kk, vv)
        assert np.allclose(st["logits"][:, 0], blk["logits"][:, j], rtol=0, atol=1e-9)
        for l in range(2):
            for b in range(B):
                kk[l][b] = np.concatenate([kk[l][b], st["k_new"][l, b]], axis=1)
                vv[l][b] = np.concatenate([vv[l][b], st["v_new"][l, b]], axis=1)
        cur = [c + 1 for c in cur]
    # permuting episodes permutes outputs
    perm = [2, 0, 1]
    pk = [[kv_k[l][b] for b in perm] for l in range(2)]
    pv = [[kv_v[l][b] for b in perm] for l in range(2)]
    blk_p = oracle.forward_block(m, x_new[perm], [plen[b] for b in perm], pk, pv)
    assert np.array_equal(blk_p["logits"], blk["logits"][perm])


def test_zero_layers_reduce_to_one_gemv_and_constructed_shift():
    """With all layer matrices zero the residual stream is the embedding, so the bin logits are
    W_lm . RMSNorm(E[t]).  With one-hot embeddings and a cyclically shifted one-hot head the
    target's next bin is (draft bin + c) mod 256, which fixes every step of verify_step by hand."""
    nb, d, c = 256, 256, 37
    sh = synth.ModelShape(2, d, 4, 64, 32, 300, n_bins=nb)
    base = sh.bin_base
    w = {k: [np.zeros(s) for _ in range(2)] for k, s in
         {"wq": (d, d), "wk": (d, d), "wv": (d, d), "wo": (d, d), "w_gate": (32, d), "w_up": (32, d),
          "w_down": (d, 32)}.items()}
    w["attn_norm"] = [np.ones(d)] * 2
    w["ffn_norm"] = [np.ones(d)] * 2
    w["final_norm"] = np.ones(d)
    E = np.zeros((300, d))
    Wl = np.zeros((300, d))
    for b in range(nb):
        E[base + b, b] = 3.0
        Wl[base + (b + c) % nb, b] = 1.0
    w["tok_emb"], w["lm_head"] = E, Wl
    m = oracle_model(sh, w)
    K = 7
    d_bins = np.array([[5, 42, 79, 116, 153, 190, 227], [250, 31, 0, 1, 2, 3, 4]])
    kv = [[np.zeros((4, 0, 64))] * 2 for _ in range(2)]
    # single GEMV check
    f = oracle.rmsnorm(E[base + d_bins[0]], np.ones(d), sh.rms_eps)
    lg = oracle.forward_block(m, E[base + d_bins][:, :, :], [0, 0])["logits"]
    assert np.allclose(lg[0], f @ Wl[base:base + nb].T, atol=1e-12)
    assert np.allclose(lg[0].max(axis=-1), 3.0 / np.sqrt(9.0 / d + sh.rms_eps), atol=1e-9)
    out = oracle.verify_step(m, kv, kv, [0, 0], first_pred=[5, 250], draft_tokens=base + d_bins,
                             rule=oracle.AcceptRule(2, 6))
    assert np.array_equal(out["target_bins"][0], [5] + list((d_bins[0] + c) % nb))
    # episode 0: drafts chain by +37 so every v_j equals d_j: all accepted, bonus = (227+37)%256
    assert out["accepted_len"][0] == 7 and out["next_token"][0] == base + (227 + c) % nb
    # episode 1: d_1 = 31 = (250+37)%256 ok, d_2 = 0 but v_2 = 68: first group fails as a whole
    assert out["accepted_len"][1] == 0 and out["next_token"][1] == base + 250


def test_skip_rows_bypass_verification():
    sh = synth.ModelShape(1, 16, 2, 8, 24, 300)
    m = oracle_model(sh, synth.make_weights(sh, seed=3))
    kv = [[np.zeros((2, 0, 8))] * 3]
    drafts = sh.bin_base + np.array([[1, 2, 3, 4, 5, 6, 7]] * 3)
    out = oracle.verify_step(m, kv, kv, [0, 0, 0], [1, 1, 1], drafts, oracle.AcceptRule(2, 6),
                             skip_mask=[0, 1, 0])
    assert out["accepted_len"][1] == 7 and out["next_token"][1] == -1
    assert np.all(out["target_bins"][1] == -1) and np.all(np.isnan(out["bin_logits"][1]))
    assert np.array_equal(out["target_bins"][0], out["target_bins"][2]) and out["target_bins"][0][0] == 1
    alone = oracle.verify_step(m, [[kv[0][0]]], [[kv[0][0]]], [0], [1], drafts[:1], oracle.AcceptRule(2, 6))
    assert np.allclose(alone["bin_logits"][0], out["bin_logits"][2], atol=1e-12)


def test_rmsnorm_rope_attention_argmax_closed_forms():
    g = np.array([0.5, -2.0, 3.0, 1.0])
    assert np.allclose(oracle.rmsnorm(np.full(4, -7.0), g, 0.0), -g)
    assert np.allclose(oracle.rmsnorm(np.array([3.0, 4.0, 0.0, 0.0]), np.ones(4), 0.0),
                       np.array([3.0, 4.0, 0, 0]) / 2.5)
    # rotation direction and pairing: hd = 4 pairs (0,2) and (1,3); theta_0 = 1, theta_1 = base^(-1/2)
    u = np.array([1.0, 1.0, 0.0, 0.0]).reshape(1, 1, 4)
    r = oracle.rope(u, np.array([np.pi / 2]), 4.0)[0, 0]
    assert np.allclose(r, [0.0, np.cos(np.pi / 4), 1.0, np.sin(np.pi / 4)], atol=1e-12)
    rng = np.random.default_rng(0)
    q, k = rng.normal(size=(1, 2, 16)), rng.normal(size=(1, 2, 16))
    assert np.allclose(oracle.rope(q, np.array([0]), 1e4), q)
    assert np.allclose(np.linalg.norm(oracle.rope(q, np.array([13]), 1e4)), np.linalg.norm(q))
    dots = [np.sum(oracle.rope(q, np.array([m_]), 1e4) * oracle.rope(k, np.array([m_ - 3]), 1e4))
            for m_ in (3, 10, 77)]
    assert np.allclose(dots, dots[0])
    # identical keys: uniform weights over the visible rows -> running mean of the values
    kk = np.tile(rng.normal(size=(1, 1, 4)), (1, 5, 1))
    vv = rng.normal(size=(1, 5, 4))
    o = oracle.attention_block(rng.normal(size=(3, 1, 4)), kk, vv, 2)
    for t in range(3):
        assert np.allclose(o[t, 0], vv[0, :3 + t].mean(axis=0))
    assert oracle.argmax_bins(np.zeros((2, 256))).tolist() == [0, 0]
    z = np.zeros(8)
    z[[3, 5]] = 2.0
    z[1] = np.nan
    assert oracle.argmax_bins(z) == 3
    assert np.isclose(oracle.silu(np.array([0.0, 1.0]))[1], 1.0 / (1.0 + np.exp(-1.0)))


def test_bf16_prefix_cache_round_trip_on_c0_shape():
    """C0-shaped run end to end on the CPU: prefill -> bf16 cache -> verify step.  Rounding the
    prefix K/V to bf16 moves the logits by far less than the parity tolerance."""
    wl = synth.WORKLOADS["C0"]
    m = oracle_model(wl.shape, synth.make_weights(wl.shape, wl.seed))
    cap = wl.prefix_len + wl.K
    kb, vb, plen, first = oracle_prefix_cache(m, wl, cap)
    drafts = wl.shape.bin_base + synth.make_drafts_uniform(wl)
    out = oracle.verify_step(m, kb, vb, plen, first, drafts, oracle.AcceptRule(wl.tau_tok, wl.tau_seq))
    from helpers import prefix_embeddings
    x = np.concatenate([prefix_embeddings(m, wl, 0), oracle.embed(m, drafts[0])])[None]
    exact = oracle.forward_block(m, x, [0])["logits"][0, wl.prefix_len:]
    rng_ = exact.max(axis=-1) - exact.min(axis=-1)
    assert np.max(np.abs(out["bin_logits"][0] - exact) / rng_[:, None]) < 2e-3
    assert out["target_bins"][0, 0] == first[0]
    assert out["accepted_len"][0] in (0, 3, 6, 7)
    assert out["next_token"][0] == wl.shape.bin_base + out["target_bins"][0, out["accepted_len"][0]]


def test_c_linear_equals_library_matmul():
    """The oracle's C routine for bf16-stored weights against numpy's matmul on the widened matrix,
    including row counts that are not a multiple of its 4-row grouping."""
    rng = np.random.default_rng(4)
    for (T, Kd, N) in [(1, 8, 1), (7, 40, 6), (5, 33, 7), (3, 256, 17), (64, 100, 50)]:
        w = synth.f32_to_bf16_bits(rng.normal(0, 0.3, (N, Kd)).astype(np.float32))
        x = rng.normal(0, 1, (T, Kd))
        ref = x @ oracle.widen_bf16(w).T
        got = oracle.linear_bf16w(x, w)
        assert got.shape == (T, N) and np.allclose(got, ref, rtol=1e-13, atol=1e-13)
    # widening is exact: the fp64 value equals the fp32 reading of the same bits
    bits = rng.integers(0, 0x7F80, 1000).astype(np.uint16)
    assert np.array_equal(oracle.widen_bf16(bits), synth.bf16_bits_to_f32(bits).astype(np.float64))
    x3 = rng.normal(0, 1, (2, 3, 40))
    w = synth.f32_to_bf16_bits(rng.normal(0, 0.3, (6, 40)).astype(np.float32))
    assert np.allclose(oracle.linear_bf16w(x3, w), x3 @ oracle.widen_bf16(w).T, atol=1e-13)
