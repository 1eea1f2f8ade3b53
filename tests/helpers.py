"""Glue for the tests: builds oracle-side objects from generated inputs.  Holds no arithmetic
of the method: it only calls oracle/ and synth/ and converts storage formats."""
import numpy as np

import oracle
import synth


def oracle_model(shape: synth.ModelShape, weights) -> oracle.OracleModel:
    return oracle.OracleModel(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim,
                              shape.d_ffn, shape.vocab, weights, shape.n_bins, shape.rms_eps,
                              shape.rope_base)


def prefix_embeddings(model: oracle.OracleModel, wl: synth.Workload, episode: int) -> np.ndarray:
    """[P, d] fp64 input rows of one episode's prefix: visual rows as given, text rows looked up."""
    emb, ids = synth.make_prefix_inputs(wl, episode)
    parts = [emb.astype(np.float64)] if wl.n_visual else []
    if wl.n_text:
        parts.append(oracle.embed(model, ids))
    return np.concatenate(parts, axis=0)


def oracle_prefix_cache(model: oracle.OracleModel, wl: synth.Workload, capacity: int, episodes=None):
    """Prefill every episode's prefix with the oracle and round the K/V once to bf16.
    Returns (k_bits, v_bits) u16[L][B][H][cap][hd], prefix_len i32[B], first_pred i32[B]."""
    sh = wl.shape
    eps = list(range(wl.batch)) if episodes is None else list(episodes)
    B, P = len(eps), wl.prefix_len
    kb = np.zeros((sh.n_layers, B, sh.n_heads, capacity, sh.head_dim), np.uint16)
    vb = np.zeros_like(kb)
    first = np.zeros(B, np.int32)
    for i, e in enumerate(eps):
        x = prefix_embeddings(model, wl, e)[None]
        out = oracle.prefill(model, x)
        kb[:, i, :, :P, :] = synth.f32_to_bf16_bits(out["k_new"][:, 0].astype(np.float32))
        vb[:, i, :, :P, :] = synth.f32_to_bf16_bits(out["v_new"][:, 0].astype(np.float32))
        first[i] = out["first_pred"][0]
    return kb, vb, np.full(B, P, np.int32), first


def direct_prefix_cache(wl: synth.Workload, capacity: int, episodes=None):
    """Prefix K/V drawn directly by the generator (no prefill), same layout as above."""
    sh = wl.shape
    eps = list(range(wl.batch)) if episodes is None else list(episodes)
    B, P = len(eps), wl.prefix_len
    kb = np.zeros((sh.n_layers, B, sh.n_heads, capacity, sh.head_dim), np.uint16)
    vb = np.zeros_like(kb)
    first = np.zeros(B, np.int32)
    for i, e in enumerate(eps):
        k, v, f = synth.make_prefix_kv_direct(wl, e, capacity)
        kb[:, i], vb[:, i], first[i] = k, v, f
    return kb, vb, np.full(B, P, np.int32), first


def teacher_forced_drafts(model, wl, kb, vb, prefix_len, first_pred, offsets):
    """Drafts d_j = clip(v_j + offset_j, 0, n_bins-1), where v_j is the oracle's own greedy
    bin given the drafts already fixed: K sequential single-token oracle forwards per episode,
    run for all episodes at once.  Returns draft bins i32[B,K]."""
    sh = wl.shape
    B, K = offsets.shape
    L, H, hd = sh.n_layers, sh.n_heads, sh.head_dim
    kf = [[oracle.widen_bf16(kb[l][b][:, :prefix_len[b]]) for b in range(B)] for l in range(L)]
    vf = [[oracle.widen_bf16(vb[l][b][:, :prefix_len[b]]) for b in range(B)] for l in range(L)]
    v_cur = np.asarray(first_pred, np.int64).copy()
    drafts = np.zeros((B, K), np.int32)
    plen = np.asarray(prefix_len, np.int64).copy()
    for j in range(K):
        drafts[:, j] = np.clip(v_cur + offsets[:, j], 0, sh.n_bins - 1)
        if j == K - 1:
            break
        x = oracle.embed(model, sh.bin_base + drafts[:, j])[:, None, :]
        out = oracle.forward_block(model, x, plen, kf, vf)
        for l in range(L):
            for b in range(B):
                kf[l][b] = np.concatenate([kf[l][b], out["k_new"][l, b]], axis=1)
                vf[l][b] = np.concatenate([vf[l][b], out["v_new"][l, b]], axis=1)
        plen += 1
        v_cur = oracle.argmax_bins(out["logits"][:, 0, :]).astype(np.int64)
    return drafts


def oracle_chunked_prefill(model: oracle.OracleModel, x_full: np.ndarray, chunks, capacity: int):
    """The prefix of ONE episode through the oracle chunk by chunk, the cache rounded to bf16 between
    chunks (the cache format is part of the boundary: later chunks read bf16 rows).  x_full: [P, d] fp64.
    Returns (k_bits, v_bits) u16 [L][1][H][cap][hd] after the last chunk, and one record per chunk:
    {"p", "n", "k_before", "v_before" (the cache the chunk started from), "k_new", "v_new" (its rows,
    unrounded, [L][H][n][hd]), "logits" (last row), "next_bin"}."""
    L, H, hd = model.n_layers, model.n_heads, model.head_dim
    kb = np.zeros((L, 1, H, capacity, hd), np.uint16)
    vb = np.zeros_like(kb)
    p, steps = 0, []
    for n in chunks:
        out = oracle.forward_block(model, x_full[None, p:p + n], [p], kb, vb)
        rec = {"p": p, "n": n, "k_before": kb.copy(), "v_before": vb.copy(), "k_new": out["k_new"][:, 0],
               "v_new": out["v_new"][:, 0], "logits": out["logits"][0, -1],
               "next_bin": int(oracle.argmax_bins(out["logits"][0, -1]))}
        kb[:, 0, :, p:p + n, :] = synth.f32_to_bf16_bits(out["k_new"][:, 0].astype(np.float32))
        vb[:, 0, :, p:p + n, :] = synth.f32_to_bf16_bits(out["v_new"][:, 0].astype(np.float32))
        steps.append(rec)
        p += n
    return kb, vb, steps
