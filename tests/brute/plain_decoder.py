"""A second, even plainer decoder used only to pin the oracle on tiny shapes.

Written separately from oracle/: scalar Python loops over tokens, heads and
channels, complex-number rotary embedding, no KV cache at all (every call runs the
whole sequence from position 0), explicit causal sums.  It follows the model family
the paper names (App. A.1: Llama-2 backbone, causal attention over all earlier
tokens; App. A.2: linear head over the 256 action bins) with the same readings for
what the paper leaves open.
"""
import cmath
import math


def _matvec(W, x):           # W: list of rows [out][in]
    return [sum(wi * xi for wi, xi in zip(row, x)) for row in W]


def _rms(x, g, eps):
    ms = sum(v * v for v in x) / len(x)
    return [v / math.sqrt(ms + eps) * gi for v, gi in zip(x, g)]


def _rotary(vec, pos, hd, base):
    """vec: one head's hd channels.  Channel pair (i, i+hd/2) is the complex number
    vec[i] + 1j*vec[i+hd/2], multiplied by exp(1j * pos * base**(-2i/hd))."""
    half = hd // 2
    out = [0.0] * hd
    for i in range(half):
        z = complex(vec[i], vec[i + half]) * cmath.exp(1j * pos * base ** (-2.0 * i / hd))
        out[i], out[i + half] = z.real, z.imag
    return out


def full_sequence_logits(W, shape, x_seq):
    """Run the decoder over the whole sequence x_seq (list of d-vectors), no cache.

    W: dict of nested Python lists (floats): wq,wk,wv,wo,w_gate,w_up,w_down per layer
    ([out][in]), attn_norm, ffn_norm per layer, final_norm, lm_bins ([n_bins][d]).
    shape: dict with n_layers, n_heads, head_dim, rms_eps, rope_base.
    Returns (logits[t][bin], feat[t][d]) for every position t.
    """
    L, H, hd = shape["n_layers"], shape["n_heads"], shape["head_dim"]
    eps, base = shape["rms_eps"], shape["rope_base"]
    S = len(x_seq)
    x = [list(v) for v in x_seq]
    for l in range(L):
        q, k, v = [], [], []
        for t in range(S):
            h = _rms(x[t], W["attn_norm"][l], eps)
            qt, kt, vt = _matvec(W["wq"][l], h), _matvec(W["wk"][l], h), _matvec(W["wv"][l], h)
            q.append([_rotary(qt[a * hd:(a + 1) * hd], t, hd, base) for a in range(H)])
            k.append([_rotary(kt[a * hd:(a + 1) * hd], t, hd, base) for a in range(H)])
            v.append([vt[a * hd:(a + 1) * hd] for a in range(H)])
        for t in range(S):
            o = []
            for a in range(H):
                sc = [sum(q[t][a][c] * k[r][a][c] for c in range(hd)) / math.sqrt(hd) for r in range(t + 1)]
                mx = max(sc)
                e = [math.exp(s - mx) for s in sc]
                z = sum(e)
                o += [sum(e[r] / z * v[r][a][c] for r in range(t + 1)) for c in range(hd)]
            proj = _matvec(W["wo"][l], o)
            x[t] = [xi + pi for xi, pi in zip(x[t], proj)]
        for t in range(S):
            h = _rms(x[t], W["ffn_norm"][l], eps)
            g, u = _matvec(W["w_gate"][l], h), _matvec(W["w_up"][l], h)
            a_ = [gi / (1.0 + math.exp(-gi)) * ui for gi, ui in zip(g, u)]
            dn = _matvec(W["w_down"][l], a_)
            x[t] = [xi + di for xi, di in zip(x[t], dn)]
    feats = [_rms(x[t], W["final_norm"], eps) for t in range(S)]
    logits = [_matvec(W["lm_bins"], f) for f in feats]
    return logits, feats


def accept_literal(d, v, tau_tok, tau_seq, sizes=(3, 3, 1), exact=(False, False, True)):
    """Literal transcription of the acceptance rule for one episode, written apart from
    the oracle: walk the groups of the repeating pattern; stop at the first group that
    is not accepted.  Returns (n, v[n])."""
    K = len(d)
    j = 0
    g = 0
    n = 0
    while j < K:
        size = sizes[g % len(sizes)]
        members = list(range(j, min(j + size, K)))
        devs = [abs(d[i] - v[i]) for i in members]
        if exact[g % len(sizes)]:
            good = max(devs) == 0
        else:
            good = max(devs) <= tau_tok and sum(devs) <= tau_seq
        if not good:
            return n, v[n]
        n = members[-1] + 1
        j += size
        g += 1
    return n, v[n]
