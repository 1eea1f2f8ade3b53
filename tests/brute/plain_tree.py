"""Second, independent formulations used only to pin the tree-verification oracle.

* accept_tree_recursive: chain selection as a recursion over sequence nodes (the oracle
  instead flattens the tree into chains and scans each chain linearly).
* masked_tree_logits: ONE forward over all tree tokens in which a token sees the prefix, its
  ancestors and itself (the oracle instead runs every chain separately).  Scalar Python.

Paper Sec. 4.2 (tree of sequences, chains checked from the root, relaxed rule per sequence).
"""
import math

from .plain_decoder import _matvec, _rms, _rotary


def accept_tree_recursive(bins, parent, first_pred, pred, tau_tok, tau_seq, sizes=(3, 3, 1),
                          exact=(False, False, True)):
    """Returns (n, path, next bin).  From a point in the tree (the token reached so far, the depth,
    the index of the next sequence in the repeating pattern) try every way the tree continues with
    one whole sequence (or with what is left of it at a leaf); keep the continuation that gets
    furthest, among equals the one ending at the lowest token index."""
    T = len(parent)
    kids = {}
    for t in range(T):
        kids.setdefault(int(parent[t]), []).append(t)

    def sequences_from(tok, size):
        """Every run of `size` tokens hanging under tok (-1: the root); shorter only where a leaf ends it."""
        out = []

        def walk(last, run):
            children = kids.get(last, [])
            if len(run) == size or (run and not children):
                out.append(run)
                return
            for c in children:
                walk(c, run + [c])

        walk(tok, [])
        return out

    def best_from(tok, g):
        """(accepted tokens beyond tok, their indices, next bin) for the best continuation."""
        target_here = first_pred if tok == -1 else pred[tok]
        best = (0, [], target_here)
        for run in sequences_from(tok, sizes[g % len(sizes)]):
            devs, prev = [], tok
            for t in run:
                devs.append(abs(bins[t] - (first_pred if prev == -1 else pred[prev])))
                prev = t
            good = (max(devs) == 0) if exact[g % len(sizes)] else (max(devs) <= tau_tok and sum(devs) <= tau_seq)
            if not good:
                continue
            more = best_from(run[-1], g + 1)
            cand = (len(run) + more[0], run + more[1], more[2])
            if cand[0] > best[0] or (cand[0] == best[0] and cand[0] > 0 and cand[1][-1] < best[1][-1]):
                best = cand
        return best

    return best_from(-1, 0)


def masked_tree_logits(W, shape, x_prefix, x_tree, parent):
    """x_prefix: list of P d-vectors (causal among themselves); x_tree: T d-vectors; parent[t] as in the
    oracle.  Tree token t sits at position P + depth(t) and sees the prefix, its ancestors and itself.
    Returns logits[t][bin] for the tree tokens."""
    L, H, hd = shape["n_layers"], shape["n_heads"], shape["head_dim"]
    eps, base = shape["rms_eps"], shape["rope_base"]
    P, T = len(x_prefix), len(x_tree)
    depth, sees = [], []
    for t in range(T):
        p = int(parent[t])
        depth.append(0 if p < 0 else depth[p] + 1)
        sees.append(([] if p < 0 else sees[p]) + [P + t])
    pos = list(range(P)) + [P + dpt for dpt in depth]
    vis = [list(range(r + 1)) for r in range(P)] + [list(range(P)) + sees[t] for t in range(T)]
    x = [list(v) for v in x_prefix] + [list(v) for v in x_tree]
    S = P + T
    for l in range(L):
        q, k, v = [], [], []
        for s in range(S):
            h = _rms(x[s], W["attn_norm"][l], eps)
            qt, kt, vt = _matvec(W["wq"][l], h), _matvec(W["wk"][l], h), _matvec(W["wv"][l], h)
            q.append([_rotary(qt[a * hd:(a + 1) * hd], pos[s], hd, base) for a in range(H)])
            k.append([_rotary(kt[a * hd:(a + 1) * hd], pos[s], hd, base) for a in range(H)])
            v.append([vt[a * hd:(a + 1) * hd] for a in range(H)])
        for s in range(S):
            o = []
            for a in range(H):
                sc = [sum(q[s][a][c] * k[r][a][c] for c in range(hd)) / math.sqrt(hd) for r in vis[s]]
                mx = max(sc)
                e = [math.exp(z - mx) for z in sc]
                z = sum(e)
                o += [sum(e[i] / z * v[r][a][c] for i, r in enumerate(vis[s])) for c in range(hd)]
            proj = _matvec(W["wo"][l], o)
            x[s] = [xi + pi for xi, pi in zip(x[s], proj)]
        for s in range(S):
            h = _rms(x[s], W["ffn_norm"][l], eps)
            g, u = _matvec(W["w_gate"][l], h), _matvec(W["w_up"][l], h)
            a_ = [gi / (1.0 + math.exp(-gi)) * ui for gi, ui in zip(g, u)]
            dn = _matvec(W["w_down"][l], a_)
            x[s] = [xi + di for xi, di in zip(x[s], dn)]
    return [_matvec(W["lm_bins"], _rms(x[P + t], W["final_norm"], eps)) for t in range(T)]
