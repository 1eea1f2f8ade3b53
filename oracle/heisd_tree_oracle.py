"""Plain CPU oracle of sequence-wise TREE verification (paper Sec. 4.2).

TEST INFRASTRUCTURE ONLY, like the rest of this package.

What the paper states (Sec. 4.2), in this module's words:

* retrieval returns the Top-K drafts instead of one; each draft is cut into kinematic
  sequences (X,Y,Z), (rX,rY,rZ), (G);
* the draft tree is built sequence by sequence, not token by token: a node is one whole
  sequence; sequences taken from different retrieval results may follow each other, except
  the gripper sequence, which is not connected across retrieval results;
* every chain from the root is verified, depth first, with the sequence-wise relaxed rule;
  when every candidate for a sequence is rejected, the target model itself supplies the
  next token.

The oracle is that statement written out: the tree is flattened into its root-to-leaf
chains, each chain is verified ALONE by the linear verify step of heisd_oracle (one plain
forward of the chain's tokens after the prefix, then the linear acceptance scan), and the
chain that gets furthest wins.  No tree attention mask appears here: that a single masked
forward over all tree tokens gives the same numbers is a property the HIP path relies on,
and the parity tests check it against this definition.

Readings where the paper is silent (listed in the design notes):

T1  cross-linking: under a parent node, the children for a non-exact sequence level are the
    distinct sequences of ALL candidates at that level; for an exact level (gripper) only the
    sequences of the candidates whose sequence the parent node carries.  A node remembers
    that candidate set.  Equal sibling sequences are merged.
T2  layout: depth-first preorder, candidates in retrieval order; a node whose tokens would
    exceed the token budget is left out together with its subtree.
T3  choice among accepted chains: the largest accepted length; among equals the chain whose
    last accepted token has the lowest index (for a preorder layout: the first in
    depth-first order).  Nothing accepted: length 0, and the next token is the target's own
    prediction after the prefix.
T4  a token whose parent index is not in [-1, own index) is padding: it is in no chain.
T5  verify-skip on a tree executes the first chain: token 0 and, from each token, its
    lowest-index child.
"""
from typing import Dict, List, Sequence, Tuple

import numpy as np

from .heisd_oracle import (AcceptRule, OracleModel, accept_block, argmax_bins, embed, forward_block)


def _levels(K: int, group_sizes: Sequence[int]) -> List[Tuple[int, int, int]]:
    """(start, end, pattern index) of the consecutive sequences covering positions 0..K-1."""
    out, j, g = [], 0, 0
    while j < K:
        size = group_sizes[g % len(group_sizes)]
        out.append((j, min(j + size, K), g % len(group_sizes)))
        j += size
        g += 1
    return out


def build_sequence_tree(candidates: np.ndarray, rule: AcceptRule, max_tokens: int) -> Tuple[np.ndarray, np.ndarray]:
    """Draft tree of R retrieved candidates (rows of `candidates`, K tokens each), readings T1/T2.
    Returns (tokens[T], parent[T]): parent[t] is the index of the token before t in its chain,
    -1 for a token that follows the prefix."""
    cand = np.asarray(candidates)
    R, K = cand.shape
    levels = _levels(K, rule.group_sizes)
    tokens: List[int] = []
    parent: List[int] = []

    def grow(level: int, last_token: int, carried: List[int]) -> None:
        if level == len(levels):
            return
        s, e, g = levels[level]
        exact = (rule.exact_group_mask >> g) & 1
        eligible = carried if exact else list(range(R))
        seen: List[Tuple[Tuple[int, ...], List[int]]] = []       # (sequence, candidates that have it)
        for c in eligible:
            seq = tuple(int(v) for v in cand[c, s:e])
            for known, owners in seen:
                if known == seq:
                    owners.append(c)
                    break
            else:
                seen.append((seq, [c]))
        for seq, owners in seen:
            if len(tokens) + len(seq) > max_tokens:
                continue
            prev = last_token
            for tok in seq:
                tokens.append(tok)
                parent.append(prev)
                prev = len(tokens) - 1
            grow(level + 1, prev, owners)

    grow(0, -1, list(range(R)))
    return np.asarray(tokens, np.int32), np.asarray(parent, np.int32)


def _valid_tokens(parent: Sequence[int]) -> List[bool]:
    """Reading T4, applied along chains: a token is in the tree iff its parent index is -1, or a
    lower index whose token is itself in the tree."""
    ok = []
    for t, p in enumerate(parent):
        p = int(p)
        ok.append(p == -1 or (0 <= p < t and ok[p]))
    return ok


def tree_chains(parent: Sequence[int]) -> List[List[int]]:
    """All root-to-leaf chains as lists of token indices, ordered by leaf index."""
    ok = _valid_tokens(parent)
    has_child = [False] * len(parent)
    for t, p in enumerate(parent):
        if ok[t] and int(p) >= 0:
            has_child[int(p)] = True
    chains = []
    for t in range(len(parent)):
        if ok[t] and not has_child[t]:
            c, cur = [], t
            while cur != -1:
                c.append(cur)
                cur = int(parent[cur])
            chains.append(c[::-1])
    return chains


def first_chain(parent: Sequence[int]) -> List[int]:
    """Reading T5: token 0, then from each token its lowest-index child."""
    ok = _valid_tokens(parent)
    if len(parent) == 0 or not ok[0] or int(parent[0]) != -1:
        return []
    chain = [0]
    while True:
        nxt = [t for t in range(len(parent)) if ok[t] and int(parent[t]) == chain[-1]]
        if not nxt:
            return chain
        chain.append(nxt[0])


def accept_tree(draft_bins: Sequence[int], parent: Sequence[int], first_pred: int, pred: Sequence[int],
                rule: AcceptRule, n_bins: int = 256) -> Tuple[int, List[int], int]:
    """Chain selection, reading T3.  draft_bins[t]: bin of tree token t; pred[t]: the target's greedy
    bin after token t given t's own chain; first_pred: its bin after the prefix.  Every chain gets the
    linear rule (accept_block) on its own; returns (n, the n accepted token indices, next bin)."""
    best_n, best_path, best_next = 0, [], int(first_pred)
    for chain in tree_chains(parent):
        d = [int(draft_bins[t]) for t in chain]
        v = [int(first_pred)] + [int(pred[t]) for t in chain]
        n, nxt = accept_block(d, v, rule, n_bins)
        if n > best_n or (n == best_n and n > 0 and chain[n - 1] < best_path[-1]):
            best_n, best_path, best_next = n, chain[:n], nxt
    return best_n, best_path, best_next


def verify_tree_step(model: OracleModel, kv_k, kv_v, prefix_len: Sequence[int], first_pred: Sequence[int],
                     tree_tokens: np.ndarray, parent: np.ndarray, rule: AcceptRule,
                     skip_mask=None) -> Dict[str, np.ndarray]:
    """Tree verify step for a batch of episodes, chain by chain.

    tree_tokens, parent: [B, T].  Returns accepted_len [B], next_token [B] (vocabulary id, -1 if
    skipped), accepted_path [B, T] (first n entries: token indices, rest -1), target_bins [B, T+1]
    ([0] = first_pred, [t+1] = greedy bin after token t; -1 for padding tokens and skipped episodes),
    bin_logits [B, T, n_bins] (NaN where not computed), k_new/v_new [L, B, H, T, hd]: the key/value
    row of every tree token as computed in its chain."""
    m = model
    tree_tokens = np.asarray(tree_tokens, dtype=np.int64)
    parent = np.asarray(parent, dtype=np.int64)
    B, T = tree_tokens.shape
    skip = np.zeros(B, dtype=bool) if skip_mask is None else np.asarray(skip_mask).astype(bool)
    accepted = np.zeros(B, dtype=np.int32)
    next_tok = np.full(B, -1, dtype=np.int32)
    path = np.full((B, T), -1, dtype=np.int32)
    tbins = np.full((B, T + 1), -1, dtype=np.int32)
    logits = np.full((B, T, m.n_bins), np.nan)
    k_new = np.zeros((m.n_layers, B, m.n_heads, T, m.head_dim))
    v_new = np.zeros_like(k_new)
    for b in range(B):
        if skip[b]:
            c = first_chain(parent[b])
            accepted[b] = len(c)
            path[b, :len(c)] = c
            continue
        tbins[b, 0] = int(first_pred[b])
        done = np.zeros(T, dtype=bool)
        for chain in tree_chains(parent[b]):
            ids = np.clip(tree_tokens[b, chain], 0, m.vocab - 1)
            out = forward_block(m, embed(m, ids)[None], [int(prefix_len[b])], [[layer[b]] for layer in kv_k],
                                [[layer[b]] for layer in kv_v])
            for i, t in enumerate(chain):
                if not done[t]:                       # a token shared by several chains has one value
                    done[t] = True
                    logits[b, t] = out["logits"][0, i]
                    k_new[:, b, :, t] = out["k_new"][:, 0, :, i]
                    v_new[:, b, :, t] = out["v_new"][:, 0, :, i]
        pred = np.full(T, -1, dtype=np.int32)
        pred[done] = argmax_bins(logits[b, done])
        tbins[b, 1:] = pred
        n, p, nb = accept_tree(tree_tokens[b] - m.bin_base, parent[b], int(first_pred[b]), pred, rule, m.n_bins)
        accepted[b] = n
        path[b, :n] = p
        next_tok[b] = m.bin_base + nb
    return {"accepted_len": accepted, "next_token": next_tok, "accepted_path": path, "target_bins": tbins,
            "bin_logits": logits, "k_new": k_new, "v_new": v_new}
