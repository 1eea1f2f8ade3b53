"""Plain fp64 CPU oracle of the target-model verify step of HeiSD.

TEST INFRASTRUCTURE ONLY: used by tests/, the smoke check and the benchmark's
cpu_baseline leg.  The product path never imports it.

What is computed, and where the paper defines it:

* Verification is one teacher-forced forward of the target model over the K draft
  tokens given the prefix, a_hat_j = M_V(a_{0:j-1}, P, W), followed by an
  accept/discard decision per draft (Sec. 2.2, Eq. 2-2).  The target decodes
  greedily: argmax over the action vocabulary (Sec. 2.1, Eq. 2-1).
* The backbone is a Llama-2-style decoder with causal attention over visual, text
  and earlier action tokens; each action dimension is one token out of 256 bins
  read out by a linear head (App. A.1, A.2).
* Draft tokens are grouped into kinematic sequences (X,Y,Z), (rX,rY,rZ), (G); a
  sequence is accepted as a whole when the sequence's bias and every token's bias
  (index distance between draft bin and target bin) stay within their ranges, and
  the gripper admits no deviation (Sec. 4.2).
* A draft whose verification is skipped is executed as is, i.e. counts as fully
  accepted (Sec. 4.1, Sec. 6.2).

Everything is the plain definition in fp64 on the bf16-valued weights widened
exactly; numpy's matmul is the only library step.  No blocking, no fusion, no
cache tricks: the KV "cache" is simply the list of earlier keys and values.

Readings where the paper is silent (all listed in the design notes): RMSNorm with
gain, rotate-half RoPE on absolute positions, multi-head attention with scale
1/sqrt(head_dim), SwiGLU FFN, untied LM head, bin b <-> token id vocab-256+b,
sequence bias = sum of the token biases of the group, inclusive thresholds, ties
in argmax go to the lowest bin.
"""
import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle_widen.so")
_lib = None


def build_native(force: bool = False) -> str:
    """Compile the oracle's one C helper (bf16 -> fp64 widening)."""
    src = os.path.join(_HERE, "widen.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        tmp = _SO + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O3", "-mavx2", "-mfma", "-fPIC", "-shared", "-fopenmp", "-o", tmp, src])
        os.replace(tmp, _SO)
    return _SO


def _native():
    global _lib
    if _lib is None:
        build_native()
        _lib = ctypes.CDLL(_SO)
        _lib.oracle_widen_bf16_f64.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64]
        _lib.oracle_widen_bf16_f64.restype = None
        _lib.oracle_linear_bf16w.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                                             ctypes.c_int64, ctypes.c_void_p]
        _lib.oracle_linear_bf16w.restype = None
    return _lib


def widen_bf16(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> the same values in fp64 (exact).  Floats pass through."""
    bits = np.ascontiguousarray(bits)
    if bits.dtype != np.uint16:
        return np.asarray(bits, dtype=np.float64)
    out = np.empty(bits.shape, dtype=np.float64)
    _native().oracle_widen_bf16_f64(bits.ctypes.data, out.ctypes.data, bits.size)
    return out


def linear_bf16w(x: np.ndarray, w_bits: np.ndarray) -> np.ndarray:
    """y = x . W^T for W given as bf16 bit patterns [out, in]; products and sums in fp64."""
    n_out, n_in = w_bits.shape
    x2 = np.ascontiguousarray(x, dtype=np.float64).reshape(-1, n_in)
    w_bits = np.ascontiguousarray(w_bits)
    y = np.empty((x2.shape[0], n_out))
    _native().oracle_linear_bf16w(x2.ctypes.data, x2.shape[0], n_in, w_bits.ctypes.data, n_out, y.ctypes.data)
    return y.reshape(x.shape[:-1] + (n_out,))


@dataclass
class OracleModel:
    """Decoder shape plus weights.  Matrices are row-major [out, in], either bf16 bit
    patterns (uint16) or floats; gains are float arrays."""
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    weights: Dict[str, object]
    n_bins: int = 256
    rms_eps: float = 1e-6
    rope_base: float = 10000.0

    @property
    def bin_base(self) -> int:
        return self.vocab - self.n_bins

    def mat(self, name: str, layer: Optional[int] = None) -> np.ndarray:
        w = self.weights[name] if layer is None else self.weights[name][layer]
        return widen_bf16(w)

    def rows(self, name: str, idx) -> np.ndarray:
        return widen_bf16(np.asarray(self.weights[name])[idx])

    def linear(self, x: np.ndarray, name: str, layer: Optional[int] = None) -> np.ndarray:
        """y = x . W^T for W = weights[name][layer] ([out, in])."""
        w = self.weights[name] if layer is None else self.weights[name][layer]
        w = np.asarray(w)
        if w.dtype == np.uint16:
            return linear_bf16w(x, w)
        return x @ np.asarray(w, dtype=np.float64).T


# ----------------------------------------------------------------------------
# decoder forward (App. A.1: Llama-2 backbone; Eq. 2-1 / Eq. 2-2: what it feeds)
# ----------------------------------------------------------------------------

def embed(model: OracleModel, ids: np.ndarray) -> np.ndarray:
    """x_j = E[t_j]: token embeddings of the given ids, fp64 [..., d]."""
    ids = np.asarray(ids)
    return model.rows("tok_emb", ids.reshape(-1)).reshape(ids.shape + (model.d_model,))


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """RMSNorm(x)_i = x_i * g_i / sqrt(mean_i(x_i^2) + eps), over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(g, dtype=np.float64)


def rope(u: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing.  u: [T, H, hd]; pos: [T] absolute positions.
    For i < hd/2 and theta_i = base^(-2i/hd), the pair (u_i, u_{i+hd/2}) is rotated by
    the angle pos * theta_i."""
    hd = u.shape[-1]
    half = hd // 2
    theta = np.asarray(base, dtype=np.float64) ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = np.asarray(pos, dtype=np.float64)[:, None, None] * theta[None, None, :]
    c, s = np.cos(ang), np.sin(ang)
    a, b = u[..., :half], u[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def attention_block(q: np.ndarray, k_all: np.ndarray, v_all: np.ndarray, p0: int) -> np.ndarray:
    """Causal attention of T new queries over p0 earlier rows plus the block itself.
    q: [T, H, hd]; k_all, v_all: [H, p0+T, hd] (earlier rows first).  Query t sees rows
    0 .. p0+t.  Returns [T, H, hd]."""
    T, H, hd = q.shape
    s = np.einsum("thd,hrd->htr", q, k_all) / np.sqrt(float(hd))
    r = np.arange(k_all.shape[1])[None, None, :]
    t = np.arange(T)[None, :, None]
    s = np.where(r <= p0 + t, s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    w = np.exp(s)
    w = w / w.sum(axis=-1, keepdims=True)
    return np.einsum("htr,hrd->thd", w, v_all)


def forward_block(model: OracleModel, x_in: np.ndarray, prefix_len: Sequence[int],
                  kv_k=None, kv_v=None, want_logits: bool = True) -> Dict[str, np.ndarray]:
    """One decoder forward over T new tokens per episode given each episode's earlier K/V.

    x_in:       [B, T, d] input embeddings of the new tokens (fp64).
    prefix_len: [B] number of earlier rows p0_b of each episode (may be 0).
    kv_k, kv_v: earlier keys/values, indexable as kv[l][b] -> [H, >=p0_b, hd]
                (bf16 bit patterns or floats); None when every p0_b is 0.
    Returns feat [B,T,d] (final-norm hidden state, the LM head's input), logits
    [B,T,n_bins] over the action bins, and the new rows k_new, v_new [L,B,H,T,hd].
    """
    m = model
    x = np.array(x_in, dtype=np.float64)
    B, T, d = x.shape
    H, hd = m.n_heads, m.head_dim
    k_new = np.zeros((m.n_layers, B, H, T, hd))
    v_new = np.zeros((m.n_layers, B, H, T, hd))
    for l in range(m.n_layers):
        h = rmsnorm(x, m.weights["attn_norm"][l], m.rms_eps)
        q = m.linear(h, "wq", l).reshape(B, T, H, hd)
        k = m.linear(h, "wk", l).reshape(B, T, H, hd)
        v = m.linear(h, "wv", l).reshape(B, T, H, hd)
        o = np.zeros((B, T, H, hd))
        for b in range(B):
            p0 = int(prefix_len[b])
            pos = p0 + np.arange(T)
            qb = rope(q[b], pos, m.rope_base)
            kb = rope(k[b], pos, m.rope_base)
            kb_h = np.transpose(kb, (1, 0, 2))            # [H, T, hd]
            vb_h = np.transpose(v[b], (1, 0, 2))
            k_new[l, b], v_new[l, b] = kb_h, vb_h
            if p0 > 0:
                kp = widen_bf16(np.asarray(kv_k[l][b])[:, :p0, :])
                vp = widen_bf16(np.asarray(kv_v[l][b])[:, :p0, :])
                k_all = np.concatenate([kp, kb_h], axis=1)
                v_all = np.concatenate([vp, vb_h], axis=1)
            else:
                k_all, v_all = kb_h, vb_h
            o[b] = attention_block(qb, k_all, v_all, p0)
        x = x + m.linear(o.reshape(B, T, d), "wo", l)
        h = rmsnorm(x, m.weights["ffn_norm"][l], m.rms_eps)
        a = silu(m.linear(h, "w_gate", l)) * m.linear(h, "w_up", l)
        x = x + m.linear(a, "w_down", l)
    feat = rmsnorm(x, m.weights["final_norm"], m.rms_eps)
    out = {"feat": feat, "k_new": k_new, "v_new": v_new}
    if want_logits:
        out["logits"] = bin_logits(m, feat)
    return out


def bin_logits(model: OracleModel, feat: np.ndarray) -> np.ndarray:
    """Logits of the n_bins action tokens only: rows bin_base .. bin_base+n_bins-1 of the LM head."""
    w = model.rows("lm_head", slice(model.bin_base, model.bin_base + model.n_bins))
    return feat @ w.T


def argmax_bins(logits: np.ndarray) -> np.ndarray:
    """Greedy choice (Eq. 2-1) over the last axis; the lowest index wins ties, NaN never wins."""
    lg = np.where(np.isnan(logits), -np.inf, logits)
    return np.argmax(lg, axis=-1).astype(np.int32)     # numpy returns the first maximum


def prefill(model: OracleModel, x_in: np.ndarray) -> Dict[str, np.ndarray]:
    """Forward of a whole prefix from nothing: x_in [B, P, d].  Gives the prefix K/V
    (k_new/v_new [L,B,H,P,hd]) and first_pred [B], the target's greedy bin after the
    last prefix position (a_hat_0 of Eq. 2-2 depends on the prefix alone)."""
    B = x_in.shape[0]
    out = forward_block(model, x_in, [0] * B, want_logits=False)
    out["logits_last"] = bin_logits(model, out["feat"][:, -1, :])
    out["first_pred"] = argmax_bins(out["logits_last"])
    return out


# ----------------------------------------------------------------------------
# sequence-wise relaxed acceptance (Sec. 4.2) and verify-skip (Sec. 4.1 / 6.2)
# ----------------------------------------------------------------------------

@dataclass(frozen=True)
class AcceptRule:
    tok_threshold: int = 15            # bias_aj: largest index bias one token may have
    seq_budget: int = 30               # bias_seq: largest summed bias of one sequence
    group_sizes: Tuple[int, ...] = (3, 3, 1)   # (X,Y,Z), (rX,rY,rZ), (G); repeats per action slice
    exact_group_mask: int = 0b100      # bit g set: group g tolerates no deviation (gripper)
    mode: int = 0                      # 0: the paper's all-or-nothing sequences; 1: token-granular variant


INF_BIAS = 2 ** 31 - 1


def _token_groups(K: int, group_sizes: Sequence[int]) -> List[Tuple[int, int, int]]:
    """Cut positions 0..K-1 into consecutive groups following the repeating pattern.
    Returns (start, end_exclusive, group_index_in_pattern); a trailing group may be cut short."""
    out, j, g = [], 0, 0
    while j < K:
        size = group_sizes[g % len(group_sizes)]
        out.append((j, min(j + size, K), g % len(group_sizes)))
        j += size
        g += 1
    return out


def accept_block(draft_bins: Sequence[int], target_bins: Sequence[int], rule: AcceptRule,
                 n_bins: int = 256) -> Tuple[int, int]:
    """Accepted length n and the target's bin at position n for one episode.

    draft_bins d_0..d_{K-1}; target_bins v_0..v_K where v_j is the target's greedy
    bin for position j given drafts 0..j-1 (v_0 comes from the prefix).  bias_j =
    |d_j - v_j|.  A sequence (group) is accepted iff every bias_j <= tok_threshold and
    the sum of its biases <= seq_budget, or, for an exact group, every bias_j = 0.
    n is the total length of the leading run of accepted groups; accepted positions
    keep the DRAFT tokens, and v_n is the token the target itself supplies next.
    """
    K = len(draft_bins)
    assert len(target_bins) == K + 1
    bias = []
    for j in range(K):
        dj = int(draft_bins[j])
        bias.append(abs(dj - int(target_bins[j])) if 0 <= dj < n_bins else INF_BIAS)
    n = 0
    if rule.mode == 0:
        for (s, e, g) in _token_groups(K, rule.group_sizes):
            grp = bias[s:e]
            if (rule.exact_group_mask >> g) & 1:
                ok = all(bj == 0 for bj in grp)
            else:
                ok = all(bj <= rule.tok_threshold for bj in grp) and sum(grp) <= rule.seq_budget
            if not ok:
                break
            n = e
    else:
        run = 0
        for (s, e, g) in _token_groups(K, rule.group_sizes):
            stop = False
            for j in range(s, e):
                run += bias[j]
                exact = (rule.exact_group_mask >> g) & 1
                if (exact and bias[j] != 0) or bias[j] > rule.tok_threshold or run > rule.seq_budget:
                    stop = True
                    break
                n = j + 1
            if stop:
                break
    return n, int(target_bins[n])


def verify_step(model: OracleModel, kv_k, kv_v, prefix_len: Sequence[int], first_pred: Sequence[int],
                draft_tokens: np.ndarray, rule: AcceptRule, skip_mask=None) -> Dict[str, np.ndarray]:
    """The whole verify step for a batch of episodes.

    kv_k, kv_v: prefix keys/values, kv[l][b] -> [H, >=prefix_len[b], hd].
    draft_tokens: [B, K] vocabulary ids.  skip_mask: [B] (nonzero = bypass).
    Returns accepted_len [B], next_token [B] (vocabulary id, -1 if skipped),
    target_bins [B, K+1] (-1 if skipped), bin_logits [B, K, n_bins] (NaN if skipped),
    feat, k_new, v_new for the verified episodes (zeros if skipped).
    """
    m = model
    draft_tokens = np.asarray(draft_tokens, dtype=np.int64)
    B, K = draft_tokens.shape
    skip = np.zeros(B, dtype=bool) if skip_mask is None else np.asarray(skip_mask).astype(bool)
    act = [b for b in range(B) if not skip[b]]
    accepted = np.full(B, K, dtype=np.int32)
    next_tok = np.full(B, -1, dtype=np.int32)
    tbins = np.full((B, K + 1), -1, dtype=np.int32)
    logits = np.full((B, K, m.n_bins), np.nan)
    feat = np.zeros((B, K, m.d_model))
    k_new = np.zeros((m.n_layers, B, m.n_heads, K, m.head_dim))
    v_new = np.zeros_like(k_new)
    if act:
        ids = np.clip(draft_tokens[act], 0, m.vocab - 1)
        x = embed(m, ids)

        class _Sel:          # view of the caches restricted to the verified episodes
            def __init__(self, kv):
                self.kv = kv

            def __getitem__(self, l):
                layer = self.kv[l]
                return [layer[b] for b in act]

        out = forward_block(m, x, [int(prefix_len[b]) for b in act], _Sel(kv_k), _Sel(kv_v))
        v_next = argmax_bins(out["logits"])                       # [n_act, K]: v_1..v_K
        for i, b in enumerate(act):
            tb = np.concatenate([[int(first_pred[b])], v_next[i]]).astype(np.int32)
            tbins[b] = tb
            n, nb = accept_block(draft_tokens[b] - m.bin_base, tb, rule, m.n_bins)
            accepted[b] = n
            next_tok[b] = m.bin_base + nb
            logits[b] = out["logits"][i]
            feat[b] = out["feat"][i]
            k_new[:, b] = out["k_new"][:, i]
            v_new[:, b] = out["v_new"][:, i]
    return {"accepted_len": accepted, "next_token": next_tok, "target_bins": tbins,
            "bin_logits": logits, "feat": feat, "k_new": k_new, "v_new": v_new}
