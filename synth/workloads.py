"""Shapes and seeded input recipes of the verify-step workloads (C0..C4).

The paper's workload is an OpenVLA-style policy: a Llama-2-7B backbone attending to
256 visual tokens per observation plus a language prompt, emitting 7 action tokens
over a 256-bin vocabulary (App. A.1/A.2).  Neither its weights nor its datasets are
used here: only the shapes.  Everything below is random and seeded.
"""
from dataclasses import dataclass, field
from typing import Dict, Tuple

import numpy as np

from . import rng


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    n_bins: int = 256
    rms_eps: float = 1e-6
    rope_base: float = 10000.0
    init_std: float = 0.02

    @property
    def bin_base(self) -> int:
        """Token id of action bin 0: the bins are the last n_bins ids of the vocabulary."""
        return self.vocab - self.n_bins

    def weight_bytes(self) -> int:
        d, f = self.d_model, self.d_ffn
        return self.n_layers * (4 * d * d + 3 * d * f) * 2


@dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    n_visual: int          # prefix rows given as N(0,1) input embeddings
    n_text: int            # prefix rows given as token ids
    text_id_hi: int        # text ids are uniform in [0, text_id_hi)
    batch: int
    K: int
    tau_tok: int = 2
    tau_seq: int = 6
    skip_p: float = 0.0
    draft: Tuple = ("uniform",)   # ("uniform",) or ("geometric", p)
    seed: int = 0

    @property
    def prefix_len(self) -> int:
        return self.n_visual + self.n_text


TINY = ModelShape(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=32000)
LLAMA7B = ModelShape(n_layers=32, d_model=4096, n_heads=32, head_dim=128, d_ffn=11008, vocab=32000)

WORKLOADS: Dict[str, Workload] = {
    "C0": Workload("C0", TINY, 0, 64, 32000, batch=1, K=7),
    "C1": Workload("C1", LLAMA7B, 256, 20, LLAMA7B.bin_base, batch=1, K=7),
    "C2": Workload("C2", LLAMA7B, 256, 20, LLAMA7B.bin_base, batch=8, K=7, draft=("geometric", 0.5)),
    "C3": Workload("C3", LLAMA7B, 512, 20, LLAMA7B.bin_base, batch=16, K=14, skip_p=0.3,
                   draft=("geometric", 0.5)),
    "C4": Workload("C4", LLAMA7B, 256, 20, LLAMA7B.bin_base, batch=64, K=7, draft=("geometric", 0.3)),
}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (storage format conversion only)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = u >> np.uint32(16)
    r &= np.uint32(1)
    r += np.uint32(0x7FFF)
    r += u
    r >>= np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_weights(shape: ModelShape, seed: int = 0) -> Dict[str, object]:
    """bf16 bit patterns of every matrix (N(0, init_std), rounded once); RMSNorm gains are 1.

    Returns {"tok_emb", "lm_head": u16[vocab,d]; "wq","wk","wv","wo","w_gate","w_up","w_down":
    lists of u16 per layer, row-major [out,in]; "attn_norm","ffn_norm": lists of f32[d];
    "final_norm": f32[d]}.
    """
    d, f, v, s = shape.d_model, shape.d_ffn, shape.vocab, shape.init_std
    w: Dict[str, object] = {}
    w["tok_emb"] = rng.normal_bf16(seed, "tok_emb", v * d, 0.0, s).reshape(v, d)
    w["lm_head"] = rng.normal_bf16(seed, "lm_head", v * d, 0.0, s).reshape(v, d)
    dims = {"wq": (d, d), "wk": (d, d), "wv": (d, d), "wo": (d, d),
            "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f)}
    for name, (o, i) in dims.items():
        w[name] = [rng.normal_bf16(seed, "%s.%d" % (name, l), o * i, 0.0, s).reshape(o, i)
                   for l in range(shape.n_layers)]
    w["attn_norm"] = [np.ones(d, np.float32) for _ in range(shape.n_layers)]
    w["ffn_norm"] = [np.ones(d, np.float32) for _ in range(shape.n_layers)]
    w["final_norm"] = np.ones(d, np.float32)
    return w


def make_prefix_inputs(wl: Workload, episode: int = 0):
    """(embeds f32[n_visual,d] ~ N(0,1), text_ids i32[n_text]) of one episode's prefix."""
    d = wl.shape.d_model
    emb = rng.normal_f32(wl.seed, "prefix.emb.%d" % episode, wl.n_visual * d).reshape(wl.n_visual, d)
    ids = rng.uniform_i32(wl.seed, "prefix.ids.%d" % episode, wl.n_text, 0, wl.text_id_hi)
    return emb, ids


def make_prefix_kv_direct(wl: Workload, episode: int = 0, capacity: int = None):
    """Prefix K/V rows drawn directly instead of by a prefill: bf16 bits [L][H][cap][hd].

    Rows 0..prefix_len-1 are N(0, init_std*sqrt(d_model)), the scale a prefill of a
    random-init model gives its keys and values; rows beyond the prefix are zero.
    Also returns a synthetic first_pred bin (uniform over the bins).
    """
    sh = wl.shape
    P = wl.prefix_len
    cap = capacity or (P + wl.K)
    std = sh.init_std * float(np.sqrt(sh.d_model))
    out = []
    for nm in ("k", "v"):
        a = np.zeros((sh.n_layers, sh.n_heads, cap, sh.head_dim), np.uint16)
        for l in range(sh.n_layers):
            r = rng.normal_bf16(wl.seed, "kv.%s.%d.%d" % (nm, episode, l),
                                sh.n_heads * P * sh.head_dim, 0.0, std)
            a[l, :, :P, :] = r.reshape(sh.n_heads, P, sh.head_dim)
        out.append(a)
    first = int(rng.uniform_i32(wl.seed, "kv.first.%d" % episode, 1, 0, sh.n_bins)[0])
    return out[0], out[1], first


def make_drafts_uniform(wl: Workload) -> np.ndarray:
    """Draft action bins i32[batch,K], uniform over the bins."""
    return rng.uniform_i32(wl.seed, "drafts", wl.batch * wl.K, 0, wl.shape.n_bins).reshape(wl.batch, wl.K)


def make_offsets_geometric(wl: Workload, p: float) -> np.ndarray:
    """Signed bin offsets i32[batch,K]: magnitude Geometric(p) on {0,1,2,...}, fair sign."""
    u = rng.uniform_f64(wl.seed, "offset.mag", wl.batch * wl.K)
    s = rng.uniform_f64(wl.seed, "offset.sign", wl.batch * wl.K)
    mag = np.floor(np.log(u) / np.log1p(-p)).astype(np.int64)     # P(mag = k) = p (1-p)^k
    sign = np.where(s < 0.5, -1, 1)
    return (mag * sign).astype(np.int32).reshape(wl.batch, wl.K)


def make_candidate_offsets(wl: Workload, n_candidates: int, p: float) -> np.ndarray:
    """Signed bin offsets i32[batch, n_candidates, K] for Top-K retrieval stand-ins: candidate r of an
    episode is the target's own continuation plus these offsets (magnitude Geometric(p) on
    {0,1,2,...}, fair sign), one independent stream per candidate."""
    out = np.zeros((wl.batch, n_candidates, wl.K), np.int32)
    for r in range(n_candidates):
        u = rng.uniform_f64(wl.seed, "cand.mag.%d" % r, wl.batch * wl.K)
        s = rng.uniform_f64(wl.seed, "cand.sign.%d" % r, wl.batch * wl.K)
        mag = np.floor(np.log(u) / np.log1p(-p)).astype(np.int64)
        out[:, r] = (mag * np.where(s < 0.5, -1, 1)).astype(np.int32).reshape(wl.batch, wl.K)
    return out


def make_retrieval_db(n_vectors: int, dim: int, seed: int = 0, payload_len: int = 7, n_bins: int = 256):
    """Stand-in for the retrieval database: n_vectors L2-normalised N(0,1) directions stored as bf16 bit
    patterns u16 [n_vectors, dim], and a payload of action bins i32 [n_vectors, payload_len] (uniform)."""
    db = np.empty((n_vectors, dim), np.uint16)
    step = max(1, (1 << 26) // dim)
    for s in range(0, n_vectors, step):
        n = min(step, n_vectors - s)
        v = rng.normal_f32(seed, "retrieval.db.%d" % s, n * dim).reshape(n, dim)
        v /= np.sqrt(np.einsum("ij,ij->i", v, v, dtype=np.float64)).astype(np.float32)[:, None]
        db[s:s + n] = f32_to_bf16_bits(v)
    payload = rng.uniform_i32(seed, "retrieval.payload", n_vectors * payload_len, 0, n_bins).reshape(n_vectors, payload_len)
    return db, payload


def make_retrieval_queries(db_bits: np.ndarray, batch: int, noise: float, seed: int = 0) -> np.ndarray:
    """Queries f32 [batch, dim]: a stored vector (rows spread over the database) plus N(0, noise^2/dim)
    per component, L2-normalised - an observation close to one seen before."""
    n, dim = db_bits.shape
    rows = (np.arange(batch, dtype=np.int64) * 7919 + 13) % n
    q = bf16_bits_to_f32(db_bits[rows]).astype(np.float64)
    q += noise / np.sqrt(dim) * rng.normal_f64(seed, "retrieval.noise", batch * dim).reshape(batch, dim)
    q /= np.sqrt((q * q).sum(axis=1, keepdims=True))
    return q.astype(np.float32)


def make_skip_mask(wl: Workload) -> np.ndarray:
    """u8[batch]: 1 = this episode's drafts bypass verification (Bernoulli(skip_p))."""
    u = rng.uniform_f64(wl.seed, "skip", wl.batch)
    return (u < wl.skip_p).astype(np.uint8)
