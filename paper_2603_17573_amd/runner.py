"""Torch-facing plumbing around the C ABI: device buffers, pointers, streams.  No arithmetic."""
import numpy as np
import torch

from . import binding as B

_SHAPE_KEYS = ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab", "n_bins", "rms_eps",
               "rope_base")
_LAYER_MATS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def _to_dev(a, device):
    """numpy uint16 (bf16 bits) -> bf16 tensor; float -> fp32 tensor; tensors pass through."""
    if isinstance(a, torch.Tensor):
        return a.to(device)
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a.astype(np.float32)).to(device)


class DeviceModel:
    """The target model's weights resident in HBM (caller-owned from the library's point of view)."""

    def __init__(self, shape, weights, device="cuda:0"):
        self.shape = {k: getattr(shape, k) for k in _SHAPE_KEYS}
        self.shape["bin_token_base"] = shape.vocab - shape.n_bins
        self.device = torch.device(device)
        self.t = {}
        for k in ("tok_emb", "lm_head", "final_norm"):
            self.t[k] = _to_dev(weights[k], self.device)
        for k in _LAYER_MATS + ("attn_norm", "ffn_norm"):
            self.t[k] = [_to_dev(w, self.device) for w in weights[k]]

    def pointers(self):
        p = {k: self.t[k].data_ptr() for k in ("tok_emb", "lm_head", "final_norm")}
        for k in _LAYER_MATS + ("attn_norm", "ffn_norm"):
            p[k] = [w.data_ptr() for w in self.t[k]]
        return p


class Verifier:
    """Owns a heisd_verify_ctx and its workspace; step() marshals tensors into one C call."""

    def __init__(self, model: DeviceModel, max_batch: int, max_k: int, kv_capacity: int):
        self.model = model
        self.max_batch, self.max_k, self.kv_capacity = max_batch, max_k, kv_capacity
        desc, self._keep = B.make_model_desc(model.shape, model.pointers(), max_batch, max_k, kv_capacity)
        nbytes = B.heisd_verify_workspace_bytes(desc)
        if nbytes == 0:
            raise ValueError("invalid model description")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=model.device)
        desc.workspace, desc.workspace_bytes = self.workspace.data_ptr(), nbytes
        self.desc = desc
        rc, ctx = B.heisd_verify_init(desc)
        if rc != 0:
            raise RuntimeError("heisd_verify_init failed (%d): %s" % (rc, B.heisd_last_error(None)))
        self.ctx = ctx

    def new_cache(self, batch: int):
        s = self.model.shape
        shp = (s["n_layers"], batch, s["n_heads"], self.kv_capacity, s["head_dim"])
        return (torch.zeros(shp, dtype=torch.bfloat16, device=self.model.device),
                torch.zeros(shp, dtype=torch.bfloat16, device=self.model.device))

    def step(self, k_cache, v_cache, prefix_len, first_pred, draft_tokens, accept, skip_mask=None,
             want_aux=True, out=None, stream=None):
        """draft_tokens i32[batch,K] on the device.  Returns dict of device tensors (enqueued on the
        stream, not synchronised).  `out` lets a timing loop reuse the output tensors."""
        batch, K = draft_tokens.shape
        dev = self.model.device
        if out is None:
            out = {"accepted_len": torch.empty(batch, dtype=torch.int32, device=dev),
                   "next_token": torch.empty(batch, dtype=torch.int32, device=dev)}
            if want_aux:
                out["target_bins"] = torch.empty(batch, K + 1, dtype=torch.int32, device=dev)
                out["bin_logits"] = torch.empty(batch, K, self.model.shape["n_bins"], dtype=torch.float32,
                                                device=dev)
        kv = B.heisd_kv_desc(k_cache.data_ptr(), v_cache.data_ptr(), prefix_len.data_ptr(),
                             first_pred.data_ptr())
        st = (stream or torch.cuda.current_stream(dev)).cuda_stream
        rc = B.heisd_verify_step(self.ctx, kv, draft_tokens.data_ptr(), K, batch, accept,
                                 skip_mask.data_ptr() if skip_mask is not None else None,
                                 out["accepted_len"].data_ptr(), out["next_token"].data_ptr(),
                                 out["target_bins"].data_ptr() if "target_bins" in out else None,
                                 out["bin_logits"].data_ptr() if "bin_logits" in out else None, st)
        if rc != 0:
            raise RuntimeError("heisd_verify_step failed (%d): %s" % (rc, B.heisd_last_error(self.ctx)))
        return out

    def tree_step(self, k_cache, v_cache, prefix_len, first_pred, tree_tokens, parent, accept, skip_mask=None,
                  want_aux=True, out=None, stream=None):
        """tree_tokens, parent: i32[batch,T] on the device.  Returns dict of device tensors."""
        batch, T = tree_tokens.shape
        dev = self.model.device
        if out is None:
            out = {"accepted_len": torch.empty(batch, dtype=torch.int32, device=dev),
                   "next_token": torch.empty(batch, dtype=torch.int32, device=dev),
                   "accepted_path": torch.empty(batch, T, dtype=torch.int32, device=dev)}
            if want_aux:
                out["target_bins"] = torch.empty(batch, T + 1, dtype=torch.int32, device=dev)
                out["bin_logits"] = torch.empty(batch, T, self.model.shape["n_bins"], dtype=torch.float32,
                                                device=dev)
        kv = B.heisd_kv_desc(k_cache.data_ptr(), v_cache.data_ptr(), prefix_len.data_ptr(),
                             first_pred.data_ptr())
        st = (stream or torch.cuda.current_stream(dev)).cuda_stream
        rc = B.heisd_verify_tree_step(self.ctx, kv, tree_tokens.data_ptr(), parent.data_ptr(), T, batch, accept,
                                      skip_mask.data_ptr() if skip_mask is not None else None,
                                      out["accepted_len"].data_ptr(), out["next_token"].data_ptr(),
                                      out["accepted_path"].data_ptr(),
                                      out["target_bins"].data_ptr() if "target_bins" in out else None,
                                      out["bin_logits"].data_ptr() if "bin_logits" in out else None, st)
        if rc != 0:
            raise RuntimeError("heisd_verify_tree_step failed (%d): %s" % (rc, B.heisd_last_error(self.ctx)))
        return out

    def prefill_chunk(self, k_cache, v_cache, prefix_len, token_ids=None, x_rows=None, want_logits=False,
                      out=None, stream=None):
        """token_ids i32[batch,n], x_rows f32[batch,n,d] on the device, or both (then a row whose id is
        negative takes its embedding from x_rows).  Returns dict of device tensors: next_bin i32[batch]
        (and last_logits f32[batch,n_bins])."""
        src = token_ids if token_ids is not None else x_rows
        batch, n = src.shape[0], src.shape[1]
        dev = self.model.device
        if out is None:
            out = {"next_bin": torch.empty(batch, dtype=torch.int32, device=dev)}
            if want_logits:
                out["last_logits"] = torch.empty(batch, self.model.shape["n_bins"], dtype=torch.float32, device=dev)
        kv = B.heisd_kv_desc(k_cache.data_ptr(), v_cache.data_ptr(), prefix_len.data_ptr(), None)
        st = (stream or torch.cuda.current_stream(dev)).cuda_stream
        rc = B.heisd_prefill_chunk(self.ctx, kv, token_ids.data_ptr() if token_ids is not None else None,
                                   x_rows.data_ptr() if x_rows is not None else None, n, batch,
                                   out["next_bin"].data_ptr(),
                                   out["last_logits"].data_ptr() if "last_logits" in out else None, st)
        if rc != 0:
            raise RuntimeError("heisd_prefill_chunk failed (%d): %s" % (rc, B.heisd_last_error(self.ctx)))
        return out

    def close(self):
        if self.ctx is not None:
            B.heisd_free(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def build_sequence_tree(candidates, accept, max_tokens):
    """Host call: candidates i32[R,K] (numpy) -> (tokens[T], parent[T]) numpy arrays."""
    cand = np.ascontiguousarray(candidates, dtype=np.int32)
    R, K = cand.shape
    tokens = np.zeros(max_tokens, np.int32)
    parent = np.zeros(max_tokens, np.int32)
    rc, n = B.heisd_build_sequence_tree(cand.ctypes.data, R, K, accept, max_tokens, tokens.ctypes.data,
                                        parent.ctypes.data)
    if rc != 0:
        raise RuntimeError("heisd_build_sequence_tree failed (%d): %s" % (rc, B.heisd_last_error(None)))
    return tokens[:n].copy(), parent[:n].copy()
