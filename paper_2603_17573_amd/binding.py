"""ctypes binding of libheisd_verify.so: the same entry points as include/heisd_verify.h.

Argument marshalling only.  Every step of the verify path runs in the library's HIP
kernels; if the library is missing this module raises instead of computing anything
itself.  PyTorch appears only as the owner of device memory and streams (callers pass
tensor.data_ptr() and torch.cuda.current_stream().cuda_stream).
"""
import ctypes
import os
from ctypes import POINTER, Structure, c_char_p, c_float, c_int32, c_size_t, c_uint32, c_void_p

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libheisd_verify.so")

HEISD_OK, HEISD_EINVAL, HEISD_EUNSUPPORTED, HEISD_ENOMEM, HEISD_EHIP = 0, -1, -2, -3, -4
HEISD_MAX_GROUPS = 8


class heisd_model_desc(Structure):
    _fields_ = [(n, c_int32) for n in ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab",
                                      "n_bins", "bin_token_base")] + \
               [("rms_eps", c_float), ("rope_base", c_float),
                ("max_batch", c_int32), ("max_k", c_int32), ("kv_capacity", c_int32),
                ("tok_emb", c_void_p)] + \
               [(n, POINTER(c_void_p)) for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down",
                                                 "attn_norm", "ffn_norm")] + \
               [("final_norm", c_void_p), ("lm_head", c_void_p),
                ("workspace", c_void_p), ("workspace_bytes", c_size_t)]


class heisd_kv_desc(Structure):
    _fields_ = [("k_cache", c_void_p), ("v_cache", c_void_p), ("prefix_len", c_void_p),
                ("first_pred", c_void_p)]


class heisd_accept_desc(Structure):
    _fields_ = [("tok_threshold", c_int32), ("seq_budget", c_int32), ("n_groups", c_int32),
                ("group_sizes", c_int32 * HEISD_MAX_GROUPS), ("exact_group_mask", c_uint32),
                ("mode", c_int32)]


_lib = None


def load():
    """Load the HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libheisd_verify.so is not built; run paper_2603_17573_amd.build.build() "
                               "(there is no CPU fallback)")
        lib = ctypes.CDLL(LIB_PATH)
        lib.heisd_verify_workspace_bytes.argtypes = [POINTER(heisd_model_desc)]
        lib.heisd_verify_workspace_bytes.restype = c_size_t
        lib.heisd_verify_init.argtypes = [POINTER(heisd_model_desc), POINTER(c_void_p)]
        lib.heisd_verify_init.restype = ctypes.c_int
        lib.heisd_verify_step.argtypes = [c_void_p, POINTER(heisd_kv_desc), c_void_p, c_int32, c_int32,
                                          POINTER(heisd_accept_desc), c_void_p, c_void_p, c_void_p,
                                          c_void_p, c_void_p, c_void_p]
        lib.heisd_verify_step.restype = ctypes.c_int
        lib.heisd_verify_tree_step.argtypes = [c_void_p, POINTER(heisd_kv_desc), c_void_p, c_void_p, c_int32, c_int32,
                                               POINTER(heisd_accept_desc), c_void_p, c_void_p, c_void_p,
                                               c_void_p, c_void_p, c_void_p, c_void_p]
        lib.heisd_verify_tree_step.restype = ctypes.c_int
        lib.heisd_build_sequence_tree.argtypes = [c_void_p, c_int32, c_int32, POINTER(heisd_accept_desc), c_int32,
                                                  c_void_p, c_void_p, POINTER(c_int32)]
        lib.heisd_build_sequence_tree.restype = ctypes.c_int
        lib.heisd_prefill_chunk.argtypes = [c_void_p, POINTER(heisd_kv_desc), c_void_p, c_void_p, c_int32, c_int32,
                                            c_void_p, c_void_p, c_void_p]
        lib.heisd_prefill_chunk.restype = ctypes.c_int
        lib.heisd_export_features.argtypes = [c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p]
        lib.heisd_export_features.restype = ctypes.c_int
        lib.heisd_feature_similarity.argtypes = [c_void_p, c_void_p, c_int32, c_int32, c_int32, c_void_p, c_void_p]
        lib.heisd_feature_similarity.restype = ctypes.c_int
        lib.heisd_skip_offline.argtypes = [c_void_p, c_int32, c_int32, c_float, c_void_p, c_void_p, c_void_p, c_void_p,
                                           c_void_p]
        lib.heisd_skip_offline.restype = ctypes.c_int
        lib.heisd_skip_decide.argtypes = [c_void_p, c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p,
                                          c_void_p, c_void_p]
        lib.heisd_skip_decide.restype = ctypes.c_int
        lib.heisd_retrieve_workspace_bytes.argtypes = [ctypes.c_int64, c_int32, c_int32]
        lib.heisd_retrieve_workspace_bytes.restype = c_size_t
        lib.heisd_retrieve_topk.argtypes = [c_void_p, ctypes.c_int64, c_int32, c_void_p, c_int32, c_int32, c_void_p,
                                            c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
        lib.heisd_retrieve_topk.restype = ctypes.c_int
        lib.heisd_retrieve_static_bytes.argtypes = []
        lib.heisd_retrieve_static_bytes.restype = c_size_t
        lib.heisd_retrieve_topk_static.argtypes = [c_void_p, ctypes.c_int64, c_int32, c_void_p, c_int32, c_int32,
                                                   c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p]
        lib.heisd_retrieve_topk_static.restype = ctypes.c_int
        lib.heisd_free.argtypes = [c_void_p]
        lib.heisd_free.restype = None
        lib.heisd_verify_profile_enable.argtypes = [c_void_p, ctypes.c_int]
        lib.heisd_verify_profile_enable.restype = ctypes.c_int
        lib.heisd_verify_profile_read.argtypes = [c_void_p, POINTER(ctypes.c_double), POINTER(ctypes.c_int64)]
        lib.heisd_verify_profile_read.restype = ctypes.c_int
        lib.heisd_verify_set_path.argtypes = [c_void_p, ctypes.c_int]
        lib.heisd_verify_set_path.restype = ctypes.c_int
        lib.heisd_verify_check.argtypes = [c_void_p]
        lib.heisd_verify_check.restype = ctypes.c_int
        lib.heisd_measure_read.argtypes = [c_void_p, c_size_t, c_int32, c_int32, c_int32, c_int32, c_void_p, c_void_p]
        lib.heisd_measure_read.restype = ctypes.c_int
        lib.heisd_measure_empty_launch.argtypes = [c_int32, c_void_p]
        lib.heisd_measure_empty_launch.restype = ctypes.c_int
        lib.heisd_verify_set_handover.argtypes = [c_void_p, ctypes.c_int]
        lib.heisd_verify_set_handover.restype = ctypes.c_int
        lib.heisd_verify_set_activations.argtypes = [c_void_p, ctypes.c_int]
        lib.heisd_verify_set_activations.restype = ctypes.c_int
        lib.heisd_debug_set_wait_limits.argtypes = [c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.heisd_debug_set_wait_limits.restype = ctypes.c_int
        lib.heisd_verify_release_projections.argtypes = [c_void_p]
        lib.heisd_verify_release_projections.restype = ctypes.c_int
        lib.heisd_debug_trace.argtypes = [c_void_p, ctypes.c_int, c_void_p, ctypes.c_int]
        lib.heisd_debug_trace.restype = ctypes.c_int
        lib.heisd_last_error.argtypes = [c_void_p]
        lib.heisd_last_error.restype = c_char_p
        _lib = lib
    return _lib


def heisd_verify_workspace_bytes(desc: heisd_model_desc) -> int:
    return int(load().heisd_verify_workspace_bytes(ctypes.byref(desc)))


def heisd_verify_init(desc: heisd_model_desc):
    """Returns (rc, ctx handle or None)."""
    ctx = c_void_p()
    rc = load().heisd_verify_init(ctypes.byref(desc), ctypes.byref(ctx))
    return rc, (ctx if rc == 0 else None)


def heisd_verify_step(ctx, kv: heisd_kv_desc, draft_tokens, K, batch, accept: heisd_accept_desc,
                      skip_mask, accepted_len, next_token, target_bins, bin_logits, stream) -> int:
    """All array arguments are integer device addresses (0/None = NULL)."""
    return load().heisd_verify_step(ctx, ctypes.byref(kv) if kv is not None else None, draft_tokens, K, batch,
                                    ctypes.byref(accept) if accept is not None else None, skip_mask,
                                    accepted_len, next_token, target_bins, bin_logits, stream)


def heisd_verify_tree_step(ctx, kv: heisd_kv_desc, tree_tokens, parent, T, batch, accept: heisd_accept_desc,
                           skip_mask, accepted_len, next_token, accepted_path, target_bins, bin_logits,
                           stream) -> int:
    """All array arguments are integer device addresses (0/None = NULL)."""
    return load().heisd_verify_tree_step(ctx, ctypes.byref(kv) if kv is not None else None, tree_tokens, parent,
                                         T, batch, ctypes.byref(accept) if accept is not None else None,
                                         skip_mask, accepted_len, next_token, accepted_path, target_bins,
                                         bin_logits, stream)


def heisd_build_sequence_tree(candidates, R, K, accept: heisd_accept_desc, max_tokens, tokens, parent):
    """candidates, tokens, parent: HOST addresses (ints) of i32 arrays.  Returns (rc, n_tokens)."""
    n = c_int32(0)
    rc = load().heisd_build_sequence_tree(candidates, R, K, ctypes.byref(accept) if accept is not None else None,
                                          max_tokens, tokens, parent, ctypes.byref(n))
    return rc, int(n.value)


def heisd_prefill_chunk(ctx, kv: heisd_kv_desc, token_ids, x_rows, n_rows, batch, next_bin, last_logits,
                        stream) -> int:
    """All array arguments are integer device addresses (0/None = NULL)."""
    return load().heisd_prefill_chunk(ctx, ctypes.byref(kv) if kv is not None else None, token_ids, x_rows, n_rows,
                                      batch, next_bin, last_logits, stream)


def heisd_export_features(ctx, row, rows_per_episode, batch, feat, stream) -> int:
    return load().heisd_export_features(ctx, row, rows_per_episode, batch, feat, stream)


def heisd_feature_similarity(a, b, n, m, d, S, stream) -> int:
    return load().heisd_feature_similarity(a, b, n, m, d, S, stream)


def heisd_skip_offline(feat, n, d, T, S, work, min_s, o_dist, stream) -> int:
    return load().heisd_skip_offline(feat, n, d, T, S, work, min_s, o_dist, stream)


def heisd_skip_decide(feat_prev, feat_last, dist, batch, d, min_s, o_dist, skip_mask, similarity, stream) -> int:
    return load().heisd_skip_decide(feat_prev, feat_last, dist, batch, d, min_s, o_dist, skip_mask, similarity, stream)


def heisd_retrieve_workspace_bytes(n_vectors, batch, K) -> int:
    return int(load().heisd_retrieve_workspace_bytes(n_vectors, batch, K))


def heisd_retrieve_topk(db, n_vectors, d, queries, batch, K, payload, payload_len, top_index, top_score, top_payload,
                        workspace, workspace_bytes, stream) -> int:
    """All array arguments are integer device addresses (0/None = NULL)."""
    return load().heisd_retrieve_topk(db, n_vectors, d, queries, batch, K, payload, payload_len, top_index, top_score,
                                      top_payload, workspace, workspace_bytes, stream)


def heisd_retrieve_static_bytes() -> int:
    return int(load().heisd_retrieve_static_bytes())


def heisd_retrieve_topk_static(db, n_vectors, d, queries, batch, K, payload, payload_len, top_index, top_score,
                               top_payload, stream) -> int:
    """All array arguments are integer device addresses (0/None = NULL)."""
    return load().heisd_retrieve_topk_static(db, n_vectors, d, queries, batch, K, payload, payload_len, top_index,
                                             top_score, top_payload, stream)


def heisd_free(ctx) -> None:
    load().heisd_free(ctx)


def heisd_last_error(ctx=None) -> str:
    return load().heisd_last_error(ctx).decode()


HEISD_PATH_AUTO, HEISD_PATH_GENERIC, HEISD_PATH_FAST, HEISD_PATH_PERSIST, HEISD_PATH_BATCH = 0, 1, 2, 3, 4


def heisd_verify_check(ctx) -> int:
    return load().heisd_verify_check(ctx)


def heisd_verify_set_path(ctx, path: int) -> int:
    return load().heisd_verify_set_path(ctx, path)


def heisd_measure_read(buf, nbytes, pattern, ksteps, in_flight, workgroups, sink, stream) -> int:
    return load().heisd_measure_read(buf, nbytes, pattern, ksteps, in_flight, workgroups, sink, stream)


def heisd_measure_empty_launch(workgroups, stream) -> int:
    return load().heisd_measure_empty_launch(workgroups, stream)


def heisd_verify_set_handover(ctx, mode: int) -> int:
    return load().heisd_verify_set_handover(ctx, mode)


HEISD_ACT_SPLIT, HEISD_ACT_BF16 = 0, 1


def heisd_debug_set_wait_limits(ctx, grid_polls: int, scale_polls: int, skip_scales: int) -> int:
    return load().heisd_debug_set_wait_limits(ctx, grid_polls, scale_polls, skip_scales)


def heisd_verify_release_projections(ctx) -> int:
    return load().heisd_verify_release_projections(ctx)


def heisd_verify_set_activations(ctx, fmt: int) -> int:
    return load().heisd_verify_set_activations(ctx, fmt)


def heisd_debug_trace(ctx, enable: bool, max_entries: int = 0):
    """Returns (rc, list of timestamps) - the list is empty unless max_entries > 0."""
    if max_entries <= 0:
        return load().heisd_debug_trace(ctx, 1 if enable else 0, None, 0), []
    buf = (ctypes.c_ulonglong * max_entries)()
    rc = load().heisd_debug_trace(ctx, 1 if enable else 0, buf, max_entries)
    return rc, list(buf[:max(rc, 0)])


KERNEL_CLASSES = ("embed", "qkv", "attn", "oproj", "gateup", "down", "lmhead", "accept", "persist")


def heisd_verify_profile_enable(ctx, enable: bool) -> int:
    return load().heisd_verify_profile_enable(ctx, 1 if enable else 0)


def heisd_verify_profile_read(ctx):
    """Returns (rc, {class: (total_ms, launches)})."""
    ms = (ctypes.c_double * len(KERNEL_CLASSES))()
    n = (ctypes.c_int64 * len(KERNEL_CLASSES))()
    rc = load().heisd_verify_profile_read(ctx, ms, n)
    return rc, {k: (ms[i], n[i]) for i, k in enumerate(KERNEL_CLASSES)}


def make_accept_desc(tok_threshold=15, seq_budget=30, group_sizes=(3, 3, 1), exact_group_mask=0b100,
                     mode=0) -> heisd_accept_desc:
    a = heisd_accept_desc()
    a.tok_threshold, a.seq_budget, a.n_groups = tok_threshold, seq_budget, len(group_sizes)
    for i in range(HEISD_MAX_GROUPS):
        a.group_sizes[i] = group_sizes[i] if i < len(group_sizes) else 0
    a.exact_group_mask, a.mode = exact_group_mask, mode
    return a


def _ptr_table(ptrs):
    arr = (c_void_p * len(ptrs))(*ptrs)
    return arr


def make_model_desc(shape: dict, ptrs: dict, max_batch, max_k, kv_capacity, workspace=0, workspace_bytes=0):
    """shape: n_layers, d_model, n_heads, head_dim, d_ffn, vocab, n_bins, bin_token_base, rms_eps,
    rope_base.  ptrs: device addresses: tok_emb, lm_head, final_norm (ints) and per-layer lists wq, wk, wv,
    wo, w_gate, w_up, w_down, attn_norm, ffn_norm.  Returns (desc, keepalive) - keep `keepalive`
    referenced while the descriptor is in use."""
    d = heisd_model_desc()
    for k in ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab", "n_bins", "bin_token_base",
              "rms_eps", "rope_base"):
        setattr(d, k, shape[k])
    d.max_batch, d.max_k, d.kv_capacity = max_batch, max_k, kv_capacity
    keep = []
    for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "attn_norm", "ffn_norm"):
        t = _ptr_table(ptrs[k])
        keep.append(t)
        setattr(d, k, ctypes.cast(t, POINTER(c_void_p)))
    d.tok_emb, d.lm_head, d.final_norm = ptrs["tok_emb"], ptrs["lm_head"], ptrs["final_norm"]
    d.workspace, d.workspace_bytes = workspace, workspace_bytes
    return d, keep
