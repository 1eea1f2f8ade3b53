"""HeiSD target-model verify step for AMD MI355X: hand-written HIP kernels behind a C ABI.

This package holds the kernels (csrc/), the build step and a ctypes binding with the same
entry points as include/heisd_verify.h, plus a small torch-facing convenience class that
only moves pointers around.
"""
from .binding import (heisd_model_desc, heisd_kv_desc, heisd_accept_desc, heisd_verify_workspace_bytes,
                      heisd_verify_init, heisd_verify_step, heisd_verify_tree_step,
                      heisd_build_sequence_tree, heisd_prefill_chunk, heisd_export_features,
                      heisd_feature_similarity, heisd_skip_offline, heisd_skip_decide,
                      heisd_retrieve_workspace_bytes, heisd_retrieve_topk, heisd_retrieve_static_bytes,
                      heisd_retrieve_topk_static, heisd_debug_trace, heisd_verify_set_handover, heisd_verify_set_activations, heisd_verify_release_projections, heisd_debug_set_wait_limits, HEISD_ACT_SPLIT, HEISD_ACT_BF16, heisd_measure_read,
                      heisd_measure_empty_launch, heisd_free, heisd_last_error,
                      heisd_verify_profile_enable, heisd_verify_profile_read, KERNEL_CLASSES,
                      heisd_verify_set_path, heisd_verify_check, HEISD_PATH_AUTO, HEISD_PATH_GENERIC, HEISD_PATH_FAST,
                      HEISD_PATH_PERSIST, HEISD_PATH_BATCH,
                      make_accept_desc, make_model_desc, HEISD_OK, HEISD_EINVAL, HEISD_EUNSUPPORTED,
                      HEISD_ENOMEM, HEISD_EHIP)
from .runner import DeviceModel, Verifier, build_sequence_tree

__all__ = [n for n in dir() if not n.startswith("_")]
