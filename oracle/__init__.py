"""Plain fp64 CPU oracle of the HeiSD target-model verify step.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and its
Python binding) may import, link or call this package; only tests/, the smoke
check and the benchmark's cpu_baseline leg do.  It shares no code with the HIP
path and imports neither it nor the input generators.
"""
from .heisd_oracle import (OracleModel, widen_bf16, linear_bf16w, embed, rmsnorm, rope, silu, attention_block,
                           forward_block, prefill, bin_logits, argmax_bins, accept_block,
                           AcceptRule, verify_step, build_native)
from .heisd_skip_oracle import (final_features, cosine, similarity_matrix, offline_stage, skip_decision)
from .heisd_retrieval_oracle import similarity_scores, top_k, retrieve
from .heisd_tree_oracle import (build_sequence_tree, tree_chains, first_chain, accept_tree, verify_tree_step)

__all__ = [n for n in dir() if not n.startswith("_")]
