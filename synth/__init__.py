"""Seeded synthetic inputs for the HeiSD verify step.

A module of its own: it draws random numbers and lays them out in the formats the
verify step's inputs are defined in.  It contains none of the method's arithmetic,
imports neither the CPU oracle nor the GPU binding, and is the only code the two
sides' tests have in common.
"""
from .rng import (normal_bf16, normal_f32, normal_f64, uniform_i32, uniform_f64,
                  stream_id, build_native)
from .workloads import (ModelShape, Workload, TINY, LLAMA7B, WORKLOADS, make_weights,
                        make_prefix_inputs, make_prefix_kv_direct, make_drafts_uniform,
                        make_offsets_geometric, make_candidate_offsets, make_skip_mask, make_retrieval_db,
                        make_retrieval_queries, bf16_bits_to_f32,
                        f32_to_bf16_bits)

__all__ = [n for n in dir() if not n.startswith("_")]
