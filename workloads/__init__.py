"""Seeded synthetic inputs shaped like the paper's serving workloads.

This module only draws inputs; it holds none of the LoRA arithmetic.  Both the HIP path and
the CPU oracle consume the arrays it returns (bf16 tensors as uint16 bit patterns), so the two
sides always see bit-identical inputs.

Shapes follow the five benchmark configurations:
  c1  tiny decode                      (64 tokens, 256->256, 8 slots, rank 8)
  c2  4B-dense-like decode layer       (256 tokens, q/k/v/o/gate/up/down, 64 slots, rank 16, Zipf)
  c3  rank-1 compact catalog           (512 tokens, 4096->4096, 1024 slots, all distinct)
  c4  30B-MoE-like packed LoRA         (2048 tokens, 128 experts top-8, 32 slots, rank 8; gate, up,
                                        and the down projection with the routing-weight combine;
                                        a variant with slot ranks drawn from {2, 4, 8})
  c5  segmented prefill                (8192 tokens, 16 lognormal segments, rank 64)
The same-batch adapter window (<= 64 distinct adapters in one decoding step), the expert
geometry (hidden 2048, expert intermediate 768, 128 experts) and the 10^6-entry catalog id
space come from the paper's serving section and its adapter tensor census.
"""
from .gen import (  # noqa: F401
    SEED0, rng, to_bf16_bits, normal_bf16, zipf_slots, lognormal_segments, topk_routing,
    DenseCase, MoECase, MoEDownCase, SegCase, routing_weights,
    dense_case, moe_case, moe_down_case, seg_case,
    c1_tiny_decode, c2_projections, c2_dense_decode, c3_rank1_catalog, c4_moe_packed,
    c4_moe_down, c4_moe_mixed_rank, c5_segmented,
)
