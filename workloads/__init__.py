"""Seeded synthetic inputs for the draft-then-verify exploration path.

This module only *describes* and *draws* inputs: loop-nest descriptors of the
tuned subgraphs, candidate schedules (tile-factor vectors plus unroll /
vectorize annotations), statement-feature tensors and cost-model weights.
It holds none of the method's arithmetic (no symbols, penalties, scores,
selection or model evaluation), so that the CPU oracle and the HIP library,
which share no code, can both be fed from it.

Everything here is a stand-in: the populations the paper explores come from
Ansor/MetaSchedule sketches of its 14 DNNs and from the TenSet dataset
(Experimental Settings; Sec. 6 "Feasibility Analysis"); neither is available,
and no item of either is reproduced.  What is kept is the structure: the
multi-level tile factorisations, unroll factors, per-subgraph population
sizes and the 164-wide per-statement feature rows (Introduction).
"""
from .rng import mix64, hash_u64, uniform01
from .subgraphs import (
    Device, Buffer, Subgraph, a100_like, toy_device,
    gemm, batched_gemm, conv2d, depthwise_conv2d, n_slots,
)
from .schedules import (
    ordered_factorizations, count_ordered_factorizations, axis_tables,
    sample_population, enumerate_all_schedules, UNROLL_VALUES, VECTOR_VALUES,
)
from .configs import Workload, make_config, bert_base_subgraphs, CONFIG_NAMES
from .costmodel import (
    FEAT_DIM, MAX_STMT, HIDDEN, FLOW_DIM, MAX_BLOCKS, EMBED, make_mlp_weights, make_statement_features,
    make_pacm_weights, make_flow_features,
    f32_to_bf16_bits, bf16_bits_to_f32,
)

__all__ = [n for n in dir() if not n.startswith("_")]
