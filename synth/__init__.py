"""Seeded synthetic inputs: DAG-shaped states, candidate sets, masks, weights, upstream grads.

This package serves both the CPU oracle's tests and the GPU library's tests/benchmarks.
It produces inputs only; it contains none of the encoder's arithmetic and imports neither
the oracle nor the GPU package.
"""
from .graphs import (Graph, layered_dag, transformer_dag, resnet_dag, inception_dag,
                     local_rewrite, shuffle_edges, local_rewrite_edit, apply_edit)
from .states import (CONFIGS, BASE_SEED, make_state, make_config, concat_states,
                     init_weights, upstream_grads, state_subset, random_states, make_edit_states)

__all__ = ["Graph", "layered_dag", "transformer_dag", "resnet_dag", "inception_dag",
           "local_rewrite", "shuffle_edges", "CONFIGS", "BASE_SEED", "make_state",
           "make_config", "concat_states", "init_weights", "upstream_grads", "state_subset", "random_states",
           "local_rewrite_edit", "apply_edit", "make_edit_states"]
