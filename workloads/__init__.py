"""Seeded synthetic inputs (decoding graphs and CTC log-likelihoods).

This module is pure data generation: it holds none of the decoder's arithmetic
and is the only code shared by the CPU oracle's tests and the HIP path's tests
and benchmark.  Everything is a deterministic function of an integer seed.
"""
from .graphs import (Graph, tiny_lexicon_graph, tlg_shaped_graph, ctc_topology_graph,
                     micro_graph, permute_arcs_within_states, dense_graph, giant_state_graph,
                     eps_layers_graph, loop_tie_graph)
from .loglikes import ctc_loglikes, random_lengths
from .configs import CONFIGS, make_config, boost_tables
from .boost import BoostFst, boost_trie, boost_fsts, random_targets

__all__ = ["Graph", "tiny_lexicon_graph", "tlg_shaped_graph", "ctc_topology_graph",
           "micro_graph", "permute_arcs_within_states", "dense_graph", "giant_state_graph",
           "eps_layers_graph", "loop_tie_graph", "ctc_loglikes", "random_lengths",
           "CONFIGS", "make_config", "boost_tables", "BoostFst", "boost_trie", "boost_fsts", "random_targets"]
