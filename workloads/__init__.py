"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP library's tests.

This package holds input *generators* only: topologies as COO arc lists and
problem lists as plain integer arrays.  It contains none of the method's
arithmetic (no max-flow, no feasibility test, no search) and imports neither
the oracle nor the HIP binding.
"""
from .topologies import (Topology, config_topology, shrunken_config5, paper_example_switch,
                         paper_example_split, paper_example_ring_unwound,
                         random_tiny, complete_digraph, directed_ring,
                         bidirectional_ring, star_switch, superposed_out_trees, rail_fabric, eulerian_fabric_1024,
                         CONFIG_NAMES)
from .problems import ProblemList, config_problems, all_sinks

__all__ = [
    "Topology", "config_topology", "shrunken_config5", "paper_example_switch", "paper_example_split",
    "paper_example_ring_unwound", "random_tiny", "complete_digraph",
    "directed_ring", "bidirectional_ring", "star_switch", "superposed_out_trees", "rail_fabric", "eulerian_fabric_1024",
    "CONFIG_NAMES",
    "ProblemList", "config_problems", "all_sinks",
]
