"""Seeded synthetic search-tree workloads.

This module only *generates inputs*: tree topologies shaped like PRM-guided
parallel tree searches (a shared prompt root, W trajectories per step, parents
re-sampled every step so that trajectories share ancestor steps) and N(0,1)
K/V/Q values.  It contains none of the attention arithmetic, and both the CPU
oracle's tests and the HIP library's tests draw their inputs from here.
"""
from .trees import (CONFIGS, Tree, TreeConfig, make_tree, make_values_host,
                    make_values_device, to_bf16_bits, bf16_bits_to_f32,
                    random_tree, with_growth_room, make_new_tokens_host,
                    make_prefill_queries_host, quantize_e4m3, make_values_fp8_host,
                    make_values_fp8_device)
from .search_sim import simulate_search

__all__ = ["CONFIGS", "Tree", "TreeConfig", "make_tree", "make_values_host",
           "make_values_device", "to_bf16_bits", "bf16_bits_to_f32",
           "random_tree", "with_growth_room", "make_new_tokens_host",
           "make_prefill_queries_host", "quantize_e4m3", "make_values_fp8_host",
           "make_values_fp8_device", "simulate_search"]
