"""CPU oracle for the batched max-flow feasibility path -- test infrastructure only.

Only tests, the smoke check and the bench's `cpu_baseline` leg may import this
package; it shares no code with the HIP library and never imports it.
"""
from .reference import (Disconnected, build_c, maxflow, aux_network, aux_maxflow,
                        aux_maxflow_batch, feasible, in_bandwidths,
                        min_compute_in_bandwidth, fraction_in_interval, smallest_true_fraction,
                        optimality_binary_search, smallest_U_k, brute_inv_xstar,
                        brute_min_cut, brute_cut_condition, aux_maxflow_batch_floor,
                        fixed_k_feasible, fixed_k_binary_search, brute_fixed_k, links, link_capacities, is_eulerian,
                        unbounded, split_flows, split_gamma, split_off, brute_split_gamma, remove_switches,
                        weighted_aux_network, weighted_aux_maxflow_batch, weighted_feasible,
                        tree_mu_network, tree_mu, brute_tree_mu, construct_trees)
