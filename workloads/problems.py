"""Problem lists for the batched feasibility path.

One problem is a triple (sink v_j, edge multiplier U_j, source-arc capacity k_j):
the auxiliary network of the paper's Section 5.2 scaled to integers, i.e. every
topology arc e gets capacity U_j * b_e and every arc s->c, c a compute node, gets
capacity k_j (candidate 1/x = U_j / k_j).  Nothing is solved here.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from .topologies import Topology


@dataclass(frozen=True)
class ProblemList:
    sink: np.ndarray        # int32 [n_problems]
    edge_mult: np.ndarray   # int32 [n_problems], U_j >= 1
    src_cap: np.ndarray     # int32 [n_problems], k_j >= 1
    # candidate-major layout: problem j = cand * n_sinks + sink_index
    n_candidates: int
    n_sinks: int

    @property
    def n_problems(self) -> int:
        return int(self.sink.shape[0])


def all_sinks(topo: Topology, cand_U, cand_k) -> ProblemList:
    """Every compute node as sink for each candidate (U, k)."""
    cand_U = np.asarray(cand_U, dtype=np.int64).reshape(-1)
    cand_k = np.asarray(cand_k, dtype=np.int64).reshape(-1)
    assert cand_U.shape == cand_k.shape
    sinks = topo.compute_nodes
    C, S = cand_U.shape[0], sinks.shape[0]
    return ProblemList(
        sink=np.tile(sinks, C).astype(np.int32),
        edge_mult=np.repeat(cand_U, S).astype(np.int32),
        src_cap=np.repeat(cand_k, S).astype(np.int32),
        n_candidates=C, n_sinks=S)


def _ceil_div(a: int, b: int) -> int:
    return -((-a) // b)


def config_candidates(cfg: int, inv_xstar: tuple[int, int] | None = None,
                      extra_parity: bool = False):
    """Candidate (U_j, k_j) lists of the five benchmark configurations.

    Configs 2 and 5 centre their candidates on the optimum 1/x* = p/q of their
    (seeded random) topology, which the caller supplies as `inv_xstar=(p, q)`:
    half of the candidates fall below it (infeasible) and half at or above.
    """
    if cfg == 1:
        U = [1]; k = [4]                        # the configured batch: 16 sinks x 1 candidate
        if extra_parity:                        # further candidates for parity tests only
            U += [4, 5, 6]; k += [4, 4, 4]
    elif cfg == 3:
        U = [44 + j for j in range(32)]; k = [8] * 32
    elif cfg == 4:
        U = [55 + j for j in range(16)]; k = [4] * 16
    elif cfg in (2, 5):
        if inv_xstar is None:
            raise ValueError("configs 2 and 5 need inv_xstar=(p, q)")
        p, q = int(inv_xstar[0]), int(inv_xstar[1])
        k0, nc = (4, 8) if cfg == 2 else (16, 16)
        base = _ceil_div(k0 * p, q) - nc // 2
        U = [max(1, base + j) for j in range(nc)]; k = [k0] * nc
    else:
        raise ValueError(f"unknown config {cfg}")
    return np.asarray(U, dtype=np.int32), np.asarray(k, dtype=np.int32)


def config_problems(cfg: int, topo: Topology, inv_xstar: tuple[int, int] | None = None,
                    extra_parity: bool = False) -> ProblemList:
    U, k = config_candidates(cfg, inv_xstar, extra_parity)
    return all_sinks(topo, U, k)
