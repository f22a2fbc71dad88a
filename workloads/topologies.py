"""Synthetic network topologies: directed graphs of compute and switch nodes with
integer link bandwidths (the input of the paper's problem definition, Section 5).

Every generator is deterministic.  A bidirectional link of bandwidth b is emitted
as two directed arcs of bandwidth b.  Parallel arcs may be emitted on purpose
(config 2): consumers must add their bandwidths (integer capacity = number of
multi-edges, Appendix E.1).

The five `config_topology(i)` graphs stand in for the paper's cluster topologies
(2-box MI250, DGX A100, fat-tree and 1024-node fabrics of Section 6), whose real
description files are not public; shapes and capacities follow the benchmark
configuration list of this repository.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 24020678

CONFIG_NAMES = {
    1: "cfg1_2box8_switch_spine",
    2: "cfg2_mi250_like_2x16_direct",
    3: "cfg3_dgx_a100_like_16x8",
    4: "cfg4_fat_tree_64x8",
    5: "cfg5_random_fabric_1024c_128s",
}


@dataclass(frozen=True)
class Topology:
    """COO digraph.  Vertex ids are 0..n_vertices-1; the super-source is NOT included."""
    name: str
    n_vertices: int
    tail: np.ndarray        # int32 [n_arcs]
    head: np.ndarray        # int32 [n_arcs]
    bandwidth: np.ndarray   # int32 [n_arcs], >= 0
    is_compute: np.ndarray  # uint8 [n_vertices], 1 = compute node, 0 = switch node

    @property
    def n_arcs(self) -> int:
        return int(self.tail.shape[0])

    @property
    def compute_nodes(self) -> np.ndarray:
        return np.flatnonzero(self.is_compute).astype(np.int32)

    @property
    def n_compute(self) -> int:
        return int(self.is_compute.sum())


class _Builder:
    def __init__(self, name: str, n_vertices: int, n_compute_prefix: int | None = None):
        self.name = name
        self.n = n_vertices
        self.t: list[int] = []
        self.h: list[int] = []
        self.b: list[int] = []
        self.is_compute = np.zeros(n_vertices, dtype=np.uint8)
        if n_compute_prefix is not None:
            self.is_compute[:n_compute_prefix] = 1

    def arc(self, u: int, v: int, bw: int) -> None:
        self.t.append(int(u)); self.h.append(int(v)); self.b.append(int(bw))

    def link(self, u: int, v: int, bw: int) -> None:
        self.arc(u, v, bw); self.arc(v, u, bw)

    def done(self) -> Topology:
        return Topology(self.name, self.n,
                        np.asarray(self.t, dtype=np.int32),
                        np.asarray(self.h, dtype=np.int32),
                        np.asarray(self.b, dtype=np.int32),
                        self.is_compute.copy())


# --------------------------------------------------------------------------- paper's worked example

def paper_example_switch(b: int = 1) -> Topology:
    """The 2-box, 8-compute-node switch topology of the paper's Section 4 figure.

    ids: box 1 compute 0..3, box 2 compute 4..7, w1 = 8, w2 = 9 (intra-box, 10b),
    w0 = 10 (inter-box, b).
    """
    g = _Builder(f"paper_2x4_switch_b{b}", 11, 8)
    for box in range(2):
        for j in range(4):
            c = 4 * box + j
            g.link(c, 8 + box, 10 * b)
            g.link(c, 10, b)
    return g.done()


def paper_example_split(b: int = 1) -> Topology:
    """Switch-free topology the paper obtains from the example by edge splitting
    (Appendix E.2 figure): a directed 10b ring inside each box and a bidirectional
    b link between c_{1,j} and c_{2,j}."""
    g = _Builder(f"paper_2x4_split_b{b}", 8, 8)
    for box in range(2):
        for j in range(4):
            g.arc(4 * box + j, 4 * box + (j + 1) % 4, 10 * b)
    for j in range(4):
        g.link(j, 4 + j, b)
    return g.done()


def paper_example_ring_unwound(b: int = 1) -> Topology:
    """The 'unwound into rings' alternative the paper's Appendix E preamble calls
    4x worse: a directed 10b ring inside each box plus ONE directed b ring through
    all eight compute nodes (box 1 forwards, crossing to box 2, box 2 backwards)."""
    g = _Builder(f"paper_2x4_ring_unwound_b{b}", 8, 8)
    for box in range(2):
        for j in range(4):
            g.arc(4 * box + j, 4 * box + (j + 1) % 4, 10 * b)
    ring = [0, 1, 2, 3, 7, 6, 5, 4]
    for i in range(8):
        g.arc(ring[i], ring[(i + 1) % 8], b)
    return g.done()


# --------------------------------------------------------------------------- textbook shapes

def complete_digraph(n: int, c: int) -> Topology:
    g = _Builder(f"K{n}_c{c}", n, n)
    for u in range(n):
        for v in range(n):
            if u != v:
                g.arc(u, v, c)
    return g.done()


def directed_ring(n: int, c: int) -> Topology:
    g = _Builder(f"dring{n}_c{c}", n, n)
    for u in range(n):
        g.arc(u, (u + 1) % n, c)
    return g.done()


def bidirectional_ring(n: int, c: int) -> Topology:
    g = _Builder(f"bring{n}_c{c}", n, n)
    for u in range(n):
        g.link(u, (u + 1) % n, c)
    return g.done()


def star_switch(n: int, c: int) -> Topology:
    """n compute nodes, each joined to one switch (id n) by a bidirectional link c."""
    g = _Builder(f"star{n}_c{c}", n + 1, n)
    for u in range(n):
        g.link(u, n, c)
    return g.done()


def random_tiny(seed: int, n_vertices: int | None = None, max_cap: int = 9,
                density: float = 0.45, switch_free: bool = False,
                strongly_connected: bool = True) -> Topology:
    """Small random digraph for brute-force checks: random compute/switch split
    (at least two compute nodes), random arcs with capacities in 1..max_cap, a few
    parallel arcs and an occasional zero-bandwidth arc and self-loop (which
    consumers must ignore)."""
    rng = np.random.default_rng(seed)
    n = int(n_vertices) if n_vertices is not None else int(rng.integers(3, 9))
    g = _Builder(f"tiny_s{seed}_n{n}", n)
    if switch_free:
        g.is_compute[:] = 1
    else:
        ncomp = int(rng.integers(2, n + 1))
        g.is_compute[rng.permutation(n)[:ncomp]] = 1
    if strongly_connected:
        order = rng.permutation(n)
        for i in range(n):
            g.arc(order[i], order[(i + 1) % n], int(rng.integers(1, max_cap + 1)))
    for u in range(n):
        for v in range(n):
            if u != v and rng.random() < density:
                g.arc(u, v, int(rng.integers(1, max_cap + 1)))
                if rng.random() < 0.15:      # parallel arc
                    g.arc(u, v, int(rng.integers(1, max_cap + 1)))
    if rng.random() < 0.3:
        g.arc(int(rng.integers(n)), int(rng.integers(n)), 0)   # zero-bandwidth arc
    if rng.random() < 0.3:
        u = int(rng.integers(n)); g.arc(u, u, int(rng.integers(1, max_cap + 1)))  # self-loop
    return g.done()


def superposed_out_trees(n: int, k: int, seed: int) -> dict:
    """Link capacities {(x, y): c} of a switch-free digraph over vertices 0..n-1 laid down as k random spanning
    out-trees per root, one unit of capacity per tree edge: a packing of k out-trees per root exists by
    construction and uses every unit, so spanning tree construction (Appendix E.3) must find one that does too.
    Capacities vary from link to link and most trees end up with a multiplicity of their own."""
    rng = np.random.default_rng(seed)
    links: dict = {}
    for root in range(n):
        for _ in range(k):
            order = [root] + [int(v) for v in rng.permutation([v for v in range(n) if v != root])]
            for i in range(1, n):
                x, y = order[int(rng.integers(0, i))], order[i]
                links[(x, y)] = links.get((x, y), 0) + 1
    return links


# --------------------------------------------------------------------------- the five benchmark configs

def _config1() -> Topology:
    g = _Builder(CONFIG_NAMES[1], 19, 16)
    for c in range(16):
        g.link(c, 16 + c // 8, 12)
    g.link(16, 18, 8)
    g.link(17, 18, 8)
    return g.done()


def _mi250_box_links(rng: np.random.Generator, n_box: int = 16, max_degree: int = 8,
                     max_mult: int = 4) -> list[tuple[int, int, int]]:
    pairs = [(i, j) for i in range(n_box) for j in range(i + 1, n_box)]
    degree = [0] * n_box
    out = []
    for idx in rng.permutation(len(pairs)):
        i, j = pairs[int(idx)]
        m = int(rng.integers(0, max_mult + 1))
        m = min(m, max_degree - degree[i], max_degree - degree[j])
        if m > 0:
            degree[i] += m; degree[j] += m
            out.append((i, j, m))
    return out


def _connected(n: int, links: list[tuple[int, int, int]]) -> bool:
    adj = [[] for _ in range(n)]
    for i, j, _ in links:
        adj[i].append(j); adj[j].append(i)
    seen = {0}; stack = [0]
    while stack:
        u = stack.pop()
        for v in adj[u]:
            if v not in seen:
                seen.add(v); stack.append(v)
    return len(seen) == n


def _config2() -> Topology:
    g = _Builder(CONFIG_NAMES[2], 33, 32)
    seed = BASE_SEED + 2
    for box in range(2):
        while True:
            links = _mi250_box_links(np.random.default_rng(seed))
            seed += 1
            if _connected(16, links):
                break
        for i, j, m in links:
            for _ in range(m):                       # m parallel links of capacity 2
                g.link(16 * box + i, 16 * box + j, 2)
        for loc in (0, 4, 8, 12):                    # 4 NIC arcs per box, capacity 1
            g.link(16 * box + loc, 32, 1)
    return g.done()


def _config3() -> Topology:
    g = _Builder(CONFIG_NAMES[3], 145, 128)
    for c in range(128):
        g.link(c, 128 + c // 8, 24)
        g.link(c, 144, 2)
    return g.done()


def _config4() -> Topology:
    g = _Builder(CONFIG_NAMES[4], 596, 512)
    for c in range(512):
        box = c // 8
        g.link(c, 512 + box, 32)
        g.link(c, 576 + box // 4, 4)
    for leaf in range(16):
        for spine in range(4):
            g.link(576 + leaf, 592 + spine, 64)
    return g.done()


def _config5(n_compute: int = 1024, n_switch: int = 128, out_degree: int = 8,
             max_cap: int = 100, seed: int = BASE_SEED + 5, name: str | None = None) -> Topology:
    n = n_compute + n_switch
    g = _Builder(name or CONFIG_NAMES[5], n, n_compute)
    rng = np.random.default_rng(seed)
    for u in range(n):
        ring_head = (u + 1) % n
        heads = [ring_head]
        while len(heads) < out_degree:
            v = int(rng.integers(n))
            if v != u and v not in heads:
                heads.append(v)
        caps = rng.integers(1, max_cap + 1, size=out_degree)
        for v, c in zip(heads, caps):
            g.arc(u, v, int(c))
    return g.done()


def rail_fabric(n_boxes: int = 128, per_box: int = 8, nvswitch_cap: int = 24, nic_cap: int = 2,
                name: str | None = None) -> Topology:
    """Eulerian switch topology shaped like a rail-optimised DGX-A100 cluster: `n_boxes` boxes of `per_box` compute
    nodes, one NVSwitch node per box (bidirectional links of `nvswitch_cap`), and `per_box` rail switches: compute
    node j of every box has a bidirectional NIC link of `nic_cap` to rail switch j.  Every link is bidirectional, so
    every vertex has equal in- and out-bandwidth.  The default is the 1024-compute instance (1160 vertices) on which
    the generator's back end -- switch removal, spanning tree construction -- is timed; it stands in for the
    1024-GPU A100 topology of the paper's generation-time table (Appendix C), whose description file is not public."""
    n_compute = n_boxes * per_box
    g = _Builder(name or f"rail_fabric_{n_boxes}x{per_box}", n_compute + n_boxes + per_box, n_compute)
    for c in range(n_compute):
        g.link(c, n_compute + c // per_box, nvswitch_cap)
        g.link(c, n_compute + n_boxes + c % per_box, nic_cap)
    return g.done()


def eulerian_fabric_1024() -> Topology:
    """128 boxes x 8 compute nodes, 128 NVSwitch nodes, 8 rail switches (see `rail_fabric`)."""
    return rail_fabric(128, 8, 24, 2, name="rail_fabric_1024c_128x8")


def config_topology(cfg: int) -> Topology:
    """Benchmark configuration `cfg` in 1..5 (see module docstring)."""
    return {1: _config1, 2: _config2, 3: _config3, 4: _config4, 5: _config5}[cfg]()


def shrunken_config5(seed: int = 7, n_compute: int = 12, n_switch: int = 4,
                     out_degree: int = 3, max_cap: int = 9) -> Topology:
    """Brute-force-sized analogue of config 5 (same recipe, 16 vertices)."""
    return _config5(n_compute, n_switch, out_degree, max_cap, seed,
                    name=f"cfg5_shrunk_s{seed}")
