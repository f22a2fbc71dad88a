"""Pins for the CPU oracle: each test checks it against something other than itself --
values the paper states for its worked example, closed forms from the min-cut theorem,
brute-force enumeration on tiny graphs, and invariants the paper's theorems fix."""
import json
import os
from fractions import Fraction
from math import ceil, log2

import math

import numpy as np
import pytest

import oracle as o
import workloads as w
from workloads.topologies import shrunken_config5

GOLD = os.path.join(os.path.dirname(__file__), "golden")
ALGOS = ("dinic", "edmonds_karp")


def _gold(name):
    with open(os.path.join(GOLD, name)) as f:
        return json.load(f)


# ---------------------------------------------------------------- the paper's worked example

@pytest.mark.parametrize("b", [1, 2, 3, 7])
def test_paper_example_bottleneck_and_search(b):
    g = _gold("paper_worked_example.json")
    topo = w.paper_example_switch(b)
    want = Fraction(*g["bottleneck_ratio_times_b"]["value"]) / b       # Section 4: 1/x* = 1/b
    assert o.brute_inv_xstar(topo) == want
    assert o.optimality_binary_search(topo) == want
    # Section 5.2 "Determine k" / Appendix E.1: U = 1/b, k = 1, capacities become {1, 10}
    U, k = o.smallest_U_k(want, topo.bandwidth)
    assert (U, k) == (Fraction(g["scaled_capacities"]["U_times_b"], b), g["scaled_capacities"]["k"])
    assert sorted({int(U * int(x)) for x in topo.bandwidth}) == g["scaled_capacities"]["value"]


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("b", [1, 3])
def test_paper_example_flows(algo, b):
    g = _gold("paper_worked_example.json")
    topo = w.paper_example_switch(b)
    # x = b: every sink receives all 8x (Section 5.2)
    for v in range(8):
        assert o.aux_maxflow(topo, v, 1, b, algo) == g["flow_at_x_equals_b_over_b"]["value"] * b
    # b < x <= 7b/3: capped at 4x + 4b (Section 5.2); x/b = 2 lies in that range
    x = 2 * b
    assert o.aux_maxflow(topo, 5, 1, x, algo) == 4 * x + 4 * b
    # x/b = 3: the single-node cut x + 11b (B+(S') = 11b, Section 5.2) binds instead
    x = 3 * b
    assert o.aux_maxflow(topo, 5, 1, x, algo) == x + g["exit_bandwidth_all_but_one_over_b"]["value"] * b
    # verdicts around the optimum
    assert o.feasible(topo, 1, b, algo)[0] is True
    assert o.feasible(topo, 99, 100 * b, algo)[0] is False   # 1/x slightly below 1/b


@pytest.mark.parametrize("b", [1, 2, 5])
def test_paper_example_variants(b):
    g = _gold("paper_worked_example.json")
    ring = w.paper_example_ring_unwound(b)
    want = Fraction(*g["ring_unwound_ratio_times_b"]["value"]) / b      # 4/b, "4x worse"
    assert o.brute_inv_xstar(ring) == want
    assert o.optimality_binary_search(ring) == want
    split = w.paper_example_split(b)
    want = Fraction(*g["after_edge_splitting_ratio_times_b"]["value"]) / b
    assert o.brute_inv_xstar(split) == want
    assert o.optimality_binary_search(split) == want


# ---------------------------------------------------------------- closed forms on the symmetric configs

def _closed_form(cfg, U, k):
    if cfg == 1:
        return min(16 * k, k + 12 * U, 8 * k + 8 * U)
    if cfg == 3:
        return min(128 * k, k + 26 * U, 8 * k + 16 * U)
    if cfg == 4:
        return min(512 * k, k + 36 * U, 8 * k + 32 * U, 32 * k + 256 * U)
    raise ValueError


def test_closed_form_file_matches_test_formulas():
    g = _gold("config_closed_forms.json")
    assert g["config1"]["F"] == "min(16k, k+12U, 8k+8U)"
    assert g["config3"]["F"] == "min(128k, k+26U, 8k+16U)"
    assert g["config4"]["F"] == "min(512k, k+36U, 8k+32U, 32k+256U)"


@pytest.mark.parametrize("cfg,cands", [
    (1, [(1, 4), (4, 4), (5, 4), (6, 4), (3, 1), (1, 1)]),
    (3, [(1, 8), (44, 8), (59, 8), (60, 8), (61, 8), (7, 1), (8, 1)]),
    (4, [(1, 4), (6, 4), (7, 4), (8, 4), (55, 4), (62, 4), (63, 4), (64, 4)]),
])
def test_config_closed_form_flows(cfg, cands):
    topo = w.config_topology(cfg)
    N = topo.n_compute
    for U, k in cands:
        ok, flows = o.feasible(topo, U, k, threads=4)
        want = _closed_form(cfg, U, k)
        assert (flows == want).all(), (cfg, U, k, want, flows[:4])
        assert ok == (want >= N * k)
    # a few sinks with the second algorithm
    for U, k in cands[:3]:
        for v in (0, N // 2, N - 1):
            assert o.aux_maxflow(topo, v, U, k, "edmonds_karp") == _closed_form(cfg, U, k)


@pytest.mark.parametrize("cfg", [1, 3, 4])
def test_config_closed_form_optimum(cfg):
    g = _gold("config_closed_forms.json")[f"config{cfg}"]
    topo = w.config_topology(cfg)
    log = []
    x = o.optimality_binary_search(topo, threads=4, log=log)
    assert x == Fraction(*g["inv_xstar"])
    U, k = o.smallest_U_k(x, topo.bandwidth)
    assert (U, k) == (Fraction(*g["U_k"][0]), g["U_k"][1])
    # iteration ceiling of Appendix F: at most ceil(log2(N * B^2)) rounds
    B = o.min_compute_in_bandwidth(topo)
    assert log[-1][1] <= ceil(log2(topo.n_compute * B * B))
    # every verdict in the log is monotone in A/D (Theorem 1)
    tested = sorted((Fraction(a, d), ok) for a, d, ok in log[:-1])
    flags = [ok for _, ok in tested]
    assert flags == sorted(flags)


def test_config1_configured_batch_is_infeasible():
    topo = w.config_topology(1)
    ok, flows = o.feasible(topo, 1, 4)
    assert not ok and (flows == 16).all()          # min(64, 4+12, 32+8) = 16 < 64


# ---------------------------------------------------------------- textbook special cases of the bound (star)

@pytest.mark.parametrize("n,c", [(3, 1), (5, 2), (6, 7)])
def test_textbook_shapes(n, c):
    assert o.optimality_binary_search(w.complete_digraph(n, c)) == Fraction(1, c)
    assert o.optimality_binary_search(w.directed_ring(n, c)) == Fraction(n - 1, c)
    if n >= 3:
        assert o.optimality_binary_search(w.bidirectional_ring(n, c)) == Fraction(n - 1, 2 * c)
    assert o.optimality_binary_search(w.star_switch(n, c)) == Fraction(n - 1, c)


def test_generic_maxflow_textbook_network():
    # classic 6-vertex example with max-flow 23 (CLRS figure 26.1 capacities)
    arcs = [(0, 1, 16), (0, 2, 13), (1, 3, 12), (2, 1, 4), (2, 4, 14), (3, 2, 9), (3, 5, 20), (4, 3, 7), (4, 5, 4)]
    t, h, c = zip(*arcs)
    for algo in ALGOS:
        assert o.maxflow(6, t, h, c, 0, 5, algo) == 23
    assert o.brute_min_cut(6, t, h, c, 0, 5) == 23
    # direction matters: nothing flows backwards
    assert o.maxflow(6, t, h, c, 5, 0) == 0


# ---------------------------------------------------------------- brute force on random tiny graphs

@pytest.mark.parametrize("seed", range(60))
def test_tiny_random_flow_equals_brute_min_cut(seed):
    topo = w.random_tiny(seed)
    rng = np.random.default_rng(1000 + seed)
    U, k = int(rng.integers(1, 5)), int(rng.integers(1, 12))
    n, tail, head, cap, s = o.aux_network(topo, U, k)
    for v in topo.compute_nodes:
        want = o.brute_min_cut(n, tail, head, cap, s, int(v))
        got_d, flow = o.maxflow(n, tail, head, cap, s, int(v), "dinic", return_arc_flow=True)
        got_e = o.maxflow(n, tail, head, cap, s, int(v), "edmonds_karp")
        assert got_d == want == got_e
        # capacity + conservation + value on the returned arc flows
        capa = np.asarray(cap, dtype=np.int64)
        assert (flow >= 0).all() and (flow <= capa).all()
        net = np.zeros(n, dtype=np.int64)
        np.add.at(net, head, flow); np.subtract.at(net, tail, flow)
        assert net[int(v)] == got_d and net[s] == -got_d
        mask = np.ones(n, bool); mask[[s, int(v)]] = False
        assert (net[mask] == 0).all()
        # bounds: k <= F <= min(N k, k + U B^-(v))
        Bv = o.in_bandwidths(topo)[int(v)]
        assert k <= got_d <= min(topo.n_compute * k, k + U * Bv)


@pytest.mark.parametrize("seed", range(80))
def test_tiny_random_search_equals_brute_bound(seed):
    topo = w.random_tiny(seed, strongly_connected=(seed % 4 != 3))
    try:
        want = o.brute_inv_xstar(topo)
    except o.Disconnected:
        with pytest.raises(o.Disconnected):
            o.optimality_binary_search(topo)
        return
    got = o.optimality_binary_search(topo, algo=ALGOS[seed % 2])
    assert got == want
    N, B = topo.n_compute, o.min_compute_in_bandwidth(topo)
    assert Fraction(N - 1, B) <= got <= N - 1 and got.denominator <= B    # Appendix E.1 range
    # Theorem 1 at and just below the optimum
    assert o.feasible(topo, got.numerator, got.denominator)[0]
    below = got - Fraction(1, 1000 * got.denominator)
    assert not o.feasible(topo, below.numerator, below.denominator)[0]


@pytest.mark.parametrize("seed", range(4))
def test_shrunken_config5_and_config2_like(seed):
    topo = shrunken_config5(seed)
    assert o.optimality_binary_search(topo) == o.brute_inv_xstar(topo)


@pytest.mark.parametrize("seed", range(40))
def test_theorem8_cut_form_switch_free(seed):
    topo = w.random_tiny(500 + seed, n_vertices=int(3 + seed % 5), switch_free=True, density=0.6)
    for k in (1, 2, 3, 5):
        assert o.brute_cut_condition(topo, k) == o.feasible(topo, 1, k)[0]


# ---------------------------------------------------------------- invariants (Theorem 1, Appendix E.1)

@pytest.mark.parametrize("cfg", [2, 3])
def test_monotone_and_scaling(cfg):
    topo = w.config_topology(cfg)
    k = 4
    prev = None
    for U in range(1, 40, 3):
        ok, flows = o.feasible(topo, U, k, threads=4)
        if prev is not None:
            assert (flows >= prev[1]).all() and ok >= prev[0]
        prev = (ok, flows)
        if U % 2:
            _, f3 = o.feasible(topo, 3 * U, 3 * k, threads=4)     # uniform scaling (Appendix E.1)
            assert (f3 == 3 * flows).all()


def test_proposition3_gcd_rule():
    assert o.smallest_U_k(Fraction(1, 3), [3, 30]) == (Fraction(1, 3), 1)
    assert o.smallest_U_k(Fraction(5, 4), [12, 8]) == (Fraction(5, 4), 1)
    assert o.smallest_U_k(Fraction(5, 6), [4, 10]) == (Fraction(5, 2), 3)
    assert o.smallest_U_k(Fraction(7, 5), [3, 4]) == (Fraction(7, 1), 5)
    # U*b_e integral, U/k = p/q, and no smaller k works
    for p, q, bw in [(5, 6, [4, 10]), (9, 8, [12, 20, 8]), (3, 7, [14, 21])]:
        U, k = o.smallest_U_k(Fraction(p, q), bw)
        assert U / k == Fraction(p, q) and all((U * b).denominator == 1 for b in bw)
        for k2 in range(1, k):
            U2 = Fraction(p, q) * k2
            assert not all((U2 * b).denominator == 1 for b in bw)


def test_fraction_gap_proposition2():
    # two different fractions with denominators <= X differ by at least 1/X^2
    X = 9
    fr = sorted({Fraction(p, q) for q in range(1, X + 1) for p in range(0, 3 * q + 1)})
    assert min(b - a for a, b in zip(fr, fr[1:])) >= Fraction(1, X * X)
    assert o.fraction_in_interval(Fraction(5, 4), Fraction(5, 4) + Fraction(1, 200), 12) == Fraction(5, 4)
    assert o.fraction_in_interval(Fraction(299, 80), Fraction(301, 80), 8) == Fraction(15, 4)


def test_threshold_search_recovers_every_bounded_fraction():
    # the search both optimisations run: for EVERY fraction p/q with q <= X inside the range, a step verdict with its
    # threshold there (closed on the feasible side, as Theorem 1's is) must give back exactly p/q, also when the threshold
    # sits on an end of the range, and within the iteration ceiling ceil(log2(width * X^2)) of Appendix F
    X = 7
    lo, hi = Fraction(1, 2), Fraction(5)
    fr = sorted({Fraction(p, q) for q in range(1, X + 1) for p in range(1, 5 * q + 1) if lo <= Fraction(p, q) <= hi})
    assert fr[0] == lo and fr[-1] == hi and len(fr) > 60
    for thr in fr:
        seen = []
        got, halvings = o.smallest_true_fraction(lambda z: z >= thr, lo, hi, X, lambda z, ok: seen.append((z, ok)))
        assert got == thr
        assert halvings == len(seen) and all(ok == (z >= thr) for z, ok in seen)
        assert halvings <= math.ceil(math.log2((hi - lo) * X * X)) + 1
    # a bracket that stops one halving too early still holds two candidates, which the last step refuses
    with pytest.raises(AssertionError):
        o.fraction_in_interval(Fraction(1, 7), Fraction(1, 6), X)              # 1/42 wide: not below 1/49


def test_planted_mistakes_are_caught():
    """Each plausible slip, planted in a copy of the oracle's network builder, changes a pinned value."""
    topo = w.paper_example_switch(1)

    def flow_with(build):
        n, t, h, c, s = build()
        return o.maxflow(n, t, h, c, s, 5)

    n, t, h, c, s = o.aux_network(topo, 1, 2)
    assert flow_with(lambda: (n, t, h, c, s)) == 12
    assert flow_with(lambda: (n, h, t, c, s)) != 12                       # transposed arcs
    c_no_sink = [0 if (tt == s and hh == 5) else cc for tt, hh, cc in zip(t, h, c)]
    assert flow_with(lambda: (n, t, h, c_no_sink, s)) != 12               # dropped s->sink arc
    c_unscaled = [cc if tt == s else 2 * cc for tt, cc in zip(t, c)]
    assert flow_with(lambda: (n, t, h, c_unscaled, s)) != 12              # wrong capacity scaling


# ---------------------------------------------------------------- fixed k (Section 5.5, Appendix E.4, Algorithm 3)

@pytest.mark.parametrize("b", [1, 2, 3, 7])
def test_fixed_k_on_the_paper_example(b):
    # the worked example needs k = 1 trees per node at U = 1/b (Section 5.2 "Determine k"), so fixing
    # k = 1 must give exactly that, and k = j must give j / b: U*/k cannot beat 1/x* = 1/b (Theorem 13's
    # left side is the optimum) and j/b is feasible because every floor(j/b * b_e) = j * b_e / b is exact
    topo = w.paper_example_switch(b)
    for k in (1, 2, 5):
        assert o.fixed_k_binary_search(topo, k) == Fraction(k, b)
    assert o.fixed_k_feasible(topo, Fraction(1, b), 1)[0]
    # just below 1/b the thin links floor to 0 and the boxes fall apart
    assert not o.fixed_k_feasible(topo, Fraction(1, b) - Fraction(1, 1000), 1)[0]


@pytest.mark.parametrize("seed", range(40))
def test_fixed_k_search_equals_enumeration(seed):
    # Algorithm 3 (bisection + the unique fraction with denominator <= max b) against trying every j / b_e
    topo = w.random_tiny(seed, max_cap=5)
    for k in (1, 2, 3):
        try:
            want = o.brute_fixed_k(topo, k, algo=ALGOS[seed % 2])
        except o.Disconnected:
            with pytest.raises(o.Disconnected):
                o.fixed_k_binary_search(topo, k)
            continue
        got = o.fixed_k_binary_search(topo, k, algo=ALGOS[(seed + 1) % 2])
        assert got == want, (seed, k)
        assert got.denominator <= int(o.links(topo)[2].max())


@pytest.mark.parametrize("seed", range(30))
def test_fixed_k_bounds_and_multiples_of_the_optimal_k(seed):
    topo = w.random_tiny(100 + seed, max_cap=6)
    try:
        inv = o.optimality_binary_search(topo)
    except o.Disconnected:
        return
    bw = o.links(topo)[2]
    U_opt, k_opt = o.smallest_U_k(inv, bw)
    for k in (1, 2, 3, 4):
        Us = o.fixed_k_binary_search(topo, k)
        # optimality bound (star) from below, Theorem 13 from above
        assert inv <= Us / k <= inv + Fraction(1, k * int(bw.min())), (seed, k)
    # with k a multiple of Proposition 3's k the optimum is reached exactly: U = j U_opt makes every
    # floor exact (U_opt b_e is an integer) and is feasible by Theorem 3
    for j in (1, 2):
        assert o.fixed_k_binary_search(topo, j * k_opt) == j * U_opt, seed


def test_fixed_k_verdict_is_monotone_and_floors_per_link():
    topo = w.config_topology(2)                          # has parallel arcs (links of capacity 2 emitted twice or more)
    N = topo.n_compute
    B = o.min_compute_in_bandwidth(topo)
    Us = [Fraction((N - 1) * 2, B) + Fraction(j, 7) for j in range(0, 60, 3)]
    verdicts = [o.fixed_k_feasible(topo, U, 2, threads=8)[0] for U in Us]
    assert verdicts == sorted(verdicts)                  # Theorem 12: feasible iff U >= U*
    # an integer multiplier floors nothing: same flows as the integer path
    comp = topo.compute_nodes
    a = o.aux_maxflow_batch(topo, comp, np.full(N, 3), np.full(N, 2))
    b = o.aux_maxflow_batch_floor(topo, comp, np.full(N, 9), np.full(N, 3), np.full(N, 2))
    assert (a == b).all()
    # two parallel arcs of bandwidth 1 are one link of bandwidth 2: at U = 1/2 it carries floor(1) = 1, not 0 + 0
    t2 = w.Topology("par", 2, np.array([0, 0, 1], dtype=np.int32), np.array([1, 1, 0], dtype=np.int32),
                    np.array([1, 1, 2], dtype=np.int32), np.array([1, 1], dtype=np.uint8))
    assert o.aux_maxflow_batch_floor(t2, [1], [1], [2], [1])[0] == 2      # k direct + 1 through the link
    assert o.fixed_k_binary_search(t2, 1) == Fraction(1, 2)


@pytest.mark.parametrize("n,c,k", [(4, 3, 1), (5, 2, 3), (6, 4, 2)])
def test_fixed_k_textbook_shapes(n, c, k):
    # complete digraph, every link c: a node's n-1 in-links carry floor(U c) each and must bring in (n-1) k
    # (cut around one node), and floor(U c) = k on every link suffices by symmetry: U* = k / c
    assert o.fixed_k_binary_search(w.complete_digraph(n, c), k) == Fraction(k, c)
    # directed ring, every link c: the link into v carries the other n-1 nodes' k units: U* = (n-1) k / c
    assert o.fixed_k_binary_search(w.directed_ring(n, c), k) == Fraction((n - 1) * k, c)


# ---------------------------------------------------------------- edge splitting (Appendix E.2, the maximum-split-off theorem)

def _scaled_eulerian(seed):
    """A small bidirectional (hence Eulerian) graph with switches, scaled by Proposition 3's (U, k) so
    that min_v F(s, v) >= N k holds with integer capacities U b_e -- the input of the edge-splitting stage."""
    rng = np.random.default_rng(4000 + seed)
    base = w.random_tiny(4000 + seed, n_vertices=int(rng.integers(4, 8)), max_cap=4, density=0.35)
    if base.is_compute.all():
        base.is_compute[int(rng.integers(0, base.n_vertices))] = 0
        if base.is_compute.sum() < 2:
            return None
    cap = {}
    for t, h, b in zip(base.tail.tolist(), base.head.tolist(), base.bandwidth.tolist()):
        if t != h and b > 0:
            key = (min(t, h), max(t, h))
            cap[key] = cap.get(key, 0) + int(b)
    tail = [a for a, b in cap] + [b for a, b in cap]
    head = [b for a, b in cap] + [a for a, b in cap]
    bw = list(cap.values()) * 2
    sym = w.Topology(f"euler{seed}", base.n_vertices, np.array(tail, dtype=np.int32), np.array(head, dtype=np.int32),
                     np.array(bw, dtype=np.int32), base.is_compute.copy())
    try:
        inv = o.optimality_binary_search(sym)
    except o.Disconnected:
        return None
    U, k = o.smallest_U_k(inv, sym.bandwidth)
    scaled = w.Topology(sym.name, sym.n_vertices, sym.tail, sym.head,
                        np.array([int(U * int(b)) for b in sym.bandwidth], dtype=np.int32), sym.is_compute)
    assert o.is_eulerian(scaled) and o.feasible(scaled, 1, k)[0]
    return scaled, k


@pytest.mark.parametrize("b", [1, 2])
def test_edge_splitting_of_the_paper_example(b):
    # Appendix E.2, the stages figure: in each box split off all 10b of (c_j, w_i), (w_i, c_{j+1}) to form a ring,
    # across boxes all b of (c_{1,j}, w_0), (w_0, c_{2,j}) and back; the result is the switch-free topology of
    # the figure, and the optimum 1/x* = 1/b is unchanged.  D = G({U b_e}) with U = 1/b, k = 1: capacities {10, 1}.
    D = w.paper_example_switch(1)
    k = 1
    for box in range(2):
        for j in range(4):
            u, t, sw = 4 * box + j, 4 * box + (j + 1) % 4, 8 + box
            assert o.split_gamma(D, k, u, sw, t) == 10
            D = o.split_off(D, u, sw, t, 10)
    for j in range(4):
        for u, t in ((j, 4 + j), (4 + j, j)):
            assert o.split_gamma(D, k, u, 10, t) == 1
            D = o.split_off(D, u, 10, t, 1)
    want = w.paper_example_split(1)
    assert o.link_capacities(D) == o.link_capacities(want)
    assert o.feasible(D, 1, k)[0] and o.optimality_binary_search(w.paper_example_split(b)) == Fraction(1, b)
    # capacity that leaves a box cannot be split onto an in-box pair: nothing can be taken
    assert o.split_gamma(w.paper_example_switch(1), 1, 0, 10, 1) == 0


@pytest.mark.parametrize("seed", range(40))
def test_split_gamma_formula_equals_its_definition(seed):
    made = _scaled_eulerian(seed)
    if made is None:
        return
    D, k = made
    cap = o.link_capacities(D)
    switches = [v for v in range(D.n_vertices) if not D.is_compute[v]]
    pairs = [(u, sw, t) for sw in switches for (u, x) in cap if x == sw for (y, t) in cap if y == sw]
    rng = np.random.default_rng(seed)
    for i in rng.permutation(len(pairs))[:6]:
        u, sw, t = pairs[int(i)]
        g_formula = o.split_gamma(D, k, u, sw, t, algo=ALGOS[seed % 2])
        assert g_formula == o.brute_split_gamma(D, k, u, sw, t, algo=ALGOS[(seed + 1) % 2]), (seed, u, sw, t)
        F1, F2 = o.split_flows(D, k, u, sw, t)
        assert (F1 >= D.n_compute * k).all() and (F2 >= D.n_compute * k).all()     # gamma >= 0 under the preconditions
        after = o.split_off(D, u, sw, t, g_formula)
        assert o.is_eulerian(after) and o.feasible(after, 1, k)[0]


def test_switch_removal_by_repeated_splitting_keeps_the_optimum():
    # Algorithm 2's loop with the oracle's gamma: every switch ends isolated and Theorem 1's condition still holds
    done = 0
    for seed in range(12):
        made = _scaled_eulerian(100 + seed)
        if made is None:
            continue
        D, k = made
        for sw in [v for v in range(D.n_vertices) if not D.is_compute[v]]:
            for (y, t) in [key for key in o.link_capacities(D) if key[0] == sw]:
                for (u, x) in [key for key in o.link_capacities(D) if key[1] == sw]:
                    cap = o.link_capacities(D)
                    if (sw, t) not in cap:
                        break
                    if (u, sw) not in cap:
                        continue
                    g = o.split_gamma(D, k, u, sw, t)
                    if g > 0:
                        D = o.split_off(D, u, sw, t, g)
                assert (sw, t) not in o.link_capacities(D)            # Appendix E.2, existence theorem: f can always be split off completely
        cap = o.link_capacities(D)
        assert all(D.is_compute[a] and D.is_compute[b] for a, b in cap)
        assert o.feasible(D, 1, k)[0]
        done += 1
    assert done >= 6


def _check_switch_removal(D, k, Dstar, table):
    cap0, cap1 = o.link_capacities(D), o.link_capacities(Dstar)
    assert all(D.is_compute[a] and D.is_compute[b] for a, b in cap1)          # every switch is isolated
    assert o.is_eulerian(Dstar) and o.feasible(Dstar, 1, k)[0]                  # Appendix E.2, existence theorem: the condition survives
    # the table accounts for exactly the capacity that was added between compute nodes (a link that touches a
    # switch may be created by one split and used up by a later one: the recovery of paths is recursive) ...
    for key in set(cap1) | set(table):
        if D.is_compute[key[0]] and D.is_compute[key[1]]:
            assert cap1.get(key, 0) == cap0.get(key, 0) + sum(table.get(key, {}).values()), key
    # ... and no switch relays more than entered it
    total_in = sum(c for (a, b), c in cap0.items() if not D.is_compute[b])
    for sw in [v for v in range(D.n_vertices) if not D.is_compute[v]]:
        relayed = sum(amount for routes in table.values() for s2, amount in routes.items() if s2 == sw)
        assert relayed <= total_in           # what a switch relays entered some switch (its own links, or links made for it)


def test_remove_switches_on_the_paper_example():
    for b, U, k in ((1, 1, 1), (2, 1, 2)):
        D = w.paper_example_switch(b)
        D = w.Topology(D.name, D.n_vertices, D.tail, D.head, (D.bandwidth * U).astype(np.int32), D.is_compute)
        Dstar, table = o.remove_switches(D, k)
        _check_switch_removal(D, k, Dstar, table)
        # in-box traffic stays on the box switch, cross-box traffic goes over the spine (the remark under the stages figure)
        for (u, t), routes in table.items():
            for sw in routes:
                assert sw == (8 + u // 4 if u // 4 == t // 4 else 10), (u, t, sw)
        # the optimum of the example survives the removal: 1/x* = 1/b, so with these capacities k / U trees fit
        assert o.optimality_binary_search(Dstar) == Fraction(U, k * b) * b


@pytest.mark.parametrize("seed", range(25))
def test_remove_switches_on_random_eulerian_graphs(seed):
    made = _scaled_eulerian(200 + seed)
    if made is None:
        return
    D, k = made
    Dstar, table = o.remove_switches(D, k, algo=ALGOS[seed % 2])
    _check_switch_removal(D, k, Dstar, table)
    # the optimum cannot improve, and D itself was at its optimum 1/x* = 1/k (scaled by Proposition 3)
    assert o.optimality_binary_search(Dstar) == o.optimality_binary_search(D) == Fraction(1, k)


# ---------------------------------------------------------------- non-uniform source capacities (Section 5.7)

def _line(bws, n):
    """compute nodes 0 .. n-1 on a directed line i -> i+1 with bandwidths bws"""
    return w.Topology("line", n, np.arange(n - 1, dtype=np.int32), np.arange(1, n, dtype=np.int32),
                      np.asarray(bws, dtype=np.int32), np.ones(n, dtype=np.uint8))


def test_weighted_closed_forms_on_lines():
    # a -> b: what reaches b is its own m_b k plus whatever of a's m_a k the link carries
    for ma, mb, B, U, k in ((3, 1, 2, 1, 1), (3, 1, 2, 2, 1), (0, 2, 5, 1, 3), (4, 0, 1, 3, 2), (2, 5, 7, 1, 4)):
        t = _line([B], 2)
        f = o.weighted_aux_maxflow_batch(t, [0, 1], [U, U], [k, k], [ma, mb])
        assert f.tolist() == [ma * k, mb * k + min(ma * k, U * B)]
    # a -> b -> c, three different weights: a permuted or dropped weight changes the value
    for (ma, mb, mc), (B1, B2), U, k in (((5, 1, 2), (3, 4), 1, 1), ((1, 7, 0), (9, 2), 2, 3), ((2, 3, 4), (1, 100), 3, 2)):
        t = _line([B1, B2], 3)
        f = o.weighted_aux_maxflow_batch(t, [2, 1], [U, U], [k, k], [ma, mb, mc])
        assert f.tolist() == [mc * k + min(U * B2, mb * k + min(U * B1, ma * k)), mb * k + min(U * B1, ma * k)]


def test_weighted_verdict_threshold_is_k_times_the_weight_sum():
    # two nodes joined both ways with bandwidth B, weights (3, 1): b must receive 3k over the link, so the
    # candidate is feasible iff U B >= 3 k -- although F(s, b) reaches N k = 2 k much earlier
    t = w.Topology("pair", 2, np.array([0, 1], np.int32), np.array([1, 0], np.int32), np.array([2, 2], np.int32), np.ones(2, np.uint8))
    for U, k, want in ((1, 1, False), (3, 2, True), (2, 2, False), (3, 3, False), (9, 6, True)):
        ok, flows = o.weighted_feasible(t, U, k, [3, 1])
        assert ok is want and flows.tolist() == [3 * k + min(k, 2 * U), k + min(3 * k, 2 * U)]
    assert o.weighted_feasible(t, 1, 2, [1, 1])[0] == o.feasible(t, 1, 2)[0]


@pytest.mark.parametrize("seed", range(30))
def test_weighted_flows_equal_brute_min_cut_and_reduce_to_the_uniform_case(seed):
    topo = w.random_tiny(2000 + seed)
    rng = np.random.default_rng(3000 + seed)
    U, k = int(rng.integers(1, 5)), int(rng.integers(1, 8))
    wts = rng.integers(0, 4, topo.n_vertices)
    comp = [int(v) for v in topo.compute_nodes]
    n, tail, head, cap, s = o.weighted_aux_network(topo, U, k, wts)
    got = o.weighted_aux_maxflow_batch(topo, comp, [U] * len(comp), [k] * len(comp), wts, algo=ALGOS[seed % 2])
    for i, v in enumerate(comp):
        assert got[i] == o.brute_min_cut(n, tail, head, cap, s, v)
    # weight 1 everywhere is the network of Section 5.2
    ones = np.ones(topo.n_vertices, dtype=np.int64)
    assert (o.weighted_aux_maxflow_batch(topo, comp, [U] * len(comp), [k] * len(comp), ones) ==
            o.aux_maxflow_batch(topo, comp, [U] * len(comp), [k] * len(comp))).all()
    assert o.weighted_feasible(topo, U, k, ones)[0] == o.feasible(topo, U, k)[0]
    # a common factor can sit in the weights or in k; scaling everything scales the flows
    a = o.weighted_aux_maxflow_batch(topo, comp, [U] * len(comp), [3 * k] * len(comp), wts)
    b = o.weighted_aux_maxflow_batch(topo, comp, [U] * len(comp), [k] * len(comp), 3 * wts)
    c = o.weighted_aux_maxflow_batch(topo, comp, [3 * U] * len(comp), [3 * k] * len(comp), wts)
    assert (a == b).all() and (c == 3 * got).all()


@pytest.mark.parametrize("seed", range(20))
def test_a_weight_is_that_many_unit_nodes_behind_wide_links(seed):
    # a compute node of weight m >= 1 sends what it and m - 1 extra unit nodes, each joined to it by a link that
    # carries its k units, would send: the flows into the original nodes agree with the uniform network's
    topo = w.random_tiny(2500 + seed)
    rng = np.random.default_rng(3500 + seed)
    U, k = int(rng.integers(1, 4)), int(rng.integers(1, 6))
    wts = np.where(np.asarray(topo.is_compute) != 0, rng.integers(1, 4, topo.n_vertices), 0)
    tail, head, bw, isc = topo.tail.tolist(), topo.head.tolist(), topo.bandwidth.tolist(), list(np.asarray(topo.is_compute).tolist())
    nv = topo.n_vertices
    for c in [int(v) for v in topo.compute_nodes]:
        for _ in range(int(wts[c]) - 1):
            tail.append(nv); head.append(c); bw.append(k); isc.append(1); nv += 1      # U * k >= k
    big = w.Topology("expanded", nv, np.asarray(tail, np.int32), np.asarray(head, np.int32), np.asarray(bw, np.int32), np.asarray(isc, np.uint8))
    comp = [int(v) for v in topo.compute_nodes]
    want = o.aux_maxflow_batch(big, comp, [U] * len(comp), [k] * len(comp))
    got = o.weighted_aux_maxflow_batch(topo, comp, [U] * len(comp), [k] * len(comp), wts)
    assert (got == want).all()


def test_weighted_floor_capacities():
    t = _line([3, 5], 3)
    # multiplier 5/2: floor(7.5) = 7 and floor(12.5) = 12
    f = o.weighted_aux_maxflow_batch(t, [2], [5], [1], [20, 1, 2], U_den=[2])
    assert f.tolist() == [2 + min(12, 1 + min(7, 20))]
    with pytest.raises(ValueError):
        o.weighted_aux_network(t, 1, 1, [1, -1, 1])


# ---------------------------------------------------------------- spanning tree construction (Appendix E.3)

def _check_trees(n, links, k, trees):
    """what the construction promises: every tree spans all vertices from its root, the multiplicities of a root
    add up to k, and no link carries more trees than its capacity"""
    use, per_root = {}, {}
    for root, m, edges in trees:
        assert m >= 1 and len(edges) == n - 1
        seen = {root}
        for x, y in edges:
            assert x in seen and y not in seen
            seen.add(y)
            use[(x, y)] = use.get((x, y), 0) + m
        assert seen == set(range(n))
        per_root[root] = per_root.get(root, 0) + m
    assert per_root == {u: k for u in range(n)}
    assert all(c <= links[e] for e, c in use.items())
    return use


@pytest.mark.parametrize("b", [1, 2, 3])
def test_trees_on_the_paper_example(b):
    # the switch-free form of the worked example (Appendix E.2 figure): optimum 1/x* = 1/b, so U = 1, k = b
    topo = w.paper_example_split(b)
    links = o.link_capacities(topo)
    assert o.feasible(topo, 1, b)[0]
    trees = o.construct_trees(8, links, b)
    use = _check_trees(8, links, b, trees)
    # the inter-box links are the bottleneck cut: 4 b leave each box and 4 roots x b trees have to cross it
    assert all(use.get((j, 4 + j), 0) == b and use.get((4 + j, j), 0) == b for j in range(4))


def test_trees_on_complete_digraphs_use_every_link():
    # K_n with capacity c on every ordered pair: c(S, V - S) = |S| (n - |S|) c >= |S| k exactly when c >= k, and
    # with c = k the n k trees need n k (n - 1) link slots, which is all there are
    for n, k in ((2, 1), (2, 5), (3, 2), (4, 3), (5, 1)):
        links = {(a, b): k for a in range(n) for b in range(n) if a != b}
        trees = o.construct_trees(n, links, k)
        use = _check_trees(n, links, k, trees)
        assert use == links
    # two nodes: the only tree of root a is the link (a, b), k times
    assert sorted(o.construct_trees(2, {(0, 1): 4, (1, 0): 4}, 4)) == [(0, 4, [(0, 1)]), (1, 4, [(1, 0)])]
    # capacity short of k on one link: the packing condition fails and the construction says so
    with pytest.raises(AssertionError):
        o.construct_trees(3, {(0, 1): 1, (1, 0): 2, (1, 2): 2, (2, 1): 2, (0, 2): 2, (2, 0): 2}, 2)


@pytest.mark.parametrize("n,k,seed", [(5, 1, 0), (7, 2, 1), (9, 2, 2), (12, 3, 3)])
def test_trees_on_superposed_random_out_trees_use_every_unit(n, k, seed):
    # a digraph laid down as k random spanning out-trees per root, one unit per tree edge: a packing exists, and any
    # packing of n k spanning out-trees uses n k (n - 1) units, which is all there are.  Capacities differ from
    # link to link, so partial mu (copies) occur all the time.
    links = w.superposed_out_trees(n, k, seed)
    assert sum(links.values()) == n * k * (n - 1)
    trees = o.construct_trees(n, links, k, algo=ALGOS[seed % 2])
    use = _check_trees(n, links, k, trees)
    assert use == links
    assert len(trees) > n or k == 1 or n <= 2       # some root needed more than one kind of tree


@pytest.mark.parametrize("seed", range(12))
def test_mu_by_max_flow_equals_its_definition(seed):
    # random small compute-only digraphs that satisfy the packing condition (a complete digraph of capacity k
    # plus random extra capacity); every mu the construction computes is checked against the cut formula
    rng = np.random.default_rng(6000 + seed)
    n = int(rng.integers(3, 6)); k = int(rng.integers(1, 4))
    links = {(a, b): k + int(rng.integers(0, 3)) for a in range(n) for b in range(n) if a != b}
    count = [0]

    def observe(g, sets, demand, i, x, y, mu):
        assert mu == o.brute_tree_mu(n, g, sets, demand, i, x, y)
        assert 0 <= mu <= min(g[(x, y)], demand[i])
        count[0] += 1

    trees = o.construct_trees(n, links, k, algo=ALGOS[seed % 2], observe=observe)
    _check_trees(n, links, k, trees)
    assert count[0] >= n * (n - 1)


@pytest.mark.parametrize("seed", range(16))
def test_trees_after_switch_removal(seed):
    # the whole back end on a small random switch topology: optimum, scaling, switch removal, trees
    inv = None
    for redraw in range(20):                               # a disconnected draw is drawn again, never skipped
        base = w.random_tiny(7000 + seed + 100 * redraw, n_vertices=int(5 + seed % 3))
        cap = {}
        for t, h, b in zip(base.tail.tolist(), base.head.tolist(), base.bandwidth.tolist()):
            if t != h and b > 0:
                key = (min(t, h), max(t, h)); cap[key] = cap.get(key, 0) + int(b)
        tail = [a for a, b in cap] + [b for a, b in cap]; head = [b for a, b in cap] + [a for a, b in cap]
        sym = w.Topology(f"euler{seed}", base.n_vertices, np.array(tail, dtype=np.int32), np.array(head, dtype=np.int32),
                         np.array(list(cap.values()) * 2, dtype=np.int32), base.is_compute.copy())
        try:
            inv = o.optimality_binary_search(sym)
            break
        except o.Disconnected:
            continue
    assert inv is not None
    Uq, k = o.smallest_U_k(inv, sym.bandwidth)
    U, kk = Uq.numerator, k * Uq.denominator
    D = w.Topology(sym.name, sym.n_vertices, sym.tail, sym.head, (sym.bandwidth.astype(np.int64) * U).astype(np.int32), sym.is_compute)
    Dstar, _ = o.remove_switches(D, kk)
    comp = [int(v) for v in sym.compute_nodes]
    idx = {v: i for i, v in enumerate(comp)}
    links = {(idx[a], idx[b]): c for (a, b), c in o.link_capacities(Dstar).items()}
    trees = o.construct_trees(len(comp), links, kk)
    _check_trees(len(comp), links, kk, trees)


@pytest.mark.parametrize("seed", range(10))
def test_mu_of_an_edge_never_rises_while_its_root_set_grows(seed):
    # what lets a construction skip an edge once it had mu = 0: growing R admits more cuts, used capacity lowers
    # them, copies raise p(S), m(R) only shrinks
    rng = np.random.default_rng(8000 + seed)
    for _ in range(200):                                   # draw again until the packing condition holds
        n = int(rng.integers(3, 7)); k = int(rng.integers(1, 5))
        # a complete digraph of capacity >= k satisfies the packing condition; odd seeds thin it out and may not
        links = {(a, b): k + int(rng.integers(0, 3)) for a in range(n) for b in range(n) if a != b and (seed % 2 == 0 or rng.random() < 0.85)}
        for a in range(n):                                 # keep a ring so that the digraph stays connected
            links.setdefault((a, (a + 1) % n), k)
        keys = sorted(links)
        topo = w.Topology("draw", n, np.array([a for a, _ in keys], np.int32), np.array([b for _, b in keys], np.int32),
                          np.array([links[e] for e in keys], np.int32), np.ones(n, np.uint8))
        if o.feasible(topo, 1, k)[0]:                      # min over v of F(s, v) >= N k: trees exist (Theorem 3)
            break
    else:
        raise AssertionError("no draw satisfied the packing condition")
    last = {}

    def observe(g, sets, demand, i, x, y, mu):
        key = (i, x, y)
        if key in last:
            assert mu <= last[key], key
        last[key] = mu

    trees = o.construct_trees(n, links, k, observe=observe)
    assert len(last) >= n * (n - 1) // 2
    _check_trees(n, links, k, trees)


# ------------------------------------------------------------------ two facts the device path leans on, shown on the oracle

@pytest.mark.parametrize("seed", range(6))
def test_mu_is_what_a_small_supply_at_x_adds_to_the_other_demands(seed):
    # mu = min{g, m(R), F(x, y; D-bar) - sum of the other demands}.  A maximum flow can be reached from any feasible
    # flow, and only min{g, m(R)} more units matter, so mu is also what a supply of min{g(x, y), m(R)} at x -- an
    # ordinary vertex, nothing saturated -- adds to the flow that delivers the other root-sets' demands to y; and
    # those demands alone always arrive in full.  (The HIP path evaluates mu in these two parts.)
    n, k = (6, 2) if seed % 2 else (5, 3)
    links = w.superposed_out_trees(n, k, 40 + seed)
    count = [0]

    def observe(g, sets, demand, i, x, y, mu):
        others = [l for l in range(len(sets)) if l != i]
        inf = sum(g.values()) + sum(demand) + 1
        sigma = n + len(others)                       # a source of its own: demands into the root-sets' vertices, the rest into x
        arcs = [(a, b, c) for (a, b), c in sorted(g.items()) if c > 0]
        for j, l in enumerate(others):
            arcs.append((sigma, n + j, int(demand[l])))
            arcs += [(n + j, r, inf) for r in sorted(sets[l])]
        def flow(extra):
            a = arcs + extra
            return o.maxflow(sigma + 1, [t for t, _, _ in a], [h for _, h, _ in a], [c for _, _, c in a], sigma, y, ALGOS[seed % 2])
        total = sum(int(demand[l]) for l in others)
        assert flow([]) == total
        supply = min(int(g[(x, y)]), int(demand[i]))
        assert flow([(sigma, x, supply)]) - total == mu
        count[0] += 1

    o.construct_trees(n, links, k, observe=observe)
    assert count[0] >= n * (n - 1)


def test_one_more_sink_never_lowers_a_split_flow():
    # the 2N max-flows of a pair (maximum-split-off theorem, Appendix E.2) differ in one sink, the compute node v (its unbounded arc into w or t makes it
    # one).  Without that arc the flow cannot be larger: what the problem without v reaches, every problem with v
    # reaches too.  (The HIP path answers from the problem without v where that already settles gamma.)
    checked = 0
    for seed in range(12):
        base = w.random_tiny(6000 + seed, n_vertices=6 + seed % 3, max_cap=5, density=0.4)
        if base.is_compute.all():
            continue
        cap = {}
        for t, h, b in zip(base.tail.tolist(), base.head.tolist(), base.bandwidth.tolist()):
            if t != h and b > 0:
                key = (min(t, h), max(t, h)); cap[key] = cap.get(key, 0) + int(b)
        tail = [a for a, b in cap] + [b for a, b in cap]; head = [b for a, b in cap] + [a for a, b in cap]
        sym = w.Topology(f"euler{seed}", base.n_vertices, np.array(tail, dtype=np.int32), np.array(head, dtype=np.int32),
                         np.array(list(cap.values()) * 2, dtype=np.int32), base.is_compute.copy())
        k = 2
        links = o.link_capacities(sym)
        comp = [v for v in range(sym.n_vertices) if sym.is_compute[v]]
        s = sym.n_vertices
        inf = o.unbounded(sym, k)
        common = [(a, b, c) for (a, b), c in sorted(links.items())] + [(s, c, k) for c in comp]
        def flow(extra, src, dst):
            a = common + [(x, y, inf) for x, y in extra if x != y]
            return min(inf, o.maxflow(s + 1, [t for t, _, _ in a], [h for _, h, _ in a], [c for _, _, c in a], src, dst))
        for sw in (v for v in range(sym.n_vertices) if not sym.is_compute[v]):
            ins = sorted(a for (a, b) in links if b == sw); outs = sorted(b for (a, b) in links if a == sw)
            for u in ins[:2]:
                for t in outs[:2]:
                    F1, F2 = o.split_flows(sym, k, u, sw, t)
                    without1 = flow([(u, s), (u, t)], u, sw)
                    without2 = flow([(sw, s), (u, t)], sw, t)
                    assert (F1 >= without1).all() and (F2 >= without2).all(), (seed, u, sw, t)
                    checked += 1
    assert checked >= 20


# ------------------------------------------------------------------ the rail fabric (back-end timing workload)

def test_rail_fabric_is_eulerian_and_has_the_box_cut_optimum():
    # every link is bidirectional, so the digraph is Eulerian; the binding cut is the one around a box: N - 8 compute nodes
    # outside, per_box * nic_cap coming in.  Tiny instances against brute force over all cuts, larger ones against the search.
    for boxes, per_box, nv, nic in ((3, 3, 6, 1), (4, 2, 5, 2), (2, 4, 9, 1)):
        t = w.rail_fabric(boxes, per_box, nv, nic)
        assert t.n_vertices == boxes * per_box + boxes + per_box and o.is_eulerian(t)
        want = Fraction(boxes * per_box - per_box, per_box * nic)
        assert o.brute_inv_xstar(t) == want == o.optimality_binary_search(t)
    t = w.rail_fabric(16, 8)
    assert o.is_eulerian(t) and o.optimality_binary_search(t, threads=8) == Fraction(120, 16)
    big = w.eulerian_fabric_1024()
    assert big.n_compute == 1024 and big.n_vertices == 1160 and o.is_eulerian(big) and o.min_compute_in_bandwidth(big) == 26
