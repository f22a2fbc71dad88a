"""GPU parity tests: the HIP library, called through its C ABI, against the CPU oracle on the
same seeded inputs.  All quantities are integers, so every comparison is bit-exact."""
from fractions import Fraction

import numpy as np
import pytest

import oracle as o
import workloads as w
from workloads.problems import config_candidates

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

if not torch.cuda.is_available():          # selected explicitly on a machine without a GPU
    pytest.skip("needs a GPU", allow_module_level=True)

import paper_2402_06787_amd as fc   # noqa: E402

DEV = torch.device("cuda:0")
_OPTIMA = {}


def _upload(topo):
    return fc.fc_graph_upload(topo.n_vertices, topo.tail, topo.head, topo.bandwidth, topo.is_compute)


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def _gpu_flows(g, sink, U, k, options=None, want_stats=False):
    flows, stats = fc.fc_maxflow_batch(g, _dev(sink), _dev(U), _dev(k), options=options, want_stats=want_stats)
    torch.cuda.synchronize()
    return flows.cpu().numpy().astype(np.int64), stats


def _golden(name):
    import json, os
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)) as f:
        return json.load(f)


def _optimum(cfg, topo):
    if cfg not in _OPTIMA:
        x = o.optimality_binary_search(topo, threads=16)
        _OPTIMA[cfg] = (x.numerator, x.denominator)
    return _OPTIMA[cfg]


# ------------------------------------------------------------------ the paper's worked example

def test_library_call_as_the_first_device_use_of_a_fresh_process():
    # A process in which this package is the first thing to touch the GPU (torch imported, nothing allocated): the binding
    # brings torch's side up before it maps the library, or the library's own HIP runtime finds no device.
    import subprocess, sys, os
    code = ("import workloads as w, paper_2402_06787_amd as fc\n"
            "t = w.config_topology(1)\n"
            "g = fc.fc_graph_upload(t.n_vertices, t.tail, t.head, t.bandwidth, t.is_compute)\n"
            "print(fc.fc_opt_throughput_search(g, 16)['inv_xstar'])\n")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, "-c", code], cwd=root, capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr[-2000:]
    assert out.stdout.strip().splitlines()[-1] == "5/4"


def test_paper_example_on_gpu():
    topo = w.paper_example_switch(1)
    with _upload(topo) as g:
        sink = np.array([5, 5, 5, 0, 7], np.int32)
        U = np.array([1, 1, 1, 1, 1], np.int32)
        k = np.array([1, 2, 3, 1, 2], np.int32)
        got, _ = _gpu_flows(g, sink, U, k)
        assert got.tolist() == [8, 12, 14, 8, 12]          # 8x; 4x+4b; x+11b (Section 5.2)
        res = fc.fc_opt_throughput_search(g, 4)
        assert res["inv_xstar"] == 1 and res["U"] == 1 and res["k"] == 1


# ------------------------------------------------------------------ the five configs, full problem lists

@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_config_flows_match_oracle(cfg):
    topo = w.config_topology(cfg)
    inv = _optimum(cfg, topo) if cfg in (2, 5) else None
    pl = w.config_problems(cfg, topo, inv, extra_parity=True)
    want = o.aux_maxflow_batch(topo, pl.sink, pl.edge_mult, pl.src_cap, threads=16)
    with _upload(topo) as g:
        got, stats = _gpu_flows(g, pl.sink, pl.edge_mult, pl.src_cap, want_stats=True)
        assert got.shape == want.shape
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, (cfg, bad[:8], got[bad[:8]], want[bad[:8]])
        assert stats["not_converged"] == 0 and stats["pushes"] > 0 and stats["arc_scans"] >= stats["pushes"]
        # bounds that hold for any correct value: k <= F <= min(N k, k + U B^-(v))
        Bin = np.asarray(o.in_bandwidths(topo), dtype=np.int64)
        k64 = pl.src_cap.astype(np.int64); U64 = pl.edge_mult.astype(np.int64)
        assert (got >= k64).all() and (got <= np.minimum(topo.n_compute * k64, k64 + U64 * Bin[pl.sink])).all()


@pytest.mark.parametrize("cfg", [1, 3, 4])
def test_config_closed_forms_on_gpu(cfg):
    topo = w.config_topology(cfg)
    formula = {1: lambda U, k: min(16 * k, k + 12 * U, 8 * k + 8 * U),
               3: lambda U, k: min(128 * k, k + 26 * U, 8 * k + 16 * U),
               4: lambda U, k: min(512 * k, k + 36 * U, 8 * k + 32 * U, 32 * k + 256 * U)}[cfg]
    cand = [(1, 4), (5, 4), (44, 8), (60, 8), (63, 4), (7, 1), (1000, 3), (3, 700)]
    pl = w.all_sinks(topo, [c[0] for c in cand], [c[1] for c in cand])
    with _upload(topo) as g:
        got, _ = _gpu_flows(g, pl.sink, pl.edge_mult, pl.src_cap)
    got = got.reshape(len(cand), topo.n_compute)
    for i, (U, k) in enumerate(cand):
        assert (got[i] == formula(U, k)).all(), (cfg, U, k)


# ------------------------------------------------------------------ random small graphs, every vertex as sink

@pytest.mark.parametrize("block", range(4))
def test_tiny_random_graphs_match_oracle(block):
    for seed in range(block * 25, block * 25 + 25):
        topo = w.random_tiny(seed, n_vertices=None if seed % 3 else 12, strongly_connected=(seed % 4 != 3))
        rng = np.random.default_rng(77 + seed)
        P = 64
        sink = rng.integers(0, topo.n_vertices, P).astype(np.int32)           # switches too
        U = rng.integers(1, 9, P).astype(np.int32)
        k = rng.integers(1, 30, P).astype(np.int32)
        k[::7] = rng.integers(20000, 3000000, k[::7].shape)                    # N*k > 65535: 32-bit state
        U[::11] = rng.integers(1 << 20, 1 << 30, U[::11].shape)                # U*b beyond 32 bits: clamped
        want = o.aux_maxflow_batch(topo, sink, U, k, algo="edmonds_karp" if seed % 2 else "dinic")
        with _upload(topo) as g:
            got, _ = _gpu_flows(g, sink, U, k)
            assert (got == want).all(), (seed, np.flatnonzero(got != want)[:5])
            if seed % 5 == 0:
                got2, _ = _gpu_flows(g, sink, U, k, options={"force_wide": 1, "use_label_table": 2})
                assert (got2 == want).all(), seed


def _funnel(n_feed, arcs_out):
    """Compute nodes 0..n_feed-1 feed one switch u, which has the arcs `arcs_out` (bandwidths) to switches w_i, each of
    which feeds the compute node t: all excess meets at u and has to be split over several admissible arcs."""
    u, t = n_feed, n_feed + 1
    tail, head, bw = [], [], []
    for c in range(n_feed):
        tail.append(c); head.append(u); bw.append(8)
    for i, cap in enumerate(arcs_out):
        wi = n_feed + 2 + i
        tail.append(u); head.append(wi); bw.append(cap)
        tail.append(wi); head.append(t); bw.append(8)
    n = n_feed + 2 + len(arcs_out)
    is_c = np.zeros(n, np.uint8); is_c[:n_feed] = 1; is_c[t] = 1
    return w.Topology("funnel", n, np.asarray(tail, np.int32), np.asarray(head, np.int32), np.asarray(bw, np.int32), is_c)


def test_residuals_near_two_to_the_31_are_split_without_wrapping():
    # N * k just below 2^31 and capacities U * b of 2^28 .. N * k: the admissible residuals of one row add up to far more
    # than 32 bits hold, while every single one, the excess and the flow value fit
    topo = _funnel(7, [1, 1, 3, 3, 3, 3])
    N = topo.n_compute
    k = (1 << 28) - 1
    assert N * k < (1 << 31) <= N * (k + 1)
    cases = [(1 << 28, k), ((1 << 28) + 12345, k), (1 << 27, k), (3 << 26, k - 77), (1 << 28, k // 3), (1 << 30, k)]
    sink = np.array([8, 0, 3] * len(cases), np.int32)                         # t, and two of the feeders
    U = np.repeat([c[0] for c in cases], 3).astype(np.int32)
    kk = np.repeat([c[1] for c in cases], 3).astype(np.int32)
    want = o.aux_maxflow_batch(topo, sink, U, kk)
    assert want.max() > (1 << 30)
    with _upload(topo) as g:
        for opts in [None, dict(lanes_per_vertex=4), dict(lanes_per_vertex=64), dict(lanes_per_vertex=16, use_label_table=2),
                     dict(lanes_per_vertex=32, threads_per_problem=128)]:
            got, _ = _gpu_flows(g, sink, U, kk, options=opts)
            assert (got == want).all(), (opts, got.tolist(), want.tolist())
    # random small graphs in the same range
    for seed in range(40):
        topo = w.random_tiny(500 + seed, n_vertices=10 + seed % 5, strongly_connected=True)
        rng = np.random.default_rng(900 + seed)
        N = topo.n_compute
        P = 48
        sink = rng.integers(0, topo.n_vertices, P).astype(np.int32)
        kk = (((1 << 31) - 1) // N - rng.integers(0, 1000, P)).astype(np.int32)
        U = rng.integers(1 << 24, 1 << 29, P).astype(np.int32)
        want = o.aux_maxflow_batch(topo, sink, U, kk)
        with _upload(topo) as g:
            for opts in [dict(lanes_per_vertex=4), dict(lanes_per_vertex=64)]:
                got, _ = _gpu_flows(g, sink, U, kk, options=opts)
                assert (got == want).all(), (seed, opts, np.flatnonzero(got != want)[:5])


# ------------------------------------------------------------------ every launch shape gives the same values

def test_option_matrix_same_values():
    topo = w.config_topology(5)
    inv = _optimum(5, topo)
    pl = w.config_problems(5, topo, inv)
    rng = np.random.default_rng(3)
    idx = np.sort(rng.choice(pl.n_problems, 96, replace=False))
    idx[:16] = np.flatnonzero(pl.sink == pl.sink[np.argmin(o.in_bandwidths(topo)[:1024])])[:16]  # the bottleneck sink
    sink, U, k = pl.sink[idx], pl.edge_mult[idx], pl.src_cap[idx]
    want = o.aux_maxflow_batch(topo, sink, U, k, threads=16)
    with _upload(topo) as g:
        for opts in [dict(threads_per_problem=64, lanes_per_vertex=4), dict(threads_per_problem=128, lanes_per_vertex=8),
                     dict(threads_per_problem=256, lanes_per_vertex=16), dict(threads_per_problem=512, lanes_per_vertex=32),
                     dict(threads_per_problem=1024, lanes_per_vertex=64), dict(use_gap=2), dict(use_label_table=2),
                     dict(force_wide=1), dict(global_relabel_steps=1), dict(global_relabel_steps=100000, global_relabel_permille=1000000),
                     dict(force_wide=1, use_gap=2, use_label_table=2, threads_per_problem=192, lanes_per_vertex=64),
                     dict(schedule=2), dict(tight_sink_percent=-1), dict(tight_sink_percent=100000),
                     dict(global_relabel_rises=1), dict(global_relabel_rises=3, use_gap=2), dict(tree_certificate=1),
                     dict(tree_certificate=1, force_wide=1)]:
            got, stats = _gpu_flows(g, sink, U, k, options=opts, want_stats=True)
            assert (got == want).all(), (opts, np.flatnonzero(got != want)[:5])
            assert stats["not_converged"] == 0


def test_every_register_budget_gives_the_same_values():
    # the solver exists in builds for 5, 6 and 7 wavefronts per SIMD; a launch gets the one for min(what the LDS of a CU
    # leaves room for, what the launch itself puts on a SIMD of the 256 CUs).  Reach each of them with both state widths
    # and with rational multipliers: 160 distinct problems, repeated to make the launch as large as the case needs.
    cases = [(5, 8, dict(threads_per_problem=256)), (5, 1, dict(threads_per_problem=320)), (5, 8, dict(threads_per_problem=384)),
             (5, 1, dict(threads_per_problem=512)),
             (4, 1, dict()), (4, 24, dict()), (4, 19, dict()), (4, 24, dict(force_wide=1, threads_per_problem=256)),
             (4, 24, dict(force_wide=1, threads_per_problem=128)),
             (3, 1, dict()), (3, 38, dict()), (3, 48, dict()), (3, 38, dict(force_wide=1, threads_per_problem=64)),
             (3, 48, dict(force_wide=1, threads_per_problem=64)), (3, 24, dict(force_wide=1, threads_per_problem=128)),
             (3, 2, dict(threads_per_problem=1024, lanes_per_vertex=4))]
    rng = np.random.default_rng(9)
    cache = {}
    for cfg, rep, opts in cases:
        if cfg not in cache:
            topo = w.config_topology(cfg)
            inv = Fraction(*_optimum(cfg, topo))
            P = 160
            sink = rng.choice(topo.compute_nodes, P).astype(np.int32)
            k = rng.integers(1, 6, P).astype(np.int32)
            den = rng.integers(1, 5, P).astype(np.int32)
            num = np.maximum(1, (inv * k.astype(object) * den.astype(object) * rng.choice([Fraction(1, 2), Fraction(9, 10), 1, Fraction(11, 10), 3], P))
                             .astype(object)).astype(np.int64).astype(np.int32)
            mt = _merged(topo)
            cache[cfg] = (topo, sink, num, den, k, o.aux_maxflow_batch(topo, sink, num, k, threads=16),
                          o.aux_maxflow_batch_floor(mt, sink, num, den, k, threads=16))
        topo, sink, num, den, k, want_int, want_floor = cache[cfg]
        tile = lambda a: np.tile(a, rep)
        with _upload(topo) as g:
            got, stats = _gpu_flows(g, tile(sink), tile(num), tile(k), options=opts, want_stats=True)
            assert (got == tile(want_int)).all() and stats["not_converged"] == 0, (cfg, rep, opts)
            got, _ = _gpu_flows_floor(g, tile(sink), tile(num), tile(den), tile(k), options=opts)
            assert (got == tile(want_floor)).all(), (cfg, rep, opts)


# ------------------------------------------------------------------ the first-arc tree certificate and the launch order

@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_tree_certificate_gives_the_same_flows(cfg):
    topo = w.config_topology(cfg)
    inv = _optimum(cfg, topo) if cfg in (2, 5) else None
    pl = w.config_problems(cfg, topo, inv, extra_parity=True)
    want = o.aux_maxflow_batch(topo, pl.sink, pl.edge_mult, pl.src_cap, threads=16)
    with _upload(topo) as g:
        got, stats = _gpu_flows(g, pl.sink, pl.edge_mult, pl.src_cap, options={"tree_certificate": 1}, want_stats=True)
        plain, stats0 = _gpu_flows(g, pl.sink, pl.edge_mult, pl.src_cap, want_stats=True)
        assert (got == want).all(), (cfg, np.flatnonzero(got != want)[:8])
        assert (plain == want).all()
        # a certified problem is not solved, so the counters can only shrink; every certified value is N * k
        assert stats["pushes"] <= stats0["pushes"] and stats["level_steps"] <= stats0["level_steps"]
        # very generous capacities: the tree carries everything for every sink
        big = np.full(pl.n_problems, 1 << 20, dtype=np.int32)
        got2, stats2 = _gpu_flows(g, pl.sink, big, pl.src_cap, options={"tree_certificate": 1}, want_stats=True)
        assert (got2 == topo.n_compute * pl.src_cap.astype(np.int64)).all()
        assert stats2["pushes"] == 0 and stats2["level_steps"] == 0


def test_repeated_calls_reorder_but_do_not_change_values():
    # every call leaves per-sink cost hints with the graph and the next call starts the expensive sinks first
    topo = w.config_topology(5)
    inv = _optimum(5, topo)
    pl = w.config_problems(5, topo, inv)
    want = o.aux_maxflow_batch(topo, pl.sink, pl.edge_mult, pl.src_cap, threads=16)
    rng = np.random.default_rng(11)
    with _upload(topo) as g:
        for rep in range(3):
            perm = rng.permutation(pl.n_problems)
            got, _ = _gpu_flows(g, pl.sink[perm], pl.edge_mult[perm], pl.src_cap[perm])
            assert (got == want[perm]).all(), rep
        U, k = config_candidates(5, inv)
        first = fc.fc_feasible(g, _dev(U), _dev(k), want_flows=True)["flows"].cpu().numpy()
        again = fc.fc_feasible(g, _dev(U), _dev(k), want_flows=True, options={"schedule": 2})["flows"].cpu().numpy()
        assert (first == again).all() and (first.reshape(-1) == want).all()


# ------------------------------------------------------------------ edge cases of the boundary

def test_empty_invalid_and_workspace_errors():
    topo = w.config_topology(1)
    with _upload(topo) as g:
        empty = torch.empty(0, dtype=torch.int32, device=DEV)
        out, stats = fc.fc_maxflow_batch(g, empty, empty, empty, want_stats=True)
        assert out.numel() == 0 and stats["pushes"] == 0
        sink = np.array([0, 19, -1, 3, 4, 5, 18], np.int32)       # 19 and -1 are not vertices; 18 is a switch
        U = np.array([1, 1, 1, 0, 1, 1, 2], np.int32)
        k = np.array([4, 4, 4, 4, 0, 2 ** 28, 4], np.int32)       # 16 * 2^28 >= 2^31
        got, _ = _gpu_flows(g, sink, U, k)
        assert got[0] == 16 and got[1:6].tolist() == [fc.FC_FLOW_INVALID] * 5
        assert got[6] == o.aux_maxflow(topo, 18, 2, 4)
        d = _dev(sink)
        small = torch.empty(8, dtype=torch.uint8, device=DEV)
        with pytest.raises(fc.FcError) as ei:
            fc.fc_maxflow_batch(g, d, d, d, d_workspace=small)
        assert ei.value.code == fc.FC_EWORKSPACE
        with pytest.raises(fc.FcError) as ei:
            fc.fc_maxflow_batch(g, d, d, d, options={"threads_per_problem": 100})
        assert ei.value.code == fc.FC_EINVAL


def test_large_graph_limits():
    # largest shapes the 32-bit on-chip layout takes on a 160 KB LDS, and one beyond every layout
    rng = np.random.default_rng(11)
    n, deg = 3000, 6
    tail = np.repeat(np.arange(n), deg).astype(np.int32)
    head = ((tail + rng.integers(1, n, tail.shape)) % n).astype(np.int32)
    head[::deg] = (np.arange(n) + 1) % n                                      # ring keeps it connected
    bw = rng.integers(1, 50, tail.shape).astype(np.int32)
    isc = (np.arange(n) % 3 != 0).astype(np.uint8)
    topo = w.Topology("limit", n, tail, head, bw, isc)
    P = 48
    sink = rng.integers(0, n, P).astype(np.int32); U = rng.integers(1, 400, P).astype(np.int32)
    k = rng.integers(1, 40, P).astype(np.int32); k[::4] = 5000                # both layouts in one batch
    want = o.aux_maxflow_batch(topo, sink, U, k, threads=16)
    with _upload(topo) as g:
        got, stats = _gpu_flows(g, sink, U, k, want_stats=True)
        assert (got == want).all() and stats["not_converged"] == 0
    n2 = 40000
    t2 = np.arange(n2, dtype=np.int32); h2 = ((t2 + 1) % n2).astype(np.int32)
    with pytest.raises(fc.FcError) as ei:
        fc.fc_graph_upload(n2, t2, h2, np.ones(n2, np.int32), np.ones(n2, np.uint8))
    assert ei.value.code == fc.FC_EUNSUPPORTED


# ------------------------------------------------------------------ verdicts (Theorem 1) and the search (Algorithm 1)

@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_feasible_matches_oracle(cfg):
    topo = w.config_topology(cfg)
    inv = _optimum(cfg, topo) if cfg in (2, 5) else None
    U, k = config_candidates(cfg, inv, extra_parity=True)
    U = np.concatenate([U, [0, 5]]).astype(np.int32); k = np.concatenate([k, [3, 0]]).astype(np.int32)   # two malformed
    with _upload(topo) as g:
        res = fc.fc_feasible(g, _dev(U), _dev(k), want_flows=True, want_stats=True)
        torch.cuda.synchronize()
        feas = res["feasible"].cpu().numpy(); wit = res["witness"].cpu().numpy(); flows = res["flows"].cpu().numpy()
    comp = topo.compute_nodes
    for c in range(len(U) - 2):
        ok, want = o.feasible(topo, int(U[c]), int(k[c]), threads=16)
        assert (flows[c] == want).all(), (cfg, c)
        assert bool(feas[c]) == ok
        short = comp[want < topo.n_compute * int(k[c])]
        assert wit[c] == (-1 if ok else short.min())
    assert feas[-2:].tolist() == [0, 0] and wit[-2:].tolist() == [-1, -1]
    assert (flows[-2:] == fc.FC_FLOW_INVALID).all()
    # Theorem 1: verdicts are monotone in U/k
    order = np.argsort([Fraction(int(a), int(b)) for a, b in zip(U[:-2], k[:-2])], kind="stable")
    f = feas[:-2][order].tolist()
    assert f == sorted(f)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_search_matches_oracle_on_configs(cfg):
    topo = w.config_topology(cfg)
    want = Fraction(*_optimum(cfg, topo))
    wantU, wantk = o.smallest_U_k(want, topo.bandwidth)
    with _upload(topo) as g:
        for cpr in (16, 3):
            res = fc.fc_opt_throughput_search(g, cpr)
            assert res["inv_xstar"] == want and res["U"] == wantU and res["k"] == wantk
            assert res["trace_len"] == len(res["trace"]) > 0
            # every verdict the GPU produced, re-evaluated by the oracle (sampled on the big config)
            trace = res["trace"] if cfg < 5 else res["trace"][:: max(1, len(res["trace"]) // 6)]
            for U, k, v in trace:
                assert bool(v) == o.feasible(topo, U, k, threads=16)[0], (U, k)
            if cfg >= 4:
                break


def test_search_on_random_and_disconnected_graphs():
    for seed in range(40):
        topo = w.random_tiny(seed, strongly_connected=(seed % 4 != 3))
        with _upload(topo) as g:
            try:
                want = o.optimality_binary_search(topo)
            except o.Disconnected:
                with pytest.raises(fc.FcError) as ei:
                    fc.fc_opt_throughput_search(g, 5)
                assert ei.value.code == fc.FC_EDISCONNECTED
                continue
            res = fc.fc_opt_throughput_search(g, 1 + seed % 7)
            assert res["inv_xstar"] == want
            assert (res["U"], res["k"]) == o.smallest_U_k(want, topo.bandwidth)
    for topo, want in [(w.paper_example_ring_unwound(2), Fraction(2)), (w.paper_example_split(3), Fraction(1, 3)),
                       (w.complete_digraph(6, 7), Fraction(1, 7)), (w.star_switch(9, 4), Fraction(2))]:
        with _upload(topo) as g:
            assert fc.fc_opt_throughput_search(g, 8)["inv_xstar"] == want


def test_scaling_identity_on_gpu():
    # multiplying every capacity, source arcs included, by t multiplies F by t (Appendix E.1)
    topo = w.config_topology(2)
    pl = w.all_sinks(topo, [3, 9, 14], [2, 5, 4])
    with _upload(topo) as g:
        base, _ = _gpu_flows(g, pl.sink, pl.edge_mult, pl.src_cap)
        for t in (2, 7, 1000):
            got, _ = _gpu_flows(g, pl.sink, pl.edge_mult * t, pl.src_cap * t)
            assert (got == t * base).all()


# ------------------------------------------------------------------ fixed k: floor(U b_e) capacities, Algorithm 3

def _gpu_flows_floor(g, sink, num, den, k, options=None, want_stats=False):
    flows, stats = fc.fc_maxflow_batch_floor(g, _dev(sink), _dev(num), _dev(den), _dev(k), options=options,
                                            want_stats=want_stats)
    torch.cuda.synchronize()
    return flows.cpu().numpy().astype(np.int64), stats


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_floor_capacity_flows_match_oracle(cfg):
    topo = w.config_topology(cfg)
    N = topo.n_compute
    inv = Fraction(*_optimum(cfg, topo))
    rng = np.random.default_rng(500 + cfg)
    # per k, multipliers scattered around k / x* (where verdicts flip) with assorted denominators
    nums, dens, ks = [], [], []
    for k in (1, 2, 3, 7):
        for den in (1, 2, 3, 5, 64, 97, 1000):
            centre = inv * k * den
            for off in (-3, -1, 0, 1, 4):
                nums.append(max(1, int(centre) + off)); dens.append(den); ks.append(k)
    nums, dens, ks = (np.array(a, dtype=np.int64) for a in (nums, dens, ks))
    if cfg == 5:                                           # 140 candidates x 1024 sinks is a lot for the oracle: sample
        pick = np.sort(rng.choice(len(nums), 24, replace=False)); nums, dens, ks = nums[pick], dens[pick], ks[pick]
    comp = topo.compute_nodes
    sink = np.tile(comp, len(nums)); num = np.repeat(nums, N); den = np.repeat(dens, N); k = np.repeat(ks, N)
    want = o.aux_maxflow_batch_floor(topo, sink, num, den, k, threads=16)
    with _upload(topo) as g:
        got, stats = _gpu_flows_floor(g, sink, num, den, k, want_stats=True)
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, (cfg, bad[:8], got[bad[:8]], want[bad[:8]])
        assert stats["not_converged"] == 0
        # a denominator of 1 is the integer path
        a, _ = _gpu_flows(g, sink[: 4 * N], num[: 4 * N], k[: 4 * N])
        b, _ = _gpu_flows_floor(g, sink[: 4 * N], num[: 4 * N], np.ones(4 * N), k[: 4 * N])
        assert (a == b).all()
        # verdict form of the same thing
        res = fc.fc_feasible_floor(g, _dev(nums), _dev(dens), _dev(ks), want_flows=True)
        torch.cuda.synchronize()
        flows = res["flows"].cpu().numpy().astype(np.int64)
        assert (flows.reshape(-1) == want).all()
        feas = res["feasible"].cpu().numpy()
        assert (feas == (want.reshape(len(nums), N) >= N * ks[:, None]).all(axis=1)).all()


def test_floor_capacity_on_tiny_random_graphs_and_malformed_input():
    for seed in range(60):
        topo = w.random_tiny(seed, n_vertices=None if seed % 3 else 12, strongly_connected=(seed % 4 != 3))
        rng = np.random.default_rng(900 + seed)
        P = 64
        sink = rng.integers(0, topo.n_vertices, P).astype(np.int32)
        num = rng.integers(1, 200, P).astype(np.int64)
        den = rng.integers(1, 40, P).astype(np.int64)
        k = rng.integers(1, 30, P).astype(np.int64)
        k[::7] = rng.integers(20000, 3000000, k[::7].shape)                    # N*k > 65535: 32-bit state
        num[::11] = rng.integers(1 << 20, 1 << 30, num[::11].shape)            # products beyond 32 bits
        den[::13] = rng.integers(1 << 20, 1 << 30, den[::13].shape)            # multipliers far below 1: most links floor to 0
        want = o.aux_maxflow_batch_floor(topo, sink, num, den, k, algo="edmonds_karp" if seed % 2 else "dinic")
        with _upload(topo) as g:
            got, _ = _gpu_flows_floor(g, sink, num, den, k)
            assert (got == want).all(), (seed, np.flatnonzero(got != want)[:5])
            if seed % 6 == 0:
                got2, _ = _gpu_flows_floor(g, sink, num, den, k, options={"force_wide": 1, "use_label_table": 2})
                assert (got2 == want).all(), seed
            if seed == 0:
                den_bad = den.copy(); den_bad[3] = 0; den_bad[9] = -5
                got3, _ = _gpu_flows_floor(g, sink, num, den_bad, k)
                assert got3[3] == fc.FC_FLOW_INVALID and got3[9] == fc.FC_FLOW_INVALID
                keep = np.ones(P, dtype=bool); keep[[3, 9]] = False
                assert (got3[keep] == want[keep]).all()


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_fixed_k_search_matches_oracle_on_configs(cfg):
    topo = w.config_topology(cfg)
    inv = Fraction(*_optimum(cfg, topo))
    bmin = int(o.links(topo)[2].min())
    with _upload(topo) as g:
        for k in ((1, 2, 5) if cfg < 5 else (2,)):
            want = o.fixed_k_binary_search(topo, k, threads=16)
            res = fc.fc_fixed_k_search(g, k, 16 if k != 2 else 3)
            assert res["U_star"] == want, (cfg, k)
            assert inv <= want / k <= inv + Fraction(1, k * bmin)              # Theorem 13 and the optimum
            trace = res["trace"] if cfg < 5 else res["trace"][:: max(1, len(res["trace"]) // 6)]
            for num, den, v in trace:                                          # every verdict the GPU produced
                assert bool(v) == o.fixed_k_feasible(topo, Fraction(num, den), k, threads=16)[0], (num, den)
    # the paper's worked example: k = 1 at U = 1/b (Section 5.2, "Determine k")
    for b in (1, 3):
        with _upload(w.paper_example_switch(b)) as g:
            assert fc.fc_fixed_k_search(g, 1, 8)["U_star"] == Fraction(1, b)
            assert fc.fc_fixed_k_search(g, 4, 2)["U_star"] == Fraction(4, b)


def test_fixed_k_search_on_random_and_disconnected_graphs():
    for seed in range(40):
        topo = w.random_tiny(700 + seed, max_cap=6, strongly_connected=(seed % 4 != 3))
        k = 1 + seed % 3
        with _upload(topo) as g:
            try:
                want = o.fixed_k_binary_search(topo, k)
            except o.Disconnected:
                with pytest.raises(fc.FcError) as ei:
                    fc.fc_fixed_k_search(g, k, 5)
                assert ei.value.code == fc.FC_EDISCONNECTED
                continue
            assert fc.fc_fixed_k_search(g, k, 1 + seed % 7)["U_star"] == want, seed


# ------------------------------------------------------------------ edge splitting: gamma of the maximum-split-off theorem (Appendix E.2)

def _switch_pairs(topo):
    cap = o.link_capacities(topo)
    switches = [v for v in range(topo.n_vertices) if not topo.is_compute[v]]
    return [(u, sw, t) for sw in switches for (u, x) in sorted(cap) if x == sw for (y, t) in sorted(cap) if y == sw]


def _gamma_on_gpu(topo, U, k, pairs, want_flows=True, options=None):
    pu, pw, pt = (np.array([p[i] for p in pairs], dtype=np.int32) for i in range(3))
    with _upload(topo) as g:
        res = fc.fc_split_gamma_batch(g, U, k, _dev(pu), _dev(pw), _dev(pt), want_flows=want_flows, want_stats=True, options=options)
        torch.cuda.synchronize()
    assert res["stats"]["not_converged"] == 0
    return res["gamma"].cpu().numpy().astype(np.int64), (res["flows"].cpu().numpy().astype(np.int64) if want_flows else None)


def _scaled(topo, U):
    return w.Topology(topo.name, topo.n_vertices, topo.tail, topo.head,
                      (np.asarray(topo.bandwidth, dtype=np.int64) * int(U)).astype(np.int32), topo.is_compute)


def test_split_gamma_on_the_paper_example():
    # Appendix E.2, stages figure: 10 b inside a box, b across boxes, nothing from the spine back into the same box
    for U, k, b in ((1, 1, 1), (3, 3, 1), (1, 2, 2)):
        topo = w.paper_example_switch(b)
        pairs = _switch_pairs(topo)
        got, flows = _gamma_on_gpu(topo, U, k, pairs)
        D = _scaled(topo, U)
        for i, (u, sw, t) in enumerate(pairs):
            F1, F2 = o.split_flows(D, k, u, sw, t)
            assert (flows[i, 0] == F1).all() and (flows[i, 1] == F2).all(), (U, k, b, u, sw, t)
            assert got[i] == o.split_gamma(D, k, u, sw, t)
        idx = {p: i for i, p in enumerate(pairs)}
        if (U, k, b) == (1, 1, 1):
            assert got[idx[(0, 8, 1)]] == 10 and got[idx[(0, 10, 4)]] == 1 and got[idx[(0, 10, 1)]] == 0


def test_split_gamma_matches_oracle_on_random_eulerian_graphs():
    checked = 0
    for seed in range(40):
        rng = np.random.default_rng(6000 + seed)
        base = w.random_tiny(6000 + seed, n_vertices=int(rng.integers(4, 10)), max_cap=5, density=0.4)
        if base.is_compute.all():
            continue
        cap = {}
        for t, h, b in zip(base.tail.tolist(), base.head.tolist(), base.bandwidth.tolist()):
            if t != h and b > 0:
                key = (min(t, h), max(t, h)); cap[key] = cap.get(key, 0) + int(b)
        tail = [a for a, b in cap] + [b for a, b in cap]; head = [b for a, b in cap] + [a for a, b in cap]
        sym = w.Topology(f"euler{seed}", base.n_vertices, np.array(tail, dtype=np.int32), np.array(head, dtype=np.int32),
                         np.array(list(cap.values()) * 2, dtype=np.int32), base.is_compute.copy())
        try:
            inv = o.optimality_binary_search(sym)
        except o.Disconnected:
            continue
        Uq, k = o.smallest_U_k(inv, sym.bandwidth)
        # integer multiplier for the library: scale k too when Proposition 3's U is a fraction
        U, kk = Uq.numerator, k * Uq.denominator
        pairs = _switch_pairs(sym)
        if not pairs:
            continue
        # a pair that is no pair: (compute node in the middle) and (a missing link)
        comp = [v for v in range(sym.n_vertices) if sym.is_compute[v]]
        bogus = [(pairs[0][0], comp[0], pairs[0][2]), (pairs[0][1], pairs[0][1], pairs[0][2]), (-1, pairs[0][1], 99)]
        got, flows = _gamma_on_gpu(sym, U, kk, pairs + bogus)
        D = _scaled(sym, U)
        for i, (u, sw, t) in enumerate(pairs):
            F1, F2 = o.split_flows(D, kk, u, sw, t, algo="edmonds_karp" if seed % 2 else "dinic")
            assert (flows[i, 0] == F1).all() and (flows[i, 1] == F2).all(), (seed, u, sw, t)
            assert got[i] == o.split_gamma(D, kk, u, sw, t), (seed, u, sw, t)
            assert got[i] >= 0
        assert (got[len(pairs):] == fc.FC_GAMMA_INVALID).all()
        early, _ = _gamma_on_gpu(sym, U, kk, pairs + bogus, want_flows=False)      # max-flows may stop early: same gamma
        assert (early == got).all(), seed
        # in two launches (first without the compute node v, then from the kept preflows): same flows, same gamma
        two, two_flows = _gamma_on_gpu(sym, U, kk, pairs + bogus, options={"split_two_launches": 1})
        assert (two == got).all() and (two_flows == flows).all(), seed
        two_early, _ = _gamma_on_gpu(sym, U, kk, pairs + bogus, want_flows=False, options={"split_two_launches": 1})
        assert (two_early == got).all(), seed
        # the second launch's problems solved forwards (all stranded excess towards v) instead of backwards from v
        for rev in (1, 2):
            alt, alt_flows = _gamma_on_gpu(sym, U, kk, pairs + bogus, options={"split_two_launches": 1, "split_reverse": rev})
            assert (alt == got).all() and (alt_flows == flows).all(), (seed, rev)
        alt, _ = _gamma_on_gpu(sym, U, kk, pairs + bogus, want_flows=False, options={"split_two_launches": 1, "split_reverse": 2})
        assert (alt == got).all(), seed
        checked += len(pairs)
    assert checked > 200


@pytest.mark.parametrize("cfg", [1, 3, 4])
def test_split_gamma_on_configs(cfg):
    # bidirectional (Eulerian) configs at their optimum (U, k) from Proposition 3; a sample of pairs per switch kind
    topo = w.config_topology(cfg)
    assert o.is_eulerian(topo)
    inv = Fraction(*_optimum(cfg, topo))
    Uq, k = o.smallest_U_k(inv, topo.bandwidth)
    U, kk = Uq.numerator, k * Uq.denominator
    pairs = _switch_pairs(topo)
    rng = np.random.default_rng(cfg)
    pick = [pairs[int(i)] for i in rng.permutation(len(pairs))[: (24 if cfg < 4 else 6)]]
    got, flows = _gamma_on_gpu(topo, U, kk, pick)
    D = _scaled(topo, U)
    for i, (u, sw, t) in enumerate(pick):
        F1, F2 = o.split_flows(D, kk, u, sw, t)
        assert (flows[i, 0] == F1).all() and (flows[i, 1] == F2).all(), (cfg, u, sw, t)
        assert got[i] == o.split_gamma(D, kk, u, sw, t)
    # initial heights from the distance tables (the default on the larger graphs) or from a search in the kernel;
    # relabel policies; lanes per vertex
    for opt in ({"use_label_table": 2}, {"global_relabel_rises": -1, "use_gap": 2}, {"global_relabel_rises": 1, "lanes_per_vertex": 4},
                {"threads_per_problem": 256, "lanes_per_vertex": 32}, {"split_two_launches": 1}, {"split_two_launches": 2},
                {"split_two_launches": 1, "threads_per_problem": 64, "global_relabel_rises": -1},
                {"split_two_launches": 1, "split_reverse": 1}, {"split_two_launches": 1, "split_reverse": 1, "lanes_per_vertex": 64, "use_gap": 2}):
        alt, alt_flows = _gamma_on_gpu(topo, U, kk, pick, options=opt)
        assert (alt == got).all() and (alt_flows == flows).all(), (cfg, opt)
    # without the flows a max-flow may stop once N k + min{c(e), c(f)} units have arrived: gamma is the same
    early, _ = _gamma_on_gpu(topo, U, kk, pick, want_flows=False)
    assert (early == got).all()
    for two in (1, 2):
        early, _ = _gamma_on_gpu(topo, U, kk, pick, want_flows=False, options={"split_two_launches": two})
        assert (early == got).all(), two
    early, _ = _gamma_on_gpu(topo, U, kk, pick, want_flows=False, options={"split_two_launches": 1, "split_reverse": 2})
    assert (early == got).all()


def test_split_gamma_on_the_1024_compute_rail_fabric():
    # Paper-scale Eulerian input (1 160 vertices): one pair over a box switch, one over a rail switch, at the optimum (127, 2);
    # graphs of 1024 vertices or more run these launches with four wavefronts per problem.  The oracle takes about 8 s a pair.
    topo = w.eulerian_fabric_1024()
    U, k = 127, 2
    D = _scaled(topo, U)
    cap = o.link_capacities(topo)
    pick = []
    for sw, i_in, i_out in ((1024, 0, 1), (topo.n_vertices - 1, 3, 100)):
        assert not topo.is_compute[sw]
        ins = sorted(u for (u, x) in cap if x == sw); outs = sorted(t for (y, t) in cap if y == sw)
        pick.append((ins[i_in], sw, outs[i_out]))
    got, flows = _gamma_on_gpu(topo, U, k, pick)
    for i, (u, sw, t) in enumerate(pick):
        F1, F2 = o.split_flows(D, k, u, sw, t)
        assert (flows[i, 0] == F1).all() and (flows[i, 1] == F2).all(), (u, sw, t)
        # the oracle's gamma, from the flows it has just computed (o.split_gamma would compute them a second time)
        capD = o.link_capacities(D)
        Nk = int(np.count_nonzero(topo.is_compute)) * k
        assert got[i] == min(capD[(u, sw)], capD[(sw, t)], int(F1.min()) - Nk, int(F2.min()) - Nk), (u, sw, t)
    for opt in ({"split_two_launches": 1}, {"split_two_launches": 2}):
        alt, alt_flows = _gamma_on_gpu(topo, U, k, pick, options=opt)
        assert (alt == got).all() and (alt_flows == flows).all(), opt
    early, _ = _gamma_on_gpu(topo, U, k, pick, want_flows=False)
    assert (early == got).all()


# ------------------------------------------------------------------ Algorithm 2: the switch-removal loop around the gamma batches

def _remove_on_gpu(D, k, options=None):
    return fc.fc_remove_switches(D.n_vertices, D.tail, D.head, D.bandwidth, D.is_compute, k, options=options)


def test_remove_switches_matches_oracle_on_the_paper_example():
    for b, U, k in ((1, 1, 1), (2, 3, 6)):
        D = _scaled(w.paper_example_switch(b), U)
        want, table = o.remove_switches(D, k)
        got = _remove_on_gpu(D, k)
        assert got["links"] == o.link_capacities(want) and got["table"] == table
        assert got["batches"] >= 1


def test_remove_switches_matches_oracle_on_random_eulerian_graphs():
    done = 0
    for seed in range(30):
        rng = np.random.default_rng(8000 + seed)
        base = w.random_tiny(8000 + seed, n_vertices=int(rng.integers(4, 9)), max_cap=4, density=0.4)
        if base.is_compute.all():
            continue
        cap = {}
        for t, h, b in zip(base.tail.tolist(), base.head.tolist(), base.bandwidth.tolist()):
            if t != h and b > 0:
                key = (min(t, h), max(t, h)); cap[key] = cap.get(key, 0) + int(b)
        tail = [a for a, b in cap] + [b for a, b in cap]; head = [b for a, b in cap] + [a for a, b in cap]
        sym = w.Topology(f"euler{seed}", base.n_vertices, np.array(tail, dtype=np.int32), np.array(head, dtype=np.int32),
                         np.array(list(cap.values()) * 2, dtype=np.int32), base.is_compute.copy())
        try:
            inv = o.optimality_binary_search(sym)
        except o.Disconnected:
            continue
        Uq, k = o.smallest_U_k(inv, sym.bandwidth)
        D = _scaled(sym, Uq.numerator)
        kk = k * Uq.denominator
        want, table = o.remove_switches(D, kk, algo="edmonds_karp" if seed % 2 else "dinic")
        got = _remove_on_gpu(D, kk)
        assert got["links"] == o.link_capacities(want), seed
        assert got["table"] == table, seed
        two = _remove_on_gpu(D, kk, options={"split_two_launches": 1})      # every batch in two launches
        assert two["links"] == got["links"] and two["table"] == got["table"], seed
        # without the preflows kept from batch to batch, without the backward second launch, without both
        for opt in ({"split_carry": 2}, {"split_reverse": 2}, {"split_carry": 2, "split_reverse": 2, "split_two_launches": 1}):
            alt = _remove_on_gpu(D, kk, options=opt)
            assert alt["links"] == got["links"] and alt["table"] == got["table"], (seed, opt)
        done += 1
    assert done >= 15
    # not Eulerian: refused; Eulerian but the condition min F >= N k fails: reported
    bad = w.directed_ring(4, 3)
    bad = w.Topology("noneuler", 4, np.append(bad.tail, 0).astype(np.int32), np.append(bad.head, 2).astype(np.int32),
                     np.append(bad.bandwidth, 1).astype(np.int32), bad.is_compute)
    with pytest.raises(fc.FcError) as ei:
        _remove_on_gpu(bad, 1)
    assert ei.value.code == fc.FC_EINVAL
    D = w.paper_example_switch(1)
    with pytest.raises(fc.FcError) as ei:
        _remove_on_gpu(D, 3)                               # the example carries k = 1 at these capacities, not 3
    assert ei.value.code == fc.FC_ENOCONVERGE


def test_remove_switches_on_config1():
    topo = w.config_topology(1)
    inv = Fraction(*_optimum(1, topo))
    Uq, k = o.smallest_U_k(inv, topo.bandwidth)
    D = _scaled(topo, Uq.numerator)
    kk = k * Uq.denominator
    want, table = o.remove_switches(D, kk)
    got = _remove_on_gpu(D, kk)
    assert got["links"] == o.link_capacities(want) and got["table"] == table
    Dstar = w.Topology("star", D.n_vertices, np.array([a for a, _ in got["links"]], dtype=np.int32),
                       np.array([b for _, b in got["links"]], dtype=np.int32),
                       np.array(list(got["links"].values()), dtype=np.int32), D.is_compute)
    assert o.feasible(Dstar, 1, kk)[0] and o.is_eulerian(Dstar)


def test_remove_switches_on_config3_in_one_and_in_two_launches_per_batch():
    # the same links and the same table whether a batch's max-flows are solved in one launch, in two, or as the library chooses
    topo = w.config_topology(3)
    D = _scaled(topo, 15)
    res = [_remove_on_gpu(D, 2, options=opt) for opt in (None, {"split_two_launches": 1}, {"split_two_launches": 2},
                                                         {"split_carry": 2}, {"split_reverse": 2}, {"split_carry": 2, "split_reverse": 2})]
    assert len(res[0]["links"]) == 504
    assert all(r["links"] == res[0]["links"] and r["table"] == res[0]["table"] for r in res[1:])
    # element by element against what the oracle's loop (Algorithm "Remove Switch Nodes") leaves on this input:
    # tests/golden/config3_dstar.json, written by tests/golden/make_config3_goldens.py from the oracle alone
    gold = _golden("config3_dstar.json")
    assert (gold["U"], gold["k"]) == (15, 2)
    assert res[0]["links"] == {(a, b): c for a, b, c in gold["links"]}
    want_table = {}
    for u, t, sw, amount in gold["table"]:
        want_table.setdefault((u, t), {})[sw] = amount
    assert res[0]["table"] == want_table


# ------------------------------------------------------------------ the per-sink tables the device builds at upload

def _check_sink_table(topo, g, sink, tab, cap):
    """What the tables promise, recomputed here from the link list alone."""
    n = topo.n_vertices
    into = {v: [] for v in range(n)}
    for (a, b), c in cap.items():
        if c > 0:
            into[b].append(a)
    dist = [n] * n; dist[sink] = 0; frontier = [sink]                     # breadth-first search against the links
    while frontier:
        nxt = []
        for x in frontier:
            for a in into[x]:
                if dist[a] == n:
                    dist[a] = dist[x] + 1; nxt.append(a)
        frontier = nxt
    assert tab["have"] & 1
    assert tab["label"].tolist() == dist
    reach = [v for v in range(n) if v != sink and dist[v] < n]
    assert tab["label_hmax"] == max([dist[v] for v in reach if topo.is_compute[v]], default=0)
    if not tab["have"] & 2:
        return False
    L = max([dist[v] for v in reach], default=0)
    lt = tab["level_table"].tolist()
    assert lt[0] == L
    want_order = sorted(reach, key=lambda v: (-dist[v], v))
    assert tab["order_vertex"][: len(reach)].tolist() == want_order
    starts = [sum(1 for v in reach if dist[v] > d) for d in range(L, 0, -1)]   # level d starts after all deeper vertices
    assert lt[1: 1 + L] == starts and lt[1 + L] == len(reach) and all(x == 0 for x in lt[2 + L:])
    row_ptr, other, pair, bw, fwd = fc.fc_graph_csr(g)
    pair_of = {}
    for u in range(n):
        for r in range(row_ptr[u], row_ptr[u + 1]):
            if fwd[r]:
                pair_of[(u, int(other[r]))] = int(pair[r])
    weight = {v: int(topo.is_compute[v]) for v in range(n)}
    num, den = (1, 0) if any(topo.is_compute[v] and dist[v] >= n for v in range(n)) else (0, 1)
    for i, v in enumerate(want_order):                                       # children come before their parents
        q, b = int(tab["first_head"][i]), int(tab["first_bw"][i])
        assert cap.get((v, q), 0) == b > 0 and dist[q] == dist[v] - 1, (sink, v, q)
        assert int(tab["first_pair"][i]) == pair_of[(v, q)]
        weight[q] += weight[v]
        if den != 0 and weight[v] * den > num * b:
            num, den = weight[v], b
    assert weight[sink] == sum(int(topo.is_compute[v]) for v in range(n) if dist[v] < n)   # a spanning in-tree: everything arrives
    rn, rd = tab["ratio"]
    assert (rd == 0) == (den == 0) and rn * den == num * rd, (sink, tab["ratio"], num, den)
    for i in range(len(reach), n):
        assert tab["first_bw"][i] == 0 and tab["order_vertex"][i] == 0
    return True


def test_sink_tables_on_random_graphs_and_configs():
    full = 0
    for seed in range(30):
        topo = w.random_tiny(35000 + seed, max_cap=9, strongly_connected=(seed % 3 != 2))
        cap = o.link_capacities(topo)
        with _upload(topo) as g:
            for sink in range(topo.n_vertices):
                full += _check_sink_table(topo, g, sink, fc.fc_graph_sink_table(g, sink), cap)
    assert full > 100
    for cfg in (1, 2, 3, 4, 5):
        topo = w.config_topology(cfg)
        cap = o.link_capacities(topo)
        rng = np.random.default_rng(35100 + cfg)
        sinks = sorted(set([0, topo.n_vertices - 1] + [int(x) for x in rng.integers(0, topo.n_vertices, 6 if cfg < 4 else 3)]))
        with _upload(topo) as g:
            for sink in sinks:
                assert _check_sink_table(topo, g, sink, fc.fc_graph_sink_table(g, sink), cap)
    # a path of 70 vertices is deeper than the level table: labels only, and the solver still gets every value right
    n = 70
    tail = list(range(n - 1)) + list(range(1, n)); head = list(range(1, n)) + list(range(n - 1))
    line = w.Topology("line70", n, np.array(tail, np.int32), np.array(head, np.int32), np.full(len(tail), 3, np.int32), np.ones(n, np.uint8))
    with _upload(line) as g:
        tab = fc.fc_graph_sink_table(g, 0)
        assert tab["have"] == 1 and tab["label"].tolist() == list(range(n))
        sink = np.arange(n, dtype=np.int32); U = np.full(n, 2, np.int32); k = np.full(n, 1, np.int32)
        assert (_gpu_flows(g, sink, U, k)[0] == o.aux_maxflow_batch(line, sink, U, k)).all()


# ------------------------------------------------------------------ in-place bandwidth updates of an uploaded graph

def _topology_of(base, cap):
    live = sorted(key for key, b in cap.items() if b > 0)
    return w.Topology(base.name + "_updated", base.n_vertices, np.array([a for a, _ in live], dtype=np.int32),
                      np.array([b for _, b in live], dtype=np.int32), np.array([cap[x] for x in live], dtype=np.int32), base.is_compute)


def _upload_with_spares(topo, spares):
    tail = np.concatenate([topo.tail, np.array([a for a, _ in spares], dtype=np.int32)]).astype(np.int32)
    head = np.concatenate([topo.head, np.array([b for _, b in spares], dtype=np.int32)]).astype(np.int32)
    bw = np.concatenate([topo.bandwidth, np.zeros(len(spares), dtype=np.int32)]).astype(np.int32)
    return fc.fc_graph_upload_with_spares(topo.n_vertices, tail, head, bw, topo.is_compute)


def test_update_arcs_matches_oracle_on_random_graphs():
    # links lowered (also to zero), raised, spare links brought to life; tables rebuilt or dropped: always the oracle's
    # values on the updated arc list, and after a rebuild also its optimum
    searched = 0
    for seed in range(40):
        rng = np.random.default_rng(33000 + seed)
        topo = w.random_tiny(33000 + seed, max_cap=7, strongly_connected=(seed % 5 != 4))
        n = topo.n_vertices
        cap = o.link_capacities(topo)
        spares = [(a, b) for a in range(n) for b in range(n) if a != b and (a, b) not in cap and rng.random() < 0.3]
        for key in spares:
            cap[key] = 0
        for a, b, c in zip(topo.tail.tolist(), topo.head.tolist(), topo.bandwidth.tolist()):
            if c == 0 and a != b:                       # the generator's own zero-bandwidth arc becomes a spare link too
                cap.setdefault((a, b), 0)
        with _upload_with_spares(topo, spares) as g:
            assert fc.fc_graph_info(g).n_arcs_merged == len(cap)
            for rnd in range(4):
                keys = sorted(cap)
                pick = [keys[int(i)] for i in rng.permutation(len(keys))[: max(1, int(len(keys) * rng.random()))]]
                new = [int(rng.integers(0, 9)) if rng.random() < 0.8 else 0 for _ in pick]
                refresh = bool((seed + rnd) % 2)
                fc.fc_graph_update_arcs(g, [a for a, _ in pick], [b for _, b in pick], new, refresh_tables=refresh)
                for key, b in zip(pick, new):
                    cap[key] = b
                now = _topology_of(topo, cap)
                if now.n_arcs == 0:
                    continue
                info = fc.fc_graph_info(g)
                assert info.min_in_bw_compute == o.min_compute_in_bandwidth(now) and info.is_eulerian == o.is_eulerian(now)
                comp = now.compute_nodes
                sink = np.tile(np.arange(n, dtype=np.int32), 3)
                U = np.repeat(np.array([1, 2, 5], np.int32), n); k = np.repeat(np.array([1, 3, 4], np.int32), n)
                want = o.aux_maxflow_batch(now, sink, U, k)
                got, stats = _gpu_flows(g, sink, U, k, want_stats=True)
                assert (got == want).all(), (seed, rnd, refresh)
                assert stats["not_converged"] == 0
                wide, _ = _gpu_flows(g, sink, U, k, options={"force_wide": 1})
                assert (wide == want).all(), (seed, rnd, refresh)
                if refresh:
                    try:
                        x = o.optimality_binary_search(now)
                    except o.Disconnected:
                        with pytest.raises(fc.FcError) as ei:
                            fc.fc_opt_throughput_search(g, 4)
                        assert ei.value.code == fc.FC_EDISCONNECTED
                        continue
                    assert fc.fc_opt_throughput_search(g, 1 + seed % 5)["inv_xstar"] == x, (seed, rnd)
                    searched += 1
    assert searched >= 30


@pytest.mark.parametrize("cfg", [3, 5])
def test_update_arcs_on_configs_matches_oracle(cfg):
    # a degraded fabric: one link in ten at a fraction of its bandwidth, a few links down, a few upgraded; the full
    # problem list against the oracle with the tables rebuilt (first pass along new first-arc trees) and without them
    topo = w.config_topology(cfg)
    rng = np.random.default_rng(34000 + cfg)
    cap = o.link_capacities(topo)
    keys = sorted(cap)
    pick = [keys[int(i)] for i in rng.permutation(len(keys))[: len(keys) // 8]]
    new = []
    for j, key in enumerate(pick):
        new.append(0 if j % 9 == 0 else (cap[key] * 3 if j % 9 == 1 else max(1, cap[key] // int(rng.integers(2, 5)))))
    inv = _optimum(cfg, topo) if cfg == 5 else None
    pl = w.config_problems(cfg, topo, inv)
    with _upload(topo) as g:
        for refresh in (False, True):
            fc.fc_graph_update_arcs(g, [a for a, _ in pick], [b for _, b in pick], new, refresh_tables=refresh)
            now = dict(cap)
            for key, b in zip(pick, new):
                now[key] = b
            changed = _topology_of(topo, now)
            want = o.aux_maxflow_batch(changed, pl.sink, pl.edge_mult, pl.src_cap, threads=16)
            got, stats = _gpu_flows(g, pl.sink, pl.edge_mult, pl.src_cap, want_stats=True)
            assert (got == want).all(), (cfg, refresh)
            assert stats["not_converged"] == 0
            # without tables every problem starts with a search for heights; with them none of these needs one up front
            if not refresh:
                assert stats["global_relabels"] >= len(pl.sink)
            cert, _ = _gpu_flows(g, pl.sink, pl.edge_mult, pl.src_cap, options={"tree_certificate": 1})
            assert (cert == want).all(), (cfg, refresh)
            # and back: the original bandwidths give the original values again
            fc.fc_graph_update_arcs(g, [a for a, _ in pick], [b for _, b in pick], [cap[key] for key in pick], refresh_tables=refresh)
            want0 = o.aux_maxflow_batch(topo, pl.sink[:256], pl.edge_mult[:256], pl.src_cap[:256], threads=16)
            got0, _ = _gpu_flows(g, pl.sink[:256], pl.edge_mult[:256], pl.src_cap[:256])
            assert (got0 == want0).all(), (cfg, refresh)
        assert fc.fc_opt_throughput_search(g, 16)["inv_xstar"] == Fraction(*_optimum(cfg, topo))


def _remove_switches_in_place(D, k):
    """Algorithm "Remove Switch Nodes" (Appendix E.2) driven from here: one uploaded graph, every gamma from
    fc_split_gamma_batch on it, every split applied to it with fc_graph_update_arcs -- no second upload."""
    cap = dict(o.link_capacities(D))
    n = D.n_vertices
    switches = [v for v in range(n) if not D.is_compute[v]]
    # links a split can create: (u, t) over the ingress tails and egress heads of a switch, whatever was created before
    ins = {v: set() for v in range(n)}; outs = {v: set() for v in range(n)}
    for (a, b) in cap:
        outs[a].add(b); ins[b].add(a)
    spares = set()
    for sw in switches:
        for u in sorted(ins[sw]):
            for t in sorted(outs[sw]):
                if u != t and (u, t) not in cap:
                    spares.add((u, t)); outs[u].add(t); ins[t].add(u)
    spares = sorted(spares)
    table = {}
    with _upload_with_spares(D, spares) as g:
        for sw in switches:
            for t in sorted(h for (a, h), c in cap.items() if a == sw and c > 0):
                for u in sorted(a for (a, h), c in cap.items() if h == sw and c > 0):
                    if cap.get((sw, t), 0) == 0:
                        break
                    if cap.get((u, sw), 0) == 0:
                        continue
                    res = fc.fc_split_gamma_batch(g, 1, k, _dev([u]), _dev([sw]), _dev([t]))
                    gam = int(res["gamma"].cpu()[0])
                    assert gam >= 0
                    if gam > 0:
                        cap[(u, sw)] -= gam; cap[(sw, t)] -= gam
                        upd = [(u, sw), (sw, t)]
                        if u != t:
                            cap[(u, t)] = cap.get((u, t), 0) + gam
                            upd.append((u, t))
                            table.setdefault((u, t), {})
                            table[(u, t)][sw] = table[(u, t)].get(sw, 0) + gam
                        fc.fc_graph_update_arcs(g, [a for a, _ in upd], [b for _, b in upd], [cap[x] for x in upd], refresh_tables=False)
                assert cap.get((sw, t), 0) == 0
    return {key: c for key, c in cap.items() if c > 0}, table


def test_switch_removal_by_in_place_updates_matches_oracle():
    # the paper's worked example, config 1 and random Eulerian switch topologies: D* and the path recovery table
    cases = []
    for b, U, k in ((1, 1, 1), (2, 3, 6)):
        cases.append((_scaled(w.paper_example_switch(b), U), k))
    topo = w.config_topology(1)
    Uq, k = o.smallest_U_k(Fraction(*_optimum(1, topo)), topo.bandwidth)
    cases.append((_scaled(topo, Uq.numerator), k * Uq.denominator))
    for seed in range(12):
        rng = np.random.default_rng(8000 + seed)
        base = w.random_tiny(8000 + seed, n_vertices=int(rng.integers(4, 9)), max_cap=4, density=0.4)
        if base.is_compute.all():
            continue
        cap = {}
        for t, h, b in zip(base.tail.tolist(), base.head.tolist(), base.bandwidth.tolist()):
            if t != h and b > 0:
                key = (min(t, h), max(t, h)); cap[key] = cap.get(key, 0) + int(b)
        tail = [a for a, b in cap] + [b for a, b in cap]; head = [b for a, b in cap] + [a for a, b in cap]
        sym = w.Topology(f"euler{seed}", base.n_vertices, np.array(tail, dtype=np.int32), np.array(head, dtype=np.int32),
                         np.array(list(cap.values()) * 2, dtype=np.int32), base.is_compute.copy())
        try:
            inv = o.optimality_binary_search(sym)
        except o.Disconnected:
            continue
        Uq, k = o.smallest_U_k(inv, sym.bandwidth)
        cases.append((_scaled(sym, Uq.numerator), k * Uq.denominator))
    assert len(cases) >= 9
    for D, k in cases:
        want, want_table = o.remove_switches(D, k)
        links, table = _remove_switches_in_place(D, k)
        assert links == o.link_capacities(want), D.name
        assert table == want_table, D.name


def test_update_arcs_errors_on_the_device():
    topo = w.config_topology(1)
    with _upload(topo) as g:
        sink = np.arange(16, dtype=np.int32); U = np.full(16, 1, np.int32); k = np.full(16, 4, np.int32)
        before, _ = _gpu_flows(g, sink, U, k)
        with pytest.raises(fc.FcError) as ei:
            fc.fc_graph_update_arcs(g, [0, 0], [16, 5], [3, 3])             # (0, 5) is no link of config 1: nothing is applied
        assert ei.value.code == fc.FC_EINVAL
        after, _ = _gpu_flows(g, sink, U, k)
        assert (before == after).all()
        fc.fc_graph_update_arcs(g, [], [], [])                             # nothing to do
        assert (_gpu_flows(g, sink, U, k)[0] == before).all()


# ------------------------------------------------------------------ launch shapes the other tests do not reach

def test_remove_switches_on_config4_keeps_the_optimum():
    # too large for the oracle's loop: check what the edge-splitting existence theorem of Appendix E.2 promises instead.  D = G({U b_e}) at the optimum
    # U / k = 63 / 4 has 1/x* = 1/k; D* must be a compute-only Eulerian digraph with the same optimum, every link
    # that was routed through a switch must be covered by its table entries, and capacity is conserved per node.
    topo = w.config_topology(4)
    U, k = 63, 4
    D = _scaled(topo, U)
    res = _remove_on_gpu(D, k)
    links, table = res["links"], res["table"]
    comp = set(int(v) for v in topo.compute_nodes)
    assert links and all(a in comp and b in comp and c > 0 for (a, b), c in links.items())
    n = topo.n_vertices
    out = np.zeros(n, np.int64); inn = np.zeros(n, np.int64)
    for (a, b), c in links.items():
        out[a] += c; inn[b] += c
    assert (out == inn).all()
    # a compute node keeps its total egress capacity: every unit that left it still leaves it
    out0 = np.zeros(n, np.int64)
    np.add.at(out0, D.tail, D.bandwidth.astype(np.int64))
    assert all(out[v] <= out0[v] for v in comp)            # detours u -> w -> u disappear, nothing is added
    direct = {}
    for a, b, c in zip(D.tail.tolist(), D.head.tolist(), D.bandwidth.tolist()):
        if a in comp and b in comp:
            direct[(a, b)] = direct.get((a, b), 0) + int(c)
    for key, c in links.items():
        assert c == direct.get(key, 0) + sum(table.get(key, {}).values()), key
    keys = sorted(links)
    with fc.fc_graph_upload(n, [a for a, b in keys], [b for a, b in keys], [links[x] for x in keys], topo.is_compute) as g:
        assert fc.fc_opt_throughput_search(g, 8)["inv_xstar"] == Fraction(1, k)


def test_large_batch_two_streams_and_degenerate_graphs():
    # 300 000 problems on a small graph: several rounds of the ordering kernel, several waves of workgroups
    topo = w.config_topology(2)
    rng = np.random.default_rng(42)
    P = 300_000
    sink = rng.integers(0, topo.n_vertices, P).astype(np.int32)
    U = rng.integers(1, 40, P).astype(np.int32)
    k = rng.integers(1, 12, P).astype(np.int32)
    want = o.aux_maxflow_batch(topo, sink, U, k, threads=16)
    with _upload(topo) as g:
        got, _ = _gpu_flows(g, sink, U, k)
        assert (got == want).all()
        # the same graph used from two streams at once, each call with its own workspace and outputs
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        half = P // 2
        a = [_dev(x[:half]) for x in (sink, U, k)]; b = [_dev(x[half:]) for x in (sink, U, k)]
        torch.cuda.synchronize()
        outs = []
        for rep in range(3):
            with torch.cuda.stream(s1):
                f1, _ = fc.fc_maxflow_batch(g, *a, stream=s1)
            with torch.cuda.stream(s2):
                f2, _ = fc.fc_maxflow_batch(g, *b, stream=s2)
            outs.append((f1, f2))
        torch.cuda.synchronize()
        for f1, f2 in outs:
            assert (f1.cpu().numpy() == want[:half]).all() and (f2.cpu().numpy() == want[half:]).all()
    # two compute nodes and nothing else; two compute nodes and no arcs at all
    pair = w.Topology("pair", 2, np.array([0, 1], dtype=np.int32), np.array([1, 0], dtype=np.int32),
                      np.array([5, 3], dtype=np.int32), np.array([1, 1], dtype=np.uint8))
    with _upload(pair) as g:
        got, _ = _gpu_flows(g, [0, 1, 1], [1, 1, 7], [4, 4, 2])
        assert got.tolist() == [4 + min(4, 3), 4 + min(4, 5), 2 + min(2, 35)]
        assert fc.fc_opt_throughput_search(g, 4)["inv_xstar"] == Fraction(1, 3)
    empty = w.Topology("noarcs", 3, np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.int32),
                       np.array([1, 0, 1], dtype=np.uint8))
    with _upload(empty) as g:
        got, _ = _gpu_flows(g, [0, 1, 2], [3, 3, 3], [5, 5, 5])
        assert got.tolist() == [5, 0, 5]
        with pytest.raises(fc.FcError) as ei:
            fc.fc_opt_throughput_search(g, 4)
        assert ei.value.code == fc.FC_EDISCONNECTED


def test_ordered_list_with_malformed_problems_and_a_ragged_length():
    # an explicit list long enough to be reordered (sinks grouped, runs of 16 per XCD), its length no multiple of
    # the run size, with sinks that are not vertices and non-positive multipliers scattered through it
    topo = w.config_topology(3)
    rng = np.random.default_rng(77)
    for P in (5003, 1031, 128 * 9 + 1):
        sink = rng.choice(topo.compute_nodes, P).astype(np.int32)
        U = rng.integers(10, 70, P).astype(np.int32); k = rng.integers(1, 9, P).astype(np.int32)
        bad = rng.random(P) < 0.06
        kind = rng.integers(0, 5, P)
        sink[bad & (kind == 0)] = -1; sink[bad & (kind == 1)] = topo.n_vertices; sink[bad & (kind == 2)] = topo.n_vertices + 1000
        U[bad & (kind == 3)] = 0; k[bad & (kind == 4)] = -3
        ok = ~bad
        want = o.aux_maxflow_batch(topo, sink[ok], U[ok], k[ok], threads=16)
        with _upload(topo) as g:
            for rep in range(2):                           # the second call sorts by the first one's cost hints
                got, stats = _gpu_flows(g, sink, U, k, want_stats=True)
                assert (got[ok] == want).all() and (got[bad] == fc.FC_FLOW_INVALID).all(), (P, rep)
                assert stats["not_converged"] == 0
            plain, _ = _gpu_flows(g, sink, U, k, options={"schedule": 2})
            assert (plain == got).all()


# ------------------------------------------------------------------ non-uniform source capacities (Section 5.7)

def _merged(topo):
    tail, head, bw = o.links(topo)
    return w.Topology(topo.name, topo.n_vertices, tail, head, bw, topo.is_compute)


@pytest.mark.parametrize("cfg", [1, 3, 4, 5])
def test_weighted_source_arcs_match_oracle(cfg):
    topo = w.config_topology(cfg)
    N, comp = topo.n_compute, topo.compute_nodes
    rng = np.random.default_rng(700 + cfg)
    wts = rng.integers(0, 4, topo.n_vertices).astype(np.int32)
    wts[comp[0]] = 3                                       # not all zero
    sum_w = int(wts[comp].sum())
    inv = Fraction(*_optimum(cfg, topo))
    # candidates around the unit-weight optimum scaled by the mean weight, plus one that needs the 32-bit state
    mean = Fraction(sum_w, N)
    cands = []
    for kk in (1, 2, 5):
        centre = inv * mean * kk
        cands += [(max(1, int(centre * f)), kk) for f in (Fraction(1, 2), Fraction(9, 10), 1, Fraction(11, 10), 2)]
    cands.append((max(1, int(inv * mean * 70000 // sum_w + 1)), 70000 // sum_w + 1))      # k * sum_w > 65535
    U = np.array([c[0] for c in cands], np.int32); k = np.array([c[1] for c in cands], np.int32)
    sinks = comp if cfg < 4 else np.sort(rng.choice(comp, 64 if cfg == 4 else 24, replace=False))
    sink = np.tile(sinks, len(cands)); Uj = np.repeat(U, len(sinks)); kj = np.repeat(k, len(sinks))
    want = o.weighted_aux_maxflow_batch(topo, sink, Uj, kj, wts)
    with _upload(topo) as g:
        before, _ = _gpu_flows(g, sink[: len(sinks)], Uj[: len(sinks)], kj[: len(sinks)])
        fc.fc_graph_set_source_weights(g, wts)
        got, stats = _gpu_flows(g, sink, Uj, kj, want_stats=True)
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, (cfg, bad[:8], got[bad[:8]], want[bad[:8]])
        assert stats["not_converged"] == 0
        assert (got <= kj.astype(np.int64) * sum_w).all()
        # all launch modes agree
        for opt in ({"use_label_table": 2}, {"force_wide": 1}, {"tree_certificate": 1}, {"schedule": 2, "use_gap": 2}):
            alt, _ = _gpu_flows(g, sink, Uj, kj, options=opt)
            assert (alt == want).all(), opt
        # verdicts: F >= k * sum of the weights at every compute node
        res = fc.fc_feasible(g, _dev(U), _dev(k), want_flows=True)
        torch.cuda.synchronize()
        feas = res["feasible"].cpu().numpy(); wit = res["witness"].cpu().numpy(); flows = res["flows"].cpu().numpy().astype(np.int64)
        if cfg < 4:
            assert (flows.reshape(-1) == want).all()
            for c in range(len(cands)):
                row = want[c * N:(c + 1) * N]
                short = comp[row < int(k[c]) * sum_w]
                assert bool(feas[c]) == (short.size == 0) and wit[c] == (-1 if short.size == 0 else short.min())
        else:
            pos = np.searchsorted(comp, sinks)
            assert (flows[:, pos].reshape(-1) == want).all()
        # floor capacities with weights (the floor is per link: the oracle gets merged links)
        mt = _merged(topo)
        num = np.repeat(U.astype(np.int64) * 3 + 1, len(sinks)); den = np.full(len(sink), 3, np.int64)
        want_f = o.weighted_aux_maxflow_batch(mt, sink[: 6 * len(sinks)], num[: 6 * len(sinks)], kj[: 6 * len(sinks)], wts, U_den=den[: 6 * len(sinks)])
        got_f, _ = _gpu_flows_floor(g, sink[: 6 * len(sinks)], num[: 6 * len(sinks)], den[: 6 * len(sinks)], kj[: 6 * len(sinks)])
        assert (got_f == want_f).all()
        # what the paper defines for unit weights only is refused, not answered wrongly
        for call in (lambda: fc.fc_opt_throughput_search(g, 4), lambda: fc.fc_fixed_k_search(g, 2, 4)):
            with pytest.raises(fc.FcError) as err:
                call()
            assert err.value.code == fc.FC_EUNSUPPORTED
        # unit weights, given explicitly or by resetting, are the uniform case again
        fc.fc_graph_set_source_weights(g, np.ones(topo.n_vertices, np.int32))
        ones, _ = _gpu_flows(g, sink[: len(sinks)], Uj[: len(sinks)], kj[: len(sinks)])
        fc.fc_graph_set_source_weights(g, None)
        after, _ = _gpu_flows(g, sink[: len(sinks)], Uj[: len(sinks)], kj[: len(sinks)])
        assert (ones == before).all() and (after == before).all()
        assert fc.fc_opt_throughput_search(g, 8)["inv_xstar"] == inv


def test_weighted_source_arcs_on_tiny_random_graphs_and_bad_weights():
    for seed in range(40):
        topo = w.random_tiny(4000 + seed)
        rng = np.random.default_rng(4500 + seed)
        comp = topo.compute_nodes
        wts = rng.integers(0, 5, topo.n_vertices).astype(np.int32)
        if wts[comp].sum() == 0:
            wts[comp[-1]] = 1
        P = 24
        sink = rng.choice(comp, P).astype(np.int32); U = rng.integers(1, 6, P).astype(np.int32); k = rng.integers(1, 9, P).astype(np.int32)
        want = o.weighted_aux_maxflow_batch(topo, sink, U, k, wts)
        with _upload(topo) as g:
            fc.fc_graph_set_source_weights(g, wts)
            got, _ = _gpu_flows(g, sink, U, k)
            assert (got == want).all(), seed
            ok, flows = o.weighted_feasible(topo, int(U[0]), int(k[0]), wts)
            res = fc.fc_feasible(g, _dev(U[:1]), _dev(k[:1]), want_flows=True)
            torch.cuda.synchronize()
            assert bool(res["feasible"].cpu().numpy()[0]) == ok and (res["flows"].cpu().numpy()[0] == flows).all()
    topo = w.config_topology(1)
    with _upload(topo) as g:
        bad = np.ones(topo.n_vertices, np.int32); bad[topo.compute_nodes[1]] = -1
        for arr, code in ((bad, fc.FC_EINVAL), (np.zeros(topo.n_vertices, np.int32), fc.FC_EINVAL),
                          (np.full(topo.n_vertices, 2 ** 30, np.int32), fc.FC_EOVERFLOW)):
            with pytest.raises(fc.FcError) as err:
                fc.fc_graph_set_source_weights(g, arr)
            assert err.value.code == code
        # a k whose product with the weight sum leaves 31 bits is a malformed problem, as N k is without weights
        fc.fc_graph_set_source_weights(g, np.full(topo.n_vertices, 2 ** 20, np.int32))
        got, _ = _gpu_flows(g, topo.compute_nodes[:2], [1, 1], [1, 2 ** 11])
        assert got[1] == fc.FC_FLOW_INVALID and got[0] == o.weighted_aux_maxflow_batch(topo, topo.compute_nodes[:1], [1], [1], np.full(topo.n_vertices, 2 ** 20))[0]


# ------------------------------------------------------------------ spanning tree construction (Appendix E.3)

def _check_trees(n, links, k, trees):
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


def _star_links(topo, U, k):
    """D* of a switch topology at (U, k): switch removal by the oracle, compute nodes renumbered 0..N-1"""
    D = _scaled(topo, U)
    Dstar, _ = o.remove_switches(D, k)
    comp = [int(v) for v in topo.compute_nodes]
    idx = {v: i for i, v in enumerate(comp)}
    return len(comp), {(idx[a], idx[b]): c for (a, b), c in o.link_capacities(Dstar).items()}


def test_tree_mu_batches_match_oracle():
    # every mu the oracle's construction computes, replayed state by state as batches on the GPU: all candidate
    # edges of the state at once, with exact flows and with early stops
    cases = [(8, o.link_capacities(w.paper_example_split(2)), 2)]
    for n, k in ((3, 2), (5, 3)):
        rng = np.random.default_rng(100 * n + k)
        cases.append((n, {(a, b): k + int(rng.integers(0, 3)) for a in range(n) for b in range(n) if a != b}, k))
    cases.append(_star_links(w.paper_example_switch(1), 1, 1) + (1,))
    for n, links, k in cases:
        states = []

        def observe(g, sets, demand, i, x, y, mu):
            if not states or states[-1][0] != (dict(g), [set(R) for R in sets], list(demand), i):
                states.append(((dict(g), [set(R) for R in sets], list(demand), i), []))
            states[-1][1].append((x, y, mu))

        o.construct_trees(n, links, k, observe=observe)
        assert states
        for (g, sets, demand, i), seen in states[:: max(1, len(states) // 25)]:
            cand = [(x, y) for (x, y) in sorted(g) if x in sets[i] and y not in sets[i]]
            want = [o.tree_mu(n, g, sets, demand, i, x, y) for (x, y) in cand]
            assert [m for (_, _, m) in seen] == want[: len(seen)]
            others = sum(demand[l] for l in range(len(sets)) if l != i)
            exact = fc.fc_tree_mu_batch(n, g, sets, demand, i, cand, want_flows=True)
            assert exact["mu"].tolist() == want
            nv, tail, head, c = o.tree_mu_network(n, g, sets, demand, i, cand[0][0])
            assert exact["flows"][0] == o.maxflow(nv, tail, head, c, cand[0][0], cand[0][1])
            assert (exact["flows"] >= others).all()
            early = fc.fc_tree_mu_batch(n, g, sets, demand, i, cand)
            assert early["mu"].tolist() == want
            # entries that are no candidate: inside to inside, outside to inside, a missing link
            inside = sorted(sets[i]); outside = [v for v in range(n) if v not in sets[i]]
            bogus = [(inside[0], inside[0]), (outside[0], inside[0]), (-1, 0), (inside[0], n)]
            res = fc.fc_tree_mu_batch(n, g, sets, demand, i, cand + bogus)
            assert res["mu"].tolist() == want + [fc.FC_MU_INVALID] * 4


def test_construct_trees_matches_oracle():
    cases = [(8, o.link_capacities(w.paper_example_split(1)), 1), (8, o.link_capacities(w.paper_example_split(3)), 3),
             (2, {(0, 1): 4, (1, 0): 4}, 4), (4, {(a, b): 3 for a in range(4) for b in range(4) if a != b}, 3),
             _star_links(w.paper_example_switch(2), 1, 2) + (2,)]
    rng = np.random.default_rng(5)
    for n in (3, 5, 6):
        k = int(rng.integers(1, 5))
        cases.append((n, {(a, b): k + int(rng.integers(0, 4)) for a in range(n) for b in range(n) if a != b}, k))
    for n, links, k in cases:
        want = o.construct_trees(n, links, k)
        got = fc.fc_construct_trees(n, links, k)
        assert got["trees"] == want, (n, k)
        _check_trees(n, links, k, got["trees"])
        assert got["batches"] >= n - 1
        # every max-flow from nothing instead of from the flows kept between launches: the same trees
        cold = fc.fc_construct_trees(n, links, k, options={"tree_warm_start": 2})
        assert cold["trees"] == want and cold["batches"] == got["batches"], (n, k)
    with pytest.raises(fc.FcError) as err:
        fc.fc_construct_trees(2, {(0, 1): 4, (1, 0): 4}, 4, options={"tree_warm_start": 3})
    assert err.value.code == fc.FC_EINVAL
    # the packing condition fails: the construction reports it
    with pytest.raises(fc.FcError) as err:
        fc.fc_construct_trees(3, {(0, 1): 1, (1, 0): 2, (1, 2): 2, (2, 1): 2, (0, 2): 2, (2, 0): 2}, 2)
    assert err.value.code == fc.FC_ENOCONVERGE


@pytest.mark.parametrize("n,k,seed", [(5, 1, 0), (9, 2, 2), (12, 3, 3), (16, 2, 4)])
def test_trees_on_superposed_random_out_trees_match_oracle(n, k, seed):
    # capacities that differ from link to link: most accepted edges come with a partial mu, so copies with a vertex
    # of their own enter the network all the time, the graph is built anew and the kept flows start over
    links = w.superposed_out_trees(n, k, seed)
    want = o.construct_trees(n, links, k)
    got = fc.fc_construct_trees(n, links, k)
    assert got["trees"] == want
    assert _check_trees(n, links, k, got["trees"]) == links            # every unit of every link is used
    cold = fc.fc_construct_trees(n, links, k, options={"tree_warm_start": 2})
    assert cold["trees"] == want and cold["batches"] == got["batches"]


@pytest.mark.parametrize("n,k,seed", [(48, 3, 11), (96, 1, 12)])
def test_trees_on_larger_superposed_out_trees_use_every_unit(n, k, seed):
    # beyond what the oracle's loop does in seconds: the construction's promises (which pin the packing down to "uses
    # every unit of every link") and the same trees with and without kept flows; copies with a vertex of their own all the time
    links = w.superposed_out_trees(n, k, seed)
    got = fc.fc_construct_trees(n, links, k)
    assert _check_trees(n, links, k, got["trees"]) == links
    cold = fc.fc_construct_trees(n, links, k, options={"tree_warm_start": 2})
    assert cold["trees"] == got["trees"]


def test_trees_on_config1_after_switch_removal_on_the_gpu():
    # the back end on the GPU alone: optimum, switch removal, trees; then the oracle's trees for the same D*
    topo = w.config_topology(1)
    inv = Fraction(*_optimum(1, topo))
    Uq, k = o.smallest_U_k(inv, topo.bandwidth)
    U, kk = Uq.numerator, k * Uq.denominator
    res = _remove_on_gpu(_scaled(topo, U), kk)
    comp = [int(v) for v in topo.compute_nodes]
    idx = {v: i for i, v in enumerate(comp)}
    links = {(idx[a], idx[b]): c for (a, b), c in res["links"].items()}
    got = fc.fc_construct_trees(len(comp), links, kk)
    _check_trees(len(comp), links, kk, got["trees"])
    assert got["trees"] == o.construct_trees(len(comp), links, kk)


def test_tree_mu_on_config3_sized_states():
    # 128 nodes and as many root-sets: the state with its root-set vertices and arcs needs most of a CU's LDS.
    # States are made up (every root-set a breadth-first ball of random size around its root), which the formula
    # does not mind; mu and the flows are compared with the oracle for every candidate edge of a few root-sets.
    topo = w.config_topology(3)
    U, k = 15, 2
    res = _remove_on_gpu(_scaled(topo, U), k)
    comp = [int(v) for v in topo.compute_nodes]
    idx = {v: i for i, v in enumerate(comp)}
    links = {(idx[a], idx[b]): c for (a, b), c in res["links"].items()}
    n = len(comp)
    out = {}
    for (a, b) in sorted(links):
        out.setdefault(a, []).append(b)
    rng = np.random.default_rng(33)
    sets = []
    for u in range(n):
        size = int(rng.integers(1, 65))
        ball, queue = [u], [u]
        while queue and len(ball) < size:
            x = queue.pop(0)
            for y in out.get(x, []):
                if y not in ball and len(ball) < size:
                    ball.append(y); queue.append(y)
        sets.append(set(ball))
    demand = [int(rng.integers(1, k + 1)) for _ in range(n)]
    g = {e: c - int(rng.integers(0, min(c, 3))) for e, c in links.items()}
    g = {e: c for e, c in g.items() if c > 0}
    for i in (0, 17, 64, 127):
        cand = [(x, y) for (x, y) in sorted(g) if x in sets[i] and y not in sets[i]][:24]
        assert cand
        want = [o.tree_mu(n, g, sets, demand, i, x, y) for (x, y) in cand]
        exact = fc.fc_tree_mu_batch(n, g, sets, demand, i, cand, want_flows=True)
        assert exact["mu"].tolist() == want, i
        for j in (0, len(cand) - 1):
            nv, tail, head, c = o.tree_mu_network(n, g, sets, demand, i, cand[j][0])
            assert exact["flows"][j] == o.maxflow(nv, tail, head, c, cand[j][0], cand[j][1])
        assert fc.fc_tree_mu_batch(n, g, sets, demand, i, cand)["mu"].tolist() == want


def test_trees_on_config3_after_switch_removal_are_valid():
    # 128 roots x 127 edges: too many max-flows for the oracle's loop, so the promises of the construction are
    # checked instead -- spanning trees, k per root, no link used beyond its capacity -- and, as a spot check,
    # the first root's tree against the oracle's construction restricted to that root-set
    topo = w.config_topology(3)
    U, k = 15, 2
    res = _remove_on_gpu(_scaled(topo, U), k)
    comp = [int(v) for v in topo.compute_nodes]
    idx = {v: i for i, v in enumerate(comp)}
    links = {(idx[a], idx[b]): c for (a, b), c in res["links"].items()}
    got = fc.fc_construct_trees(len(comp), links, k)
    use = _check_trees(len(comp), links, k, got["trees"])
    # element by element against the oracle's construction on the same D* (tests/golden/config3_trees.json, written by
    # tests/golden/make_config3_goldens.py from the oracle alone): same roots, multiplicities and edges in the same order
    gold = _golden("config3_trees.json")
    assert (gold["n"], gold["k"]) == (len(comp), k)
    want = [(r, m, [(e[i], e[i + 1]) for i in range(0, len(e), 2)]) for r, m, e in gold["trees"]]
    assert got["trees"] == want
    # config 3 is symmetric and tight: every unit of every link is used by some tree
    assert sum(use.values()) == len(comp) * k * (len(comp) - 1)
    assert got["batches"] < len(comp) * (len(comp) - 1)                # the look-ahead saves launches
    # the flows kept between launches change nothing: same trees as with every max-flow started from nothing
    cold = fc.fc_construct_trees(len(comp), links, k, options={"tree_warm_start": 2})
    assert cold["trees"] == got["trees"] and cold["batches"] == got["batches"]
    # how far a launch looks ahead changes the number of launches, never a tree (1: no speculation at all)
    for chain in (1, 5, 64):
        alt = fc.fc_construct_trees(len(comp), links, k, options={"tree_chain_states": chain})
        assert alt["trees"] == got["trees"], chain
        assert (alt["batches"] > got["batches"]) == (chain < 32), (chain, alt["batches"], got["batches"])
    # first steps of root 0 by the oracle: same edges in the same order
    n = len(comp)
    g = dict(links); sets = [{u} for u in range(n)]; demand = [k] * n
    for step in range(6):
        x, y = got["trees"][0][2][step]
        cand = [(a, b) for (a, b) in sorted(g) if a in sets[0] and b not in sets[0]]
        first = next((a, b) for (a, b) in cand if o.tree_mu(n, g, sets, demand, 0, a, b) > 0)
        assert first == (x, y), step
        mu = o.tree_mu(n, g, sets, demand, 0, x, y)
        assert mu == got["trees"][0][1]
        sets[0].add(y); g[(x, y)] -= mu
        if g[(x, y)] == 0:
            del g[(x, y)]


# ------------------------------------------------------------------ the loops at size: states replayed by the oracle

def _replay_sampled_states(n, links, k, trees, samples):
    """States along a finished construction without copies (one root-set per root, multiplicity k), rebuilt from the
    returned trees: before edge j of root-set i is added, the root-sets before i span, i holds its root and its first j
    heads, the later ones are single vertices, and every edge added so far has used k units of its link.  For each
    sampled (i, j) the oracle evaluates mu for the candidate edges in (x, y) order: all before the library's edge must be
    0 and the library's edge must have mu = k (Appendix E.3, the theorem that computes mu by one max-flow)."""
    assert len(trees) == n and all(m == k and r == i for i, (r, m, _) in enumerate(trees))
    full = set(range(n))
    checked = 0
    for i, j in samples:
        g = dict(links)
        for l in range(i + 1):
            for (x, y) in (trees[l][2] if l < i else trees[l][2][:j]):
                g[(x, y)] -= k
                if g[(x, y)] == 0:
                    del g[(x, y)]
        assert all(c > 0 for c in g.values())
        sets = [set(full) for _ in range(i)] + [{i} | {y for _, y in trees[i][2][:j]}] + [{l} for l in range(i + 1, n)]
        demand = [k] * n
        chosen = trees[i][2][j]
        for (x, y) in sorted(g):
            if x in sets[i] and y not in sets[i]:
                mu = o.tree_mu(n, g, sets, demand, i, x, y)
                checked += 1
                if (x, y) == chosen:
                    assert mu == k, (i, j, x, y, mu)
                    break
                assert mu == 0, (i, j, x, y, mu)
        else:
            raise AssertionError(("the library's edge is no candidate", i, j))
    return checked


def test_trees_on_config4_sampled_states_replayed_by_the_oracle():
    # 512 roots x 511 edges: far too many max-flows for the oracle's loop.  The construction's promises are checked in full;
    # 20 states sampled along the library's own construction are rebuilt and every candidate edge up to the one the library
    # took is evaluated by the oracle
    topo = w.config_topology(4)
    U, k = 63, 4
    res = _remove_on_gpu(_scaled(topo, U), k)
    comp = [int(v) for v in topo.compute_nodes]
    idx = {v: i for i, v in enumerate(comp)}
    links = {(idx[a], idx[b]): c for (a, b), c in res["links"].items()}
    n = len(comp)
    got = fc.fc_construct_trees(n, links, k)
    use = _check_trees(n, links, k, got["trees"])
    assert sum(use.values()) == n * k * (n - 1)
    rng = np.random.default_rng(404)
    samples = [(0, 0), (0, n - 2), (n - 1, n - 2), (n - 1, 0)] + [(int(rng.integers(0, n)), int(rng.integers(0, n - 1))) for _ in range(16)]
    assert _replay_sampled_states(n, links, k, got["trees"], samples) >= len(samples)


def test_back_end_on_a_rail_fabric_warm_and_cold_and_replayed():
    # 32 boxes x 8 compute nodes, NVSwitch per box, 8 rail switches (the 1024-compute instance of the same generator is the
    # back end's timing workload): search, switch removal, trees; the trees from kept flows equal the trees with every
    # max-flow started from nothing; sampled states are replayed by the oracle; D* keeps the optimum
    topo = w.rail_fabric(32, 8)
    assert o.is_eulerian(topo)
    with _upload(topo) as g:
        sr = fc.fc_opt_throughput_search(g, 16)
    assert sr["inv_xstar"] == Fraction(256 - 8, 8 * 2)                    # the cut around one box: 248 outside, 16 coming in
    U, k = sr["U"].numerator, sr["k"] * sr["U"].denominator
    D = _scaled(topo, U)
    res = _remove_on_gpu(D, k)
    comp = [int(v) for v in topo.compute_nodes]
    assert all(a in set(comp) and b in set(comp) and c > 0 for (a, b), c in res["links"].items())
    links = {(a, b): c for (a, b), c in res["links"].items()}            # compute nodes are 0..255 already
    n = len(comp)
    keys = sorted(links)
    with fc.fc_graph_upload(n, [a for a, b in keys], [b for a, b in keys], [links[x] for x in keys], np.ones(n, np.uint8)) as g:
        assert fc.fc_opt_throughput_search(g, 8)["inv_xstar"] == Fraction(1, k)
    warm = fc.fc_construct_trees(n, links, k)
    use = _check_trees(n, links, k, warm["trees"])
    assert sum(use.values()) == n * k * (n - 1)
    cold = fc.fc_construct_trees(n, links, k, options={"tree_warm_start": 2})
    assert cold["trees"] == warm["trees"]
    rng = np.random.default_rng(405)
    samples = [(0, 0), (n - 1, n - 2)] + [(int(rng.integers(0, n)), int(rng.integers(0, n - 1))) for _ in range(10)]
    assert _replay_sampled_states(n, links, k, warm["trees"], samples) >= len(samples)

