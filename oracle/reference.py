"""CPU ORACLE -- TEST INFRASTRUCTURE ONLY (tests, the smoke check and the bench's
`cpu_baseline` leg may use it; the product path never does).

Plain definitions of everything the batched feasibility path outputs, written from
the paper (ForestColl, arXiv 2402.06787):

* F(s, v): max-flow value in the auxiliary network of Section 5.2 / Appendix E.1
  (`aux_network`, `aux_maxflow`), solved by the C routines of `maxflow.c`
  (Dinic, Edmonds-Karp), or by brute-force cut enumeration (`brute_min_cut`).
* the feasibility verdict of Theorem 1 / the integer form after Proposition 3
  (`feasible`).
* 1/x* by the search of Algorithm 1 in exact rational arithmetic (`optimality_binary_search`,
  around `smallest_true_fraction`), or by enumerating every cut of the bound (star) of
  Section 4 (`brute_inv_xstar`).
* (U, k) by the gcd rule of Section 5.2 "Determine k" / Proposition 3 (`smallest_U_k`).
* the non-uniform variant (Section 5.7): source arcs of capacity m_c * k (`weighted_aux_network`,
  `weighted_aux_maxflow_batch`, `weighted_feasible`).
* edge splitting (Appendix E.2): the 2N max-flows and gamma of the maximum-split-off theorem (`split_flows`,
  `split_gamma`), gamma by its definition (`brute_split_gamma`), the split graph (`split_off`), and the loop of
  Algorithm 2 around them (`remove_switches`).
* spanning tree construction (Appendix E.3): mu by one max-flow on the network D-bar (`tree_mu`), mu by its
  definition over all cuts (`brute_tree_mu`), and the construction loop around it (`construct_trees`).
* the fixed-k variant (Section 5.5, Appendix E.4): the verdict on the network with capacities
  floor(U b_e) for a rational U (`fixed_k_feasible`), U* by the search of Algorithm 3 in
  exact rationals (`fixed_k_binary_search`), or by trying every fraction j / b_e
  (`brute_fixed_k`).

Readings of the paper taken here (each also listed in the design notes):
 - Algorithm 1 tests "max-flow is N x"; Theorem 1 says ">= N x".  They are the same
   because s emits at most N x; `feasible` uses >= and asserts <=.
 - s is joined to every compute node including the sink itself, so F >= k.
 - B^-(v) in Algorithm 1 is the in-bandwidth of v in the input graph G (no source
   arc), taken over compute nodes only.
 - a rational candidate 1/x = A/D is tested on integers by uniform scaling
   (Appendix E.1): arc capacities A*b_e, source arcs D, threshold N*D.
 - the final interval is closed: the fraction with denominator <= B may sit on an
   end point (the initial lower bound can equal 1/x*).
 - parallel arcs add up; self-loops and zero-bandwidth arcs carry nothing.
 - if some cut with compute nodes on both sides has no exiting bandwidth the bound
   is infinite (the paper assumes B^+(S) >= 1): `Disconnected` is raised.
 - non-uniform allgather (Section 5.7, last sentence): compute node c sends a weight m_c >= 0 (an
   integer) instead of one unit, the arc (s, c) gets capacity m_c * k, and the verdict is
   F(s, v) >= k * sum_c m_c for every compute node v -- what s emits when all its arcs are full, as
   N k is in the uniform case.  The paper says only that the source arcs are adjusted.
 - spanning tree construction: the arcs (s_i, r) of D-bar are "unbounded"; they get the finite capacity
   sum of all g(e) + sum of the other demands + 1, more than any finite cut.  "Pick an edge" is read as: the
   first edge leaving the root-set in (x, y) order whose mu is positive; root-sets are grown in creation order.
 - fixed k: "link e with bandwidth b_e" is one ordered vertex pair with the summed bandwidth of
   its parallel arcs (`links`); floor(U b_e) is taken per link; max_e b_e (termination width and
   denominator bound of Algorithm 3) is over links; the verdict is F >= N k as in Algorithm 1.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from fractions import Fraction
from math import gcd

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libfc_oracle.so")
_SRC = os.path.join(_HERE, "maxflow.c")
_lib_handle = None

ALGO = {"dinic": 0, "edmonds_karp": 1}
_I64_GUARD = 1 << 62


class Disconnected(Exception):
    """Some compute node cannot reach another one: the bound (star) is infinite."""


def build_c(force: bool = False) -> str:
    """Compile maxflow.c into libfc_oracle.so with gcc -O2 (plain C, pthreads)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        tmp = _SO + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-pthread",
                               "-Wall", "-Wextra", "-o", tmp, _SRC])
        os.replace(tmp, _SO)
    return _SO


def _lib():
    global _lib_handle
    if _lib_handle is None:
        lib = ctypes.CDLL(build_c())
        p32 = ctypes.POINTER(ctypes.c_int32); p64 = ctypes.POINTER(ctypes.c_int64)
        pu8 = ctypes.POINTER(ctypes.c_uint8)
        lib.fco_maxflow.restype = ctypes.c_int64
        lib.fco_maxflow.argtypes = [ctypes.c_int32, ctypes.c_int64, p32, p32, p64,
                                    ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, p64]
        lib.fco_aux_maxflow_batch.restype = ctypes.c_int32
        lib.fco_aux_maxflow_batch.argtypes = [ctypes.c_int32, ctypes.c_int64, p32, p32, p32, pu8,
                                              ctypes.c_int64, p32, p64, p64, p64,
                                              ctypes.c_int32, ctypes.c_int32]
        lib.fco_aux_maxflow_batch_floor.restype = ctypes.c_int32
        lib.fco_aux_maxflow_batch_floor.argtypes = [ctypes.c_int32, ctypes.c_int64, p32, p32, p32, pu8,
                                                    ctypes.c_int64, p32, p64, p64, p64, p64,
                                                    ctypes.c_int32, ctypes.c_int32]
        _lib_handle = lib
    return _lib_handle


def _ptr(a, ty):
    return a.ctypes.data_as(ctypes.POINTER(ty))


# ------------------------------------------------------------------ F(x, y; D)

def maxflow(n_vertices, tail, head, cap, src, dst, algo="dinic", return_arc_flow=False):
    """Value of a maximum src->dst flow in the digraph (tail, head, cap) -- the
    quantity F(x, y; D) of the Appendix E preamble."""
    tail = np.ascontiguousarray(tail, dtype=np.int32)
    head = np.ascontiguousarray(head, dtype=np.int32)
    cap_py = [int(c) for c in np.asarray(cap).reshape(-1)]
    if sum(c for t, c in zip(tail.tolist(), cap_py) if t == src) >= _I64_GUARD:
        raise OverflowError("source out-capacity exceeds the int64 guard")
    cap = np.asarray([min(c, _I64_GUARD) for c in cap_py], dtype=np.int64)
    m = tail.shape[0]
    arc_flow = np.zeros(m, dtype=np.int64) if return_arc_flow else None
    f = _lib().fco_maxflow(int(n_vertices), m, _ptr(tail, ctypes.c_int32), _ptr(head, ctypes.c_int32),
                           _ptr(cap, ctypes.c_int64), int(src), int(dst), ALGO[algo],
                           _ptr(arc_flow, ctypes.c_int64) if return_arc_flow else None)
    if f < 0:
        raise ValueError("bad arguments to the oracle max-flow")
    return (int(f), arc_flow) if return_arc_flow else int(f)


def aux_network(topo, U, k):
    """Auxiliary network of Section 5.2 on integers: vertices V + {s}, s = n_vertices;
    arc e with capacity U*b_e; arc (s, c) with capacity k for every compute node c."""
    comp = np.flatnonzero(topo.is_compute).astype(np.int32)
    s = topo.n_vertices
    tail = np.concatenate([topo.tail.astype(np.int32), np.full(comp.shape[0], s, dtype=np.int32)])
    head = np.concatenate([topo.head.astype(np.int32), comp])
    cap = [int(U) * int(b) for b in topo.bandwidth.tolist()] + [int(k)] * comp.shape[0]
    return topo.n_vertices + 1, tail, head, cap, s


def aux_maxflow(topo, sink, U, k, algo="dinic"):
    """F(s, sink) in the auxiliary network with edge multiplier U and source arcs k."""
    n, tail, head, cap, s = aux_network(topo, U, k)
    return maxflow(n, tail, head, cap, s, int(sink), algo)


def aux_maxflow_batch(topo, sink, U, k, algo="dinic", threads=1):
    """F(s, sink_j) for every problem j = (sink_j, U_j, k_j); int64 values.
    `threads` > 1 shards the problem list statically over POSIX threads."""
    sink = np.ascontiguousarray(sink, dtype=np.int32)
    U = np.ascontiguousarray(U, dtype=np.int64)
    k = np.ascontiguousarray(k, dtype=np.int64)
    P = sink.shape[0]
    assert U.shape[0] == P and k.shape[0] == P
    if P == 0:
        return np.zeros(0, dtype=np.int64)
    if sink.min() < 0 or sink.max() >= topo.n_vertices or U.min() < 0 or k.min() < 0:
        raise ValueError("bad problem list")
    max_b = int(topo.bandwidth.max()) if topo.n_arcs else 0
    if int(U.max()) * max_b >= _I64_GUARD or int(k.max()) * topo.n_compute >= _I64_GUARD:
        raise OverflowError("capacities exceed the int64 guard")
    tail = np.ascontiguousarray(topo.tail, dtype=np.int32)
    head = np.ascontiguousarray(topo.head, dtype=np.int32)
    bw = np.ascontiguousarray(topo.bandwidth, dtype=np.int32)
    isc = np.ascontiguousarray(topo.is_compute, dtype=np.uint8)
    out = np.full(P, -1, dtype=np.int64)
    rc = _lib().fco_aux_maxflow_batch(topo.n_vertices, topo.n_arcs, _ptr(tail, ctypes.c_int32),
                                      _ptr(head, ctypes.c_int32), _ptr(bw, ctypes.c_int32),
                                      _ptr(isc, ctypes.c_uint8), P, _ptr(sink, ctypes.c_int32),
                                      _ptr(U, ctypes.c_int64), _ptr(k, ctypes.c_int64),
                                      _ptr(out, ctypes.c_int64), ALGO[algo], int(threads))
    if rc != 0 or (out < 0).any():
        raise RuntimeError("oracle batch failed")
    return out


# ------------------------------------------------------------------ non-uniform source capacities (Section 5.7)

def _compute_weights(topo, weights):
    """weights: one nonnegative integer per vertex (entries of switches are ignored)."""
    wts = [int(x) for x in np.asarray(weights).tolist()]
    if len(wts) != topo.n_vertices or any(x < 0 for x in wts):
        raise ValueError("weights: one nonnegative integer per vertex")
    return [wts[v] if topo.is_compute[v] else 0 for v in range(topo.n_vertices)]


def weighted_aux_network(topo, U, k, weights, U_den=1):
    """The auxiliary network when compute node c sends m_c = weights[c] units instead of one: arc e
    with capacity floor(U * b_e / U_den), arc (s, c) with capacity m_c * k for every compute node c."""
    wts = _compute_weights(topo, weights)
    comp = np.flatnonzero(topo.is_compute).astype(np.int32)
    s = topo.n_vertices
    tail = np.concatenate([topo.tail.astype(np.int32), np.full(comp.shape[0], s, dtype=np.int32)])
    head = np.concatenate([topo.head.astype(np.int32), comp])
    cap = [int(U) * int(b) // int(U_den) for b in topo.bandwidth.tolist()] + [wts[int(c)] * int(k) for c in comp.tolist()]
    return topo.n_vertices + 1, tail, head, cap, s


def weighted_aux_maxflow_batch(topo, sink, U, k, weights, U_den=None, algo="dinic"):
    """F(s, sink_j) in the weighted auxiliary network for every problem j = (sink_j, U_j [/ U_den_j], k_j).
    With U_den the capacities are floor(U_j b_e / U_den_j) per arc (the caller passes merged links when the
    floor is to be taken per link)."""
    sink = np.asarray(sink).tolist(); U = np.asarray(U).tolist(); k = np.asarray(k).tolist()
    den = [1] * len(sink) if U_den is None else np.asarray(U_den).tolist()
    out = np.zeros(len(sink), dtype=np.int64)
    for j in range(len(sink)):
        n, tail, head, cap, s = weighted_aux_network(topo, U[j], k[j], weights, den[j])
        out[j] = maxflow(n, tail, head, cap, s, int(sink[j]), algo)
    return out


def weighted_feasible(topo, U, k, weights, algo="dinic"):
    """Verdict of the non-uniform variant: min over compute nodes v of F(s, v) >= k * sum_c m_c.
    Returns (verdict, flows)."""
    wts = _compute_weights(topo, weights)
    comp = np.flatnonzero(topo.is_compute).astype(np.int32)
    flows = weighted_aux_maxflow_batch(topo, comp, [int(U)] * len(comp), [int(k)] * len(comp), weights, None, algo)
    need = int(k) * sum(wts)
    assert (flows <= need).all(), "s cannot emit more than k * sum of the weights"
    return bool((flows >= need).all()), flows


# ------------------------------------------------------------------ verdict (Theorem 1 / Theorem 3)

def feasible(topo, U, k, algo="dinic", threads=1):
    """Candidate 1/x = U/k is feasible iff min over compute nodes v of F(s, v) >= N*k.
    Returns (verdict, flows) with flows[i] = F(s, i-th compute node)."""
    comp = np.flatnonzero(topo.is_compute).astype(np.int32)
    N = comp.shape[0]
    flows = aux_maxflow_batch(topo, comp, np.full(N, int(U), dtype=np.int64),
                              np.full(N, int(k), dtype=np.int64), algo, threads)
    assert (flows <= N * int(k)).all(), "s cannot emit more than N*k"
    return bool((flows >= N * int(k)).all()), flows


# ------------------------------------------------------------------ Algorithm 1, literally

def in_bandwidths(topo):
    """B^-_G(v) for every vertex: total bandwidth of arcs entering v from other vertices."""
    B = [0] * topo.n_vertices
    for t, h, b in zip(topo.tail.tolist(), topo.head.tolist(), topo.bandwidth.tolist()):
        if t != h:
            B[h] += int(b)
    return B


def min_compute_in_bandwidth(topo):
    B = in_bandwidths(topo)
    return min(B[v] for v in range(topo.n_vertices) if topo.is_compute[v])


def fraction_in_interval(l: Fraction, r: Fraction, max_den: int) -> Fraction:
    """The fraction p/q in the closed interval [l, r] with q <= max_den, by brute force over denominators.
    It must be unique (two different fractions with denominators <= max_den are at least 1 / max_den^2 apart,
    Proposition 2)."""
    found = set()
    for q in range(1, max_den + 1):
        p_lo = -((-l.numerator * q) // l.denominator)      # ceil(l*q)
        p_hi = (r.numerator * q) // r.denominator           # floor(r*q)
        for p in range(p_lo, p_hi + 1):
            found.add(Fraction(p, q))
    if len(found) != 1:
        raise AssertionError(f"expected exactly one fraction in [{l}, {r}] with q <= {max_den}: {sorted(found)}")
    return found.pop()


def smallest_true_fraction(verdict, below: Fraction, above: Fraction, max_den: int, note=None) -> Fraction:
    """The threshold of a monotone verdict when that threshold is known to be a fraction with denominator
    <= max_den inside [below, above]: verdict(z) is False for z under the threshold and True from it on,
    `above` is known to be True.  The bracket is halved in exact rationals -- the lower end only ever moves to
    a False point, the upper end to a True point, so the threshold stays inside -- until it is narrower than
    the gap 1 / max_den^2 between two such fractions (Proposition 2); the threshold is then the only such
    fraction the closed bracket holds.  This is the search of Algorithm 1 and of Algorithm 3; what differs
    between them is the verdict, the range and the denominator bound.  `note(z, verdict)` sees every test."""
    lo, hi = Fraction(below), Fraction(above)
    gap = Fraction(1, max_den * max_den)
    halvings = 0
    while hi - lo >= gap:
        z = (lo + hi) / 2
        ok = bool(verdict(z))
        if note is not None:
            note(z, ok)
        lo, hi = (lo, z) if ok else (z, hi)
        halvings += 1
    return fraction_in_interval(lo, hi, max_den), halvings


def optimality_binary_search(topo, algo="dinic", threads=1, log=None):
    """1/x* as a Fraction, by the search of Algorithm 1 in exact rationals.  Theorem 1: a candidate 1/x is at
    or above 1/x* exactly when every compute node receives N x from s in the auxiliary network; Appendix E.1:
    1/x* lies in [(N-1)/B, N-1] and its denominator is at most B = min over compute nodes of B^-(v).  A
    candidate A/D is tested on integers (capacities A b_e, source arcs D).  `log`, if a list, receives
    (A, D, verdict) for every candidate tested and a final ("rounds", count, None)."""
    N = topo.n_compute
    if N < 2:
        raise ValueError("need at least two compute nodes")
    B = min_compute_in_bandwidth(topo)
    if B < 1 or not feasible(topo, N - 1, 1, algo, threads)[0]:
        raise Disconnected()
    note = None if log is None else (lambda z, ok: log.append((z.numerator, z.denominator, ok)))
    result, rounds = smallest_true_fraction(lambda z: feasible(topo, z.numerator, z.denominator, algo, threads)[0],
                                            Fraction(N - 1, B), Fraction(N - 1), B, note)
    if log is not None:
        log.append(("rounds", rounds, None))
    return result


def smallest_U_k(inv_xstar: Fraction, bandwidths):
    """Proposition 3: with 1/x* = p/q in lowest terms, g = gcd(q, {b_e}):
    U = p/g (a rational), k = q/g (an integer)."""
    p, q = inv_xstar.numerator, inv_xstar.denominator
    g = q
    for b in bandwidths:
        if int(b) > 0:
            g = gcd(g, int(b))
    return Fraction(p, g), q // g


# ------------------------------------------------------------------ fixed k (Section 5.5, Appendix E.4, Algorithm 3)

def links(topo):
    """The links of the topology: one per ordered vertex pair, its bandwidth the sum over the
    listed arcs of that pair (an integer bandwidth stands for that many unit multi-edges,
    Appendix E.1, so parallel arcs are one link); self-loops and zero bandwidths dropped.
    Flooring is per link, so this has to happen before it."""
    acc = {}
    for t, h, b in zip(topo.tail.tolist(), topo.head.tolist(), topo.bandwidth.tolist()):
        if t != h and b > 0:
            acc[(t, h)] = acc.get((t, h), 0) + int(b)
    keys = sorted(acc)
    tail = np.array([t for t, _ in keys], dtype=np.int32)
    head = np.array([h for _, h in keys], dtype=np.int32)
    bw = np.array([acc[key] for key in keys], dtype=np.int32)
    return tail, head, bw


def aux_maxflow_batch_floor(topo, sink, U_num, U_den, k, algo="dinic", threads=1):
    """F(s, sink_j) in the network of the fixed-k test: problem j has the rational
    multiplier U_j = U_num_j / U_den_j, every link e gets capacity floor(U_j * b_e)
    and every arc (s, c) capacity k_j.  int64 values."""
    sink = np.ascontiguousarray(sink, dtype=np.int32)
    U_num = np.ascontiguousarray(U_num, dtype=np.int64)
    U_den = np.ascontiguousarray(U_den, dtype=np.int64)
    k = np.ascontiguousarray(k, dtype=np.int64)
    P = sink.shape[0]
    assert U_num.shape[0] == P and U_den.shape[0] == P and k.shape[0] == P
    if P == 0:
        return np.zeros(0, dtype=np.int64)
    if sink.min() < 0 or sink.max() >= topo.n_vertices or U_num.min() < 0 or U_den.min() < 1 or k.min() < 0:
        raise ValueError("bad problem list")
    max_b = int(topo.bandwidth.max()) if topo.n_arcs else 0
    if int(U_num.max()) * max_b >= _I64_GUARD or int(k.max()) * topo.n_compute >= _I64_GUARD:
        raise OverflowError("capacities exceed the int64 guard")
    tail, head, bw = links(topo)
    isc = np.ascontiguousarray(topo.is_compute, dtype=np.uint8)
    out = np.full(P, -1, dtype=np.int64)
    rc = _lib().fco_aux_maxflow_batch_floor(topo.n_vertices, tail.shape[0], _ptr(tail, ctypes.c_int32),
                                            _ptr(head, ctypes.c_int32), _ptr(bw, ctypes.c_int32),
                                            _ptr(isc, ctypes.c_uint8), P, _ptr(sink, ctypes.c_int32),
                                            _ptr(U_num, ctypes.c_int64), _ptr(U_den, ctypes.c_int64),
                                            _ptr(k, ctypes.c_int64), _ptr(out, ctypes.c_int64),
                                            ALGO[algo], int(threads))
    if rc != 0 or (out < 0).any():
        raise RuntimeError("oracle batch failed")
    return out


def fixed_k_feasible(topo, U: Fraction, k, algo="dinic", threads=1):
    """The test of Algorithm 3 (Theorems 11, 12 of Appendix E.4): with capacities floor(U b_e) and
    source arcs k, is min over compute nodes v of F(s, v) >= N k?  Returns (verdict, flows)."""
    U = Fraction(U)
    comp = np.flatnonzero(topo.is_compute).astype(np.int32)
    N = comp.shape[0]
    flows = aux_maxflow_batch_floor(topo, comp, np.full(N, U.numerator, dtype=np.int64),
                                    np.full(N, U.denominator, dtype=np.int64),
                                    np.full(N, int(k), dtype=np.int64), algo, threads)
    assert (flows <= N * int(k)).all(), "s cannot emit more than N*k"
    return bool((flows >= N * int(k)).all()), flows


def fixed_k_binary_search(topo, k, algo="dinic", threads=1, log=None):
    """U* = 1/y*, the smallest U for which k edge-disjoint out-trees per compute node exist in
    G({floor(U b_e)}) (the communication time is M/(N k) * U*), by the search of Algorithm 3 in exact
    rationals.  Appendix E.4: the verdict is monotone in U, U* lies in [(N-1) k / B, (N-1) k], and some
    U* b_e is an integer, so its denominator is at most the largest link bandwidth.  `log`, if a list,
    receives (U, verdict) per test."""
    N = topo.n_compute
    k = int(k)
    if N < 2 or k < 1:
        raise ValueError("need at least two compute nodes and k >= 1")
    B = min_compute_in_bandwidth(topo)
    if B < 1 or not fixed_k_feasible(topo, Fraction((N - 1) * k), k, algo, threads)[0]:
        raise Disconnected()
    bmax = int(links(topo)[2].max())
    note = None if log is None else (lambda z, ok: log.append((z, ok)))
    return smallest_true_fraction(lambda z: fixed_k_feasible(topo, z, k, algo, threads)[0],
                                  Fraction((N - 1) * k, B), Fraction((N - 1) * k), bmax, note)[0]


def brute_fixed_k(topo, k, algo="dinic"):
    """U* for a fixed k without any search: at U* some U* b_e is an integer (else U* could be
    lowered, Appendix E.4), so U* is the smallest feasible member of { j / b : b a link bandwidth,
    j >= 1 } up to the upper end (N - 1) k of the paper's range.  Small graphs only."""
    N = topo.n_compute
    k = int(k)
    top = (N - 1) * k
    if not fixed_k_feasible(topo, Fraction(top), k, algo)[0]:
        raise Disconnected()
    bws = sorted(set(links(topo)[2].tolist()))
    cands = sorted({Fraction(j, b) for b in bws for j in range(1, top * b + 1)})
    assert len(cands) <= 200000
    for U in cands:                                     # increasing: the first feasible one is U*
        if fixed_k_feasible(topo, U, k, algo)[0]:
            return U
    raise AssertionError("the upper end of the range was feasible")


# ------------------------------------------------------------------ edge splitting (Appendix E.2, the maximum-split-off theorem)

def link_capacities(topo):
    """{(tail, head): bandwidth} over the links."""
    tail, head, bw = links(topo)
    return {(int(t), int(h)): int(b) for t, h, b in zip(tail.tolist(), head.tolist(), bw.tolist())}


def is_eulerian(topo):
    """Every vertex has equal in- and out-capacity (the precondition of the edge-splitting theorems)."""
    bal = [0] * topo.n_vertices
    for (t, h), b in link_capacities(topo).items():
        bal[t] -= b
        bal[h] += b
    return all(x == 0 for x in bal)


def unbounded(topo, k):
    """A finite stand-in for the infinite capacities of the split-off networks: more than every finite
    cut can carry (all link capacities plus all source arcs), so a flow of at least this much means
    an all-infinite path.  Flow values are reported capped at it."""
    return sum(link_capacities(topo).values()) + topo.n_compute * int(k) + 1


def split_flows(topo, k, u, w, t, algo="dinic"):
    """The 2N max-flows of the maximum-split-off theorem (Appendix E.2) for splitting off e = (u, w), f = (w, t) in the integer-capacity
    digraph D = topo (capacities are the link bandwidths).  With s joined to every compute node by k:
      F1[v] = F(u, w; D_k + infinite arcs (u, s), (u, t), (v, w)),
      F2[v] = F(w, t; D_k + infinite arcs (w, s), (u, t), (v, t)),   v over the compute nodes,
    each capped at `unbounded`.  Returns (F1, F2) as int64 arrays in compute-node order."""
    u, w, t, k = int(u), int(w), int(t), int(k)
    cap = link_capacities(topo)
    if (u, w) not in cap or (w, t) not in cap:
        raise ValueError("e = (u, w) and f = (w, t) must be links of the graph")
    comp = [v for v in range(topo.n_vertices) if topo.is_compute[v]]
    s = topo.n_vertices
    INF = unbounded(topo, k)
    base = [(a, b, c) for (a, b), c in sorted(cap.items())] + [(s, c, k) for c in comp]

    def flow(extra, src, dst):
        arcs = base + [(a, b, INF) for a, b in extra if a != b]
        tail = np.array([a for a, _, _ in arcs], dtype=np.int32)
        head = np.array([b for _, b, _ in arcs], dtype=np.int32)
        return min(INF, maxflow(topo.n_vertices + 1, tail, head, [c for _, _, c in arcs], src, dst, algo))

    F1 = np.array([flow([(u, s), (u, t), (v, w)], u, w) for v in comp], dtype=np.int64)
    F2 = np.array([flow([(w, s), (u, t), (v, t)], w, t) for v in comp], dtype=np.int64)
    return F1, F2


def split_gamma(topo, k, u, w, t, algo="dinic"):
    """gamma of the maximum-split-off theorem (Appendix E.2): the most capacity of e = (u, w) and f = (w, t) that can be replaced by a
    direct arc (u, t) while min over compute nodes v of F(s, v) stays >= N k."""
    cap = link_capacities(topo)
    F1, F2 = split_flows(topo, k, u, w, t, algo)
    Nk = topo.n_compute * int(k)
    return int(min(cap[(int(u), int(w))], cap[(int(w), int(t))], int(F1.min()) - Nk, int(F2.min()) - Nk))


def split_off(topo, u, w, t, amount):
    """D^{ef}: `amount` of the capacity of (u, w) and of (w, t) replaced by capacity on (u, t)."""
    from workloads import Topology
    u, w, t, amount = int(u), int(w), int(t), int(amount)
    cap = link_capacities(topo)
    assert 0 <= amount <= min(cap[(u, w)], cap[(w, t)])
    cap[(u, w)] -= amount
    cap[(w, t)] -= amount
    if u != t:                                          # splitting off a detour u -> w -> u just removes it
        cap[(u, t)] = cap.get((u, t), 0) + amount
    keys = sorted(key for key, c in cap.items() if c > 0)
    return Topology(topo.name + "_split", topo.n_vertices, np.array([a for a, _ in keys], dtype=np.int32),
                    np.array([b for _, b in keys], dtype=np.int32), np.array([cap[key] for key in keys], dtype=np.int32),
                    np.array(topo.is_compute, dtype=np.uint8))


def brute_split_gamma(topo, k, u, w, t, algo="dinic"):
    """gamma by its definition: try every amount 0..min(c_e, c_f), split it off, and test Theorem 1's
    condition on the result; the feasible amounts must form a prefix and gamma is the largest."""
    cap = link_capacities(topo)
    top = min(cap[(int(u), int(w))], cap[(int(w), int(t))])
    ok = [feasible(split_off(topo, u, w, t, a), 1, k, algo)[0] for a in range(top + 1)]
    assert ok[0], "the graph itself must satisfy min F(s, v) >= N k"
    best = max(a for a in range(top + 1) if ok[a])
    assert all(ok[: best + 1]), "feasible split amounts form a prefix"
    return best


def remove_switches(topo, k, algo="dinic"):
    """Algorithm 2 (Remove Switch Nodes) on the integer-capacity Eulerian digraph D = topo: for every
    switch w, every egress link f = (w, t) and every ingress link e = (u, w), split off gamma (the maximum-split-off theorem)
    when it is positive.  Switches, egress heads and ingress tails are visited in increasing id order;
    the links of w are listed when the loop over them starts, as in the pseudocode.  Returns (D*, table)
    with D* the resulting compute-only digraph and table[(u, t)][w] the capacity of (u, t) that is
    routed through switch w (the path recovery table)."""
    D = topo
    table = {}
    for w in [v for v in range(topo.n_vertices) if not topo.is_compute[v]]:
        for t in sorted(h for (a, h) in link_capacities(D) if a == w):
            for u in sorted(a for (a, h) in link_capacities(D) if h == w):
                cap = link_capacities(D)
                if (w, t) not in cap:
                    break                                   # f has been used up
                if (u, w) not in cap:
                    continue
                g = split_gamma(D, k, u, w, t, algo)
                if g > 0:
                    D = split_off(D, u, w, t, g)
                    if u != t:
                        table.setdefault((u, t), {})
                        table[(u, t)][w] = table[(u, t)].get(w, 0) + g
            if (w, t) in link_capacities(D):
                raise AssertionError("an egress link of a switch could not be split off completely (the existence theorem of Appendix E.2 promises it can)")
    return D, table


# ------------------------------------------------------------------ spanning tree construction (Appendix E.3)

def tree_mu_network(n, cap, sets, demand, grow, x):
    """The flow network D-bar of Appendix E.3 for growing root-set `grow` from vertex x: the digraph with
    capacities cap[(a, b)] = g(a, b), one extra vertex s_i per root-set i != grow, an arc (x, s_i) of capacity
    m(R_i) and an arc (s_i, r) for every r in R_i that carries anything (capacity: more than every finite cut)."""
    others = [i for i in range(len(sets)) if i != grow]
    inf = sum(cap.values()) + sum(demand[i] for i in others) + 1
    tail, head, c = [], [], []
    for (a, b), g in sorted(cap.items()):
        if g > 0 and a != b:
            tail.append(a); head.append(b); c.append(int(g))
    for j, i in enumerate(others):
        tail.append(x); head.append(n + j); c.append(int(demand[i]))
        for r in sorted(sets[i]):
            tail.append(n + j); head.append(r); c.append(inf)
    return n + len(others), np.array(tail, dtype=np.int32), np.array(head, dtype=np.int32), c


def tree_mu(n, cap, sets, demand, grow, x, y, algo="dinic"):
    """mu for the edge (x, y), x in R_grow, y outside it (Appendix E.3, the theorem that computes mu by one
    max-flow): min{ g(x, y), m(R_grow), F(x, y; D-bar) - sum of m(R_i) over i != grow }."""
    assert x in sets[grow] and y not in sets[grow] and cap.get((x, y), 0) > 0
    nv, tail, head, c = tree_mu_network(n, cap, sets, demand, grow, x)
    F = maxflow(nv, tail, head, c, int(x), int(y), algo)
    return min(int(cap[(x, y)]), int(demand[grow]), F - sum(demand[i] for i in range(len(sets)) if i != grow))


def brute_tree_mu(n, cap, sets, demand, grow, x, y):
    """mu by its definition (Appendix E.3, the formula taken from Berczi and Frank): min of g(x, y), m(R_grow) and
    c(S, V - S) - p(S) over all S with x in S, y not in S, R_grow not inside S, where p(S) adds up m(R_i)
    over the root-sets R_i inside S."""
    assert n <= 14
    best = min(int(cap[(x, y)]), int(demand[grow]))
    masks = [sum(1 << r for r in R) for R in sets]
    for S in range(1 << n):
        if not (S >> x) & 1 or (S >> y) & 1 or (masks[grow] & ~S) == 0:
            continue
        cut = sum(g for (a, b), g in cap.items() if (S >> a) & 1 and not (S >> b) & 1)
        p = sum(demand[i] for i in range(len(sets)) if (masks[i] & ~S) == 0)
        best = min(best, cut - p)
    return best


def construct_trees(n, links, k, algo="dinic", observe=None):
    """Spanning Tree Construction (Appendix E.3) on the compute-only digraph D* = links {(a, b): capacity} over
    vertices 0 .. n-1: every root u starts with R = {u} of multiplicity k; a root-set that does not span yet is
    grown by the first edge (x, y) in (x, y) order that leaves it and has mu > 0; if mu is less than its
    multiplicity a copy keeps the rest.  Root-sets are taken in creation order.  Returns a list of
    (root, multiplicity, edges in the order they were added); the multiplicities of a root add up to k.
    `observe(g, sets, demand, i, x, y, mu)`, if given, sees every mu that is computed."""
    g = {key: int(c) for key, c in links.items() if c > 0 and key[0] != key[1]}
    sets = [{u} for u in range(n)]
    demand = [int(k)] * n
    root = list(range(n))
    edges = [[] for _ in range(n)]
    full = set(range(n))
    while True:
        todo = [i for i in range(len(sets)) if sets[i] != full]
        if not todo:
            break
        i = todo[0]
        while sets[i] != full:
            grown = False
            for (x, y) in sorted(g):
                if x in sets[i] and y not in sets[i]:
                    mu = tree_mu(n, g, sets, demand, i, x, y, algo)
                    if observe is not None:
                        observe(g, sets, demand, i, x, y, mu)
                    if mu == 0:
                        continue
                    assert mu > 0
                    if mu < demand[i]:
                        sets.append(set(sets[i])); demand.append(demand[i] - mu); root.append(root[i])
                        edges.append(list(edges[i])); demand[i] = mu
                    edges[i].append((x, y)); sets[i].add(y)
                    g[(x, y)] -= mu
                    if g[(x, y)] == 0:
                        del g[(x, y)]
                    grown = True
                    break
            if not grown:
                raise AssertionError("no edge leaving the root-set can be added (the packing condition does not hold)")
    return [(root[i], demand[i], edges[i]) for i in range(len(sets))]


# ------------------------------------------------------------------ brute force (tiny graphs only)

def brute_inv_xstar(topo):
    """max over S subset of V, S not containing all compute nodes, of |S n V_c| / B^+(S)
    (the bound (star) of Section 4) by enumerating all 2^|V| subsets.  Raises
    Disconnected when a subset holding a compute node has no exiting bandwidth."""
    n = topo.n_vertices
    assert n <= 16
    arcs = [(t, h, int(b)) for t, h, b in zip(topo.tail.tolist(), topo.head.tolist(),
                                              topo.bandwidth.tolist()) if t != h and b > 0]
    comp_mask = 0
    for v in range(n):
        if topo.is_compute[v]:
            comp_mask |= 1 << v
    best = Fraction(0)
    for S in range(1, 1 << n):
        if S & comp_mask == comp_mask:
            continue                                   # S contains every compute node
        inside = bin(S & comp_mask).count("1")
        if inside == 0:
            continue
        out_bw = sum(b for t, h, b in arcs if (S >> t) & 1 and not (S >> h) & 1)
        if out_bw == 0:
            raise Disconnected()
        best = max(best, Fraction(inside, out_bw))
    return best


def brute_min_cut(n_vertices, tail, head, cap, src, dst):
    """min over vertex sets A containing src and not dst of the capacity leaving A."""
    assert n_vertices <= 16
    arcs = list(zip(np.asarray(tail).tolist(), np.asarray(head).tolist(), [int(c) for c in cap]))
    others = [v for v in range(n_vertices) if v not in (src, dst)]
    best = None
    for bits in range(1 << len(others)):
        A = 1 << src
        for i, v in enumerate(others):
            if (bits >> i) & 1:
                A |= 1 << v
        c = sum(cp for t, h, cp in arcs if (A >> t) & 1 and not (A >> h) & 1)
        best = c if best is None else min(best, c)
    return best


def brute_cut_condition(topo, k):
    """Theorem 8's cut form on a switch-free integer digraph D:
    c(S, complement of S; D) >= |S| * k for every proper non-empty subset S of V."""
    n = topo.n_vertices
    assert n <= 16 and topo.is_compute.all()
    arcs = [(t, h, int(b)) for t, h, b in zip(topo.tail.tolist(), topo.head.tolist(),
                                              topo.bandwidth.tolist()) if t != h]
    for S in range(1, (1 << n) - 1):
        c = sum(b for t, h, b in arcs if (S >> t) & 1 and not (S >> h) & 1)
        if c < bin(S).count("1") * k:
            return False
    return True
