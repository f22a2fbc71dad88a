"""Thin ctypes binding of libfcmaxflow.so: argument marshalling only.

Every function has the name of the C entry point it calls (see include/fc_maxflow.h).
Device buffers are torch tensors on the GPU; torch is used for device memory and streams
only.  There is no CPU fallback: if the shared library is missing, loading fails.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from fractions import Fraction

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libfcmaxflow.so")

FC_OK = 0
FC_EINVAL, FC_EOVERFLOW, FC_EDISCONNECTED, FC_ENOMEM = -1, -2, -3, -4
FC_EWORKSPACE, FC_EDEVICE, FC_ENOCONVERGE, FC_EUNSUPPORTED = -5, -6, -7, -8
FC_FLOW_INVALID, FC_FLOW_NOCONVERGE, FC_FLOW_UNSUPPORTED = -1, -2, -3
FC_GAMMA_INVALID = -2147483648

EXPORTED = ["fc_graph_build", "fc_graph_upload", "fc_graph_upload_with_spares", "fc_graph_update_arcs", "fc_graph_sink_table", "fc_graph_free", "fc_graph_info", "fc_graph_csr", "fc_graph_set_source_weights",
            "fc_maxflow_batch_workspace_bytes", "fc_maxflow_batch", "fc_maxflow_batch_static", "fc_maxflow_batch_floor", "fc_feasible_workspace_bytes",
            "fc_feasible_floor", "fc_fixed_k_search", "fc_fixed_k_search_with_verdicts",
            "fc_split_gamma_workspace_bytes", "fc_split_gamma_batch", "fc_remove_switches", "fc_tree_mu_batch", "fc_construct_trees",
            "fc_feasible", "fc_opt_throughput_search", "fc_search_with_verdicts", "fc_strerror"]


class FcError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


class fc_rational(ctypes.Structure):
    _fields_ = [("num", ctypes.c_int64), ("den", ctypes.c_int64)]


class fc_stats(ctypes.Structure):
    _fields_ = [("pushes", ctypes.c_uint64), ("relabels", ctypes.c_uint64), ("arc_scans", ctypes.c_uint64),
                ("global_relabels", ctypes.c_uint64), ("gr_arc_scans", ctypes.c_uint64),
                ("level_steps", ctypes.c_uint64), ("discharges", ctypes.c_uint64),
                ("not_converged", ctypes.c_uint64), ("device_ms", ctypes.c_float)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class fc_options(ctypes.Structure):
    _fields_ = [("threads_per_problem", ctypes.c_int32), ("lanes_per_vertex", ctypes.c_int32),
                ("global_relabel_steps", ctypes.c_int32), ("global_relabel_permille", ctypes.c_int32),
                ("global_relabel_rises", ctypes.c_int32), ("tight_sink_percent", ctypes.c_int32),
                ("use_gap", ctypes.c_int32), ("use_label_table", ctypes.c_int32),
                ("force_wide", ctypes.c_int32), ("max_level_steps", ctypes.c_int32),
                ("src_cap_bound", ctypes.c_int32), ("tree_certificate", ctypes.c_int32), ("schedule", ctypes.c_int32),
                ("tree_warm_start", ctypes.c_int32), ("split_two_launches", ctypes.c_int32),
                ("stats_time_only", ctypes.c_int32), ("split_carry", ctypes.c_int32), ("split_reverse", ctypes.c_int32), ("tree_chain_states", ctypes.c_int32)]


VERDICT_FN = ctypes.CFUNCTYPE(ctypes.c_int, ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32),
                              ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_uint8))

_lib = None


def load_library():
    """dlopen the in-tree library and declare the C signatures.  Raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is not built; run `python -m paper_2402_06787_amd.build`")
    _ensure_gpu_ready()                                  # before the library (and the HIP runtime it links) is mapped: see there
    lib = ctypes.CDLL(LIB_PATH)
    c = ctypes
    vp, i32, i64, sz = c.c_void_p, c.c_int32, c.c_int64, c.c_size_t
    lib.fc_graph_build.restype = c.c_int
    lib.fc_graph_build.argtypes = [i32, i64, vp, vp, vp, vp, c.POINTER(vp)]
    lib.fc_graph_upload.restype = c.c_int
    lib.fc_graph_upload.argtypes = [i32, i64, vp, vp, vp, vp, c.POINTER(vp)]
    lib.fc_graph_upload_with_spares.restype = c.c_int
    lib.fc_graph_upload_with_spares.argtypes = [i32, i64, vp, vp, vp, vp, c.POINTER(vp)]
    lib.fc_graph_update_arcs.restype = c.c_int
    lib.fc_graph_update_arcs.argtypes = [vp, i64, vp, vp, vp, i32, vp]
    lib.fc_graph_sink_table.restype = c.c_int
    lib.fc_graph_sink_table.argtypes = [vp, i32, c.POINTER(i32), vp, c.POINTER(i32), vp, vp, vp, vp, vp, vp]
    lib.fc_graph_free.restype = c.c_int
    lib.fc_graph_free.argtypes = [vp]
    lib.fc_graph_info.restype = c.c_int
    lib.fc_graph_info.argtypes = [vp, c.POINTER(i32), c.POINTER(i64), c.POINTER(i64), c.POINTER(i32),
                                  c.POINTER(i32), c.POINTER(i32)]
    lib.fc_graph_set_source_weights.restype = c.c_int
    lib.fc_graph_set_source_weights.argtypes = [vp, vp]
    lib.fc_graph_csr.restype = c.c_int
    lib.fc_graph_csr.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.fc_maxflow_batch_workspace_bytes.restype = sz
    lib.fc_maxflow_batch_workspace_bytes.argtypes = [vp, i64]
    lib.fc_maxflow_batch.restype = c.c_int
    lib.fc_maxflow_batch.argtypes = [vp, i64, vp, vp, vp, vp, vp, sz, vp, c.POINTER(fc_options), c.POINTER(fc_stats)]
    lib.fc_maxflow_batch_static.restype = c.c_int
    lib.fc_maxflow_batch_static.argtypes = [vp, i64, vp, vp, vp, vp, vp, c.POINTER(fc_options)]
    lib.fc_feasible_workspace_bytes.restype = sz
    lib.fc_feasible_workspace_bytes.argtypes = [vp, i32]
    lib.fc_feasible.restype = c.c_int
    lib.fc_feasible.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, sz, vp, c.POINTER(fc_options), c.POINTER(fc_stats)]
    lib.fc_opt_throughput_search.restype = c.c_int
    lib.fc_opt_throughput_search.argtypes = [vp, i32, c.POINTER(fc_rational), c.POINTER(fc_rational),
                                             c.POINTER(i64), c.POINTER(i32), vp, c.POINTER(fc_options),
                                             vp, vp, vp, i32, c.POINTER(i32)]
    lib.fc_search_with_verdicts.restype = c.c_int
    lib.fc_search_with_verdicts.argtypes = [i32, i64, i32, i32, VERDICT_FN, vp, c.POINTER(fc_rational),
                                            c.POINTER(fc_rational), c.POINTER(i64), c.POINTER(i32)]
    lib.fc_maxflow_batch_floor.restype = c.c_int
    lib.fc_maxflow_batch_floor.argtypes = [vp, i64, vp, vp, vp, vp, vp, vp, sz, vp, c.POINTER(fc_options), c.POINTER(fc_stats)]
    lib.fc_feasible_floor.restype = c.c_int
    lib.fc_feasible_floor.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp, c.POINTER(fc_options), c.POINTER(fc_stats)]
    lib.fc_fixed_k_search.restype = c.c_int
    lib.fc_fixed_k_search.argtypes = [vp, i32, i32, c.POINTER(fc_rational), c.POINTER(i32), vp, c.POINTER(fc_options),
                                      vp, vp, vp, i32, c.POINTER(i32)]
    lib.fc_fixed_k_search_with_verdicts.restype = c.c_int
    lib.fc_fixed_k_search_with_verdicts.argtypes = [i32, i64, i32, i32, i32, VERDICT_FN, vp, c.POINTER(fc_rational),
                                                    c.POINTER(i32)]
    lib.fc_split_gamma_workspace_bytes.restype = sz
    lib.fc_split_gamma_workspace_bytes.argtypes = [vp, i64]
    lib.fc_split_gamma_batch.restype = c.c_int
    lib.fc_split_gamma_batch.argtypes = [vp, i32, i32, i64, vp, vp, vp, vp, vp, vp, sz, vp, c.POINTER(fc_options), c.POINTER(fc_stats)]
    lib.fc_tree_mu_batch.restype = c.c_int
    lib.fc_tree_mu_batch.argtypes = [i32, i64, vp, vp, vp, i32, vp, vp, vp, i32, i64, vp, vp, vp, vp, vp, c.POINTER(fc_options)]
    lib.fc_construct_trees.restype = c.c_int
    lib.fc_construct_trees.argtypes = [i32, i64, vp, vp, vp, i32, i64, c.POINTER(i64), vp, vp, vp, vp, c.POINTER(i64), vp, c.POINTER(fc_options)]
    lib.fc_remove_switches.restype = c.c_int
    lib.fc_remove_switches.argtypes = [i32, i64, vp, vp, vp, vp, i32, i64, c.POINTER(i64), vp, vp, vp,
                                       i64, c.POINTER(i64), vp, vp, vp, vp, c.POINTER(i64), vp, c.POINTER(fc_options)]
    lib.fc_strerror.restype = c.c_char_p
    lib.fc_strerror.argtypes = [c.c_int]
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load_library().fc_strerror(int(code)).decode()


def _check(code: int, where: str):
    if code != FC_OK:
        raise FcError(code, where)


def _np(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def _host_ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None and a.size else None


def _opts(options):
    if options is None:
        return None
    if isinstance(options, fc_options):
        return ctypes.byref(options)
    o = fc_options()
    for key, val in dict(options).items():
        setattr(o, key, int(val))
    return ctypes.byref(o)


@dataclass
class GraphInfo:
    n_compute: int
    n_arcs_merged: int
    min_in_bw_compute: int
    max_bw: int
    gcd_bw: int
    is_eulerian: bool


class Graph:
    """Owns an fc_graph handle; freed on `close()` or garbage collection."""

    def __init__(self, handle: int, n_vertices: int):
        self.handle = ctypes.c_void_p(handle)
        self.n_vertices = n_vertices

    def close(self):
        if self.handle:
            load_library().fc_graph_free(self.handle)
            self.handle = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


def _graph_call(fn_name, n_vertices, tail, head, bandwidth, is_compute) -> Graph:
    lib = load_library()
    tail = _np(tail, np.int32); head = _np(head, np.int32); bandwidth = _np(bandwidth, np.int32)
    is_compute = _np(is_compute, np.uint8)
    if not (tail.shape == head.shape == bandwidth.shape) or tail.ndim != 1:
        raise ValueError("tail, head, bandwidth must be 1-d arrays of equal length")
    if is_compute.shape != (int(n_vertices),):
        raise ValueError("is_compute must have n_vertices entries")
    out = ctypes.c_void_p(None)
    rc = getattr(lib, fn_name)(int(n_vertices), int(tail.shape[0]), _host_ptr(tail), _host_ptr(head),
                               _host_ptr(bandwidth), _host_ptr(is_compute), ctypes.byref(out))
    _check(rc, fn_name)
    return Graph(out.value, int(n_vertices))


def fc_graph_build(n_vertices, tail, head, bandwidth, is_compute) -> Graph:
    return _graph_call("fc_graph_build", n_vertices, tail, head, bandwidth, is_compute)


def fc_graph_upload(n_vertices, tail, head, bandwidth, is_compute) -> Graph:
    return _graph_call("fc_graph_upload", n_vertices, tail, head, bandwidth, is_compute)


def fc_graph_upload_with_spares(n_vertices, tail, head, bandwidth, is_compute) -> Graph:
    """fc_graph_upload, except that an arc of bandwidth 0 becomes a link that carries nothing yet."""
    return _graph_call("fc_graph_upload_with_spares", n_vertices, tail, head, bandwidth, is_compute)


def fc_graph_update_arcs(g: Graph, tail, head, bandwidth, refresh_tables: bool = True, stream=None) -> None:
    """Give the existing links (tail[i], head[i]) the bandwidths bandwidth[i], in place (host arrays)."""
    tail = _np(tail, np.int32); head = _np(head, np.int32); bandwidth = _np(bandwidth, np.int32)
    if not (tail.shape == head.shape == bandwidth.shape) or tail.ndim != 1:
        raise ValueError("tail, head, bandwidth must be 1-d arrays of equal length")
    _check(load_library().fc_graph_update_arcs(g.handle, int(tail.shape[0]), _host_ptr(tail), _host_ptr(head), _host_ptr(bandwidth),
                                               1 if refresh_tables else 0, _stream_ptr_for_host_call(stream)),
           "fc_graph_update_arcs")


def fc_graph_sink_table(g: Graph, sink: int) -> dict:
    """The per-sink tables the device holds for `sink` (see the header): dict with `have`, and when present `label`,
    `label_hmax`, `level_table`, `order_vertex`, `first_head`, `first_pair`, `first_bw`, `ratio`."""
    n = g.n_vertices
    have, hmax = ctypes.c_int32(0), ctypes.c_int32(0)
    label = np.zeros(n, np.int32); lt = np.zeros(64, np.int32); ratio = np.zeros(2, np.int32)
    ov, fh, fp, fb = (np.zeros(n, np.int32) for _ in range(4))
    _check(load_library().fc_graph_sink_table(g.handle, int(sink), ctypes.byref(have), _host_ptr(label), ctypes.byref(hmax), _host_ptr(lt),
                                              _host_ptr(ov), _host_ptr(fh), _host_ptr(fp), _host_ptr(fb), _host_ptr(ratio)),
           "fc_graph_sink_table")
    out = {"have": have.value}
    if have.value & 1:
        out.update(label=label, label_hmax=hmax.value)
    if have.value & 2:
        out.update(level_table=lt, order_vertex=ov, first_head=fh, first_pair=fp, first_bw=fb, ratio=(int(ratio[0]), int(ratio[1])))
    return out


def fc_graph_info(g: Graph) -> GraphInfo:
    c = ctypes
    nc, m, mb, mx, gc, eu = c.c_int32(), c.c_int64(), c.c_int64(), c.c_int32(), c.c_int32(), c.c_int32()
    _check(load_library().fc_graph_info(g.handle, c.byref(nc), c.byref(m), c.byref(mb), c.byref(mx),
                                        c.byref(gc), c.byref(eu)), "fc_graph_info")
    return GraphInfo(nc.value, m.value, mb.value, mx.value, gc.value, bool(eu.value))


def fc_graph_set_source_weights(g: Graph, weights) -> None:
    """weights: one nonnegative integer per vertex (host array), or None for unit weights."""
    lib = load_library()
    if weights is None:
        _check(lib.fc_graph_set_source_weights(g.handle, None), "fc_graph_set_source_weights")
        return
    wts = _np(weights, np.int32)
    if wts.shape[0] != g.n_vertices:
        raise ValueError("weights: one entry per vertex")
    _check(lib.fc_graph_set_source_weights(g.handle, _host_ptr(wts)), "fc_graph_set_source_weights")


def fc_graph_csr(g: Graph):
    info = fc_graph_info(g)
    M = 2 * info.n_arcs_merged
    row_ptr = np.zeros(g.n_vertices + 1, np.int32)
    other = np.zeros(M, np.int32); pair = np.zeros(M, np.int32); bw = np.zeros(M, np.int32)
    fwd = np.zeros(M, np.uint8)
    _check(load_library().fc_graph_csr(g.handle, _host_ptr(row_ptr), _host_ptr(other), _host_ptr(pair),
                                       _host_ptr(bw), _host_ptr(fwd)), "fc_graph_csr")
    return row_ptr, other, pair, bw, fwd


# ------------------------------------------------------------------ device calls (torch tensors)

def _dev_ptr(t, dtype, n, name):
    import torch
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != dtype or not t.is_contiguous() or t.numel() < n:
        raise ValueError(f"{name}: need a contiguous {dtype} device tensor with at least {n} elements")
    return ctypes.c_void_p(t.data_ptr())


_gpu_ready = False


def _ensure_gpu_ready():
    """The library links the system HIP runtime, torch brings one of its own, and a process that uses both holds both.
    When the library's runtime is mapped before torch has put anything on the device, its first hipMalloc has been seen
    to report that there is no device (torch's runtime then comes up second and the two do not agree on the device).  So
    torch's side is brought up -- one allocation -- before the library is loaded; torch is what provides device memory to
    this binding anyway.  Without a GPU nothing is done and the library reports FC_EDEVICE by itself."""
    global _gpu_ready
    if not _gpu_ready:
        import torch
        if not torch.cuda.is_available():                 # (without a GPU the library reports FC_EDEVICE by itself)
            return
        torch.cuda.init()
        torch.empty(1, device="cuda")
        torch.cuda.synchronize()
        _gpu_ready = True


def _stream_ptr(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _stream_ptr_for_host_call(stream):
    """For the entry points that take host arrays and validate them before any device call: without a GPU the
    default stream is passed as null, so that what they reject is still reported as such (and everything else
    fails in the library with FC_EDEVICE)."""
    import torch
    if stream is None and not torch.cuda.is_available():
        return ctypes.c_void_p(0)
    return _stream_ptr(stream)


def fc_maxflow_batch_workspace_bytes(g: Graph, n_problems: int) -> int:
    return int(load_library().fc_maxflow_batch_workspace_bytes(g.handle, int(n_problems)))


def fc_maxflow_batch(g: Graph, d_sink, d_edge_mult, d_src_cap, d_flow_out=None, d_workspace=None,
                     stream=None, options=None, want_stats=False):
    """Returns (d_flow_out, stats dict or None).  Allocates outputs/workspace with torch if not given."""
    import torch
    P = int(d_sink.numel())
    if d_flow_out is None:
        d_flow_out = torch.empty(P, dtype=torch.int32, device=d_sink.device)
    need = fc_maxflow_batch_workspace_bytes(g, P)
    if d_workspace is None:
        d_workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=d_sink.device)
    st = fc_stats() if want_stats else None
    rc = load_library().fc_maxflow_batch(
        g.handle, P, _dev_ptr(d_sink, torch.int32, P, "d_sink"), _dev_ptr(d_edge_mult, torch.int32, P, "d_edge_mult"),
        _dev_ptr(d_src_cap, torch.int32, P, "d_src_cap"), _dev_ptr(d_flow_out, torch.int32, P, "d_flow_out"),
        ctypes.c_void_p(d_workspace.data_ptr()), d_workspace.numel(), _stream_ptr(stream), _opts(options),
        ctypes.byref(st) if st is not None else None)
    _check(rc, "fc_maxflow_batch")
    return d_flow_out, (st.as_dict() if st is not None else None)


FC_MAXFLOW_BATCH_STATIC_MAX_PROBLEMS = 262144


def fc_maxflow_batch_static(g: Graph, d_sink, d_edge_mult, d_src_cap, d_flow_out, stream=None, options=None):
    """fc_maxflow_batch without a workspace: the library's static device array holds the scratch.  The caller
    passes every buffer; nothing is allocated here or in the library.  Returns d_flow_out."""
    import torch
    P = int(d_sink.numel())
    rc = load_library().fc_maxflow_batch_static(
        g.handle, P, _dev_ptr(d_sink, torch.int32, P, "d_sink"), _dev_ptr(d_edge_mult, torch.int32, P, "d_edge_mult"),
        _dev_ptr(d_src_cap, torch.int32, P, "d_src_cap"), _dev_ptr(d_flow_out, torch.int32, P, "d_flow_out"),
        _stream_ptr(stream), _opts(options))
    _check(rc, "fc_maxflow_batch_static")
    return d_flow_out


def fc_feasible_workspace_bytes(g: Graph, n_candidates: int) -> int:
    return int(load_library().fc_feasible_workspace_bytes(g.handle, int(n_candidates)))


def fc_feasible(g: Graph, d_edge_mult, d_src_cap, want_flows=False, want_witness=True, d_workspace=None,
                stream=None, options=None, want_stats=False):
    """Returns dict(feasible=uint8 tensor, witness=int32 tensor|None, flows=int32 [C, N]|None, stats)."""
    import torch
    C = int(d_edge_mult.numel())
    dev = d_edge_mult.device
    N = fc_graph_info(g).n_compute
    feas = torch.empty(C, dtype=torch.uint8, device=dev)
    wit = torch.empty(C, dtype=torch.int32, device=dev) if want_witness else None
    flows = torch.empty(C * N, dtype=torch.int32, device=dev) if want_flows else None
    need = fc_feasible_workspace_bytes(g, C)
    if d_workspace is None:
        d_workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    st = fc_stats() if want_stats else None
    rc = load_library().fc_feasible(
        g.handle, C, _dev_ptr(d_edge_mult, torch.int32, C, "d_edge_mult"), _dev_ptr(d_src_cap, torch.int32, C, "d_src_cap"),
        _dev_ptr(feas, torch.uint8, C, "feasible"), _dev_ptr(wit, torch.int32, C, "witness"),
        _dev_ptr(flows, torch.int32, C * N, "flows"), ctypes.c_void_p(d_workspace.data_ptr()), d_workspace.numel(),
        _stream_ptr(stream), _opts(options), ctypes.byref(st) if st is not None else None)
    _check(rc, "fc_feasible")
    return {"feasible": feas, "witness": wit, "flows": flows.view(C, N) if flows is not None else None,
            "stats": st.as_dict() if st is not None else None}


def fc_opt_throughput_search(g: Graph, candidates_per_round: int = 16, stream=None, options=None,
                             trace_capacity: int = 4096):
    """Returns dict(inv_xstar=Fraction, U=Fraction, k=int, rounds=int, trace=[(U, k, verdict), ...])."""
    c = ctypes
    r1, r2, kk, rounds, tlen = fc_rational(), fc_rational(), c.c_int64(), c.c_int32(), c.c_int32()
    tU = np.zeros(trace_capacity, np.int32); tk = np.zeros(trace_capacity, np.int32)
    tv = np.zeros(trace_capacity, np.uint8)
    rc = load_library().fc_opt_throughput_search(
        g.handle, int(candidates_per_round), c.byref(r1), c.byref(r2), c.byref(kk), c.byref(rounds),
        _stream_ptr(stream), _opts(options), _host_ptr(tU), _host_ptr(tk), _host_ptr(tv), trace_capacity, c.byref(tlen))
    _check(rc, "fc_opt_throughput_search")
    nt = min(tlen.value, trace_capacity)
    return {"inv_xstar": Fraction(r1.num, r1.den), "U": Fraction(r2.num, r2.den), "k": int(kk.value),
            "rounds": int(rounds.value), "trace": [(int(tU[i]), int(tk[i]), int(tv[i])) for i in range(nt)],
            "trace_len": int(tlen.value)}


def fc_search_with_verdicts(n_compute: int, min_in_bw: int, gcd_bw: int, candidates_per_round: int, verdict_fn):
    """Host-only search logic.  `verdict_fn(list of (U, k))` returns a list of 0/1 verdicts
    (or raises); returns dict(inv_xstar, U, k, rounds)."""
    c = ctypes
    err = []

    def _cb(_ctx, n, pU, pk, pout):
        try:
            res = verdict_fn([(int(pU[i]), int(pk[i])) for i in range(n)])
            for i in range(n):
                pout[i] = 1 if res[i] else 0
            return FC_OK
        except Exception as exc:            # never let an exception cross the C boundary
            err.append(exc)
            return FC_EINVAL

    cb = VERDICT_FN(_cb)
    r1, r2, kk, rounds = fc_rational(), fc_rational(), c.c_int64(), c.c_int32()
    rc = load_library().fc_search_with_verdicts(int(n_compute), int(min_in_bw), int(gcd_bw), int(candidates_per_round),
                                               cb, None, c.byref(r1), c.byref(r2), c.byref(kk), c.byref(rounds))
    if err:
        raise err[0]
    _check(rc, "fc_search_with_verdicts")
    return {"inv_xstar": Fraction(r1.num, r1.den), "U": Fraction(r2.num, r2.den), "k": int(kk.value),
            "rounds": int(rounds.value)}


# ------------------------------------------------------------------ fixed k (rational multipliers, floor capacities)

def fc_maxflow_batch_floor(g: Graph, d_sink, d_mult_num, d_mult_den, d_src_cap, d_flow_out=None, d_workspace=None,
                           stream=None, options=None, want_stats=False):
    """fc_maxflow_batch with the rational multiplier num/den per problem.  Returns (d_flow_out, stats or None)."""
    import torch
    P = int(d_sink.numel())
    if d_flow_out is None:
        d_flow_out = torch.empty(P, dtype=torch.int32, device=d_sink.device)
    need = fc_maxflow_batch_workspace_bytes(g, P)
    if d_workspace is None:
        d_workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=d_sink.device)
    st = fc_stats() if want_stats else None
    rc = load_library().fc_maxflow_batch_floor(
        g.handle, P, _dev_ptr(d_sink, torch.int32, P, "d_sink"), _dev_ptr(d_mult_num, torch.int32, P, "d_mult_num"),
        _dev_ptr(d_mult_den, torch.int32, P, "d_mult_den"), _dev_ptr(d_src_cap, torch.int32, P, "d_src_cap"),
        _dev_ptr(d_flow_out, torch.int32, P, "d_flow_out"), ctypes.c_void_p(d_workspace.data_ptr()), d_workspace.numel(),
        _stream_ptr(stream), _opts(options), ctypes.byref(st) if st is not None else None)
    _check(rc, "fc_maxflow_batch_floor")
    return d_flow_out, (st.as_dict() if st is not None else None)


def fc_feasible_floor(g: Graph, d_mult_num, d_mult_den, d_src_cap, want_flows=False, want_witness=True, d_workspace=None,
                      stream=None, options=None, want_stats=False):
    """fc_feasible with the rational multiplier num/den per candidate; same result dict."""
    import torch
    C = int(d_mult_num.numel())
    dev = d_mult_num.device
    N = fc_graph_info(g).n_compute
    feas = torch.empty(C, dtype=torch.uint8, device=dev)
    wit = torch.empty(C, dtype=torch.int32, device=dev) if want_witness else None
    flows = torch.empty(C * N, dtype=torch.int32, device=dev) if want_flows else None
    need = fc_feasible_workspace_bytes(g, C)
    if d_workspace is None:
        d_workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    st = fc_stats() if want_stats else None
    rc = load_library().fc_feasible_floor(
        g.handle, C, _dev_ptr(d_mult_num, torch.int32, C, "d_mult_num"), _dev_ptr(d_mult_den, torch.int32, C, "d_mult_den"),
        _dev_ptr(d_src_cap, torch.int32, C, "d_src_cap"), _dev_ptr(feas, torch.uint8, C, "feasible"),
        _dev_ptr(wit, torch.int32, C, "witness"), _dev_ptr(flows, torch.int32, C * N, "flows"),
        ctypes.c_void_p(d_workspace.data_ptr()), d_workspace.numel(), _stream_ptr(stream), _opts(options),
        ctypes.byref(st) if st is not None else None)
    _check(rc, "fc_feasible_floor")
    return {"feasible": feas, "witness": wit, "flows": flows.view(C, N) if flows is not None else None,
            "stats": st.as_dict() if st is not None else None}


def fc_fixed_k_search(g: Graph, k: int, candidates_per_round: int = 16, stream=None, options=None,
                      trace_capacity: int = 4096):
    """Returns dict(U_star=Fraction, rounds=int, trace=[(num, den, verdict), ...])."""
    c = ctypes
    r, rounds, tlen = fc_rational(), c.c_int32(), c.c_int32()
    tn = np.zeros(trace_capacity, np.int32); td = np.zeros(trace_capacity, np.int32)
    tv = np.zeros(trace_capacity, np.uint8)
    rc = load_library().fc_fixed_k_search(
        g.handle, int(k), int(candidates_per_round), c.byref(r), c.byref(rounds), _stream_ptr(stream), _opts(options),
        _host_ptr(tn), _host_ptr(td), _host_ptr(tv), trace_capacity, c.byref(tlen))
    _check(rc, "fc_fixed_k_search")
    nt = min(tlen.value, trace_capacity)
    return {"U_star": Fraction(r.num, r.den), "rounds": int(rounds.value),
            "trace": [(int(tn[i]), int(td[i]), int(tv[i])) for i in range(nt)], "trace_len": int(tlen.value)}


def fc_fixed_k_search_with_verdicts(n_compute: int, min_in_bw: int, max_bw: int, k: int, candidates_per_round: int,
                                    verdict_fn):
    """Host-only search logic of the fixed-k search.  `verdict_fn(list of (num, den))` returns 0/1 verdicts
    (1 iff num/den >= U*); returns dict(U_star, rounds)."""
    c = ctypes
    err = []

    def _cb(_ctx, n, pn, pd, pout):
        try:
            res = verdict_fn([(int(pn[i]), int(pd[i])) for i in range(n)])
            for i in range(n):
                pout[i] = 1 if res[i] else 0
            return FC_OK
        except Exception as exc:            # never let an exception cross the C boundary
            err.append(exc)
            return FC_EINVAL

    cb = VERDICT_FN(_cb)
    r, rounds = fc_rational(), c.c_int32()
    rc = load_library().fc_fixed_k_search_with_verdicts(int(n_compute), int(min_in_bw), int(max_bw), int(k),
                                                       int(candidates_per_round), cb, None, c.byref(r), c.byref(rounds))
    if err:
        raise err[0]
    _check(rc, "fc_fixed_k_search_with_verdicts")
    return {"U_star": Fraction(r.num, r.den), "rounds": int(rounds.value)}


# ------------------------------------------------------------------ edge splitting (gamma of Appendix E.2's maximum-split-off theorem)

def fc_split_gamma_workspace_bytes(g: Graph, n_pairs: int) -> int:
    return int(load_library().fc_split_gamma_workspace_bytes(g.handle, int(n_pairs)))


def fc_split_gamma_batch(g: Graph, U: int, k: int, d_u, d_w, d_t, want_flows=False, d_workspace=None, stream=None,
                         options=None, want_stats=False):
    """gamma for every pair e = (u, w), f = (w, t) in G({U b_e}).  Returns dict(gamma=int32 tensor,
    flows=int32 [n_pairs, 2, N] or None, stats)."""
    import torch
    n_pairs = int(d_u.numel())
    dev = d_u.device
    N = fc_graph_info(g).n_compute
    gamma = torch.empty(n_pairs, dtype=torch.int32, device=dev)
    flows = torch.empty(n_pairs * 2 * N, dtype=torch.int32, device=dev) if want_flows else None
    need = fc_split_gamma_workspace_bytes(g, n_pairs)
    if d_workspace is None:
        d_workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    st = fc_stats() if want_stats else None
    rc = load_library().fc_split_gamma_batch(
        g.handle, int(U), int(k), n_pairs, _dev_ptr(d_u, torch.int32, n_pairs, "d_u"), _dev_ptr(d_w, torch.int32, n_pairs, "d_w"),
        _dev_ptr(d_t, torch.int32, n_pairs, "d_t"), _dev_ptr(gamma, torch.int32, n_pairs, "gamma"),
        _dev_ptr(flows, torch.int32, n_pairs * 2 * N, "flows"), ctypes.c_void_p(d_workspace.data_ptr()), d_workspace.numel(),
        _stream_ptr(stream), _opts(options), ctypes.byref(st) if st is not None else None)
    _check(rc, "fc_split_gamma_batch")
    return {"gamma": gamma, "flows": flows.view(n_pairs, 2, N) if flows is not None else None,
            "stats": st.as_dict() if st is not None else None}


def fc_remove_switches(n_vertices, tail, head, capacity, is_compute, k: int, stream=None, options=None):
    """Algorithm 2 on the integer-capacity Eulerian digraph given as host arrays.  Returns dict(links={(u, t): cap},
    table={(u, t): {w: amount}}, batches=int)."""
    c = ctypes
    lib = load_library()
    tail = _np(tail, np.int32); head = _np(head, np.int32); capacity = _np(capacity, np.int32)
    is_compute = _np(is_compute, np.uint8)
    n_out, n_routes, batches = c.c_int64(0), c.c_int64(0), c.c_int64(0)
    out_cap = route_cap = max(1024, 4 * int(tail.shape[0]))      # a guess that normally fits
    for _ in range(2):                                   # the call reports the sizes it needs when they do not fit
        ot = np.zeros(max(out_cap, 1), np.int32); oh = np.zeros_like(ot); oc = np.zeros_like(ot)
        ru = np.zeros(max(route_cap, 1), np.int32); rt = np.zeros_like(ru); rw = np.zeros_like(ru); ra = np.zeros_like(ru)
        rc = lib.fc_remove_switches(int(n_vertices), int(tail.shape[0]), _host_ptr(tail), _host_ptr(head), _host_ptr(capacity),
                                    _host_ptr(is_compute), int(k), out_cap, c.byref(n_out), _host_ptr(ot), _host_ptr(oh),
                                    _host_ptr(oc), route_cap, c.byref(n_routes), _host_ptr(ru), _host_ptr(rt), _host_ptr(rw),
                                    _host_ptr(ra), c.byref(batches), _stream_ptr_for_host_call(stream), _opts(options))
        if rc == FC_EWORKSPACE and (n_out.value > out_cap or n_routes.value > route_cap):
            out_cap, route_cap = int(n_out.value), int(n_routes.value)
            continue
        break
    _check(rc, "fc_remove_switches")
    links = {(int(ot[i]), int(oh[i])): int(oc[i]) for i in range(n_out.value)}
    table = {}
    for i in range(n_routes.value):
        table.setdefault((int(ru[i]), int(rt[i])), {})[int(rw[i])] = int(ra[i])
    return {"links": links, "table": table, "batches": int(batches.value)}


FC_MU_INVALID = FC_GAMMA_INVALID


def _links_arrays(links):
    keys = sorted(links)
    return (np.array([a for a, _ in keys], dtype=np.int32), np.array([b for _, b in keys], dtype=np.int32),
            np.array([int(links[key]) for key in keys], dtype=np.int32))


def fc_tree_mu_batch(n_vertices, links, sets, demand, grow_set, edges, want_flows=False, stream=None, options=None):
    """mu (Appendix E.3) for the candidate edges [(x, y), ...] of root-set `grow_set` in the state (links =
    {(a, b): remaining capacity}, sets = list of vertex collections, demand = list of multiplicities).
    Returns dict(mu=int32 array, flows=int32 array or None)."""
    tail, head, cap = _links_arrays(links)
    ptr = np.zeros(len(sets) + 1, dtype=np.int64)
    for i, R in enumerate(sets):
        ptr[i + 1] = ptr[i] + len(R)
    mem = np.array([int(r) for R in sets for r in sorted(R)], dtype=np.int32)
    dem = _np(demand, np.int32)
    ex = np.array([int(e[0]) for e in edges], dtype=np.int32); ey = np.array([int(e[1]) for e in edges], dtype=np.int32)
    mu = np.zeros(max(len(edges), 1), dtype=np.int32)
    flows = np.zeros(max(len(edges), 1), dtype=np.int32) if want_flows else None
    rc = load_library().fc_tree_mu_batch(int(n_vertices), int(tail.shape[0]), _host_ptr(tail), _host_ptr(head), _host_ptr(cap),
                                         len(sets), _host_ptr(ptr), _host_ptr(mem), _host_ptr(dem), int(grow_set), len(edges),
                                         _host_ptr(ex), _host_ptr(ey), _host_ptr(mu), _host_ptr(flows) if flows is not None else None,
                                         _stream_ptr_for_host_call(stream), _opts(options))
    _check(rc, "fc_tree_mu_batch")
    return {"mu": mu[: len(edges)], "flows": flows[: len(edges)] if flows is not None else None}


def fc_construct_trees(n_vertices, links, k: int, stream=None, options=None):
    """Spanning tree construction (Appendix E.3) on D* = links {(a, b): capacity} over vertices 0..n_vertices-1.
    Returns dict(trees=[(root, multiplicity, [(x, y), ...]), ...], batches=int)."""
    c = ctypes
    tail, head, cap = _links_arrays(links)
    n = int(n_vertices)
    n_trees, batches = c.c_int64(0), c.c_int64(0)
    room = max(4 * n, 64)
    for _ in range(2):                                   # the call reports the size it needs when the guess was short
        root = np.zeros(room, np.int32); mult = np.zeros(room, np.int32)
        exs = np.zeros(room * max(n - 1, 1), np.int32); eys = np.zeros_like(exs)
        rc = load_library().fc_construct_trees(n, int(tail.shape[0]), _host_ptr(tail), _host_ptr(head), _host_ptr(cap), int(k), room,
                                               c.byref(n_trees), _host_ptr(root), _host_ptr(mult), _host_ptr(exs), _host_ptr(eys),
                                               c.byref(batches), _stream_ptr_for_host_call(stream), _opts(options))
        if rc == FC_EWORKSPACE and n_trees.value > room:
            room = int(n_trees.value)
            continue
        break
    _check(rc, "fc_construct_trees")
    trees = []
    for i in range(n_trees.value):
        lo = i * (n - 1)
        trees.append((int(root[i]), int(mult[i]), [(int(exs[lo + q]), int(eys[lo + q])) for q in range(n - 1)]))
    return {"trees": trees, "batches": int(batches.value)}
