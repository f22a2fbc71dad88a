"""GPU test of the entry point that allocates nothing: fc_maxflow_batch_static, called through the C ABI, must give
exactly the values of fc_maxflow_batch (which themselves are checked against the oracle elsewhere, and here again)
on two calls in a row, the second on a smaller input that leaves the first call's contents in the static array."""
import numpy as np
import pytest

import oracle as o
import workloads as w

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

if not torch.cuda.is_available():          # selected explicitly on a machine without a GPU
    pytest.skip("needs a GPU", allow_module_level=True)

import paper_2402_06787_amd as fc   # noqa: E402

DEV = torch.device("cuda:0")


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def test_static_scratch_entry_point_matches_the_workspace_one():
    topo = w.config_topology(4)                       # 512 compute nodes, 8192 problems: the launch order is used
    pl = w.config_problems(4, topo)
    with fc.fc_graph_upload(topo.n_vertices, topo.tail, topo.head, topo.bandwidth, topo.is_compute) as g:
        rng = np.random.default_rng(5)
        first = np.arange(pl.n_problems)
        second = np.sort(rng.choice(pl.n_problems, 1500, replace=False))     # smaller, ragged, still ordered (> 2 x CUs)
        third = second[:37]                                                  # small enough to run without an order
        for idx in (first, second, third):
            sink, U, k = _dev(pl.sink[idx]), _dev(pl.edge_mult[idx]), _dev(pl.src_cap[idx])
            want, _ = fc.fc_maxflow_batch(g, sink, U, k)
            out = torch.full((len(idx),), -77, dtype=torch.int32, device=DEV)
            before = torch.cuda.memory_stats(DEV)["allocation.all.allocated"]      # allocations so far (never goes down)
            got = fc.fc_maxflow_batch_static(g, sink, U, k, out)
            assert torch.cuda.memory_stats(DEV)["allocation.all.allocated"] == before   # the binding asked torch for nothing
            torch.cuda.synchronize()
            assert torch.equal(got, want), int((got != want).sum())
            if len(idx) <= 1500:
                ref = o.aux_maxflow_batch(topo, pl.sink[idx], pl.edge_mult[idx], pl.src_cap[idx], threads=16)
                assert (got.cpu().numpy().astype(np.int64) == ref).all()
        # too many problems for the static array: refused before anything is launched
        big = fc.FC_MAXFLOW_BATCH_STATIC_MAX_PROBLEMS + 1
        z = torch.ones(big, dtype=torch.int32, device=DEV)
        with pytest.raises(fc.FcError) as err:
            fc.fc_maxflow_batch_static(g, z, z, z, torch.empty(big, dtype=torch.int32, device=DEV))
        assert err.value.code == fc.FC_EWORKSPACE
        # malformed problems get the same markers as from the workspace entry point
        sink = _dev([0, -1, topo.n_vertices, 3]); U = _dev([60, 60, 60, 0]); k = _dev([4, 4, 4, 4])
        want, _ = fc.fc_maxflow_batch(g, sink, U, k)
        got = fc.fc_maxflow_batch_static(g, sink, U, k, torch.empty(4, dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        assert torch.equal(got, want) and got.cpu().tolist()[1:] == [fc.FC_FLOW_INVALID] * 3
