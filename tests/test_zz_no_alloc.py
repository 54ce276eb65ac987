"""spechub_verify_static (the entry point that allocates nothing: the arrival counters of the
in-kernel walk live in a device array of the library's own) against spechub_verify, through the
C ABI: two calls in a row, the second on a smaller batch."""
import ctypes as C

import pytest
import torch

from paper_2411_05289_amd import binding as B
from paper_2411_05289_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"
KEYS = ("outcome", "token", "flags", "accept_depth", "emitted")


def _case(Bn, V, depth, seed, stats):
    wl = W.config(3, device=DEV, B=Bn, V=V, depth=depth, seed=seed)
    pb = B.Problem.from_workload(wl)
    if stats:
        pb = pb.with_draft_stats()
    u_d = B.philox_uniform(seed, 1, wl.B * wl.N, 2, device=DEV).view(wl.B, wl.N, 2)
    u_v = B.philox_uniform(seed, 2, wl.B * wl.N, 3, device=DEV).view(wl.B, wl.N, 3)
    tokens = B.spechub_draft(pb, u_d)["tokens"]
    return pb, tokens, u_v


@pytest.mark.parametrize("stats", [True, False], ids=["draft_records", "self_contained"])
def test_static_entry_point_matches_spechub_verify(stats):
    # first call: 48 trees of 31 nodes, rows in registers; second call: 5 trees of 15 nodes, streamed
    # rows; third: 3 trees of 7 nodes, rows short enough for one wavefront per node
    for Bn, V, depth, seed in ((48, 32000, 5, 71), (5, 70016, 4, 72), (3, 600, 3, 74)):
        pb, tokens, u_v = _case(Bn, V, depth, seed, stats)
        want = B.spechub_verify(pb, tokens, u_v, flags=True, walk=True)              # walk as its own launch
        want_ws = B.spechub_verify(pb, tokens, u_v, workspace=B.alloc_workspace(pb), flags=True, walk=True)
        out = B.alloc_result(pb, flags=True, walk=True)
        for t in out.values():
            t.fill_(-9)
        before = torch.cuda.memory_allocated()
        B.spechub_verify_static(pb, tokens, u_v, out)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        for key in KEYS:
            assert torch.equal(out[key], want[key]), (Bn, key)
            assert torch.equal(out[key], want_ws[key]), (Bn, key)
        # and once more on the same inputs: the counters were left at zero
        for t in out.values():
            t.fill_(-9)
        B.spechub_verify_static(pb, tokens, u_v, out)
        torch.cuda.synchronize()
        for key in KEYS:
            assert torch.equal(out[key], want[key]), (Bn, key, "second call")


def test_static_entry_point_refuses_what_it_cannot_hold():
    pb, tokens, u_v = _case(2, 600, 3, 73, False)
    cp = B._c_problem(pb)
    res = B._Result()
    out = B.alloc_result(pb, flags=True, walk=True)
    for name in ("outcome", "token", "flags", "accept_depth", "emitted"):
        setattr(res, name, out[name].data_ptr())
    fn = B.lib().spechub_verify_static
    cp.B = 65537                                  # more trees than the library's array has counters
    assert fn(C.byref(cp), B._ptr(tokens), B._ptr(u_v), C.byref(res), None) == -7
    cp.B = 2
    res.emitted = None                            # the walk outputs are the point of the call
    assert fn(C.byref(cp), B._ptr(tokens), B._ptr(u_v), C.byref(res), None) == -1
    torch.cuda.synchronize()
