"""CPU-side checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects what the host can detect before anything is
launched (no GPU is touched: every call below fails validation)."""
import ctypes as C
import os
import re

import pytest

from paper_2411_05289_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mdsd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\(", text)) - {"defined"})


def test_header_symbols_are_exported():
    L = B.lib()
    names = declared_functions()
    assert set(B.EXPORTS) <= set(names)
    for n in names:
        assert hasattr(L, n), "libmdsd.so does not export %s" % n


def test_version_and_strerror():
    assert B.version() >= 100
    assert B.strerror(0) == "ok"
    assert "NULL" in B.strerror(-1)


def _problem(**kw):
    p = B._Problem()
    p.target, p.draft = 0x1000, 0x2000     # never dereferenced: validation fails first
    p.ld_t = p.ld_d = 64
    p.dtype, p.kind = B.BF16, B.LOGITS
    p.temp_target = p.temp_draft = 1.0
    p.B, p.N, p.V, p.k, p.depth = 1, 3, 64, 2, 2
    p.first_child = None
    for k, v in kw.items():
        setattr(p, k, v)
    return p


@pytest.mark.parametrize("kw,code", [
    (dict(V=1), -2), (dict(B=-1), -2), (dict(N=4), -2), (dict(ld_t=8), -2), (dict(depth=0), -2),
    (dict(k=3, N=4), -3), (dict(k=0), -3), (dict(temp_target=0.0), -4), (dict(temp_draft=-1.0), -4),
    (dict(dtype=7), -5), (dict(kind=2), -5), (dict(target=0x1002, draft=0x2000), -6),
    (dict(target=0x1001), -6), (dict(draft=None), -1), (dict(ld_t=65), -6),
])
def test_spechub_verify_rejects_bad_problems(kw, code):
    L = B.lib()
    p = _problem(**kw)
    res = B._Result()
    res.outcome, res.token = 0x3000, 0x4000
    rc = L.spechub_verify(C.byref(p), C.c_void_p(0x5000), C.c_void_p(0x6000), C.byref(res), None, 0, None)
    assert rc == code


def test_empty_batch_is_accepted_and_launches_nothing():
    """B = 0: every entry point returns MDSD_OK before it looks at a pointer or the GPU."""
    L = B.lib()
    p = _problem(B=0, target=None, draft=None)
    res = B._Result()
    for f in (L.spechub_verify, L.rrs_verify, L.rrsw_verify, L.spechub_verify_path, L.rrs_verify_path,
              L.rrsw_verify_path):
        assert f(C.byref(p), None, None, C.byref(res), None, 0, None) == 0
    assert L.spechub_draft(C.byref(p), None, None, None, None, None, 0, None) == 0
    assert L.rrs_draft(C.byref(p), None, None, None, None, 0, None) == 0
    assert L.rrsw_draft(C.byref(p), None, None, None, None, 0, None) == 0
    assert L.mdsd_tree_walk(C.byref(p), None, None, None, None, None) == 0
    assert L.mdsd_philox_uniform(1, 0, 0, 4, None, None, None) == 0


def test_null_arguments():
    L = B.lib()
    p = _problem()
    res = B._Result()
    assert L.spechub_verify(C.byref(p), None, C.c_void_p(0x6000), C.byref(res), None, 0, None) == -1
    res.outcome, res.token = 0x3000, 0x4000
    res.accept_depth = 0x7000          # emitted missing
    assert L.rrs_verify(C.byref(p), C.c_void_p(0x5000), C.c_void_p(0x6000), C.byref(res), None, 0, None) == -1
    assert L.spechub_draft(C.byref(p), None, C.c_void_p(0x5000), None, None, None, 0, None) == -1
    assert L.rrs_draft(None, C.c_void_p(0x5000), C.c_void_p(0x5000), None, None, 0, None) == -1
    assert L.mdsd_philox_uniform(1, 0, 4, 4, None, None, None) == -1
    assert L.mdsd_philox_uniform(1, 0, 4, 0, C.c_void_p(0x5000), None, None) == -2


def test_rrs_accepts_k_up_to_8_and_rejects_9():
    L = B.lib()
    res = B._Result()
    p = _problem(k=9, N=10, depth=2)
    assert L.rrs_verify(C.byref(p), C.c_void_p(0x5000), C.c_void_p(0x6000), C.byref(res), None, 0, None) == -3
    p = _problem(k=2, N=3, V=10**7, ld_t=10**7, ld_d=10**7)
    assert L.rrsw_verify(C.byref(p), C.c_void_p(0x5000), C.c_void_p(0x6000), C.byref(res), None, 0, None) == -2


@pytest.mark.parametrize("name", ["spechub_verify_path", "rrs_verify_path", "rrsw_verify_path"])
def test_path_calls_need_the_walk_outputs_and_refuse_resid_prob(name):
    fn = getattr(B.lib(), name)
    p = _problem()
    args = (C.byref(p), C.c_void_p(0x5000), C.c_void_p(0x6000))
    res = B._Result()
    res.outcome, res.token = 0x3000, 0x4000
    assert fn(*args, C.byref(res), None, 0, None) == -1            # accept_depth / emitted missing
    res.accept_depth, res.emitted = 0x7000, 0x8000
    res.resid_prob = 0x9000
    assert fn(*args, C.byref(res), None, 0, None) == -9            # no residual rows from the path call
    assert "not available" in B.strerror(-9)
    bad = _problem(V=1)
    res.resid_prob = None
    assert fn(C.byref(bad), C.c_void_p(0x5000), C.c_void_p(0x6000), C.byref(res), None, 0, None) == -2


def test_workspace_is_one_counter_per_tree_and_checked():
    p = _problem()
    assert B.lib().mdsd_workspace_bytes(C.byref(p)) == 4 * p.B
    assert B.lib().mdsd_workspace_bytes(None) == 0
    # a workspace that is too small, or not 4-byte aligned, is refused before anything is launched
    res = B._Result()
    res.outcome, res.token = 0x7000, 0x8000
    res.accept_depth, res.emitted = 0x9000, 0xA000
    fn = B.lib().spechub_verify
    assert fn(C.byref(p), C.c_void_p(0x5000), C.c_void_p(0x6000), C.byref(res), C.c_void_p(0xB000), 4 * p.B - 1, None) == -7
    assert fn(C.byref(p), C.c_void_p(0x5000), C.c_void_p(0x6000), C.byref(res), C.c_void_p(0xB002), 4 * p.B, None) == -6


def test_binding_refuses_cpu_tensors():
    import torch
    t = torch.zeros((1, 3, 64), dtype=torch.bfloat16)
    pb = B.Problem(t, t, B.LOGITS, 2, 2)
    with pytest.raises(ValueError):
        B.spechub_verify(pb, torch.zeros((1, 3), dtype=torch.int32), torch.zeros((1, 3, 3)))
