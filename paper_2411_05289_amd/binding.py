"""Thin Python binding of the C ABI in ``include/mdsd.h``.

Argument marshalling only: torch supplies device memory and the HIP stream;
every step of the method runs inside ``libmdsd.so``.  There is no fallback: if
the library has not been built, or a tensor is not on the GPU, the call raises.
"""
from __future__ import annotations

import ctypes as C
import os
import dataclasses
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmdsd.so")

FP32, BF16 = 0, 1
PROBS, LOGITS = 0, 1
NONE, BAD_PAIR, BAD_TOKEN, UNVISITED = -1, -2, -3, -4
FLAG_DEGENERATE_HUB, FLAG_ZERO_RESIDUAL, FLAG_Q_EXHAUSTED, FLAG_BAD_PAIR, FLAG_BAD_TOKEN = 1, 2, 4, 8, 16

EXPORTS = ("mdsd_workspace_bytes", "spechub_draft", "spechub_verify", "spechub_verify_static", "rrs_draft", "rrsw_draft",
           "rrs_verify", "rrsw_verify", "spechub_verify_path", "rrs_verify_path", "rrsw_verify_path",
           "mdsd_tree_walk", "mdsd_philox_uniform", "mdsd_strerror", "mdsd_version")


class MdsdError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s: %s (%d)" % (where, strerror(code), code))


class _Problem(C.Structure):
    _fields_ = [
        ("target", C.c_void_p), ("draft", C.c_void_p),
        ("ld_t", C.c_int64), ("ld_d", C.c_int64),
        ("dtype", C.c_int32), ("kind", C.c_int32),
        ("temp_target", C.c_float), ("temp_draft", C.c_float),
        ("B", C.c_int32), ("N", C.c_int32), ("V", C.c_int32),
        ("k", C.c_int32), ("depth", C.c_int32),
        ("first_child", C.c_void_p),
        ("draft_stats", C.c_void_p),
    ]


class _Result(C.Structure):
    _fields_ = [
        ("outcome", C.c_void_p), ("token", C.c_void_p), ("resid_mass", C.c_void_p),
        ("flags", C.c_void_p), ("resid_prob", C.c_void_p), ("accept_depth", C.c_void_p),
        ("emitted", C.c_void_p),
    ]


_lib = None


def lib():
    """The loaded HIP library.  Raises if it is missing: there is no CPU path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libmdsd.so is not built (run `python -m paper_2411_05289_amd.build`); "
                "this package has no fallback path")
        L = C.CDLL(LIB_PATH)
        L.mdsd_workspace_bytes.restype = C.c_size_t
        L.mdsd_workspace_bytes.argtypes = [C.c_void_p]
        L.mdsd_strerror.restype = C.c_char_p
        L.mdsd_strerror.argtypes = [C.c_int]
        L.mdsd_version.restype = C.c_int
        dv = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.spechub_draft.argtypes = dv
        L.rrs_draft.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.rrsw_draft.argtypes = L.rrs_draft.argtypes
        vv = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        for f in (L.spechub_verify, L.rrs_verify, L.rrsw_verify,
                  L.spechub_verify_path, L.rrs_verify_path, L.rrsw_verify_path):
            f.argtypes = vv
            f.restype = C.c_int
        for f in (L.spechub_draft, L.rrs_draft, L.rrsw_draft):
            f.restype = C.c_int
        L.spechub_verify_static.argtypes = [C.c_void_p] * 5
        L.spechub_verify_static.restype = C.c_int
        L.mdsd_tree_walk.argtypes = [C.c_void_p] * 6
        L.mdsd_tree_walk.restype = C.c_int
        L.mdsd_philox_uniform.argtypes = [C.c_uint64, C.c_uint32, C.c_int64, C.c_int32, C.c_void_p,
                                          C.c_void_p, C.c_void_p]
        L.mdsd_philox_uniform.restype = C.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().mdsd_strerror(code).decode()


def version() -> int:
    return lib().mdsd_version()


@dataclass
class Problem:
    """Rows of one batch of token trees (device tensors) and the tree shape."""
    target: Optional[torch.Tensor]   # [B,N,V] float32 or bfloat16; None for draft-only use
    draft: torch.Tensor              # [B,N,V]
    kind: int                        # PROBS | LOGITS
    k: int
    depth: int
    temp_target: float = 1.0
    temp_draft: float = 1.0
    first_child: Optional[torch.Tensor] = None  # [N] int32 on device, or None
    # [B,N,4] float32 on device, or None: one record per node (max stored draft element, draft
    # mass outside the hub, hub index as int32 bits, 0) that spechub_draft writes and
    # spechub_verify reads instead of scanning the draft row for them again
    draft_stats: Optional[torch.Tensor] = None

    def with_draft_stats(self) -> "Problem":
        """The same problem with a fresh record array attached."""
        B, N, _ = self.draft.shape
        stats = torch.zeros((B, N, 4), dtype=torch.float32, device=self.draft.device)
        return dataclasses.replace(self, draft_stats=stats)

    @staticmethod
    def from_workload(wl) -> "Problem":
        return Problem(wl.target, wl.draft, LOGITS if wl.kind == "logits" else PROBS, wl.k, wl.depth,
                       wl.temp_target, wl.temp_draft, wl.first_child)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _check_rows(t: torch.Tensor, name: str):
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % name)
    if t.dim() != 3 or t.stride(2) != 1 or t.stride(0) != t.shape[1] * t.stride(1):
        raise ValueError("%s must be [B,N,V] with unit stride in V and B-major rows" % name)
    if t.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("%s must be float32 or bfloat16" % name)


def _check_dev(t: torch.Tensor, name: str, dtype, shape):
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous() or tuple(t.shape) != tuple(shape):
        raise ValueError("%s must be a contiguous %s GPU tensor of shape %s" % (name, dtype, tuple(shape)))


def _c_problem(pb: Problem) -> _Problem:
    _check_rows(pb.draft, "draft")
    B, N, V = pb.draft.shape
    cp = _Problem()
    if pb.target is not None:
        _check_rows(pb.target, "target")
        if pb.target.shape != pb.draft.shape or pb.target.dtype != pb.draft.dtype:
            raise ValueError("target and draft must agree in shape and dtype")
        cp.target = pb.target.data_ptr()
        cp.ld_t = pb.target.stride(1)
    else:
        cp.target = None
        cp.ld_t = pb.draft.stride(1)
    cp.draft = pb.draft.data_ptr()
    cp.ld_d = pb.draft.stride(1)
    cp.dtype = FP32 if pb.draft.dtype == torch.float32 else BF16
    cp.kind = pb.kind
    cp.temp_target, cp.temp_draft = pb.temp_target, pb.temp_draft
    cp.B, cp.N, cp.V, cp.k, cp.depth = B, N, V, pb.k, pb.depth
    if pb.first_child is not None:
        _check_dev(pb.first_child, "first_child", torch.int32, (N,))
        cp.first_child = pb.first_child.data_ptr()
    else:
        cp.first_child = None
    if pb.draft_stats is not None:
        _check_dev(pb.draft_stats, "draft_stats", torch.float32, (B, N, 4))
        cp.draft_stats = pb.draft_stats.data_ptr()
    else:
        cp.draft_stats = None
    return cp


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def workspace_bytes(pb: Problem) -> int:
    cp = _c_problem(pb)
    return int(lib().mdsd_workspace_bytes(C.byref(cp)))


def _draft(fn_name, pb: Problem, u: torch.Tensor, out, with_hub: bool):
    cp = _c_problem(pb)
    B, N, _ = pb.draft.shape
    dev = pb.draft.device
    _check_dev(u, "u", torch.float32, (B, N, pb.k))
    out = {} if out is None else out
    if "tokens" not in out:
        out["tokens"] = torch.empty((B, N), dtype=torch.int32, device=dev)
    if "flags" not in out:
        out["flags"] = torch.empty((B, N), dtype=torch.int32, device=dev)
    if with_hub and "hub" not in out:
        out["hub"] = torch.empty((B, N), dtype=torch.int32, device=dev)
    _check_dev(out["tokens"], "tokens", torch.int32, (B, N))
    fn = getattr(lib(), fn_name)
    if with_hub:
        rc = fn(C.byref(cp), _ptr(u), _ptr(out["tokens"]), _ptr(out["hub"]), _ptr(out["flags"]), None, 0, _stream())
    else:
        rc = fn(C.byref(cp), _ptr(u), _ptr(out["tokens"]), _ptr(out["flags"]), None, 0, _stream())
    if rc != 0:
        raise MdsdError(rc, fn_name)
    return out


def spechub_draft(pb: Problem, u: torch.Tensor, out=None):
    """Sample the (x1, x2) ~ Q pair of every internal node.  -> dict(tokens, hub, flags)."""
    return _draft("spechub_draft", pb, u, out, True)


def rrs_draft(pb: Problem, u: torch.Tensor, out=None):
    return _draft("rrs_draft", pb, u, out, False)


def rrsw_draft(pb: Problem, u: torch.Tensor, out=None):
    return _draft("rrsw_draft", pb, u, out, False)


def alloc_result(pb: Problem, *, resid_mass=False, flags=True, resid_prob=False, walk=True):
    """Output tensors for a verify call (so that a timed loop allocates nothing)."""
    B, N, V = pb.draft.shape
    dev = pb.draft.device
    out = dict(outcome=torch.empty((B, N), dtype=torch.int32, device=dev),
               token=torch.empty((B, N), dtype=torch.int32, device=dev))
    if resid_mass:
        out["resid_mass"] = torch.empty((B, N), dtype=torch.float32, device=dev)
    if flags:
        out["flags"] = torch.empty((B, N), dtype=torch.int32, device=dev)
    if resid_prob:
        out["resid_prob"] = torch.empty((B, N, V), dtype=torch.float32, device=dev)
    if walk:
        out["accept_depth"] = torch.empty((B,), dtype=torch.int32, device=dev)
        out["emitted"] = torch.empty((B, pb.depth), dtype=torch.int32, device=dev)
    return out


def alloc_workspace(pb: Problem) -> torch.Tensor:
    """A zero-filled workspace for the verify calls (one arrival counter per tree): handed to a
    verify call together with walk=True, the kernel walks the trees itself.  Every call leaves
    it zero-filled, so one workspace serves call after call on one stream."""
    n = workspace_bytes(pb)
    return torch.zeros(((n + 3) // 4,), dtype=torch.int32, device=pb.draft.device)


def _verify(fn_name, pb: Problem, tokens: torch.Tensor, u: torch.Tensor, out, workspace=None, **want):
    cp = _c_problem(pb)
    if pb.target is None:
        raise ValueError("verify needs target rows")
    B, N, _ = pb.draft.shape
    _check_dev(tokens, "tokens", torch.int32, (B, N))
    _check_dev(u, "u", torch.float32, (B, N, pb.k + 1))
    if out is None:
        out = alloc_result(pb, **want)
    res = _Result()
    for name in ("outcome", "token", "resid_mass", "flags", "resid_prob", "accept_depth", "emitted"):
        t = out.get(name)
        if t is not None and not (t.is_cuda and t.is_contiguous()):
            raise ValueError("output %s must be a contiguous GPU tensor" % name)
        setattr(res, name, None if t is None else t.data_ptr())
    if workspace is not None and not (workspace.is_cuda and workspace.is_contiguous()):
        raise ValueError("workspace must be a contiguous GPU tensor")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = getattr(lib(), fn_name)(C.byref(cp), _ptr(tokens), _ptr(u), C.byref(res), _ptr(workspace), ws_bytes, _stream())
    if rc != 0:
        raise MdsdError(rc, fn_name)
    return out


def spechub_verify(pb: Problem, tokens, u, out=None, workspace=None, **want):
    """Alg. 3 on every node plus the tree walk.  -> dict(outcome, token, [resid_mass],
    [flags], [resid_prob], [accept_depth, emitted])."""
    return _verify("spechub_verify", pb, tokens, u, out, workspace, **want)


def spechub_verify_static(pb: Problem, tokens, u, out):
    """spechub_verify with the walk inside its kernel on the library's own arrival counters: the
    call allocates nothing (`out`, from alloc_result(..., walk=True), is the caller's)."""
    cp = _c_problem(pb)
    B, N, _ = pb.draft.shape
    _check_dev(tokens, "tokens", torch.int32, (B, N))
    _check_dev(u, "u", torch.float32, (B, N, pb.k + 1))
    res = _Result()
    for name in ("outcome", "token", "resid_mass", "flags", "resid_prob", "accept_depth", "emitted"):
        t = out.get(name)
        if t is not None and not (t.is_cuda and t.is_contiguous()):
            raise ValueError("output %s must be a contiguous GPU tensor" % name)
        setattr(res, name, None if t is None else t.data_ptr())
    rc = lib().spechub_verify_static(C.byref(cp), _ptr(tokens), _ptr(u), C.byref(res), _stream())
    if rc != 0:
        raise MdsdError(rc, "spechub_verify_static")
    return out


def rrs_verify(pb: Problem, tokens, u, out=None, workspace=None, **want):
    return _verify("rrs_verify", pb, tokens, u, out, workspace, **want)


def rrsw_verify(pb: Problem, tokens, u, out=None, workspace=None, **want):
    return _verify("rrsw_verify", pb, tokens, u, out, workspace, **want)


def spechub_verify_path(pb: Problem, tokens, u, out=None, **want):
    """Alg. 3 on the nodes the walk visits only (one workgroup per tree).  -> dict(outcome,
    token, [resid_mass], [flags], accept_depth, emitted); unvisited nodes: UNVISITED."""
    return _verify("spechub_verify_path", pb, tokens, u, out, **want)


def rrs_verify_path(pb: Problem, tokens, u, out=None, **want):
    return _verify("rrs_verify_path", pb, tokens, u, out, **want)


def rrsw_verify_path(pb: Problem, tokens, u, out=None, **want):
    return _verify("rrsw_verify_path", pb, tokens, u, out, **want)


def tree_walk(pb: Problem, outcome, token, accept_depth=None, emitted=None):
    B, N, _ = pb.draft.shape
    cp = _c_problem(pb)
    dev = pb.draft.device
    ad = torch.empty((B,), dtype=torch.int32, device=dev) if accept_depth is None else accept_depth
    em = torch.empty((B, pb.depth), dtype=torch.int32, device=dev) if emitted is None else emitted
    _check_dev(ad, "accept_depth", torch.int32, (B,))
    _check_dev(em, "emitted", torch.int32, (B, pb.depth))
    rc = lib().mdsd_tree_walk(C.byref(cp), _ptr(outcome), _ptr(token), _ptr(ad), _ptr(em), _stream())
    if rc != 0:
        raise MdsdError(rc, "mdsd_tree_walk")
    return ad, em


# Up to this many tree nodes per batch, StepPlan.run() lets the verify kernel walk the trees
# itself (two launches per step).  The arrival count keeps a finished workgroup about a
# microsecond longer on its compute unit, which costs more than the walk's own launch
# (2-3 us) once a batch is several times what the chip holds at once: measured on one MI355X,
# 31-node trees at V = 32000, the two placements timed in turns in one process: B = 16 26.4 against
# 26.6 us per step, B = 32 36.9 / 37.5, B = 64 54.6 / 54.9, B = 96 73.5 / 73.5, B = 128 91.6 / 91.1,
# B = 256 171.1 / 166.7, B = 1024 632 / 621.
WALK_IN_VERIFY_MAX_NODES = 3000


class StepPlan:
    """Marshalled arguments of one draft + verify + walk step, so that a serving loop pays
    two or three foreign calls per step and nothing else.  The tensors handed in must stay
    alive and in place for the life of the plan.  walk_in_verify: True = the verify kernel
    walks the trees (one launch), False = mdsd_tree_walk as a launch of its own, None = by
    batch size (WALK_IN_VERIFY_MAX_NODES)."""

    def __init__(self, method: str, pb: Problem, u_draft, u_verify, *, flags=True, hand_stats=True,
                 walk_in_verify=None):
        if method not in ("spechub", "rrs", "rrsw"):
            raise ValueError("unknown method %r" % method)
        if hand_stats and pb.draft_stats is None:
            pb = pb.with_draft_stats()   # spechub_draft -> spechub_verify hand-over of the row statistics
        B, N, _ = pb.draft.shape
        dev = pb.draft.device
        self.method, self.pb = method, pb
        self.walk_in_verify = (B * N <= WALK_IN_VERIFY_MAX_NODES) if walk_in_verify is None else bool(walk_in_verify)
        self._cp = _c_problem(pb)
        _check_dev(u_draft, "u_draft", torch.float32, (B, N, pb.k))
        _check_dev(u_verify, "u_verify", torch.float32, (B, N, pb.k + 1))
        self.tokens = torch.empty((B, N), dtype=torch.int32, device=dev)
        self.hub = torch.empty((B, N), dtype=torch.int32, device=dev)
        self.draft_flags = torch.empty((B, N), dtype=torch.int32, device=dev)
        self.out = alloc_result(pb, flags=flags, walk=True)
        self._keep = (u_draft, u_verify)
        res = _Result()
        for name in ("outcome", "token", "flags"):
            t = self.out.get(name)
            setattr(res, name, None if t is None else t.data_ptr())
        self._res = res          # no walk outputs: the walk is its own call below
        L = lib()
        pbp, resp = C.byref(self._cp), C.byref(res)
        ud, uv = _ptr(u_draft), _ptr(u_verify)
        tk, hb, df = _ptr(self.tokens), _ptr(self.hub), _ptr(self.draft_flags)
        oc, tok = _ptr(self.out["outcome"]), _ptr(self.out["token"])
        ad, em = _ptr(self.out["accept_depth"]), _ptr(self.out["emitted"])
        if method == "spechub":
            self._draft = lambda st: L.spechub_draft(pbp, ud, tk, hb, df, None, 0, st)
        else:
            fn = L.rrs_draft if method == "rrs" else L.rrsw_draft
            self._draft = lambda st: fn(pbp, ud, tk, df, None, 0, st)
        vfn = {"spechub": L.spechub_verify, "rrs": L.rrs_verify, "rrsw": L.rrsw_verify}[method]
        self._verify = lambda st: vfn(pbp, tk, uv, resp, None, 0, st)
        # verify with the walk inside its kernel: the result structure carries the walk outputs
        # and the call gets the (zero-filled, self-resetting) workspace
        self.workspace = alloc_workspace(pb)
        wsp, wsn = _ptr(self.workspace), self.workspace.numel() * 4
        fres = _Result()
        for name in ("outcome", "token", "flags", "accept_depth", "emitted"):
            t = self.out.get(name)
            setattr(fres, name, None if t is None else t.data_ptr())
        self._fres = fres
        fresp = C.byref(fres)
        self._verify_walk = lambda st: vfn(pbp, tk, uv, fresp, wsp, wsn, st)
        # path-only: its result structure carries the walk outputs, the walk is in the kernel
        pres = _Result()
        for name in ("outcome", "token", "flags", "accept_depth", "emitted"):
            t = self.out.get(name)
            setattr(pres, name, None if t is None else t.data_ptr())
        self._pres = pres
        presp = C.byref(pres)
        pfn = {"spechub": L.spechub_verify_path, "rrs": L.rrs_verify_path,
               "rrsw": L.rrsw_verify_path}[method]
        self._verify_path = lambda st: pfn(pbp, tk, uv, presp, None, 0, st)
        self._walk = lambda st: L.mdsd_tree_walk(pbp, oc, tok, ad, em, st)

    def draft(self, stream=None):
        rc = self._draft(_stream() if stream is None else stream)
        if rc != 0:
            raise MdsdError(rc, self.method + "_draft")

    def verify(self, stream=None):
        rc = self._verify(_stream() if stream is None else stream)
        if rc != 0:
            raise MdsdError(rc, self.method + "_verify")

    def verify_and_walk(self, stream=None):
        """verify with the tree walk inside its kernel (one launch)."""
        rc = self._verify_walk(_stream() if stream is None else stream)
        if rc != 0:
            raise MdsdError(rc, self.method + "_verify")

    def verify_path(self, stream=None):
        rc = self._verify_path(_stream() if stream is None else stream)
        if rc != 0:
            raise MdsdError(rc, self.method + "_verify_path")

    def walk(self, stream=None):
        rc = self._walk(_stream() if stream is None else stream)
        if rc != 0:
            raise MdsdError(rc, "mdsd_tree_walk")

    def run(self, stream=None):
        st = _stream() if stream is None else stream
        self.draft(st)
        if self.walk_in_verify:
            self.verify_and_walk(st)
        else:
            self.verify(st)
            self.walk(st)
        return self.out


def philox_uniform(seed: int, stream_id: int, rows: int, slots: int, device="cuda", want_words=False):
    """[rows, slots] float32 uniforms in [0,1) from Philox4x32-10 (and the raw words)."""
    out = torch.empty((rows, slots), dtype=torch.float32, device=device)
    words = torch.empty((rows, slots), dtype=torch.int32, device=device) if want_words else None
    rc = lib().mdsd_philox_uniform(C.c_uint64(seed), C.c_uint32(stream_id), C.c_int64(rows),
                                   C.c_int32(slots), _ptr(out), _ptr(words), _stream())
    if rc != 0:
        raise MdsdError(rc, "mdsd_philox_uniform")
    return (out, words) if want_words else out
