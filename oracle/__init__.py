"""ctypes front end of the fp64 CPU oracle (``mdsd_oracle.c``).

TEST INFRASTRUCTURE.  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the HIP library
and its Python binding never do.  It holds no arithmetic of its own: every
number comes from the C file, which states the method step by step.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mdsd_oracle.c")
_SO = os.path.join(_HERE, "libmdsd_oracle.so")

SPECHUB, RRS, RRSW = 0, 1, 2
FP32, BF16 = 0, 1
PROBS, LOGITS = 0, 1

FLAG_DEGENERATE_HUB = 1
FLAG_ZERO_RESIDUAL = 2
FLAG_Q_EXHAUSTED = 4
FLAG_BAD_PAIR = 8
FLAG_BAD_TOKEN = 16


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (never tuned beyond that)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        tmp = _SO + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _SO)
    return _SO


class _Problem(C.Structure):
    _fields_ = [
        ("target", C.c_void_p), ("draft", C.c_void_p),
        ("ld_t", C.c_int64), ("ld_d", C.c_int64),
        ("dtype", C.c_int), ("kind", C.c_int),
        ("temp_target", C.c_double), ("temp_draft", C.c_double),
        ("B", C.c_int), ("N", C.c_int), ("V", C.c_int), ("k", C.c_int), ("depth", C.c_int),
        ("first_child", C.c_void_p),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_icdf.restype = C.c_int
        _lib.orc_argmax.restype = C.c_int
        _lib.orc_spechub_draft.restype = C.c_int
        _lib.orc_spechub_verify.restype = C.c_int
        _lib.orc_rrs_verify.restype = C.c_int
        _lib.orc_rrs_draft.restype = C.c_int
        _lib.orc_batch_verify.restype = C.c_int
        _lib.orc_batch_draft.restype = C.c_int
    return _lib


def _dp(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


# ---------------------------------------------------------------- single node
def softmax(logits, T=1.0):
    l = _f64(logits)
    out = np.empty_like(l)
    lib().orc_softmax(_dp(l), C.c_int(l.size), C.c_double(T), _dp(out))
    return out


def argmax(v):
    v = _f64(v)
    return int(lib().orc_argmax(_dp(v), C.c_int(v.size)))


def icdf(w, u):
    """-> (token, W, margin)"""
    w = _f64(w)
    W = C.c_double()
    m = C.c_double()
    x = lib().orc_icdf(_dp(w), C.c_int(w.size), C.c_double(u), C.byref(W), C.byref(m))
    return int(x), W.value, m.value


def spechub_draft(q, a, u0, u1):
    """-> (x1, x2, flags, margin)"""
    q = _f64(q)
    x1, x2, m = C.c_int(), C.c_int(), C.c_double()
    fl = lib().orc_spechub_draft(_dp(q), C.c_int(q.size), C.c_int(a), C.c_double(u0),
                                 C.c_double(u1), C.byref(x1), C.byref(x2), C.byref(m))
    return x1.value, x2.value, int(fl), m.value


def spechub_verify(p, q, a, x1, x2, r0, r1, u, want_w=False):
    """-> dict(outcome, token, resid_mass, margin, flags[, w])"""
    p, q = _f64(p), _f64(q)
    tok, rm, m, fl = C.c_int(), C.c_double(), C.c_double(), C.c_int()
    w = np.empty(p.size) if want_w else None
    oc = lib().orc_spechub_verify(_dp(p), _dp(q), C.c_int(p.size), C.c_int(a), C.c_int(x1),
                                  C.c_int(x2), C.c_double(r0), C.c_double(r1), C.c_double(u),
                                  C.byref(tok), C.byref(rm), C.byref(m), C.byref(fl), _dp(w))
    out = dict(outcome=int(oc), token=tok.value, resid_mass=rm.value, margin=m.value,
               flags=fl.value)
    if want_w:
        out["w"] = w
    return out


def rrs_verify(p, q, x, r, u, without_replacement=False, want_P=False):
    """-> dict(outcome, token, margin, flags, mass[, P])"""
    p, q = _f64(p), _f64(q)
    k = len(x)
    xs = np.ascontiguousarray(x, dtype=np.int32)
    rs = _f64(r)
    tok, m, fl = C.c_int(), C.c_double(), C.c_int()
    P = np.empty(p.size) if want_P else None
    mass = np.zeros(max(k, 1))
    oc = lib().orc_rrs_verify(_dp(p), _dp(q), C.c_int(p.size), C.c_int(k), _dp(xs), _dp(rs),
                              C.c_double(u), C.c_int(1 if without_replacement else 0),
                              C.byref(tok), C.byref(m), C.byref(fl), _dp(P), _dp(mass))
    out = dict(outcome=int(oc), token=tok.value, margin=m.value, flags=fl.value,
               mass=mass[:k].copy())
    if want_P:
        out["P"] = P
    return out


def rrs_draft(q, u, without_replacement=False):
    """-> (tokens, flags, margin)"""
    q = _f64(q)
    us = _f64(u)
    k = us.size
    x = np.empty(k, dtype=np.int32)
    m = C.c_double()
    fl = lib().orc_rrs_draft(_dp(q), C.c_int(q.size), C.c_int(k), _dp(us),
                             C.c_int(1 if without_replacement else 0), _dp(x), C.byref(m))
    return x, int(fl), m.value


def tree_walk(outcome, token, k, depth, first_child=None):
    oc = np.ascontiguousarray(outcome, dtype=np.int32)
    tk = np.ascontiguousarray(token, dtype=np.int32)
    fc = None if first_child is None else np.ascontiguousarray(first_child, dtype=np.int32)
    em = np.empty(depth, dtype=np.int32)
    d = C.c_int32()
    lib().orc_tree_walk(_dp(oc), _dp(tk), C.c_int(oc.size), C.c_int(k), _dp(fc),
                        C.c_int(depth), C.byref(d), _dp(em))
    return d.value, em


# ---------------------------------------------------------------- batches
def _rows(a, dtype):
    """numpy view of the stored rows: float32, or uint16 holding bf16 bits."""
    a = np.ascontiguousarray(a)
    if dtype == FP32:
        assert a.dtype == np.float32
    else:
        assert a.dtype == np.uint16
    return a


def _problem(target, draft, dtype, kind, temp_target, temp_draft, B, N, V, k, depth,
             first_child, keep):
    t = _rows(target, dtype)
    d = _rows(draft, dtype) if draft is not None else t
    fc = None if first_child is None else np.ascontiguousarray(first_child, dtype=np.int32)
    keep.extend([t, d, fc])
    assert t.shape == (B, N, V) and d.shape == (B, N, V)
    pb = _Problem()
    pb.target, pb.draft = t.ctypes.data, d.ctypes.data
    pb.ld_t = pb.ld_d = V
    pb.dtype, pb.kind = dtype, kind
    # the temperature the library sees is an fp32 number; use its exact value
    pb.temp_target = float(np.float32(temp_target))
    pb.temp_draft = float(np.float32(temp_draft))
    pb.B, pb.N, pb.V, pb.k, pb.depth = B, N, V, k, depth
    pb.first_child = None if fc is None else fc.ctypes.data
    return pb


def batch_verify(method, target, draft, tokens, u, *, dtype, kind, k, depth,
                 temp_target=1.0, temp_draft=1.0, first_child=None, want_resid_prob=False,
                 nthreads=1):
    """Verify every node of every tree.  Rows are [B,N,V] numpy arrays (float32, or
    uint16 = bf16 bits); tokens [B,N] int32 child-indexed; u [B,N,k+1] float32."""
    B, N, V = target.shape
    keep = []
    pb = _problem(target, draft, dtype, kind, temp_target, temp_draft, B, N, V, k, depth,
                  first_child, keep)
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    u = np.ascontiguousarray(u, dtype=np.float32)
    assert tokens.shape == (B, N) and u.shape == (B, N, k + 1)
    out = dict(
        outcome=np.empty((B, N), np.int32), token=np.empty((B, N), np.int32),
        resid_mass=np.empty((B, N)), margin=np.empty((B, N)),
        flags=np.empty((B, N), np.int32), accept_depth=np.empty(B, np.int32),
        emitted=np.empty((B, depth), np.int32))
    rp = np.empty((B, N, V)) if want_resid_prob else None
    rc = lib().orc_batch_verify(C.byref(pb), C.c_int(method), _dp(tokens), _dp(u),
                                _dp(out["outcome"]), _dp(out["token"]), _dp(out["resid_mass"]),
                                _dp(out["margin"]), _dp(out["flags"]), _dp(out["accept_depth"]),
                                _dp(out["emitted"]), _dp(rp), C.c_int(nthreads))
    if rc != 0:
        raise ValueError("oracle rejected the problem (SpecHub needs k == 2)")
    if want_resid_prob:
        out["resid_prob"] = rp
    return out


def batch_draft(method, draft, u, *, dtype, kind, k, depth, temp_draft=1.0, first_child=None,
                nthreads=1):
    """Sample the children tokens of every internal node.  u is [B,N,k] float32."""
    B, N, V = draft.shape
    keep = []
    pb = _problem(draft, draft, dtype, kind, temp_draft, temp_draft, B, N, V, k, depth,
                  first_child, keep)
    u = np.ascontiguousarray(u, dtype=np.float32)
    assert u.shape == (B, N, k)
    out = dict(tokens=np.full((B, N), -1, np.int32), hub=np.empty((B, N), np.int32),
               margin=np.empty((B, N)), flags=np.empty((B, N), np.int32))
    rc = lib().orc_batch_draft(C.byref(pb), C.c_int(method), _dp(u), _dp(out["tokens"]),
                               _dp(out["hub"]), _dp(out["margin"]), _dp(out["flags"]),
                               C.c_int(nthreads))
    if rc != 0:
        raise ValueError("oracle rejected the problem (SpecHub needs k == 2)")
    return out


# ---------------------------------------------------------------- Philox
def philox4x32_10(ctr, key):
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    o = np.empty(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_dp(c), _dp(k), _dp(o))
    return o


def philox_uniform(seed, stream, rows, slots, want_words=False):
    out = np.empty((rows, slots), dtype=np.float32)
    words = np.empty((rows, slots), dtype=np.uint32) if want_words else None
    lib().orc_philox_uniform(C.c_uint64(seed), C.c_uint32(stream), C.c_int64(rows),
                             C.c_int(slots), _dp(out), _dp(words))
    return (out, words) if want_words else out
