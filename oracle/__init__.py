"""ctypes front end of the CPU oracle (oracle/confu_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's
CPU-baseline leg.  It shares no code with the GPU library and never imports it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "confu_oracle.c")
_LIB = os.path.join(_HERE, "libconfu_oracle.so")

RULE_GREEDY, RULE_DETERMINISTIC, RULE_DRAFT_WOR, RULE_DRAFT_WR, RULE_SAMPLE_MATCH = 0, 1, 2, 3, 4
FINAL_BONUS, FINAL_RESIDUAL = 0, 1
KIND_NODE, KIND_CONTEMPLATE = 0, 1

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64, -O2, OpenMP over independent rows only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-fast-math",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


class OracleError(RuntimeError):
    def __init__(self, code: int):
        super().__init__({1: "malformed tree", 2: "bad argument", 3: "out of memory"}.get(code, str(code)))
        self.code = code


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def ancestor_matrix(parent, kind) -> np.ndarray:
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    kind = np.ascontiguousarray(kind, dtype=np.uint8)
    M = len(parent)
    anc = np.zeros((M, M), dtype=np.uint8)
    rc = _load().oracle_ancestor_matrix(M, _p(parent, ctypes.c_int32), _p(kind, ctypes.c_uint8),
                                        _p(anc, ctypes.c_uint8))
    if rc:
        raise OracleError(rc)
    return anc


def visibility_matrix(parent, kind, P: int, s: int) -> np.ndarray:
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    kind = np.ascontiguousarray(kind, dtype=np.uint8)
    M = len(parent)
    vis = np.zeros((M, P + M), dtype=np.uint8)
    rc = _load().oracle_visibility_matrix(M, int(P), int(s), _p(parent, ctypes.c_int32),
                                          _p(kind, ctypes.c_uint8), _p(vis, ctypes.c_uint8))
    if rc:
        raise OracleError(rc)
    return vis


def tree_attention(q, k, v, parent, kind, *, soft_len: int, scale: float, return_lse: bool = False):
    """q [M,Hq,D], k/v [P+M,Hkv,D] (any float dtype, widened to fp64), one sequence.
    Returns out [M,Hq,D] fp64 (and lse [Hq,M])."""
    q = np.ascontiguousarray(q, dtype=np.float64)
    k = np.ascontiguousarray(k, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64)
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    kind = np.ascontiguousarray(kind, dtype=np.uint8)
    M, Hq, D = q.shape
    L, Hkv, D2 = k.shape
    if D2 != D or v.shape != k.shape or len(parent) != M or len(kind) != M or L < M:
        raise ValueError("shape mismatch")
    P = L - M
    out = np.empty((M, Hq, D), dtype=np.float64)
    lse = np.empty((Hq, M), dtype=np.float64) if return_lse else None
    rc = _load().oracle_tree_attention(
        M, Hq, Hkv, D, P, int(soft_len), ctypes.c_double(scale),
        _p(q, ctypes.c_double), _p(k, ctypes.c_double), _p(v, ctypes.c_double),
        _p(parent, ctypes.c_int32), _p(kind, ctypes.c_uint8),
        _p(out, ctypes.c_double), _p(lse, ctypes.c_double))
    if rc:
        raise OracleError(rc)
    return (out, lse) if return_lse else out


def tree_accept(target_logits, draft_logits, token, parent, uniforms, *, temperature: float, rule: int,
                con_anchor=None) -> dict:
    """One sequence.  target_logits/draft_logits float32 [T,V]; see confu_oracle.c."""
    tl = np.ascontiguousarray(target_logits, dtype=np.float32)
    dl = None if draft_logits is None else np.ascontiguousarray(draft_logits, dtype=np.float32)
    token = np.ascontiguousarray(token, dtype=np.int32)
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    un = None if uniforms is None else np.ascontiguousarray(uniforms, dtype=np.float32)
    ca = None if con_anchor is None else np.ascontiguousarray(con_anchor, dtype=np.int32)
    T, V = tl.shape
    if dl is not None and dl.shape != tl.shape:
        raise ValueError("draft/target shape mismatch")
    if len(token) != T or len(parent) != T or (un is not None and len(un) != 2 * T):
        raise ValueError("shape mismatch")
    path = np.empty(T, dtype=np.int32)
    outs = [ctypes.c_int32() for _ in range(5)]
    rc = _load().oracle_tree_accept(
        T, V, 0 if ca is None else len(ca), ctypes.c_double(temperature), int(rule),
        _p(tl, ctypes.c_float), _p(dl, ctypes.c_float), _p(token, ctypes.c_int32),
        _p(parent, ctypes.c_int32), _p(un, ctypes.c_float), _p(ca, ctypes.c_int32),
        _p(path, ctypes.c_int32), *[ctypes.byref(o) for o in outs])
    if rc:
        raise OracleError(rc)
    n_acc, ftok, fkind, last, scon = (int(o.value) for o in outs)
    return {"path": path, "n_accepted": n_acc, "final_token": ftok, "final_kind": fkind,
            "last_node": last, "selected_con": scon}


def tree_accept_many(target_logits, draft_logits, token, parent, uniforms, *, temperature: float, rule: int):
    """uniforms float32 [n, 2T]; the other inputs as in tree_accept. Returns int32 arrays [n]."""
    tl = np.ascontiguousarray(target_logits, dtype=np.float32)
    dl = None if draft_logits is None else np.ascontiguousarray(draft_logits, dtype=np.float32)
    token = np.ascontiguousarray(token, dtype=np.int32)
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    un = np.ascontiguousarray(uniforms, dtype=np.float32)
    T, V = tl.shape
    n = un.shape[0]
    if un.shape[1] != 2 * T:
        raise ValueError("uniforms must be [n, 2T]")
    o = [np.empty(n, dtype=np.int32) for _ in range(4)]
    rc = _load().oracle_tree_accept_many(
        n, T, V, ctypes.c_double(temperature), int(rule), _p(tl, ctypes.c_float), _p(dl, ctypes.c_float),
        _p(token, ctypes.c_int32), _p(parent, ctypes.c_int32), _p(un, ctypes.c_float),
        *[_p(a, ctypes.c_int32) for a in o])
    if rc:
        raise OracleError(rc)
    return {"n_accepted": o[0], "final_token": o[1], "final_kind": o[2], "last_node": o[3]}
