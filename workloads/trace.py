"""Stack-distance trace tools of Sec. 4.2 as a seeded input generator (no method arithmetic).

Alg. 1 profiles a trace of the embedding lookups of one categorical feature: the list ``u`` of
unique accesses in order of first appearance and the distribution ``p`` of stack distances
(``p[0]``: share of first-time accesses; ``p[d]``, d >= 1: share of accesses whose id sat at position
d from the top of the stack of most recently used ids, 1 = the access just before).  Alg. 2
generates a synthetic trace from ``(u, p)`` with the same locality: it draws a distance from ``p``
restricted to what has been emitted so far, takes a new id from the front of ``u`` for d = 0, else
re-uses the d-th most recently used id.

Two implementations that must agree exactly (tests/test_trace_tools.py):
  * ``profile_trace_py`` / ``generate_trace_py``: the two algorithms as plain list operations, step
    by step in the paper's order; O(n * stack depth), for small inputs;
  * ``profile_trace`` / ``generate_trace``: workloads/trace_tools.c (same steps, the stack kept
    under a Fenwick tree), for traces of millions of lookups.
Random numbers are an INPUT of the generator (one uniform number in [0, 1) per emitted access), so
both implementations can be driven by the same stream.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "trace_tools.c")
_LIB = os.path.join(_HERE, "libtrace_tools.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC],
                       check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.trace_profile.restype = C.c_int
        _lib.trace_generate.restype = C.c_int
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


# ------------------------------------------------------------------ Alg. 1
def profile_trace_py(tr: Sequence[int]) -> Tuple[List[int], np.ndarray]:
    """Alg. 1 with a Python list as the stack (top = end of the list)."""
    stack: List[int] = []
    u: List[int] = []
    counts: List[int] = [0]
    for a in tr:
        d = 0
        for pos in range(1, len(stack) + 1):          # position from the top
            if stack[-pos] == a:
                d = pos
                break
        if d == 0:
            u.append(a)
        else:
            del stack[-d]
        while len(counts) <= d:
            counts.append(0)
        counts[d] += 1
        stack.append(a)
    n = max(len(tr), 1)
    return u, np.asarray(counts, dtype=np.float64) / n


def profile_trace(tr: np.ndarray, id_bound: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Alg. 1 at scale.  tr: int64 ids in [0, id_bound).  Returns (u int64, p float64)."""
    tr = np.ascontiguousarray(tr, dtype=np.int64)
    n = int(tr.size)
    if id_bound is None:
        id_bound = int(tr.max()) + 1 if n else 1
    u = np.empty(max(n, 1), dtype=np.int64)
    cnt = np.zeros(n + 1, dtype=np.int64)
    n_u, max_d = C.c_int64(0), C.c_int64(0)
    st = lib().trace_profile(_ptr(tr), C.c_int64(n), C.c_int64(int(id_bound)), _ptr(u), C.byref(n_u), _ptr(cnt),
                             C.byref(max_d))
    if st != 0:
        raise ValueError("trace_profile status %d" % st)
    return u[:n_u.value].copy(), cnt[:max_d.value + 1].astype(np.float64) / max(n, 1)


# ------------------------------------------------------------------ Alg. 2
def _draw_distance(cum: np.ndarray, s: int, unseen: bool, r: float, boost: float) -> int:
    """A distance from p restricted to [0 or 1, s] (see trace_tools.c: the same rule, written out)."""
    top = min(s, len(cum) - 1)
    if unseen:
        total = cum[top] + boost
        target = r * total
        if not total > 0.0 or target < cum[0] + boost:
            return 0
        for d in range(1, top + 1):
            if cum[d] + boost > target:
                return d
        return top
    mass = cum[top] - cum[0]
    if not mass > 0.0:
        return 1
    target = cum[0] + r * mass
    for d in range(1, top + 1):
        if cum[d] > target:
            return d
    return top


def generate_trace_py(u: Sequence[int], p: np.ndarray, r: Sequence[float], min_new: float = 0.0) -> List[int]:
    """Alg. 2 with a Python list: unseen ids at the front in order, used ids appended at the back."""
    lst = list(u)
    n_unseen = len(lst)
    cum = np.cumsum(np.asarray(p, dtype=np.float64))
    boost = max(float(min_new) - cum[0], 0.0)
    s = 0
    out: List[int] = []
    for ri in r:
        d = _draw_distance(cum, s, n_unseen > 0, float(ri), boost)
        if d == 0:
            a = lst.pop(0)                            # remove from the front
            n_unseen -= 1
            s += 1
        else:
            a = lst.pop(len(lst) - d)                 # remove from the back at position d
        lst.append(a)
        out.append(a)
    return out


def generate_trace(u: np.ndarray, p: np.ndarray, r: np.ndarray, min_new: float = 0.0) -> np.ndarray:
    """Alg. 2 at scale.  r: float64 uniform numbers in [0, 1), one per access to emit."""
    u = np.ascontiguousarray(u, dtype=np.int64)
    r = np.ascontiguousarray(r, dtype=np.float64)
    cum = np.ascontiguousarray(np.cumsum(np.asarray(p, dtype=np.float64)))
    out = np.empty(r.size, dtype=np.int64)
    st = lib().trace_generate(_ptr(u), C.c_int64(u.size), _ptr(cum), C.c_int64(cum.size), _ptr(r),
                              C.c_int64(r.size), C.c_double(float(min_new)), _ptr(out))
    if st != 0:
        raise ValueError("trace_generate status %d" % st)
    return out
