"""CPU oracle for the MoE layer -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end of ``moe_oracle.c`` (plain C, double arithmetic).
Only the tests, the smoke check and the benchmark's CPU-baseline leg may use
it; the product path never does, and nothing here imports the HIP package.

Arrays: ``dtype`` 0 means float32 arrays, 1 means bfloat16 bit patterns held in
``numpy.uint16`` arrays.  Every result is float64 (or int32 for indices).

What each function computes is stated next to its C definition; in short
(paper section 2.1 for the gate-selects-k-of-n_e structure, the notation table
of section 4.2 for h1, h2, n_e, k, dt, section 3.3 for the micro-batch):

    route       logits = x Wr^T (+bias); top-k by descending logit, ties to the
                lower index; weights = softmax over the k selected logits
    permute     histogram, exclusive scan, stable placement of rows by expert
    expert_ffn  o = W2 (round_dt(silu(W1 x) * W3 x)) per routed row
    combine     y[t] = sum_s w[t,s] * o[row_of[t,s]]
    layer       the four in sequence, optionally for a subset of tokens
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP on); returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i32, vp, dbl = ctypes.c_int, ctypes.c_void_p, ctypes.c_double
        lib.oracle_round_bf16.restype = dbl
        lib.oracle_round_bf16.argtypes = [dbl]
        lib.oracle_num_threads.restype = i32
        lib.oracle_route.restype = None
        lib.oracle_route.argtypes = [i32] * 5 + [vp] * 8
        lib.oracle_permute.restype = None
        lib.oracle_permute.argtypes = [i32] * 3 + [vp] * 5
        lib.oracle_gather_rows.restype = None
        lib.oracle_gather_rows.argtypes = [i32] * 4 + [vp] * 3
        lib.oracle_expert_ffn.restype = None
        lib.oracle_expert_ffn.argtypes = [i32] * 5 + [vp] * 6 + [i32] + [vp] * 3
        lib.oracle_combine.restype = None
        lib.oracle_combine.argtypes = [i32] * 3 + [vp] * 4
        _lib = lib
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(a: np.ndarray, dtype: int, shape: Sequence[int], name: str) -> np.ndarray:
    want = np.uint16 if dtype == 1 else np.float32
    if a.dtype != want:
        raise TypeError(f"{name}: expected {want} for dtype={dtype}, got {a.dtype}")
    if tuple(a.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {a.shape}")
    return np.ascontiguousarray(a)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def round_bf16(v: float) -> float:
    """Nearest bfloat16 value (ties to even) of a double."""
    return float(_load().oracle_round_bf16(float(v)))


def route(x, Wr, k: int, dtype: int, bias=None):
    """Returns dict(ids[T,k] i32, w[T,k] f64, logits[T,E] f64, gap_next[T], gap_inner[T])."""
    T, H = x.shape
    E = Wr.shape[0]
    if not (1 <= k <= E <= 1024):
        raise ValueError("need 1 <= k <= E <= 1024")
    x = _check(x, dtype, (T, H), "x")
    Wr = _check(Wr, dtype, (E, H), "Wr")
    b = None if bias is None else np.ascontiguousarray(np.asarray(bias, dtype=np.float64).reshape(E))
    ids = np.zeros((T, k), np.int32)
    w = np.zeros((T, k), np.float64)
    logits = np.zeros((T, E), np.float64)
    gn = np.zeros(T, np.float64)
    gi = np.zeros(T, np.float64)
    _load().oracle_route(T, H, E, k, dtype, _ptr(x), _ptr(Wr), _ptr(b), _ptr(ids), _ptr(w),
                         _ptr(logits), _ptr(gn), _ptr(gi))
    return dict(ids=ids, w=w, logits=logits, gap_next=gn, gap_inner=gi)


def permute(ids: np.ndarray, E: int):
    """Returns dict(counts[E], offsets[E+1], row_src[R], row_of[R]) (all int32)."""
    T, k = ids.shape
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    if ids.size and (ids.min() < 0 or ids.max() >= E):
        raise ValueError("expert id out of range")
    R = T * k
    counts = np.zeros(E, np.int32)
    offsets = np.zeros(E + 1, np.int32)
    row_src = np.zeros(R, np.int32)
    row_of = np.zeros(R, np.int32)
    _load().oracle_permute(T, k, E, _ptr(ids), _ptr(counts), _ptr(offsets), _ptr(row_src), _ptr(row_of))
    return dict(counts=counts, offsets=offsets, row_src=row_src, row_of=row_of)


def gather_rows(x: np.ndarray, row_src: np.ndarray, k: int, dtype: int) -> np.ndarray:
    T, H = x.shape
    R = row_src.shape[0]
    x = _check(x, dtype, (T, H), "x")
    row_src = np.ascontiguousarray(row_src, dtype=np.int32)
    out = np.zeros((R, H), x.dtype)
    _load().oracle_gather_rows(R, H, k, dtype, _ptr(x), _ptr(row_src), _ptr(out))
    return out


def expert_ffn(x_perm, offsets, W1, W3, W2, dtype: int, row_w=None, sel=None,
               want_h: bool = True, want_o: bool = True):
    """SwiGLU expert FFN on permuted rows.  ``sel`` (int rows) restricts the work.

    Returns (h[n_sel,F] f64 or None, o[n_sel,H] f64 or None).
    """
    R, H = x_perm.shape
    E, F, H2 = W1.shape
    if H2 != H:
        raise ValueError("W1 must be [E,F,H]")
    x_perm = _check(x_perm, dtype, (R, H), "x_perm")
    W1 = _check(W1, dtype, (E, F, H), "W1")
    W3 = _check(W3, dtype, (E, F, H), "W3")
    W2 = _check(W2, dtype, (E, H, F), "W2")
    offsets = np.ascontiguousarray(offsets, dtype=np.int32)
    if offsets.shape != (E + 1,):
        raise ValueError("offsets must be [E+1]")
    rw = None if row_w is None else np.ascontiguousarray(np.asarray(row_w, dtype=np.float64).reshape(R))
    if sel is None:
        n_sel, selp = R, None
    else:
        selp = np.ascontiguousarray(sel, dtype=np.int32)
        n_sel = int(selp.shape[0])
        if n_sel and (selp.min() < 0 or selp.max() >= R):
            raise ValueError("selected row out of range")
    h = np.zeros((n_sel, F), np.float64) if want_h else None
    o = np.zeros((n_sel, H), np.float64) if want_o else None
    _load().oracle_expert_ffn(R, H, F, E, dtype, _ptr(x_perm), _ptr(offsets), _ptr(W1), _ptr(W3), _ptr(W2),
                              _ptr(rw), n_sel, _ptr(selp), _ptr(h), _ptr(o))
    return h, o


def combine(o: np.ndarray, row_of: np.ndarray, k: int, w=None) -> np.ndarray:
    """y[T,H] f64 from o[R,H] f64."""
    R, H = o.shape
    T = R // k
    o = np.ascontiguousarray(o, dtype=np.float64)
    row_of = np.ascontiguousarray(row_of, dtype=np.int32).reshape(R)
    wp = None if w is None else np.ascontiguousarray(np.asarray(w, dtype=np.float64).reshape(T, k))
    y = np.zeros((T, H), np.float64)
    _load().oracle_combine(T, H, k, _ptr(o), _ptr(row_of), _ptr(wp), _ptr(y))
    return y


def layer(x, Wr, W1, W3, W2, k: int, dtype: int, bias=None, tokens=None):
    """The whole layer.  ``tokens`` (int array) restricts the expert FFN and the
    output to those tokens (routing and permutation are always done in full).

    Returns dict with everything route() and permute() return plus
    ``y`` [n_tokens,H] f64 and ``tokens``.
    """
    T, H = x.shape
    E = Wr.shape[0]
    rt = route(x, Wr, k, dtype, bias)
    pm = permute(rt["ids"], E)
    xp = gather_rows(x, pm["row_src"], k, dtype)
    tok = np.arange(T, dtype=np.int32) if tokens is None else np.ascontiguousarray(tokens, dtype=np.int32)
    flat = (tok[:, None].astype(np.int64) * k + np.arange(k)[None, :]).reshape(-1)
    rows = pm["row_of"][flat]
    _, o = expert_ffn(xp, pm["offsets"], W1, W3, W2, dtype, sel=rows, want_h=False)
    y = combine(o, np.arange(rows.shape[0], dtype=np.int32), k, w=rt["w"][tok])
    out = dict(rt)
    out.update(pm)
    out["x_perm"] = xp
    out["y"] = y
    out["tokens"] = tok
    return out
