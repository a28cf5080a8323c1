"""CPU oracle for the PaRO update-stage hot path (plan + schedules in
``plan.py``, arithmetic in ``update.c``).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg, never by the product package.  It shares no code
with the HIP library and takes no input from it.

Arrays are numpy; bf16 data travels as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

from . import plan
from .plan import (AG, HORING, HRING, RING, RS, Layout, accumulate_two_step, all_legal_strategies,  # noqa: F401
                   chunk_of_rank,
                   default_sched, fold_order, group_of, layout, owner_of_chunk, pack_slot,
                   schedule, segments, simulate, state_range, strategy_legal, volumes)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liborc.so")
_SRC = os.path.join(_HERE, "update.c")
_lib = None


def build(force: bool = True) -> str:
    """Compile update.c with gcc into oracle/liborc.so."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-fPIC",
               "-shared", "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_SO)
        i64, f32, f64, i32, vp = (ctypes.c_int64, ctypes.c_float, ctypes.c_double, ctypes.c_int,
                                  ctypes.c_void_p)
        L.orc_fold_bf16.argtypes = [vp, i32, i32, i64, vp]
        L.orc_fold_f32.argtypes = [vp, i32, i32, i64, vp]
        L.orc_sumsq.argtypes = [vp, i64]
        L.orc_sumsq.restype = f64
        L.orc_clip_coef.argtypes = [f64, f32, f32]
        L.orc_clip_coef.restype = f64
        for fn in (L.orc_adam64, L.orc_adam32):
            fn.argtypes = [i64, vp, vp, vp, vp, f64, f32, f32, f32, f32, f32, i32, i32]
        L.orc_bf16_rne.argtypes = [vp, i64, vp]
        L.orc_f16_rne.argtypes = [vp, i64, vp]
        L.orc_max_threads.restype = i32
        L.orc_set_threads.argtypes = [i32]
        _lib = L
    return _lib


def _ptr(a: np.ndarray) -> int:
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data


def threads() -> int:
    return int(lib().orc_max_threads())


def set_threads(n: int) -> None:
    lib().orc_set_threads(int(n))


# ------------------------------------------------------------------ arithmetic
def fold(srcs: Sequence[np.ndarray], group_len: int, out: Optional[np.ndarray] = None) -> np.ndarray:
    """srcs: the P contributions already listed in fold order; all uint16 (bf16
    bits) or all float32.  Returns the fp32 fold (see update.c)."""
    P = len(srcs)
    n = srcs[0].shape[0]
    assert P % group_len == 0 and all(s.shape[0] == n and s.dtype == srcs[0].dtype for s in srcs)
    if srcs[0].dtype == np.float16:                 # fp16 -> fp32 is exact
        srcs = [s.astype(np.float32) for s in srcs]
    srcs = [np.ascontiguousarray(s) for s in srcs]
    if out is None:
        out = np.empty(n, np.float32)
    assert out.dtype == np.float32 and out.shape[0] == n and out.flags["C_CONTIGUOUS"]
    ptrs = (ctypes.c_void_p * P)(*[_ptr(s) for s in srcs])
    if srcs[0].dtype == np.uint16:
        lib().orc_fold_bf16(ptrs, P, group_len, n, _ptr(out))
    elif srcs[0].dtype == np.float32:
        lib().orc_fold_f32(ptrs, P, group_len, n, _ptr(out))
    else:
        raise TypeError(srcs[0].dtype)
    return out


def sumsq(g: np.ndarray) -> float:
    assert g.dtype == np.float32
    g = np.ascontiguousarray(g)
    return float(lib().orc_sumsq(_ptr(g), g.shape[0]))


def clip_coef(total_sumsq: float, grad_scale: float, max_norm: float) -> float:
    return float(lib().orc_clip_coef(float(total_sumsq), float(grad_scale), float(max_norm)))


def adam(g, p, m, v, *, sc: float, lr, beta1, beta2, eps, weight_decay, step: int, adamw: bool = True,
         literal32: bool = False) -> None:
    """In-place Adam on fp32 arrays.  sc = grad_scale * clip coefficient (a
    double).  literal32 selects the all-fp32 evaluation, else fp64 rounded once."""
    for a in (g, p, m, v):
        assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"] and a.shape == g.shape
    fn = lib().orc_adam32 if literal32 else lib().orc_adam64
    fn(g.shape[0], _ptr(g), _ptr(p), _ptr(m), _ptr(v), float(sc), lr, beta1, beta2, eps, weight_decay,
       int(step), 1 if adamw else 0)


def bf16_rne(p: np.ndarray) -> np.ndarray:
    assert p.dtype == np.float32
    p = np.ascontiguousarray(p)
    out = np.empty(p.shape[0], np.uint16)
    lib().orc_bf16_rne(_ptr(p), p.shape[0], _ptr(out))
    return out


def f16_rne(p: np.ndarray) -> np.ndarray:
    """fp32 -> fp16 bit patterns, IEEE round to nearest even, overflow to infinity;
    a NaN becomes the quiet NaN of its sign (see update.c)."""
    assert p.dtype == np.float32
    p = np.ascontiguousarray(p)
    out = np.empty(p.shape[0], np.uint16)
    lib().orc_f16_rne(_ptr(p), p.shape[0], _ptr(out))
    return out


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    return (h.astype(np.uint32) << 16).view(np.float32)


# ------------------------------------------------------------- the path itself
def reduce_shard(lay: Layout, strategy: str, sched: int, rank: int, contribs, layout_kind: str = "chunk"):
    """Fold the P contributions over the rank's update range (the range of its
    optimizer state).  Every chunk inside the range is folded in the order of the
    reduce-scatter that delivers it to the chunk's owner, so replicas held by
    several ranks are identical.  Returns (g, sumsq over the rank's own chunk).

    chunk layout:   contribs[q] = array over the update range (uint16 or float32)
    tensor layout:  contribs[q][t] = rank q's full gradient of tensor t."""
    ob, ol = state_range(lay, rank, strategy[2])
    g = np.zeros(ol, np.float32)
    L = lay.L
    for c in range(ob // L, (ob + ol) // L):
        order, gl = fold_order(lay.P, lay.G, sched, c)
        lo = c * L - ob
        if layout_kind == "chunk":
            fold([contribs[q][lo:lo + L] for q in order], gl, out=g[lo:lo + L])
        else:
            for (t, toff, soff, n) in segments(lay, c * L, L):
                fold([contribs[q][t][toff:toff + n] for q in order], gl, out=g[lo + soff:lo + soff + n])
    own = chunk_of_rank(rank, lay.P, lay.G) * L - ob
    return g, sumsq(g[own:own + L])


def range_sumsq(lay: Layout, strategy: str, rank: int, g: np.ndarray) -> float:
    """Sum of squares over the rank's whole update range (g: the reduced gradient over that
    range): one sum per chunk, the chunks' sums added in chunk order.  It is the norm a rank can
    form on its own; where the optimizer state is sharded over all ranks it equals the
    own-chunk value reduce_shard returns."""
    ob, ol = state_range(lay, rank, strategy[2])
    assert g.shape[0] == ol
    tot = 0.0
    for lo in range(0, ol, lay.L):
        tot += sumsq(g[lo:lo + lay.L])
    return tot


def adam_shard(lay: Layout, strategy: str, rank: int, g, p, m, v, *, total_sumsq: float, hp: dict,
               step: int, no_decay: Optional[Sequence[int]] = None, literal32: bool = False) -> float:
    """Clip coefficient from the global sum of squares, then Adam over the update
    range, tensor by tensor where some tensors are exempt from weight decay.
    hp: lr, beta1, beta2, eps, weight_decay, grad_scale, max_norm, adamw,
    skip_nonfinite.  Returns the clip coefficient (NaN for a skipped step)."""
    f = np.float32
    if hp.get("skip_nonfinite", False) and not np.isfinite(total_sumsq):
        return float("nan")                            # overflow somewhere: the step is skipped, nothing changes
    coef = clip_coef(total_sumsq, f(hp["grad_scale"]), f(hp.get("max_norm", 0.0)))
    sc = float(f(hp["grad_scale"])) * coef
    kw = dict(sc=sc, lr=f(hp["lr"]), beta1=f(hp["beta1"]), beta2=f(hp["beta2"]), eps=f(hp["eps"]),
              step=step, adamw=bool(hp.get("adamw", True)), literal32=literal32)
    wd = f(hp["weight_decay"])
    if no_decay is None:
        adam(g, p, m, v, weight_decay=wd, **kw)
        return coef
    ob, ol = state_range(lay, rank, strategy[2])
    covered = 0
    for (t, _toff, soff, n) in segments(lay, ob, ol):
        s = slice(soff, soff + n)
        adam(g[s], p[s], m[s], v[s], weight_decay=f(0.0) if no_decay[t] else wd, **kw)
        covered = soff + n
    if covered < ol:                                  # padding: decays like any element; stays 0
        s = slice(covered, ol)
        adam(g[s], p[s], m[s], v[s], weight_decay=wd, **kw)
    return coef
