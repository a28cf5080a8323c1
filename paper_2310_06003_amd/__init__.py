"""Python binding of libparo (see include/paro.h): argument marshalling only.

Every step of the path runs inside the HIP library; there is no Python or CPU
fallback - if ``libparo.so`` has not been built, importing this package raises.
Functions carry the C names.  Device buffers are passed as integer addresses
(``tensor.data_ptr()``), streams as ``torch.cuda.current_stream().cuda_stream``.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import (POINTER, Structure, byref, c_char, c_char_p, c_double, c_float, c_int, c_int32, c_int64, c_uint8,
                    c_void_p)
from typing import List, Optional, Sequence, Tuple

# The caller's device buffers and streams come from PyTorch, which ships its own copy of the HIP
# runtime.  A process must run on ONE runtime: load torch's first, so that libparo.so's dependency on
# libamdhip64 binds to the copy that owns those buffers and streams (a second, separately loaded
# runtime sees no device).
import torch  # noqa: F401  (imported for its side effect on the loader)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libparo.so")

PARO_OK, PARO_EINVAL, PARO_ESTRATEGY, PARO_ERANGE, PARO_ENOMEM, PARO_EHIP, PARO_EALIGN = 0, -1, -2, -3, -4, -5, -6
PARO_SCHED_DEFAULT, PARO_RING, PARO_HRING, PARO_HORING = -1, 0, 1, 2
PARO_BF16, PARO_F32, PARO_F16 = 0, 1, 2
PARO_CHUNK, PARO_TENSORS = 0, 1
PARO_RS, PARO_AG = 0, 1
PARO_MAX_RANKS = 256
PARO_STATIC_MAX_CHUNK = 1 << 30

if not os.path.exists(_SO):
    raise ImportError(
        f"{_SO} is missing: build it first (python paper_2310_06003_amd/build.py, or __graft_entry__.build()). "
        "There is no fallback path.")
_lib = ctypes.CDLL(_SO)


class ParoError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libparo error {code}: {text}")
        self.code = code


class paro_plan_opts_t(Structure):
    _fields_ = [("sched", c_int32), ("align_elems", c_int32), ("grad_dtype", POINTER(c_uint8)),
                ("no_decay", POINTER(c_uint8)), ("pack_dtype", c_int32), ("reserved_", c_int32)]


class paro_seg_t(Structure):
    _fields_ = [("tensor", c_int64), ("tensor_off", c_int64), ("shard_off", c_int64), ("len", c_int64)]


class paro_msg_t(Structure):
    _fields_ = [("phase", c_int32), ("step", c_int32), ("ring", c_int32), ("send_to", c_int32),
                ("recv_from", c_int32), ("pad_", c_int32), ("send_off", c_int64), ("send_len", c_int64),
                ("recv_off", c_int64), ("recv_len", c_int64)]


class paro_adam_t(Structure):
    _fields_ = [("lr", c_float), ("beta1", c_float), ("beta2", c_float), ("eps", c_float),
                ("weight_decay", c_float), ("grad_scale", c_float), ("max_norm", c_float), ("step", c_int32),
                ("adamw", c_int32), ("skip_nonfinite", c_int32)]


class paro_cost_t(Structure):
    _fields_ = [(k, c_double) for k in ("mem_param", "mem_grad", "mem_os", "fwd_ag_intra", "fwd_ag_inter",
                                        "bwd_ag_intra", "bwd_ag_inter", "bwd_rs_intra", "bwd_rs_inter",
                                        "upd_g_intra", "upd_g_inter", "upd_ag_intra", "upd_ag_inter")] + \
               [("recommended", c_int32 * 4), ("derived", c_int32)]


EXPORTS = {
    "paro_strategy_legal": (c_int, [c_char_p]),
    "paro_plan": (c_int, [c_int, c_int, c_char_p, POINTER(c_int64), c_int64, POINTER(paro_plan_opts_t),
                          POINTER(c_void_p)]),
    "paro_plan_destroy": (None, [c_void_p]),
    "paro_total": (c_int64, [c_void_p]),
    "paro_shard_len": (c_int64, [c_void_p]),
    "paro_padded_total": (c_int64, [c_void_p]),
    "paro_sched": (c_int, [c_void_p]),
    "paro_chunk_of_rank": (c_int, [c_void_p, c_int]),
    "paro_owner_of_chunk": (c_int, [c_void_p, c_int]),
    "paro_range": (c_int, [c_void_p, c_int, c_char, POINTER(c_int64), POINTER(c_int64)]),
    "paro_segments": (c_int64, [c_void_p, c_int, POINTER(paro_seg_t), c_int64]),
    "paro_fold_order": (c_int, [c_void_p, c_int, POINTER(c_int32), POINTER(c_int32)]),
    "paro_schedule": (c_int64, [c_void_p, c_int, c_int, c_int, POINTER(paro_msg_t), c_int64]),
    "paro_pack_slot": (c_int, [c_void_p, c_int, POINTER(c_int64), POINTER(c_int64), POINTER(c_int64)]),
    "paro_reduce_shard": (c_int, [c_void_p, c_int, POINTER(c_void_p), c_int, c_void_p, c_void_p, c_void_p]),
    "paro_adam_shard": (c_int, [c_void_p, c_int, POINTER(paro_adam_t), c_void_p, c_void_p, c_void_p, c_void_p,
                                c_void_p, c_void_p, c_void_p]),
    "paro_pack_params": (c_int, [c_void_p, c_int, c_void_p, c_void_p, c_void_p]),
    "paro_step_fused": (c_int, [c_void_p, c_int, POINTER(c_void_p), c_int, POINTER(paro_adam_t), c_void_p, c_void_p,
                                c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
    "paro_step_fused_static": (c_int, [c_void_p, c_int, POINTER(c_void_p), POINTER(paro_adam_t), c_void_p, c_void_p,
                                       c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
    "paro_ring_hop": (c_int, [c_void_p, c_void_p, c_int, c_void_p, c_int, c_void_p, c_int64, c_void_p]),
    "paro_collective_step": (c_int64, [c_void_p, c_int, c_int, c_int, c_int, c_int, c_int, POINTER(c_void_p),
                                       c_void_p]),
    "paro_cost": (c_int, [c_char_p, c_double, c_double, c_int, c_int, c_int, c_int, c_int, POINTER(paro_cost_t)]),
    "paro_two_step_saving": (c_double, [c_double, c_int, c_int, c_int]),
    "paro_last_error": (c_char_p, []),
}
for _name, (_res, _args) in EXPORTS.items():
    _fn = getattr(_lib, _name)          # AttributeError here = a declared symbol is not exported
    _fn.restype = _res
    _fn.argtypes = _args


def paro_last_error() -> str:
    return (_lib.paro_last_error() or b"").decode()


def _check(rc: int) -> int:
    if rc < 0:
        raise ParoError(int(rc), paro_last_error())
    return int(rc)


def paro_strategy_legal(strategy: str) -> bool:
    return bool(_lib.paro_strategy_legal(strategy.encode()))


class Plan:
    """Owns a paro_plan_t*; destroyed with the object."""

    def __init__(self, handle: int, P: int, n_tensors: int):
        self.handle = c_void_p(handle)
        self.P = P
        self.n_tensors = n_tensors

    def __del__(self):
        h, self.handle = getattr(self, "handle", None), None
        if h and _lib is not None:          # at interpreter shutdown the module may already be torn down
            _lib.paro_plan_destroy(h)


def paro_plan(P: int, G: int, strategy: str, tensor_sizes: Sequence[int], *, sched: int = PARO_SCHED_DEFAULT,
              align_elems: int = 0, grad_dtype: Optional[Sequence[int]] = None,
              no_decay: Optional[Sequence[int]] = None, pack_dtype: int = PARO_BF16) -> Plan:
    T = len(tensor_sizes)
    sizes = (c_int64 * max(T, 1))(*tensor_sizes)
    opts = paro_plan_opts_t(sched, align_elems, None, None, pack_dtype, 0)
    keep = []
    if grad_dtype is not None:
        assert len(grad_dtype) == T
        a = (c_uint8 * T)(*grad_dtype)
        keep.append(a)
        opts.grad_dtype = ctypes.cast(a, POINTER(c_uint8))
    if no_decay is not None:
        assert len(no_decay) == T
        a = (c_uint8 * T)(*no_decay)
        keep.append(a)
        opts.no_decay = ctypes.cast(a, POINTER(c_uint8))
    out = c_void_p()
    _check(_lib.paro_plan(P, G, strategy.encode() if strategy is not None else None, sizes, T, byref(opts),
                          byref(out)))
    return Plan(out.value, P, T)


def paro_total(plan: Plan) -> int:
    return _check(_lib.paro_total(plan.handle))


def paro_shard_len(plan: Plan) -> int:
    return _check(_lib.paro_shard_len(plan.handle))


def paro_padded_total(plan: Plan) -> int:
    return _check(_lib.paro_padded_total(plan.handle))


def paro_sched(plan: Plan) -> int:
    return _check(_lib.paro_sched(plan.handle))


def paro_chunk_of_rank(plan: Plan, rank: int) -> int:
    return _check(_lib.paro_chunk_of_rank(plan.handle, rank))


def paro_owner_of_chunk(plan: Plan, chunk: int) -> int:
    return _check(_lib.paro_owner_of_chunk(plan.handle, chunk))


def paro_range(plan: Plan, rank: int, state: str) -> Tuple[int, int]:
    b, n = c_int64(), c_int64()
    _check(_lib.paro_range(plan.handle, rank, state.encode(), byref(b), byref(n)))
    return b.value, n.value


def paro_segments(plan: Plan, rank: int) -> List[Tuple[int, int, int, int]]:
    n = _check(_lib.paro_segments(plan.handle, rank, None, 0))
    buf = (paro_seg_t * max(n, 1))()
    _check(_lib.paro_segments(plan.handle, rank, buf, n))
    return [(s.tensor, s.tensor_off, s.shard_off, s.len) for s in buf[:n]]


def paro_fold_order(plan: Plan, chunk: int) -> Tuple[List[int], int]:
    ranks = (c_int32 * plan.P)()
    gl = c_int32()
    _check(_lib.paro_fold_order(plan.handle, chunk, ranks, byref(gl)))
    return list(ranks), gl.value


def paro_schedule(plan: Plan, rank: int, collective: int, sched: int = PARO_SCHED_DEFAULT) -> List[paro_msg_t]:
    n = _check(_lib.paro_schedule(plan.handle, rank, sched, collective, None, 0))
    buf = (paro_msg_t * max(n, 1))()
    _check(_lib.paro_schedule(plan.handle, rank, sched, collective, buf, n))
    return list(buf[:n])


def paro_pack_slot(plan: Plan, rank: int) -> Tuple[int, int, int]:
    a, b, c = c_int64(), c_int64(), c_int64()
    _check(_lib.paro_pack_slot(plan.handle, rank, byref(a), byref(b), byref(c)))
    return a.value, b.value, c.value


def make_adam(*, lr, beta1, beta2, eps, weight_decay, grad_scale, max_norm=0.0, step=1, adamw=True,
              skip_nonfinite=False) -> paro_adam_t:
    return paro_adam_t(lr, beta1, beta2, eps, weight_decay, grad_scale, max_norm, step, 1 if adamw else 0,
                       1 if skip_nonfinite else 0)


def _ptr_array(ptrs: Sequence[int]):
    return (c_void_p * len(ptrs))(*ptrs)


def paro_reduce_shard(plan: Plan, rank: int, contrib: Sequence[int], layout: int, grad_out: int, sumsq_out: int,
                      stream: int = 0) -> None:
    _check(_lib.paro_reduce_shard(plan.handle, rank, _ptr_array(contrib), layout, grad_out, sumsq_out, stream))


def paro_adam_shard(plan: Plan, rank: int, hp: paro_adam_t, grad: int, total_sumsq: int, p: int, m: int, v: int,
                    dst_base: int = 0, stream: int = 0) -> None:
    _check(_lib.paro_adam_shard(plan.handle, rank, byref(hp), grad, total_sumsq, p, m, v, dst_base, stream))


def paro_pack_params(plan: Plan, rank: int, p: int, dst_base: int, stream: int = 0) -> None:
    _check(_lib.paro_pack_params(plan.handle, rank, p, dst_base, stream))


def paro_step_fused(plan: Plan, rank: int, contrib: Sequence[int], layout: int, hp: paro_adam_t, grad_scratch: int,
                    sumsq_scratch: int, p: int, m: int, v: int, dst_base: int, stream: int = 0) -> None:
    _check(_lib.paro_step_fused(plan.handle, rank, _ptr_array(contrib), layout, byref(hp), grad_scratch,
                                sumsq_scratch, p, m, v, dst_base, stream))


def paro_step_fused_static(plan: Plan, rank: int, contrib: Sequence[int], hp: paro_adam_t, grad_scratch: int,
                           sumsq_scratch: int, p: int, m: int, v: int, dst_base: int, stream: int = 0) -> None:
    _check(_lib.paro_step_fused_static(plan.handle, rank, _ptr_array(contrib), byref(hp), grad_scratch,
                                       sumsq_scratch, p, m, v, dst_base, stream))


def paro_ring_hop(plan: Plan, partial_in: int, in_dtype: int, local: int, local_dtype: int, out: int, n: int,
                  stream: int = 0) -> None:
    _check(_lib.paro_ring_hop(plan.handle, partial_in, in_dtype, local, local_dtype, out, n, stream))


def paro_collective_step(plan: Plan, rank: int, sched: int, collective: int, phase: int, ring: int, step: int,
                         bufs: Sequence[int], stream: int = 0) -> int:
    return _check(_lib.paro_collective_step(plan.handle, rank, sched, collective, phase, ring, step,
                                            _ptr_array(bufs), stream))


def paro_cost(strategy: str, psi: float, psi_trainable: float, N: int, M: int, s: int, K: int = 12,
              sched: int = PARO_SCHED_DEFAULT) -> dict:
    out = paro_cost_t()
    _check(_lib.paro_cost(strategy.encode(), psi, psi_trainable, N, M, s, K, sched, byref(out)))
    d = {k: getattr(out, k) for k, _ in paro_cost_t._fields_ if k not in ("recommended", "derived")}
    d["recommended"] = list(out.recommended)
    d["derived"] = bool(out.derived)
    return d


def paro_two_step_saving(psi: float, N: int, M: int, s: int) -> float:
    return float(_lib.paro_two_step_saving(psi, N, M, s))
