"""Shared plumbing of the GPU parity tests: moves seeded inputs to both sides and
compares.  Holds no arithmetic of the method."""
from __future__ import annotations

import numpy as np
import torch

import oracle as orc
import workloads as wl
from parity import check_bf16_within_one_ulp, check_moments_and_params, ulp_distance_f32

DEV = "cuda:0"


def np_of(t: torch.Tensor) -> np.ndarray:
    """torch tensor -> numpy; bf16 travels as uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()            # float16 stays float16: numpy knows the format


def stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def hp_dict(P, max_norm=0.0, adamw=True, **over):
    hp = dict(wl.ADAM_DEFAULT)
    hp.update(grad_scale=1.0 / P, max_norm=max_norm, adamw=adamw)
    hp.update(over)
    return hp


def hp_struct(paro, hp, step):
    return paro.make_adam(lr=hp["lr"], beta1=hp["beta1"], beta2=hp["beta2"], eps=hp["eps"],
                          weight_decay=hp["weight_decay"], grad_scale=hp["grad_scale"],
                          max_norm=hp["max_norm"], step=step, adamw=hp["adamw"],
                          skip_nonfinite=hp.get("skip_nonfinite", False))


class PtrTable:
    """Device array of per-tensor device pointers for one simulated rank."""

    def __init__(self, tensors):
        self.keep = tensors
        # an absent tensor (None: outside the range the step covers) gets a valid address all the same
        spare = next(t for t in tensors if t is not None).data_ptr()
        ptrs = [spare if t is None else (t.data_ptr() if t.numel() else 0) for t in tensors]
        self.table = torch.tensor(ptrs, dtype=torch.int64, device=DEV)

    def ptr(self):
        return self.table.data_ptr()


def l2_terms(hp, step):
    """What parity.check_moments_and_params needs to propagate an error of the L2-decayed
    gradient into the parameter: the step's scalars, formed as the contract forms them."""
    f = np.float32
    b1, b2 = float(f(hp["beta1"])), float(f(hp["beta2"]))
    bc1, bc2 = float(f(1.0 - b1 ** step)), float(f(1.0 - b2 ** step))
    return dict(step_size=float(f(hp["lr"])) / bc1, sqrt_bc2=float(np.sqrt(bc2)), eps=float(f(hp["eps"])))


def compare_step(gpu, ref, *, p_old, m_old, g_hat, what, report=None, hist=None, literal=None, fmt="bf16",
                 g_terms=None, v_old=None, l2=None):
    """gpu / ref: dicts with p, m, v (fp32 numpy) and q (uint16 bf16 bits).  ref is the
    fp64 evaluation (the 1e-6 contract).  literal, when given, is the oracle's all-fp32
    evaluation in the kernel's operation order: IEEE arithmetic leaves no freedom there,
    so it must match bit for bit."""
    tol_p = check_moments_and_params(gpu["p"], gpu["m"], gpu["v"], ref["p"], ref["m"], ref["v"], p_old=p_old,
                                     m_old=m_old, g_hat=g_hat, what=what, hist=hist, g_terms=g_terms, v_old=v_old,
                                     l2=l2)
    check_bf16_within_one_ulp(gpu["q"], ref["q"], what, ref_p=ref["p"], tol_p=tol_p, fmt=fmt)
    if literal is not None:
        for k in ("p", "m", "v", "q"):
            a, b = gpu[k], literal[k]
            if k != "q":        # +0 and -0 are the same value (they differ only for masked-out weight decay)
                a, b = a + np.float32(0), b + np.float32(0)
            assert a.tobytes() == b.tobytes(), f"{what}: {k} differs from the fp32-literal oracle"
    if report is not None:
        report.append((what, ulp_distance_f32(gpu["p"], ref["p"]), ulp_distance_f32(gpu["v"], ref["v"])))


def oracle_update(lay, strategy, rank, g, p, m, v, *, total_sumsq, hp, step, no_decay=None, literal32=False,
                  fmt="bf16"):
    """Oracle Adam + pack on copies; returns dict(p, m, v, q, coef)."""
    p, m, v = p.copy(), m.copy(), v.copy()
    coef = orc.adam_shard(lay, strategy, rank, g, p, m, v, total_sumsq=total_sumsq, hp=hp, step=step,
                          no_decay=no_decay, literal32=literal32)
    return dict(p=p, m=m, v=v, q=orc.f16_rne(p) if fmt == "f16" else orc.bf16_rne(p), coef=coef)
