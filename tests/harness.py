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


def flat_inputs(P, n, seed, dtype=wl.BF16, integer=False, dist="normal"):
    dev = wl.chunk_contribs(P, n, seed, dtype=dtype, device=DEV, integer=integer, dist=dist)
    return dev, [np_of(t) for t in dev]


def run_rank(paro, pl, lay, strategy, sched, rank, dev, host, state, hp, step, report=None, check_unfused=True):
    """One rank, chunk layout: reduce, fused step, unfused step; all against the oracle.
    lay.align must be the plan's alignment."""
    ob, ol = orc.state_range(lay, rank, strategy[2])
    contrib = [t[ob:ob + ol] for t in dev]
    g = torch.empty(ol, dtype=torch.float32, device=DEV)
    ss = torch.zeros(1, dtype=torch.float64, device=DEV)
    paro.paro_reduce_shard(pl, rank, [c.data_ptr() for c in contrib], paro.PARO_CHUNK, g.data_ptr(), ss.data_ptr(),
                           stream())
    g_ref, ss_ref = orc.reduce_shard(lay, strategy, sched, rank, [h[ob:ob + ol] for h in host], "chunk")
    g_gpu = np_of(g)
    what = f"{strategy}/sched{sched}/rank{rank}"
    assert g_gpu.tobytes() == g_ref.tobytes(), what + ": reduced gradient differs"
    assert abs(float(ss.item()) - ss_ref) <= 1e-12 * ss_ref, what

    p0, m0, v0 = (a[ob:ob + ol].copy() for a in state)
    # the fused step forms its norm over the rank's whole update range (= the own-chunk value where the
    # optimizer state is sharded over all ranks); the split calls below are handed the same total
    total = orc.range_sumsq(lay, strategy, rank, g_ref)
    if strategy[2] == "G":
        assert total == ss_ref
    ref = oracle_update(lay, strategy, rank, g_ref, p0, m0, v0, total_sumsq=total, hp=hp, step=step)
    lit = oracle_update(lay, strategy, rank, g_ref, p0, m0, v0, total_sumsq=total, hp=hp, step=step, literal32=True)
    g_hat = float(np.float32(hp["grad_scale"])) * ref["coef"] * g_ref.astype(np.float64)

    dst_len, slot_off, slot_len = orc.pack_slot(lay, rank, strategy)
    assert slot_len == ol

    def fresh():
        return [torch.from_numpy(a.copy()).to(DEV) for a in (p0, m0, v0)]

    # fused
    p, m, v = fresh()
    dst = torch.zeros(dst_len, dtype=torch.bfloat16, device=DEV)
    gs = torch.empty(ol, dtype=torch.float32, device=DEV)
    ss2 = torch.zeros(1, dtype=torch.float64, device=DEV)
    paro.paro_step_fused(pl, rank, [c.data_ptr() for c in contrib], paro.PARO_CHUNK, hp_struct(paro, hp, step),
                         gs.data_ptr(), ss2.data_ptr(), p.data_ptr(), m.data_ptr(), v.data_ptr(), dst.data_ptr(),
                         stream())
    q_all = np_of(dst)
    fused = dict(p=np_of(p), m=np_of(m), v=np_of(v), q=q_all[slot_off:slot_off + slot_len])
    compare_step(fused, ref, p_old=p0, m_old=m0, g_hat=g_hat, what=what + " fused", report=report, literal=lit)
    assert (fused["q"] == orc.bf16_rne(fused["p"])).all(), what + ": pack is not the rounding of the stored p"
    assert not q_all[:slot_off].any() and not q_all[slot_off + slot_len:].any(), what + ": wrote outside the slot"
    if hp["max_norm"] > 0:
        assert np_of(gs).tobytes() == g_ref.tobytes() and abs(float(ss2.item()) - total) <= 1e-12 * total

    if check_unfused:
        p, m, v = fresh()
        dst2 = torch.zeros(dst_len, dtype=torch.bfloat16, device=DEV)
        tot = torch.tensor([total], dtype=torch.float64, device=DEV)
        paro.paro_adam_shard(pl, rank, hp_struct(paro, hp, step), g.data_ptr(), tot.data_ptr(), p.data_ptr(),
                             m.data_ptr(), v.data_ptr(), 0, stream())
        paro.paro_pack_params(pl, rank, p.data_ptr(), dst2.data_ptr(), stream())
        for name, t in (("p", p), ("m", m), ("v", v)):
            assert np_of(t).tobytes() == fused[name].tobytes(), what + f": unfused {name} differs from fused"
        assert np_of(dst2).tobytes() == q_all.tobytes()
    return fused, ref
