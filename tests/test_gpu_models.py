"""GPU parity on the model-shaped tensor lists: the GPT-2-small-shaped list
(P=8, G=8, three steps, clipping with the true global norm) and the ragged
10,000-tensor list (P=8, G=4, Student-t gradients, mixed fp32/bf16 inputs,
five steps).  Every rank, every step, full parity."""
import numpy as np
import pytest
import torch

import oracle as orc
import workloads as wl
from harness import DEV, PtrTable, compare_step, hp_dict, hp_struct, np_of, oracle_update, stream

pytestmark = pytest.mark.gpu


def _host_views(ts: wl.TensorSet, sizes, dtypes):
    """numpy views of a rank's tensors, copied to the host one flat stream at a time."""
    flat = {k: np_of(v) for k, v in ts.flat.items()}
    out = []
    for t, n in enumerate(sizes):
        k = dtypes[t] if dtypes is not None else wl.BF16
        out.append(flat[k][ts.start[t]:ts.start[t] + n])
    return out


def _multi_step(paro, cfg, strategy, steps, seed, *, fused):
    P, G, sizes = cfg.P, cfg.G, cfg.sizes
    lay = orc.layout(P, G, sizes)
    sched = orc.default_sched(P, G)
    pl = paro.paro_plan(P, G, strategy, sizes, grad_dtype=cfg.dtypes, no_decay=cfg.no_decay)
    n = P * lay.L
    state = [np_of(t) for t in wl.master_state(n, seed)]
    for a in state:
        a[lay.total:] = 0
    rng = [orc.state_range(lay, r, strategy[2]) for r in range(P)]
    ora = [[a[b:b + ln].copy() for a in state] for (b, ln) in rng]
    lit = [[a.copy() for a in st] for st in ora]
    gpu = [[torch.from_numpy(a.copy()).to(DEV) for a in st] for st in ora]
    hist = [dict() for _ in range(P)]
    hp = hp_dict(P, max_norm=cfg.max_norm)
    coefs = []
    for step in range(1, steps + 1):
        sets = wl.tensor_contribs(P, sizes, cfg.dtypes, seed, step, dist=cfg.dist, device=DEV)
        tables = [PtrTable(s.tensors) for s in sets]
        host = [_host_views(s, sizes, cfg.dtypes) for s in sets]
        ptrs = [t.ptr() for t in tables]
        # sweep 1 on every rank
        g_gpu, ss_gpu, g_ref, ss_ref = [], [], [], []
        for r in range(P):
            ol = rng[r][1]
            g = torch.empty(ol, dtype=torch.float32, device=DEV)
            ss = torch.zeros(1, dtype=torch.float64, device=DEV)
            if not fused:
                paro.paro_reduce_shard(pl, r, ptrs, paro.PARO_TENSORS, g.data_ptr(), ss.data_ptr(), stream())
            gr, sr = orc.reduce_shard(lay, strategy, sched, r, host, "tensors")
            if not fused:
                assert np_of(g).tobytes() == gr.tobytes(), f"step {step} rank {r}: reduced gradient differs"
                assert abs(float(ss.item()) - sr) <= 1e-12 * sr
            g_gpu.append(g)
            ss_gpu.append(ss)
            g_ref.append(gr)
            ss_ref.append(sr)
        # the cross-rank sum of the norm contributions: the harness stands in for the all-reduce
        total_ref = 0.0
        for s in ss_ref:
            total_ref += s
        if not fused:
            total_gpu = 0.0
            for s in ss_gpu:
                total_gpu += float(s.item())
            tot = torch.tensor([total_gpu], dtype=torch.float64, device=DEV)
        for r in range(P):
            ob, ol = rng[r]
            p, m, v = gpu[r]
            dst_len, slot_off, slot_len = orc.pack_slot(lay, r, strategy)
            dst = torch.zeros(dst_len, dtype=torch.bfloat16, device=DEV)
            if fused:      # one call; the norm is this rank's own
                total = ss_ref[r]
                paro.paro_step_fused(pl, r, ptrs, paro.PARO_TENSORS, hp_struct(paro, hp, step), g_gpu[r].data_ptr(),
                                     ss_gpu[r].data_ptr(), p.data_ptr(), m.data_ptr(), v.data_ptr(), dst.data_ptr(),
                                     stream())
                assert np_of(g_gpu[r]).tobytes() == g_ref[r].tobytes()
            else:
                total = total_ref
                paro.paro_adam_shard(pl, r, hp_struct(paro, hp, step), g_gpu[r].data_ptr(), tot.data_ptr(),
                                     p.data_ptr(), m.data_ptr(), v.data_ptr(), 0, stream())
                paro.paro_pack_params(pl, r, p.data_ptr(), dst.data_ptr(), stream())
            ref = oracle_update(lay, strategy, r, g_ref[r], *ora[r], total_sumsq=total, hp=hp, step=step,
                                no_decay=cfg.no_decay)
            li = oracle_update(lay, strategy, r, g_ref[r], *lit[r], total_sumsq=total, hp=hp, step=step,
                               no_decay=cfg.no_decay, literal32=True)
            g_hat = float(np.float32(hp["grad_scale"])) * ref["coef"] * g_ref[r].astype(np.float64)
            q_all = np_of(dst)
            got = dict(p=np_of(p), m=np_of(m), v=np_of(v), q=q_all[slot_off:slot_off + slot_len])
            compare_step(got, ref, p_old=ora[r][0], m_old=ora[r][1], g_hat=g_hat,
                         what=f"{cfg.name} {strategy} step {step} rank {r}", hist=hist[r], literal=li)
            assert not q_all[:slot_off].any() and not q_all[slot_off + slot_len:].any()
            ora[r] = [ref["p"], ref["m"], ref["v"]]
            lit[r] = [li["p"], li["m"], li["v"]]
            coefs.append(ref["coef"])
        del sets, tables, host
    return coefs


def test_gpt2_small_three_steps_true_global_norm(paro):
    cfg = wl.config("gpt2")
    assert sum(cfg.sizes) == 124_356_864 and len(cfg.sizes) == 100
    coefs = _multi_step(paro, cfg, "NGG", cfg.steps, seed=2, fused=False)
    print(f"\n[gpt2 NGG] clip coefficients per step: {sorted(set(round(c, 6) for c in coefs))}")


def test_gpt2_small_fused_step(paro):
    cfg = wl.config("gpt2")
    _multi_step(paro, cfg, "GGG", 1, seed=2, fused=True)


def test_ragged_five_steps_clipping_triggers(paro):
    cfg = wl.config("ragged")
    assert len(cfg.sizes) == 10000 and min(cfg.sizes) >= 1 and max(cfg.sizes) <= 65536
    coefs = _multi_step(paro, cfg, cfg.strategy, cfg.steps, seed=5, fused=False)
    assert max(coefs) < 1.0, "the heavy-tailed gradients must trigger clipping"
    print(f"\n[ragged] Psi = {sum(cfg.sizes)}, clip coefficient range {min(coefs):.4f} .. {max(coefs):.4f}")


def test_ragged_fused_two_steps(paro):
    cfg = wl.config("ragged")
    _multi_step(paro, cfg, cfg.strategy, 2, seed=6, fused=True)
