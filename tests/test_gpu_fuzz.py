"""GPU parity on randomly drawn small configurations: cluster shape, strategy, schedule, tensor
list (empty, tiny, tile-sized and large tensors), gradient dtypes, weight-decay mask, layout,
alignment of the per-tensor gradients, clipping, decay style, with and without the per-tile
table, with sweep 1's two-blocks-per-wave shape forced on (it is otherwise kept for launches of
196 608 blocks and more).  Every rank of every configuration, fused entry point, full parity."""
import numpy as np
import pytest
import torch

import oracle as orc
import workloads as wl
from harness import DEV, PtrTable, compare_step, hp_dict, hp_struct, l2_terms, np_of, oracle_update, stream

pytestmark = pytest.mark.gpu

SHAPES = [(1, 1), (2, 1), (2, 2), (3, 1), (4, 2), (6, 3), (6, 2), (8, 4), (8, 8), (12, 4), (16, 8)]


def _draw_config(seed):
    rng = np.random.default_rng(1000 + seed)
    P, G = SHAPES[int(rng.integers(len(SHAPES)))]
    strategy = orc.all_legal_strategies()[int(rng.integers(14))]
    n_t = int(rng.integers(1, 40))
    kinds = rng.integers(0, 5, n_t)
    sizes = []
    for k in kinds:
        if k == 0:
            sizes.append(0)
        elif k == 1:
            sizes.append(int(rng.integers(1, 20)))
        elif k == 2:
            sizes.append(int(rng.integers(100, 5000)))
        elif k == 3:
            sizes.append(max(1, 2048 * int(rng.integers(1, 6)) + int(rng.integers(-9, 10))))
        else:
            sizes.append(256 * int(rng.integers(1, 40)) + int(rng.integers(-3, 4)))
    if sum(sizes) == 0:
        sizes[0] = 777
    tensors_layout = bool(rng.integers(2))
    if tensors_layout:
        dtypes = [int(x) for x in rng.integers(0, 3, n_t)]
    else:
        dtypes = [int(rng.integers(0, 3))] * n_t
    no_decay = [int(x) for x in rng.integers(0, 2, n_t)] if rng.integers(2) else None
    return dict(P=P, G=G, strategy=strategy, sizes=sizes, dtypes=dtypes, no_decay=no_decay,
                tensors_layout=tensors_layout, align=int(rng.choice([1, 4, 8, 128])),
                max_norm=float(rng.choice([0.0, 0.002])), adamw=bool(rng.integers(2)),
                sched=int(rng.choice([orc.RING, orc.HRING, orc.HORING])), table=bool(rng.integers(4)),
                step=int(rng.integers(1, 50)))


@pytest.mark.parametrize("seed", range(48))
def test_random_configuration(paro, seed, monkeypatch):
    c = _draw_config(seed)
    if not c["table"]:
        monkeypatch.setenv("PARO_TILE_TABLE_MAX_TILES", "0")
    if seed % 2:
        monkeypatch.setenv("PARO_PAIR_MIN_BLOCKS", "0")       # tensor layout, P <= 8: a wave takes two blocks
    P, G, strategy, sizes, dtypes, no_decay = c["P"], c["G"], c["strategy"], c["sizes"], c["dtypes"], c["no_decay"]
    lay = orc.layout(P, G, sizes)
    sched = c["sched"]
    pl = paro.paro_plan(P, G, strategy, sizes, sched=sched, grad_dtype=dtypes, no_decay=no_decay)
    hp = dict(hp_dict(P, max_norm=c["max_norm"]), adamw=c["adamw"])
    n = P * lay.L
    state = [np_of(t) for t in wl.master_state(n, 200 + seed)]
    for a in state:
        a[lay.total:] = 0
    if c["tensors_layout"]:
        sets = wl.tensor_contribs(P, sizes, dtypes, 300 + seed, 1, device=DEV, align_elems=c["align"])
        tables = [PtrTable(s.tensors) for s in sets]
        host = [[np_of(t) for t in s.tensors] for s in sets]
    else:
        dev = wl.chunk_contribs(P, n, 300 + seed, dtype=dtypes[0], device=DEV)
        for t in dev:
            t[lay.total:] = 0
        host = [np_of(t) for t in dev]
    what0 = f"seed {seed} {c}"
    for rank in range(P):
        ob, ol = orc.state_range(lay, rank, strategy[2])
        if c["tensors_layout"]:
            g_ref, ss_ref = orc.reduce_shard(lay, strategy, sched, rank, host, "tensors")
            ptrs, kind = [t.ptr() for t in tables], paro.PARO_TENSORS
        else:
            g_ref, ss_ref = orc.reduce_shard(lay, strategy, sched, rank, [h[ob:ob + ol] for h in host], "chunk")
            ptrs, kind = [t[ob:ob + ol].data_ptr() for t in dev], paro.PARO_CHUNK
        ss_ref = orc.range_sumsq(lay, strategy, rank, g_ref)      # the fused step's norm: over the whole update range
        old = [a[ob:ob + ol].copy() for a in state]
        ref = oracle_update(lay, strategy, rank, g_ref, *old, total_sumsq=ss_ref, hp=hp, step=c["step"], no_decay=no_decay)
        lit = oracle_update(lay, strategy, rank, g_ref, *old, total_sumsq=ss_ref, hp=hp, step=c["step"],
                            no_decay=no_decay, literal32=True)
        p, m, v = (torch.from_numpy(a.copy()).to(DEV) for a in old)
        dst_len, slot_off, slot_len = orc.pack_slot(lay, rank, strategy)
        dst = torch.zeros(dst_len, dtype=torch.bfloat16, device=DEV)
        gs = torch.empty(ol, dtype=torch.float32, device=DEV)
        ss = torch.zeros(1, dtype=torch.float64, device=DEV)
        paro.paro_step_fused(pl, rank, ptrs, kind, hp_struct(paro, hp, c["step"]), gs.data_ptr(), ss.data_ptr(),
                             p.data_ptr(), m.data_ptr(), v.data_ptr(), dst.data_ptr(), stream())
        what = f"{what0} rank {rank}"
        if c["max_norm"] > 0:
            assert np_of(gs).tobytes() == g_ref.tobytes(), what
            assert abs(float(ss.item()) - ss_ref) <= 1e-12 * max(ss_ref, 1e-300), what
        g_hat = float(np.float32(hp["grad_scale"])) * ref["coef"] * g_ref.astype(np.float64)
        g_terms = None
        if not c["adamw"]:
            decays = np.ones(ol, bool)
            if no_decay is not None:
                for (t, _toff, soff, ln) in orc.segments(lay, ob, ol):
                    decays[soff:soff + ln] = not no_decay[t]
            wd_p = np.where(decays, float(np.float32(hp["weight_decay"])) * old[0].astype(np.float64), 0.0)
            g_terms = np.abs(g_hat) + np.abs(wd_p)
            g_hat = g_hat + wd_p
        q_all = np_of(dst)
        got = dict(p=np_of(p), m=np_of(m), v=np_of(v), q=q_all[slot_off:slot_off + slot_len])
        compare_step(got, ref, p_old=old[0], m_old=old[1], g_hat=g_hat, g_terms=g_terms, v_old=old[2], what=what,
                     literal=lit, l2=None if c["adamw"] else l2_terms(hp, c["step"]))
        assert not q_all[:slot_off].any() and not q_all[slot_off + slot_len:].any(), what + ": wrote outside the slot"
