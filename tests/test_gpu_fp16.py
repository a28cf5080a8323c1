"""GPU parity of the fp16 + loss-scaling variant: fp16 gradient contributions (exact
up-conversion), un-scaling folded into grad_scale, fp16 packed parameters, and the
skipped step when a gradient has overflowed."""
import numpy as np
import pytest
import torch

import oracle as orc
import workloads as wl
from harness import DEV, PtrTable, compare_step, hp_dict, hp_struct, np_of, oracle_update, stream

pytestmark = pytest.mark.gpu
LOSS_SCALE = 1024.0


def _setup(paro, P, G, strategy, total, seed):
    lay = orc.layout(P, G, [total])
    pl = paro.paro_plan(P, G, strategy, [total], grad_dtype=[wl.F16], pack_dtype=paro.PARO_F16)
    n = P * lay.L
    dev = wl.chunk_contribs(P, n, seed, dtype=wl.F16, device=DEV)
    for t in dev:
        t.mul_(LOSS_SCALE)                         # what a scaled loss puts on the wire
    state = [np_of(t) for t in wl.master_state(n, seed)]
    return lay, pl, dev, state


def _step(paro, pl, lay, strategy, rank, dev, state, hp, step):
    ob, ol = orc.state_range(lay, rank, strategy[2])
    contrib = [t[ob:ob + ol] for t in dev]
    p0, m0, v0 = (a[ob:ob + ol].copy() for a in state)
    p, m, v = (torch.from_numpy(a.copy()).to(DEV) for a in (p0, m0, v0))
    dst_len, slot_off, slot_len = orc.pack_slot(lay, rank, strategy)
    dst = torch.full((dst_len,), 3.0, dtype=torch.float16, device=DEV)
    g = torch.empty(ol, dtype=torch.float32, device=DEV)
    ss = torch.zeros(1, dtype=torch.float64, device=DEV)
    paro.paro_step_fused(pl, rank, [c.data_ptr() for c in contrib], paro.PARO_CHUNK, hp_struct(paro, hp, step),
                         g.data_ptr(), ss.data_ptr(), p.data_ptr(), m.data_ptr(), v.data_ptr(), dst.data_ptr(),
                         stream())
    q = np_of(dst).view(np.uint16)
    got = dict(p=np_of(p), m=np_of(m), v=np_of(v), q=q[slot_off:slot_off + slot_len], g=np_of(g), ss=float(ss.item()),
               q_all=q)
    return got, (p0, m0, v0), [np_of(c) for c in contrib], (slot_off, slot_len)


@pytest.mark.parametrize("P,G,strategy", [(8, 4, "IIG"), (4, 2, "NIG"), (4, 4, "GGG")])
def test_fp16_step_with_loss_scale(paro, P, G, strategy):
    lay, pl, dev, state = _setup(paro, P, G, strategy, P * 8 * 700 + 24, seed=3)
    hp = hp_dict(P, max_norm=0.01, grad_scale=1.0 / (P * LOSS_SCALE), skip_nonfinite=True)
    for rank in (0, P - 1):
        got, (p0, m0, v0), host, _ = _step(paro, pl, lay, strategy, rank, dev, state, hp, 2)
        g_ref, ss_ref = orc.reduce_shard(lay, strategy, orc.default_sched(P, G), rank, host, "chunk")
        assert got["g"].tobytes() == g_ref.tobytes()
        assert abs(got["ss"] - ss_ref) <= 1e-12 * ss_ref
        ref = oracle_update(lay, strategy, rank, g_ref, p0, m0, v0, total_sumsq=ss_ref, hp=hp, step=2, fmt="f16")
        lit = oracle_update(lay, strategy, rank, g_ref, p0, m0, v0, total_sumsq=ss_ref, hp=hp, step=2, fmt="f16",
                            literal32=True)
        assert ref["coef"] < 1.0
        g_hat = float(np.float32(hp["grad_scale"])) * ref["coef"] * g_ref.astype(np.float64)
        compare_step(got, ref, p_old=p0, m_old=m0, g_hat=g_hat, what=f"fp16 {strategy} rank {rank}", literal=lit,
                     fmt="f16")
        assert (got["q"] == orc.f16_rne(got["p"])).all()


@pytest.mark.parametrize("poison", [float("inf"), float("-inf"), float("nan")])
def test_overflowed_gradient_skips_the_step(paro, poison):
    P, G, strategy = 8, 4, "IIG"
    lay, pl, dev, state = _setup(paro, P, G, strategy, P * 8 * 300, seed=4)
    rank = 5
    ob, ol = orc.state_range(lay, rank, "G")
    dev[2][ob + ol - 3] = poison                     # one element of one rank's contribution
    hp = hp_dict(P, max_norm=0.0, grad_scale=1.0 / (P * LOSS_SCALE), skip_nonfinite=True)
    got, (p0, m0, v0), host, (slot_off, slot_len) = _step(paro, pl, lay, strategy, rank, dev, state, hp, 1)
    assert not np.isfinite(got["ss"])
    g_ref, ss_ref = orc.reduce_shard(lay, strategy, orc.default_sched(P, G), rank, host, "chunk")
    assert not np.isfinite(ss_ref)
    fin = np.isfinite(g_ref)
    assert got["g"][fin].tobytes() == g_ref[fin].tobytes() and (~np.isfinite(got["g"][~fin])).all()
    ref = oracle_update(lay, strategy, rank, g_ref, p0, m0, v0, total_sumsq=ss_ref, hp=hp, step=1, fmt="f16")
    for k, old in (("p", p0), ("m", m0), ("v", v0)):
        assert got[k].tobytes() == old.tobytes() == ref[k].tobytes(), k
    assert (got["q_all"] == np.float16(3.0).view(np.uint16)).all(), "a skipped step must not pack"
    # without the flag the same input does update (and poisons the state): the flag is what skips
    hp2 = dict(hp, skip_nonfinite=False, max_norm=1.0)
    got2, *_ = _step(paro, pl, lay, strategy, rank, dev, state, hp2, 1)
    assert not np.isfinite(got2["p"]).all()


@pytest.mark.parametrize("strategy", ["III", "NNN"])
def test_overflow_outside_the_own_chunk_skips_every_replica(paro, strategy):
    """Optimizer state sharded inside the group only / not at all: a rank updates chunks that other
    ranks own.  The fused step's norm covers the whole update range, so an overflowed gradient in
    ANY chunk of it skips the step, and every rank that holds a replica of that chunk skips alike
    (with the norm of the own chunk alone the replicas would part ways)."""
    P, G = 4, 2
    lay, pl, dev, state = _setup(paro, P, G, strategy, P * 8 * 600, seed=6)
    victim = 2 * lay.L + 77                          # flat index inside chunk 2 (owner: rank 1)
    dev[3][victim] = float("inf")
    hp = hp_dict(P, max_norm=0.0, grad_scale=1.0 / (P * LOSS_SCALE), skip_nonfinite=True)
    sched = orc.default_sched(P, G)
    for rank in range(P):
        ob, ol = orc.state_range(lay, rank, strategy[2])
        covers = ob <= victim < ob + ol
        got, (p0, m0, v0), host, _ = _step(paro, pl, lay, strategy, rank, dev, state, hp, 1)
        g_ref, own_ss = orc.reduce_shard(lay, strategy, sched, rank, host, "chunk")
        total = orc.range_sumsq(lay, strategy, rank, g_ref)
        ref = oracle_update(lay, strategy, rank, g_ref, p0, m0, v0, total_sumsq=total, hp=hp, step=1, fmt="f16")
        if covers:
            assert not np.isfinite(got["ss"]) and not np.isfinite(total)
            if orc.chunk_of_rank(rank, P, G) != 2:
                assert np.isfinite(own_ss), "the rank's own chunk is clean: only the range-wide norm sees the overflow"
            for k, old in (("p", p0), ("m", m0), ("v", v0)):
                assert got[k].tobytes() == old.tobytes() == ref[k].tobytes(), (rank, k)
            assert (got["q_all"] == np.float16(3.0).view(np.uint16)).all()
        else:
            assert np.isfinite(got["ss"]) and abs(got["ss"] - total) <= 1e-12 * total
            lit = oracle_update(lay, strategy, rank, g_ref, p0, m0, v0, total_sumsq=total, hp=hp, step=1, fmt="f16",
                                literal32=True)
            g_hat = float(np.float32(hp["grad_scale"])) * g_ref.astype(np.float64)
            compare_step(got, ref, p_old=p0, m_old=m0, g_hat=g_hat, what=f"{strategy} rank {rank}", literal=lit, fmt="f16")
    assert strategy != "NNN" or all(orc.state_range(lay, r, "N")[1] == P * lay.L for r in range(P))


def test_tensor_layout_with_three_dtypes(paro):
    rng = np.random.default_rng(9)
    sizes = [int(s) for s in rng.integers(0, 12, 30)] + [4100, 1, 9000, 2047, 6, 3000]
    dtypes = [int(x) for x in rng.integers(0, 3, len(sizes))]
    P, G, strategy = 4, 2, "IIG"
    lay = orc.layout(P, G, sizes)
    for align in (1, 128):
        pl = paro.paro_plan(P, G, strategy, sizes, grad_dtype=dtypes)
        sets = wl.tensor_contribs(P, sizes, dtypes, 70, 1, device=DEV, align_elems=align)
        tables = [PtrTable(s.tensors) for s in sets]
        host = [[np_of(t) for t in s.tensors] for s in sets]
        for rank in range(P):
            ob, ol = orc.state_range(lay, rank, "G")
            g = torch.empty(ol, dtype=torch.float32, device=DEV)
            ss = torch.zeros(1, dtype=torch.float64, device=DEV)
            paro.paro_reduce_shard(pl, rank, [t.ptr() for t in tables], paro.PARO_TENSORS, g.data_ptr(), ss.data_ptr(),
                                   stream())
            g_ref, ss_ref = orc.reduce_shard(lay, strategy, orc.default_sched(P, G), rank, host, "tensors")
            assert np_of(g).tobytes() == g_ref.tobytes(), (align, rank)
            assert abs(float(ss.item()) - ss_ref) <= 1e-12 * ss_ref


def test_ring_hop_with_fp16(paro):
    pl = paro.paro_plan(4, 2, "IIG", [4096])
    n = 2048 * 5 + 3
    a = wl.draw(n + 5, 1, dtype=wl.F16, scale=1.0, device=DEV)
    for db in (wl.BF16, wl.F32, wl.F16):
        b = wl.draw(n + 5, 2, dtype=db, scale=1.0, device=DEV)
        out = torch.zeros(n + 5, dtype=torch.float32, device=DEV)
        paro.paro_ring_hop(pl, a.data_ptr(), wl.F16, b.data_ptr(), db, out.data_ptr(), n, stream())
        fb = np_of(b)
        fb = orc.bf16_bits_to_f32(fb) if fb.dtype == np.uint16 else fb.astype(np.float32)
        want = (np_of(a).astype(np.float32) + fb).astype(np.float32)
        assert np_of(out)[:n].tobytes() == want[:n].tobytes() and not np_of(out)[n:].any()
