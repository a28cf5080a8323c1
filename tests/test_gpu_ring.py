"""GPU parity for the steps around the Update stage: one ring hop / accumulation,
whole reduce-scatters and all-gathers played from the message tables over ranks
simulated as buffers in one GPU's memory, and gradient accumulation with the
grouped two-step reduce-scatter.  Everything here is bit-exact."""
import numpy as np
import pytest
import torch

import oracle as orc
import workloads as wl
from harness import DEV, np_of, stream

pytestmark = pytest.mark.gpu
SCHEDS = [orc.RING, orc.HRING, orc.HORING]
TD = {wl.BF16: torch.bfloat16, wl.F32: torch.float32}


def _as_f32(a):
    return orc.bf16_bits_to_f32(a) if a.dtype == np.uint16 else a


@pytest.mark.parametrize("n", [0, 1, 7, 8, 2048 * 3 + 5, 1 << 20])
def test_ring_hop_every_dtype_pair(paro, n):
    pl = paro.paro_plan(4, 2, "IIG", [4096])
    for da in (wl.BF16, wl.F32):
        for db in (wl.BF16, wl.F32):
            a = wl.draw(max(n, 8), 11 + da, dtype=da, device=DEV)
            b = wl.draw(max(n, 8), 13 + db, dtype=db, scale=1.0, device=DEV)
            out = torch.full((max(n, 8),), 7.0, dtype=torch.float32, device=DEV)
            paro.paro_ring_hop(pl, a.data_ptr(), da, b.data_ptr(), db, out.data_ptr(), n, stream())
            want = (_as_f32(np_of(a)) + _as_f32(np_of(b))).astype(np.float32)      # one fp32 add per element
            got = np_of(out)
            assert got[:n].tobytes() == want[:n].tobytes()
            assert (got[n:] == 7.0).all(), "wrote past n"
    # in place on an fp32 operand (accumulation)
    acc = wl.draw(max(n, 8), 17, dtype=wl.F32, device=DEV)
    x = wl.draw(max(n, 8), 19, dtype=wl.BF16, device=DEV)
    want = (np_of(acc) + _as_f32(np_of(x))).astype(np.float32)
    paro.paro_ring_hop(pl, acc.data_ptr(), wl.F32, x.data_ptr(), wl.BF16, acc.data_ptr(), n, stream())
    assert np_of(acc)[:n].tobytes() == want[:n].tobytes()
    with pytest.raises(paro.ParoError):
        paro.paro_ring_hop(pl, x.data_ptr(), wl.BF16, acc.data_ptr(), wl.F32, x.data_ptr(), n, stream())


def _play(paro, pl, P, sched, collective, bufs, phases=None):
    """Every rank's steps in schedule order: phase, then ring 0 before ring 1, then step."""
    keys = sorted({(m.phase, m.ring, m.step) for r in range(P) for m in paro.paro_schedule(pl, r, collective, sched)})
    ptrs = [b.data_ptr() for b in bufs]
    moved = 0
    for (phase, ring, step) in keys:
        if phases is not None and phase not in phases:
            continue
        for r in range(P):
            moved += paro.paro_collective_step(pl, r, sched, collective, phase, ring, step, ptrs, stream())
    return moved


@pytest.mark.parametrize("P,G", [(8, 4), (9, 3), (4, 4), (6, 1), (16, 8)])
def test_reduce_scatter_played_on_device_equals_the_fold(paro, P, G):
    total = P * 8 * 300 - 11
    lay = orc.layout(P, G, [total])
    L = lay.L
    contrib = wl.chunk_contribs(P, P * L, 23, device=DEV)             # bf16, one flat gradient per rank
    host = [np_of(c) for c in contrib]
    for sched in SCHEDS:
        pl = paro.paro_plan(P, G, "GGG", [total], sched=sched)
        work = [c.float() for c in contrib]                           # exact up-conversion
        moved = _play(paro, pl, P, sched, paro.PARO_RS, work)
        intra_inter = sum(sum(orc.volumes(lay, sched, r, orc.RS)) for r in range(P))
        assert moved == intra_inter
        sim = [orc.bf16_bits_to_f32(h) for h in host]
        orc.simulate(lay, sched, orc.RS, sim)
        for r in range(P):
            c = orc.chunk_of_rank(r, P, G)
            got = np_of(work[r][c * L:(c + 1) * L])
            assert got.tobytes() == sim[r][c * L:(c + 1) * L].tobytes(), (sched, r)
            # and the one-pass fold of the update stage gives the same bits
            g = torch.empty(L, dtype=torch.float32, device=DEV)
            paro.paro_reduce_shard(pl, r, [t[c * L:(c + 1) * L].data_ptr() for t in contrib], paro.PARO_CHUNK,
                                   g.data_ptr(), 0, stream())
            assert np_of(g).tobytes() == got.tobytes(), (sched, r)


@pytest.mark.parametrize("P,G", [(8, 4), (9, 3), (4, 4), (6, 1)])
def test_all_gather_played_on_device_completes(paro, P, G):
    total = P * 8 * 100 - 3
    lay = orc.layout(P, G, [total])
    L = lay.L
    full = wl.draw(P * L, 29, dtype=wl.BF16, scale=1.0, device=DEV)
    for sched in SCHEDS:
        pl = paro.paro_plan(P, G, "NGG", [total], sched=sched)
        bufs = []
        for r in range(P):
            b = torch.zeros(P * L, dtype=torch.bfloat16, device=DEV)
            c = orc.chunk_of_rank(r, P, G)
            b[c * L:(c + 1) * L] = full[c * L:(c + 1) * L]          # what paro_pack_params leaves in the slot
            bufs.append(b)
        moved = _play(paro, pl, P, sched, paro.PARO_AG, bufs)
        assert moved == P * (P - 1) * L                              # everybody receives everything else once
        for r in range(P):
            assert torch.equal(bufs[r], full), (sched, r)


@pytest.mark.parametrize("P,G,s", [(8, 4, 3), (4, 2, 2), (16, 8, 2)])
def test_accumulation_with_two_step_reduce_scatter(paro, P, G, s):
    """Sec. 3.3: per micro-batch an intra-group reduce-scatter, accumulation into the persistent
    gradient block, one inter-group reduce-scatter at the end - against the oracle, bit for bit."""
    total = P * 8 * 64
    lay = orc.layout(P, G, [total])
    L, g = lay.L, P // G
    pl = paro.paro_plan(P, G, "IIG", [total], sched=paro.PARO_HRING)
    mbs = [wl.chunk_contribs(P, P * L, 31 + b, device=DEV) for b in range(s)]
    acc = [None] * P
    for b in range(s):
        work = [c.float() for c in mbs[b]]
        _play(paro, pl, P, paro.PARO_HRING, paro.PARO_RS, work, phases={1})
        for r in range(P):
            lo, n = orc.state_range(lay, r, "I")
            if b == 0:
                acc[r] = work[r][lo:lo + n].clone()
            else:
                paro.paro_ring_hop(pl, acc[r].data_ptr(), wl.F32, work[r][lo:lo + n].data_ptr(), wl.F32,
                                   acc[r].data_ptr(), n, stream())
    work = []
    for r in range(P):
        w = torch.zeros(P * L, dtype=torch.float32, device=DEV)
        lo, n = orc.state_range(lay, r, "I")
        w[lo:lo + n] = acc[r]
        work.append(w)
    moved = _play(paro, pl, P, paro.PARO_HRING, paro.PARO_RS, work, phases={2})
    assert moved == P * (g - 1) * L                                   # Eq. 1's second term, once per mini-batch
    want = orc.accumulate_two_step(lay, [[orc.bf16_bits_to_f32(np_of(c)) for c in mb] for mb in mbs])
    for r in range(P):
        c = orc.chunk_of_rank(r, P, G)
        assert np_of(work[r][c * L:(c + 1) * L]).tobytes() == want[r].tobytes(), r
