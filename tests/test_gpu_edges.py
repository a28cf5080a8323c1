"""GPU parity on inputs and plans at the edges of the contract: signed zeros, non-finite
gradient contributions without the skip, a plan alignment other than the default, update
ranges of several chunks at a size where every chunk is thousands of blocks."""
import numpy as np
import pytest
import torch

import oracle as orc
import workloads as wl
from harness import (DEV, PtrTable, compare_step, flat_inputs, hp_dict, hp_struct, np_of, oracle_update, run_rank,
                     stream)

pytestmark = pytest.mark.gpu

SCHEDS = [orc.RING, orc.HRING, orc.HORING]
NP_DTYPE = {wl.BF16: np.uint16, wl.F32: np.float32, wl.F16: np.float16}


def _to_dev(a: np.ndarray, dtype: int) -> torch.Tensor:
    """numpy bit patterns -> device tensor of the gradient dtype."""
    if dtype == wl.BF16:
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).to(DEV)
    return torch.from_numpy(a.copy()).to(DEV)


def _signed_zero_mix(n, P, dtype, seed):
    """Per rank: values from {-0, +0, x, -x} with many zeros, so that sums of only -0, sums with
    one +0 among -0s, and exact cancellations x + (-x) all occur.  Elements [0, 64) are -0 in
    every rank.  Returned as numpy arrays of the dtype's storage type."""
    rng = np.random.default_rng(seed)
    x = rng.integers(1, 5, n).astype(np.float32)
    out = []
    for _ in range(P):
        kind = rng.choice(4, n, p=[0.55, 0.15, 0.15, 0.15])
        v = np.where(kind == 0, np.float32(-0.0), np.where(kind == 1, np.float32(0.0), np.where(kind == 2, x, -x)))
        v = v.astype(np.float32)
        v[:64] = -0.0
        if dtype == wl.BF16:
            out.append((v.view(np.uint32) >> 16).astype(np.uint16))       # small integers and zeros: exact in bf16
        elif dtype == wl.F16:
            out.append(v.astype(np.float16))
        else:
            out.append(v)
    return out


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32, wl.F16])
def test_signed_zeros_chunk_layout(paro, dtype):
    """An element whose contributions are all -0 comes out -0 (the fold never adds to a +0 start
    value), and every other mix of zeros gives the oracle's sign: the reduced gradient bit for bit."""
    P, G = 8, 4
    sizes = [P * (2048 * 3 + 264)]
    lay = orc.layout(P, G, sizes)
    n = P * lay.L
    host = _signed_zero_mix(n, P, dtype, seed=5)
    dev = [_to_dev(h, dtype) for h in host]
    host_o = [h for h in host]
    seen_neg_zero = 0
    for sched in SCHEDS:
        for strategy in ("IIG", "NNN"):
            pl = paro.paro_plan(P, G, strategy, sizes, sched=sched, grad_dtype=[dtype])
            for rank in (0, 3, 6):
                ob, ol = orc.state_range(lay, rank, strategy[2])
                g = torch.empty(ol, dtype=torch.float32, device=DEV)
                ss = torch.zeros(1, dtype=torch.float64, device=DEV)
                paro.paro_reduce_shard(pl, rank, [t[ob:ob + ol].data_ptr() for t in dev], paro.PARO_CHUNK, g.data_ptr(),
                                       ss.data_ptr(), stream())
                g_ref, ss_ref = orc.reduce_shard(lay, strategy, sched, rank, [h[ob:ob + ol] for h in host_o], "chunk")
                got = np_of(g)
                assert got.tobytes() == g_ref.tobytes(), (sched, strategy, rank)
                assert float(ss.item()) == ss_ref                 # small integers: exact
                bits = got.view(np.uint32)
                if ob == 0:
                    assert (bits[:64] == 0x80000000).all(), "all -0 contributions must give -0"
                seen_neg_zero += int((bits == 0x80000000).sum())
                assert (bits == 0).sum() > 0
    assert seen_neg_zero > 1000


def _tensor_rank(paro, pl, lay, strategy, sched, rank, tables, host, state, hp, step, no_decay=None, what=""):
    """One rank, tensor layout: fused step against the oracle (reduced gradient and sum of
    squares when the step stores them)."""
    ob, ol = orc.state_range(lay, rank, strategy[2])
    g_ref, _own = orc.reduce_shard(lay, strategy, sched, rank, host, "tensors")
    ss_ref = orc.range_sumsq(lay, strategy, rank, g_ref)          # the fused step's norm: over the whole update range
    old = [a[ob:ob + ol].copy() for a in state]
    ref = oracle_update(lay, strategy, rank, g_ref, *old, total_sumsq=ss_ref, hp=hp, step=step, no_decay=no_decay)
    lit = oracle_update(lay, strategy, rank, g_ref, *old, total_sumsq=ss_ref, hp=hp, step=step, no_decay=no_decay,
                        literal32=True)
    p, m, v = (torch.from_numpy(a.copy()).to(DEV) for a in old)
    dst_len, slot_off, slot_len = orc.pack_slot(lay, rank, strategy)
    dst = torch.zeros(dst_len, dtype=torch.bfloat16, device=DEV)
    gs = torch.empty(ol, dtype=torch.float32, device=DEV)
    ss = torch.zeros(1, dtype=torch.float64, device=DEV)
    paro.paro_step_fused(pl, rank, [t.ptr() for t in tables], paro.PARO_TENSORS, hp_struct(paro, hp, step),
                         gs.data_ptr(), ss.data_ptr(), p.data_ptr(), m.data_ptr(), v.data_ptr(), dst.data_ptr(), stream())
    what = f"{what} {strategy} sched{sched} rank{rank}"
    if hp["max_norm"] > 0:
        assert np_of(gs).tobytes() == g_ref.tobytes(), what + ": reduced gradient"
        assert abs(float(ss.item()) - ss_ref) <= 1e-12 * ss_ref, what
    g_hat = float(np.float32(hp["grad_scale"])) * ref["coef"] * g_ref.astype(np.float64)
    q_all = np_of(dst)
    got = dict(p=np_of(p), m=np_of(m), v=np_of(v), q=q_all[slot_off:slot_off + slot_len])
    compare_step(got, ref, p_old=old[0], m_old=old[1], g_hat=g_hat, what=what, literal=lit)
    assert not q_all[:slot_off].any() and not q_all[slot_off + slot_len:].any(), what + ": wrote outside the slot"
    return got


def test_signed_zeros_tensor_layout(paro):
    """The same in the tensor layout, with tensor boundaries inside blocks (per-lane loads) and
    padding at the end (whose gradient is +0)."""
    P, G, strategy = 4, 2, "IIG"
    sizes = [700, 3, 2048 * 3, 1, 5000, 0, 2049, 9001]
    dtypes = [wl.BF16, wl.F32, wl.F16, wl.BF16, wl.F32, wl.BF16, wl.F16, wl.BF16]
    lay = orc.layout(P, G, sizes)
    per_rank = [[] for _ in range(P)]
    for t, (s, dt) in enumerate(zip(sizes, dtypes)):
        vals = _signed_zero_mix(max(s, 64), P, dt, seed=20 + t)
        for q in range(P):
            per_rank[q].append(vals[q][:s])
    dev_sets = [[_to_dev(a, dt) if a.size else torch.empty(0, dtype=wl.TORCH_DTYPE[dt], device=DEV)
                 for a, dt in zip(per_rank[q], dtypes)] for q in range(P)]
    tables = [PtrTable(ts) for ts in dev_sets]
    pl = paro.paro_plan(P, G, strategy, sizes, grad_dtype=dtypes)
    sched = orc.default_sched(P, G)
    neg = 0
    for rank in range(P):
        ob, ol = orc.state_range(lay, rank, strategy[2])
        g = torch.empty(ol, dtype=torch.float32, device=DEV)
        ss = torch.zeros(1, dtype=torch.float64, device=DEV)
        paro.paro_reduce_shard(pl, rank, [t.ptr() for t in tables], paro.PARO_TENSORS, g.data_ptr(), ss.data_ptr(),
                               stream())
        g_ref, ss_ref = orc.reduce_shard(lay, strategy, sched, rank, per_rank, "tensors")
        got = np_of(g)
        assert got.tobytes() == g_ref.tobytes(), rank
        assert float(ss.item()) == ss_ref
        neg += int((got.view(np.uint32) == 0x80000000).sum())
        pad = got[max(0, lay.total - ob):]
        assert (pad.view(np.uint32) == 0).all(), "padding is +0"
    assert neg > 100


def _plant_nonfinite(host, dtype, seed, where):
    """Overwrites a few elements of a few ranks with +inf, -inf, NaN (several payloads); returns
    the set of touched element indices.  `where`: candidate indices."""
    rng = np.random.default_rng(seed)
    inf, ninf, nans = {wl.BF16: (0x7F80, 0xFF80, (0x7FC0, 0xFFC1, 0x7F81, 0x7FFF)),
                       wl.F16: (0x7C00, 0xFC00, (0x7E00, 0xFE01, 0x7C01, 0x7FFF)),
                       wl.F32: (0x7F800000, 0xFF800000, (0x7FC00000, 0xFFC00001, 0x7F800001, 0x7FFFFFFF))}[dtype]
    touched = set()
    picks = rng.choice(where, 60, replace=False)
    for k, e in enumerate(picks):
        e = int(e)
        raw = [h.view(np.uint16 if dtype != wl.F32 else np.uint32) for h in host]
        kind = k % 6
        q = int(rng.integers(0, len(host)))
        q2 = (q + 1 + int(rng.integers(0, len(host) - 1))) % len(host)
        if kind == 0:
            raw[q][e] = inf
        elif kind == 1:
            raw[q][e] = ninf
        elif kind == 2:                       # +inf and -inf meet: NaN
            raw[q][e] = inf
            raw[q2][e] = ninf
        elif kind == 3:                       # two +inf: stays +inf
            raw[q][e] = inf
            raw[q2][e] = inf
        else:
            raw[q][e] = nans[(k // 6) % 4]
            if kind == 5:
                raw[q2][e] = nans[(k // 6 + 1) % 4]
        touched.add(e)
    return np.array(sorted(touched))


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32, wl.F16])
def test_nonfinite_contributions_without_skip(paro, dtype):
    """Infinities and NaNs among the contributions, skip_nonfinite off, no clipping: the path is
    element-wise, so every other element is untouched and must match as always; at the planted
    elements the reduced gradient is the oracle's up to the payload of a NaN (which operand's
    payload an add of two NaNs keeps, and the sign of inf - inf, are the adder's choice), and p, m, v
    and the packed value are non-finite exactly where the oracle's are."""
    P, G, strategy = 8, 4, "IIG"
    sizes = [P * 2048 * 5 + 24]
    lay = orc.layout(P, G, sizes)
    n = P * lay.L
    dev0, host = flat_inputs(P, n, seed=61, dtype=dtype)
    host = [h.copy() for h in host]
    touched = _plant_nonfinite(host, dtype, 62, np.arange(lay.total))
    dev = [_to_dev(h, dtype) for h in host]
    state = [np_of(t) for t in wl.master_state(n, 63)]
    hp = hp_dict(P, max_norm=0.0)
    for sched in (orc.RING, orc.HORING):
        pl = paro.paro_plan(P, G, strategy, sizes, sched=sched, grad_dtype=[dtype])
        hit = 0
        for rank in range(P):
            ob, ol = orc.state_range(lay, rank, strategy[2])
            g = torch.empty(ol, dtype=torch.float32, device=DEV)
            ss = torch.zeros(1, dtype=torch.float64, device=DEV)
            ptrs = [t[ob:ob + ol].data_ptr() for t in dev]
            paro.paro_reduce_shard(pl, rank, ptrs, paro.PARO_CHUNK, g.data_ptr(), ss.data_ptr(), stream())
            with np.errstate(invalid="ignore", over="ignore"):
                g_ref, ss_ref = orc.reduce_shard(lay, strategy, sched, rank, [h[ob:ob + ol] for h in host], "chunk")
            got = np_of(g)
            nan_ref = np.isnan(g_ref)
            assert (np.isnan(got) == nan_ref).all(), "NaN in other places than the oracle's"
            assert got[~nan_ref].tobytes() == g_ref[~nan_ref].tobytes()          # infinities included, bit for bit
            mine = touched[(touched >= ob) & (touched < ob + ol)] - ob
            assert not np.isfinite(g_ref[mine]).any()
            hit += int((~np.isfinite(got)).sum())
            if mine.size:
                assert not np.isfinite(float(ss.item())) and not np.isfinite(ss_ref)
            # the update, one sweep, no skip
            old = [a[ob:ob + ol].copy() for a in state]
            with np.errstate(invalid="ignore", over="ignore"):
                ref = oracle_update(lay, strategy, rank, g_ref, *old, total_sumsq=0.0, hp=hp, step=1)
                lit = oracle_update(lay, strategy, rank, g_ref, *old, total_sumsq=0.0, hp=hp, step=1, literal32=True)
            p, m, v = (torch.from_numpy(a.copy()).to(DEV) for a in old)
            dst_len, slot_off, slot_len = orc.pack_slot(lay, rank, strategy)
            dst = torch.zeros(dst_len, dtype=torch.bfloat16, device=DEV)
            paro.paro_step_fused(pl, rank, ptrs, paro.PARO_CHUNK, hp_struct(paro, hp, 1), 0, 0, p.data_ptr(), m.data_ptr(),
                                 v.data_ptr(), dst.data_ptr(), stream())
            gpu = dict(p=np_of(p), m=np_of(m), v=np_of(v), q=np_of(dst)[slot_off:slot_off + slot_len])
            fin = np.isfinite(g_ref)
            for k in ("p", "m", "v"):
                assert (np.isnan(gpu[k]) == np.isnan(lit[k])).all(), k
                both = ~np.isnan(lit[k])
                assert gpu[k][both].tobytes() == lit[k][both].tobytes(), k     # +-inf moments bit for bit
            assert not np.isfinite(gpu["p"][~fin]).any(), "a non-finite gradient must make its parameter non-finite"
            qn = (gpu["q"] & 0x7FFF) > 0x7F80
            assert (qn == np.isnan(lit["p"])).all() and (gpu["q"][~qn] == lit["q"][~qn]).all()
            g_hat = float(np.float32(hp["grad_scale"])) * g_ref[fin].astype(np.float64)
            compare_step({k: a[fin] for k, a in gpu.items()}, {k: a[fin] for k, a in ref.items() if k != "coef"},
                         p_old=old[0][fin], m_old=old[1][fin], g_hat=g_hat, what=f"finite elements, rank {rank}",
                         literal={k: a[fin] for k, a in lit.items() if k != "coef"})
        assert hit >= 55


def test_plan_alignment_64_through_the_device_calls(paro):
    """align_elems = 64 changes the chunk length, hence every range, slot and fold: chunk and
    tensor layout, every rank, against the oracle laid out with the same alignment."""
    P, G = 4, 2
    sizes = [5000, 0, 17, 4096 + 3, 1, 2048 * 2]
    no_decay = [0, 1, 1, 0, 1, 0]
    lay8, lay = orc.layout(P, G, sizes), orc.layout(P, G, sizes, align=64)
    assert lay.L % 64 == 0 and lay.L != lay8.L
    n = P * lay.L
    dev, host = flat_inputs(P, n, seed=71)
    for t, h in zip(dev, host):
        t[lay.total:] = 0
        h[lay.total:] = 0
    state = [np_of(t) for t in wl.master_state(n, 72)]
    for a in state:
        a[lay.total:] = 0
    sets = wl.tensor_contribs(P, sizes, None, 73, 1, device=DEV, align_elems=1)
    tables = [PtrTable(s.tensors) for s in sets]
    host_t = [[np_of(t) for t in s.tensors] for s in sets]
    for strategy in ("IIG", "NIG", "III"):
        sched = orc.default_sched(P, G)
        pl = paro.paro_plan(P, G, strategy, sizes, align_elems=64)
        assert paro.paro_shard_len(pl) == lay.L and paro.paro_padded_total(pl) == n
        plm = paro.paro_plan(P, G, strategy, sizes, align_elems=64, no_decay=no_decay)
        for rank in range(P):
            assert paro.paro_range(pl, rank, "O") == orc.state_range(lay, rank, strategy[2])
            assert paro.paro_pack_slot(pl, rank) == orc.pack_slot(lay, rank, strategy)
            for max_norm in (0.0, 0.004):
                hp = hp_dict(P, max_norm=max_norm)
                run_rank(paro, pl, lay, strategy, sched, rank, dev, host, state, hp, 2)
                _tensor_rank(paro, plm, lay, strategy, sched, rank, tables, host_t, state, hp, 2, no_decay=no_decay,
                             what=f"align64 clip{max_norm}")


@pytest.mark.parametrize("strategy,ranks", [("III", (0, 3)), ("NNN", (2,)), ("NNI", (1,))])
def test_update_range_of_several_chunks_at_size(paro, strategy, ranks):
    """Optimizer state sharded inside the group only (2 chunks per rank) or not at all (4 chunks):
    one launch per chunk, each in its own fold order, at L = 2^22 (16 384 blocks per chunk, a
    two-level sum of the partial sums) - chunk layout through every entry point, then tensor layout
    with a decay mask (one masked launch per chunk, each with its per-tile table) on a list whose
    tensors straddle the chunk edges."""
    P, G = 4, 2
    L = 1 << 22
    sizes = [3 * (1 << 21) + 5, (1 << 22) - 5 - 768, 768, 1 << 22, (1 << 21) - 8]
    assert sum(sizes) == P * L - 8
    no_decay = [0, 0, 1, 1, 0]
    lay = orc.layout(P, G, sizes)
    assert lay.L == L
    n = P * L
    sched = orc.default_sched(P, G)
    dev, host = flat_inputs(P, n, seed=81)
    for t, h in zip(dev, host):
        t[lay.total:] = 0
        h[lay.total:] = 0
    state = [np_of(t) for t in wl.master_state(n, 82)]
    for a in state:
        a[lay.total:] = 0
    pl = paro.paro_plan(P, G, strategy, sizes)
    for rank in ranks:
        ob, ol = orc.state_range(lay, rank, strategy[2])
        assert ol >= 2 * L
        run_rank(paro, pl, lay, strategy, sched, rank, dev, host, state, hp_dict(P, max_norm=0.5), 1)
        run_rank(paro, pl, lay, strategy, sched, rank, dev, host, state, hp_dict(P, max_norm=0.0), 2,
                 check_unfused=False)
    sets = wl.tensor_contribs(P, sizes, None, 83, 1, device=DEV)
    tables = [PtrTable(s.tensors) for s in sets]
    host_t = [[np_of(t) for t in s.tensors] for s in sets]
    plm = paro.paro_plan(P, G, strategy, sizes, no_decay=no_decay)
    for rank in ranks[:1]:
        for max_norm in (0.5, 0.0):
            _tensor_rank(paro, plm, lay, strategy, sched, rank, tables, host_t, state, hp_dict(P, max_norm=max_norm), 1,
                         no_decay=no_decay, what=f"multi-chunk clip{max_norm}")


@pytest.mark.parametrize("mode", ["per-block table", "search", "two blocks per wave"])
def test_blocks_holding_hundreds_of_tensors(paro, mode, monkeypatch):
    """Runs of one- to three-element tensors: blocks of 256 elements that hold up to 256 tensors.  A block
    finds its elements' tensors with one table entry per lane (64 segment starts) and falls back to a
    per-lane search through the table when more than 64 tensors start inside it - both happen here, next
    to ordinary blocks, with mixed dtypes and a decay mask, in the tensor layout and (for the mask) the
    chunk layout."""
    if mode == "search":
        monkeypatch.setenv("PARO_TILE_TABLE_MAX_TILES", "0")
    if mode == "two blocks per wave":
        monkeypatch.setenv("PARO_PAIR_MIN_BLOCKS", "0")
    rng = np.random.default_rng(77)
    sizes = ([1] * 300 + [5000] + [int(x) for x in rng.integers(1, 4, 400)] + [700, 0, 0, 3] + [2] * 90 + [4096]
             + [int(x) for x in rng.integers(1, 9, 200)] + [1] * 70 + [9])
    dtypes = [int(x) for x in rng.integers(0, 3, len(sizes))]
    no_decay = [int(x) for x in rng.integers(0, 2, len(sizes))]
    P, G = 4, 2
    lay = orc.layout(P, G, sizes)
    starts = np.cumsum([0] + sizes[:-1])[np.array(sizes) > 0]
    per_block = np.bincount(starts // 256)
    assert per_block.max() > 200 and (per_block > 64).sum() >= 2 and ((per_block > 1) & (per_block <= 64)).sum() >= 2
    n = P * lay.L
    state = [np_of(t) for t in wl.master_state(n, 78)]
    for a in state:
        a[lay.total:] = 0
    sets = wl.tensor_contribs(P, sizes, dtypes, 79, 1, device=DEV, align_elems=1)
    tables = [PtrTable(s.tensors) for s in sets]
    host_t = [[np_of(t) for t in s.tensors] for s in sets]
    dev, host = flat_inputs(P, n, seed=80)
    for t, h in zip(dev, host):
        t[lay.total:] = 0
        h[lay.total:] = 0
    for strategy in ("IIG", "III"):
        sched = orc.default_sched(P, G)
        plm = paro.paro_plan(P, G, strategy, sizes, grad_dtype=dtypes, no_decay=no_decay)
        plc = paro.paro_plan(P, G, strategy, sizes, no_decay=no_decay)          # chunk layout: one dtype
        for rank in range(P):
            for max_norm in (0.01, 0.0):
                hp = dict(hp_dict(P, max_norm=max_norm), weight_decay=0.1)
                _tensor_rank(paro, plm, lay, strategy, sched, rank, tables, host_t, state, hp, 3, no_decay=no_decay,
                             what=f"tiny tensors, {mode}, clip {max_norm}")
            # chunk layout with the mask: sweep 2 / the single sweep look the tensors up for the decay flag only
            ob, ol = orc.state_range(lay, rank, strategy[2])
            g_ref, _ = orc.reduce_shard(lay, strategy, sched, rank, [h[ob:ob + ol] for h in host], "chunk")
            hp = dict(hp_dict(P, max_norm=0.01), weight_decay=0.1)
            total = orc.range_sumsq(lay, strategy, rank, g_ref)
            old = [a[ob:ob + ol].copy() for a in state]
            ref = oracle_update(lay, strategy, rank, g_ref, *old, total_sumsq=total, hp=hp, step=3, no_decay=no_decay)
            lit = oracle_update(lay, strategy, rank, g_ref, *old, total_sumsq=total, hp=hp, step=3, no_decay=no_decay,
                                literal32=True)
            p, m, v = (torch.from_numpy(a.copy()).to(DEV) for a in old)
            dst_len, slot_off, slot_len = orc.pack_slot(lay, rank, strategy)
            dst = torch.zeros(dst_len, dtype=torch.bfloat16, device=DEV)
            gs = torch.empty(ol, dtype=torch.float32, device=DEV)
            ss = torch.zeros(1, dtype=torch.float64, device=DEV)
            paro.paro_step_fused(plc, rank, [t[ob:ob + ol].data_ptr() for t in dev], paro.PARO_CHUNK, hp_struct(paro, hp, 3),
                                 gs.data_ptr(), ss.data_ptr(), p.data_ptr(), m.data_ptr(), v.data_ptr(), dst.data_ptr(), stream())
            got = dict(p=np_of(p), m=np_of(m), v=np_of(v), q=np_of(dst)[slot_off:slot_off + slot_len])
            g_hat = float(np.float32(hp["grad_scale"])) * ref["coef"] * g_ref.astype(np.float64)
            compare_step(got, ref, p_old=old[0], m_old=old[1], g_hat=g_hat, what=f"tiny tensors, chunk + mask, rank {rank}",
                         literal=lit)
