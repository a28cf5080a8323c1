"""GPU parity, small cases (the oracle finishes in well under a second each):
the tiny configuration over every strategy and schedule, integer gradients,
fp32 contributions, edge cases of the layout, special values in the pack."""
import numpy as np
import pytest
import torch

import oracle as orc
import workloads as wl
from harness import (DEV, PtrTable, compare_step, flat_inputs, hp_dict, hp_struct, l2_terms, np_of, oracle_update, run_rank,
                     stream)
from parity import ulp_distance_f32

pytestmark = pytest.mark.gpu

SCHEDS = [orc.RING, orc.HRING, orc.HORING]


def test_tiny_every_strategy_and_schedule(paro):
    """P=4, G=2, one tensor of 2^20, bf16 N(0,1e-3) gradients, N(0,0.02) parameters,
    one step without clipping - for all 14 strategies x 3 schedules x 4 ranks."""
    cfg = wl.config("tiny")
    P, G = cfg.P, cfg.G
    lay = orc.layout(P, G, cfg.sizes)
    n = P * lay.L
    dev, host = flat_inputs(P, n, seed=0)
    state = [np_of(t) for t in wl.master_state(n, 0)]
    hp = hp_dict(P)
    report = []
    union = {}
    for strategy in orc.all_legal_strategies():
        for sched in SCHEDS:
            pl = paro.paro_plan(P, G, strategy, cfg.sizes, sched=sched)
            for rank in range(P):
                fused, _ = run_rank(paro, pl, lay, strategy, sched, rank, dev, host, state, hp, 1, report,
                                     check_unfused=(sched == orc.HORING))
                ob, ol = orc.state_range(lay, rank, strategy[2])
                key = (sched,)
                flat = union.setdefault(key, {})
                # whatever the strategy, an element's result is the same bits (replicas agree,
                # shards tile the model)
                for name in ("p", "m", "v", "q"):
                    buf = flat.setdefault(name, {})
                    for c in range(ob // lay.L, (ob + ol) // lay.L):
                        piece = fused[name][c * lay.L - ob:(c + 1) * lay.L - ob].tobytes()
                        assert buf.setdefault(c, piece) == piece, (strategy, sched, rank, name, c)
    worst_p = max(r[1] for r in report)
    worst_v = max(r[2] for r in report)
    print(f"\n[tiny] max ulp distance to the fp64 reference: p {worst_p}, v {worst_v} over {len(report)} rank-cases")
    for key, flat in union.items():
        assert sorted(flat["p"]) == list(range(P))


def test_fp32_literal_evaluation_distance(paro):
    """How far the kernel is from the oracle's all-fp32 evaluation (same operation
    order): reported, and bounded by a few ulp."""
    P, G = 4, 2
    lay = orc.layout(P, G, [1 << 18])
    n = P * lay.L
    dev, host = flat_inputs(P, n, seed=3)
    state = [np_of(t) for t in wl.master_state(n, 3)]
    state[1] = np_of(wl.draw(n, 91, scale=1e-4, dtype=wl.F32))
    state[2] = np.abs(np_of(wl.draw(n, 92, scale=1e-7, dtype=wl.F32)))
    pl = paro.paro_plan(P, G, "GGG", [1 << 18])
    for max_norm, adamw, step in ((0.0, True, 1), (0.05, True, 4), (0.05, False, 9)):
        hp = hp_dict(P, max_norm=max_norm, adamw=adamw)
        rank = 2
        fused, ref = run_rank(paro, pl, lay, "GGG", orc.HORING, rank, dev, host, state, hp, step)
        ob, ol = orc.state_range(lay, rank, "G")
        g_ref, ss_ref = orc.reduce_shard(lay, "GGG", orc.HORING, rank, [h[ob:ob + ol] for h in host], "chunk")
        lit = oracle_update(lay, "GGG", rank, g_ref, *(a[ob:ob + ol] for a in state), total_sumsq=ss_ref, hp=hp,
                            step=step, literal32=True)
        d = {k: ulp_distance_f32(fused[k], lit[k]) for k in ("p", "m", "v")}
        print(f"\n[literal32] max_norm={max_norm} adamw={adamw} step={step}: ulp distance {d}, coef {ref['coef']:.6f}")
        if max_norm > 0:
            assert ref["coef"] < 1.0
        assert max(d.values()) <= 2
        assert (fused["q"] == lit["q"]).mean() > 0.999


def test_integer_gradients_reduce_exactly(paro):
    P, G = 8, 4
    lay = orc.layout(P, G, [P * 5000 + 13])
    n = P * lay.L
    for dtype in (wl.BF16, wl.F32):
        dev, host = flat_inputs(P, n, seed=11, dtype=dtype, integer=True)
        as_f32 = [orc.bf16_bits_to_f32(h) if h.dtype == np.uint16 else h for h in host]
        exact = np.sum([a.astype(np.int64) for a in as_f32], axis=0)
        for sched in SCHEDS:
            pl = paro.paro_plan(P, G, "IIG", [P * 5000 + 13], sched=sched,
                                grad_dtype=[dtype])
            for rank in (0, 5):
                ob, ol = orc.state_range(lay, rank, "G")
                g = torch.empty(ol, dtype=torch.float32, device=DEV)
                ss = torch.zeros(1, dtype=torch.float64, device=DEV)
                paro.paro_reduce_shard(pl, rank, [t[ob:ob + ol].data_ptr() for t in dev], paro.PARO_CHUNK,
                                       g.data_ptr(), ss.data_ptr(), stream())
                got = np_of(g)
                assert (got.astype(np.int64) == exact[ob:ob + ol]).all() and (got == np.round(got)).all()
                assert float(ss.item()) == float(np.sum(exact[ob:ob + ol] ** 2))


def test_fp32_contributions_chunk_layout(paro):
    P, G = 6, 3
    sizes = [70001]
    lay = orc.layout(P, G, sizes)
    n = P * lay.L
    dev, host = flat_inputs(P, n, seed=21, dtype=wl.F32)
    state = [np_of(t) for t in wl.master_state(n, 21)]
    for strategy, sched in (("IIG", orc.HORING), ("NNI", orc.HRING), ("GGG", orc.RING)):
        pl = paro.paro_plan(P, G, strategy, sizes, sched=sched, grad_dtype=[wl.F32])
        for rank in range(P):
            run_rank(paro, pl, lay, strategy, sched, rank, dev, host, state, hp_dict(P, max_norm=0.01), 3)


@pytest.mark.parametrize("P,G,total", [(1, 1, 1), (1, 1, 4099), (4, 2, 1), (4, 4, 3), (8, 2, 8 * 8 * 300 - 1),
                                        (64, 8, 64 * 2048 + 8), (256, 16, 256 * 24), (2, 2, 2 * 256),
                                        (2, 1, 2 * 264 - 5)])
def test_layout_edge_cases(paro, P, G, total):
    """One element (a shard that is almost all padding), P = 1, a ragged last tile,
    a shard of exactly one tile plus 8, the largest supported P, a shard of exactly one
    block of 256 elements, one block plus 8 with a ragged end."""
    lay = orc.layout(P, G, [total])
    n = P * lay.L
    dev, host = flat_inputs(P, n, seed=31)
    for t, h in zip(dev, host):                 # padding carries zero gradient
        t[total:] = 0
        h[total:] = 0
    state = [np_of(t) for t in wl.master_state(n, 31)]
    for a in state:
        a[total:] = 0
    sched = orc.default_sched(P, G)
    pl = paro.paro_plan(P, G, "GGG", [total])
    ranks = sorted({0, P - 1, P // 2})
    for rank in ranks:
        fused, ref = run_rank(paro, pl, lay, "GGG", sched, rank, dev, host, state, hp_dict(P, max_norm=1e-4), 2)
        ob, ol = orc.state_range(lay, rank, "G")
        pad = slice(max(0, total - ob), ol)
        for k in ("p", "m", "v", "q"):
            assert not fused[k][pad].any(), "padding must stay zero"


def test_pack_special_values(paro):
    """NaN, infinities, ties, denormals, the largest finite value: bit-exact."""
    bits = np.array([0x3F808000, 0x3F818000, 0x3F808001, 0x3F807FFF, 0x7F7FFFFF, 0xFF7FFFFF, 0x7F800000, 0xFF800000,
                     0x7FC00000, 0xFFC00001, 0x7F800001, 0xFF80FFFF, 0x80000000, 0x00000000, 0x00008000, 0x00018000,
                     0x00000001, 0x807FFFFF], np.uint32)
    rng = np.random.default_rng(5)
    allbits = np.concatenate([bits, rng.integers(0, 1 << 32, 1 << 16, dtype=np.uint64).astype(np.uint32),
                              (np.arange(1 << 16, dtype=np.uint32) << 16) | 0x8000])
    n = (allbits.size + 7) // 8 * 8
    x = np.zeros(n, np.uint32)
    x[:allbits.size] = allbits
    pl = paro.paro_plan(1, 1, "GGG", [n])
    p = torch.from_numpy(x.view(np.float32).copy()).to(DEV)
    dst = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    paro.paro_pack_params(pl, 0, p.data_ptr(), dst.data_ptr(), stream())
    assert np_of(dst).tobytes() == orc.bf16_rne(x.view(np.float32)).tobytes()


@pytest.mark.parametrize("fmt", [wl.BF16, wl.F16])
def test_pack_every_fp32_bit_pattern(paro, fmt):
    """All 2^32 fp32 bit patterns through the pack, in blocks of 2^27: bit-exact
    against the oracle's rounding.  For fp16 the payload of a NaN is not part of the
    contract: a NaN must come out as a NaN of the same sign."""
    n = 1 << 27
    pl = paro.paro_plan(1, 1, "GGG", [n], pack_dtype=fmt)
    low = torch.arange(n, dtype=torch.int32, device=DEV)
    low_h = np.arange(n, dtype=np.uint32)
    dst = torch.zeros(n, dtype=torch.int16, device=DEV)
    for b in range(32):
        hi = b << 27
        bits = low | (hi - (1 << 32) if hi >= (1 << 31) else hi)
        p = bits.view(torch.float32)
        paro.paro_pack_params(pl, 0, p.data_ptr(), dst.data_ptr(), stream())
        got = dst.cpu().numpy().view(np.uint16)
        x = (low_h | np.uint32(hi)).view(np.float32)
        if fmt == wl.BF16:
            assert got.tobytes() == orc.bf16_rne(x).tobytes(), f"bf16 pack differs in block {b}"
        else:
            ref = orc.f16_rne(x)
            nan = np.isnan(x)
            assert (got[~nan] == ref[~nan]).all(), f"fp16 pack differs in block {b}"
            g_nan = got[nan]
            assert ((g_nan & 0x7FFF) > 0x7C00).all() and ((g_nan >> 15) == (ref[nan] >> 15)).all()


def test_runs_are_bit_identical(paro):
    P, G = 16, 8
    sizes = [16 * 3 * 2048 * 11]
    lay = orc.layout(P, G, sizes)
    dev, _ = flat_inputs(P, lay.L, seed=41)
    pl = paro.paro_plan(P, G, "IIG", sizes)
    outs = []
    for _ in range(3):
        g = torch.empty(lay.L, dtype=torch.float32, device=DEV)
        ss = torch.zeros(1, dtype=torch.float64, device=DEV)
        paro.paro_reduce_shard(pl, 3, [t.data_ptr() for t in dev], paro.PARO_CHUNK, g.data_ptr(), ss.data_ptr(),
                               stream())
        outs.append((np_of(g).tobytes(), float(ss.item())))
    assert outs[0] == outs[1] == outs[2]


@pytest.mark.parametrize("table", ["per-tile table", "search", "two blocks per wave"])
def test_tensor_layout_small_ragged(paro, table, monkeypatch):
    """Tensor layout on a small ragged list: empty and one-element tensors, mixed
    dtypes, unaligned tensor bases, a weight-decay mask, every rank, 2 steps - with
    the plan's per-tile table, without it (every block searches the offset table), and with
    sweep 1's shape for large launches of few ranks forced on (a wave takes two blocks)."""
    if table == "search":
        monkeypatch.setenv("PARO_TILE_TABLE_MAX_TILES", "0")
    if table == "two blocks per wave":
        monkeypatch.setenv("PARO_PAIR_MIN_BLOCKS", "0")
    rng = np.random.default_rng(8)
    sizes = [int(s) for s in rng.integers(0, 9, 40)] + [5000, 1, 0, 7, 20000, 3, 2049, 2047, 1, 1, 9000]
    dtypes = [int(x) for x in rng.integers(0, 2, len(sizes))]
    no_decay = [int(x) for x in rng.integers(0, 2, len(sizes))]
    for (P, G, strategy, align) in ((4, 2, "IIG", 1), (4, 2, "NIG", 128), (2, 2, "III", 1), (4, 1, "NNN", 8)):
        lay = orc.layout(P, G, sizes)
        sched = orc.default_sched(P, G)
        pl = paro.paro_plan(P, G, strategy, sizes, grad_dtype=dtypes, no_decay=no_decay)
        n = P * lay.L
        state = [np_of(t) for t in wl.master_state(n, 51)]
        for a in state:
            a[lay.total:] = 0
        for max_norm in (0.0, 0.002):
            hp = hp_dict(P, max_norm=max_norm)
            # every rank keeps its own copy of its range on both sides (replicas of a range clip with
            # their own rank's norm here, so they may drift apart - as they would on the GPU side)
            ora_state = [[a[slice(*_rng(lay, r, strategy))].copy() for a in state] for r in range(P)]
            lit_state = [[a.copy() for a in st] for st in ora_state]
            hist = [dict() for _ in range(P)]
            gpu_state = [[torch.from_numpy(a.copy()).to(DEV) for a in ora_state[r]] for r in range(P)]
            for step in (1, 2):
                sets = wl.tensor_contribs(P, sizes, dtypes, 60, step, device=DEV, align_elems=align)
                tables = [PtrTable(s.tensors) for s in sets]
                host = [[np_of(t) for t in s.tensors] for s in sets]
                for rank in range(P):
                    ob, ol = orc.state_range(lay, rank, strategy[2])
                    g_ref, _own = orc.reduce_shard(lay, strategy, sched, rank, host, "tensors")
                    ss_ref = orc.range_sumsq(lay, strategy, rank, g_ref)      # the fused step's norm
                    old = ora_state[rank]
                    ref = oracle_update(lay, strategy, rank, g_ref, *old, total_sumsq=ss_ref, hp=hp, step=step,
                                        no_decay=no_decay)
                    lit = oracle_update(lay, strategy, rank, g_ref, *lit_state[rank], total_sumsq=ss_ref, hp=hp,
                                        step=step, no_decay=no_decay, literal32=True)
                    p, m, v = gpu_state[rank]
                    dst_len, slot_off, slot_len = orc.pack_slot(lay, rank, strategy)
                    dst = torch.zeros(dst_len, dtype=torch.bfloat16, device=DEV)
                    gs = torch.empty(ol, dtype=torch.float32, device=DEV)
                    ss = torch.zeros(1, dtype=torch.float64, device=DEV)
                    paro.paro_step_fused(pl, rank, [t.ptr() for t in tables], paro.PARO_TENSORS,
                                         hp_struct(paro, hp, step), gs.data_ptr(), ss.data_ptr(), p.data_ptr(),
                                         m.data_ptr(), v.data_ptr(), dst.data_ptr(), stream())
                    what = f"{strategy} align{align} clip{max_norm} step{step} rank{rank}"
                    if max_norm > 0:
                        assert np_of(gs).tobytes() == g_ref.tobytes(), what
                        assert abs(float(ss.item()) - ss_ref) <= 1e-12 * ss_ref
                        assert ref["coef"] < 1.0
                    g_hat = float(np.float32(hp["grad_scale"])) * ref["coef"] * g_ref.astype(np.float64)
                    got = dict(p=np_of(p), m=np_of(m), v=np_of(v), q=np_of(dst)[slot_off:slot_off + slot_len])
                    compare_step(got, ref, p_old=old[0], m_old=old[1], g_hat=g_hat, what=what, hist=hist[rank],
                                 literal=lit)
                    ora_state[rank] = [ref["p"], ref["m"], ref["v"]]
                    lit_state[rank] = [lit["p"], lit["m"], lit["v"]]


@pytest.mark.parametrize("P,G,strategy", [(256, 16, "IGG"), (64, 8, "NIG"), (12, 3, "IIG")])
def test_tensor_layout_many_ranks(paro, P, G, strategy, monkeypatch):
    """Tensor layout at large P (the pointer staging covers up to 256 sources), shards of a
    few tiles that hold both whole-tensor tiles and tiles with boundaries; sampled ranks.
    P = 12 runs without the per-tile table."""
    if P == 12:
        monkeypatch.setenv("PARO_TILE_TABLE_MAX_TILES", "0")
    rng = np.random.default_rng(P)
    sizes = [int(s) for s in rng.integers(1, 30, 25)] + [40000, 3, 8192, 2048 * 9, 77, 1_500_000, 123456, 5]
    dtypes = [int(x) for x in rng.choice([wl.BF16, wl.F32, wl.F16], len(sizes))]
    lay = orc.layout(P, G, sizes)
    sched = orc.default_sched(P, G)
    pl = paro.paro_plan(P, G, strategy, sizes, grad_dtype=dtypes)
    sets = wl.tensor_contribs(P, sizes, dtypes, 70, 1, device=DEV)
    tables = [PtrTable(s.tensors) for s in sets]
    host = [[np_of(t) for t in s.tensors] for s in sets]
    n = P * lay.L
    state = [np_of(t) for t in wl.master_state(n, 71)]
    for a in state:
        a[lay.total:] = 0
    hp = hp_dict(P, max_norm=0.001)
    for rank in sorted({0, 1, G, P // 2 + 1, P - 1}):
        ob, ol = orc.state_range(lay, rank, strategy[2])
        g_ref, ss_ref = orc.reduce_shard(lay, strategy, sched, rank, host, "tensors")
        old = [a[ob:ob + ol].copy() for a in state]
        ref = oracle_update(lay, strategy, rank, g_ref, *old, total_sumsq=ss_ref, hp=hp, step=1)
        lit = oracle_update(lay, strategy, rank, g_ref, *old, total_sumsq=ss_ref, hp=hp, step=1, literal32=True)
        p, m, v = (torch.from_numpy(a.copy()).to(DEV) for a in old)
        dst_len, slot_off, slot_len = orc.pack_slot(lay, rank, strategy)
        dst = torch.zeros(dst_len, dtype=torch.bfloat16, device=DEV)
        gs = torch.empty(ol, dtype=torch.float32, device=DEV)
        ss = torch.zeros(1, dtype=torch.float64, device=DEV)
        paro.paro_step_fused(pl, rank, [t.ptr() for t in tables], paro.PARO_TENSORS, hp_struct(paro, hp, 1),
                             gs.data_ptr(), ss.data_ptr(), p.data_ptr(), m.data_ptr(), v.data_ptr(), dst.data_ptr(),
                             stream())
        what = f"P{P} {strategy} rank{rank}"
        assert np_of(gs).tobytes() == g_ref.tobytes(), what
        assert abs(float(ss.item()) - ss_ref) <= 1e-12 * ss_ref and ref["coef"] < 1.0
        g_hat = float(np.float32(hp["grad_scale"])) * ref["coef"] * g_ref.astype(np.float64)
        got = dict(p=np_of(p), m=np_of(m), v=np_of(v), q=np_of(dst)[slot_off:slot_off + slot_len])
        compare_step(got, ref, p_old=old[0], m_old=old[1], g_hat=g_hat, what=what, literal=lit)


def test_chunk_layout_with_decay_mask(paro):
    """Chunk-layout contributions with a per-tensor weight-decay mask (the tensors only matter
    for the mask): clipped two-sweep step and unclipped single sweep, L2 and decoupled decay."""
    P, G, strategy = 4, 2, "IIG"
    sizes = [3000, 17, 2048, 1, 4096 + 5, 700, 9000]
    no_decay = [0, 1, 0, 1, 1, 0, 1]
    lay = orc.layout(P, G, sizes)
    sched = orc.default_sched(P, G)
    n = P * lay.L
    dev, host = flat_inputs(P, n, seed=81)
    for t, h in zip(dev, host):
        t[lay.total:] = 0
        h[lay.total:] = 0
    state = [np_of(t) for t in wl.master_state(n, 82)]
    for a in state:
        a[lay.total:] = 0
    pl = paro.paro_plan(P, G, strategy, sizes, no_decay=no_decay)
    for adamw in (True, False):
        for max_norm in (0.0, 0.003):
            hp = dict(hp_dict(P, max_norm=max_norm), adamw=adamw, weight_decay=0.1)
            for rank in range(P):
                ob, ol = orc.state_range(lay, rank, strategy[2])
                contrib = [t[ob:ob + ol] for t in dev]
                g_ref, ss_ref = orc.reduce_shard(lay, strategy, sched, rank, [h[ob:ob + ol] for h in host], "chunk")
                old = [a[ob:ob + ol].copy() for a in state]
                ref = oracle_update(lay, strategy, rank, g_ref, *old, total_sumsq=ss_ref, hp=hp, step=2,
                                    no_decay=no_decay)
                lit = oracle_update(lay, strategy, rank, g_ref, *old, total_sumsq=ss_ref, hp=hp, step=2,
                                    no_decay=no_decay, literal32=True)
                p, m, v = (torch.from_numpy(a.copy()).to(DEV) for a in old)
                dst_len, slot_off, slot_len = orc.pack_slot(lay, rank, strategy)
                dst = torch.zeros(dst_len, dtype=torch.bfloat16, device=DEV)
                gs = torch.empty(ol, dtype=torch.float32, device=DEV)
                ss = torch.zeros(1, dtype=torch.float64, device=DEV)
                paro.paro_step_fused(pl, rank, [c.data_ptr() for c in contrib], paro.PARO_CHUNK,
                                     hp_struct(paro, hp, 2), gs.data_ptr(), ss.data_ptr(), p.data_ptr(), m.data_ptr(),
                                     v.data_ptr(), dst.data_ptr(), stream())
                g_hat = float(np.float32(hp["grad_scale"])) * ref["coef"] * g_ref.astype(np.float64)
                g_terms = None
                if not adamw:                   # L2: wd * p joins the gradient where the tensor decays
                    decays = np.ones(ol, bool)
                    for (t, _toff, soff, ln) in orc.segments(lay, ob, ol):
                        decays[soff:soff + ln] = not no_decay[t]
                    wd_p = np.where(decays, float(np.float32(hp["weight_decay"])) * old[0].astype(np.float64), 0.0)
                    g_terms = np.abs(g_hat) + np.abs(wd_p)
                    g_hat = g_hat + wd_p
                got = dict(p=np_of(p), m=np_of(m), v=np_of(v), q=np_of(dst)[slot_off:slot_off + slot_len])
                compare_step(got, ref, p_old=old[0], m_old=old[1], g_hat=g_hat, g_terms=g_terms, v_old=old[2],
                             what=f"mask adamw={adamw} clip={max_norm} rank{rank}", literal=lit,
                             l2=None if adamw else l2_terms(hp, 2))


def test_tensor_layout_ranks_with_different_alignment(paro):
    """Per-tensor gradients whose alignment differs from rank to rank: the vector-load / element-load
    choice is made source by source."""
    P, G, strategy = 4, 2, "IIG"
    sizes = [20000, 4096, 30000, 8192]
    dtypes = [wl.BF16, wl.F32, wl.F16, wl.BF16]
    lay = orc.layout(P, G, sizes)
    sched = orc.default_sched(P, G)
    pl = paro.paro_plan(P, G, strategy, sizes, grad_dtype=dtypes)
    aligned = wl.tensor_contribs(P, sizes, dtypes, 90, 1, device=DEV, align_elems=128)
    skewed = wl.tensor_contribs(P, [s + 1 for s in sizes], dtypes, 90, 1, device=DEV, align_elems=1)
    per_rank = []
    for q in range(P):
        if q % 2 == 0:
            per_rank.append(aligned[q].tensors)
        else:                                   # every tensor starts one element into its (longer) twin
            per_rank.append([t[1:] for t in skewed[q].tensors])
    tables = [PtrTable(ts) for ts in per_rank]
    host = [[np_of(t) for t in ts] for ts in per_rank]
    assert any(t.data_ptr() % 8 for t in per_rank[1]) and not any(t.data_ptr() % 16 for t in per_rank[0])
    for rank in range(P):
        ob, ol = orc.state_range(lay, rank, strategy[2])
        g_ref, ss_ref = orc.reduce_shard(lay, strategy, sched, rank, host, "tensors")
        g = torch.empty(ol, dtype=torch.float32, device=DEV)
        ss = torch.zeros(1, dtype=torch.float64, device=DEV)
        paro.paro_reduce_shard(pl, rank, [t.ptr() for t in tables], paro.PARO_TENSORS, g.data_ptr(), ss.data_ptr(),
                               stream())
        assert np_of(g).tobytes() == g_ref.tobytes(), f"rank {rank}"
        assert abs(float(ss.item()) - ss_ref) <= 1e-12 * ss_ref


def _rng(lay, rank, strategy):
    ob, ol = orc.state_range(lay, rank, strategy[2])
    return ob, ob + ol
