"""Pins for the oracle's integer side (plan, ownership, schedules): what the
paper's tables, its Fig. 4 example, Eq. 1 and plain brute force fix."""
import itertools
import os

import numpy as np
import pytest

import oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")
SHAPES = [(P, G) for P in range(1, 17) for G in range(1, P + 1) if P % G == 0]
SCHEDS = [orc.RING, orc.HRING, orc.HORING]


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


# ---- Table 1 / Principle 1 -------------------------------------------------
def test_legal_strategies_are_exactly_table1():
    table = [r[0] for r in _rows("table1_strategies.txt")]
    assert len(table) == 14
    assert orc.all_legal_strategies() == table          # same set AND the table's own order
    every = ["".join(t) for t in itertools.product("NIG", repeat=3)]
    assert sum(not orc.strategy_legal(s) for s in every) == 13   # "eliminate 13 out of 27"
    for bad in ("", "GG", "GGGG", "XGG", "ggg", "GGN", "IGN", "GGI"):
        assert not orc.strategy_legal(bad)


# ---- Table 2: memory closed forms ---------------------------------------------
@pytest.mark.parametrize("P,G", [(16, 8), (64, 8), (4, 2), (9, 3), (8, 8), (8, 1)])
def test_table2_memory(P, G):
    psi = 8 * P * 35                                    # divisible by 8P: no padding
    lay = orc.layout(P, G, [psi])
    assert lay.L * P == psi
    div = {"1": 1, "M": G, "N": P}
    K = 12
    for name, strat, dp, dg, dos in _rows("table2_memory.txt"):
        assert orc.strategy_legal(strat)
        for r in range(P):
            lens = [orc.state_range(lay, r, c)[1] for c in strat]
            assert 2 * lens[0] == 2 * psi // div[dp], name
            assert 2 * lens[1] == 2 * psi // div[dg], name
            assert K * lens[2] == K * psi // div[dos], name


# ---- ownership ----------------------------------------------------------------
@pytest.mark.parametrize("P,G", SHAPES)
def test_every_element_owned_exactly_once_and_ranges_nest(P, G):
    for total in {1, max(1, P - 1), P, P + 1, 8 * P - 1, 8 * P, 8 * P + 1, 1000}:
        lay = orc.layout(P, G, [total])
        assert lay.L % 8 == 0 and lay.L * P >= total and (lay.L - 8) * P < total
        count = np.zeros(P * lay.L, np.int32)
        for r in range(P):
            b, n = orc.state_range(lay, r, "G")
            count[b:b + n] += 1
            c = orc.chunk_of_rank(r, P, G)
            assert orc.owner_of_chunk(c, P, G) == r and b == c * lay.L
            # global range inside intra-group range inside everything
            bi, ni = orc.state_range(lay, r, "I")
            bn, nn = orc.state_range(lay, r, "N")
            assert bn <= bi <= b and b + n <= bi + ni <= bn + nn
            assert ni == lay.L * (P // G) and nn == P * lay.L
        assert (count == 1).all()
        # an intra-group sharded state: each group holds one full replica
        for j in range(P // G):
            cnt = np.zeros(P * lay.L, np.int32)
            for i in range(G):
                b, n = orc.state_range(lay, j * G + i, "I")
                cnt[b:b + n] += 1
            assert (cnt == 1).all()
    if G == P or G == 1:                                 # no grouping: ZeRO's chunk r -> rank r
        assert [orc.chunk_of_rank(r, P, G) for r in range(P)] == list(range(P))


def test_inter_group_peers_complete_the_intra_group_shard():
    # Sec. 3.2 (PaRO-IGG/IIG): the inter-group ring members (same local index)
    # together own exactly the intra-group shard of that local index.
    P, G = 16, 8
    lay = orc.layout(P, G, [8 * P * 3])
    for i in range(G):
        bi, ni = orc.state_range(lay, i, "I")
        got = sorted(orc.state_range(lay, j * G + i, "G")[0] for j in range(P // G))
        assert got == [bi + k * lay.L for k in range(P // G)]


def test_segments_brute_force():
    rng = np.random.default_rng(3)
    for _ in range(30):
        T = int(rng.integers(1, 12))
        sizes = [int(x) for x in rng.integers(0, 40, T)]
        if sum(sizes) == 0:
            sizes[0] = 5
        P, G = [(4, 2), (6, 3), (8, 8), (3, 1)][int(rng.integers(0, 4))]
        lay = orc.layout(P, G, sizes)
        flat_tensor = np.full(P * lay.L, -1)
        flat_off = np.full(P * lay.L, -1)
        for t, s in enumerate(sizes):
            flat_tensor[lay.offsets[t]:lay.offsets[t] + s] = t
            flat_off[lay.offsets[t]:lay.offsets[t] + s] = np.arange(s)
        for r in range(P):
            for letter in "NIG":
                b, n = orc.state_range(lay, r, letter)
                got_t = np.full(n, -1)
                got_o = np.full(n, -1)
                for (t, toff, soff, ln) in orc.segments(lay, b, n):
                    assert ln > 0
                    got_t[soff:soff + ln] = t
                    got_o[soff:soff + ln] = toff + np.arange(ln)
                assert (got_t == flat_tensor[b:b + n]).all() and (got_o == flat_off[b:b + n]).all()


def test_pack_slot():
    P, G = 16, 8
    g = P // G
    lay = orc.layout(P, G, [8 * P * 5])
    L = lay.L
    r = 13                                   # group j = 1, local i = 5
    assert orc.pack_slot(lay, r, "IIG") == (g * L, 1 * L, L)      # sub-slot j of the group block
    assert orc.pack_slot(lay, r, "IGG") == (g * L, 1 * L, L)
    assert orc.pack_slot(lay, r, "GGG") == (L, 0, L)
    assert orc.pack_slot(lay, r, "NIG") == (P * L, (5 * g + 1) * L, L)
    assert orc.pack_slot(lay, r, "III") == (g * L, 0, g * L)
    assert orc.pack_slot(lay, r, "NNI") == (P * L, 5 * g * L, g * L)
    assert orc.pack_slot(lay, r, "NNN") == (P * L, 0, P * L)


# ---- fold order: literal message passing vs the closed form --------------------
def _contribs(P, n, seed):
    rng = np.random.default_rng(seed)
    # wide dynamic range so that a different association order changes bits
    return [(rng.standard_normal(n) * 10.0 ** rng.integers(-3, 4, n)).astype(np.float32) for _ in range(P)]


@pytest.mark.parametrize("P,G", [(9, 3), (4, 2), (16, 8), (8, 8), (8, 1), (12, 4), (6, 2), (1, 1), (2, 1), (2, 2)])
@pytest.mark.parametrize("sched", SCHEDS)
def test_reduce_scatter_simulation_matches_fold_order(P, G, sched):
    lay = orc.layout(P, G, [P * 8 * 2 - 3])
    L = lay.L
    x = _contribs(P, P * L, seed=P * 100 + G)
    bufs = [a.copy() for a in x]
    orc.simulate(lay, sched, orc.RS, bufs)
    differs_from_naive = False
    for r in range(P):
        c = orc.chunk_of_rank(r, P, G)
        order, gl = orc.fold_order(P, G, sched, c)
        assert sorted(order) == list(range(P)) and order[-1] == r      # owner adds last
        want = orc.fold([x[q][c * L:(c + 1) * L] for q in order], gl)
        got = bufs[r][c * L:(c + 1) * L]
        assert got.tobytes() == want.tobytes()
        naive = orc.fold([x[q][c * L:(c + 1) * L] for q in range(P)], P)
        differs_from_naive |= naive.tobytes() != want.tobytes()
        # and it is the sum: fp64 reference within the fp32 chain bound
        ref = np.sum([a[c * L:(c + 1) * L].astype(np.float64) for a in x], axis=0)
        mag = np.sum([np.abs(a[c * L:(c + 1) * L]).astype(np.float64) for a in x], axis=0)
        assert (np.abs(got - ref) <= (P - 1) * 2.0 ** -24 * mag * 1.01 + 1e-300).all()
    if P >= 4:
        assert differs_from_naive        # the inputs do tell fold orders apart


def test_hring_and_horing_give_the_same_bits_but_differ_from_flat_ring():
    P, G = 12, 4
    lay = orc.layout(P, G, [P * 16])
    x = _contribs(P, P * lay.L, seed=7)
    res = {}
    for sched in SCHEDS:
        bufs = [a.copy() for a in x]
        orc.simulate(lay, sched, orc.RS, bufs)
        res[sched] = b"".join(bufs[r][orc.chunk_of_rank(r, P, G) * lay.L:][:lay.L].tobytes() for r in range(P))
    assert res[orc.HRING] == res[orc.HORING]
    assert res[orc.RING] != res[orc.HRING]


@pytest.mark.parametrize("P,G", [(9, 3), (4, 2), (16, 8), (8, 8), (8, 1), (12, 4)])
@pytest.mark.parametrize("sched", SCHEDS)
def test_all_gather_simulation_completes(P, G, sched):
    lay = orc.layout(P, G, [P * 8])
    L = lay.L
    full = np.arange(P * L, dtype=np.float32) + 1
    bufs = []
    for r in range(P):
        b = np.zeros(P * L, np.float32)
        c = orc.chunk_of_rank(r, P, G)
        b[c * L:(c + 1) * L] = full[c * L:(c + 1) * L]
        bufs.append(b)
    orc.simulate(lay, sched, orc.AG, bufs)
    for r in range(P):
        assert (bufs[r] == full).all()


def test_small_integers_reduce_exactly():
    P, G = 8, 4
    lay = orc.layout(P, G, [P * 64])
    rng = np.random.default_rng(0)
    x = [rng.integers(-8, 9, P * lay.L).astype(np.float32) for _ in range(P)]
    exact = np.sum(x, axis=0, dtype=np.int64)
    for sched in SCHEDS:
        bufs = [a.copy() for a in x]
        orc.simulate(lay, sched, orc.RS, bufs)
        for r in range(P):
            c = orc.chunk_of_rank(r, P, G)
            assert (bufs[r][c * lay.L:(c + 1) * lay.L].astype(np.int64) == exact[c * lay.L:(c + 1) * lay.L]).all()


# ---- Fig. 4 worked example -------------------------------------------------------
def test_fig4_example_steps():
    kv = {k: int(v) for k, v in _rows("fig4_horing.txt")}
    P, g = kv["N"], kv["g"]
    G = P // g
    lay = orc.layout(P, G, [P * 8])
    for r in range(P):
        ms = orc.schedule(lay, orc.HORING, r, orc.AG)
        steps = lambda ph, ring: len({m.step for m in ms if m.phase == ph and m.ring == ring})   # noqa: E731
        assert steps(1, 0) == kv["phase1_intra_steps"]
        assert steps(1, 1) == kv["phase1_inter_steps"]
        assert steps(2, 0) == kv["phase2_intra_steps"]
        assert steps(2, 1) == 0
        j, i = orc.group_of(r, G)
        own = orc.chunk_of_rank(r, P, G) * lay.L
        # phase 1, first step: the rank's OWN shard goes out on both rings
        first = [m for m in ms if m.phase == 1 and m.step == 1]
        assert sorted((m.ring, m.send_off, m.send_len) for m in first) == [(0, own, lay.L), (1, own, lay.L)]
        for m in ms:
            jt, it = orc.group_of(m.send_to, G)
            assert (jt == j and it == (i + 1) % G) if m.ring == 0 else (it == i and jt == (j + 1) % g)
        # phase 2 hands on exactly what came over the inter-group ring: g-1 chunks per step
        for k in range(1, G):
            assert sum(m.send_len for m in ms if m.phase == 2 and m.step == k) == (g - 1) * lay.L


# ---- Table 3 volumes and Eq. 1 -----------------------------------------------------
@pytest.mark.parametrize("P,G", [(9, 3), (16, 8), (64, 8), (4, 2), (12, 4), (8, 8), (8, 1)])
def test_table3_volumes(P, G):
    g = P // G
    lay = orc.layout(P, G, [P * 8 * 3])
    L = lay.L
    psi = P * L
    for coll in (orc.RS, orc.AG):
        for sched in (orc.HRING, orc.HORING):
            for r in range(P):
                intra, inter = orc.volumes(lay, sched, r, coll)
                # rows PaRO-IGG backward R-S(G) / PaRO-NIG update A-G(P), per GPU
                assert inter == (g - 1) * psi // P
                assert intra == (G - 1) * psi // G if g > 1 else intra == (G - 1) * L
        # flat ring (rows ZeRO-1/2/3): every link carries Psi/N * (N-1); g of the N links
        # cross groups (when there is more than one group)
        tot_intra = tot_inter = 0
        for r in range(P):
            a, b = orc.volumes(lay, orc.RING, r, coll)
            tot_intra += a
            tot_inter += b
        n_inter = g if g > 1 else 0
        assert tot_inter == n_inter * (psi // P) * (P - 1)
        assert tot_intra == (P - n_inter) * (psi // P) * (P - 1)


@pytest.mark.parametrize("P,G", [(16, 8), (64, 8), (4, 2), (12, 4), (8, 8), (8, 1)])
@pytest.mark.parametrize("s", [1, 2, 8, 10])
def test_eq1_saving_of_grouped_two_step_reduce_scatter(P, G, s):
    g = P // G
    lay = orc.layout(P, G, [P * 8 * 5])
    psi = P * lay.L
    glob = sum(orc.volumes(lay, orc.RING, 0, orc.RS))                       # one global reduce-scatter
    hr = orc.schedule(lay, orc.HRING, 0, orc.RS)
    intra = sum(m.send_len for m in hr if m.ring == 0)                       # intra-group reduce-scatter
    inter = sum(m.send_len for m in hr if m.ring == 1)                       # inter-group reduce-scatter
    delta = s * glob - (s * intra + inter)
    assert delta * P == psi * (s - 1) * (g - 1)
    if g == 1 or s == 1:
        assert delta == 0


def test_degenerate_groupings_collapse_to_the_flat_ring():
    for P, G in [(8, 8), (8, 1)]:
        for c in range(P):
            flat, _ = orc.fold_order(P, G, orc.RING, c)
            for sched in (orc.HRING, orc.HORING):
                order, gl = orc.fold_order(P, G, sched, c)
                assert order == flat and gl in (1, P)


def test_layout_rejects_bad_shapes():
    for P, G in [(0, 1), (4, 3), (4, 0), (-2, 1)]:
        with pytest.raises(ValueError):
            orc.layout(P, G, [10])
    with pytest.raises(ValueError):
        orc.layout(4, 2, [])
    with pytest.raises(ValueError):
        orc.layout(4, 2, [3, -1])


# ---- gradient accumulation with the grouped two-step reduce-scatter (Sec. 3.3) ---------
def test_split_phases_equal_the_whole_collective():
    P, G = 12, 4
    lay = orc.layout(P, G, [P * 16])
    x = _contribs(P, P * lay.L, seed=21)
    whole = [a.copy() for a in x]
    orc.simulate(lay, orc.HRING, orc.RS, whole)
    split = [a.copy() for a in x]
    orc.simulate(lay, orc.HRING, orc.RS, split, phases={1})
    # after the intra-group phase every rank holds its group's partial of its whole block
    for r in range(P):
        j, i = orc.group_of(r, G)
        lo, n = orc.state_range(lay, r, "I")
        order = [j * G + (i + l) % G for l in range(1, G + 1)]
        want = orc.fold([x[q][lo:lo + n] for q in order], G)
        assert split[r][lo:lo + n].tobytes() == want.tobytes()
    orc.simulate(lay, orc.HRING, orc.RS, split, phases={2})
    for r in range(P):
        c = orc.chunk_of_rank(r, P, G)
        assert split[r][c * lay.L:(c + 1) * lay.L].tobytes() == whole[r][c * lay.L:(c + 1) * lay.L].tobytes()


@pytest.mark.parametrize("P,G,s", [(8, 4, 3), (4, 2, 1), (6, 3, 4), (4, 4, 2), (4, 1, 2)])
def test_accumulation_closed_form_order(P, G, s):
    g = P // G
    lay = orc.layout(P, G, [P * 24])
    L = lay.L
    mbs = [_contribs(P, P * L, seed=100 + b) for b in range(s)]
    got = orc.accumulate_two_step(lay, mbs)
    for r in range(P):
        j, i = orc.group_of(r, G)
        c = orc.chunk_of_rank(r, P, G)
        sl = slice(c * L, (c + 1) * L)
        # per group: intra-group ring fold of each micro-batch, micro-batches added in order;
        # then the groups in inter-group ring order, the owner's group last
        sums = []
        for k in range(1, g + 1):
            jj = (j + k) % g
            members = [jj * G + (i + l) % G for l in range(1, G + 1)]
            per_mb = [orc.fold([mbs[b][q][sl] for q in members], G) for b in range(s)]
            sums.append(orc.fold(per_mb, s))
        want = orc.fold(sums, g)
        assert got[r].tobytes() == want.tobytes()


def test_accumulation_small_integers_exact():
    P, G, s = 8, 4, 5
    lay = orc.layout(P, G, [P * 40])
    rng = np.random.default_rng(3)
    mbs = [[rng.integers(-8, 9, P * lay.L).astype(np.float32) for _ in range(P)] for _ in range(s)]
    exact = np.sum([np.sum(mb, axis=0, dtype=np.int64) for mb in mbs], axis=0)
    got = orc.accumulate_two_step(lay, mbs)
    for r in range(P):
        c = orc.chunk_of_rank(r, P, G)
        assert (got[r].astype(np.int64) == exact[c * lay.L:(c + 1) * lay.L]).all()
