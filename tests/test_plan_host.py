"""Host logic of libparo (no GPU needed): its tables against the oracle's, bit for
bit, plus error behaviour and the exported symbols."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SHAPES = [(1, 1), (2, 1), (2, 2), (4, 2), (6, 2), (6, 3), (8, 1), (8, 4), (8, 8), (9, 3), (12, 4), (16, 8), (64, 8)]


def test_library_exports_every_declared_symbol(paro):
    text = open(os.path.join(ROOT, "include", "paro.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(paro_[a-z_0-9]+)\s*\(", text))
    assert {"paro_plan", "paro_reduce_shard", "paro_adam_shard", "paro_pack_params", "paro_step_fused"} <= declared
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2310_06003_amd", "libparo.so"))
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(paro.EXPORTS)            # the binding covers the same names


def test_header_is_plain_c_and_the_host_calls_link_from_c(paro, tmp_path):
    """The boundary is a C interface: the header compiles as C99, and a C program links against
    the library and gets the plan's tables (host calls only: no GPU needed)."""
    import subprocess
    src = tmp_path / "use_paro.c"
    src.write_text(r'''
#include <stdio.h>
#include "paro.h"
int main(void) {
    int64_t sizes[3] = {1000, 0, 24};
    paro_plan_t *pl = 0;
    if (paro_plan(4, 2, "IIG", sizes, 3, 0, &pl) != PARO_OK) { printf("plan: %s\n", paro_last_error()); return 1; }
    int64_t b = -1, n = -1;
    if (paro_range(pl, 3, 'O', &b, &n) != PARO_OK) return 2;
    printf("%lld %lld %lld %d %d\n", (long long)paro_total(pl), (long long)paro_shard_len(pl), (long long)b,
           paro_chunk_of_rank(pl, 3), paro_strategy_legal("GNN"));
    if (paro_plan(4, 3, "IIG", sizes, 3, 0, &pl) != PARO_EINVAL) return 3;
    paro_plan_destroy(pl);
    return 0;
}
''')
    exe = tmp_path / "use_paro"
    libdir = os.path.join(ROOT, "paper_2310_06003_amd")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), str(src),
                    "-o", str(exe), "-L", libdir, "-l:libparo.so", "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    lay = orc.layout(4, 2, [1000, 0, 24])
    ob, _ = orc.state_range(lay, 3, "G")
    assert [int(x) for x in out] == [lay.total, lay.L, ob, orc.chunk_of_rank(3, 4, 2), 0]


def test_bench_refuses_more_than_one_gpu():
    """This build measures one GPU's share: bench.py says so and exits for any other count."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout == ""


def test_strategies(paro):
    import itertools
    for s in ("".join(t) for t in itertools.product("NIG", repeat=3)):
        assert paro.paro_strategy_legal(s) == orc.strategy_legal(s)
        if orc.strategy_legal(s):
            paro.paro_plan(4, 2, s, [100])
        else:
            with pytest.raises(paro.ParoError) as ei:
                paro.paro_plan(4, 2, s, [100])
            assert ei.value.code == paro.PARO_ESTRATEGY
    for bad in ("", "GG", "GGGG", "XGG", "ggg"):
        assert not paro.paro_strategy_legal(bad)
        with pytest.raises(paro.ParoError) as ei:
            paro.paro_plan(4, 2, bad, [100])
        assert ei.value.code == paro.PARO_ESTRATEGY


def test_plan_errors(paro):
    E = paro.PARO_EINVAL
    for args in [(0, 1, "GGG", [8]), (4, 3, "GGG", [8]), (4, 0, "GGG", [8]), (257, 1, "GGG", [8]),
                 (4, 2, "GGG", []), (4, 2, "GGG", [5, -1]), (4, 2, "GGG", [0, 0])]:
        with pytest.raises(paro.ParoError) as ei:
            paro.paro_plan(*args)
        assert ei.value.code == E, args
        assert paro.paro_last_error()
    for kw in [dict(sched=7), dict(align_elems=4), dict(align_elems=12), dict(grad_dtype=[3]), dict(pack_dtype=1), dict(pack_dtype=5)]:
        with pytest.raises(paro.ParoError) as ei:
            paro.paro_plan(4, 2, "GGG", [8], **kw)
        assert ei.value.code == E, kw
    pl = paro.paro_plan(4, 2, "IIG", [100])
    for fn, a in [(paro.paro_chunk_of_rank, 4), (paro.paro_chunk_of_rank, -1), (paro.paro_owner_of_chunk, 4),
                  (paro.paro_segments, 9), (paro.paro_pack_slot, 4)]:
        with pytest.raises(paro.ParoError) as ei:
            fn(pl, a)
        assert ei.value.code == paro.PARO_ERANGE
    with pytest.raises(paro.ParoError) as ei:
        paro.paro_range(pl, 0, "X")
    assert ei.value.code == E
    with pytest.raises(paro.ParoError) as ei:
        paro.paro_fold_order(pl, 4)
    assert ei.value.code == paro.PARO_ERANGE


@pytest.mark.parametrize("P,G", SHAPES)
def test_layout_ownership_ranges_slots(paro, P, G):
    rng = np.random.default_rng(P * 31 + G)
    for sizes in ([1], [P - 1 or 1], [8 * P], [8 * P + 1], [int(x) for x in rng.integers(0, 50, 9)] + [3]):
        lay = orc.layout(P, G, sizes)
        for strat in orc.all_legal_strategies():
            pl = paro.paro_plan(P, G, strat, sizes)
            assert (paro.paro_total(pl), paro.paro_shard_len(pl), paro.paro_padded_total(pl)) == \
                   (lay.total, lay.L, P * lay.L)
            assert paro.paro_sched(pl) == orc.default_sched(P, G)
            for r in range(P):
                assert paro.paro_chunk_of_rank(pl, r) == orc.chunk_of_rank(r, P, G)
                assert paro.paro_owner_of_chunk(pl, r) == orc.owner_of_chunk(r, P, G)
                for k, st in enumerate("PGO"):
                    assert paro.paro_range(pl, r, st) == orc.state_range(lay, r, strat[k])
                ob, ol = orc.state_range(lay, r, strat[2])
                assert paro.paro_segments(pl, r) == orc.segments(lay, ob, ol)
                assert paro.paro_pack_slot(pl, r) == orc.pack_slot(lay, r, strat)


def test_align_option(paro):
    pl = paro.paro_plan(4, 2, "GGG", [1000], align_elems=64)
    lay = orc.layout(4, 2, [1000], align=64)
    assert paro.paro_shard_len(pl) == lay.L == 256


@pytest.mark.parametrize("P,G", SHAPES)
def test_fold_order_and_schedules(paro, P, G):
    lay = orc.layout(P, G, [P * 24 - 5])
    for sched in (orc.RING, orc.HRING, orc.HORING):
        pl = paro.paro_plan(P, G, "GGG", [P * 24 - 5], sched=sched)
        assert paro.paro_sched(pl) == sched
        for c in range(P):
            assert paro.paro_fold_order(pl, c) == orc.fold_order(P, G, sched, c)
        for coll in (orc.RS, orc.AG):
            for r in range(P):
                got = sorted((m.phase, m.ring, m.step, m.send_to, m.recv_from, m.send_off, m.send_len, m.recv_off,
                              m.recv_len) for m in paro.paro_schedule(pl, r, coll))
                want = sorted((m.phase, m.ring, m.step, m.send_to, m.recv_from, m.send_off, m.send_len, m.recv_off,
                               m.recv_len) for m in orc.schedule(lay, sched, r, coll))
                assert got == want
                # an explicit kind overrides the plan's own
                other = paro.paro_schedule(pl, r, coll, sched=orc.RING)
                assert len(other) == P - 1


def test_device_calls_reject_bad_arguments_before_touching_the_gpu(paro):
    pl = paro.paro_plan(4, 2, "IIG", [4096])
    hp = paro.make_adam(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, grad_scale=0.25)
    ok = 1 << 20                                         # a fake, aligned, never dereferenced address
    def code(fn, *a):
        with pytest.raises(paro.ParoError) as ei:
            fn(*a)
        return ei.value.code
    assert code(paro.paro_reduce_shard, pl, 7, [ok] * 4, paro.PARO_CHUNK, ok, ok) == paro.PARO_ERANGE
    assert code(paro.paro_reduce_shard, pl, 0, [ok, ok, 0, ok], paro.PARO_CHUNK, ok, ok) == paro.PARO_EINVAL
    assert code(paro.paro_reduce_shard, pl, 0, [ok, ok + 2, ok, ok], paro.PARO_CHUNK, ok, ok) == paro.PARO_EALIGN
    assert code(paro.paro_reduce_shard, pl, 0, [ok] * 4, 5, ok, ok) == paro.PARO_EINVAL
    assert code(paro.paro_reduce_shard, pl, 0, [ok] * 4, paro.PARO_CHUNK, ok + 4, ok) == paro.PARO_EALIGN
    assert code(paro.paro_reduce_shard, pl, 0, [ok] * 4, paro.PARO_CHUNK, 0, ok) == paro.PARO_EINVAL
    assert code(paro.paro_adam_shard, pl, 0, hp, ok, 0, ok, ok + 8, ok, 0) == paro.PARO_EALIGN
    hp_clip = paro.make_adam(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, grad_scale=0.25,
                             max_norm=1.0)
    assert code(paro.paro_adam_shard, pl, 0, hp_clip, ok, 0, ok, ok, ok, 0) == paro.PARO_EINVAL
    hp_bad = paro.make_adam(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, grad_scale=0.25, step=0)
    assert code(paro.paro_adam_shard, pl, 0, hp_bad, ok, 0, ok, ok, ok, 0) == paro.PARO_EINVAL
    assert code(paro.paro_adam_shard, pl, 0, hp, ok, 0, ok, ok, ok, ok + 2) == paro.PARO_EALIGN
    assert code(paro.paro_pack_params, pl, 0, ok, ok + 2) == paro.PARO_EALIGN
    assert code(paro.paro_step_fused, pl, 0, [ok] * 4, paro.PARO_CHUNK, hp_clip, 0, ok, ok, ok, ok, ok) == paro.PARO_EINVAL
    mixed = paro.paro_plan(4, 2, "IIG", [64, 64], grad_dtype=[0, 1])
    assert code(paro.paro_reduce_shard, mixed, 0, [ok] * 4, paro.PARO_CHUNK, ok, ok) == paro.PARO_EINVAL


def test_ring_and_collective_calls_reject_bad_arguments(paro):
    pl = paro.paro_plan(4, 2, "IIG", [4096])
    ok = 1 << 20

    def code(fn, *a):
        with pytest.raises(paro.ParoError) as ei:
            fn(*a)
        return ei.value.code
    assert code(paro.paro_ring_hop, pl, 0, 0, ok, 0, ok, 8) == paro.PARO_EINVAL
    assert code(paro.paro_ring_hop, pl, ok, 0, ok + 2, 0, ok, 8) == paro.PARO_EALIGN
    assert code(paro.paro_ring_hop, pl, ok, 3, ok, 0, ok, 8) == paro.PARO_EINVAL
    assert code(paro.paro_ring_hop, pl, ok, 0, ok, 1, ok, -1) == paro.PARO_EINVAL
    assert code(paro.paro_ring_hop, pl, ok, 0, ok * 2, 1, ok, 8) == paro.PARO_EINVAL      # out aliases a bf16 operand
    assert code(paro.paro_ring_hop, pl, ok, 2, ok * 2, 1, ok, 8) == paro.PARO_EINVAL      # ... or an fp16 one
    bufs = [ok] * 4
    assert code(paro.paro_collective_step, pl, 4, paro.PARO_RING, paro.PARO_RS, 1, 0, 1, bufs) == paro.PARO_ERANGE
    assert code(paro.paro_collective_step, pl, 0, 9, paro.PARO_RS, 1, 0, 1, bufs) == paro.PARO_EINVAL
    assert code(paro.paro_collective_step, pl, 0, paro.PARO_RING, 7, 1, 0, 1, bufs) == paro.PARO_EINVAL
    assert code(paro.paro_collective_step, pl, 0, paro.PARO_RING, paro.PARO_RS, 1, 0, 1, [ok, 0, ok, ok]) == paro.PARO_EINVAL
    assert code(paro.paro_collective_step, pl, 0, paro.PARO_RING, paro.PARO_AG, 1, 0, 1, [ok, ok + 8, ok, ok]) == paro.PARO_EALIGN
    hp = paro.make_adam(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, grad_scale=0.25,
                        skip_nonfinite=True)
    assert code(paro.paro_adam_shard, pl, 0, hp, ok, 0, ok, ok, ok, 0) == paro.PARO_EINVAL          # needs the total
    assert code(paro.paro_step_fused, pl, 0, [ok] * 4, paro.PARO_CHUNK, hp, 0, ok, ok, ok, ok, ok) == paro.PARO_EINVAL
