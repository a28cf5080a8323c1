"""GPU parity at the benchmark's full sizes, in the launch configuration the
benchmark times.

Llama-7B share (P=16, G=8, IIG, 421 M shard params): the oracle streams the whole
shard in blocks, so the reduced gradient, the sum of squares, Adam's p, m, v and
the packed parameters are all checked in full, element by element.

65B share (P=64, G=8, IGG, 1.02 G shard params, two-level HO-Ring order): the
oracle folds sampled blocks only (the full fold would move 130 GB to the host);
the sum of squares is checked against an fp64 reduction of the verified
gradient, and Adam + pack run with a norm total supplied by the harness, as a
cross-rank sum would supply it.

Both shards again in the tensor layout (the models' tensor lists, every simulated
rank handing over per-tensor gradients), checked on every block that holds a
tensor boundary plus random ones."""
import numpy as np
import pytest
import torch

import oracle as orc
import workloads as wl
from harness import DEV, PtrTable, compare_step, hp_dict, hp_struct, np_of, oracle_update, stream

pytestmark = pytest.mark.gpu

BLOCK = 1 << 24


def _need_memory(gib):
    import gc
    gc.collect()
    torch.cuda.empty_cache()                    # what earlier tests left in torch's allocator
    free, _ = torch.cuda.mem_get_info()
    if free < gib * (1 << 30):
        pytest.skip(f"needs {gib} GiB of free device memory")


def _sample_blocks(L, block, n_random, seed):
    nb = (L + block - 1) // block
    rng = np.random.default_rng(seed)
    picks = {0, nb - 1} | {int(x) for x in rng.integers(0, nb, n_random)}
    return [(b * block, min(block, L - b * block)) for b in sorted(picks)]


def test_llama7b_share_full_size(paro):
    _need_memory(40)
    cfg = wl.config("llama7b_share")
    P, G, strategy, rank = cfg.P, cfg.G, cfg.strategy, 5
    lay = orc.layout(P, G, cfg.sizes)
    L = lay.L
    assert L == 421_150_976 and lay.total == 6_738_415_616
    sched = orc.default_sched(P, G)
    assert sched == orc.HORING
    pl = paro.paro_plan(P, G, strategy, cfg.sizes)
    order, gl = orc.fold_order(P, G, sched, orc.chunk_of_rank(rank, P, G))

    contrib = wl.chunk_contribs(P, L, 7, device=DEV)
    p, m, v = wl.master_state(L, 7, device=DEV)
    p_old, m_old, v_old = p.clone(), m.clone(), v.clone()        # the state before the step, for the oracle

    dst_len, slot_off, slot_len = paro.paro_pack_slot(pl, rank)
    assert (dst_len, slot_off, slot_len) == orc.pack_slot(lay, rank, strategy) == (2 * L, 0, L)
    dst = torch.zeros(dst_len, dtype=torch.bfloat16, device=DEV)
    g = torch.empty(L, dtype=torch.float32, device=DEV)
    ss = torch.zeros(1, dtype=torch.float64, device=DEV)
    hp = hp_dict(P, max_norm=cfg.max_norm)
    paro.paro_step_fused(pl, rank, [t.data_ptr() for t in contrib], paro.PARO_CHUNK, hp_struct(paro, hp, 1),
                         g.data_ptr(), ss.data_ptr(), p.data_ptr(), m.data_ptr(), v.data_ptr(), dst.data_ptr(),
                         stream())
    torch.cuda.synchronize()

    # the oracle streams the shard: full parity of the reduced gradient, full sum of squares
    total_ref = 0.0
    g_ref = np.empty(L, np.float32)
    for lo in range(0, L, BLOCK):
        n = min(BLOCK, L - lo)
        gr = orc.fold([np_of(contrib[q][lo:lo + n]) for q in order], gl, out=g_ref[lo:lo + n])
        assert np_of(g[lo:lo + n]).tobytes() == gr.tobytes(), f"reduced gradient differs in block at {lo}"
        total_ref += orc.sumsq(gr)
    assert abs(float(ss.item()) - total_ref) <= 1e-12 * total_ref
    coef = orc.clip_coef(total_ref, np.float32(hp["grad_scale"]), np.float32(hp["max_norm"]))
    assert coef < 1.0
    print(f"\n[llama7b share] sum of squares {total_ref:.6e}, clip coefficient {coef:.6f}")

    # ... and then Adam and the pack over EVERY block of the shard (p, m, v, packed bf16)
    worst_p = worst_v = 0
    for lo in range(0, L, BLOCK):
        n = min(BLOCK, L - lo)
        p0, m0, v0 = (np_of(t[lo:lo + n]) for t in (p_old, m_old, v_old))
        gb = g_ref[lo:lo + n]
        ref = oracle_update(lay, strategy, rank, gb, p0, m0, v0, total_sumsq=total_ref, hp=hp, step=1)
        lit = oracle_update(lay, strategy, rank, gb, p0, m0, v0, total_sumsq=total_ref, hp=hp, step=1, literal32=True)
        got = dict(p=np_of(p[lo:lo + n]), m=np_of(m[lo:lo + n]), v=np_of(v[lo:lo + n]),
                   q=np_of(dst[slot_off + lo:slot_off + lo + n]))
        g_hat = float(np.float32(hp["grad_scale"])) * coef * gb.astype(np.float64)
        report = []
        compare_step(got, ref, p_old=p0, m_old=m0, g_hat=g_hat, what=f"llama7b block at {lo}", literal=lit,
                     report=report)
        worst_p, worst_v = max(worst_p, report[0][1]), max(worst_v, report[0][2])
    print(f"[llama7b share] all {(L + BLOCK - 1) // BLOCK} blocks: p, m, v, packed bf16 within the contract and equal to the "
          f"fp32-literal oracle bit for bit; largest distance to the fp64 reference: v {worst_v} ulp, p {worst_p} ulp "
          f"(p counts elements that are cancelled differences, judged on their terms)")
    assert not bool(dst[L:].any()), "the other group's slot of the parameter block must stay untouched"


def _tensor_layout_at_full_size(paro, sizes, P, G, strategy, rank, L_want, need_gib, seed):
    """One rank's shard of a model's tensor list, each simulated rank handing over per-tensor
    gradients: the fold and the sum of squares against the oracle on every block that holds a
    tensor boundary plus random ones, then the fused step on those samples."""
    _need_memory(need_gib)
    lay = orc.layout(P, G, sizes)
    L = lay.L
    assert L == L_want
    sched = orc.default_sched(P, G)
    pl = paro.paro_plan(P, G, strategy, sizes)
    ob, ol = orc.state_range(lay, rank, strategy[2])
    assert paro.paro_range(pl, rank, "O") == (ob, ol) and ol == L
    sets = wl.tensor_contribs_over_range(P, sizes, ob, ol, seed, device=DEV)
    tables = [PtrTable(s.tensors) for s in sets]
    ptrs = [t.ptr() for t in tables]
    segs = orc.segments(lay, ob, ol)
    assert len(segs) >= 5                                     # the range crosses several tensors

    p, m, v = wl.master_state(L, seed, device=DEV)
    blk = 1 << 22
    nb = (L + blk - 1) // blk
    rng = np.random.default_rng(3)
    picks = {0, nb - 1} | {int(x) for x in rng.integers(0, nb, 4)} | {soff // blk for (_t, _o, soff, _n) in segs}
    picks = [(b * blk, min(blk, L - b * blk)) for b in sorted(picks)]
    old = {lo: [np_of(t[lo:lo + n]) for t in (p, m, v)] for lo, n in picks}

    dst_len, slot_off, slot_len = paro.paro_pack_slot(pl, rank)
    assert (dst_len, slot_off, slot_len) == orc.pack_slot(lay, rank, strategy)
    dst = torch.zeros(dst_len, dtype=torch.bfloat16, device=DEV)
    g = torch.empty(L, dtype=torch.float32, device=DEV)
    ss = torch.zeros(1, dtype=torch.float64, device=DEV)
    hp = hp_dict(P, max_norm=1.0)
    paro.paro_step_fused(pl, rank, ptrs, paro.PARO_TENSORS, hp_struct(paro, hp, 1), g.data_ptr(), ss.data_ptr(),
                         p.data_ptr(), m.data_ptr(), v.data_ptr(), dst.data_ptr(), stream())
    torch.cuda.synchronize()

    order, gl = orc.fold_order(P, G, sched, orc.chunk_of_rank(rank, P, G))
    g_blocks = {}
    for lo, n in picks:
        gr = np.empty(n, np.float32)
        for (t, toff, soff, ln) in orc.segments(lay, ob + lo, n):       # the oracle's own map: flat range -> tensors
            orc.fold([np_of(sets[q].tensors[t][toff:toff + ln]) for q in order], gl, out=gr[soff:soff + ln])
        assert np_of(g[lo:lo + n]).tobytes() == gr.tobytes(), f"reduced gradient differs in block at {lo}"
        g_blocks[lo] = gr
    chk = 0.0
    for lo in range(0, L, 1 << 27):
        chk += float(g[lo:lo + (1 << 27)].double().square().sum().item())
    total = float(ss.item())
    assert abs(total - chk) <= 1e-11 * chk
    coef = orc.clip_coef(total, np.float32(hp["grad_scale"]), np.float32(hp["max_norm"]))
    assert coef < 1.0
    for lo, n in picks:
        p0, m0, v0 = old[lo]
        ref = oracle_update(lay, strategy, rank, g_blocks[lo], p0, m0, v0, total_sumsq=total, hp=hp, step=1)
        lit = oracle_update(lay, strategy, rank, g_blocks[lo], p0, m0, v0, total_sumsq=total, hp=hp, step=1,
                            literal32=True)
        got = dict(p=np_of(p[lo:lo + n]), m=np_of(m[lo:lo + n]), v=np_of(v[lo:lo + n]),
                   q=np_of(dst[slot_off + lo:slot_off + lo + n]))
        g_hat = float(np.float32(hp["grad_scale"])) * coef * g_blocks[lo].astype(np.float64)
        compare_step(got, ref, p_old=p0, m_old=m0, g_hat=g_hat, what=f"tensor layout, block at {lo}", literal=lit)


def test_ragged_list_at_size_two_blocks_per_wave(paro):
    """38 000 tensors of the ragged list's law (sizes log-uniform in [1, 65536], a quarter fp32), P = 4:
    a shard of 56 M parameters = 217 000 blocks, where sweep 1 of the tensor layout lets a wave take two
    blocks.  One rank in full: reduced gradient and sum of squares, then the fused step."""
    sizes, dtypes = wl.ragged_sizes(38000, seed=9), wl.ragged_dtypes(38000, seed=99)
    P, G, strategy, rank = 4, 2, "IIG", 2
    lay = orc.layout(P, G, sizes)
    assert lay.L // 256 >= 196608, "the list must be large enough for the two-block shape"
    sched = orc.default_sched(P, G)
    pl = paro.paro_plan(P, G, strategy, sizes, grad_dtype=dtypes)
    sets = wl.tensor_contribs(P, sizes, dtypes, 17, 1, dist="student_t", device=DEV, align_elems=1)
    tables = [PtrTable(s.tensors) for s in sets]
    host = []
    for s in sets:
        flat = {k: np_of(v) for k, v in s.flat.items()}
        host.append([flat[dtypes[t]][s.start[t]:s.start[t] + n] for t, n in enumerate(sizes)])
    ob, ol = orc.state_range(lay, rank, strategy[2])
    g_ref, ss_ref = orc.reduce_shard(lay, strategy, sched, rank, host, "tensors")
    p, m, v = wl.master_state(ol, 18, device=DEV)
    old = [np_of(t) for t in (p, m, v)]
    dst_len, slot_off, slot_len = orc.pack_slot(lay, rank, strategy)
    dst = torch.zeros(dst_len, dtype=torch.bfloat16, device=DEV)
    g = torch.empty(ol, dtype=torch.float32, device=DEV)
    ss = torch.zeros(1, dtype=torch.float64, device=DEV)
    hp = hp_dict(P, max_norm=1.0)
    paro.paro_step_fused(pl, rank, [t.ptr() for t in tables], paro.PARO_TENSORS, hp_struct(paro, hp, 1), g.data_ptr(),
                         ss.data_ptr(), p.data_ptr(), m.data_ptr(), v.data_ptr(), dst.data_ptr(), stream())
    assert np_of(g).tobytes() == g_ref.tobytes(), "reduced gradient differs"
    assert abs(float(ss.item()) - ss_ref) <= 1e-12 * ss_ref
    ref = oracle_update(lay, strategy, rank, g_ref, *old, total_sumsq=ss_ref, hp=hp, step=1)
    lit = oracle_update(lay, strategy, rank, g_ref, *old, total_sumsq=ss_ref, hp=hp, step=1, literal32=True)
    assert ref["coef"] < 1.0
    got = dict(p=np_of(p), m=np_of(m), v=np_of(v), q=np_of(dst)[slot_off:slot_off + slot_len])
    g_hat = float(np.float32(hp["grad_scale"])) * ref["coef"] * g_ref.astype(np.float64)
    compare_step(got, ref, p_old=old[0], m_old=old[1], g_hat=g_hat, what="ragged list at size", literal=lit)


def test_llama7b_share_tensor_layout(paro):
    """The 291-tensor Llama-7B list, P = 16, rank 5's shard (20 tensors meet it)."""
    sizes = wl.llama7b_sizes()
    assert len(sizes) == 291 and sum(sizes) == 6_738_415_616
    _tensor_layout_at_full_size(paro, sizes, 16, 8, "IIG", 5, 421_150_976, 40, seed=11)


def test_llama65b_share_tensor_layout(paro):
    """The 723-tensor 65B list, P = 64, rank 21's shard: 64 simulated ranks' per-tensor gradients
    (about 180 GB), two-level HO-Ring order, a per-tile table for a chunk of half a million tiles."""
    sizes = wl.llama65b_sizes()
    assert len(sizes) == 723 and sum(sizes) == 65_285_660_672
    _tensor_layout_at_full_size(paro, sizes, 64, 8, "IGG", 21, 1_020_088_448, 210, seed=13)


def test_llama65b_share_full_size(paro):
    _need_memory(200)
    cfg = wl.config("llama65b_share")
    P, G, strategy = cfg.P, cfg.G, cfg.strategy
    rank = 21                                   # group 2, local index 5
    lay = orc.layout(P, G, cfg.sizes)
    L = lay.L
    assert L == 1_020_088_448 and lay.total == 65_285_660_672
    sched = orc.default_sched(P, G)
    pl = paro.paro_plan(P, G, strategy, cfg.sizes)
    order, gl = orc.fold_order(P, G, sched, orc.chunk_of_rank(rank, P, G))
    assert gl == G and order[-1] == rank and paro.paro_fold_order(pl, orc.chunk_of_rank(rank, P, G)) == (order, gl)

    contrib = wl.chunk_contribs(P, L, 9, device=DEV)
    p, m, v = wl.master_state(L, 9, device=DEV)
    blk = 1 << 22
    picks = _sample_blocks(L, blk, 4, seed=2)
    old = {lo: [np_of(t[lo:lo + n]) for t in (p, m, v)] for lo, n in picks}
    dst_len, slot_off, slot_len = paro.paro_pack_slot(pl, rank)
    assert (dst_len, slot_off, slot_len) == (8 * L, 2 * L, L)          # sub-slot j = 2 of the group block
    dst = torch.zeros(dst_len, dtype=torch.bfloat16, device=DEV)
    g = torch.empty(L, dtype=torch.float32, device=DEV)
    ss = torch.zeros(1, dtype=torch.float64, device=DEV)
    ptrs = [t.data_ptr() for t in contrib]

    paro.paro_reduce_shard(pl, rank, ptrs, paro.PARO_CHUNK, g.data_ptr(), ss.data_ptr(), stream())
    torch.cuda.synchronize()
    g_blocks = {}
    for lo, n in picks:
        gr = orc.fold([np_of(contrib[q][lo:lo + n]) for q in order], gl)
        assert np_of(g[lo:lo + n]).tobytes() == gr.tobytes(), f"reduced gradient differs in block at {lo}"
        g_blocks[lo] = gr
    # property: the scalar is the sum of squares of the (sample-verified) gradient
    chk = 0.0
    for lo in range(0, L, 1 << 27):
        chk += float(g[lo:lo + (1 << 27)].double().square().sum().item())
    assert abs(float(ss.item()) - chk) <= 1e-11 * chk

    # Adam + pack with a total as a cross-rank sum would deliver it (64 shards of about this size)
    total = 64 * 65000.0
    hp = hp_dict(P, max_norm=cfg.max_norm)
    tot = torch.tensor([total], dtype=torch.float64, device=DEV)
    paro.paro_adam_shard(pl, rank, hp_struct(paro, hp, 1), g.data_ptr(), tot.data_ptr(), p.data_ptr(), m.data_ptr(),
                         v.data_ptr(), dst.data_ptr(), stream())
    torch.cuda.synchronize()
    coef = orc.clip_coef(total, np.float32(hp["grad_scale"]), np.float32(hp["max_norm"]))
    assert coef < 1.0
    for lo, n in picks:
        p0, m0, v0 = old[lo]
        ref = oracle_update(lay, strategy, rank, g_blocks[lo], p0, m0, v0, total_sumsq=total, hp=hp, step=1)
        lit = oracle_update(lay, strategy, rank, g_blocks[lo], p0, m0, v0, total_sumsq=total, hp=hp, step=1,
                            literal32=True)
        got = dict(p=np_of(p[lo:lo + n]), m=np_of(m[lo:lo + n]), v=np_of(v[lo:lo + n]),
                   q=np_of(dst[slot_off + lo:slot_off + lo + n]))
        g_hat = float(np.float32(hp["grad_scale"])) * coef * g_blocks[lo].astype(np.float64)
        compare_step(got, ref, p_old=p0, m_old=m0, g_hat=g_hat, what=f"llama65b block at {lo}", literal=lit)

    # the single-sweep path (no clipping) at P = 64, from the same starting state, on the samples
    del g
    p2, m2, v2 = wl.master_state(L, 9, device=DEV)
    hp2 = hp_dict(P, max_norm=0.0)
    dst.zero_()
    paro.paro_step_fused(pl, rank, ptrs, paro.PARO_CHUNK, hp_struct(paro, hp2, 1), 0, 0, p2.data_ptr(),
                         m2.data_ptr(), v2.data_ptr(), dst.data_ptr(), stream())
    torch.cuda.synchronize()
    for lo, n in picks:
        p0, m0, v0 = old[lo]
        ref = oracle_update(lay, strategy, rank, g_blocks[lo], p0, m0, v0, total_sumsq=0.0, hp=hp2, step=1)
        lit = oracle_update(lay, strategy, rank, g_blocks[lo], p0, m0, v0, total_sumsq=0.0, hp=hp2, step=1,
                            literal32=True)
        got = dict(p=np_of(p2[lo:lo + n]), m=np_of(m2[lo:lo + n]), v=np_of(v2[lo:lo + n]),
                   q=np_of(dst[slot_off + lo:slot_off + lo + n]))
        g_hat = float(np.float32(hp2["grad_scale"])) * g_blocks[lo].astype(np.float64)
        compare_step(got, ref, p_old=p0, m_old=m0, g_hat=g_hat, what=f"llama65b single sweep, block at {lo}",
                     literal=lit)
    assert not bool(dst[:slot_off].any()) and not bool(dst[slot_off + L:].any())
