"""The entry point that allocates nothing, paro_step_fused_static, against paro_step_fused:
same inputs, every output bit for bit, on two calls in a row of which the second is smaller;
then the single sweep, a multi-chunk update range, and the limits it must refuse."""
import numpy as np
import pytest
import torch

import workloads as wl
from harness import DEV, hp_dict, hp_struct, np_of, stream

pytestmark = pytest.mark.gpu


def _both_entries(paro, P, G, strategy, sizes, rank, seed, max_norm, step, fresh_plan_for_static=True):
    """Runs the step through both entry points from the same starting state; returns nothing,
    asserts that g, sum of squares, p, m, v and the whole packed buffer agree bit for bit."""
    pl = paro.paro_plan(P, G, strategy, sizes)
    # a plan of its own that has never made a device call: the static entry must not need one
    pl_static = paro.paro_plan(P, G, strategy, sizes) if fresh_plan_for_static else pl
    ob, ol = paro.paro_range(pl, rank, "O")
    dst_len, slot_off, slot_len = paro.paro_pack_slot(pl, rank)
    contrib = wl.chunk_contribs(P, ol, seed, device=DEV)
    ptrs = [t.data_ptr() for t in contrib]
    hp = hp_dict(P, max_norm=max_norm)
    outs = []
    for entry in ("plan", "static"):
        p, m, v = wl.master_state(ol, seed, device=DEV)
        dst = torch.zeros(dst_len, dtype=torch.bfloat16, device=DEV)
        g = torch.full((ol,), 7.0, dtype=torch.float32, device=DEV)
        ss = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
        for k in range(1, step + 1):
            if entry == "plan":
                paro.paro_step_fused(pl, rank, ptrs, paro.PARO_CHUNK, hp_struct(paro, hp, k), g.data_ptr(),
                                     ss.data_ptr(), p.data_ptr(), m.data_ptr(), v.data_ptr(), dst.data_ptr(), stream())
            else:
                paro.paro_step_fused_static(pl_static, rank, ptrs, hp_struct(paro, hp, k), g.data_ptr(), ss.data_ptr(),
                                            p.data_ptr(), m.data_ptr(), v.data_ptr(), dst.data_ptr(), stream())
        torch.cuda.synchronize()
        outs.append({k: np_of(t).tobytes() for k, t in (("g", g), ("ss", ss), ("p", p), ("m", m), ("v", v), ("q", dst))})
    what = f"P{P} G{G} {strategy} rank{rank} n{ol} clip{max_norm}"
    for k in outs[0]:
        assert outs[0][k] == outs[1][k], f"{what}: {k} differs between paro_step_fused and paro_step_fused_static"
    if max_norm > 0:
        assert np.frombuffer(outs[1]["ss"], np.float64)[0] > 0
    return outs[1]


def test_static_entry_equals_plan_entry_two_calls_second_smaller(paro):
    """Two calls in a row on the shared static array: a shard of 9.4 M elements (36 864 partial
    sums, two-level finalize), then one of 70 k (a single level) whose partial sums land where the
    first call's still lie."""
    big = _both_entries(paro, 16, 8, "IIG", [16 * 2048 * 288 + 40], 5, seed=3, max_norm=0.05, step=2)
    small = _both_entries(paro, 4, 2, "IIG", [4 * 70000 - 3], 1, seed=4, max_norm=0.05, step=1)
    assert big["ss"] != small["ss"]


def test_static_entry_single_sweep_and_wide_update_range(paro):
    """No clipping (one sweep, no scratch at all), and an update range of several chunks
    (optimizer state sharded inside the group only / not at all)."""
    _both_entries(paro, 8, 4, "IGG", [8 * 2048 * 33], 6, seed=5, max_norm=0.0, step=1)
    _both_entries(paro, 8, 4, "III", [8 * 2048 * 20 + 8], 3, seed=6, max_norm=0.02, step=1)
    _both_entries(paro, 4, 2, "NNN", [4 * 2048 * 9], 2, seed=7, max_norm=0.02, step=1, fresh_plan_for_static=False)


def test_static_entry_refuses_what_it_cannot_do(paro):
    P, sizes = 4, [4 * 4096]
    masked = paro.paro_plan(P, 2, "IIG", sizes + [64], no_decay=[0, 1])
    hp = hp_struct(paro, hp_dict(P, max_norm=1.0), 1)
    a = torch.zeros(8192, dtype=torch.float32, device=DEV)
    with pytest.raises(paro.ParoError) as e:
        paro.paro_step_fused_static(masked, 0, [a.data_ptr()] * P, hp, a.data_ptr(), a.data_ptr(), a.data_ptr(),
                                    a.data_ptr(), a.data_ptr(), a.data_ptr(), stream())
    assert e.value.code == paro.PARO_EINVAL and "mask" in str(e.value)
    huge = paro.paro_plan(2, 1, "GGG", [2 * paro.PARO_STATIC_MAX_CHUNK + 16])     # host only: nothing is allocated
    with pytest.raises(paro.ParoError) as e:
        paro.paro_step_fused_static(huge, 0, [a.data_ptr()] * 2, hp, a.data_ptr(), a.data_ptr(), a.data_ptr(),
                                    a.data_ptr(), a.data_ptr(), a.data_ptr(), stream())
    assert e.value.code == paro.PARO_ERANGE and "PARO_STATIC_MAX_CHUNK" in str(e.value)
    mixed = paro.paro_plan(P, 2, "IIG", [4096, 4096 * 3], grad_dtype=[paro.PARO_BF16, paro.PARO_F32])
    with pytest.raises(paro.ParoError) as e:
        paro.paro_step_fused_static(mixed, 0, [a.data_ptr()] * P, hp, a.data_ptr(), a.data_ptr(), a.data_ptr(),
                                    a.data_ptr(), a.data_ptr(), a.data_ptr(), stream())
    assert e.value.code == paro.PARO_EINVAL
    torch.cuda.synchronize()
