"""The fused step inside a HIP graph: the device entry points only enqueue kernels on the
caller's stream (no allocation, no synchronisation, no memset after the plan's first device
call), so a captured step must replay to the eager result, every time."""
import pytest
import torch

import workloads as wl
from harness import DEV, PtrTable, hp_dict, hp_struct, np_of

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("layout", ["chunk", "chunk, the entry point that allocates nothing", "tensors with a decay mask"])
@pytest.mark.parametrize("max_norm", [0.0, 0.01])
def test_fused_step_replays_from_a_graph(paro, max_norm, layout):
    P, G, strategy, rank = 8, 4, "IIG", 3
    if layout.startswith("chunk"):
        sizes = [P * 2048 * 40 + 24]
        pl = paro.paro_plan(P, G, strategy, sizes)
        L = paro.paro_shard_len(pl)
        contrib = wl.chunk_contribs(P, L, 5, device=DEV)
        ptrs = [t.data_ptr() for t in contrib]
        kind = paro.PARO_CHUNK
    else:               # per-tensor gradients, boundaries inside blocks, a mask: the per-tile table is in play
        sizes = [70000, 3, 2048 * 7, 12345, 1, 300000, 77]
        pl = paro.paro_plan(P, G, strategy, sizes, grad_dtype=[0, 1, 0, 2, 0, 0, 1], no_decay=[0, 1, 0, 0, 1, 0, 1])
        L = paro.paro_shard_len(pl)
        sets = wl.tensor_contribs(P, sizes, [0, 1, 0, 2, 0, 0, 1], 5, 1, device=DEV)
        tables = [PtrTable(ts.tensors) for ts in sets]
        ptrs = [t.ptr() for t in tables]
        kind = paro.PARO_TENSORS
    hp = hp_dict(P, max_norm=max_norm)
    hs = hp_struct(paro, hp, 3)
    dst_len, slot_off, slot_len = paro.paro_pack_slot(pl, rank)

    def state():
        p, m, v = wl.master_state(L, 5, device=DEV)
        return dict(p=p, m=m, v=v, dst=torch.zeros(dst_len, dtype=torch.bfloat16, device=DEV),
                    g=torch.empty(L, dtype=torch.float32, device=DEV),
                    ss=torch.zeros(1, dtype=torch.float64, device=DEV))

    def step(s, stream):
        if "allocates nothing" in layout:       # its plan never makes a device call of the allocating kind
            paro.paro_step_fused_static(pl, rank, ptrs, hs, s["g"].data_ptr(), s["ss"].data_ptr(),
                                        s["p"].data_ptr(), s["m"].data_ptr(), s["v"].data_ptr(), s["dst"].data_ptr(), stream)
        else:
            paro.paro_step_fused(pl, rank, ptrs, kind, hs, s["g"].data_ptr(), s["ss"].data_ptr(),
                                 s["p"].data_ptr(), s["m"].data_ptr(), s["v"].data_ptr(), s["dst"].data_ptr(), stream)

    # eager: three steps in a row, the state after each kept
    eager = state()
    step(eager, torch.cuda.current_stream().cuda_stream)      # also creates the plan's device tables
    want = []
    ref = state()
    for _ in range(3):
        step(ref, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        want.append({k: np_of(ref[k]).tobytes() for k in ("p", "m", "v", "dst")})

    graphed = state()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        step(graphed, side.cuda_stream)
        graph.capture_end()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    # capture enqueues nothing: the state is still the initial one
    assert np_of(graphed["p"]).tobytes() == np_of(state()["p"]).tobytes()
    for k in range(3):
        graph.replay()
        torch.cuda.synchronize()
        _ = float(graphed["ss"].item())                         # eager work and a sync between replays
        got = {name: np_of(graphed[name]).tobytes() for name in ("p", "m", "v", "dst")}
        assert got == want[k], f"replay {k + 1} differs from the eager step"
