#!/usr/bin/env python3
"""Benchmark of the PaRO update-stage hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input that is
already resident in HBM: sweep 1 (ordered fold of the P gradient contributions
+ sum of squares) and sweep 2 (clip + Adam + bf16 pack).  The timed loop issues
the two sweeps through paro_reduce_shard and paro_adam_shard(dst) - exactly the
launches paro_step_fused makes when clipping - so that HIP events recorded on
the launch stream between them give each sweep's own duration; the one-call
entry point is timed right after as a cross-check.

Prints ONE JSON line.  `value` = shard parameters updated per second.
`roofline` is for the dominant kernel (sweep 1, the fold): algorithmic bytes
(2P + 4 per parameter: P bf16 reads, one fp32 write) over its mean duration,
against 8 TB/s; `copy_ref` is what a plain device copy of 3.4 GB reaches in the same
process (`roofline.frac_of_copy` = the fold's rate over the copy's).  `cpu_baseline` times the CPU oracle on a bounded sample of the
same buffers on this machine's host cores (a baseline, not a target).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama7b_share",
                    choices=["llama7b_share", "llama65b_share", "tiny_share", "ragged", "ragged_large"],
                    help="llama7b_share: the configuration the metric is quoted on.  ragged: the 10 000-tensor list "
                         "(sizes log-uniform in [1, 65536], 25 %% fp32 / 75 %% bf16 gradients, P = 8, G = 4; a shard of "
                         "7.3 M parameters, cache-resident - no roofline claim); ragged_large: the same law with 160 000 "
                         "tensors (a shard of about 118 M parameters, 2.4 GB of contributions per sweep).  Both use the "
                         "tensor layout")
    ap.add_argument("--no-clip", action="store_true", help="single-sweep path (max_norm = 0)")
    ap.add_argument("--layout", default="chunk", choices=["chunk", "tensors"],
                    help="chunk: contributions are buffers in shard coordinates (the default, the configuration the "
                         "metric is quoted on); tensors: the same shard of the Llama-7B tensor list, each simulated "
                         "rank handing over per-tensor gradients (llama7b_share only)")
    ap.add_argument("--cpu-sample", type=int, default=0,
                    help="elements of the shard the oracle is timed on with all threads (0 = the whole shard, "
                         "about 10 s of CPU work in all at the default workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--extras", action="store_true",
                    help="also time the steps around the update stage (ring hop, all-gather landing copy) at the "
                         "same shard size and add them to the JSON line under 'extras'")
    ap.add_argument("--copy-ref", action="store_true",
                    help="only run a plain 4 GiB device copy three times (reference for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    return ap.parse_args()


def measured_traffic(workload: str, kernel: str):
    """HBM bytes per launch of the dominant kernel from rocprofv3 --pmc runs (counters cannot be
    read from inside this process), when a summary for this kernel and workload has been
    committed under profiles/; returns (bytes or None, where the figure comes from)."""
    name = f"traffic_{kernel}_{workload}.txt"
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None, None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch:"):
            return float(line.split(":", 1)[1]), f"profiles/{name} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, earlier run)"
    return None, None


def stats(ms):
    """mean / median / min of per-launch durations in ms."""
    import numpy as np
    a = np.asarray(ms, dtype=np.float64)
    return {"mean": float(a.mean()), "median": float(np.median(a)), "min": float(a.min()), "n": int(a.size)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU's share of the step; it runs on exactly one GPU "
              f"(got --gpus {args.gpus}).", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from __graft_entry__ import ensure_built, library_identity
    ensure_built()                             # builds libparo.so if there is none or its sources changed since
    import paper_2310_06003_amd as paro        # raises if there is no library: no fallback path
    import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if args.copy_ref:
        n = (4 << 30) // 4
        a = torch.ones(n, dtype=torch.float32, device=dev)
        b = torch.zeros(n, dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_ref_bytes_read": 4 << 30, "copy_ref_bytes_written": 4 << 30, "launches": 3}))
        return

    ragged = args.workload.startswith("ragged")
    if args.workload == "tiny_share":           # quick functional check of the script itself
        cfg = wl.Config("tiny_share", 16, 8, "IIG", [16 * 2048 * 64], max_norm=1.0)
    elif args.workload == "ragged_large":       # the ragged list's law, 16 times as many tensors
        cfg = wl.config("ragged")
        cfg.sizes, cfg.dtypes = wl.ragged_sizes(160000, seed=5), wl.ragged_dtypes(160000, seed=55)
    else:
        cfg = wl.config(args.workload)
    if ragged:
        args.layout = "tensors"
        args.no_cpu_baseline = True             # the oracle is timed on the headline workload only
    P, G, strategy = cfg.P, cfg.G, cfg.strategy
    rank = 5 if P == 16 else (21 if P == 64 else (3 if ragged else 0))
    max_norm = 0.0 if args.no_clip else cfg.max_norm
    sizes = cfg.sizes
    if args.layout == "tensors" and not ragged:
        assert args.workload == "llama7b_share", "--layout tensors goes with the llama7b_share workload"
        sizes = wl.llama7b_sizes()                 # the same Psi as a list of 291 tensors
    pl = paro.paro_plan(P, G, strategy, sizes, grad_dtype=cfg.dtypes)
    L = paro.paro_shard_len(pl)
    ob, ol = paro.paro_range(pl, rank, "O")
    assert ol == L
    dst_len, slot_off, slot_len = paro.paro_pack_slot(pl, rank)

    contrib_bytes_per_rank = 2 * L              # bytes one rank contributes to the range (bf16)
    if ragged:
        sets = wl.tensor_contribs(P, sizes, cfg.dtypes, 7, 1, dist=cfg.dist, device=dev)
        tables = [torch.tensor([t.data_ptr() if t.numel() else 0 for t in ts.tensors], dtype=torch.int64, device=dev)
                  for ts in sets]
        ptrs = [t.data_ptr() for t in tables]
        layout = paro.PARO_TENSORS
        contrib = None
        contrib_bytes_per_rank = sum(n * (4 if cfg.dtypes[t] == wl.F32 else 2) for (t, _o, _s, n) in paro.paro_segments(pl, rank))
    elif args.layout == "tensors":
        # per simulated rank, only the tensors that meet this rank's range exist; the pointer table gives
        # the others a valid address, which the step never reads
        sets = wl.tensor_contribs_over_range(P, sizes, ob, ol, 7, device=dev)
        tables = []
        for ts in sets:
            spare = ts.flat[wl.BF16].data_ptr()
            tables.append(torch.tensor([spare if t is None else t.data_ptr() for t in ts.tensors],
                                       dtype=torch.int64, device=dev))
        ptrs = [t.data_ptr() for t in tables]
        layout = paro.PARO_TENSORS
        # the same bytes in shard coordinates (for the CPU baseline and the extras)
        first = next(t for t, x in enumerate(sets[0].tensors) if x is not None)
        lo = ob - sum(sizes[:first])
        contrib = [ts.flat[wl.BF16][lo:lo + ol] for ts in sets]
    else:
        contrib = wl.chunk_contribs(P, L, 7, device=dev)
        ptrs = [t.data_ptr() for t in contrib]
        layout = paro.PARO_CHUNK
    p, m, v = wl.master_state(L, 7, device=dev)
    dst = torch.zeros(dst_len, dtype=torch.bfloat16, device=dev)
    g = torch.empty(L, dtype=torch.float32, device=dev)
    ss = torch.zeros(1, dtype=torch.float64, device=dev)
    hp = dict(wl.ADAM_DEFAULT, grad_scale=1.0 / P, max_norm=max_norm, adamw=True)
    st = torch.cuda.current_stream().cuda_stream

    def split_step(k, ev=None):
        hs = paro.make_adam(step=k, **hp)
        if max_norm > 0:
            if ev:
                ev[0].record()
            paro.paro_reduce_shard(pl, rank, ptrs, layout, g.data_ptr(), ss.data_ptr(), st)
            if ev:
                ev[1].record()
            paro.paro_adam_shard(pl, rank, hs, g.data_ptr(), ss.data_ptr(), p.data_ptr(), m.data_ptr(), v.data_ptr(),
                                 dst.data_ptr(), st)
            if ev:
                ev[2].record()
        else:
            if ev:
                ev[0].record()
            paro.paro_step_fused(pl, rank, ptrs, layout, hs, 0, 0, p.data_ptr(), m.data_ptr(), v.data_ptr(),
                                 dst.data_ptr(), st)
            if ev:
                ev[1].record()
                ev[2].record()

    def fused_step(k):
        paro.paro_step_fused(pl, rank, ptrs, layout, paro.make_adam(step=k, **hp), g.data_ptr(),
                             ss.data_ptr(), p.data_ptr(), m.data_ptr(), v.data_ptr(), dst.data_ptr(), st)

    K, W = args.steps, args.warmup
    for k in range(1, W + 1):
        split_step(k)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        split_step(W + 1 + k, events[k])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_step = elapsed * 1e3 / K
    sweep1 = [e[0].elapsed_time(e[1]) for e in events]
    sweep2 = [e[1].elapsed_time(e[2]) for e in events]
    ms1, ms2 = float(np.mean(sweep1)), float(np.mean(sweep2))
    step_ev = [e[0].elapsed_time(e[2]) for e in events]           # one step on the device, launch gaps included

    # the one-call entry point, same work
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        fused_step(W + K + 1 + k)
    torch.cuda.synchronize()
    ms_fused_entry = (time.perf_counter() - t0) * 1e3 / K

    clip = max_norm > 0
    bytes_step = P * contrib_bytes_per_rank + (34 if clip else 26) * L
    bytes_dom = P * contrib_bytes_per_rank + (4 if clip else 26) * L
    dom_ms = ms1
    achieved = bytes_dom / (dom_ms * 1e-3) / 1e9
    dom_kernel = ("k_reduce4t" if args.layout == "tensors" else "k_reduce4") if clip else "k_fused4"
    traffic, traffic_source = measured_traffic(args.workload, dom_kernel)      # summaries are per kernel and workload
    out = {
        "metric": "shard_params_updated_per_s (fused reduce+Adam+pack step)",
        "value": L / (ms_step * 1e-3),
        "unit": "params/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": ms_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "layout": args.layout, "P": P, "G": G, "strategy": strategy,
                   "schedule": ["ring", "h-ring", "ho-ring"][paro.paro_sched(pl)], "rank": rank,
                   "shard_params": L, "contrib_dtype": "bf16/f32 per tensor" if ragged else "bf16", "tensors": len(sizes),
                   "clip_max_norm": max_norm,
                   "sweeps": 2 if clip else 1},
        "hbm_gbps_step": bytes_step / (ms_step * 1e-3) / 1e9,
        "hbm_frac_step": bytes_step / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "algorithmic_bytes_per_param_step": bytes_step / L,
        "ms_fused_entry": ms_fused_entry,
        "ms_per_step_device": stats(step_ev),
        "library": library_identity(),
        "kernels": {
            "sweep1_fold_sumsq": {"ms": ms1, "ms_stats": stats(sweep1), "bytes_per_param": bytes_dom / L,
                                  "gbps": bytes_dom / (ms1 * 1e-3) / 1e9,
                                  "gbps_median": bytes_dom / (float(np.median(sweep1)) * 1e-3) / 1e9,
                                  "gbps_best": bytes_dom / (min(sweep1) * 1e-3) / 1e9},
        },
        "roofline": {"kernel": dom_kernel + (" (fold + sum of squares)" if clip else " (fold + Adam + pack)"),
                     "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": traffic_source,
                     "launch_ms": stats(sweep1)},
    }
    if clip:
        out["kernels"]["sweep2_adam_pack"] = {"ms": ms2, "ms_stats": stats(sweep2), "bytes_per_param": 30,
                                              "gbps": 30 * L / (ms2 * 1e-3) / 1e9,
                                              "gbps_median": 30 * L / (float(np.median(sweep2)) * 1e-3) / 1e9,
                                              "gbps_best": 30 * L / (min(sweep2) * 1e-3) / 1e9}

    def timed(fn, reps=10):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    # what a plain copy reaches on this machine, same process: the library's own copy kernel (the all-gather
    # landing copy) moving a message of 2L bf16 elements = as many bytes as g holds, each way
    cp = paro.paro_plan(2, 2, "NGG", [4 * L])
    assert paro.paro_shard_len(cp) == 2 * L
    ca = torch.zeros(4 * L, dtype=torch.bfloat16, device=dev)
    cb = torch.ones(4 * L, dtype=torch.bfloat16, device=dev)
    ms_copy = timed(lambda: paro.paro_collective_step(cp, 0, paro.PARO_RING, paro.PARO_AG, 1, 0, 1,
                                                      [ca.data_ptr(), cb.data_ptr()], st))
    copy_gbps = 8 * L / (ms_copy * 1e-3) / 1e9
    del ca, cb
    out["copy_ref"] = {"kernel": "k_copy16", "bytes_read": 4 * L, "bytes_written": 4 * L, "ms": ms_copy,
                       "gbps": copy_gbps}
    out["roofline"]["frac_of_copy"] = achieved / copy_gbps
    out["hbm_frac_of_copy_step"] = out["hbm_gbps_step"] / copy_gbps

    if ragged:
        # the chunk layout at the same shard size and rank count (all-bf16 contributions in shard coordinates):
        # what the tensor layout's bookkeeping costs on top of the plain sweeps
        cpl = paro.paro_plan(P, G, strategy, [P * L])
        cc = wl.chunk_contribs(P, L, 9, device=dev)
        cptrs = [t.data_ptr() for t in cc]
        ms_c1 = timed(lambda: paro.paro_reduce_shard(cpl, rank, cptrs, paro.PARO_CHUNK, g.data_ptr(), ss.data_ptr(), st), 20)
        out["chunk_layout_ref"] = {"sweep1_ms": ms_c1, "bytes_per_param": 2 * P + 4,
                                   "gbps": (2 * P + 4) * L / (ms_c1 * 1e-3) / 1e9,
                                   "tensor_layout_sweep1_over_chunk_layout": float(np.median(sweep1)) / ms_c1,
                                   "tensor_layout_sweep1_gbps_over_chunk_layout":
                                       bytes_dom / (float(np.median(sweep1)) * 1e-3) / 1e9 / ((2 * P + 4) * L / (ms_c1 * 1e-3) / 1e9)}
        del cc

    if args.extras and not ragged:
        wire = torch.zeros(L, dtype=torch.float32, device=dev)          # partial arriving over the ring (fp32)
        ms_hop = timed(lambda: paro.paro_ring_hop(pl, wire.data_ptr(), paro.PARO_F32, contrib[0].data_ptr(),
                                                  paro.PARO_BF16, g.data_ptr(), L, st))
        ms_acc = timed(lambda: paro.paro_ring_hop(pl, g.data_ptr(), paro.PARO_F32, wire.data_ptr(), paro.PARO_F32,
                                                  g.data_ptr(), L, st))
        # all-gather landing: one peer's packed chunk copied into this rank's parameter buffer (P = 2 toy plan
        # whose chunk is this shard, so that one step moves exactly L bf16 elements)
        ag = paro.paro_plan(2, 2, "NGG", [2 * L])
        assert paro.paro_shard_len(ag) == L
        pa = torch.zeros(2 * L, dtype=torch.bfloat16, device=dev)
        pb = torch.ones(2 * L, dtype=torch.bfloat16, device=dev)
        ms_ag = timed(lambda: paro.paro_collective_step(ag, 0, paro.PARO_RING, paro.PARO_AG, 1, 0, 1,
                                                        [pa.data_ptr(), pb.data_ptr()], st))
        ms_pack = timed(lambda: paro.paro_pack_params(pl, rank, p.data_ptr(), dst.data_ptr(), st))
        out["extras"] = {
            "pack_alone_f32_to_bf16": {"ms": ms_pack, "bytes_per_param": 6, "gbps": 6 * L / (ms_pack * 1e-3) / 1e9},
            "ring_hop_f32_plus_bf16": {"ms": ms_hop, "bytes_per_param": 10, "gbps": 10 * L / (ms_hop * 1e-3) / 1e9},
            "accumulate_f32_inplace": {"ms": ms_acc, "bytes_per_param": 12, "gbps": 12 * L / (ms_acc * 1e-3) / 1e9},
            "all_gather_landing_copy_bf16": {"ms": ms_ag, "bytes_per_param": 4, "gbps": 4 * L / (ms_ag * 1e-3) / 1e9},
        }
        del wire, pa, pb

    if not args.no_cpu_baseline:
        import oracle as orc
        n = min(args.cpu_sample, L) if args.cpu_sample > 0 else L
        order, gl = orc.fold_order(P, G, orc.default_sched(P, G), orc.chunk_of_rank(rank, P, G))
        host = [contrib[q][:n].cpu().view(torch.int16).numpy().view(np.uint16) for q in order]
        p0, m0, v0 = wl.master_state(n, 7)
        hp32 = {k: np.float32(x) for k, x in wl.ADAM_DEFAULT.items()}

        def oracle_step(threads, n_el):
            orc.set_threads(threads)
            pp, mm, vv = (a[:n_el].numpy().copy() for a in (p0, m0, v0))
            srcs = [h[:n_el] for h in host]
            t = time.perf_counter()
            gg = orc.fold(srcs, gl)
            tot = orc.sumsq(gg)
            coef = orc.clip_coef(tot, np.float32(1.0 / P), np.float32(max_norm))
            orc.adam(gg, pp, mm, vv, sc=float(np.float32(1.0 / P)) * coef, step=1, **hp32)
            orc.bf16_rne(pp)
            return n_el / (time.perf_counter() - t)

        nthreads = orc.threads()
        oracle_step(nthreads, min(n, 1 << 20))                       # page in
        rate_all = max(oracle_step(nthreads, n) for _ in range(2))
        n1 = min(n, 1 << 27)
        rate_one = oracle_step(1, n1)
        orc.set_threads(nthreads)
        out["cpu_baseline"] = {"value": rate_all, "unit": "params/s", "cores": nthreads, "kind": "oracle",
                               "sample": (f"{'the whole shard' if n == L else 'first ' + str(n) + ' shard elements'} of the "
                                          f"same buffers ({n} elements), all {P} contributions, one fused step (fold + "
                                          f"sum of squares + clip + Adam fp64 + pack), best of 2"),
                               "single_thread": {"value": rate_one, "cores": 1, "sample_elements": n1},
                               "host_cpus": os.cpu_count()}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
