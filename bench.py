#!/usr/bin/env python3
"""Benchmark of the SparseLoCo compress + aggregate path on one MI355X.

One "step" is one worker-round: sl_compress of one worker's pseudo-gradient
(error-feedback accumulate, chunk Top-k, 2-bit quantizer, residual, payload) and
sl_decompress_avg_apply of R workers' payloads fused with the outer SGD step,
over the whole tensor list.  Inputs are synthetic and resident in HBM before
the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E peak
PROFILE_TAGS = {4: "1p8B"}


def cpu_baseline(w, sample_layers):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: the
    tensors of the first `sample_layers` transformer layers, R workers compressed
    (each timed) and one aggregation (timed)."""
    import numpy as np
    import torch
    from oracle import oracle
    from paper_2508_15706_amd import synth

    names = tuple(f"l{l}." for l in range(sample_layers))
    specs = [s for s in w.specs if s.name.startswith(names)] or list(w.specs)
    base = min(s.offset for s in specs)
    descs = [(s.rows, s.cols, s.offset - base, s.layout) for s in specs]
    n = max(d[2] + d[0] * d[1] for d in descs)
    n_el = sum(d[0] * d[1] for d in descs)
    g = torch.Generator().manual_seed(synth.seed_for(w.config_id, 50, 0))
    t_comp, pays = [], []
    for r in range(w.R):
        e = (torch.randn(n, generator=g) * w.scale).numpy()
        d = (torch.randn(n, generator=g) * w.scale).numpy()
        t0 = time.perf_counter()
        pays.append(oracle.compress(descs, w.k, e, d, w.beta))
        t_comp.append(time.perf_counter() - t0)
    theta = (torch.randn(n, generator=g) * 0.02).numpy()
    t0 = time.perf_counter()
    oracle.decompress_avg_apply(descs, w.k, theta, pays, w.lr)
    t_apply = time.perf_counter() - t0
    t_round = sum(t_comp) / len(t_comp) + t_apply
    return {
        "value": n_el / t_round / 1e9, "unit": "Gelem/s", "cores": oracle.max_threads(),
        "kind": "oracle",
        "sample": f"tensors of the first {sample_layers} layers of the list ({len(specs)} tensors, "
                  f"{n_el} elements): mean of R={w.R} compress calls + one aggregation; "
                  f"cpu work {sum(t_comp) + t_apply:.1f} s",
        "ms_compress": 1e3 * sum(t_comp) / len(t_comp), "ms_apply": 1e3 * t_apply,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--k", type=int, default=None)
    ap.add_argument("--workers", type=int, default=None,
                    help="number of workers R whose payloads are aggregated (default: the configuration's)")
    ap.add_argument("--flat", action="store_true", help="cut every tensor into runs of 4096")
    ap.add_argument("--bits", type=int, default=2, choices=[1, 2, 3, 4, 32],
                    help="payload value width (the paper's setting is 2; 32 = unquantized fp32)")
    ap.add_argument("--graph", action="store_true",
                    help="time the steps as replays of a captured HIP graph (takes the launch overhead "
                         "out of small configurations; per-kernel times still come from eager steps)")
    ap.add_argument("--outer-steps", action="store_true",
                    help="also time the dense outer steps of the DiLoCo family (extra arenas: R + 1)")
    ap.add_argument("--delta-buffers", type=int, default=3)
    ap.add_argument("--cpu-layers", type=int, default=4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mode", choices=["deferred", "eager"], default="deferred",
                    help="deferred: the error update of a round is folded into the next round's "
                         "read of e (SL_COMPRESS_DEFER_RESIDUAL + pending); eager: scattered update "
                         "inside every sl_compress")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the R workers are R payload buffers on "
              "it, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2508_15706_amd import binding as sl
    from paper_2508_15706_amd import synth

    sl.lib()                                   # fails loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    w = synth.workload(args.config, k=args.k, flat=args.flat)
    if args.workers is not None:
        if not 1 <= args.workers <= 64:
            raise SystemExit("--workers must be between 1 and 64")
        w.R = args.workers
    descs = [s.desc() for s in w.specs]
    plan = sl.sl_plan_create(descs, w.k) if args.bits == 2 else sl.sl_plan_create_bits(descs, w.k, args.bits)
    N, n_chunks, arena = plan.num_elements, plan.num_chunks, w.arena
    ws = sl.alloc_workspace(plan)

    # state: theta, worker 0's error buffer (persistent), R payload buffers
    theta = torch.empty(arena, dtype=torch.float32, device=dev)
    synth.fill_theta(w, theta)
    e0 = torch.zeros(arena, dtype=torch.float32, device=dev)
    pays = [sl.alloc_payload(plan) for _ in range(w.R)]
    deltas = [torch.empty(arena, dtype=torch.float32, device=dev) for _ in range(args.delta_buffers)]

    # set-up (untimed): the other workers' payloads of this round, each from its own delta
    scratch_e = torch.zeros(arena, dtype=torch.float32, device=dev)
    for r in range(1, w.R):
        synth.fill_delta(w, deltas[0], 1, r)
        scratch_e.zero_()
        sl.sl_compress(plan, scratch_e, deltas[0], w.beta, pays[r], ws)
    del scratch_e
    for i, d in enumerate(deltas):             # worker 0's pseudo-gradients of successive rounds
        synth.fill_delta(w, d, 1 + i, 0)
    torch.cuda.synchronize()

    # worker 0's payload alternates between two buffers so that the previous round's
    # payload can be handed back as `pending`
    own = [pays[0], sl.alloc_payload(plan)]
    state = {"pending": None, "i": 0}

    def step(mode):
        i = state["i"]
        out = own[i % 2]
        if mode == "deferred":
            sl.sl_compress(plan, e0, deltas[i % len(deltas)], w.beta, out, ws,
                           flags=sl.SL_COMPRESS_DEFER_RESIDUAL, pending=state["pending"])
            state["pending"] = out
        else:
            sl.sl_compress(plan, e0, deltas[i % len(deltas)], w.beta, out, ws, pending=state["pending"])
            state["pending"] = None
        sl.sl_decompress_avg_apply(plan, theta, [out] + pays[1:], w.lr)
        state["i"] = i + 1

    def timed(mode, steps):
        for _ in range(args.warmup):
            step(mode)
        torch.cuda.synchronize()
        sl.sl_profile_begin(plan, steps)
        t0 = time.perf_counter()
        for _ in range(steps):
            step(mode)
        if state["pending"] is not None:
            # the last round's error update is applied inside the timed region, so that no
            # work of the K rounds is left outstanding when the clock stops
            sl.sl_residual_apply(plan, e0, state["pending"])
            state["pending"] = None
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        return dt, sl.sl_profile_end(plan)

    other = "eager" if args.mode == "deferred" else "deferred"
    dt_other, prof_other = timed(other, max(2, args.steps // 4))
    ms_other = 1e3 * dt_other / max(2, args.steps // 4)
    dt, prof = timed(args.mode, args.steps)
    ms_step = 1e3 * dt / args.steps

    graph_info = None
    if args.graph:
        # one graph = one full cycle of the step's buffer rotation (two payload buffers, the
        # delta buffers), so that every replay continues the chain exactly as eager steps would
        import math
        cycle = 2 * len(deltas) // math.gcd(2, len(deltas))
        if state["i"] % cycle:
            for _ in range(cycle - state["i"] % cycle):
                step(args.mode)
        if state["pending"] is None and args.mode == "deferred":
            for _ in range(cycle):
                step(args.mode)                  # the captured first step expects a pending payload
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for _ in range(cycle):
                    step(args.mode)
        torch.cuda.synchronize()
        replays = max(1, -(-args.steps // cycle))
        for _ in range(max(1, args.warmup // cycle)):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        if state["pending"] is not None:
            sl.sl_residual_apply(plan, e0, state["pending"])
            state["pending"] = None
        torch.cuda.synchronize()
        ms_eager = ms_step
        ms_step = 1e3 * (time.perf_counter() - t0) / (replays * cycle)
        graph_info = {"steps_per_graph": cycle, "replays": replays, "eager_ms_per_step": ms_eager}
        args.steps = replays * cycle

    rec = 3 * w.k // 2 + w.k * args.bits // 8
    hdr = 0 if args.bits == 32 else max(16, 4 << args.bits)
    bytes_round = 20 * N + (w.R + 1) * rec * n_chunks + hdr * len(descs) * (w.R + 1)
    # dominant kernel: accumulate + select.  Algorithmic bytes per launch: read e and
    # delta, write e (12 B/element) + the packed indices it writes (3k/2 B per chunk)
    sel_ms = prof["select"][0]
    sel_bytes = 12 * N + (3 * w.k // 2 + (4 * w.k if args.bits == 32 else 0)) * n_chunks
    sel_gbs = sel_bytes / (sel_ms * 1e-3) / 1e9 if sel_ms > 0 else 0.0
    apply_ms = prof["apply"][0]
    apply_bytes = 8 * N + w.R * (rec * n_chunks + hdr * len(descs))
    compress_ms = sum(prof[p][0] for p in ("select", "stats", "codes", "lut", "residual"))

    # a plain device copy of the same footprint as a practical ceiling (context only)
    src, dst = deltas[0], deltas[1 % len(deltas)]
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    dst.copy_(src)
    ev0.record()
    for _ in range(5):
        dst.copy_(src)
    ev1.record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 8 * arena / (ev0.elapsed_time(ev1) * 1e-3) / 1e9

    # HBM bytes per launch of the dominant kernel as measured with rocprofv3 counters
    # (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy; written by
    # paper_2508_15706_amd/rocprof_summary.py from a profiled run of this same command)
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_config{w.config_id}_{PROFILE_TAGS.get(w.config_id, '')}.json")
    if os.path.exists(tpath) and not args.flat and args.k is None and args.bits == 2 and args.workers is None:
        tk = json.load(open(tpath))["kernels"]
        name = next((n for n in tk if n.startswith("k_select")), None)
        if name and tk[name]["fetch_bytes"] is not None and tk[name]["write_bytes"] is not None:
            traffic = tk[name]["fetch_bytes"] + tk[name]["write_bytes"]

    out = {
        "metric": "pseudo-gradient elements compressed+aggregated/sec",
        "value": N / (ms_step * 1e-3) / 1e9,
        "unit": "Gelem/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config {w.config_id}: {w.name}, {len(descs)} fp32 tensors, "
                               f"N={N}, chunk 4096 ({'flat runs' if args.flat else '64x64 tiles / 1-D runs'}), "
                               f"k={w.k}, R={w.R}, beta={w.beta}, lr={w.lr}, "
                               f"{'fp32' if args.bits == 32 else str(args.bits) + '-bit'} values, {args.mode} residual",
                   "n_elements": N, "n_chunks": n_chunks, "k": w.k, "R": w.R, "value_bits": args.bits},
        "roofline": {"bound": "hbm", "kernel": "k_select (EF accumulate + chunk Top-k)",
                     "achieved": sel_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": sel_gbs / HBM_PEAK_GBS, "traffic": traffic,
                     "ms": sel_ms, "algorithmic_bytes": sel_bytes},
        "path_hbm": {"algorithmic_bytes_per_step": bytes_round,
                     "achieved_GBps": bytes_round / (ms_step * 1e-3) / 1e9,
                     "frac_of_peak": bytes_round / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "device_copy_GBps": copy_gbs},
        "mode": args.mode, "hip_graph": graph_info,
        "other_mode": {"mode": other, "ms_per_step": ms_other, "value": N / (ms_other * 1e-3) / 1e9,
                       "kernels_ms": {p: prof_other[p][0] for p in prof_other}},
        "kernels_ms": {p: prof[p][0] for p in prof},
        "compress_ms": compress_ms, "apply_ms": apply_ms,
        "apply_GBps": apply_bytes / (apply_ms * 1e-3) / 1e9 if apply_ms > 0 else 0.0,
    }
    # index coder (not part of the timed step): coded size and transcoding time of one payload
    def time_ms(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    if args.bits == 2:
        coded = torch.empty(sl.sl_rice_max_bytes(plan), dtype=torch.uint8, device=dev)
        back = sl.alloc_payload(plan)
        enc_ms = time_ms(lambda: sl.sl_rice_encode(plan, own[0], coded, ws))
        coded_bytes = int(coded[8:16].cpu().numpy().view("uint64")[0])
        dec_ms = time_ms(lambda: sl.sl_rice_decode(plan, coded, coded_bytes, back))
        out["index_coder"] = {
            "plain_bytes": plan.payload_bytes, "coded_bytes": coded_bytes,
            "bits_per_index": coded_bytes * 8 / (n_chunks * w.k) - 2.0,
            "lossless": bool(torch.equal(back[:plan.payload_bytes], own[0][:plan.payload_bytes])),
            "encode_ms": enc_ms, "decode_ms": dec_ms,
        }
    if args.outer_steps:
        # the DiLoCo-family entry points, each timed alone on the same list (context rows, not
        # part of the step): algorithmic bytes = 4 B per element per stream touched
        mom = torch.zeros(arena, dtype=torch.float32, device=dev)
        dirs = [torch.empty(arena, dtype=torch.float32, device=dev) for _ in range(w.R)]
        for r, dbuf in enumerate(dirs):
            synth.fill_delta(w, dbuf, 2, r)
        rows = {
            "lom_direction": (lambda: sl.sl_lom_direction(plan, mom, deltas[0], 0.9, dirs[0]), 16 * N),
            "dense_avg_apply": (lambda: sl.sl_dense_avg_apply(plan, theta, None, dirs, w.lr), (w.R + 2) * 4 * N),
            "dense_avg_apply_nesterov": (lambda: sl.sl_dense_avg_apply(plan, theta, mom, dirs, w.lr, 0.9),
                                         (w.R + 4) * 4 * N),
            "decompress_avg_apply_nesterov": (
                lambda: sl.sl_decompress_avg_apply_nesterov(plan, theta, mom, [own[0]] + pays[1:], w.lr, 0.9),
                apply_bytes + 8 * N),
            "sub_topk": (lambda: sl.sl_sub_topk(plan, mom), 4 * N + 4 * w.k * n_chunks),
        }
        out["outer_steps"] = {}
        for name, (fn, nbytes) in rows.items():
            if name == "sub_topk":
                synth.fill_delta(w, mom, 3, 0)
            ms = time_ms(fn, reps=10)
            out["outer_steps"][name] = {"ms": ms, "algorithmic_GBps": nbytes / (ms * 1e-3) / 1e9}
        del mom, dirs
    if not args.no_cpu_baseline:
        del deltas, theta, e0
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_layers)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
