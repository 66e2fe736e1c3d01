#!/usr/bin/env python3
"""Benchmark of the SparseLoCo compress + aggregate path on one MI355X.

One "step" is one worker-round: the compression of one worker's pseudo-gradient
(error-feedback accumulate, chunk Top-k, 2-bit quantizer, residual, payload) and
the aggregate of R workers' payloads fused with the outer SGD step, over the
whole tensor list.  Inputs are synthetic and resident in HBM before the timed
region.  Two wire formats are timed in the same run: the plain one (12-bit
indices: sl_compress + sl_decompress_avg_apply) and the coded one (Rice-coded
indices emitted by the compressor and decoded inside the aggregate:
sl_compress_coded + sl_decompress_avg_apply_coded); --wire chooses which of them
is the line's `value` (default: the coded one, the format whose sizes the paper's
Table 1 prints), the other is reported under `other_wire`.
Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4 | --list paper512M] [--wire plain|coded]
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E peak
PROFILE_TAGS = {4: "1p8B"}
# Table 1 of the paper (512M model, R = 8, H = 15): pseudo-gradient size per worker and sync in MB at
# density 0.78 % (k = 32) and 3.12 % (k = 128), and the bits per index its coder reaches
# (appendix "Compression of indices in Top-k")
PAPER_TABLE1_MB = {32: 5.45, 128: 17.21}
PAPER_INDEX_BITS = {32: 8.9, 128: 6.6, 256: 5.6}


def sources_sha():
    """Hash of the kernel sources: a counter profile is only quoted while it matches them."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2508_15706_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:16]


def cpu_baseline(w, descs, host, sample_desc):
    """The CPU oracle, as it stands, on the benchmarked list itself: one compress of worker 0 from host
    copies of the bench's own e and delta, one aggregate of host copies of the R payloads the GPU
    produced.  Its outputs are compared with the GPU's for the same round (a whole-list parity check
    that costs nothing extra)."""
    import numpy as np
    from oracle import oracle

    t0 = time.perf_counter()
    pay = oracle.compress(descs, w.k, host["e"], host["delta"], w.beta)
    t_comp = time.perf_counter() - t0
    same_payload = bool(np.array_equal(pay, host["payloads"][0]))
    same_e = bool(np.array_equal(host["e"].view(np.uint32), host["e_gpu"].view(np.uint32)))
    t0 = time.perf_counter()
    oracle.decompress_avg_apply(descs, w.k, host["theta"], host["payloads"], w.lr)
    t_apply = time.perf_counter() - t0
    same_theta = bool(np.array_equal(host["theta"].view(np.uint32), host["theta_gpu"].view(np.uint32)))
    n_el = sum(d[0] * d[1] for d in descs)
    return {
        "value": n_el / (t_comp + t_apply) / 1e9, "unit": "Gelem/s", "cores": oracle.max_threads(),
        "kind": "oracle",
        "sample": f"{sample_desc}: one compress of worker 0 (host copies of the bench's e and delta) + one "
                  f"aggregate of the R={w.R} payloads; cpu work {t_comp + t_apply:.1f} s",
        "ms_compress": 1e3 * t_comp, "ms_apply": 1e3 * t_apply,
        "gpu_equals_oracle": {"payload": same_payload, "e": same_e, "theta": same_theta},
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--list", choices=["config", "paper178M", "paper512M", "paper2B"], default="config",
                    help="the tensor list: the configuration's (default) or one of the paper's own three "
                         "architectures (vocabulary 32000, every dimension a multiple of 64)")
    ap.add_argument("--wire", choices=["plain", "coded"], default="coded",
                    help="wire format of the timed steps: Rice-coded indices emitted by the compressor and "
                         "decoded inside the aggregate (default), or plain 12-bit indices")
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
    ap.add_argument("--cpu-sample-layers", type=int, default=None,
                    help="time the CPU oracle on the tensors of the first layers only (default: the whole list "
                         "while it has at most 2.5e9 elements)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-times", action="store_true",
                    help="skip the extra steps that are run with per-kernel events after the timed ones; the "
                         "per-kernel fields are then 0")
    ap.add_argument("--mode", choices=["deferred", "eager"], default="deferred",
                    help="deferred: the error update of a round is folded into the next round's "
                         "read of e (SL_COMPRESS_DEFER_RESIDUAL + pending); eager: scattered update "
                         "inside every compress call")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the R workers are R payload buffers on "
              "it, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2508_15706_amd import binding as sl
    from paper_2508_15706_amd import synth

    sl.lib()                                   # fails loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    if args.list == "config":
        w = synth.workload(args.config, k=args.k, flat=args.flat)
        list_name = f"config {w.config_id}: {w.name}"
    else:
        w = synth.paper_workload(args.list, k=args.k, flat=args.flat)
        list_name = f"the paper's own {w.name[6:]} architecture"
    if args.workers is not None:
        if not 1 <= args.workers <= 64:
            raise SystemExit("--workers must be between 1 and 64")
        w.R = args.workers
    # A tensor with fewer than k elements has no Top-k (the paper's density sweep reaches k = 2048, its norm
    # vectors have 1024 to 2560 elements): on the paper's own lists such tensors are left out, and the line says so.
    dropped = 0
    if args.list != "config":
        kept = [s for s in w.specs if s.numel >= w.k]
        dropped = len(w.specs) - len(kept)
        if dropped:
            w.specs = synth._finish(kept, args.flat)
    descs = [s.desc() for s in w.specs]
    plan = sl.sl_plan_create(descs, w.k) if args.bits == 2 else sl.sl_plan_create_bits(descs, w.k, args.bits)
    N, n_chunks, arena = plan.num_elements, plan.num_chunks, w.arena
    ws = sl.alloc_workspace(plan)
    cap = sl.sl_rice_max_bytes(plan)
    if cap == 0:
        raise SystemExit("list too long for the coded format")

    # state: theta, worker 0's error buffer (persistent), R payloads in both wire formats
    theta = torch.empty(arena, dtype=torch.float32, device=dev)
    synth.fill_theta(w, theta)
    e0 = torch.zeros(arena, dtype=torch.float32, device=dev)
    pays = [sl.alloc_payload(plan) for _ in range(w.R)]
    wires = [torch.zeros(cap, dtype=torch.uint8, device=dev) for _ in range(w.R)]
    deltas = [torch.empty(arena, dtype=torch.float32, device=dev) for _ in range(args.delta_buffers)]

    # set-up (untimed): the other workers' payloads of this round, each from its own delta
    scratch_e = torch.zeros(arena, dtype=torch.float32, device=dev)
    for r in range(1, w.R):
        synth.fill_delta(w, deltas[0], 1, r)
        scratch_e.zero_()
        sl.sl_compress_coded(plan, scratch_e, deltas[0], w.beta, pays[r], wires[r], ws)
    del scratch_e
    for i, d in enumerate(deltas):             # worker 0's pseudo-gradients of successive rounds
        synth.fill_delta(w, d, 1 + i, 0)
    torch.cuda.synchronize()
    wire_bytes = [cap] + [sl.coded_size(wires[r]) for r in range(1, w.R)]   # worker 0's: the buffer's capacity

    # worker 0's payload alternates between two buffers so that the previous round's
    # record can be handed back as `pending`
    own = [pays[0], sl.alloc_payload(plan)]
    state = {"pending": None, "i": 0}

    def step(mode, wire):
        i = state["i"]
        out = own[i % 2]
        flags = sl.SL_COMPRESS_DEFER_RESIDUAL if mode == "deferred" else sl.SL_COMPRESS_DEFAULT
        if wire == "coded":
            sl.sl_compress_coded(plan, e0, deltas[i % len(deltas)], w.beta, out, wires[0], ws, flags=flags,
                                 pending=state["pending"])
            sl.sl_decompress_avg_apply_coded(plan, theta, wires, wire_bytes, w.lr)
        else:
            sl.sl_compress(plan, e0, deltas[i % len(deltas)], w.beta, out, ws, flags=flags, pending=state["pending"])
            sl.sl_decompress_avg_apply(plan, theta, [out] + pays[1:], w.lr)
        state["pending"] = out if mode == "deferred" else None
        state["i"] = i + 1

    def flush():
        if state["pending"] is not None:
            sl.sl_residual_apply(plan, e0, state["pending"])
            state["pending"] = None

    # The library's per-kernel events cost a few microseconds per kernel.  On the benchmark lists that is
    # nothing and they are recorded over the timed steps themselves; on a list of a few hundred chunks it
    # would be a large part of the step, so there the K timed steps run bare and the events are recorded
    # over extra steps afterwards.
    events_inline = n_chunks >= 16384 and not args.no_kernel_times

    def timed(mode, wire, steps):
        for _ in range(args.warmup):
            step(mode, wire)
        torch.cuda.synchronize()
        if events_inline:
            sl.sl_profile_begin(plan, steps)
        t0 = time.perf_counter()
        for _ in range(steps):
            step(mode, wire)
        # the last round's error update is applied inside the timed region, so that no
        # work of the K rounds is left outstanding when the clock stops
        flush()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        prof = {p: (0.0, 0) for p in sl.PROF_PHASES}
        if events_inline:
            prof = sl.sl_profile_end(plan)
        elif not args.no_kernel_times:
            n_ev = max(4, steps // 2)
            step(mode, wire)
            sl.sl_profile_begin(plan, n_ev)
            for _ in range(n_ev):
                step(mode, wire)
            flush()
            torch.cuda.synchronize()
            prof = sl.sl_profile_end(plan)
        return 1e3 * dt / steps, prof

    few = max(2, args.steps // 4)
    other_mode = "eager" if args.mode == "deferred" else "deferred"
    other_wire = "coded" if args.wire == "plain" else "plain"
    ms_other_mode, prof_other_mode = timed(other_mode, args.wire, few)
    ms_other_wire, prof_other_wire = timed(args.mode, other_wire, max(few, args.steps // 2))
    ms_step, prof = timed(args.mode, args.wire, args.steps)
    own_coded_bytes = sl.coded_size(wires[0])      # (one of the two loops wrote worker 0's coded payload)

    graph_info = None
    if args.graph:
        # one graph = one full cycle of the step's buffer rotation (two payload buffers, the
        # delta buffers), so that every replay continues the chain exactly as eager steps would
        import math
        cycle = 2 * len(deltas) // math.gcd(2, len(deltas))
        if state["i"] % cycle:
            for _ in range(cycle - state["i"] % cycle):
                step(args.mode, args.wire)
        if state["pending"] is None and args.mode == "deferred":
            for _ in range(cycle):
                step(args.mode, args.wire)       # the captured first step expects a pending payload
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for _ in range(cycle):
                    step(args.mode, args.wire)
        torch.cuda.synchronize()
        replays = max(1, -(-args.steps // cycle))
        for _ in range(max(1, args.warmup // cycle)):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        flush()
        torch.cuda.synchronize()
        ms_eager = ms_step
        ms_step = 1e3 * (time.perf_counter() - t0) / (replays * cycle)
        graph_info = {"steps_per_graph": cycle, "replays": replays, "eager_ms_per_step": ms_eager}
        args.steps = replays * cycle

    # ---- algorithmic bytes.  Plain wire: 20 B per element + (R + 1) payloads of 7k/4 B per chunk and a
    # table per tensor.  Coded wire: the payloads at their coded sizes (worker 0's written, R read).
    rec = 3 * w.k // 2 + w.k * args.bits // 8
    hdr = 0 if args.bits == 32 else max(16, 4 << args.bits)
    plain_payload = rec * n_chunks + hdr * len(descs)
    coded_read = own_coded_bytes + sum(wire_bytes[1:])

    def path_bytes(wire):
        return 20 * N + ((w.R + 1) * plain_payload if wire == "plain" else own_coded_bytes + coded_read)

    def index_bytes(wire):      # what kernel A writes per launch besides e: the index part of the payload
        if wire == "plain":
            return (3 * w.k // 2 + (4 * w.k if args.bits == 32 else 0)) * n_chunks
        return own_coded_bytes - (w.k * args.bits // 8) * n_chunks - hdr * len(descs)

    # dominant kernel: accumulate + select.  Algorithmic bytes per launch: read e and delta, write e
    # (12 B per element) + the index part of the payload
    sel_ms = prof["select"][0]
    sel_bytes = 12 * N + index_bytes(args.wire)
    sel_gbs = sel_bytes / (sel_ms * 1e-3) / 1e9 if sel_ms > 0 else 0.0
    apply_ms = prof["apply"][0]
    apply_bytes = 8 * N + (w.R * plain_payload if args.wire == "plain" else coded_read)
    compress_ms = sum(prof[p][0] for p in ("select", "stats", "codes", "lut", "residual", "index"))

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
    synth.fill_delta(w, dst, 1 + (1 % len(deltas)), 0)      # the copy overwrote a pseudo-gradient: restore it

    # HBM bytes per launch of the dominant kernel as measured with rocprofv3 counters (FETCH_SIZE +
    # WRITE_SIZE, scaled by a plain copy; written by paper_2508_15706_amd/rocprof_summary.py from profiled
    # runs of this same command).  Quoted only while the profile was taken with the kernel sources of this
    # tree and for this command's workload; otherwise null, with the reason.
    traffic, traffic_source = None, "no counter profile for this workload"
    tag = PROFILE_TAGS.get(w.config_id, "")
    tpath = os.path.join(ROOT, "profiles", f"traffic_config{w.config_id}_{tag}_{args.wire}.json")
    default_workload = (args.list == "config" and not args.flat and args.k is None and args.bits == 2 and
                        args.workers is None and args.mode == "deferred")
    if os.path.exists(tpath) and default_workload:
        tj = json.load(open(tpath))
        name = next((n for n in tj["kernels"] if n.startswith("k_select")), None)
        if tj.get("sources_sha") != sources_sha():
            traffic_source = f"profiles/{os.path.basename(tpath)} is older than the kernel sources: not quoted"
        elif name and tj["kernels"][name]["fetch_bytes"] is not None and tj["kernels"][name]["write_bytes"] is not None:
            traffic = tj["kernels"][name]["fetch_bytes"] + tj["kernels"][name]["write_bytes"]
            traffic_source = (f"profiles/{os.path.basename(tpath)}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of "
                              f"`bench.py {tj.get('bench_args', '')}` at kernel sources {tj['sources_sha']} "
                              "(a separate run, not this one)")

    def frac(nbytes, ms):
        return nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS

    out = {
        "metric": "pseudo-gradient elements compressed+aggregated/sec",
        "value": N / (ms_step * 1e-3) / 1e9,
        "unit": "Gelem/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{list_name}, {len(descs)} fp32 tensors, "
                               f"N={N}, chunk 4096 ({'flat runs' if args.flat else '64x64 tiles / 1-D runs'}), "
                               f"k={w.k}, R={w.R}, beta={w.beta}, lr={w.lr}, "
                               f"{'fp32' if args.bits == 32 else str(args.bits) + '-bit'} values, {args.mode} residual, "
                               f"{args.wire} wire format",
                   "n_elements": N, "n_chunks": n_chunks, "k": w.k, "R": w.R, "value_bits": args.bits,
                   "wire": args.wire, "arena_bytes": 4 * arena, "tensors_smaller_than_k_left_out": dropped},
        "argv": " ".join(sys.argv[1:]),
        "roofline": {"bound": "hbm", "kernel": "k_select (EF accumulate + chunk Top-k)",
                     "achieved": sel_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": sel_gbs / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "ms": sel_ms, "algorithmic_bytes": sel_bytes},
        "path_hbm": {"algorithmic_bytes_per_step": path_bytes(args.wire),
                     "achieved_GBps": path_bytes(args.wire) / (ms_step * 1e-3) / 1e9,
                     "frac_of_peak": frac(path_bytes(args.wire), ms_step),
                     "device_copy_GBps": copy_gbs},
        "mode": args.mode, "hip_graph": graph_info,
        "kernel_events": "over the timed steps" if events_inline else "over extra steps after the timed ones",
        "other_mode": {"mode": other_mode, "ms_per_step": ms_other_mode, "value": N / (ms_other_mode * 1e-3) / 1e9,
                       "kernels_ms": {p: prof_other_mode[p][0] for p in prof_other_mode}},
        "other_wire": {"wire": other_wire, "ms_per_step": ms_other_wire, "value": N / (ms_other_wire * 1e-3) / 1e9,
                       "algorithmic_bytes_per_step": path_bytes(other_wire),
                       "frac_of_peak": frac(path_bytes(other_wire), ms_other_wire),
                       "kernels_ms": {p: prof_other_wire[p][0] for p in prof_other_wire}},
        "kernels_ms": {p: prof[p][0] for p in prof},
        "compress_ms": compress_ms, "apply_ms": apply_ms,
        "apply_GBps": apply_bytes / (apply_ms * 1e-3) / 1e9 if apply_ms > 0 else 0.0,
        "payload": {"plain_bytes": plain_payload, "coded_bytes": own_coded_bytes,
                    "bits_per_index": (own_coded_bytes - hdr * len(descs)) * 8 / (n_chunks * w.k) - args.bits,
                    "paper_bits_per_index": PAPER_INDEX_BITS.get(w.k)},
    }
    if args.list == "paper512M" and args.bits == 2 and w.k in PAPER_TABLE1_MB:
        # Table 1 of the paper quotes the message size per worker on this very model
        out["payload"]["table1"] = {"coded_MB": own_coded_bytes / 1e6, "paper_MB": PAPER_TABLE1_MB[w.k],
                                    "density_percent": 100.0 * w.k / 4096}

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

    # the stand-alone transcoders (not part of the timed step)
    back = sl.alloc_payload(plan)
    coded2 = torch.zeros(cap, dtype=torch.uint8, device=dev)
    enc_ms = time_ms(lambda: sl.sl_rice_encode(plan, pays[w.R - 1], coded2, ws))
    dec_ms = time_ms(lambda: sl.sl_rice_decode(plan, coded2, sl.coded_size(coded2), back))
    out["payload"]["transcoders"] = {
        "encode_ms": enc_ms, "decode_ms": dec_ms,
        "lossless": bool(torch.equal(back[:plan.payload_bytes], pays[w.R - 1][:plan.payload_bytes])),
        "equals_compressor_output": bool(w.R < 2 or torch.equal(coded2[:wire_bytes[-1]], wires[-1][:wire_bytes[-1]]))}
    del back, coded2

    if args.outer_steps:
        # the DiLoCo-family entry points, each timed alone on the same list (context rows, not
        # part of the step): algorithmic bytes = 4 B per element per stream touched
        mom = torch.zeros(arena, dtype=torch.float32, device=dev)
        dirs = [torch.empty(arena, dtype=torch.float32, device=dev) for _ in range(w.R)]
        for r, dbuf in enumerate(dirs):
            synth.fill_delta(w, dbuf, 2, r)
        pl_apply = 8 * N + w.R * plain_payload
        rows = {
            "lom_direction": (lambda: sl.sl_lom_direction(plan, mom, deltas[0], 0.9, dirs[0]), 16 * N),
            "dense_avg_apply": (lambda: sl.sl_dense_avg_apply(plan, theta, None, dirs, w.lr), (w.R + 2) * 4 * N),
            "dense_avg_apply_nesterov": (lambda: sl.sl_dense_avg_apply(plan, theta, mom, dirs, w.lr, 0.9),
                                         (w.R + 4) * 4 * N),
            "decompress_avg_apply_nesterov": (
                lambda: sl.sl_decompress_avg_apply_nesterov(plan, theta, mom, [own[0]] + pays[1:], w.lr, 0.9),
                pl_apply + 8 * N),
            "decompress_avg_apply_nesterov_coded": (
                lambda: sl.sl_decompress_avg_apply_nesterov_coded(plan, theta, mom, wires, wire_bytes, w.lr, 0.9),
                8 * N + coded_read + 8 * N),
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
        # One more round on the GPU (eager, plain wire, state as the timed rounds left it) with host copies
        # of its inputs taken first; the oracle then does the same round on the host's cores.
        layers = args.cpu_sample_layers
        if layers is None and N > 2_500_000_000:
            layers = 4
        if layers is None:
            sub_specs, sample_desc = list(w.specs), "the whole benchmarked list"
        else:
            names = tuple(f"l{l}." for l in range(layers))
            sub_specs = [s for s in w.specs if s.name.startswith(names)] or list(w.specs)
            sample_desc = (f"the tensors of the first {layers} layers of the list ({len(sub_specs)} tensors, "
                           f"{sum(s.numel for s in sub_specs)} elements)")
        lo = min(s.offset for s in sub_specs)
        hi = max(s.offset + s.numel for s in sub_specs)
        sub_descs = [(s.rows, s.cols, s.offset - lo, s.layout) for s in sub_specs]
        sub_plan = plan if layers is None else (sl.sl_plan_create(sub_descs, w.k) if args.bits == 2 else None)
        if sub_plan is None or args.bits != 2:
            out["cpu_baseline"] = None
        else:
            d_dev = deltas[state["i"] % len(deltas)]
            host = {"e": e0[lo:hi].cpu().numpy(), "delta": d_dev[lo:hi].cpu().numpy(),
                    "theta": theta[lo:hi].cpu().numpy()}
            sub_pays = [sl.alloc_payload(sub_plan) for _ in range(w.R)]
            sub_ws = sl.alloc_workspace(sub_plan)
            e_sub, th_sub = e0[lo:hi], theta[lo:hi]
            if layers is not None:       # the other workers' payloads on the sub-list
                tmp_e = torch.zeros(hi - lo, dtype=torch.float32, device=dev)
                tmp_d = torch.empty(arena, dtype=torch.float32, device=dev)
                for r in range(1, w.R):
                    synth.fill_delta(w, tmp_d, 1, r)
                    tmp_e.zero_()
                    sl.sl_compress(sub_plan, tmp_e, tmp_d[lo:hi], w.beta, sub_pays[r], sub_ws)
                del tmp_e, tmp_d
            else:
                sub_pays[1:] = pays[1:]
            sl.sl_compress(sub_plan, e_sub, d_dev[lo:hi], w.beta, sub_pays[0], sub_ws)
            sl.sl_decompress_avg_apply(sub_plan, th_sub, sub_pays, w.lr)
            torch.cuda.synchronize()
            host["payloads"] = [p[:sub_plan.payload_bytes].cpu().numpy() for p in sub_pays]
            host["e_gpu"] = e_sub.cpu().numpy()
            host["theta_gpu"] = th_sub.cpu().numpy()
            del deltas, theta, e0, e_sub, th_sub
            out["cpu_baseline"] = cpu_baseline(w, sub_descs, host, sample_desc)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
