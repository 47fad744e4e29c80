#!/usr/bin/env python3
"""Benchmark of the Tier-2 attention step on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input already resident
in HBM: gh_kv_append -> gh_decode_attention_out -> gh_decode_reduce on one stream (the attention
kernel stores the final rows of the heads whose strip one worker covered alone; the merge completes
the others).  The same row is re-appended at the same position every step, so each step moves
identical bytes.

Prints ONE JSON line on stdout (diagnostics go to stderr):
  value     sequence-steps per second over the timed steps (wall clock, sync on both sides)
  roofline  the attention kernel's algorithmic bytes per launch / its mean duration between HIP
            events on the launch stream, against the 8 TB/s HBM peak
  cpu_baseline  the float64 oracle timed on the host cores on a bounded sample of the same workload
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E peak

# HBM bytes per attention launch (FETCH_SIZE + WRITE_SIZE, each scaled by what the same counter
# reads for a plain 1 GiB device copy) are read from profiles/traffic.json, which
# `python -m paper_2501_11779_amd.rocprof_summary` writes together with the rocprofv3 summaries in
# profiles/; they are valid for this file's default step only.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")


def measured_traffic(name):
    """(bytes per attention launch, where the figure comes from) or (None, None)."""
    try:
        with open(TRAFFIC_FILE) as fh:
            rec = json.load(fh)[name]
        return rec["attention_bytes_per_launch"], (
            f"profiles/traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on {rec['kernel']}, "
            f"scaled by a 1 GiB device copy (factors {rec['fetch_factor']:.4f} / "
            f"{rec['write_factor']:.4f}); summary {rec['summary']}")
    except (OSError, KeyError, ValueError):
        return None, None

CONFIG_OF = {"c1": "configs[0]", "c2": "configs[1]", "c3": "configs[2]", "c4": "configs[3]",
             "c5": "configs[4]"}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(inp, target_s=12.0):
    """Time the oracle (append + attention) on the first S sequences of the workload."""
    import numpy as np
    import torch
    from oracle import gh_oracle as O
    from paper_2501_11779_amd import workloads as W

    w = inp["workload"]
    B = w.batch

    def run(S):
        slots = torch.from_numpy(inp["slots"][:S].astype(np.int64)).to(inp["k_cache"].device)
        kc = W.bits(inp["k_cache"].index_select(0, slots))
        vc = W.bits(inp["v_cache"].index_select(0, slots))
        q, kn, vn = W.bits(inp["q"][:S]), W.bits(inp["k_new"][:S]), W.bits(inp["v_new"][:S])
        strides = W.cache_shape_and_strides(S, w.n_kv_heads, inp["capacity"], w.head_dim,
                                            inp["layout"])[1]
        p = O.make_problem(S, w.n_q_heads, w.n_kv_heads, w.head_dim, W.DTYPE_CODE[w.dtype], S,
                           inp["capacity"], inp["scale"], strides)
        sid = np.arange(S, dtype=np.int32)
        pos = inp["lengths"][:S].astype(np.int32)
        t0 = time.perf_counter()
        O.kv_append(p, kc, vc, kn, vn, sid, pos)
        O.decode_attention(p, q, kc, vc, sid, pos + 1)
        return time.perf_counter() - t0

    S0 = min(B, 16)                      # one sequence per host thread: a fair rate estimate
    t_probe = run(S0)
    S = int(max(S0, min(B, round(S0 * target_s / max(t_probe, 1e-6)))))
    S = min(S, 512)
    t = run(S)
    return {"value": S / t, "unit": "sequence-steps/s", "cores": O.num_threads(), "kind": "oracle",
            "sample": f"first {S} of {B} sequences of the same workload (float64 append + attention, "
                      f"{t:.2f} s)"}


def one_thread_oracle(names=("c1", "c2")):
    """The oracle on ONE host thread over the whole of the small workloads, for scale."""
    import numpy as np
    from oracle import gh_oracle as O
    from paper_2501_11779_amd import workloads as W

    out = {}
    threads = O.num_threads()
    O.set_num_threads(1)
    try:
        for name in names:
            w = W.WORKLOADS[name]
            inp = W.make_inputs(w, "cpu")
            kc, vc = W.bits(inp["k_cache"]), W.bits(inp["v_cache"])
            p = O.make_problem(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, W.DTYPE_CODE[w.dtype],
                               inp["n_slots"], inp["capacity"], inp["scale"], inp["strides"])
            sid, pos = inp["slots"].astype(np.int32), inp["lengths"].astype(np.int32)
            t0 = time.perf_counter()
            O.kv_append(p, kc, vc, W.bits(inp["k_new"]), W.bits(inp["v_new"]), sid, pos)
            O.decode_attention(p, W.bits(inp["q"]), kc, vc, sid, pos + 1)
            t = time.perf_counter() - t0
            out[name] = {"value": w.batch / t, "unit": "sequence-steps/s", "cores": 1,
                         "sample": f"all {w.batch} sequences, {t:.2f} s"}
    finally:
        O.set_num_threads(threads)
    return out


def time_default_step(name, steps, warmup, keep):
    """Append + attention + merge of workload `name` in the library's default launch, timed like
    the headline workload (wall clock for the step, HIP events on the launch stream per kernel).
    The tensors are appended to `keep`: a later workload placed in memory that an earlier one gave
    back runs 2-3% slower than in memory the process takes for the first time."""
    import numpy as np
    import torch
    from paper_2501_11779_amd import binding as G
    from paper_2501_11779_amd import workloads as W

    w = W.WORKLOADS[name]
    inp = W.make_inputs(w, "cuda")
    p = G.problem_from_inputs(inp)
    ws = G.alloc_workspace(p)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), device="cuda", dtype=torch.float32)
    keep.append((inp, ws, out))
    ctx = inp["lengths"].astype(np.int64) + 1
    attn_bytes = W.attention_bytes(w, ctx)

    def step(ev=None):
        G.check(G.gh_kv_append(p, inp["k_cache"], inp["v_cache"], inp["k_new"], inp["v_new"],
                               inp["slot_id"], inp["pos"], None))
        if ev is not None:
            ev[0].record()
        G.check(G.gh_decode_attention_out(p, inp["q"], inp["k_cache"], inp["v_cache"], inp["slot_id"],
                                          inp["ctx_len"], ws, out, G.GH_OUT_F32))
        if ev is not None:
            ev[1].record()
        G.check(G.gh_decode_reduce(p, ws, inp["ctx_len"], out))
        if ev is not None:
            ev[2].record()

    for _ in range(warmup):
        step()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(evs[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    attn_ms = np.array([e[0].elapsed_time(e[1]) for e in evs])
    red_ms = np.array([e[1].elapsed_time(e[2]) for e in evs])
    achieved = attn_bytes / (float(attn_ms.mean()) * 1e-3) / 1e9
    traffic, _ = measured_traffic(name)
    res = {"workload": f"{CONFIG_OF[name]}: B={w.batch}, H={w.n_q_heads}, H_kv={w.n_kv_heads}, "
                       f"{w.dtype}, lengths={list(w.lengths)}, seed={w.seed}",
           "steps": steps, "warmup": warmup, "ms_per_step": elapsed / steps * 1e3,
           "sequence_steps_per_s": w.batch * steps / elapsed,
           "attention_ms_mean": float(attn_ms.mean()), "attention_ms_median": float(np.median(attn_ms)),
           "attention_ms_min": float(attn_ms.min()), "reduce_ms": float(red_ms.mean()),
           "algorithmic_bytes_per_launch": attn_bytes, "attention_GBps": achieved,
           "frac": achieved / HBM_PEAK_GBS, "traffic": traffic}
    log(f"{name}: step {res['ms_per_step']:.4f} ms | attention mean {attn_ms.mean():.4f} median "
        f"{np.median(attn_ms):.4f} min {attn_ms.min():.4f} ms = {achieved:.0f} GB/s = "
        f"{res['frac'] * 100:.1f}% | reduce {red_ms.mean():.4f} ms")
    del inp, ws, out
    torch.cuda.empty_cache()
    return res


def ceiling(args):
    """Rate of the streaming-read probe over 8 GiB: 2048 waves (two per SIMD), and reads only
    with 1024 (one per SIMD, the attention kernel's grid)."""
    import torch
    from paper_2501_11779_amd import binding as G

    n_waves, nbytes = 2048, 8 << 30
    src = torch.ones(nbytes // 4, dtype=torch.int32, device="cuda")
    rec = torch.empty(n_waves * 1024, dtype=torch.int32, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    tiles_per_wave = nbytes // (n_waves * 16384)
    rows = {}
    cases = [("reads only", 0, 0, n_waves), ("reads only, one wave per SIMD", 0, 0, n_waves // 2)]
    for every in (64, 16):           # a 4 KiB store per 1 MiB / 256 KiB read by a wave
        for name, pol in (("plain", G.GH_PROBE_STORE_PLAIN), ("non-temporal", G.GH_PROBE_STORE_NT),
                          ("write-through", G.GH_PROBE_STORE_WRITE_THROUGH)):
            cases.append((f"4 KiB {name} store per {every} tiles", every, pol, n_waves))
    for label, every, pol, waves in cases:
        def run():
            G.check(G.gh_probe_stream_read(src, nbytes, waves, every, pol, rec, sink))
        for _ in range(args.warmup):
            run()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        torch.cuda.synchronize()
        ev[0].record()
        for _ in range(args.steps):
            run()
        ev[1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[1]) / args.steps
        rows[label] = {"ms": ms, "GBps": nbytes / ms / 1e6}
        log(f"stream probe, {label}: {ms:.4f} ms, {rows[label]['GBps']:.0f} GB/s = "
            f"{rows[label]['GBps'] / HBM_PEAK_GBS * 100:.1f}% of {HBM_PEAK_GBS:.0f}")
    print(json.dumps({"metric": "streaming-read probe (measurement aid, not the hot path)",
                      "value": rows["reads only"]["GBps"], "unit": "GB/s", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup,
                      "config": {"workload": f"8 GiB read once by {n_waves} waves, {tiles_per_wave} "
                                             f"tiles of 16 KiB each", "cases": rows}}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c4", choices=sorted(CONFIG_OF))
    ap.add_argument("--kernel", default="auto", choices=["auto", "valu", "mfma", "strips"],
                    help="strips: with --one-launch, a workgroup per strip (GH_KERNEL_STRIPS)")
    ap.add_argument("--chunk-rows", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--batch", type=int, default=0, help="experiment: override the batch size")
    ap.add_argument("--const-len", type=int, default=0,
                    help="experiment: every sequence has this many cached rows")
    ap.add_argument("--capacity", type=int, default=0,
                    help="experiment: rows per cache slot (default: longest context + 1)")
    ap.add_argument("--mixed", type=int, default=0, metavar="T",
                    help="experiment: the last 2*T batch entries become two prefill chunks of T "
                         "tokens each (entries sharing a slot with consecutive positions)")
    ap.add_argument("--prefill", type=int, default=0, metavar="T",
                    help="experiment: the whole batch is B/T prefill chunks of T tokens each, every "
                         "chunk on its own slot behind the cached rows the workload draws")
    ap.add_argument("--group", type=int, default=0, metavar="T",
                    help="experiment: declare tokens_per_group = T (rows kT..kT+T-1 share a slot); "
                         "the GB/s printed then counts every row's K/V as if read separately")
    ap.add_argument("--out16", action="store_true",
                    help="experiment: the merge stores the model's 16-bit type (gh_decode_reduce_native)")
    ap.add_argument("--records-only", action="store_true",
                    help="gh_decode_attention instead of gh_decode_attention_out: every strip writes "
                         "partial records, also where one worker covered it alone and could store "
                         "the final rows (the default step stores those directly)")
    ap.add_argument("--one-launch", action="store_true",
                    help="time the step as one gh_decode_step launch (append + attention + merge "
                         "fused) instead of gh_kv_append + gh_decode_attention + gh_decode_reduce")
    ap.add_argument("--paged", action="store_true",
                    help="keep the caches in a gh_slot_pool (virtual slots, pages mapped on demand)")
    ap.add_argument("--page-rows", type=int, default=1024)
    ap.add_argument("--paged-layout", choices=["token_major", "head_blocked"], default="token_major",
                    help="order of a page's rows: [row][kv head] or [kv head][row]")
    ap.add_argument("--virtual-capacity", type=int, default=0,
                    help="rows per virtual slot in --paged mode (default: 3x the mean context)")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step replayed from a HIP graph (one step per graph); the "
                         "JSON line keeps the eager figures and adds config.hip_graph_ms_per_step")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy, the known-size kernel that "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per attention launch from rocprofv3 counters, if measured")
    ap.add_argument("--ceiling", action="store_true",
                    help="measurement aid instead of the step: the streaming-read probe of "
                         "include/gh_probe.h (pure reads in the attention kernel's access shape, "
                         "alone and with record-sized stores in each store policy)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short timings of the other full-size workloads that the default "
                         "run adds under config.other_workloads")
    ap.add_argument("--other-steps", type=int, default=30)
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path shards by sequence, with no "
                 "exchange step between shards, but no multi-GPU launcher is part of it); "
                 "run with --gpus 1")

    import numpy as np
    import torch
    from paper_2501_11779_amd import binding as G
    from paper_2501_11779_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    G.lib()
    props = torch.cuda.get_device_properties(0)
    log(f"device: {props.name} CUs={props.multi_processor_count} "
        f"mem={props.total_memory / 2**30:.0f} GiB host_cpus={os.cpu_count()}")

    if args.ceiling:
        return ceiling(args)
    w = W.WORKLOADS[args.workload]
    if args.batch or args.const_len:
        import dataclasses
        w = dataclasses.replace(
            w, batch=args.batch or w.batch,
            lengths=("const", args.const_len) if args.const_len else w.lengths,
            note=w.note + " [EXPERIMENT: overridden batch/lengths]")
    t0 = time.perf_counter()
    lengths = slots = None
    if args.mixed:
        T = args.mixed
        assert 2 * T < w.batch
        lengths = W.draw_lengths(w).copy()
        slots = W.draw_slots(w, w.batch).copy()
        for i, base in enumerate((1024, 3000)):            # cached rows of the two prompts
            first = w.batch - (2 - i) * T
            lengths[first:first + T] = base + np.arange(T)
            slots[first:first + T] = slots[first]
        import dataclasses
        w = dataclasses.replace(w, note=w.note + f" [EXPERIMENT: two {T}-token prefill chunks]")
    if args.prefill:
        T = args.prefill
        assert w.batch % T == 0 and not args.mixed
        base = W.draw_lengths(w)[: w.batch // T]
        lengths = (np.repeat(base, T) + np.tile(np.arange(T), w.batch // T)).astype(np.int32)
        slots = np.repeat(W.draw_slots(w, w.batch)[: w.batch // T], T)
        import dataclasses
        w = dataclasses.replace(w, note=w.note + f" [EXPERIMENT: {w.batch // T} prefill chunks of "
                                                 f"{T} tokens, tokens_per_group={args.group}]")
    inp = W.make_inputs(w, "cuda", capacity=args.capacity or None, lengths=lengths, slots=slots,
                        layout="token_major" if args.paged else "head_major")
    torch.cuda.synchronize()
    pool = None
    paged_info = None
    cpu = None
    if args.paged:
        if not args.no_cpu_baseline:
            cpu = cpu_baseline(inp)          # needs the generated tensors, which the pool replaces
        from paper_2501_11779_amd.paged import into_pool, pages_needed
        need = pages_needed(inp["lengths"], args.page_rows)
        vcap = args.virtual_capacity or max(int(inp["lengths"].max()) + 1,
                                            int(3 * need * args.page_rows / w.batch))
        pool = G.SlotPool(inp["n_slots"], vcap, w.n_kv_heads, w.head_dim, args.page_rows, need,
                          layout=args.paged_layout)
        inp = into_pool(pool, inp, poison=False)
        st = pool.stats()
        paged_info = {"page_rows": args.page_rows, "page_bytes": st.page_bytes,
                      "virtual_GB": st.virtual_bytes / 1e9, "physical_GB": st.physical_bytes / 1e9,
                      "oversubscription": st.virtual_bytes / st.physical_bytes,
                      "layout": args.paged_layout + ", HIP virtual memory"}
        log(f"paged slots: {paged_info}")
    kernel = {"auto": G.GH_KERNEL_AUTO, "valu": G.GH_KERNEL_VALU, "mfma": G.GH_KERNEL_MFMA,
              "strips": G.GH_KERNEL_STRIPS}[args.kernel]
    p = G.problem_from_inputs(inp, chunk_rows=args.chunk_rows, kernel=kernel,
                              tokens_per_group=args.group)
    ws = G.alloc_workspace(p)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), device="cuda",
                      dtype=W.TORCH_DTYPE[w.dtype] if args.out16 else torch.float32)
    reduce = G.gh_decode_reduce_native if args.out16 else G.gh_decode_reduce
    ctx = inp["lengths"].astype(np.int64) + 1
    step_bytes = W.algorithmic_bytes(w, ctx)
    attn_bytes = W.attention_bytes(w, ctx)
    flops = W.algorithmic_flops(w, ctx)
    if args.group > 1:
        # a declared group streams its slot once (the rows of its longest token): K/V rows count
        # once per group, q once per entry
        row_bytes = 2 * w.n_kv_heads * w.head_dim * W.ELEM_BYTES
        saved = int((ctx.sum() - ctx.reshape(-1, args.group).max(axis=1).sum()) * row_bytes)
        attn_bytes -= saved
        step_bytes -= saved
    chunk_rows, n_chunks = G.gh_decode_chunk_rows(p), G.gh_decode_num_chunks(p)
    log(f"workload {w.name}: B={w.batch} H={w.n_q_heads}/{w.n_kv_heads} d={w.head_dim} {w.dtype} "
        f"sum(n_b)={int(ctx.sum())} step_bytes={step_bytes / 1e9:.3f} GB "
        f"attn_bytes={attn_bytes / 1e9:.3f} GB chunk_rows={chunk_rows} n_chunks={n_chunks} "
        f"workspace={ws.numel() * 4 / 1e6:.1f} MB setup={time.perf_counter() - t0:.1f} s")

    # gh_decode_step does not take batches whose entries share a slot (prefill chunks).
    one_launch = args.one_launch
    assert not (one_launch and (args.mixed or args.prefill or args.group))
    early = not args.records_only
    if one_launch:
        G.check(G.gh_decode_step_init(p, ws))

    def step(events=None):
        if one_launch:
            if events is not None:
                events[0].record()
            G.check(G.gh_decode_step(p, inp["q"], inp["k_new"], inp["v_new"], inp["k_cache"],
                                     inp["v_cache"], inp["slot_id"], inp["pos"], ws, out,
                                     G.GH_OUT_NATIVE if args.out16 else G.GH_OUT_F32))
            if events is not None:
                events[1].record()
                events[2].record()
            return
        G.check(G.gh_kv_append(p, inp["k_cache"], inp["v_cache"], inp["k_new"], inp["v_new"],
                               inp["slot_id"], inp["pos"], None))
        if events is not None:
            events[0].record()
        if early:
            G.check(G.gh_decode_attention_out(p, inp["q"], inp["k_cache"], inp["v_cache"],
                                              inp["slot_id"], inp["ctx_len"], ws, out,
                                              G.GH_OUT_NATIVE if args.out16 else G.GH_OUT_F32))
        else:
            G.check(G.gh_decode_attention(p, inp["q"], inp["k_cache"], inp["v_cache"], inp["slot_id"],
                                          inp["ctx_len"], ws))
        if events is not None:
            events[1].record()
        G.check(reduce(p, ws, inp["ctx_len"], out))
        if events is not None:
            events[2].record()

    if args.pmc_calibration:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    attn_ms = np.array([e[0].elapsed_time(e[1]) for e in evs])
    red_ms = np.array([e[1].elapsed_time(e[2]) for e in evs])
    ms_per_step = elapsed / args.steps * 1e3
    attn_avg_s = float(attn_ms.mean()) * 1e-3
    # the one-launch kernel does the whole sequence-step: its algorithmic bytes are the step's
    # (K/V rows, q, the result, the appended rows in and out), not the attention's alone
    kernel_bytes = step_bytes if one_launch else attn_bytes
    achieved = kernel_bytes / attn_avg_s / 1e9
    log(f"step {ms_per_step:.4f} ms | {'step kernel' if one_launch else 'attention'} mean {attn_ms.mean():.4f} ms median "
        f"{np.median(attn_ms):.4f} min {attn_ms.min():.4f} | reduce mean {red_ms.mean():.4f} ms | "
        f"attention {achieved:.0f} GB/s = {achieved / HBM_PEAK_GBS * 100:.1f}% of {HBM_PEAK_GBS:.0f} | "
        f"whole step {step_bytes / (elapsed / args.steps) / 1e9:.0f} GB/s | "
        f"{flops / attn_avg_s / 1e12:.1f} TFLOP/s algorithmic")

    graph_ms = None
    if args.graph:
        # the three calls only launch kernels (no allocation, no memset, nothing read back), so a
        # step is captured as it is; lengths and slots stay device arrays the replay re-reads
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        for _ in range(args.warmup):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) / args.steps * 1e3
        log(f"HIP graph replay: {graph_ms:.4f} ms per step (eager {ms_per_step:.4f})")

    plain = args.kernel == "auto" and not (
        args.one_launch or args.chunk_rows or args.batch or args.const_len or args.capacity or args.paged or args.mixed
        or args.prefill or args.group or args.out16 or args.records_only)
    traffic, traffic_source = (args.traffic_bytes, "command line") if args.traffic_bytes is not None \
        else measured_traffic(w.name) if plain else (None, None)
    result = {
        "metric": "decode-attention sequence-steps/sec (achieved HBM GB/s and % of peak under roofline)",
        "value": w.batch * args.steps / elapsed,
        "unit": "sequence-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{CONFIG_OF[w.name]} ({w.note}): B={w.batch}, H={w.n_q_heads}, "
                               f"H_kv={w.n_kv_heads}, d={w.head_dim}, lengths={list(w.lengths)}, "
                               f"seed={w.seed}",
                   "kernel": args.kernel, "chunk_rows": chunk_rows, "n_chunks": n_chunks,
                   "step": ("gh_decode_step (append + attention + merge in one launch)" if one_launch
                            else "gh_kv_append + gh_decode_attention" + ("_out" if early else "")
                            + " + " + ("gh_decode_reduce_native" if args.out16 else "gh_decode_reduce")),
                   "paged_slots": paged_info, "hip_graph_ms_per_step": graph_ms,
                   "step_algorithmic_bytes": step_bytes,
                   "step_GBps": step_bytes / (elapsed / args.steps) / 1e9,
                   "attention_ms_mean": float(attn_ms.mean()),
                   "attention_ms_median": float(np.median(attn_ms)),
                   "attention_ms_min": float(attn_ms.min()),
                   "reduce_ms": float(red_ms.mean())},
        "roofline": {"bound": "hbm", "kernel": "gh_decode_step" if one_launch else
                     "gh_decode_attention_out" if early else "gh_decode_attention",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes_per_launch": kernel_bytes,
                     "avg_launch_ms": float(attn_ms.mean())},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu if cpu is not None else cpu_baseline(inp)
        log(f"cpu_baseline: {result['cpu_baseline']}")
        result["cpu_baseline"]["one_thread"] = one_thread_oracle()
        log(f"one-thread oracle: {result['cpu_baseline']['one_thread']}")
    if plain and w.name == "c4" and not args.no_other_workloads:
        # the other full-size workloads of the target, each for a few steps in the same launch
        # configuration, so that one run's record covers them all
        # (the headline workload's tensors stay allocated: memory handed back to the driver and
        # taken again comes in smaller physical pieces, and the kernels then run 2-3% slower)
        keep = []
        result["config"]["other_workloads"] = {
            name: time_default_step(name, args.other_steps, 10, keep) for name in ("c3", "c5", "c2", "c1")}
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
