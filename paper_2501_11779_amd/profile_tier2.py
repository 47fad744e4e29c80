"""Measure the Tier-2 curve the configuration search needs: time of one layer's attention step
(the fastest of gh_kv_append + gh_decode_attention + gh_decode_reduce, gh_decode_step, and
gh_decode_step with a workgroup per strip) against batch size, every context at the
maximum sequence length (Appendix C: kernels are profiled at batch sizes about sqrt(2) apart and
the attention time is taken at full sequence length).  Needs an MI355X.

    python -m paper_2501_11779_amd.profile_tier2 [--seq-len 2048] [--heads 64] [--kv-heads 8]
                                                 [--out paper_2501_11779_amd/data/<name>.json]
"""
import argparse
import json
import os
import sys

import numpy as np
import torch

from . import binding as G
from . import workloads as W
from .config_search import profile_batch_sizes


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--seq-len", type=int, default=2048)
    ap.add_argument("--heads", type=int, default=64)
    ap.add_argument("--kv-heads", type=int, default=8)
    ap.add_argument("--dtype", default="bf16")
    ap.add_argument("--max-batch", type=int, default=4096)
    ap.add_argument("--repeats", type=int, default=15)
    ap.add_argument("--out", default=os.path.join(os.path.dirname(os.path.abspath(__file__)), "data",
                                                  "tier2_mi355x_llama2_70b.json"))
    args = ap.parse_args()
    assert torch.cuda.is_available(), "needs a GPU"
    G.lib()
    S, H, Hkv, Bmax = args.seq_len, args.heads, args.kv_heads, args.max_batch
    w = W.Workload("profile", Bmax, H, Hkv, 128, args.dtype, ("const", S - 1), 4242)
    inp = W.make_inputs(w, "cuda", poison=False)
    batches, seconds, how = [], [], []
    per_variant = {"three_launches": [], "one_launch": [], "one_launch_strips": []}
    for B in profile_batch_sizes(Bmax):
        dt = G.GH_BF16 if args.dtype == "bf16" else G.GH_F16
        sub = dict(inp)
        for key in ("q", "k_new", "v_new", "slot_id", "pos", "ctx_len"):
            sub[key] = inp[key][:B].contiguous()
        out = torch.empty((B, H, 128), dtype=torch.float32, device="cuda")

        def timed(run):
            for _ in range(3):
                run()
            torch.cuda.synchronize()
            times = []
            for _ in range(args.repeats):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                run()
                e1.record()
                torch.cuda.synchronize()
                times.append(e0.elapsed_time(e1) * 1e-3)
            return float(np.median(times))

        # the step three ways: the three calls, one launch with the library's split, and one launch
        # with a workgroup per strip (every context has the same length here, its best case)
        p = G.make_problem(B, H, Hkv, 128, dt, inp["n_slots"], inp["capacity"], S, inp["strides"],
                           inp["scale"])
        ws = G.alloc_step_workspace(p)
        t3 = timed(lambda: G.decode_step(p, sub, ws, out))
        t1 = timed(lambda: G.decode_step_one_launch(p, sub, ws, out))
        ps = G.make_problem(B, H, Hkv, 128, dt, inp["n_slots"], inp["capacity"], S, inp["strides"],
                            inp["scale"], kernel=G.GH_KERNEL_STRIPS)
        ts = timed(lambda: G.decode_step_one_launch(ps, sub, ws, out))
        for name, t in (("three_launches", t3), ("one_launch", t1), ("one_launch_strips", ts)):
            per_variant[name].append(t)
        t, name = min((t3, "three_launches"), (t1, "one_launch"), (ts, "one_launch_strips"))
        batches.append(B)
        seconds.append(t)
        how.append(name)
        print(f"B={B:5d}  three launches {t3 * 1e6:8.1f} us  one launch {t1 * 1e6:8.1f} us  strips "
              f"{ts * 1e6:8.1f} us  -> {B / t:12.0f} sequence-steps/s ({name})", file=sys.stderr, flush=True)
    doc = {"what": "one layer's attention step on one MI355X, every context at seq_len rows",
           "seq_len": S, "n_q_heads": H, "n_kv_heads": Hkv, "head_dim": 128, "dtype": args.dtype,
           "batch": batches, "seconds": seconds, "fastest": how, "seconds_by_variant": per_variant}
    with open(args.out, "w") as f:
        json.dump(doc, f, indent=1)
    print(args.out)


if __name__ == "__main__":
    main()
