"""Benchmark of the Cerberus verify step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 7b|13b|tiny] [--no-graph] [--no-cpu]
                    [--ar] [--batch B [--mixed]] [--prefix L] [--tree p63|p120|p150] [--medusa-heads]
                    [--param name=value]

A step is one full pass of the hot path over one batch: tree assembly, 32 decoder layers over the
64-node tree with tree-masked attention against a 1024-row KV prefix, LM head and per-node argmax,
acceptance, KV compaction, entropy gate, Cerberus heads and top-k (gate forced to the parallel path,
so the heads always run).  Weights, KV prefix and candidates are synthetic (seeded, random-init) and
resident in HBM before the timed region.  Prints ONE JSON line.  The default is the headline
configuration; --ar (plain auto-regressive step), --batch/--mixed, --workload 13b and --medusa-heads
time the secondary configurations with the same contract.
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

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
GEMM_KINDS = ["qkv", "attn_out", "ffn_gate_up", "ffn_down", "lm_head", "head_resblocks", "head_fc"]


def algorithmic_bytes(cfg: dict, T: int, L: int, elem: int = 2) -> dict:
    """Bytes one step must move when every weight and every live KV row is read once."""
    d, F, V, NL, Hc = cfg["d_model"], cfg["d_ffn"], cfg["vocab"], cfg["n_layers"], cfg["n_cerb_heads"]
    from paper_2410_13344_amd import synth
    layer_w = (3 * d * d + d * d + 2 * F * d + d * F) * elem
    heads = 0
    for i, widths in enumerate(synth.head_block_widths(cfg)):
        heads += sum(w * w + w for w in widths) * elem + V * widths[-1] * elem
    out = {
        "layer_weights": NL * layer_w,
        "lm_head": V * d * elem,
        "kv_prefix_read": NL * 2 * L * d * elem,
        "tree_kv_write_read": NL * 2 * T * d * elem * 2,
        "heads": heads,
        "embedding_rows": T * d * elem,
    }
    out["total"] = sum(out.values())
    return out


def cpu_baseline(cfg: dict, W_dev: dict, parent, rank, L: int, cap: int, reps: int = 2) -> dict:
    """Times the CPU oracle, as it stands, on the same workload: `reps` whole steps (all layers, all
    tree nodes, LM head, gate, heads, top-k) from the same seeded weights and KV prefix."""
    import numpy as np
    import torch
    from oracle import cerberus_oracle as orc
    from paper_2410_13344_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1

    W = synth.to_host_f32(W_dev)
    kv_t = synth.make_kv_prefix(cfg, 1, cap, seed=0, dtype=torch.bfloat16, device="cuda")
    kv = [(kv_t[l, 0, 0].double().cpu().numpy(), kv_t[l, 1, 0].double().cpu().numpy()) for l in range(cfg["n_layers"])]
    del kv_t
    root = int(synth.make_token_ids(1, cfg["vocab"], seed=2)[0])
    cand = synth.make_candidates(cfg, 1, seed=3)[0].numpy()
    times = []
    for _ in range(reps):
        st = orc.new_state(kv, L, root, cand, 0)      # rows >= L are rewritten by every step
        t0 = time.perf_counter()
        orc.verify_step(cfg, W, parent, rank, st)
        times.append(time.perf_counter() - t0)
    return {"value": round(float(np.mean(times)) * 1e6, 1), "unit": "us/step", "cores": int(threads), "kind": "oracle",
            "sample": f"{reps} whole verify steps of this workload (every layer and tree node, LM head, gate, heads, "
                      f"top-k), mean of {', '.join(f'{t:.2f}' for t in times)} s",
            "measured_s": round(float(np.sum(times)), 3)}


def profiled_traffic_mb():
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, scaled by the calibration copy), or None when no summary is there."""
    path = os.path.join(ROOT, "profiles", "verify_step_7b_t64_l1024.txt")
    try:
        for line in open(path):
            if line.startswith("average over all launches: fetch"):
                parts = line.split()
                return float(parts[5]) + float(parts[8])
    except (OSError, ValueError, IndexError):
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="7b", choices=["7b", "13b", "tiny"])
    ap.add_argument("--prefix", type=int, default=None)
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--param", action="append", default=[], help="library tuning knob name=value")
    ap.add_argument("--prefill", type=int, default=0, metavar="N",
                    help="time the prompt phase (cerberus_prefill) of N tokens from an empty cache; value is per pass of "
                         "up to CERBERUS_MAX_TREE rows")
    ap.add_argument("--decode", type=int, default=0, metavar="N",
                    help="time N chained steps per call (cerberus_decode: device-side gate, token log); value is per step")
    ap.add_argument("--tree", default=None, help="candidate tree: p63 (default, 64 nodes), p120 or p150 (top-10 per head)")
    ap.add_argument("--medusa-heads", action="store_true",
                    help="independent d-wide heads (special_block = -1) instead of the linked Cerberus heads")
    ap.add_argument("--ar", action="store_true", help="time the plain auto-regressive step (tree of size 1, no heads)")
    ap.add_argument("--gate-threshold", type=float, default=None,
                    help="entropy threshold of the gate (default +inf: the gate always says parallel, so the heads run "
                         "after every step; -1: it always says auto-regressive and the heads are skipped)")
    ap.add_argument("--ar-direct", action="store_true",
                    help="with --ar: call cerberus_ar_step (launches sized for one row per sequence) instead of "
                         "reaching the step through the gate flag of cerberus_verify_step")
    ap.add_argument("--batch", type=int, default=1, help="sequences per launch (prefix lengths spread over [prefix/2, prefix])")
    ap.add_argument("--mixed", action="store_true", help="with --batch: every third sequence takes the auto-regressive step")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference dispatch for scaling profiler byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the path has no inter-GPU part); run with --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2410_13344_amd import binding as B
    from paper_2410_13344_amd import synth

    if not os.path.exists(B.LIB_PATH):
        from paper_2410_13344_amd.build import build_library
        build_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)

    name = args.workload
    over = {"special_block": -1} if args.medusa_heads else {}
    tree_name = args.tree or ("tiny" if name == "tiny" else "p63")
    if tree_name in ("p120", "p150"):
        over["topk"] = 10                              # Section 5.1: top-10 predictions per head for the larger trees
    if args.gate_threshold is not None:
        over["entropy_threshold"] = args.gate_threshold
    cfg = synth.make_config(name, **over)              # entropy_threshold = +inf unless given: gate forced parallel
    L = args.prefix if args.prefix is not None else {"7b": 1024, "13b": 2048, "tiny": 128}[name]
    parent, rank = synth.make_tree(tree_name, cfg["n_cerb_heads"])
    T = len(parent)
    Bn = args.batch
    assert 1 <= Bn <= 16
    Ls = [L] if Bn == 1 else [int(round(L / 2 + (L - L / 2) * b / (Bn - 1))) for b in range(Bn)]
    flags = [1 if (args.ar or (args.mixed and b % 3 == 2)) else 0 for b in range(Bn)]
    cap = ((max(Ls) + T + max(args.decode, 1) * (cfg["n_cerb_heads"] + 1) + 127) // 128 + 1) * 128
    if args.prefill:
        cap = ((args.prefill + T + 127) // 128 + 1) * 128
    dtype = B.CERBERUS_BF16
    W = synth.make_weights(cfg, seed=0, dtype=torch.bfloat16, device="cuda")
    eng = B.Engine(cfg, W, parent, rank, dtype, Bn, cap)
    for kv in args.param:
        k, v = kv.split("=")
        eng.set_param(k, int(v))
    st = eng.new_state()
    st.kv.copy_(synth.make_kv_prefix(cfg, Bn, cap, seed=0, dtype=torch.bfloat16, device="cuda"))
    st.root_token.copy_(synth.make_token_ids(Bn, cfg["vocab"], seed=2).to(torch.int32).cuda())
    st.cand.copy_(synth.make_candidates(cfg, Bn, seed=3).cuda())
    flag_dev = torch.tensor(flags, dtype=torch.int32, device="cuda")
    L_dev = torch.tensor(Ls, dtype=torch.int32, device="cuda")

    log_tokens = torch.zeros((Bn, max(args.decode, 1) * (cfg["n_cerb_heads"] + 1)), dtype=torch.int32, device="cuda")
    log_count = torch.zeros(Bn, dtype=torch.int32, device="cuda")
    per_call = max(args.decode, 1)
    if args.prefill:
        prompt_dev = synth.make_token_ids(args.prefill, cfg["vocab"], seed=4).cuda()
        per_call = (args.prefill + B.CERBERUS_MAX_TREE - 1) // B.CERBERUS_MAX_TREE          # passes per call

    def step():
        st.kv_len.copy_(L_dev)          # every repetition sees the configured prefix lengths ...
        st.gate_flag.copy_(flag_dev)    # ... and step kinds (the threshold is +inf, so the gate itself says parallel)
        if args.prefill:
            st.kv_len.zero_()
            eng.prefill(st, Bn, 0, prompt_dev)
        elif args.decode:
            log_count.zero_()
            eng.decode(st, Bn, args.decode, log_tokens, log_count)
        elif args.ar_direct:
            eng.ar_step(st, Bn)
        else:
            eng.verify_step(st, Bn)

    graph = None
    if not args.no_graph:
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            for _ in range(2):
                step()
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
    run = graph.replay if graph is not None else step

    if args.calib_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    accepted = 0
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) / (args.steps * per_call) * 1e3
    accepted = (args.prefill if args.prefill else int(log_count.sum()) if args.decode else int(st.accept_len[:Bn].sum())) * args.steps
    assert int(st.status[0]) == 0, "device status word set"

    # per-step distribution from events (separate pass)
    n_ev = min(args.steps, 50)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_ev)]
    for a, b in evs:
        a.record()
        run()
        b.record()
    torch.cuda.synchronize()
    lat = np.array([a.elapsed_time(b) for a, b in evs]) * 1e3 / per_call

    # dominant kernel: the weight-streaming GEMM.  Every kind is replayed back to back over all
    # layers (fresh weights each launch, so no cache reuse) between two events on this stream.
    gemm = {}
    tot_bytes = tot_ms = 0.0
    n_launch = 0
    for kind, kname in enumerate(GEMM_KINDS):
        rows = 1 if kind >= 5 else sum(1 if f else T for f in flags)
        reps = 3 if kind <= 3 else 20
        B.cerberus_bench_gemm(eng.ctx, kind, rows)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            nbytes = B.cerberus_bench_gemm(eng.ctx, kind, rows)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        launches = cfg["n_layers"] if kind <= 3 else (cfg["n_resblocks"] if kind == 5 else 1)
        gemm[kname] = {"ms_per_step": round(ms, 4), "launches": launches, "GB": round(nbytes / 1e9, 4),
                       "GBps": round(nbytes / ms / 1e6, 1), "us_per_launch": round(ms * 1e3 / launches, 2)}
        if kind <= 4:     # the MT=4 kernel instance (tree rows); head GEMMs run the 16-row instance
            tot_bytes += nbytes
            tot_ms += ms
            n_launch += launches
    achieved = tot_bytes / tot_ms / 1e6
    alg = algorithmic_bytes(cfg, T, L)
    if Bn > 1 or args.ar:               # weights once; KV rows and tree rows per sequence; heads only if some sequence runs them
        per = [algorithmic_bytes(cfg, 1 if f else T, l) for f, l in zip(flags, Ls)]
        alg = dict(per[0])
        for k in ("kv_prefix_read", "tree_kv_write_read", "embedding_rows"):
            alg[k] = sum(q[k] for q in per)
        if bool((st.gate_flag[:Bn] != 0).all()):   # the gate after the step sent every sequence down the one-token path
            alg["heads"] = 0
        alg["total"] = sum(v for k, v in alg.items() if k != "total")

    out = {
        "metric": "verify_step_latency", "value": round(ms_per_step * 1e3, 1), "unit": "us",
        "n_gpus": 1, "steps": args.steps * per_call, "warmup": args.warmup * per_call, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": (f"{name}-shape bf16, {T}-node tree, KV prefix {L}, batch 1, gate forced parallel"
                                + (", independent (Medusa-style) heads" if args.medusa_heads else "")
                                + (f", {args.decode} chained steps per call" if args.decode else "")
                                + (f"; prompt phase of {args.prefill} tokens from an empty cache, {per_call} passes per call, "
                                   "tokens_per_s = prompt tokens" if args.prefill else "")
                                if Bn == 1 and not args.ar else
                                f"{name}-shape bf16, batch {Bn}, KV prefixes {Ls}, step kinds (1 = auto-regressive) {flags}, "
                                f"{T}-node tree"),
                   "graph": graph is not None},
        "latency_us": {"p10": round(float(np.percentile(lat, 10)), 1), "p50": round(float(np.percentile(lat, 50)), 1),
                       "p90": round(float(np.percentile(lat, 90)), 1)},
        "tokens_per_s": round(accepted / (t1 - t0), 2),
        "step_algorithmic_GB": round(alg["total"] / 1e9, 4),
        "step_hbm_frac": round(alg["total"] / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9), 4),
        "roofline": {"bound": "hbm", "kernel": "k_gemm_bf16<4,2> (QKV, O, gate/up, down, LM head)",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": (profiled_traffic_mb() if name == "7b" and L == 1024 and Bn == 1 and T == 64 and not args.ar else None),
                     "traffic_unit": "MB per launch (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, profiles/)",
                     "algorithmic_MB_per_launch": round(tot_bytes / n_launch / 1e6, 1),
                     "avg_launch_us": round(tot_ms * 1e3 / n_launch, 2), "launches_per_step": n_launch,
                     "per_kind": gemm},
    }
    if not args.no_cpu and Bn == 1 and not args.ar:
        out["cpu_baseline"] = cpu_baseline(cfg, W, parent, rank, L, cap)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
