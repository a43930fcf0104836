"""Benchmark of the Cerberus verify step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 7b|13b|tiny] [--no-graph] [--no-cpu]
                    [--ar] [--batch B [--mixed]] [--prefix L] [--tree p63|p120|p150] [--medusa-heads]
                    [--schedule N] [--param name=value]

A step is one full pass of the hot path over one batch: tree assembly, 32 decoder layers over the
64-node tree with tree-masked attention against a 1024-row KV prefix, LM head and per-node argmax,
acceptance, KV compaction, entropy gate, Cerberus heads and top-k (gate forced to the parallel path,
so the heads always run).  Weights, KV prefix and candidates are synthetic (seeded, random-init) and
resident in HBM before the timed region.  Prints ONE JSON line.  The default is the headline
configuration; --ar (plain auto-regressive step), --batch/--mixed (seeded prefixes uniform in 512..4096,
step kinds Bernoulli(0.3)), --workload 13b, --medusa-heads and --schedule N (N consecutive steps with
the gate active: per step 30 % hand over to an auto-regressive step, accepted lengths uniform in 1..5)
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
MFMA_PEAK_TFLOPS = 2500.0      # MI355X published dense bf16 MFMA rate
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


def gemm_flops(cfg: dict, rows: int, head_rows: int) -> dict:
    """Multiply-add work of one step: 2*N*K per row of every layer GEMM and the LM head over `rows` tree
    rows; the decoding heads over `head_rows` rows (one per sequence whose gate said parallel)."""
    d, F, V, NL = cfg["d_model"], cfg["d_ffn"], cfg["vocab"], cfg["n_layers"]
    from paper_2410_13344_amd import synth
    layers = 2.0 * rows * NL * (3 * d * d + d * d + 2 * F * d + d * F)
    lm = 2.0 * rows * V * d
    heads = 0.0
    for widths in synth.head_block_widths(cfg):
        heads += 2.0 * head_rows * (sum(w * w for w in widths) + V * widths[-1])
    return {"layers": layers, "lm_head": lm, "heads": heads}


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


def _oracle_step_seconds(cfg, W, parent, rank, kv_t, b, L, root, cand, flag) -> float:
    """One oracle step of sequence b of a device cache tensor (rows 0..L-1 are the prefix)."""
    import numpy as np
    from oracle import cerberus_oracle as orc
    rows = L + len(parent) + 8
    kv = [(kv_t[l, 0, b, :, :rows].double().cpu().numpy(), kv_t[l, 1, b, :, :rows].double().cpu().numpy())
          for l in range(cfg["n_layers"])]
    st = orc.new_state(kv, L, root, cand, flag)
    t0 = time.perf_counter()
    orc.verify_step(cfg, W, parent, rank, st)
    return time.perf_counter() - t0


def _threads() -> int:
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] or [1]))
    except Exception:
        return os.cpu_count() or 1


def cpu_baseline_batch(cfg, W_dev, parent, rank, kv_t, Ls, flags, roots, cands) -> dict:
    """The oracle on a bounded sample of a batch launch: the first tree sequence and the first
    auto-regressive one, scaled to the batch's counts of each kind (sequences are independent)."""
    from paper_2410_13344_amd import synth
    W = synth.to_host_f32(W_dev)
    t_kind, n_kind = {}, {0: flags.count(0), 1: flags.count(1)}
    for kind in (0, 1):
        if n_kind[kind]:
            b = flags.index(kind)
            t_kind[kind] = _oracle_step_seconds(cfg, W, parent, rank, kv_t, b, Ls[b], int(roots[b]), cands[b].numpy(), kind)
    total = sum(t_kind[k] * n_kind[k] for k in t_kind)
    return {"value": round(total * 1e6, 1), "unit": "us/step", "cores": _threads(), "kind": "oracle",
            "sample": "one whole step of the first tree sequence (%s s) and of the first auto-regressive sequence (%s s), "
                      "scaled to the batch's %d tree and %d auto-regressive sequences" % (
                          "%.2f" % t_kind.get(0, 0.0), "%.2f" % t_kind.get(1, 0.0), n_kind[0], n_kind[1]),
            "measured_s": round(sum(t_kind.values()), 3)}


def cpu_baseline_schedule(cfg, W_dev, parent, rank, kv_t, L, root, cand, n_tree, n_ar, tokens) -> dict:
    """The oracle on a bounded sample of the gated schedule: two tree steps and two auto-regressive steps,
    extrapolated to the schedule's step counts."""
    from paper_2410_13344_amd import synth
    W = synth.to_host_f32(W_dev)
    tt = [_oracle_step_seconds(cfg, W, parent, rank, kv_t, 0, L, root, cand, 0) for _ in range(2)]
    ta = [_oracle_step_seconds(cfg, W, parent, rank, kv_t, 0, L, root, cand, 1) for _ in range(2)]
    total = n_tree * sum(tt) / 2 + n_ar * sum(ta) / 2
    return {"value": round(tokens / total, 3), "unit": "tokens/s", "cores": _threads(), "kind": "oracle",
            "sample": "2 tree steps (%.2f, %.2f s) and 2 auto-regressive steps (%.2f, %.2f s) at prefix %d, extrapolated to "
                      "the schedule's %d tree and %d auto-regressive steps (%.0f s)" % (tt[0], tt[1], ta[0], ta[1], L, n_tree, n_ar, total),
            "measured_s": round(sum(tt) + sum(ta), 3)}


def profiled_traffic_mb(kernel, summary):
    """HBM bytes per launch of `kernel` from a committed rocprofv3 --pmc summary under profiles/ (FETCH_SIZE +
    WRITE_SIZE, scaled by the calibration copy), or None when the summary has no line for it."""
    path = os.path.join(ROOT, "profiles", summary)
    try:
        for line in open(path):
            if line.startswith(f"traffic {kernel}:"):
                parts = line.split(":", 1)[1].split()
                return round(float(parts[1]) + float(parts[4]), 1)       # "fetch X MB, write Y MB per launch"
    except (OSError, ValueError, IndexError):
        pass
    return None


def run_schedule(args, cfg, eng, st, parent, rank, L0, W) -> dict:
    """configs[2]: n consecutive steps with the gate active.  Per step s: ar_s ~ Bernoulli(0.3) decides the
    forced gate input (0.5 z: ~11.8 bits > T = 9 -> the NEXT step is auto-regressive; 3 z: ~5.5 bits ->
    parallel) and a_s ~ U{1..5} is the accepted length planted in the forced per-node argmax (a random tree
    path of depth a_s - 1, a token no child carries at its end).  The node tokens the plant refers to are
    formed on the device from the state's own root and candidates just before the step (a few small
    torch kernels, outside the per-step events), so nothing crosses to the host between steps."""
    import numpy as np
    import torch
    from paper_2410_13344_amd import binding as B
    from paper_2410_13344_amd import synth
    n, T, Hc, V, d = args.schedule, len(parent), cfg["n_cerb_heads"], cfg["vocab"], cfg["d_model"]
    taps = B.DeviceTaps(cfg, 1, T, logits=False, forced_argmax=True, forced_gate=True)
    eng.set_taps(taps)
    rng = np.random.default_rng(11)
    depth = [0] * T
    for i in range(1, T):
        depth[i] = depth[parent[i]] + 1
    children = {i: [c for c in range(T) if parent[c] == i] for i in range(T)}
    z = synth.make_gate_states(n, d, seed=5, lo=1.0, hi=1.0)
    ar_next = rng.random(n) < 0.3
    gate_in = (torch.where(torch.from_numpy(ar_next)[:, None], 0.5, 3.0) * z).to(torch.float32).cuda()       # [n][d]
    is_ar = np.concatenate([[False], ar_next[:-1]])                    # the kind of step s is what step s-1's gate said
    # per step: path nodes (padded with -1) as device index tensors
    src = torch.zeros((n, Hc), dtype=torch.int64)                    # node whose token is wanted at path position j
    dst = torch.zeros((n, Hc), dtype=torch.int64)                    # node that gets it as its forced argmax
    end = torch.zeros(n, dtype=torch.int64)
    for s_ in range(n):
        a_want = int(rng.integers(1, Hc + 2))
        path = [0]
        while len(path) < a_want and not is_ar[s_] and children[path[-1]]:
            path.append(int(rng.choice(children[path[-1]])))
        for j in range(Hc):                                           # unused slots point at the path's end, which
            dst[s_, j] = path[j] if j + 1 < len(path) else path[-1]   # the sentinel overwrites afterwards
            src[s_, j] = path[j + 1] if j + 1 < len(path) else 0
        end[s_] = path[-1]
    src, dst, end = src.cuda(), dst.cuda(), end.cuda()
    dm1 = torch.tensor([max(depth[i] - 1, 0) for i in range(T)], dtype=torch.int64, device="cuda")
    rk = torch.tensor(list(rank), dtype=torch.int64, device="cuda")
    sentinel = torch.tensor([(1000 + s_) % V for s_ in range(n)], dtype=torch.int32, device="cuda")
    minus1 = torch.full((T,), -1, dtype=torch.int32, device="cuda")

    st.kv_len[0] = L0
    st.gate_flag[0] = 0
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    acc = torch.zeros(n, dtype=torch.int32, device="cuda")
    flags_seen = torch.zeros(n, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s_ in range(n):
        tok = st.cand[0][dm1, rk].to(torch.int32)                      # token of every node of the full tree
        tok[0] = st.root_token[0]
        forced = minus1.clone()
        forced[dst[s_]] = tok[src[s_]]
        forced[end[s_]] = sentinel[s_]
        taps.forced_node_argmax.copy_(forced)
        taps.forced_gate_hidden[0].copy_(gate_in[s_])
        flags_seen[s_] = st.gate_flag[0]
        evs[s_][0].record()
        eng.verify_step(st, 1)
        evs[s_][1].record()
        acc[s_] = st.accept_len[0]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    assert int(st.status[0]) == 0, "device status word set"
    lat = np.array([a.elapsed_time(b) for a, b in evs]) * 1e3          # us
    acc = acc.cpu().numpy()
    seen = flags_seen.cpu().numpy().astype(bool)
    assert np.array_equal(seen, is_ar), "the gate did not follow the schedule"
    tokens = int(acc.sum())

    def stats(v):
        return {"n": int(len(v)), "mean": round(float(np.mean(v)), 1), "p50": round(float(np.median(v)), 1),
                "p10": round(float(np.percentile(v, 10)), 1), "p90": round(float(np.percentile(v, 90)), 1)}
    out = {
        "metric": "verify_step_latency", "value": round(float(np.mean(lat)), 1), "unit": "us", "n_gpus": 1, "steps": n, "warmup": 0,
        "ms_per_step": round(float(np.mean(lat)) / 1e3, 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}-shape bf16, {T}-node tree, KV prefix {L0} growing to {int(st.kv_len[0])}, batch 1, gate "
                               f"active (threshold 9 bits): {n} consecutive steps, 30 % hand over to an auto-regressive step, planted "
                               "accepted lengths uniform in 1..5", "graph": False},
        "tree_steps_us": stats(lat[~is_ar]), "ar_steps_us": stats(lat[is_ar]),
        "accepted_tokens": tokens, "mean_accept_len": round(tokens / n, 3),
        "tokens_per_s": round(tokens / (float(lat.sum()) * 1e-6), 2),
        "tokens_per_s_wall": round(tokens / (t1 - t0), 2),
        "note": "tokens_per_s = accepted tokens / sum of the per-step device latencies (events around every step); "
                "tokens_per_s_wall includes the host loop and the small kernels that plant the schedule",
    }
    if not args.no_cpu:
        kv_t = synth.make_kv_prefix(cfg, 1, L0 + T + 16, seed=0, dtype=torch.bfloat16, device="cuda")
        out["cpu_baseline"] = cpu_baseline_schedule(cfg, W, parent, rank, kv_t, L0, int(synth.make_token_ids(1, V, seed=2)[0]),
                                                    synth.make_candidates(cfg, 1, seed=3)[0].numpy(), int((~is_ar).sum()),
                                                    int(is_ar.sum()), tokens)
    return out


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
    ap.add_argument("--batch", type=int, default=1,
                    help="sequences per launch; prefix lengths drawn uniformly from 512..prefix (default 4096), seed 21")
    ap.add_argument("--mixed", action="store_true",
                    help="with --batch: every sequence takes the auto-regressive step with probability 0.3 (same seed)")
    ap.add_argument("--schedule", type=int, default=0, metavar="N",
                    help="N consecutive steps with the gate active (threshold 9 bits): per step the gate's input is forced "
                         "so that 30 %% of the steps hand over to an auto-regressive step, and an accepted length drawn "
                         "uniformly from 1..5 is planted; reports tree and auto-regressive steps separately")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference dispatch for scaling profiler byte counters)")
    args = ap.parse_args()
    if args.ar_direct:
        args.ar = True          # same step kind, rows and byte count; only the entry point differs (launches sized for one row)
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
    Bn = args.batch
    assert 1 <= Bn <= 16
    L = args.prefix if args.prefix is not None else (4096 if Bn > 1 else {"7b": 1024, "13b": 2048, "tiny": 128}[name])
    parent, rank = synth.make_tree(tree_name, cfg["n_cerb_heads"])
    T = len(parent)
    if Bn == 1:
        Ls, flags = [L], [1 if args.ar else 0]
    else:   # seeded: prefixes uniform in 512..L, step kinds Bernoulli(0.3), at least one sequence of each kind
        rng_b = np.random.default_rng(21)
        Ls = [int(v) for v in rng_b.integers(min(512, L), L + 1, size=Bn)]
        flags = [int(v) for v in (rng_b.random(Bn) < 0.3)] if args.mixed else [0] * Bn
        if args.mixed:
            flags[0], flags[1] = 0, 1
        if args.ar:
            flags = [1] * Bn
    if args.schedule:
        assert Bn == 1 and not args.ar and not args.decode and not args.prefill
        over["entropy_threshold"] = 9.0
        cfg = synth.make_config(name, **over)
    cap = ((max(Ls) + T + max(args.decode, args.schedule, 1) * (cfg["n_cerb_heads"] + 1) + 127) // 128 + 1) * 128
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

    if args.schedule:
        print(json.dumps(run_schedule(args, cfg, eng, st, parent, rank, L, W)))
        return 0

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
        # the dominant kernel is the split-K GEMM instance for tree rows (O, down, LM head; also QKV and gate/up
        # where the step does not run those as whole-K fused launches); head GEMMs run the 16-row instance
        how = B.cerberus_bench_gemm(eng.ctx, 100 + kind, rows) if kind in (0, 2, 4) else 0.0   # 1: whole-K fused, 2 + NT: team kernel
        fused_kind = kind in (0, 2) and how == 1.0
        gemm[kname]["kernel"] = ("k_qkv_rope" if kind == 0 else "k_gate_up_swiglu") if fused_kind else "k_gemm_team<%d>" % int(how - 2) if how >= 2.0 else (
            "k_gemm_bf16<1,2,1,true>" if kind > 4 else "k_gemm_bf16_rows<1>" if rows > 256 and kind in (3, 4)
            else "k_gemm_bf16<4,2,1,%s>" % ("true" if rows <= 64 else "false"))
    # the roofline object covers the kernel of the layer stack that takes the most time in a step
    by_kernel = {}
    for kname in GEMM_KINDS[:5]:
        g = by_kernel.setdefault(gemm[kname]["kernel"], {"kinds": [], "ms_per_step": 0.0, "bytes": 0.0, "launches": 0})
        g["kinds"].append(kname)
        g["ms_per_step"] += gemm[kname]["ms_per_step"]
        g["bytes"] += gemm[kname]["GB"] * 1e9
        g["launches"] += gemm[kname]["launches"]
    for g in by_kernel.values():
        g["GBps"] = round(g["bytes"] / g["ms_per_step"] / 1e6, 1)
        g["frac"] = round(g["bytes"] / g["ms_per_step"] / 1e6 / HBM_PEAK_GBS, 4)
        g["ms_per_step"] = round(g["ms_per_step"], 4)
    dom = max(by_kernel, key=lambda k: by_kernel[k]["ms_per_step"])
    tot_bytes, tot_ms, n_launch = by_kernel[dom]["bytes"], by_kernel[dom]["ms_per_step"], by_kernel[dom]["launches"]
    achieved = tot_bytes / tot_ms / 1e6
    for g in by_kernel.values():
        del g["bytes"]
    # the two workloads whose committed profile carries the counter passes
    pmc_summary = None
    if name == "7b" and T == 64 and not args.ar:
        if Bn == 1 and L == 1024:        # (also the decode, prefill and independent-heads runs: same kernel, same rows)
            pmc_summary = "verify_step_7b_t64_l1024.txt"
        elif Bn == 8 and args.mixed and args.prefix is None and not args.decode and not args.prefill and not args.medusa_heads:
            pmc_summary = "verify_step_7b_batch8_mixed.txt"
    alg = algorithmic_bytes(cfg, T, L)
    if Bn > 1 or args.ar:               # weights once; KV rows and tree rows per sequence; heads only if some sequence runs them
        per = [algorithmic_bytes(cfg, 1 if f else T, l) for f, l in zip(flags, Ls)]
        alg = dict(per[0])
        for k in ("kv_prefix_read", "tree_kv_write_read", "embedding_rows"):
            alg[k] = sum(q[k] for q in per)
        if bool((st.gate_flag[:Bn] != 0).all()):   # the gate after the step sent every sequence down the one-token path
            alg["heads"] = 0
        alg["total"] = sum(v for k, v in alg.items() if k != "total")

    # MFMA side: multiply-add work of the GEMMs over the time of the GEMM launches (the survey's definition);
    # the kernels execute twice that on the matrix cores (hi and lo activation plane).
    rows_step = sum(1 if f else T for f in flags)
    head_rows = int((st.gate_flag[:Bn] == 0).sum())
    fl = gemm_flops(cfg, rows_step, head_rows)
    gemm_ms = sum(v["ms_per_step"] for v in gemm.values())
    fl_total = sum(fl.values())
    mfma = {"flops": fl_total, "executed_flops": 2 * fl_total, "gemm_ms": round(gemm_ms, 4),
            "achieved_TFLOPs": round(fl_total / (gemm_ms * 1e-3) / 1e12, 1), "peak": MFMA_PEAK_TFLOPS,
            "frac": round(fl_total / (gemm_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS, 4),
            "frac_executed": round(2 * fl_total / (gemm_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS, 4),
            "note": "flops = 2*N*K*rows of every GEMM of the step; gemm_ms = their launches timed back to back with events; "
                    "executed counts both activation planes"}
    t_hbm = alg["total"] / (HBM_PEAK_GBS * 1e9)
    t_mfma = 2 * fl_total / (MFMA_PEAK_TFLOPS * 1e12)
    step_s = ms_per_step * 1e-3

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
                                f"{T}-node tree" + (", cerberus_ar_step called directly" if args.ar_direct else "")),
                   "graph": graph is not None},
        "latency_us": {"p10": round(float(np.percentile(lat, 10)), 1), "p50": round(float(np.percentile(lat, 50)), 1),
                       "p90": round(float(np.percentile(lat, 90)), 1)},
        "tokens_per_s": round(accepted / (t1 - t0), 2),
        "step_algorithmic_GB": round(alg["total"] / 1e9, 4),
        "step_hbm_frac": round(alg["total"] / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9), 4),
        "step_mfma_frac": round(t_mfma / step_s, 4),
        "step_bound": {"hbm_time_at_peak_ms": round(t_hbm * 1e3, 3), "mfma_time_at_peak_ms": round(t_mfma * 1e3, 3),
                       "binding": "hbm" if t_hbm >= t_mfma else "mfma", "rows": rows_step, "sum_prefix": int(sum(Ls))},
        "roofline": {"bound": "hbm", "kernel": dom + " (" + ", ".join(by_kernel[dom]["kinds"]) + ")",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": profiled_traffic_mb(dom, pmc_summary) if pmc_summary else None,
                     "traffic_unit": "MB per launch",
                     "traffic_source": (f"read from the committed summary profiles/{pmc_summary} (rocprofv3 --pmc FETCH_SIZE + "
                                        "WRITE_SIZE of an earlier run of this command); not measured by this run") if pmc_summary
                                       else "no counter summary is committed for this workload",
                     "by_kernel": by_kernel,
                     "mfma": mfma,
                     "algorithmic_MB_per_launch": round(tot_bytes / n_launch / 1e6, 1),
                     "avg_launch_us": round(tot_ms * 1e3 / n_launch, 2), "launches_per_step": n_launch,
                     "per_kind": gemm},
    }
    if not args.no_cpu and Bn == 1 and not args.ar:
        out["cpu_baseline"] = cpu_baseline(cfg, W, parent, rank, L, cap, reps=1 if name == "13b" else 2)
    elif not args.no_cpu and Bn > 1 and not args.decode and not args.prefill:
        kv_t = synth.make_kv_prefix(cfg, Bn, cap, seed=0, dtype=torch.bfloat16, device="cuda")
        out["cpu_baseline"] = cpu_baseline_batch(cfg, W, parent, rank, kv_t, Ls, flags,
                                                 synth.make_token_ids(Bn, cfg["vocab"], seed=2), synth.make_candidates(cfg, Bn, seed=3))
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
