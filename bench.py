#!/usr/bin/env python3
"""Benchmark of the tree-based parallel decoding hot path on one MI355X.

One step = one verification pass of a whole model over one batch of token trees:
    for each of the L layers: spec_tree_attention_append (KV append fused into tree attention; distinct
                              per-layer caches)
    spec_verify_greedy, spec_verify_stochastic                        (once per pass)
    spec_kv_commit of the greedy path over all L layers
Inputs are resident in HBM before the timed region. Prints ONE JSON line: the headline workload (config 4, the
largest single-GPU configuration) measured in full, and a `per_config` list with the same measurement of the
other bf16 workloads (configs 2, 3, 5) on fewer timed steps, each in a child process of its own.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--no-per-config] [--no-graph] [--no-cpu-baseline]

`--lm-head` measures something else and prints its own JSON line: verification from hidden states (the LM head fused
with the arg-max, or with the logits' softmax statistics) next to a library GEMM followed by the verifier on its logits.
"""
import argparse
import gc
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
HEADLINE_CONFIG = 4
SETTLE_SECONDS = 3.0           # pause after a process that freed a large workload, before the next measurement
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "tree_attention_bf16_hbm_traffic.txt")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=HEADLINE_CONFIG, help="headline workload (BASELINE config number, 2..5)")
    ap.add_argument("--layers", type=int, default=0, help="layers per pass (0 = every layer of the model the shape comes from)")
    ap.add_argument("--no-per-config", action="store_true", help="measure the headline workload only")
    ap.add_argument("--per-config-entry", action="store_true",
                    help="measure --config and print it as one entry of `per_config` (what a default run starts as a "
                         "child process for each of the other workloads)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--attn-only", action="store_true", help="time only the attention launches (profiling aid)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run three plain 256 MiB device copies, the known-size reference for rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE readings")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="instead of the verification pass: the attention launch of --config (2, 3 or 4: equal prefix "
                         "lengths, 128 elements per row) next to a kernel that issues only its memory requests")
    ap.add_argument("--lm-head", action="store_true",
                    help="instead of the verification pass: the LM-head entry points against a library GEMM + verifier, "
                         "at 16 .. 256 tree nodes per pass (hidden 4096, vocabulary 32000)")
    return ap.parse_args()


def counter_traffic_bytes(cfg_id):
    """HBM bytes per attention launch of this workload as rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE counted them
    (a committed summary under profiles/, which also records the commit it was taken at); None when that file
    is not next to this script."""
    try:
        for line in open(TRAFFIC_FILE):
            m = re.match(r"\s*config\s+(\d+)\s*:.*\btotal_bytes=(\d+)", line)
            if m and int(m.group(1)) == cfg_id:
                return int(m.group(2))
    except OSError:
        pass
    return None


def build_workload(cfg, n_layers, dev):
    """Layer 0 is the host-generated, seeded input the parity tests use; the other layers' buffers are
    filled on the device (their values do not matter for timing, their distinct addresses do)."""
    import torch
    from paper_2305_09781_amd import workloads as wl

    inp = wl.make_attention_inputs(cfg)
    g = torch.Generator(device=dev)
    g.manual_seed(cfg.seed)
    dt = cfg.torch_dtype
    W = {"prefix_len": inp["prefix_len"].to(dev), "tree_parent": inp["tree_parent"].to(dev),
         "tree_depth": inp["tree_depth"].to(dev), "q": [], "k_new": [], "v_new": [], "k_cache": [], "v_cache": [],
         "out": [], "host": inp}
    for l in range(n_layers):
        for name in ("q", "k_new", "v_new", "k_cache", "v_cache"):
            if l == 0:
                W[name].append(inp[name][0].to(dev))
            else:
                W[name].append(torch.randn(inp[name][0].shape, generator=g, device=dev, dtype=torch.float32).to(dt))
        W["out"].append(torch.empty_like(W["q"][l]))
    return W


def measure(cfg_id, args, steps, warmup, want_cpu_baseline, want_read_probe):
    """One workload, measured in full: the whole pass (graph replay, wall clock around `steps` replays), the
    dominant kernel (events on the launch stream around back-to-back attention launches), the once-per-pass
    steps on their own."""
    import torch

    from paper_2305_09781_amd import binding as spec
    from paper_2305_09781_amd import probe_binding as probe
    from paper_2305_09781_amd import workloads as wl

    dev = "cuda:0"
    cfg = wl.CONFIGS[cfg_id]
    e = 2 if cfg.dtype == "bf16" else 4
    per_layer_cache = 2 * cfg.B * cfg.H * cfg.S_cap * cfg.D * e
    L = args.layers or cfg.layers
    L = max(1, min(L, int(200e9 // per_layer_cache), 128))
    W = build_workload(cfg, L, dev)
    B, N, H, D = cfg.B, cfg.N, cfg.H, cfg.D
    pl, par, dep = W["prefix_len"], W["tree_parent"], W["tree_depth"]
    max_prefix = int(W["host"]["prefix_len"].max())

    desc = spec.make_desc(W["q"][0], W["k_cache"][0], max_prefix_len=max_prefix)
    ws_bytes = spec.spec_tree_attention_workspace_bytes(desc)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
    status = torch.zeros(B, dtype=torch.int32, device=dev)

    # verification inputs (the 65B-shaped config names no vocabulary: LLaMA's 32000, as in the 7B shapes)
    vcfg = cfg if cfg.V else wl.Config(cfg.cfg, cfg.name, cfg.dtype, B=B, H=H, D=D, P=cfg.P, N=N, tree=cfg.tree,
                                       widths=cfg.widths, V=32000)
    par_np = W["host"]["tree_parent"].numpy()
    gi = wl.make_verify_inputs(vcfg, mode="greedy", parent=par_np)
    si = wl.make_verify_inputs(vcfg, mode="stochastic", parent=par_np)
    g_logits, g_tok = gi["logits"].to(dev), gi["tree_token"].to(dev)
    s_dev = {k: si[k].to(dev) for k in ("logits", "probs_ssm", "ssm_row", "tree_token", "u_accept", "u_order", "u_final")}
    Lmax = N
    g_out = (torch.empty((B, Lmax), dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
             torch.empty((B, Lmax), dtype=torch.int32, device=dev), torch.empty((B, N), dtype=torch.int32, device=dev))
    s_out = (torch.empty((B, Lmax), dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
             torch.empty((B, Lmax), dtype=torch.int32, device=dev))
    s_ws = torch.empty(spec.spec_verify_stochastic_workspace_bytes(B, N, vcfg.V), dtype=torch.uint8, device=dev)
    pl_out = torch.empty_like(pl)

    def attention_layers():
        for l in range(L):
            spec.spec_tree_attention_append(W["q"][l], W["k_new"][l], W["v_new"][l], W["k_cache"][l], W["v_cache"][l], par,
                                            dep, pl, out=W["out"][l], workspace=ws, status=status, desc=desc)

    rope_cos, rope_sin = (t.to(dev) for t in wl.make_rope_tables(cfg.S_cap, D))

    def attention_layers_rope():   # the same launches with the rotary embedding of q and the new K rows fused in
        for l in range(L):
            spec.spec_tree_attention_append_rope(W["q"][l], W["k_new"][l], W["v_new"][l], W["k_cache"][l], W["v_cache"][l],
                                                 par, dep, pl, rope_cos, rope_sin, out=W["out"][l], workspace=ws,
                                                 status=status, max_prefix_len=max_prefix)

    def greedy():
        spec.spec_verify_greedy(g_logits, g_tok, par, Lmax=Lmax, status=status, out=g_out)

    def stochastic():
        spec.spec_verify_stochastic(s_dev["logits"], s_dev["probs_ssm"], s_dev["ssm_row"], s_dev["tree_token"], par,
                                    s_dev["u_accept"], s_dev["u_order"], s_dev["u_final"], Lmax=Lmax, workspace=s_ws,
                                    status=status, out=s_out)

    def commit():
        spec.spec_kv_commit(W["k_cache"], W["v_cache"], g_out[0], g_out[1], pl, N, prefix_len_out=pl_out, status=status)

    def one_pass():
        attention_layers()
        greedy()
        stochastic()
        commit()

    work = attention_layers if args.attn_only else one_pass

    def make_runner(fn):
        if args.no_graph:
            return fn
        fn()                                  # eager once: first-call set-up happens outside capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            fn()
        return graph.replay

    run = make_runner(work)
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / steps
    assert int(status.abs().sum().item()) == 0, "a request was flagged malformed during the benchmark"

    # ---- dominant kernel: tree attention, timed live with events on the launch stream
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def time_us(fn, reps, per=1, repeats=5):
        """Median over `repeats` event-timed batches of `reps` replays each (after three untimed replays)."""
        r = run if fn is work else make_runner(fn)
        for _ in range(3):
            r()
        batches = []
        for _ in range(repeats):
            torch.cuda.synchronize()
            ev0.record()
            for _ in range(reps):
                r()
            ev1.record()
            torch.cuda.synchronize()
            batches.append(ev0.elapsed_time(ev1) * 1e3 / (reps * per))
        return sorted(batches)[len(batches) // 2]

    attn_us = time_us(attention_layers, max(5, min(steps, 50)), per=L)
    attn_rope_us = time_us(attention_layers_rope, max(5, min(steps, 20)), per=L) if cfg.dtype == "bf16" else None
    sum_p = int(W["host"]["prefix_len"].sum())
    # fused append + attention: prefix K,V read (2P), new K,V read (2N) and written to the cache (2N), Q in, O out
    attn_bytes = e * H * D * (2 * sum_p + 6 * B * N)
    achieved = attn_bytes / (attn_us * 1e-6) / 1e9
    # the once-per-pass steps, each replayed on its own
    greedy_us, stoch_us, commit_us = time_us(greedy, 20), time_us(stochastic, 20), time_us(commit, 20)

    read_stream_gbs = None
    if want_read_probe:
        # practical ceiling on this machine for a launch of this size: a plain read kernel, one launch per buffer,
        # over distinct buffers of the attention launch's byte count (>= 2 GB in total, far beyond the 256 MB
        # Infinity Cache), timed the same way
        n_probe = max(2, int(2e9 // attn_bytes) + 1)
        probes = [torch.empty(attn_bytes // 16 * 16, dtype=torch.uint8, device=dev).fill_(l + 1) for l in range(n_probe)]
        sink = torch.zeros(16, dtype=torch.uint8, device=dev)

        def read_all():
            for pb in probes:
                probe.spec_probe_read_stream(pb, sink)
        read_all()
        torch.cuda.synchronize()
        ev0.record()
        for _ in range(3):
            read_all()
        ev1.record()
        torch.cuda.synchronize()
        read_stream_gbs = 3 * n_probe * (attn_bytes // 16 * 16) / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
        del probes

    dense_flops = 4.0 * H * D * N * float(W["host"]["prefix_len"].double().add(N).sum())
    wide = N > 16
    res = {
        "cfg": cfg.cfg,
        "workload": f"config {cfg.cfg}: {cfg.name} B={B} H={H} D={D} prefix={cfg.P} tree N={N} vocab={vcfg.V} "
                    f"layers/pass={L}" + (" (attention only)" if args.attn_only else ""),
        "ms_per_step": ms_per_step, "value": B * N / (ms_per_step * 1e-3), "steps": steps,
        "attn_us": attn_us, "attn_rope_us": attn_rope_us, "attn_bytes": attn_bytes, "achieved": achieved,
        "greedy_us": greedy_us, "stoch_us": stoch_us, "commit_us": commit_us, "L": L,
        "kernel": ("tree_attention_bf16_wide32_kernel" if N > 64 and D == 128 else
                   "tree_attention_bf16_wide_kernel" if wide else "tree_attention_bf16_kernel")
                  + " (KV append fused; + attn_combine_kernel when the key range is split)",
        "read_stream_gbs": read_stream_gbs, "dense_flops": dense_flops, "dtype": cfg.dtype,
        "traffic": counter_traffic_bytes(cfg.cfg),
    }
    if args.pmc_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    if want_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cfg, W["host"], gi, si, L)
    del W, s_dev, g_logits, ws, s_ws, run
    gc.collect()
    torch.cuda.empty_cache()
    return res


def lm_head_comparison(args):
    """Greedy / stochastic verification from hidden states: spec_verify_greedy_lm_head and spec_lm_head_logits_stats
    next to torch.matmul (the library GEMM) writing bf16 logits followed by spec_verify_greedy on them. HIP-graph
    replay over several distinct weight matrices (a 32000 x 4096 head is 262 MB, more than the Infinity Cache)."""
    import numpy as np
    import torch

    from paper_2305_09781_amd import binding as spec
    from paper_2305_09781_amd import workloads as wl

    dev = "cuda:0"
    K, V, N = 4096, 32000, 16
    Ws = [torch.randn((V, K), device=dev, dtype=torch.float32).mul_(0.05).to(torch.bfloat16) for _ in range(6)]
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def time_us(fn, reps=10):
        fn()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            fn()
        for _ in range(2):
            graph.replay()
        torch.cuda.synchronize()
        ev0.record()
        for _ in range(reps):
            graph.replay()
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) * 1e3 / (reps * len(Ws))

    rows = []
    for B in (1, 2, 4, 6, 8, 16):
        M = B * N
        h = torch.randn((M, K), device=dev, dtype=torch.bfloat16)
        par = torch.from_numpy(np.stack([wl.tree_expansion(wl.EXPANSION_EVAL * 16, N) for _ in range(B)]).astype(np.int32)).to(dev)
        tok = torch.randint(0, V, (B, N), device=dev, dtype=torch.int32)
        ws = torch.empty(spec.spec_lm_head_argmax_workspace_bytes(M, V), dtype=torch.uint8, device=dev)
        ws2 = torch.empty(int(spec.load().spec_lm_head_logits_stats_workspace_bytes(M, V)), dtype=torch.uint8, device=dev)
        logits = torch.empty((B, N, V), device=dev, dtype=torch.bfloat16)

        def fused():
            for W in Ws:
                spec.spec_verify_greedy_lm_head(h, W, tok, par, workspace=ws)

        def gemm_then_verify():
            for W in Ws:
                torch.matmul(h, W.t(), out=logits.view(M, V))
                spec.spec_verify_greedy(logits, tok, par)

        def gemm_only():
            for W in Ws:
                torch.matmul(h, W.t(), out=logits.view(M, V))

        def head_only():
            for W in Ws:
                spec.spec_lm_head_argmax(h, W, workspace=ws)

        def logits_and_stats():
            for W in Ws:
                spec.spec_lm_head_logits_stats(h, W, 1.0, workspace=ws2)

        us = {"fused_greedy_verify_us": time_us(fused), "library_gemm_plus_greedy_verify_us": time_us(gemm_then_verify),
              "lm_head_argmax_us": time_us(head_only), "lm_head_logits_and_stats_us": time_us(logits_and_stats),
              "library_gemm_us": time_us(gemm_only)}
        weight_bytes = V * K * 2 + M * K * 2
        rows.append({"rows": M, **{k: round(v, 2) for k, v in us.items()},
                     "lm_head_argmax_frac_of_hbm_peak": round(weight_bytes / us["lm_head_argmax_us"] / 1e3 / HBM_PEAK_GBS, 3)})
    print(json.dumps({"metric": "verification from hidden states, microseconds per pass (hidden 4096, vocabulary 32000, "
                                "trees of 16 nodes)", "n_gpus": 1, "dtype": "bf16", "data": "synthetic", "rows": rows}))


def roofline_of(r):
    d = {"bound": "hbm", "achieved": r["achieved"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": r["achieved"] / HBM_PEAK_GBS,
         # counter-measured HBM bytes per launch of this shape, read from the committed rocprofv3 --pmc summary
         # (which names the commit it was taken at): not measured in this run; null when the summary is not
         # next to this script
         "traffic": r["traffic"],
         "traffic_source": "profiles/tree_attention_bf16_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, offline)",
         "kernel": r["kernel"], "bytes_per_launch": r["attn_bytes"], "us_per_launch": r["attn_us"],
         # the two products as dense contractions over all N x (prefix + N) pairs, against the bf16 MFMA
         # peak: what the matrix cores would be charged with if this were the bound (it is not)
         "dense_equivalent_tflops": r["dense_flops"] / (r["attn_us"] * 1e-6) / 1e12,
         "frac_of_bf16_mfma_peak": r["dense_flops"] / (r["attn_us"] * 1e-6) / 2.5e15}
    if r["read_stream_gbs"]:
        d["measured_read_stream_gbs"] = r["read_stream_gbs"]
        d["frac_of_measured_read_stream"] = r["achieved"] / r["read_stream_gbs"]
    return d


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2305_09781_amd import binding as spec

    spec.load()

    def need_gpu():
        if not torch.cuda.is_available():
            print("bench.py: no GPU visible", file=sys.stderr)
            sys.exit(2)
        torch.cuda.set_device(0)

    if args.lm_head:
        need_gpu()
        lm_head_comparison(args)
        return
    if args.traffic_probe:
        need_gpu()
        traffic_probe(args)
        return

    if args.per_config_entry:   # child of a default run: one workload, printed as an entry of `per_config`
        need_gpu()
        print(json.dumps(per_config_entry(measure(args.config, args, args.steps, args.warmup, False, False))))
        return
    # The other workloads, each measured by a child process of its own (this file with --per-config-entry) before
    # this process touches the GPU: after a process frees tens of GB the driver clears that memory in the
    # background for some seconds, and a workload measured meanwhile runs about 4 % slower (config 3 right after a
    # config 4 run: 44.7 us per launch against 43.1 otherwise). Hence also the pauses.
    per = None
    if not args.no_per_config and not args.attn_only:
        import subprocess
        per = []
        time.sleep(SETTLE_SECONDS)   # whatever ran on the machine before this may have just freed its memory
        for c in (2, 3, 4, 5):
            if c == args.config:
                continue
            cmd = [sys.executable, os.path.abspath(__file__), "--config", str(c), "--per-config-entry",
                   "--steps", str(max(3, min(args.steps, 10))), "--warmup", str(min(args.warmup, 3))]
            if args.no_graph:
                cmd.append("--no-graph")
            if args.layers:
                cmd += ["--layers", str(args.layers)]
            child = subprocess.run(cmd, capture_output=True, text=True)
            lines = [ln for ln in child.stdout.splitlines() if ln.startswith("{")]
            if child.returncode != 0 or not lines:
                # said loudly, and the headline measurement still runs: its line is what the caller came for
                sys.stderr.write(child.stderr[-2000:])
                sys.stderr.write("bench.py: measuring config %d in a child process failed (exit %d)\n" % (c, child.returncode))
                per.append({"workload": "config %d" % c, "error": "child process exited with %d" % child.returncode})
            else:
                per.append(json.loads(lines[-1]))
            time.sleep(SETTLE_SECONDS)
        time.sleep(SETTLE_SECONDS)
    need_gpu()
    head = measure(args.config, args, args.steps, args.warmup, not args.no_cpu_baseline, True)
    tokens = head["value"] * head["ms_per_step"] * 1e-3          # tree tokens per pass (B * N)
    result = {
        "metric": "verified tree tokens/sec (whole verification pass: L layers of KV append + tree attention, "
                  "greedy + stochastic verification, KV commit) + achieved HBM GB/s",
        "value": head["value"], "unit": "tree tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": head["workload"],
                   "launch": "eager" if args.no_graph else "hip-graph replay",
                   "layer_tree_tokens_per_s": tokens / (head["attn_us"] * 1e-6),
                   "attention_us_per_layer": head["attn_us"], "layer_algorithmic_bytes": head["attn_bytes"],
                   # the same launch with the rotary embedding of q and of the new K rows fused in
                   "attention_with_rotary_us_per_layer": head["attn_rope_us"],
                   "greedy_verify_us": head["greedy_us"], "greedy_verify_tree_tokens_per_s": tokens / (head["greedy_us"] * 1e-6),
                   "stochastic_verify_us": head["stoch_us"],
                   "stochastic_verify_tree_tokens_per_s": tokens / (head["stoch_us"] * 1e-6),
                   "commit_all_layers_us": head["commit_us"]},
        "roofline": roofline_of(head),
    }
    if "cpu_baseline" in head:
        result["cpu_baseline"] = head["cpu_baseline"]
    if per is not None:
        result["per_config"] = per
    print(json.dumps(result))


def per_config_entry(r):
    return {"workload": r["workload"], "tree_tokens_per_s": r["value"], "ms_per_step": r["ms_per_step"],
            "steps": r["steps"], "us_per_launch": r["attn_us"], "us_per_launch_with_rotary": r["attn_rope_us"],
            "bytes_per_launch": r["attn_bytes"],
            "roofline": {"bound": "hbm", "achieved": r["achieved"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": r["achieved"] / HBM_PEAK_GBS, "traffic": r["traffic"]},
            "greedy_verify_us": r["greedy_us"], "stochastic_verify_us": r["stoch_us"],
            "commit_all_layers_us": r["commit_us"]}


def traffic_probe(args):
    """The attention launch of one workload next to spec_probe_attention_traffic: the same memory requests (K/V
    stream through an LDS ring, queries, new rows, appended rows, outputs) with no arithmetic. One JSON line."""
    import torch

    from paper_2305_09781_amd import binding as spec
    from paper_2305_09781_amd import probe_binding as probe
    from paper_2305_09781_amd import workloads as wl

    dev = "cuda:0"
    cfg = wl.CONFIGS[args.config]
    prefix = cfg.P if isinstance(cfg.P, int) else None
    if cfg.dtype != "bf16" or cfg.D != 128 or prefix is None:
        print("bench.py --traffic-probe: config %d has no equal prefix lengths / 128-element bf16 rows" % args.config,
              file=sys.stderr)
        sys.exit(2)
    L = args.layers or min(cfg.layers, 32)
    W = build_workload(cfg, L, dev)
    pl, par, dep = W["prefix_len"], W["tree_parent"], W["tree_depth"]
    desc = spec.make_desc(W["q"][0], W["k_cache"][0], max_prefix_len=prefix)
    ws = torch.empty(max(spec.spec_tree_attention_workspace_bytes(desc), 256), dtype=torch.uint8, device=dev)
    status = torch.zeros(cfg.B, dtype=torch.int32, device=dev)

    def attention():
        for l in range(L):
            spec.spec_tree_attention_append(W["q"][l], W["k_new"][l], W["v_new"][l], W["k_cache"][l], W["v_cache"][l], par,
                                            dep, pl, out=W["out"][l], workspace=ws, status=status, desc=desc)

    def requests(flags):
        def run():
            for l in range(L):
                probe.spec_probe_attention_traffic(W["k_cache"][l], W["v_cache"][l], W["q"][l], W["k_new"][l], W["v_new"][l],
                                                   W["out"][l], prefix, flags)
        return run

    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def time_us(fn, reps=10, repeats=5):
        fn()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            fn()
        for _ in range(3):
            graph.replay()
        batches = []
        for _ in range(repeats):
            torch.cuda.synchronize()
            ev0.record()
            for _ in range(reps):
                graph.replay()
            ev1.record()
            torch.cuda.synchronize()
            batches.append(ev0.elapsed_time(ev1) * 1e3 / (reps * L))
        return sorted(batches)[len(batches) // 2]

    Q, NEW, APP, OUT = probe.TRAFFIC_QUERIES, probe.TRAFFIC_NEW_ROWS, probe.TRAFFIC_APPEND, probe.TRAFFIC_OUTPUTS
    attn_us = time_us(attention)
    sets = [("kv_stream", 0), ("kv_stream+queries", Q), ("kv_stream+new_rows", NEW), ("kv_stream+new_rows+appended_rows", NEW | APP),
            ("kv_stream+outputs", OUT), ("everything", Q | NEW | APP | OUT)]
    req = {name: time_us(requests(flags)) for name, flags in sets}
    attn_us_again = time_us(attention)
    e = 2
    attn_bytes = e * cfg.H * cfg.D * cfg.B * (2 * prefix + 6 * cfg.N)
    print(json.dumps({
        "mode": "traffic-probe", "workload": "config %d: %s B=%d H=%d D=%d prefix=%d tree N=%d" % (
            cfg.cfg, cfg.name, cfg.B, cfg.H, cfg.D, prefix, cfg.N),
        "layers": L, "bytes_per_launch": attn_bytes,
        "attention_us_per_launch": [attn_us, attn_us_again],
        "memory_requests_only_us_per_launch": req,
        "memory_requests_only_gbs": attn_bytes / (req["everything"] * 1e-6) / 1e9,
        "attention_over_memory_requests_only": min(attn_us, attn_us_again) / req["everything"]}))


def cpu_baseline(cfg, host, gi, si, L):
    """The CPU oracle, as it stands, on a bounded sample of the same workload."""
    import torch
    from oracle import spec_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = 1
    B, N = cfg.B, cfg.N
    budget_s = 12.0
    # attention + append of one layer, request by request, repeated over the batch until the time
    # budget is used (about 12 s of CPU work; a slow configuration stops inside the first batch)
    t0 = time.perf_counter()
    done = 0
    pl = host["prefix_len"].numpy()
    par = host["tree_parent"].numpy()
    while True:
        b = done % B
        kc = host["k_cache"][0][b:b + 1].double().numpy()
        vc = host["v_cache"][0][b:b + 1].double().numpy()
        orc.kv_append(kc, vc, host["k_new"][0][b:b + 1].double().numpy(), host["v_new"][0][b:b + 1].double().numpy(),
                      pl[b:b + 1])
        orc.tree_attention(host["q"][0][b:b + 1].double().numpy(), kc, vc, par[b:b + 1], pl[b:b + 1])
        done += 1
        if time.perf_counter() - t0 > budget_s or done >= 64 * B:
            break
    t_layer = (time.perf_counter() - t0) * B / done
    t0 = time.perf_counter()
    gp, gl, _, _ = orc.verify_greedy(gi["logits"].numpy(), gi["tree_token"].numpy(), par)
    orc.verify_stochastic(si["logits"].numpy(), si["probs_ssm"].numpy(), si["ssm_row"].numpy(), si["tree_token"].numpy(),
                          par, si["u_accept"].numpy(), si["u_order"].numpy(), si["u_final"].numpy())
    t_verify = time.perf_counter() - t0
    t0 = time.perf_counter()
    kc = host["k_cache"][0].view(dtype=torch.int16 if cfg.dtype == "bf16" else torch.int32).numpy().copy()
    orc.kv_commit([kc], [kc.copy()], gp, gl, pl, N=N)
    t_commit = time.perf_counter() - t0
    t_pass = L * (t_layer + t_commit) + t_verify
    return {"value": B * N / t_pass, "unit": "tree tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"oracle (numpy float64) timed on {done} request-layers of append+attention (batch of {B}; "
                      f"{t_layer:.2f} s per layer of the batch), one greedy + one stochastic verification "
                      f"({t_verify:.2f} s), one layer's commit ({t_commit:.3f} s); pass time = L*(layer+commit)+verify "
                      f"with L={L}"}


if __name__ == "__main__":
    main()
