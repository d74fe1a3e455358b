#!/usr/bin/env python3
"""Benchmark of the tree-based parallel decoding hot path on one MI355X.

One step = one verification pass of a whole model over one batch of token trees:
    for each of the L layers: spec_tree_attention_append (KV append fused into tree attention; distinct
                              per-layer caches)
    spec_verify_greedy, spec_verify_stochastic                        (once per pass)
    spec_kv_commit of the greedy path over all L layers
Inputs are resident in HBM before the timed region. Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--no-graph] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth

# HBM bytes per attention launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a plain copy of
# known size (profiles/tree_attention_bf16_configs2-5_hbm_traffic.txt), per launch of the workload's shape.
MEASURED_TRAFFIC_BYTES = {2: int((67237.9 * 2.000 + 3189.0) * 1024), 3: int((90357.2 * 2.000 + 49164.0) * 1024),
                          4: int((549066.4 * 2.000 + 49154.8) * 1024),
                          5: int(((400755.5 + 7107.0) * 2.000 + 12367.2 + 1024.0) * 1024)}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="workload (BASELINE config number, 2..5)")
    ap.add_argument("--layers", type=int, default=0, help="layers per pass (0 = as many of the model's layers as fit)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--attn-only", action="store_true", help="time only the attention launches (profiling aid)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run three plain 256 MiB device copies, the known-size reference for rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE readings")
    return ap.parse_args()


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
        for name in ("q", "k_new", "v_new"):
            if l == 0:
                W[name].append(inp[name][0].to(dev))
            else:
                W[name].append(torch.randn(inp[name][0].shape, generator=g, device=dev, dtype=torch.float32).to(dt))
        for name in ("k_cache", "v_cache"):
            if l == 0:
                W[name].append(inp[name][0].to(dev))
            else:
                W[name].append(torch.randn(inp[name][0].shape, generator=g, device=dev, dtype=torch.float32).to(dt))
        W["out"].append(torch.empty_like(W["q"][l]))
    return W


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2305_09781_amd import binding as spec
    from paper_2305_09781_amd import probe_binding as probe
    from paper_2305_09781_amd import workloads as wl

    spec.load()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = wl.CONFIGS[args.config]
    e = 2 if cfg.dtype == "bf16" else 4
    per_layer_cache = 2 * cfg.B * cfg.H * cfg.S_cap * cfg.D * e
    L = args.layers or cfg.layers
    L = max(1, min(L, int(200e9 // per_layer_cache)))
    if cfg.cfg == 4 and not args.layers:
        L = 16          # 65B shape: 16 of the 80 layers (17.7 GB of caches) keep set-up time bounded
    W = build_workload(cfg, L, dev)
    B, N, H, D = cfg.B, cfg.N, cfg.H, cfg.D
    pl, par, dep = W["prefix_len"], W["tree_parent"], W["tree_depth"]
    max_prefix = int(W["host"]["prefix_len"].max())

    desc = spec.make_desc(W["q"][0], W["k_cache"][0], max_prefix_len=max_prefix)
    ws_bytes = spec.spec_tree_attention_workspace_bytes(desc)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
    status = torch.zeros(B, dtype=torch.int32, device=dev)

    # verification inputs (vocabulary of the 7B model also for the 65B-shaped config, which names none)
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

    def one_pass():
        for l in range(L):
            spec.spec_tree_attention_append(W["q"][l], W["k_new"][l], W["v_new"][l], W["k_cache"][l], W["v_cache"][l], par,
                                            dep, pl, out=W["out"][l], workspace=ws, status=status, desc=desc)
        spec.spec_verify_greedy(g_logits, g_tok, par, Lmax=Lmax, status=status, out=g_out)
        spec.spec_verify_stochastic(s_dev["logits"], s_dev["probs_ssm"], s_dev["ssm_row"], s_dev["tree_token"], par,
                                    s_dev["u_accept"], s_dev["u_order"], s_dev["u_final"], Lmax=Lmax, workspace=s_ws,
                                    status=status, out=s_out)
        spec.spec_kv_commit(W["k_cache"], W["v_cache"], g_out[0], g_out[1], pl, N, prefix_len_out=pl_out, status=status)

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
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    assert int(status.abs().sum().item()) == 0, "a request was flagged malformed during the benchmark"

    # ---- dominant kernel: tree attention, timed live with events on the launch stream
    run_attn = make_runner(attention_layers) if not args.attn_only else run
    for _ in range(3):
        run_attn()
    reps = max(5, min(args.steps, 50))
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(reps):
        run_attn()
    ev1.record()
    torch.cuda.synchronize()
    attn_us = ev0.elapsed_time(ev1) * 1e3 / (reps * L)
    sum_p = int(W["host"]["prefix_len"].sum())
    # fused append + attention: prefix K,V read (2P), new K,V read (2N) and written to the cache (2N), Q in, O out
    attn_bytes = e * H * D * (2 * sum_p + 6 * B * N)
    achieved = attn_bytes / (attn_us * 1e-6) / 1e9
    layer_bytes = attn_bytes

    # the once-per-pass steps, each timed on its own (graph replay, events): verified tree tokens per second of
    # verification time, as the metric's per-verifier figure
    def time_us(fn, reps=20):
        r = make_runner(fn)
        for _ in range(3):
            r()
        torch.cuda.synchronize()
        ev0.record()
        for _ in range(reps):
            r()
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) * 1e3 / reps
    greedy_us = time_us(lambda: spec.spec_verify_greedy(g_logits, g_tok, par, Lmax=Lmax, status=status, out=g_out))
    stoch_us = time_us(lambda: spec.spec_verify_stochastic(
        s_dev["logits"], s_dev["probs_ssm"], s_dev["ssm_row"], s_dev["tree_token"], par, s_dev["u_accept"], s_dev["u_order"],
        s_dev["u_final"], Lmax=Lmax, workspace=s_ws, status=status, out=s_out))
    commit_us = time_us(lambda: spec.spec_kv_commit(W["k_cache"], W["v_cache"], g_out[0], g_out[1], pl, N,
                                                    prefix_len_out=pl_out, status=status))

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
    result = {
        "metric": "verified tree tokens/sec (whole verification pass: L layers of KV append + tree attention, "
                  "greedy + stochastic verification, KV commit) + achieved HBM GB/s",
        "value": B * N / (ms_per_step * 1e-3), "unit": "tree tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"config {cfg.cfg}: {cfg.name} B={B} H={H} D={D} prefix={cfg.P} tree N={N} "
                               f"vocab={vcfg.V} layers/pass={L}" + (" (attention only)" if args.attn_only else ""),
                   "launch": "eager" if args.no_graph else "hip-graph replay",
                   "layer_tree_tokens_per_s": B * N / (attn_us * 1e-6),
                   "attention_us_per_layer": attn_us, "layer_algorithmic_bytes": layer_bytes,
                   "greedy_verify_us": greedy_us, "greedy_verify_tree_tokens_per_s": B * N / (greedy_us * 1e-6),
                   "stochastic_verify_us": stoch_us, "stochastic_verify_tree_tokens_per_s": B * N / (stoch_us * 1e-6),
                   "commit_all_layers_us": commit_us},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.cfg),
                     "kernel": ("tree_attention_bf16_kernel" if N <= 16 else "tree_attention_bf16_wide_kernel")
                               + " (KV append fused; + attn_combine_kernel when the key range is split)",
                     "bytes_per_launch": attn_bytes,
                     "us_per_launch": attn_us,
                     "measured_read_stream_gbs": read_stream_gbs, "frac_of_measured_read_stream": achieved / read_stream_gbs,
                     # the two products as dense contractions over all N x (prefix + N) pairs, against the bf16
                     # MFMA peak: what the matrix cores would be charged with if this were the bound (it is not)
                     "dense_equivalent_tflops": dense_flops / (attn_us * 1e-6) / 1e12,
                     "frac_of_bf16_mfma_peak": dense_flops / (attn_us * 1e-6) / 2.5e15},
    }

    if args.pmc_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, vcfg, W["host"], gi, si, L)
    print(json.dumps(result))


def cpu_baseline(cfg, vcfg, host, gi, si, L):
    """The CPU oracle, as it stands, on a bounded sample of the same workload."""
    import numpy as np
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
    kc = host["k_cache"][0].view(dtype=__import__("torch").int16 if cfg.dtype == "bf16" else __import__("torch").int32).numpy().copy()
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
