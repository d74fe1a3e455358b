"""Greedy verification from hidden states: the fused LM head + arg-max (spec_verify_greedy_lm_head) next to the
two-step alternative (a library GEMM that writes bf16 logits, then spec_verify_greedy on them).

    python -m paper_2305_09781_amd.lm_head_study [--batches 1,2,4,8] [--tree 16] [--hidden 4096] [--vocab 32000]

One JSON line per batch size: microseconds per verification from hidden states to the accepted path, HIP-graph
replay over several distinct weight matrices (a 32000 x 4096 head is 262 MB, more than the 256 MB Infinity
Cache, and the copies rotate). Synthetic weights and hidden states; the timing does not depend on their values.
"""
from __future__ import annotations

import argparse
import json

import numpy as np
import torch

from . import binding as spec
from . import workloads as wl


def _time_us(fn, per_replay: int, reps: int = 10) -> float:
    fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    for _ in range(2):
        g.replay()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (reps * per_replay)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--batches", default="1,2,4,8")
    ap.add_argument("--tree", type=int, default=16)
    ap.add_argument("--hidden", type=int, default=4096)
    ap.add_argument("--vocab", type=int, default=32000)
    ap.add_argument("--weights", type=int, default=6, help="distinct weight matrices the timing rotates over")
    args = ap.parse_args()
    spec.load()
    dev = "cuda:0"
    K, V, N = args.hidden, args.vocab, args.tree
    Ws = [torch.randn((V, K), device=dev, dtype=torch.float32).mul_(0.05).to(torch.bfloat16) for _ in range(args.weights)]
    for B in [int(x) for x in args.batches.split(",")]:
        M = B * N
        h = torch.randn((M, K), device=dev, dtype=torch.bfloat16)
        par = torch.from_numpy(np.stack([wl.tree_expansion(wl.EXPANSION_EVAL * 16, N) for _ in range(B)]).astype(np.int32)).to(dev)
        tok = torch.randint(0, V, (B, N), device=dev, dtype=torch.int32)
        ws = torch.empty(spec.spec_lm_head_argmax_workspace_bytes(M, V), dtype=torch.uint8, device=dev)
        logits = torch.empty((B, N, V), device=dev, dtype=torch.bfloat16)

        def fused():
            for W in Ws:
                spec.spec_verify_greedy_lm_head(h, W, tok, par, workspace=ws)

        def two_step():
            for W in Ws:
                torch.matmul(h, W.t(), out=logits.view(M, V))
                spec.spec_verify_greedy(logits, tok, par)

        def head_only():
            for W in Ws:
                spec.spec_lm_head_argmax(h, W, workspace=ws)

        us_f, us_t, us_h = _time_us(fused, len(Ws)), _time_us(two_step, len(Ws)), _time_us(head_only, len(Ws))
        weight_bytes = V * K * 2 + M * K * 2
        print(json.dumps({"batch": B, "tree_nodes": N, "rows": M, "hidden": K, "vocab": V,
                          "fused_verify_us": round(us_f, 2), "library_gemm_plus_verify_us": round(us_t, 2),
                          "speedup": round(us_t / us_f, 3), "lm_head_argmax_us": round(us_h, 2),
                          "lm_head_gbs": round(weight_bytes / us_h / 1e3, 1),
                          "lm_head_frac_of_hbm_peak": round(weight_bytes / us_h / 1e3 / 8000.0, 3)}), flush=True)


if __name__ == "__main__":
    main()
