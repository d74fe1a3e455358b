"""HIP-graph replays of the entry points next to the path (fused rotary call, the call on the library's own scratch
array, LM head with statistics, the stochastic verifier from statistics) against the same calls made eagerly
(`pytest -m gpu`). Every replay is compared, with eager launches and synchronisations in between."""
import numpy as np
import pytest
import torch

from paper_2305_09781_amd import workloads as wl
from test_gpu_parity import DEV, _dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("N,D", [(16, 128), (100, 128), (40, 64)])
def test_replays_of_the_newer_entry_points_match_eager(spec, N, D):
    B, H, V, K = 2, 2, 3000, 512
    cfg = wl.Config(86, "graph2", "bf16", B=B, H=H, D=D, P=(300, 500), N=N, tree="random_branching", V=V)
    L = 2
    inp = wl.make_attention_inputs(cfg, n_layers=L)
    S = inp["k_cache"][0].shape[2]
    cos, sin = (_dev(t) for t in wl.make_rope_tables(S, D))
    ver = wl.make_verify_inputs(cfg, mode="stochastic", parent=inp["tree_parent"].numpy())
    pl, par, dep = _dev(inp["prefix_len"]), _dev(inp["tree_parent"]), _dev(inp["tree_depth"])
    q, kn, vn = [_dev(x) for x in inp["q"]], [_dev(x) for x in inp["k_new"]], [_dev(x) for x in inp["v_new"]]
    k0, v0 = [_dev(x) for x in inp["k_cache"]], [_dev(x) for x in inp["v_cache"]]
    kcs, vcs = [x.clone() for x in k0], [x.clone() for x in v0]
    outs = [torch.empty_like(x) for x in q]
    rng = np.random.default_rng(9)
    hidden = _dev(torch.from_numpy(rng.standard_normal((B * N, K)).astype(np.float32)).to(torch.bfloat16))
    weight = _dev(torch.from_numpy((rng.standard_normal((V, K)) * 0.05).astype(np.float32)).to(torch.bfloat16))
    lm_out = (torch.empty((B * N, V), dtype=torch.bfloat16, device=DEV), torch.empty(B * N, dtype=torch.int32, device=DEV),
              torch.empty(B * N, dtype=torch.float32, device=DEV), torch.empty(B * N, dtype=torch.float32, device=DEV))
    lm_ws = torch.empty(int(spec.load().spec_lm_head_logits_stats_workspace_bytes(B * N, V)), dtype=torch.uint8, device=DEV)
    sdev = {k: _dev(ver[k]) for k in ("probs_ssm", "ssm_row", "tree_token", "u_accept", "u_order", "u_final")}
    s_ws = torch.empty(int(spec.load().spec_verify_stochastic_stats_workspace_bytes(B, V)), dtype=torch.uint8, device=DEV)
    vout = (torch.empty((B, N), dtype=torch.int32, device=DEV), torch.empty(B, dtype=torch.int32, device=DEV),
            torch.empty((B, N), dtype=torch.int32, device=DEV))
    ws = torch.empty(64 << 20, dtype=torch.uint8, device=DEV)
    status = torch.zeros(B, dtype=torch.int32, device=DEV)
    pl_out = torch.empty_like(pl)
    mp = int(inp["prefix_len"].max())

    def one_pass():
        # layer 0: rotation + append + attention in one launch, key range in chunks (partials + combine)
        spec.spec_tree_attention_append_rope(q[0], kn[0], vn[0], kcs[0], vcs[0], par, dep, pl, cos, sin, out=outs[0], workspace=ws,
                                             status=status, max_prefix_len=mp, plan=(128, 0, 0))
        # layer 1: the call that allocates nothing, partials in the library's scratch array
        spec.spec_tree_attention_append_static(q[1], kn[1], vn[1], kcs[1], vcs[1], par, dep, pl, outs[1], status=status,
                                               max_prefix_len=mp, plan=(128, 0, 0))
        spec.spec_lm_head_logits_stats(hidden, weight, 1.0, workspace=lm_ws, out=lm_out)
        spec.spec_verify_stochastic_stats(lm_out[0].view(B, N, V), lm_out[2], lm_out[3], sdev["probs_ssm"], sdev["ssm_row"],
                                          sdev["tree_token"], par, sdev["u_accept"], sdev["u_order"], sdev["u_final"],
                                          workspace=s_ws, status=status, out=vout)
        spec.spec_kv_commit(kcs, vcs, vout[0], vout[1], pl, N, prefix_len_out=pl_out, status=status)

    def snapshot():
        torch.cuda.synchronize()
        return [o.clone() for o in outs] + [c.clone() for c in kcs + vcs] + [x.clone() for x in vout + lm_out] + [pl_out.clone()]

    def reset():
        for l in range(L):
            kcs[l].copy_(k0[l])
            vcs[l].copy_(v0[l])
            outs[l].zero_()
        for x in vout:
            x.fill_(-7)
        for x in lm_out:
            x.zero_()
        pl_out.zero_()

    one_pass()
    want = snapshot()
    assert int(status.abs().sum()) == 0 and int(want[2 * L + 2 * L + 1].max()) >= 1      # accepted_len
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        one_pass()
    for rep in range(4):
        reset()
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for i, (a, b_) in enumerate(zip(want, got)):
            assert torch.equal(a, b_), f"replay {rep}: tensor {i} differs from the eager pass"
        one_pass()                      # eager work between replays
        torch.cuda.synchronize()
    assert int(status.abs().sum()) == 0
