"""Sequence-based decoding baseline (Section 4.2; the comparison of Figure 11): host-side decomposition of
a token tree into root-to-leaf sequences (CPU tests) and, on the GPU, agreement of sequence-based decoding
with the oracle's tree attention on every node (Definition 4.1: a node's tree attention is the attention
output of its own sequence)."""
import numpy as np
import pytest
import torch

from oracle import spec_oracle as orc
from paper_2305_09781_amd import sequence_baseline as sb
from paper_2305_09781_amd import workloads as wl


def test_leaf_paths_of_the_figure_4_shaped_tree():
    # t2 -> t3 -> {t4 -> t5, t6 -> t7, t8 -> t9}: three sequences sharing (t2, t3); nodes in depth-first order
    parent = [-1, 0, 1, 2, 1, 4, 1, 6]
    assert sb.leaf_paths(parent) == [[0, 1, 2, 3], [0, 1, 4, 5], [0, 1, 6, 7]]
    assert sb.leaf_paths([-1]) == [[0]]
    assert sb.leaf_paths([-1, 0, 1, 2]) == [[0, 1, 2, 3]]          # a chain is its own single sequence
    assert sb.leaf_paths([-1, 0, 0, 0]) == [[0, 1], [0, 2], [0, 3]]


@pytest.mark.parametrize("seed", range(5))
def test_decompose_covers_every_node_at_its_depth(seed):
    rng = np.random.default_rng(seed)
    B, N = 3, 1 + int(rng.integers(1, 40))
    parent = np.stack([wl.tree_random_parent(rng, N) for _ in range(B)])
    dec = sb.decompose(parent)
    n_leaves = sum(len(set(range(N)) - set(int(p) for p in parent[b][1:])) for b in range(B))
    assert dec.nodes.shape[0] == n_leaves == len(dec.request) == len(dec.length)
    for s in range(dec.nodes.shape[0]):
        b, ln = dec.request[s], dec.length[s]
        path = dec.nodes[s, :ln]
        assert path[0] == 0 and all(parent[b][path[i]] == path[i - 1] for i in range(1, ln))
        assert (dec.nodes[s, ln:] == path[-1]).all()                # padding repeats the leaf
    depth = np.stack([wl.depth_of(parent[b]) for b in range(B)])
    for b in range(B):
        for i in range(N):
            s, pos = dec.owner[b, i]
            assert dec.request[s] == b and dec.nodes[s, pos] == i and pos == depth[b, i] and pos < dec.length[s]


DEV = "cuda:0"


@pytest.mark.gpu
@pytest.mark.parametrize("case", [("bf16", 2, 2, 128, (40, 200), 16, "expansion"), ("bf16", 2, 2, 64, (10, 90), 24, "random_branching"),
                                  ("f32", 1, 2, 64, (30, 60), 9, "random_parent")])
def test_sequence_based_decoding_matches_tree_attention(spec, case):
    dtype, B, H, D, P, N, tree = case
    cfg = wl.Config(93, "seq", dtype, B=B, H=H, D=D, P=P, N=N, tree=tree, widths=wl.EXPANSION_EVAL * 2)
    inp = wl.make_attention_inputs(cfg, seed=77 + N, S_cap=P[1] + N + 3)
    dev = lambda t: t.to(DEV)
    mp = int(inp["prefix_len"].max())
    args = [dev(inp[k][0]) for k in ("q", "k_new", "v_new", "k_cache", "v_cache")]
    seq = sb.SequenceBatch(*args, dev(inp["prefix_len"]), inp["tree_parent"].numpy(), mp)
    f64 = lambda t: t.double().numpy()
    kc, vc = f64(inp["k_cache"][0]), f64(inp["v_cache"][0])
    orc.kv_append(kc, vc, f64(inp["k_new"][0]), f64(inp["v_new"][0]), inp["prefix_len"].numpy())
    ref = orc.tree_attention(f64(inp["q"][0]), kc, vc, inp["tree_parent"].numpy(), inp["prefix_len"].numpy())
    for run in (seq.run_batched, seq.run_per_sequence):
        seq.out.zero_()
        run(spec)
        torch.cuda.synchronize()
        got = seq.tree_outputs().double().cpu().numpy()
        err = np.abs(got - ref)
        if dtype == "f32":
            assert err.max() <= 1e-5
        else:
            assert (err <= 2e-2 + 1e-2 * np.abs(ref)).all(), err.max()
    # each sequence's cache now holds prefix + its own tokens, in sequence order
    s0 = 0
    b0, ln = seq.dec.request[s0], seq.dec.length[s0]
    p0 = int(inp["prefix_len"][b0])
    want = inp["k_new"][0][b0, seq.dec.nodes[s0, :ln]].transpose(0, 1)          # [H, ln, D]
    assert torch.equal(seq.k_cache[s0, :, p0:p0 + ln].cpu(), want)
