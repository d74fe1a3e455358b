"""GPU-vs-oracle parity of token-tree construction (Section 3) through the C ABI: top-k expansion step and
token tree merge (Definition 3.2), bit-exact; and a flow that feeds a merged tree straight into attention,
verification and commit without visiting the host."""
import numpy as np
import pytest
import torch

from oracle import spec_oracle as orc
from paper_2305_09781_amd import workloads as wl
from test_oracle_tree_build import _random_trees

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(x):
    if isinstance(x, np.ndarray):
        x = torch.from_numpy(np.ascontiguousarray(x))
    return x.to(DEV)


@pytest.mark.parametrize("case", [(3, 4, 23, 5, "f32"), (2, 3, 32000, 3, "f32"), (2, 1, 777, 16, "bf16"), (1, 2, 5, 5, "f32")])
def test_expand_topk_matches_oracle(spec, case):
    B, F, V, k, dt = case
    rng = np.random.default_rng(V + k)
    logits = torch.from_numpy(np.round(rng.standard_normal((B, F, V)) * 3, 2).astype(np.float32))   # coarse: ties occur
    if dt == "bf16":
        logits = logits.to(torch.bfloat16)
    N = 1 + F * k + 2
    slots = torch.from_numpy(rng.permutation(np.arange(1, N))[:F * k].reshape(F, k).astype(np.int32))
    tok = torch.full((B, N), -5, dtype=torch.int32)
    want = tok.numpy().copy()
    picks = orc.expand_topk(logits.float().numpy(), k)
    for b in range(B):
        for f in range(F):
            want[b, slots[f].numpy()] = picks[b, f]
    got = spec.spec_tree_expand_topk(_dev(logits), k, _dev(slots), _dev(tok))
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), want)


def test_expand_topk_builds_the_evaluation_tree_level_by_level(spec):
    """Expansion configuration <1,1,3,1,1,1,1,1> truncated to 16 nodes: one call per level fills the tokens
    of a tree whose shape (parent array, child slots) is static."""
    cfg = wl.CONFIGS[2]
    parent = wl.make_trees(cfg, np.random.default_rng(0))[0]
    depth = wl.depth_of(parent)
    N, B, V = len(parent), 3, 512
    rng = np.random.default_rng(1)
    tok = torch.zeros((B, N), dtype=torch.int32, device=DEV)
    ref = np.zeros((B, N), dtype=np.int32)
    for level in range(int(depth.max())):
        frontier = [u for u in range(N) if depth[u] == level and any(parent[v] == u for v in range(N))]
        kids = [[v for v in range(N) if parent[v] == u] for u in frontier]
        k = max(len(c) for c in kids)
        if any(len(c) != k for c in kids):      # truncated level: expand the full-width nodes and the others separately
            groups = {}
            for u, c in zip(frontier, kids):
                groups.setdefault(len(c), []).append((u, c))
        else:
            groups = {k: list(zip(frontier, kids))}
        for kk, items in groups.items():
            logits = torch.from_numpy(rng.standard_normal((B, len(items), V)).astype(np.float32))
            slots = torch.tensor([c for _, c in items], dtype=torch.int32)
            spec.spec_tree_expand_topk(_dev(logits), kk, _dev(slots), tok)
            picks = orc.expand_topk(logits.numpy(), kk)
            for j, (_, c) in enumerate(items):
                ref[:, c] = picks[:, j]
    torch.cuda.synchronize()
    assert np.array_equal(tok.cpu().numpy(), ref)


def test_expand_topk_errors(spec):
    lg = torch.zeros((1, 1, 8), device=DEV)
    tok = torch.zeros((1, 4), dtype=torch.int32, device=DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    spec.spec_tree_expand_topk(lg, 2, torch.tensor([[1, 9]], dtype=torch.int32, device=DEV), tok, status=status)
    torch.cuda.synchronize()
    assert status.item() == orc.ST_BAD_TREE and tok.cpu().tolist() == [[0, 0, 0, 0]]
    with pytest.raises(spec.SpecError) as e:
        spec.spec_tree_expand_topk(lg, 9, torch.zeros((1, 9), dtype=torch.int32, device=DEV), tok)
    assert e.value.code == spec.ERR_UNSUPPORTED


@pytest.mark.parametrize("seed", range(8))
def test_tree_merge_matches_oracle(spec, seed):
    rng = np.random.default_rng(100 + seed)
    B = 5
    M, Nin = [(1, 1), (2, 7), (3, 16), (4, 40), (3, 128), (8, 128), (2, 33), (5, 9)][seed]
    V = [3, 4, 6, 50, 5, 3, 1000, 2][seed]
    Ps, Ts, Ss = [], [], []
    for b in range(B):
        P, T, S = _random_trees(rng, M, Nin, max(V, Nin))
        Ps.append(P); Ts.append(T); Ss.append(S)
    P, T, S = np.stack(Ps), np.stack(Ts), np.stack(Ss).astype(np.int32)
    refs = [orc.tree_merge(P[b], T[b], S[b], 128) for b in range(B)]
    n_out = min(128, max(r[4] for r in refs) + 3)
    refs = [orc.tree_merge(P[b], T[b], S[b], n_out) for b in range(B)]
    status = torch.zeros(B, dtype=torch.int32, device=DEV)
    par, dep, tok, ssm, size, node_map = spec.spec_tree_merge(_dev(P), _dev(T), _dev(S), n_out, status=status)
    torch.cuda.synchronize()
    for b in range(B):
        rp, rd, rt, rs, rsize, rmap, rst = refs[b]
        assert status[b].item() == rst
        assert size[b].item() == rsize
        assert np.array_equal(par[b].cpu().numpy(), rp) and np.array_equal(dep[b].cpu().numpy(), rd)
        assert np.array_equal(tok[b].cpu().numpy(), rt) and np.array_equal(ssm[b].cpu().numpy(), rs)
        assert np.array_equal(node_map[b].cpu().numpy(), rmap)


def test_tree_merge_status_cases(spec):
    P = np.array([[[-1, 0, 1], [-1, 0, 0]]] * 5, dtype=np.int32)
    T = np.array([[[1, 2, 3], [1, 4, 5]]] * 5, dtype=np.int32)
    S = np.array([[3, 3]] * 5, dtype=np.int32)
    T[1, 1, 0] = 9          # roots differ
    P[2, 0, 1] = 2          # parent after child
    S[3, 0] = 0             # empty tree
    T[4, 0, 2] = -1         # real node without a token
    for n_out, want in ((5, [0, 1, 1, 1, 1]), (4, [orc.ST_CAPACITY, 1, 1, 1, 1])):
        status = torch.zeros(5, dtype=torch.int32, device=DEV)
        par, dep, tok, ssm, size, node_map = spec.spec_tree_merge(_dev(P), _dev(T), _dev(S), n_out, status=status)
        torch.cuda.synchronize()
        assert status.cpu().tolist() == want
        for b in range(5):
            rp, rd, rt, rs, rsize, rmap, rst = orc.tree_merge(P[b], T[b], S[b], n_out)
            assert rst == want[b] and size[b].item() == rsize
            assert np.array_equal(par[b].cpu().numpy(), rp) and np.array_equal(tok[b].cpu().numpy(), rt)
            assert np.array_equal(dep[b].cpu().numpy(), rd) and np.array_equal(node_map[b].cpu().numpy(), rmap)
    with pytest.raises(spec.SpecError) as e:
        spec.spec_tree_merge(_dev(np.zeros((1, 9, 128), np.int32)), _dev(np.zeros((1, 9, 128), np.int32)),
                             _dev(np.ones((1, 9), np.int32)), 16)
    assert e.value.code == spec.ERR_UNSUPPORTED


def test_merged_tree_flows_into_attention_verification_and_commit(spec):
    """Three SSM trees per request -> merge on the device -> fused append + tree attention -> multi-step
    speculative sampling with out_ssm selecting the draft row -> commit; every stage against the oracle,
    padding nodes included."""
    rng = np.random.default_rng(7)
    B, M, Nin, V, H, D, n_out = 4, 3, 12, 64, 2, 128, 32
    Ps, Ts, Ss = zip(*[_random_trees(rng, M, Nin, V) for _ in range(B)])
    P, T, S = np.stack(Ps), np.stack(Ts), np.stack(Ss).astype(np.int32)
    par, dep, tok, ssm, size, _ = spec.spec_tree_merge(_dev(P), _dev(T), _dev(S), n_out)
    torch.cuda.synchronize()
    refs = [orc.tree_merge(P[b], T[b], S[b], n_out) for b in range(B)]
    rpar = np.stack([r[0] for r in refs]); rtok = np.stack([r[2] for r in refs]); rssm = np.stack([r[3] for r in refs])
    assert np.array_equal(par.cpu().numpy(), rpar) and np.array_equal(tok.cpu().numpy(), rtok)
    # attention over the merged (padded) tree
    cfg = wl.Config(99, "flow", "bf16", B=B, H=H, D=D, P=(20, 70), N=n_out, tree="random_parent")
    inp = wl.make_attention_inputs(cfg, seed=3, S_cap=70 + n_out)
    kc, vc = _dev(inp["k_cache"][0]), _dev(inp["v_cache"][0])
    out = spec.spec_tree_attention_append(_dev(inp["q"][0]), _dev(inp["k_new"][0]), _dev(inp["v_new"][0]), kc, vc, par, dep,
                                          _dev(inp["prefix_len"]), max_prefix_len=70)
    f64 = lambda t: t.double().numpy()
    kco, vco = f64(inp["k_cache"][0]), f64(inp["v_cache"][0])
    orc.kv_append(kco, vco, f64(inp["k_new"][0]), f64(inp["v_new"][0]), inp["prefix_len"].numpy())
    ref = orc.tree_attention(f64(inp["q"][0]), kco, vco, rpar, inp["prefix_len"].numpy())
    err = np.abs(out.double().cpu().numpy() - ref)
    assert (err <= 2e-2 + 1e-2 * np.abs(ref)).all()
    # verification: one draft row per (request, SSM); a node is tested against the SSM that proposed it
    logits = rng.standard_normal((B, n_out, V)).astype(np.float32) * 2
    probs = np.exp(rng.standard_normal((B * M, V)))
    probs = (probs / probs.sum(1, keepdims=True)).astype(np.float32)
    ssm_row = np.where(rssm >= 0, rssm + M * np.arange(B)[:, None], 0).astype(np.int32)
    ua, uo, uf = (rng.random((B, n_out), dtype=np.float32), rng.random((B, n_out), dtype=np.float32), rng.random(B, dtype=np.float32))
    from oracle import vetting
    ua, uf, _ = vetting.vet_uniforms(logits, probs, ssm_row, rtok, rpar, ua, uo, uf, rng)
    rp, rl, rt, rs = orc.verify_stochastic(logits, probs, ssm_row, rtok, rpar, ua, uo, uf)
    path, ln, toks = spec.spec_verify_stochastic(_dev(logits), _dev(probs), _dev(ssm_row), tok, par, _dev(ua), _dev(uo), _dev(uf))
    torch.cuda.synchronize()
    assert np.array_equal(path.cpu().numpy(), rp) and np.array_equal(ln.cpu().numpy(), rl) and np.array_equal(toks.cpu().numpy(), rt)
    sz = size.cpu().numpy()
    for b in range(B):
        assert all(0 <= n < sz[b] for n in rp[b, :rl[b]])            # padding nodes are never on the accepted path
    gp, gl, gt, _ = orc.verify_greedy(logits, rtok, rpar)
    path_g, ln_g, toks_g, _ = spec.spec_verify_greedy(_dev(logits), tok, par)
    torch.cuda.synchronize()
    assert np.array_equal(path_g.cpu().numpy(), gp) and np.array_equal(toks_g.cpu().numpy(), gt)
    # commit of the accepted path
    new_len = spec.spec_kv_commit([kc], [vc], path, ln, _dev(inp["prefix_len"]), N=n_out)
    torch.cuda.synchronize()
    kb = inp["k_cache"][0].view(torch.int16).numpy().copy()
    vb = inp["v_cache"][0].view(torch.int16).numpy().copy()
    orc.kv_append(kb, vb, inp["k_new"][0].view(torch.int16).numpy(), inp["v_new"][0].view(torch.int16).numpy(), inp["prefix_len"].numpy())
    rlen, rst = orc.kv_commit([kb], [vb], rp, rl, inp["prefix_len"].numpy(), N=n_out)
    assert np.array_equal(new_len.cpu().numpy(), rlen) and (rst == 0).all()
    for b in range(B):
        assert np.array_equal(kc[b, :, :rlen[b]].view(torch.int16).cpu().numpy(), kb[b, :, :rlen[b]])
        assert np.array_equal(vc[b, :, :rlen[b]].view(torch.int16).cpu().numpy(), vb[b, :, :rlen[b]])
