"""spec_tree_attention_append_static (the entry point that allocates nothing) against spec_tree_attention_append
through the C ABI: same kernels, same launch plan, so outputs and caches must agree bit for bit, and both stay
within the bf16 bar of the oracle. Two calls in a row per shape pair, the second with a smaller input, so the
library's scratch array still holds the first call's partial results when the second runs."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import spec_oracle as orc
from paper_2305_09781_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(t):
    return t.to(DEV)


def _bits(t):
    return t.cpu().contiguous().view(torch.int16).numpy()


def _inputs(B, H, P, N, tree, seed):
    cfg = wl.Config(86, "static", "bf16", B=B, H=H, D=128, P=P if P[0] != P[1] else P[0], N=N, tree=tree,
                    widths=wl.EXPANSION_EVAL * 2)
    return wl.make_attention_inputs(cfg, seed=seed, S_cap=P[1] + N + 3)


def _both_ways(spec, inp):
    """(out, k_cache, v_cache) from the workspace entry point and from the static one, on fresh copies."""
    res = []
    par, dep, pl = _dev(inp["tree_parent"]), _dev(inp["tree_depth"]), _dev(inp["prefix_len"])
    mp = int(inp["prefix_len"].max())
    for static in (False, True):
        q, kn, vn = _dev(inp["q"][0]), _dev(inp["k_new"][0]), _dev(inp["v_new"][0])
        kc, vc = _dev(inp["k_cache"][0]), _dev(inp["v_cache"][0])
        status = torch.zeros(q.shape[0], dtype=torch.int32, device=DEV)
        if static:
            out = torch.full_like(q, 7.0)
            spec.spec_tree_attention_append_static(q, kn, vn, kc, vc, par, dep, pl, out, status=status, max_prefix_len=mp)
        else:
            out = spec.spec_tree_attention_append(q, kn, vn, kc, vc, par, dep, pl, status=status, max_prefix_len=mp)
        torch.cuda.synchronize()
        assert (status.cpu().numpy() == 0).all()
        res.append((out, kc, vc))
    return res


def _oracle(inp):
    f64 = lambda t: t.double().numpy()
    kc, vc = f64(inp["k_cache"][0]), f64(inp["v_cache"][0])
    pl = inp["prefix_len"].numpy()
    assert (orc.kv_append(kc, vc, f64(inp["k_new"][0]), f64(inp["v_new"][0]), pl) == 0).all()
    return orc.tree_attention(f64(inp["q"][0]), kc, vc, inp["tree_parent"].numpy(), pl), kc, vc


PAIRS = [
    # first call, then a smaller one: (B, H, (P lo, hi), N, tree)
    ((1, 4, (700, 700), 16, "expansion"), (1, 2, (300, 300), 16, "expansion")),                   # fixed chunks, few-query kernel
    ((2, 2, (300, 1100), 64, "random_branching"), (1, 2, (280, 280), 40, "random_branching")),    # wide kernel
    ((2, 4, (3000, 5000), 32, "expansion"), (2, 2, (2100, 2600), 17, "random_branching")),        # several requests, long shares
    ((2, 3, (40, 90), 16, "random_parent"), (1, 3, (10, 10), 5, "random_parent")),                # whole key ranges: no scratch used
]


@pytest.mark.parametrize("pair", PAIRS, ids=lambda p: f"B{p[0][0]}H{p[0][1]}P{p[0][2][1]}N{p[0][3]}-then-B{p[1][0]}H{p[1][1]}P{p[1][2][1]}N{p[1][3]}")
def test_static_scratch_entry_point_matches_the_workspace_one(spec, pair):
    for i, (B, H, P, N, tree) in enumerate(pair):
        inp = _inputs(B, H, P, N, tree, seed=8600 + 10 * N + i)
        (o_ws, k_ws, v_ws), (o_st, k_st, v_st) = _both_ways(spec, inp)
        assert np.array_equal(_bits(o_st), _bits(o_ws)), f"call {i}: outputs differ"
        assert np.array_equal(_bits(k_st), _bits(k_ws)) and np.array_equal(_bits(v_st), _bits(v_ws)), f"call {i}: caches differ"
        ref, kco, vco = _oracle(inp)
        err = np.abs(o_st.double().cpu().numpy() - ref)
        assert (err <= 2e-2 + 1e-2 * np.abs(ref)).all(), f"call {i}: max abs err {err.max():.3e}"
        assert np.array_equal(k_st.double().cpu().numpy(), kco) and np.array_equal(v_st.double().cpu().numpy(), vco)


def test_static_scratch_entry_point_flags_and_rejects(spec):
    """Status handling is the workspace call's; a shape whose plan needs more than the array is refused on the
    host (no launch), and so is a missing k_new."""
    inp = _inputs(2, 2, (300, 1100), 33, "random_branching", seed=8700)
    inp["tree_parent"][0, 20] = 25
    par, dep, pl = _dev(inp["tree_parent"]), _dev(inp["tree_depth"]), _dev(inp["prefix_len"])
    q, kn, vn = _dev(inp["q"][0]), _dev(inp["k_new"][0]), _dev(inp["v_new"][0])
    kc, vc = _dev(inp["k_cache"][0]), _dev(inp["v_cache"][0])
    status = torch.zeros(2, dtype=torch.int32, device=DEV)
    out = torch.full_like(q, 7.0)
    spec.spec_tree_attention_append_static(q, kn, vn, kc, vc, par, dep, pl, out, status=status, max_prefix_len=1100)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [orc.ST_BAD_TREE, 0] and (out[0].float() == 0).all()
    f64 = lambda t: t.double().numpy()
    kco, vco = f64(inp["k_cache"][0][1:]), f64(inp["v_cache"][0][1:])
    orc.kv_append(kco, vco, f64(inp["k_new"][0][1:]), f64(inp["v_new"][0][1:]), inp["prefix_len"].numpy()[1:])
    ref = orc.tree_attention(f64(inp["q"][0][1:]), kco, vco, inp["tree_parent"].numpy()[1:], inp["prefix_len"].numpy()[1:])
    err = np.abs(out[1:].double().cpu().numpy() - ref)
    assert (err <= 2e-2 + 1e-2 * np.abs(ref)).all()
    d = spec.make_desc(q, kc, max_prefix_len=1100, k_new=kn)
    ptr = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = spec.load().spec_tree_attention_append_static(ctypes.byref(d), ptr(q), None, None, ptr(kc), ptr(vc), ptr(par),
                                                       ptr(dep), ptr(pl), ptr(out), None, None)
    assert rc == spec.ERR_INVALID_ARG
