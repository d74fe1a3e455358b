"""Pins for the oracle's rotary-embedding append (a step adjacent to the path: the paper's LLaMA models
rotate keys by position; tree tokens sit at prefix_len + depth). CPU only. The rotation is pinned to complex
multiplication written separately, to its group properties and to the plain append at angle zero."""
import numpy as np
import pytest
import torch

from oracle import spec_oracle as orc
from paper_2305_09781_amd import workloads as wl


def test_rotation_is_complex_multiplication_and_preserves_norms():
    rng = np.random.default_rng(0)
    D = 16
    x = rng.standard_normal((3, D))
    ang = rng.uniform(-7, 7, size=D // 2)
    got = orc.rope_rotate(x, np.cos(ang), np.sin(ang))
    z = (x[:, :D // 2] + 1j * x[:, D // 2:]) * np.exp(1j * ang)           # pair (j, j + D/2) as a complex number
    assert np.allclose(got[:, :D // 2], z.real, atol=1e-14) and np.allclose(got[:, D // 2:], z.imag, atol=1e-14)
    assert np.allclose((got ** 2).sum(-1), (x ** 2).sum(-1))
    quarter = orc.rope_rotate(x, np.zeros(D // 2), np.ones(D // 2))      # 90 degrees: (a, b) -> (-b, a)
    assert np.array_equal(quarter[:, :D // 2], -x[:, D // 2:]) and np.array_equal(quarter[:, D // 2:], x[:, :D // 2])
    back = orc.rope_rotate(got, np.cos(-ang), np.sin(-ang))
    assert np.allclose(back, x, atol=1e-13)


def test_rounding_to_the_storage_type_is_one_rounding_to_nearest_even():
    """bfloat16 keeps 8 significant bits: hand-derived cases, among them a value that rounding through float32
    first would get wrong, and agreement with a library conversion of values that float32 holds exactly."""
    r = lambda x: float(orc.round_to_storage(np.array([x]), "bf16")[0])
    assert r(1.0) == 1.0 and r(-0.15625) == -0.15625 and r(0.0) == 0.0
    assert r(1.0 + 2.0 ** -8) == 1.0                       # a tie: to the even neighbour (down)
    assert r(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6       # a tie: to the even neighbour (up)
    assert r(1.0 + 2.0 ** -8 + 2.0 ** -30) == 1.0 + 2.0 ** -7   # just above the tie
    assert r(-(3.0 + 2.0 ** -7)) == -3.0 and r(-(3.0 + 3 * 2.0 ** -7)) == -(3.0 + 2.0 ** -5)   # spacing 2^-6 in [2, 4)
    # 1 + 2^-8 + 2^-40 lies above the tie; float32 first rounds it onto the tie, which then goes down: double rounding
    x = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert r(x) == 1.0 + 2.0 ** -7
    assert float(torch.tensor([x], dtype=torch.float64).to(torch.float32).to(torch.bfloat16).double()[0]) == 1.0
    rng = np.random.default_rng(3)
    v = rng.standard_normal(4000).astype(np.float32) * np.float32(10.0) ** rng.integers(-3, 4, 4000).astype(np.float32)
    assert np.array_equal(orc.round_to_storage(v.astype(np.float64), "bf16"), torch.from_numpy(v).to(torch.bfloat16).double().numpy())
    w = rng.standard_normal(100)
    assert np.array_equal(orc.round_to_storage(w, "f32"), w.astype(np.float32).astype(np.float64))


def test_scores_depend_only_on_relative_position():
    """The property rotary embeddings exist for: <R(m) q, R(n) k> is a function of m - n."""
    rng = np.random.default_rng(1)
    D = 32
    cos, sin = (t.double().numpy() for t in wl.make_rope_tables(64, D))
    q, k = rng.standard_normal(D), rng.standard_normal(D)
    ref = orc.rope_rotate(q, cos[9], sin[9]) @ orc.rope_rotate(k, cos[4], sin[4])
    for m, n in ((5, 0), (30, 25), (63, 58)):
        assert abs(orc.rope_rotate(q, cos[m], sin[m]) @ orc.rope_rotate(k, cos[n], sin[n]) - ref) < 1e-5
    assert abs(orc.rope_rotate(q, cos[9], sin[9]) @ orc.rope_rotate(k, cos[5], sin[5]) - ref) > 1e-3
    # table generator: position 0 is the identity, frequency 0 advances one radian per position
    assert np.array_equal(cos[0], np.ones(D // 2)) and np.array_equal(sin[0], np.zeros(D // 2))
    assert abs(cos[3, 0] - np.cos(3.0)) < 1e-7 and abs(sin[3, D // 2 - 1] - np.sin(3.0 * 10000.0 ** (-(D - 2) / D))) < 1e-7


@pytest.mark.parametrize("storage", ["bf16", "f32"])
def test_append_with_rotation_positions_rounding_and_status(storage):
    cfg = wl.Config(95, "rope", storage, B=3, H=2, D=16, P=(3, 9), N=6, tree="random_parent")
    inp = wl.make_attention_inputs(cfg, seed=4, S_cap=9 + 6)
    f64 = lambda t: t.double().numpy()
    kn, vn = f64(inp["k_new"][0]), f64(inp["v_new"][0])
    pl, dep = inp["prefix_len"].numpy(), inp["tree_depth"].numpy()
    cos, sin = wl.make_rope_tables(9 + 6, cfg.D)
    # all-zero angles: exactly the plain append
    kc, vc = f64(inp["k_cache"][0]), f64(inp["v_cache"][0])
    kc0, vc0 = kc.copy(), vc.copy()
    orc.kv_append(kc0, vc0, kn, vn, pl)
    st = orc.kv_append_rope(kc, vc, kn, vn, pl, dep, np.ones((15, 8)), np.zeros((15, 8)), storage)
    assert (st == 0).all() and np.array_equal(kc, kc0) and np.array_equal(vc, vc0)
    # real tables: row p+i holds k_new[i] rotated by position p + depth[i] (not p + i), rounded to the storage type
    kc, vc = f64(inp["k_cache"][0]), f64(inp["v_cache"][0])
    st = orc.kv_append_rope(kc, vc, kn, vn, pl, dep, cos, sin, storage)
    assert (st == 0).all() and np.array_equal(vc, vc0)
    dt = torch.bfloat16 if storage == "bf16" else torch.float32
    for b in range(cfg.B):
        for i in range(cfg.N):
            pos = pl[b] + dep[b, i]
            z = (kn[b, i, :, :8] + 1j * kn[b, i, :, 8:]) * np.exp(1j * np.arctan2(f64(sin)[pos], f64(cos)[pos]))
            want = torch.from_numpy(np.concatenate([z.real, z.imag], -1)).to(dt).double().numpy()
            got = kc[b, :, pl[b] + i]
            assert np.abs(got - want).max() <= (2.0 ** -7 if storage == "bf16" else 2e-6) * np.abs(want).max()
            assert np.array_equal(torch.from_numpy(got).to(dt).double().numpy(), got)      # representable in the storage type
    siblings = [(i, j) for i in range(cfg.N) for j in range(i) if dep[0, i] == dep[0, j]]
    assert siblings, "the tree should have two nodes of equal depth (same position, different rows)"
    # a position outside the tables or a tree that does not fit: request untouched, flagged
    kc = f64(inp["k_cache"][0])
    before = kc.copy()
    st = orc.kv_append_rope(kc, vc, kn, vn, pl, dep, cos[:int(pl.max())], sin[:int(pl.max())], storage)
    assert st[np.argmax(pl)] == orc.ST_CAPACITY and np.array_equal(kc[np.argmax(pl)], before[np.argmax(pl)])


@pytest.mark.parametrize("storage", ["bf16", "f32"])
def test_query_rotation_positions_rounding_and_status(storage):
    cfg = wl.Config(95, "ropeq", storage, B=3, H=2, D=16, P=(3, 9), N=6, tree="random_parent")
    inp = wl.make_attention_inputs(cfg, seed=5, S_cap=9 + 6)
    q = inp["q"][0].double().numpy()
    pl, dep = inp["prefix_len"].numpy(), inp["tree_depth"].numpy()
    cos, sin = (t.double().numpy() for t in wl.make_rope_tables(15, cfg.D))
    same, st = orc.rope_queries(q, pl, dep, np.ones((15, 8)), np.zeros((15, 8)), 15, storage)
    assert (st == 0).all() and np.array_equal(same, q)                         # angle zero: untouched
    got, st = orc.rope_queries(q, pl, dep, cos, sin, 15, storage)
    assert (st == 0).all() and not np.array_equal(got, q)
    dt = torch.bfloat16 if storage == "bf16" else torch.float32
    for b in range(cfg.B):
        for i in range(cfg.N):
            pos = pl[b] + dep[b, i]                                            # the depth, not the row index
            z = (q[b, i, :, :8] + 1j * q[b, i, :, 8:]) * np.exp(1j * np.arctan2(sin[pos], cos[pos]))
            want = np.concatenate([z.real, z.imag], -1)
            assert np.abs(got[b, i] - want).max() <= (2.0 ** -7 if storage == "bf16" else 2e-6) * np.abs(want).max()
    assert np.array_equal(torch.from_numpy(got).to(dt).double().numpy(), got)
    assert np.array_equal(q, inp["q"][0].double().numpy())                     # the input is not modified
    # tables too short for the longest request, or a tree that does not fit: that request keeps its q
    short = int(pl.max())
    got, st = orc.rope_queries(q, pl, dep, cos[:short], sin[:short], 15, storage)
    worst = int(np.argmax(pl))
    assert st[worst] == orc.ST_CAPACITY and np.array_equal(got[worst], q[worst])
    _, st = orc.rope_queries(q, pl, dep, cos, sin, int(pl.max()) + cfg.N - 1, storage)
    assert st[worst] == orc.ST_CAPACITY
    # the same flags as the key side
    kc, vc = inp["k_cache"][0].double().numpy(), inp["v_cache"][0].double().numpy()
    st_k = orc.kv_append_rope(kc, vc, inp["k_new"][0].double().numpy(), inp["v_new"][0].double().numpy(), pl, dep,
                              cos[:short], sin[:short], storage)
    _, st_q = orc.rope_queries(q, pl, dep, cos[:short], sin[:short], 15, storage)
    assert np.array_equal(st_k, st_q)


def test_tree_attention_with_rotated_q_and_k_depends_on_relative_positions_only():
    """No prefix, queries and keys both rotated: moving every position by the same offset (tables read from row
    s on) leaves the tree attention output alone, up to the float32 rounding of the rotated operands; rotating
    only one side does not."""
    cfg = wl.Config(95, "ropeqa", "f32", B=2, H=2, D=16, P=0, N=7, tree="random_parent")
    inp = wl.make_attention_inputs(cfg, seed=6, S_cap=8)
    f64 = lambda t: t.double().numpy()
    q, kn, vn = f64(inp["q"][0]), f64(inp["k_new"][0]), f64(inp["v_new"][0])
    pl, dep, par = inp["prefix_len"].numpy(), inp["tree_depth"].numpy(), inp["tree_parent"].numpy()
    cos, sin = (f64(t) for t in wl.make_rope_tables(40, cfg.D))

    def run(s, rotate_q=True):
        kc, vc = f64(inp["k_cache"][0]), f64(inp["v_cache"][0])
        assert (orc.kv_append_rope(kc, vc, kn, vn, pl, dep, cos[s:], sin[s:], "f32") == 0).all()
        qr = orc.rope_queries(q, pl, dep, cos[s:], sin[s:], 8, "f32")[0] if rotate_q else q
        return orc.tree_attention(qr, kc, vc, par, pl)

    base = run(0)
    for s in (1, 5, 30):
        assert np.abs(run(s) - base).max() < 2e-5
    assert np.abs(run(5, rotate_q=False) - run(0, rotate_q=False)).max() > 1e-3
    kc, vc = f64(inp["k_cache"][0]), f64(inp["v_cache"][0])
    orc.kv_append(kc, vc, kn, vn, pl)
    assert np.abs(orc.tree_attention(q, kc, vc, par, pl) - base).max() > 1e-3   # the embedding does something
