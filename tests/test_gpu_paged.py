"""GPU-vs-oracle parity of the paged-cache entry points through the C ABI (needs an MI355X: `pytest -m gpu`).

The cache of every layer is a pool of blocks behind a block table; the steps are those of the contiguous
entry points. Bars as there: attention max-abs 1e-5 (float32 inputs), |g-o| <= 2e-2 + 1e-2*|o| (bf16 inputs,
oracle in float64, not rounded); append and commit bit-exact over the WHOLE pool (so a row written to a wrong
block shows up), status words equal."""
import numpy as np
import pytest
import torch

from oracle import spec_oracle as orc
from paper_2305_09781_amd import workloads as wl
from test_gpu_parity import DEV, _balanced_wgs, _bits, _check_attention, _chunk_keys, _dev, _f64, _oracle_append_attention, _plan

pytestmark = pytest.mark.gpu


def _paged_inputs(dtype, B, H, H_kv, D, P, N, tree, bt, seed, max_blocks=None, unused_entry=-1):
    cfg = wl.Config(93, "paged", dtype, B=B, H=H, D=D, P=P if P[0] != P[1] else P[0], N=N, tree=tree,
                    widths=wl.EXPANSION_EVAL * 16, H_kv=H_kv)
    S = ((P[1] + N + bt - 1) // bt) * bt
    inp = wl.make_attention_inputs(cfg, seed=seed, S_cap=S)
    rng = np.random.default_rng(seed + 17)
    pools, table = wl.to_paged([inp["k_cache"][0], inp["v_cache"][0]], inp["prefix_len"].numpy(), N, bt, rng,
                               max_blocks=max_blocks, unused_entry=unused_entry)
    return cfg, inp, pools[0], pools[1], table


PAGED_ATTENTION = [
    # dtype, B, H, H_kv, D, (P lo, hi), N, tree, block_tokens, forced chunk, balanced workgroups
    ("bf16", 3, 4, 4, 128, (100, 400), 16, "expansion", 64, 0, 0),          # one query tile, blocks of one key tile
    ("bf16", 3, 4, 4, 128, (100, 400), 16, "expansion", 128, 96, 0),        # chunks (rounded up to a tile multiple)
    ("bf16", 2, 4, 4, 64, (0, 300), 7, "random_parent", 64, 0, 7),          # balanced deal, empty prefix possible
    ("bf16", 2, 8, 2, 128, (60, 330), 40, "random_branching", 64, 0, 0),    # grouped heads, tree rows cross a block
    ("bf16", 2, 2, 2, 128, (190, 260), 128, "random_branching", 256, 0, 0), # widest tree, one block holds many tiles
    ("bf16", 2, 2, 2, 128, (130, 700), 64, "expansion", 128, 128, 0),       # four-wavefront shape, chunks
    ("bf16", 4, 2, 1, 128, (0, 520), 33, "random_parent", 64, 0, 9),        # balanced, grouped, ragged
    ("f32", 2, 3, 3, 64, (30, 200), 12, "random_parent", 64, 0, 0),
    ("f32", 2, 4, 2, 128, (30, 200), 20, "expansion", 128, 64, 0),
]


@pytest.mark.parametrize("case", PAGED_ATTENTION, ids=lambda c: f"{c[0]}-B{c[1]}-H{c[2]}/{c[3]}-N{c[6]}-bt{c[8]}-c{c[9]}-w{c[10]}")
@pytest.mark.parametrize("fused", [False, True])
def test_paged_append_and_attention(spec, case, fused):
    dtype, B, H, H_kv, D, P, N, tree, bt, chunk, wgs = case
    # entries of blocks a request does not reach may hold anything: a huge value must be neither used nor flagged
    cfg, inp, kp, vp, table = _paged_inputs(dtype, B, H, H_kv, D, P, N, tree, bt, seed=500 + N + bt, unused_entry=1 << 30)
    pl, par = inp["prefix_len"].numpy(), inp["tree_parent"].numpy()
    kpo, vpo = _f64(kp), _f64(vp)
    st_ref = orc.kv_append_paged(kpo, vpo, table.numpy(), bt, table.shape[1] * bt, _f64(inp["k_new"][0]),
                                 _f64(inp["v_new"][0]), pl)
    ref = orc.tree_attention_paged(_f64(inp["q"][0]), kpo, vpo, table.numpy(), bt, par, pl)
    assert (st_ref == 0).all()
    kpd, vpd, tab = _dev(kp), _dev(vp), _dev(table)
    status = torch.zeros(B, dtype=torch.int32, device=DEV)
    args = (tab, _dev(inp["tree_parent"]), _dev(inp["tree_depth"]), _dev(inp["prefix_len"]))
    kn, vn = _dev(inp["k_new"][0]), _dev(inp["v_new"][0])
    with _chunk_keys(chunk), _balanced_wgs(wgs):
        if fused:
            out = spec.spec_tree_attention_append_paged(_dev(inp["q"][0]), kn, vn, kpd, vpd, *args, status=status,
                                                        max_prefix_len=int(pl.max()), plan=_plan())
        else:
            spec.spec_kv_append_paged(kn, vn, kpd, vpd, tab, _dev(inp["prefix_len"]), status=status)
            out = spec.spec_tree_attention_paged(_dev(inp["q"][0]), kpd, vpd, *args, status=status,
                                                 max_prefix_len=int(pl.max()), plan=_plan())
    torch.cuda.synchronize()
    assert (status.cpu().numpy() == 0).all()
    # the whole pool, bit for bit: the appended rows are in place and nothing else moved
    assert np.array_equal(kpd.double().cpu().numpy(), kpo) and np.array_equal(vpd.double().cpu().numpy(), vpo)
    _check_attention(out, ref, inp["q"][0].dtype)


@pytest.mark.parametrize("seed", range(24))
def test_randomised_paged_shapes_and_plans(spec, seed):
    """Random small shapes (grouped heads, head dim, tree size, ragged prefixes down to zero, block sizes) under a
    random launch plan, fused or not, some requests sharing their prefix blocks: parity, the pool bit for bit."""
    rng = np.random.default_rng(7000 + seed)
    dtype = "bf16" if rng.random() < 0.8 else "f32"
    D = int(rng.choice([64, 128]))
    H_kv = int(rng.integers(1, 4))
    N = int(rng.choice([1, 5, 16, 17, 32, 33, 64, 65, 100, 128]))
    group = int(rng.integers(1, 9)) if rng.random() < 0.3 else int(rng.integers(1, 3))
    B = int(rng.integers(1, 5))
    hi = int(rng.choice([0, 40, 130, 400, 700]))
    lo = int(rng.integers(0, hi + 1))
    bt = int(rng.choice([64, 128, 512]))
    tree = str(rng.choice(["random_parent", "random_branching", "expansion"]))
    cfg, inp, kp, vp, table = _paged_inputs(dtype, B, H_kv * group, H_kv, D, (lo, hi), N, tree, bt, seed=8000 + seed,
                                            unused_entry=int(rng.choice([-1, 1 << 30, -(1 << 31)])))
    pl, par = inp["prefix_len"].numpy(), inp["tree_parent"].numpy()
    plan = int(rng.integers(0, 3))
    chunk = int(rng.choice([32, 64, 96, 160])) if plan == 1 else 0
    wgs = int(rng.integers(1, 12)) if plan == 2 and dtype == "bf16" else 0
    fused = bool(rng.integers(0, 2))
    kpo, vpo = _f64(kp), _f64(vp)
    st_ref = orc.kv_append_paged(kpo, vpo, table.numpy(), bt, table.shape[1] * bt, _f64(inp["k_new"][0]),
                                 _f64(inp["v_new"][0]), pl)
    ref = orc.tree_attention_paged(_f64(inp["q"][0]), kpo, vpo, table.numpy(), bt, par, pl)
    assert (st_ref == 0).all()
    kpd, vpd, tab = _dev(kp), _dev(vp), _dev(table)
    status = torch.zeros(B, dtype=torch.int32, device=DEV)
    args = (tab, _dev(inp["tree_parent"]), _dev(inp["tree_depth"]), _dev(inp["prefix_len"]))
    kn, vn = _dev(inp["k_new"][0]), _dev(inp["v_new"][0])
    with _chunk_keys(chunk), _balanced_wgs(wgs):
        if fused:
            out = spec.spec_tree_attention_append_paged(_dev(inp["q"][0]), kn, vn, kpd, vpd, *args, status=status,
                                                        max_prefix_len=int(pl.max()), plan=_plan())
        else:
            spec.spec_kv_append_paged(kn, vn, kpd, vpd, tab, _dev(inp["prefix_len"]), status=status)
            out = spec.spec_tree_attention_paged(_dev(inp["q"][0]), kpd, vpd, *args, status=status,
                                                 max_prefix_len=int(pl.max()), plan=_plan())
    torch.cuda.synchronize()
    assert (status.cpu().numpy() == 0).all()
    assert np.array_equal(kpd.double().cpu().numpy(), kpo) and np.array_equal(vpd.double().cpu().numpy(), vpo)
    _check_attention(out, ref, inp["q"][0].dtype)


@pytest.mark.parametrize("c,bt", [(2, 64), (3, 128), (4, 128), (5, 256)])
def test_full_size_configs_paged_every_request_and_head(spec, c, bt):
    """The benchmark's shapes with the caches scattered over a pool (fused append + attention), compared with
    the oracle on every (request, head) pair on the logical caches the pool stands for, request by request;
    the appended rows are read back through the table, bit for bit."""
    cfg = wl.CONFIGS[c]
    inp = wl.make_attention_inputs(cfg)
    pl = inp["prefix_len"].numpy()
    pools, table = wl.to_paged([inp["k_cache"][0], inp["v_cache"][0]], pl, cfg.N, bt, np.random.default_rng(c))
    kpd, vpd = _dev(pools[0]), _dev(pools[1])
    status = torch.zeros(cfg.B, dtype=torch.int32, device=DEV)
    out = spec.spec_tree_attention_append_paged(_dev(inp["q"][0]), _dev(inp["k_new"][0]), _dev(inp["v_new"][0]), kpd, vpd,
                                                _dev(table), _dev(inp["tree_parent"]), _dev(inp["tree_depth"]),
                                                _dev(inp["prefix_len"]), status=status, max_prefix_len=int(pl.max()))
    torch.cuda.synchronize()
    assert (status.cpu().numpy() == 0).all()
    out_h, kp_host, vp_host, tab = out.cpu(), kpd.cpu(), vpd.cpu(), table.numpy()
    for b in range(cfg.B):
        ref, kco, vco = _oracle_append_attention(inp, bsel=[b])
        _check_attention(out_h[b:b + 1], ref, torch.bfloat16)
        for s_ in range(int(pl[b]), int(pl[b]) + cfg.N):          # the appended rows, read back through the table
            e, r = int(tab[b, s_ // bt]), s_ % bt
            assert np.array_equal(kp_host[e, :, r].double().numpy(), kco[0, :, s_])
            assert np.array_equal(vp_host[e, :, r].double().numpy(), vco[0, :, s_])


def test_paged_equals_contiguous_on_the_device(spec):
    """Same logical caches, contiguous and paged: the wide kernel serves both, so the outputs agree closely
    (identical arithmetic per tile; only the few-query kernel of the contiguous call may order sums differently)."""
    cfg, inp, kp, vp, table = _paged_inputs("bf16", 3, 4, 4, 128, (100, 500), 48, "random_branching", 64, seed=77)
    pl = inp["prefix_len"]
    common = (_dev(inp["tree_parent"]), _dev(inp["tree_depth"]), _dev(pl))
    kn, vn = _dev(inp["k_new"][0]), _dev(inp["v_new"][0])
    out_c = spec.spec_tree_attention_append(_dev(inp["q"][0]), kn, vn, _dev(inp["k_cache"][0]), _dev(inp["v_cache"][0]),
                                            *common, max_prefix_len=int(pl.max()))
    out_p = spec.spec_tree_attention_append_paged(_dev(inp["q"][0]), kn, vn, _dev(kp), _dev(vp), _dev(table), *common,
                                                  max_prefix_len=int(pl.max()))
    torch.cuda.synchronize()
    assert np.array_equal(_bits(out_c), _bits(out_p))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_paged_commit_bit_exact(spec, dtype):
    B, H, D, N, bt, L = 4, 3, 64, 24, 64, 3
    cfg = wl.Config(92, "pcommit", dtype, B=B, H=H, D=D, P=(50, 300), N=N, tree="random_branching")
    inp = wl.make_attention_inputs(cfg, seed=41, n_layers=L, S_cap=384)
    rng = np.random.default_rng(5)
    pl, par = inp["prefix_len"].numpy(), inp["tree_parent"].numpy()
    caches = [c for l in range(L) for c in (inp["k_cache"][l], inp["v_cache"][l])]
    pools, table = wl.to_paged(caches, pl, N, bt, rng)
    path, ln = wl.random_accepted_paths(rng, par, max_len=9)
    path[1, :3], ln[1] = [0, 2, 1], 3                           # malformed: untouched, flagged
    kpo = [_bits(p).copy() for p in pools[0::2]]
    vpo = [_bits(p).copy() for p in pools[1::2]]
    out_ref, st_ref = orc.kv_commit_paged(kpo, vpo, table.numpy(), bt, table.shape[1] * bt, path, ln, pl, N)
    kd, vd = [_dev(p) for p in pools[0::2]], [_dev(p) for p in pools[1::2]]
    status = torch.zeros(B, dtype=torch.int32, device=DEV)
    out = spec.spec_kv_commit_paged(kd, vd, _dev(table), _dev(path), _dev(ln), _dev(inp["prefix_len"]), N, status=status)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), out_ref) and np.array_equal(status.cpu().numpy(), st_ref)
    assert st_ref[1] == orc.ST_BAD_PATH
    for l in range(L):
        # rows at and beyond the new prefix length are unspecified: compare through the table up to it, and the
        # blocks no request's tree rows touch bit for bit
        n_rows = out_ref
        assert np.array_equal(orc.paged_gather(_bits(kd[l]), table.numpy(), bt, n_rows),
                              orc.paged_gather(kpo[l], table.numpy(), bt, n_rows))
        assert np.array_equal(orc.paged_gather(_bits(vd[l]), table.numpy(), bt, n_rows),
                              orc.paged_gather(vpo[l], table.numpy(), bt, n_rows))
        tree_blocks = {int(table[b, j]) for b in range(B) for j in range(int(pl[b]) // bt, (int(pl[b]) + N - 1) // bt + 1)}
        for e in set(range(pools[0].shape[0])) - tree_blocks:
            assert np.array_equal(_bits(kd[l][e]), _bits(pools[2 * l][e]))


def test_paged_rope_append(spec):
    B, H, D, N, bt = 3, 2, 128, 20, 64
    cfg = wl.Config(91, "prope", "bf16", B=B, H=H, D=D, P=(40, 200), N=N, tree="random_branching")
    inp = wl.make_attention_inputs(cfg, seed=9, S_cap=256)
    pools, table = wl.to_paged([inp["k_cache"][0], inp["v_cache"][0]], inp["prefix_len"].numpy(), N, bt,
                               np.random.default_rng(2))
    cos, sin = wl.make_rope_tables(256, D)
    kco, vco = _f64(inp["k_cache"][0]), _f64(inp["v_cache"][0])
    orc.kv_append_rope(kco, vco, _f64(inp["k_new"][0]), _f64(inp["v_new"][0]), inp["prefix_len"].numpy(),
                       inp["tree_depth"].numpy(), cos.numpy(), sin.numpy(), "bf16")
    kpd, vpd = _dev(pools[0]), _dev(pools[1])
    status = torch.zeros(B, dtype=torch.int32, device=DEV)
    spec.spec_kv_append_rope_paged(_dev(inp["k_new"][0]), _dev(inp["v_new"][0]), kpd, vpd, _dev(table),
                                   _dev(inp["tree_depth"]), _dev(inp["prefix_len"]), _dev(cos), _dev(sin), status=status)
    torch.cuda.synchronize()
    assert (status.cpu().numpy() == 0).all()
    n_rows = inp["prefix_len"].numpy() + N
    got_k = orc.paged_gather(kpd.double().cpu().numpy(), table.numpy(), bt, n_rows)
    got_v = orc.paged_gather(vpd.double().cpu().numpy(), table.numpy(), bt, n_rows)
    for b in range(B):
        n = int(n_rows[b])
        assert np.array_equal(got_v[b, :, :n], vco[b, :, :n])
        assert (np.abs(got_k[b, :, :n] - kco[b, :, :n]) <= 2.0 ** -7 * np.abs(kco[b, :, :n]) + 1e-6).all()


def test_paged_q_and_k_rope_append(spec):
    """The one-launch form on paged caches: the pools as after spec_kv_append_rope_paged bit for bit, q within
    one unit in the last place of the oracle; a bad table entry among the tree's blocks flags the request."""
    B, H, H_kv, D, N, bt = 3, 4, 2, 128, 20, 64
    cfg = wl.Config(91, "pqrope", "bf16", B=B, H=H, H_kv=H_kv, D=D, P=(40, 200), N=N, tree="random_branching")
    inp = wl.make_attention_inputs(cfg, seed=10, S_cap=256)
    pl, dep = inp["prefix_len"].numpy(), inp["tree_depth"].numpy()
    pools, table = wl.to_paged([inp["k_cache"][0], inp["v_cache"][0]], pl, N, bt, np.random.default_rng(3))
    cos, sin = wl.make_rope_tables(256, D)
    q_ref, st_ref = orc.rope_queries(_f64(inp["q"][0]), pl, dep, cos.numpy(), sin.numpy(), 256, "bf16")
    assert (st_ref == 0).all()
    kp1, vp1 = _dev(pools[0]), _dev(pools[1])
    spec.spec_kv_append_rope_paged(_dev(inp["k_new"][0]), _dev(inp["v_new"][0]), kp1, vp1, _dev(table),
                                   _dev(inp["tree_depth"]), _dev(inp["prefix_len"]), _dev(cos), _dev(sin))
    q, kp, vp = _dev(inp["q"][0]), _dev(pools[0]), _dev(pools[1])
    status = torch.zeros(B, dtype=torch.int32, device=DEV)
    spec.spec_qk_rope_append(q, _dev(inp["k_new"][0]), _dev(inp["v_new"][0]), kp, vp, _dev(inp["tree_depth"]),
                             _dev(inp["prefix_len"]), _dev(cos), _dev(sin), status=status, block_table=_dev(table))
    torch.cuda.synchronize()
    assert (status.cpu().numpy() == 0).all()
    assert np.array_equal(_bits(kp), _bits(kp1)) and np.array_equal(_bits(vp), _bits(vp1))
    got = q.double().cpu().numpy()
    assert (np.abs(got - q_ref) <= 2.0 ** -7 * np.abs(q_ref) + 1e-6).all()
    bad = table.clone()
    bad[1, int(pl[1]) // bt] = pools[0].shape[0] + 3
    status.zero_()
    spec.spec_qk_rope_append(_dev(inp["q"][0]), _dev(inp["k_new"][0]), _dev(inp["v_new"][0]), _dev(pools[0]), _dev(pools[1]),
                             _dev(inp["tree_depth"]), _dev(inp["prefix_len"]), _dev(cos), _dev(sin), status=status,
                             block_table=_dev(bad))
    torch.cuda.synchronize()
    assert status.cpu().numpy().tolist() == [0, orc.ST_BAD_BLOCK, 0]


def test_shared_prefix_blocks(spec):
    """Two requests whose tables name the same physical blocks for a common prefix get the outputs of two
    requests with private copies."""
    B, H, D, N, bt = 2, 4, 128, 16, 64
    cfg = wl.Config(90, "share", "bf16", B=B, H=H, D=D, P=192, N=N, tree="expansion", widths=wl.EXPANSION_EVAL * 2)
    inp = wl.make_attention_inputs(cfg, seed=12, S_cap=256)
    inp["k_cache"][0][1, :, :192] = inp["k_cache"][0][0, :, :192]
    inp["v_cache"][0][1, :, :192] = inp["v_cache"][0][0, :, :192]
    pools, table = wl.to_paged([inp["k_cache"][0], inp["v_cache"][0]], inp["prefix_len"].numpy(), N, bt,
                               np.random.default_rng(4))
    shared = table.clone()
    shared[1, :3] = table[0, :3]                                   # 192 rows = three blocks of 64
    ref = orc.tree_attention(_f64(inp["q"][0]), *_appended(inp), inp["tree_parent"].numpy(), inp["prefix_len"].numpy())
    for tab in (table, shared):
        out = spec.spec_tree_attention_append_paged(_dev(inp["q"][0]), _dev(inp["k_new"][0]), _dev(inp["v_new"][0]),
                                                    _dev(pools[0]), _dev(pools[1]), _dev(tab), _dev(inp["tree_parent"]),
                                                    _dev(inp["tree_depth"]), _dev(inp["prefix_len"]), max_prefix_len=192)
        torch.cuda.synchronize()
        _check_attention(out, ref, torch.bfloat16)


def _appended(inp):
    kc, vc = _f64(inp["k_cache"][0]), _f64(inp["v_cache"][0])
    orc.kv_append(kc, vc, _f64(inp["k_new"][0]), _f64(inp["v_new"][0]), inp["prefix_len"].numpy())
    return kc, vc


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_block_outside_the_pool_is_flagged_and_never_written(spec, dtype):
    B, H, D, N, bt = 3, 2, 128, 16, 64
    cfg, inp, kp, vp, table = _paged_inputs(dtype, B, H, H, D, (100, 300), N, "expansion", bt, seed=23)
    pl = inp["prefix_len"].numpy()
    bad = table.clone()
    blk_tree = int(pl[1]) // bt                                    # the block holding request 1's first tree row
    bad[1, blk_tree] = kp.shape[0]                                 # one past the pool
    bad[2, 0] = -5                                                 # request 2: a prefix block
    kpo, vpo = _f64(kp), _f64(vp)
    st_ref = orc.kv_append_paged(kpo, vpo, bad.numpy(), bt, table.shape[1] * bt, _f64(inp["k_new"][0]),
                                 _f64(inp["v_new"][0]), pl)
    assert st_ref.tolist() == [0, orc.ST_BAD_BLOCK, 0]
    for fused in (False, True):
        kpd, vpd = _dev(kp), _dev(vp)
        status = torch.zeros(B, dtype=torch.int32, device=DEV)
        args = (_dev(bad), _dev(inp["tree_parent"]), _dev(inp["tree_depth"]), _dev(inp["prefix_len"]))
        kn, vn = _dev(inp["k_new"][0]), _dev(inp["v_new"][0])
        if fused:
            out = spec.spec_tree_attention_append_paged(_dev(inp["q"][0]), kn, vn, kpd, vpd, *args, status=status,
                                                        max_prefix_len=int(pl.max()), plan=_plan())
        else:
            spec.spec_kv_append_paged(kn, vn, kpd, vpd, _dev(bad), _dev(inp["prefix_len"]), status=status)
            torch.cuda.synchronize()
            assert status.cpu().numpy().tolist() == st_ref.tolist()
            out = spec.spec_tree_attention_paged(_dev(inp["q"][0]), kpd, vpd, *args, status=status,
                                                 max_prefix_len=int(pl.max()), plan=_plan())
        torch.cuda.synchronize()
        # requests 1 and 2 are flagged (their outputs are unspecified), request 0 is served
        assert status.cpu().numpy().tolist() == [0, orc.ST_BAD_BLOCK, orc.ST_BAD_BLOCK]
        # the pool holds exactly what the oracle's append left: rows of the bad block were dropped, not redirected
        assert np.array_equal(kpd.double().cpu().numpy(), kpo) and np.array_equal(vpd.double().cpu().numpy(), vpo)
        ref0 = orc.tree_attention_paged(_f64(inp["q"][0][:1]), kpo, vpo, table.numpy()[:1], bt,
                                        inp["tree_parent"].numpy()[:1], pl[:1])
        _check_attention(out[:1], ref0, inp["q"][0].dtype)
        assert torch.isfinite(out.float()).all()
    # commit: a request with a tree block outside the pool is left alone
    path, ln = np.zeros((B, 2), dtype=np.int32), np.ones(B, dtype=np.int32)
    path[:, 1], ln[:] = 1, 2
    status = torch.zeros(B, dtype=torch.int32, device=DEV)
    kpd = _dev(kp)
    out = spec.spec_kv_commit_paged([kpd], [_dev(vp)], _dev(bad), _dev(path), _dev(ln), _dev(inp["prefix_len"]), N, status=status)
    torch.cuda.synchronize()
    assert status.cpu().numpy().tolist() == [0, orc.ST_BAD_BLOCK, 0]
    assert out.cpu().numpy().tolist() == [int(pl[0]) + 2, int(pl[1]), int(pl[2]) + 2]


def test_paged_host_side_errors(spec):
    cfg, inp, kp, vp, table = _paged_inputs("bf16", 2, 2, 2, 128, (10, 100), 8, "random_parent", 64, seed=3)
    q, tab = _dev(inp["q"][0]), _dev(table)
    kpd, vpd = _dev(kp), _dev(vp)
    rest = (_dev(inp["tree_parent"]), _dev(inp["tree_depth"]), _dev(inp["prefix_len"]))
    import ctypes
    d, pg = spec.make_paged_desc(q, kpd, tab)
    out = torch.empty_like(q)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)

    def call(desc, pages):
        return spec.load().spec_tree_attention_paged(ctypes.byref(desc), ctypes.byref(pages) if pages is not None else None,
                                                     q.data_ptr(), kpd.data_ptr(), vpd.data_ptr(), rest[0].data_ptr(),
                                                     rest[1].data_ptr(), rest[2].data_ptr(), out.data_ptr(), ws.data_ptr(),
                                                     ws.numel(), None, None)
    assert call(d, pg) == 0
    torch.cuda.synchronize()
    assert call(d, None) == spec.ERR_INVALID_ARG
    for field, val, code in (("block_tokens", 96, spec.ERR_UNSUPPORTED), ("block_tokens", 32, spec.ERR_UNSUPPORTED),
                             ("max_blocks", 0, spec.ERR_INVALID_ARG), ("n_blocks", 0, spec.ERR_INVALID_ARG),
                             ("block_table", None, spec.ERR_INVALID_ARG), ("max_blocks", 1, spec.ERR_CAPACITY)):
        d2, pg2 = spec.make_paged_desc(q, kpd, tab)
        setattr(pg2, field, val)
        assert call(d2, pg2) == code, field
    assert spec.spec_tree_attention_paged_workspace_bytes(d, spec.KvPages(None, 1, 64, 1)) == 0
