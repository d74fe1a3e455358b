"""Rotary embedding inside the fused append + attention launch, GPU vs oracle through the C ABI (`pytest -m gpu`).

What is unique is compared bit for bit: the caches after the one-launch call equal the caches after
spec_qk_rope_append (whose rotation is held to one unit in the last place of the float64 oracle), `out` equals
the attention launched on what spec_qk_rope_append left behind, and q is not modified. `out` is also held to the
attention bar (|g-o| <= 2e-2 + 1e-2*|o|) of the float64 oracle on the rotated operands. Shapes cover every bf16
kernel (few-query, 2 / 4 / 8 wavefronts of 16 queries, 4 wavefronts of 32 queries), every launch plan and the
paged cache."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import spec_oracle as orc
from paper_2305_09781_amd import workloads as wl
from test_gpu_parity import DEV, _balanced_wgs, _bits, _check_attention, _chunk_keys, _dev, _f64, _heads_per_wg, _plan

pytestmark = pytest.mark.gpu

CASES = [
    # B, H, H_kv, D, (P lo, hi), N, tree, forced chunk, balanced workgroups, heads per workgroup
    (3, 4, 4, 128, (30, 200), 16, "expansion", 0, 0, 0),           # few-query kernel
    (2, 3, 3, 64, (0, 90), 9, "random_parent", 0, 0, 0),           # few-query kernel, D = 64, empty prefix possible
    (2, 4, 4, 128, (100, 400), 16, "expansion", 96, 0, 0),         # few-query kernel, chunks
    (3, 2, 2, 64, (20, 300), 12, "random_branching", 0, 5, 0),     # few-query kernel, balanced deal
    (2, 3, 3, 128, (0, 130), 30, "random_branching", 0, 0, 0),     # 2 x 2 wavefronts
    (2, 4, 4, 64, (50, 260), 64, "expansion", 0, 0, 0),            # 4 wavefronts, D = 64
    (2, 4, 4, 128, (50, 260), 40, "random_branching", 128, 0, 0),  # 4 wavefronts, chunks
    (2, 8, 2, 128, (70, 300), 16, "random_parent", 0, 0, 0),       # grouped heads: 4 query tiles on one K/V head
    (2, 16, 1, 128, (40, 300), 16, "expansion", 0, 0, 0),          # 2 query groups per K/V head: both rotate, one stores
    (2, 3, 3, 64, (30, 280), 100, "random_branching", 0, 0, 0),    # 8 wavefronts of 16 queries (D = 64)
    (2, 4, 4, 64, (30, 280), 128, "expansion", 0, 0, 2),           # ... two heads per workgroup as one stream
    (2, 2, 2, 64, (100, 500), 77, "random_branching", 0, 7, 0),    # ... balanced deal
    (2, 3, 3, 128, (30, 280), 128, "expansion", 0, 0, 0),          # 4 wavefronts of 32 queries
    (3, 2, 2, 128, (0, 300), 65, "random_branching", 0, 0, 0),     # ... ragged tree tail, empty prefix possible
    (2, 2, 2, 128, (200, 700), 100, "random_branching", 128, 0, 0),  # ... chunks
    (2, 3, 3, 128, (100, 500), 90, "random_parent", 0, 7, 0),      # ... balanced deal
    (2, 6, 1, 128, (64, 64), 128, "random_branching", 0, 0, 0),    # ... one K/V head, six query groups
]


def _inputs(B, H, H_kv, D, P, N, tree, seed, S=None):
    cfg = wl.Config(97, "ropefused", "bf16", B=B, H=H, H_kv=H_kv, D=D, P=P if P[0] != P[1] else P[0], N=N, tree=tree,
                    widths=wl.EXPANSION_EVAL * 16)
    S = S or P[1] + N + 3
    return cfg, wl.make_attention_inputs(cfg, seed=seed, S_cap=S), S


@pytest.mark.parametrize("case", CASES, ids=lambda c: f"B{c[0]}-H{c[1]}/{c[2]}-D{c[3]}-N{c[5]}-c{c[7]}-w{c[8]}-h{c[9]}")
def test_rotary_embedding_inside_the_fused_launch(spec, case):
    B, H, H_kv, D, P, N, tree, chunk, wgs, hpw = case
    cfg, inp, S = _inputs(B, H, H_kv, D, P, N, tree, seed=900 + N + H)
    cos, sin = wl.make_rope_tables(S, D)
    pl, dep, par = inp["prefix_len"].numpy(), inp["tree_depth"].numpy(), inp["tree_parent"].numpy()
    mp = int(pl.max())
    dev = {k: _dev(inp[k][0]) for k in ("q", "k_new", "v_new")}
    tree_args = (_dev(inp["tree_parent"]), _dev(inp["tree_depth"]), _dev(inp["prefix_len"]))
    cs, sn = _dev(cos), _dev(sin)
    # two launches: rotate q in place and K on its way into the cache, then attend
    q2, kc2, vc2 = dev["q"].clone(), _dev(inp["k_cache"][0]), _dev(inp["v_cache"][0])
    spec.spec_qk_rope_append(q2, dev["k_new"], dev["v_new"], kc2, vc2, tree_args[1], tree_args[2], cs, sn)
    with _chunk_keys(chunk), _balanced_wgs(wgs), _heads_per_wg(hpw):
        out2 = spec.spec_tree_attention(q2, kc2, vc2, *tree_args, max_prefix_len=mp, plan=_plan())
    # one launch
    kc, vc = _dev(inp["k_cache"][0]), _dev(inp["v_cache"][0])
    status = torch.zeros(B, dtype=torch.int32, device=DEV)
    with _chunk_keys(chunk), _balanced_wgs(wgs), _heads_per_wg(hpw):
        out = spec.spec_tree_attention_append_rope(dev["q"], dev["k_new"], dev["v_new"], kc, vc, *tree_args, cs, sn,
                                                   status=status, max_prefix_len=mp, plan=_plan())
    torch.cuda.synchronize()
    assert (status.cpu().numpy() == 0).all()
    assert np.array_equal(_bits(dev["q"]), _bits(inp["q"][0]))                       # q is an input only
    assert np.array_equal(_bits(kc), _bits(kc2)) and np.array_equal(_bits(vc), _bits(vc2))
    assert np.array_equal(_bits(out), _bits(out2))
    # the rotation against the oracle (one unit in the last place), then the attention on the rotated bits
    kco, vco = _f64(inp["k_cache"][0]), _f64(inp["v_cache"][0])
    orc.kv_append_rope(kco, vco, _f64(inp["k_new"][0]), _f64(inp["v_new"][0]), pl, dep, cos.numpy(), sin.numpy(), "bf16")
    got_k = kc.double().cpu().numpy()
    assert (np.abs(got_k - kco) <= 2.0 ** -7 * np.abs(kco) + 1e-6).all() and (got_k != kco).mean() < 0.02
    assert np.array_equal(vc.double().cpu().numpy(), vco)
    q_ref, _ = orc.rope_queries(_f64(inp["q"][0]), pl, dep, cos.numpy(), sin.numpy(), S, "bf16")
    got_q = q2.double().cpu().numpy()
    assert (np.abs(got_q - q_ref) <= 2.0 ** -7 * np.abs(q_ref) + 1e-6).all()
    want = orc.tree_attention(got_q, got_k, vc.double().cpu().numpy(), par, pl)
    _check_attention(out, want, torch.bfloat16)


@pytest.mark.parametrize("case", [(2, 4, 4, 128, (100, 400), 16, "expansion", 64, 0, 0),
                                  (2, 8, 2, 128, (60, 330), 40, "random_branching", 64, 0, 0),
                                  (2, 2, 2, 128, (190, 460), 128, "random_branching", 256, 128, 0),
                                  (2, 2, 2, 64, (130, 400), 100, "expansion", 128, 0, 5)],
                         ids=lambda c: f"B{c[0]}-H{c[1]}/{c[2]}-D{c[3]}-N{c[5]}-bt{c[7]}-c{c[8]}-w{c[9]}")
def test_rotary_embedding_inside_the_fused_launch_paged(spec, case):
    B, H, H_kv, D, P, N, tree, bt, chunk, wgs = case
    S = ((P[1] + N + bt - 1) // bt) * bt
    cfg, inp, _ = _inputs(B, H, H_kv, D, P, N, tree, seed=950 + N, S=S)
    rng = np.random.default_rng(5)
    pools, table = wl.to_paged([inp["k_cache"][0], inp["v_cache"][0]], inp["prefix_len"].numpy(), N, bt, rng)
    cos, sin = wl.make_rope_tables(S, D)
    pl, par = inp["prefix_len"].numpy(), inp["tree_parent"].numpy()
    mp = int(pl.max())
    q, kn, vn = (_dev(inp[k][0]) for k in ("q", "k_new", "v_new"))
    tab, cs, sn = _dev(table), _dev(cos), _dev(sin)
    tree_args = (_dev(inp["tree_parent"]), _dev(inp["tree_depth"]), _dev(inp["prefix_len"]))
    q2, kp2, vp2 = q.clone(), _dev(pools[0]), _dev(pools[1])
    spec.spec_qk_rope_append(q2, kn, vn, kp2, vp2, tree_args[1], tree_args[2], cs, sn, block_table=tab)
    with _chunk_keys(chunk), _balanced_wgs(wgs):
        out2 = spec.spec_tree_attention_paged(q2, kp2, vp2, tab, *tree_args, max_prefix_len=mp, plan=_plan())
    kp, vp = _dev(pools[0]), _dev(pools[1])
    status = torch.zeros(B, dtype=torch.int32, device=DEV)
    with _chunk_keys(chunk), _balanced_wgs(wgs):
        out = spec.spec_tree_attention_append_rope(q, kn, vn, kp, vp, *tree_args, cs, sn, status=status, max_prefix_len=mp,
                                                   plan=_plan(), block_table=tab)
    torch.cuda.synchronize()
    assert (status.cpu().numpy() == 0).all()
    assert np.array_equal(_bits(kp), _bits(kp2)) and np.array_equal(_bits(vp), _bits(vp2))   # the whole pools
    assert np.array_equal(_bits(out), _bits(out2))
    want = orc.tree_attention_paged(q2.double().cpu().numpy(), kp.double().cpu().numpy(), vp.double().cpu().numpy(),
                                    table.numpy(), bt, par, pl)
    _check_attention(out, want, torch.bfloat16)


@pytest.mark.parametrize("seed", range(20))
def test_randomised_shapes_and_plans_with_the_rotation_fused_in(spec, seed):
    """Random small shapes (grouped heads, head dim, tree size from one node to 128, ragged prefixes down to zero)
    under a random launch plan, contiguous or paged: the one-launch call against the oracle's rotation (one unit in
    the last place) and the oracle's attention on the rotated bits, the caches bit-equal to spec_qk_rope_append's."""
    rng = np.random.default_rng(9100 + seed)
    D = int(rng.choice([64, 128]))
    H_kv = int(rng.integers(1, 4))
    N = int(rng.choice([1, 5, 16, 17, 32, 33, 64, 65, 100, 128]))
    group = int(rng.integers(1, 9)) if rng.random() < 0.3 else int(rng.integers(1, 3))
    B = int(rng.integers(1, 5))
    hi = int(rng.choice([0, 40, 130, 400, 700]))
    lo = int(rng.integers(0, hi + 1))
    tree = str(rng.choice(["random_parent", "random_branching", "expansion"]))
    bt = int(rng.choice([0, 0, 64, 128]))                        # 0: contiguous cache
    S = hi + N + 3 if bt == 0 else ((hi + N + bt - 1) // bt) * bt
    cfg, inp, _ = _inputs(B, H_kv * group, H_kv, D, (lo, hi), N, tree, seed=9200 + seed, S=S)
    plan = int(rng.integers(0, 3))
    chunk = int(rng.choice([32, 64, 96, 160])) if plan == 1 else 0
    wgs = int(rng.integers(1, 12)) if plan == 2 else 0
    cos, sin = wl.make_rope_tables(S + int(rng.integers(0, 5)), D)
    pl, dep, par = inp["prefix_len"].numpy(), inp["tree_depth"].numpy(), inp["tree_parent"].numpy()
    q, kn, vn = (_dev(inp[k][0]) for k in ("q", "k_new", "v_new"))
    tree_args = (_dev(inp["tree_parent"]), _dev(inp["tree_depth"]), _dev(inp["prefix_len"]))
    cs, sn = _dev(cos), _dev(sin)
    caches, tab = [inp["k_cache"][0], inp["v_cache"][0]], None
    if bt:
        caches, table = wl.to_paged(caches, pl, N, bt, np.random.default_rng(seed))
        tab = _dev(table)
    q2, kc2, vc2 = q.clone(), _dev(caches[0]), _dev(caches[1])
    spec.spec_qk_rope_append(q2, kn, vn, kc2, vc2, tree_args[1], tree_args[2], cs, sn, block_table=tab)
    kc, vc = _dev(caches[0]), _dev(caches[1])
    status = torch.zeros(B, dtype=torch.int32, device=DEV)
    with _chunk_keys(chunk), _balanced_wgs(wgs):
        out = spec.spec_tree_attention_append_rope(q, kn, vn, kc, vc, *tree_args, cs, sn, status=status, max_prefix_len=int(pl.max()),
                                                   plan=_plan(), block_table=tab)
    torch.cuda.synchronize()
    assert (status.cpu().numpy() == 0).all()
    assert np.array_equal(_bits(q), _bits(inp["q"][0]))
    assert np.array_equal(_bits(kc), _bits(kc2)) and np.array_equal(_bits(vc), _bits(vc2))
    q_ref, _ = orc.rope_queries(_f64(inp["q"][0]), pl, dep, cos.numpy(), sin.numpy(), S, "bf16")
    got_q = q2.double().cpu().numpy()
    assert (np.abs(got_q - q_ref) <= 2.0 ** -7 * np.abs(q_ref) + 1e-6).all()
    kco, vco = _f64(inp["k_cache"][0]), _f64(inp["v_cache"][0])       # the logical caches, rotated rows appended
    orc.kv_append_rope(kco, vco, _f64(inp["k_new"][0]), _f64(inp["v_new"][0]), pl, dep, cos.numpy(), sin.numpy(), "bf16")
    if bt:
        got = orc.tree_attention_paged(got_q, kc.double().cpu().numpy(), vc.double().cpu().numpy(), table.numpy(), bt, par, pl)
        # the pool's appended rows against the oracle's, read through the table
        for b in range(B):
            rows = np.arange(pl[b], pl[b] + N)
            blk, off = table.numpy()[b, rows // bt], rows % bt
            gk = kc.double().cpu().numpy()[blk, :, off]              # [N, H_kv, D]
            want_k = kco[b][:, rows].transpose(1, 0, 2)
            assert (np.abs(gk - want_k) <= 2.0 ** -7 * np.abs(want_k) + 1e-6).all()
    else:
        got_k = kc.double().cpu().numpy()
        assert (np.abs(got_k - kco) <= 2.0 ** -7 * np.abs(kco) + 1e-6).all()
        assert np.array_equal(vc.double().cpu().numpy(), vco)
        got = orc.tree_attention(got_q, got_k, vc.double().cpu().numpy(), par, pl)
    _check_attention(out, got, torch.bfloat16)


def test_outputs_depend_on_relative_positions_only(spec):
    """What the rotary embedding is for, through the whole launch: with every position shifted by the same amount
    (tables that start s rows later) the scores, and so the outputs, stay the same up to the rounding of the
    rotated operands. The prefix rows are rotated on the host by the oracle, the tree rows by the launch."""
    B, H, D, N, P = 2, 2, 128, 24, 90
    cfg, inp, S = _inputs(B, H, H, D, (P, P), N, "random_branching", seed=31)
    cos, sin = wl.make_rope_tables(S + 64, D)
    pl, par = inp["prefix_len"].numpy(), inp["tree_parent"].numpy()
    outs = []
    for shift in (0, 37):
        c, s_ = cos[shift:].contiguous(), sin[shift:].contiguous()
        kc = _f64(inp["k_cache"][0])
        for b in range(B):                                            # prefix row j sits at position j (+ shift)
            for j in range(P):
                kc[b, :, j] = orc.round_to_storage(orc.rope_rotate(kc[b, :, j], c[j].double().numpy(), s_[j].double().numpy()), "bf16")
        kcd, vcd = _dev(torch.from_numpy(kc).to(torch.bfloat16)), _dev(inp["v_cache"][0])
        outs.append(spec.spec_tree_attention_append_rope(_dev(inp["q"][0]), _dev(inp["k_new"][0]), _dev(inp["v_new"][0]), kcd, vcd,
                                                         _dev(inp["tree_parent"]), _dev(inp["tree_depth"]), _dev(inp["prefix_len"]),
                                                         _dev(c), _dev(s_)).double().cpu().numpy())
    # two bf16 roundings of differently rotated operands: the bf16 attention bar, not bit equality
    assert (np.abs(outs[0] - outs[1]) <= 2e-2 + 1e-2 * np.abs(outs[0])).all()
    assert np.abs(outs[0]).max() > 0.05                                # and not trivially: the outputs are not zeros


@pytest.mark.parametrize("c", [2, 3, 4, 5])
def test_full_size_configs_with_the_rotation_fused_in(spec, c):
    """The benchmark's shapes at full size, in the plan the library chooses: caches and outputs of the one-launch call
    equal, bit for bit, those of spec_qk_rope_append followed by the attention launch (every request, head, node and
    the whole cache); the last request's last head is also held to the oracle on the rotated bits."""
    cfg = wl.CONFIGS[c]
    inp = wl.make_attention_inputs(cfg)
    S = inp["k_cache"][0].shape[2]
    cos, sin = wl.make_rope_tables(S, cfg.D)
    pl, par = inp["prefix_len"].numpy(), inp["tree_parent"].numpy()
    mp = int(pl.max())
    q, kn, vn = (_dev(inp[k][0]) for k in ("q", "k_new", "v_new"))
    tree_args = (_dev(inp["tree_parent"]), _dev(inp["tree_depth"]), _dev(inp["prefix_len"]))
    cs, sn = _dev(cos), _dev(sin)
    q2, kc2, vc2 = q.clone(), _dev(inp["k_cache"][0]), _dev(inp["v_cache"][0])
    spec.spec_qk_rope_append(q2, kn, vn, kc2, vc2, tree_args[1], tree_args[2], cs, sn)
    out2 = spec.spec_tree_attention(q2, kc2, vc2, *tree_args, max_prefix_len=mp)
    kc, vc = _dev(inp["k_cache"][0]), _dev(inp["v_cache"][0])
    status = torch.zeros(cfg.B, dtype=torch.int32, device=DEV)
    out = spec.spec_tree_attention_append_rope(q, kn, vn, kc, vc, *tree_args, cs, sn, status=status, max_prefix_len=mp)
    torch.cuda.synchronize()
    assert (status.cpu().numpy() == 0).all()
    assert torch.equal(kc.view(torch.int16), kc2.view(torch.int16)) and torch.equal(vc.view(torch.int16), vc2.view(torch.int16))
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))
    b, h = cfg.B - 1, cfg.H - 1
    want = orc.tree_attention(q2[b:b + 1, :, h:h + 1].double().cpu().numpy(), kc[b:b + 1, h:h + 1].double().cpu().numpy(),
                              vc[b:b + 1, h:h + 1].double().cpu().numpy(), par[b:b + 1], pl[b:b + 1])
    _check_attention(out[b:b + 1, :, h:h + 1], want, torch.bfloat16)


@pytest.mark.parametrize("N,D", [(16, 128), (48, 64), (128, 128)])
def test_tables_shorter_than_a_request_needs(spec, N, D):
    """prefix_len + N beyond the tables: that request is neither appended nor attended (zeros, SPEC_ST_CAPACITY),
    the others come out as with long tables; a malformed tree still gives zeros and its own flag."""
    B, H = 3, 2
    cfg, inp, S = _inputs(B, H, H, D, (40, 300), N, "random_branching", seed=77 + N)
    inp["prefix_len"][:] = torch.tensor([120, 300, 250], dtype=inp["prefix_len"].dtype)   # request 1 is the longest
    cos, sin = wl.make_rope_tables(S, D)
    short = 300 + N - 1                                          # one position short for request 1 only
    assert int(np.delete(inp["prefix_len"].numpy(), 1).max()) + N <= short
    q, kn, vn = (_dev(inp[k][0]) for k in ("q", "k_new", "v_new"))
    tree_args = (_dev(inp["tree_parent"]), _dev(inp["tree_depth"]), _dev(inp["prefix_len"]))
    kc_full, vc_full = _dev(inp["k_cache"][0]), _dev(inp["v_cache"][0])
    out_full = spec.spec_tree_attention_append_rope(q, kn, vn, kc_full, vc_full, *tree_args, _dev(cos), _dev(sin))
    kc, vc = _dev(inp["k_cache"][0]), _dev(inp["v_cache"][0])
    status = torch.zeros(B, dtype=torch.int32, device=DEV)
    out = spec.spec_tree_attention_append_rope(q, kn, vn, kc, vc, *tree_args, _dev(cos[:short].contiguous()),
                                               _dev(sin[:short].contiguous()), status=status)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, orc.ST_CAPACITY, 0]
    assert (out[1].float() == 0).all()
    assert np.array_equal(_bits(kc[1]), _bits(inp["k_cache"][0][1])) and np.array_equal(_bits(vc[1]), _bits(inp["v_cache"][0][1]))
    for b in (0, 2):
        assert np.array_equal(_bits(out[b]), _bits(out_full[b])) and np.array_equal(_bits(kc[b]), _bits(kc_full[b]))
    # malformed tree
    bad = inp["tree_parent"].clone()
    bad[0, N - 1] = N + 3
    status.zero_()
    out = spec.spec_tree_attention_append_rope(q, kn, vn, _dev(inp["k_cache"][0]), _dev(inp["v_cache"][0]), _dev(bad),
                                               tree_args[1], tree_args[2], _dev(cos), _dev(sin), status=status)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [orc.ST_BAD_TREE, 0, 0] and (out[0].float() == 0).all()
    assert np.array_equal(_bits(out[2]), _bits(out_full[2]))


def test_fused_rope_rejects_bad_arguments(spec):
    cfg, inp, S = _inputs(1, 2, 2, 64, (10, 10), 4, "random_parent", seed=1)
    cos, sin = wl.make_rope_tables(S, 64)
    t = [_dev(inp[k][0]) for k in ("q", "k_new", "v_new", "k_cache", "v_cache")] + [_dev(inp["tree_parent"]), _dev(inp["tree_depth"]),
                                                                                   _dev(inp["prefix_len"])]
    with pytest.raises(ValueError):
        spec.spec_tree_attention_append_rope(*t, _dev(cos[:, :16].contiguous()), _dev(sin[:, :16].contiguous()))
    d = spec.make_desc(t[0], t[3], k_new=t[1])
    ptr = lambda x: ctypes.c_void_p(x.data_ptr())
    cs, sn, out = _dev(cos), _dev(sin), torch.empty_like(t[0])
    call = spec.load().spec_tree_attention_append_rope
    ok_args = [ptr(x) for x in t]
    assert call(ctypes.byref(d), *ok_args, None, ptr(sn), S, ptr(out), None, 0, None, None) != 0       # no cosines
    assert call(ctypes.byref(d), *ok_args, ptr(cs), ptr(sn), 0, ptr(out), None, 0, None, None) != 0    # empty tables
    assert call(ctypes.byref(d), ok_args[0], None, *ok_args[2:], ptr(cs), ptr(sn), S, ptr(out), None, 0, None, None) != 0
    # float32 inputs: the one-launch form is the bf16 kernels'
    f = [x.float() if x.dtype == torch.bfloat16 else x for x in t]
    d32 = spec.make_desc(f[0], f[3], k_new=f[1])
    out32 = torch.empty_like(f[0])
    rc = call(ctypes.byref(d32), *[ptr(x) for x in f], ptr(cs), ptr(sn), S, ptr(out32), None, 0, None, None)
    assert rc != 0 and b"unsupported" in spec.load().spec_strerror(rc).lower()
