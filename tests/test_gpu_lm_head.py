"""GPU-vs-oracle parity of the LM head in front of the greedy verifier, through the C ABI (`pytest -m gpu`).

The arg-max is an integer decided by floating point: the kernel accumulates bf16 products in float32 on the
matrix cores, the oracle in float64. A row whose two best logits are further apart than the float32 error bound
of the sums must agree exactly; for a closer pair either token is a correct answer, and the test checks that the
kernel's token is one of the (near-)maxima. Error bound of a K-term float32 sum of products: K * 2^-24 * sum |h w|
(worst case; the inputs here have |h|, |w| <= 8, so the bound is computed from them, not guessed)."""
import numpy as np
import pytest
import torch

from oracle import spec_oracle as orc
from paper_2305_09781_amd import workloads as wl
from test_gpu_parity import DEV, _dev

pytestmark = pytest.mark.gpu


def _inputs(M, K, V, seed, scale=1.0):
    rng = np.random.default_rng(seed)
    h = torch.from_numpy(rng.standard_normal((M, K)).astype(np.float32) * scale).to(torch.bfloat16)
    w = torch.from_numpy(rng.standard_normal((V, K)).astype(np.float32) * 0.05).to(torch.bfloat16)
    return h, w


def _check_rows(arg_gpu, max_gpu, h, w):
    hd, wd = h.double().numpy(), w.double().numpy()
    logits = orc.lm_head_logits(hd, wd)
    arg, top, gap = orc.lm_head_argmax(hd, wd)
    bound = hd.shape[1] * 2.0 ** -24 * (np.abs(hd) @ np.abs(wd).T).max(axis=1)      # float32 accumulation, worst case
    sure = gap > 2 * bound
    assert sure.mean() > 0.9                                                           # the test is not vacuous
    assert np.array_equal(arg_gpu[sure], arg[sure])
    picked = logits[np.arange(len(arg_gpu)), arg_gpu]
    assert (picked >= top - 2 * bound).all()                                           # a near-maximum otherwise
    if max_gpu is not None:
        assert (np.abs(max_gpu - top) <= bound + 1e-6 * np.abs(top)).all()
    return arg


@pytest.mark.parametrize("M,K,V", [(128, 4096, 32000), (16, 4096, 32000), (1, 512, 1000), (17, 256, 130), (64, 1280, 4097),
                                   (200, 1024, 5000), (33, 768, 127), (128, 2048, 129), (48, 2304, 700),
                                   (65, 512, 200), (96, 1024, 1000), (97, 1536, 4097), (129, 512, 128), (300, 1024, 999),
                                   (128, 768, 300)])
def test_lm_head_argmax(spec, M, K, V):
    h, w = _inputs(M, K, V, seed=M + K + V)
    arg, mx = spec.spec_lm_head_argmax(_dev(h), _dev(w), want_max=True)
    torch.cuda.synchronize()
    _check_rows(arg.cpu().numpy(), mx.cpu().numpy().astype(np.float64), h, w)


def test_lm_head_exact_ties_take_the_lowest_token(spec):
    """Duplicate rows of the weight matrix give bit-identical logits: the lower token id must win, also across
    wavefronts, workgroups and the partial merge."""
    M, K, V = 40, 256, 1500
    h, w = _inputs(M, K, V, seed=5)
    w[:] *= 0.1
    big = torch.from_numpy(np.random.default_rng(1).standard_normal(K).astype(np.float32)).to(torch.bfloat16)
    for v in (3, 17, 130, 700, 1499):                      # same strong row at five places: lane, wavefront, workgroup apart
        w[v] = big
    h[:, :] = big.float().abs().to(torch.bfloat16) * torch.sign(big.float()).to(torch.bfloat16)   # aligned with it: huge logit
    arg, _ = spec.spec_lm_head_argmax(_dev(h), _dev(w))
    torch.cuda.synchronize()
    assert (arg.cpu().numpy() == 3).all()
    w[3] = 0
    arg, _ = spec.spec_lm_head_argmax(_dev(h), _dev(w))
    torch.cuda.synchronize()
    assert (arg.cpu().numpy() == 17).all()


@pytest.mark.parametrize("B,N,K,V", [(8, 16, 4096, 32000), (3, 40, 512, 2000), (2, 128, 256, 300)])
def test_verify_greedy_from_hidden_states(spec, B, N, K, V):
    """Hidden states -> accepted path without logits in memory, against VerifyGreedy on the oracle's logits."""
    rng = np.random.default_rng(B * N + K)
    h, w = _inputs(B * N, K, V, seed=K + V)
    par = np.stack([wl.tree_random_parent(rng, N) for _ in range(B)]).astype(np.int32)
    # Rows whose two best logits are closer than float32 rounding could legitimately go either way: such a row is
    # drawn again (same seeded stream) until every decision of the walk is unique.
    for _ in range(20):
        arg_ref, _, gap = orc.lm_head_argmax(h.double().numpy(), w.double().numpy())
        close = np.nonzero(gap <= 1e-3)[0]
        if len(close) == 0:
            break
        h[close] = torch.from_numpy(rng.standard_normal((len(close), K)).astype(np.float32)).to(torch.bfloat16)
    assert (gap > 1e-3).all()
    tok = rng.integers(0, V, size=(B, N)).astype(np.int32)
    for b in range(B):                                     # plant matches so that paths grow
        for u in range(N):
            kids = [v for v in range(N) if par[b, v] == u]
            if kids and rng.random() < 0.7:
                tok[b, kids[int(rng.integers(0, len(kids)))]] = arg_ref[b * N + u]
    logits = orc.lm_head_logits(h.double().numpy(), w.double().numpy()).reshape(B, N, V)
    path, ln, out, node_arg = orc.verify_greedy(logits, tok, par)
    status = torch.zeros(B, dtype=torch.int32, device=DEV)
    g = spec.spec_verify_greedy_lm_head(_dev(h), _dev(w), _dev(tok), _dev(par), status=status)
    torch.cuda.synchronize()
    Lmax = g[0].shape[1]
    assert (status.cpu().numpy() == 0).all() and ln.max() > 1
    assert np.array_equal(g[3].cpu().numpy(), node_arg) and np.array_equal(g[1].cpu().numpy(), ln)
    assert np.array_equal(g[0].cpu().numpy(), path[:, :Lmax]) and np.array_equal(g[2].cpu().numpy(), out[:, :Lmax])


def test_lm_head_host_side_errors(spec):
    h, w = _inputs(4, 256, 100, seed=1)
    hd, wd = _dev(h), _dev(w)
    ws = torch.empty(1 << 16, dtype=torch.uint8, device=DEV)
    arg = torch.empty(4, dtype=torch.int32, device=DEV)
    lib = spec.load()
    call = lambda M, K, V, hp, wp, ap, wsp, nb: lib.spec_lm_head_argmax(M, K, V, hp, wp, ap, None, wsp, nb, None)
    assert call(4, 256, 100, hd.data_ptr(), wd.data_ptr(), arg.data_ptr(), ws.data_ptr(), ws.numel()) == 0
    torch.cuda.synchronize()
    assert call(4, 128, 100, hd.data_ptr(), wd.data_ptr(), arg.data_ptr(), ws.data_ptr(), ws.numel()) == spec.ERR_UNSUPPORTED
    assert call(0, 256, 100, hd.data_ptr(), wd.data_ptr(), arg.data_ptr(), ws.data_ptr(), ws.numel()) == spec.ERR_INVALID_ARG
    assert call(4, 256, 100, None, wd.data_ptr(), arg.data_ptr(), ws.data_ptr(), ws.numel()) == spec.ERR_INVALID_ARG
    assert call(4, 256, 100, hd.data_ptr(), wd.data_ptr(), None, ws.data_ptr(), ws.numel()) == spec.ERR_INVALID_ARG
    assert call(4, 256, 100, hd.data_ptr(), wd.data_ptr(), arg.data_ptr(), ws.data_ptr(), 16) == spec.ERR_WORKSPACE
    assert call(4, 256, 100, hd.data_ptr(), wd.data_ptr(), arg.data_ptr(), None, 0) == spec.ERR_WORKSPACE
    assert spec.spec_lm_head_argmax_workspace_bytes(0, 5) == 0


# ------------------------------------------------------------------------------------------------
# LM head in front of the stochastic verifier: bf16 logits + per-row softmax statistics in one pass
# ------------------------------------------------------------------------------------------------

def _stats_case(spec, M, K, V, temperature, seed):
    """Logits against the float64 product (within one unit in the last place of bf16 plus the float32 accumulation
    bound); maximum, arg-max and sum of exponentials against the oracle's statistics OF THE LOGITS THE KERNEL
    STORED (they are defined on the stored values)."""
    from oracle import spec_oracle as orc
    h, w = _inputs(M, K, V, seed=seed)
    logits, arg, mx, se = spec.spec_lm_head_logits_stats(_dev(h), _dev(w), temperature=temperature)
    torch.cuda.synchronize()
    hd, wd = h.double().numpy(), w.double().numpy()
    want = orc.lm_head_logits(hd, wd)
    got = logits.double().cpu().numpy()
    bound = hd.shape[1] * 2.0 ** -24 * (np.abs(hd) @ np.abs(wd).T)
    assert (np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + bound + 1e-30).all()
    ra, rm, rz = orc.softmax_stats(got, temperature)
    assert np.array_equal(arg.cpu().numpy(), ra)
    assert np.array_equal(mx.double().cpu().numpy(), rm)
    assert np.allclose(se.double().cpu().numpy(), rz, rtol=2e-5, atol=0)
    return logits, mx, se


@pytest.mark.parametrize("M,K,V,T", [(128, 4096, 32000, 1.0), (16, 4096, 32000, 0.7), (1, 512, 1000, 1.0), (17, 256, 130, 1.6),
                                     (64, 1280, 4097, 1.0), (200, 1024, 5001, 0.9), (33, 768, 127, 1.0),
                                     (65, 512, 200, 1.0), (96, 1024, 1002, 0.8), (129, 1536, 4097, 1.3)])
def test_lm_head_logits_and_softmax_statistics(spec, M, K, V, T):
    _stats_case(spec, M, K, V, T, seed=M + K + V)


@pytest.mark.parametrize("temperature", [1.0, 0.8])
def test_stochastic_verification_from_the_lm_head_statistics(spec, temperature):
    """hidden states -> spec_lm_head_logits_stats -> spec_verify_stochastic_stats: the same accepted path and tokens
    as spec_verify_stochastic on the stored logits (the statistics replace its first pass, nothing else), and as
    the oracle's VerifyStochastic on those logits with uniforms vetted against them."""
    from oracle import spec_oracle as orc
    from oracle import vetting
    cfg = wl.Config(2, "lmh-stoch", "bf16", B=8, H=1, D=64, P=1, N=16, tree="expansion", widths=wl.EXPANSION_EVAL, V=4000)
    K = 512
    par_np = wl.make_trees(cfg, np.random.default_rng(3))
    h, w = _inputs(cfg.B * cfg.N, K, cfg.V, seed=77, scale=1.5)
    logits2d, _, mx, se = spec.spec_lm_head_logits_stats(_dev(h), _dev(w), temperature=temperature)
    torch.cuda.synchronize()
    logits = logits2d.view(cfg.B, cfg.N, cfg.V)
    lg = logits.float().cpu()
    # drafts near the LLM and children sampled from them, built on the logits the kernel stored
    rng = np.random.default_rng(5)
    probs_t, ssm_row, tok = wl.make_ssm(cfg, rng, lg, par_np, tau=1.2)
    probs = probs_t.numpy()
    ua, uo, uf = wl.make_uniforms(rng, cfg.B, cfg.N)
    args = (lg.numpy(), probs, ssm_row, tok, par_np)
    ua, uf, _ = vetting.vet_uniforms(*args, ua, uo, uf, rng, temperature=temperature)
    rp, rl, rt, rs = orc.verify_stochastic(*args, ua, uo, uf, temperature=temperature)
    dev_args = (_dev(probs), _dev(ssm_row), _dev(tok), _dev(par_np), _dev(ua), _dev(uo), _dev(uf))
    status = torch.zeros(cfg.B, dtype=torch.int32, device=DEV)
    p1, l1, t1 = spec.spec_verify_stochastic_stats(logits, mx, se, *dev_args, temperature=temperature, status=status)
    p2, l2, t2 = spec.spec_verify_stochastic(logits, *dev_args, temperature=temperature)
    torch.cuda.synchronize()
    assert np.array_equal(p1.cpu().numpy(), rp) and np.array_equal(l1.cpu().numpy(), rl) and np.array_equal(t1.cpu().numpy(), rt)
    assert np.array_equal(status.cpu().numpy(), rs)
    assert torch.equal(p1, p2) and torch.equal(l1, l2) and torch.equal(t1, t2)
    assert rl.max() > 1


def test_lm_head_stats_reject_bad_arguments(spec):
    h, w = _inputs(4, 256, 100, seed=1)
    with pytest.raises(spec.SpecError) as e:
        spec.spec_lm_head_logits_stats(_dev(h), _dev(w), temperature=0.0)
    assert e.value.code == spec.ERR_INVALID_ARG
    with pytest.raises(spec.SpecError) as e:
        spec.spec_lm_head_logits_stats(_dev(h), _dev(w), workspace=torch.empty(256, dtype=torch.uint8, device=DEV)[:8])
    assert e.value.code == spec.ERR_WORKSPACE
