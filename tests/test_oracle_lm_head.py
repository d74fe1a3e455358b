"""Pins for the oracle's LM head (the LLM's output projection in front of VerifyGreedy of Algorithm 2: for greedy
decoding only O(u) = argmax of the logits is needed). CPU only. The function is a matrix product and an arg-max:
it is pinned to a scalar triple loop, to one-hot weights (where the product is a gather), to a hand-derived
case with a tie, and to the greedy verifier run on the materialised logits."""
import numpy as np
import pytest

from oracle import spec_oracle as orc
from paper_2305_09781_amd import workloads as wl


@pytest.mark.parametrize("seed", range(3))
def test_scalar_triple_loop(seed):
    rng = np.random.default_rng(seed)
    M, K, V = 5, 7, 9
    h, w = rng.standard_normal((M, K)), rng.standard_normal((V, K))
    arg, top, gap = orc.lm_head_argmax(h, w)
    for m in range(M):
        best, best_v, second = -np.inf, -1, -np.inf
        for v in range(V):
            acc = 0.0
            for k in range(K):
                acc += h[m, k] * w[v, k]
            if acc > best:
                second, best, best_v = best, acc, v
            elif acc > second:
                second = acc
        assert arg[m] == best_v and abs(top[m] - best) < 1e-12 and abs(gap[m] - (best - second)) < 1e-12


def test_one_hot_weights_gather_and_hand_derived_tie():
    rng = np.random.default_rng(3)
    M, K = 4, 6
    h = rng.standard_normal((M, K))
    w = np.eye(K)[[3, 0, 5, 3]]                      # token v reads hidden dimension (3, 0, 5, 3)[v]
    logits = orc.lm_head_logits(h, w)
    assert np.array_equal(logits, h[:, [3, 0, 5, 3]])
    arg, top, gap = orc.lm_head_argmax(h, w)
    for m in range(M):
        cols = h[m, [3, 0, 5, 3]]
        assert arg[m] == int(np.argmax(cols)) and top[m] == cols.max()
        if arg[m] in (0, 3):
            assert arg[m] == 0 and gap[m] == 0.0      # tokens 0 and 3 tie: the lower id wins, no gap
    # hand-derived: hidden (1, 2), weights rows (1,0) (0,1) (1,1) (2,0.5) -> logits 1, 2, 3, 3: token 2
    arg, top, gap = orc.lm_head_argmax(np.array([[1.0, 2.0]]), np.array([[1.0, 0], [0, 1.0], [1, 1], [2, 0.5]]))
    assert arg[0] == 2 and top[0] == 3.0 and gap[0] == 0.0


def test_greedy_verifier_on_the_materialised_logits():
    """VerifyGreedy needs nothing but O(u): running it on the logits and walking with the LM head's arg-max agree."""
    rng = np.random.default_rng(11)
    B, N, K, V = 3, 9, 16, 12
    par = np.stack([wl.tree_random_parent(rng, N) for _ in range(B)])
    h, w = rng.standard_normal((B * N, K)), rng.standard_normal((V, K))
    logits = orc.lm_head_logits(h, w).reshape(B, N, V)
    arg, _, _ = orc.lm_head_argmax(h, w)
    tok = rng.integers(0, V, size=(B, N)).astype(np.int32)
    for b in range(B):                               # plant some matches so that paths are longer than one node
        for u in range(N):
            kids = [v for v in range(N) if par[b, v] == u]
            if kids and rng.random() < 0.7:
                tok[b, kids[0]] = arg[b * N + u]
    path, ln, out, node_arg = orc.verify_greedy(logits, tok, par)
    assert np.array_equal(node_arg.reshape(-1), arg)
    assert (ln >= 1).all() and ln.max() > 1


def test_softmax_stats_closed_form_ties_and_the_verifier_it_feeds():
    """softmax_stats: hand-derived values, the tie rule, P(x) rebuilt from (m, Z) against a library softmax, and
    the use it is made for: the first ratio test of VerifyStochastic at a node needs P(x) only, so a walk that
    meets no rejection is decided by the statistics alone."""
    import scipy.special
    # logits (0, ln 2, ln 2): max ln 2 at token 1 (lowest id of the tie), Z = 1/2 + 1 + 1
    arg, m, z = orc.softmax_stats(np.array([[0.0, np.log(2.0), np.log(2.0)]]))
    assert arg[0] == 1 and abs(m[0] - np.log(2.0)) < 1e-15 and abs(z[0] - 2.5) < 1e-12
    # temperature 1/2 squares the ratios: Z = 1/4 + 1 + 1
    _, _, z2 = orc.softmax_stats(np.array([[0.0, np.log(2.0), np.log(2.0)]]), temperature=0.5)
    assert abs(z2[0] - 2.25) < 1e-12
    rng = np.random.default_rng(4)
    x = rng.standard_normal((5, 7, 33)) * 3
    for T in (1.0, 0.7, 1.9):
        arg, m, z = orc.softmax_stats(x, T)
        p = np.exp((x - m[..., None]) / T) / z[..., None]
        assert np.allclose(p, scipy.special.softmax(x / T, axis=-1), rtol=1e-12, atol=0)
        assert np.array_equal(arg, x.argmax(-1)) and np.array_equal(m, x.max(-1))
    # a chain tree whose every child is accepted (draft = LLM, so r * Q(x) <= P(x) always): the path is the chain,
    # and every acceptance test r * Q(x) <= P(x) can be re-evaluated from the statistics
    B, N, V = 2, 6, 17
    par = np.tile(np.arange(-1, N - 1, dtype=np.int32), (B, 1))
    logits = rng.standard_normal((B, N, V)) * 2
    arg, m, z = orc.softmax_stats(logits)
    probs = scipy.special.softmax(logits, axis=-1).reshape(B * N, V).astype(np.float32)
    tok = rng.integers(0, V, size=(B, N)).astype(np.int32)
    row = np.zeros((B, N), dtype=np.int32)
    for b in range(B):
        for v in range(1, N):
            row[b, v] = b * N + par[b, v]
    ua = rng.random((B, N), dtype=np.float32) * 0.99
    path, ln, out, st = orc.verify_stochastic(logits, probs, row, tok, par, ua, rng.random((B, N), dtype=np.float32),
                                              rng.random(B, dtype=np.float32))
    assert (ln == N).all() and (st == 0).all()
    for b in range(B):
        for v in range(1, N):
            u, xx = par[b, v], tok[b, v]
            p_stats = np.exp(logits[b, u, xx] - m[b, u]) / z[b, u]
            assert np.float32(ua[b, v]) * probs[row[b, v], xx] <= np.float32(p_stats) * (1 + 1e-6)
