"""Pins for the oracle's naive-sampling verifier (Section 4.3; Theorem 4.3; the baseline of Table 3). CPU only.

Nothing here re-types the oracle's arithmetic: the inverse CDF is checked by a scalar brute-force loop, the
walk by exhaustive integration over the uniforms (exact acceptance and emission laws in closed form), the
rejection probability against Theorem 4.3's closed form next to multi-step speculative sampling's, and the
low-temperature limit against the greedy verifier."""
import itertools
import math

import numpy as np
import pytest

from oracle import spec_oracle as orc
from paper_2305_09781_amd import workloads as wl


def _softmax(z):
    e = np.exp(z - np.max(z))
    return e / e.sum()


def test_inverse_cdf_brute_force_and_edges():
    rng = np.random.default_rng(0)
    V = 7
    logits = rng.standard_normal((2, 3, V)) * 2
    u = rng.random((2, 3)).astype(np.float32)
    u[0, 0], u[0, 1] = 0.0, np.float32(1 - 2.0 ** -24)
    got, margins = orc.sample_nodes(logits, u)
    for b in range(2):
        for n in range(3):
            p = _softmax(logits[b, n])
            run, want = 0.0, V - 1
            for k in range(V):                      # scalar definition: first k with CDF(k) > r
                run += p[k]
                if run > float(u[b, n]):
                    want = k
                    break
            assert got[b, n] == want
            assert margins[b, n] >= 0
    assert got[0, 0] == 0 and got[0, 1] == V - 1
    # temperature: T -> 0 puts all mass on the argmax
    cold, _ = orc.sample_nodes(logits, u, temperature=1e-3)
    assert (cold == logits.argmax(-1)).all()


def test_first_step_law_is_exactly_the_llm_distribution():
    """The measure of uniforms that emit token x first is P(x): integrate over a fine grid of u."""
    rng = np.random.default_rng(1)
    V, M = 5, 20000
    logits = np.tile(rng.standard_normal((1, 1, V)) * 1.5, (M, 1, 1))
    u = ((np.arange(M) + 0.5) / M).astype(np.float32).reshape(M, 1)
    toks = np.zeros((M, 1), dtype=np.int32)
    par = -np.ones((M, 1), dtype=np.int32)
    _, ln, out, _ = orc.verify_naive(logits, toks, par, u)
    assert (ln == 1).all()
    freq = np.bincount(out[:, 0], minlength=V) / M
    assert np.abs(freq - _softmax(logits[0, 0])).max() <= 1.5 / M * V


@pytest.mark.parametrize("seed", range(4))
def test_acceptance_probability_matches_closed_form_and_theorem_4_3(seed):
    """One level, k children with tokens x_1..x_k: naive sampling accepts iff the drawn token is one of
    them, so P(accept) = sum of P over the distinct child tokens and P(move to child j) = P(x_j) for the
    lowest-index child carrying x_j. Multi-step speculative sampling's rejection probability (closed
    form, children drawn from their draft distributions, random order) is never larger."""
    rng = np.random.default_rng(seed)
    V, k, M = 4, 3, 8000
    p_logits = rng.standard_normal(V) * 2
    p = _softmax(p_logits)
    child_tok = rng.integers(0, V, size=k)
    N = 1 + k
    logits = np.zeros((M, N, V))
    logits[:, 0] = p_logits
    toks = np.tile(np.concatenate([[0], child_tok]).astype(np.int32), (M, 1))
    par = np.tile(np.array([-1] + [0] * k, dtype=np.int32), (M, 1))
    u = np.full((M, N), 0.5, dtype=np.float32)
    u[:, 0] = (np.arange(M) + 0.5) / M
    path, ln, out, _ = orc.verify_naive(logits, toks, par, u)
    moved = ln >= 2
    want_accept = sum(p[x] for x in set(int(t) for t in child_tok))
    assert abs(moved.mean() - want_accept) <= 2.0 / M * V
    for j in range(k):
        first = j == [int(t) for t in child_tok].index(int(child_tok[j]))
        want = p[child_tok[j]] if first else 0.0
        assert abs((path[:, 1] == 1 + j).mean() - want) <= 2.0 / M * V
    assert (out[moved, 0] == toks[moved, path[moved, 1]]).all()          # emitted token = the child's token
    # Theorem 4.3 in closed form (naive: 1 - sum over distinct child tokens; multi-step: product of rejections)
    qs = [_softmax(rng.standard_normal(V) * 2) for _ in range(k)]
    rej_ns = rej_mss = 0.0
    for tup in itertools.product(range(V), repeat=k):
        w = math.prod(qs[j][tup[j]] for j in range(k))
        rej_ns += w * (1.0 - sum(p[x] for x in set(tup)))
        for order in itertools.permutations(range(k)):
            pp, reach = p.copy(), 1.0
            for j in order:
                x = tup[j]
                a = 1.0 if qs[j][x] <= 0 else min(1.0, pp[x] / qs[j][x])
                reach *= 1.0 - a
                r = np.maximum(0.0, pp - qs[j])
                if r.sum() > 0:
                    pp = r / r.sum()
            rej_mss += w * reach / math.factorial(k)
    assert rej_mss <= rej_ns + 1e-12


@pytest.mark.parametrize("seed", range(3))
def test_low_temperature_limit_is_the_greedy_verifier(seed):
    cfg = wl.Config(94, "ns", "f32", B=3, H=1, D=64, P=4, N=12, tree="random_parent", V=16, logit_std=2.0)
    inp = wl.make_verify_inputs(cfg, seed=seed, mode="greedy")
    logits, tok, par = inp["logits"].numpy(), inp["tree_token"].numpy(), inp["tree_parent"].numpy()
    gp, gl, gt, _ = orc.verify_greedy(logits, tok, par)
    u = np.random.default_rng(seed).random((cfg.B, cfg.N)).astype(np.float32)
    npth, nl, nt, _ = orc.verify_naive(logits, tok, par, u, temperature=1e-4)
    assert np.array_equal(gp, npth) and np.array_equal(gl, nl) and np.array_equal(gt, nt)


def test_walk_invariants_and_duplicate_children():
    rng = np.random.default_rng(5)
    B, N, V = 6, 10, 6
    par = np.stack([wl.tree_random_parent(rng, N) for _ in range(B)])
    tok = rng.integers(0, V, size=(B, N)).astype(np.int32)       # small vocabulary: duplicate sibling tokens occur
    logits = rng.standard_normal((B, N, V))
    u = rng.random((B, N)).astype(np.float32)
    path, ln, out, samp = orc.verify_naive(logits, tok, par, u)
    for b in range(B):
        assert path[b, 0] == 0 and 1 <= ln[b] <= N
        for k in range(1, ln[b]):
            v, prev = path[b, k], path[b, k - 1]
            assert par[b, v] == prev and tok[b, v] == samp[b, prev] == out[b, k - 1]
            same = [c for c in range(N) if par[b, c] == prev and tok[b, c] == tok[b, v]]
            assert v == min(same)                                   # lowest-index child among duplicates
        last = path[b, ln[b] - 1]
        assert out[b, ln[b] - 1] == samp[b, last]
        assert all(tok[b, c] != samp[b, last] for c in range(N) if par[b, c] == last)
        assert (path[b, ln[b]:] == -1).all() and (out[b, ln[b]:] == -1).all()
