"""Keeps stochastic-verification test inputs away from rounding-fragile decisions.

TEST INFRASTRUCTURE ONLY (uses the CPU oracle). Every ratio test r*Q(x) <= P(x) and the final
inverse-CDF draw compare floating-point sums over the vocabulary; a GPU sums in another order, so a
decision whose two sides agree to within rounding could legitimately flip. For a bit-exact comparison
the uniforms of a request are re-drawn (from the same seeded stream) until every decision the oracle
takes for it has a margin far above float32 summation noise.
"""
import numpy as np

from . import spec_oracle as orc

ACCEPT_MARGIN = 1e-4   # relative gap of a ratio test; float32 softmax noise is ~1e-6
CDF_MARGIN = 2e-6      # distance of the final draw from a CDF step, as a fraction of the total mass


def vet_uniforms(logits, probs_ssm, ssm_row, tree_token, tree_parent, u_accept, u_order, u_final, rng,
                 temperature=1.0, max_rounds=200):
    """Returns (u_accept, u_final, n_redraws) such that the oracle's margins exceed the thresholds for
    every request. u_order is left alone (the order is an exact comparison of inputs)."""
    u_accept = np.array(u_accept, dtype=np.float32, copy=True)
    u_final = np.array(u_final, dtype=np.float32, copy=True)
    B, N = u_accept.shape
    redraws = 0
    todo = list(range(B))
    for _ in range(max_rounds):
        if not todo:
            break
        idx = np.array(todo)
        _, _, _, _, margins = orc.verify_stochastic(
            np.asarray(logits)[idx], probs_ssm, np.asarray(ssm_row)[idx], np.asarray(tree_token)[idx],
            np.asarray(tree_parent)[idx], u_accept[idx], np.asarray(u_order)[idx], u_final[idx],
            temperature=temperature, return_margins=True)
        nxt = []
        for j, b in enumerate(todo):
            if margins[j, 0] < ACCEPT_MARGIN or margins[j, 1] < CDF_MARGIN:
                u_accept[b] = np.minimum(rng.random(N, dtype=np.float32), np.float32(1 - 2.0 ** -24))
                u_final[b] = min(rng.random(dtype=np.float32), np.float32(1 - 2.0 ** -24))
                redraws += 1
                nxt.append(b)
        todo = nxt
    if todo:
        raise RuntimeError("could not find robust uniforms")
    return u_accept, u_final, redraws


def vet_sample_uniforms(logits, u_sample, rng, temperature=1.0, max_rounds=200):
    """Returns (u_sample, n_redraws) such that every node's inverse-CDF draw keeps CDF_MARGIN from a step."""
    u_sample = np.array(u_sample, dtype=np.float32, copy=True)
    redraws = 0
    for _ in range(max_rounds):
        _, margins = orc.sample_nodes(logits, u_sample, temperature)
        bad = margins < CDF_MARGIN
        if not bad.any():
            return u_sample, redraws
        n = int(bad.sum())
        u_sample[bad] = np.minimum(rng.random(n, dtype=np.float32), np.float32(1 - 2.0 ** -24))
        redraws += n
    raise RuntimeError("could not find robust uniforms")
