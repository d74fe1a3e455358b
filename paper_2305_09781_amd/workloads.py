"""Seeded synthetic workloads for tree-based parallel decoding.

This module only *draws data*: tree shapes, Q/K/V values, logits, draft distributions, tokens and
uniform random numbers. It contains none of the method's arithmetic (no attention, no verification,
no cache update) and is the only code used by both the CPU oracle's tests and the GPU path.

The shapes stand in for the paper's evaluation workloads (Section 6.1): LLaMA-7B (32 heads x 128,
32 layers, vocabulary 32000) and LLaMA-65B (64 heads x 128, 80 layers); token trees follow the
expansion configuration <1,1,3,1,1,1,1,1> used there; the rate at which a speculated child matches
the LLM's choice follows Table 1.

Everything is generated on the host with numpy's PCG64, rounded to the storage dtype on the host
(round-to-nearest-even for bf16) and returned as CPU torch tensors, so every consumer sees identical
bytes.
"""
from __future__ import annotations

import concurrent.futures
import dataclasses
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

BASE_SEED = 20230509 * 10

# Probability that one child of a node with c children carries the LLM's argmax token (greedy runs);
# mid-range of the greedy rows of Table 1 for top-1..top-4 (index = number of children).
GREEDY_MATCH_RATE = {1: 0.66, 2: 0.77, 3: 0.81, 4: 0.84}

EXPANSION_EVAL = (1, 1, 3, 1, 1, 1, 1, 1)  # Section 6.1


@dataclasses.dataclass(frozen=True)
class Config:
    """One named workload. `P` is the KV prefix length, or (lo, hi) for a ragged batch."""
    cfg: int
    name: str
    dtype: str            # "f32" | "bf16"
    B: int
    H: int
    D: int
    P: object             # int or (lo, hi)
    N: int
    tree: str             # "random_parent" | "expansion" | "random_branching"
    widths: Tuple[int, ...] = ()
    V: int = 0
    logit_std: float = 3.0
    n_ssm: int = 1
    layers: int = 32      # layers of the model the shape comes from
    H_kv: int = 0         # key/value heads (0: as many as query heads)

    @property
    def kv_heads(self) -> int:
        return self.H_kv if self.H_kv > 0 else self.H

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def max_prefix(self) -> int:
        return self.P if isinstance(self.P, int) else self.P[1]

    @property
    def S_cap(self) -> int:
        return self.max_prefix + self.N

    @property
    def seed(self) -> int:
        return BASE_SEED + self.cfg


CONFIGS: Dict[int, Config] = {
    1: Config(1, "tiny-fp32", "f32", B=1, H=4, D=64, P=128, N=8, tree="random_parent", V=64, logit_std=2.0, layers=1),
    2: Config(2, "llama7b-tree16", "bf16", B=8, H=32, D=128, P=1024, N=16, tree="expansion",
              widths=EXPANSION_EVAL, V=32000, layers=32),
    3: Config(3, "llama7b-wide128", "bf16", B=16, H=32, D=128, P=512, N=128, tree="random_branching",
              V=32000, n_ssm=3, layers=32),
    4: Config(4, "llama65b-tree64", "bf16", B=16, H=64, D=128, P=2048, N=64, tree="expansion",
              widths=EXPANSION_EVAL * 2, V=0, layers=80),
    5: Config(5, "llama7b-long", "bf16", B=4, H=32, D=128, P=(8192, 16384), N=32, tree="expansion",
              widths=(1, 1, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1), V=32000, layers=32),
}


# --------------------------------------------------------------------------------------------------
# tree shapes (Definition 3.1: every node has a parent; node 0 is the root, parent[0] = -1)
# --------------------------------------------------------------------------------------------------

def depth_of(parent: Sequence[int]) -> np.ndarray:
    """depth[0] = 0, depth[i] = depth[parent[i]] + 1 (requires parent[i] < i)."""
    d = np.zeros(len(parent), dtype=np.int32)
    for i in range(1, len(parent)):
        d[i] = d[parent[i]] + 1
    return d


def children_of(parent: Sequence[int]) -> List[List[int]]:
    ch: List[List[int]] = [[] for _ in parent]
    for i in range(1, len(parent)):
        ch[parent[i]].append(i)
    return ch


def dfs_relabel(parent: Sequence[int]) -> np.ndarray:
    """Renumber the nodes in depth-first (pre-order) visiting order, children in their given order."""
    ch = children_of(parent)
    order: List[int] = []
    stack = [0]
    while stack:
        u = stack.pop()
        order.append(u)
        stack.extend(reversed(ch[u]))
    new_id = {old: new for new, old in enumerate(order)}
    out = np.full(len(parent), -1, dtype=np.int32)
    for old in range(1, len(parent)):
        out[new_id[old]] = new_id[parent[old]]
    return out


def tree_random_parent(rng: np.random.Generator, n: int) -> np.ndarray:
    """parent[i] uniform in {0..i-1}; a valid topological order that is generally not depth-first."""
    p = np.full(n, -1, dtype=np.int32)
    for i in range(1, n):
        p[i] = rng.integers(0, i)
    return p


def tree_expansion(widths: Sequence[int], n: int) -> np.ndarray:
    """Expansion-based tree (Section 3): every node of level j gets widths[j] children. The tree is
    generated level by level, cut to its first n nodes in generation order, then renumbered
    depth-first."""
    parent = [-1]
    level = [0]
    for k in widths:
        if len(parent) >= n:      # only the first n nodes in generation order are kept
            break
        nxt = []
        for u in level:
            for _ in range(k):
                if len(parent) < n:
                    parent.append(u)
                    nxt.append(len(parent) - 1)
        level = nxt
    if len(parent) < n:
        raise ValueError(f"expansion {tuple(widths)} yields {len(parent)} nodes < {n}")
    return dfs_relabel(parent[:n])


def tree_random_branching(rng: np.random.Generator, n: int, max_children: int = 4, max_depth: int = 16) -> np.ndarray:
    """Repeatedly give a random childless node of depth < max_depth between 1 and max_children
    children until n nodes exist; renumbered depth-first. Looks like a merge of several drafts."""
    parent = [-1]
    depth = [0]
    leaves = [0]
    while len(parent) < n:
        cand = [u for u in leaves if depth[u] < max_depth]
        u = cand[int(rng.integers(0, len(cand)))]
        leaves.remove(u)
        c = int(rng.integers(1, max_children + 1))
        for _ in range(c):
            if len(parent) == n:
                break
            parent.append(u)
            depth.append(depth[u] + 1)
            leaves.append(len(parent) - 1)
    return dfs_relabel(parent)


def make_trees(cfg: Config, rng: np.random.Generator) -> np.ndarray:
    """tree_parent [B, N] int32 for a config."""
    out = np.zeros((cfg.B, cfg.N), dtype=np.int32)
    for b in range(cfg.B):
        if cfg.tree == "random_parent":
            out[b] = tree_random_parent(rng, cfg.N)
        elif cfg.tree == "expansion":
            out[b] = tree_expansion(cfg.widths, cfg.N)
        elif cfg.tree == "random_branching":
            out[b] = tree_random_branching(rng, cfg.N)
        else:
            raise ValueError(cfg.tree)
    return out


# --------------------------------------------------------------------------------------------------
# attention-side tensors
# --------------------------------------------------------------------------------------------------

_BIG = 1 << 22     # elements per independently seeded block of a large array


def _normal(rng: np.random.Generator, shape, dtype: torch.dtype, scale: float = 1.0) -> torch.Tensor:
    """N(0, scale) values of `shape` in `dtype`. Large arrays are filled block-wise by child generators
    whose seeds are drawn from `rng`, on a few threads; the result does not depend on the threading."""
    n = int(np.prod(shape))
    if n <= _BIG:
        x = rng.standard_normal(shape, dtype=np.float32)
    else:
        x = np.empty(n, dtype=np.float32)
        nblk = (n + _BIG - 1) // _BIG
        seeds = rng.integers(0, 2 ** 63 - 1, size=nblk)

        def fill(i):
            lo, hi = i * _BIG, min((i + 1) * _BIG, n)
            np.random.Generator(np.random.PCG64(int(seeds[i]))).standard_normal(out=x[lo:hi], dtype=np.float32)

        with concurrent.futures.ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(fill, range(nblk)))
        x = x.reshape(shape)
    if scale != 1.0:
        x *= np.float32(scale)
    return torch.from_numpy(x).to(dtype)


def make_prefix_len(cfg: Config, rng: np.random.Generator) -> np.ndarray:
    if isinstance(cfg.P, int):
        return np.full(cfg.B, cfg.P, dtype=np.int32)
    lo, hi = cfg.P
    return rng.integers(lo, hi + 1, size=cfg.B).astype(np.int32)


def make_attention_inputs(cfg: Config, seed: Optional[int] = None, n_layers: int = 1,
                          S_cap: Optional[int] = None) -> Dict[str, object]:
    """Per-layer Q, new K/V of the tree tokens and caches holding the prefix.

    Cache rows at and beyond prefix_len[b] hold large finite garbage (N(0,1)*100) so that any read of
    a row that should not be visible shows up in the outputs.
    Returns CPU tensors: q : [L][B,N,H,D]; k_new, v_new : [L][B,N,H_kv,D]; k_cache, v_cache : [L][B,H_kv,S_cap,D];
    prefix_len [B] int32; tree_parent, tree_depth [B,N] int32.
    """
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    S = cfg.S_cap if S_cap is None else S_cap
    dt = cfg.torch_dtype
    parent = make_trees(cfg, rng)
    depth = np.stack([depth_of(p) for p in parent])
    prefix_len = make_prefix_len(cfg, rng)
    if int(prefix_len.max()) + cfg.N > S:
        raise ValueError("S_cap too small")
    out: Dict[str, object] = {
        "cfg": cfg, "S_cap": S,
        "tree_parent": torch.from_numpy(parent), "tree_depth": torch.from_numpy(depth),
        "prefix_len": torch.from_numpy(prefix_len),
        "q": [], "k_new": [], "v_new": [], "k_cache": [], "v_cache": [],
    }
    for _ in range(n_layers):
        out["q"].append(_normal(rng, (cfg.B, cfg.N, cfg.H, cfg.D), dt))
        out["k_new"].append(_normal(rng, (cfg.B, cfg.N, cfg.kv_heads, cfg.D), dt))
        out["v_new"].append(_normal(rng, (cfg.B, cfg.N, cfg.kv_heads, cfg.D), dt))
        for name in ("k_cache", "v_cache"):
            c = torch.empty((cfg.B, cfg.kv_heads, S, cfg.D), dtype=dt)
            for b in range(cfg.B):
                p = int(prefix_len[b])
                c[b, :, :p] = _normal(rng, (cfg.kv_heads, p, cfg.D), dt)
                c[b, :, p:] = _normal(rng, (cfg.kv_heads, S - p, cfg.D), dt, scale=100.0)
            out[name].append(c)
    return out


def to_paged(caches: Sequence[torch.Tensor], prefix_len, N: int, block_tokens: int, rng: np.random.Generator,
             spare_blocks: int = 3, max_blocks: Optional[int] = None, unused_entry: int = -1):
    """Re-lays contiguous caches [B,H_kv,S_cap,D] out as pools of blocks behind one block table (a storage
    layout only: no arithmetic of the method). Request b gets ceil((prefix_len[b] + N) / block_tokens) blocks,
    placed at random in the pool among `spare_blocks` unused ones; the pool's other rows hold large finite
    garbage; table entries of blocks a request does not reach hold `unused_entry`.
    Returns (pools: list of [n_blocks,H_kv,block_tokens,D], block_table int32 [B,max_blocks])."""
    B, H, S, D = caches[0].shape
    bt = block_tokens
    need_blocks = (S + bt - 1) // bt
    mb = need_blocks if max_blocks is None else max_blocks
    used = [min(mb, (int(prefix_len[b]) + N + bt - 1) // bt) for b in range(B)]
    n_blocks = sum(used) + spare_blocks
    perm = rng.permutation(n_blocks)
    table = np.full((B, mb), unused_entry, dtype=np.int32)
    nxt = 0
    for b in range(B):
        for j in range(used[b]):
            table[b, j] = perm[nxt]
            nxt += 1
    pools = []
    for c in caches:
        pool = _normal(rng, (n_blocks, H, bt, D), c.dtype, scale=100.0)
        for b in range(B):
            for j in range(used[b]):
                rows = min(bt, S - j * bt)
                if rows > 0:
                    pool[int(table[b, j]), :, :rows] = c[b, :, j * bt:j * bt + rows]
        pools.append(pool)
    return pools, torch.from_numpy(table)


# --------------------------------------------------------------------------------------------------
# verification-side tensors
# --------------------------------------------------------------------------------------------------

def make_logits(cfg: Config, rng: np.random.Generator, dtype: torch.dtype = torch.float32) -> torch.Tensor:
    """LLM logits [B,N,V] ~ N(0, std) (std, not variance)."""
    return _normal(rng, (cfg.B, cfg.N, cfg.V), torch.float32, scale=cfg.logit_std).to(dtype)


def plant_greedy_tokens(rng: np.random.Generator, logits: torch.Tensor, parent: np.ndarray) -> np.ndarray:
    """tree_token [B,N]: for a node with c children, with probability GREEDY_MATCH_RATE[c] one child
    (uniformly chosen) carries the position of the node's largest logit; siblings are distinct unless
    the vocabulary is too small for that."""
    B, N, V = logits.shape
    top = torch.argmax(logits.float(), dim=-1).numpy()   # only used to place a matching token
    tok = rng.integers(0, V, size=(B, N)).astype(np.int32)
    for b in range(B):
        ch = children_of(parent[b])
        for u in range(N):
            c = len(ch[u])
            if c == 0:
                continue
            used = set()
            hit = -1
            if rng.random() < GREEDY_MATCH_RATE.get(c, 0.84):
                hit = ch[u][int(rng.integers(0, c))]
            for v in ch[u]:
                if v == hit:
                    t = int(top[b, u])
                else:
                    t = int(rng.integers(0, V))
                    for _ in range(32):      # distinct non-matching siblings when the vocabulary allows it
                        if t not in used and t != int(top[b, u]):
                            break
                        t = int(rng.integers(0, V))
                used.add(t)
                tok[b, v] = t
    return tok


def _softmax_rows(x: np.ndarray) -> np.ndarray:
    """Row softmax used only to manufacture draft distributions (inputs), in float64."""
    x = x.astype(np.float64)
    x = x - x.max(axis=-1, keepdims=True)
    e = np.exp(x)
    return e / e.sum(axis=-1, keepdims=True)


def make_ssm(cfg: Config, rng: np.random.Generator, logits: torch.Tensor, parent: np.ndarray,
             tau: Optional[float] = 1.2, n_ssm: Optional[int] = None):
    """Draft (SSM) distributions and the tokens they propose.

    One row of `probs_ssm` per (parent node, SSM) that owns children. tau=None draws the row
    independently of the LLM (softmax of N(0, logit_std)); otherwise it is
    softmax(llm_logits[parent] + tau * N(0,1)). Every child's token is sampled from its row.
    Returns probs_ssm [R,V] float32, ssm_row [B,N] int32 (-1 at the root), tree_token [B,N] int32.
    """
    B, N, V = logits.shape
    m = cfg.n_ssm if n_ssm is None else n_ssm
    rows: List[np.ndarray] = []
    ssm_row = np.full((B, N), -1, dtype=np.int32)
    tok = np.zeros((B, N), dtype=np.int32)
    lg = logits.float().numpy()
    for b in range(B):
        tok[b, 0] = int(rng.integers(0, V))
        ch = children_of(parent[b])
        for u in range(N):
            if not ch[u]:
                continue
            owner = rng.integers(0, m, size=len(ch[u]))
            for s in sorted(set(int(o) for o in owner)):
                if tau is None:
                    z = rng.standard_normal(V) * cfg.logit_std
                else:
                    z = lg[b, u].astype(np.float64) + tau * rng.standard_normal(V)
                qrow = _softmax_rows(z[None, :])[0].astype(np.float32)
                rows.append(qrow)
                r = len(rows) - 1
                cdf = np.cumsum(qrow.astype(np.float64))
                for v, o in zip(ch[u], owner):
                    if int(o) != s:
                        continue
                    ssm_row[b, v] = r
                    tok[b, v] = min(int(np.searchsorted(cdf, rng.random() * cdf[-1], side="right")), V - 1)
    probs = np.stack(rows) if rows else np.zeros((0, V), dtype=np.float32)
    return torch.from_numpy(probs), ssm_row, tok


def make_uniforms(rng: np.random.Generator, B: int, N: int):
    """u_accept [B,N], u_order [B,N], u_final [B]: float32 in [0,1)."""
    def u(shape):
        x = rng.random(shape, dtype=np.float32)
        return np.minimum(x, np.float32(1.0 - 2.0 ** -24))
    return u((B, N)), u((B, N)), u((B,))


def make_verify_inputs(cfg: Config, seed: Optional[int] = None, mode: str = "greedy",
                       parent: Optional[np.ndarray] = None, logits_dtype: torch.dtype = torch.float32,
                       tau: Optional[float] = 1.2) -> Dict[str, object]:
    """Inputs of one verification call. mode = "greedy" | "stochastic"."""
    rng = np.random.default_rng((cfg.seed if seed is None else seed) + 500)
    if parent is None:
        parent = make_trees(cfg, rng)
    logits = make_logits(cfg, rng, logits_dtype)
    out: Dict[str, object] = {"cfg": cfg, "tree_parent": torch.from_numpy(np.ascontiguousarray(parent)),
                              "logits": logits}
    if mode == "greedy":
        out["tree_token"] = torch.from_numpy(plant_greedy_tokens(rng, logits, parent))
    else:
        probs, ssm_row, tok = make_ssm(cfg, rng, logits, parent, tau=tau)
        ua, uo, uf = make_uniforms(rng, cfg.B, cfg.N)
        out.update(probs_ssm=probs, ssm_row=torch.from_numpy(ssm_row), tree_token=torch.from_numpy(tok),
                   u_accept=torch.from_numpy(ua), u_order=torch.from_numpy(uo), u_final=torch.from_numpy(uf))
        out["rng"] = rng   # stream continues for re-draws of fragile uniforms
    return out


def random_accepted_paths(rng: np.random.Generator, parent: np.ndarray, max_len: int = 9):
    """For the commit-only config: per request a path length ~ U{1..max_len} (cut to the tree's
    depth), a uniformly random node of that depth, and its root-to-node chain.
    Returns accepted_path [B,Lmax] int32 (padded with -1), accepted_len [B] int32."""
    B, N = parent.shape
    Lmax = int(max(depth_of(p).max() for p in parent)) + 1
    path = np.full((B, Lmax), -1, dtype=np.int32)
    ln = np.zeros(B, dtype=np.int32)
    for b in range(B):
        d = depth_of(parent[b])
        want = min(int(rng.integers(1, max_len + 1)), int(d.max()) + 1)
        nodes = np.nonzero(d == want - 1)[0]
        u = int(nodes[int(rng.integers(0, len(nodes)))])
        chain = []
        while u >= 0:
            chain.append(u)
            u = int(parent[b, u])
        chain.reverse()
        path[b, :len(chain)] = chain
        ln[b] = len(chain)
    return path, ln


def make_rope_tables(n_positions: int, D: int, theta: float = 10000.0):
    """cos / sin tables [n_positions, D/2] of the rotary embedding, float32 (computed in float64):
    angle(position, j) = position * theta ** (-2 j / D). Inputs of the append-with-rotation call."""
    j = np.arange(D // 2, dtype=np.float64)
    ang = np.arange(n_positions, dtype=np.float64)[:, None] * theta ** (-2.0 * j / D)[None, :]
    return torch.from_numpy(np.cos(ang).astype(np.float32)), torch.from_numpy(np.sin(ang).astype(np.float32))
