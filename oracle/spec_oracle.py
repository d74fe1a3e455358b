"""CPU oracle for tree-based parallel decoding (SpecInfer, arxiv 2305.09781).

TEST INFRASTRUCTURE ONLY. This file is the plain, slow, float64 statement of what the hot path
computes. It is imported by tests, by the smoke check and by the benchmark's CPU-baseline leg, and
by nothing else; it shares no code with the GPU library and never calls it.

What each function follows:
  ancestor_matrix        Definition 3.1 (S_u = S_parent(u) ++ {t_u}) and Section 4.2 (topology-aware
                         causal mask: a tree token may see its ancestors and itself, nothing else)
  kv_append              Section 4.2, "depth-first search to update key-value cache": one cache
                         region holds the whole tree, token i at row prefix_len + i
  rope_queries           the queries of the tree tokens under the same embedding (position prefix_len + depth)
  rope_rotate, kv_append_rope  the same append with the rotary embedding of the paper's LLaMA models
                         applied to the keys at position prefix_len + depth (a step adjacent to the path)
  tree_attention         Definition 4.1 with the attention equations of Section 4.1 (scores scaled by
                         1/sqrt(d), masked entries -inf, softmax, times V)
  verify_greedy          Algorithm 2, VerifyGreedy
  verify_stochastic      Algorithm 2, VerifyStochastic (multi-step speculative sampling)
  sample_nodes, verify_naive  naive sampling, the alternative of Section 4.3 (Theorem 4.3, Table 3)
  expand_topk, tree_merge     Section 3: one step of expansion-based construction; Definition 3.2
  kv_commit              Algorithm 2 main loop (verified tokens are appended to the sequence), so the
                         K/V rows of the accepted path must become the contiguous prefix
  lm_head_logits, lm_head_argmax, softmax_stats
                         the LLM's output projection in front of VerifyGreedy (Algorithm 2 takes O(u) from the
                         LLM's distribution at node u; for greedy decoding only its arg-max is needed): logits =
                         hidden . W^T, O(u) = argmax, lowest token id on ties. A step adjacent to the path.
  paged_rows, paged_gather, kv_append_paged, tree_attention_paged, kv_commit_paged
                         the same steps on a cache kept as a pool of blocks behind a block table (a
                         storage layout next to the path, not in the paper): logical row s of request b
                         is row s % block_tokens of block table[b, s // block_tokens], nothing else changes

Parity pins (tests/test_oracle_*.py): per-path brute-force causal attention, chain/star/N=1 special
cases against a library routine, constant-V and non-interference invariants (attention); exhaustive
path enumeration and incremental decoding on a bigram model (greedy); exact cell-by-cell enumeration
against a closed-form law, Theorem 4.2 and 4.3 in closed form, chi-square over many seeds
(stochastic); brute-force inverse CDF, the exact first-step law, the closed-form rejection probability of
Theorem 4.3 and the low-temperature limit against the greedy verifier (naive sampling); round trips and
overlapping-path cases (append / commit); sequence-set equality by brute force, idempotence, chains
merging into a trie (tree merge); scalar selection loop and the argmax special case (top-k); identity
tables against the contiguous functions, invariance under a relabelling of the blocks, shared prefix blocks
and a hand-derived two-block case (paged caches); scalar triple loop, one-hot weights and a hand-derived case
(LM head). No function is unpinned.

Readings taken where the paper is silent are listed next to each function.
"""
from __future__ import annotations

import numpy as np

# status bits reported per request for data-dependent faults
ST_BAD_TREE = 1        # parent[0] != -1, or parent[i] not in [0, i), or depth[i] != depth[parent[i]] + 1
ST_CAPACITY = 2        # prefix_len + N > S_cap, or prefix_len < 0
ST_BAD_PATH = 4        # accepted path: len out of range, path[0] != 0, not strictly increasing, or out of range
ST_ZERO_RESIDUAL = 8   # residual distribution had no mass left (kept previous distribution)
ST_BAD_BLOCK = 16      # paged cache: a block-table entry the request uses lies outside the pool


# ---------------------------------------------------------------------------------------------
# token tree helpers (Definition 3.1)
# ---------------------------------------------------------------------------------------------

def tree_status(parent, depth=None):
    """0 if `parent` (and `depth`, if given) describe a valid linearised token tree, else ST_BAD_TREE."""
    parent = np.asarray(parent)
    n = len(parent)
    if n == 0 or parent[0] != -1:
        return ST_BAD_TREE
    for i in range(1, n):
        if not (0 <= parent[i] < i):
            return ST_BAD_TREE
    if depth is not None:
        depth = np.asarray(depth)
        if depth[0] != 0:
            return ST_BAD_TREE
        for i in range(1, n):
            if depth[i] != depth[parent[i]] + 1:
                return ST_BAD_TREE
    return 0


def ancestor_matrix(parent):
    """anc[i, a] = True iff a is i itself or an ancestor of i (the tokens of S_i inside the tree)."""
    parent = np.asarray(parent)
    n = len(parent)
    anc = np.zeros((n, n), dtype=bool)
    for i in range(n):
        u = i
        while u >= 0:
            anc[i, u] = True
            u = int(parent[u])
    return anc


def children(parent, u):
    return [v for v in range(len(parent)) if parent[v] == u]


# ---------------------------------------------------------------------------------------------
# KV append  (Section 4.2)
# ---------------------------------------------------------------------------------------------

def kv_append(k_cache, v_cache, k_new, v_new, prefix_len):
    """cache[b, h, prefix_len[b] + i, :] = new[b, i, h, :] for every tree token i. In place.

    k_cache, v_cache: [B,H,S_cap,D]; k_new, v_new: [B,N,H,D]. Returns status [B]; a request whose
    tree does not fit (prefix_len + N > S_cap) is left untouched and flagged ST_CAPACITY."""
    B, N = k_new.shape[0], k_new.shape[1]
    S_cap = k_cache.shape[2]
    status = np.zeros(B, dtype=np.int32)
    for b in range(B):
        p = int(prefix_len[b])
        if p < 0 or p + N > S_cap:
            status[b] |= ST_CAPACITY
            continue
        for i in range(N):
            k_cache[b, :, p + i, :] = k_new[b, i, :, :]
            v_cache[b, :, p + i, :] = v_new[b, i, :, :]
    return status


def rope_rotate(x, cos, sin):
    """Rotary position embedding of one position, half-split pairing: dimension i < D/2 is paired with
    i + D/2 and the pair is rotated by the angle whose cosine / sine are cos[i] / sin[i].
    x [..., D], cos, sin [D/2]; float64."""
    x = np.asarray(x, dtype=np.float64)
    h = x.shape[-1] // 2
    x1, x2 = x[..., :h], x[..., h:]
    return np.concatenate([x1 * cos - x2 * sin, x2 * cos + x1 * sin], axis=-1)


def round_to_storage(x, storage):
    """float64 values rounded ONCE, to nearest with ties to even, to the storage type: "bf16" (8 significant
    bits; values in bfloat16's normal range, which rotated activations are) or "f32". Returned as float64."""
    x = np.asarray(x, dtype=np.float64)
    if storage != "bf16":
        return x.astype(np.float32).astype(np.float64)
    m, e = np.frexp(x)                       # x = m * 2**e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0) / 256.0, e)   # np.rint rounds halves to even


def kv_append_rope(k_cache, v_cache, k_new, v_new, prefix_len, tree_depth, rope_cos, rope_sin, storage="bf16"):
    """KV append with the rotary embedding applied to the keys on the way in: tree token i of request b
    sits at sequence position prefix_len[b] + tree_depth[b,i] (its depth below the last verified token,
    not its row in the cache), K is rotated by that position's table row and rounded to the cache's
    storage type ("bf16" or "f32"); V is copied. rope_cos, rope_sin: [rope_len, D/2] tables supplied by
    the caller (float32 values). Returns status [B]: ST_CAPACITY if the tree does not fit the cache or a
    position lies outside the tables (request untouched)."""
    B, N = k_new.shape[0], k_new.shape[1]
    S_cap = k_cache.shape[2]
    rope_cos = np.asarray(rope_cos, dtype=np.float64)
    rope_sin = np.asarray(rope_sin, dtype=np.float64)
    status = np.zeros(B, dtype=np.int32)
    for b in range(B):
        p = int(prefix_len[b])
        pos = [p + int(tree_depth[b, i]) for i in range(N)]
        if p < 0 or p + N > S_cap or min(pos) < 0 or max(pos) >= rope_cos.shape[0]:
            status[b] |= ST_CAPACITY
            continue
        for i in range(N):
            rot = rope_rotate(k_new[b, i], rope_cos[pos[i]], rope_sin[pos[i]])          # [H, D]
            k_cache[b, :, p + i, :] = round_to_storage(rot, storage)
            v_cache[b, :, p + i, :] = v_new[b, i, :, :]
    return status


# ---------------------------------------------------------------------------------------------
# tree attention  (Definition 4.1, Section 4.1 equations, Section 4.2 mask)
# ---------------------------------------------------------------------------------------------

def rope_queries(q, prefix_len, tree_depth, rope_cos, rope_sin, S_cap, storage="bf16"):
    """The queries of the tree tokens under the rotary embedding: row (b, i) of every head rotated by position
    prefix_len[b] + tree_depth[b,i] and rounded to the storage type. q [B,N,H,D]; returns (rotated copy,
    status [B]); a request that does not fit S_cap or has a position outside the tables keeps its q
    (ST_CAPACITY), exactly like kv_append_rope."""
    q = np.array(q, dtype=np.float64)
    B, N = q.shape[0], q.shape[1]
    rope_cos = np.asarray(rope_cos, dtype=np.float64)
    rope_sin = np.asarray(rope_sin, dtype=np.float64)
    status = np.zeros(B, dtype=np.int32)
    for b in range(B):
        p = int(prefix_len[b])
        pos = [p + int(tree_depth[b, i]) for i in range(N)]
        if p < 0 or p + N > S_cap or min(pos) < 0 or max(pos) >= rope_cos.shape[0]:
            status[b] |= ST_CAPACITY
            continue
        for i in range(N):
            rot = rope_rotate(q[b, i], rope_cos[pos[i]], rope_sin[pos[i]])
            q[b, i] = round_to_storage(rot, storage)
    return q, status


def tree_attention(q, k_cache, v_cache, tree_parent, prefix_len, softmax_scale=None):
    """Attention output of every tree node over (cached prefix) ++ (its own root-to-node path).

    q: [B,N,H,D]; caches [B,H_kv,S_cap,D] already holding the tree rows at prefix_len[b] + i. H_kv = H
    is the paper's multi-head attention; with fewer K/V heads (grouped-query attention, an extension)
    query head h reads K/V head h // (H / H_kv).
    Returns float64 [B,N,H,D]. A = Q K^T / sqrt(d); mask(A) puts -inf wherever key j is a tree token
    that is neither node i nor one of its ancestors; H = softmax(mask(A)) V.
    Readings: d is the head dimension; a row is never fully masked (a node sees itself)."""
    q = np.asarray(q, dtype=np.float64)
    B, N, H, D = q.shape
    scale = 1.0 / np.sqrt(D) if softmax_scale is None else float(softmax_scale)
    out = np.zeros((B, N, H, D), dtype=np.float64)
    for b in range(B):
        p = int(prefix_len[b])
        L = p + N
        visible = np.concatenate([np.ones((N, p), dtype=bool), ancestor_matrix(tree_parent[b])], axis=1)
        group = H // k_cache.shape[1]
        for h in range(H):
            K = np.asarray(k_cache[b, h // group, :L, :], dtype=np.float64)
            V = np.asarray(v_cache[b, h // group, :L, :], dtype=np.float64)
            A = (q[b, :, h, :] @ K.T) * scale
            A = np.where(visible, A, -np.inf)
            W = np.exp(A - A.max(axis=1, keepdims=True))
            W = W / W.sum(axis=1, keepdims=True)
            out[b, :, h, :] = W @ V
    return out


# ---------------------------------------------------------------------------------------------
# greedy verification  (Algorithm 2, VerifyGreedy)
# ---------------------------------------------------------------------------------------------

def verify_greedy(logits, tree_token, tree_parent):
    """O(u) = argmax of the LLM's logits at node u (lowest token id on ties). Starting at the root,
    move to a child whose token equals O(u) while one exists (lowest node index if several);
    finally append O(u) of the last node reached.

    logits [B,N,V]; returns accepted_path [B,N] (node indices, root first, padded -1),
    accepted_len [B], out_tokens [B,N] (tokens of the accepted children, then the bonus token,
    padded -1; same count as path nodes), node_argmax [B,N]."""
    logits = np.asarray(logits)
    B, N, V = logits.shape
    path = np.full((B, N), -1, dtype=np.int32)
    toks = np.full((B, N), -1, dtype=np.int32)
    ln = np.zeros(B, dtype=np.int32)
    node_argmax = np.zeros((B, N), dtype=np.int32)
    for b in range(B):
        for u in range(N):
            node_argmax[b, u] = int(np.argmax(logits[b, u]))   # first occurrence = lowest id
        u = 0
        k = 0
        path[b, 0] = 0
        while True:
            nxt = -1
            for v in children(tree_parent[b], u):
                if int(tree_token[b, v]) == int(node_argmax[b, u]):
                    nxt = v
                    break
            if nxt < 0:
                break
            toks[b, k] = tree_token[b, nxt]
            k += 1
            path[b, k] = nxt
            u = nxt
        toks[b, k] = node_argmax[b, u]
        ln[b] = k + 1
    return path, ln, toks, node_argmax


# ---------------------------------------------------------------------------------------------
# stochastic verification  (Algorithm 2, VerifyStochastic: multi-step speculative sampling)
# ---------------------------------------------------------------------------------------------

def verify_stochastic(logits, probs_ssm, ssm_row, tree_token, tree_parent, u_accept, u_order, u_final,
                      temperature=1.0, return_margins=False):
    """Multi-step speculative sampling over a token tree.

    At node u: P = softmax(logits[u] / temperature). The children of u are tried in ascending order of
    (u_order[v], v) -- a uniformly random order without replacement. Child s with token x and draft
    distribution Q = probs_ssm[ssm_row[s]] passes iff r <= P(x)/Q(x), r = u_accept[s], evaluated as
    r * Q(x) <= P(x) on float32-rounded values (no division; Q(x) = 0 passes). If it passes, x is
    emitted and the walk moves to s. Otherwise P := norm(max(0, P - Q)) and s is dropped. When no child
    is left (or u is a leaf) the final token is drawn from the current P by inverse CDF over
    ascending token id: the first k with cumsum(P)[k] > u_final * sum(P).

    Readings: the residual persists only across the siblings of one node; an all-zero residual keeps
    the previous P and sets ST_ZERO_RESIDUAL; uniforms are float32 in [0,1) supplied by the caller; a
    node with a negative token is padding (see tree_merge) and is skipped.

    Returns accepted_path [B,N], accepted_len [B], out_tokens [B,N], status [B] and, if asked,
    margins [B,2]: [:,0] the smallest relative gap |r Q(x) - P(x)| / max(...) over the ratio tests
    taken, [:,1] the distance of the final draw's target from the nearest CDF step as a fraction of
    the total mass. They tell how far each decision is from flipping under rounding noise."""
    logits = np.asarray(logits, dtype=np.float64)
    probs_ssm = np.asarray(probs_ssm, dtype=np.float64)
    B, N, V = logits.shape
    path = np.full((B, N), -1, dtype=np.int32)
    toks = np.full((B, N), -1, dtype=np.int32)
    ln = np.zeros(B, dtype=np.int32)
    status = np.zeros(B, dtype=np.int32)
    margins = np.full((B, 2), np.inf)
    for b in range(B):
        u = 0
        k = 0
        path[b, 0] = 0
        while True:
            z = logits[b, u] / float(temperature)
            P = np.exp(z - z.max())
            P = P / P.sum()
            H = sorted((v for v in children(tree_parent[b], u) if int(tree_token[b, v]) >= 0),
                       key=lambda v: (float(u_order[b, v]), v))   # token < 0: padding node, never a candidate
            accepted = False
            for s in H:
                x = int(tree_token[b, s])
                Q = probs_ssm[int(ssm_row[b, s])]
                r = np.float32(u_accept[b, s])
                lhs = np.float32(r * np.float32(Q[x]))
                rhs = np.float32(P[x])
                denom = max(float(rhs), float(lhs), 1e-300)
                margins[b, 0] = min(margins[b, 0], abs(float(lhs) - float(rhs)) / denom)
                if lhs <= rhs:
                    toks[b, k] = x
                    k += 1
                    path[b, k] = s
                    u = s
                    accepted = True
                    break
                R = np.maximum(0.0, P - Q)
                Z = R.sum()
                if Z > 0.0:
                    P = R / Z
                else:
                    status[b] |= ST_ZERO_RESIDUAL
            if not accepted:
                break
        cdf = np.cumsum(P)
        target = float(np.float32(u_final[b])) * cdf[-1]
        x_next = int(np.searchsorted(cdf, target, side="right"))   # first k with cdf[k] > target
        x_next = min(x_next, V - 1)
        lo = cdf[x_next - 1] if x_next > 0 else -np.inf
        margins[b, 1] = min((target - lo) / cdf[-1], (cdf[x_next] - target) / cdf[-1])
        toks[b, k] = x_next
        ln[b] = k + 1
    if return_margins:
        return path, ln, toks, status, margins
    return path, ln, toks, status


# ---------------------------------------------------------------------------------------------
# naive sampling  (Section 4.3: the straightforward alternative multi-step speculative sampling is
# compared with; Theorem 4.3, Table 3)
# ---------------------------------------------------------------------------------------------

def sample_nodes(logits, u_sample, temperature=1.0):
    """x_u ~ softmax(logits[u] / temperature) for every node, drawn by inverse CDF over ascending token
    id with the caller's uniform: the first k with cumsum(P)[k] > u_sample[u] * sum(P).

    Returns node_sample [B,N] and margins [B,N]: the distance of each draw's target from the nearest
    CDF step as a fraction of the total mass."""
    logits = np.asarray(logits, dtype=np.float64)
    B, N, V = logits.shape
    out = np.zeros((B, N), dtype=np.int32)
    margins = np.zeros((B, N))
    for b in range(B):
        for u in range(N):
            z = logits[b, u] / float(temperature)
            P = np.exp(z - z.max())
            cdf = np.cumsum(P)
            target = float(np.float32(u_sample[b, u])) * cdf[-1]
            x = min(int(np.searchsorted(cdf, target, side="right")), V - 1)
            lo = cdf[x - 1] if x > 0 else -np.inf
            margins[b, u] = min((target - lo) / cdf[-1], (cdf[x] - target) / cdf[-1])
            out[b, u] = x
    return out, margins


def verify_naive(logits, tree_token, tree_parent, u_sample, temperature=1.0):
    """Naive sampling: at node u draw x ~ P(. | u, LLM); if x is the token of a child of u (lowest node
    index if several children carry it), emit x and move there; otherwise emit x and stop.

    Readings: one uniform per node, supplied by the caller; inverse CDF as in sample_nodes.
    Returns accepted_path [B,N], accepted_len [B], out_tokens [B,N], node_sample [B,N]."""
    node_sample, _ = sample_nodes(logits, u_sample, temperature)
    B, N = node_sample.shape
    path = np.full((B, N), -1, dtype=np.int32)
    toks = np.full((B, N), -1, dtype=np.int32)
    ln = np.zeros(B, dtype=np.int32)
    for b in range(B):
        u = 0
        k = 0
        path[b, 0] = 0
        while True:
            x = int(node_sample[b, u])
            toks[b, k] = x
            nxt = -1
            for v in children(tree_parent[b], u):
                if int(tree_token[b, v]) == x:
                    nxt = v
                    break
            if nxt < 0:
                break
            k += 1
            path[b, k] = nxt
            u = nxt
        ln[b] = k + 1
    return path, ln, toks, node_sample


# ---------------------------------------------------------------------------------------------
# token-tree construction  (Section 3: expansion-based construction, Definition 3.2 token tree merge)
# ---------------------------------------------------------------------------------------------

def expand_topk(logits, k):
    """Expansion-based construction, one step: the k most likely next tokens of every frontier node,
    most likely first (ties: lowest token id). logits [..., V] -> token ids [..., k]."""
    logits = np.asarray(logits, dtype=np.float64)
    V = logits.shape[-1]
    flat = logits.reshape(-1, V)
    out = np.zeros((flat.shape[0], k), dtype=np.int32)
    for r in range(flat.shape[0]):
        ids = sorted(range(V), key=lambda i: (-flat[r, i], i))
        out[r] = ids[:k]
    return out.reshape(logits.shape[:-1] + (k,))


def tree_merge(in_parent, in_token, in_size, n_out):
    """Token tree merge (Definition 3.2) of the M trees of one request: the merged tree holds exactly the
    token sequences S_u of the input trees, each once. Input tree i has in_size[i] nodes (root first,
    parent[u] < u) out of the Nin slots of in_parent[i] / in_token[i]; all roots carry the same token.

    Readings (the paper fixes none of these): a merged node's children are ordered by first appearance
    when the trees are scanned in order i = 0..M-1, nodes in index order; nodes are numbered in
    depth-first (pre-)order; out_ssm is the lowest tree index whose tree holds the node's sequence;
    slots past the merged size are padding nodes (parent 0, depth 1, token -1, ssm -1) that no verifier
    ever accepts.

    Returns (parent [n_out], depth [n_out], token [n_out], ssm [n_out], size, node_map [M,Nin], status):
    node_map[i,u] = merged index of input node u of tree i (-1 for unused slots); status ST_BAD_TREE for
    a malformed input tree or differing root tokens, ST_CAPACITY if more than n_out sequences (size 0)."""
    in_parent = np.asarray(in_parent)
    in_token = np.asarray(in_token)
    M, Nin = in_parent.shape
    node_map = np.full((M, Nin), -1, dtype=np.int32)
    pad = (np.zeros(n_out, np.int32), np.ones(n_out, np.int32), np.full(n_out, -1, np.int32), np.full(n_out, -1, np.int32))

    def fail(bit):
        par, dep, tok, ssm = (a.copy() for a in pad)
        par[0], dep[0] = -1, 0
        return par, dep, tok, ssm, 0, np.full((M, Nin), -1, dtype=np.int32), bit

    nodes = []          # merged nodes in order of first appearance: [parent id, token, tree index]
    trie = {}
    for i in range(M):
        sz = int(in_size[i])
        if sz < 1 or sz > Nin or int(in_parent[i, 0]) != -1 or int(in_token[i, 0]) != int(in_token[0, 0]):
            return fail(ST_BAD_TREE)
        if i == 0:
            nodes.append([-1, int(in_token[0, 0]), 0])
        ids = [0] * sz
        for u in range(1, sz):
            p = int(in_parent[i, u])
            if not (0 <= p < u) or int(in_token[i, u]) < 0:
                return fail(ST_BAD_TREE)
            key = (ids[p], int(in_token[i, u]))
            if key not in trie:
                trie[key] = len(nodes)
                nodes.append([ids[p], int(in_token[i, u]), i])
            ids[u] = trie[key]
        node_map[i, :sz] = ids
    if len(nodes) > n_out:
        return fail(ST_CAPACITY)
    kids = [[] for _ in nodes]
    for j in range(1, len(nodes)):
        kids[nodes[j][0]].append(j)
    order = []          # depth-first pre-order
    stack = [0]
    while stack:
        j = stack.pop()
        order.append(j)
        stack.extend(reversed(kids[j]))
    new_id = {j: n for n, j in enumerate(order)}
    par, dep, tok, ssm = (a.copy() for a in pad)
    for j, (pj, tj, sj) in enumerate(nodes):
        n = new_id[j]
        par[n] = -1 if pj < 0 else new_id[pj]
        tok[n], ssm[n] = tj, sj
    for n in range(len(nodes)):
        dep[n] = 0 if par[n] < 0 else dep[par[n]] + 1
    node_map = np.where(node_map >= 0, np.vectorize(lambda j: new_id.get(j, -1))(node_map), -1).astype(np.int32)
    return par, dep, tok, ssm, len(nodes), node_map, 0


# ---------------------------------------------------------------------------------------------
# KV commit  (Algorithm 2 main loop: S.append(t) for every verified token)
# ---------------------------------------------------------------------------------------------

def path_status(path_b, len_b, parent_b):
    """0 if path_b[:len_b] is a root-to-node chain of the tree, else ST_BAD_PATH."""
    n = len(parent_b)
    if not (1 <= len_b <= n) or len_b > len(path_b) or path_b[0] != 0:
        return ST_BAD_PATH
    for k in range(1, len_b):
        if not (0 < path_b[k] < n) or parent_b[path_b[k]] != path_b[k - 1]:
            return ST_BAD_PATH
    return 0


def kv_commit(k_caches, v_caches, accepted_path, accepted_len, prefix_len, N=None):
    """For every layer's cache and every request: row prefix_len + k <- row prefix_len + path[k],
    k = 0..len-1 (K and V), so the accepted tokens' K/V become the contiguous continuation of the
    prefix. Returns (prefix_len_out = prefix_len + len, status [B]). In place; rows at and beyond
    the new prefix length are unspecified afterwards.

    Only the structure a copy needs is checked here (path[0] = 0, strictly increasing, inside the
    tree's N rows); requests failing it are left untouched with prefix_len_out = prefix_len."""
    B = len(prefix_len)
    out_len = np.array(prefix_len, dtype=np.int32).copy()
    status = np.zeros(B, dtype=np.int32)
    for b in range(B):
        p = int(prefix_len[b])
        n = int(accepted_len[b])
        pb = [int(x) for x in accepted_path[b][:max(n, 0)]]
        limit = (k_caches[0].shape[2] - p) if N is None else N
        if p < 0 or p + limit > k_caches[0].shape[2]:      # the tree region does not fit: skipped
            status[b] |= ST_CAPACITY
            continue
        ok = 1 <= n <= len(accepted_path[b]) and pb[0] == 0 and all(pb[k] > pb[k - 1] for k in range(1, n)) \
            and pb[-1] < limit
        if not ok:
            status[b] |= ST_BAD_PATH
            continue
        for kc, vc in zip(k_caches, v_caches):
            for k in range(n):           # increasing k is safe: destination row <= source row
                kc[b, :, p + k, :] = kc[b, :, p + pb[k], :]
                vc[b, :, p + k, :] = vc[b, :, p + pb[k], :]
        out_len[b] = p + n
    return out_len, status


# ---------------------------------------------------------------------------------------------
# Paged caches: the same steps on a pool of blocks behind a block table
# ---------------------------------------------------------------------------------------------

def paged_rows(block_table, block_tokens, n_blocks, b, rows):
    """(block, row inside the block, entry inside the pool?) of every logical row in `rows` of request b."""
    out = []
    for s in rows:
        e = int(block_table[b, s // block_tokens])
        out.append((e, s % block_tokens, 0 <= e < n_blocks))
    return out


def paged_gather(pool, block_table, block_tokens, n_rows):
    """The logical caches [B,H,max(n_rows),D] a pool [n_blocks,H,block_tokens,D] stands for: rows
    0..n_rows[b]-1 of request b (the rest zero). Every entry used must lie inside the pool."""
    B = block_table.shape[0]
    n_blocks, H, _, D = pool.shape
    out = np.zeros((B, H, int(max(n_rows)), D), dtype=pool.dtype)
    for b in range(B):
        for s, (e, r, ok) in enumerate(paged_rows(block_table, block_tokens, n_blocks, b, range(int(n_rows[b])))):
            assert ok, "paged_gather: block-table entry outside the pool"
            out[b, :, s, :] = pool[e, :, r, :]
    return out


def kv_append_paged(k_pool, v_pool, block_table, block_tokens, S_cap, k_new, v_new, prefix_len):
    """kv_append on paged caches: logical row prefix_len[b] + i of request b receives new[b, i]. In place.
    A request that does not fit its logical capacity S_cap is skipped (ST_CAPACITY); a row whose block
    lies outside the pool is not written and the request is flagged ST_BAD_BLOCK."""
    B, N = k_new.shape[0], k_new.shape[1]
    status = np.zeros(B, dtype=np.int32)
    for b in range(B):
        p = int(prefix_len[b])
        if p < 0 or p + N > S_cap:
            status[b] |= ST_CAPACITY
            continue
        for i, (e, r, ok) in enumerate(paged_rows(block_table, block_tokens, k_pool.shape[0], b, range(p, p + N))):
            if not ok:
                status[b] |= ST_BAD_BLOCK
                continue
            k_pool[e, :, r, :] = k_new[b, i, :, :]
            v_pool[e, :, r, :] = v_new[b, i, :, :]
    return status


def tree_attention_paged(q, k_pool, v_pool, block_table, block_tokens, tree_parent, prefix_len, softmax_scale=None):
    """tree_attention over the logical caches the pools stand for (every request must fit and use blocks
    inside the pool: the failure cases are those of the contiguous function plus ST_BAD_BLOCK, whose output
    is unspecified)."""
    N = q.shape[1]
    n_rows = [int(p) + N for p in prefix_len]
    k = paged_gather(k_pool, block_table, block_tokens, n_rows)
    v = paged_gather(v_pool, block_table, block_tokens, n_rows)
    return tree_attention(q, k, v, tree_parent, prefix_len, softmax_scale)


def kv_commit_paged(k_pools, v_pools, block_table, block_tokens, S_cap, accepted_path, accepted_len, prefix_len, N):
    """kv_commit on paged caches: logical row prefix_len + k <- logical row prefix_len + path[k]. In place.
    Returns (prefix_len_out, status). A request with a block of its tree rows [prefix_len, prefix_len + N)
    outside the pool is left untouched and flagged ST_BAD_BLOCK."""
    B = len(prefix_len)
    out_len = np.array(prefix_len, dtype=np.int32).copy()
    status = np.zeros(B, dtype=np.int32)
    n_blocks = k_pools[0].shape[0]
    for b in range(B):
        p = int(prefix_len[b])
        n = int(accepted_len[b])
        pb = [int(x) for x in accepted_path[b][:max(n, 0)]]
        if p < 0 or p + N > S_cap:
            status[b] |= ST_CAPACITY
            continue
        ok = 1 <= n <= len(accepted_path[b]) and n <= N and pb[0] == 0 and \
            all(pb[k] > pb[k - 1] for k in range(1, n)) and pb[-1] < N
        if not ok:
            status[b] |= ST_BAD_PATH
            continue
        where = paged_rows(block_table, block_tokens, n_blocks, b, range(p, p + N))
        if not all(w[2] for w in where):
            status[b] |= ST_BAD_BLOCK
            continue
        for kc, vc in zip(k_pools, v_pools):
            for k in range(n):           # increasing k is safe: destination row <= source row
                (ed, rd, _), (es, rs, _) = where[k], where[pb[k]]
                kc[ed, :, rd, :] = kc[es, :, rs, :]
                vc[ed, :, rd, :] = vc[es, :, rs, :]
        out_len[b] = p + n
    return out_len, status


# ---------------------------------------------------------------------------------------------
# LM head in front of the greedy verifier
# ---------------------------------------------------------------------------------------------

def lm_head_logits(hidden, weight):
    """logits[m, v] = sum_k hidden[m, k] * weight[v, k] in float64 (hidden [M,K], weight [V,K])."""
    return np.asarray(hidden, dtype=np.float64) @ np.asarray(weight, dtype=np.float64).T


def lm_head_argmax(hidden, weight):
    """O(u) for every row: (argmax over the vocabulary with the lowest token id on ties, the maximum, and
    the gap to the runner-up: a row whose gap is within float32 rounding of zero has no unique answer)."""
    logits = lm_head_logits(hidden, weight)
    arg = logits.argmax(axis=1).astype(np.int32)          # numpy: first maximum = lowest id
    top = logits.max(axis=1)
    rest = logits.copy()
    rest[np.arange(logits.shape[0]), arg] = -np.inf
    gap = top - rest.max(axis=1) if logits.shape[1] > 1 else np.full(logits.shape[0], np.inf)
    return arg, top, gap


def softmax_stats(logits, temperature=1.0):
    """What VerifyStochastic needs of the LLM's distribution at a node before any rejection (Algorithm 2:
    P(x | u) = softmax(logits[u] / T)[x]) without the whole row: per row (arg-max with the lowest token id on
    ties, the maximum m, Z = sum_x exp((logits[x] - m) / T)), so that P(x) = exp((logits[x] - m) / T) / Z.
    logits [..., V] (the values as stored, e.g. already rounded to bf16); float64."""
    x = np.asarray(logits, dtype=np.float64)
    m = x.max(axis=-1)
    z = np.exp((x - m[..., None]) / float(temperature)).sum(axis=-1)
    return x.argmax(axis=-1).astype(np.int32), m, z
