"""CPU oracle for SpecExtend's verification-side hot path.  TEST INFRASTRUCTURE.

Plain, slow, fp64 numpy.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this file; the product path never does, and this
file imports nothing from the product.  It shares no code, table or helper
with the HIP kernels.

What the paper fixes (SpecExtend, arXiv 2505.20776):
  * Sec. 3.1: during verification the draft-tree tokens are the queries; they
    attend to the target model's cached prefix and, under the tree-structured
    mask of tree attention, to tree tokens.  Hybrid Tree Attention is the
    FlashDecoding-compatible way of computing exactly that, so the oracle for
    it is the plain definition: ONE softmax per (head, tree row) over
    prefix keys + ancestor-or-self tree keys  -> `verify_attention`.
  * Sec. 3.2.1: the prefix is cut into fixed-size chunks which are ranked by
    their average attention score for one query token, the top-k chunks are
    kept (Alg. 1 SelectChunks) and only those stay in the draft model's KV
    cache (Alg. 1 UpdateDraftCache)  -> `chunk_scores`, `select_chunks`,
    `gather_draft_kv`.

Readings where the paper is silent (each listed in the design notes):
  scale 1/sqrt(d); query head h uses KV head h // G; "scores" are post-softmax
  probabilities normalised over the whole row (prefix + visible tree keys);
  "average" = mean over the tokens actually in the chunk and over all query
  heads; a ragged last chunk averages over its real length; ties go to the
  lower chunk index; kept chunks are listed in ascending position; the gather
  copies bytes verbatim and reports original positions.

Pins (tests/test_oracle_*.py): hybrid == single softmax; chain tree == causal
attention (own routine and torch SDPA); one-node tree == single-token decode;
row sums; closed forms for Q = 0 and for a one-hot row; key-shift invariance;
chunk / tree permutation laws; GQA duplication; top-k versus brute-force
subset search; gather round trips; literal-loop brute force on tiny inputs.
The paper prints no worked numeric example for any of these quantities, so
beyond those pins the numeric values are "parity unpinned by the paper".

Closing the step (what follows the attention in Alg. 1): `accept_greedy` is the
Verify / Correct loop of Alg. 1 at temperature 0 - a drafted token is accepted
exactly when it equals the target model's arg-max token for its position, the
first mismatch is replaced by that arg-max token, and when every drafted token
on the path is accepted the target's next arg-max token is appended - walked
down the draft tree (tree attention, Sec. 2: the children of a node are
alternative drafts for the position after it).  Readings: among several children
with the accepted token the lowest node index wins; roots (parent -1) are the
drafts for the first new position.  `commit_tree_kv` appends the accepted
nodes' K/V rows to the target cache behind the prefix, byte for byte.  Pins:
the chain tree against the literal sequential loop of Alg. 1, a recursive
reformulation on random trees, maximality and chain invariants.

The score path the paper itself describes (Sec. 3.2.1: the last layer is computed as
standard attention and the attention scores are read from it) needs the whole
probability matrix: `attention_probabilities` writes every row of it out with a
literal loop over rows.  Pins: rows sum to one, hidden tree keys are exactly zero,
p @ V reproduces `verify_attention`, chunk sums reproduce its chunk mass, uniform
rows for Q = 0.

Prefill (Sec. 3.1: FlashAttention is applied to the prefill of target and draft model; it
computes exact attention without writing the score matrix, so its oracle is the plain
definition of causal self-attention): `prefill_attention`, one row at a time.  Pins: torch's
scaled_dot_product_attention with a causal mask, `causal_attention_tail`, the chain-tree case
of `verify_attention`, the running-mean closed form for Q = 0, independence of later keys.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "ancestor_mask", "verify_attention", "chunk_scores", "hybrid_attention",
    "select_chunks", "gather_draft_kv", "causal_attention_tail", "accept_greedy", "commit_tree_kv",
    "attention_probabilities", "prefill_attention",
]


def ancestor_mask(parent) -> np.ndarray:
    """vis[i, j] = True iff tree node j is node i itself or one of its ancestors.

    `parent[i] < i`, and -1 marks a root (Sec. 2 tree attention / Sec. 3.1: a
    tree token may only see the tokens on its own root-to-node path).
    """
    parent = np.asarray(parent, dtype=np.int64)
    n = len(parent)
    vis = np.zeros((n, n), dtype=bool)
    for i in range(n):
        p = int(parent[i])
        if p >= i or p < -1:
            raise ValueError(f"parent[{i}]={p} is not a topological parent index")
        if p >= 0:
            vis[i, :] = vis[p, :]
        vis[i, i] = True
    return vis


def _as64(x):
    return np.asarray(x, dtype=np.float64)


def verify_attention(q, k_prefix, v_prefix, k_tree, v_tree, parent, *, scale=None,
                     chunk_size=None):
    """Full masked attention of the tree tokens in a single softmax (Sec. 3.1).

    q [T,Hq,d]; k_prefix,v_prefix [Hkv,L,d]; k_tree,v_tree [Hkv,T,d]; parent [T].
    Returns (out [T,Hq,d], lse [Hq,T], chunk_mass) where chunk_mass [Hq,T,C] is
    the softmax probability that falls into each prefix chunk (None when
    chunk_size is None).  Everything in fp64.
    """
    q, k_prefix, v_prefix, k_tree, v_tree = map(_as64, (q, k_prefix, v_prefix, k_tree, v_tree))
    n_tree, n_q_heads, d = q.shape
    n_kv_heads, plen, _ = k_prefix.shape
    assert n_q_heads % n_kv_heads == 0
    group = n_q_heads // n_kv_heads
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    vis = ancestor_mask(parent)
    out = np.zeros((n_tree, n_q_heads, d))
    lse = np.zeros((n_q_heads, n_tree))
    n_chunks = None
    mass = None
    if chunk_size is not None:
        n_chunks = (plen + chunk_size - 1) // chunk_size
        mass = np.zeros((n_q_heads, n_tree, n_chunks))
    for h in range(n_q_heads):
        g = h // group
        keys = np.concatenate([k_prefix[g], k_tree[g]], axis=0)          # [L+T, d]
        vals = np.concatenate([v_prefix[g], v_tree[g]], axis=0)
        s = scale * (q[:, h, :] @ keys.T)                                  # [T, L+T]
        allowed = np.concatenate([np.ones((n_tree, plen), dtype=bool), vis], axis=1)
        s = np.where(allowed, s, -np.inf)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        z = e.sum(axis=1, keepdims=True)
        p = e / z
        out[:, h, :] = p @ vals
        lse[h, :] = (m + np.log(z))[:, 0]
        if mass is not None:
            for c in range(n_chunks):
                lo, hi = c * chunk_size, min((c + 1) * chunk_size, plen)
                mass[h, :, c] = p[:, lo:hi].sum(axis=1)
    return out, lse, mass


def attention_probabilities(q, k_prefix, k_tree, parent, *, scale=None):
    """The materialised attention scores of standard attention (Sec. 3.2.1): p [Hq, T, L+T],
    row (h, i) = softmax over the prefix keys and the tree keys node i may see, exactly 0
    for the hidden tree keys.  Columns 0..L-1 are the prefix, L..L+T-1 the tree nodes."""
    q, k_prefix, k_tree = map(_as64, (q, k_prefix, k_tree))
    n_tree, n_q_heads, d = q.shape
    n_kv_heads, plen, _ = k_prefix.shape
    group = n_q_heads // n_kv_heads
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    parent = np.asarray(parent, dtype=np.int64)
    p = np.zeros((n_q_heads, n_tree, plen + n_tree))
    for h in range(n_q_heads):
        g = h // group
        for i in range(n_tree):
            cols = list(range(plen))
            node = i
            while node >= 0:                      # the node itself, then up to its root
                cols.append(plen + node)
                node = int(parent[node])
            cols = np.asarray(sorted(cols))
            keys = np.concatenate([k_prefix[g], k_tree[g]], axis=0)[cols]
            logits = scale * (keys @ q[i, h])
            w = np.exp(logits - logits.max())
            p[h, i, cols] = w / w.sum()
    return p


def chunk_scores(q, k_prefix, v_prefix, k_tree, v_tree, parent, chunk_size, *, scale=None):
    """Per-chunk average attention score for every tree row (Sec. 3.2.1).

    score[i, c] = mean over query heads of ( mean over the tokens of chunk c of
    p[h, i, token] ), p being the full-row softmax of `verify_attention`.
    Returns [T, C] fp64.
    """
    plen = np.asarray(k_prefix).shape[1]
    _, _, mass = verify_attention(q, k_prefix, v_prefix, k_tree, v_tree, parent,
                                  scale=scale, chunk_size=chunk_size)
    n_chunks = mass.shape[2]
    sizes = np.array([min((c + 1) * chunk_size, plen) - c * chunk_size for c in range(n_chunks)],
                     dtype=np.float64)
    return (mass / sizes[None, None, :]).mean(axis=0)


def _softmax_part(qh, keys, vals, scale, allowed=None):
    """Softmax attention over one key subset: (o [T,d], lse [T]); rows that see
    no key get lse = -inf and o = 0."""
    s = scale * (qh @ keys.T)
    if allowed is not None:
        s = np.where(allowed, s, -np.inf)
    m = s.max(axis=1, keepdims=True) if s.shape[1] else np.full((s.shape[0], 1), -np.inf)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    e = np.exp(s - m_safe)
    z = e.sum(axis=1, keepdims=True)
    with np.errstate(divide="ignore", invalid="ignore"):
        o = np.where(z > 0, (e @ vals) / np.where(z > 0, z, 1.0), 0.0)
        lse = np.where(z[:, 0] > 0, m_safe[:, 0] + np.log(np.where(z[:, 0] > 0, z[:, 0], 1.0)), -np.inf)
    return o, lse


def prefill_attention(q, k_all, v_all, *, scale=None, rows=None):
    """Causal self-attention of the prefill stage (Sec. 3.1), by its definition.

    q [Tq,Hq,d] are the queries of the last Tq positions of a context of N keys
    (Tq = N for a whole prompt, Tq < N for a later piece of a prompt processed in
    pieces); k_all, v_all [Hkv,N,d].  Query i sits at position N - Tq + i and sees keys
    0..that position.  `rows` restricts the computation to some query indices (the
    others come back as zeros / -inf).  Returns (out [Tq,Hq,d], lse [Hq,Tq]).
    """
    q, k_all, v_all = map(_as64, (q, k_all, v_all))
    n_q, n_q_heads, d = q.shape
    n_kv_heads, n_all, _ = k_all.shape
    if n_q > n_all:
        raise ValueError("more queries than keys")
    group = n_q_heads // n_kv_heads
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.zeros((n_q, n_q_heads, d))
    lse = np.full((n_q_heads, n_q), -np.inf)
    for i in (range(n_q) if rows is None else rows):
        n_seen = n_all - n_q + int(i) + 1
        for h in range(n_q_heads):
            g = h // group
            logits = scale * (k_all[g, :n_seen] @ q[i, h])
            top = logits.max()
            w = np.exp(logits - top)
            z = w.sum()
            out[i, h] = (w @ v_all[g, :n_seen]) / z
            lse[h, i] = top + np.log(z)
    return out, lse


def hybrid_attention(q, k_prefix, v_prefix, k_tree, v_tree, parent, *, split_points=(), scale=None):
    """The hybrid form: independent softmaxes over prefix segments and over the
    tree keys, recombined by log-sum-exp weights.  `split_points` are the
    interior cut positions of the prefix (any positions, they need not respect
    chunk boundaries).  Mathematically identical to `verify_attention`; kept
    as a separately written routine so the identity can be tested.
    Returns (out [T,Hq,d], lse [Hq,T]).
    """
    q, k_prefix, v_prefix, k_tree, v_tree = map(_as64, (q, k_prefix, v_prefix, k_tree, v_tree))
    n_tree, n_q_heads, d = q.shape
    n_kv_heads, plen, _ = k_prefix.shape
    group = n_q_heads // n_kv_heads
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    vis = ancestor_mask(parent)
    cuts = [0] + sorted(int(c) for c in split_points) + [plen]
    out = np.zeros((n_tree, n_q_heads, d))
    lse = np.zeros((n_q_heads, n_tree))
    for h in range(n_q_heads):
        g = h // group
        parts = []
        for lo, hi in zip(cuts[:-1], cuts[1:]):
            parts.append(_softmax_part(q[:, h, :], k_prefix[g, lo:hi], v_prefix[g, lo:hi], scale))
        parts.append(_softmax_part(q[:, h, :], k_tree[g], v_tree[g], scale, allowed=vis))
        lses = np.stack([p[1] for p in parts], axis=0)                   # [parts, T]
        top = lses.max(axis=0)
        total = top + np.log(np.exp(lses - top[None, :]).sum(axis=0))
        acc = np.zeros((n_tree, d))
        for o, l in parts:
            acc += np.exp(l - total)[:, None] * o
        out[:, h, :] = acc
        lse[h, :] = total
    return out, lse


def causal_attention_tail(q_tail, k_all, v_all, *, scale=None):
    """Causal self-attention outputs of the LAST T positions of a sequence.

    q_tail [T,Hq,d] are the queries of positions N-T..N-1; k_all, v_all
    [Hkv,N,d].  Position n sees keys 0..n.  Written row by row, on purpose not
    sharing the masking code above (used to pin the chain-tree special case).
    Returns out [T,Hq,d].
    """
    q_tail, k_all, v_all = map(_as64, (q_tail, k_all, v_all))
    n_tail, n_q_heads, d = q_tail.shape
    n_kv_heads, n_all, _ = k_all.shape
    group = n_q_heads // n_kv_heads
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.zeros((n_tail, n_q_heads, d))
    for t in range(n_tail):
        last = n_all - n_tail + t            # index of the newest visible key
        for h in range(n_q_heads):
            g = h // group
            logits = scale * (k_all[g, :last + 1] @ q_tail[t, h])
            w = np.exp(logits - logits.max())
            out[t, h] = (w / w.sum()) @ v_all[g, :last + 1]
    return out


def select_chunks(scores_row, k):
    """Alg. 1 SelectChunks: the min(k, C) chunks with the largest score, ties
    to the lower index, returned in ascending chunk order (int32)."""
    s = _as64(scores_row).ravel()
    if not np.all(np.isfinite(s)):
        raise ValueError("scores must be finite")
    if k < 0:
        raise ValueError("k must be non-negative")
    order = sorted(range(len(s)), key=lambda c: (-s[c], c))
    keep = order[:min(int(k), len(s))]
    return np.asarray(sorted(keep), dtype=np.int32)


def gather_draft_kv(k_src, v_src, idx, chunk_size):
    """Alg. 1 UpdateDraftCache: keep only the chunks in `idx` (in that order).

    k_src, v_src [Ld,H,L,d] of any dtype; values are copied verbatim.  Returns
    (k_dst, v_dst [Ld,H,n_tok,d], pos int32 [n_tok]) where pos holds each kept
    token's original position; a ragged last chunk contributes only its real
    tokens.
    """
    k_src = np.asarray(k_src)
    v_src = np.asarray(v_src)
    plen = k_src.shape[2]
    n_chunks = (plen + chunk_size - 1) // chunk_size
    pos = []
    for c in np.asarray(idx, dtype=np.int64).ravel():
        if c < 0 or c >= n_chunks:
            raise ValueError(f"chunk index {c} out of range")
        pos.extend(range(int(c) * chunk_size, min((int(c) + 1) * chunk_size, plen)))
    pos = np.asarray(pos, dtype=np.int64)
    k_dst = np.ascontiguousarray(k_src[:, :, pos, :])
    v_dst = np.ascontiguousarray(v_src[:, :, pos, :])
    return k_dst, v_dst, pos.astype(np.int32)


def accept_greedy(parent, draft_token, target_token, first_target):
    """Alg. 1 Verify / Correct at temperature 0 along the draft tree.

    parent[i] < i (-1 = root): tree shape.  draft_token[i]: the token drafted at
    node i.  target_token[i]: the target model's arg-max token for the position
    after node i.  first_target: its arg-max token for the first new position.
    Returns (path, next_token): the accepted nodes from the top down, and the
    token that follows them (the correction of the first mismatch, or the bonus
    token when a leaf was reached).
    """
    parent = np.asarray(parent)
    draft_token = np.asarray(draft_token)
    target_token = np.asarray(target_token)
    path = []
    cur, want = -1, int(first_target)
    while True:
        matches = [i for i in range(len(parent)) if parent[i] == cur and draft_token[i] == want]
        if not matches:
            return path, want
        cur = min(matches)
        path.append(cur)
        want = int(target_token[cur])


def commit_tree_kv(k_cache, v_cache, k_tree, v_tree, path, prefix_len):
    """Accepted tree tokens enter the target cache: cache[:, prefix_len + i, :] = tree[:, path[i], :].

    k_cache / v_cache [Hkv, capacity, d], k_tree / v_tree [Hkv, T, d]; returns the
    updated copies and the new prefix length.  Verbatim copies (any dtype).
    """
    k_new = np.array(k_cache, copy=True)
    v_new = np.array(v_cache, copy=True)
    for i, node in enumerate(path):
        k_new[:, prefix_len + i, :] = k_tree[:, node, :]
        v_new[:, prefix_len + i, :] = v_tree[:, node, :]
    return k_new, v_new, prefix_len + len(path)
