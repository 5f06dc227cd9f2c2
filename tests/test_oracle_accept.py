"""Pins for the oracle's greedy tree acceptance and KV commit (CPU only).

The paper gives the loop for a linear draft (Alg. 1: Verify, Correct, bonus token
when everything is accepted); on a draft tree the same loop runs down one path.
Nothing here calls the HIP path.
"""
import numpy as np
import pytest

import oracle as orc
from workloads import chain_tree, eagle_style_tree, random_parent_tree, tree_depths, wide_tree


def alg1_sequential(draft, target_next, first_target):
    """Alg. 1 lines 'if Verify ... else Correct; break' and 'if all accepted: sample q_{K+1}' written out for a
    linear draft at temperature 0: target_next[i] is the arg-max of q_{i+2} (the position after draft i)."""
    accepted = []
    q_argmax = [first_target] + list(target_next)        # q_1 .. q_{K+1}
    for i, tok in enumerate(draft):
        if tok == q_argmax[i]:                            # Verify
            accepted.append(i)
        else:                                             # Correct, break
            return accepted, q_argmax[i]
    return accepted, q_argmax[len(draft)]                 # all K accepted: bonus token from q_{K+1}


@pytest.mark.parametrize("seed", range(8))
def test_chain_equals_alg1_loop(seed):
    rng = np.random.default_rng(seed)
    K = int(rng.integers(1, 12))
    draft = rng.integers(0, 3, size=K)
    target_next = rng.integers(0, 3, size=K)
    first = int(rng.integers(0, 3))
    # make long accepted prefixes likely
    n_ok = int(rng.integers(0, K + 1))
    q = [first] + list(target_next)
    for i in range(n_ok):
        draft[i] = q[i]
    path, nxt = orc.accept_greedy(chain_tree(K), draft, target_next, first)
    ref_path, ref_next = alg1_sequential(draft, target_next, first)
    assert path == ref_path and nxt == ref_next


def accepted_by_recursion(parent, draft, target_next, first_target):
    """Independent formulation: node i is accepted iff its parent is accepted (or i is a root), its token is the one
    the target wants after the parent, and no lower-indexed sibling has that token too."""
    T = len(parent)
    ok = np.zeros(T, dtype=bool)
    for i in range(T):                                    # parent[i] < i: one pass suffices
        par = parent[i]
        if par >= 0 and not ok[par]:
            continue
        want = first_target if par < 0 else target_next[par]
        if draft[i] != want:
            continue
        if any(parent[j] == par and draft[j] == want for j in range(i)):
            continue
        ok[i] = True
    return ok


@pytest.mark.parametrize("seed", range(40))
def test_random_trees_against_recursion(seed):
    rng = np.random.default_rng(100 + seed)
    T = int(rng.integers(1, 40))
    parent = random_parent_tree(T, 6, rng) if seed % 3 else wide_tree(T, 3, rng) if T > 3 else chain_tree(T)
    if seed % 5 == 0 and T > 2:                           # several roots
        parent = np.array(parent); parent[1] = -1
    vocab = int(rng.integers(1, 4))
    draft = rng.integers(0, vocab, size=T)
    target_next = rng.integers(0, vocab, size=T)
    first = int(rng.integers(0, vocab))
    path, nxt = orc.accept_greedy(parent, draft, target_next, first)
    ok = accepted_by_recursion(parent, draft, target_next, first)
    assert sorted(path) == list(np.flatnonzero(ok))
    # the path is a chain from a root downwards
    for a, b in zip([-1] + path[:-1], path):
        assert parent[b] == a
    depth = tree_depths(parent)
    assert [depth[i] for i in path] == list(range(len(path)))
    # tokens along the path are what the target wanted, and the walk is maximal
    wants = [first] + [int(target_next[i]) for i in path]
    assert [int(draft[i]) for i in path] == wants[:-1] and nxt == wants[-1]
    last = path[-1] if path else -1
    assert not any(parent[j] == last and draft[j] == nxt for j in range(T))


def test_nothing_and_everything():
    parent = eagle_style_tree(30, 6, np.random.default_rng(3))
    T = len(parent)
    draft = np.arange(T) + 10
    target_next = np.full(T, 5)
    assert orc.accept_greedy(parent, draft, target_next, 7) == ([], 7)          # no root carries token 7
    # follow the deepest node's ancestor chain
    depth = tree_depths(parent)
    leaf = int(np.argmax(depth))
    chain = []
    i = leaf
    while i >= 0:
        chain.append(i); i = int(parent[i])
    chain.reverse()
    target_next = np.full(T, -1)
    for a, b in zip(chain[:-1], chain[1:]):
        target_next[a] = draft[b]
    target_next[leaf] = 99
    path, nxt = orc.accept_greedy(parent, draft, target_next, int(draft[chain[0]]))
    assert path == chain and nxt == 99


def test_commit_copies_rows_verbatim():
    rng = np.random.default_rng(5)
    Hkv, cap, d, T, L = 3, 50, 8, 12, 37
    kc = rng.integers(0, 2**16, size=(Hkv, cap, d)).astype(np.uint16)
    vc = rng.integers(0, 2**16, size=(Hkv, cap, d)).astype(np.uint16)
    kt = rng.integers(0, 2**16, size=(Hkv, T, d)).astype(np.uint16)
    vt = rng.integers(0, 2**16, size=(Hkv, T, d)).astype(np.uint16)
    path = [0, 2, 5, 11]
    kn, vn, newL = orc.commit_tree_kv(kc, vc, kt, vt, path, L)
    assert newL == L + 4 and kn.dtype == kc.dtype
    for i, node in enumerate(path):
        assert (kn[:, L + i] == kt[:, node]).all() and (vn[:, L + i] == vt[:, node]).all()
    untouched = np.ones(cap, dtype=bool); untouched[L:L + 4] = False
    assert (kn[:, untouched] == kc[:, untouched]).all() and (vn[:, untouched] == vc[:, untouched]).all()
    assert (kc[:, L] != kn[:, L]).any()                   # the input was not modified in place
    k0, v0, l0 = orc.commit_tree_kv(kc, vc, kt, vt, [], L)
    assert l0 == L and (k0 == kc).all() and (v0 == vc).all()
