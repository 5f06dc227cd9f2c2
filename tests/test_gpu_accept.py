"""GPU parity of the steps that close a verification step: greedy acceptance along the draft tree,
commit of the accepted K/V rows into the target cache, chunk scores for the last accepted row.
Integer and byte work: exact against the oracle."""
import numpy as np
import pytest
import torch

import oracle as orc
from parity_util import check_scores, oracle_all
from workloads import chain_tree, config_tree, config_workload, eagle_style_tree, random_parent_tree, wide_tree

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hx():
    from paper_2505_20776_amd import harness
    return harness


def _tokens_following(parent, rng, vocab, follow):
    """Draft / target tokens: with probability `follow` the target's wish after a node is one of its children's
    tokens, so that long accepted paths occur."""
    T = len(parent)
    draft = rng.integers(0, vocab, size=T)
    target = rng.integers(0, vocab, size=T)
    for i in range(T):
        kids = [j for j in range(T) if parent[j] == i]
        if kids and rng.random() < follow:
            target[i] = draft[kids[int(rng.integers(len(kids)))]]
    roots = [j for j in range(T) if parent[j] < 0]
    first = int(draft[roots[int(rng.integers(len(roots)))]]) if rng.random() < follow else int(rng.integers(vocab))
    return draft, target, first


@pytest.mark.parametrize("seed", range(24))
def test_accept_exact(hx, seed):
    rng = np.random.default_rng(500 + seed)
    T = int(rng.choice([1, 2, 7, 16, 60, 64, 65, 100, 128]))
    kind = seed % 4
    parent = (chain_tree(T) if kind == 0 or T < 4 else random_parent_tree(T, 10, rng) if kind == 1
              else eagle_style_tree(T, 6, rng) if kind == 2 else wide_tree(T, 4, rng))
    parent = np.array(parent[:T])
    if seed % 6 == 5 and T > 3:
        parent[2] = -1                                       # a second root
    draft, target, first = _tokens_following(parent, rng, vocab=int(rng.integers(1, 6)), follow=0.85)
    print(f"[case] accept seed={seed} T={T} kind={kind}", flush=True)
    path, nxt, raw, _ = hx.run_accept(parent, draft, target, first)
    ref_path, ref_next = orc.accept_greedy(parent, draft, target, first)
    assert path == ref_path and nxt == ref_next
    assert (raw[len(path):] == -1).all()


def test_accept_whole_chain_and_nothing(hx):
    T = 128
    parent = chain_tree(T)
    draft = np.arange(T) % 7
    target = np.roll(draft, -1); target[-1] = 42
    path, nxt, _, _ = hx.run_accept(parent, draft, target, int(draft[0]))
    assert path == list(range(T)) and nxt == 42
    path, nxt, raw, _ = hx.run_accept(parent, draft, target, 99)
    assert path == [] and nxt == 99 and (raw == -1).all()


@pytest.mark.parametrize("n_accept", [0, 1, 5, 9])
def test_commit_exact(hx, n_accept):
    import paper_2505_20776_amd as sx
    rng = np.random.default_rng(7 + n_accept)
    layers, Hkv, T, d, L, cap = 3, 8, 60, 128, 1000, 1024
    dev = "cuda"
    bits = lambda *s: torch.from_numpy(rng.integers(0, 2**15, size=s).astype(np.int16)).to(dev).view(torch.bfloat16)
    kt, vt, kc, vc = bits(layers, Hkv, T, d), bits(layers, Hkv, T, d), bits(layers, Hkv, cap, d), bits(layers, Hkv, cap, d)
    path_h = np.full(T, -1, dtype=np.int32)
    path_h[:n_accept] = rng.choice(T, size=n_accept, replace=False)
    path = torch.from_numpy(path_h).to(dev)
    n_dev = torch.tensor([n_accept], dtype=torch.int32, device=dev)
    as_u16 = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
    refs = [orc.commit_tree_kv(as_u16(kc[y]), as_u16(vc[y]), as_u16(kt[y]), as_u16(vt[y]),
                               [int(x) for x in path_h[:n_accept]], L) for y in range(layers)]
    print(f"[case] commit n_accept={n_accept}", flush=True)
    sx.commit_tree_kv(kt, vt, kc, vc, path, n_dev, 16, T, layers, Hkv, d, 2, L, cap)
    torch.cuda.synchronize()
    for y, (ref_k, ref_v, new_len) in enumerate(refs):
        assert new_len == L + n_accept
        assert (as_u16(kc[y]) == ref_k).all() and (as_u16(vc[y]) == ref_v).all()


def test_commit_strided_cache(hx):
    """The cache as a slice of a larger allocation (stride_l > d, stride_h > capacity * stride_l)."""
    import paper_2505_20776_amd as sx
    rng = np.random.default_rng(11)
    Hkv, T, d, L, cap = 2, 12, 64, 30, 40
    dev = "cuda"
    big_k = torch.from_numpy(rng.integers(0, 2**15, size=(Hkv, cap + 3, 2 * d)).astype(np.int16)).to(dev)
    big_v = big_k.clone() + 1
    kt = torch.from_numpy(rng.integers(0, 2**15, size=(Hkv, T, d)).astype(np.int16)).to(dev)
    vt = kt.clone() + 3
    before_k, before_v = big_k.cpu().numpy().copy(), big_v.cpu().numpy().copy()
    path_h = np.array([3, 7, 11] + [-1] * 9, dtype=np.int32)
    sx.commit_tree_kv(kt, vt, big_k, big_v, torch.from_numpy(path_h).to(dev),
                      torch.tensor([3], dtype=torch.int32, device=dev), 4, T, 1, Hkv, d, 2, L, cap,
                      cache_stride_h=(cap + 3) * 2 * d, cache_stride_l=2 * d)
    torch.cuda.synchronize()
    exp_k, exp_v = before_k.copy(), before_v.copy()
    for i, node in enumerate([3, 7, 11]):
        exp_k[:, L + i, :d] = kt.cpu().numpy()[:, node]
        exp_v[:, L + i, :d] = vt.cpu().numpy()[:, node]
    assert (big_k.cpu().numpy() == exp_k).all() and (big_v.cpu().numpy() == exp_v).all()


def test_scores_for_last_accepted_row(hx):
    """verify -> accept -> chunk scores of the last accepted node, row index never leaving the device."""
    import paper_2505_20776_amd as sx
    wl = config_workload(2, sharp=True)
    ref_out, ref_lse, ref_scores = oracle_all(wl)
    T = wl.n_tree
    rng = np.random.default_rng(21)
    draft, target, first = _tokens_following(np.asarray(wl.parent), rng, vocab=5, follow=1.0)
    ref_path, _ = orc.accept_greedy(wl.parent, draft, target, first)
    assert len(ref_path) >= 2                                # the seed gives a real path
    dev = "cuda"
    q, kp, vp = hx.to_device(wl.q, wl.dtype, dev), hx.to_device(wl.k_prefix, wl.dtype, dev), hx.to_device(wl.v_prefix, wl.dtype, dev)
    kt, vt = hx.to_device(wl.k_tree, wl.dtype, dev), hx.to_device(wl.v_tree, wl.dtype, dev)
    parent = torch.from_numpy(np.asarray(wl.parent, dtype=np.int32)).to(dev)
    buf = hx.make_buffers(dtype=wl.dtype, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim,
                          prefix_len=wl.prefix_len, n_tree=T, chunk_size=wl.chunk_size, want_scores=True)
    sx.verify_attn(buf.desc, q, kp, vp, kt, vt, parent, buf.out, buf.lse, buf.workspace)
    path, nxt, raw, (path_dev, n_dev) = hx.run_accept(np.asarray(wl.parent), draft, target, first)
    assert path == ref_path
    C = ref_scores.shape[1]
    one = torch.empty(C, dtype=torch.float32, device=dev)
    sx.chunk_scores_accepted(buf.desc, buf.workspace, path_dev, n_dev, one)
    torch.cuda.synchronize()
    check_scores(one.cpu().numpy()[None], ref_scores[path[-1]][None], "scores of the last accepted row")
    # nothing accepted: row 0
    n_dev.zero_()
    sx.chunk_scores_accepted(buf.desc, buf.workspace, path_dev, n_dev, one)
    torch.cuda.synchronize()
    check_scores(one.cpu().numpy()[None], ref_scores[0][None], "scores with an empty path")
