"""Pins for the fp64 oracle: invariants, closed forms, special cases that reduce
to textbook / library routines, and literal-loop brute force on tiny inputs.

The paper (SpecExtend, arXiv 2505.20776) prints no worked numeric example for
attention outputs, chunk scores or selections, so each pin below is something
its definitions (Sec. 3.1, Sec. 3.2.1, Alg. 1) and the mathematics fix.  Each
is chosen so that a plausible slip in the oracle (dropped term, wrong sign or
index, transposed operand, wrong normaliser) breaks at least one of them.
"""
import itertools
import math

import numpy as np
import pytest
import torch

import oracle as orc
from workloads import (chain_tree, config_workload, eagle_style_tree, random_parent_tree,
                       tree_depths, wide_tree)


def _rand_case(seed, T=7, Hq=4, Hkv=2, d=8, L=37, std=1.0, max_depth=3):
    rng = np.random.default_rng(seed)
    parent = random_parent_tree(T, max_depth, rng)
    mk = lambda *s: rng.standard_normal(s) * std
    return dict(q=mk(T, Hq, d), k_prefix=mk(Hkv, L, d), v_prefix=mk(Hkv, L, d),
                k_tree=mk(Hkv, T, d), v_tree=mk(Hkv, T, d), parent=parent)


# ---------------------------------------------------------------------------
# I13: literal nested loops on tiny inputs (a third, independent routine)
# ---------------------------------------------------------------------------

def _brute(q, kp, vp, kt, vt, parent, chunk):
    T, Hq, d = len(q), len(q[0]), len(q[0][0])
    Hkv, L = len(kp), len(kp[0])
    G = Hq // Hkv
    C = (L + chunk - 1) // chunk
    out = [[[0.0] * d for _ in range(Hq)] for _ in range(T)]
    lse = [[0.0] * T for _ in range(Hq)]
    score = [[0.0] * C for _ in range(T)]
    for i in range(T):
        path = []
        n = i
        while n != -1:
            path.append(n)
            n = parent[n]
        for h in range(Hq):
            g = h // G
            logits, values, where = [], [], []
            for j in range(L):
                logits.append(sum(q[i][h][x] * kp[g][j][x] for x in range(d)) / math.sqrt(d))
                values.append(vp[g][j])
                where.append(j)
            for j in sorted(path):
                logits.append(sum(q[i][h][x] * kt[g][j][x] for x in range(d)) / math.sqrt(d))
                values.append(vt[g][j])
                where.append(None)
            z = sum(math.exp(s) for s in logits)
            lse[h][i] = math.log(z)
            for s, v, w in zip(logits, values, where):
                p = math.exp(s) / z
                for x in range(d):
                    out[i][h][x] += p * v[x]
                if w is not None:
                    c = w // chunk
                    size = min((c + 1) * chunk, L) - c * chunk
                    score[i][c] += p / size / Hq
    return np.array(out), np.array(lse), np.array(score)


@pytest.mark.parametrize("L,T,d,chunk,Hq,Hkv", [(3, 2, 2, 2, 1, 1), (5, 3, 2, 2, 2, 1), (5, 4, 3, 2, 4, 2)])
def test_brute_force_tiny(L, T, d, chunk, Hq, Hkv):
    rng = np.random.default_rng(100 + L + T)
    parent = [-1] + [int(rng.integers(0, i)) for i in range(1, T)]
    mk = lambda *s: rng.standard_normal(s)
    q, kp, vp, kt, vt = mk(T, Hq, d), mk(Hkv, L, d), mk(Hkv, L, d), mk(Hkv, T, d), mk(Hkv, T, d)
    bo, bl, bs = _brute(q.tolist(), kp.tolist(), vp.tolist(), kt.tolist(), vt.tolist(), parent, chunk)
    out, lse, _ = orc.verify_attention(q, kp, vp, kt, vt, parent)
    sc = orc.chunk_scores(q, kp, vp, kt, vt, parent, chunk)
    np.testing.assert_allclose(out, bo, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, bl, rtol=0, atol=1e-13)
    np.testing.assert_allclose(sc, bs, rtol=0, atol=1e-14)


def test_hand_computed_two_keys():
    """One prefix key + root, d=1: the softmax is a logistic function."""
    q = np.array([[[2.0]]])
    kp = np.array([[[1.0]]]); vp = np.array([[[10.0]]])
    kt = np.array([[[-1.0]]]); vt = np.array([[[-10.0]]])
    out, lse, mass = orc.verify_attention(q, kp, vp, kt, vt, [-1], chunk_size=4)
    p0 = 1.0 / (1.0 + math.exp(-4.0))            # logits +2 and -2, scale 1
    assert abs(out[0, 0, 0] - (10 * p0 - 10 * (1 - p0))) < 1e-13
    assert abs(lse[0, 0] - math.log(math.exp(2) + math.exp(-2))) < 1e-13
    assert abs(mass[0, 0, 0] - p0) < 1e-14


# ---------------------------------------------------------------------------
# I1: hybrid (split softmaxes + log-sum-exp merge) == one softmax
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("seed,splits", [(1, ()), (2, (16,)), (3, (5, 6, 30)), (4, (1, 2, 3, 36))])
def test_hybrid_equals_full(seed, splits):
    c = _rand_case(seed, std=2.0)
    out, lse, _ = orc.verify_attention(**c)
    ho, hl = orc.hybrid_attention(**c, split_points=splits)
    np.testing.assert_allclose(ho, out, rtol=0, atol=1e-12)
    np.testing.assert_allclose(hl, lse, rtol=0, atol=1e-12)


# ---------------------------------------------------------------------------
# I2: a chain-shaped tree is causal attention of the last T positions
# ---------------------------------------------------------------------------

def test_chain_equals_causal_own_routine_and_sdpa():
    T, L, Hq, Hkv, d = 6, 29, 4, 2, 16
    c = _rand_case(7, T=T, Hq=Hq, Hkv=Hkv, d=d, L=L)
    c["parent"] = chain_tree(T)
    out, _, _ = orc.verify_attention(**c)
    k_all = np.concatenate([c["k_prefix"], c["k_tree"]], axis=1)
    v_all = np.concatenate([c["v_prefix"], c["v_tree"]], axis=1)
    own = orc.causal_attention_tail(c["q"], k_all, v_all)
    np.testing.assert_allclose(out, own, rtol=0, atol=1e-12)
    # library routine: full causal SDPA over L+T positions with arbitrary head queries, take the tail
    G = Hq // Hkv
    q_full = np.zeros((Hq, L + T, d)); q_full[:, L:, :] = np.transpose(c["q"], (1, 0, 2))
    kk = np.repeat(k_all, G, axis=0); vv = np.repeat(v_all, G, axis=0)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q_full), torch.from_numpy(kk), torch.from_numpy(vv), is_causal=True).numpy()
    np.testing.assert_allclose(out, np.transpose(ref[:, L:, :], (1, 0, 2)), rtol=0, atol=1e-12)


# ---------------------------------------------------------------------------
# I3: a one-node tree is single-token decode over L+1 keys
# ---------------------------------------------------------------------------

def test_single_node_is_decode():
    c = _rand_case(9, T=1, L=21)
    out, lse, _ = orc.verify_attention(**c)
    Hq, Hkv = c["q"].shape[1], c["k_prefix"].shape[0]
    for h in range(Hq):
        g = h // (Hq // Hkv)
        keys = np.vstack([c["k_prefix"][g], c["k_tree"][g]])
        vals = np.vstack([c["v_prefix"][g], c["v_tree"][g]])
        logits = keys @ c["q"][0, h] / math.sqrt(keys.shape[1])
        w = np.exp(logits); w /= w.sum()
        np.testing.assert_allclose(out[0, h], w @ vals, atol=1e-13)
        assert abs(lse[h, 0] - math.log(np.exp(logits).sum())) < 1e-12


# ---------------------------------------------------------------------------
# I4: probability bookkeeping (normaliser and ragged chunk)
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("L,chunk", [(37, 8), (40, 8), (5, 2), (7, 16)])
def test_mass_sums_to_one(L, chunk):
    c = _rand_case(11 + L, L=L, std=1.5)
    _, lse, mass = orc.verify_attention(**c, chunk_size=chunk)
    sc = orc.chunk_scores(**c, chunk_size=chunk)
    vis = orc.ancestor_mask(c["parent"])
    Hq, Hkv, d = c["q"].shape[1], c["k_prefix"].shape[0], c["q"].shape[2]
    G = Hq // Hkv
    C = mass.shape[2]
    sizes = np.array([min((j + 1) * chunk, L) - j * chunk for j in range(C)])
    assert sizes.sum() == L
    tree_mass = np.zeros((Hq, len(c["parent"])))
    for h in range(Hq):
        s = c["q"][:, h, :] @ c["k_tree"][h // G].T / math.sqrt(d)
        tree_mass[h] = (np.exp(s - lse[h][:, None]) * vis).sum(axis=1)
    np.testing.assert_allclose(mass.sum(axis=2) + tree_mass, 1.0, atol=1e-12)
    # head-averaged, size-weighted scores add up to the mean prefix mass
    np.testing.assert_allclose((sc * sizes[None, :]).sum(axis=1), mass.sum(axis=2).mean(axis=0), atol=1e-12)


# ---------------------------------------------------------------------------
# I5: closed form when all logits are equal
# ---------------------------------------------------------------------------

def test_zero_query_closed_form():
    L, chunk = 45, 8
    c = _rand_case(13, L=L)
    c["q"] = np.zeros_like(c["q"])
    out, lse, _ = orc.verify_attention(**c)
    sc = orc.chunk_scores(**c, chunk_size=chunk)
    depth = tree_depths(c["parent"])
    vis = orc.ancestor_mask(c["parent"])
    Hq, Hkv = c["q"].shape[1], c["k_prefix"].shape[0]
    for i in range(len(c["parent"])):
        n = L + depth[i] + 1
        np.testing.assert_allclose(sc[i], 1.0 / n, atol=1e-15)
        np.testing.assert_allclose(lse[:, i], math.log(n), atol=1e-13)
        for h in range(Hq):
            g = h // (Hq // Hkv)
            mean_v = (c["v_prefix"][g].sum(0) + c["v_tree"][g][vis[i]].sum(0)) / n
            np.testing.assert_allclose(out[i, h], mean_v, atol=1e-13)


# ---------------------------------------------------------------------------
# I6: adding one vector to every key changes nothing
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("mag", [0.5, 30.0])
def test_key_shift_invariance(mag):
    c = _rand_case(17)
    out, lse, _ = orc.verify_attention(**c)
    sc = orc.chunk_scores(**c, chunk_size=8)
    delta = np.random.default_rng(5).standard_normal(c["q"].shape[2]) * mag
    c2 = dict(c, k_prefix=c["k_prefix"] + delta, k_tree=c["k_tree"] + delta)
    out2, _, _ = orc.verify_attention(**c2)
    sc2 = orc.chunk_scores(**c2, chunk_size=8)
    np.testing.assert_allclose(out2, out, atol=1e-9)
    np.testing.assert_allclose(sc2, sc, atol=1e-11)
    ho, _ = orc.hybrid_attention(**c2, split_points=(9, 20))
    np.testing.assert_allclose(ho, out, atol=1e-9)


# ---------------------------------------------------------------------------
# I7: one dominant key
# ---------------------------------------------------------------------------

def test_one_hot_limit():
    L, chunk, hot = 40, 8, 19
    c = _rand_case(19, L=L, Hq=2, Hkv=1, std=0.1)
    d = c["q"].shape[2]
    qdir = c["q"].mean(axis=(0, 1)); qdir /= np.linalg.norm(qdir)
    c["q"] = c["q"] * 0 + qdir                        # all queries identical
    c["k_prefix"][0, hot] = qdir * 60.0 * math.sqrt(d)  # logit 60 above the rest (~0)
    out, _, _ = orc.verify_attention(**c)
    sc = orc.chunk_scores(**c, chunk_size=chunk)
    np.testing.assert_allclose(out, np.broadcast_to(c["v_prefix"][0, hot], out.shape), atol=1e-12)
    expect = np.zeros(L // chunk); expect[hot // chunk] = 1.0 / chunk
    np.testing.assert_allclose(sc, np.broadcast_to(expect, sc.shape), atol=1e-12)


# ---------------------------------------------------------------------------
# I8 / I9: permutation laws
# ---------------------------------------------------------------------------

def test_chunk_permutations():
    L, chunk = 48, 8
    c = _rand_case(23, L=L)
    out, _, _ = orc.verify_attention(**c)
    sc = orc.chunk_scores(**c, chunk_size=chunk)
    rng = np.random.default_rng(3)
    inner = np.concatenate([j * chunk + rng.permutation(chunk) for j in range(L // chunk)])
    c2 = dict(c, k_prefix=c["k_prefix"][:, inner], v_prefix=c["v_prefix"][:, inner])
    np.testing.assert_allclose(orc.verify_attention(**c2)[0], out, atol=1e-12)
    np.testing.assert_allclose(orc.chunk_scores(**c2, chunk_size=chunk), sc, atol=1e-13)
    cp = rng.permutation(L // chunk)
    outer = np.concatenate([np.arange(j * chunk, (j + 1) * chunk) for j in cp])
    c3 = dict(c, k_prefix=c["k_prefix"][:, outer], v_prefix=c["v_prefix"][:, outer])
    np.testing.assert_allclose(orc.verify_attention(**c3)[0], out, atol=1e-12)
    np.testing.assert_allclose(orc.chunk_scores(**c3, chunk_size=chunk), sc[:, cp], atol=1e-13)


def test_tree_relabelling_and_constant_v():
    c = _rand_case(29, T=6)
    parent = np.array([-1, 0, 0, 1, 2, 1], dtype=np.int32)
    c["parent"] = parent
    out, lse, _ = orc.verify_attention(**c)
    # swap the two children of the root (nodes 1 <-> 2) and relabel consistently
    perm = np.array([0, 2, 1, 4, 3, 5])       # new index -> old index; old 3,5 hang off old 1; old 4 off old 2
    old_to_new = np.argsort(perm)
    new_parent = np.array([-1 if parent[o] < 0 else old_to_new[parent[o]] for o in perm], dtype=np.int32)
    assert all(new_parent[i] < i for i in range(6))
    c2 = dict(c, q=c["q"][perm], k_tree=c["k_tree"][:, perm], v_tree=c["v_tree"][:, perm], parent=new_parent)
    out2, lse2, _ = orc.verify_attention(**c2)
    np.testing.assert_allclose(out2, out[perm], atol=1e-12)
    np.testing.assert_allclose(lse2, lse[:, perm], atol=1e-12)
    const = np.random.default_rng(1).standard_normal(c["q"].shape[2])
    c3 = dict(c, v_prefix=np.broadcast_to(const, c["v_prefix"].shape), v_tree=np.broadcast_to(const, c["v_tree"].shape))
    np.testing.assert_allclose(orc.verify_attention(**c3)[0], np.broadcast_to(const, out.shape), atol=1e-12)


def test_mask_is_ancestor_or_self():
    parent = [-1, 0, 0, 1, 3, -1, 5]
    vis = orc.ancestor_mask(parent)
    expect = np.zeros((7, 7), dtype=bool)
    for i, anc in enumerate([[0], [0, 1], [0, 2], [0, 1, 3], [0, 1, 3, 4], [5], [5, 6]]):
        expect[i, anc] = True
    assert (vis == expect).all()
    with pytest.raises(ValueError):
        orc.ancestor_mask([-1, 1])
    # a sibling's value must not leak: make sibling V huge and check it has no effect
    c = _rand_case(31, T=3); c["parent"] = np.array([-1, 0, 0], dtype=np.int32)
    base = orc.verify_attention(**c)[0]
    c["v_tree"][:, 2] += 1e6
    after = orc.verify_attention(**c)[0]
    np.testing.assert_array_equal(after[:2], base[:2])
    assert np.abs(after[2] - base[2]).max() > 1.0


# ---------------------------------------------------------------------------
# I10: grouped-query mapping
# ---------------------------------------------------------------------------

def test_gqa_duplication():
    c = _rand_case(37, Hq=6, Hkv=2)
    G = 3
    out, lse, _ = orc.verify_attention(**c)
    sc = orc.chunk_scores(**c, chunk_size=8)
    dup = dict(c, **{n: np.repeat(c[n], G, axis=0) for n in ("k_prefix", "v_prefix", "k_tree", "v_tree")})
    out2, lse2, _ = orc.verify_attention(**dup)
    np.testing.assert_allclose(out2, out, atol=1e-14)
    np.testing.assert_allclose(lse2, lse, atol=1e-14)
    np.testing.assert_allclose(orc.chunk_scores(**dup, chunk_size=8), sc, atol=1e-15)
    # and the mapping is h // G, not h % G: head 1 must use KV head 0
    c2 = dict(c); c2["k_prefix"] = c["k_prefix"].copy(); c2["k_prefix"][1] += 5.0
    out3 = orc.verify_attention(**c2)[0]
    np.testing.assert_array_equal(out3[:, :G], out[:, :G])
    assert np.abs(out3[:, G:] - out[:, G:]).max() > 1e-3


def test_scale_default_and_override():
    c = _rand_case(41)
    d = c["q"].shape[2]
    a = orc.verify_attention(**c)[0]
    b = orc.verify_attention(**c, scale=1.0 / math.sqrt(d))[0]
    np.testing.assert_array_equal(a, b)
    c2 = dict(c, q=c["q"] * 2.0)
    np.testing.assert_allclose(orc.verify_attention(**c2, scale=0.5 / math.sqrt(d))[0], a, atol=1e-13)


# ---------------------------------------------------------------------------
# I11: top-k selection
# ---------------------------------------------------------------------------

def test_select_matches_subset_brute_force():
    rng = np.random.default_rng(43)
    for trial in range(20):
        C = int(rng.integers(2, 10)); k = int(rng.integers(1, C + 1))
        s = rng.random(C)
        best = max(itertools.combinations(range(C), k), key=lambda idx: sum(s[i] for i in idx))
        got = orc.select_chunks(s, k)
        assert got.dtype == np.int32
        assert list(got) == sorted(best)


def test_select_edge_cases():
    s = np.array([0.5, 0.9, 0.5, 0.1, 0.9, 0.5])
    assert list(orc.select_chunks(s, 3)) == [0, 1, 4]        # tie among the 0.5s -> lowest index
    assert list(orc.select_chunks(s, 4)) == [0, 1, 2, 4]
    assert list(orc.select_chunks(s, 6)) == [0, 1, 2, 3, 4, 5]
    assert list(orc.select_chunks(s, 99)) == [0, 1, 2, 3, 4, 5]
    assert list(orc.select_chunks(s, 0)) == []
    with pytest.raises(ValueError):
        orc.select_chunks(np.array([0.1, np.nan]), 1)
    sel = orc.select_chunks(s, 2)
    assert list(sel) == sorted(sel)


def test_needles_are_selected_on_toy_config():
    wl = config_workload(1)
    sc = orc.chunk_scores(wl.q, wl.k_prefix, wl.v_prefix, wl.k_tree, wl.v_tree, wl.parent, wl.chunk_size)
    sel = orc.select_chunks(sc[wl.score_row], wl.top_k)
    assert set(wl.needle_chunks) <= set(int(x) for x in sel)
    assert len(sel) == wl.top_k


# ---------------------------------------------------------------------------
# I12: gather
# ---------------------------------------------------------------------------

def test_gather_round_trip_and_tail():
    rng = np.random.default_rng(47)
    Ld, H, L, d, B = 2, 3, 21, 4, 8                 # chunks: 8, 8, 5
    ks = rng.integers(0, 2 ** 16, size=(Ld, H, L, d)).astype(np.uint16)
    vs = rng.integers(0, 2 ** 16, size=(Ld, H, L, d)).astype(np.uint16)
    kd, vd, pos = orc.gather_draft_kv(ks, vs, [0, 1, 2], B)
    assert kd.dtype == np.uint16 and (kd == ks).all() and (vd == vs).all()
    assert list(pos) == list(range(L))
    kd, vd, pos = orc.gather_draft_kv(ks, vs, [2, 0], B)
    assert list(pos) == [16, 17, 18, 19, 20] + list(range(8))
    assert kd.shape == (Ld, H, 13, d)
    back_k = np.zeros_like(ks); back_k[:, :, pos] = kd        # scatter back
    assert (back_k[:, :, pos] == ks[:, :, pos]).all()
    assert (kd[:, :, :5] == ks[:, :, 16:21]).all() and (vd[:, :, 5:] == vs[:, :, 0:8]).all()
    with pytest.raises(ValueError):
        orc.gather_draft_kv(ks, vs, [3], B)
    kd, vd, pos = orc.gather_draft_kv(ks, vs, [], B)
    assert kd.shape == (Ld, H, 0, d) and len(pos) == 0


# ---------------------------------------------------------------------------
# generators: structural checks the configurations promise
# ---------------------------------------------------------------------------

def test_generated_trees_are_valid():
    for seed in range(5):
        rng = np.random.default_rng(seed)
        for parent, dmax in [(random_parent_tree(8, 4, rng), 4), (eagle_style_tree(60, 6, rng), 6),
                             (wide_tree(128, 4, rng), 4), (chain_tree(16), 15)]:
            assert parent[0] == -1
            assert all(-1 <= parent[i] < i for i in range(len(parent)))
            assert tree_depths(parent).max() <= dmax
            orc.ancestor_mask(parent)
    p = eagle_style_tree(60, 6, np.random.default_rng(2999))
    assert 4 <= int((p == 0).sum()) <= 8
    assert tree_depths(chain_tree(16)).tolist() == list(range(16))


def test_bf16_inputs_are_exact():
    from workloads import bf16_bits_to_f32, f32_to_bf16_bits
    wl = config_workload(2, prefix_len=64)
    for a in (wl.q, wl.k_prefix, wl.v_tree):
        assert (bf16_bits_to_f32(f32_to_bf16_bits(a)) == a).all()
        t = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
        assert (t == a).all()
    x = np.random.default_rng(0).standard_normal(1000).astype(np.float32)
    assert (bf16_bits_to_f32(f32_to_bf16_bits(x)) == torch.from_numpy(x).to(torch.bfloat16).float().numpy()).all()


# ---------------------------------------------------------------------------
# the materialised probability matrix of standard attention (Sec. 3.2.1)
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("seed", range(4))
def test_probability_matrix_against_the_fused_definition(seed):
    c = _rand_case(300 + seed, T=9, Hq=4, Hkv=2, d=8, L=41, std=1.5, max_depth=4)
    chunk = 8
    p = orc.attention_probabilities(c["q"], c["k_prefix"], c["k_tree"], c["parent"])
    out, lse, mass = orc.verify_attention(**c, chunk_size=chunk)
    T, Hq, L = 9, 4, 41
    assert p.shape == (Hq, T, L + T)
    np.testing.assert_allclose(p.sum(axis=2), 1.0, rtol=0, atol=1e-13)
    vis = orc.ancestor_mask(c["parent"])
    assert (p[:, :, L:][:, ~vis] == 0.0).all()                 # hidden tree keys carry exactly nothing
    assert (p[:, :, L:][:, vis] > 0.0).all() and (p[:, :, :L] > 0.0).all()
    G = Hq // 2
    for h in range(Hq):
        vals = np.concatenate([c["v_prefix"][h // G], c["v_tree"][h // G]], axis=0)
        np.testing.assert_allclose(p[h] @ vals, out[:, h, :], rtol=0, atol=1e-12)
        # a row's logits come back from p and lse: log p = logit - lse
        keys = np.concatenate([c["k_prefix"][h // G], c["k_tree"][h // G]], axis=0)
        logit = (c["q"][:, h, :] @ keys.T) / math.sqrt(8)
        seen = np.concatenate([np.ones((T, L), dtype=bool), vis], axis=1)
        np.testing.assert_allclose(np.log(p[h][seen]), (logit - lse[h][:, None])[seen], rtol=0, atol=1e-11)
    for cidx in range(mass.shape[2]):
        lo, hi = cidx * chunk, min((cidx + 1) * chunk, L)
        np.testing.assert_allclose(p[:, :, lo:hi].sum(axis=2), mass[:, :, cidx], rtol=0, atol=1e-13)
    # and the scores are chunk means of p averaged over heads
    sc = orc.chunk_scores(**c, chunk_size=chunk)
    sizes = np.array([min((k + 1) * chunk, L) - k * chunk for k in range(mass.shape[2])])
    mine = np.stack([p[:, :, k * chunk:k * chunk + sizes[k]].mean(axis=2) for k in range(len(sizes))], axis=2).mean(axis=0)
    np.testing.assert_allclose(mine, sc, rtol=0, atol=1e-14)


def test_probability_matrix_uniform_for_zero_query():
    c = _rand_case(310, T=6, Hq=2, Hkv=1, d=4, L=10, max_depth=5)
    p = orc.attention_probabilities(np.zeros_like(c["q"]), c["k_prefix"], c["k_tree"], c["parent"])
    vis = orc.ancestor_mask(c["parent"])
    for i in range(6):
        n_seen = 10 + int(vis[i].sum())
        np.testing.assert_allclose(p[:, i, :10], 1.0 / n_seen, rtol=0, atol=1e-15)
        np.testing.assert_allclose(p[:, i, 10:], np.broadcast_to(vis[i] / n_seen, (2, 6)), rtol=0, atol=1e-15)


def test_probability_matrix_matches_brute_force_scores():
    rng = np.random.default_rng(311)
    T, Hq, Hkv, d, L, chunk = 4, 4, 2, 3, 5, 2
    parent = [-1, 0, 0, 2]
    mk = lambda *s: rng.standard_normal(s)
    q, kp, vp, kt, vt = mk(T, Hq, d), mk(Hkv, L, d), mk(Hkv, L, d), mk(Hkv, T, d), mk(Hkv, T, d)
    _, _, score = _brute(q.tolist(), kp.tolist(), vp.tolist(), kt.tolist(), vt.tolist(), parent, chunk)
    p = orc.attention_probabilities(q, kp, kt, parent)
    sizes = [2, 2, 1]
    mine = np.stack([p[:, :, 2 * k:2 * k + sizes[k]].mean(axis=2) for k in range(3)], axis=2).mean(axis=0)
    np.testing.assert_allclose(mine, score, rtol=0, atol=1e-14)


# ---------------------------------------------------------------------------
# prefill: causal self-attention (Sec. 3.1)
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("n_q,n_all", [(19, 19), (7, 19), (1, 5)])
def test_prefill_against_sdpa_and_tail_routine(n_q, n_all):
    rng = np.random.default_rng(400 + n_q)
    Hq, Hkv, d = 4, 2, 8
    q = rng.standard_normal((n_q, Hq, d)) * 1.3
    k = rng.standard_normal((Hkv, n_all, d)) * 1.3
    v = rng.standard_normal((Hkv, n_all, d))
    out, lse = orc.prefill_attention(q, k, v)
    np.testing.assert_allclose(out, orc.causal_attention_tail(q, k, v), rtol=0, atol=1e-13)
    # library routine: torch SDPA in fp64 with an explicit lower-right causal mask
    qt = torch.from_numpy(q).permute(1, 0, 2)[None]                                  # [1,Hq,Tq,d]
    kt = torch.from_numpy(np.repeat(k, Hq // Hkv, axis=0))[None]
    vt = torch.from_numpy(np.repeat(v, Hq // Hkv, axis=0))[None]
    mask = torch.ones(n_q, n_all, dtype=torch.bool).tril(diagonal=n_all - n_q)
    ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)
    # lse against its definition on one row
    i, h = n_q - 1, 3
    logits = (k[h // 2, :n_all] @ q[i, h]) / math.sqrt(d)
    assert abs(lse[h, i] - math.log(sum(math.exp(x) for x in logits))) < 1e-12


def test_prefill_equals_chain_tree_verification():
    """A prompt is a chain: verifying a chain tree with an empty prefix is causal self-attention."""
    rng = np.random.default_rng(410)
    T, Hq, Hkv, d = 12, 4, 2, 8
    q, k, v = rng.standard_normal((T, Hq, d)), rng.standard_normal((Hkv, T, d)), rng.standard_normal((Hkv, T, d))
    out, lse = orc.prefill_attention(q, k, v)
    empty = np.zeros((Hkv, 0, d))
    ref_out, ref_lse, _ = orc.verify_attention(q, empty, empty, k, v, chain_tree(T))
    np.testing.assert_allclose(out, ref_out, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, ref_lse, rtol=0, atol=1e-13)


def test_prefill_closed_form_and_causality():
    rng = np.random.default_rng(411)
    N, Hq, Hkv, d = 9, 2, 1, 4
    k, v = rng.standard_normal((Hkv, N, d)), rng.standard_normal((Hkv, N, d))
    out, lse = orc.prefill_attention(np.zeros((N, Hq, d)), k, v)
    for i in range(N):                                           # Q = 0: running mean of V, lse = log(count)
        np.testing.assert_allclose(out[i, 0], v[0, :i + 1].mean(axis=0), rtol=0, atol=1e-14)
        assert abs(lse[1, i] - math.log(i + 1)) < 1e-14
    q = rng.standard_normal((N, Hq, d))
    a, _ = orc.prefill_attention(q, k, v)
    k2, v2 = k.copy(), v.copy()
    k2[:, 5:] += 3.0
    v2[:, 5:] -= 2.0
    b, _ = orc.prefill_attention(q, k2, v2)
    assert (a[:5] == b[:5]).all() and not np.allclose(a[5:], b[5:])   # a row never sees later keys
    # rows= computes exactly those rows
    c, lc = orc.prefill_attention(q, k, v, rows=[2, 7])
    assert (c[[2, 7]] == a[[2, 7]]).all() and (c[[0, 1, 3, 4, 5, 6, 8]] == 0).all() and np.isinf(lc[:, 0]).all()


# ---------------------------------------------------------------------------
# the paper's own retrieval settings (tests/golden/retrieval_settings.txt)
# ---------------------------------------------------------------------------

def _golden_settings():
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "retrieval_settings.txt")
    out = {}
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            name, value = line.split()
            out[name] = int(value)
    return out


def test_paper_retrieval_settings_give_the_paper_working_cache_sizes():
    """Table 8 / App. C: top-k chunks of the adopted chunk size are exactly the adopted working caches
    (32 x 32 = 1K tokens for Vicuna-68M, 64 x 32 = 2K for EAGLE), through SelectChunks + UpdateDraftCache."""
    g = _golden_settings()
    rng = np.random.default_rng(8)
    plen = 8192                                                   # the ablation's input length
    n_chunks = plen // g["chunk_size"]
    scores = rng.random(n_chunks)
    src = rng.integers(0, 2 ** 15, size=(1, 2, plen, 4)).astype(np.uint16)
    for model in ("vicuna68m", "eagle"):
        idx = orc.select_chunks(scores, g[f"top_k_{model}"])
        k_dst, v_dst, pos = orc.gather_draft_kv(src, src, idx, g["chunk_size"])
        assert k_dst.shape[2] == g[f"working_cache_{model}"] == len(pos)
        assert g[f"top_k_{model}"] * g["chunk_size"] == g[f"working_cache_{model}"]
    # the numbered benchmark configurations use the paper's chunk size and the smaller top-k
    wl = config_workload(2)
    assert wl.chunk_size == g["chunk_size"] and wl.top_k == g["top_k_vicuna68m"]
    assert wl.chunk_size * wl.top_k == g["working_cache_vicuna68m"]
