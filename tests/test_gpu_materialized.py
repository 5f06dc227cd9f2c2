"""GPU parity of the score path as Sec. 3.2.1 words it: standard attention with the probability matrix
written out, scores read from the matrix.  Checked against the oracle's matrix element by element, against
the oracle's outputs and scores, and against the fused path's scores."""
import numpy as np
import pytest
import torch

import oracle as orc
from parity_util import check_attention, check_scores, oracle_all
from workloads import (chain_tree, config_workload, eagle_style_tree, make_workload, random_parent_tree, wide_tree)

pytestmark = pytest.mark.gpu

# P: fp32 exponentials of fp32 logits of bf16 inputs; relative to the row's largest entry
PROB_EPS = 2e-5


@pytest.fixture(scope="module")
def hx():
    from paper_2505_20776_amd import harness
    return harness


def _check_all(hx, wl, what):
    print(f"[case] materialized {what}: L={wl.prefix_len} T={wl.n_tree} Hq={wl.n_q_heads} Hkv={wl.n_kv_heads}", flush=True)
    ref_out, ref_lse, ref_scores = oracle_all(wl)
    ref_p = orc.attention_probabilities(wl.q, wl.k_prefix, wl.k_tree, wl.parent)
    res = hx.run_materialized(wl)
    p = res["probs"].astype(np.float64)
    assert np.isfinite(p).all()
    err = np.abs(p - ref_p).max(axis=2)
    bar = PROB_EPS * ref_p.max(axis=2)
    assert (err <= bar).all(), f"{what}: P err {float((err / bar).max()):.2f} x the bar"
    assert (p[ref_p == 0.0] == 0.0).all(), f"{what}: hidden tree keys must be exactly zero"
    np.testing.assert_allclose(p.sum(axis=2), 1.0, rtol=0, atol=1e-4)
    check_attention(wl, res, ref_out, ref_lse, what)
    if ref_scores is not None:
        check_scores(res["scores"], ref_scores, what)
    return res, ref_scores


SHAPES = [
    # Hq, Hkv, L, tree, B
    (32, 8, 2048, "eagle60", 32),
    (32, 8, 1, "eagle60", 32),
    (32, 8, 63, "single", 32),
    (32, 8, 1000 + 13, "wide128", 64),
    (8, 8, 700, "chain16", 48),          # G = 1, chunk size that is no multiple of 32
    (16, 2, 1111, "rand8", 32),          # G = 8: 64 rows per KV head
    (64, 2, 300, "eagle60", 32),         # G = 32: 1920 rows per KV head, several row groups
]


def _tree(kind, rng):
    return {"eagle60": lambda: eagle_style_tree(60, 6, rng), "single": lambda: chain_tree(1),
            "wide128": lambda: wide_tree(128, 4, rng), "chain16": lambda: chain_tree(16),
            "rand8": lambda: random_parent_tree(8, 4, rng)}[kind]()


@pytest.mark.parametrize("Hq,Hkv,L,tree,B", SHAPES)
def test_shapes(hx, Hq, Hkv, L, tree, B):
    rng = np.random.default_rng(Hq * 1000 + L)
    wl = make_workload(f"mat_{tree}", seed=L * 7 + 1, dtype="bf16", n_q_heads=Hq, n_kv_heads=Hkv, head_dim=128,
                       prefix_len=L, parent=_tree(tree, rng), chunk_size=B, top_k=4, n_needles=0, value_std=1.0)
    _check_all(hx, wl, f"shape {tree}")


def test_empty_prefix(hx):
    rng = np.random.default_rng(5)
    wl = make_workload("empty", seed=5, dtype="bf16", n_q_heads=32, n_kv_heads=8, head_dim=128, prefix_len=0,
                       parent=eagle_style_tree(60, 6, rng), chunk_size=32, top_k=4, n_needles=0, value_std=1.0)
    _check_all(hx, wl, "empty prefix")


def test_agrees_with_the_fused_path_and_row_choice_on_device(hx):
    import paper_2505_20776_amd as sx
    wl = config_workload(2, sharp=True)
    res, ref_scores = _check_all(hx, wl, "config 2 sharp")
    fused = hx.run_verify(wl)
    for r in range(wl.n_tree):
        top = ref_scores[r].max()
        assert np.abs(res["scores"][r].astype(np.float64) - fused["scores"][r]).max() <= 2e-4 * top
    assert np.abs(res["out"] - fused["out"]).max() <= 2e-2 * np.abs(fused["out"]).max()
    # the row of the last accepted node, read on the device
    path = torch.tensor([0, 3, 17] + [-1] * (wl.n_tree - 3), dtype=torch.int32, device="cuda")
    n_acc = torch.tensor([3], dtype=torch.int32, device="cuda")
    one = torch.empty(ref_scores.shape[1], dtype=torch.float32, device="cuda")
    sx.chunk_scores_materialized(res["desc"], res["workspace"], 0, one, path=path, n_accept=n_acc)
    torch.cuda.synchronize()
    assert (one.cpu().numpy() == res["scores"][17]).all()
    n_acc.zero_()
    sx.chunk_scores_materialized(res["desc"], res["workspace"], 0, one, path=path, n_accept=n_acc)
    torch.cuda.synchronize()
    assert (one.cpu().numpy() == res["scores"][0]).all()


def test_fp32_output_and_strided_cache(hx):
    """fp32 output of bf16 inputs; K/V prefix as a slice of a capacity-sized cache."""
    import paper_2505_20776_amd as sx
    rng = np.random.default_rng(77)
    L, cap = 777, 1024
    wl = make_workload("mat_strided", seed=77, dtype="bf16", n_q_heads=8, n_kv_heads=2, head_dim=128, prefix_len=L,
                       parent=eagle_style_tree(26, 5, rng), chunk_size=32, top_k=4, n_needles=0, value_std=1.0)
    ref_out, ref_lse, ref_scores = oracle_all(wl)
    dev = "cuda"
    kc = torch.zeros((2, cap, 128), dtype=torch.bfloat16, device=dev)
    vc = torch.zeros_like(kc)
    kc[:, :L] = hx.to_device(wl.k_prefix, "bf16", dev)
    vc[:, :L] = hx.to_device(wl.v_prefix, "bf16", dev)
    desc = sx.make_desc(dtype=sx.SPECEXT_BF16, out_dtype=sx.SPECEXT_F32, n_q_heads=8, n_kv_heads=2, head_dim=128,
                        prefix_len=L, n_tree=26, chunk_size=32, want_scores=True, kp_stride_h=cap * 128)
    ws = torch.empty(sx.materialized_bytes(desc), dtype=torch.uint8, device=dev)
    out = torch.empty((26, 8, 128), dtype=torch.float32, device=dev)
    lse = torch.empty((8, 26), dtype=torch.float32, device=dev)
    parent = torch.from_numpy(np.asarray(wl.parent, dtype=np.int32)).to(dev)
    sx.attn_materialized(desc, hx.to_device(wl.q, "bf16", dev), kc, vc, hx.to_device(wl.k_tree, "bf16", dev),
                         hx.to_device(wl.v_tree, "bf16", dev), parent, out, lse, ws)
    one = torch.empty(ref_scores.shape[1], dtype=torch.float32, device=dev)
    sx.chunk_scores_materialized(desc, ws, 5, one)
    torch.cuda.synchronize()
    check_attention(wl, {"out": out.cpu().numpy(), "lse": lse.cpu().numpy()}, ref_out, ref_lse, "strided fp32 out")
    check_scores(one.cpu().numpy()[None], ref_scores[5][None], "strided scores")


@pytest.mark.parametrize("seed", range(12))
def test_random_shapes(hx, seed):
    rng = np.random.default_rng(92000 + seed)
    Hkv = int(rng.choice([1, 2, 8]))
    G = int(rng.choice([1, 2, 4, 8]))
    T = int(rng.choice([1, 2, 9, 16, 33, 60, 64, 65, 128]))
    L = int(rng.choice([0, 1, 31, 32, 33, 64, 200, 513, 1000, 2049]))
    B = int(rng.choice([16, 32, 48, 64]))
    parent = np.asarray((chain_tree(T) if T < 4 or seed % 3 == 0 else random_parent_tree(T, 10, rng) if seed % 3 == 1
                         else eagle_style_tree(T, 6, rng))[:T])
    wl = make_workload(f"matrand{seed}", seed=seed * 17 + 3, dtype="bf16", n_q_heads=Hkv * G, n_kv_heads=Hkv,
                       head_dim=128, prefix_len=L, parent=parent, chunk_size=B, top_k=4, n_needles=0, value_std=1.0)
    _check_all(hx, wl, f"random shape {seed}")


def test_malformed_parent_sets_status(hx):
    rng = np.random.default_rng(6)
    wl = make_workload("badparent", seed=6, dtype="bf16", n_q_heads=8, n_kv_heads=2, head_dim=128, prefix_len=100,
                       parent=eagle_style_tree(20, 5, rng), chunk_size=32, top_k=4, n_needles=0, value_std=1.0)
    res = hx.run_materialized(wl)
    assert int(res["workspace"][:4].view(torch.int32).item()) == 0
    wl.parent = wl.parent.copy()
    wl.parent[7] = 9                                             # not a topological parent: node 7 becomes a root
    res = hx.run_materialized(wl)
    assert int(res["workspace"][:4].view(torch.int32).item()) == 1
    fixed = wl.parent.copy()
    fixed[7] = -1
    ref_p = orc.attention_probabilities(wl.q, wl.k_prefix, wl.k_tree, fixed)
    assert np.abs(res["probs"] - ref_p).max() <= PROB_EPS * ref_p.max()
