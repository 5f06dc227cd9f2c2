"""GPU parity: the HIP path through the C ABI versus the fp64 oracle, element by element.

Bars (stated where they are applied, see parity_util): out max-abs <= 2e-3 for
fp32 inputs and <= 2e-2 for bf16 inputs, both also relative to max|O|; lse
<= 2e-3; chunk scores within 1e-4 of the row's largest score; chunk indices by
the tolerance-aware top-k rule (exact where the margin is wide); gathered KV
bit-exact.
"""
import numpy as np
import pytest
import torch

import oracle as orc
from parity_util import (TOL, check_attention, check_scores, check_selection, oracle_all)
from workloads import (Workload, chain_tree, config_tree, config_workload, eagle_style_tree, make_workload,
                       random_parent_tree, wide_tree)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hx():
    from paper_2505_20776_amd import harness
    return harness


def _full_check(hx, wl, what, **kw):
    print(f"[case] {what} L={wl.prefix_len} T={wl.n_tree} Hq={wl.n_q_heads} Hkv={wl.n_kv_heads} d={wl.head_dim} "
          f"{wl.dtype} B={wl.chunk_size} {kw}", flush=True)
    ref_out, ref_lse, ref_scores = oracle_all(wl)
    res = hx.run_verify(wl, **kw)
    assert res["status"] == 0
    rel = check_attention(wl, res, ref_out, ref_lse, what)
    if ref_scores is not None and res["scores"] is not None:
        check_scores(res["scores"], ref_scores, what)
    return res, ref_out, ref_lse, ref_scores, rel


# --------------------------------------------------------------------------
# configuration 1: fp32 toy, all split counts
# --------------------------------------------------------------------------

@pytest.mark.parametrize("splits", [0, 1, 3, 8])
def test_toy_fp32(hx, splits):
    wl = config_workload(1)
    res, _, _, ref_scores, _ = _full_check(hx, wl, f"toy splits={splits}", num_splits=splits)
    sel, n, raw = hx.run_select(res["scores"][wl.score_row], wl.top_k)
    assert n == wl.top_k
    check_selection(sel, ref_scores[wl.score_row], wl.top_k, "toy")
    assert set(wl.needle_chunks) <= set(int(i) for i in sel)


def test_toy_sharp_and_ragged(hx):
    for plen in (512, 500, 33, 31, 1):
        wl = config_workload(1, sharp=True, prefix_len=plen)
        _full_check(hx, wl, f"toy sharp L={plen}")


# --------------------------------------------------------------------------
# configuration 2: one Llama-3.1-8B-shaped layer, bf16
# --------------------------------------------------------------------------

@pytest.mark.parametrize("sharp", [False, True])
def test_llama_layer_2k(hx, sharp):
    wl = config_workload(2, sharp=sharp)
    res, _, _, ref_scores, rel = _full_check(hx, wl, f"cfg2 sharp={sharp}")
    print(f"    relative out error {rel:.3e}", flush=True)
    for row in (wl.score_row, wl.n_tree - 1):
        sel, n, _ = hx.run_select(res["scores"][row], wl.top_k)
        check_selection(sel, ref_scores[row], wl.top_k, f"cfg2 row {row}")
    sel, _, _ = hx.run_select(res["scores"][wl.score_row], wl.top_k)
    assert set(wl.needle_chunks) <= set(int(i) for i in sel)


@pytest.mark.parametrize("splits", [1, 2, 5, 13, 27, 32, 47, 64])
def test_llama_layer_split_counts(hx, splits):
    wl = config_workload(2, sharp=True, prefix_len=2048 - 37)
    _full_check(hx, wl, f"cfg2 ragged splits={splits}", num_splits=splits)


def test_fp32_output_of_bf16_inputs(hx):
    wl = config_workload(2, sharp=True, prefix_len=777)
    _full_check(hx, wl, "cfg2 fp32 out", out_dtype="f32")


# --------------------------------------------------------------------------
# shapes: ragged tails, tiny and maximal trees, head_dim 64, other group sizes
# --------------------------------------------------------------------------

SHAPES = [
    # dtype, Hq, Hkv, d, L, tree, B
    ("bf16", 32, 8, 128, 1, "eagle60", 32),
    ("bf16", 32, 8, 128, 63, "eagle60", 32),
    ("bf16", 32, 8, 128, 65, "single", 32),
    ("bf16", 32, 8, 128, 4096 + 13, "wide128", 64),
    ("bf16", 32, 8, 128, 3000, "chain16", 64),
    ("bf16", 32, 8, 128, 2100, "eagle30", 32),      # 120 rows per KV head: 4-wave row-split kernel
    ("bf16", 32, 8, 128, 40, "eagle30", 32),        # barely more than one tile
    ("bf16", 8, 8, 128, 1500, "eagle60", 32),       # G = 1
    ("bf16", 16, 2, 128, 1111, "rand8", 32),        # G = 8
    ("bf16", 8, 2, 64, 2049, "eagle60", 32),        # head_dim 64
    ("bf16", 32, 8, 128, 2048, "eagle60", 48),      # chunk size not a multiple of 32
    ("f32", 8, 2, 128, 700, "rand8", 32),
    ("f32", 4, 1, 64, 129, "chain16", 16),
]


# head_dim 64 on the matrix cores (two keys per LDS row): the small draft model's shape (12 heads of 64, no
# grouping), grouped heads with more than 128 rows per KV head (8-wave kernel), prefixes around the 64-key
# tile (the shifted last tile with even and odd lengths, with chunk scores spanning its two score blocks)
D64_SHAPES = [
    # Hq, Hkv, L, tree, B, splits
    (12, 12, 1024, "eagle60", 32, 0),
    (12, 12, 1000, "eagle60", 32, 0),
    (12, 12, 64, "eagle60", 32, 0),
    (12, 12, 65, "eagle30", 32, 1),
    (12, 12, 127, "eagle60", 32, 0),
    (12, 12, 191, "single", 64, 2),
    (8, 2, 3001, "eagle60", 32, 0),          # 240 rows per KV head: 8 waves
    (16, 4, 4096 + 37, "wide128", 64, 5),    # 512 rows per KV head: two row groups
    (4, 4, 777, "chain16", 32, 3),
]


@pytest.mark.parametrize("Hq,Hkv,L,tree,B,splits", D64_SHAPES)
def test_head_dim_64_matrix_core_path(hx, Hq, Hkv, L, tree, B, splits):
    import paper_2505_20776_amd as sx
    rng = np.random.default_rng(Hq * 100 + L)
    wl = make_workload(f"d64_{tree}", seed=L + Hq, dtype="bf16", n_q_heads=Hq, n_kv_heads=Hkv, head_dim=64,
                       prefix_len=L, parent=_tree(tree, rng), chunk_size=B, top_k=4, n_needles=0, value_std=1.0)
    res, ref_out, ref_lse, ref_scores, _ = _full_check(hx, wl, f"d=64 {tree}", num_splits=splits)
    # the vector-ALU kernel on the same problem: two independent kernels, one answer
    valu = hx.run_verify(wl, num_splits=splits, flags=sx.SPECEXT_FLAG_VALU_PREFIX)
    assert np.abs(valu["out"] - res["out"]).max() <= 2e-2 * np.abs(ref_out).max()
    assert np.abs(valu["scores"] - res["scores"]).max() <= 1e-4 * ref_scores.max()


def _tree(kind, rng):
    return {"eagle60": lambda: eagle_style_tree(60, 6, rng), "eagle30": lambda: eagle_style_tree(30, 5, rng),
            "single": lambda: chain_tree(1),
            "wide128": lambda: wide_tree(128, 4, rng), "chain16": lambda: chain_tree(16),
            "rand8": lambda: random_parent_tree(8, 4, rng)}[kind]()


@pytest.mark.parametrize("dtype,Hq,Hkv,d,L,tree,B", SHAPES)
def test_shapes(hx, dtype, Hq, Hkv, d, L, tree, B):
    rng = np.random.default_rng(Hq * 1000 + L)
    wl = make_workload(f"shape_{tree}", seed=L * 7 + d, dtype=dtype, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d,
                       prefix_len=L, parent=_tree(tree, rng), chunk_size=B, top_k=4, n_needles=0, value_std=1.0)
    _full_check(hx, wl, f"shape {tree}")


def test_empty_prefix(hx):
    rng = np.random.default_rng(5)
    wl = make_workload("empty", seed=5, dtype="bf16", n_q_heads=32, n_kv_heads=8, head_dim=128, prefix_len=0,
                       parent=eagle_style_tree(60, 6, rng), chunk_size=32, top_k=4, n_needles=0, value_std=1.0)
    ref_out, ref_lse, _ = orc.verify_attention(wl.q, wl.k_prefix, wl.v_prefix, wl.k_tree, wl.v_tree, wl.parent)
    res = hx.run_verify(wl, want_scores=False)
    check_attention(wl, res, ref_out, ref_lse, "empty prefix")


def test_chain_tree_is_causal(hx):
    """The chain case checked against the separately written causal routine."""
    wl = make_workload("chain", seed=77, dtype="bf16", n_q_heads=32, n_kv_heads=8, head_dim=128, prefix_len=900,
                       parent=chain_tree(16), chunk_size=64, top_k=4, n_needles=0, value_std=1.0)
    res = hx.run_verify(wl)
    k_all = np.concatenate([wl.k_prefix, wl.k_tree], axis=1)
    v_all = np.concatenate([wl.v_prefix, wl.v_tree], axis=1)
    ref = orc.causal_attention_tail(wl.q, k_all, v_all)
    err = np.abs(res["out"] - ref).max()
    assert err <= TOL["bf16"] * np.abs(ref).max()


# --------------------------------------------------------------------------
# adversarial logits: a ramp (the max moves on every tile) and a +40 outlier
# --------------------------------------------------------------------------

def _directional(seed, L, ramp=None, outlier=None):
    rng = np.random.default_rng(seed)
    parent = eagle_style_tree(60, 6, rng)
    wl = make_workload("adv", seed=seed, dtype="bf16", n_q_heads=32, n_kv_heads=8, head_dim=128, prefix_len=L,
                       parent=parent, chunk_size=32, top_k=8, n_needles=0, value_std=0.25)
    d = wl.head_dim
    u = np.zeros(d, dtype=np.float32); u[3] = 1.0
    from workloads import quantize
    wl.q = quantize(wl.q * 0.1 + u * 4.0, "bf16")            # every query points along u
    if ramp is not None:
        steps = np.linspace(0.0, ramp, L, dtype=np.float32)     # logit grows along the sequence
        wl.k_prefix = quantize(wl.k_prefix + steps[None, :, None] * u[None, None, :], "bf16")
    if outlier is not None:
        pos, mag = outlier
        wl.k_prefix[:, pos, :] = quantize(u * mag, "bf16")
    return wl


def test_ramp_logits(hx):
    wl = _directional(901, 3000, ramp=float(60.0 * np.sqrt(128) / 4.0))   # logits climb by about 60 over the prefix
    _full_check(hx, wl, "ramp")
    wl = _directional(902, 3000, ramp=-float(60.0 * np.sqrt(128) / 4.0))
    _full_check(hx, wl, "descending ramp")


def test_outlier_key(hx):
    mag = float(40.0 * np.sqrt(128) / 4.0)
    for pos in (0, 1234, 2999):
        wl = _directional(903 + pos, 3000, outlier=(pos, mag))
        res, ref_out, _, ref_scores, _ = _full_check(hx, wl, f"outlier at {pos}")
        c = pos // wl.chunk_size
        size = min(wl.chunk_size, wl.prefix_len - c * wl.chunk_size)     # the last chunk is ragged
        assert abs(res["scores"][0, c] * size - 1.0) < 1e-3


# --------------------------------------------------------------------------
# strides, status word, determinism
# --------------------------------------------------------------------------

def test_strided_inputs(hx):
    import paper_2505_20776_amd as sx
    wl = config_workload(2, sharp=True, prefix_len=1000)
    ref_out, ref_lse, _ = orc.verify_attention(wl.q, wl.k_prefix, wl.v_prefix, wl.k_tree, wl.v_tree, wl.parent)
    T, Hq, d, Hkv, L = wl.n_tree, wl.n_q_heads, wl.head_dim, wl.n_kv_heads, wl.prefix_len
    cap = L + 24                                        # cache allocated longer than it is filled
    kp = torch.zeros((Hkv, cap, 2 * d), dtype=torch.bfloat16, device="cuda")   # rows padded to 2d elements
    vp = torch.zeros_like(kp)
    kp[:, :L, :d] = hx.to_device(wl.k_prefix, "bf16"); vp[:, :L, :d] = hx.to_device(wl.v_prefix, "bf16")
    qq = torch.zeros((T, Hq + 1, d), dtype=torch.bfloat16, device="cuda"); qq[:, :Hq] = hx.to_device(wl.q, "bf16")
    oo = torch.full((T, Hq, d + 8), 9.0, dtype=torch.bfloat16, device="cuda")
    buf = hx.make_buffers(dtype="bf16", n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, prefix_len=L, n_tree=T)
    buf.desc.q_stride_t = (Hq + 1) * d
    buf.desc.kp_stride_h = cap * 2 * d; buf.desc.kp_stride_l = 2 * d
    buf.desc.o_stride_t = Hq * (d + 8); buf.desc.o_stride_h = d + 8
    parent = torch.from_numpy(wl.parent).cuda()
    sx.verify_attn(buf.desc, qq, kp, vp, hx.to_device(wl.k_tree, "bf16"), hx.to_device(wl.v_tree, "bf16"), parent,
                   oo, buf.lse, buf.workspace)
    torch.cuda.synchronize()
    res = {"out": oo[:, :, :d].float().cpu().numpy(), "lse": buf.lse.cpu().numpy()}
    check_attention(wl, res, ref_out, ref_lse, "strided")
    assert (oo[:, :, d:].float() == 9.0).all()          # padding untouched


def test_malformed_parent_sets_status(hx):
    wl = config_workload(1)
    wl.parent = wl.parent.copy(); wl.parent[3] = 5           # forward reference
    res = hx.run_verify(wl)
    assert res["status"] == 1
    assert np.isfinite(res["out"]).all()
    wl.parent[3] = 1
    assert hx.run_verify(wl)["status"] == 0
    # the same on a Llama-shaped bf16 layer (matrix-core prefix kernel, fp16 partials, merge shared by four waves):
    # the bad entry ends that node's ancestor walk, everything stays finite, nothing else changes
    wl = config_workload(2, prefix_len=777)
    good = hx.run_verify(wl)
    assert good["status"] == 0
    before = wl.parent.copy()
    wl.parent = wl.parent.copy(); wl.parent[7] = 9
    bad = hx.run_verify(wl)
    assert bad["status"] == 1 and np.isfinite(bad["out"]).all() and np.isfinite(bad["lse"]).all()
    walks_through_7 = np.zeros(wl.n_tree, dtype=bool)
    for t in range(wl.n_tree):
        a = t
        while a >= 0:
            if a == 7:
                walks_through_7[t] = True
                break
            a = int(before[a])
    assert (bad["out"][~walks_through_7] == good["out"][~walks_through_7]).all()


def test_run_to_run_bit_identical(hx):
    wl = config_workload(2, sharp=True, prefix_len=3000)
    a = hx.run_verify(wl)
    b = hx.run_verify(wl)
    assert (a["out"] == b["out"]).all() and (a["lse"] == b["lse"]).all() and (a["scores"] == b["scores"]).all()


# --------------------------------------------------------------------------
# scale of V: the split partials cross HBM as fp16 after a per-row power-of-two
# rescale, so the output must follow V through any power of two (exactly representable
# in bf16) with the same relative accuracy
# --------------------------------------------------------------------------

@pytest.mark.parametrize("log2_scale", [-40, 24, 100])
def test_value_scale(hx, log2_scale):
    import dataclasses
    wl = config_workload(2, sharp=True)
    ref_out, ref_lse, _ = oracle_all(wl)
    f = np.float32(2.0) ** log2_scale
    big = dataclasses.replace(wl, v_prefix=wl.v_prefix * f, v_tree=wl.v_tree * f)
    res = hx.run_verify(big, want_scores=False)
    assert res["status"] == 0
    res["out"] = (res["out"].astype(np.float64) / float(f)).astype(np.float32)
    check_attention(wl, res, ref_out, ref_lse, f"V x 2^{log2_scale}")


@pytest.mark.parametrize("step_log2", [7, 30, 60])
def test_value_scale_differs_per_split(hx, step_log2):
    """The fp16 partials carry a per-row exponent per split: V whose magnitude alternates between neighbouring
    splits by a factor 2^step (so partials with very different exponents meet in the merge) must still
    match the oracle on the same values."""
    import dataclasses
    wl = config_workload(2, sharp=True, prefix_len=4096)
    res0 = hx.run_verify(wl, want_scores=False)
    per = wl.prefix_len // res0["num_splits"]
    scale = np.where((np.arange(wl.prefix_len) // per) % 2 == 1, np.float32(2.0) ** step_log2, np.float32(1.0)).astype(np.float32)
    big = dataclasses.replace(wl, v_prefix=wl.v_prefix * scale[None, :, None])
    ref_out, ref_lse, _ = oracle_all(big)
    res = hx.run_verify(big, want_scores=False)
    assert res["status"] == 0 and res["num_splits"] == res0["num_splits"]
    # the bar is relative to the largest output: bring both sides back to the unscaled magnitude first
    down = 2.0 ** -step_log2
    res["out"] = (res["out"].astype(np.float64) * down).astype(np.float32)
    check_attention(big, res, ref_out * down, ref_lse, f"V x 2^{step_log2} on odd splits")


# --------------------------------------------------------------------------
# SelectChunks on its own: bit-exact against the oracle on the same fp32 values
# --------------------------------------------------------------------------

@pytest.mark.parametrize("n,k", [(1, 1), (16, 4), (64, 32), (512, 32), (512, 512), (512, 600), (1000, 0),
                                 (1024, 77), (1025, 77), (4097, 100), (65536, 2048)])
def test_select_exact(hx, n, k):
    rng = np.random.default_rng(n + k)
    s = rng.random(n).astype(np.float32)
    sel, n_out, raw = hx.run_select(s, k)
    ref = orc.select_chunks(s, k)
    assert n_out == min(n, k) and list(sel) == list(ref)
    assert (raw[n_out:] == -1).all()


def test_select_ties_and_signs(hx):
    rng = np.random.default_rng(4)
    s = rng.integers(0, 4, size=777).astype(np.float32)         # heavy ties
    for k in (1, 5, 200, 776):
        sel, _, _ = hx.run_select(s, k)
        assert list(sel) == list(orc.select_chunks(s, k))
    s = (rng.standard_normal(300) * 3).astype(np.float32); s[7] = 0.0; s[9] = -0.0
    for k in (3, 150, 299):
        sel, _, _ = hx.run_select(s, k)
        assert list(sel) == list(orc.select_chunks(s, k))
    s = np.full(100, 0.25, dtype=np.float32)
    sel, _, _ = hx.run_select(s, 10)
    assert list(sel) == list(range(10))
    # keys that differ only in their lowest byte, in their lowest two bytes, and across the sign
    base = np.float32(1.0).view(np.uint32)
    for spread, n in ((7, 900), (70000, 1024), (3, 130)):
        bits = (base + rng.integers(0, spread, size=n)).astype(np.uint32)
        s = bits.view(np.float32).copy()
        s[::5] *= -1.0
        for k in (1, 17, n // 2, n - 1):
            sel, _, _ = hx.run_select(s, k)
            assert list(sel) == list(orc.select_chunks(s, k)), (spread, n, k)


# --------------------------------------------------------------------------
# UpdateDraftCache on its own: byte-exact
# --------------------------------------------------------------------------

def test_gather_exact(hx):
    rng = np.random.default_rng(8)
    Ld, H, L, d, B = 2, 3, 1000 - 37, 128, 32               # ragged last chunk of 3 tokens
    bits_k = torch.from_numpy(rng.integers(-2 ** 15, 2 ** 15, size=(Ld, H, L, d)).astype(np.int16)).cuda()
    bits_v = torch.from_numpy(rng.integers(-2 ** 15, 2 ** 15, size=(Ld, H, L, d)).astype(np.int16)).cuda()
    ks, vs = bits_k.view(torch.bfloat16), bits_v.view(torch.bfloat16)
    C = (L + B - 1) // B
    for idx in ([0, 5, 7, C - 1], [C - 1, 3, 3, 0], list(range(C)), [2]):
        kd, vd, pos, n = hx.run_gather(ks, vs, np.array(idx), B)
        rk, rv, rpos = orc.gather_draft_kv(bits_k.cpu().numpy(), bits_v.cpu().numpy(), idx, B)
        assert n == len(rpos) and list(pos[:n]) == list(rpos) and (pos[n:] == -1).all()
        assert (kd.view(torch.int16)[:, :, :n].cpu().numpy() == rk).all()
        assert (vd.view(torch.int16)[:, :, :n].cpu().numpy() == rv).all()
        assert (kd[:, :, n:].float() == 77).all() and (vd[:, :, n:].float() == 77).all()   # nothing written behind
    # n_idx on the device limits the list; invalid entries are skipped
    kd, vd, pos, n = hx.run_gather(ks, vs, np.array([4, 9, 1, 2]), B, n_idx=2)
    rk, rv, rpos = orc.gather_draft_kv(bits_k.cpu().numpy(), bits_v.cpu().numpy(), [4, 9], B)
    assert n == 2 * B and (kd.view(torch.int16)[:, :, :n].cpu().numpy() == rk).all() and list(pos[:n]) == list(rpos)
    kd, vd, pos, n = hx.run_gather(ks, vs, np.array([4, -1, C + 3, 6]), B)
    rk, rv, rpos = orc.gather_draft_kv(bits_k.cpu().numpy(), bits_v.cpu().numpy(), [4, 6], B)
    assert n == 2 * B and (vd.view(torch.int16)[:, :, :n].cpu().numpy() == rv).all() and list(pos[:n]) == list(rpos)
    # fp32 elements, head_dim 64
    src = torch.from_numpy(rng.standard_normal((1, 2, 300, 64)).astype(np.float32)).cuda()
    kd, vd, pos, n = hx.run_gather(src, src * 2, np.array([1, 0]), 100)
    assert (kd[0, :, :100] == src[0, :, 100:200]).all() and (vd[0, :, 100:200] == 2 * src[0, :, 0:100]).all()


# --------------------------------------------------------------------------
# configuration 3: 8K prefix, scores -> top-32 of 256 -> gather 1x8x1024x128
# --------------------------------------------------------------------------

def test_config3_retrieval_pipeline(hx):
    wl = config_workload(3)
    res, ref_out, ref_lse, ref_scores, rel = _full_check(hx, wl, "cfg3")
    print(f"    relative out error {rel:.3e}", flush=True)
    row = wl.score_row
    sel, n, _ = hx.run_select(res["scores"][row], wl.top_k)
    same = check_selection(sel, ref_scores[row], wl.top_k, "cfg3")
    assert set(wl.needle_chunks) <= set(int(i) for i in sel)
    dk, dv = hx.to_device(wl.draft_k, "bf16"), hx.to_device(wl.draft_v, "bf16")
    kd, vd, pos, length = hx.run_gather(dk, dv, sel, wl.chunk_size)
    assert kd.shape == (1, 8, 1024, 128) and length == 1024
    # bit-exact against the GPU's own index list ...
    from workloads import f32_to_bf16_bits
    rk, rv, rpos = orc.gather_draft_kv(f32_to_bf16_bits(wl.draft_k), f32_to_bf16_bits(wl.draft_v), sel, wl.chunk_size)
    assert (kd.view(torch.int16).cpu().numpy().view(np.uint16) == rk).all()
    assert (vd.view(torch.int16).cpu().numpy().view(np.uint16) == rv).all()
    assert list(pos) == list(rpos)
    # ... and against the oracle's own selection when the sets agree
    if same:
        ok, ov, _ = orc.gather_draft_kv(f32_to_bf16_bits(wl.draft_k), f32_to_bf16_bits(wl.draft_v),
                                        orc.select_chunks(ref_scores[row], wl.top_k), wl.chunk_size)
        assert (kd.view(torch.int16).cpu().numpy().view(np.uint16) == ok).all()


# --------------------------------------------------------------------------
# draft side: tree attention of the draft model over its compacted cache (App. D: a
# working cache of about 1K tokens), here with a StreamingLLM-style union of the sink
# chunk, the most recent chunks and the retrieved ones
# --------------------------------------------------------------------------

def test_draft_attention_over_compacted_cache(hx):
    import dataclasses
    from workloads import bf16_bits_to_f32, f32_to_bf16_bits
    wl = config_workload(3, sharp=True)
    _, _, ref_scores = oracle_all(wl)
    C = wl.n_chunks
    picked = set(int(i) for i in orc.select_chunks(ref_scores[wl.score_row], wl.top_k - 4))
    keep = sorted(picked | {0, C - 3, C - 2, C - 1})         # sink + recent + retrieved
    dk, dv = hx.to_device(wl.draft_k, "bf16"), hx.to_device(wl.draft_v, "bf16")
    print(f"[case] draft side over {len(keep)} chunks", flush=True)
    kd, vd, pos, length = hx.run_gather(dk, dv, np.array(keep), wl.chunk_size)
    rk, rv, rpos = orc.gather_draft_kv(f32_to_bf16_bits(wl.draft_k), f32_to_bf16_bits(wl.draft_v), keep, wl.chunk_size)
    assert length == len(rpos) == len(keep) * wl.chunk_size and list(pos[:length]) == list(rpos)
    # the draft model's tree attention over that cache, GPU gather -> GPU attention vs oracle gather -> oracle attention
    gpu_k = bf16_bits_to_f32(kd.view(torch.int16).cpu().numpy().view(np.uint16)[0, :, :length])
    gpu_v = bf16_bits_to_f32(vd.view(torch.int16).cpu().numpy().view(np.uint16)[0, :, :length])
    small = dataclasses.replace(wl, k_prefix=gpu_k, v_prefix=gpu_v, prefix_len=length)
    res = hx.run_verify(small, want_scores=False)
    assert res["status"] == 0
    ref_out, ref_lse, _ = orc.verify_attention(wl.q, bf16_bits_to_f32(rk[0]), bf16_bits_to_f32(rv[0]), wl.k_tree,
                                               wl.v_tree, wl.parent)
    check_attention(small, res, ref_out, ref_lse, "draft side")


# --------------------------------------------------------------------------
# configuration 5: stress shapes with a ragged prefix
# --------------------------------------------------------------------------

@pytest.mark.parametrize("variant", ["wide", "chain"])
def test_config5_stress(hx, variant):
    wl = config_workload(5, variant=variant, sharp=(variant == "wide"))
    res, ref_out, ref_lse, ref_scores, rel = _full_check(hx, wl, f"cfg5 {variant}")
    assert res["scores"].shape[1] == 512
    sel, n, _ = hx.run_select(res["scores"][0], wl.top_k)
    check_selection(sel, ref_scores[0], wl.top_k, f"cfg5 {variant}")
    if variant == "chain":
        k_all = np.concatenate([wl.k_prefix, wl.k_tree], axis=1)
        v_all = np.concatenate([wl.v_prefix, wl.v_tree], axis=1)
        ref = orc.causal_attention_tail(wl.q, k_all, v_all)
        assert np.abs(res["out"] - ref).max() <= TOL["bf16"] * np.abs(ref).max()


# --------------------------------------------------------------------------
# configuration 4 at full size, in the launch configuration the benchmark times
# (automatic split count), all layers' worth of distinct caches sampled
# --------------------------------------------------------------------------

def test_config4_full_size_sampled(hx):
    rng = np.random.default_rng(4242)
    for layer in (0, 13, 31):
        for sharp in ((False, True) if layer == 31 else (False,)):
            wl = config_workload(4, item=layer, sharp=sharp)
            print(f"[case] cfg4 layer {layer} sharp={sharp}", flush=True)
            res = hx.run_verify(wl)
            assert res["status"] == 0
            heads = sorted(int(h) for h in rng.choice(wl.n_q_heads, size=6, replace=False))
            G = wl.n_q_heads // wl.n_kv_heads
            for h in heads:
                g = h // G
                sub = Workload(name="s", dtype=wl.dtype, n_q_heads=1, n_kv_heads=1, head_dim=wl.head_dim,
                               prefix_len=wl.prefix_len, chunk_size=wl.chunk_size, top_k=wl.top_k,
                               parent=wl.parent, score_row=0, needle_chunks=[], q=wl.q[:, h:h + 1],
                               k_prefix=wl.k_prefix[g:g + 1], v_prefix=wl.v_prefix[g:g + 1],
                               k_tree=wl.k_tree[g:g + 1], v_tree=wl.v_tree[g:g + 1])
                ro, rl, _ = orc.verify_attention(sub.q, sub.k_prefix, sub.v_prefix, sub.k_tree, sub.v_tree, sub.parent)
                part = {"out": res["out"][:, h:h + 1], "lse": res["lse"][h:h + 1]}
                check_attention(sub, part, ro, rl, f"cfg4 layer {layer} head {h}")
            if layer == 31:
                # scores come from the last layer: all heads needed, full oracle on this one layer
                _, _, ref_scores = oracle_all(wl)
                check_scores(res["scores"], ref_scores, "cfg4 scores")
                sel, n, _ = hx.run_select(res["scores"][wl.score_row], wl.top_k)
                check_selection(sel, ref_scores[wl.score_row], wl.top_k, "cfg4 select")
                assert set(wl.needle_chunks) <= set(int(i) for i in sel)


# --------------------------------------------------------------------------
# the vector-ALU prefix kernel on bf16 inputs (the matrix-core kernel's fallback
# for other head sizes / chunk sizes) against the oracle, and the two kernels
# against each other
# --------------------------------------------------------------------------

def test_valu_prefix_kernel_on_bf16(hx):
    import paper_2505_20776_amd as sx
    wl = config_workload(2, sharp=True, prefix_len=2048 - 37)
    ref_out, ref_lse, ref_scores = oracle_all(wl)
    a = hx.run_verify(wl, flags=sx.SPECEXT_FLAG_VALU_PREFIX)
    check_attention(wl, a, ref_out, ref_lse, "valu kernel")
    check_scores(a["scores"], ref_scores, "valu kernel")
    b = hx.run_verify(wl)
    assert np.abs(a["out"] - b["out"]).max() <= 2e-2 * np.abs(ref_out).max()
    assert np.abs(a["scores"] - b["scores"]).max() <= 1e-4 * ref_scores.max()


# --------------------------------------------------------------------------
# the longest input the paper evaluates (128K tokens, Table 6), ragged by 21 tokens: every output,
# lse and score against the oracle
# --------------------------------------------------------------------------

def test_prefix_128k(hx):
    L = 131072 - 21
    wl = config_workload(4, item=3, prefix_len=L, sharp=True)
    print(f"[case] 128K prefix, L={L}", flush=True)
    res, ref_out, ref_lse, ref_scores, rel = _full_check(hx, wl, "128K prefix")
    sel, n, _ = hx.run_select(res["scores"][wl.score_row], wl.top_k)
    check_selection(sel, ref_scores[wl.score_row], wl.top_k, "128K select")
    assert n == wl.top_k and set(wl.needle_chunks) <= set(int(i) for i in sel)


# --------------------------------------------------------------------------
# seeded random shapes: every supported combination of dtype, head_dim, group size, tree size and kind,
# prefix length (including 0 and lengths around tile and split boundaries), chunk size and split count
# --------------------------------------------------------------------------

@pytest.mark.parametrize("seed", range(48))
def test_random_shapes(hx, seed):
    rng = np.random.default_rng(70000 + seed)
    dtype = "bf16" if rng.random() < 0.75 else "f32"
    d = 128 if rng.random() < 0.7 else 64
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 2, 4, 8]))
    T = int(rng.choice([1, 2, 3, 8, 15, 16, 17, 33, 60, 64, 65, 100, 128]))
    L = int(rng.choice([0, 1, 31, 32, 33, 63, 64, 65, 127, 129, 255, 257, 511, 1000, 1025, 2047, 3001, 4100]))
    B = int(rng.choice([16, 32, 48, 64]))
    splits = int(rng.choice([0, 0, 1, 2, 3, 5, 8]))
    kind = int(rng.integers(4))
    parent = (chain_tree(T) if kind == 0 or T < 4 else random_parent_tree(T, 12, rng) if kind == 1
              else eagle_style_tree(T, 6, rng) if kind == 2 else wide_tree(T, 4, rng))
    parent = np.asarray(parent[:T])
    if T > 5 and rng.random() < 0.25:
        parent[int(rng.integers(1, T))] = -1                   # a forest
    wl = make_workload(f"rand{seed}", seed=seed * 13 + 5, dtype=dtype, n_q_heads=Hkv * G, n_kv_heads=Hkv, head_dim=d,
                       prefix_len=L, parent=parent, chunk_size=B, top_k=4, n_needles=0,
                       value_std=1.0 if rng.random() < 0.5 else None)
    _full_check(hx, wl, f"random shape {seed}", num_splits=splits)


@pytest.mark.parametrize("seed", range(24))
def test_random_select_and_gather(hx, seed):
    """Seeded random score vectors (ties, signs, denormals, all lengths up to the 65536 limit) and random chunk
    lists (repeats, out-of-range entries, ragged source) : both exact."""
    rng = np.random.default_rng(81000 + seed)
    n = int(rng.choice([1, 2, 63, 64, 65, 511, 512, 1023, 1024, 1025, 4096, 5000, 65535, 65536]))
    kind = seed % 4
    s = (rng.standard_normal(n).astype(np.float32) if kind == 0 else
         rng.integers(-3, 4, size=n).astype(np.float32) if kind == 1 else
         (rng.random(n) * 1e-40).astype(np.float32) if kind == 2 else            # denormals and zeros
         np.abs(rng.standard_normal(n)).astype(np.float32) * np.float32(1e-4))
    k = int(rng.choice([0, 1, 2, 31, 32, 33, n // 2, n - 1 if n > 1 else 1, n, n + 5]))
    sel, n_out, raw = hx.run_select(s, k)
    ref = orc.select_chunks(s, k)
    assert n_out == len(ref) and list(sel) == list(ref), f"select n={n} k={k} kind={kind}"
    assert (raw[n_out:] == -1).all()
    # gather
    Ld, H, d = int(rng.choice([1, 2])), int(rng.choice([1, 3, 8])), int(rng.choice([64, 128]))
    B = int(rng.choice([16, 32, 100]))
    L = int(rng.integers(B, 40 * B))
    C = (L + B - 1) // B
    src_k = torch.from_numpy(rng.integers(-2 ** 15, 2 ** 15, size=(Ld, H, L, d)).astype(np.int16)).cuda()
    src_v = torch.from_numpy(rng.integers(-2 ** 15, 2 ** 15, size=(Ld, H, L, d)).astype(np.int16)).cuda()
    idx = rng.integers(-2, C + 2, size=int(rng.integers(1, 20)))
    valid = [int(c) for c in idx if 0 <= c < C]
    kd, vd, pos, length = hx.run_gather(src_k.view(torch.bfloat16), src_v.view(torch.bfloat16), idx, B)
    rk, rv, rpos = orc.gather_draft_kv(src_k.cpu().numpy(), src_v.cpu().numpy(), valid, B)
    assert length == len(rpos) and list(pos[:length]) == list(rpos) and (pos[length:] == -1).all()
    assert (kd.view(torch.int16)[:, :, :length].cpu().numpy() == rk).all()
    assert (vd.view(torch.int16)[:, :, :length].cpu().numpy() == rv).all()
