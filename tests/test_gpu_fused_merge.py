"""The tree pass and merge as the tail of the prefix launch (SPECEXT_FLAG_FUSED_MERGE) against the fp64
oracle and against the default two-launch form, through the C ABI.

Covers the hand-over between workgroups: all split counts that form runs with, a workspace reused over
many calls and shapes (nothing is reset between calls), the path where workgroups stop waiting and the
last one to finish merges their rows (SPECEXT_FLAG_SHORT_WAIT forces it from the host; every kernel
still exits normally), an uninitialised workspace (reported through the status word, nothing
computed), and bit-reproducibility."""
import numpy as np
import pytest
import torch

from parity_util import check_attention, oracle_all
from workloads import chain_tree, config_workload, eagle_style_tree, make_workload, wide_tree

pytestmark = pytest.mark.gpu


def _device_inputs(wl):
    from paper_2505_20776_amd import harness
    dev = "cuda"
    t = [harness.to_device(a, wl.dtype, dev) for a in (wl.q, wl.k_prefix, wl.v_prefix, wl.k_tree, wl.v_tree)]
    t.append(torch.from_numpy(np.asarray(wl.parent, dtype=np.int32)).to(dev))
    return t


def _run(wl, flags, num_splits=0, buf=None, inputs=None):
    import paper_2505_20776_amd as sx
    from paper_2505_20776_amd import harness
    q, kp, vp, kt, vt, parent = inputs or _device_inputs(wl)
    if buf is None:
        buf = harness.make_buffers(dtype=wl.dtype, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                                   head_dim=wl.head_dim, prefix_len=wl.prefix_len, n_tree=wl.n_tree,
                                   num_splits=num_splits, flags=flags)
    buf.out.fill_(float("nan"))
    buf.lse.fill_(float("nan"))
    sx.verify_attn(buf.desc, q, kp, vp, kt, vt, parent, buf.out, buf.lse, buf.workspace)
    torch.cuda.synchronize()
    status = int(buf.workspace[:4].view(torch.int32).item())
    return {"out": buf.out.float().cpu().numpy(), "lse": buf.lse.cpu().numpy(), "status": status,
            "raw": buf.out.clone(), "buf": buf}


def _wl(L, tree, seed, Hq=32, Hkv=8):
    rng = np.random.default_rng(seed)
    parent = {"eagle60": lambda: eagle_style_tree(60, 6, rng), "wide128": lambda: wide_tree(128, 4, rng),
              "chain16": lambda: chain_tree(16), "eagle26": lambda: eagle_style_tree(26, 6, rng)[:26]}[tree]()
    return make_workload(f"fused_{tree}", seed=seed, dtype="bf16", n_q_heads=Hq, n_kv_heads=Hkv, head_dim=128,
                         prefix_len=L, parent=parent, chunk_size=32, top_k=4, n_needles=0, value_std=1.0)


CASES = [  # L, tree, splits, Hq, Hkv
    (16384 - 37, "eagle60", 0, 32, 8),      # 32 splits, 8 rows per slice, four groups share a row's splits
    (2048, "eagle60", 0, 32, 8),            # 8 splits, 30 rows per slice
    (1000, "eagle26", 0, 8, 2),             # 4-wave kernel, 26 rows per slice in two passes
    (1000, "eagle26", 1, 8, 2),             # one split: the workgroup merges alone
    (4096 + 13, "wide128", 0, 32, 8),       # two row groups per KV head
    (3000, "chain16", 0, 32, 8),            # 64 rows per KV head, depth 16 (two batches of ancestors)
    (9000, "eagle60", 27, 32, 8),           # a split count that does not divide the rows
]


@pytest.mark.parametrize("L,tree,splits,Hq,Hkv", CASES)
def test_fused_matches_oracle_and_two_launch_form(L, tree, splits, Hq, Hkv):
    import paper_2505_20776_amd as sx
    wl = _wl(L, tree, seed=L + splits, Hq=Hq, Hkv=Hkv)
    print(f"[case] fused merge L={L} tree={tree} splits={splits} Hq={Hq} Hkv={Hkv}", flush=True)
    ref_out, ref_lse, _ = oracle_all(wl)
    fused = _run(wl, sx.SPECEXT_FLAG_FUSED_MERGE, splits)
    plain = _run(wl, 0, splits)
    assert fused["status"] == 0 and plain["status"] == 0
    check_attention(wl, fused, ref_out, ref_lse, "fused")
    # the two forms read the same split partials and differ in summation order only
    assert np.abs(fused["out"] - plain["out"]).max() <= 2 ** -7 * np.abs(ref_out).max()
    assert np.abs(fused["lse"] - plain["lse"]).max() <= 1e-5
    # handing every slice to the last workgroup changes nothing, bit for bit
    short = _run(wl, sx.SPECEXT_FLAG_FUSED_MERGE | sx.SPECEXT_FLAG_SHORT_WAIT, splits)
    assert short["status"] == 0
    assert torch.equal(short["raw"].view(torch.int16), fused["raw"].view(torch.int16))
    assert np.array_equal(short["lse"], fused["lse"])


def test_one_workspace_many_calls_and_shapes():
    import paper_2505_20776_amd as sx
    from paper_2505_20776_amd import harness
    big = _wl(8192, "eagle60", seed=5)
    small = _wl(1500, "eagle60", seed=6)
    ws_desc = harness.make_buffers(dtype="bf16", n_q_heads=32, n_kv_heads=8, head_dim=128, prefix_len=8192, n_tree=60,
                                   flags=sx.SPECEXT_FLAG_FUSED_MERGE)
    first = {}
    for rep in range(3):
        for name, wl in (("big", big), ("small", small), ("big-short-wait", big)):
            flags = sx.SPECEXT_FLAG_FUSED_MERGE | (sx.SPECEXT_FLAG_SHORT_WAIT if "short" in name else 0)
            buf = harness.make_buffers(dtype="bf16", n_q_heads=32, n_kv_heads=8, head_dim=128,
                                       prefix_len=wl.prefix_len, n_tree=60, flags=flags)
            buf.workspace = ws_desc.workspace          # initialised once, shared by every call below
            res = _run(wl, flags, buf=buf)
            assert res["status"] == 0
            key = name.split("-")[0]
            if key not in first:
                ref_out, ref_lse, _ = oracle_all(wl)
                check_attention(wl, res, ref_out, ref_lse, name)
                first[key] = res["raw"]
            else:
                assert torch.equal(res["raw"].view(torch.int16), first[key].view(torch.int16)), f"{name} rep {rep}"


def test_uninitialised_workspace_is_reported():
    import paper_2505_20776_amd as sx
    wl = _wl(4096, "eagle60", seed=9)
    q, kp, vp, kt, vt, parent = _device_inputs(wl)
    desc = sx.make_desc(dtype=sx.SPECEXT_BF16, n_q_heads=32, n_kv_heads=8, head_dim=128, prefix_len=4096, n_tree=60,
                        flags=sx.SPECEXT_FLAG_FUSED_MERGE)
    ws = torch.full((sx.workspace_bytes(desc),), 0x5A, dtype=torch.uint8, device="cuda")     # never initialised
    out = torch.full((60, 32, 128), 7.0, dtype=torch.bfloat16, device="cuda")
    lse = torch.full((32, 60), 7.0, dtype=torch.float32, device="cuda")
    sx.verify_attn(desc, q, kp, vp, kt, vt, parent, out, lse, ws)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) == 2
    assert bool((out == 7.0).all()) and bool((lse == 7.0).all())
    # the same call after the init works, and without the flag no init is needed at all
    sx.workspace_init(ws)
    sx.verify_attn(desc, q, kp, vp, kt, vt, parent, out, lse, ws)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) == 0
    ref_out, ref_lse, _ = oracle_all(wl)
    check_attention(wl, {"out": out.float().cpu().numpy(), "lse": lse.cpu().numpy()}, ref_out, ref_lse, "after init")
    ws2 = torch.full((sx.workspace_bytes(desc),), 0x5A, dtype=torch.uint8, device="cuda")
    desc.flags = 0
    sx.verify_attn(desc, q, kp, vp, kt, vt, parent, out, lse, ws2)
    torch.cuda.synchronize()
    assert int(ws2[:4].view(torch.int32).item()) == 0


def test_fused_malformed_parent_and_static_entry():
    import paper_2505_20776_amd as sx
    from paper_2505_20776_amd import harness
    wl = _wl(2048 + 5, "eagle60", seed=11)
    q, kp, vp, kt, vt, parent = _device_inputs(wl)
    bad = np.asarray(wl.parent, dtype=np.int32).copy()
    bad[7] = 9
    buf = harness.make_buffers(dtype="bf16", n_q_heads=32, n_kv_heads=8, head_dim=128, prefix_len=wl.prefix_len,
                               n_tree=60, flags=sx.SPECEXT_FLAG_FUSED_MERGE)
    res = _run(wl, sx.SPECEXT_FLAG_FUSED_MERGE, buf=buf, inputs=(q, kp, vp, kt, vt, torch.from_numpy(bad).cuda()))
    assert res["status"] == 1
    # the entry point on the library's own scratch memory takes the flag as well
    good = _run(wl, sx.SPECEXT_FLAG_FUSED_MERGE)
    out2 = torch.full_like(buf.out, float("nan"))
    lse2 = torch.full_like(buf.lse, float("nan"))
    status = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    for _ in range(2):
        sx.verify_attn_static(buf.desc, q, kp, vp, kt, vt, parent, out2, lse2, status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    assert torch.equal(out2.view(torch.int16), good["raw"].view(torch.int16))
