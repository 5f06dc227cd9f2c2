"""specext_verify_attn_static (the entry point for callers that cannot allocate) against
specext_verify_attn on the same inputs, through the C ABI.

Both run the same kernels, one on the caller's workspace, one on the library's static
scratch array, so the outputs must be bit-identical; the workspace path itself is held to
the oracle by test_gpu_parity.  Two calls in a row share the scratch array, the second on
a smaller problem, so stale contents of the first must not leak into the second.  The
oracle bar (bf16 inputs: 2e-2 of max|O|, lse 2e-3) is applied to the static path as well.
"""
import numpy as np
import pytest
import torch

from parity_util import check_attention, oracle_all
from workloads import config_workload

pytestmark = pytest.mark.gpu


def _run_both(wl, poison_allocator=False):
    import paper_2505_20776_amd as sx
    from paper_2505_20776_amd import harness

    dev = "cuda"
    q, kp, vp, kt, vt = (harness.to_device(a, wl.dtype, dev) for a in (wl.q, wl.k_prefix, wl.v_prefix, wl.k_tree, wl.v_tree))
    parent = torch.from_numpy(np.asarray(wl.parent, dtype=np.int32)).to(dev)
    buf = harness.make_buffers(dtype=wl.dtype, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim,
                               prefix_len=wl.prefix_len, n_tree=wl.n_tree)
    sx.verify_attn(buf.desc, q, kp, vp, kt, vt, parent, buf.out, buf.lse, buf.workspace)
    out2 = torch.full_like(buf.out, float("nan"))
    lse2 = torch.full_like(buf.lse, float("nan"))
    status = torch.full((1,), -7, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"] if poison_allocator else None
    sx.verify_attn_static(buf.desc, q, kp, vp, kt, vt, parent, out2, lse2, status)
    torch.cuda.synchronize()
    if poison_allocator:
        # the call went through no torch allocation either
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    assert int(status.item()) == 0
    assert torch.equal(out2.view(torch.int16) if out2.dtype == torch.bfloat16 else out2.view(torch.int32),
                       buf.out.view(torch.int16) if buf.out.dtype == torch.bfloat16 else buf.out.view(torch.int32))
    assert torch.equal(lse2.view(torch.int32), buf.lse.view(torch.int32))
    return {"out": out2.float().cpu().numpy(), "lse": lse2.cpu().numpy()}


def test_static_entry_matches_workspace_entry_twice():
    # first call: the Llama-3.1-8B layer shape with 32 splits over a ragged prefix; second call: a smaller
    # problem (fewer rows, fewer splits, shorter prefix) on the scratch the first one left behind
    first = config_workload(2, sharp=True, prefix_len=8192 - 37)
    second = config_workload(2, sharp=True, prefix_len=1024 + 5)
    for wl, name in ((first, "first"), (second, "second (smaller)")):
        print(f"[case] static entry, {name}: L={wl.prefix_len} T={wl.n_tree}", flush=True)
        res = _run_both(wl, poison_allocator=True)
        ref_out, ref_lse, _ = oracle_all(wl)
        check_attention(wl, res, ref_out, ref_lse, f"static {name}")


def test_static_entry_fp32_toy_and_malformed_parent():
    import paper_2505_20776_amd as sx
    from paper_2505_20776_amd import harness

    wl = config_workload(1)
    res = _run_both(wl)
    ref_out, ref_lse, _ = oracle_all(wl)
    check_attention(wl, res, ref_out, ref_lse, "static toy")
    # a parent index that is not smaller than its node is reported through status_out
    dev = "cuda"
    q, kp, vp, kt, vt = (harness.to_device(a, wl.dtype, dev) for a in (wl.q, wl.k_prefix, wl.v_prefix, wl.k_tree, wl.v_tree))
    bad = np.asarray(wl.parent, dtype=np.int32).copy()
    bad[3] = 5
    buf = harness.make_buffers(dtype=wl.dtype, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim,
                               prefix_len=wl.prefix_len, n_tree=wl.n_tree)
    status = torch.zeros((1,), dtype=torch.int32, device=dev)
    sx.verify_attn_static(buf.desc, q, kp, vp, kt, vt, torch.from_numpy(bad).to(dev), buf.out, buf.lse, status)
    torch.cuda.synchronize()
    assert int(status.item()) == 1


def test_static_entry_rejects_what_it_cannot_hold():
    import paper_2505_20776_amd as sx
    from paper_2505_20776_amd import harness

    dev = "cuda"
    dummy = torch.zeros(64, dtype=torch.bfloat16, device=dev)
    par = torch.zeros(128, dtype=torch.int32, device=dev)
    # 128-node tree at 256 splits: the fp32-sized partial region alone is 537 MB
    big = sx.make_desc(dtype=sx.SPECEXT_BF16, n_q_heads=32, n_kv_heads=8, head_dim=128, prefix_len=1 << 20, n_tree=128,
                       num_splits=256)
    assert sx.workspace_bytes(big) > (48 << 20)
    rc = sx.verify_attn_static(big, dummy, dummy, dummy, dummy, dummy, par, dummy, None, None, check=False)
    assert rc == -3
    scored = sx.make_desc(dtype=sx.SPECEXT_BF16, n_q_heads=32, n_kv_heads=8, head_dim=128, prefix_len=2048, n_tree=60,
                          chunk_size=32, want_scores=True)
    rc = sx.verify_attn_static(scored, dummy, dummy, dummy, dummy, dummy, par, dummy, None, None, check=False)
    assert rc == -2
