"""The retrieval calls exactly as the benchmark and a serving loop issue them, through the C ABI:
specext_chunk_scores for ONE row (the root and a leaf), specext_chunk_scores_select (scores and top-k in
one launch) against the two separate calls bit for bit and against the oracle, verification without an lse
output, and sentinel regions around every output buffer (the harness allocates them for every test; here
they are asserted explicitly on the largest shapes)."""
import numpy as np
import pytest
import torch

import oracle as orc
from parity_util import SCORE_EPS, check_attention, check_scores, check_selection, oracle_all
from workloads import config_workload

pytestmark = pytest.mark.gpu


def _verify_with_scores(wl):
    import paper_2505_20776_amd as sx
    from paper_2505_20776_amd import harness
    dev = "cuda"
    t = [harness.to_device(a, wl.dtype, dev) for a in (wl.q, wl.k_prefix, wl.v_prefix, wl.k_tree, wl.v_tree)]
    parent = torch.from_numpy(np.asarray(wl.parent, dtype=np.int32)).to(dev)
    buf = harness.make_buffers(dtype=wl.dtype, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim,
                               prefix_len=wl.prefix_len, n_tree=wl.n_tree, chunk_size=wl.chunk_size, want_scores=True)
    sx.verify_attn(buf.desc, *t, parent, buf.out, buf.lse, buf.workspace)
    return buf


@pytest.mark.parametrize("cfg,plen", [(3, 8192), (2, 2048 - 37), (1, 512), (4, 40000)])
def test_single_row_scores_and_fused_selection(cfg, plen):
    import paper_2505_20776_amd as sx
    from paper_2505_20776_amd import harness
    wl = config_workload(cfg, sharp=True, prefix_len=plen)
    print(f"[case] single-row scores cfg {cfg} L={plen}", flush=True)
    buf = _verify_with_scores(wl)
    ref = orc.chunk_scores(wl.q, wl.k_prefix, wl.v_prefix, wl.k_tree, wl.v_tree, wl.parent, wl.chunk_size)
    C = ref.shape[1]
    leaf = wl.n_tree - 1
    k = wl.top_k
    for row in (0, leaf):
        one, one_base = harness.guarded((C,), torch.float32)
        one.fill_(float("nan"))
        sx.chunk_scores(buf.desc, buf.workspace, row, one)                     # the call the benchmark times
        idx = torch.full((k,), -7, dtype=torch.int32, device="cuda")
        n_out = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        sx.select_chunks(one, C, k, idx, n_out)
        both, both_base = harness.guarded((C,), torch.float32)
        both.fill_(float("nan"))
        idx2, idx2_base = harness.guarded((k,), torch.int32)
        n2, n2_base = harness.guarded((1,), torch.int32)
        sx.chunk_scores_select(buf.desc, buf.workspace, row, k, idx2, n2, scores=both)
        torch.cuda.synchronize()
        buf.check_guards()
        for b in (one_base, both_base, idx2_base, n2_base):
            assert harness.guards_intact(b)
        got = one.cpu().numpy()
        check_scores(got[None], ref[row][None], f"row {row}")
        check_selection(idx.cpu().numpy()[:int(n_out.item())], ref[row], k, f"row {row}")
        # one launch or two: the same bits
        assert torch.equal(both.view(torch.int32), one.view(torch.int32))
        assert torch.equal(idx2, idx) and int(n2.item()) == int(n_out.item()) == min(k, C)
        # and the decision itself, taken on the kernel's own scores, is exact
        assert list(idx.cpu().numpy()[:min(k, C)]) == list(orc.select_chunks(got, k))
    if C <= 1024:
        # without a scores output, and with the row read from an accepted path on the device
        idx3 = torch.full((k,), -7, dtype=torch.int32, device="cuda")
        n3 = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        path = torch.tensor([0, leaf] + [-1] * (wl.n_tree - 2), dtype=torch.int32, device="cuda")[:wl.n_tree]
        n_acc = torch.tensor([min(2, wl.n_tree)], dtype=torch.int32, device="cuda")
        sx.chunk_scores_select(buf.desc, buf.workspace, 0, k, idx3, n3, path=path, n_accept=n_acc)
        torch.cuda.synchronize()
        assert torch.equal(idx3, idx2)                                         # idx2 holds the leaf row's selection
    else:
        rc = sx.chunk_scores_select(buf.desc, buf.workspace, 0, k, idx2, n2, check=False)
        assert rc == -1                                                        # more than 1024 chunks need a scores buffer


def test_verify_without_lse_output():
    import paper_2505_20776_amd as sx
    from paper_2505_20776_amd import harness
    for wl in (config_workload(2, sharp=True, prefix_len=3000), config_workload(1), config_workload(2, sharp=True, prefix_len=33)):
        dev = "cuda"
        t = [harness.to_device(a, wl.dtype, dev) for a in (wl.q, wl.k_prefix, wl.v_prefix, wl.k_tree, wl.v_tree)]
        if wl.prefix_len == 0:
            t[1] = t[2] = None
        parent = torch.from_numpy(np.asarray(wl.parent, dtype=np.int32)).to(dev)
        a = harness.make_buffers(dtype=wl.dtype, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                                 head_dim=wl.head_dim, prefix_len=wl.prefix_len, n_tree=wl.n_tree)
        b = harness.make_buffers(dtype=wl.dtype, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                                 head_dim=wl.head_dim, prefix_len=wl.prefix_len, n_tree=wl.n_tree)
        sx.verify_attn(a.desc, *t, parent, a.out, a.lse, a.workspace)
        sx.verify_attn(b.desc, *t, parent, b.out, None, b.workspace)
        torch.cuda.synchronize()
        a.check_guards()
        b.check_guards()
        assert torch.equal(a.out.view(torch.uint8), b.out.view(torch.uint8))
        ref_out, ref_lse, _ = oracle_all(wl)
        check_attention(wl, {"out": b.out.float().cpu().numpy(), "lse": a.lse.cpu().numpy()}, ref_out, ref_lse, "no lse")


@pytest.mark.parametrize("what", ["cfg4", "cfg5wide", "cfg5chain", "128k"])
def test_nothing_is_written_outside_the_buffers(what):
    """Every run through harness.run_verify checks the sentinels; this spells the requirement out for the
    largest launch shapes (scores for all rows, then one row, selection and gather behind them)."""
    from paper_2505_20776_amd import harness
    wl = {"cfg4": lambda: config_workload(4, item=7), "cfg5wide": lambda: config_workload(5, variant="wide"),
          "cfg5chain": lambda: config_workload(5, variant="chain"),
          "128k": lambda: config_workload(4, item=1, prefix_len=131072 - 21)}[what]()
    print(f"[case] sentinels {what}: L={wl.prefix_len} T={wl.n_tree}", flush=True)
    res = harness.run_verify(wl)                     # asserts the sentinels of workspace, out, lse, scores
    assert res["status"] == 0 and np.isfinite(res["out"]).all() and np.isfinite(res["scores"]).all()
    sel, n, raw = harness.run_select(res["scores"][0], wl.top_k)          # asserts those of idx_out, n_out
    src = harness.to_device(wl.k_prefix[None].copy(), wl.dtype)
    kd, vd, pos, length = harness.run_gather(src, src, sel, wl.chunk_size)     # and of k_dst, v_dst, pos_out, len_out
    rk, _, rpos = orc.gather_draft_kv(src.float().cpu().numpy(), src.float().cpu().numpy(), sel, wl.chunk_size)
    assert length == len(rpos) and (kd[:, :, :length].float().cpu().numpy() == rk).all()
