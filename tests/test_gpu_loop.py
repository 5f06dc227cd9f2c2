"""Several decoding iterations in a row on the GPU against the oracle: verify attention on every layer over a
growing, ragged prefix -> greedy acceptance -> commit of the accepted K/V rows -> every few iterations (the
retrieval cadence of App. C / Table 8) chunk scores of the last accepted token, top-k selection and the draft-cache
gather.  State carried from one iteration to the next (cache contents, prefix length) must stay identical on
both sides, so a mistake in any one step shows up in all later ones."""
import numpy as np
import pytest
import torch

import oracle as orc
from parity_util import TOL, check_scores, check_selection
from workloads import eagle_style_tree, quantize

pytestmark = pytest.mark.gpu


def _tokens(parent, rng, vocab, follow):
    T = len(parent)
    draft = rng.integers(0, vocab, size=T)
    target = rng.integers(0, vocab, size=T)
    for i in range(T):
        kids = [j for j in range(T) if parent[j] == i]
        if kids and rng.random() < follow:
            target[i] = draft[kids[int(rng.integers(len(kids)))]]
    roots = [j for j in range(T) if parent[j] < 0]
    first = int(draft[roots[int(rng.integers(len(roots)))]]) if rng.random() < follow else int(rng.integers(vocab))
    return draft.astype(np.int32), target.astype(np.int32), first


@pytest.mark.parametrize("cadence,start_len", [(2, 1000), (4, 2049)])
def test_decoding_iterations(cadence, start_len):
    import paper_2505_20776_amd as sx
    from paper_2505_20776_amd import harness as hx

    dev = "cuda"
    layers, Hq, Hkv, d, T, B, topk, iters = 2, 8, 2, 128, 26, 32, 8, 8
    cap = start_len + iters * T
    rng = np.random.default_rng(9000 + cadence)
    std = 1.0 / np.sqrt(d)
    normal = lambda *s: quantize((rng.standard_normal(s) * std).astype(np.float32), "bf16")
    sharp = lambda *s: quantize((rng.standard_normal(s) * 3.0 * std ** 0.5).astype(np.float32), "bf16")

    # host (oracle) state: target caches per layer, one draft-model layer of the same length
    k_cache = [np.zeros((Hkv, cap, d), np.float32) for _ in range(layers)]
    v_cache = [np.zeros((Hkv, cap, d), np.float32) for _ in range(layers)]
    for y in range(layers):
        k_cache[y][:, :start_len] = sharp(Hkv, start_len, d)
        v_cache[y][:, :start_len] = normal(Hkv, start_len, d)
    dk_full = np.zeros((1, Hkv, cap, d), np.float32)
    dv_full = np.zeros((1, Hkv, cap, d), np.float32)
    dk_full[:, :, :start_len] = normal(1, Hkv, start_len, d)
    dv_full[:, :, :start_len] = normal(1, Hkv, start_len, d)

    # device state
    to_bf = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(torch.bfloat16)
    kc_dev = to_bf(np.stack(k_cache))                       # [layers, Hkv, cap, d]
    vc_dev = to_bf(np.stack(v_cache))
    dk_dev, dv_dev = to_bf(dk_full), to_bf(dv_full)
    work_cap = topk * B
    wk_dev = torch.zeros((1, Hkv, work_cap, d), dtype=torch.bfloat16, device=dev)
    wv_dev = torch.zeros_like(wk_dev)
    pos_dev = torch.empty(work_cap, dtype=torch.int32, device=dev)
    len_dev = torch.empty(1, dtype=torch.int32, device=dev)
    path_dev = torch.empty(T, dtype=torch.int32, device=dev)
    nacc_dev = torch.empty(1, dtype=torch.int32, device=dev)
    next_dev = torch.empty(1, dtype=torch.int32, device=dev)
    idx_dev = torch.empty(topk, dtype=torch.int32, device=dev)
    nout_dev = torch.empty(1, dtype=torch.int32, device=dev)
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)

    L = start_len
    retrievals = 0
    total_accepted = 0
    for it in range(iters):
        parent = np.asarray(eagle_style_tree(T, 6, rng)[:T], dtype=np.int32)
        draft, target, first = _tokens(parent, rng, vocab=3, follow=0.9)
        q = [sharp(T, Hq, d) for _ in range(layers)]
        kt = [sharp(Hkv, T, d) for _ in range(layers)]
        vt = [normal(Hkv, T, d) for _ in range(layers)]
        dkt, dvt = normal(1, Hkv, T, d), normal(1, Hkv, T, d)
        print(f"[case] loop cadence={cadence} iteration={it} prefix={L}", flush=True)

        # ---- device: one iteration ----
        kt_dev, vt_dev = to_bf(np.stack(kt)), to_bf(np.stack(vt))
        dkt_dev, dvt_dev = to_bf(dkt), to_bf(dvt)
        parent_dev = i32(parent)
        outs = []
        for y in range(layers):
            last = y == layers - 1
            buf = hx.make_buffers(dtype="bf16", n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, prefix_len=L, n_tree=T,
                                  chunk_size=B if last else 0, want_scores=last)
            buf.desc.kp_stride_h = cap * d
            buf.desc.kp_stride_l = d
            sx.verify_attn(buf.desc, to_bf(q[y]), kc_dev[y], vc_dev[y], kt_dev[y], vt_dev[y], parent_dev, buf.out,
                           buf.lse, buf.workspace)
            outs.append(buf)
        sx.accept_greedy(parent_dev, i32(draft), i32(target), i32([first]), T, path_dev, nacc_dev, next_dev)
        retrieve = (it + 1) % cadence == 0
        n_chunks = (L + B - 1) // B
        if retrieve:
            scores_dev = torch.empty(n_chunks, dtype=torch.float32, device=dev)
            sx.chunk_scores_accepted(outs[-1].desc, outs[-1].workspace, path_dev, nacc_dev, scores_dev)
            sx.select_chunks(scores_dev, n_chunks, topk, idx_dev, nout_dev)
            sx.gather_draft_kv(dk_dev, dv_dev, wk_dev, wv_dev, idx_dev, nout_dev, topk, 1, Hkv, L, work_cap, d, B, 2,
                               pos_dev, len_dev, src_cap=cap)
        sx.commit_tree_kv(kt_dev, vt_dev, kc_dev, vc_dev, path_dev, nacc_dev, T, T, layers, Hkv, d, 2, L, cap)
        sx.commit_tree_kv(dkt_dev, dvt_dev, dk_dev, dv_dev, path_dev, nacc_dev, T, T, 1, Hkv, d, 2, L, cap)
        torch.cuda.synchronize()
        n_acc = int(nacc_dev.item())                          # the host learns the new length here

        # ---- oracle: the same iteration ----
        ref_path, ref_next = orc.accept_greedy(parent, draft, target, first)
        assert [int(x) for x in path_dev.cpu().numpy()[:n_acc]] == ref_path and int(next_dev.item()) == ref_next
        for y in range(layers):
            ref_out, ref_lse, _ = orc.verify_attention(q[y], k_cache[y][:, :L], v_cache[y][:, :L], kt[y], vt[y], parent)
            got = outs[y].out.float().cpu().numpy()
            err = np.abs(got - ref_out).max()
            assert err <= TOL["bf16"] and err <= TOL["bf16"] * np.abs(ref_out).max(), \
                f"iteration {it} layer {y}: out err {err:.3e} (max|O| {np.abs(ref_out).max():.3e})"
            assert np.abs(outs[y].lse.cpu().numpy() - ref_lse).max() <= 2e-3
        if retrieve:
            y = layers - 1
            ref_scores = orc.chunk_scores(q[y], k_cache[y][:, :L], v_cache[y][:, :L], kt[y], vt[y], parent, B)
            row = ref_path[-1] if ref_path else 0
            got_scores = scores_dev.cpu().numpy()
            check_scores(got_scores[None], ref_scores[row][None], f"iteration {it} scores")
            n_sel = int(nout_dev.item())
            got_idx = idx_dev.cpu().numpy()[:n_sel]
            check_selection(got_idx, ref_scores[row], topk, f"iteration {it} selection")
            # the decision itself, taken in the kernel's precision: exact
            assert list(got_idx) == list(orc.select_chunks(got_scores, topk))
            ref_wk, ref_wv, ref_pos = orc.gather_draft_kv(dk_full[:, :, :L], dv_full[:, :, :L], got_idx, B)
            n_tok = int(len_dev.item())
            assert n_tok == ref_wk.shape[2]
            assert (wk_dev[:, :, :n_tok].float().cpu().numpy() == ref_wk).all()
            assert (wv_dev[:, :, :n_tok].float().cpu().numpy() == ref_wv).all()
            assert (pos_dev.cpu().numpy()[:n_tok] == ref_pos).all()
            retrievals += 1
        new_len = L
        for y in range(layers):
            k_cache[y], v_cache[y], new_len = orc.commit_tree_kv(k_cache[y], v_cache[y], kt[y], vt[y], ref_path, L)
        dk_full[0], dv_full[0], _ = orc.commit_tree_kv(dk_full[0], dv_full[0], dkt[0], dvt[0], ref_path, L)
        assert (kc_dev.float().cpu().numpy() == np.stack(k_cache)).all()
        assert (vc_dev.float().cpu().numpy() == np.stack(v_cache)).all()
        assert (dk_dev.float().cpu().numpy() == dk_full).all() and (dv_dev.float().cpu().numpy() == dv_full).all()
        total_accepted += len(ref_path)
        L = new_len
    assert retrievals == iters // cadence
    assert total_accepted >= iters                           # the token recipe gives real accepted paths
    assert L == start_len + total_accepted
