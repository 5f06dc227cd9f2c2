"""Shared comparison rules for the GPU parity tests (HIP path versus fp64 oracle)."""
import numpy as np

import oracle as orc

# max-abs error bars of the path: fp32 inputs, and bf16 inputs with fp32 accumulation
TOL = {"f32": 2e-3, "bf16": 2e-2}
# chunk scores: relative to the largest score of the row (fp32 sums of fp32 exponentials)
SCORE_EPS = 1e-4


def oracle_all(wl):
    out, lse, _ = orc.verify_attention(wl.q, wl.k_prefix, wl.v_prefix, wl.k_tree, wl.v_tree, wl.parent)
    scores = None
    if wl.prefix_len > 0:
        scores = orc.chunk_scores(wl.q, wl.k_prefix, wl.v_prefix, wl.k_tree, wl.v_tree, wl.parent, wl.chunk_size)
    return out, lse, scores


def check_attention(wl, res, ref_out, ref_lse, what=""):
    tol = TOL[wl.dtype]
    err = np.abs(res["out"].astype(np.float64) - ref_out)
    scale = np.abs(ref_out).max()
    assert np.isfinite(res["out"]).all(), f"{what}: non-finite output"
    assert err.max() <= tol, f"{what}: out max-abs err {err.max():.3e} > {tol}"
    # the literal workloads have |O| ~ 1e-3, so the absolute bar alone would accept zeros
    assert err.max() <= tol * max(scale, 1e-30), f"{what}: out err {err.max():.3e} relative to max|O|={scale:.3e} > {tol}"
    lerr = np.abs(res["lse"].astype(np.float64) - ref_lse).max()
    assert lerr <= 2e-3, f"{what}: lse err {lerr:.3e}"
    return err.max() / scale


def check_scores(res_scores, ref_scores, what=""):
    assert np.isfinite(res_scores).all(), f"{what}: non-finite scores"
    for r in range(ref_scores.shape[0]):
        eps = SCORE_EPS * ref_scores[r].max()
        e = np.abs(res_scores[r].astype(np.float64) - ref_scores[r]).max()
        assert e <= eps, f"{what}: row {r} score err {e:.3e} > {eps:.3e}"


def check_selection(gpu_idx, ref_scores_row, k, what=""):
    """Tolerance-aware top-k rule: every chunk clearly above the k-th score must be
    chosen, nothing clearly below it may be, output ascending and distinct; where
    the k-th / (k+1)-th margin is wide the set must equal the oracle's exactly."""
    ref_scores_row = np.asarray(ref_scores_row, dtype=np.float64)
    n = len(ref_scores_row)
    k_eff = min(k, n)
    gpu_idx = np.asarray(gpu_idx)
    assert gpu_idx.dtype == np.int32
    assert len(gpu_idx) == k_eff, f"{what}: {len(gpu_idx)} chunks, expected {k_eff}"
    assert (np.diff(gpu_idx) > 0).all(), f"{what}: not strictly ascending"
    if k_eff == 0:
        return True
    assert gpu_idx.min() >= 0 and gpu_idx.max() < n
    ref_idx = orc.select_chunks(ref_scores_row, k)
    srt = np.sort(ref_scores_row)[::-1]
    theta = srt[k_eff - 1]
    eps = SCORE_EPS * ref_scores_row.max()
    chosen = set(int(i) for i in gpu_idx)
    must = set(int(i) for i in np.nonzero(ref_scores_row > theta + eps)[0])
    assert must <= chosen, f"{what}: clear winners missing: {sorted(must - chosen)}"
    assert all(ref_scores_row[i] >= theta - eps for i in chosen), f"{what}: a clearly losing chunk was chosen"
    wide = k_eff == n or (theta - srt[k_eff]) > 2 * eps
    if wide:
        assert list(gpu_idx) == list(ref_idx), f"{what}: wide margin but sets differ"
    return list(gpu_idx) == list(ref_idx)
