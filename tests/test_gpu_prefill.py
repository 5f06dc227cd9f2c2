"""GPU parity of the prefill attention kernel (causal self-attention, Sec. 3.1) against the oracle's
definition: whole prompts and later pieces of a prompt, ragged sizes, group sizes, output types, and the
benchmark's 16K prompt on sampled rows."""
import numpy as np
import pytest
import torch

import oracle as orc
from workloads import quantize

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2        # max-abs, also relative to max|O| (bf16 inputs and probabilities, fp32 accumulation)
TOL_LSE = 2e-3


@pytest.fixture(scope="module")
def hx():
    from paper_2505_20776_amd import harness
    return harness


def _draw(seed, tq, n, hq, hkv, d=128, std=1.0):
    rng = np.random.default_rng(seed)
    mk = lambda *s: quantize((rng.standard_normal(s) * std).astype(np.float32), "bf16")
    return mk(tq, hq, d), mk(hkv, n, d), mk(hkv, n, d)


def _check(out, lse, ref_out, ref_lse, rows, what):
    assert np.isfinite(out).all() and np.isfinite(lse).all(), f"{what}: non-finite result"
    err = np.abs(out[rows] - ref_out[rows]).max()
    top = np.abs(ref_out[rows]).max()
    assert err <= TOL_BF16 and err <= TOL_BF16 * top, f"{what}: out err {err:.3e}, max|O| {top:.3e}"
    lerr = np.abs(lse[:, rows] - ref_lse[:, rows]).max()
    assert lerr <= TOL_LSE, f"{what}: lse err {lerr:.3e}"


CASES = [
    # q_len, kv_len, Hq, Hkv
    (64, 64, 8, 2),          # exactly one row group
    (32, 32, 8, 2),          # the smallest context
    (1, 32, 8, 2),           # one query
    (200, 200, 32, 8),       # ragged, several groups
    (257, 257, 8, 8),        # G = 1: 256 tokens per group and one over
    (100, 100, 16, 2),       # G = 8
    (40, 40, 64, 2),         # G = 32: 8 tokens per group, key ranges shorter than a tile
    (70, 300, 32, 8),        # a later piece of a prompt
    (5, 1000, 8, 2),         # a short piece behind a long context
    (513, 1029, 8, 2),       # ragged piece, ragged context
]


@pytest.mark.parametrize("tq,n,hq,hkv", CASES)
def test_against_oracle(hx, tq, n, hq, hkv):
    q, k, v = _draw(tq * 31 + n, tq, n, hq, hkv)
    print(f"[case] prefill q_len={tq} kv_len={n} Hq={hq} Hkv={hkv}", flush=True)
    ref_out, ref_lse = orc.prefill_attention(q, k, v)
    out, lse = hx.run_prefill(q, k, v)
    _check(out, lse, ref_out, ref_lse, slice(None), f"prefill {tq}/{n}")


def test_fp32_output_capacity_sized_cache_and_reproducibility(hx):
    q, k, v = _draw(99, 150, 333, 8, 2)
    ref_out, ref_lse = orc.prefill_attention(q, k, v)
    out, lse = hx.run_prefill(q, k, v, out_dtype="f32", kv_capacity=512)
    _check(out, lse, ref_out, ref_lse, slice(None), "fp32 out, capacity-sized cache")
    out_b, lse_b = hx.run_prefill(q, k, v, kv_capacity=512)
    assert np.abs(out_b - out).max() <= 2.0 ** -8 * np.abs(out).max()          # the same numbers rounded to bf16
    again, lse2 = hx.run_prefill(q, k, v, out_dtype="f32", kv_capacity=512)
    assert (again == out).all() and (lse2 == lse).all()


def test_equals_chain_tree_verification_on_gpu(hx):
    """A 64-token prompt both ways: as prefill, and as a chain tree behind an empty prefix."""
    from workloads import chain_tree, make_workload
    wl = make_workload("chain", seed=3, dtype="bf16", n_q_heads=8, n_kv_heads=2, head_dim=128, prefix_len=0,
                       parent=chain_tree(64), chunk_size=32, top_k=1, n_needles=0, value_std=1.0)
    res = hx.run_verify(wl, want_scores=False)
    out, lse = hx.run_prefill(wl.q, wl.k_tree, wl.v_tree)
    assert np.abs(out - res["out"]).max() <= TOL_BF16 * np.abs(res["out"]).max()
    assert np.abs(lse - res["lse"]).max() <= TOL_LSE


def test_full_size_prompt_sampled_rows(hx):
    """The benchmark's shape: a 16384-token prompt, 32 query heads over 8 KV heads; rows sampled where the
    tiling has its edges (group and tile boundaries, first and last rows) and at random."""
    tq = n = 16384
    q, k, v = _draw(16384, tq, n, 32, 8)
    rng = np.random.default_rng(1)
    rows = sorted(set([0, 1, 31, 32, 33, 63, 64, 65, 127, 128, 255, 256, 4095, 4096, 8191, 16320, 16383] +
                      [int(x) for x in rng.integers(0, tq, size=24)]))
    print(f"[case] prefill full size, {len(rows)} sampled rows", flush=True)
    ref_out, ref_lse = orc.prefill_attention(q, k, v, rows=rows)
    out, lse = hx.run_prefill(q, k, v)
    _check(out, lse, ref_out, ref_lse, rows, "prefill 16K")
    # properties that hold for every row: finite, and inside the hull of V's range per column block
    assert np.isfinite(out).all()
    assert np.abs(out).max() <= np.abs(v).max() * (1 + 2.0 ** -7)


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes(hx, seed):
    rng = np.random.default_rng(91000 + seed)
    hkv = int(rng.choice([1, 2, 4, 8]))
    g = int(rng.choice([1, 2, 3, 4, 8, 16]))
    n = int(rng.choice([32, 33, 63, 64, 65, 96, 127, 128, 129, 255, 300, 517, 700]))
    tq = n if rng.random() < 0.5 else int(rng.integers(1, n + 1))
    q, k, v = _draw(91000 + seed, tq, n, hkv * g, hkv)
    print(f"[case] prefill random {seed}: q_len={tq} kv_len={n} Hq={hkv * g} Hkv={hkv}", flush=True)
    ref_out, ref_lse = orc.prefill_attention(q, k, v)
    out, lse = hx.run_prefill(q, k, v, out_dtype="f32" if seed % 3 == 0 else "bf16",
                              kv_capacity=n + int(rng.integers(0, 3)) * 8)
    _check(out, lse, ref_out, ref_lse, slice(None), f"prefill random {seed}")
