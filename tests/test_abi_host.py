"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before launching."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sx():
    import paper_2505_20776_amd as sx
    if not os.path.exists(os.path.join(ROOT, "paper_2505_20776_amd", "libspecext.so")):
        from paper_2505_20776_amd.build import build_library
        build_library(verbose=False)
    sx.load_library()
    return sx


def _header_symbols():
    text = open(os.path.join(ROOT, "include", "specext.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(specext_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(sx):
    lib = sx.load_library()
    names = _header_symbols()
    assert set(names) == set(sx.binding.EXPORTED)
    for n in names:
        assert getattr(lib, n) is not None


def test_descriptor_layout_matches_header(sx):
    # 14 four-byte fields then 8 eight-byte strides, naturally aligned
    assert ctypes.sizeof(sx.specext_desc) == 14 * 4 + 8 * 8
    assert sx.specext_desc.q_stride_t.offset == 56


def _good(sx, **kw):
    base = dict(dtype=sx.SPECEXT_BF16, n_q_heads=32, n_kv_heads=8, head_dim=128, prefix_len=4096, n_tree=60,
                chunk_size=32, want_scores=True, num_splits=8)
    base.update(kw)
    return sx.make_desc(**base)


def test_workspace_and_splits(sx):
    d = _good(sx)
    assert sx.num_splits(d) == 8
    ws = sx.workspace_bytes(d)
    rows = 32 * 60
    assert ws >= 8 * rows * 128 * 4 + rows * 128 * 2 * 4
    assert ws % 256 == 0
    # splits never cut a chunk: keys per split is a multiple of lcm(64, B)
    d = _good(sx, prefix_len=1000, num_splits=7, chunk_size=48)
    assert 1 <= sx.num_splits(d) <= 7
    d = _good(sx, prefix_len=0)
    assert sx.num_splits(d) == 0 and sx.workspace_bytes(d) > 0
    d = _good(sx, prefix_len=300, num_splits=200, n_tree=8)
    assert sx.num_splits(d) == 3                        # matrix-core key-split kernel: 128-key granule
    d = _good(sx, prefix_len=300, num_splits=200)
    assert sx.num_splits(d) == 5                        # matrix-core row-split kernel: 64-key granule
    d = _good(sx, prefix_len=100, num_splits=200, flags=sx.SPECEXT_FLAG_VALU_PREFIX)
    assert sx.num_splits(d) == 2                        # vector-ALU kernel: 64-key granule


@pytest.mark.parametrize("field,value,status", [
    ("struct_size", 4, -1), ("n_q_heads", 0, -1), ("n_kv_heads", 5, -1), ("prefix_len", -1, -1),
    ("n_tree", 0, -1), ("chunk_size", 0, -1), ("num_splits", -2, -1), ("softmax_scale", -1.0, -1),
    ("dtype", 7, -2), ("head_dim", 96, -2), ("n_tree", 129, -2), ("num_splits", 257, -2),
    ("q_stride_h", 12, -2), ("kp_stride_l", 64, -1), ("reserved", 1, -1), ("flags", 16, -1),
])
def test_bad_descriptor_is_rejected(sx, field, value, status):
    d = _good(sx)
    setattr(d, field, value)
    assert sx.workspace_bytes(d) == 0
    assert sx.num_splits(d) == status
    rc = sx.verify_attn(d, 256, 256, 256, 256, 256, 256, 256, None, 256, workspace_nbytes=1 << 40, stream=0,
                        check=False)
    assert rc == status
    assert sx.chunk_scores(d, 256, -1, 256, workspace_nbytes=1 << 40, stream=0, check=False) == status


def test_bad_pointers_are_rejected_before_launch(sx):
    d = _good(sx)
    ws = sx.workspace_bytes(d)
    ok = 4096
    args = [ok] * 7
    for i in (0, 1, 2, 3, 4, 5, 6):                        # each required pointer null in turn
        a = list(args); a[i] = None
        assert sx.verify_attn(d, *a, None, ok, workspace_nbytes=ws, stream=0, check=False) == -1
    assert sx.verify_attn(d, *args, None, None, workspace_nbytes=ws, stream=0, check=False) == -1
    a = list(args); a[1] = ok + 8                          # misaligned k_prefix
    assert sx.verify_attn(d, *a, None, ok, workspace_nbytes=ws, stream=0, check=False) == -2
    assert sx.verify_attn(d, *args, None, ok + 64, workspace_nbytes=ws, stream=0, check=False) == -2
    assert sx.verify_attn(d, *args, None, ok, workspace_nbytes=ws - 1, stream=0, check=False) == -3
    with pytest.raises(sx.SpecextError):
        sx.verify_attn(d, *args, None, ok, workspace_nbytes=0, stream=0)
    # chunk_scores needs want_scores and a valid row
    assert sx.chunk_scores(d, ok, 60, ok, workspace_nbytes=ws, stream=0, check=False) == -1
    assert sx.chunk_scores(d, ok, -2, ok, workspace_nbytes=ws, stream=0, check=False) == -1
    assert sx.chunk_scores(d, None, 0, ok, workspace_nbytes=ws, stream=0, check=False) == -1
    assert sx.chunk_scores(d, ok, 0, ok, workspace_nbytes=16, stream=0, check=False) == -3
    d2 = _good(sx, want_scores=False)
    assert sx.chunk_scores(d2, ok, 0, ok, workspace_nbytes=ws, stream=0, check=False) == -1


def test_select_and_gather_argument_checks(sx):
    ok = 4096
    assert sx.select_chunks(None, 4, 2, ok, ok, stream=0, check=False) == -1
    assert sx.select_chunks(ok, 0, 2, ok, ok, stream=0, check=False) == -1
    assert sx.select_chunks(ok, 4, -1, ok, ok, stream=0, check=False) == -1
    assert sx.select_chunks(ok, 4, 2, None, ok, stream=0, check=False) == -1
    assert sx.select_chunks(ok, 4, 2, ok, None, stream=0, check=False) == -1
    assert sx.select_chunks(ok, 70000, 2, ok, ok, stream=0, check=False) == -2
    assert sx.select_chunks(ok + 2, 4, 2, ok, ok, stream=0, check=False) == -2
    g = dict(max_idx=4, n_layers=1, n_kv_heads=8, src_len=1024, dst_cap=128, head_dim=128, chunk_size=32,
             elem_bytes=2, stream=0, check=False)
    assert sx.gather_draft_kv(None, ok, ok, ok, ok, None, **g) == -1
    assert sx.gather_draft_kv(ok, ok, ok, ok, None, None, **g) == -1
    assert sx.gather_draft_kv(ok, ok, ok, ok, ok, None, **dict(g, dst_cap=127)) == -1
    assert sx.gather_draft_kv(ok, ok, ok, ok, ok, None, **dict(g, chunk_size=0)) == -1
    assert sx.gather_draft_kv(ok, ok, ok, ok, ok, None, **dict(g, src_cap=1023)) == -1   # capacity below the length
    assert sx.gather_draft_kv(ok, ok, ok, ok, ok, None, **dict(g, head_dim=100, elem_bytes=1)) == -2
    assert sx.gather_draft_kv(ok + 4, ok, ok, ok, ok, None, **g) == -2
    assert sx.gather_draft_kv(ok, ok, ok, ok, ok, None, **dict(g, n_layers=9000)) == -2


def test_accept_and_commit_argument_checks(sx):
    ok = 4096
    a = dict(stream=0, check=False)
    assert sx.accept_greedy(None, ok, ok, ok, 8, ok, ok, ok, **a) == -1
    assert sx.accept_greedy(ok, ok, ok, None, 8, ok, ok, ok, **a) == -1
    assert sx.accept_greedy(ok, ok, ok, ok, 0, ok, ok, ok, **a) == -1
    assert sx.accept_greedy(ok, ok, ok, ok, 129, ok, ok, ok, **a) == -2
    assert sx.accept_greedy(ok, ok + 2, ok, ok, 8, ok, ok, ok, **a) == -2
    c = dict(max_accept=8, n_tree=60, n_layers=32, n_kv_heads=8, head_dim=128, elem_bytes=2, prefix_len=1000, cache_capacity=1024,
             stream=0, check=False)
    assert sx.commit_tree_kv(None, ok, ok, ok, ok, ok, **c) == -1
    assert sx.commit_tree_kv(ok, ok, ok, ok, ok, None, **c) == -1
    assert sx.commit_tree_kv(ok, ok, ok, ok, ok, ok, **dict(c, prefix_len=1020)) == -1      # 1020 + 8 > capacity
    assert sx.commit_tree_kv(ok, ok, ok, ok, ok, ok, **dict(c, max_accept=-1)) == -1
    assert sx.commit_tree_kv(ok, ok, ok, ok, ok, ok, **dict(c, head_dim=100, elem_bytes=1)) == -2
    assert sx.commit_tree_kv(ok, ok, ok, ok, ok, ok, **dict(c, cache_stride_l=64)) == -2     # rows would overlap
    assert sx.commit_tree_kv(ok + 8, ok, ok, ok, ok, ok, **c) == -2
    d = _good(sx)
    ws = sx.workspace_bytes(d)
    assert sx.chunk_scores_accepted(d, ok, None, ok, ok, workspace_nbytes=ws, **a) == -1
    assert sx.chunk_scores_accepted(d, ok, ok, ok, ok, workspace_nbytes=ws - 1, **a) == -3
    assert sx.chunk_scores_accepted(_good(sx, want_scores=False), ok, ok, ok, ok, workspace_nbytes=ws, **a) == -1


def test_strerror(sx):
    assert sx.strerror(0) == "ok"
    assert "workspace" in sx.strerror(-3)
    assert sx.strerror(-99) == "unknown status"


def test_materialized_argument_checks(sx):
    d64 = sx.make_desc(dtype=sx.SPECEXT_BF16, n_q_heads=8, n_kv_heads=2, head_dim=64, prefix_len=100, n_tree=8)
    f32 = sx.make_desc(dtype=sx.SPECEXT_F32, n_q_heads=8, n_kv_heads=2, head_dim=128, prefix_len=100, n_tree=8)
    assert sx.materialized_bytes(d64) == 0 and sx.materialized_ld(d64) == -2
    assert sx.materialized_bytes(f32) == 0 and sx.materialized_ld(f32) == -2
    ok = sx.make_desc(dtype=sx.SPECEXT_BF16, n_q_heads=8, n_kv_heads=2, head_dim=128, prefix_len=100, n_tree=8,
                      chunk_size=32, want_scores=True)
    assert sx.materialized_ld(ok) == 128
    a = 4096
    assert sx.attn_materialized(ok, a, a, a, a, a, a, a, a, a, workspace_nbytes=16, stream=0, check=False) == -3
    nbytes = sx.materialized_bytes(ok)
    assert sx.chunk_scores_materialized(ok, a, 8, a, workspace_nbytes=nbytes, stream=0, check=False) == -1
    assert sx.chunk_scores_materialized(ok, a, 0, a, path=a, workspace_nbytes=nbytes, stream=0, check=False) == -1


def test_prefill_argument_checks(sx):
    a = 4096
    base = dict(n_q_heads=8, n_kv_heads=2, head_dim=128, q_len=64, kv_len=64, stream=0, check=False)
    assert sx.prefill_attn(None, a, a, a, None, **base) == -1
    assert sx.prefill_attn(a, a, a, a, None, **dict(base, q_len=65)) == -1           # more queries than keys
    assert sx.prefill_attn(a, a, a, a, None, **dict(base, n_kv_heads=3)) == -1
    assert sx.prefill_attn(a, a, a, a, None, **dict(base, head_dim=64)) == -2
    assert sx.prefill_attn(a, a, a, a, None, **dict(base, dtype=sx.SPECEXT_F32)) == -2
    assert sx.prefill_attn(a, a, a, a, None, **dict(base, q_len=8, kv_len=16)) == -2   # under one tile of keys
    assert sx.prefill_attn(a + 2, a, a, a, None, **base) == -2
    assert sx.prefill_attn(a, a, a, a, None, **dict(base, kv_stride_l=100)) == -2


def test_calibration_argument_checks(sx):
    """The measurement aids refuse bad arguments before anything is launched (no GPU is touched)."""
    lib = sx.load_library()
    mix = lambda mode, n, iters, wgs: lib.specext_calib_issue_mix(mode, n, iters, wgs, None, None)
    bad = [mix(0, 4, 10, 1), mix(5, 4, 10, 1), mix(1, 4, 0, 1), mix(1, 4, 10, 0)]
    assert all(rc < 0 for rc in bad) and len(set(bad)) == 1
    invalid = bad[0]
    unsupported = mix(1, 3, 10, 1)          # vector instructions per matrix one: 0, 4 or 8
    assert unsupported < 0 and unsupported != invalid
    assert mix(1, 4, (1 << 24) + 1, 1) == unsupported
    assert lib.specext_calib_mfma(0, 32, 1, None, None) == invalid
    assert lib.specext_calib_mfma(10, 24, 1, None, None) == invalid
    assert lib.specext_calib_stream_read(None, 32768, None, None) == invalid
