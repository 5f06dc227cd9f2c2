"""Device-buffer plumbing around the binding: allocate torch tensors for a
problem, call the C entry points, bring results back.  Marshalling only; every
step of the method runs in the HIP kernels."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

from . import binding as sx


def to_device(a: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    """fp32 numpy values (exactly representable in `dtype`) -> device tensor of that dtype."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def dtype_code(dtype: str) -> int:
    return {"f32": sx.SPECEXT_F32, "bf16": sx.SPECEXT_BF16}[dtype]


GUARD_BYTES = 4096          # sentinel bytes on each side of every buffer a kernel writes
GUARD_FILL = 0xA5


def guarded(shape, dtype: torch.dtype, device="cuda"):
    """A tensor of `shape` that sits between two sentinel regions of GUARD_BYTES bytes each.
    Returns (tensor, base); guards_intact(base) tells whether a kernel wrote outside the tensor."""
    n = 1
    for x in shape:
        n *= int(x)
    nbytes = n * torch.empty((), dtype=dtype).element_size()
    base = torch.full((nbytes + 2 * GUARD_BYTES,), GUARD_FILL, dtype=torch.uint8, device=device)
    return base[GUARD_BYTES:GUARD_BYTES + nbytes].view(dtype).view(*shape), base


def guards_intact(base: torch.Tensor) -> bool:
    return bool((base[:GUARD_BYTES] == GUARD_FILL).all()) and bool((base[-GUARD_BYTES:] == GUARD_FILL).all())


@dataclass
class VerifyBuffers:
    desc: sx.specext_desc
    out: torch.Tensor
    lse: torch.Tensor
    workspace: torch.Tensor
    scores: Optional[torch.Tensor]
    bases: dict

    def check_guards(self) -> None:
        """Raises if anything was written in front of or behind workspace, out, lse or scores."""
        for name, base in self.bases.items():
            assert guards_intact(base), f"a kernel wrote outside the {name} buffer"


def make_buffers(*, dtype: str, n_q_heads: int, n_kv_heads: int, head_dim: int, prefix_len: int, n_tree: int,
                 chunk_size: int = 0, want_scores: bool = False, num_splits: int = 0, out_dtype: Optional[str] = None,
                 softmax_scale: float = 0.0, flags: int = 0, device="cuda") -> VerifyBuffers:
    odt = out_dtype or dtype
    desc = sx.make_desc(dtype=dtype_code(dtype), out_dtype=dtype_code(odt), n_q_heads=n_q_heads,
                        n_kv_heads=n_kv_heads, head_dim=head_dim, prefix_len=prefix_len, n_tree=n_tree,
                        chunk_size=chunk_size, want_scores=want_scores, num_splits=num_splits,
                        softmax_scale=softmax_scale, flags=flags)
    nbytes = sx.workspace_bytes(desc)
    if nbytes == 0:
        raise ValueError("descriptor rejected by specext_workspace_bytes")
    bases = {}
    ws, bases["workspace"] = guarded((nbytes,), torch.uint8, device)
    sx.workspace_init(ws)
    out, bases["out"] = guarded((n_tree, n_q_heads, head_dim), torch.bfloat16 if odt == "bf16" else torch.float32, device)
    lse, bases["lse"] = guarded((n_q_heads, n_tree), torch.float32, device)
    scores = None
    if want_scores:
        n_chunks = (prefix_len + chunk_size - 1) // chunk_size
        scores, bases["scores"] = guarded((n_tree, max(n_chunks, 1)), torch.float32, device)
    return VerifyBuffers(desc, out, lse, ws, scores, bases)


def run_verify(wl, *, num_splits: int = 0, want_scores: bool = True, out_dtype: Optional[str] = None,
               flags: int = 0):
    """Run verify_attn (+ chunk_scores for every row) on a workloads.Workload.
    Returns dict of numpy arrays: out fp32 [T,Hq,d], lse [Hq,T], scores [T,C] or None, status int."""
    dev = "cuda"
    q = to_device(wl.q, wl.dtype, dev)
    kp = to_device(wl.k_prefix, wl.dtype, dev)
    vp = to_device(wl.v_prefix, wl.dtype, dev)
    kt = to_device(wl.k_tree, wl.dtype, dev)
    vt = to_device(wl.v_tree, wl.dtype, dev)
    parent = torch.from_numpy(np.asarray(wl.parent, dtype=np.int32)).to(dev)
    want_scores = want_scores and wl.prefix_len > 0
    buf = make_buffers(dtype=wl.dtype, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim,
                       prefix_len=wl.prefix_len, n_tree=wl.n_tree, chunk_size=wl.chunk_size,
                       want_scores=want_scores, num_splits=num_splits, out_dtype=out_dtype, flags=flags,
                       device=dev)
    sx.verify_attn(buf.desc, q, kp if wl.prefix_len else None, vp if wl.prefix_len else None, kt, vt, parent,
                   buf.out, buf.lse, buf.workspace)
    if want_scores:
        sx.chunk_scores(buf.desc, buf.workspace, -1, buf.scores)
    torch.cuda.synchronize()
    buf.check_guards()
    status = int(buf.workspace[:4].view(torch.int32).item())
    return {
        "out": buf.out.float().cpu().numpy(),
        "lse": buf.lse.cpu().numpy(),
        "scores": buf.scores.cpu().numpy() if want_scores else None,
        "status": status,
        "num_splits": sx.num_splits(buf.desc),
    }


def run_select(scores_row: np.ndarray, k: int):
    """select_chunks on one row of scores; returns (idx int32 [min(k,C)], n_out, raw idx buffer)."""
    s = torch.from_numpy(np.ascontiguousarray(scores_row, dtype=np.float32)).cuda()
    idx, idx_base = guarded((max(k, 1),), torch.int32)
    n_out, n_base = guarded((1,), torch.int32)
    idx.fill_(-7)
    n_out.fill_(-7)
    sx.select_chunks(s, s.numel(), k, idx, n_out)
    torch.cuda.synchronize()
    assert guards_intact(idx_base) and guards_intact(n_base), "select_chunks wrote outside idx_out / n_out"
    n = int(n_out.item())
    raw = idx.cpu().numpy()
    return raw[:n].copy(), n, raw[:k].copy()


def run_gather(k_src: torch.Tensor, v_src: torch.Tensor, idx: np.ndarray, chunk_size: int, *,
               n_idx: Optional[int] = None, max_idx: Optional[int] = None):
    """gather_draft_kv on [Ld,H,L,d] device tensors.  Returns (k_dst, v_dst, pos, length) with the
    destination sized max_idx * chunk_size tokens and pre-filled with a canary pattern."""
    ld, hh, plen, d = k_src.shape
    idx_t = torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int32)).cuda()
    max_idx = int(len(idx) if max_idx is None else max_idx)
    cap = max_idx * chunk_size
    k_dst, k_base = guarded((ld, hh, cap, d), k_src.dtype)
    v_dst, v_base = guarded((ld, hh, cap, d), k_src.dtype)
    k_dst.fill_(77)
    v_dst.fill_(77)
    pos, pos_base = guarded((max(cap, 1),), torch.int32)
    length, len_base = guarded((1,), torch.int32)
    pos.fill_(-5)
    length.fill_(-5)
    n_idx_t = None if n_idx is None else torch.tensor([n_idx], dtype=torch.int32, device="cuda")
    if idx_t.numel() == 0:
        idx_t = torch.zeros(1, dtype=torch.int32, device="cuda")
    sx.gather_draft_kv(k_src, v_src, k_dst, v_dst, idx_t, n_idx_t, max_idx, ld, hh, plen, cap, d, chunk_size,
                       k_src.element_size(), pos, length)
    torch.cuda.synchronize()
    for name, base in (("k_dst", k_base), ("v_dst", v_base), ("pos_out", pos_base), ("len_out", len_base)):
        assert guards_intact(base), f"gather_draft_kv wrote outside {name}"
    return k_dst, v_dst, pos.cpu().numpy()[:cap], int(length.item())


def run_accept(parent: np.ndarray, draft_token: np.ndarray, target_token: np.ndarray, first_target: int):
    """accept_greedy on host arrays; returns (path list, next token, raw path buffer, device tensors (path, n))."""
    dev = "cuda"
    t = len(parent)
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    path = torch.full((t,), -9, dtype=torch.int32, device=dev)
    n_acc = torch.full((1,), -9, dtype=torch.int32, device=dev)
    nxt = torch.full((1,), -9, dtype=torch.int32, device=dev)
    sx.accept_greedy(to(parent), to(draft_token), to(target_token), to(np.array([first_target])), t, path, n_acc, nxt)
    torch.cuda.synchronize()
    raw = path.cpu().numpy()
    n = int(n_acc.item())
    return [int(x) for x in raw[:n]], int(nxt.item()), raw, (path, n_acc)


def run_materialized(wl, *, out_dtype: Optional[str] = None, want_probs: bool = True):
    """attn_materialized (+ chunk_scores_materialized for every row) on a workloads.Workload.
    Returns dict of numpy arrays: out [T,Hq,d], lse [Hq,T], probs [Hq,T,L+T] (padding cut), scores [T,C] or None."""
    dev = "cuda"
    odt = out_dtype or wl.dtype
    want_scores = wl.prefix_len > 0
    desc = sx.make_desc(dtype=dtype_code(wl.dtype), out_dtype=dtype_code(odt), n_q_heads=wl.n_q_heads,
                        n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim, prefix_len=wl.prefix_len, n_tree=wl.n_tree,
                        chunk_size=wl.chunk_size if want_scores else 0, want_scores=want_scores)
    nbytes = sx.materialized_bytes(desc)
    if nbytes == 0:
        raise ValueError("descriptor rejected by specext_materialized_bytes")
    ld = sx.materialized_ld(desc)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    q, kt, vt = to_device(wl.q, wl.dtype, dev), to_device(wl.k_tree, wl.dtype, dev), to_device(wl.v_tree, wl.dtype, dev)
    kp = to_device(wl.k_prefix, wl.dtype, dev) if wl.prefix_len else None
    vp = to_device(wl.v_prefix, wl.dtype, dev) if wl.prefix_len else None
    parent = torch.from_numpy(np.asarray(wl.parent, dtype=np.int32)).to(dev)
    out = torch.empty((wl.n_tree, wl.n_q_heads, wl.head_dim), dtype=torch.bfloat16 if odt == "bf16" else torch.float32,
                      device=dev)
    lse = torch.empty((wl.n_q_heads, wl.n_tree), dtype=torch.float32, device=dev)
    sx.attn_materialized(desc, q, kp, vp, kt, vt, parent, out, lse, ws)
    scores = None
    if want_scores:
        n_chunks = (wl.prefix_len + wl.chunk_size - 1) // wl.chunk_size
        scores = torch.empty((wl.n_tree, n_chunks), dtype=torch.float32, device=dev)
        for row in range(wl.n_tree):
            sx.chunk_scores_materialized(desc, ws, row, scores[row])
    torch.cuda.synchronize()
    probs = None
    if want_probs:
        n = wl.prefix_len + wl.n_tree
        mat = ws[256:256 + wl.n_q_heads * wl.n_tree * ld * 4].view(torch.float32).view(wl.n_q_heads, wl.n_tree, ld)
        assert bool((mat[:, :, n:] == 0).all()), "padding columns must be zero"
        probs = mat[:, :, :n].cpu().numpy()
    return {"out": out.float().cpu().numpy(), "lse": lse.cpu().numpy(), "probs": probs,
            "scores": scores.cpu().numpy() if want_scores else None, "desc": desc, "workspace": ws}


def run_prefill(q: np.ndarray, k: np.ndarray, v: np.ndarray, *, out_dtype: str = "bf16", kv_capacity: int = 0):
    """prefill_attn on host arrays (values exactly representable in bf16): q [Tq,Hq,d], k/v [Hkv,N,d].
    kv_capacity > N places K/V in a capacity-sized cache.  Returns (out fp32 [Tq,Hq,d], lse [Hq,Tq])."""
    dev = "cuda"
    tq, hq, d = q.shape
    hkv, n, _ = k.shape
    cap = max(kv_capacity, n)
    kd = torch.zeros((hkv, cap, d), dtype=torch.bfloat16, device=dev)
    vd = torch.zeros_like(kd)
    kd[:, :n] = to_device(k, "bf16", dev)
    vd[:, :n] = to_device(v, "bf16", dev)
    out = torch.full((tq, hq, d), float("nan"), dtype=torch.bfloat16 if out_dtype == "bf16" else torch.float32,
                     device=dev)
    lse = torch.full((hq, tq), float("nan"), dtype=torch.float32, device=dev)
    sx.prefill_attn(to_device(q, "bf16", dev), kd, vd, out, lse, hq, hkv, d, tq, n, out_dtype=dtype_code(out_dtype),
                    kv_stride_h=cap * d if cap != n else 0)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), lse.cpu().numpy()
