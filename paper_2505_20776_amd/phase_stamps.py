"""Where the time of the row-split prefix kernel goes, from wall-clock stamps the kernel leaves per workgroup.

Needs the profiling build of the library and one MI355X:

    python -m paper_2505_20776_amd.build --stamps
    SPECEXT_LIBRARY=paper_2505_20776_amd/libspecext_stamps.so python -m paper_2505_20776_amd.phase_stamps [--prefix 16384] [--merge fused]

Runs the Llama-3.1-8B layer shape of the benchmark (60-node tree, 8 layers of distinct K/V so that every launch
streams from HBM), reads the stamps of the last launch of each pass and prints, in microseconds after the first
workgroup's start and averaged over the passes: workgroup start, first key tile ready, last key tile done, partial
stores issued (and, with --merge fused, the phases of the merge tail; otherwise those of the merge kernel: its data
arriving and its stores), the spread between XCDs and the time per key tile.  The stamps come from the GPU's 100 MHz wall clock: 10 ns resolution.
Last, per wave of the eight-wave workgroups, the key loop itself in cycles of the shader clock (s_memtime; its rate
against the wall clock is printed): waiting for the own loads, waiting at the barrier, the two halves of the wave's
loop order, and the tile period, averaged over the tiles 5..19 of all workgroups.  --num-splits forces the split
count (16 at a 64K prefix leaves half the compute units idle).
"""
import argparse
import ctypes

import numpy as np
import torch

import paper_2505_20776_amd as sx
from paper_2505_20776_amd import harness
from workloads import config_tree


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--prefix", type=int, default=16384)
    ap.add_argument("--merge", choices=["two-launch", "fused"], default="two-launch")
    ap.add_argument("--passes", type=int, default=6)
    ap.add_argument("--num-splits", type=int, default=0)
    a = ap.parse_args()
    lib = sx.load_library()
    if not hasattr(lib, "specext_debug_stamps_offset"):
        raise SystemExit("this library was built without -DSPECEXT_TAIL_STAMPS: see the module's docstring")
    lib.specext_debug_stamps_offset.restype = ctypes.c_size_t
    lib.specext_debug_stamps_offset.argtypes = [ctypes.POINTER(sx.specext_desc)]
    dev, Hq, Hkv, d, L, n_layers = "cuda", 32, 8, 128, a.prefix, 8
    parent_np = config_tree(4)
    T = len(parent_np)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1)
    rn = lambda *s: (torch.randn(*s, generator=gen, device=dev) * d ** -0.5).to(torch.bfloat16)
    q = [rn(T, Hq, d) for _ in range(n_layers)]
    kp, vp = [rn(Hkv, L, d) for _ in range(n_layers)], [rn(Hkv, L, d) for _ in range(n_layers)]
    kt, vt = [rn(Hkv, T, d) for _ in range(n_layers)], [rn(Hkv, T, d) for _ in range(n_layers)]
    parent = torch.from_numpy(parent_np).to(dev)
    fused = a.merge == "fused"
    buf = harness.make_buffers(dtype="bf16", n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, prefix_len=L, n_tree=T,
                               flags=sx.SPECEXT_FLAG_FUSED_MERGE if fused else 0, num_splits=a.num_splits)
    S = sx.num_splits(buf.desc)
    off = int(lib.specext_debug_stamps_offset(ctypes.byref(buf.desc)))
    assert off > 0
    n_st = 7 if fused else 4
    acc = []
    # the merge kernel of the two-launch form (four rows per workgroup) leaves its own stamps 2 MiB further on,
    # where the spare half of the partial region is large enough
    n_merge_wg = (Hq * T + 3) // 4
    merge_fits = S * Hq * T * d * 2 >= (2 << 20) + n_merge_wg * 64
    merge_acc = []
    # the per-wave loop stamps (eight-wave workgroups only) lie 4 MiB into the spare half, 80 words per wave
    n_rows = Hq // Hkv * T
    loop_fits = n_rows > 128 and S * Hq * T * d * 2 >= (4 << 20) + Hkv * S * 8 * 80 * 4
    loop_acc = []
    for it in range(a.passes + 2):
        for l in range(n_layers):
            sx.verify_attn(buf.desc, q[l], kp[l], vp[l], kt[l], vt[l], parent, buf.out, buf.lse, buf.workspace)
        torch.cuda.synchronize()
        st = buf.workspace[off:off + Hkv * S * 64].view(torch.int64).cpu().numpy().reshape(Hkv, S, 8).astype(np.float64)
        if it >= 2:
            acc.append((st[:, :, :n_st] - st[:, :, 0].min()) / 100.0)
            if loop_fits:
                lo = off + (4 << 20)
                loop_acc.append(buf.workspace[lo:lo + Hkv * S * 8 * 80 * 4].view(torch.int32).cpu().numpy()
                                .reshape(Hkv * S, 8, 80).astype(np.int64) & 0xffffffff)
            if not fused and merge_fits:
                ms = buf.workspace[off + (2 << 20):off + (2 << 20) + n_merge_wg * 64].view(torch.int64).cpu().numpy()
                ms = ms.reshape(n_merge_wg, 8)[:, :6].astype(np.float64)
                merge_acc.append(((ms - ms[:, 0].min()) / 100.0, (ms[:, 0].min() - st[:, :, 3].max()) / 100.0))
    us = np.mean(acc, axis=0)
    names = (["workgroup start", "last key tile done (tail entry)", "own partial acknowledged, flag stored", "tree part done",
              "all flags seen", "own slice merged and written", "done"] if fused else
             ["workgroup start", "first key tile ready", "last key tile done", "partial stores issued"])
    tiles = -(-(-(-L // S)) // 32)
    print(f"prefix {L}, {S} splits x {Hkv} KV heads = {S * Hkv} workgroups, {tiles} key tiles each, merge: {a.merge}")
    print(f"{'phase':42s} {'min':>8s} {'median':>8s} {'max':>8s}   (us after the first workgroup's start)")
    for i, n in enumerate(names):
        v = us[:, :, i]
        print(f"{n:42s} {v.min():8.2f} {np.median(v):8.2f} {v.max():8.2f}")
    last = 1 if fused else 2
    print("last key tile done, mean per KV head (one head per XCD):", " ".join(f"{us[h, :, last].mean():.2f}" for h in range(Hkv)))
    if not fused:
        print(f"key-tile loop: {np.median(us[:, :, 2] - us[:, :, 1]) / tiles:.3f} us per tile (median workgroup)")
    if loop_acc and tiles > 5:
        n_t = min(16, tiles - 4)            # stamped tiles: 4 .. 4 + n_t - 1
        ticks = np.median([(w[:, :, 65] - w[:, :, 64]) & 0xffffffff for w in loop_acc])
        wall = np.median([(w[:, :, 67] - w[:, :, 66]) & 0xffffffff for w in loop_acc])
        print(f"key loop per wave, cycles of the shader clock ({100.0 * ticks / wall:.0f} MHz by s_memtime against the wall clock), "
              f"mean over tiles 5..{3 + n_t} of all workgroups:")
        cols = ["own loads arrived", "barrier", "first half", "second half", "tile period"]
        table = np.zeros((len(loop_acc), 8, 5))
        for k, w in enumerate(loop_acc):
            x = w[:, :, :64].reshape(-1, 8, 16, 4)[:, :, :n_t, :]
            arrived, behind, half, end = x[..., 0], x[..., 1], x[..., 2], x[..., 3]
            parts = [(arrived[:, :, 1:] - end[:, :, :-1]), (behind - arrived)[:, :, 1:], (half - behind)[:, :, 1:],
                     (end - half)[:, :, 1:], (behind[:, :, 1:] - behind[:, :, :-1])]
            for c, part in enumerate(parts):
                table[k, :, c] = (part & 0xffffffff).astype(np.float64).mean(axis=(0, 2))
        table = table.mean(axis=0)
        print(f"{'wave':>4s} " + " ".join(f"{c:>18s}" for c in cols))
        for w in range(8):
            order = "second product, logits | softmax" if w < 4 else "softmax of the tile before | second product, logits"
            print(f"{w:4d} " + " ".join(f"{table[w, c]:18.0f}" for c in range(5)) + f"   ({order})")
    if merge_acc:
        mus = np.mean([a for a, _ in merge_acc], axis=0)
        gap = np.mean([b for _, b in merge_acc])
        print(f"merge kernel, {n_merge_wg} workgroups; its first workgroup starts {gap:.2f} us after the prefix kernel's last "
              "partial store was issued")
        print(f"{'phase':42s} {'min':>8s} {'median':>8s} {'max':>8s}   (us after the merge kernel's first workgroup's start)")
        for i, n in enumerate(["workgroup start", "parent array arrived", "first half of the partials, query arrived",
                               "tree K/V rows, other partials arrived", "outputs: stores issued",
                               "outputs: stores acknowledged"]):
            v = mus[:, i]
            print(f"{n:42s} {v.min():8.2f} {np.median(v):8.2f} {v.max():8.2f}")


if __name__ == "__main__":
    main()
