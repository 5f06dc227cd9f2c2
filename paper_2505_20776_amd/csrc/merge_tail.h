// Tree pass and log-sum-exp merge of Hybrid Tree Attention (SpecExtend Sec. 3.1) as the
// tail of the row-split prefix kernel: no second launch, no launch boundary per layer.
//
// The S workgroups that split the prefix of one (KV head, row group) each leave a
// partial (reference, row sum, unnormalised O as fp16) per row in the workspace.  The
// rows of the group are cut into at most S slices of R consecutive rows and workgroup s
// owns slice s: it computes the tree part of its rows (ancestor walk through parent[],
// online softmax), then folds the S partials of its rows and the tree part together and
// writes out and lse.
//
// A dependent trip to memory costs more than a microsecond while the other workgroups
// still stream K/V, so the protocol is built to put as few of them as possible between
// the last workgroup's last tile and the end of the kernel:
//   1. a workgroup writes its partial with device-scope stores (they pass the per-XCD
//      L2), waits until they are acknowledged and then stores flags[split] = epoch + 1
//      (epoch was read when the kernel started; nothing is reset between calls);
//   2. it polls the S flags (one load instruction) until all carry epoch + 1, at most
//      p.spin_limit times, then reads the partials of its slice at device scope;
//   3. a workgroup that runs out of polls sets its bit in `abandon` and leaves its slice
//      behind.  So no workgroup ever waits without bound for one that may not be running;
//   4. every workgroup ends with done += 1.  The one that brings it to S knows that all
//      partials are in memory and that nobody will touch the block again: it merges the
//      abandoned slices, clears done / abandon and raises epoch for the next call.
// The result is complete whatever the scheduling.  Sums are fp32 in a fixed order that
// depends only on the shape (never on which workgroup ran a slice or when): results are
// bit-reproducible from run to run.
#pragma once

#include "mfma_util.h"

namespace specext {

// Build with -DSPECEXT_TAIL_STAMPS to have every workgroup leave wall-clock stamps (100 MHz
// counter) of the tail's phases in the unused upper half of the partial-output region
// (sized for fp32, holding fp16): a profiling aid, off in the shipped library.
#ifdef SPECEXT_TAIL_STAMPS
#define SPECEXT_STAMP(i) do { if (threadIdx.x == 0) stamps[i] = wall_clock64(); } while (0)
#else
#define SPECEXT_STAMP(i) do { } while (0)
#endif

__device__ __forceinline__ float lane_value(float v, int src_lane) {
  return __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane << 2, __float_as_int(v)));
}

__device__ __forceinline__ void unpack_bf16x8(const uintx4 w, float (&v)[8]) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const uint32_t word = w[e];
    v[2 * e] = __uint_as_float(word << 16);
    v[2 * e + 1] = __uint_as_float(word & 0xffff0000u);
  }
}

// workgroup barrier that waits for this wave's LDS traffic only (not for loads, stores or
// atomics still on their way to memory, which __syncthreads would drain)
__device__ __forceinline__ void tail_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

constexpr int kTailSlot = 132;          // floats per LDS slot: 128 columns, reference, row sum, padding
// LDS the tail owns for the whole kernel (behind the rings and the waves' private areas):
// parent[] (filled in the kernel's prologue), a few control words, one tree slot per group
constexpr int kTailCtlOff = SPECEXT_MAX_TREE * 4;
constexpr int kTailTreeOff = kTailCtlOff + 64;
constexpr int tail_private_bytes(int threads) { return kTailTreeOff + (threads / 16) * kTailSlot * 4; }

// What a group of 16 lanes has requested for the tree part of its row: the query row and
// the K/V rows of the node and up to seven ancestors.
struct TreeLoads {
  int t, h, next;          // node, query head, first ancestor not yet requested (-1: none left)
  int anc[8];
  uintx4 q, k[8], v[8];
};

// NT threads per workgroup; bf16 inputs, head_dim 128, fp16 partials (what the row-split
// kernel writes).  `lds` is the workgroup's dynamic LDS area, whose first bytes (the K/V
// rings) are free for reuse once every wave has passed the tail's first barrier; `priv` is
// the tail's own area: parent[] is there since the prologue and the control words are zero.  epoch and
// cookie_ok were read when the kernel started.
template <int NT>
__device__ __forceinline__ void tree_merge_tail(const AttnParams& p, unsigned char* lds, unsigned char* priv,
                                                int split, int g, int z, int rows_per_wg, uint32_t epoch,
                                                bool cookie_ok) {
  constexpr int K = NT / 16;            // groups of 16 lanes; a group works on one row at a time
  constexpr int kSlot = kTailSlot;
  constexpr int kD = 128;
  int* parent_lds = reinterpret_cast<int*>(priv);                        // [SPECEXT_MAX_TREE]
  int* ctl = reinterpret_cast<int*>(priv + kTailCtlOff);                 // [16]
  float* tree_slot = reinterpret_cast<float*>(priv + kTailTreeOff);      // [K][kSlot]
  float* part_slot = reinterpret_cast<float*>(lds);                      // [K][kSlot], in the ring area

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int li = lane & 15;
  const int grp0 = lane & 48;
  const int k = tid >> 4;
  const int n_rows = p.Hq * p.T;
  SyncBlock* sb = p.sync + (z * p.Hkv + g);
#ifdef SPECEXT_TAIL_STAMPS
  unsigned long long* stamps = reinterpret_cast<unsigned long long*>(
      reinterpret_cast<unsigned char*>(p.part_o) + static_cast<size_t>(p.S) * n_rows * kD * 2) +
      ((z * p.Hkv + g) * p.S + split) * 8;
#endif
  SPECEXT_STAMP(1);

  // an uninitialised workspace has no valid hand-over block: report it and touch nothing
  if (!cookie_ok) {
    if (split == 0 && g == 0 && z == 0 && tid == 0) *p.status = 2;
    return;
  }
  const uint32_t tag = epoch + 1;

  const int row_base = z * rows_per_wg;                        // first row (of the KV head) of this row group
  const int rows_here = min(rows_per_wg, p.M - row_base);
  const int R = (rows_here + p.S - 1) / p.S;                   // rows per slice
  const int n_slices = (rows_here + R - 1) / R;                // <= S
  const int Rb = min(R, K);                                    // rows per pass over a slice
  const int P = max(1, min(K / Rb, p.S));                      // groups that share the splits of one row
  const int r_in = k % Rb;                                     // this group's row within a pass
  const int j_sub = k / Rb;                                    // which share of the splits it folds (< P, else idle)
  const uint16_t* part_h = reinterpret_cast<const uint16_t*>(p.part_o);
  const float inv_g = 1.0f / static_cast<float>(p.G);

  // row m of KV head g -> tree node
  auto node_of = [&](int m) { return static_cast<int>((static_cast<float>(m) + 0.5f) * inv_g); };

  // walk up to eight ancestors (node first) and request their K/V rows; a malformed
  // parent entry ends the walk (the node then counts as a root)
  auto request_batch = [&](TreeLoads& tl) {
    int a = tl.next;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      tl.anc[u] = a;
      if (a >= 0) {
        const int par = parent_lds[a];
        a = (par >= a || par < -1) ? -1 : par;
      }
    }
    tl.next = a;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (__any(tl.anc[u] >= 0)) {
        const int64_t off = g * p.kt_sh + max(tl.anc[u], 0) * p.kt_st + li * 8;
        tl.k[u] = *reinterpret_cast<const uintx4*>(static_cast<const uint16_t*>(p.kt) + off);
        tl.v[u] = *reinterpret_cast<const uintx4*>(static_cast<const uint16_t*>(p.vt) + off);
      }
    }
  };
  auto tree_request = [&](int m, TreeLoads& tl) {
    tl.t = node_of(m);
    tl.h = g * p.G + (m - tl.t * p.G);
    tl.q = *reinterpret_cast<const uintx4*>(static_cast<const uint16_t*>(p.q) + tl.t * p.q_st + tl.h * p.q_sh + li * 8);
    tl.next = tl.t;
    request_batch(tl);
  };

  // ---- tree part of a row from what tree_request brought (further batches of eight
  // ancestors are requested here): softmax over the node and its ancestors, left in
  // `slot` as (O, reference, sum)
  auto tree_finish = [&](TreeLoads& tl, float* slot) {
    float q[8], o[8];
    unpack_bf16x8(tl.q, q);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      q[e] *= p.scale_log2;
      o[e] = 0.f;
    }
    float run_max = -INFINITY, run_sum = 0.f;
    while (true) {
      float sc[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        sc[u] = -INFINITY;
        if (__any(tl.anc[u] >= 0)) {
          float kk[8];
          unpack_bf16x8(tl.k[u], kk);
          float dot = 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e) dot = fmaf(q[e], kk[e], dot);
          dot = row16_sum(dot);
          if (tl.anc[u] >= 0) sc[u] = dot;
        }
      }
      const float bm = fmaxf(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3])), fmaxf(fmaxf(sc[4], sc[5]), fmaxf(sc[6], sc[7])));
      const float new_max = fmaxf(run_max, bm);
      // a group whose chain ended in an earlier batch sees only -inf here and keeps what it has
      const float alpha = new_max > -INFINITY ? fast_exp2(run_max - new_max) : 1.f;
      run_max = new_max;
      run_sum *= alpha;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] *= alpha;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (__any(tl.anc[u] >= 0)) {
          const float pr = tl.anc[u] >= 0 ? fast_exp2(sc[u] - new_max) : 0.f;
          float vv[8];
          unpack_bf16x8(tl.v[u], vv);
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = fmaf(pr, vv[e], o[e]);
          run_sum += pr;
        }
      }
      if (!__any(tl.next >= 0)) break;
      request_batch(tl);
    }
    *reinterpret_cast<floatx4*>(slot + li * 8) = floatx4{o[0], o[1], o[2], o[3]};
    *reinterpret_cast<floatx4*>(slot + li * 8 + 4) = floatx4{o[4], o[5], o[6], o[7]};
    if (li == 0) *reinterpret_cast<floatx2*>(slot + kD) = floatx2{run_max, run_sum};
  };

  // ---- this group's share of the prefix splits of global row rid (splits j_sub, j_sub + P, ...),
  // 16 per round: lane i of the group holds (reference, sum) of the round's i-th split and
  // its weight; the partial outputs are added in split order with the weights fetched
  // from their lanes
  auto merge_partial = [&](int rid, float* slot) {
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.f;
    float run_max = -INFINITY, run_sum = 0.f;
    for (int s0 = j_sub; __any(s0 < p.S); s0 += 16 * P) {
      const int s_mine = s0 + li * P;
      floatx2 ml = {-INFINITY, 0.f};
      if (s_mine < p.S) {
        ml = load_device_scope_8(p.part_ml + (static_cast<int64_t>(s_mine) * n_rows + rid) * 2);
        if (!(ml[1] > 0.f)) ml = floatx2{-INFINITY, 0.f};       // an empty split contributes nothing
      }
      float w = 0.f;
      bool weighted = false;
#pragma unroll
      for (int u0 = 0; u0 < 16; u0 += 8) {
        if (!__any(s0 + u0 * P < p.S)) break;
        uintx4 raw[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int s = min(s0 + (u0 + u) * P, p.S - 1);         // splits past the end re-read the last one, weight 0
          raw[u] = load_device_scope_16(part_h + (static_cast<int64_t>(s) * n_rows + rid) * kD + li * 8);
        }
        if (!weighted) {
          weighted = true;
          const float new_max = fmaxf(run_max, row16_max(ml[0]));
          const float alpha = new_max > -INFINITY ? fast_exp2(run_max - new_max) : 1.f;
          w = ml[1] > 0.f ? fast_exp2(ml[0] - new_max) : 0.f;
          run_max = new_max;
          run_sum = fmaf(run_sum, alpha, row16_sum(ml[1] * w));
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] *= alpha;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const float wu = lane_value(w, grp0 + u0 + u);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            // through a scalar: this compiler takes element 0 when a vector element is bit-cast directly
            const uint32_t word = raw[u][e];
            const halfx2 hh = __builtin_bit_cast(halfx2, word);
            o[2 * e] = fmaf(static_cast<float>(hh[0]), wu, o[2 * e]);
            o[2 * e + 1] = fmaf(static_cast<float>(hh[1]), wu, o[2 * e + 1]);
          }
        }
      }
    }
    *reinterpret_cast<floatx4*>(slot + li * 8) = floatx4{o[0], o[1], o[2], o[3]};
    *reinterpret_cast<floatx4*>(slot + li * 8 + 4) = floatx4{o[4], o[5], o[6], o[7]};
    if (li == 0) *reinterpret_cast<floatx2*>(slot + kD) = floatx2{run_max, run_sum};
  };

  // ---- row m: tree part + the P shares of the prefix part -> out, lse
  auto finalize = [&](int m) {
    const float* ts = tree_slot + r_in * kSlot;
    float mx = ts[kD];
    for (int j = 0; j < P; ++j) mx = fmaxf(mx, part_slot[(j * Rb + r_in) * kSlot + kD]);
    const float wt = fast_exp2(ts[kD] - mx);
    float total = ts[kD + 1] * wt;
    float o[8];
    {
      const floatx4 a = *reinterpret_cast<const floatx4*>(ts + li * 8), b = *reinterpret_cast<const floatx4*>(ts + li * 8 + 4);
      o[0] = a[0] * wt; o[1] = a[1] * wt; o[2] = a[2] * wt; o[3] = a[3] * wt;
      o[4] = b[0] * wt; o[5] = b[1] * wt; o[6] = b[2] * wt; o[7] = b[3] * wt;
    }
    for (int j = 0; j < P; ++j) {
      const float* ps = part_slot + (j * Rb + r_in) * kSlot;
      const float wj = ps[kD + 1] > 0.f ? fast_exp2(ps[kD] - mx) : 0.f;
      total = fmaf(ps[kD + 1], wj, total);
      const floatx4 a = *reinterpret_cast<const floatx4*>(ps + li * 8), b = *reinterpret_cast<const floatx4*>(ps + li * 8 + 4);
      o[0] = fmaf(a[0], wj, o[0]); o[1] = fmaf(a[1], wj, o[1]); o[2] = fmaf(a[2], wj, o[2]); o[3] = fmaf(a[3], wj, o[3]);
      o[4] = fmaf(b[0], wj, o[4]); o[5] = fmaf(b[1], wj, o[5]); o[6] = fmaf(b[2], wj, o[6]); o[7] = fmaf(b[3], wj, o[7]);
    }
    const float inv = 1.f / total;
    const int t = node_of(m);
    const int h = g * p.G + (m - t * p.G);
    const int64_t ooff = t * p.o_st + h * p.o_sh + li * 8;
    if (p.out_dtype == SPECEXT_BF16) {
      uintx4 w;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        w[e] = static_cast<uint32_t>(float_to_bf16_bits(o[2 * e] * inv)) |
               (static_cast<uint32_t>(float_to_bf16_bits(o[2 * e + 1] * inv)) << 16);
      *reinterpret_cast<uintx4*>(static_cast<uint16_t*>(p.out) + ooff) = w;
    } else {
      floatx4* of = reinterpret_cast<floatx4*>(static_cast<float*>(p.out) + ooff);
      of[0] = floatx4{o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv};
      of[1] = floatx4{o[4] * inv, o[5] * inv, o[6] * inv, o[7] * inv};
    }
    if (li == 0) {
      const float l2 = mx + log2f(total);
      p.lse2[g * p.M + m] = l2;
      if (p.lse) p.lse[h * p.T + t] = l2 * kLn2;
    }
  };

  // ---- one slice, Rb rows per pass; tree_ready: the tree parts of its first pass are in LDS already
  auto do_slice = [&](int s, bool tree_ready) {
    const int lo = row_base + s * R;
    const int n = min(R, rows_here - s * R);
    for (int r0 = 0; r0 < n; r0 += Rb) {
      const bool row_ok = r0 + r_in < n;
      const int m = lo + min(r0 + r_in, n - 1);          // groups past the slice's end repeat its last row and store nothing
      // a group that also has the tree part of a row requests that first and finishes it
      // after its share of the partials, so that all its loads are in flight together
      const bool tree_here = !(tree_ready && r0 == 0) && k < Rb;
      TreeLoads tl;
      if (tree_here) tree_request(m, tl);
      if (j_sub < P) merge_partial(g * p.M + m, part_slot + k * kSlot);
      if (tree_here) tree_finish(tl, tree_slot + k * kSlot);
      tail_barrier();
      if (k < Rb && row_ok) finalize(m);
      tail_barrier();
    }
  };

  // ---- 1. the partial stores of this wave are on their way; request what the tree part
  // of the own slice's first pass needs, then wait for both
  const bool owner = split < n_slices;
  TreeLoads own;
  if (owner && k < Rb) {
    const int n = min(R, rows_here - split * R);
    tree_request(row_base + split * R + min(r_in, n - 1), own);
  }
  if (tid < p.T) {
    const int par = parent_lds[tid];
    if (par >= tid || par < -1) ctl[3] = 1;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  tail_barrier();                          // every wave's partial is acknowledged and it has left the K/V rings
  if (tid == 0) __hip_atomic_store(&sb->flags[split], tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (split == 0 && g == 0 && z == 0 && tid == 0) *p.status = ctl[3] ? 1 : 0;
  SPECEXT_STAMP(2);
  if (owner && k < Rb) tree_finish(own, tree_slot + k * kSlot);
  SPECEXT_STAMP(3);

  // ---- 2. wave 0 polls the flags of all splits, lane s the flag of split s
  if (tid < 64) {
    int ok = owner ? 0 : 1;                // a workgroup without a slice has nothing to wait for
    for (int it = 0; !ok && it <= p.spin_limit; ++it) {
      const uint32_t f = lane < p.S ? __hip_atomic_load(&sb->flags[lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : tag;
      ok = __all(f == tag) ? 1 : 0;
      if (!ok) __builtin_amdgcn_s_sleep(2);
    }
    // 3. out of polls: leave the slice to the workgroup that finishes last
    if (!ok && lane == 0) {
      __hip_atomic_fetch_or(&sb->abandon, uint64_t{1} << split, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    if (lane == 0) ctl[1] = ok;
  }
  tail_barrier();
  SPECEXT_STAMP(4);
  if (ctl[1] && owner) do_slice(split, true);     // partials are read at device scope: never a stale cache line
  SPECEXT_STAMP(5);

  // ---- 4. done; the last one to get here takes over the abandoned slices and prepares the next call
  if (tid == 0) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    ctl[2] = static_cast<int>(__hip_atomic_fetch_add(&sb->done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  }
  tail_barrier();
  if (ctl[2] == p.S - 1) {
    if (tid == 0) {
      const uint64_t ab = __hip_atomic_load(&sb->abandon, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      ctl[4] = static_cast<int>(ab & 0xffffffffu);
      ctl[5] = static_cast<int>(ab >> 32);
    }
    tail_barrier();
    uint64_t todo = static_cast<uint32_t>(ctl[4]) | (static_cast<uint64_t>(static_cast<uint32_t>(ctl[5])) << 32);
    while (todo) {
      const int s = __builtin_ctzll(todo);
      todo &= todo - 1;
      do_slice(s, false);
    }
    if (tid == 0) {
      __hip_atomic_store(&sb->abandon, uint64_t{0}, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(&sb->done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(&sb->epoch, tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  SPECEXT_STAMP(6);
}

}  // namespace specext
