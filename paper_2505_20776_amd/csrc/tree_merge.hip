// Tree pass and log-sum-exp merge of Hybrid Tree Attention (SpecExtend Sec. 3.1).
//
// One wavefront per query row (tree node t of query head h).  The lanes hold
// the head dimension.  The wave first walks the node's ancestor chain through
// parent[] (the tree mask lets a node see itself and its ancestors only) with
// an online softmax, then folds in the prefix splits in split order, each
// weighted by exp2(max_split - max_total).  The merge is a fixed-order fp32
// reduction: no atomics, bit-reproducible from run to run.
#include "common.h"

namespace specext {
namespace {

constexpr int kWavesPerBlock = 4;

template <int D, bool IN_BF16>
__device__ __forceinline__ void load_vec(const void* base, int64_t off, int lane, float (&v)[D / 64]) {
  constexpr int E = D / 64;
  if (IN_BF16) {
    const uint16_t* b = static_cast<const uint16_t*>(base) + off + lane * E;
    if (E == 2) {
      const uint32_t w = *reinterpret_cast<const uint32_t*>(b);
      v[0] = __uint_as_float(w << 16);
      v[E - 1] = __uint_as_float(w & 0xffff0000u);
    } else {
      v[0] = bf16_bits_to_float(b[0]);
    }
  } else {
    const float* b = static_cast<const float*>(base) + off + lane * E;
#pragma unroll
    for (int e = 0; e < E; ++e) v[e] = b[e];
  }
}

// PART_BF16: the prefix kernel wrote its partial outputs as bf16 (row-split matrix-core
// kernel, D = 128) instead of fp32; a lane's two values are then one 32-bit word.
template <int D, bool IN_BF16, bool PART_BF16>
__global__ __launch_bounds__(kWavesPerBlock * 64) void tree_merge_kernel(AttnParams p) {
  constexpr int E = D / 64;
  static_assert(!PART_BF16 || E == 2, "bf16 partials are written for head_dim 128 only");
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);   // rid
  const int n_rows = p.Hq * p.T;
  if (blockIdx.x == 0 && threadIdx.x < 64) {
    // single writer of the status word: 1 if any parent index is not a topological one
    bool bad = false;
    for (int i = lane; i < p.T; i += 64) {
      const int par = p.parent[i];
      bad |= (par >= i) || (par < -1);
    }
    const bool any_bad = __any(bad);
    if (lane == 0) *p.status = any_bad ? 1 : 0;
  }
  if (row >= n_rows) return;
  const int g = row / p.M;
  const int m = row - g * p.M;
  const int t = m / p.G;
  const int h = g * p.G + m % p.G;

  // The loads of the first 32 split partials are issued before anything else so that
  // their latency overlaps the tree pass below; they do not depend on it.
  constexpr int kPre = 32;
  const int64_t split_stride = static_cast<int64_t>(n_rows) * D;
  const float* po_row = p.part_o + static_cast<int64_t>(row) * D + lane * E;
  const uint32_t* po_row_h = reinterpret_cast<const uint32_t*>(p.part_o) + static_cast<int64_t>(row) * (D / 2) + lane;
  constexpr int PE = PART_BF16 ? 1 : E;          // 32-bit words a lane holds per partial
  // raw words of split s (fetch) and their fp32 values (decode)
  auto fetch = [&](int64_t s, uint32_t (&w)[PE]) {
    if (PART_BF16) {
      w[0] = po_row_h[s * (split_stride / 2)];
    } else {
#pragma unroll
      for (int e = 0; e < PE; ++e) w[e] = __float_as_uint(po_row[s * split_stride + e]);
    }
  };
  auto decode = [&](const uint32_t (&w)[PE], float (&v)[E]) {
    if (PART_BF16) {
      v[0] = __uint_as_float(w[0] << 16);
      v[E - 1] = __uint_as_float(w[0] & 0xffff0000u);
    } else {
#pragma unroll
      for (int e = 0; e < E; ++e) v[e] = __uint_as_float(w[e]);
    }
  };
  float2 ml_first = make_float2(-INFINITY, 0.f);
  if (lane < p.S) ml_first = *reinterpret_cast<const float2*>(p.part_ml + (static_cast<int64_t>(lane) * n_rows + row) * 2);
  uint32_t pre[kPre][PE];
#pragma unroll
  for (int u = 0; u < kPre; ++u) {
    if (u < p.S) fetch(u, pre[u]);
  }

  float q[E], o[E];
  load_vec<D, IN_BF16>(p.q, t * p.q_st + h * p.q_sh, lane, q);
#pragma unroll
  for (int e = 0; e < E; ++e) {
    q[e] *= p.scale_log2;
    o[e] = 0.f;
  }
  float run_max = -INFINITY, run_sum = 0.f;

  // tree part: node t and its ancestors.  The parent array (at most 128 entries) is
  // held two per lane and the chain is walked with cross-lane reads, without touching
  // memory; the ancestors' K/V rows are then fetched eight at a time so that their
  // load latencies overlap.  A malformed entry ends the walk (the node is then
  // treated as a root).
  const int par_lo = lane < p.T ? p.parent[lane] : -1;
  const int par_hi = lane + 64 < p.T ? p.parent[lane + 64] : -1;
  int a = t;
  while (a >= 0) {
    int anc[8];
    int n_anc = 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      anc[u] = a;
      if (a >= 0) {
        ++n_anc;
        const int par = a < 64 ? __builtin_amdgcn_readlane(par_lo, a) : __builtin_amdgcn_readlane(par_hi, a - 64);
        a = (par >= a || par < -1) ? -1 : par;
      }
    }
    float kk[8][E], vv[8][E];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (u < n_anc) {
        load_vec<D, IN_BF16>(p.kt, g * p.kt_sh + anc[u] * p.kt_st, lane, kk[u]);
        load_vec<D, IN_BF16>(p.vt, g * p.kt_sh + anc[u] * p.kt_st, lane, vv[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (u < n_anc) {
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) dot = fmaf(q[e], kk[u][e], dot);
        const float s = wave_sum(dot);
        const float new_max = fmaxf(run_max, s);
        const float alpha = exp2f(run_max - new_max);
        const float pr = exp2f(s - new_max);
#pragma unroll
        for (int e = 0; e < E; ++e) o[e] = fmaf(pr, vv[u][e], o[e] * alpha);
        run_sum = fmaf(run_sum, alpha, pr);
        run_max = new_max;
      }
    }
  }

  // prefix splits.  Lane s first takes (max, sum) of split s (64 splits per round), the
  // wave agrees on the common maximum, and lane s keeps the weight exp2(max_s - max_total)
  // of its split.  The partial outputs are then added in split order with the weights
  // broadcast from their lanes; the loads do not depend on one another, so several
  // are in flight at once.  Fixed order, no atomics: bit-reproducible.
  for (int s0 = 0; s0 < p.S; s0 += 64) {
    const int s_mine = s0 + lane;
    float ms = -INFINITY, ls = 0.f;
    if (s_mine < p.S) {
      const float2 ml = s0 == 0 ? ml_first
                                : *reinterpret_cast<const float2*>(p.part_ml + (static_cast<int64_t>(s_mine) * n_rows + row) * 2);
      if (ml.y > 0.f) {              // an empty split contributes nothing
        ms = ml.x;
        ls = ml.y;
      }
    }
    const float new_max = fmaxf(run_max, wave_max(ms));
    if (new_max == -INFINITY) continue;          // nothing so far and nothing in this round (wave-uniform)
    const float alpha = exp2f(run_max - new_max);
    const float w = ls > 0.f ? exp2f(ms - new_max) : 0.f;
    run_max = new_max;
    run_sum = fmaf(run_sum, alpha, wave_sum(ls * w));
#pragma unroll
    for (int e = 0; e < E; ++e) o[e] *= alpha;
    const int s_end = min(64, p.S - s0);
    int s = 0;
    if (s0 == 0) {                   // the preloaded partials, in split order
#pragma unroll
      for (int u = 0; u < kPre; ++u) {
        if (u < s_end) {
          const float wu = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w), u));
          float v[E];
          decode(pre[u], v);
#pragma unroll
          for (int e = 0; e < E; ++e) o[e] = fmaf(v[e], wu, o[e]);
        }
      }
      s = min(kPre, s_end);
    }
    for (; s + 8 <= s_end; s += 8) {
      uint32_t raw[8][PE];
#pragma unroll
      for (int u = 0; u < 8; ++u) fetch(s0 + s + u, raw[u]);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float wu = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w), s + u));
        float v[E];
        decode(raw[u], v);
#pragma unroll
        for (int e = 0; e < E; ++e) o[e] = fmaf(v[e], wu, o[e]);
      }
    }
    for (; s < s_end; ++s) {
      const float wu = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w), s));
      uint32_t raw[PE];
      fetch(s0 + s, raw);
      float v[E];
      decode(raw, v);
#pragma unroll
      for (int e = 0; e < E; ++e) o[e] = fmaf(v[e], wu, o[e]);
    }
  }

  const float inv = 1.f / run_sum;
  const int64_t ooff = t * p.o_st + h * p.o_sh + lane * E;
  if (p.out_dtype == SPECEXT_BF16) {
    uint16_t* ob = static_cast<uint16_t*>(p.out) + ooff;
    if (E == 2) {
      const uint32_t w = static_cast<uint32_t>(float_to_bf16_bits(o[0] * inv)) |
                         (static_cast<uint32_t>(float_to_bf16_bits(o[E - 1] * inv)) << 16);
      *reinterpret_cast<uint32_t*>(ob) = w;
    } else {
      ob[0] = float_to_bf16_bits(o[0] * inv);
    }
  } else {
    float* of = static_cast<float*>(p.out) + ooff;
#pragma unroll
    for (int e = 0; e < E; ++e) of[e] = o[e] * inv;
  }
  if (lane == 0) {
    const float l2 = run_max + log2f(run_sum);
    p.lse2[row] = l2;
    if (p.lse) p.lse[h * p.T + t] = l2 * kLn2;
  }
}

}  // namespace

hipError_t launch_tree_merge(const AttnParams& p, hipStream_t stream) {
  const int n_rows = p.Hq * p.T;
  dim3 grid((n_rows + kWavesPerBlock - 1) / kWavesPerBlock);
  dim3 block(kWavesPerBlock * 64);
  const bool bf16 = p.in_dtype == SPECEXT_BF16;
  if (p.part_bf16 && !(p.d == 128 && bf16)) return hipErrorInvalidValue;
  if (p.d == 128) {
    if (p.part_bf16) tree_merge_kernel<128, true, true><<<grid, block, 0, stream>>>(p);
    else if (bf16) tree_merge_kernel<128, true, false><<<grid, block, 0, stream>>>(p);
    else tree_merge_kernel<128, false, false><<<grid, block, 0, stream>>>(p);
  } else {
    if (bf16) tree_merge_kernel<64, true, false><<<grid, block, 0, stream>>>(p);
    else tree_merge_kernel<64, false, false><<<grid, block, 0, stream>>>(p);
  }
  return hipGetLastError();
}

}  // namespace specext
