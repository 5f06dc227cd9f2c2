// Tree pass and log-sum-exp merge of Hybrid Tree Attention (SpecExtend Sec. 3.1).
//
// Sixteen lanes per query row (tree node t of query head h), four rows per
// wavefront; a lane holds D/16 consecutive elements of the head dimension.  Each
// group of 16 lanes folds in the prefix splits in split order, each weighted by
// exp2(max_split - max_total), and walks its node's ancestor chain through parent[]
// (the tree mask lets a node see itself and its ancestors only) with an online
// softmax over batches of eight ancestors.  The order of these steps is fixed
// (first 16 splits, tree part, remaining splits) and every sum is an fp32
// reduction in a fixed order: no atomics, bit-reproducible from run to run.
//
// The prefix kernels leave one partial per (split, row): (max, sum) in base-2 units
// plus the unnormalised output, in fp32 or (row-split matrix-core kernel, which first
// rescales the triple by a power of two per row) in fp16.
#include "mfma_util.h"

namespace specext {
namespace {

constexpr int kWavesPerBlock = 1;             // small workgroups: the rows spread over every compute unit
constexpr int kRowsPerWave = 4;
constexpr int kRowsPerBlock = kWavesPerBlock * kRowsPerWave;

// N consecutive values starting at element `off` of a bf16 or fp32 array, as fp32
template <int N, bool BF16>
__device__ __forceinline__ void load_row_part(const void* base, int64_t off, float (&v)[N]) {
  if (BF16) {
    const uint32_t* b = reinterpret_cast<const uint32_t*>(static_cast<const uint16_t*>(base) + off);
    uint32_t w[N / 2];
    if constexpr (N == 8) {
      const uint4 x = *reinterpret_cast<const uint4*>(b);
      w[0] = x.x; w[1] = x.y; w[N / 2 - 2] = x.z; w[N / 2 - 1] = x.w;
    } else {
      const uint2 x = *reinterpret_cast<const uint2*>(b);
      w[0] = x.x; w[1] = x.y;
    }
#pragma unroll
    for (int e = 0; e < N / 2; ++e) {
      v[2 * e] = __uint_as_float(w[e] << 16);
      v[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
    }
  } else {
    const float4* b = reinterpret_cast<const float4*>(static_cast<const float*>(base) + off);
#pragma unroll
    for (int e = 0; e < N / 4; ++e) {
      const float4 x = b[e];
      v[4 * e] = x.x; v[4 * e + 1] = x.y; v[4 * e + 2] = x.z; v[4 * e + 3] = x.w;
    }
  }
}

// value of `v` in lane `src` (any lane of the wave) for every lane
__device__ __forceinline__ float lane_read(float v, int src) {
  return __int_as_float(__builtin_amdgcn_ds_bpermute(src << 2, __float_as_int(v)));
}

// HAS_PREFIX: at least one prefix split exists (p.S > 0).  It is a template parameter so that the
// up-front loads below are issued without branches around them: with branches the
// compiler can no longer count which loads are still pending and waits for all of them
// where only the first is needed.
template <int D, bool IN_BF16, bool PART_F16, bool HAS_PREFIX>
__global__ __launch_bounds__(kWavesPerBlock * 64) void tree_merge_kernel(AttnParams p) {
  constexpr int E = D / 16;                      // elements per lane: 8 or 4
  static_assert(!PART_F16 || D == 128, "fp16 partials are written for head_dim 128 only");
  __shared__ int parent_lds[SPECEXT_MAX_TREE];
  const int lane = threadIdx.x & 63;
  const int li = lane & 15;                      // position inside the row's group
  const int grp0 = lane & 48;                    // first lane of the group
  const int n_rows = p.Hq * p.T;
  // parent[] first (at most two entries per thread): everything that follows waits for it
  constexpr int kThreads = kWavesPerBlock * 64;
  constexpr int kParPerThread = (SPECEXT_MAX_TREE + kThreads - 1) / kThreads;
  int par_reg[kParPerThread];
#pragma unroll
  for (int i = 0; i < kParPerThread; ++i) {
    const int idx = threadIdx.x + i * kThreads;
    par_reg[i] = idx < p.T ? p.parent[idx] : -1;
  }
  const int row_raw = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 4);
  const bool live = row_raw < n_rows;
  const int row = live ? row_raw : n_rows - 1;   // groups past the end repeat the last row and store nothing
  // row = g * M + t * G + (head within the group); the quotients through a float
  // reciprocal, exact for rows below 2^20 (the ABI caps n_q_heads * n_tree there)
  const int g = static_cast<int>((static_cast<float>(row) + 0.5f) * (1.0f / static_cast<float>(p.M)));
  const int m = row - g * p.M;
  const int t = static_cast<int>((static_cast<float>(m) + 0.5f) * (1.0f / static_cast<float>(p.G)));
  const int h = g * p.G + (m - t * p.G);

  // Everything below is ordered so that no wait is longer than it must be: loads return in
  // issue order, so the parent array (first, above) is followed by the query, the
  // (max, sum) pairs and the first 16 split partials, which depend on nothing; then, once
  // the ancestor chain is known, come the tree K/V rows and behind them the next 16
  // partials (a compute unit takes in only about 16 bytes per clock, so a longer burst
  // would only block the wave at the load queue).  The arithmetic takes the same order.
  float q[E], o[E];
  load_row_part<E, IN_BF16>(p.q, t * p.q_st + h * p.q_sh + li * E, q);
  constexpr int kRound = 16;                     // splits whose (max, sum) one group holds, one per lane
  constexpr int kPre = PART_F16 ? 32 : 16;       // partials requested up front
  constexpr int PW = PART_F16 ? E / 2 : E;       // 32-bit words a lane holds per partial
  const int64_t split_stride = static_cast<int64_t>(n_rows) * D;
  const uint32_t* po_words = PART_F16 ? reinterpret_cast<const uint32_t*>(p.part_o) + (static_cast<int64_t>(row) * D + li * E) / 2
                                      : reinterpret_cast<const uint32_t*>(p.part_o) + static_cast<int64_t>(row) * D + li * E;
  const int64_t split_words = PART_F16 ? split_stride / 2 : split_stride;
  auto fetch_from = [&](const uint32_t* src, uint32_t (&w)[PW]) {
    // streaming loads: see tree_merge_shared_kernel
    if constexpr (PW == 4) {
      const uintx4 x = __builtin_nontemporal_load(reinterpret_cast<const uintx4*>(src));
      w[0] = x[0]; w[1] = x[1]; w[2] = x[2]; w[3] = x[3];
    } else if constexpr (PW == 8) {
      const uintx4 x = __builtin_nontemporal_load(reinterpret_cast<const uintx4*>(src));
      const uintx4 y = __builtin_nontemporal_load(reinterpret_cast<const uintx4*>(src + 4));
      w[0] = x[0]; w[1] = x[1]; w[2] = x[2]; w[3] = x[3];
      w[4] = y[0]; w[5] = y[1]; w[6] = y[2]; w[7] = y[3];
    } else {
      const uintx2 x = __builtin_nontemporal_load(reinterpret_cast<const uintx2*>(src));
      w[0] = x[0]; w[1] = x[1];
    }
  };
  auto fetch = [&](int s, uint32_t (&w)[PW]) { fetch_from(po_words + s * split_words, w); };
  auto accumulate = [&](const uint32_t (&w)[PW], float weight) {
    if constexpr (PART_F16) {
#pragma unroll
      for (int e = 0; e < E / 2; ++e) {
        const halfx2 hh = __builtin_bit_cast(halfx2, w[e]);
        o[2 * e] = fmaf(static_cast<float>(hh[0]), weight, o[2 * e]);
        o[2 * e + 1] = fmaf(static_cast<float>(hh[1]), weight, o[2 * e + 1]);
      }
    } else {
#pragma unroll
      for (int e = 0; e < E; ++e) o[e] = fmaf(__uint_as_float(w[e]), weight, o[e]);
    }
  };
  // (max, sum) of split s; splits past the end read the last split and count as empty
  auto load_ml = [&](int s) {
    const int sc = min(s, p.S - 1);
    float2 ml = *reinterpret_cast<const float2*>(p.part_ml + (static_cast<int64_t>(sc) * n_rows + row) * 2);
    if (s >= p.S || !(ml.y > 0.f)) ml = make_float2(-INFINITY, 0.f);     // an empty split contributes nothing
    return ml;
  };
  float2 ml_pre[kPre / kRound];
  uint32_t pre[kPre][PW];
  if (HAS_PREFIX) {
#pragma unroll
    for (int r = 0; r < kPre / kRound; ++r) ml_pre[r] = load_ml(r * kRound + li);
  }
  // splits past the end fetch the last split again (never used)
  const uint32_t* pre_src = po_words;
  const uint32_t* const pre_last = po_words + (p.S - 1) * split_words;
  auto request_partials = [&](auto first_c) {      // kRound of them, starting at split FIRST
    constexpr int first = decltype(first_c)::value;
#pragma unroll
    for (int u = first; u < first + kRound; ++u) {
      fetch_from(pre_src, pre[u]);
      if (pre_src != pre_last) pre_src += split_words;
    }
  };
  if (HAS_PREFIX) request_partials(std::integral_constant<int, 0>{});

  {
    bool bad = false;
#pragma unroll
    for (int i = 0; i < kParPerThread; ++i) {
      const int idx = threadIdx.x + i * kThreads;
      if (idx < p.T) {
        parent_lds[idx] = par_reg[i];
        bad |= (par_reg[i] >= idx) || (par_reg[i] < -1);
      }
    }
    if (blockIdx.x == 0) {
      // single writer of the status word: 1 if any parent index is not a topological one
      __shared__ int any_bad;
      if (threadIdx.x == 0) any_bad = 0;
      __syncthreads();
      if (bad) any_bad = 1;
      __syncthreads();
      if (threadIdx.x == 0) *p.status = any_bad;
    } else {
      __syncthreads();
    }
  }

  // ancestor chain of the row's node, eight per batch; the first batch's K/V rows are
  // requested here.  A malformed parent entry ends the walk (the node is then treated as
  // a root).  A group that has run out of ancestors keeps going with weight zero.
  int a = t;
  int anc[8];
  uint32_t kraw[8][IN_BF16 ? E / 2 : E], vraw[8][IN_BF16 ? E / 2 : E];
  constexpr int RW = IN_BF16 ? E / 2 : E;        // 32-bit words a lane holds per K or V row
  auto request_batch = [&]() {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      anc[u] = a;
      if (a >= 0) {
        const int par = parent_lds[a];
        a = (par >= a || par < -1) ? -1 : par;
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (__any(anc[u] >= 0)) {
        const int64_t off = g * p.kt_sh + max(anc[u], 0) * p.kt_st + li * E;
        const uint32_t* ksrc = IN_BF16 ? reinterpret_cast<const uint32_t*>(static_cast<const uint16_t*>(p.kt) + off)
                                       : reinterpret_cast<const uint32_t*>(static_cast<const float*>(p.kt) + off);
        const uint32_t* vsrc = IN_BF16 ? reinterpret_cast<const uint32_t*>(static_cast<const uint16_t*>(p.vt) + off)
                                       : reinterpret_cast<const uint32_t*>(static_cast<const float*>(p.vt) + off);
#pragma unroll
        for (int e = 0; e < RW; e += 2) {
          const uint2 kx = *reinterpret_cast<const uint2*>(ksrc + e), vx = *reinterpret_cast<const uint2*>(vsrc + e);
          kraw[u][e] = kx.x; kraw[u][e + 1] = kx.y;
          vraw[u][e] = vx.x; vraw[u][e + 1] = vx.y;
        }
      }
    }
  };
  auto unpack_row = [&](const uint32_t (&w)[RW], float (&v)[E]) {
    if constexpr (IN_BF16) {
#pragma unroll
      for (int e = 0; e < E / 2; ++e) {
        v[2 * e] = __uint_as_float(w[e] << 16);
        v[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
      }
    } else {
#pragma unroll
      for (int e = 0; e < E; ++e) v[e] = __uint_as_float(w[e]);
    }
  };
  request_batch();
  // the second half of the up-front partials goes behind the K/V rows: by now the
  // first half has drained from the load queue, and it is not needed before the tree part
  if (HAS_PREFIX && kPre > kRound) request_partials(std::integral_constant<int, kPre - kRound>{});

#pragma unroll
  for (int e = 0; e < E; ++e) {
    q[e] *= p.scale_log2;
    o[e] = 0.f;
  }
  float run_max = -INFINITY, run_sum = 0.f;

  // prefix splits, 16 per round.  Lane i of a group holds (max, sum) of split s0 + i, the
  // group agrees on the common maximum, and lane i keeps the weight of its split.  The
  // partial outputs are then added in split order with the weights fetched from their
  // lanes.  Fixed order, no atomics: bit-reproducible.
  auto merge_round = [&](float2 ml, int s0, auto&& partial_of) {
    const float ms = ml.x, ls = ml.y;
    const float new_max = fmaxf(run_max, row16_max(ms));
    const bool any = new_max > -INFINITY;          // false only while nothing has been seen at all
    const float alpha = any ? fast_exp2(run_max - new_max) : 1.f;
    const float w = ls > 0.f ? fast_exp2(ms - new_max) : 0.f;             // weight of the split's unnormalised output
    const float wsum = ls * w;                                             // the split's share of the row sum
    run_max = new_max;
    run_sum = fmaf(run_sum, alpha, row16_sum(wsum));
#pragma unroll
    for (int e = 0; e < E; ++e) o[e] *= alpha;
    partial_of(w, min(kRound, p.S - s0));
  };
  auto merge_preloaded = [&](auto r_c) {
    constexpr int r = decltype(r_c)::value;
    if (HAS_PREFIX && r * kRound < p.S) {
      merge_round(ml_pre[r], r * kRound, [&](float w, int s_end) {
#pragma unroll
        for (int u = 0; u < kRound; ++u) {
          if (u < s_end) accumulate(pre[r * kRound + u], lane_read(w, grp0 + u));
        }
      });
    }
  };
  merge_preloaded(std::integral_constant<int, 0>{});

  // tree part: the batch's eight logits first (independent of one another), then one
  // online-softmax step for the whole batch
  while (true) {
    float sc[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      sc[u] = -INFINITY;
      if (__any(anc[u] >= 0)) {
        float kk[E];
        unpack_row(kraw[u], kk);
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) dot = fmaf(q[e], kk[e], dot);
        dot = row16_sum(dot);
        if (anc[u] >= 0) sc[u] = dot;
      }
    }
    float bm = fmaxf(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3])), fmaxf(fmaxf(sc[4], sc[5]), fmaxf(sc[6], sc[7])));
    const float new_max = fmaxf(run_max, bm);      // finite: the first batch holds the node itself
    const float alpha = fast_exp2(run_max - new_max);
    run_max = new_max;
    run_sum *= alpha;
#pragma unroll
    for (int e = 0; e < E; ++e) o[e] *= alpha;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (__any(anc[u] >= 0)) {
        const float pr = fast_exp2(sc[u] - new_max);
        float vv[E];
        unpack_row(vraw[u], vv);
#pragma unroll
        for (int e = 0; e < E; ++e) o[e] = fmaf(pr, vv[e], o[e]);
        run_sum += pr;
      }
    }
    if (!__any(a >= 0)) break;
    request_batch();
  }

  if (kPre > kRound) merge_preloaded(std::integral_constant<int, (kPre > kRound ? 1 : 0)>{});
  for (int s0 = kPre; HAS_PREFIX && s0 < p.S; s0 += kRound) {
    merge_round(load_ml(s0 + li), s0, [&](float w, int s_end) {
      int s = 0;
      for (; s + 8 <= s_end; s += 8) {
        uint32_t raw[8][PW];
#pragma unroll
        for (int u = 0; u < 8; ++u) fetch(s0 + s + u, raw[u]);
#pragma unroll
        for (int u = 0; u < 8; ++u) accumulate(raw[u], lane_read(w, grp0 + s + u));
      }
      for (; s < s_end; ++s) {
        uint32_t raw[PW];
        fetch(s0 + s, raw);
        accumulate(raw, lane_read(w, grp0 + s));
      }
    });
  }

  if (!live) return;
  const float inv = 1.f / run_sum;
  const int64_t ooff = t * p.o_st + h * p.o_sh + li * E;
  if (p.out_dtype == SPECEXT_BF16) {
    uint32_t w[E / 2];
#pragma unroll
    for (int e = 0; e < E / 2; ++e)
      w[e] = static_cast<uint32_t>(float_to_bf16_bits(o[2 * e] * inv)) |
             (static_cast<uint32_t>(float_to_bf16_bits(o[2 * e + 1] * inv)) << 16);
    uint32_t* ob = reinterpret_cast<uint32_t*>(static_cast<uint16_t*>(p.out) + ooff);
    if (E == 8) {
      *reinterpret_cast<uint4*>(ob) = make_uint4(w[0], w[1], w[E / 2 - 2], w[E / 2 - 1]);
    } else {
      *reinterpret_cast<uint2*>(ob) = make_uint2(w[0], w[1]);
    }
  } else {
    float4* of = reinterpret_cast<float4*>(static_cast<float*>(p.out) + ooff);
#pragma unroll
    for (int e = 0; e < E / 4; ++e) of[e] = make_float4(o[4 * e] * inv, o[4 * e + 1] * inv, o[4 * e + 2] * inv, o[4 * e + 3] * inv);
  }
  if (li == 0) {
    const float l2 = run_max + log2f(run_sum);
    p.lse2[row] = l2;
    if (p.lse) p.lse[h * p.T + t] = l2 * kLn2;
  }
}


// ---------------------------------------------------------------------------------------
// The same result for the hot configuration (head_dim 128, bf16 inputs, fp16 partials,
// at most 64 splits), with the work of four rows shared by four wavefronts.
//
// The kernel above gives a row's whole merge to sixteen lanes of one wave: the launch then
// has fewer waves than the chip has SIMDs, every wave runs alone on its SIMD and the
// kernel's duration is the time one wave takes to issue its ~2400 instructions.  Here the
// four waves of a workgroup serve the same four rows and each takes a quarter of the items
// of the row's softmax: PER consecutive prefix splits and every fourth node of the ancestor
// chain.  A wave reduces its items to a partial (max, sum, output) in the usual way, the four
// partials meet in LDS, and wave w finishes row w.  Per wave the instruction stream is a
// quarter as long and two waves share a SIMD, so issue time no longer bounds the kernel.
// Every sum keeps a fixed order: bit-reproducible from run to run.
constexpr int kShareWaves = 4;               // 8 measured no faster
constexpr int kShareSlot = 132;               // floats per (wave, row) slot: 128 outputs, max, sum, padding

template <int PER>
__global__ __launch_bounds__(kShareWaves * 64) void tree_merge_shared_kernel(AttnParams p) {
  constexpr int D = 128, E = 8;
  constexpr int kThreads = kShareWaves * 64;
  static_assert(SPECEXT_MAX_TREE <= kThreads, "one parent entry per thread");
  static_assert(PER >= 1 && PER <= 16, "a group of 16 lanes holds one (max, sum) pair per lane");
  __shared__ int parent_lds[SPECEXT_MAX_TREE];
  __shared__ __attribute__((aligned(16))) float slots[kShareWaves][kRowsPerWave][kShareSlot];
  __shared__ int any_bad;
  const int tid = threadIdx.x;
#ifdef SPECEXT_TAIL_STAMPS
  // profiling build: 100 MHz wall-clock stamps of this workgroup's phases (0 start, 1 parent array there, 2 the
  // partials requested up front and the query there, 3 tree K/V rows and the other partials there, 4 stores issued,
  // 5 stores acknowledged), left in the unused upper half of the partial-output region, 2 MiB in; the waits that
  // separate 2 and 3 are extra
  unsigned long long phase_stamp[6];
  phase_stamp[0] = wall_clock64();
#endif
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15;
  const int rg = lane >> 4;                      // row of the workgroup this group of 16 lanes works for
  const int grp0 = lane & 48;
  const int n_rows = p.Hq * p.T;

  // parent[] first, then everything else that depends on nothing; loads return in issue order
  const int par_reg = tid < p.T ? p.parent[tid] : -1;
  const int row_raw = blockIdx.x * kRowsPerWave + rg;
  const bool live = row_raw < n_rows;
  const int row = live ? row_raw : n_rows - 1;   // groups past the end repeat the last row and store nothing
  const int g = static_cast<int>((static_cast<float>(row) + 0.5f) * (1.0f / static_cast<float>(p.M)));
  const int m = row - g * p.M;
  const int t = static_cast<int>((static_cast<float>(m) + 0.5f) * (1.0f / static_cast<float>(p.G)));
  const int h = g * p.G + (m - t * p.G);

  // this wave's splits: s_lo .. s_lo + PER - 1; those past the last split read the last one
  // again and count as empty
  const int s_lo = wave * PER;
  const int s_last = p.S - 1;
  const floatx2 ml_raw = __builtin_nontemporal_load(reinterpret_cast<const floatx2*>(
      p.part_ml + (static_cast<int64_t>(min(s_lo + li, s_last)) * n_rows + row) * 2));
  float2 ml = make_float2(ml_raw[0], ml_raw[1]);
  const bool ml_valid = li < PER && s_lo + li <= s_last;
  const int64_t split_words = static_cast<int64_t>(n_rows) * D / 2;
  const uint32_t* po = reinterpret_cast<const uint32_t*>(p.part_o) + (static_cast<int64_t>(row) * D + li * E) / 2;
  uintx4 raw[PER];
  // (streaming loads: partial lines left behind in the L2s would be hit by the next launch's partial stores, which
  // costs that launch 1.3 - 2 us at prefixes of 2K - 4K tokens, whose K/V stream is too short to evict them first)
  constexpr int kFirst = PER >= 4 ? PER / 2 : PER;      // partials requested before the tree K/V rows
#pragma unroll
  for (int u = 0; u < kFirst; ++u) raw[u] = __builtin_nontemporal_load(reinterpret_cast<const uintx4*>(po + min(s_lo + u, s_last) * split_words));
  float q[E];
  load_row_part<E, true>(p.q, t * p.q_st + h * p.q_sh + li * E, q);

  {
    bool bad = false;
#ifdef SPECEXT_TAIL_STAMPS
    asm volatile("" :: "v"(par_reg));
    phase_stamp[1] = wall_clock64();
#endif
    if (tid < p.T) {
      parent_lds[tid] = par_reg;
      bad = (par_reg >= tid) || (par_reg < -1);
    }
    if (blockIdx.x == 0) {
      // single writer of the status word: 1 if any parent index is not a topological one
      if (tid == 0) any_bad = 0;
      __syncthreads();
      if (bad) any_bad = 1;
      __syncthreads();
      if (tid == 0) *p.status = any_bad;
    } else {
      __syncthreads();
    }
  }

  // Ancestor chain of the row's node (the node itself first).  Every wave walks the whole
  // chain and keeps the nodes at positions wave, wave + 4, ...; kAnc of them per batch.  A
  // malformed parent entry ends the walk (the node is then treated as a root).
  constexpr int kAnc = 8 / kShareWaves;
  int a = t;
  int anc[kAnc];
  uintx4 kraw[kAnc], vraw[kAnc];
  auto request_batch = [&]() {
#pragma unroll
    for (int u = 0; u < kAnc; ++u) {
#pragma unroll
      for (int w = 0; w < kShareWaves; ++w) {
        if (w == wave) anc[u] = a;
        if (a >= 0) {
          const int par = parent_lds[a];
          a = (par >= a || par < -1) ? -1 : par;
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kAnc; ++u) {
      const int64_t off = g * p.kt_sh + max(anc[u], 0) * p.kt_st + li * E;
      kraw[u] = *reinterpret_cast<const uintx4*>(static_cast<const uint16_t*>(p.kt) + off);
      vraw[u] = *reinterpret_cast<const uintx4*>(static_cast<const uint16_t*>(p.vt) + off);
    }
  };
  request_batch();
  // the rest of the partials goes behind the K/V rows, which would otherwise queue behind all of them
#pragma unroll
  for (int u = kFirst; u < PER; ++u) raw[u] = __builtin_nontemporal_load(reinterpret_cast<const uintx4*>(po + min(s_lo + u, s_last) * split_words));

#ifdef SPECEXT_TAIL_STAMPS
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * kAnc + PER - kFirst) : "memory");      // the loads requested up front
  phase_stamp[2] = wall_clock64();
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  phase_stamp[3] = wall_clock64();
#endif
  // the wave's prefix splits: lane i of a group holds (max, sum) of split s_lo + i
  if (!ml_valid || !(ml.y > 0.f)) ml = make_float2(-INFINITY, 0.f);        // an empty split contributes nothing
  float run_max = row16_max(ml.x);
  const float wgt = ml.y > 0.f ? fast_exp2(ml.x - run_max) : 0.f;
  float run_sum = row16_sum(ml.y * wgt);
  float o[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    q[e] *= p.scale_log2;
    o[e] = 0.f;
  }
#pragma unroll
  for (int u = 0; u < PER; ++u) {
    const float w = lane_read(wgt, grp0 + u);
#pragma unroll
    for (int e = 0; e < E / 2; ++e) {
      const uint32_t word = raw[u][e];
      const halfx2 hh = __builtin_bit_cast(halfx2, word);
      o[2 * e] = fmaf(static_cast<float>(hh[0]), w, o[2 * e]);
      o[2 * e + 1] = fmaf(static_cast<float>(hh[1]), w, o[2 * e + 1]);
    }
  }

  // the wave's share of the tree part, one online-softmax step per batch
  while (true) {
    float sc[kAnc];
#pragma unroll
    for (int u = 0; u < kAnc; ++u) {
      float dot = 0.f;
#pragma unroll
      for (int e = 0; e < E / 2; ++e) {
        const uint32_t word = kraw[u][e];
        dot = fmaf(q[2 * e], __uint_as_float(word << 16), dot);
        dot = fmaf(q[2 * e + 1], __uint_as_float(word & 0xffff0000u), dot);
      }
      dot = row16_sum(dot);
      sc[u] = anc[u] >= 0 ? dot : -INFINITY;
    }
    float bm = sc[0];
#pragma unroll
    for (int u = 1; u < kAnc; ++u) bm = fmaxf(bm, sc[u]);
    const float new_max = fmaxf(run_max, bm);
    // nothing seen so far and nothing in this batch: keep the empty state
    const float alpha = new_max > -INFINITY ? fast_exp2(run_max - new_max) : 1.f;
    run_max = new_max;
    run_sum *= alpha;
#pragma unroll
    for (int e = 0; e < E; ++e) o[e] *= alpha;
#pragma unroll
    for (int u = 0; u < kAnc; ++u) {
      const float pr = anc[u] >= 0 ? fast_exp2(sc[u] - new_max) : 0.f;
#pragma unroll
      for (int e = 0; e < E / 2; ++e) {
        const uint32_t word = vraw[u][e];
        o[2 * e] = fmaf(pr, __uint_as_float(word << 16), o[2 * e]);
        o[2 * e + 1] = fmaf(pr, __uint_as_float(word & 0xffff0000u), o[2 * e + 1]);
      }
      run_sum += pr;
    }
    if (!__any(a >= 0)) break;
    request_batch();
  }

  // the wave's partial goes to LDS; wave w then finishes row w, two output elements per lane
  {
    float* slot = &slots[wave][rg][0];
    *reinterpret_cast<float4*>(slot + li * E) = make_float4(o[0], o[1], o[2], o[3]);
    *reinterpret_cast<float4*>(slot + li * E + 4) = make_float4(o[4], o[5], o[6], o[7]);
    if (li == 0) *reinterpret_cast<float2*>(slot + D) = make_float2(run_max, run_sum);
  }
  __syncthreads();
  const int frow = blockIdx.x * kRowsPerWave + wave;
  if (wave >= kRowsPerWave || frow >= n_rows) return;
  float2 st[kShareWaves];
#pragma unroll
  for (int w = 0; w < kShareWaves; ++w) st[w] = *reinterpret_cast<const float2*>(&slots[w][wave][D]);
  float top = st[0].x;
#pragma unroll
  for (int w = 1; w < kShareWaves; ++w) top = fmaxf(top, st[w].x);     // finite: wave 0 holds the node itself
  float total = 0.f;
  float2 acc = make_float2(0.f, 0.f);
#pragma unroll
  for (int w = 0; w < kShareWaves; ++w) {
    const float wt = st[w].y > 0.f ? fast_exp2(st[w].x - top) : 0.f;
    total = fmaf(st[w].y, wt, total);
    const float2 v = *reinterpret_cast<const float2*>(&slots[w][wave][lane * 2]);
    acc.x = fmaf(v.x, wt, acc.x);
    acc.y = fmaf(v.y, wt, acc.y);
  }
  const float inv = 1.f / total;
  const int fg = static_cast<int>((static_cast<float>(frow) + 0.5f) * (1.0f / static_cast<float>(p.M)));
  const int fm = frow - fg * p.M;
  const int ft = static_cast<int>((static_cast<float>(fm) + 0.5f) * (1.0f / static_cast<float>(p.G)));
  const int fh = fg * p.G + (fm - ft * p.G);
  const int64_t ooff = ft * p.o_st + fh * p.o_sh + lane * 2;
  if (p.out_dtype == SPECEXT_BF16) {
    *reinterpret_cast<uint32_t*>(static_cast<uint16_t*>(p.out) + ooff) =
        static_cast<uint32_t>(float_to_bf16_bits(acc.x * inv)) |
        (static_cast<uint32_t>(float_to_bf16_bits(acc.y * inv)) << 16);
  } else {
    *reinterpret_cast<float2*>(static_cast<float*>(p.out) + ooff) = make_float2(acc.x * inv, acc.y * inv);
  }
  if (lane == 0) {
    const float l2 = top + log2f(total);
    p.lse2[frow] = l2;
    if (p.lse) p.lse[fh * p.T + ft] = l2 * kLn2;
  }
#ifdef SPECEXT_TAIL_STAMPS
  phase_stamp[4] = wall_clock64();
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  phase_stamp[5] = wall_clock64();
  const size_t spare = static_cast<size_t>(p.S) * p.Hq * p.T * D * 2;        // bytes of that upper half
  if (tid == 0 && spare >= (size_t{2} << 20) + static_cast<size_t>(gridDim.x) * 64) {
    unsigned long long* st = reinterpret_cast<unsigned long long*>(reinterpret_cast<unsigned char*>(p.part_o) + spare + (2 << 20)) +
                             blockIdx.x * 8;
#pragma unroll
    for (int i = 0; i < 6; ++i) st[i] = phase_stamp[i];
  }
#endif
}

}  // namespace

hipError_t launch_tree_merge(const AttnParams& p, hipStream_t stream) {
  const int n_rows = p.Hq * p.T;
  dim3 grid((n_rows + kRowsPerBlock - 1) / kRowsPerBlock);
  dim3 block(kWavesPerBlock * 64);
  const bool bf16 = p.in_dtype == SPECEXT_BF16;
  if (p.part_f16 && !(p.d == 128 && bf16)) return hipErrorInvalidValue;
  const bool pre = p.S > 0;
#ifndef SPECEXT_MERGE_ONE_WAVE_PER_ROWS
  if (p.part_f16 && p.S >= 1 && p.S <= 16 * kShareWaves) {
    dim3 shared_block(kShareWaves * 64);
    const int per = (p.S + kShareWaves - 1) / kShareWaves;       // splits per wave, rounded up to a power of two
    if (per <= 1) tree_merge_shared_kernel<1><<<grid, shared_block, 0, stream>>>(p);
    else if (per <= 2) tree_merge_shared_kernel<2><<<grid, shared_block, 0, stream>>>(p);
    else if (per <= 4) tree_merge_shared_kernel<4><<<grid, shared_block, 0, stream>>>(p);
    else if (per <= 8) tree_merge_shared_kernel<8><<<grid, shared_block, 0, stream>>>(p);
    else tree_merge_shared_kernel<16><<<grid, shared_block, 0, stream>>>(p);
    return hipGetLastError();
  }
#endif
#define SPECEXT_LAUNCH(D_, BF_, F16_)                                                              \
  do {                                                                                             \
    if (pre) tree_merge_kernel<D_, BF_, F16_, true><<<grid, block, 0, stream>>>(p);                \
    else tree_merge_kernel<D_, BF_, F16_, false><<<grid, block, 0, stream>>>(p);                   \
  } while (0)
  if (p.d == 128) {
    if (p.part_f16) SPECEXT_LAUNCH(128, true, true);
    else if (bf16) SPECEXT_LAUNCH(128, true, false);
    else SPECEXT_LAUNCH(128, false, false);
  } else {
    if (bf16) SPECEXT_LAUNCH(64, true, false);
    else SPECEXT_LAUNCH(64, false, false);
  }
#undef SPECEXT_LAUNCH
  return hipGetLastError();
}

}  // namespace specext
