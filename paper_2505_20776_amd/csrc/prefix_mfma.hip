// Prefix pass of Hybrid Tree Attention (SpecExtend Sec. 3.1) on the gfx950
// matrix cores: bf16 K/V streamed once from HBM, fp32 accumulation.
//
// Work decomposition (FlashDecoding-style split over the KV length, laid out
// for 256 compute units with only a handful of KV heads):
//   grid  = (splits, KV heads, row groups); a row group is 32*RB query rows
//           (row m = tree node * G + head-in-group) of one KV head.
//   block = 4 wavefronts.  All four work on the SAME rows and take the 32-key
//           tiles of the split round-robin, each with a private LDS staging
//           area, so the main loop has no workgroup barrier.  At the end the
//           four partial (max, sum, O) sets are merged through LDS and one
//           partial per (split, row) goes to the workspace.
//   Row groups of the same (split, head) read the same K/V; their workgroup
//   ids are congruent modulo 8 so that they land on one XCD and share its L2.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, everything transposed so that
// a lane owns one query row in both products):
//   S^T[key][row]  = K[key][:] . Q[row][:]      A = K tile (LDS), B = Q (registers)
//   O^T[dcol][row] += V^T[dcol][key] P^T[key][row]   A = V^T (LDS transpose
//   read ds_read_b64_tr_b16), B = P^T taken straight from the S^T accumulator
//   registers: the key order the accumulator layout implies is used as the
//   contraction order and V is fetched in that same order, so P never moves
//   between lanes.
// Row max / row sum therefore live in one lane pair (lane, lane^32).
#include "mfma_util.h"

namespace specext {
namespace {

constexpr int kWaves = 4;
constexpr int kTile = 32;                         // keys per wave tile
constexpr int kD = 128;                           // head_dim this kernel is written for
constexpr int kRowBytes = kD * 2;                 // one bf16 K or V row in LDS
constexpr int kTileBytes = kTile * kRowBytes;     // 8 KB: one K (or V) tile
constexpr int kKSlots = 3;                        // ring of K tiles per wave
constexpr int kVSlots = 2;                        // ring of V tiles per wave
constexpr int kStageBytes = (kKSlots + kVSlots) * kTileBytes;   // 40 KB per wave, 160 KB per workgroup
constexpr int kMergeFloatsPerWave = 4 * 2 * 16 * 64;   // O^T dump at RB = 2
constexpr int kMergeBytes = kWaves * kMergeFloatsPerWave * 4 + kWaves * 2 * 2 * 32 * 4;
constexpr int kLdsBytes = kMergeBytes > kWaves * kStageBytes ? kMergeBytes : kWaves * kStageBytes;
// Wait until at most 8 * groups vector-memory operations are outstanding.
__device__ __forceinline__ void wait_vm_groups(int groups) {
  switch (groups) {
    case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    case 1: asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); break;
    case 2: asm volatile("s_waitcnt vmcnt(16)" ::: "memory"); break;
    case 3: asm volatile("s_waitcnt vmcnt(24)" ::: "memory"); break;
    case 4: asm volatile("s_waitcnt vmcnt(32)" ::: "memory"); break;
    default: asm volatile("s_waitcnt vmcnt(40)" ::: "memory"); break;
  }
}

template <int RB, bool SCORES>
__global__ __launch_bounds__(kWaves * 64) void prefix_mfma_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c32 = lane & 31;
  const int hf = lane >> 5;

  const int split = blockIdx.x;
  const int g = blockIdx.y;
  const int row0 = blockIdx.z * (32 * RB);

  const int key_lo = split * p.keys_per_split;
  const int key_hi = min(p.L, key_lo + p.keys_per_split);
  const int n_tiles = (key_hi - key_lo + kTile - 1) / kTile;
  // this wave takes tiles wave, wave + 4, ...: n of them, numbered j = 0 .. n-1
  const int n = (n_tiles - wave + kWaves - 1) / kWaves;

  const int64_t row_bytes = p.kp_sl * 2;
  const unsigned char* kbase = static_cast<const unsigned char*>(p.kp) + static_cast<int64_t>(g) * p.kp_sh * 2;
  const unsigned char* vbase = static_cast<const unsigned char*>(p.vp) + static_cast<int64_t>(g) * p.kp_sh * 2;

  // ---- Q fragments (B operand of S^T): lane = row c32, 8 consecutive d per k-step ----
  bf16x8 qf[RB][8];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int m = row0 + 32 * rb + c32;
    const bool ok = m < p.M;
    const int t = ok ? m / p.G : 0;
    const int h = g * p.G + (ok ? m % p.G : 0);
    const uint16_t* qp = static_cast<const uint16_t*>(p.q) + t * p.q_st + h * p.q_sh + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      uintx4 w = {0u, 0u, 0u, 0u};
      if (ok) w = *reinterpret_cast<const uintx4*>(qp + 16 * ks);
      qf[rb][ks] = __builtin_bit_cast(bf16x8, w);
    }
  }
  // All query loads have landed before the main loop starts; said through the builtin
  // so that the compiler's own wait bookkeeping sees it and adds no vmcnt wait of its
  // own inside the loop (0x0F70 = vmcnt(0), other counters untouched).
  __builtin_amdgcn_s_waitcnt(0x0F70);

  // ---- per-wave LDS staging: a ring of 3 K tiles and a ring of 2 V tiles, each
  // tile 32 rows x 256 B, filled by direct global->LDS loads: one load instruction
  // writes 1 KB = 4 consecutive rows, lane i landing at byte 16*i.  The 16-byte
  // chunks of a row are XOR-swizzled (K: chunk ^ (row & 15), V: chunk ^
  // ((row & 3) << 2)) so that the operand reads are bank-conflict free; since the
  // LDS side of such a load is fixed, the swizzle is applied to the global address.
  unsigned char* stage = lds + wave * kStageBytes;
  const unsigned stage_lds = static_cast<unsigned>(reinterpret_cast<uintptr_t>((lds_void*)stage));
  const int ld_row = lane >> 4;          // row within the 4-row block of one load
  const int ld_slot = lane & 15;         // LDS chunk slot this lane fills
  unsigned k_voff[4];                    // per-lane global byte offset of K loads, by (it & 3)
#pragma unroll
  for (int i = 0; i < 4; ++i)
    k_voff[i] = static_cast<unsigned>(ld_row * row_bytes) + ((ld_slot ^ ((4 * i + ld_row) & 15)) << 4);
  const unsigned v_voff = static_cast<unsigned>(ld_row * row_bytes) + ((ld_slot ^ (ld_row << 2)) << 4);

  // K operand read: row c32, chunk (2*ks + hf) ^ (c32 & 15)
  const int k_rd_base = c32 * kRowBytes + ((hf ^ (c32 & 1)) << 4);
  const int k_rd_xor = c32 & 14;
  // V transpose read: a group of 16 lanes reads 4 keys x 16 dcols
  const int li = lane & 15;
  const int grp_col = (lane >> 4) & 1;                  // which 16-column half of the 32-dcol block
  const int v_key_in = 4 * hf + (li >> 2);              // + 16 * j (+ 8)
  const int v_rd_base = v_key_in * kRowBytes + ((2 * grp_col + ((li & 3) >> 1)) << 4) + ((li & 1) << 3);
  const int v_q4 = li >> 2;                             // (row & 3) of the row this lane addresses

  floatx16 acc_o[4][RB];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc_o[db][rb][r] = 0.f;
  float ref[RB], run_sum[RB];        // reference logit (raw units) the exponentials are taken against; lane-partial sum
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    ref[rb] = -INFINITY;
    run_sum[rb] = 0.f;
  }
  const float c = p.scale_log2;
  const float lazy_raw = kLazyLog2 / c;      // the threshold in raw-logit units

  // First key of the 32 rows tile j loads.  The last tile of a ragged split is shifted
  // back so that it ends exactly at key_hi (no load ever leaves the prefix); its rows
  // below the tile's own first key were already handled by another tile and are masked.
  auto tile_key0 = [&](int j) { return key_lo + (wave + kWaves * j) * kTile; };
  auto tile_first_row = [&](int j) { return min(tile_key0(j), key_hi - kTile); };

  // The loads are issued through inline assembly on purpose: the compiler then does
  // not know that they write LDS and leaves the waiting to the explicit s_waitcnt,
  // instead of draining the whole load queue (and with it the prefetch of later
  // tiles) before the first LDS read of every tile.
  auto issue_tile = [&](const unsigned char* base, int j, unsigned dst, bool is_k) {
    const unsigned char* src = base + static_cast<int64_t>(tile_first_row(j)) * row_bytes;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const unsigned char* r = src + it * 4 * row_bytes;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :: "s"(dst + it * 1024), "v"(is_k ? k_voff[it & 3] : v_voff), "s"(r) : "memory", "m0");
    }
  };
  auto issue_k = [&](int j) { issue_tile(kbase, j, stage_lds + (j % kKSlots) * kTileBytes, true); };
  auto issue_v = [&](int j) { issue_tile(vbase, j, stage_lds + (kKSlots + j % kVSlots) * kTileBytes, false); };

  bf16x8 kf[8];
  auto read_k = [&](int j) {
    const unsigned char* kst = stage + (j % kKSlots) * kTileBytes + k_rd_base;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const uintx4 kw = *reinterpret_cast<const uintx4*>(kst + (((2 * ks) ^ k_rd_xor) << 4));
      kf[ks] = __builtin_bit_cast(bf16x8, kw);
    }
  };
  bf16x8 vf[4][2];
  auto read_v = [&](int j) {
    const unsigned char* vst = stage + (kKSlots + j % kVSlots) * kTileBytes + v_rd_base;
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      const unsigned char* col = vst + ((db ^ v_q4) << 6);
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4*)(col + (16 * jj) * kRowBytes));
        const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4*)(col + (16 * jj + 8) * kRowBytes));
        const shortx8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        vf[db][jj] = __builtin_bit_cast(bf16x8, both);
      }
    }
  };

  floatx16 s_v[RB];        // logits of the tile whose softmax comes next
  float tile_max[RB];
  bf16x8 pf[RB][2];

  // mask the rows of a shifted last tile that belong to an earlier tile, then the lane-local row max
  auto mask_and_max = [&](int j, bool may_be_shifted) {
    if (may_be_shifted) {
      const int key0 = tile_key0(j);
      const int first_row = tile_first_row(j);
      if (first_row < key0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = first_row + 8 * (r >> 2) + 4 * hf + (r & 3);
          if (key < key0) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) s_v[rb][r] = -INFINITY;
          }
        }
      }
    }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      float mx = fmaxf(s_v[rb][0], s_v[rb][1]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) mx = fmaxf(mx, fmaxf(s_v[rb][r], s_v[rb][r + 1]));
      tile_max[rb] = mx;
    }
  };
  // move the references up if some row of this wave outgrew its own by the lazy margin
  auto lazy_rescale = [&]() {
    bool grow = false;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) grow |= tile_max[rb] > ref[rb] + lazy_raw;
    if (__any(grow)) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const float mx = fmaxf(tile_max[rb], __shfl_xor(tile_max[rb], 32, 64));
        const float new_ref = fmaxf(ref[rb], mx);
        const float alpha = fast_exp2((ref[rb] - new_ref) * c);     // 0 on the first tile
        ref[rb] = new_ref;
        run_sum[rb] *= alpha;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc_o[db][rb][r] *= alpha;
      }
    }
  };
  // exponentials of s_v against the references -> P^T fragments, row sums, score blocks
  auto exp_and_pack = [&](int j) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const float mc = ref[rb] * c;
      float part = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pr = fast_exp2(fmaf(s_v[rb][r], c, -mc));
        s_v[rb][r] = pr;
        part += pr;
      }
      run_sum[rb] += part;
      if (SCORES) {
        const float tot = part + __shfl_xor(part, 32, 64);
        const int m = row0 + 32 * rb + c32;
        if (hf == 0 && m < p.M) {
          float* cp = p.chunk_part + ((static_cast<int64_t>(g) * p.n_sub + tile_key0(j) / kTile) * p.M + m) * 2;
          *reinterpret_cast<floatx2*>(cp) = floatx2{tot, mc};
        }
      }
      pf[rb][0] = pack8(s_v[rb], 0);
      pf[rb][1] = pack8(s_v[rb], 8);
    }
  };
  // S^T = K Q^T for the tile whose K fragments are in kf
  auto qk = [&](floatx16 (&acc_s)[RB]) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc_s[rb][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        acc_s[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[rb][ks], acc_s[rb], 0, 0, 0);
  };
  auto pv = [&]() {
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          acc_o[db][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db][jj], pf[rb][jj], acc_o[db][rb], 0, 0, 0);
  };

  if (n > 0) {
    // prologue: fill the rings (K0 V0 K1 V1 K2, and K3 once K0 has left its slot), logits of tile 0
    issue_k(0);
    issue_v(0);
    if (n > 1) {
      issue_k(1);
      issue_v(1);
    }
    if (n > 2) issue_k(2);
    wait_vm_groups(1 + (n > 1 ? 2 : 0) + (n > 2 ? 1 : 0));     // K0 landed
    read_k(0);
    qk(s_v);
    if (n > 3) {
      __builtin_amdgcn_sched_barrier(0);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      issue_k(3);                                              // K3 shares the ring slot of K0
      __builtin_amdgcn_sched_barrier(0);
    }
    mask_and_max(0, true);

    // Steady state for tile j: the logits of tile j sit in s_v.  While the matrix cores
    // compute the logits of tile j+1, the vector ALUs turn s_v into P(j); then P(j) V(j)
    // runs on the matrix cores while the row maxima of tile j+1 are taken.  Loads issued
    // in iteration i are V(i+2) then K(i+4), so at the top of iteration j the operations
    // younger than the needed V(j) and K(j+1) are K(j+2), V(j+1), K(j+3).
    int j = 0;
    // iterations whose loads all exist and whose next tile cannot be the shifted one: no branches
    for (; j + 4 < n; ++j) {
      asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
      read_v(j);
      read_k(j + 1);
      lazy_rescale();
      floatx16 s_next[RB];
      exp_and_pack(j);
      qk(s_next);
#pragma unroll
      for (int i = 0; i < 16; ++i) {             // one matrix op, then its share of the softmax ALU work
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, RB * 4, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // both ring slots read above are in registers now
      issue_v(j + 2);
      issue_k(j + 4);
      __builtin_amdgcn_sched_barrier(0);
      pv();
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) s_v[rb] = s_next[rb];
      mask_and_max(j + 1, false);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
        __builtin_amdgcn_sched_group_barrier(0x002, RB, 1);
      }
    }
    // the last (up to four) iterations: loads and the next tile exist only conditionally
    for (; j < n; ++j) {
      wait_vm_groups((j + 2 < n ? 1 : 0) + (j + 1 < n ? 1 : 0) + (j + 3 < n ? 1 : 0));
      read_v(j);
      const bool has_next = j + 1 < n;
      if (has_next) read_k(j + 1);
      lazy_rescale();
      exp_and_pack(j);
      if (has_next) {
        floatx16 s_next[RB];
        qk(s_next);
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (j + 2 < n) issue_v(j + 2);
        if (j + 4 < n) issue_k(j + 4);
        __builtin_amdgcn_sched_barrier(0);
        pv();
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) s_v[rb] = s_next[rb];
        mask_and_max(j + 1, true);
      } else {
        pv();
      }
    }
  }

  // ---- merge the four waves' partials through LDS; wave w finishes dcols 32w..32w+31 ----
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    run_sum[rb] += __shfl_xor(run_sum[rb], 32, 64);
    ref[rb] = fmaxf(ref[rb], __shfl_xor(ref[rb], 32, 64));      // both lanes of a pair hold the same value already
  }
  __syncthreads();                                  // every wave is done with its staging area
  float* dump = reinterpret_cast<float*>(lds);
  float* ml = dump + kWaves * kMergeFloatsPerWave;  // [wave][rb][2][32]
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        dump[wave * kMergeFloatsPerWave + ((db * 2 + rb) * 16 + r) * 64 + lane] = acc_o[db][rb][r];
  if (hf == 0) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      ml[((wave * 2 + rb) * 2 + 0) * 32 + c32] = ref[rb] * c;
      ml[((wave * 2 + rb) * 2 + 1) * 32 + c32] = run_sum[rb];
    }
  }
  __syncthreads();
  const int db = wave;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float mw[kWaves], lw[kWaves];
    float m_tot = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      mw[w] = ml[((w * 2 + rb) * 2 + 0) * 32 + c32];
      lw[w] = ml[((w * 2 + rb) * 2 + 1) * 32 + c32];
      m_tot = fmaxf(m_tot, mw[w]);
    }
    float l_tot = 0.f;
    float o[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) o[r] = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float wgt = lw[w] > 0.f ? fast_exp2(mw[w] - m_tot) : 0.f;   // a wave without tiles contributes nothing
      l_tot = fmaf(lw[w], wgt, l_tot);
#pragma unroll
      for (int r = 0; r < 16; ++r)
        o[r] = fmaf(dump[w * kMergeFloatsPerWave + ((db * 2 + rb) * 16 + r) * 64 + lane], wgt, o[r]);
    }
    const int m = row0 + 32 * rb + c32;
    if (m < p.M) {
      const int64_t slot = static_cast<int64_t>(split) * p.Hq * p.T + g * p.M + m;
      float* po = p.part_o + slot * kD + 32 * db + 4 * hf;
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4)
        *reinterpret_cast<floatx4*>(po + 8 * r4) = floatx4{o[4 * r4], o[4 * r4 + 1], o[4 * r4 + 2], o[4 * r4 + 3]};
      if (db == 0 && hf == 0) {
        p.part_ml[slot * 2] = m_tot;
        p.part_ml[slot * 2 + 1] = l_tot;
      }
    }
  }
}

template <int RB, bool SCORES>
hipError_t launch_one(const AttnParams& p, hipStream_t stream) {
  // the kernel needs more than the default 64 KB of dynamic LDS: raise the cap once per device
  static std::atomic<bool> attr_set[64];
  auto kernel = prefix_mfma_kernel<RB, SCORES>;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!attr_set[dev].load(std::memory_order_acquire)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    attr_set[dev].store(true, std::memory_order_release);
  }
  dim3 grid(p.S, p.Hkv, (p.M + 32 * RB - 1) / (32 * RB));
  kernel<<<grid, dim3(kWaves * 64), kLdsBytes, stream>>>(p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_prefix_mfma(const AttnParams& p, hipStream_t stream) {
  if (p.S <= 0) return hipSuccess;
  // one 32-row block per workgroup (problems with more rows take the row-split kernel)
  return p.want_scores ? launch_one<1, true>(p, stream) : launch_one<1, false>(p, stream);
}

}  // namespace specext
