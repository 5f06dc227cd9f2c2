// Prefix pass of Hybrid Tree Attention (SpecExtend Sec. 3.1) on the gfx950
// matrix cores, row-split form: bf16 K/V streamed ONCE from HBM into ONE compute
// unit each, fp32 accumulation.  Used when a KV head has more than 64 query rows
// (tree nodes x heads in the GQA group); smaller problems take the key-split kernel.
//
// Why this shape: a compute unit can take in only about 30 GB/s (the whole chip
// about 7.5 TB/s, measured, whether the data comes from L2 or from HBM), so every
// K/V byte must enter exactly one compute unit.  That compute unit therefore owns
// all query rows of the KV head for its slice of the prefix:
//   grid  = (splits, KV heads, row groups of 128*RB rows)
//   block = 4 wavefronts; wave w owns rows [32*RB*w, 32*RB*(w+1)) of the row group
//           and keeps their queries and running output in registers.
//   The split's keys are walked in tiles of 32.  K and V tiles are filled by direct
//   global->LDS loads into two rings of kRing tiles (each wave issues a quarter of
//   every tile), one workgroup barrier per tile, and every wave reads every tile.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, everything transposed so that a
// lane owns one query row in both products):
//   S^T[key][row]   = K[key][:] . Q[row][:]          A = K tile (LDS), B = Q (registers)
//   O^T[dcol][row] += V^T[dcol][key] P^T[key][row]   A = V^T (LDS transpose read
//   ds_read_b64_tr_b16), B = P^T taken straight from the S^T accumulator registers:
//   the key order that layout implies is used as the contraction order and V is
//   fetched in that same order, so P never moves between lanes.
// Software pipeline per tile j: exponentials of tile j on the vector ALUs while the
// matrix cores compute the logits of tile j+1, then P(j) V(j) on the matrix cores
// while the row maxima of tile j+1 are taken.
#include "mfma_util.h"

namespace specext {
namespace {

constexpr int kWaves = 4;
constexpr int kTile = 32;                         // keys per tile
constexpr int kD = 128;                           // head_dim this kernel is written for
constexpr int kRowBytes = kD * 2;                 // one bf16 K or V row in LDS
constexpr int kTileBytes = kTile * kRowBytes;     // 8 KB
#ifndef SPECEXT_ROWS_RING
#define SPECEXT_ROWS_RING 4
#endif
constexpr int kRing = SPECEXT_ROWS_RING;          // tiles per ring (K ring and V ring)
constexpr int kLdsBytes = 2 * kRing * kTileBytes; // 128 KB

template <int RB, bool SCORES>
__global__ __launch_bounds__(kWaves * 64) void prefix_rows_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c32 = lane & 31;
  const int hf = lane >> 5;

  const int split = blockIdx.x;
  const int g = blockIdx.y;
  const int row0 = blockIdx.z * (kWaves * 32 * RB) + wave * (32 * RB);

  const int key_lo = split * p.keys_per_split;
  const int key_hi = min(p.L, key_lo + p.keys_per_split);
  const int n = (key_hi - key_lo + kTile - 1) / kTile;          // tiles of this split (>= 1)

  const int64_t row_bytes = p.kp_sl * 2;
  const unsigned char* kbase = static_cast<const unsigned char*>(p.kp) + static_cast<int64_t>(g) * p.kp_sh * 2;
  const unsigned char* vbase = static_cast<const unsigned char*>(p.vp) + static_cast<int64_t>(g) * p.kp_sh * 2;

  // ---- Q fragments (B operand of S^T): lane = row c32, 8 consecutive d per k-step.
  // Loaded with inline assembly further down (after the first K tile has been
  // requested) so that waiting for them does not also wait for the tile prefetch.
  bf16x8 qf[RB][8];

  // ---- LDS rings.  A tile is 32 rows x 256 B; one direct load writes 1 KB = 4
  // consecutive rows, lane i landing at byte 16*i.  The 16-byte chunks of a row are
  // XOR-swizzled (K: chunk ^ (row & 15), V: chunk ^ ((row & 3) << 2)) so that the
  // operand reads are bank-conflict free; the LDS side of a direct load being fixed,
  // the swizzle is applied to the global address.  Wave w fills blocks 2w and 2w+1
  // (rows 8w .. 8w+7) of every tile.
  unsigned char* kring = lds;
  unsigned char* vring = lds + kRing * kTileBytes;
  const unsigned kring_lds = static_cast<unsigned>(reinterpret_cast<uintptr_t>((lds_void*)kring));
  const unsigned vring_lds = kring_lds + kRing * kTileBytes;
  const int ld_row = lane >> 4;          // row within the 4-row block of one load
  const int ld_slot = lane & 15;         // LDS chunk slot this lane fills
  unsigned k_voff[2];
#pragma unroll
  for (int u = 0; u < 2; ++u)
    k_voff[u] = static_cast<unsigned>(ld_row * row_bytes) + ((ld_slot ^ ((4 * (2 * wave + u) + ld_row) & 15)) << 4);
  const unsigned v_voff = static_cast<unsigned>(ld_row * row_bytes) + ((ld_slot ^ (ld_row << 2)) << 4);

  // First key of the 32 rows tile t loads.  The last tile of a ragged split is shifted
  // back so that it ends exactly at key_hi (no load ever leaves the prefix); its rows
  // below the tile's own first key belong to the tile before and are masked.
  auto tile_key0 = [&](int t) { return key_lo + t * kTile; };
  auto tile_first_row = [&](int t) { return min(tile_key0(t), key_hi - kTile); };
  auto issue_k = [&](int t) {
    const unsigned char* src = kbase + static_cast<int64_t>(tile_first_row(t)) * row_bytes;
    const unsigned dst = kring_lds + (t % kRing) * kTileBytes;
#pragma unroll
    for (int u = 0; u < 2; ++u)
      load_to_lds_16(dst + (2 * wave + u) * 1024, k_voff[u], src + (2 * wave + u) * 4 * row_bytes);
  };
  auto issue_v = [&](int t) {
    const unsigned char* src = vbase + static_cast<int64_t>(tile_first_row(t)) * row_bytes;
    const unsigned dst = vring_lds + (t % kRing) * kTileBytes;
#pragma unroll
    for (int u = 0; u < 2; ++u)
      load_to_lds_16(dst + (2 * wave + u) * 1024, v_voff, src + (2 * wave + u) * 4 * row_bytes);
  };

  // K operand read: row c32, chunk (2*ks + hf) ^ (c32 & 15)
  const int k_rd_base = c32 * kRowBytes + ((hf ^ (c32 & 1)) << 4);
  const int k_rd_xor = c32 & 14;
  // V transpose read: a group of 16 lanes reads 4 keys x 16 dcols
  const int li = lane & 15;
  const int grp_col = (lane >> 4) & 1;                  // which 16-column half of the 32-dcol block
  const int v_key_in = 4 * hf + (li >> 2);              // + 16 * jj (+ 8)
  const int v_rd_base = v_key_in * kRowBytes + ((2 * grp_col + ((li & 3) >> 1)) << 4) + ((li & 1) << 3);
  const int v_q4 = li >> 2;                             // (row & 3) of the row this lane addresses

  bf16x8 kf[8];
  auto read_k = [&](int t) {
    const unsigned char* kst = kring + (t % kRing) * kTileBytes + k_rd_base;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const uintx4 kw = *reinterpret_cast<const uintx4*>(kst + (((2 * ks) ^ k_rd_xor) << 4));
      kf[ks] = __builtin_bit_cast(bf16x8, kw);
    }
  };
  bf16x8 vf[4][2];
  auto read_v = [&](int t) {
    const unsigned char* vst = vring + (t % kRing) * kTileBytes + v_rd_base;
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

  // single-fragment forms of the two reads, for the pipelined loop that streams them
  auto read_k_frag = [&](const unsigned char* kst, int ks) {
    const uintx4 kw = *reinterpret_cast<const uintx4*>(kst + (((2 * ks) ^ k_rd_xor) << 4));
    return __builtin_bit_cast(bf16x8, kw);
  };
  auto read_v_frag = [&](const unsigned char* vst, int v) {          // v = 2 * db + jj
    const unsigned char* col = vst + (((v >> 1) ^ v_q4) << 6);
    const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4*)(col + (16 * (v & 1)) * kRowBytes));
    const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4*)(col + (16 * (v & 1) + 8) * kRowBytes));
    const shortx8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
  };

  floatx16 acc_o[4][RB];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc_o[db][rb][r] = 0.f;
  float ref[RB], run_sum[RB];        // reference logit (raw units) of the exponentials; lane-partial row sum
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    ref[rb] = -INFINITY;
    run_sum[rb] = 0.f;
  }
  const float c = p.scale_log2;
  const float lazy_raw = kLazyLog2 / c;      // the lazy margin in raw-logit units

  float tile_max[RB];
  bf16x8 pf[RB][2];

  auto mask_shifted = [&](floatx16 (&sv)[RB], int t) {
    const int key0 = tile_key0(t);
    const int first_row = tile_first_row(t);
    if (first_row < key0) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = first_row + 8 * (r >> 2) + 4 * hf + (r & 3);
        if (key < key0) {
#pragma unroll
          for (int rb = 0; rb < RB; ++rb) sv[rb][r] = -INFINITY;
        }
      }
    }
  };
  auto row_max = [&](const floatx16 (&sv)[RB]) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      float mx = fmaxf(sv[rb][0], sv[rb][1]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) mx = fmaxf(mx, fmaxf(sv[rb][r], sv[rb][r + 1]));
      tile_max[rb] = mx;
    }
  };
  auto lazy_rescale = [&]() {
    bool grow = false;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) grow |= tile_max[rb] > ref[rb] + lazy_raw;
    if (__any(grow)) {     // some row of this wave outgrew its reference: move every reference up
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
  auto store_score_block = [&](int rb, float part, float mc, int t) {
    const float tot = part + __shfl_xor(part, 32, 64);
    const int m = row0 + 32 * rb + c32;
    if (hf == 0 && m < p.M) {
      float* cp = p.chunk_part + ((static_cast<int64_t>(g) * p.n_sub + tile_key0(t) / kTile) * p.M + m) * 2;
      *reinterpret_cast<floatx2*>(cp) = floatx2{tot, mc};
    }
  };
  // exponentials of sv against the references -> P^T fragments, row sums, score blocks
  auto exp_and_pack = [&](floatx16 (&sv)[RB], int t) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const float mc = ref[rb] * c;
      float part = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pr = fast_exp2(fmaf(sv[rb][r], c, -mc));
        sv[rb][r] = pr;
        part += pr;
      }
      run_sum[rb] += part;
      if (SCORES) store_score_block(rb, part, mc, t);
      pf[rb][0] = pack8(sv[rb], 0);
      pf[rb][1] = pack8(sv[rb], 8);
    }
  };
  const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  auto qk = [&](floatx16 (&acc_s)[RB]) {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        acc_s[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[rb][ks], ks == 0 ? zero16 : acc_s[rb], 0, 0, 0);
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

  // One pipelined tile step with the instruction order pinned by scheduling barriers
  // (a lone wave per SIMD overlaps matrix and vector work only if the two kinds of
  // instruction alternate in its stream): the 8*RB matrix ops of the logits of tile
  // t+1 (into nxt) alternate with the exponentials of tile t (in cur), two values per
  // matrix op; then the 8*RB matrix ops of P(t) V(t) alternate with the row maxima of nxt.
  auto pipelined_step = [&](floatx16 (&cur)[RB], floatx16 (&nxt)[RB], int t) {
    const unsigned char* kst = kring + ((t + 1) % kRing) * kTileBytes + k_rd_base;
    const unsigned char* vst = vring + (t % kRing) * kTileBytes + v_rd_base;
    float mc[RB], part[RB];
    uintx4 pw[RB][2];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      mc[rb] = ref[rb] * c;
      part[rb] = 0.f;
    }
    bf16x8 kq[3], vq[3];           // operand fragments, read from LDS two steps ahead of their use
    kq[0] = read_k_frag(kst, 0);
    kq[1] = read_k_frag(kst, 1);
#pragma unroll
    for (int i = 0; i < 8 * RB; ++i) {
      const int ks = i / RB, rbm = i % RB;
      if (rbm == 0 && ks + 2 < 8) kq[(ks + 2) % 3] = read_k_frag(kst, ks + 2);
      if (i == 8 * RB - 2) vq[0] = read_v_frag(vst, 0);
      if (i == 8 * RB - 1) vq[1] = read_v_frag(vst, 1);
      nxt[rbm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kq[ks % 3], qf[rbm][ks], ks == 0 ? zero16 : nxt[rbm], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      const int rb = i / 8, r = 2 * (i % 8);
      const float p0 = fast_exp2(fmaf(cur[rb][r], c, -mc[rb]));
      const float p1 = fast_exp2(fmaf(cur[rb][r + 1], c, -mc[rb]));
      part[rb] += p0 + p1;
      const floatx2 f2 = {p0, p1};
      pw[rb][r / 8][(r % 8) / 2] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f2, bf16x2));
      if (i % 8 == 7) {
        run_sum[rb] += part[rb];
        if (SCORES) store_score_block(rb, part[rb], mc[rb], t);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      pf[rb][0] = __builtin_bit_cast(bf16x8, pw[rb][0]);
      pf[rb][1] = __builtin_bit_cast(bf16x8, pw[rb][1]);
    }
    float mx[RB];
#pragma unroll
    for (int i = 0; i < 8 * RB; ++i) {
      const int v = i / RB, rbm = i % RB;
      if (rbm == 0 && v + 2 < 8) vq[(v + 2) % 3] = read_v_frag(vst, v + 2);
      acc_o[v >> 1][rbm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vq[v % 3], pf[rbm][v & 1], acc_o[v >> 1][rbm], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      const int rb = i / 8, r = 2 * (i % 8);
      mx[rb] = r == 0 ? fmaxf(nxt[rb][0], nxt[rb][1]) : fmaxf(mx[rb], fmaxf(nxt[rb][r], nxt[rb][r + 1]));
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) tile_max[rb] = mx[rb];
  };

  // Each wave's loads form the sequence K0 V0 K1 V1 ... (two instructions per entry;
  // K(t) has index 2t, V(t) index 2t+1).  Before iteration j every entry with index
  // <= min(2(j + kRing - 1), 2n - 1) has been issued.
  auto last_issued = [&](int j) { return min(2 * (j + kRing - 1), 2 * n - 1); };

  // prologue: K0 first, then the queries, then V0 K1 V1 ... K(kRing-1)
  issue_k(0);
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int m = min(row0 + 32 * rb + c32, p.M - 1);       // padding rows repeat the last real row (never stored)
    const int t = m / p.G;
    const int h = g * p.G + m % p.G;
    const uint16_t* qp = static_cast<const uint16_t*>(p.q) + t * p.q_st + h * p.q_sh + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(qf[rb][ks]) : "v"(qp + 16 * ks) : "memory");
  }
  int issued_after_q = 0;                 // load instructions younger than the query loads
  if (0 < n) {
    issue_v(0);
    issued_after_q += 2;
  }
#pragma unroll
  for (int t = 1; t < kRing; ++t) {
    if (t < n) {
      issue_k(t);
      issued_after_q += 2;
      if (t < kRing - 1) {
        issue_v(t);
        issued_after_q += 2;
      }
    }
  }
  // K0 and the queries have landed (everything older than the loads counted above);
  // the fragments are operands of the wait so that no use of them can move above it
  wait_vmcnt_even(issued_after_q);
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
    asm volatile("" : "+v"(qf[rb][0]), "+v"(qf[rb][1]), "+v"(qf[rb][2]), "+v"(qf[rb][3]), "+v"(qf[rb][4]),
                      "+v"(qf[rb][5]), "+v"(qf[rb][6]), "+v"(qf[rb][7]) :: "memory");
  lds_barrier();                                // everybody's part of K0 has landed
  read_k(0);
  floatx16 s_a[RB], s_b[RB];       // logits of the current / the next tile, swapping roles
  qk(s_a);
  if (n == 1) mask_shifted(s_a, 0);
  row_max(s_a);

  auto top_of_iteration = [&](int jj) {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(4 * (kRing - 2)) : "memory");   // own parts of V(jj), K(jj+1) landed
    lds_barrier();                   // all parts landed; everyone is done with the slots of V(jj-1) and K(jj)
    issue_v(jj - 1 + kRing);
    issue_k(jj + kRing);
    lazy_rescale();
  };
  int j = 0;
  // steady state, two tiles per trip: every load still exists and no tile is the split's last
  for (; j + 1 + kRing < n; j += 2) {
    top_of_iteration(j);
    pipelined_step(s_a, s_b, j);
    top_of_iteration(j + 1);
    pipelined_step(s_b, s_a, j + 1);
  }
  // the remaining iterations: loads run out, the last tile may be shifted
  for (; j < n; ++j) {
    const bool has_next = j + 1 < n;
    const int need = has_next ? 2 * (j + 1) : 2 * j + 1;
    wait_vmcnt_even(2 * (last_issued(j) - need));
    lds_barrier();
    if (j - 1 + kRing < n) issue_v(j - 1 + kRing);
    if (j + kRing < n) issue_k(j + kRing);
    read_v(j);
    if (has_next) read_k(j + 1);
    lazy_rescale();
    exp_and_pack(s_a, j);
    if (has_next) {
      qk(s_b);
      pv();
      if (j + 2 == n) mask_shifted(s_b, j + 1);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) s_a[rb] = s_b[rb];
      row_max(s_a);
    } else {
      pv();
    }
  }

  // ---- partial results of this split: unnormalised O, reference (base-2 units) and row sum ----
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const float l_tot = run_sum[rb] + __shfl_xor(run_sum[rb], 32, 64);
    const int m = row0 + 32 * rb + c32;
    if (m < p.M) {
      const int64_t slot = static_cast<int64_t>(split) * p.Hq * p.T + g * p.M + m;
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        float* po = p.part_o + slot * kD + 32 * db + 4 * hf;
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
          *reinterpret_cast<floatx4*>(po + 8 * r4) = floatx4{acc_o[db][rb][4 * r4], acc_o[db][rb][4 * r4 + 1],
                                                             acc_o[db][rb][4 * r4 + 2], acc_o[db][rb][4 * r4 + 3]};
      }
      if (hf == 0) {
        p.part_ml[slot * 2] = ref[rb] * c;
        p.part_ml[slot * 2 + 1] = l_tot;
      }
    }
  }
}

template <int RB, bool SCORES>
hipError_t launch_rows(const AttnParams& p, hipStream_t stream) {
  // the kernel needs more than the default 64 KB of dynamic LDS: raise the cap once per device
  static std::atomic<bool> attr_set[64];
  auto kernel = prefix_rows_kernel<RB, SCORES>;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!attr_set[dev].load(std::memory_order_acquire)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    attr_set[dev].store(true, std::memory_order_release);
  }
  const int rows_per_wg = kWaves * 32 * RB;
  dim3 grid(p.S, p.Hkv, (p.M + rows_per_wg - 1) / rows_per_wg);
  kernel<<<grid, dim3(kWaves * 64), kLdsBytes, stream>>>(p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_prefix_mfma_rows(const AttnParams& p, hipStream_t stream) {
  if (p.S <= 0) return hipSuccess;
  if (p.rows_per_group == 256) {
    return p.want_scores ? launch_rows<2, true>(p, stream) : launch_rows<2, false>(p, stream);
  }
  return p.want_scores ? launch_rows<1, true>(p, stream) : launch_rows<1, false>(p, stream);
}

}  // namespace specext
