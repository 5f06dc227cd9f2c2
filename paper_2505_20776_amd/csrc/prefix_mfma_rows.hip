// Prefix pass of Hybrid Tree Attention (SpecExtend Sec. 3.1) on the gfx950
// matrix cores, row-split form: bf16 K/V streamed ONCE from HBM into ONE compute
// unit each, fp32 accumulation.  Used when a KV head has more than 64 query rows
// (tree nodes x heads in the GQA group); smaller problems take the key-split kernel.
//
// Why this shape.  Measured on MI355X: a compute unit takes in only about 30 GB/s
// (the whole chip about 7.5 TB/s, whether the data comes from L2 or from HBM), so
// every K/V byte must enter exactly one compute unit; and a lone wave per SIMD
// overlaps its matrix and vector instructions poorly, while two waves per SIMD
// overlap them well.  Hence:
//   grid  = (splits, KV heads, row groups of 32*WAVES rows)
//   block = WAVES (8 or 4) wavefronts, at most 256 registers each, so that two
//           waves share a SIMD; wave w owns rows [32w, 32w+32) of the row group and
//           keeps their queries and running output in registers.
//   The split's keys are walked in tiles of 32.  K and V tiles are filled by direct
//   global->LDS loads into two rings of kRing tiles (every wave issues its share of
//   every tile), one workgroup barrier per tile, and every wave reads every tile.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, everything transposed so that a
// lane owns one query row in both products):
//   S^T[key][row]   = K[key][:] . Q[row][:]          A = K tile (LDS), B = Q (registers)
//   O^T[dcol][row] += V^T[dcol][key] P^T[key][row]   A = V^T (LDS transpose read
//   ds_read_b64_tr_b16), B = P^T taken straight from the S^T accumulator registers:
//   the key order that layout implies is used as the contraction order and V is
//   fetched in that same order, so P never moves between lanes.
#include "mfma_util.h"

namespace specext {
namespace {

constexpr int kTile = 32;                         // keys per tile
constexpr int kD = 128;                           // head_dim this kernel is written for
constexpr int kRowBytes = kD * 2;                 // one bf16 K or V row in LDS
constexpr int kTileBytes = kTile * kRowBytes;     // 8 KB
#ifndef SPECEXT_ROWS_RING
#define SPECEXT_ROWS_RING 4
#endif
constexpr int kRing = SPECEXT_ROWS_RING;          // tiles per ring (K ring and V ring)
constexpr int kPatchStride = 64 + 4;              // floats per row of the output staging patch (padded against bank conflicts)
constexpr int kRingBytes = 2 * kRing * kTileBytes;
constexpr int lds_bytes(int waves) { return kRingBytes > waves * 32 * kPatchStride * 4 ? kRingBytes : waves * 32 * kPatchStride * 4; }
#ifndef SPECEXT_ROWS_SKEW
#define SPECEXT_ROWS_SKEW 0
#endif
constexpr bool kSkewHalves = SPECEXT_ROWS_SKEW != 0;   // upper half of the waves runs half a tile behind

template <int WAVES, bool SCORES>
__global__ __launch_bounds__(WAVES * 64) void prefix_rows_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  constexpr int kLoadsPerWave = 8 / WAVES;       // 1 KB blocks of a tile that one wave fills (per K or V)

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c32 = lane & 31;
  const int hf = lane >> 5;

  const int split = blockIdx.x;
  const int g = blockIdx.y;
  const int row0 = blockIdx.z * (WAVES * 32) + wave * 32;
  const int m = row0 + c32;                      // this lane's query row of the KV head

  const int key_lo = split * p.keys_per_split;
  const int key_hi = min(p.L, key_lo + p.keys_per_split);
  const int n = (key_hi - key_lo + kTile - 1) / kTile;          // tiles of this split (>= 1)

  const int64_t row_bytes = p.kp_sl * 2;
  const unsigned char* kbase = static_cast<const unsigned char*>(p.kp) + static_cast<int64_t>(g) * p.kp_sh * 2;
  const unsigned char* vbase = static_cast<const unsigned char*>(p.vp) + static_cast<int64_t>(g) * p.kp_sh * 2;

  // ---- LDS rings.  A tile is 32 rows x 256 B; one direct load writes 1 KB = 4
  // consecutive rows, lane i landing at byte 16*i.  The 16-byte chunks of a row are
  // XOR-swizzled (K: chunk ^ (row & 15), V: chunk ^ ((row & 3) << 2)) so that the
  // operand reads are bank-conflict free; the LDS side of a direct load being fixed,
  // the swizzle is applied to the global address.
  unsigned char* kring = lds;
  unsigned char* vring = lds + kRing * kTileBytes;
  const unsigned kring_lds = static_cast<unsigned>(reinterpret_cast<uintptr_t>((lds_void*)kring));
  const unsigned vring_lds = kring_lds + kRing * kTileBytes;
  const int ld_row = lane >> 4;          // row within the 4-row block of one load
  const int ld_slot = lane & 15;         // LDS chunk slot this lane fills
  unsigned k_voff[kLoadsPerWave];
#pragma unroll
  for (int u = 0; u < kLoadsPerWave; ++u)
    k_voff[u] = static_cast<unsigned>(ld_row * row_bytes) +
                ((ld_slot ^ ((4 * (kLoadsPerWave * wave + u) + ld_row) & 15)) << 4);
  const unsigned v_voff = static_cast<unsigned>(ld_row * row_bytes) + ((ld_slot ^ (ld_row << 2)) << 4);

  // First key of the 32 rows tile t loads.  The last tile of a ragged split is shifted
  // back so that it ends exactly at key_hi (no load ever leaves the prefix); its rows
  // below the tile's own first key belong to the tile before and are masked.
  auto tile_key0 = [&](int t) { return key_lo + t * kTile; };
  auto tile_first_row = [&](int t) { return min(tile_key0(t), key_hi - kTile); };
  auto issue_tile = [&](int t) {                  // this wave's share of K(t), then of V(t)
    const int64_t off = static_cast<int64_t>(tile_first_row(t)) * row_bytes;
    const unsigned slot = (t % kRing) * kTileBytes;
#pragma unroll
    for (int u = 0; u < kLoadsPerWave; ++u) {
      const int blk = kLoadsPerWave * wave + u;
      load_to_lds_16(kring_lds + slot + blk * 1024, k_voff[u], kbase + off + blk * 4 * row_bytes);
    }
#pragma unroll
    for (int u = 0; u < kLoadsPerWave; ++u) {
      const int blk = kLoadsPerWave * wave + u;
      load_to_lds_16(vring_lds + slot + blk * 1024, v_voff, vbase + off + blk * 4 * row_bytes);
    }
  };

  // prologue: the first kRing-2 tiles are requested, and in between the queries
  // (B operand of S^T: lane = row c32, 8 consecutive d per k-step) with plain loads
  // in inline assembly, so that waiting for them does not drain the tile prefetch
  issue_tile(0);
  bf16x8 qf[8];
  {
    const int mq = min(m, p.M - 1);               // padding rows repeat the last real row (never stored)
    const uint16_t* qp =
        static_cast<const uint16_t*>(p.q) + (mq / p.G) * p.q_st + (g * p.G + mq % p.G) * p.q_sh + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(qf[ks]) : "v"(qp + 16 * ks) : "memory");
  }
  int younger = 0;                                // load instructions issued after the query loads
#pragma unroll
  for (int t = 1; t < kRing - 2; ++t) {
    if (t < n) {
      issue_tile(t);
      younger += 2 * kLoadsPerWave;
    }
  }
  wait_vmcnt_even(younger);                       // tile 0 (this wave's share) and the queries have landed
  asm volatile("" : "+v"(qf[0]), "+v"(qf[1]), "+v"(qf[2]), "+v"(qf[3]), "+v"(qf[4]), "+v"(qf[5]), "+v"(qf[6]),
                    "+v"(qf[7]) :: "memory");     // no use of the fragments may move above the wait

  // K operand read: row c32, chunk (2*ks + hf) ^ (c32 & 15)
  const int k_rd_base = c32 * kRowBytes + ((hf ^ (c32 & 1)) << 4);
  const int k_rd_xor = c32 & 14;
  // V transpose read: a group of 16 lanes reads 4 keys x 16 dcols
  const int li = lane & 15;
  const int grp_col = (lane >> 4) & 1;                  // which 16-column half of the 32-dcol block
  const int v_key_in = 4 * hf + (li >> 2);              // + 16 * jj (+ 8)
  const int v_rd_base = v_key_in * kRowBytes + ((2 * grp_col + ((li & 3) >> 1)) << 4) + ((li & 1) << 3);
  const int v_q4 = li >> 2;                             // (row & 3) of the row this lane addresses

  floatx16 acc_o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_o[db][r] = 0.f;
  float ref = -INFINITY;       // reference logit (raw units) the exponentials are taken against
  float run_sum = 0.f;         // lane-partial row sum
  const float c = p.scale_log2;
  const float lazy_raw = kLazyLog2 / c;      // the lazy margin in raw-logit units
  const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // Each wave's loads form the sequence K0 V0 K1 V1 ... (kLoadsPerWave instructions per
  // entry).  After barrier j every wave is done with tile j-2 (see the skew below), so
  // tile j-2+kRing is requested into that slot; before iteration j the tiles up to
  // min(j + kRing - 3, n - 1) have been requested and tile j is needed.
  auto top = [&](int j) {
    const int younger_tiles = min(j + kRing - 3, n - 1) - j;
    if (younger_tiles == kRing - 3) {
      asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * kLoadsPerWave * (kRing - 3)) : "memory");
    } else {
      wait_vmcnt_even(2 * kLoadsPerWave * younger_tiles);
    }
    lds_barrier();            // every share of tile j has landed
    if (j - 2 + kRing < n) issue_tile(j - 2 + kRing);
  };

  floatx16 s;                  // logits, then probabilities, of the tile in flight
  bf16x8 vf[4][2];             // its V^T fragments
  // first half of a tile: logits, V^T fragments requested, shifted-tile mask
  auto logits = [&](int j) {
    const unsigned char* kst = kring + (j % kRing) * kTileBytes + k_rd_base;
    s = zero16;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const uintx4 kw = *reinterpret_cast<const uintx4*>(kst + (((2 * ks) ^ k_rd_xor) << 4));
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kw), qf[ks], s, 0, 0, 0);
    }
    const unsigned char* vst = vring + (j % kRing) * kTileBytes + v_rd_base;
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
    const int key0 = tile_key0(j);
    const int first_row = tile_first_row(j);
    if (first_row < key0) {          // rows of a shifted last tile that belong to the tile before
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = first_row + 8 * (r >> 2) + 4 * hf + (r & 3);
        if (key < key0) s[r] = -INFINITY;
      }
    }
  };
  // second half: online softmax (one query row per lane pair, the reference moves
  // lazily), then O^T += V^T P^T
  auto softmax_pv = [&](int j) {
    float mx = fmaxf(s[0], s[1]);
#pragma unroll
    for (int r = 2; r < 16; r += 2) mx = fmaxf(mx, fmaxf(s[r], s[r + 1]));
    if (__any(mx > ref + lazy_raw)) {     // some row of this wave outgrew its reference: move every reference up
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float new_ref = fmaxf(ref, mx);
      const float alpha = fast_exp2((ref - new_ref) * c);     // 0 on the first tile
      ref = new_ref;
      run_sum *= alpha;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[db][r] *= alpha;
    }
    const float mc = ref * c;
    float part = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      s[r] = fast_exp2(fmaf(s[r], c, -mc));
      part += s[r];
    }
    run_sum += part;
    if (SCORES) {
      const float tot = part + __shfl_xor(part, 32, 64);
      if (hf == 0 && m < p.M) {
        float* cp = p.chunk_part + ((static_cast<int64_t>(g) * p.n_sub + tile_key0(j) / kTile) * p.M + m) * 2;
        *reinterpret_cast<floatx2*>(cp) = floatx2{tot, mc};
      }
    }
    const bf16x8 pf0 = pack8(s, 0);
    const bf16x8 pf1 = pack8(s, 8);
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db][0], pf0, acc_o[db], 0, 0, 0);
      acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db][1], pf1, acc_o[db], 0, 0, 0);
    }
  };

  // The waves of the upper half of the workgroup run half a tile behind the lower
  // half: between two barriers the lower half does logits(j) then softmax_pv(j), the
  // upper half softmax_pv(j-1) then logits(j).  The two waves that share a SIMD (w and
  // w + WAVES/2) are thus in different phases, and one's matrix work overlaps the
  // other's vector work.  Both halves pass the same n barriers.
  if (!kSkewHalves || wave < WAVES / 2) {
    for (int j = 0; j < n; ++j) {
      top(j);
      logits(j);
      softmax_pv(j);
    }
  } else {
    top(0);
    logits(0);
    for (int j = 1; j < n; ++j) {
      top(j);
      softmax_pv(j - 1);
      logits(j);
    }
    softmax_pv(n - 1);
  }

  // ---- partial results of this split: unnormalised O, reference (base-2 units) and row sum.
  // O^T sits in registers with a lane owning one row; it goes through a wave-private
  // LDS patch (two halves of 64 columns) so that the global stores are 256-byte runs.
  const float l_tot = run_sum + __shfl_xor(run_sum, 32, 64);
  lds_barrier();                                   // every wave is done with the tile rings
  float* patch = reinterpret_cast<float*>(lds) + wave * (32 * kPatchStride);
  const int64_t slot0 = static_cast<int64_t>(split) * p.Hq * p.T + g * p.M + row0;     // slot of the wave's first row
  const int rows_here = min(32, p.M - row0);       // <= 0 for a wave of padding rows only
#pragma unroll
  for (int half = 0; half < 2; ++half) {
#pragma unroll
    for (int d2 = 0; d2 < 2; ++d2) {
      const int db = 2 * half + d2;
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4)
        *reinterpret_cast<floatx4*>(patch + c32 * kPatchStride + 32 * d2 + 8 * r4 + 4 * hf) =
            floatx4{acc_o[db][4 * r4], acc_o[db][4 * r4 + 1], acc_o[db][4 * r4 + 2], acc_o[db][4 * r4 + 3]};
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int row = 4 * it + (lane >> 4);
      const floatx4 v = *reinterpret_cast<const floatx4*>(patch + row * kPatchStride + 4 * (lane & 15));
      if (row < rows_here)
        *reinterpret_cast<floatx4*>(p.part_o + (slot0 + row) * kD + 64 * half + 4 * (lane & 15)) = v;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
  }
  if (hf == 0 && m < p.M) {
    p.part_ml[(slot0 + c32) * 2] = ref * c;
    p.part_ml[(slot0 + c32) * 2 + 1] = l_tot;
  }
}

template <int WAVES, bool SCORES>
hipError_t launch_rows(const AttnParams& p, hipStream_t stream) {
  auto kernel = prefix_rows_kernel<WAVES, SCORES>;
  constexpr int kLdsBytes = lds_bytes(WAVES);
  if (kLdsBytes > 64 * 1024) {
    // more than the default 64 KB of dynamic LDS: raise the cap once per device
    static std::atomic<bool> attr_set[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!attr_set[dev].load(std::memory_order_acquire)) {
      const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
      if (e != hipSuccess) return e;
      attr_set[dev].store(true, std::memory_order_release);
    }
  }
  const int rows_per_wg = WAVES * 32;
  dim3 grid(p.S, p.Hkv, (p.M + rows_per_wg - 1) / rows_per_wg);
  kernel<<<grid, dim3(WAVES * 64), kLdsBytes, stream>>>(p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_prefix_mfma_rows(const AttnParams& p, hipStream_t stream) {
  if (p.S <= 0) return hipSuccess;
  if (p.rows_per_group == 256) {
    return p.want_scores ? launch_rows<8, true>(p, stream) : launch_rows<8, false>(p, stream);
  }
  return p.want_scores ? launch_rows<4, true>(p, stream) : launch_rows<4, false>(p, stream);
}

}  // namespace specext
