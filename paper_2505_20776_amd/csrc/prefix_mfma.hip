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
#include "common.h"

namespace specext {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float floatx2;
typedef __attribute__((ext_vector_type(4))) float floatx4;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((ext_vector_type(4))) short shortx4;
typedef __attribute__((ext_vector_type(8))) short shortx8;
typedef __attribute__((ext_vector_type(4))) uint32_t uintx4;

constexpr int kWaves = 4;
constexpr int kTile = 32;                         // keys per wave tile
constexpr int kD = 128;                           // head_dim this kernel is written for
constexpr int kRowBytes = kD * 2;                 // one bf16 K or V row
constexpr int kStageBytes = 2 * kTile * kRowBytes;  // K tile + V tile of one wave
constexpr int kMergeFloatsPerWave = 4 * 2 * 16 * 64;   // O^T dump at RB = 2
constexpr int kLdsBytes = kWaves * kMergeFloatsPerWave * 4 + kWaves * 2 * 2 * 32 * 4;

typedef __attribute__((address_space(3))) shortx4 lds_shortx4;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ bf16x8 pack8(const floatx16& v, int first) {
  bf16x8 out;
#pragma unroll
  for (int e = 0; e < 8; e += 2) {
    floatx2 f = {v[first + e], v[first + e + 1]};
    bf16x2 b = __builtin_convertvector(f, bf16x2);
    out[e] = b[0];
    out[e + 1] = b[1];
  }
  return out;
}

template <int RB, bool SCORES>
__global__ __launch_bounds__(kWaves * 64) void prefix_mfma_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int c32 = lane & 31;
  const int hf = lane >> 5;

  // blockIdx.x enumerates (row group, split, head) with the row group slowest, so
  // that ids of one (split, head) differ by a multiple of S * Hkv.
  const int split = blockIdx.x;
  const int g = blockIdx.y;
  const int row0 = blockIdx.z * (32 * RB);

  const int key_lo = split * p.keys_per_split;
  const int key_hi = min(p.L, key_lo + p.keys_per_split);
  const int n_tiles = (key_hi - key_lo + kTile - 1) / kTile;

  const uint16_t* __restrict__ kbase = static_cast<const uint16_t*>(p.kp) + static_cast<int64_t>(g) * p.kp_sh;
  const uint16_t* __restrict__ vbase = static_cast<const uint16_t*>(p.vp) + static_cast<int64_t>(g) * p.kp_sh;

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

  // ---- per-wave LDS staging: K tile then V tile, 32 rows x 256 B each, 16-byte
  // chunks XOR-swizzled so that the operand reads below are bank-conflict free ----
  unsigned char* kst = lds + wave * kStageBytes;
  unsigned char* vst = kst + kTile * kRowBytes;

  // global -> LDS mapping of one tile: 8 steps, step `it` covers keys 4*it .. 4*it+3
  const int ld_key = lane >> 4;        // + 4 * it
  const int ld_ch = lane & 15;
  // K operand read: row c32, chunk (2*ks + hf) ^ (c32 & 15)
  const int k_rd_base = c32 * kRowBytes + ((hf ^ (c32 & 1)) << 4);
  const int k_rd_xor = c32 & 14;
  // V transpose read: group of 16 lanes reads 4 keys x 16 dcols
  const int li = lane & 15;
  const int grp_col = (lane >> 4) & 1;                  // which 16-column half of the 32-dcol block
  const int v_key_in = 4 * hf + (li >> 2);              // + 16 * j (+ 8)
  const int v_rd_base = v_key_in * kRowBytes + ((2 * grp_col + ((li & 3) >> 1)) << 4) + ((li & 1) << 3);
  const int v_q4 = li >> 2;                             // (key & 3) of the row this lane addresses

  floatx16 acc_o[4][RB];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc_o[db][rb][r] = 0.f;
  float run_max[RB], run_sum[RB];                       // raw-logit max; lane-partial sum
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    run_max[rb] = -INFINITY;
    run_sum[rb] = 0.f;
  }
  const float c = p.scale_log2;

  uintx4 stage_k[8], stage_v[8];
  auto issue_loads = [&](int tile) {
    const int key0 = key_lo + tile * kTile;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int j = min(key0 + 4 * it + ld_key, p.L - 1);    // rows past the end repeat the last key
      const int64_t off = static_cast<int64_t>(j) * p.kp_sl + ld_ch * 8;
      stage_k[it] = *reinterpret_cast<const uintx4*>(kbase + off);
      stage_v[it] = *reinterpret_cast<const uintx4*>(vbase + off);
    }
  };

  int tile = wave;
  if (tile < n_tiles) issue_loads(tile);

  for (; tile < n_tiles; tile += kWaves) {
    // registers -> LDS (swizzled)
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int key = 4 * it + ld_key;
      *reinterpret_cast<uintx4*>(kst + key * kRowBytes + ((ld_ch ^ (key & 15)) << 4)) = stage_k[it];
      *reinterpret_cast<uintx4*>(vst + key * kRowBytes + ((ld_ch ^ ((key & 3) << 2)) << 4)) = stage_v[it];
    }
    const int next = tile + kWaves;
    if (next < n_tiles) issue_loads(next);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- S^T = K Q^T ----
    floatx16 acc_s[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc_s[rb][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const uintx4 kw = *reinterpret_cast<const uintx4*>(kst + k_rd_base + (((2 * ks) ^ k_rd_xor) << 4));
      const bf16x8 kf = __builtin_bit_cast(bf16x8, kw);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        acc_s[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[rb][ks], acc_s[rb], 0, 0, 0);
    }

    // ---- mask keys past the end of the split (last tile only) ----
    const int key0 = key_lo + tile * kTile;
    if (key0 + kTile > key_hi) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = key0 + 8 * (r >> 2) + 4 * hf + (r & 3);
        if (key >= key_hi) {
#pragma unroll
          for (int rb = 0; rb < RB; ++rb) acc_s[rb][r] = -INFINITY;
        }
      }
    }

    // ---- online softmax, one query row per lane pair ----
    float tile_max[RB];
    bool grow = false;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      float mx = acc_s[rb][0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, acc_s[rb][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      tile_max[rb] = mx;
      grow |= mx > run_max[rb];
    }
    if (__any(grow)) {     // the running max moved for some row of this wave: rescale (rare in steady state)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const float new_max = fmaxf(run_max[rb], tile_max[rb]);
        const float alpha = fast_exp2((run_max[rb] - new_max) * c);     // 0 on the first tile
        run_max[rb] = new_max;
        run_sum[rb] *= alpha;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc_o[db][rb][r] *= alpha;
      }
    }
    bf16x8 pf[RB][2];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const float mc = run_max[rb] * c;
      float part = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pr = fast_exp2(fmaf(acc_s[rb][r], c, -mc));
        acc_s[rb][r] = pr;
        part += pr;
      }
      run_sum[rb] += part;
      if (SCORES) {
        const float tot = part + __shfl_xor(part, 32, 64);
        const int m = row0 + 32 * rb + c32;
        if (hf == 0 && m < p.M) {
          float* cp = p.chunk_part + ((static_cast<int64_t>(g) * p.n_sub + key0 / kTile) * p.M + m) * 2;
          *reinterpret_cast<floatx2*>(cp) = floatx2{tot, mc};
        }
      }
      pf[rb][0] = pack8(acc_s[rb], 0);
      pf[rb][1] = pack8(acc_s[rb], 8);
    }

    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      const int col_off = v_rd_base + ((db ^ v_q4) << 6);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (lds_shortx4*)(vst + col_off + (16 * j) * kRowBytes));
        const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (lds_shortx4*)(vst + col_off + (16 * j + 8) * kRowBytes));
        const shortx8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        const bf16x8 vf = __builtin_bit_cast(bf16x8, both);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          acc_o[db][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[rb][j], acc_o[db][rb], 0, 0, 0);
      }
    }
    __builtin_amdgcn_wave_barrier();
  }

  // ---- merge the four waves' partials through LDS; wave w finishes dcols 32w..32w+31 ----
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) run_sum[rb] += __shfl_xor(run_sum[rb], 32, 64);
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
      ml[((wave * 2 + rb) * 2 + 0) * 32 + c32] = run_max[rb] * c;
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

bool prefix_mfma_supports(const AttnParams& p) { return p.use_mfma != 0; }

hipError_t launch_prefix_mfma(const AttnParams& p, hipStream_t stream) {
  if (p.S <= 0) return hipSuccess;
  if (p.rows_per_group == 64) {
    return p.want_scores ? launch_one<2, true>(p, stream) : launch_one<2, false>(p, stream);
  }
  return p.want_scores ? launch_one<1, true>(p, stream) : launch_one<1, false>(p, stream);
}

}  // namespace specext
