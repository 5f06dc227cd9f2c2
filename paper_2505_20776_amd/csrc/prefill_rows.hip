// Prefill attention (SpecExtend Sec. 3.1: FlashAttention for the prefill stage of the
// target and the draft model): exact causal self-attention with an online softmax, no
// score matrix in memory, on the gfx950 matrix cores.  bf16 Q/K/V, head_dim 128, fp32
// accumulation.
//
// Shape.  The query rows of a KV head (row m = token * G + head-in-group, as in the
// verification kernels) are cut into groups of 256; a workgroup of 8 wavefronts owns one
// group (wave w its rows [32w, 32w+32), queries and running output in registers) and
// walks the keys 0 .. position of the group's last token in tiles of 32.  K and V tiles
// arrive by direct global->LDS loads into two rings of kRing tiles, one workgroup barrier
// per tile, every wave reads every tile.  Only the tiles on the diagonal are masked
// (a key is hidden from a row whose token comes before it).  At the end every row is
// normalised and written as one 256-byte piece.
//
//   grid = (KV heads, row groups); row groups are taken from the last (longest key range)
//   to the first so that the long workgroups start first, and neighbouring workgroups in
//   dispatch order are the KV heads of one row group, which land on different XCDs: the
//   workgroups that share a head's K/V share an L2.
//
// Matrix-core mapping as in the verification prefix kernel: S^T = K Q^T (A = K tile from
// LDS, B = Q registers), O^T += V^T P^T (A = V^T by LDS transpose reads, B = P^T straight
// from the S^T accumulators), so that a lane owns one query row in both products.
#include "mfma_util.h"

namespace specext {
namespace {

constexpr int kTile = 32;
constexpr int kD = 128;
constexpr int kRowBytes = kD * 2;
constexpr int kTileBytes = kTile * kRowBytes;     // 8 KB
constexpr int kRing = 4;                          // tiles per ring (K ring and V ring)
constexpr int kRingBytes = 2 * kRing * kTileBytes;
constexpr int kWaves = 8;
// Behind the rings every wave has a private area: first the staging of its 32 query rows
// (32 x 256 B), at the end the staging of its 32 output rows, 256 bytes at a time (rows
// padded to 264 B so that the 8-byte column writes fall into distinct banks).
constexpr int kPatchStride = kRowBytes + 8;
constexpr int kPrivBytes = 32 * kPatchStride;
constexpr int kLdsBytes = kRingBytes + kWaves * kPrivBytes;
static_assert(kLdsBytes <= 160 * 1024, "rings and private areas must fit the 160 KB of LDS");
constexpr int kLoadsPerTile = 2;                  // direct loads per wave and tile: 1 KB of K, 1 KB of V

template <int I>
using ic = std::integral_constant<int, I>;
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(ic<I>{});
    static_for<I + 1, N>(f);
  }
}

__global__ __launch_bounds__(kWaves * 64) void prefill_rows_kernel(PrefillParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c32 = lane & 31;
  const int hf = lane >> 5;

  const int g = blockIdx.x;
  const int grp = gridDim.y - 1 - blockIdx.y;
  const int row0 = grp * (kWaves * 32) + wave * 32;
  const int m = row0 + c32;                                       // this lane's query row of the KV head
  const int m_last = min(p.M, (grp + 1) * (kWaves * 32)) - 1;      // last real row of the group
  const int key_hi = p.q_off + m_last / p.G + 1;                  // keys that row sees (<= N)
  const int load_hi = max(key_hi, kTile);                         // whole tiles are loaded; N >= 32
  const int n = (load_hi + kTile - 1) / kTile;                    // tiles of this workgroup
  const int my_pos = p.q_off + min(m, p.M - 1) / p.G;             // newest key this lane's row sees
  const int wave_first_pos = p.q_off + min(row0, p.M - 1) / p.G;  // ... the wave's first row sees

  const int64_t row_bytes = p.k_sl * 2;
  const unsigned char* kbase = static_cast<const unsigned char*>(p.k) + static_cast<int64_t>(g) * p.k_sh * 2;
  const unsigned char* vbase = static_cast<const unsigned char*>(p.v) + static_cast<int64_t>(g) * p.k_sh * 2;

  // LDS rings: a tile is 32 rows x 256 B; one direct load writes 1 KB = 4 consecutive rows,
  // lane i landing at byte 16*i.  The 16-byte chunks of a row are XOR-swizzled (K: chunk ^
  // (row & 15), V: chunk ^ ((row & 3) << 2)) so that the operand reads are free of bank
  // conflicts; the LDS side of a direct load being fixed, the swizzle is applied to the
  // global address.
  const unsigned kring_lds = static_cast<unsigned>(reinterpret_cast<uintptr_t>((lds_void*)lds));
  const unsigned vring_lds = kring_lds + kRing * kTileBytes;
  const int ld_row = lane >> 4;
  const int ld_slot = lane & 15;
  const unsigned k_voff = static_cast<unsigned>(ld_row * row_bytes) + ((ld_slot ^ ((4 * wave + ld_row) & 15)) << 4);
  const unsigned v_voff = static_cast<unsigned>(ld_row * row_bytes) + ((ld_slot ^ (ld_row << 2)) << 4);

  // Tile t covers keys [32t, 32t+32); the last tile is shifted back so that it ends exactly
  // at load_hi (no load leaves the cache); its rows below 32t belong to the tile before
  // and are masked.
  auto tile_first_row = [&](int t) { return min(t * kTile, load_hi - kTile); };
  auto issue_tile = [&](auto slot_c, int t) {
    constexpr unsigned slot = decltype(slot_c)::value * kTileBytes;
    const int64_t off = (static_cast<int64_t>(tile_first_row(t)) + 4 * wave) * row_bytes;
    load_to_lds_16(kring_lds + slot + wave * 1024, k_voff, kbase + off);
    load_to_lds_16(vring_lds + slot + wave * 1024, v_voff, vbase + off);
  };
  auto younger_than_tile = [&](int t) { return kLoadsPerTile * (min(t + kRing - 1, n) - min(t + 1, n)); };

  // prologue: tile 0, then the wave's queries, then tiles 1 .. kRing-2
  issue_tile(ic<0>{}, 0);
  const unsigned priv_lds = kring_lds + kRingBytes + wave * kPrivBytes;
  {
    // load u brings rows 4u..4u+3 of the wave (1 KB); the lane that fills LDS chunk slot
    // `ld_slot` of row r fetches chunk ld_slot ^ (r & 15) of that query row (the K swizzle,
    // so that the fragment reads below use the K read offsets)
    const int t0 = min(row0, p.M - 1) / p.G;
    const unsigned char* qbase = static_cast<const unsigned char*>(p.q) + static_cast<int64_t>(t0) * p.q_st * 2;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int r = 4 * u + ld_row;
      const int mq = min(row0 + r, p.M - 1);               // padding rows repeat the last real row (never stored)
      const int tq = mq / p.G;
      const int hq = g * p.G + (mq - tq * p.G);
      const unsigned voff = static_cast<unsigned>(((tq - t0) * p.q_st + hq * p.q_sh) * 2) + ((ld_slot ^ (r & 15)) << 4);
      load_to_lds_16(priv_lds + u * 1024, voff, qbase);
    }
  }
  static_for<1, kRing - 1>([&](auto u_c) {
    constexpr int u = decltype(u_c)::value;
    if (u < n) issue_tile(ic<u>{}, u);
  });

  // K operand read: row c32, chunk (2*ks + hf) ^ (c32 & 15)
  unsigned k_rd[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) k_rd[ks] = c32 * kRowBytes + ((((2 * ks) ^ (c32 & 14)) | (hf ^ (c32 & 1))) << 4);
  // V transpose read: a group of 16 lanes reads 4 keys x 16 dcols
  const int li = lane & 15;
  const int grp_col = (lane >> 4) & 1;
  const int v_key_in = 4 * hf + (li >> 2);
  const int v_q4 = li >> 2;
  unsigned v_rd[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
    v_rd[db] = kRing * kTileBytes + v_key_in * kRowBytes + ((db ^ v_q4) << 6) + ((2 * grp_col + ((li & 3) >> 1)) << 4) +
               ((li & 1) << 3);

  bf16x8 qf[8];
  unsigned char* priv = lds + kRingBytes + wave * kPrivBytes;
  floatx16 acc_o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_o[db][r] = 0.f;
  float ref = -INFINITY;       // reference logit (raw units) the exponentials are taken against
  float run_sum = 0.f;         // lane-partial row sum
  const float c = p.scale_log2;
  const float lazy_raw = kLazyLog2 / c;
  const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // One tile: logits, mask on the diagonal, online softmax (one query row per lane pair,
  // the reference moves lazily), O^T += V^T P^T.
  auto tile = [&](auto slot_c, int j) {
    constexpr int slot = decltype(slot_c)::value * kTileBytes;
    floatx16 s = zero16;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const uintx4 kw = *reinterpret_cast<const uintx4*>(lds + k_rd[ks] + slot);
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kw), qf[ks], s, 0, 0, 0);
    }
    bf16x8 vf[4][2];
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      const unsigned char* col = lds + v_rd[db] + slot;
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4*)(col + (16 * jj) * kRowBytes));
        const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4*)(col + (16 * jj + 8) * kRowBytes));
        const shortx8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        vf[db][jj] = __builtin_bit_cast(bf16x8, both);
      }
    }
    const int key0 = j * kTile;
    const int first_row = tile_first_row(j);
    if (first_row < key0 || first_row + kTile - 1 > wave_first_pos) {
      // register r holds key first_row + 4*hf + 8*(r/4) + r%4: hidden when it belongs to the
      // tile before (shifted last tile) or comes after this row's token
      const int lo_thr = key0 - first_row - 4 * hf;
      const int hi_thr = my_pos - first_row - 4 * hf;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int idx = 8 * (r >> 2) + (r & 3);
        if (idx < lo_thr || idx > hi_thr) s[r] = -INFINITY;
      }
    }
    float mx = fmaxf(s[0], s[1]);
#pragma unroll
    for (int r = 2; r < 16; r += 2) mx = fmaxf(mx, fmaxf(s[r], s[r + 1]));
    if (__any(mx > ref + lazy_raw)) {     // some row of this wave outgrew its reference: move every reference up
      mx = halves_max(mx);
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
    const bf16x8 pf0 = pack8(s, 0);
    const bf16x8 pf1 = pack8(s, 8);
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db][0], pf0, acc_o[db], 0, 0, 0);
      acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db][1], pf1, acc_o[db], 0, 0, 0);
    }
  };

  // Each wave's loads form the sequence (K, V of tile 0), (K, V of tile 1), ...  Before tile t
  // is read every wave waits for its own share of it and meets the others at a barrier; behind
  // that barrier every wave has also left tile t-1, whose ring slot takes tile t + kRing - 1.
  for (int t0 = 0; t0 < n; t0 += kRing) {
    static_for<0, kRing>([&](auto u_c) {
      constexpr int u = decltype(u_c)::value;
      const int t = t0 + u;
      if (t < n) {
        if (t == 0) {
          wait_vmcnt_even(younger_than_tile(0));           // also covers the wave's own queries
#pragma unroll
          for (int ks = 0; ks < 8; ++ks)
            qf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uintx4*>(priv + k_rd[ks]));
        } else if (t + kRing - 1 <= n) {
          asm volatile("s_waitcnt vmcnt(%0)" :: "n"(kLoadsPerTile * (kRing - 2)) : "memory");
        } else {
          wait_vmcnt_even(younger_than_tile(t));
        }
        lds_barrier();
        if (t + kRing - 1 < n) issue_tile(ic<(u + kRing - 1) % kRing>{}, t + kRing - 1);
        tile(ic<u>{}, t);
      }
    });
  }

  // ---- normalise and write.  O^T sits in registers with a lane owning one row; it goes
  // through the wave's private LDS area, 256 bytes per row at a time (all 128 columns as
  // bf16, or 64 columns as fp32), so that the global stores are whole 256-byte pieces.
  const float l_tot = halves_sum(run_sum);
  const float inv = 1.0f / l_tot;
  const int rows_here = min(32, p.M - row0);       // <= 0 for a wave of padding rows only
  const int passes = p.out_dtype == SPECEXT_BF16 ? 1 : 2;
  for (int pass = 0; pass < passes; ++pass) {
    if (pass == 1) __builtin_amdgcn_wave_barrier();
    if (p.out_dtype == SPECEXT_BF16) {
#pragma unroll
      for (int db = 0; db < 4; ++db) {
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          uintx2 w;
          const floatx2 f0 = {acc_o[db][4 * r4] * inv, acc_o[db][4 * r4 + 1] * inv};
          const floatx2 f1 = {acc_o[db][4 * r4 + 2] * inv, acc_o[db][4 * r4 + 3] * inv};
          w[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f0, bf16x2));
          w[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f1, bf16x2));
          *reinterpret_cast<uintx2*>(priv + c32 * kPatchStride + (32 * db + 8 * r4 + 4 * hf) * 2) = w;
        }
      }
    } else {
#pragma unroll
      for (int d2 = 0; d2 < 2; ++d2) {
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          floatx4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = (pass == 0 ? acc_o[d2][4 * r4 + e] : acc_o[2 + d2][4 * r4 + e]) * inv;
          // 16 bytes at column 32*d2 + 8*r4 + 4*hf of the 64-column half; rows padded by 8 B
          // are only 8-byte aligned, so two 8-byte writes
          unsigned char* dst = priv + c32 * kPatchStride + (32 * d2 + 8 * r4 + 4 * hf) * 4;
          *reinterpret_cast<floatx2*>(dst) = floatx2{w[0], w[1]};
          *reinterpret_cast<floatx2*>(dst + 8) = floatx2{w[2], w[3]};
        }
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int row = 4 * it + (lane >> 4);
      const uintx2* src = reinterpret_cast<const uintx2*>(priv + row * kPatchStride + 16 * (lane & 15));
      const uintx2 a = src[0], b = src[1];
      if (row < rows_here) {
        const int mr = row0 + row;
        const int tr = mr / p.G;
        const int hr = g * p.G + (mr - tr * p.G);
        const int64_t o = static_cast<int64_t>(tr) * p.o_st + static_cast<int64_t>(hr) * p.o_sh;
        unsigned char* dst = p.out_dtype == SPECEXT_BF16
                                 ? static_cast<unsigned char*>(p.out) + o * 2 + 16 * (lane & 15)
                                 : static_cast<unsigned char*>(p.out) + o * 4 + 256 * pass + 16 * (lane & 15);
        *reinterpret_cast<uintx4*>(dst) = uintx4{a[0], a[1], b[0], b[1]};
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
  if (p.lse && hf == 0 && m < p.M) {
    const int tr = m / p.G;
    const int hr = g * p.G + (m - tr * p.G);
    p.lse[static_cast<int64_t>(hr) * p.Tq + tr] = (ref * c + __builtin_amdgcn_logf(l_tot)) * kLn2;
  }
}

}  // namespace

hipError_t launch_prefill_rows(const PrefillParams& p, hipStream_t stream) {
  auto kernel = prefill_rows_kernel;
  static std::atomic<bool> attr_set[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!attr_set[dev].load(std::memory_order_acquire)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    attr_set[dev].store(true, std::memory_order_release);
  }
  const int rows_per_wg = kWaves * 32;
  dim3 grid(p.Hkv, (p.M + rows_per_wg - 1) / rows_per_wg);
  kernel<<<grid, dim3(kWaves * 64), kLdsBytes, stream>>>(p);
  return hipGetLastError();
}

}  // namespace specext
