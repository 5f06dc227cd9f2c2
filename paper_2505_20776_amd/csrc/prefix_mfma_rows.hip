// Prefix pass of Hybrid Tree Attention (SpecExtend Sec. 3.1) on the gfx950
// matrix cores, row-split form: bf16 K/V streamed ONCE from HBM into ONE compute
// unit each, fp32 accumulation.  Used when a KV head has more than 32 query rows
// (tree nodes x heads in the GQA group); smaller problems take the key-split kernel.
//
// Why this shape.  Measured on MI355X: the memory system delivers the same 5.5 - 6 TB/s
// whether the bytes come from L2, the Infinity Cache or HBM, so every byte that passes
// a compute unit counts and every K/V byte must enter exactly one compute unit; and a
// lone wave per SIMD overlaps its matrix and vector instructions poorly, while two
// waves per SIMD overlap them better.  Hence:
//   grid  = (splits, KV heads, row groups of 32*WAVES rows)
//   block = WAVES (8 or 4) wavefronts, at most 256 registers each, so that two
//           waves share a SIMD; wave w owns rows [32w, 32w+32) of the row group and
//           keeps their queries and running output in registers.
//   The split's keys are walked in tiles of 32.  K and V tiles are filled by direct
//   global->LDS loads into two rings of kRing tiles (every wave issues its share of
//   every tile); the ring is cut into kStages stages of kStageTiles tiles with one
//   workgroup barrier per stage (one tile per stage by default), and every wave reads
//   every tile.  The loop is unrolled over the ring so that every LDS address is a
//   loop-invariant register plus an immediate.
//   A workgroup leaves one partial per row: (reference, row sum, unnormalised O), the
//   triple rescaled by a power of two per row so that O fits fp16 whatever V's scale.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, everything transposed so that a
// lane owns one query row in both products):
//   S^T[key][row]   = K[key][:] . Q[row][:]          A = K tile (LDS), B = Q (registers)
//   O^T[dcol][row] += V^T[dcol][key] P^T[key][row]   A = V^T (LDS transpose read
//   ds_read_b64_tr_b16), B = P^T taken straight from the S^T accumulator registers:
//   the key order that layout implies is used as the contraction order and V is
//   fetched in that same order, so P never moves between lanes.
#include "merge_tail.h"
#include "mfma_util.h"

namespace specext {
namespace {

constexpr int kTile = 32;                         // keys per tile
constexpr int kD = 128;                           // head_dim this kernel is written for
constexpr int kRowBytes = kD * 2;                 // one bf16 K or V row in LDS
constexpr int kTileBytes = kTile * kRowBytes;     // 8 KB
#ifndef SPECEXT_ROWS_STAGE_TILES
#define SPECEXT_ROWS_STAGE_TILES 1
#endif
#ifndef SPECEXT_ROWS_STAGES
#define SPECEXT_ROWS_STAGES 4
#endif
constexpr int kStageTiles = SPECEXT_ROWS_STAGE_TILES;   // tiles between two workgroup barriers
// Stages per ring (>= 2), a template parameter of the kernel.  The deep ring is for long splits; a split of few tiles
// (a workgroup of eight waves only) takes a ring of two stages: measured 0.5 - 0.9 us shorter per launch up to 16 tiles
// per split, equal at 32, 1 - 2 % longer at 64 and more (and much longer with four waves, whose tiles are consumed
// faster than one tile of look-ahead arrives).
constexpr int kDeepStages = SPECEXT_ROWS_STAGES;
constexpr int kShortStages = 2;
constexpr int kShortSplitTiles = 24;                    // splits of at most this many tiles take the short ring
constexpr int ring_bytes(int stages) { return 2 * kStageTiles * stages * kTileBytes; }
// Behind the rings every wave has a private area: first the staging of its 32 query
// rows (32 x 256 B), at the end the staging of its 32 partial output rows as fp16
// (rows padded to 264 B so that the 8-byte column writes fall into distinct banks).
constexpr int kPatchStride = kRowBytes + 8;
constexpr int kPrivBytes = 32 * kPatchStride;
// Behind those, the area of the fused tree-pass / merge tail (parent[], control words, tree slots).
constexpr int lds_bytes(int waves, int stages) { return ring_bytes(stages) + waves * kPrivBytes + tail_private_bytes(waves * 64); }
static_assert(kDeepStages >= 2 && lds_bytes(8, kDeepStages) <= 160 * 1024, "rings and private areas must fit the 160 KB of LDS");

template <int I>
using ic = std::integral_constant<int, I>;
// f(ic<0>{}), f(ic<1>{}), ..., f(ic<N-1>{})
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(ic<I>{});
    static_for<I + 1, N>(f);
  }
}

// KPR = keys per 256-byte LDS row: 1 for head_dim 128.  For head_dim 64 (KPR = 2, keys
// contiguous in memory) two consecutive keys share a row and the whole tile machinery -
// loads, swizzles, operand reads - is the same; a tile is then 64 keys, the logits of the
// even and of the odd keys of the rows come from the first and the second half of the
// K fragments against the same four query fragments, and the even / odd probabilities
// meet V^T's first / second pair of 32-column blocks in the same two output blocks.
template <int WAVES, bool SCORES, int KPR, int STAGES>
__global__ __launch_bounds__(WAVES * 64) void prefix_rows_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  constexpr int kStages = STAGES;
  constexpr int kRing = kStageTiles * kStages;            // tiles per ring (K ring and V ring)
  constexpr int kRingBytes = ring_bytes(kStages);
  constexpr int kLoadsPerWave = 8 / WAVES;       // 1 KB blocks of a tile that one wave fills (per K or V)
  constexpr int kKeysPerTile = kTile * KPR;
  constexpr int kQSteps = 8 / KPR;               // 16-wide contraction steps of one query row
  constexpr int kOBlocks = 4 / KPR;              // 32-column blocks of the output
  constexpr int kHeadDim = kD / KPR;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c32 = lane & 31;
  const int hf = lane >> 5;
#ifdef SPECEXT_TAIL_STAMPS
  // profiling build: wall-clock stamps (100 MHz) of this workgroup's phases, left in the unused upper half
  // of the partial-output region (sized for fp32, holding fp16): 0 start, 1 first tile ready, 2 last tile
  // done, 3 partial stores issued (the fused tail, when it runs, overwrites 1.. with its own phases)
  const unsigned long long stamp_start = wall_clock64();
  unsigned long long stamp_first = 0, stamp_loop = 0;
  // and, per wave, shader-clock stamps inside the key loop (low 32 bits of s_memtime) for the 16 tiles from
  // kLoopStampTile0 on: 0 this wave's loads of the tile have arrived, 1 behind the barrier, 2 between the two
  // halves of the loop order (before the second product in the rotated order, before the softmax otherwise),
  // 3 the tile's last instruction issued.  Lane 4 * (tile - kLoopStampTile0) + k of loop_stamps holds stamp k.
  constexpr int kLoopStampTile0 = 4;
  int loop_stamps = 0;
  unsigned long long ls_arrived = 0, ls_barrier = 0, ls_half = 0, ls_end = 0;
  const unsigned long long ls_begin = __builtin_amdgcn_s_memtime();
#define SPECEXT_LOOP_STAMP(var)              \
  do {                                       \
    __builtin_amdgcn_sched_barrier(0);       \
    var = __builtin_amdgcn_s_memtime();      \
    __builtin_amdgcn_sched_barrier(0);       \
  } while (0)
#else
#define SPECEXT_LOOP_STAMP(var) do { } while (0)
#endif

  const int split = p.head_fastest ? blockIdx.y : blockIdx.x;
  const int g = p.head_fastest ? blockIdx.x : blockIdx.y;
  const int row0 = blockIdx.z * (WAVES * 32) + wave * 32;
  const int m = row0 + c32;                      // this lane's query row of the KV head
  // a wave whose 32 rows are all padding (fewer rows than the workgroup covers) still loads its
  // share of every tile and meets every barrier, but does no arithmetic
  const bool wave_live = row0 < p.M;

  const int key_lo = split * p.keys_per_split;
  const int key_hi = min(p.L, key_lo + p.keys_per_split);
  const int n = (key_hi - key_lo + kKeysPerTile - 1) / kKeysPerTile;          // tiles of this split (>= 1)

  const int64_t key_bytes = p.kp_sl * 2;
  const int64_t row_bytes = key_bytes * KPR;     // from one LDS row's first key to the next one's (KPR = 2: kp_sl = 64)
  const unsigned char* kbase = static_cast<const unsigned char*>(p.kp) + static_cast<int64_t>(g) * p.kp_sh * 2;
  const unsigned char* vbase = static_cast<const unsigned char*>(p.vp) + static_cast<int64_t>(g) * p.kp_sh * 2;

  // ---- LDS rings.  A tile is 32 rows x 256 B; one direct load writes 1 KB = 4
  // consecutive rows, lane i landing at byte 16*i.  The 16-byte chunks of a row are
  // XOR-swizzled (K: chunk ^ (row & 15), V: chunk ^ ((row & 3) << 2)) so that the
  // operand reads are bank-conflict free; the LDS side of a direct load being fixed,
  // the swizzle is applied to the global address.
  const unsigned kring_lds = static_cast<unsigned>(reinterpret_cast<uintptr_t>((lds_void*)lds));
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
  // back so that it ends exactly at key_hi (no load ever leaves the prefix); its keys
  // below the tile's own first key belong to the tile before and are masked.
  auto tile_key0 = [&](int t) { return key_lo + t * kKeysPerTile; };
  auto tile_first_row = [&](int t) { return min(tile_key0(t), key_hi - kKeysPerTile); };
  // this wave's share of K(t), then of V(t), into ring slot SLOT (a compile-time constant,
  // so that every LDS address below is a loop-invariant register plus an immediate)
  auto issue_tile = [&](auto slot_c, int t) {
    constexpr unsigned slot = decltype(slot_c)::value * kTileBytes;
    const int64_t off = static_cast<int64_t>(tile_first_row(t)) * key_bytes;
#pragma unroll
    for (int u = 0; u < kLoadsPerWave; ++u) {
      const int blk = kLoadsPerWave * wave + u;
      load_to_lds_16_stream(kring_lds + slot + blk * 1024, k_voff[u], kbase + off + blk * 4 * row_bytes);
    }
#pragma unroll
    for (int u = 0; u < kLoadsPerWave; ++u) {
      const int blk = kLoadsPerWave * wave + u;
      load_to_lds_16_stream(vring_lds + slot + blk * 1024, v_voff, vbase + off + blk * 4 * row_bytes);
    }
  };
  // stage s = tiles [s * kStageTiles, (s + 1) * kStageTiles) of the split, cut at n; it
  // lives in ring stage s % kStages
  const int n_stages = (n + kStageTiles - 1) / kStageTiles;
  auto issue_stage = [&](auto ring_stage_c, int s) {
    constexpr int ring_stage = decltype(ring_stage_c)::value;
    static_for<0, kStageTiles>([&](auto i_c) {
      constexpr int i = decltype(i_c)::value;
      const int t = s * kStageTiles + i;
      if (t < n) issue_tile(ic<ring_stage * kStageTiles + i>{}, t);
    });
  };
  // load instructions of this wave that are younger than those of stage s, once the
  // stages up to s + kStages - 2 have been requested
  constexpr int kLoadsPerTile = 2 * kLoadsPerWave;
  auto younger_than_stage = [&](int s) {
    return kLoadsPerTile * (min((s + kStages - 1) * kStageTiles, n) - min((s + 1) * kStageTiles, n));
  };

  // prologue: the first kStages-1 stages are requested, and after the first of them
  // the queries (B operand of S^T: lane = row c32, 8 consecutive d per k-step) with
  // plain loads in inline assembly, so that waiting for them does not drain the prefetch
  issue_stage(ic<0>{}, 0);
  const unsigned priv_lds = kring_lds + kRingBytes + wave * kPrivBytes;
  {
    // load u brings rows 4u..4u+3 of the wave (1 KB); the lane that fills LDS chunk
    // slot `ld_slot` of row r fetches chunk ld_slot ^ (r & 15) of that query row (the K
    // swizzle, so that the fragment reads below use the K read offsets)
    const float inv_g = 1.0f / static_cast<float>(p.G);
    const unsigned char* qbase = static_cast<const unsigned char*>(p.q);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int r = 4 * u + ld_row;
      const int mq = min(row0 + r, p.M - 1);               // padding rows repeat the last real row (never stored)
      const int tq = static_cast<int>((static_cast<float>(mq) + 0.5f) * inv_g);   // mq / G, exact for mq < 2^20
      const int hq = g * p.G + (mq - tq * p.G);
      // (a 64-wide query row has eight 16-byte chunks: the lanes of the other eight slots re-read them, unused)
      const unsigned voff = static_cast<unsigned>((tq * p.q_st + hq * p.q_sh) * 2) +
                            (((ld_slot ^ (r & 15)) & (KPR == 2 ? 7 : 15)) << 4);
      load_to_lds_16(priv_lds + u * 1024, voff, qbase);
    }
  }
  // Fused tail: parent[] goes to the tail's LDS area with one direct load per wave (lane i
  // of wave w fills entry 64 w + i; lanes past the tree re-read its last entry), and the
  // hand-over block's epoch and the workspace's initialisation mark are read now, long
  // before the tail needs them.  These loads are older than those of the next stages, so
  // the counted waits below stay valid (they only ever wait for more).
  unsigned char* tail_priv = lds + kRingBytes + WAVES * kPrivBytes;
  uint32_t epoch = 0;
  bool cookie_ok = true;
  if (p.fused_tail) {
    if (wave * 64 < p.T) {
      const unsigned tail_lds = kring_lds + kRingBytes + WAVES * kPrivBytes;
      const unsigned voff = static_cast<unsigned>(min(static_cast<int>(threadIdx.x), p.T - 1)) * 4u;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                   :: "s"(tail_lds + wave * 256), "v"(voff), "s"(p.parent) : "memory", "m0");
    }
    if (threadIdx.x < 16) reinterpret_cast<int*>(tail_priv + kTailCtlOff)[threadIdx.x] = 0;
    epoch = p.sync[blockIdx.z * p.Hkv + g].epoch;
    cookie_ok = p.cookie == nullptr || *p.cookie == kWorkspaceCookie;
  }
  static_for<1, kStages - 1>([&](auto u_c) {
    constexpr int u = decltype(u_c)::value;
    if (u < n_stages) issue_stage(ic<u>{}, u);
  });

  // K operand read: row c32, chunk (2*ks + hf) ^ (c32 & 15)
  unsigned k_rd[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) k_rd[ks] = c32 * kRowBytes + ((((2 * ks) ^ (c32 & 14)) | (hf ^ (c32 & 1))) << 4);
  // V transpose read: a group of 16 lanes reads 4 keys x 16 dcols
  const int li = lane & 15;
  const int grp_col = (lane >> 4) & 1;                  // which 16-column half of the 32-dcol block
  const int v_key_in = 4 * hf + (li >> 2);              // + 16 * jj (+ 8)
  const int v_q4 = li >> 2;                             // (row & 3) of the row this lane addresses
  unsigned v_rd[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
    v_rd[db] = kRing * kTileBytes + v_key_in * kRowBytes + ((db ^ v_q4) << 6) + ((2 * grp_col + ((li & 3) >> 1)) << 4) +
               ((li & 1) << 3);

  // The operand reads of the loop take these as LDS addresses plus the ring slot's immediate; pinned
  // in registers so that the compiler does not rebuild each one with an addition per use.
  unsigned k_addr[8], v_addr[4];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    k_addr[ks] = kring_lds + k_rd[ks];
    asm volatile("" : "+v"(k_addr[ks]));
  }
#pragma unroll
  for (int db = 0; db < 4; ++db) {
    v_addr[db] = kring_lds + v_rd[db];
    asm volatile("" : "+v"(v_addr[db]));
  }

  // queries: B operand of S^T (lane = row c32, 8 consecutive d per k-step), read from
  // the private area once the first wait below has passed
  bf16x8 qf[kQSteps];
  unsigned char* priv = lds + kRingBytes + wave * kPrivBytes;
  floatx16 acc_o[kOBlocks];
#pragma unroll
  for (int db = 0; db < kOBlocks; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_o[db][r] = 0.f;
  float ref = -INFINITY;       // reference logit (raw units) the exponentials are taken against
  float run_sum = 0.f;         // lane-partial row sum
  const float c = p.scale_log2;
  const float lazy_raw = kLazyLog2 / c;      // the lazy margin in raw-logit units
  const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // where this lane's (sum, reference) pair of tile j goes: score_base + j * score_step
  float* score_base = nullptr;
  const int score_step = p.M * 2;
  if (SCORES) score_base = p.chunk_part + ((static_cast<int64_t>(g) * p.n_sub + key_lo / kTile) * p.M + min(m, p.M - 1)) * 2;

  // One tile in two parts.  Front: the logits (matrix pipe) and the V^T fragments, everything
  // the tile needs from its ring slot SLOT.  Back: online softmax (vector ALU; one query row
  // per lane pair, the reference moves lazily) and O^T += V^T P^T (matrix pipe) from
  // registers alone.  The two waves of a SIMD leave every barrier together, and with the
  // same instruction stream they would want the matrix pipe at the same time and the
  // vector ALU at the same time, one unit idling while the other is contended.  So the two
  // take their steps in different orders behind a barrier, each with one long matrix
  // phase and one vector phase that fall on the other's vector and matrix phase:
  //   upper wave:  softmax of the tile before | its second product, this tile's logits
  //   lower wave:  second product of the tile before, this tile's logits | its softmax
  // Waves w and w + 4 of a workgroup share a SIMD (measured: rotating the upper four gains,
  // rotating every other wave or every other pair loses).  In a workgroup of four waves
  // every wave has its SIMD to itself and keeps the plain order.
  const bool rotated = (wave & 4) != 0;
  floatx16 s[KPR];               // the tile's logits, then its probabilities
  bf16x8 vf[4][2];               // the tile's V^T fragments
  auto tile_front = [&](auto slot_c) __attribute__((always_inline)) {
    constexpr int slot = decltype(slot_c)::value * kTileBytes;
#pragma unroll
    for (int kp = 0; kp < KPR; ++kp) {
      s[kp] = zero16;
#pragma unroll
      for (int ks = 0; ks < kQSteps; ++ks) {
        const uintx4 kw = *reinterpret_cast<const lds_uintx4*>(static_cast<uintptr_t>(k_addr[ks + kp * kQSteps] + slot));
        s[kp] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kw), qf[ks], s[kp], 0, 0, 0);
      }
    }
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      const unsigned col = v_addr[db] + slot;
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4*)static_cast<uintptr_t>(col + (16 * jj) * kRowBytes));
        const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4*)static_cast<uintptr_t>(col + (16 * jj + 8) * kRowBytes));
        const shortx8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        vf[db][jj] = __builtin_bit_cast(bf16x8, both);
      }
    }
  };
  bf16x8 pf[KPR][2];             // the tile's probabilities as the second product takes them
  auto tile_softmax = [&](int j) __attribute__((always_inline)) {
    const int key0 = tile_key0(j);
    const int first_key = tile_first_row(j);
    // register r of s[kp] holds key first_key + KPR * (4*hf + 8*(r/4) + r%4) + kp
    const int skip = key0 - first_key - KPR * 4 * hf;     // > 0 only in a shifted last tile: keys of the tile before
    if (first_key < key0) {
#pragma unroll
      for (int kp = 0; kp < KPR; ++kp)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          if (KPR * (8 * (r >> 2) + (r & 3)) + kp < skip) s[kp][r] = -INFINITY;
        }
    }
    float mx = fmaxf(s[0][0], s[0][1]);
#pragma unroll
    for (int kp = 0; kp < KPR; ++kp)
#pragma unroll
      for (int r = 0; r < 16; r += 2) mx = fmaxf(mx, fmaxf(s[kp][r], s[kp][r + 1]));
    if (__any(mx > ref + lazy_raw)) {     // some row of this wave outgrew its reference: move every reference up
      mx = halves_max(mx);
      const float new_ref = fmaxf(ref, mx);
      const float alpha = fast_exp2((ref - new_ref) * c);     // 0 on the first tile
      ref = new_ref;
      run_sum *= alpha;
#pragma unroll
      for (int db = 0; db < kOBlocks; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[db][r] *= alpha;
    }
    const float mc = ref * c;
    // exponentials; their sums per 32-key score block: a tile is one block (KPR = 1) or two
    // (KPR = 2: the keys of LDS rows 0..15, registers 0..7, then those of rows 16..31)
    float part[KPR];
#pragma unroll
    for (int b = 0; b < KPR; ++b) part[b] = 0.f;
    if (KPR == 2 && SCORES && first_key < key0) {
      // shifted last tile: its rows no longer line up with the score blocks; sort every key by its position
#pragma unroll
      for (int kp = 0; kp < KPR; ++kp)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          s[kp][r] = fast_exp2(fmaf(s[kp][r], c, -mc));
          if (KPR * (8 * (r >> 2) + (r & 3)) + kp - skip >= kTile) part[KPR - 1] += s[kp][r];
          else part[0] += s[kp][r];
        }
    } else {
#pragma unroll
      for (int kp = 0; kp < KPR; ++kp)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          s[kp][r] = fast_exp2(fmaf(s[kp][r], c, -mc));
          part[KPR == 2 ? (r >> 3) : 0] += s[kp][r];
        }
    }
#pragma unroll
    for (int b = 0; b < KPR; ++b) run_sum += part[b];
    if (SCORES) {
#pragma unroll
      for (int b = 0; b < KPR; ++b) {
        const float tot = halves_sum(part[b]);
        if (hf == 0 && m < p.M && key0 + b * kTile < key_hi) {
          *reinterpret_cast<floatx2*>(score_base + (j * KPR + b) * score_step) = floatx2{tot, mc};
        }
      }
    }
#pragma unroll
    for (int kp = 0; kp < KPR; ++kp) {
      pf[kp][0] = pack8(s[kp], 0);
      pf[kp][1] = pack8(s[kp], 8);
    }
  };
  auto tile_second_product = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int db = 0; db < kOBlocks; ++db) {
#pragma unroll
      for (int kp = 0; kp < KPR; ++kp) {
        acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db + kp * kOBlocks][0], pf[kp][0], acc_o[db], 0, 0, 0);
        acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db + kp * kOBlocks][1], pf[kp][1], acc_o[db], 0, 0, 0);
      }
    }
  };
  auto tile_back = [&](int j) __attribute__((always_inline)) {
    tile_softmax(j);
    tile_second_product();
  };

  // Each wave's loads form the sequence (K, V of tile 0), (K, V of tile 1), ...  Before
  // stage s is read every wave waits for its own share of it and meets the others at a
  // barrier; behind that barrier every wave has also left stage s-1, whose ring stage
  // takes the loads of stage s + kStages - 1.  Between two barriers the waves run free.
  // The loop exists once per order of the steps, so that each order gets its own register
  // allocation.
  auto key_loop = [&](auto order_c) __attribute__((always_inline)) {
    // 0: front, back; 1: back of the tile before, front; 2: second product of the tile before, front, softmax
    constexpr int kOrder = decltype(order_c)::value;
    constexpr bool kRot = kOrder == 1;
    for (int s0 = 0; s0 < n_stages; s0 += kStages) {
      static_for<0, kStages>([&](auto u_c) {
        constexpr int u = decltype(u_c)::value;
        const int s = s0 + u;
        if (s < n_stages) {
          if (s == 0) {
            wait_vmcnt_even(younger_than_stage(0));        // also covers the wave's own queries
#pragma unroll
            for (int ks = 0; ks < kQSteps; ++ks)
              qf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uintx4*>(priv + k_rd[ks]));
          } else if ((s + kStages - 1) * kStageTiles <= n) {
            asm volatile("s_waitcnt vmcnt(%0)" :: "n"(kLoadsPerTile * kStageTiles * (kStages - 2)) : "memory");
          } else {
            wait_vmcnt_even(younger_than_stage(s));
          }
          SPECEXT_LOOP_STAMP(ls_arrived);
          lds_barrier();
          SPECEXT_LOOP_STAMP(ls_barrier);
#ifdef SPECEXT_TAIL_STAMPS
          if (s == 0) stamp_first = wall_clock64();
#endif
          if (s + kStages - 1 < n_stages) issue_stage(ic<(u + kStages - 1) % kStages>{}, s + kStages - 1);
          static_for<0, kStageTiles>([&](auto i_c) {
            constexpr int i = decltype(i_c)::value;
            const int j = s * kStageTiles + i;
            if (j < n && wave_live) {
              if constexpr (kOrder == 2) {
                if (j > 0) tile_second_product();
                tile_front(ic<u * kStageTiles + i>{});
                SPECEXT_LOOP_STAMP(ls_half);
                tile_softmax(j);
              } else if constexpr (kRot) {
                if (j > 0) tile_softmax(j - 1);
                SPECEXT_LOOP_STAMP(ls_half);
                if (j > 0) tile_second_product();
                tile_front(ic<u * kStageTiles + i>{});
              } else {
                tile_front(ic<u * kStageTiles + i>{});
                SPECEXT_LOOP_STAMP(ls_half);
                tile_back(j);
              }
            }
#ifdef SPECEXT_TAIL_STAMPS
            SPECEXT_LOOP_STAMP(ls_end);
            if (j >= kLoopStampTile0 && j < kLoopStampTile0 + 16) {
              // (plain copies: operands of inline assembly alone are not captured by the enclosing lambdas)
              int reg = loop_stamps;
              const int at = 4 * (j - kLoopStampTile0);
              const int t0 = static_cast<int>(ls_arrived), t1 = static_cast<int>(ls_barrier), t2 = static_cast<int>(ls_half),
                        t3 = static_cast<int>(ls_end);
              asm volatile("s_mov_b32 m0, %2\n\tv_writelane_b32 %0, %1, m0" : "+v"(reg) : "s"(t0), "s"(at) : "m0");
              asm volatile("s_mov_b32 m0, %2\n\tv_writelane_b32 %0, %1, m0" : "+v"(reg) : "s"(t1), "s"(at + 1) : "m0");
              asm volatile("s_mov_b32 m0, %2\n\tv_writelane_b32 %0, %1, m0" : "+v"(reg) : "s"(t2), "s"(at + 2) : "m0");
              asm volatile("s_mov_b32 m0, %2\n\tv_writelane_b32 %0, %1, m0" : "+v"(reg) : "s"(t3), "s"(at + 3) : "m0");
              loop_stamps = reg;
            }
#endif
          });
        }
      });
    }
    if (kRot && wave_live) tile_back(n - 1);
    if (kOrder == 2 && wave_live) tile_second_product();
  };
  if (rotated) key_loop(ic<1>{});
  else key_loop(ic<(WAVES == 8 ? 2 : 0)>{});

#ifdef SPECEXT_TAIL_STAMPS
  stamp_loop = wall_clock64();
#endif
  const float l_tot = halves_sum(run_sum);
  const int64_t slot0 = static_cast<int64_t>(split) * p.Hq * p.T + g * p.M + row0;     // slot of the wave's first row
  if constexpr (KPR == 2) {
    // ---- head_dim 64: the partial goes out as it is, (reference, row sum) and the unnormalised
    // O in fp32 (what the merge kernel reads for this head size); a lane owns one row and
    // holds four consecutive columns per register quad
    if (m < p.M) {
      float* dst = p.part_o + (slot0 + c32) * kHeadDim;
#pragma unroll
      for (int db = 0; db < kOBlocks; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
          __builtin_nontemporal_store(floatx4{acc_o[db][4 * r4], acc_o[db][4 * r4 + 1], acc_o[db][4 * r4 + 2], acc_o[db][4 * r4 + 3]},
                                      reinterpret_cast<floatx4*>(dst + 32 * db + 8 * r4 + 4 * hf));
      if (hf == 0) __builtin_nontemporal_store(floatx2{ref * c, l_tot}, reinterpret_cast<floatx2*>(p.part_ml + (slot0 + c32) * 2));
    }
  } else {
  // ---- partial results of this split: the triple (reference, row sum, unnormalised O)
  // is rescaled by the power of two that brings the row's largest |O| just below 1
  // (O * 2^-e, sum * 2^-e, reference + e describe the same partial), and O goes out as
  // fp16: every row keeps 11 bits against its own largest element whatever the scale of
  // V.  O^T sits in registers with a lane owning one row; it goes through the wave's
  // private LDS area so that the global stores are whole 256-byte rows.
  float row_max = 0.f;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; r += 2) row_max = fmaxf(row_max, fmaxf(fabsf(acc_o[db][r]), fabsf(acc_o[db][r + 1])));
  row_max = halves_max(row_max);
  const int row_exp = (row_max > 0.f && row_max < INFINITY) ? __builtin_amdgcn_frexp_expf(row_max) : 0;
  const float row_scale = __builtin_amdgcn_ldexpf(1.0f, -row_exp);
  auto to_half2 = [&](float x, float y) {
    const floatx2 f = {x * row_scale, y * row_scale};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, halfx2));
  };
  const int rows_here = min(32, p.M - row0);       // <= 0 for a wave of padding rows only
#pragma unroll
  for (int db = 0; db < 4; ++db) {
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      uintx2 w;
      w[0] = to_half2(acc_o[db][4 * r4], acc_o[db][4 * r4 + 1]);
      w[1] = to_half2(acc_o[db][4 * r4 + 2], acc_o[db][4 * r4 + 3]);
      *reinterpret_cast<uintx2*>(priv + c32 * kPatchStride + (32 * db + 8 * r4 + 4 * hf) * 2) = w;
    }
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_wave_barrier();
  uint16_t* part_h = reinterpret_cast<uint16_t*>(p.part_o);
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int row = 4 * it + (lane >> 4);
    const uintx2* src = reinterpret_cast<const uintx2*>(priv + row * kPatchStride + 16 * (lane & 15));
    const uintx2 a = src[0], b = src[1];
    // Separate merge launch: non-temporal stores, so that the partials leave the L2 as they are
    // written instead of waiting there for the write-back at the end of the kernel (measured:
    // 1.4 us per launch).  Merge in this launch: device-scope stores, which the workgroups of
    // the other XCDs can read back without cache maintenance.
    if (row < rows_here) {
      const uintx4 v = {a[0], a[1], b[0], b[1]};
      uint16_t* dst = part_h + (slot0 + row) * kD + 8 * (lane & 15);
      if (p.fused_tail) store_device_scope_16(dst, v);
      else __builtin_nontemporal_store(v, reinterpret_cast<uintx4*>(dst));
    }
  }
  if (hf == 0 && m < p.M) {
    const floatx2 v = {ref * c + static_cast<float>(row_exp), l_tot * row_scale};
    float* dst = p.part_ml + (slot0 + c32) * 2;
    if (p.fused_tail) store_device_scope_8(dst, v);
    else __builtin_nontemporal_store(v, reinterpret_cast<floatx2*>(dst));
  }
  }
#ifdef SPECEXT_TAIL_STAMPS
  if (KPR == 1 && WAVES == 8) {
    // the loop stamps of every wave: 80 words per wave, 4 MiB into the spare half of the partial region (when
    // that half reaches so far): words 0..63 the register above, 64 / 65 the shader-clock counter at the kernel's
    // start and here, 66 / 67 the 100 MHz wall clock at the same two points
    const size_t spare = static_cast<size_t>(p.S) * p.Hq * p.T * kD * 2;
    const size_t n_wg = static_cast<size_t>(gridDim.x) * gridDim.y * gridDim.z;
    if (spare >= (4u << 20) + n_wg * WAVES * 80 * 4) {
      const unsigned long long ls_done = __builtin_amdgcn_s_memtime();
      int* st = reinterpret_cast<int*>(reinterpret_cast<unsigned char*>(p.part_o) + spare + (4u << 20)) +
                ((((blockIdx.z * p.Hkv + g) * p.S + split) * WAVES + wave) * 80);
      st[lane] = loop_stamps;
      if (lane == 0) {
        st[64] = static_cast<int>(ls_begin);
        st[65] = static_cast<int>(ls_done);
        st[66] = static_cast<int>(stamp_start);
        st[67] = static_cast<int>(wall_clock64());
      }
    }
  }
  if (KPR == 1 && threadIdx.x == 0) {
    unsigned long long* st = reinterpret_cast<unsigned long long*>(reinterpret_cast<unsigned char*>(p.part_o) +
                                                                   static_cast<size_t>(p.S) * p.Hq * p.T * kD * 2) +
                             ((blockIdx.z * p.Hkv + g) * p.S + split) * 8;
    st[0] = stamp_start;
    st[1] = stamp_first;
    st[2] = stamp_loop;
    st[3] = wall_clock64();
  }
#endif
  // tree pass and merge in the same launch: this workgroup merges its slice of the head's rows
  if constexpr (KPR == 1) {
    if (p.fused_tail) tree_merge_tail<WAVES * 64>(p, lds, tail_priv, split, g, blockIdx.z, WAVES * 32, epoch, cookie_ok);
  }
}

template <int WAVES, bool SCORES, int KPR, int STAGES = kDeepStages>
hipError_t launch_rows(const AttnParams& p, hipStream_t stream) {
  auto kernel = prefix_rows_kernel<WAVES, SCORES, KPR, STAGES>;
  constexpr int kLdsBytes = lds_bytes(WAVES, STAGES);
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
  dim3 grid(p.head_fastest ? p.Hkv : p.S, p.head_fastest ? p.S : p.Hkv, (p.M + rows_per_wg - 1) / rows_per_wg);
  kernel<<<grid, dim3(WAVES * 64), kLdsBytes, stream>>>(p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_prefix_mfma_rows(const AttnParams& p, hipStream_t stream) {
  if (p.S <= 0) return hipSuccess;
  const bool big = p.rows_per_group == 256;
  if (p.d == 64) {
    if (big) return p.want_scores ? launch_rows<8, true, 2>(p, stream) : launch_rows<8, false, 2>(p, stream);
    return p.want_scores ? launch_rows<4, true, 2>(p, stream) : launch_rows<4, false, 2>(p, stream);
  }
  if (big) {
    const int split_tiles = (p.keys_per_split + kTile - 1) / kTile;
    if (split_tiles <= kShortSplitTiles)
      return p.want_scores ? launch_rows<8, true, 1, kShortStages>(p, stream) : launch_rows<8, false, 1, kShortStages>(p, stream);
    return p.want_scores ? launch_rows<8, true, 1>(p, stream) : launch_rows<8, false, 1>(p, stream);
  }
  return p.want_scores ? launch_rows<4, true, 1>(p, stream) : launch_rows<4, false, 1>(p, stream);
}

}  // namespace specext
