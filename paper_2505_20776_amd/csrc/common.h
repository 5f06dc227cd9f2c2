// Internal declarations shared by the HIP translation units of libspecext.
// Nothing here is part of the public ABI (see include/specext.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "specext.h"

namespace specext {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Hand-over between the workgroups that share the rows of one KV head when the tree pass
// and the merge run as the tail of the prefix kernel: one block per (KV head, row group)
// in the workspace header.  specext_workspace_init clears the blocks once; every call leaves
// `done` and `abandon` at zero and `epoch` one higher, so no call depends on what the one
// before left in `flags`.
struct SyncBlock {
  uint32_t epoch;        // calls completed on this block; flag values of the current call are epoch + 1
  uint32_t done;         // workgroups that have finished (or given up) in the current call
  uint64_t abandon;      // bit s: the owner of slice s stopped waiting; the last workgroup to finish merges it
  uint32_t pad[12];
  uint32_t flags[64];    // flags[s] == epoch + 1: the partial results of prefix split s are in memory
};
static_assert(sizeof(SyncBlock) == 320, "SyncBlock layout");
constexpr int kMaxSyncBlocks = 256;
constexpr uint64_t kWorkspaceCookie = 0x53504558544e4431ull;   // written by specext_workspace_init

// One verification-attention problem with every default resolved.  Passed to
// kernels by value.  Rows of a KV head g are numbered m = t * G + hg
// (t = tree node, hg = query head within the group); the global row id is
// rid = g * M + m with M = T * G.  All softmax bookkeeping is kept in the
// base-2 domain: logits are multiplied by scale * log2(e) once.
struct AttnParams {
  const void* q;
  const void* kp;
  const void* vp;
  const void* kt;
  const void* vt;
  const int32_t* parent;
  void* out;
  float* lse;          // user output, natural log, [Hq][T]; may be null
  // workspace pieces
  int32_t* status;     // [1]
  float* lse2;         // [Hq*T] base-2 log-sum-exp per rid
  float* part_ml;      // [S][Hq*T][2]  (running max, running sum) per split
  float* part_o;       // [S][Hq*T][d]  unnormalised partial outputs
  float* chunk_part;   // [Hkv][n_sub][M][2]  (sum of exp2(s - ref), ref) per score block; null unless want_scores
  SyncBlock* sync;     // [kMaxSyncBlocks] hand-over blocks of the fused tail
  const uint64_t* cookie;   // kWorkspaceCookie once the workspace was initialised; null = do not check (library-owned memory)
  int32_t Hq, Hkv, G, d, L, T, M;
  int32_t B, C, S, keys_per_split, want_scores;
  int32_t score_gran, n_sub;      // keys per score block (32 on the MFMA path, else B) and their count
  int32_t use_mfma;               // 0 vector-ALU kernel, 1 matrix-core key-split kernel, 2 matrix-core row-split kernel
  int32_t rows_per_group;         // query rows of one KV head that one workgroup covers
  int32_t part_f16;               // part_o [S][rows][d] holds the unnormalised O as fp16 (1: row-split kernel) or fp32 (0)
  int32_t fused_tail;             // 1: the row-split kernel also runs the tree pass and the merge (no second launch)
  int32_t head_fastest;           // row-split kernel: grid x = KV head, y = split (else x = split, y = KV head)
  int32_t spin_limit;             // polls of the arrival counter before a workgroup hands its slice to the last arriver
  int32_t in_dtype, out_dtype;
  float scale_log2;
  int64_t q_st, q_sh, kp_sh, kp_sl, kt_sh, kt_st, o_st, o_sh;
};

// Standard attention with the probability matrix written out (the score path of
// Sec. 3.2.1 as the paper describes it): the problem plus the two buffers it needs.
struct MatParams {
  AttnParams a;               // inputs, outputs, shapes, strides, scale (workspace pieces unused)
  float* probs;               // [Hq][T][ld] logits, then probabilities
  float* part;                // [pv_splits][Hkv][m_pad][d] partial outputs of P V
  int32_t ld;                 // row pitch of probs in elements, a multiple of 64 >= L + T
  int32_t m_pad;              // rows of a KV head rounded up to whole 32-row blocks
  int32_t logit_keys_per_block, pv_keys_per_split, pv_splits;   // multiples of 32 keys
};

// Causal self-attention of the prefill stage: query i of q_len sits at position
// q_off + i of a context of N keys.  Row numbering as above (m = token * G + hg).
struct PrefillParams {
  const void* q;
  const void* k;
  const void* v;
  void* out;
  float* lse;                 // natural log, [Hq][Tq]; may be null
  int32_t Hq, Hkv, G, Tq, N, M, q_off, out_dtype;
  float scale_log2;
  int64_t q_st, q_sh, k_sh, k_sl, o_st, o_sh;
};

// Launchers (each returns a hipError_t from the launch itself).
hipError_t launch_prefill_rows(const PrefillParams& p, hipStream_t stream);
hipError_t launch_materialized(const MatParams& mp, hipStream_t stream);
hipError_t launch_materialized_scores(const MatParams& mp, int32_t score_row, const int32_t* row_path,
                                      const int32_t* row_count, float* scores, hipStream_t stream);
hipError_t launch_prefix_generic(const AttnParams& p, hipStream_t stream);
hipError_t launch_prefix_mfma(const AttnParams& p, hipStream_t stream);        // key-split kernel (use_mfma == 1)
hipError_t launch_prefix_mfma_rows(const AttnParams& p, hipStream_t stream);   // row-split kernel (use_mfma == 2)
hipError_t launch_tree_merge(const AttnParams& p, hipStream_t stream);
// score_row >= 0: that row; -1: every row; row_path != nullptr: the row is read on the device,
// row_path[*row_count - 1] (row 0 when *row_count <= 0)
hipError_t launch_chunk_scores(const AttnParams& p, int32_t score_row, const int32_t* row_path,
                               const int32_t* row_count, float* scores, hipStream_t stream);
// chunk scores of one row and their top-k in one launch; needs p.C <= 1024
hipError_t launch_score_select(const AttnParams& p, int32_t score_row, const int32_t* row_path,
                               const int32_t* row_count, int32_t k, float* scores, int32_t* idx_out, int32_t* n_out,
                               hipStream_t stream);
hipError_t launch_accept_greedy(const int32_t* parent, const int32_t* draft_token, const int32_t* target_token,
                                const int32_t* first_target, int32_t n_tree, int32_t* path_out,
                                int32_t* n_accept_out, int32_t* next_token_out, hipStream_t stream);
hipError_t launch_commit_tree_kv(const void* k_tree, const void* v_tree, void* k_cache, void* v_cache,
                                 const int32_t* path, const int32_t* n_accept, int32_t max_accept, int32_t n_tree,
                                 int32_t n_layers, int32_t n_kv_heads, int32_t prefix_len, int32_t row_bytes,
                                 int64_t tree_sl_bytes, int64_t tree_sh_bytes, int64_t tree_st_bytes,
                                 int64_t cache_sy_bytes, int64_t cache_sh_bytes, int64_t cache_sl_bytes,
                                 hipStream_t stream);
hipError_t launch_select_chunks(const float* scores, int32_t n_chunks, int32_t k, int32_t* idx_out,
                                int32_t* n_out, hipStream_t stream);
hipError_t launch_gather(const void* k_src, const void* v_src, void* k_dst, void* v_dst,
                         const int32_t* idx, const int32_t* n_idx, int32_t max_idx, int32_t n_lh,
                         int32_t src_len, int32_t src_cap, int32_t dst_cap, int32_t row_bytes,
                         int32_t chunk_size, int32_t* pos_out, int32_t* len_out, hipStream_t stream);

// bf16 helpers (bit-level; round to nearest even on the way down)
__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

// Wave-wide reductions on the vector ALU's data-parallel-primitive paths (no LDS
// round trips): four steps inside each row of 16 lanes (quad swaps, half mirror,
// mirror), then the four row totals are read out and combined.  Every lane gets
// the result.
#define SPECEXT_DPP(v, ctrl) \
  __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), (ctrl), 0xf, 0xf, false))

__device__ __forceinline__ float wave_sum(float v) {
  v += SPECEXT_DPP(v, 0xB1);    // quad_perm [1,0,3,2]
  v += SPECEXT_DPP(v, 0x4E);    // quad_perm [2,3,0,1]
  v += SPECEXT_DPP(v, 0x141);   // row_half_mirror
  v += SPECEXT_DPP(v, 0x140);   // row_mirror
  const int b = __float_as_int(v);
  return (__int_as_float(__builtin_amdgcn_readlane(b, 0)) + __int_as_float(__builtin_amdgcn_readlane(b, 16))) +
         (__int_as_float(__builtin_amdgcn_readlane(b, 32)) + __int_as_float(__builtin_amdgcn_readlane(b, 48)));
}

// the same two reductions over each aligned group of 16 lanes (one DPP row); every
// lane of a group receives its group's result
__device__ __forceinline__ float row16_sum(float v) {
  v += SPECEXT_DPP(v, 0xB1);
  v += SPECEXT_DPP(v, 0x4E);
  v += SPECEXT_DPP(v, 0x141);
  v += SPECEXT_DPP(v, 0x140);
  return v;
}

__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, SPECEXT_DPP(v, 0xB1));
  v = fmaxf(v, SPECEXT_DPP(v, 0x4E));
  v = fmaxf(v, SPECEXT_DPP(v, 0x141));
  v = fmaxf(v, SPECEXT_DPP(v, 0x140));
  return v;
}

__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, SPECEXT_DPP(v, 0xB1));
  v = fmaxf(v, SPECEXT_DPP(v, 0x4E));
  v = fmaxf(v, SPECEXT_DPP(v, 0x141));
  v = fmaxf(v, SPECEXT_DPP(v, 0x140));
  const int b = __float_as_int(v);
  return fmaxf(fmaxf(__int_as_float(__builtin_amdgcn_readlane(b, 0)), __int_as_float(__builtin_amdgcn_readlane(b, 16))),
               fmaxf(__int_as_float(__builtin_amdgcn_readlane(b, 32)), __int_as_float(__builtin_amdgcn_readlane(b, 48))));
}

}  // namespace specext
