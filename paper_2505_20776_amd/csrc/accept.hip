// What follows the attention in one verification step (SpecExtend Alg. 1): the
// Verify / Correct loop at temperature 0 walked down the draft tree, and the commit of
// the accepted tree tokens' K/V rows into the target cache.
#include "common.h"

namespace specext {
namespace {

// One wavefront; lane i holds nodes i and i + 64 (n_tree <= 128).  At each step the
// children of the current node that carry the wanted token are found with two ballots,
// the lowest index wins, and the next wanted token is read across lanes.  At most
// n_tree steps, so the walk also ends on a malformed parent array.
__global__ __launch_bounds__(64) void accept_greedy_kernel(const int* __restrict__ parent,
                                                          const int* __restrict__ draft_token,
                                                          const int* __restrict__ target_token,
                                                          const int* __restrict__ first_target, int n_tree,
                                                          int* __restrict__ path_out, int* __restrict__ n_accept_out,
                                                          int* __restrict__ next_token_out) {
  const int lane = threadIdx.x;
  const bool has0 = lane < n_tree, has1 = lane + 64 < n_tree;
  const int par0 = has0 ? parent[lane] : -2, par1 = has1 ? parent[lane + 64] : -2;
  const int tok0 = has0 ? draft_token[lane] : 0, tok1 = has1 ? draft_token[lane + 64] : 0;
  const int tgt0 = has0 ? target_token[lane] : 0, tgt1 = has1 ? target_token[lane + 64] : 0;
  int cur = -1;
  int want = *first_target;
  int n = 0;
  for (int step = 0; step < n_tree; ++step) {
    const uint64_t m0 = __ballot(has0 && par0 == cur && tok0 == want);
    const uint64_t m1 = __ballot(has1 && par1 == cur && tok1 == want);
    int c;
    if (m0) c = __builtin_ctzll(m0);
    else if (m1) c = 64 + __builtin_ctzll(m1);
    else break;
    if (lane == 0) path_out[n] = c;
    ++n;
    cur = c;
    want = c < 64 ? __builtin_amdgcn_readlane(tgt0, c) : __builtin_amdgcn_readlane(tgt1, c - 64);
  }
  for (int i = n + lane; i < n_tree; i += 64) path_out[i] = -1;
  if (lane == 0) {
    *n_accept_out = n;
    *next_token_out = want;
  }
}

// grid (max_accept, layers * KV heads, 2): one workgroup copies one accepted row of K (z = 0)
// or V (z = 1) of one (layer, head), 16 bytes per thread.
__global__ __launch_bounds__(64) void commit_tree_kv_kernel(const uint4* __restrict__ k_tree,
                                                            const uint4* __restrict__ v_tree,
                                                            uint4* __restrict__ k_cache, uint4* __restrict__ v_cache,
                                                            const int* __restrict__ path,
                                                            const int* __restrict__ n_accept, int max_accept,
                                                            int n_tree, int n_kv_heads, int prefix_len, int row_vecs,
                                                            int64_t tree_sl, int64_t tree_sh, int64_t tree_st,
                                                            int64_t cache_sy, int64_t cache_sh, int64_t cache_sl) {
  const int i = blockIdx.x;
  const int n = min(max(*n_accept, 0), max_accept);
  if (i >= n) return;
  const int node = path[i];
  if (node < 0 || node >= n_tree) return;
  const int layer = blockIdx.y / n_kv_heads;
  const int g = blockIdx.y - layer * n_kv_heads;
  const uint4* src = (blockIdx.z ? v_tree : k_tree) + layer * tree_sl + g * tree_sh + node * tree_st;
  uint4* dst = (blockIdx.z ? v_cache : k_cache) + layer * cache_sy + g * cache_sh +
               (static_cast<int64_t>(prefix_len) + i) * cache_sl;
  for (int v = threadIdx.x; v < row_vecs; v += 64) dst[v] = src[v];
}

}  // namespace

hipError_t launch_accept_greedy(const int32_t* parent, const int32_t* draft_token, const int32_t* target_token,
                                const int32_t* first_target, int32_t n_tree, int32_t* path_out,
                                int32_t* n_accept_out, int32_t* next_token_out, hipStream_t stream) {
  accept_greedy_kernel<<<dim3(1), dim3(64), 0, stream>>>(parent, draft_token, target_token, first_target, n_tree,
                                                        path_out, n_accept_out, next_token_out);
  return hipGetLastError();
}

hipError_t launch_commit_tree_kv(const void* k_tree, const void* v_tree, void* k_cache, void* v_cache,
                                 const int32_t* path, const int32_t* n_accept, int32_t max_accept, int32_t n_tree,
                                 int32_t n_layers, int32_t n_kv_heads, int32_t prefix_len, int32_t row_bytes,
                                 int64_t tree_sl_bytes, int64_t tree_sh_bytes, int64_t tree_st_bytes,
                                 int64_t cache_sy_bytes, int64_t cache_sh_bytes, int64_t cache_sl_bytes,
                                 hipStream_t stream) {
  if (max_accept <= 0) return hipSuccess;
  dim3 grid(max_accept, n_layers * n_kv_heads, 2);
  commit_tree_kv_kernel<<<grid, dim3(64), 0, stream>>>(
      static_cast<const uint4*>(k_tree), static_cast<const uint4*>(v_tree), static_cast<uint4*>(k_cache),
      static_cast<uint4*>(v_cache), path, n_accept, max_accept, n_tree, n_kv_heads, prefix_len, row_bytes / 16,
      tree_sl_bytes / 16, tree_sh_bytes / 16, tree_st_bytes / 16, cache_sy_bytes / 16, cache_sh_bytes / 16,
      cache_sl_bytes / 16);
  return hipGetLastError();
}

}  // namespace specext
