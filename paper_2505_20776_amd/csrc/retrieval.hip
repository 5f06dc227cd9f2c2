// Cross-model Retrieval kernels (SpecExtend Sec. 3.2.1 and Alg. 1):
//   chunk_scores_kernel  - normalise the per-chunk exponential sums left by
//                          the prefix pass, average over chunk tokens and heads
//   select_kernel        - SelectChunks: top-k by radix select, ascending output
//   gather_*_kernel      - UpdateDraftCache: copy the chosen chunks verbatim
#include "common.h"

namespace specext {
namespace {

// --------------------------------------------------------------------------
// chunk scores
// --------------------------------------------------------------------------

// scores[r][c] = (1/Hq) * sum_h  sum_blocks  blocksum(h, t) * exp2(ref - lse2(h, t)) / |c|
// The prefix pass leaves one (sum, ref) pair per score block (score_gran keys;
// a chunk is a whole number of blocks).  Heads and blocks are added in
// ascending order: a fixed-order fp32 sum.
__global__ __launch_bounds__(256) void chunk_scores_kernel(AttnParams p, int first_row, float* scores) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  const int t = first_row + blockIdx.y;
  if (c >= p.C) return;
  const int size = min(p.B, p.L - c * p.B);
  const int per_chunk = p.B / p.score_gran;
  const int sub_lo = c * per_chunk;
  const int sub_hi = min(sub_lo + per_chunk, p.n_sub);
  float acc = 0.f;
  for (int h = 0; h < p.Hq; ++h) {
    const int g = h / p.G;
    const int m = t * p.G + (h - g * p.G);
    const float l2 = p.lse2[g * p.M + m];
    for (int sb = sub_lo; sb < sub_hi; ++sb) {
      const float* cp = p.chunk_part + ((static_cast<int64_t>(g) * p.n_sub + sb) * p.M + m) * 2;
      acc += cp[0] * exp2f(cp[1] - l2);
    }
  }
  scores[static_cast<int64_t>(blockIdx.y) * p.C + c] = acc / (static_cast<float>(size) * static_cast<float>(p.Hq));
}

// --------------------------------------------------------------------------
// top-k selection
// --------------------------------------------------------------------------

constexpr int kSelThreads = 1024;

// Map a finite float to a uint32 whose unsigned order is the float order.
__device__ __forceinline__ uint32_t orderable(float f) {
  f += 0.0f;                                   // -0 -> +0 so they compare equal
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Exclusive block prefix sum of one int per thread; returns the block total in `total`.
__device__ __forceinline__ int block_exclusive_scan(int v, int* wave_sums, int& total) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int n = __shfl_up(incl, off, 64);
    if (lane >= off) incl += n;
  }
  __syncthreads();                              // wave_sums may still be read from the previous call
  if (lane == 63) wave_sums[wave] = incl;
  __syncthreads();
  int base = 0;
  total = 0;
  const int n_waves = blockDim.x >> 6;
  for (int w = 0; w < n_waves; ++w) {
    const int s = wave_sums[w];
    if (w < wave) base += s;
    total += s;
  }
  return base + incl - v;
}

// One workgroup.  Four rounds of an 8-bit radix select find the key value of
// the k-th largest score and how many scores are strictly larger; a final
// pass in index order emits every larger score plus the lowest-indexed ties.
__global__ __launch_bounds__(kSelThreads) void select_kernel(const float* __restrict__ scores, int n, int k,
                                                            int* __restrict__ idx_out, int* __restrict__ n_out) {
  __shared__ int hist[256];
  __shared__ int wave_sums[kSelThreads / 64];
  __shared__ uint32_t sh_prefix;
  __shared__ int sh_need;

  const int k_eff = min(k, n);
  if (threadIdx.x == 0) *n_out = k_eff;
  for (int i = k_eff + threadIdx.x; i < k; i += blockDim.x) idx_out[i] = -1;
  if (k_eff == 0) return;

  uint32_t prefix = 0;      // high bits fixed so far
  uint32_t mask = 0;
  int need = k_eff;         // rank still wanted among keys matching the prefix
  for (int shift = 24; shift >= 0; shift -= 8) {
    for (int b = threadIdx.x; b < 256; b += blockDim.x) hist[b] = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
      const uint32_t key = orderable(scores[i]);
      if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      int above = 0;
      int b = 255;
      for (; b > 0; --b) {
        if (above + hist[b] >= need) break;
        above += hist[b];
      }
      sh_prefix = prefix | (static_cast<uint32_t>(b) << shift);
      sh_need = need - above;
    }
    __syncthreads();
    prefix = sh_prefix;
    need = sh_need;
    mask |= 255u << shift;
    __syncthreads();
  }
  // prefix is now the k-th largest key; `need` ties (>= 1) are taken, lowest index first
  int out_base = 0, tie_base = 0;
  for (int start = 0; start < n; start += blockDim.x) {
    const int i = start + threadIdx.x;
    uint32_t key = 0;
    if (i < n) key = orderable(scores[i]);
    const int is_tie = (i < n && key == prefix) ? 1 : 0;
    const int is_gt = (i < n && key > prefix) ? 1 : 0;
    int tie_total;
    const int tie_rank = tie_base + block_exclusive_scan(is_tie, wave_sums, tie_total);
    const int take = is_gt | (is_tie & (tie_rank < need ? 1 : 0));
    int take_total;
    const int pos = out_base + block_exclusive_scan(take, wave_sums, take_total);
    if (take) idx_out[pos] = i;
    out_base += take_total;
    tie_base += tie_total;
  }
}

// --------------------------------------------------------------------------
// draft-KV gather
// --------------------------------------------------------------------------

__device__ __forceinline__ int chunk_tokens(int c, int n_chunks, int src_len, int chunk_size) {
  if (c < 0 || c >= n_chunks) return 0;
  return min(chunk_size, src_len - c * chunk_size);
}

// grid (max_idx, n_layers * n_heads, 2): one workgroup copies one chunk of one
// (layer, head) of K (z = 0) or V (z = 1), 16 bytes per thread per step.
__global__ __launch_bounds__(256) void gather_copy_kernel(const uint4* __restrict__ k_src, const uint4* __restrict__ v_src,
                                                         uint4* __restrict__ k_dst, uint4* __restrict__ v_dst,
                                                         const int* __restrict__ idx, const int* __restrict__ n_idx,
                                                         int max_idx, int src_len, int dst_cap, int row_vecs,
                                                         int chunk_size) {
  __shared__ int sh_off[4];
  const int r = blockIdx.x;
  const int n_used = n_idx ? min(max(*n_idx, 0), max_idx) : max_idx;
  if (r >= n_used) return;
  const int n_chunks = (src_len + chunk_size - 1) / chunk_size;
  const int c = idx[r];
  const int tokens = chunk_tokens(c, n_chunks, src_len, chunk_size);
  if (tokens == 0) return;
  // destination token offset = tokens of all earlier list entries
  int part = 0;
  for (int i = threadIdx.x; i < r; i += blockDim.x) part += chunk_tokens(idx[i], n_chunks, src_len, chunk_size);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
  if ((threadIdx.x & 63) == 0) sh_off[threadIdx.x >> 6] = part;
  __syncthreads();
  const int dst_tok = sh_off[0] + sh_off[1] + sh_off[2] + sh_off[3];

  const int64_t lh = blockIdx.y;
  const uint4* src = (blockIdx.z == 0 ? k_src : v_src) + (lh * src_len + static_cast<int64_t>(c) * chunk_size) * row_vecs;
  uint4* dst = (blockIdx.z == 0 ? k_dst : v_dst) + (lh * dst_cap + dst_tok) * row_vecs;
  const int n_vecs = tokens * row_vecs;
  for (int i = threadIdx.x; i < n_vecs; i += blockDim.x) dst[i] = src[i];
}

// One workgroup: original positions of the kept tokens, -1 behind them, and the total.
__global__ __launch_bounds__(256) void gather_meta_kernel(const int* __restrict__ idx, const int* __restrict__ n_idx,
                                                         int max_idx, int src_len, int dst_cap, int chunk_size,
                                                         int* __restrict__ pos_out, int* __restrict__ len_out) {
  const int n_used = n_idx ? min(max(*n_idx, 0), max_idx) : max_idx;
  const int n_chunks = (src_len + chunk_size - 1) / chunk_size;
  int off = 0;
  for (int r = 0; r < n_used; ++r) {
    const int c = idx[r];
    const int tokens = chunk_tokens(c, n_chunks, src_len, chunk_size);
    if (pos_out)
      for (int tk = threadIdx.x; tk < tokens; tk += blockDim.x) pos_out[off + tk] = c * chunk_size + tk;
    off += tokens;
  }
  if (pos_out)
    for (int i = off + threadIdx.x; i < dst_cap; i += blockDim.x) pos_out[i] = -1;
  if (len_out && threadIdx.x == 0) *len_out = off;
}

}  // namespace

hipError_t launch_chunk_scores(const AttnParams& p, int32_t score_row, float* scores, hipStream_t stream) {
  const int rows = score_row < 0 ? p.T : 1;
  dim3 grid((p.C + 255) / 256, rows);
  chunk_scores_kernel<<<grid, dim3(256), 0, stream>>>(p, score_row < 0 ? 0 : score_row, scores);
  return hipGetLastError();
}

hipError_t launch_select_chunks(const float* scores, int32_t n_chunks, int32_t k, int32_t* idx_out,
                                int32_t* n_out, hipStream_t stream) {
  select_kernel<<<dim3(1), dim3(kSelThreads), 0, stream>>>(scores, n_chunks, k, idx_out, n_out);
  return hipGetLastError();
}

hipError_t launch_gather(const void* k_src, const void* v_src, void* k_dst, void* v_dst,
                         const int32_t* idx, const int32_t* n_idx, int32_t max_idx, int32_t n_lh,
                         int32_t src_len, int32_t dst_cap, int32_t row_bytes, int32_t chunk_size,
                         int32_t* pos_out, int32_t* len_out, hipStream_t stream) {
  if (pos_out || len_out) {
    gather_meta_kernel<<<dim3(1), dim3(256), 0, stream>>>(idx, n_idx, max_idx, src_len, dst_cap, chunk_size,
                                                          pos_out, len_out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (max_idx > 0 && n_lh > 0) {
    dim3 grid(max_idx, n_lh, 2);
    gather_copy_kernel<<<grid, dim3(256), 0, stream>>>(
        static_cast<const uint4*>(k_src), static_cast<const uint4*>(v_src), static_cast<uint4*>(k_dst),
        static_cast<uint4*>(v_dst), idx, n_idx, max_idx, src_len, dst_cap, row_bytes / 16, chunk_size);
    return hipGetLastError();
  }
  return hipSuccess;
}

}  // namespace specext
