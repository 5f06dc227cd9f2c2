// Cross-model Retrieval kernels (SpecExtend Sec. 3.2.1 and Alg. 1):
//   chunk_scores_kernel  - normalise the per-chunk exponential sums left by
//                          the prefix pass, average over chunk tokens and heads
//   select_*_kernel      - SelectChunks: top-k by ranking (short inputs) or radix select, ascending output
//   gather_*_kernel      - UpdateDraftCache: copy the chosen chunks verbatim
#include "common.h"

namespace specext {
namespace {

// --------------------------------------------------------------------------
// chunk scores
// --------------------------------------------------------------------------

// scores[r][c] = (1/Hq) * sum_h  sum_blocks  blocksum(h, t) * exp2(ref - lse2(h, t)) / |c|
// The prefix pass leaves one (sum, ref) pair per score block (score_gran keys;
// a chunk is a whole number of blocks).  A workgroup handles 64 chunks; the heads
// of a chunk are dealt to four threads (head h goes to thread h mod 4), each adds
// its heads in ascending order, and the four partial sums are combined in a fixed
// order: a deterministic fp32 sum.
__global__ __launch_bounds__(256) void chunk_scores_kernel(AttnParams p, int first_row, const int* row_path,
                                                          const int* row_count, float* scores) {
  __shared__ float partial[4][64];
  const int cl = threadIdx.x & 63;
  const int part = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  int t = first_row + blockIdx.y;
  if (row_path) {                                // the row comes from the acceptance walk: its last accepted node
    const int cnt = min(*row_count, p.T);            // never past the path array, whatever the count says
    const int node = cnt > 0 ? row_path[cnt - 1] : 0;
    t = (node >= 0 && node < p.T) ? node : 0;
  }
  float acc = 0.f;
  if (c < p.C) {
    const int per_chunk = p.B / p.score_gran;
    const int sub_lo = c * per_chunk;
    const int sub_hi = min(sub_lo + per_chunk, p.n_sub);
    for (int h = part; h < p.Hq; h += 4) {
      const int g = h / p.G;
      const int m = t * p.G + (h - g * p.G);
      const float l2 = p.lse2[g * p.M + m];
      for (int sb = sub_lo; sb < sub_hi; ++sb) {
        const float2 cp = *reinterpret_cast<const float2*>(
            p.chunk_part + ((static_cast<int64_t>(g) * p.n_sub + sb) * p.M + m) * 2);
        acc += cp.x * exp2f(cp.y - l2);
      }
    }
  }
  partial[part][cl] = acc;
  __syncthreads();
  if (part == 0 && c < p.C) {
    const int size = min(p.B, p.L - c * p.B);
    const float tot = ((partial[0][cl] + partial[1][cl]) + partial[2][cl]) + partial[3][cl];
    scores[static_cast<int64_t>(blockIdx.y) * p.C + c] = tot / (static_cast<float>(size) * static_cast<float>(p.Hq));
  }
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

// Block-wide count of a predicate (up to kSelPerThread flags per thread, bit u of
// `flags` = flag u); every thread gets the total.  Wave counts come from ballots;
// `slots` must hold blockDim.x / 64 ints and alternate between two buffers from
// call to call so that one barrier per call is enough.
__device__ __forceinline__ int block_count(unsigned flags, int n_flags, int* slots) {
  int c = 0;
  for (int u = 0; u < n_flags; ++u) c += __popcll(__ballot((flags >> u) & 1u));
  if ((threadIdx.x & 63) == 0) slots[threadIdx.x >> 6] = c;
  __syncthreads();
  // all sixteen slots are read at once (slots of absent waves hold zero), one LDS round trip
  const int4 a = *reinterpret_cast<const int4*>(slots), b = *reinterpret_cast<const int4*>(slots + 4),
             cc = *reinterpret_cast<const int4*>(slots + 8), d = *reinterpret_cast<const int4*>(slots + 12);
  return ((a.x + a.y) + (a.z + a.w)) + ((b.x + b.y) + (b.z + b.w)) + ((cc.x + cc.y) + (cc.z + cc.w)) +
         ((d.x + d.y) + (d.z + d.w));
}

// One workgroup.  The key value V of the k-th largest score is built bit by bit from
// the top: a bit stays set if at least k keys are >= the candidate.  Scores above V
// are all taken; of the scores equal to V the lowest-indexed ones fill what is left.
// A last pass in index order (block scans over the keep flags) writes the output
// ascending.  Threads hold up to kSelPerThread keys in registers; longer inputs are
// re-read from memory.
constexpr int kSelPerThread = 4;

__global__ __launch_bounds__(kSelThreads) void select_kernel(const float* __restrict__ scores, int n, int k,
                                                            int* __restrict__ idx_out, int* __restrict__ n_out) {
  __shared__ __attribute__((aligned(16))) int slots[2][kSelThreads / 64];
  __shared__ int wave_sums[kSelThreads / 64];

  const int k_eff = min(k, n);
  if (threadIdx.x == 0) *n_out = k_eff;
  for (int i = k_eff + threadIdx.x; i < k; i += blockDim.x) idx_out[i] = -1;
  if (k_eff == 0) return;
  if (threadIdx.x < 2 * (kSelThreads / 64)) slots[0][threadIdx.x] = 0;      // slots of absent waves stay zero
  __syncthreads();

  const bool in_regs = n <= kSelThreads * kSelPerThread;
  uint32_t mine[kSelPerThread];
#pragma unroll
  for (int u = 0; u < kSelPerThread; ++u) {
    const int i = u * kSelThreads + threadIdx.x;
    mine[u] = (in_regs && i < n) ? orderable(scores[i]) : 0u;       // 0 is below every real key
  }
  // how many keys are >= cand (block-wide)
  auto count_ge = [&](uint32_t cand, int* slot) {
    if (in_regs) {
      unsigned flags = 0;
#pragma unroll
      for (int u = 0; u < kSelPerThread; ++u) flags |= (mine[u] >= cand ? 1u : 0u) << u;
      const int n_flags = min(kSelPerThread, (n + kSelThreads - 1) / kSelThreads);
      return block_count(flags, n_flags, slot);
    }
    int total = 0;                     // long input: 32 keys per thread per round of ballots
    for (int base = 0; base < n; base += blockDim.x * 32) {
      unsigned flags = 0;
      for (int u = 0; u < 32; ++u) {
        const int i = base + u * blockDim.x + threadIdx.x;
        flags |= ((i < n && orderable(scores[i]) >= cand) ? 1u : 0u) << u;
      }
      // (an extra barrier keeps the slot buffer of the previous call intact)
      __syncthreads();
      total += block_count(flags, 32, slot);
    }
    return total;
  };
  uint32_t v = 0;
  int round = 0;
  for (int bit = 31; bit >= 0; --bit, ++round) {
    const uint32_t cand = v | (1u << bit);
    if (count_ge(cand, slots[round & 1]) >= k_eff) v = cand;
  }
  // v is the k-th largest key.  Keys above it: n_gt < k_eff; ties needed: k_eff - n_gt >= 1
  const int n_gt = v == 0xffffffffu ? 0 : count_ge(v + 1u, slots[round & 1]);
  const int need = k_eff - n_gt;
  int out_base = 0, tie_base = 0;
  for (int start = 0; start < n; start += blockDim.x) {
    const int i = start + threadIdx.x;
    uint32_t key = 0;
    if (i < n) key = orderable(scores[i]);
    const int is_tie = (i < n && key == v) ? 1 : 0;
    const int is_gt = (i < n && key > v) ? 1 : 0;
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

// Short inputs (n <= kRankMax) get one key per thread and the byte-wise selection below.
constexpr int kRankMax = 1024;

// One workgroup (blockDim.x a multiple of 64, at least n threads), thread i holding the score
// of chunk i.  The key of the k-th largest score is found a byte at a time from the top:
// a 256-bin histogram (LDS atomics) of the keys that match the bytes fixed so far, a
// suffix scan over the bins, and the bin that holds the k-th key fixes the next byte - four
// rounds instead of one compare of every key with every other.  Every wave does the scan
// for itself (four bins per lane), so a round costs one barrier.  Keys above the threshold
// are all taken; of the keys equal to it the lowest-indexed ones fill what is left; ballots
// and one exchange of per-wave counts give the ascending output.
struct RadixLds {
  __attribute__((aligned(16))) int hist[4][256];     // one histogram per round, all cleared up front
  int wave_counts[kSelThreads / 64][2];              // per wave: keys above the threshold, keys equal to it
};

__device__ __forceinline__ void radix_select_and_write(float score, int n, int k, int* __restrict__ idx_out,
                                                       int* __restrict__ n_out, RadixLds& sh) {
  const int i = threadIdx.x;
  const int lane = i & 63;
  const int wave = i >> 6;
  const int k_eff = min(k, n);
  if (i == 0) *n_out = k_eff;
  for (int u = k_eff + i; u < k; u += blockDim.x) idx_out[u] = -1;
  if (k_eff == 0) return;
  const bool live = i < n;
  const uint32_t key = live ? orderable(score) : 0u;
  for (int u = i; u < 4 * 256; u += blockDim.x) (&sh.hist[0][0])[u] = 0;
  __syncthreads();
  uint32_t prefix = 0;           // the bytes of the threshold fixed so far (higher bytes first)
  int need = k_eff;              // keys still to take among those that match `prefix` in the fixed bytes
#pragma unroll
  for (int round = 0; round < 4; ++round) {
    const int shift = 24 - 8 * round;
    const bool match = live && (round == 0 || (key >> (shift + 8)) == (prefix >> (shift + 8)));
    if (match) atomicAdd(&sh.hist[round][(key >> shift) & 255u], 1);
    __syncthreads();
    // lane l looks at bins 255 - 4l (first) down to 252 - 4l; `above` = keys in higher bins
    const int4 h = *reinterpret_cast<const int4*>(&sh.hist[round][252 - 4 * lane]);
    const int bins[4] = {h.w, h.z, h.y, h.x};
    const int mine = (h.x + h.y) + (h.z + h.w);
    int incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int up = __shfl_up(incl, off, 64);
      if (lane >= off) incl += up;
    }
    int above = incl - mine;
    int bin = -1, left = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (above < need && need <= above + bins[j]) {
        bin = 255 - 4 * lane - j;
        left = need - above;
      }
      above += bins[j];
    }
    // exactly one lane found the bin (1 <= need <= number of matching keys)
    const int src = __ffsll(static_cast<long long>(__ballot(bin >= 0))) - 1;
    prefix |= static_cast<uint32_t>(__shfl(bin, src, 64)) << shift;
    need = __shfl(left, src, 64);
  }
  // prefix is the k-th largest key; `need` of the keys equal to it are taken, lowest index first
  const bool greater = live && key > prefix;
  const bool is_tie = live && key == prefix;
  const uint64_t bal_greater = __ballot(greater), bal_tie = __ballot(is_tie);
  if (lane == 0) {
    sh.wave_counts[wave][0] = __popcll(bal_greater);
    sh.wave_counts[wave][1] = __popcll(bal_tie);
  }
  __syncthreads();
  int ties_before = 0, pos = 0;
  for (int w = 0; w < wave; ++w) {
    const int gr = sh.wave_counts[w][0], ti = sh.wave_counts[w][1];
    pos += gr + min(max(need - ties_before, 0), ti);
    ties_before += ti;
  }
  const uint64_t lower = (uint64_t{1} << lane) - 1;
  const int tie_rank = ties_before + __popcll(bal_tie & lower);
  const bool take = greater || (is_tie && tie_rank < need);
  const uint64_t bal_take = __ballot(take);
  if (take) idx_out[pos + __popcll(bal_take & lower)] = i;
}

__global__ __launch_bounds__(kRankMax) void select_short_kernel(const float* __restrict__ scores, int n, int k,
                                                              int* __restrict__ idx_out, int* __restrict__ n_out) {
  __shared__ RadixLds radix;
  const int i = threadIdx.x;
  radix_select_and_write(i < n ? scores[i] : 0.f, n, k, idx_out, n_out, radix);
}

// Chunk scores of one tree row and the top-k over them in one launch (at most kRankMax
// chunks, 1024 threads).  Scores with the arithmetic of chunk_scores_kernel - the heads of
// a chunk are dealt to four threads (head h to thread h mod 4), each adds its heads in
// ascending order, the four sums are combined in the same fixed order: the same bits -
// a quarter of the threads' number of chunks per pass, all loads of a thread requested
// before the first is used; then the byte-wise selection above.  scores may be null.
__global__ __launch_bounds__(kRankMax) void score_select_kernel(AttnParams p, int score_row, const int* row_path,
                                                               const int* row_count, int k, float* scores,
                                                               int* __restrict__ idx_out, int* __restrict__ n_out) {
  __shared__ RadixLds radix;
  __shared__ float partial[kRankMax][4];
  int t = score_row;
  if (row_path) {
    const int cnt = min(*row_count, p.T);
    const int node = cnt > 0 ? row_path[cnt - 1] : 0;
    t = (node >= 0 && node < p.T) ? node : 0;
  }
  const int part = threadIdx.x & 3;
  const int per_chunk = p.B / p.score_gran;
  constexpr int kHeadsAtOnce = 8;                // heads of one thread whose loads are in flight together
  constexpr int kChunksAtOnce = 2;               // chunks of one thread, likewise
  const int chunks_per_pass = blockDim.x / 4;
  for (int c0 = 0; c0 < p.C; c0 += kChunksAtOnce * chunks_per_pass) {
    int cs[kChunksAtOnce], sub_lo[kChunksAtOnce], sub_hi[kChunksAtOnce];
    float acc[kChunksAtOnce];
#pragma unroll
    for (int j = 0; j < kChunksAtOnce; ++j) {
      cs[j] = c0 + j * chunks_per_pass + (threadIdx.x >> 2);
      const int cl = min(cs[j], p.C - 1);                        // chunks past the end re-read the last one, unused
      sub_lo[j] = cl * per_chunk;
      sub_hi[j] = min(sub_lo[j] + per_chunk, p.n_sub);
      acc[j] = 0.f;
    }
    for (int hb = part; hb < p.Hq; hb += 4 * kHeadsAtOnce) {
      float l2[kHeadsAtOnce];
      float2 first[kChunksAtOnce][kHeadsAtOnce];
      const float* src[kChunksAtOnce][kHeadsAtOnce];
#pragma unroll
      for (int u = 0; u < kHeadsAtOnce; ++u) {
        const int h = min(hb + 4 * u, p.Hq - 1);                 // heads past the end re-read the last one, unused
        const int g = h / p.G;
        const int m = t * p.G + (h - g * p.G);
        l2[u] = p.lse2[g * p.M + m];
#pragma unroll
        for (int j = 0; j < kChunksAtOnce; ++j) {
          src[j][u] = p.chunk_part + ((static_cast<int64_t>(g) * p.n_sub + sub_lo[j]) * p.M + m) * 2;
          first[j][u] = *reinterpret_cast<const float2*>(src[j][u]);
        }
      }
#pragma unroll
      for (int j = 0; j < kChunksAtOnce; ++j) {
#pragma unroll
        for (int u = 0; u < kHeadsAtOnce; ++u) {
          if (hb + 4 * u < p.Hq) {
            acc[j] += first[j][u].x * exp2f(first[j][u].y - l2[u]);
            for (int sb = sub_lo[j] + 1; sb < sub_hi[j]; ++sb) {
              const float2 cp = *reinterpret_cast<const float2*>(src[j][u] + static_cast<int64_t>(sb - sub_lo[j]) * p.M * 2);
              acc[j] += cp.x * exp2f(cp.y - l2[u]);
            }
          }
        }
      }
    }
#pragma unroll
    for (int j = 0; j < kChunksAtOnce; ++j)
      if (cs[j] < p.C) partial[cs[j]][part] = acc[j];
  }
  __syncthreads();
  const int c = threadIdx.x;
  float score = 0.f;
  if (c < p.C) {
    const int size = min(p.B, p.L - c * p.B);
    score = (((partial[c][0] + partial[c][1]) + partial[c][2]) + partial[c][3]) / (static_cast<float>(size) * static_cast<float>(p.Hq));
    if (scores) scores[c] = score;
  }
  radix_select_and_write(score, p.C, k, idx_out, n_out, radix);
}

// --------------------------------------------------------------------------
// draft-KV gather
// --------------------------------------------------------------------------

__device__ __forceinline__ int chunk_tokens(int c, int n_chunks, int src_len, int chunk_size) {
  if (c < 0 || c >= n_chunks) return 0;
  return min(chunk_size, src_len - c * chunk_size);
}

// grid (max_idx, n_layers * n_heads, 2): one workgroup copies one chunk of one
// (layer, head) of K (z = 0) or V (z = 1), 16 bytes per thread per step.  The workgroups
// of (layer, head) 0 of K also do the bookkeeping: each writes the original positions of
// its chunk's tokens, and the one of list entry 0 the total and the -1 behind it.
__global__ __launch_bounds__(256) void gather_copy_kernel(const uint4* __restrict__ k_src, const uint4* __restrict__ v_src,
                                                         uint4* __restrict__ k_dst, uint4* __restrict__ v_dst,
                                                         const int* __restrict__ idx, const int* __restrict__ n_idx,
                                                         int max_idx, int src_len, int src_cap, int dst_cap,
                                                         int row_vecs, int chunk_size, int* __restrict__ pos_out,
                                                         int* __restrict__ len_out) {
  __shared__ int sh_off[4];
  const int r = blockIdx.x;
  const int n_used = n_idx ? min(max(*n_idx, 0), max_idx) : max_idx;
  const int n_chunks = (src_len + chunk_size - 1) / chunk_size;
  const bool book = blockIdx.y == 0 && blockIdx.z == 0 && (pos_out || len_out);
  if (book && r == 0) {
    // tokens of the whole list (fixed order), then the tail of pos_out
    int part = 0;
    for (int i = threadIdx.x; i < n_used; i += blockDim.x) part += chunk_tokens(idx[i], n_chunks, src_len, chunk_size);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
    if ((threadIdx.x & 63) == 0) sh_off[threadIdx.x >> 6] = part;
    __syncthreads();
    const int total = sh_off[0] + sh_off[1] + sh_off[2] + sh_off[3];
    __syncthreads();
    if (pos_out)
      for (int i = total + threadIdx.x; i < dst_cap; i += blockDim.x) pos_out[i] = -1;
    if (len_out && threadIdx.x == 0) *len_out = total;
  }
  if (r >= n_used) return;
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
  if (book && pos_out)
    for (int tk = threadIdx.x; tk < tokens; tk += blockDim.x) pos_out[dst_tok + tk] = c * chunk_size + tk;

  const int64_t lh = blockIdx.y;
  const uint4* src = (blockIdx.z == 0 ? k_src : v_src) + (lh * src_cap + static_cast<int64_t>(c) * chunk_size) * row_vecs;
  uint4* dst = (blockIdx.z == 0 ? k_dst : v_dst) + (lh * dst_cap + dst_tok) * row_vecs;
  const int n_vecs = tokens * row_vecs;
  for (int i = threadIdx.x; i < n_vecs; i += blockDim.x) dst[i] = src[i];
}

// The bookkeeping alone (an empty list or no (layer, head) to copy): original positions of
// the kept tokens, -1 behind them, and the total.  One workgroup; entry r of the list is
// handled by thread r (lists longer than the block go round by round, carrying the
// running offset), offsets come from a block scan.
__global__ __launch_bounds__(256) void gather_meta_kernel(const int* __restrict__ idx, const int* __restrict__ n_idx,
                                                         int max_idx, int src_len, int dst_cap, int chunk_size,
                                                         int* __restrict__ pos_out, int* __restrict__ len_out) {
  __shared__ int wave_sums[4];
  const int n_used = n_idx ? min(max(*n_idx, 0), max_idx) : max_idx;
  const int n_chunks = (src_len + chunk_size - 1) / chunk_size;
  int base = 0;
  for (int r0 = 0; r0 < n_used; r0 += blockDim.x) {
    const int r = r0 + threadIdx.x;
    int c = -1, tokens = 0;
    if (r < n_used) {
      c = idx[r];
      tokens = chunk_tokens(c, n_chunks, src_len, chunk_size);
    }
    int total;
    const int off = base + block_exclusive_scan(tokens, wave_sums, total);
    if (pos_out)
      for (int tk = 0; tk < tokens; ++tk) pos_out[off + tk] = c * chunk_size + tk;
    base += total;
  }
  if (pos_out)
    for (int i = base + threadIdx.x; i < dst_cap; i += blockDim.x) pos_out[i] = -1;
  if (len_out && threadIdx.x == 0) *len_out = base;
}

}  // namespace

hipError_t launch_chunk_scores(const AttnParams& p, int32_t score_row, const int32_t* row_path,
                               const int32_t* row_count, float* scores, hipStream_t stream) {
  const int rows = (score_row < 0 && !row_path) ? p.T : 1;
  dim3 grid((p.C + 63) / 64, rows);
  chunk_scores_kernel<<<grid, dim3(256), 0, stream>>>(p, score_row < 0 ? 0 : score_row, row_path, row_count, scores);
  return hipGetLastError();
}

hipError_t launch_score_select(const AttnParams& p, int32_t score_row, const int32_t* row_path,
                               const int32_t* row_count, int32_t k, float* scores, int32_t* idx_out, int32_t* n_out,
                               hipStream_t stream) {
  if (p.C > kRankMax) return hipErrorInvalidValue;
  // at least one thread per chunk (selection), up to eight (scores: two chunks in flight per thread, four threads
  // per chunk, so that 1024 threads take in 512 chunks in one pass)
  const int threads = p.C <= 128 ? 256 : p.C <= 256 ? 512 : 1024;
  score_select_kernel<<<dim3(1), dim3(threads), 0, stream>>>(p, score_row, row_path, row_count, k, scores, idx_out, n_out);
  return hipGetLastError();
}

hipError_t launch_select_chunks(const float* scores, int32_t n_chunks, int32_t k, int32_t* idx_out,
                                int32_t* n_out, hipStream_t stream) {
  // a small input needs only as many waves as it has scores (fewer waves, cheaper barriers)
  const int threads = n_chunks >= kSelThreads ? kSelThreads : ((n_chunks + 63) / 64) * 64;
  if (n_chunks <= kRankMax) {
    select_short_kernel<<<dim3(1), dim3(threads), 0, stream>>>(scores, n_chunks, k, idx_out, n_out);
  } else {
    select_kernel<<<dim3(1), dim3(threads), 0, stream>>>(scores, n_chunks, k, idx_out, n_out);
  }
  return hipGetLastError();
}

hipError_t launch_gather(const void* k_src, const void* v_src, void* k_dst, void* v_dst,
                         const int32_t* idx, const int32_t* n_idx, int32_t max_idx, int32_t n_lh,
                         int32_t src_len, int32_t src_cap, int32_t dst_cap, int32_t row_bytes,
                         int32_t chunk_size, int32_t* pos_out, int32_t* len_out, hipStream_t stream) {
  if (max_idx > 0 && n_lh > 0) {
    dim3 grid(max_idx, n_lh, 2);
    gather_copy_kernel<<<grid, dim3(256), 0, stream>>>(
        static_cast<const uint4*>(k_src), static_cast<const uint4*>(v_src), static_cast<uint4*>(k_dst),
        static_cast<uint4*>(v_dst), idx, n_idx, max_idx, src_len, src_cap, dst_cap, row_bytes / 16, chunk_size,
        pos_out, len_out);
    return hipGetLastError();
  }
  if (pos_out || len_out) {
    gather_meta_kernel<<<dim3(1), dim3(256), 0, stream>>>(idx, n_idx, max_idx, src_len, dst_cap, chunk_size,
                                                          pos_out, len_out);
    return hipGetLastError();
  }
  return hipSuccess;
}

}  // namespace specext
