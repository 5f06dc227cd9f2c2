// The score path as the paper itself describes it (SpecExtend Sec. 3.2.1): the last
// layer's verification attention computed as STANDARD attention - the whole matrix
// of attention scores written out to memory, a row softmax over it, the product
// with V - and the chunk scores read from that matrix.  Kept beside the fused path
// (prefix pass + tree/merge pass, which never writes the matrix) as an independent
// way to the same numbers and to measure what the fusion saves.
//
//   mat_logits_kernel       logits of all query rows against the prefix keys, on the
//                           matrix cores (v_mfma_f32_32x32x16_bf16, A = Q, B = K, both
//                           fragments are plain 16-byte row loads), fp32, base-2 units
//   mat_tree_logits_kernel  logits against the tree keys, -inf where the tree mask hides
//   mat_softmax_kernel      one workgroup per row: max, sum, normalise in place (the row
//                           is held in registers between the passes), lse
//   mat_pv_kernel           O = P V over a split of the keys, matrix cores (A = P rounded
//                           to bf16, B = V gathered per lane), fp32 partial per split
//   mat_reduce_kernel       partials summed in split order, written in the output type
//   mat_scores_kernel       mean of P over the tokens of each chunk and over all heads (fixed order)
//
// P layout: fp32 [Hq][T][ld], ld a multiple of 64 >= L + T; columns 0..L-1 are the
// prefix, L..L+T-1 the tree nodes, the padding behind them is written as zero.
#include "mfma_util.h"

namespace specext {
namespace {

constexpr int kD = 128;

// (t, h) of row m of KV head g (m = t * G + hg) -> first element of its P row
__device__ __forceinline__ int64_t prow(const MatParams& mp, int g, int m) {
  const int t = m / mp.a.G;
  const int h = g * mp.a.G + (m - t * mp.a.G);
  return (static_cast<int64_t>(h) * mp.a.T + t) * mp.ld;
}

__device__ __forceinline__ const uint16_t* q_row(const MatParams& mp, int g, int m) {
  const int t = m / mp.a.G;
  const int h = g * mp.a.G + (m - t * mp.a.G);
  return static_cast<const uint16_t*>(mp.a.q) + t * mp.a.q_st + h * mp.a.q_sh;
}

// grid (key blocks, KV heads, row groups); wave w of a workgroup owns rows
// [32 (z * waves + w), +32) of the KV head and walks the block's keys in tiles of 32.
__global__ __launch_bounds__(512) void mat_logits_kernel(MatParams mp) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int c32 = lane & 31, hf = lane >> 5;
  const int g = blockIdx.y;
  const int row0 = (blockIdx.z * (blockDim.x >> 6) + wave) * 32;
  if (row0 >= mp.a.M) return;
  const int L = mp.a.L;
  const int key_lo = blockIdx.x * mp.logit_keys_per_block;
  const int key_hi = min(L, key_lo + mp.logit_keys_per_block);

  bf16x8 qf[8];
  {
    const uint16_t* qr = q_row(mp, g, min(row0 + c32, mp.a.M - 1));
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      qf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uintx4*>(qr + 16 * ks + 8 * hf));
  }
  int64_t out_row[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int m = row0 + 8 * (i >> 2) + 4 * hf + (i & 3);
    out_row[i] = m < mp.a.M ? prow(mp, g, m) : -1;
  }
  const uint16_t* kbase = static_cast<const uint16_t*>(mp.a.kp) + g * mp.a.kp_sh;
  const float c = mp.a.scale_log2;
  for (int key0 = key_lo; key0 < key_hi; key0 += 32) {
    const int key = key0 + c32;
    const uint16_t* kr = kbase + static_cast<int64_t>(min(key, L - 1)) * mp.a.kp_sl + 8 * hf;
    floatx16 s = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const bf16x8 kf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uintx4*>(kr + 16 * ks));
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[ks], kf, s, 0, 0, 0);
    }
    if (key < key_hi) {
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (out_row[i] >= 0) mp.probs[out_row[i] + key] = s[i] * c;
    }
  }
}

// grid (T, Hq), one thread per tree key.
__global__ __launch_bounds__(128) void mat_tree_logits_kernel(MatParams mp) {
  const int t = blockIdx.x, h = blockIdx.y, j = threadIdx.x;
  if (t == 0 && h == 0) {
    // single writer of the status word: 1 if any parent index is not a topological one
    const bool bad = j < mp.a.T && (mp.a.parent[j] >= j || mp.a.parent[j] < -1);
    const int any_bad = __syncthreads_or(bad);
    if (j == 0) *mp.a.status = any_bad ? 1 : 0;
  }
  if (j >= mp.a.T) return;
  const int g = h / mp.a.G;
  bool seen = false;
  int node = t;
  for (int step = 0; node >= 0 && step < mp.a.T; ++step) {      // the node itself, then up to its root
    seen |= node == j;
    const int up = mp.a.parent[node];
    node = up < node ? up : -1;
  }
  float logit = -INFINITY;
  if (seen) {
    const uint16_t* qr = static_cast<const uint16_t*>(mp.a.q) + t * mp.a.q_st + h * mp.a.q_sh;
    const uint16_t* kr = static_cast<const uint16_t*>(mp.a.kt) + g * mp.a.kt_sh + j * mp.a.kt_st;
    float acc = 0.f;
    for (int x = 0; x < kD; ++x) acc = fmaf(bf16_bits_to_float(qr[x]), bf16_bits_to_float(kr[x]), acc);
    logit = acc * mp.a.scale_log2;
  }
  mp.probs[(static_cast<int64_t>(h) * mp.a.T + t) * mp.ld + mp.a.L + j] = logit;
}

__device__ __forceinline__ float block_max(float v, float* sh) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
}
__device__ __forceinline__ float block_sum(float v, float* sh) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  return (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

// grid (T, Hq), 256 threads per row.  The first kCached float4 per thread stay in
// registers between the passes (rows up to 256 * 4 * kCached elements are read
// once); longer rows re-read the rest.
constexpr int kCached = 20;
__global__ __launch_bounds__(256) void mat_softmax_kernel(MatParams mp) {
  __shared__ float sh[4];
  const int t = blockIdx.x, h = blockIdx.y;
  const int n = mp.a.L + mp.a.T;
  float* row = mp.probs + (static_cast<int64_t>(h) * mp.a.T + t) * mp.ld;
  floatx4* row4 = reinterpret_cast<floatx4*>(row);
  const int nvec = mp.ld / 4;                       // the row including its padding, whole float4
  const int tid = threadIdx.x;
  floatx4 keep[kCached];
  float mx = -INFINITY;
#pragma unroll
  for (int u = 0; u < kCached; ++u) {
    const int v = tid + 256 * u;
    floatx4 x = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    if (v < nvec) {
      x = row4[v];
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (4 * v + e >= n) x[e] = -INFINITY;       // padding columns
    }
    keep[u] = x;
    mx = fmaxf(mx, fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])));
  }
  for (int v = tid + 256 * kCached; v < nvec; v += 256) {
    const floatx4 x = row4[v];
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (4 * v + e < n) mx = fmaxf(mx, x[e]);
  }
  mx = block_max(mx, sh);
  float sum = 0.f;
#pragma unroll
  for (int u = 0; u < kCached; ++u) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      keep[u][e] = fast_exp2(keep[u][e] - mx);      // exp2(-inf) = 0 for hidden keys and padding
      sum += keep[u][e];
    }
  }
  for (int v = tid + 256 * kCached; v < nvec; v += 256) {
    const floatx4 x = row4[v];
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (4 * v + e < n) sum += fast_exp2(x[e] - mx);
  }
  sum = block_sum(sum, sh);
  const float inv = 1.0f / sum;
#pragma unroll
  for (int u = 0; u < kCached; ++u) {
    const int v = tid + 256 * u;
    if (v < nvec) row4[v] = keep[u] * inv;
  }
  for (int v = tid + 256 * kCached; v < nvec; v += 256) {
    floatx4 x = row4[v];
#pragma unroll
    for (int e = 0; e < 4; ++e) x[e] = 4 * v + e < n ? fast_exp2(x[e] - mx) * inv : 0.f;
    row4[v] = x;
  }
  if (mp.a.lse && tid == 0) mp.a.lse[h * mp.a.T + t] = (mx + __builtin_amdgcn_logf(sum)) * kLn2;
}

// grid (splits, KV heads, row groups); wave w owns 32 rows x 128 output columns and
// walks the split's keys (prefix and tree keys in one index) in tiles of 32.
__global__ __launch_bounds__(512) void mat_pv_kernel(MatParams mp) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int c32 = lane & 31, hf = lane >> 5;
  const int g = blockIdx.y;
  const int row0 = (blockIdx.z * (blockDim.x >> 6) + wave) * 32;
  if (row0 >= mp.a.M) return;
  const int L = mp.a.L;
  const int n = L + mp.a.T;
  const int key_lo = blockIdx.x * mp.pv_keys_per_split;
  const int key_hi = min((n + 31) / 32 * 32, key_lo + mp.pv_keys_per_split);
  const float* prow_ptr = mp.probs + prow(mp, g, min(row0 + c32, mp.a.M - 1)) + 8 * hf;
  const uint16_t* vp = static_cast<const uint16_t*>(mp.a.vp) + g * mp.a.kp_sh + c32;
  const uint16_t* vt = static_cast<const uint16_t*>(mp.a.vt) + g * mp.a.kt_sh + c32;
  floatx16 acc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[db][i] = 0.f;
  for (int key0 = key_lo; key0 < key_hi; key0 += 32) {
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const floatx4 p0 = *reinterpret_cast<const floatx4*>(prow_ptr + key0 + 16 * ks);
      const floatx4 p1 = *reinterpret_cast<const floatx4*>(prow_ptr + key0 + 16 * ks + 4);
      bf16x8 pf;
#pragma unroll
      for (int e = 0; e < 4; e += 2) {
        const bf16x2 lo = __builtin_convertvector(floatx2{p0[e], p0[e + 1]}, bf16x2);
        const bf16x2 hi = __builtin_convertvector(floatx2{p1[e], p1[e + 1]}, bf16x2);
        pf[e] = lo[0];
        pf[e + 1] = lo[1];
        pf[4 + e] = hi[0];
        pf[4 + e + 1] = hi[1];
      }
      uint16_t vv[4][8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int key = min(key0 + 16 * ks + 8 * hf + e, n - 1);      // beyond the row P is zero
        const uint16_t* vr = key < L ? vp + static_cast<int64_t>(key) * mp.a.kp_sl
                                     : vt + static_cast<int64_t>(key - L) * mp.a.kt_st;
#pragma unroll
        for (int db = 0; db < 4; ++db) vv[db][e] = vr[32 * db];
      }
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        uintx4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = vv[db][2 * e] | (static_cast<uint32_t>(vv[db][2 * e + 1]) << 16);
        acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf, __builtin_bit_cast(bf16x8, w), acc[db], 0, 0, 0);
      }
    }
  }
  float* part = mp.part + ((static_cast<int64_t>(blockIdx.x) * mp.a.Hkv + g) * mp.m_pad + row0) * kD + c32;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) part[(8 * (i >> 2) + 4 * hf + (i & 3)) * kD + 32 * db] = acc[db][i];
}

// grid (T, Hq), 128 threads = output columns
__global__ __launch_bounds__(128) void mat_reduce_kernel(MatParams mp) {
  const int t = blockIdx.x, h = blockIdx.y, x = threadIdx.x;
  const int g = h / mp.a.G;
  const int m = t * mp.a.G + (h - g * mp.a.G);
  float acc = 0.f;
#pragma unroll 8
  for (int s = 0; s < mp.pv_splits; ++s)
    acc += mp.part[((static_cast<int64_t>(s) * mp.a.Hkv + g) * mp.m_pad + m) * kD + x];
  const int64_t o = t * mp.a.o_st + h * mp.a.o_sh + x;
  if (mp.a.out_dtype == SPECEXT_BF16)
    static_cast<uint16_t*>(mp.a.out)[o] = float_to_bf16_bits(acc);
  else
    static_cast<float*>(mp.a.out)[o] = acc;
}

// grid (ceil(C / 8)), 256 threads: a workgroup scores 8 chunks; wave w takes heads
// w, w+4, ...; inside a wave 8 lanes share a chunk (lane part p sums tokens p, p+8, ...
// of it, the 8 partial sums are combined in a fixed butterfly); the four waves' totals
// are added in wave order.
__global__ __launch_bounds__(256) void mat_scores_kernel(MatParams mp, int first_row, const int* __restrict__ row_path,
                                                        const int* __restrict__ row_count, float* __restrict__ scores) {
  __shared__ float sh[4][8];
  int row = first_row;
  if (row_path) {
    const int cnt = min(*row_count, mp.a.T);
    row = cnt > 0 ? row_path[cnt - 1] : 0;
    row = min(max(row, 0), mp.a.T - 1);
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int part = lane & 7, slot = lane >> 3;
  const int c = blockIdx.x * 8 + slot;
  float total = 0.f;
  if (c < mp.a.C) {
    const int lo = c * mp.a.B;
    const int size = min(mp.a.B, mp.a.L - lo);
    const float inv = 1.0f / static_cast<float>(size);
    for (int h = wave; h < mp.a.Hq; h += 4) {
      const float* pr = mp.probs + (static_cast<int64_t>(h) * mp.a.T + row) * mp.ld + lo;
      float acc = 0.f;
      for (int k = part; k < size; k += 8) acc += pr[k];
      total += acc * inv;
    }
  }
  total += __shfl_xor(total, 1, 64);
  total += __shfl_xor(total, 2, 64);
  total += __shfl_xor(total, 4, 64);
  if (part == 0) sh[wave][slot] = total;
  __syncthreads();
  if (wave == 0 && part == 0 && c < mp.a.C)
    scores[c] = ((sh[0][slot] + sh[1][slot]) + (sh[2][slot] + sh[3][slot])) / static_cast<float>(mp.a.Hq);
}

}  // namespace

hipError_t launch_materialized(const MatParams& mp, hipStream_t stream) {
  const int row_blocks = (mp.a.M + 31) / 32;
  const int waves = row_blocks < 8 ? row_blocks : 8;
  const int row_groups = (row_blocks + waves - 1) / waves;
  if (mp.a.L > 0) {
    dim3 grid((mp.a.L + mp.logit_keys_per_block - 1) / mp.logit_keys_per_block, mp.a.Hkv, row_groups);
    mat_logits_kernel<<<grid, dim3(64 * waves), 0, stream>>>(mp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  mat_tree_logits_kernel<<<dim3(mp.a.T, mp.a.Hq), dim3(128), 0, stream>>>(mp);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  mat_softmax_kernel<<<dim3(mp.a.T, mp.a.Hq), dim3(256), 0, stream>>>(mp);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  mat_pv_kernel<<<dim3(mp.pv_splits, mp.a.Hkv, row_groups), dim3(64 * waves), 0, stream>>>(mp);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  mat_reduce_kernel<<<dim3(mp.a.T, mp.a.Hq), dim3(128), 0, stream>>>(mp);
  return hipGetLastError();
}

hipError_t launch_materialized_scores(const MatParams& mp, int32_t score_row, const int32_t* row_path,
                                      const int32_t* row_count, float* scores, hipStream_t stream) {
  mat_scores_kernel<<<dim3((mp.a.C + 7) / 8), dim3(256), 0, stream>>>(mp, score_row, row_path, row_count, scores);
  return hipGetLastError();
}

}  // namespace specext
