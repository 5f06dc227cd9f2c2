// Prefix pass of Hybrid Tree Attention (SpecExtend Sec. 3.1), generic kernel.
//
// fp32 arithmetic on the vector ALUs for any supported dtype, head_dim and
// chunk size.  It is the product path for fp32 inputs and for shapes the MFMA
// kernel does not take.  One thread owns one query row (a tree node of one
// query head), keeps the query and the running output in registers, and walks
// its split of the prefix in tiles of 32 keys staged through LDS as fp32.
// Softmax is the usual online form in base 2; per-chunk sums of the
// exponentials are flushed with the reference maximum they were taken against
// so that a later kernel can normalise them (Sec. 3.2.1 chunk scores).
#include "common.h"

namespace specext {
namespace {

constexpr int kTileKeys = 32;
constexpr int kRowsPerBlock = 64;

template <int D, bool BF16>
__global__ __launch_bounds__(kRowsPerBlock) void prefix_generic_kernel(AttnParams p) {
  __shared__ __attribute__((aligned(16))) float k_tile[kTileKeys * D];
  __shared__ __attribute__((aligned(16))) float v_tile[kTileKeys * D];

  const int split = blockIdx.x;
  const int g = blockIdx.y;
  const int m = blockIdx.z * kRowsPerBlock + threadIdx.x;
  const bool row_ok = m < p.M;
  const int t = row_ok ? m / p.G : 0;
  const int h = g * p.G + (row_ok ? m % p.G : 0);
  const int rid = g * p.M + m;

  const int key_lo = split * p.keys_per_split;
  const int key_hi = min(p.L, key_lo + p.keys_per_split);

  float q[D];
  float o[D];
#pragma unroll
  for (int x = 0; x < D; ++x) o[x] = 0.f;
  if (BF16) {
    const uint16_t* qp = static_cast<const uint16_t*>(p.q) + t * p.q_st + h * p.q_sh;
#pragma unroll
    for (int x = 0; x < D; ++x) q[x] = bf16_bits_to_float(qp[x]) * p.scale_log2;
  } else {
    const float* qp = static_cast<const float*>(p.q) + t * p.q_st + h * p.q_sh;
#pragma unroll
    for (int x = 0; x < D; ++x) q[x] = qp[x] * p.scale_log2;
  }

  float run_max = -INFINITY;
  float run_sum = 0.f;
  float chunk_sum = 0.f;            // sum of exp2(s - run_max) over the open chunk

  for (int base = key_lo; base < key_hi; base += kTileKeys) {
    __syncthreads();
    // cooperative, coalesced tile load; rows past the end repeat the last valid key
    constexpr int kVec = BF16 ? 8 : 4;            // elements per 16-byte load
    constexpr int kVecPerRow = D / kVec;
    for (int i = threadIdx.x; i < kTileKeys * kVecPerRow; i += kRowsPerBlock) {
      const int r = i / kVecPerRow;
      const int c = (i % kVecPerRow) * kVec;
      const int j = min(base + r, p.L - 1);
      if (BF16) {
        const uint16_t* kb = static_cast<const uint16_t*>(p.kp) + g * p.kp_sh + j * p.kp_sl + c;
        const uint16_t* vb = static_cast<const uint16_t*>(p.vp) + g * p.kp_sh + j * p.kp_sl + c;
        const uint4 kk = *reinterpret_cast<const uint4*>(kb);
        const uint4 vv = *reinterpret_cast<const uint4*>(vb);
        const uint32_t kw[4] = {kk.x, kk.y, kk.z, kk.w};
        const uint32_t vw[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          k_tile[r * D + c + 2 * e] = __uint_as_float(kw[e] << 16);
          k_tile[r * D + c + 2 * e + 1] = __uint_as_float(kw[e] & 0xffff0000u);
          v_tile[r * D + c + 2 * e] = __uint_as_float(vw[e] << 16);
          v_tile[r * D + c + 2 * e + 1] = __uint_as_float(vw[e] & 0xffff0000u);
        }
      } else {
        const float* kb = static_cast<const float*>(p.kp) + g * p.kp_sh + j * p.kp_sl + c;
        const float* vb = static_cast<const float*>(p.vp) + g * p.kp_sh + j * p.kp_sl + c;
        *reinterpret_cast<float4*>(&k_tile[r * D + c]) = *reinterpret_cast<const float4*>(kb);
        *reinterpret_cast<float4*>(&v_tile[r * D + c]) = *reinterpret_cast<const float4*>(vb);
      }
    }
    __syncthreads();

    const int n_keys = min(kTileKeys, key_hi - base);
    float s[kTileKeys];
    float tile_max = -INFINITY;
#pragma unroll
    for (int r = 0; r < kTileKeys; ++r) {
      float acc = 0.f;
#pragma unroll
      for (int x = 0; x < D; x += 4) {
        const float4 kk = *reinterpret_cast<const float4*>(&k_tile[r * D + x]);
        acc = fmaf(q[x], kk.x, acc);
        acc = fmaf(q[x + 1], kk.y, acc);
        acc = fmaf(q[x + 2], kk.z, acc);
        acc = fmaf(q[x + 3], kk.w, acc);
      }
      s[r] = r < n_keys ? acc : -INFINITY;
      tile_max = fmaxf(tile_max, s[r]);
    }
    const float new_max = fmaxf(run_max, tile_max);
    const float alpha = exp2f(run_max - new_max);      // 0 on the first tile
    run_max = new_max;
    run_sum *= alpha;
    chunk_sum *= alpha;
#pragma unroll
    for (int x = 0; x < D; ++x) o[x] *= alpha;
#pragma unroll
    for (int r = 0; r < kTileKeys; ++r) {
      const float pr = exp2f(s[r] - new_max);          // 0 for masked keys
      run_sum += pr;
#pragma unroll
      for (int x = 0; x < D; x += 4) {
        const float4 vv = *reinterpret_cast<const float4*>(&v_tile[r * D + x]);
        o[x] = fmaf(pr, vv.x, o[x]);
        o[x + 1] = fmaf(pr, vv.y, o[x + 1]);
        o[x + 2] = fmaf(pr, vv.z, o[x + 2]);
        o[x + 3] = fmaf(pr, vv.w, o[x + 3]);
      }
      if (p.want_scores && r < n_keys) {
        chunk_sum += pr;
        const int j = base + r;
        if ((j + 1) % p.B == 0 || j + 1 == key_hi) {   // chunk closes (splits start on chunk boundaries)
          if (row_ok) {
            float* cp = p.chunk_part + ((static_cast<int64_t>(g) * p.n_sub + j / p.B) * p.M + m) * 2;
            cp[0] = chunk_sum;
            cp[1] = new_max;
          }
          chunk_sum = 0.f;
        }
      }
    }
  }

  if (row_ok) {
    const int64_t slot = static_cast<int64_t>(split) * p.Hq * p.T + rid;
    p.part_ml[slot * 2] = run_max;
    p.part_ml[slot * 2 + 1] = run_sum;
    float* po = p.part_o + slot * D;
#pragma unroll
    for (int x = 0; x < D; x += 4)
      *reinterpret_cast<float4*>(po + x) = make_float4(o[x], o[x + 1], o[x + 2], o[x + 3]);
  }
}

}  // namespace

hipError_t launch_prefix_generic(const AttnParams& p, hipStream_t stream) {
  if (p.S <= 0) return hipSuccess;
  dim3 grid(p.S, p.Hkv, (p.M + kRowsPerBlock - 1) / kRowsPerBlock);
  dim3 block(kRowsPerBlock);
  const bool bf16 = p.in_dtype == SPECEXT_BF16;
  if (p.d == 128) {
    if (bf16) prefix_generic_kernel<128, true><<<grid, block, 0, stream>>>(p);
    else prefix_generic_kernel<128, false><<<grid, block, 0, stream>>>(p);
  } else {
    if (bf16) prefix_generic_kernel<64, true><<<grid, block, 0, stream>>>(p);
    else prefix_generic_kernel<64, false><<<grid, block, 0, stream>>>(p);
  }
  return hipGetLastError();
}

}  // namespace specext
