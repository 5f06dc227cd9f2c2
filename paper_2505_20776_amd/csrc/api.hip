// C ABI of libspecext: argument validation, workspace layout, kernel dispatch.
// See include/specext.h for the contract of every entry point.
#include <atomic>
#include <cmath>
#include <cstring>

#include "common.h"

namespace specext {
namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct WorkspaceLayout {
  size_t status_off, lse2_off, part_ml_off, part_o_off, chunk_off, total;
};
// Head of every workspace, the same for every descriptor (so that one specext_workspace_init
// serves whatever problems the workspace is later used for): status word at byte 0, the
// initialisation mark at byte 8, the hand-over blocks of the fused merge tail from byte 256 on.
constexpr size_t kCookieOff = 8;
constexpr size_t kSyncOff = 256;
constexpr size_t kHeaderBytes = kSyncOff + kMaxSyncBlocks * sizeof(SyncBlock);
static_assert(kHeaderBytes == SPECEXT_WORKSPACE_HEADER_BYTES, "the header states the size of the workspace head");
constexpr int kDefaultSpinLimit = 1 << 16;     // polls of roughly a microsecond each

__global__ void workspace_init_kernel(uint32_t* head) {
  for (unsigned i = threadIdx.x; i < kHeaderBytes / 4; i += blockDim.x) {
    uint32_t v = 0;
    if (i == kCookieOff / 4) v = static_cast<uint32_t>(kWorkspaceCookie);
    if (i == kCookieOff / 4 + 1) v = static_cast<uint32_t>(kWorkspaceCookie >> 32);
    head[i] = v;
  }
}

// Compute-unit count of the current device, cached per process.
int device_cu_count() {
  static std::atomic<int> cached{0};
  int v = cached.load(std::memory_order_relaxed);
  if (v > 0) return v;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
  cached.store(cus, std::memory_order_relaxed);
  return cus;
}

int64_t gcd64(int64_t a, int64_t b) {
  while (b) {
    const int64_t t = a % b;
    a = b;
    b = t;
  }
  return a;
}

// Validate the descriptor and resolve every default.  Pointers are not looked at here.
int resolve(const specext_desc* d, AttnParams* p) {
  if (!d || d->struct_size != sizeof(specext_desc)) return SPECEXT_ERR_INVALID_ARG;
  if (d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->prefix_len < 0 || d->n_tree <= 0 || d->num_splits < 0)
    return SPECEXT_ERR_INVALID_ARG;
  if (d->n_q_heads % d->n_kv_heads != 0) return SPECEXT_ERR_INVALID_ARG;
  if (d->want_scores && d->chunk_size <= 0) return SPECEXT_ERR_INVALID_ARG;
  // bounds that keep the 32-bit length arithmetic below exact (rounding a length up to a chunk or a split unit)
  if (d->prefix_len > (1 << 30) || (d->want_scores && d->chunk_size > (1 << 24))) return SPECEXT_ERR_UNSUPPORTED;
  if (!(d->softmax_scale >= 0.f) || std::isinf(d->softmax_scale)) return SPECEXT_ERR_INVALID_ARG;
  if (d->reserved != 0 || (d->flags & ~(SPECEXT_FLAG_VALU_PREFIX | SPECEXT_FLAG_PREFIX_ONLY | SPECEXT_FLAG_FUSED_MERGE |
                                       SPECEXT_FLAG_SHORT_WAIT)) != 0) return SPECEXT_ERR_INVALID_ARG;
  if (d->dtype != SPECEXT_F32 && d->dtype != SPECEXT_BF16) return SPECEXT_ERR_UNSUPPORTED;
  if (d->out_dtype != SPECEXT_F32 && d->out_dtype != d->dtype) return SPECEXT_ERR_UNSUPPORTED;
  if (d->head_dim != 64 && d->head_dim != 128) return SPECEXT_ERR_UNSUPPORTED;
  if (d->n_tree > SPECEXT_MAX_TREE || d->num_splits > SPECEXT_MAX_SPLITS) return SPECEXT_ERR_UNSUPPORTED;
  if (static_cast<int64_t>(d->n_q_heads) * d->n_tree > (1 << 20)) return SPECEXT_ERR_UNSUPPORTED;

  std::memset(p, 0, sizeof(*p));
  p->Hq = d->n_q_heads;
  p->Hkv = d->n_kv_heads;
  p->G = p->Hq / p->Hkv;
  p->d = d->head_dim;
  p->L = d->prefix_len;
  p->T = d->n_tree;
  p->M = p->T * p->G;
  p->want_scores = d->want_scores ? 1 : 0;
  p->B = p->want_scores ? d->chunk_size : 1;
  p->C = p->want_scores ? (p->L + p->B - 1) / p->B : 0;
  p->in_dtype = d->dtype;
  p->out_dtype = d->out_dtype;
  const float scale = d->softmax_scale > 0.f ? d->softmax_scale : 1.0f / std::sqrt(static_cast<float>(p->d));
  p->scale_log2 = scale * kLog2e;
  p->q_st = d->q_stride_t ? d->q_stride_t : static_cast<int64_t>(p->Hq) * p->d;
  p->q_sh = d->q_stride_h ? d->q_stride_h : p->d;
  p->kp_sh = d->kp_stride_h ? d->kp_stride_h : static_cast<int64_t>(p->L) * p->d;
  p->kp_sl = d->kp_stride_l ? d->kp_stride_l : p->d;
  p->kt_sh = d->kt_stride_h ? d->kt_stride_h : static_cast<int64_t>(p->T) * p->d;
  p->kt_st = d->kt_stride_t ? d->kt_stride_t : p->d;
  p->o_st = d->o_stride_t ? d->o_stride_t : static_cast<int64_t>(p->Hq) * p->d;
  p->o_sh = d->o_stride_h ? d->o_stride_h : p->d;
  const int64_t strides[] = {p->q_st, p->q_sh, p->kp_sh, p->kp_sl, p->kt_sh, p->kt_st, p->o_st, p->o_sh};
  for (int64_t s : strides)
    if (s < 0 || s % 8 != 0) return SPECEXT_ERR_UNSUPPORTED;
  if (p->q_sh < p->d || p->kp_sl < p->d || p->kt_st < p->d || p->o_sh < p->d) return SPECEXT_ERR_INVALID_ARG;

  // Which prefix kernel runs.  The matrix-core kernels take bf16, d = 128, at least one
  // full 32-key tile and, when scores are wanted, chunk sizes that are whole tiles.
  // Up to 32 query rows per KV head: the key-split kernel (the four waves of a
  // workgroup share the rows and split the keys).  More rows: the row-split kernel
  // (a workgroup owns 128 or 256 rows, so each K/V byte enters one compute unit only;
  // measured faster from 33 rows on, also when most of a workgroup's rows are padding).
  // Their address arithmetic inside a tile and inside Q is 32-bit, hence the stride limits.
  const bool mfma_common = p->in_dtype == SPECEXT_BF16 && (!p->want_scores || p->B % 32 == 0) &&
                           !(d->flags & SPECEXT_FLAG_VALU_PREFIX) && p->kp_sl <= (1 << 24) &&
                           (p->T - 1) * p->q_st + (p->Hq - 1) * p->q_sh + p->d < (int64_t{1} << 30);
  const bool mfma_ok = mfma_common && p->d == 128 && p->L >= 32;
  // head_dim 64 (small draft models): the row-split kernel with two keys per LDS row, which needs the
  // keys of a head contiguous in memory and at least one 64-key tile
  const bool mfma64_ok = mfma_common && p->d == 64 && p->kp_sl == 64 && p->L >= 64;
  if (mfma64_ok) {
    p->use_mfma = 2;
    p->rows_per_group = p->M > 128 ? 256 : 128;
    p->part_f16 = 0;
  } else if (!mfma_ok) {
    p->use_mfma = 0;
    p->rows_per_group = 64;
  } else if (p->M <= 32) {
    p->use_mfma = 1;
    p->rows_per_group = 32;
  } else {
    p->use_mfma = 2;
    p->rows_per_group = p->M > 128 ? 256 : 128;
    p->part_f16 = 1;
  }
  p->score_gran = p->use_mfma ? 32 : p->B;
  p->n_sub = p->want_scores ? (p->L + p->score_gran - 1) / p->score_gran : 0;

  // Split the prefix.  Every split but the last holds keys_per_split keys: a
  // multiple of the kernel's key granule (4 waves x 32 keys on the matrix-core
  // path, 64 otherwise) and, with scores, of the chunk size, so that no chunk
  // is shared by two splits.
  if (p->L == 0) {
    p->S = 0;
    p->keys_per_split = 128;
    return SPECEXT_OK;
  }
  int64_t unit = p->use_mfma == 1 ? 128 : 64;
  if (p->want_scores) unit = unit / gcd64(unit, p->B) * p->B;
  int want = d->num_splits;
  if (want == 0) {
    // one workgroup per compute unit: splits x KV heads x row groups ~ CU count
    const int cus = device_cu_count();
    const int row_groups = (p->M + p->rows_per_group - 1) / p->rows_per_group;
    want = cus / (p->Hkv * row_groups);
    // short prefixes: eight key tiles per split, four while that keeps the split count at 16 or
    // below (measured at 1K - 8K tokens: more splits shorten the prefix kernel by less than they
    // add to the merge, fewer leave most compute units idle)
    const int by_256 = static_cast<int>((p->L + 255) / 256), by_128 = static_cast<int>((p->L + 127) / 128);
    const int by_len = by_256 > (by_128 < 16 ? by_128 : 16) ? by_256 : (by_128 < 16 ? by_128 : 16);
    if (want > by_len) want = by_len;
    if (want < 1) want = 1;
  }
  if (want > SPECEXT_MAX_SPLITS) want = SPECEXT_MAX_SPLITS;
  int64_t per = (p->L + want - 1) / want;
  per = (per + unit - 1) / unit * unit;
  p->keys_per_split = static_cast<int32_t>(per);
  p->S = static_cast<int32_t>((p->L + per - 1) / per);
  // Tree pass and merge as the tail of the prefix launch (on request): row-split kernel
  // only, and only when all its workgroups fit the device at once (one per compute unit),
  // so that in the normal case nobody waits for a workgroup that has not started.
  const int64_t row_groups = (p->M + p->rows_per_group - 1) / p->rows_per_group;
  // Workgroups are dealt to the eight XCDs in turn: with the KV head in the fastest grid index and a
  // multiple of eight heads, all splits of a head run on one XCD, and the head's queries (the only
  // bytes its workgroups share) are fetched from HBM once instead of once per XCD.  Same run time
  // (measured), 3.4 MB less HBM traffic per launch at the Llama-3.1-8B shape.
  p->head_fastest = p->Hkv % 8 == 0 ? 1 : 0;
  p->spin_limit = (d->flags & SPECEXT_FLAG_SHORT_WAIT) ? 0 : kDefaultSpinLimit;
  p->fused_tail = p->use_mfma == 2 && p->part_f16 && p->S <= 64 && p->L > 0 && p->Hkv * row_groups <= kMaxSyncBlocks &&
                  p->S * p->Hkv * row_groups <= device_cu_count() &&
                  (d->flags & SPECEXT_FLAG_FUSED_MERGE) && !(d->flags & SPECEXT_FLAG_PREFIX_ONLY);
  return SPECEXT_OK;
}

WorkspaceLayout layout_of(const AttnParams& p) {
  WorkspaceLayout w;
  const size_t rows = static_cast<size_t>(p.Hq) * p.T;
  size_t off = 0;
  w.status_off = off;
  off += kHeaderBytes;
  w.lse2_off = off;
  off += align_up(rows * sizeof(float));
  w.part_ml_off = off;
  off += align_up(static_cast<size_t>(p.S) * rows * 2 * sizeof(float));
  w.part_o_off = off;
  off += align_up(static_cast<size_t>(p.S) * rows * p.d * sizeof(float));
  w.chunk_off = off;
  if (p.want_scores) off += align_up(rows * static_cast<size_t>(p.n_sub) * 2 * sizeof(float));
  w.total = off;
  return w;
}

void bind_workspace(AttnParams* p, const WorkspaceLayout& w, void* workspace) {
  char* base = static_cast<char*>(workspace);
  p->status = reinterpret_cast<int32_t*>(base + w.status_off);
  p->lse2 = reinterpret_cast<float*>(base + w.lse2_off);
  p->part_ml = reinterpret_cast<float*>(base + w.part_ml_off);
  p->part_o = reinterpret_cast<float*>(base + w.part_o_off);
  p->chunk_part = p->want_scores ? reinterpret_cast<float*>(base + w.chunk_off) : nullptr;
  p->sync = reinterpret_cast<SyncBlock*>(base + kSyncOff);
  p->cookie = reinterpret_cast<const uint64_t*>(base + kCookieOff);
}

inline bool aligned16(const void* ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15u) == 0; }

// Shapes of the materialised path: row pitch, key blocking of its two matrix products
// (about one workgroup per compute unit each), byte offsets of its two buffers.
struct MatLayout {
  size_t probs_off, part_off, total;
};
int resolve_materialized(const specext_desc* d, MatParams* mp, MatLayout* w) {
  const int rc = resolve(d, &mp->a);
  if (rc != SPECEXT_OK) return rc;
  const AttnParams& a = mp->a;
  if (a.in_dtype != SPECEXT_BF16 || a.d != 128) return SPECEXT_ERR_UNSUPPORTED;
  const int64_t n = static_cast<int64_t>(a.L) + a.T;
  const int64_t ld = (n + 63) / 64 * 64;
  if (ld * a.Hq * a.T > (int64_t{1} << 32)) return SPECEXT_ERR_UNSUPPORTED;   // a matrix of more than 16 GiB
  mp->ld = static_cast<int32_t>(ld);
  const int row_blocks = (a.M + 31) / 32;
  const int waves = row_blocks < 8 ? row_blocks : 8;
  const int row_groups = (row_blocks + waves - 1) / waves;
  mp->m_pad = row_groups * waves * 32;
  const int cus = device_cu_count();
  int want = cus / (a.Hkv * row_groups);
  if (want < 1) want = 1;
  auto per_block = [&](int64_t keys) {
    int64_t per = (keys + want - 1) / want;
    per = (per + 31) / 32 * 32;
    return static_cast<int32_t>(per < 32 ? 32 : per);
  };
  mp->logit_keys_per_block = per_block(a.L);
  mp->pv_keys_per_split = per_block(n);
  mp->pv_splits = static_cast<int32_t>((n + mp->pv_keys_per_split - 1) / mp->pv_keys_per_split);
  size_t off = kAlign;
  w->probs_off = off;
  off += align_up(static_cast<size_t>(a.Hq) * a.T * ld * sizeof(float));
  w->part_off = off;
  off += align_up(static_cast<size_t>(mp->pv_splits) * a.Hkv * mp->m_pad * a.d * sizeof(float));
  w->total = off;
  return SPECEXT_OK;
}

// Scratch memory of specext_verify_attn_static: one array per GPU that loads this code
// object, held until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the device address it returns (one per device) is what the kernels
// are given.
constexpr size_t kStaticScratchBytes = size_t{SPECEXT_STATIC_SCRATCH_MIB} << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

void* static_scratch_of_current_device() {
  constexpr int kMaxDevices = 64;
  static std::atomic<void*> cached[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* ptr = cached[dev].load(std::memory_order_acquire);
  if (ptr) return ptr;
  if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
  cached[dev].store(ptr, std::memory_order_release);
  return ptr;
}

// specext_verify_attn on an explicit workspace; status_word != nullptr redirects the status word
int verify_attn_on(const specext_desc* desc, const void* q, const void* k_prefix, const void* v_prefix,
                   const void* k_tree, const void* v_tree, const int32_t* parent, void* out, float* lse,
                   void* workspace, size_t workspace_bytes, int32_t* status_word, bool library_memory, void* stream) {
  AttnParams p;
  const int rc = resolve(desc, &p);
  if (rc != SPECEXT_OK) return rc;
  if (!q || !k_tree || !v_tree || !parent || !out || !workspace) return SPECEXT_ERR_INVALID_ARG;
  if (p.L > 0 && (!k_prefix || !v_prefix)) return SPECEXT_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_prefix) || !aligned16(v_prefix) || !aligned16(k_tree) || !aligned16(v_tree) ||
      !aligned16(out) || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0 ||
      (reinterpret_cast<uintptr_t>(parent) & 3u) != 0 || (reinterpret_cast<uintptr_t>(lse) & 3u) != 0)
    return SPECEXT_ERR_UNSUPPORTED;
  const WorkspaceLayout w = layout_of(p);
  if (workspace_bytes < w.total) return SPECEXT_ERR_WORKSPACE_TOO_SMALL;
  p.q = q;
  p.kp = k_prefix;
  p.vp = v_prefix;
  p.kt = k_tree;
  p.vt = v_tree;
  p.parent = parent;
  p.out = out;
  p.lse = lse;
  bind_workspace(&p, w, workspace);
  if (library_memory) p.cookie = nullptr;      // the static scratch array: zero when the code object is loaded, cleared by every call
  if (status_word) p.status = status_word;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (p.S > 0) {
    const hipError_t e = p.use_mfma == 2   ? launch_prefix_mfma_rows(p, s)
                         : p.use_mfma == 1 ? launch_prefix_mfma(p, s)
                                           : launch_prefix_generic(p, s);
    if (e != hipSuccess) return SPECEXT_ERR_LAUNCH_FAILED;
  }
  if ((desc->flags & SPECEXT_FLAG_PREFIX_ONLY) || (p.fused_tail && p.S > 0)) return SPECEXT_OK;
  if (launch_tree_merge(p, s) != hipSuccess) return SPECEXT_ERR_LAUNCH_FAILED;
  return SPECEXT_OK;
}

}  // namespace
}  // namespace specext

using namespace specext;

extern "C" {

const char* specext_strerror(int status) {
  switch (status) {
    case SPECEXT_OK: return "ok";
    case SPECEXT_ERR_INVALID_ARG: return "invalid argument";
    case SPECEXT_ERR_UNSUPPORTED: return "unsupported dtype, shape or alignment";
    case SPECEXT_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case SPECEXT_ERR_LAUNCH_FAILED: return "kernel launch failed";
    default: return "unknown status";
  }
}

size_t specext_workspace_bytes(const specext_desc* desc) {
  AttnParams p;
  if (resolve(desc, &p) != SPECEXT_OK) return 0;
  return layout_of(p).total;
}

int specext_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  if (!workspace) return SPECEXT_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) return SPECEXT_ERR_UNSUPPORTED;
  if (workspace_bytes < kHeaderBytes) return SPECEXT_ERR_WORKSPACE_TOO_SMALL;
  workspace_init_kernel<<<1, 1024, 0, static_cast<hipStream_t>(stream)>>>(static_cast<uint32_t*>(workspace));
  return hipGetLastError() == hipSuccess ? SPECEXT_OK : SPECEXT_ERR_LAUNCH_FAILED;
}

#ifdef SPECEXT_TAIL_STAMPS
// Profiling builds only (not in the public header): byte offset, inside the workspace, of the phase stamps the
// row-split prefix kernel leaves per workgroup - eight 64-bit wall-clock values (100 MHz) for workgroup
// (row group z, KV head g, split s) at index ((z * Hkv + g) * S + s) * 8.  0 if the descriptor takes another kernel.
size_t specext_debug_stamps_offset(const specext_desc* desc) {
  AttnParams p;
  if (resolve(desc, &p) != SPECEXT_OK || p.use_mfma != 2 || !p.part_f16) return 0;
  return layout_of(p).part_o_off + static_cast<size_t>(p.S) * p.Hq * p.T * p.d * 2;
}
#endif

int specext_num_splits(const specext_desc* desc) {
  AttnParams p;
  const int rc = resolve(desc, &p);
  if (rc != SPECEXT_OK) return rc;
  return p.S;
}

int specext_verify_attn(const specext_desc* desc, const void* q, const void* k_prefix, const void* v_prefix,
                        const void* k_tree, const void* v_tree, const int32_t* parent, void* out, float* lse,
                        void* workspace, size_t workspace_bytes, void* stream) {
  return verify_attn_on(desc, q, k_prefix, v_prefix, k_tree, v_tree, parent, out, lse, workspace, workspace_bytes,
                        nullptr, false, stream);
}

int specext_verify_attn_static(const specext_desc* desc, const void* q, const void* k_prefix, const void* v_prefix,
                               const void* k_tree, const void* v_tree, const int32_t* parent, void* out, float* lse,
                               int32_t* status_out, void* stream) {
  AttnParams p;
  const int rc = resolve(desc, &p);
  if (rc != SPECEXT_OK) return rc;
  // the chunk partial sums would have to outlive the call for specext_chunk_scores, which
  // takes the caller's workspace: the layer that feeds the retrieval uses specext_verify_attn
  if (p.want_scores) return SPECEXT_ERR_UNSUPPORTED;
  if (reinterpret_cast<uintptr_t>(status_out) & 3u) return SPECEXT_ERR_UNSUPPORTED;
  if (layout_of(p).total > kStaticScratchBytes) return SPECEXT_ERR_WORKSPACE_TOO_SMALL;
  void* ws = static_scratch_of_current_device();
  if (!ws) return SPECEXT_ERR_LAUNCH_FAILED;
  return verify_attn_on(desc, q, k_prefix, v_prefix, k_tree, v_tree, parent, out, lse, ws, kStaticScratchBytes,
                        status_out, true, stream);
}

int specext_chunk_scores(const specext_desc* desc, const void* workspace, size_t workspace_bytes,
                         int32_t score_row, float* scores, void* stream) {
  AttnParams p;
  const int rc = resolve(desc, &p);
  if (rc != SPECEXT_OK) return rc;
  if (!workspace || !scores || !p.want_scores || p.C <= 0) return SPECEXT_ERR_INVALID_ARG;
  if (score_row < -1 || score_row >= p.T) return SPECEXT_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0 || (reinterpret_cast<uintptr_t>(scores) & 3u) != 0)
    return SPECEXT_ERR_UNSUPPORTED;
  const WorkspaceLayout w = layout_of(p);
  if (workspace_bytes < w.total) return SPECEXT_ERR_WORKSPACE_TOO_SMALL;
  bind_workspace(&p, w, const_cast<void*>(workspace));
  if (launch_chunk_scores(p, score_row, nullptr, nullptr, scores, static_cast<hipStream_t>(stream)) != hipSuccess)
    return SPECEXT_ERR_LAUNCH_FAILED;
  return SPECEXT_OK;
}

int specext_chunk_scores_accepted(const specext_desc* desc, const void* workspace, size_t workspace_bytes,
                                  const int32_t* path, const int32_t* n_accept, float* scores, void* stream) {
  AttnParams p;
  const int rc = resolve(desc, &p);
  if (rc != SPECEXT_OK) return rc;
  if (!workspace || !scores || !path || !n_accept || !p.want_scores || p.C <= 0) return SPECEXT_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0 || (reinterpret_cast<uintptr_t>(scores) & 3u) ||
      (reinterpret_cast<uintptr_t>(path) & 3u) || (reinterpret_cast<uintptr_t>(n_accept) & 3u))
    return SPECEXT_ERR_UNSUPPORTED;
  const WorkspaceLayout w = layout_of(p);
  if (workspace_bytes < w.total) return SPECEXT_ERR_WORKSPACE_TOO_SMALL;
  bind_workspace(&p, w, const_cast<void*>(workspace));
  if (launch_chunk_scores(p, 0, path, n_accept, scores, static_cast<hipStream_t>(stream)) != hipSuccess)
    return SPECEXT_ERR_LAUNCH_FAILED;
  return SPECEXT_OK;
}

int specext_chunk_scores_select(const specext_desc* desc, const void* workspace, size_t workspace_bytes,
                                int32_t score_row, const int32_t* path, const int32_t* n_accept, int32_t k,
                                float* scores, int32_t* idx_out, int32_t* n_out, void* stream) {
  AttnParams p;
  const int rc = resolve(desc, &p);
  if (rc != SPECEXT_OK) return rc;
  if (!workspace || !n_out || !p.want_scores || p.C <= 0 || k < 0 || (k > 0 && !idx_out)) return SPECEXT_ERR_INVALID_ARG;
  if ((path == nullptr) != (n_accept == nullptr)) return SPECEXT_ERR_INVALID_ARG;
  if (!path && (score_row < 0 || score_row >= p.T)) return SPECEXT_ERR_INVALID_ARG;
  if (p.C > 65536) return SPECEXT_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0 || (reinterpret_cast<uintptr_t>(scores) & 3u) ||
      (reinterpret_cast<uintptr_t>(path) & 3u) || (reinterpret_cast<uintptr_t>(n_accept) & 3u) ||
      (reinterpret_cast<uintptr_t>(idx_out) & 3u) || (reinterpret_cast<uintptr_t>(n_out) & 3u))
    return SPECEXT_ERR_UNSUPPORTED;
  // beyond what one workgroup ranks, the two steps run as two launches and need the scores in memory
  if (p.C > 1024 && !scores) return SPECEXT_ERR_INVALID_ARG;
  const WorkspaceLayout w = layout_of(p);
  if (workspace_bytes < w.total) return SPECEXT_ERR_WORKSPACE_TOO_SMALL;
  bind_workspace(&p, w, const_cast<void*>(workspace));
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int32_t row = path ? 0 : score_row;
  if (p.C <= 1024) {
    if (launch_score_select(p, row, path, n_accept, k, scores, idx_out, n_out, s) != hipSuccess)
      return SPECEXT_ERR_LAUNCH_FAILED;
    return SPECEXT_OK;
  }
  if (launch_chunk_scores(p, row, path, n_accept, scores, s) != hipSuccess) return SPECEXT_ERR_LAUNCH_FAILED;
  if (launch_select_chunks(scores, p.C, k, idx_out, n_out, s) != hipSuccess) return SPECEXT_ERR_LAUNCH_FAILED;
  return SPECEXT_OK;
}

size_t specext_materialized_bytes(const specext_desc* desc) {
  MatParams mp;
  MatLayout w;
  if (resolve_materialized(desc, &mp, &w) != SPECEXT_OK) return 0;
  return w.total;
}

int specext_materialized_ld(const specext_desc* desc) {
  MatParams mp;
  MatLayout w;
  const int rc = resolve_materialized(desc, &mp, &w);
  return rc != SPECEXT_OK ? rc : mp.ld;
}

int specext_attn_materialized(const specext_desc* desc, const void* q, const void* k_prefix, const void* v_prefix,
                              const void* k_tree, const void* v_tree, const int32_t* parent, void* out, float* lse,
                              void* workspace, size_t workspace_bytes, void* stream) {
  MatParams mp;
  MatLayout w;
  const int rc = resolve_materialized(desc, &mp, &w);
  if (rc != SPECEXT_OK) return rc;
  AttnParams& p = mp.a;
  if (!q || !k_tree || !v_tree || !parent || !out || !workspace) return SPECEXT_ERR_INVALID_ARG;
  if (p.L > 0 && (!k_prefix || !v_prefix)) return SPECEXT_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_prefix) || !aligned16(v_prefix) || !aligned16(k_tree) || !aligned16(v_tree) ||
      !aligned16(out) || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0 ||
      (reinterpret_cast<uintptr_t>(parent) & 3u) != 0 || (reinterpret_cast<uintptr_t>(lse) & 3u) != 0)
    return SPECEXT_ERR_UNSUPPORTED;
  if (workspace_bytes < w.total) return SPECEXT_ERR_WORKSPACE_TOO_SMALL;
  p.q = q;
  p.kp = k_prefix;
  p.vp = v_prefix;
  p.kt = k_tree;
  p.vt = v_tree;
  p.parent = parent;
  p.out = out;
  p.lse = lse;
  p.status = static_cast<int32_t*>(workspace);
  mp.probs = reinterpret_cast<float*>(static_cast<char*>(workspace) + w.probs_off);
  mp.part = reinterpret_cast<float*>(static_cast<char*>(workspace) + w.part_off);
  if (launch_materialized(mp, static_cast<hipStream_t>(stream)) != hipSuccess) return SPECEXT_ERR_LAUNCH_FAILED;
  return SPECEXT_OK;
}

int specext_chunk_scores_materialized(const specext_desc* desc, const void* workspace, size_t workspace_bytes,
                                      int32_t score_row, const int32_t* path, const int32_t* n_accept,
                                      float* scores, void* stream) {
  MatParams mp;
  MatLayout w;
  const int rc = resolve_materialized(desc, &mp, &w);
  if (rc != SPECEXT_OK) return rc;
  if (!workspace || !scores || !mp.a.want_scores || mp.a.C <= 0) return SPECEXT_ERR_INVALID_ARG;
  if ((path == nullptr) != (n_accept == nullptr)) return SPECEXT_ERR_INVALID_ARG;
  if (!path && (score_row < 0 || score_row >= mp.a.T)) return SPECEXT_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0 || (reinterpret_cast<uintptr_t>(scores) & 3u) ||
      (reinterpret_cast<uintptr_t>(path) & 3u) || (reinterpret_cast<uintptr_t>(n_accept) & 3u))
    return SPECEXT_ERR_UNSUPPORTED;
  if (workspace_bytes < w.total) return SPECEXT_ERR_WORKSPACE_TOO_SMALL;
  mp.probs = reinterpret_cast<float*>(static_cast<char*>(const_cast<void*>(workspace)) + w.probs_off);
  mp.part = nullptr;
  if (launch_materialized_scores(mp, path ? 0 : score_row, path, n_accept, scores,
                                 static_cast<hipStream_t>(stream)) != hipSuccess)
    return SPECEXT_ERR_LAUNCH_FAILED;
  return SPECEXT_OK;
}

int specext_prefill_attn(const void* q, const void* k, const void* v, void* out, float* lse, int32_t n_q_heads,
                         int32_t n_kv_heads, int32_t head_dim, int32_t q_len, int32_t kv_len, int32_t dtype,
                         int32_t out_dtype, float softmax_scale, int64_t q_stride_t, int64_t q_stride_h,
                         int64_t kv_stride_h, int64_t kv_stride_l, int64_t o_stride_t, int64_t o_stride_h,
                         void* stream) {
  if (!q || !k || !v || !out) return SPECEXT_ERR_INVALID_ARG;
  if (n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads != 0 || q_len <= 0 || kv_len < q_len ||
      head_dim <= 0)
    return SPECEXT_ERR_INVALID_ARG;
  if (!(softmax_scale >= 0.f) || std::isinf(softmax_scale)) return SPECEXT_ERR_INVALID_ARG;
  if (dtype != SPECEXT_BF16 || (out_dtype != SPECEXT_BF16 && out_dtype != SPECEXT_F32) || head_dim != 128 ||
      kv_len < 32)
    return SPECEXT_ERR_UNSUPPORTED;
  PrefillParams p;
  std::memset(&p, 0, sizeof(p));
  p.Hq = n_q_heads;
  p.Hkv = n_kv_heads;
  p.G = n_q_heads / n_kv_heads;
  p.Tq = q_len;
  p.N = kv_len;
  p.q_off = kv_len - q_len;
  p.out_dtype = out_dtype;
  if (static_cast<int64_t>(q_len) * p.G > (1 << 24)) return SPECEXT_ERR_UNSUPPORTED;
  p.M = q_len * p.G;
  const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / std::sqrt(static_cast<float>(head_dim));
  p.scale_log2 = scale * kLog2e;
  p.q_st = q_stride_t ? q_stride_t : static_cast<int64_t>(n_q_heads) * head_dim;
  p.q_sh = q_stride_h ? q_stride_h : head_dim;
  p.k_sl = kv_stride_l ? kv_stride_l : head_dim;
  p.k_sh = kv_stride_h ? kv_stride_h : static_cast<int64_t>(kv_len) * p.k_sl;
  p.o_st = o_stride_t ? o_stride_t : static_cast<int64_t>(n_q_heads) * head_dim;
  p.o_sh = o_stride_h ? o_stride_h : head_dim;
  const int64_t strides[] = {p.q_st, p.q_sh, p.k_sh, p.k_sl, p.o_st, p.o_sh};
  for (int64_t s : strides)
    if (s < 0 || s % 8 != 0) return SPECEXT_ERR_UNSUPPORTED;
  if (p.q_sh < head_dim || p.k_sl < head_dim || p.o_sh < head_dim) return SPECEXT_ERR_INVALID_ARG;
  // 32-bit address arithmetic inside a K/V tile and inside the queries of one workgroup
  if (p.k_sl > (1 << 24) || p.q_st > (1 << 20) || static_cast<int64_t>(n_q_heads) * p.q_sh > (1 << 24))
    return SPECEXT_ERR_UNSUPPORTED;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || (reinterpret_cast<uintptr_t>(lse) & 3u))
    return SPECEXT_ERR_UNSUPPORTED;
  p.q = q;
  p.k = k;
  p.v = v;
  p.out = out;
  p.lse = lse;
  if (launch_prefill_rows(p, static_cast<hipStream_t>(stream)) != hipSuccess) return SPECEXT_ERR_LAUNCH_FAILED;
  return SPECEXT_OK;
}

int specext_accept_greedy(const int32_t* parent, const int32_t* draft_token, const int32_t* target_token,
                          const int32_t* first_target, int32_t n_tree, int32_t* path_out, int32_t* n_accept_out,
                          int32_t* next_token_out, void* stream) {
  if (!parent || !draft_token || !target_token || !first_target || !path_out || !n_accept_out || !next_token_out ||
      n_tree <= 0)
    return SPECEXT_ERR_INVALID_ARG;
  if (n_tree > SPECEXT_MAX_TREE) return SPECEXT_ERR_UNSUPPORTED;
  const void* ptrs[] = {parent, draft_token, target_token, first_target, path_out, n_accept_out, next_token_out};
  for (const void* q : ptrs)
    if (reinterpret_cast<uintptr_t>(q) & 3u) return SPECEXT_ERR_UNSUPPORTED;
  if (launch_accept_greedy(parent, draft_token, target_token, first_target, n_tree, path_out, n_accept_out,
                           next_token_out, static_cast<hipStream_t>(stream)) != hipSuccess)
    return SPECEXT_ERR_LAUNCH_FAILED;
  return SPECEXT_OK;
}

int specext_commit_tree_kv(const void* k_tree, const void* v_tree, void* k_cache, void* v_cache,
                           const int32_t* path, const int32_t* n_accept, int32_t max_accept, int32_t n_tree,
                           int32_t n_layers, int32_t n_kv_heads, int32_t head_dim, int32_t elem_bytes,
                           int32_t prefix_len, int32_t cache_capacity, int64_t tree_stride_layer,
                           int64_t tree_stride_h, int64_t tree_stride_t, int64_t cache_stride_layer,
                           int64_t cache_stride_h, int64_t cache_stride_l, void* stream) {
  if (!k_tree || !v_tree || !k_cache || !v_cache || !path || !n_accept) return SPECEXT_ERR_INVALID_ARG;
  if (max_accept < 0 || n_tree <= 0 || n_layers <= 0 || n_kv_heads <= 0 || head_dim <= 0 || elem_bytes <= 0 ||
      prefix_len < 0 || tree_stride_layer < 0 || tree_stride_h < 0 || tree_stride_t < 0 || cache_stride_layer < 0 ||
      cache_stride_h < 0 || cache_stride_l < 0)
    return SPECEXT_ERR_INVALID_ARG;
  if (static_cast<int64_t>(prefix_len) + max_accept > cache_capacity) return SPECEXT_ERR_INVALID_ARG;
  if (n_tree > SPECEXT_MAX_TREE || max_accept > SPECEXT_MAX_TREE ||
      static_cast<int64_t>(n_layers) * n_kv_heads > 65535)
    return SPECEXT_ERR_UNSUPPORTED;
  const int64_t row_bytes = static_cast<int64_t>(head_dim) * elem_bytes;
  const int64_t tst = (tree_stride_t ? tree_stride_t : head_dim) * elem_bytes;
  const int64_t tsh = tree_stride_h ? tree_stride_h * elem_bytes : n_tree * tst;
  const int64_t tsl = tree_stride_layer ? tree_stride_layer * elem_bytes : n_kv_heads * tsh;
  const int64_t csl = (cache_stride_l ? cache_stride_l : head_dim) * elem_bytes;
  const int64_t csh = cache_stride_h ? cache_stride_h * elem_bytes : cache_capacity * csl;
  const int64_t csy = cache_stride_layer ? cache_stride_layer * elem_bytes : n_kv_heads * csh;
  if (row_bytes % 16 || tsl % 16 || tsh % 16 || tst % 16 || csy % 16 || csh % 16 || csl % 16 || tst < row_bytes ||
      csl < row_bytes)
    return SPECEXT_ERR_UNSUPPORTED;
  if (!aligned16(k_tree) || !aligned16(v_tree) || !aligned16(k_cache) || !aligned16(v_cache) ||
      (reinterpret_cast<uintptr_t>(path) & 3u) || (reinterpret_cast<uintptr_t>(n_accept) & 3u))
    return SPECEXT_ERR_UNSUPPORTED;
  if (launch_commit_tree_kv(k_tree, v_tree, k_cache, v_cache, path, n_accept, max_accept, n_tree, n_layers,
                            n_kv_heads, prefix_len, static_cast<int32_t>(row_bytes), tsl, tsh, tst, csy, csh, csl,
                            static_cast<hipStream_t>(stream)) != hipSuccess)
    return SPECEXT_ERR_LAUNCH_FAILED;
  return SPECEXT_OK;
}

int specext_select_chunks(const float* scores, int32_t n_chunks, int32_t k, int32_t* idx_out, int32_t* n_out,
                          void* stream) {
  if (!scores || !n_out || n_chunks <= 0 || k < 0 || (k > 0 && !idx_out)) return SPECEXT_ERR_INVALID_ARG;
  if (n_chunks > 65536) return SPECEXT_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(scores) & 3u) || (reinterpret_cast<uintptr_t>(idx_out) & 3u) ||
      (reinterpret_cast<uintptr_t>(n_out) & 3u))
    return SPECEXT_ERR_UNSUPPORTED;
  if (launch_select_chunks(scores, n_chunks, k, idx_out, n_out, static_cast<hipStream_t>(stream)) != hipSuccess)
    return SPECEXT_ERR_LAUNCH_FAILED;
  return SPECEXT_OK;
}

int specext_gather_draft_kv(const void* k_src, const void* v_src, void* k_dst, void* v_dst, const int32_t* idx,
                            const int32_t* n_idx, int32_t max_idx, int32_t n_layers, int32_t n_kv_heads,
                            int32_t src_len, int32_t src_cap, int32_t dst_cap, int32_t head_dim,
                            int32_t chunk_size, int32_t elem_bytes, int32_t* pos_out, int32_t* len_out,
                            void* stream) {
  if (!k_src || !v_src || !k_dst || !v_dst || !idx) return SPECEXT_ERR_INVALID_ARG;
  if (max_idx < 0 || n_layers <= 0 || n_kv_heads <= 0 || src_len <= 0 || dst_cap < 0 || head_dim <= 0 ||
      chunk_size <= 0 || elem_bytes <= 0)
    return SPECEXT_ERR_INVALID_ARG;
  if (static_cast<int64_t>(max_idx) * chunk_size > dst_cap) return SPECEXT_ERR_INVALID_ARG;
  if (src_cap == 0) src_cap = src_len;
  if (src_cap < src_len) return SPECEXT_ERR_INVALID_ARG;
  const int64_t row_bytes = static_cast<int64_t>(head_dim) * elem_bytes;
  const int64_t n_lh = static_cast<int64_t>(n_layers) * n_kv_heads;
  if (row_bytes % 16 != 0 || row_bytes > (1 << 20) || n_lh > 65535) return SPECEXT_ERR_UNSUPPORTED;
  if (!aligned16(k_src) || !aligned16(v_src) || !aligned16(k_dst) || !aligned16(v_dst)) return SPECEXT_ERR_UNSUPPORTED;
  if (launch_gather(k_src, v_src, k_dst, v_dst, idx, n_idx, max_idx, static_cast<int32_t>(n_lh), src_len, src_cap,
                    dst_cap, static_cast<int32_t>(row_bytes), chunk_size, pos_out, len_out,
                    static_cast<hipStream_t>(stream)) != hipSuccess)
    return SPECEXT_ERR_LAUNCH_FAILED;
  return SPECEXT_OK;
}

}  // extern "C"
