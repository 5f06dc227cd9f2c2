// Host-side argument validation of the C ABI under AddressSanitizer and
// UndefinedBehaviorSanitizer (host code only).  Links api.hip, the only translation unit
// with host logic, against stub launchers, so that no kernel is compiled or launched and no
// GPU is needed: every call below either returns an error before anything would be
// launched, or reaches a stub.  Exit code 0 = every expectation held and no sanitizer fired.
#include <cstdio>
#include <cstring>
#include <vector>

#include "common.h"

namespace specext {
hipError_t launch_prefill_rows(const PrefillParams&, hipStream_t) { return hipSuccess; }
hipError_t launch_materialized(const MatParams&, hipStream_t) { return hipSuccess; }
hipError_t launch_materialized_scores(const MatParams&, int32_t, const int32_t*, const int32_t*, float*, hipStream_t) { return hipSuccess; }
hipError_t launch_prefix_generic(const AttnParams&, hipStream_t) { return hipSuccess; }
hipError_t launch_prefix_mfma(const AttnParams&, hipStream_t) { return hipSuccess; }
hipError_t launch_prefix_mfma_rows(const AttnParams&, hipStream_t) { return hipSuccess; }
hipError_t launch_tree_merge(const AttnParams&, hipStream_t) { return hipSuccess; }
hipError_t launch_chunk_scores(const AttnParams&, int32_t, const int32_t*, const int32_t*, float*, hipStream_t) { return hipSuccess; }
hipError_t launch_score_select(const AttnParams&, int32_t, const int32_t*, const int32_t*, int32_t, float*, int32_t*, int32_t*, hipStream_t) { return hipSuccess; }
hipError_t launch_accept_greedy(const int32_t*, const int32_t*, const int32_t*, const int32_t*, int32_t, int32_t*, int32_t*, int32_t*, hipStream_t) { return hipSuccess; }
hipError_t launch_commit_tree_kv(const void*, const void*, void*, void*, const int32_t*, const int32_t*, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, hipStream_t) { return hipSuccess; }
hipError_t launch_select_chunks(const float*, int32_t, int32_t, int32_t*, int32_t*, hipStream_t) { return hipSuccess; }
hipError_t launch_gather(const void*, const void*, void*, void*, const int32_t*, const int32_t*, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t*, int32_t*, hipStream_t) { return hipSuccess; }
}  // namespace specext

static int failures = 0;
#define EXPECT(cond) do { if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

static specext_desc good_desc() {
  specext_desc d;
  std::memset(&d, 0, sizeof(d));
  d.struct_size = sizeof(d);
  d.dtype = SPECEXT_BF16;
  d.out_dtype = SPECEXT_BF16;
  d.n_q_heads = 32;
  d.n_kv_heads = 8;
  d.head_dim = 128;
  d.prefix_len = 4096;
  d.n_tree = 60;
  d.chunk_size = 32;
  d.want_scores = 1;
  d.num_splits = 8;
  return d;
}

int main() {
  // pointers that are never dereferenced on the host: aligned, non-null
  void* const ok = reinterpret_cast<void*>(uintptr_t{1} << 20);
  void* const odd = reinterpret_cast<void*>((uintptr_t{1} << 20) + 2);
  int32_t* const iok = static_cast<int32_t*>(ok);
  float* const fok = static_cast<float*>(ok);

  specext_desc d = good_desc();
  const size_t ws = specext_workspace_bytes(&d);
  EXPECT(ws > SPECEXT_WORKSPACE_HEADER_BYTES);
  EXPECT(specext_workspace_bytes(nullptr) == 0);
  EXPECT(specext_num_splits(&d) == 8);
  EXPECT(std::strlen(specext_strerror(-3)) > 0 && std::strlen(specext_strerror(12345)) > 0);

  // descriptor fields, one at a time
  struct Case { void (*mutate)(specext_desc&); int want; };
  const Case cases[] = {
      {[](specext_desc& x) { x.struct_size = 8; }, -1},           {[](specext_desc& x) { x.n_q_heads = 0; }, -1},
      {[](specext_desc& x) { x.n_kv_heads = 5; }, -1},            {[](specext_desc& x) { x.prefix_len = -1; }, -1},
      {[](specext_desc& x) { x.n_tree = 0; }, -1},                {[](specext_desc& x) { x.n_tree = 129; }, -2},
      {[](specext_desc& x) { x.num_splits = -1; }, -1},           {[](specext_desc& x) { x.num_splits = 257; }, -2},
      {[](specext_desc& x) { x.chunk_size = 0; }, -1},            {[](specext_desc& x) { x.chunk_size = (1 << 24) + 1; }, -2},
      {[](specext_desc& x) { x.chunk_size = 0x7fffffff; }, -2},   {[](specext_desc& x) { x.softmax_scale = -1.f; }, -1},
      {[](specext_desc& x) { x.prefix_len = 0x7fffffff; }, -2},   {[](specext_desc& x) { x.prefix_len = (1 << 30) + 1; }, -2},
      {[](specext_desc& x) { x.dtype = 7; }, -2},                 {[](specext_desc& x) { x.out_dtype = 3; }, -2},
      {[](specext_desc& x) { x.head_dim = 96; }, -2},             {[](specext_desc& x) { x.flags = 1u << 20; }, -1},
      {[](specext_desc& x) { x.reserved = 1; }, -1},              {[](specext_desc& x) { x.q_stride_h = 12; }, -2},
      {[](specext_desc& x) { x.kp_stride_l = 64; }, -1},          {[](specext_desc& x) { x.n_q_heads = 1 << 20; x.n_kv_heads = 1 << 20; }, -2},
  };
  for (const Case& c : cases) {
    specext_desc x = good_desc();
    c.mutate(x);
    EXPECT(specext_workspace_bytes(&x) == 0);
    EXPECT(specext_num_splits(&x) == c.want);
    EXPECT(specext_verify_attn(&x, ok, ok, ok, ok, ok, iok, ok, fok, ok, size_t{1} << 40, nullptr) == c.want);
    EXPECT(specext_verify_attn_static(&x, ok, ok, ok, ok, ok, iok, ok, fok, iok, nullptr) == c.want);
  }
  // extreme but valid sizes: no overflow in the layout arithmetic
  {
    specext_desc x = good_desc();
    x.prefix_len = 1 << 30;
    x.chunk_size = 1 << 24;
    x.num_splits = 256;
    x.n_tree = 128;
    EXPECT(specext_workspace_bytes(&x) > 0);
    EXPECT(specext_num_splits(&x) > 0);
    x.num_splits = 0;
    EXPECT(specext_workspace_bytes(&x) > 0);
    EXPECT(specext_verify_attn_static(&x, ok, ok, ok, ok, ok, iok, ok, fok, iok, nullptr) == -2);   // want_scores
    x.want_scores = 0;
    x.num_splits = 256;
    EXPECT(specext_verify_attn_static(&x, ok, ok, ok, ok, ok, iok, ok, fok, iok, nullptr) == -3);   // too large for the scratch
  }

  // pointers and sizes of verify_attn
  EXPECT(specext_verify_attn(&d, nullptr, ok, ok, ok, ok, iok, ok, fok, ok, ws, nullptr) == -1);
  EXPECT(specext_verify_attn(&d, ok, nullptr, ok, ok, ok, iok, ok, fok, ok, ws, nullptr) == -1);
  EXPECT(specext_verify_attn(&d, ok, ok, ok, ok, ok, nullptr, ok, fok, ok, ws, nullptr) == -1);
  EXPECT(specext_verify_attn(&d, ok, ok, ok, ok, ok, iok, ok, fok, nullptr, ws, nullptr) == -1);
  EXPECT(specext_verify_attn(&d, odd, ok, ok, ok, ok, iok, ok, fok, ok, ws, nullptr) == -2);
  EXPECT(specext_verify_attn(&d, ok, ok, ok, ok, ok, iok, ok, fok, static_cast<char*>(ok) + 64, ws, nullptr) == -2);
  EXPECT(specext_verify_attn(&d, ok, ok, ok, ok, ok, iok, ok, fok, ok, ws - 1, nullptr) == -3);
  EXPECT(specext_verify_attn(&d, ok, ok, ok, ok, ok, iok, ok, nullptr, ok, ws, nullptr) == 0);     // reaches the stubs
  EXPECT(specext_workspace_init(nullptr, ws, nullptr) == -1);
  EXPECT(specext_workspace_init(odd, ws, nullptr) == -2);
  EXPECT(specext_workspace_init(ok, 100, nullptr) == -3);

  // scores, selection
  EXPECT(specext_chunk_scores(&d, ok, ws, 60, fok, nullptr) == -1);
  EXPECT(specext_chunk_scores(&d, ok, ws, -2, fok, nullptr) == -1);
  EXPECT(specext_chunk_scores(&d, nullptr, ws, 0, fok, nullptr) == -1);
  EXPECT(specext_chunk_scores(&d, ok, 16, 0, fok, nullptr) == -3);
  EXPECT(specext_chunk_scores(&d, ok, ws, 0, fok, nullptr) == 0);
  EXPECT(specext_chunk_scores_accepted(&d, ok, ws, nullptr, iok, fok, nullptr) == -1);
  EXPECT(specext_chunk_scores_select(&d, ok, ws, 0, nullptr, nullptr, 32, nullptr, iok, iok, nullptr) == 0);
  EXPECT(specext_chunk_scores_select(&d, ok, ws, 60, nullptr, nullptr, 32, nullptr, iok, iok, nullptr) == -1);
  EXPECT(specext_chunk_scores_select(&d, ok, ws, 0, iok, nullptr, 32, nullptr, iok, iok, nullptr) == -1);
  EXPECT(specext_chunk_scores_select(&d, ok, ws, 0, nullptr, nullptr, -1, nullptr, iok, iok, nullptr) == -1);
  EXPECT(specext_chunk_scores_select(&d, ok, ws, 0, nullptr, nullptr, 32, nullptr, iok, nullptr, nullptr) == -1);
  {
    specext_desc x = good_desc();
    x.prefix_len = 40000;                       // 1250 chunks: two launches, needs the scores buffer
    const size_t w2 = specext_workspace_bytes(&x);
    EXPECT(specext_chunk_scores_select(&x, ok, w2, 0, nullptr, nullptr, 32, nullptr, iok, iok, nullptr) == -1);
    EXPECT(specext_chunk_scores_select(&x, ok, w2, 0, nullptr, nullptr, 32, fok, iok, iok, nullptr) == 0);
  }
  EXPECT(specext_select_chunks(nullptr, 8, 2, iok, iok, nullptr) == -1);
  EXPECT(specext_select_chunks(fok, 0, 2, iok, iok, nullptr) == -1);
  EXPECT(specext_select_chunks(fok, 70000, 2, iok, iok, nullptr) == -2);
  EXPECT(specext_select_chunks(fok, 8, 2, iok, iok, nullptr) == 0);

  // gather, commit, acceptance, prefill, calibration
  EXPECT(specext_gather_draft_kv(ok, ok, ok, ok, iok, iok, 4, 1, 8, 100, 0, 4 * 32, 128, 32, 2, iok, iok, nullptr) == 0);
  EXPECT(specext_gather_draft_kv(ok, ok, ok, ok, iok, iok, 4, 1, 8, 100, 0, 4 * 32 - 1, 128, 32, 2, iok, iok, nullptr) == -1);
  EXPECT(specext_gather_draft_kv(ok, ok, ok, ok, iok, iok, 4, 1, 8, 100, 50, 4 * 32, 128, 32, 2, iok, iok, nullptr) == -1);
  EXPECT(specext_gather_draft_kv(ok, ok, ok, ok, iok, iok, 4, 1, 8, 100, 0, 4 * 32, 3, 32, 2, iok, iok, nullptr) == -2);
  EXPECT(specext_gather_draft_kv(ok, ok, ok, ok, iok, iok, 0x7fffffff, 1, 8, 100, 0, 0x7fffffff, 128, 32, 2, iok, iok, nullptr) == -1);
  EXPECT(specext_commit_tree_kv(ok, ok, ok, ok, iok, iok, 60, 60, 32, 8, 128, 2, 1000, 1060, 0, 0, 0, 0, 0, 0, nullptr) == 0);
  EXPECT(specext_commit_tree_kv(ok, ok, ok, ok, iok, iok, 60, 60, 32, 8, 128, 2, 0x7fffffff, 0x7fffffff, 0, 0, 0, 0, 0, 0, nullptr) == -1);
  EXPECT(specext_commit_tree_kv(ok, ok, ok, ok, iok, iok, 200, 60, 32, 8, 128, 2, 1000, 2000, 0, 0, 0, 0, 0, 0, nullptr) == -2);
  EXPECT(specext_accept_greedy(iok, iok, iok, iok, 60, iok, iok, iok, nullptr) == 0);
  EXPECT(specext_accept_greedy(iok, iok, iok, iok, 129, iok, iok, iok, nullptr) == -2);
  EXPECT(specext_accept_greedy(iok, iok, nullptr, iok, 60, iok, iok, iok, nullptr) == -1);
  EXPECT(specext_prefill_attn(ok, ok, ok, ok, fok, 32, 8, 128, 4096, 4096, SPECEXT_BF16, SPECEXT_BF16, 0.f, 0, 0, 0, 0, 0, 0, nullptr) == 0);
  EXPECT(specext_prefill_attn(ok, ok, ok, ok, fok, 32, 8, 128, 4096, 100, SPECEXT_BF16, SPECEXT_BF16, 0.f, 0, 0, 0, 0, 0, 0, nullptr) == -1);
  EXPECT(specext_prefill_attn(ok, ok, ok, ok, fok, 32, 8, 64, 4096, 4096, SPECEXT_BF16, SPECEXT_BF16, 0.f, 0, 0, 0, 0, 0, 0, nullptr) == -2);
  EXPECT(specext_prefill_attn(ok, ok, ok, ok, fok, 32, 8, 128, 0x7fffffff, 0x7fffffff, SPECEXT_BF16, SPECEXT_BF16, 0.f, 0, 0, 0, 0, 0, 0, nullptr) == -2);
  std::printf(failures ? "%d expectation(s) failed\n" : "all expectations held\n", failures);
  return failures ? 1 : 0;
}
