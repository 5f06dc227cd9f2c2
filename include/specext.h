/*
 * specext.h - C ABI of the SpecExtend verification hot path for AMD MI355X (gfx950).
 *
 * Implements, as hand-written HIP kernels, the verification-side operations of
 * SpecExtend (arXiv 2505.20776):
 *   - Hybrid Tree Attention (Sec. 3.1): the draft tree's tokens attend to the
 *     target model's cached prefix (split over the KV length, FlashDecoding
 *     style) and, under the tree mask, to each other; the parts are merged
 *     exactly by log-sum-exp.
 *   - Cross-model Retrieval (Sec. 3.2.1, Alg. 1): per-chunk average attention
 *     scores of one query token, top-k chunk selection (SelectChunks) and the
 *     compaction of the draft model's KV cache to the chosen chunks
 *     (UpdateDraftCache).
 *   - The rest of the step in Alg. 1: greedy acceptance along the draft tree and
 *     the commit of the accepted tokens' K/V rows into the target cache.
 *
 * Conventions common to every entry point
 *   - Every tensor argument is a DEVICE pointer owned by the caller.  The
 *     library allocates nothing, frees nothing and keeps no pointer after the
 *     call returns.  `stream` is the caller's hipStream_t passed as void*
 *     (NULL = the default stream).  All work is enqueued asynchronously on it;
 *     no entry point synchronises with the host.
 *   - Return value: SPECEXT_OK (0) or a negative specext_status.  Errors that
 *     the host can see (null pointers, unsupported shapes, misaligned
 *     pointers, workspace too small) are reported BEFORE anything is launched
 *     and leave all outputs untouched.  Data-dependent errors (a parent index
 *     that is not smaller than its node) are reported through the status word
 *     in the workspace, see specext_verify_attn.
 *   - Row-major layouts, last index fastest.  L = prefix_len, T = n_tree,
 *     Hq / Hkv = query / KV heads, G = Hq / Hkv, d = head_dim,
 *     B = chunk_size, C = ceil(L / B).
 *   - Thread safety: no global mutable state except a per-process cache of
 *     device properties; concurrent calls on different streams are safe as
 *     long as they use different workspaces.
 */
#ifndef SPECEXT_H_
#define SPECEXT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum specext_status {
  SPECEXT_OK = 0,
  SPECEXT_ERR_INVALID_ARG = -1,        /* null pointer, non-positive size, bad struct_size ... */
  SPECEXT_ERR_UNSUPPORTED = -2,        /* dtype / head_dim / n_tree / alignment outside what the kernels handle */
  SPECEXT_ERR_WORKSPACE_TOO_SMALL = -3,
  SPECEXT_ERR_LAUNCH_FAILED = -4       /* the HIP runtime refused a launch */
} specext_status;

typedef enum specext_dtype {
  SPECEXT_F32 = 0,
  SPECEXT_BF16 = 1
} specext_dtype;

/* desc->flags: run the prefix pass on the vector ALUs (fp32 FMA) even where the
 * matrix-core kernel applies; for cross-checking the two kernels. */
#define SPECEXT_FLAG_VALU_PREFIX 1u
/* desc->flags: specext_verify_attn runs only the split prefix pass and stops
 * before the tree pass and merge, so out / lse are not written.  For timing the
 * prefix kernel on its own. */
#define SPECEXT_FLAG_PREFIX_ONLY 2u
/* desc->flags: run the tree pass and the merge as the tail of the prefix launch instead
 * of as a second launch, where that is possible (bf16, head_dim 128, more than 32 rows per
 * KV head, all workgroups resident at once; otherwise the flag has no effect).  The
 * workgroups hand their split results to each other through the workspace header, which
 * must have been prepared with specext_workspace_init.  Same results as the two-launch
 * form up to the rounding of a different (fixed) summation order; bit-reproducible from
 * run to run.  On MI355X the two launches measure faster at every prefix length (a
 * dependent trip through memory costs more than the launch boundary it replaces), so this
 * form is off unless asked for. */
#define SPECEXT_FLAG_FUSED_MERGE 4u
/* desc->flags, with SPECEXT_FLAG_FUSED_MERGE: a workgroup polls for the other splits'
 * results once instead of up to 65537 times before it leaves its rows to the workgroup
 * that finishes last.  Results are unchanged; for testing that hand-over. */
#define SPECEXT_FLAG_SHORT_WAIT 8u

#define SPECEXT_MAX_TREE 128           /* largest supported n_tree */
#define SPECEXT_MAX_SPLITS 256         /* largest supported num_splits */
#define SPECEXT_WORKSPACE_HEADER_BYTES 82176   /* head of every workspace, see specext_workspace_init */
#define SPECEXT_STATIC_SCRATCH_MIB 48  /* scratch of specext_verify_attn_static, MiB per GPU */

/*
 * Problem descriptor (plain data).  Set struct_size = sizeof(specext_desc).
 * A stride of 0 means "densely packed" for the layouts given below.
 */
typedef struct specext_desc {
  uint32_t struct_size;
  int32_t dtype;          /* specext_dtype of q, k_*, v_* */
  int32_t out_dtype;      /* specext_dtype of `out`; F32 or the input dtype */
  int32_t n_q_heads;      /* Hq */
  int32_t n_kv_heads;     /* Hkv, must divide Hq; query head h reads KV head h / G */
  int32_t head_dim;       /* d: 64 or 128 */
  int32_t prefix_len;     /* 0 <= L <= 2^30 cached positions */
  int32_t n_tree;         /* T in [1, SPECEXT_MAX_TREE] */
  int32_t chunk_size;     /* 0 < B <= 2^24; only read when want_scores != 0.  The bf16 matrix-core
                             kernels need B to be a multiple of 32 (and, for head_dim 64, kp_stride_l = 64);
                             other values take the vector-ALU kernel. */
  int32_t want_scores;    /* != 0: also leave per-chunk partial sums in the workspace */
  int32_t num_splits;     /* pieces the prefix is cut into; 0 = choose automatically */
  float softmax_scale;    /* 0 = 1/sqrt(d) */
  uint32_t flags;         /* bit set of SPECEXT_FLAG_* */
  uint32_t reserved;      /* must be 0 */
  /* element strides; the d elements of one vector are always contiguous */
  int64_t q_stride_t, q_stride_h;       /* q[t][h][:]        default Hq*d, d  */
  int64_t kp_stride_h, kp_stride_l;     /* k_prefix[g][j][:] default L*d,  d  (v_prefix uses the same) */
  int64_t kt_stride_h, kt_stride_t;     /* k_tree[g][t][:]   default T*d,  d  (v_tree uses the same) */
  int64_t o_stride_t, o_stride_h;       /* out[t][h][:]      default Hq*d, d  */
} specext_desc;

/* Static text for a status code. */
const char* specext_strerror(int status);

/*
 * Upper bound, in bytes, of the workspace specext_verify_attn needs for this
 * descriptor (split partials, final log-sum-exp, chunk partial sums when
 * want_scores, and the status word).  Returns 0 for an invalid descriptor.
 * Host-only; needs a visible GPU only when num_splits == 0 (to read the
 * compute-unit count).
 */
size_t specext_workspace_bytes(const specext_desc* desc);

/*
 * Prepare a workspace for specext_verify_attn with SPECEXT_FLAG_FUSED_MERGE: once after
 * it is allocated (or whenever its first SPECEXT_WORKSPACE_HEADER_BYTES were overwritten
 * by something else), before its first use, on a stream ordered before that use.  The
 * head of every workspace does not depend on the descriptor - status word, an
 * initialisation mark and the hand-over blocks through which the workgroups of one
 * launch pass their split results to each other; every call leaves them ready for the
 * next, so one workspace serves any sequence of calls and descriptors after a single
 * init.  workspace_bytes must be at least SPECEXT_WORKSPACE_HEADER_BYTES and the pointer
 * 256-byte aligned.  A fused call on a workspace that was never initialised sets the
 * status word to 2 and writes neither out nor lse.  Calls without the flag need no init.
 */
int specext_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/*
 * Hybrid Tree Attention for one layer (Sec. 3.1).
 *
 *   q         [T, Hq, d]   queries of the tree tokens           (desc->dtype)
 *   k_prefix  [Hkv, L, d]  cached keys of the prefix, v_prefix likewise
 *   k_tree    [Hkv, T, d]  keys of the tree tokens, v_tree likewise
 *   parent    int32 [T]    parent[i] < i; -1 marks a root (whose conceptual
 *                          parent is the last prefix token).  Forests allowed.
 *   out       [T, Hq, d]   softmax(scale * q k^T over prefix keys and the
 *                          ancestor-or-self tree keys) v      (desc->out_dtype)
 *   lse       fp32 [Hq, T] natural-log sum-exp of each row; may be NULL
 *   workspace at least specext_workspace_bytes(desc) bytes, 256-byte aligned.
 *
 * Pointers must be 16-byte aligned and strides multiples of 8 elements.
 * Arithmetic: logits, softmax statistics and the P V sums are fp32 (P and V enter the
 * matrix cores as bf16).  With bf16 inputs, head_dim 128 and more than 32 rows per KV
 * head the per-split partial outputs cross memory as fp16 after a per-row power-of-two
 * rescale (11 bits against the row's largest element, whatever the scale of V); the
 * rescale exponent travels in the split's softmax reference, so the magnitudes of V
 * must stay within 2^-100 ... 2^100 and those of two splits of one row within a factor
 * of about 2^100 of each other, or a split's weight underflows.
 * The first int32 of the workspace is a status word: 0 after a good call,
 * 1 if some parent[i] was >= i or < -1 (that node is then treated as a root),
 * 2 if SPECEXT_FLAG_FUSED_MERGE was set and the workspace was never initialised
 * (nothing was computed).
 * With want_scores the workspace afterwards holds what specext_chunk_scores
 * consumes; it stays valid until the next call that uses this workspace.
 */
int specext_verify_attn(const specext_desc* desc, const void* q, const void* k_prefix,
                        const void* v_prefix, const void* k_tree, const void* v_tree,
                        const int32_t* parent, void* out, float* lse, void* workspace,
                        size_t workspace_bytes, void* stream);

/*
 * specext_verify_attn for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same inputs, outputs, kernels and results as specext_verify_attn; the
 * split partials live in a scratch array of SPECEXT_STATIC_SCRATCH_MIB MiB that is
 * part of the library's device code (every GPU that loads the library holds its own
 * copy until the process ends).  The call allocates and frees nothing.
 *
 *   status_out  device int32 [1] that receives the status word (0, or 1 for a
 *               malformed parent index); may be NULL
 *
 * Limits: a descriptor whose specext_workspace_bytes exceeds the scratch array is
 * rejected with SPECEXT_ERR_WORKSPACE_TOO_SMALL before anything is launched (the
 * Llama-3.1-8B layer shape fits at every prefix length with a 60-node tree at up to
 * 48 splits and with a 128-node tree at up to 22, the automatic split counts
 * included); want_scores != 0 is SPECEXT_ERR_UNSUPPORTED, because the
 * chunk partial sums must outlive the call for specext_chunk_scores - the one layer
 * that feeds the retrieval uses specext_verify_attn.  Every call on a GPU shares that
 * GPU's array: calls that overlap in time on one GPU (different streams) race on it
 * and must not be made; calls on one stream, or otherwise ordered, are safe.
 */
int specext_verify_attn_static(const specext_desc* desc, const void* q, const void* k_prefix,
                               const void* v_prefix, const void* k_tree, const void* v_tree,
                               const int32_t* parent, void* out, float* lse, int32_t* status_out,
                               void* stream);

/*
 * Chunk scores (Sec. 3.2.1): scores[r][c] = mean over query heads of the mean,
 * over the tokens actually in chunk c, of the attention probability that tree
 * row r gives to those tokens (normalised over the row's full key set).
 *
 *   desc, workspace   exactly what the preceding specext_verify_attn call on
 *                     the same stream was given, with want_scores != 0
 *   score_row         tree row to score, or -1 for every row
 *   scores            fp32 [C] (one row) or fp32 [T, C] (score_row == -1)
 */
int specext_chunk_scores(const specext_desc* desc, const void* workspace, size_t workspace_bytes,
                         int32_t score_row, float* scores, void* stream);

/*
 * SelectChunks (Alg. 1): the min(k, n_chunks) chunks with the largest score.
 * Ties go to the lower chunk index.  Scores must be finite.
 *
 *   scores   fp32 [n_chunks], n_chunks in [1, 65536]
 *   k        >= 0
 *   idx_out  int32 [k]; the first min(k, n_chunks) entries receive the chosen
 *            chunk indices in ascending order, the rest are set to -1
 *   n_out    int32 [1] on the device: min(k, n_chunks)
 */
int specext_select_chunks(const float* scores, int32_t n_chunks, int32_t k, int32_t* idx_out,
                          int32_t* n_out, void* stream);

/*
 * UpdateDraftCache (Alg. 1): compact the draft model's KV cache to the chosen
 * chunks, copying bytes verbatim, in the order of idx.
 *
 *   k_src, v_src  [n_layers, n_kv_heads, src_cap, head_dim] elements of elem_bytes, of
 *                 which the first src_len tokens of every (layer, head) are valid;
 *                 src_cap = 0 means src_cap = src_len (a dense cache); src_cap <
 *                 src_len is SPECEXT_ERR_INVALID_ARG
 *   k_dst, v_dst  [n_layers, n_kv_heads, dst_cap, head_dim]; token slot
 *                 r*chunk_size + t of the output receives token
 *                 idx[r]*chunk_size + t of the source.  A ragged last source
 *                 chunk contributes only its real tokens and later chunks
 *                 follow it without a gap.
 *   idx           device int32 [max_idx]; entries < 0 or >= ceil(src_len/chunk_size) are skipped
 *   n_idx         device int32 [1] (how many entries of idx are used, clamped to
 *                 max_idx) or NULL to use all max_idx entries
 *   dst_cap       token capacity of the destination; must be >= max_idx * chunk_size
 *   pos_out       int32 [dst_cap] original position of every written token
 *                 (-1 beyond len_out); may be NULL
 *   len_out       device int32 [1]: tokens written; may be NULL
 *
 * head_dim * elem_bytes must be a multiple of 16 and all four cache pointers
 * 16-byte aligned.
 */
int specext_gather_draft_kv(const void* k_src, const void* v_src, void* k_dst, void* v_dst,
                            const int32_t* idx, const int32_t* n_idx, int32_t max_idx,
                            int32_t n_layers, int32_t n_kv_heads, int32_t src_len, int32_t src_cap,
                            int32_t dst_cap, int32_t head_dim, int32_t chunk_size, int32_t elem_bytes,
                            int32_t* pos_out, int32_t* len_out, void* stream);

/*
 * Verify / Correct of Alg. 1 at temperature 0, walked down the draft tree (the
 * children of a node are the alternative drafts for the position after it, as in
 * the tree attention of Sec. 2): starting above the roots with the token the
 * target model wants first, the child that carries the wanted token is accepted
 * (the lowest node index if several do) and the token the target wants after
 * that child is wanted next; the walk ends at the first position where no child
 * matches.
 *
 *   parent         int32 [n_tree], parent[i] < i, -1 = root; n_tree in [1, 128]
 *   draft_token    int32 [n_tree]: the token drafted at each node
 *   target_token   int32 [n_tree]: the target model's arg-max token for the
 *                  position after each node
 *   first_target   device int32 [1]: its arg-max token for the first new position
 *   path_out       int32 [n_tree]: accepted nodes from the top down, then -1
 *   n_accept_out   device int32 [1]: how many nodes were accepted (0 .. n_tree)
 *   next_token_out device int32 [1]: the token that follows the accepted ones (the
 *                  correction of the first mismatch, or the bonus token after a
 *                  fully accepted path)
 */
int specext_accept_greedy(const int32_t* parent, const int32_t* draft_token, const int32_t* target_token,
                          const int32_t* first_target, int32_t n_tree, int32_t* path_out,
                          int32_t* n_accept_out, int32_t* next_token_out, void* stream);

/*
 * The accepted tree tokens enter the target model's KV cache (the step after
 * verification in Alg. 1: x_{n+1} <- accepted token, n <- n + 1):
 * cache[y, g, prefix_len + i, :] = tree[y, g, path[i], :] for i < n_accept, bytes
 * verbatim, for K and for V, for every layer y in one launch.
 *
 *   k_tree, v_tree    [n_layers, n_kv_heads, n_tree, head_dim] elements of elem_bytes
 *                     (the tree K/V that the layers' specext_verify_attn calls were given)
 *   k_cache, v_cache  [n_layers, n_kv_heads, cache_capacity, head_dim]
 *   path, n_accept    as written by specext_accept_greedy (device); entries outside
 *                     [0, n_tree) are skipped, n_accept is clamped to max_accept
 *   max_accept        launch bound on the accepted length (<= 128);
 *                     prefix_len + max_accept must not exceed cache_capacity
 *   *_stride_*        in elements; 0 = contiguous in the shapes above (separate
 *                     per-layer allocations: one call per layer with n_layers = 1)
 *
 * head_dim * elem_bytes and every stride in bytes must be multiples of 16 and the
 * four tensor pointers 16-byte aligned.
 */
int specext_commit_tree_kv(const void* k_tree, const void* v_tree, void* k_cache, void* v_cache,
                           const int32_t* path, const int32_t* n_accept, int32_t max_accept, int32_t n_tree,
                           int32_t n_layers, int32_t n_kv_heads, int32_t head_dim, int32_t elem_bytes,
                           int32_t prefix_len, int32_t cache_capacity, int64_t tree_stride_layer,
                           int64_t tree_stride_h, int64_t tree_stride_t, int64_t cache_stride_layer,
                           int64_t cache_stride_h, int64_t cache_stride_l, void* stream);

/*
 * specext_chunk_scores for the row of the last accepted token (Sec. 3.2.1: the
 * query of the ranking is the last accepted token), read on the device so that no
 * host round trip sits between acceptance and retrieval: scores the tree row
 * path[*n_accept - 1], or row 0 when nothing was accepted.
 *
 *   desc, workspace   as for specext_chunk_scores
 *   path, n_accept    as written by specext_accept_greedy (device)
 *   scores            fp32 [C]
 */
int specext_chunk_scores_accepted(const specext_desc* desc, const void* workspace, size_t workspace_bytes,
                                  const int32_t* path, const int32_t* n_accept, float* scores, void* stream);

/*
 * specext_chunk_scores for one tree row followed by specext_select_chunks over that
 * row's scores (Sec. 3.2.1; SelectChunks of Alg. 1), in one launch when there are at most
 * 1024 chunks (two launches beyond that).  Same scores and the same selection, bit for
 * bit, as the two calls.
 *
 *   desc, workspace   as for specext_chunk_scores
 *   score_row         the tree row when path is NULL (0 <= score_row < n_tree); else the
 *                     row is path[*n_accept - 1] read on the device (row 0 when nothing
 *                     was accepted), path and n_accept as written by specext_accept_greedy
 *   k, idx_out, n_out as for specext_select_chunks
 *   scores            fp32 [C] that also receives the scores, or NULL (allowed up to
 *                     1024 chunks; beyond that SPECEXT_ERR_INVALID_ARG)
 */
int specext_chunk_scores_select(const specext_desc* desc, const void* workspace, size_t workspace_bytes,
                                int32_t score_row, const int32_t* path, const int32_t* n_accept, int32_t k,
                                float* scores, int32_t* idx_out, int32_t* n_out, void* stream);

/*
 * Prefill attention (Sec. 3.1: FlashAttention is applied to the prefill stage of the
 * target and of the draft model): exact causal self-attention, computed tile by
 * tile with an online softmax, no score matrix in memory.
 *
 *   q        [q_len, n_q_heads, head_dim]: the queries of the LAST q_len positions of
 *            a context of kv_len tokens (q_len = kv_len for a whole prompt; smaller for a
 *            later piece of a prompt that is processed in pieces)
 *   k, v     [n_kv_heads, kv_len, head_dim] (the KV cache layout of specext_verify_attn;
 *            the caller has written the new tokens' K/V before the call)
 *   out      [q_len, n_q_heads, head_dim] of out_dtype (bf16 or fp32)
 *   lse      fp32 [n_q_heads, q_len], natural log of the softmax denominator; may be NULL
 *   query i sits at position kv_len - q_len + i and sees keys 0 .. that position;
 *   query head h uses KV head h / (n_q_heads / n_kv_heads)
 *   softmax_scale  0 = 1/sqrt(head_dim)
 *   *_stride_*     in elements, 0 = contiguous in the shapes above; multiples of 8
 *
 * All pointers device, 16-byte aligned (lse 4).  dtype must be SPECEXT_BF16, head_dim
 * 128 and kv_len >= 32 (SPECEXT_ERR_UNSUPPORTED otherwise; a shorter prompt is a chain
 * tree for specext_verify_attn with an empty prefix).  Results are bit-reproducible.
 */
int specext_prefill_attn(const void* q, const void* k, const void* v, void* out, float* lse, int32_t n_q_heads,
                         int32_t n_kv_heads, int32_t head_dim, int32_t q_len, int32_t kv_len, int32_t dtype,
                         int32_t out_dtype, float softmax_scale, int64_t q_stride_t, int64_t q_stride_h,
                         int64_t kv_stride_h, int64_t kv_stride_l, int64_t o_stride_t, int64_t o_stride_h,
                         void* stream);

/*
 * The score path as Sec. 3.2.1 words it: the last layer's verification attention
 * as STANDARD attention - the matrix of attention scores is written to memory,
 * softmaxed row by row and multiplied with V - and the chunk scores are read from
 * that matrix.  Same inputs, outputs and results as specext_verify_attn followed
 * by specext_chunk_scores; it exists as an independent check of the fused path
 * and to measure what the fusion saves.  bf16 inputs with head_dim 128 only
 * (anything else: SPECEXT_ERR_UNSUPPORTED); num_splits and flags are ignored.
 *
 *   specext_materialized_bytes  workspace size for desc (0 if desc is rejected)
 *   specext_materialized_ld     row pitch ld of the matrix in elements (a multiple
 *                               of 64 >= prefix_len + n_tree), or a negative status
 *   workspace   device, 256-byte aligned, >= specext_materialized_bytes(desc).
 *               Its first int32 is the status word of specext_verify_attn (1 if a parent
 *               index was malformed; that node is then treated as a root).
 *               After specext_attn_materialized the matrix P lies at byte 256 of it:
 *               fp32 [n_q_heads][n_tree][ld]; columns 0..prefix_len-1 are the prefix
 *               keys, prefix_len..prefix_len+n_tree-1 the tree nodes (exactly 0 where
 *               the tree mask hides a node), the padding behind them is 0.
 *   q ... lse   as for specext_verify_attn
 *
 * specext_chunk_scores_materialized reads that matrix: scores[c] = mean over heads of
 * the mean of P[h][row][tokens of chunk c].  desc must have want_scores and
 * chunk_size set; row = score_row when path is NULL (0 <= score_row < n_tree), else
 * path[*n_accept - 1] read on the device (row 0 when nothing was accepted), path and
 * n_accept as written by specext_accept_greedy.
 */
size_t specext_materialized_bytes(const specext_desc* desc);
int specext_materialized_ld(const specext_desc* desc);
int specext_attn_materialized(const specext_desc* desc, const void* q, const void* k_prefix, const void* v_prefix,
                              const void* k_tree, const void* v_tree, const int32_t* parent, void* out, float* lse,
                              void* workspace, size_t workspace_bytes, void* stream);
int specext_chunk_scores_materialized(const specext_desc* desc, const void* workspace, size_t workspace_bytes,
                                      int32_t score_row, const int32_t* path, const int32_t* n_accept,
                                      float* scores, void* stream);

/*
 * Number of prefix splits specext_verify_attn uses for this descriptor when
 * desc->num_splits == 0 (else returns desc->num_splits clamped to what is
 * valid).  Returns a negative specext_status on an invalid descriptor.
 */
int specext_num_splits(const specext_desc* desc);

/*
 * Measurement aids, not part of the method: what the GPU at hand sustains in a pure
 * HBM read stream and in pure dense bf16 matrix-core work, so that a benchmark can
 * quote the kernels above against measured ceilings next to the published ones
 * (the roofline that bounds the prefix pass of Sec. 3.1: K/V bytes per launch against
 * HBM bandwidth, 4 d T G Hkv L flops per launch against the bf16 matrix rate).
 *
 * specext_calib_stream_read: reads every byte of [src, src + bytes) once with
 *   coalesced 16-byte loads.  src device, 16-byte aligned; bytes a positive multiple of
 *   32768; sink: device uint32 [1] or NULL (never written for real data).  Time it with
 *   events on `stream`; bytes / time is the read bandwidth.  Use a buffer much larger
 *   than the 256 MB last-level cache.
 * specext_calib_mfma: `workgroups` workgroups of four wavefronts, each wavefront
 *   issuing iters x 16 matrix instructions (tile = 32: v_mfma_f32_32x32x16_bf16,
 *   tile = 16: v_mfma_f32_16x16x32_bf16) on register operands of roughly unit variance
 *   and nothing else.  Returns the number of floating-point operations of the launch
 *   (> 0), or a negative specext_status.  sink: device float [1] or NULL.
 * specext_calib_issue_mix: how matrix and vector instructions share a SIMD (what bounds the
 *   tile loop of the prefix pass, whose every tile is 16 matrix instructions and some 70
 *   vector instructions per wavefront, two wavefronts per SIMD).  `workgroups` workgroups of
 *   eight wavefronts, wavefronts w and w + 4 on one SIMD; per iteration a wavefront issues 16
 *   v_mfma_f32_32x32x16_bf16, or 16 x vector_per_matrix vector instructions (three fused
 *   multiply-adds and one exponential in every four), or both in turns.  mode 1: wavefronts
 *   0..3 matrix only (the others leave at once); 2: wavefronts 4..7 vector only; 3: both of
 *   these together; 4: all eight wavefronts, one matrix instruction then vector_per_matrix
 *   vector ones.  vector_per_matrix: 0, 4 or 8.  Time it with events on `stream`.  Returns
 *   SPECEXT_OK or a negative specext_status; nothing is launched on an error.
 */
int specext_calib_stream_read(const void* src, size_t bytes, uint32_t* sink, void* stream);
int64_t specext_calib_mfma(int32_t iters, int32_t tile, int32_t workgroups, float* sink, void* stream);
int specext_calib_issue_mix(int32_t mode, int32_t vector_per_matrix, int32_t iters, int32_t workgroups, float* sink,
                            void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SPECEXT_H_ */
