/*
 * pillar.h -- C ABI of the PillarAttn hot path on MI355X (gfx950).
 *
 * One round of PillarAttn (paper Section 4.1) for one transformer layer:
 *
 *   pillar_verify_attn    full attention of the k+1 speculative query
 *                         positions over each request's whole paged KV-Cache,
 *                         which also emits the per-token attention-score
 *                         statistic of the verification step;
 *   pillar_select_topk    Top-K of that statistic per (request, KV head): the
 *                         critical tokens of the next k draft steps;
 *   pillar_sparse_decode  draft attention that loads only the selected rows
 *                         (paged attention at page size 1, Section 4.2).
 *
 * Conventions shared by every entry point
 *   - Every pointer inside pillar_kv_t and every tensor argument is a DEVICE
 *     pointer owned by the caller; the pillar_kv_t struct itself lives on the
 *     host.  The library never allocates, frees or synchronises: all work is
 *     enqueued on `hip_stream` (a hipStream_t, NULL = the default stream) and
 *     the call returns at once.  Scratch memory comes in through `workspace`
 *     (device, 256-byte aligned, at least pillar_workspace_bytes() bytes); its
 *     contents are meaningless between calls and calls sharing one workspace
 *     must be ordered on one stream.  Calls can be captured into a HIP graph;
 *     make one ordinary call with the same shapes first (the first launch of
 *     a kernel may set a function attribute, which is not a stream operation).
 *   - Return value: PILLAR_OK or a negative pillar_status.  Argument errors
 *     are detected on the host before anything is launched, so a failed call
 *     has no effect on the device.  Page ids and token indices stored in
 *     device memory cannot be checked on the host: values outside their
 *     documented ranges are undefined behaviour.
 *   - Outputs are bit-identical from run to run for identical inputs.
 *   - Tensors are dense C-order arrays unless a stride argument is given.
 *   - bf16 is the upper half of an IEEE float32; fp8 is OCP e4m3 (bias 7,
 *     largest finite 448, no infinities), dequantised as code * scale with
 *     one fp32 scale per (page, KV head) for K and one for V.
 *
 * Supported shapes: head_dim 64 or 128; num_q_heads a multiple of
 * num_kv_heads with group size G <= 16; page_size a power of two in 1..256;
 * 0 <= spec_len_k <= 15 and (spec_len_k+1)*G <= 64.  Anything else returns
 * PILLAR_EUNSUPPORTED.
 */
#ifndef PILLAR_H_
#define PILLAR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PILLAR_OK = 0,
  PILLAR_EINVAL = -1,        /* NULL pointer, non-positive size, inconsistent shapes */
  PILLAR_EUNSUPPORTED = -2,  /* well-formed but outside the supported shapes/dtypes */
  PILLAR_EWORKSPACE = -3,    /* workspace NULL, misaligned or too small */
  PILLAR_EHIP = -4,          /* the HIP runtime refused a launch */
  PILLAR_ETOOLARGE = -5      /* pillar_sparse_decode_static only: needs more than its fixed scratch */
} pillar_status;

typedef enum { PILLAR_F32 = 0, PILLAR_BF16 = 1, PILLAR_FP8_E4M3 = 2 } pillar_dtype;

/* The paged KV-Cache of one layer and the requests that read it.
 * Token t of request b is row  block_table[b*block_table_stride + t/page_size]
 * (a page id), slot t % page_size; its K vector for KV head g starts at element
 *   page*stride_page + g*stride_head + slot*stride_slot
 * of k_pool (same for v_pool) and is head_dim contiguous elements.
 * seq_lens[b] counts every token whose K/V is already in the pool, including
 * the k+1 speculative tokens of a verification step. */
typedef struct {
  int32_t batch;               /* B  >= 1 */
  int32_t num_q_heads;         /* Hq */
  int32_t num_kv_heads;        /* Hkv, divides Hq */
  int32_t head_dim;            /* D  */
  int32_t page_size;           /* P  */
  int32_t q_dtype;             /* PILLAR_F32 | PILLAR_BF16: type of q and of out */
  int32_t kv_dtype;            /* PILLAR_F32 | PILLAR_BF16 | PILLAR_FP8_E4M3 */
  float   sm_scale;            /* logit scale, normally 1/sqrt(D) */
  const void* k_pool;          /* device */
  const void* v_pool;          /* device */
  int64_t stride_page;         /* element strides; stride_slot >= head_dim */
  int64_t stride_head;
  int64_t stride_slot;
  const float* k_scale;        /* device [num_pages][Hkv], fp8 only, else NULL */
  const float* v_scale;
  int32_t num_pages;
  int32_t block_table_stride;  /* row length of block_table, in entries */
  const int32_t* block_table;  /* device [B][block_table_stride] */
  const int32_t* seq_lens;     /* device [B], 1 <= seq_lens[b] <= max_seq_len */
  int32_t max_seq_len;         /* host-known bound, <= block_table_stride*page_size */
  int32_t flags;               /* 0 or an OR of pillar_flag values; unknown bits: PILLAR_EINVAL */
} pillar_kv_t;

/* Per-call choices, carried in pillar_kv_t.flags.
 *   PILLAR_FLAG_EXACT_SCORES     the verification reads K twice (once for the
 *       log-sum-exp of every row, once more with V) and builds the score
 *       statistic from fp32 probabilities, instead of reading K once and
 *       rebuilding the statistic from 16-bit stashed exponentials.  Slower
 *       (about 1.15x); scores then carry fp32 rounding only.
 *   PILLAR_FLAG_GENERIC_KERNELS  every stage runs its plain vector-ALU kernel
 *       even where a matrix-core kernel exists: a second implementation to
 *       cross-check the fast one against.  Much slower. */
typedef enum { PILLAR_FLAG_EXACT_SCORES = 1, PILLAR_FLAG_GENERIC_KERNELS = 2 } pillar_flag;

/* Library version, major*10000 + minor*100 + patch. */
int pillar_version(void);

/* Static, NUL-terminated description of a status code. */
const char* pillar_status_string(int status);

/* Bytes of workspace that any of the three stage calls below may need for
 * this cache description, speculative length and largest budget.  Returns 0
 * when the description is invalid.  Host-only arithmetic. */
size_t pillar_workspace_bytes(const pillar_kv_t* kv, int32_t spec_len_k, int32_t max_budget);

/* Verification attention (Section 4.1, "Overhead-free identification").
 *   q      [B][k+1][Hq][D] q_dtype; row i is the query at position
 *          seq_lens[b]-(k+1)+i and attends to tokens 0..that position.
 *   out    [B][k+1][Hq][D] q_dtype: softmax(sm_scale * q K^T) V.
 *   lse    [B][k+1][Hq] fp32 natural-log-sum-exp of the logits, or NULL.
 *   scores [B][Hkv][score_stride] fp32, or NULL to skip the statistic:
 *          scores[b][g][t] = mean over the (k+1)*G rows of KV head g of the
 *          softmax probability that row assigns to token t (0 where the
 *          causal mask hides t).  Entries t >= seq_lens[b] are not written.
 *          score_stride >= max_seq_len.  Accuracy on the matrix-core path
 *          (bf16 queries): |error| <= 4.9e-4 * score + 2^-62, because every
 *          row's exponential is kept to 11 significant bits and a probability
 *          below 2^-62 (2.2e-19) counts as 0; with PILLAR_FLAG_EXACT_SCORES
 *          the error is that of fp32 arithmetic.
 *   Every request must hold its own speculative tokens: seq_lens[b] >= k+1.
 *   A query row that sees no token at all (seq_lens[b] < k+1) gets out = 0 and
 *   lse = -inf and adds nothing to the statistic. */
int pillar_verify_attn(const pillar_kv_t* kv, const void* q, int32_t spec_len_k,
                       void* out, float* lse, float* scores, int64_t score_stride,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* pillar_verify_attn and pillar_select_topk in one call: the critical tokens
 * are selected from the score statistic while it is still on the chip, so it
 * makes no round trip through memory between two launches.  Arguments as in
 * the two calls; `scores` may be NULL when the caller does not want the
 * statistic itself.  Results are identical to the two calls made in turn.
 * The workspace needs pillar_workspace_bytes() bytes as for every call. */
int pillar_verify_select(const pillar_kv_t* kv, const void* q, int32_t spec_len_k,
                         void* out, float* lse, float* scores, int64_t score_stride,
                         const int32_t* budgets, int32_t max_budget,
                         int32_t* indices, int32_t* counts,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/* Verification of requests that speculate different numbers of tokens
 * (Section 5.4: heterogeneous request configurations).  spec_lens: device [B],
 * 0 <= spec_lens[b] <= spec_len_max.  Request b has spec_lens[b]+1 queries, the
 * first of its spec_len_max+1 slots in q / out / lse, query i at position
 * seq_lens[b]-(spec_lens[b]+1)+i; its statistic is the mean over
 * (spec_lens[b]+1)*G rows; out and lse of the unused slots are not written.
 * With budgets / indices / counts non-NULL the critical tokens are selected as
 * by pillar_verify_select (all three NULL and max_budget 0: no selection).
 * Served by the matrix-core kernels only: bf16 queries, bf16 or fp8 KV,
 * head_dim 128, pages of >= 16 tokens, neither flag set; anything else returns
 * PILLAR_EUNSUPPORTED.  seq_lens[b] >= spec_lens[b]+1 as above. */
int pillar_verify_hetero(const pillar_kv_t* kv, const void* q, int32_t spec_len_max,
                         const int32_t* spec_lens, void* out, float* lse, float* scores,
                         int64_t score_stride, const int32_t* budgets, int32_t max_budget,
                         int32_t* indices, int32_t* counts,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/* Critical-token selection (Section 4.1: Top-K on the averaged scores).
 *   scores   as written by pillar_verify_attn (all >= 0).
 *   budgets  device [B]: sparsity budget K of each request (>= 0).
 *   indices  device [B][Hkv][max_budget] int32: for each (b, g) the
 *            K' = min(budgets[b], seq_lens[b], max_budget) positions of
 *            largest score among 0..seq_lens[b]-1, equal scores resolved
 *            towards the lower position, stored in ascending position order
 *            and padded with -1.
 *   counts   device [B] int32: K' of each request. */
int pillar_select_topk(const float* scores, int64_t score_stride, const int32_t* seq_lens,
                       const int32_t* budgets, int32_t batch, int32_t num_kv_heads,
                       int32_t max_seq_len, int32_t max_budget,
                       int32_t* indices, int32_t* counts,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* Sparse draft attention (Sections 1 and 4.2): one query row per request
 * attends to the listed rows only, no mask.
 *   q        [B][Hq][D] q_dtype.
 *   indices  device [B][Hkv][max_budget] int32 token positions in
 *            0..seq_lens[b]-1, any order; counts device [B], the first
 *            counts[b] entries of every head's list are used
 *            (0 <= counts[b] <= max_budget).
 *   out      [B][Hq][D] q_dtype (zeros where counts[b] == 0).
 *   lse      [B][Hq] fp32 or NULL (-inf where counts[b] == 0). */
int pillar_sparse_decode(const pillar_kv_t* kv, const void* q, const int32_t* indices,
                         const int32_t* counts, int32_t max_budget, void* out, float* lse,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/* One iteration of a unified batch (Section 4.2: "Unified Batch Scheduler" and
 * "Fused Sparse and Full Attention"): in the same iteration the requests listed
 * in verify_ids are in their verification phase and those in draft_ids in a
 * draft phase.  Per request the results are those of pillar_verify_select
 * (verify_ids) or pillar_sparse_decode (draft_ids) for that request alone:
 *   verify_ids  device [n_verify], draft_ids device [n_draft]: request indices
 *               in 0..batch-1, no request in both, none twice; the counts are
 *               host values (the scheduler that forms the batch knows them).
 *   q_verify / out_verify / lse_verify / scores, q_draft / out_draft / lse_draft,
 *   budgets / indices / counts: the full-batch tensors of the two calls, indexed
 *               by request id.  Only the rows of listed requests are read or
 *               written: a verifying request gets new out / lse / scores rows
 *               and a new index list and count; a drafting request reads its
 *               current list and gets out_draft / lse_draft rows.
 * Both phases run in ONE grid: the workgroups of the streaming verification
 * pass and those of the draft step are dispatched to their code path on the
 * chip.  (A draft sum may be grouped differently than by pillar_sparse_decode:
 * the results agree to rounding, not necessarily bit for bit, when a KV head
 * has more than 32 query rows.)  Either list may be empty.  Matrix-core shapes only (bf16 queries, bf16 or fp8 KV, head_dim
 * 128, pages of >= 16 tokens, rows of up to 32768 tokens, flags 0); anything
 * else returns PILLAR_EUNSUPPORTED.  Workspace: pillar_workspace_bytes(). */
int pillar_mixed_step(const pillar_kv_t* kv, const int32_t* verify_ids, int32_t n_verify,
                      const int32_t* draft_ids, int32_t n_draft,
                      const void* q_verify, int32_t spec_len_k, void* out_verify, float* lse_verify,
                      float* scores, int64_t score_stride,
                      const int32_t* budgets, int32_t max_budget, int32_t* indices, int32_t* counts,
                      const void* q_draft, void* out_draft, float* lse_draft,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* pillar_sparse_decode for callers that can hand over no workspace and must
 * not cause an allocation: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * result bits as pillar_sparse_decode, but the partial results of index lists
 * longer than one workgroup's span of 512 rows go to a 32 MiB array inside the
 * library (one copy per GPU, held until the process ends) instead of a
 * workspace.  A shape whose pillar_sparse_decode would need more than those
 * 32 MiB (batch * Hkv * ceil(max_budget / 512) spans of G rows of 128 floats;
 * about 15000 spans at G = 4; lists of up to 512 rows need none) returns
 * PILLAR_ETOOLARGE and launches nothing.
 * Calls no allocator.  All calls on one GPU share the one array: two such
 * calls that overlap in time on the same GPU (different streams) race; order
 * them.  The first call on a device looks the array's address up; make it
 * outside any stream capture. */
int pillar_sparse_decode_static(const pillar_kv_t* kv, const void* q, const int32_t* indices,
                                const int32_t* counts, int32_t max_budget, void* out, float* lse,
                                void* hip_stream);

/* The write that precedes a verification: the K/V rows of the n_new newest
 * tokens of every request go into their pages (append, then attend:
 * seq_lens already counts them).  k_new, v_new: device [B][n_new][Hkv][D] in
 * kv_dtype; row i of request b is written at position seq_lens[b]-n_new+i
 * (rows whose position would be negative are skipped).  WRITES into the pools
 * that pillar_kv_t describes.  bf16 and fp32 pools only: an fp8 pool returns
 * PILLAR_EUNSUPPORTED (its page scales would have to be recomputed). */
int pillar_append_kv(const pillar_kv_t* kv, const void* k_new, const void* v_new,
                     int32_t n_new, void* hip_stream);

/* Index lists from other sources for pillar_sparse_decode (Section 4.2: at
 * page size 1 any token set is a list).
 *
 * pillar_window_indices: the static "attention sinks + recent window" pattern
 * of the sliding-window drafts the paper compares against (Sections 1, 3.3
 * and 5.2).  For
 * request b, K' = min(budgets[b], seq_lens[b], max_budget); every head's list
 * holds the first min(sink_tokens, K') positions and the last K' minus that
 * many, ascending, padded with -1; counts[b] = K'.  All arrays on the device,
 * layouts as in pillar_select_topk.
 *
 * pillar_extend_indices: tokens generated since the last verification have no
 * score yet but must be visible to a draft step: appends the positions
 * first_new[b] .. first_new[b]+n_new[b]-1 to every head's list of request b
 * (as many as fit below max_budget) and adds that number to counts[b]. */
int pillar_window_indices(const int32_t* seq_lens, const int32_t* budgets, int32_t batch,
                          int32_t num_kv_heads, int32_t sink_tokens, int32_t max_budget,
                          int32_t* indices, int32_t* counts, void* hip_stream);
int pillar_extend_indices(int32_t* indices, int32_t* counts, const int32_t* first_new,
                          const int32_t* n_new, int32_t batch, int32_t num_kv_heads,
                          int32_t max_budget, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PILLAR_H_ */
