/*
 * hg_attn.h -- C ABI of the partitioned decode-attention library for AMD MI355X (gfx950).
 *
 * The operation (paper Section 2.1 and Section 4.2): during decode, ONE new query token per
 * sequence attends over that sequence's whole KV cache.  With per-head dimension d,
 *
 *     s_j = scale * (q . k_j),   p = softmax_j(s),   out = sum_j p_j v_j,      scale = 1/sqrt(d).
 *
 * The logit stage is independent per cached token, so the cache can be cut along the token axis
 * into positional ranges held by different executors (Section 4.2; Section 4.2.3, Token Mapper),
 * and the recombined result has to equal monolithic execution (Section 4.2.3, Token
 * Concatenator; Section 4.6 step 5).  This library expresses one range's contribution as the
 * softmax statistics
 *
 *     m = max_j s_j,    l = sum_j exp(s_j - m),    O = sum_j exp(s_j - m) v_j      (j in range)
 *
 * and recombines triples exactly:
 *
 *     M = max_p m_p,  w_p = exp(m_p - M),  L = sum_p w_p l_p,  out = sum_p w_p O_p / L.
 *
 * That is algebraically the same as concatenating the ranges' raw logits in token order and
 * taking one softmax, but a range's result is d+2 numbers instead of one logit and one value
 * row per token.
 *
 * General conventions
 *   - Every pointer marked DEVICE is memory of the current HIP device, owned by the caller.
 *     Every pointer marked HOST is ordinary host memory; it is consumed before the call returns
 *     and may be freed or reused immediately afterwards.
 *   - The library allocates nothing.  Scratch memory comes in through `workspace`
 *     (DEVICE, 256-byte aligned, at least the size the matching *_workspace_size call reports).
 *   - All device work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream).  No call declared in this header synchronises with the device.
 *   - A launch that the HIP runtime refuses is reported as HG_ERR_LAUNCH from that launch's own
 *     return value; the runtime's per-thread "last error" is neither read nor cleared, so errors
 *     the caller's own HIP calls left behind are never taken for this library's.
 *   - Validation is finished on the host before anything is enqueued: on any error status
 *     nothing has been launched and no output byte has been touched.
 *   - The cache of sequence b holds seq_lens[b] valid tokens, the current token included (its
 *     K and V are appended before attention, Section 2.1); no mask is applied.
 *   - Grouped-query attention: query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - Arithmetic: K, V, q are read in `dtype`; products, sums, exponentials, the triples and
 *     the outputs are fp32.  Inputs containing Inf or NaN give undefined results.
 *   - Concurrent calls must not share a workspace.
 */
#ifndef HG_ATTN_H
#define HG_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum hg_status {
    HG_OK = 0,
    HG_ERR_NULL = -1,      /* a required pointer is NULL                                        */
    HG_ERR_SHAPE = -2,     /* batch/heads/head_dim/strides/alignment/counts not supported       */
    HG_ERR_DTYPE = -3,     /* dtype is not HG_F16, HG_F32 or HG_BF16                            */
    HG_ERR_RANGE = -4,     /* a range or CSR offset is malformed or exceeds its sequence        */
    HG_ERR_WORKSPACE = -5, /* workspace NULL, misaligned or smaller than required               */
    HG_ERR_LAUNCH = -6     /* the HIP runtime refused a copy or a launch (details on stderr)    */
} hg_status;

typedef enum hg_dtype { HG_F16 = 0, HG_F32 = 1, HG_BF16 = 2 } hg_dtype; /* storage of q, K and V */

/*
 * One decode-attention problem: a batch of sequences, one query token each.
 *   q   DEVICE  [batch][n_q_heads][head_dim], contiguous, 16-byte aligned.
 *   k,v DEVICE  element (b, g, t, c) is at base + b*stride_b + g*stride_h + t*stride_t + c,
 *               strides counted in ELEMENTS; the channel stride is 1.  Bases are 16-byte aligned
 *               and every stride is a multiple of 16 bytes, so each row is 16-byte aligned.
 *               K and V use the same strides.  Rows at t >= seq_lens[b] are never read.
 *               A row stride of 64 MiB or more is refused (HG_ERR_SHAPE): the kernels address
 *               the rows of one workgroup's share with 32-bit byte offsets.
 *   seq_lens HOST [batch], 0 <= seq_lens[b].
 *   head_dim 64 or 128.  n_q_heads % n_kv_heads == 0.
 *   scale   multiplies q.k before the softmax (natural-log domain); callers pass 1/sqrt(head_dim).
 *
 * Paged cache (block_table != NULL; the KV manager of a paged serving stack, Section 4.8):
 *   block_table DEVICE int32 [batch][max_blocks]: token t of sequence b lives in physical block
 *               block_table[b][t / block_tokens], at row t % block_tokens of that block.
 *   block_tokens power of two, 16 .. 65536;  max_blocks >= ceil(max seq_lens / block_tokens).
 *   k, v        element (block p, head g, row r, c) is at base + p*stride_b + g*stride_h + r*stride_t + c:
 *               stride_b is the distance between physical blocks.  Table entries are not checked
 *               (they are device memory): every entry a valid token maps to must be a valid block.
 *               Limits of a paged descriptor: block stride below 4 GiB, row stride below 16 MiB.
 *   Every call that takes a descriptor accepts a paged one.
 */
typedef struct hg_attn_desc {
    const void *q;
    const void *k;
    const void *v;
    int64_t stride_b, stride_h, stride_t;
    const int32_t *seq_lens;
    int32_t batch, n_q_heads, n_kv_heads, head_dim;
    int32_t dtype; /* hg_dtype */
    float scale;
    const int32_t *block_table; /* NULL: contiguous cache */
    int32_t block_tokens, max_blocks;
} hg_attn_desc;

/* Tokens [begin, end) of sequence `seq` (the Token Mapper's positional range, Section 4.2.3).
 * 0 <= begin <= end <= seq_lens[seq]; begin == end is an empty range. */
typedef struct hg_range {
    int32_t seq, begin, end;
} hg_range;

/* Text for a status code; never NULL; static storage. */
const char *hg_strerror(hg_status status);

/*
 * hg_attn_partial -- partial softmax statistics of each listed range (Section 4.2: every
 * executor computes the logits of the keys it holds; here it also folds them into (m, l, O)).
 *
 *   ranges   HOST   [n_ranges]; any order, may overlap or leave gaps; each is computed on its own.
 *   m, l     DEVICE [n_ranges][n_q_heads] fp32.   m is the true maximum of the scaled logits in
 *                   natural-log units; l and O are relative to that m.
 *   o        DEVICE [n_ranges][n_q_heads][head_dim] fp32.
 *   An empty range yields m = -inf, l = 0, O = 0.  At most 2^31-1 tokens in all ranges together.
 *   workspace/ws_bytes  see hg_attn_partial_workspace_size (same desc and ranges).
 *
 * Merging the triples of ranges that tile [0, seq_lens[b]) exactly once reproduces hg_attn_full.
 */
hg_status hg_attn_partial_workspace_size(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges,
                                         size_t *bytes);
hg_status hg_attn_partial(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, float *m, float *l,
                          float *o, void *workspace, size_t ws_bytes, void *stream);

/*
 * hg_attn_merge -- exact recombination of triples (Section 4.2.3, Token Concatenator, in
 * statistics form).
 *
 *   m, l, o    DEVICE triples laid out as hg_attn_partial writes them ([n_triples][n_q_heads]...).
 *   group_ptr  HOST   CSR offsets [n_groups+1], non-decreasing, group_ptr[0] >= 0: group i merges
 *                     triples group_ptr[i] .. group_ptr[i+1]-1, separately for every query head.
 *                     The order of the triples inside a group does not matter.
 *   out        DEVICE [n_groups][n_q_heads][head_dim] fp32.
 *   lse_out    DEVICE [n_groups][n_q_heads] fp32 or NULL:  M + log L  (natural log).
 *   Triples with l == 0 are ignored; a group with L == 0 gives out = 0, lse = -inf.
 */
hg_status hg_attn_merge_workspace_size(int32_t n_groups, size_t *bytes);
hg_status hg_attn_merge(const float *m, const float *l, const float *o, const int32_t *group_ptr, int32_t n_groups,
                        int32_t n_q_heads, int32_t head_dim, float *out, float *lse_out, void *workspace,
                        size_t ws_bytes, void *stream);

/*
 * hg_attn_partial_merge -- hg_attn_partial followed by hg_attn_merge in one call (Sections 4.2.2
 * and 4.2.3 on one device: the triples of every range and the recombined output of every group),
 * for callers that want both.  The results are those of the two calls (the merged output up to
 * the order of summation).  group_ptr must cover the ranges exactly (group_ptr[0] == 0,
 * group_ptr[n_groups] == n_ranges) and the ranges of a group belong to one sequence.  When the input is small -- one query head per lane group
 * (32-bit storage, or 16-bit storage without a query group), a contiguous cache, at most 16
 * groups and 64 ranges, few enough (group, KV head) pairs for one workgroup each and few enough
 * tokens per group for a workgroup to stream them in the time a launch takes -- the whole call
 * is one kernel launch instead of three; otherwise it runs the two calls' kernels.
 *   workspace   DEVICE, 256-byte aligned, hg_attn_partial_merge_workspace_size bytes.
 *   Other arguments as for hg_attn_partial and hg_attn_merge; lse_out may be NULL.
 */
hg_status hg_attn_partial_merge_workspace_size(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges,
                                               const int32_t *group_ptr, int32_t n_groups, size_t *bytes);
hg_status hg_attn_partial_merge(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, const int32_t *group_ptr,
                                int32_t n_groups, float *m, float *l, float *o, float *out, float *lse_out, void *workspace,
                                size_t ws_bytes, void *stream);

/*
 * hg_attn_merge2 -- the same recombination over the triples of TWO producers, each with its own
 * arrays and CSR (Section 4.2.3; Section 4.6 step 5: the concatenator joins what the executor of
 * the offloaded tokens returns with what the executor of the resident tokens computed): group i
 * merges triples group_ptr_a[i] .. group_ptr_a[i+1]-1 of set A with triples group_ptr_b[i] ..
 * group_ptr_b[i+1]-1 of set B.  Either set may be empty for a group.  Saves the caller the
 * gather of both results into one array.  Arguments as for hg_attn_merge.
 */
hg_status hg_attn_merge2_workspace_size(int32_t n_groups, size_t *bytes);
hg_status hg_attn_merge2(const float *m_a, const float *l_a, const float *o_a, const int32_t *group_ptr_a, const float *m_b,
                         const float *l_b, const float *o_b, const int32_t *group_ptr_b, int32_t n_groups, int32_t n_q_heads,
                         int32_t head_dim, float *out, float *lse_out, void *workspace, size_t ws_bytes, void *stream);

/*
 * hg_attn_full -- the unsplit reference path ("monolithic execution", Section 4.2.3): softmax
 * attention of every sequence over its whole cache [0, seq_lens[b]).
 *
 *   out      DEVICE [batch][n_q_heads][head_dim] fp32.
 *   lse_out  DEVICE [batch][n_q_heads] fp32 or NULL.
 *   A sequence with seq_lens[b] == 0 gives out = 0, lse = -inf.
 */
hg_status hg_attn_full_workspace_size(const hg_attn_desc *desc, size_t *bytes);
hg_status hg_attn_full(const hg_attn_desc *desc, float *out, float *lse_out, void *workspace, size_t ws_bytes,
                       void *stream);

/*
 * hg_attn_logits -- the raw scaled logits of each listed range: what an executor ships in the
 * paper's own wire format (Section 4.2.2, Logits Calculator: logits as a compact vector, the
 * matching V rows travel separately).
 *
 *   logits  DEVICE [n_q_heads][ltok] fp32, ltok = total length of the ranges; the logits of range
 *           r occupy columns pre[r] .. pre[r] + len_r - 1, pre[r] = total length of the ranges
 *           listed before r.  Natural-log units: scale * (q . k_j).  Reads K only.
 */
hg_status hg_attn_logits_workspace_size(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges,
                                        size_t *bytes);
hg_status hg_attn_logits(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, float *logits,
                         void *workspace, size_t ws_bytes, void *stream);

/*
 * hg_attn_concat -- the paper-literal Token Concatenator (Section 4.2.3; Section 4.6 step 5):
 * the logits of a group's ranges are taken as ONE vector (they are adjacent columns of `logits`
 * because a group's ranges are consecutive table entries), ONE softmax is applied over it, and
 * the scores weight the V rows of those ranges.  Reads V and the logits, each once; K and q are
 * not read.  (The softmax over the whole vector is evaluated piecewise with running maxima and an
 * exact merge of the pieces, so the logits need no pass of their own.)
 *
 *   ranges     HOST  the table the logits were produced with (same order).
 *   logits     DEVICE [n_q_heads][ltok] fp32 as written by hg_attn_logits (or by any other
 *              executor: a CPU, another GPU).
 *   group_ptr  HOST  CSR [n_groups+1] over the RANGES, group_ptr[0] == 0 and
 *              group_ptr[n_groups] == n_ranges; all ranges of a group belong to one sequence.
 *              List a group's ranges in ascending token order to restore the original order;
 *              the result does not depend on it.  n_groups <= 65535.
 *   out        DEVICE [n_groups][n_q_heads][head_dim] fp32;  lse_out DEVICE [n_groups][n_q_heads] or NULL.
 *   A group without tokens gives out = 0, lse = -inf.
 */
hg_status hg_attn_concat_workspace_size(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges,
                                        int32_t n_groups, size_t *bytes);
hg_status hg_attn_concat(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, const float *logits,
                         const int32_t *group_ptr, int32_t n_groups, float *out, float *lse_out, void *workspace,
                         size_t ws_bytes, void *stream);

/*
 * hg_attn_select -- Post-QK^T token selection (Section 4.3.1; Section 4.5): the executor that
 * holds the offloaded tokens has computed the logits of ALL of them; per (group, query head) only
 * the top_k highest are kept, and those logits with their V rows are folded into one (m, l, O)
 * triple that hg_attn_merge combines with the triples of the resident tokens.
 *
 *   ranges, logits, group_ptr   as for hg_attn_concat (a group = the offloaded ranges of one sequence).
 *   top_k    1 .. 4096.  A group with fewer tokens keeps all of them.  The decision is taken on
 *            the fp32 logits as given; ties at the threshold (equal values; -0.0 equals +0.0) go
 *            to the lower column (earlier range in the table, earlier token).
 *   sel      DEVICE int32 [n_groups][n_q_heads][top_k] or NULL: the kept TOKEN positions of each
 *            head in ascending column order, padded with -1.
 *   m, l     DEVICE [n_groups][n_q_heads] fp32;  o  DEVICE [n_groups][n_q_heads][head_dim] fp32.
 *            An empty group yields (-inf, 0, 0).
 *   Reads the logits and the kept V rows only: one pass over the logits for top_k <= 1024, about
 *   five for larger top_k or when the quick bound fails (sorted or masked rows).  Groups longer
 *   than 16384 tokens are selected in two or three stages (candidates per part, then among those).
 *   Logits must not contain NaN; -inf (masked tokens) is fine.
 */
hg_status hg_attn_select_workspace_size(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges,
                                        const int32_t *group_ptr, int32_t n_groups, int32_t top_k, size_t *bytes);
hg_status hg_attn_select(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, const float *logits,
                         const int32_t *group_ptr, int32_t n_groups, int32_t top_k, int32_t *sel, float *m, float *l,
                         float *o, void *workspace, size_t ws_bytes, void *stream);

/*
 * hg_attn_topk -- the whole Post-QK^T executor stage in one call (Section 4.3.1; Section 4.6 step
 * 1): logits of every token of the listed ranges with THIS descriptor's query, top_k per (group,
 * query head), kept logits and V rows folded into one (m, l, O) triple.  The result is what
 * hg_attn_logits followed by hg_attn_select gives, bit for bit (the same fp32 logits decide, ties
 * go to the lower column), but the logits never travel through memory: the scan keeps a running
 * lower bound of each head's top_k-th largest logit and writes out only the logits that reach it
 * (a few per cent of them on unordered data; all of them if the logits arrive in ascending
 * order, which costs time, never correctness).
 *
 *   ranges, group_ptr, top_k, sel, m, l, o   as for hg_attn_select.
 *   workspace   DEVICE, 256-byte aligned, hg_attn_topk_workspace_size bytes: room for the worst
 *               case of the scan (2 x 4 bytes per (query head, token of the ranges); 4 x 4 with
 *               very many ranges per group or groups beyond 2^20 tokens).
 *   The filtering scan exists for top_k <= 256 (contiguous and paged caches), for one query head
 *   per KV head (any storage type) and for 16-bit storage with head_dim 128 and two or more query
 *   heads per KV head; it is chosen when the groups are long (see hg_attn_set_topk_mode).  Other cases
 *   run the two-call sequence inside, with the logits in the workspace.
 */
hg_status hg_attn_topk_workspace_size(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges,
                                      const int32_t *group_ptr, int32_t n_groups, int32_t top_k, size_t *bytes);
hg_status hg_attn_topk(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, const int32_t *group_ptr,
                       int32_t n_groups, int32_t top_k, int32_t *sel, float *m, float *l, float *o, void *workspace,
                       size_t ws_bytes, void *stream);

/*
 * hg_attn_gather -- attention statistics over a LISTED set of tokens per (group, query head): the
 * executor's side of a selection that was decided elsewhere.  Under Pre-QK^T selection (Section
 * 4.3.2; Section 4.6 step 1) the token selector names the tokens before the logits exist and the
 * executor computes logits and value sums for exactly those; the same call serves a Post-QK^T
 * selection taken with another query (the list hg_attn_select wrote for a proxy query, Section
 * 4.2.1, evaluated here with the true query).
 *
 *   group_seq  HOST   [n_groups]: the sequence each group's tokens belong to.
 *   index      DEVICE int32 [n_groups][n_q_heads][max_k]: token positions of sequence
 *              group_seq[g], in any order; negative entries are padding (the layout and padding
 *              of hg_attn_select's `sel`).  Entries are not checked (device memory): every
 *              non-negative one must be below seq_lens[group_seq[g]].  A token listed twice
 *              counts twice.
 *   max_k      1 .. 1048576.
 *   m, l, o    as hg_attn_partial writes them, one triple per (group, head); a list without
 *              tokens yields (-inf, 0, 0).
 */
hg_status hg_attn_gather_workspace_size(int32_t n_groups, size_t *bytes);
hg_status hg_attn_gather(const hg_attn_desc *desc, const int32_t *group_seq, int32_t n_groups, const int32_t *index,
                         int32_t max_k, float *m, float *l, float *o, void *workspace, size_t ws_bytes, void *stream);

/*
 * Feedback scheduler policy (Algorithm 1): host-only integer logic that sizes the offloaded
 * executor's work from the measured stage latencies.  One call = one tick.
 *
 *   state->k         tokens the offloaded executor keeps per head (the K of hg_attn_select);
 *                    hg_sched_init sets it to k_min with the Post-QK^T strategy.
 *   t_gpu            latency of the GPU stage (attention + FFN of the current layer),
 *   t_cpu, t_tx      latency of the offloaded logit stage and of its transfer, same unit.
 *   k_min            offline accuracy threshold; k_max = tokens available to the executor;
 *   k_step           how far one tick moves K (the paper leaves the step open).
 *
 * If t_cpu + t_tx <= t_gpu the offloaded stage is hidden behind the GPU stage and K grows by
 * k_step (at most k_max); otherwise K shrinks by k_step but not below k_min; and if K is already
 * k_min the strategy switches to Pre-QK^T (select before computing logits).  The strategy of a
 * tick is Post-QK^T unless that last case applies.  A state whose k lies outside
 * [k_min, k_max] is clamped first.
 */
typedef enum hg_select_strategy { HG_SELECT_POST_QK = 0, HG_SELECT_PRE_QK = 1 } hg_select_strategy;
typedef struct hg_sched_state {
    int32_t k;
    int32_t strategy; /* hg_select_strategy */
} hg_sched_state;
hg_status hg_sched_init(hg_sched_state *state, int32_t k_min);
hg_status hg_sched_step(hg_sched_state *state, float t_gpu, float t_cpu, float t_tx, int32_t k_min, int32_t k_max,
                        int32_t k_step);

/*
 * Host-side planning, exposed for inspection and tests.  The tokens of all ranges, repeated for
 * every stream (KV head x chunk of query heads sharing it), form one linear work space that is
 * cut into equal spans, one workgroup each, so that every workgroup streams the same number of
 * bytes whatever the shape of the partition table.  Reports the span length in tokens and the
 * number of workgroups the library would launch for this problem.  No device work.
 */
hg_status hg_attn_plan(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, int32_t *span_tokens,
                       int64_t *n_workgroups);

/* Identifies the sources this binary was built from (a hash of the HIP sources and headers taken
 * by the build step, or "unknown"); static storage.  Lets a loader refuse a stale binary. */
const char *hg_attn_build_id(void);

/*
 * hg_attn_partial_static -- hg_attn_partial for callers that cannot allocate device memory and
 * have no workspace to pass: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments and results as hg_attn_partial, but the segment records go to
 * a buffer of HG_ATTN_STATIC_SCRATCH_BYTES bytes that is part of the library's device image (every
 * GPU the library runs on holds its own copy until the process ends).  The call allocates
 * nothing on the device.
 *
 *   HG_ERR_WORKSPACE  the problem needs more scratch than the static buffer holds (what
 *                     hg_attn_partial_workspace_size reports for it); nothing has been enqueued.
 *                     A message with both sizes goes to stderr.
 *   All calls on one GPU share that GPU's buffer: two calls whose device work may overlap (other
 *   streams, other threads) race on it.  Calls on one stream are ordered and safe.  Nothing in
 *   the buffer has to start at zero: every record a call reads it has written itself.
 *   The first call on a device looks the buffer's address up (and, like any first launch, loads
 *   the device code); make that call outside a graph capture.
 */
#define HG_ATTN_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
hg_status hg_attn_partial_static(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, float *m, float *l,
                                 float *o, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HG_ATTN_H */
