/*
 * blendstep_builder.h - host-side batch builder: BlendServe's resource-aware
 * prefix tree (Section 5.1), layer-wise sort and conditional node splitting
 * (Section 5.2, Algorithms 1 and 2) and dual scan with memory partition
 * (Section 5.3, Algorithm 3), in the single-step form
 * that feeds bs_blend_step.  Pure CPU code: no HIP call is made.
 *
 * All pointers are HOST memory.  Functions return 0 or a negative bs_status
 * (blendstep.h); bs_builder_last_error gives the message.
 */
#ifndef BLENDSTEP_BUILDER_H
#define BLENDSTEP_BUILDER_H

#include "blendstep.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Constants of the performance model of Section 4.1: rho = Comp / Mem with
 * Comp = 2 (tokens) P_model / compute and Mem = (loaded tokens) kv_bytes / bandwidth. */
typedef struct bs_cost_model {
  int64_t p_model;    /* model parameters */
  int64_t kv_bytes;   /* bytes of K and V per token over all layers ("H_kv * L * 4") */
  double compute;     /* FLOP/s */
  double bandwidth;   /* bytes/s */
  int64_t mem_bytes;  /* M: KV-cache capacity the dual scanner partitions */
  int32_t page_size;  /* tokens per KV page */
} bs_cost_model;

typedef struct bs_builder bs_builder;

int bs_builder_create(const bs_cost_model *cm, bs_builder **out);
void bs_builder_destroy(bs_builder *b);
const char *bs_builder_last_error(const bs_builder *b);

/* Add a request: its prompt token ids (copied), estimated output length d_est >= 0
 * (Section 5.1, output length sampling, is outside this library: the estimate is an
 * input) and n_cached, the number of its tokens whose KV is already cached;
 * n_cached >= n_tokens means the request is decoding with context n_cached.
 * Returns the request's index (>= 0) or a negative bs_status. */
int bs_builder_add(bs_builder *b, const int32_t *tokens, int32_t n_tokens, int32_t d_est, int32_t n_cached);

/* Memory model behind B, before bs_builder_finalize.
 *   BS_MEM_EXPANDED (default): Section 4.1's Mem(r) summed over requests; a cached prefix
 *     is charged to every request that holds it (Section 3.3: a prefix-cache hit saves
 *     no bandwidth).
 *   BS_MEM_SHARED: an extension for a decode kernel that reads the pages of a shared
 *     segment once per step (Appendix A.2): loaded tokens of the subtree when all its
 *     requests decode together, each segment charged once per step while any request
 *     below it still decodes,
 *       S(leaf) = 2 own d + d^2, S(N) = 2 len(N) max_d(N) + sum S(child),
 *       B(R) = S(R) + 2 start(R) max_d(R);
 *     equal to the default wherever nothing is shared.  bs_builder_split is defined for
 *     the default only (it reasons with sums over leaves) and fails otherwise. */
enum { BS_MEM_EXPANDED = 0, BS_MEM_SHARED = 1 };
int bs_builder_set_mem_model(bs_builder *b, int mem_model);

/* kv_bytes of bs_cost_model ("H_kv * L * 2 * 2" of Section 4.1) for the attention
 * variants of Section 7: bytes of cached state per token over all layers.  MHA: keys and
 * values of n_heads heads; MQA: of one head; GQA: of n_kv_heads heads (must divide
 * n_heads); MLA: one latent of latent_dim plus a shared rotary key of rope_dim per
 * layer.  Arguments a variant does not use are ignored.  Returns a negative bs_status
 * on invalid arguments.  Host only. */
enum { BS_ATTN_MHA = 0, BS_ATTN_MQA = 1, BS_ATTN_GQA = 2, BS_ATTN_MLA = 3 };
int64_t bs_kv_bytes_per_token(int variant, int32_t n_layers, int32_t n_heads, int32_t head_dim, int32_t n_kv_heads,
                              int32_t latent_dim, int32_t rope_dim, int32_t elem_bytes);

/* Build the compressed trie over all prompts (every request a leaf, every internal
 * node a maximal shared segment), annotate every node with
 *   A = distinct prompt tokens of its subtree with the root path counted once + sum d_i
 *   B = sum (2 p_i d_i + d_i^2)            (rho is proportional to A / B)
 * sort every node's children by rho, compute-intensive first (exact comparison of
 * A1 B2 against A2 B1 in 128-bit integers; B = 0 is +infinity; ties to the subtree
 * with the smaller request index), and number the nodes in DFS pre-order. */
int bs_builder_finalize(bs_builder *b);

/* Conditional node splitting (Section 5.2, Algorithm 2, with the stopping conditions of
 * Section 5.4).  Rounds of: stop if the leaf densities (p + d) / (2 p d + d^2), left to
 * right, are non-increasing (C1); take as outliers the leaves l below a non-root node X
 * such that X without l would change places with the sibling Q next to it while l belongs
 * on the far side of all of Q (the density of a node is sum A / sum B, so one
 * memory-intensive request drags every subtree that holds it); if there is none, the
 * leaves outside a longest non-increasing subsequence (patience procedure) that are not
 * already direct children of the root - where the outlier of an adjacent violation is
 * such a child, its neighbour instead; of those whose shared prefix (the tokens recomputed once
 * they stop sharing it) is at most t, cheapest first (ties: smaller request index), cut as
 * many as the total budget of recomputed tokens allows (budget_tokens < 0: no limit) and
 * re-insert them as direct children of the root; none taken = stop (C2); rebuild, re-sort.
 * Every leaf moves at most once.  Call after bs_builder_finalize; the tree, the leaf
 * order and the batches reflect the result.  `info` may be NULL. */
typedef struct bs_split_info {
  int32_t n_split;            /* leaves relocated by this call */
  int32_t rounds;             /* rounds that relocated at least one leaf */
  int32_t monotone;           /* 1 if the final leaf densities are non-increasing */
  int64_t recompute_tokens;   /* sum of the relocated leaves' shared prefix lengths */
} bs_split_info;
int bs_builder_split(bs_builder *b, int64_t t, int64_t budget_tokens, bs_split_info *info);

/* The sorted tree in DFS pre-order.  bs_builder_tree_size gives the array lengths;
 * bs_builder_tree fills caller-provided arrays: per node its parent (-1 for the
 * root), token range [start, end) of its segment, request index (-1 for internal
 * nodes), the position of its first leaf in the leaf order, its number of leaves,
 * A and B; and leaf_order[n_requests], the request indices from left to right. */
int bs_builder_tree_size(const bs_builder *b, int32_t *n_nodes, int32_t *n_requests);
int bs_builder_tree(const bs_builder *b, int32_t *parent, int32_t *start, int32_t *end, int32_t *req,
                    int32_t *first_leaf, int32_t *leaf_count, int64_t *A, int64_t *B, int32_t *leaf_order);

/* What Algorithm 3 computed for the step. */
typedef struct bs_scan_info {
  double rho_rt, rho_l, rho_r; /* densities of the (first branching) root and of its leftmost / rightmost subtree */
  double m_l, m_r;             /* memory partition, M_L + M_R = M and M_L rho_L + M_R rho_R = M rho_rt (clamped to [0, M]) */
  int64_t n_l, n_r;            /* decode requests per side, floor(M_X / ((p_X + d_X/2) kv_bytes)), at least 1 */
  int64_t c_l, c_r;            /* prefill token budgets per side, floor(N_X p_X / d_X); -1 = unlimited (d_X = 0) */
  int32_t n_prefill, n_decode; /* sequences admitted to the batch */
} bs_scan_info;

/* A batch owned by the library: `batch` points into memory freed by bs_batch_free. */
typedef struct bs_batch_owned {
  bs_batch batch;
  const int32_t *seq_request; /* [n_seq] request index of each sequence */
  int64_t n_pages;            /* physical pages the page tables refer to: ids 0 .. n_pages-1 */
  bs_scan_info info;
} bs_batch_owned;

/* One step: partition M between the two ends of the leaf order, then scan the leaves
 * inwards from both ends, admitting up to N_X decoding requests and up to C_X prefill
 * tokens per side (the last prompt may be cut: chunked prefill).  prefill_budget and
 * decode_budget (<= 0: none) cap C_L + C_R and N_L + N_R, split in proportion.  The
 * descriptor lists prefill segments first (in admission order), then decode
 * sequences in leaf order; prefix nodes are the trie nodes with at least two admitted
 * decode members and at least one whole page, physical pages are numbered node pages
 * first (DFS order), then each sequence's private pages in sequence order. */
int bs_builder_next_batch(bs_builder *b, int64_t prefill_budget, int64_t decode_budget, bs_batch_owned **out);

/* The descriptor of an explicit step, for a driver that keeps the requests' state itself
 * (Section 5.3: the runtime batch is re-formed every iteration from the requests in flight;
 * Appendix A.2): n_pre prefill segments - request, prompt tokens whose KV is already cached,
 * rows to compute this step (cached + chunk <= prompt length) - in the order given, then n_dec
 * decode sequences - request, tokens cached before this step (>= prompt length) - emitted in
 * leaf order.  A request may appear once.  Prefix nodes and page numbering as in
 * bs_builder_next_batch; `info` of the result is zero. */
int bs_builder_emit(bs_builder *b, int32_t n_pre, const int32_t *pre_req, const int32_t *pre_cached,
                    const int32_t *pre_chunk, int32_t n_dec, const int32_t *dec_req, const int32_t *dec_ctx,
                    bs_batch_owned **out);
void bs_batch_free(bs_batch_owned *batch);

/* ---------------------------------------------------------------------------------------------
 * Multi-step driver: a pool of requests served to completion, one descriptor per step.
 *
 * The paper's engine re-forms the runtime batch every iteration (Section 3.2; Appendix A.2, batch
 * scheduler): every decoding request contributes one row, the rest of the token budget goes to
 * prefill chunks (Section 2.2), and new requests are admitted from the two ends of the sorted leaf
 * order, one scanner per end, the KV memory split between the two by Algorithm 3 (Section 5.3) and a
 * step's prefill rows split C_L : C_R, each side keeping room for one average request of its own.  A
 * request that ends before its estimate frees its memory at once, one that runs past it is charged
 * a token per step, and one admitted from the compute-intensive end whose output reaches
 * relocate_pct per cent of its estimate moves, with its own reservation, to the memory-intensive
 * partition (Section 5.4).  A shared prompt segment is computed once, by the first resident request
 * that needs it (requests that need a segment somebody is still computing wait), counted once in
 * the memory account while any request below it is resident, and its KV pages are referenced by
 * all of them (Appendix A.2, runtime prefix tree).
 *
 * KV pages are physical and stable: a page is taken from the pool (smallest free number first)
 * when a step first writes into it and keeps its number until its request finishes (private pages)
 * or the last resident request below its segment leaves (shared pages), so the caller's pool
 * carries real keys and values from step to step.  Sharing is page-granular: a segment that ends at
 * token e shares the whole pages below e / 16 (below (e - 1) / 16 where some prompt ends exactly at
 * e), and a request admitted behind complete segments starts at the first token after their pages.
 *
 * The scheduler reads the builder's finalized (and possibly split) tree; the builder must outlive
 * it and must not change meanwhile.  Requests are taken as not yet prefilled (n_cached is ignored).
 */
typedef struct bs_sched_cfg {
  int64_t mem_tokens;    /* M: tokens of KV the account may hold */
  int32_t token_budget;  /* rows of a step */
  int32_t n_pages;       /* physical pages of the caller's pool */
  int32_t relocate_pct;  /* see above; 0 = requests stay in the partition that admitted them; 200 is the usual value */
  int32_t row_multiple;  /* steps of more rows than this are cut to a multiple of it (Appendix A.2 uses 128); 1 = off */
} bs_sched_cfg;

typedef struct bs_sched_stats {
  int64_t steps, rows, prefill_rows, decode_rows, prompt_tokens_skipped, tokens_out, finished, peak_tokens, peak_pages,
          relocated, mem_left, mem_right;  /* mem_*: tokens of the two partitions */
} bs_sched_stats;

typedef struct bs_sched bs_sched;

/* d_true[n_requests]: the output length after which each request ends (>= 1; it stands in for the
 * end-of-sequence events a serving engine sees; admission and reservation use the builder's
 * estimates only).  order: NULL = the leaf order of the sorted tree, scanned from both ends;
 * else a permutation of the requests that one scanner walks from the left with all the memory
 * (the orders that the resource-aware one is compared with). */
int bs_sched_create(const bs_builder *b, const bs_sched_cfg *cfg, const int32_t *d_true, const int32_t *order,
                    bs_sched **out);
void bs_sched_destroy(bs_sched *s);
const char *bs_sched_last_error(const bs_sched *s);

/* The next step's descriptor (free it with bs_batch_free; `info` is zero; n_pages is the pool size),
 * with the scheduler's state already advanced past the step: the caller runs the steps in the order
 * it receives them.  Returns BS_OK, BS_SCHED_DONE when every request has been served (*out = NULL),
 * BS_ENOMEM when the page pool is exhausted, BS_EINVAL when nothing fits the memory at all. */
#define BS_SCHED_DONE 1
int bs_sched_next(bs_sched *s, bs_batch_owned **out);
int bs_sched_get_stats(const bs_sched *s, bs_sched_stats *out);

#ifdef __cplusplus
}
#endif
#endif /* BLENDSTEP_BUILDER_H */
