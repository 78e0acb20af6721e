/*
 * blendstep.h - C ABI of the MI355X blended decoder-layer step.
 *
 * One call runs one forward step of one Llama-style decoder layer over a
 * "dense batch" in the sense of BlendServe (Section 2.2, chunked prefill; Section
 * 4.2): compute-bound prefill rows and memory-bound decode rows side by side,
 * the decode rows attending to a paged KV cache whose shared-prefix pages
 * (Section 2.2, prefix sharing; Appendix A.2, runtime prefix tree) are referenced
 * once and read once per prefix group.
 *
 * Conventions
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device
 *     memory on the context's device.  All buffers are caller-owned unless said
 *     otherwise; the library keeps only its context workspace.
 *   - bf16 = bfloat16, row-major, innermost index last.
 *   - Every function returns 0 (BS_OK) or a negative bs_status; the message of
 *     the last failure on a context is kept for bs_last_error().  Nothing
 *     throws or aborts across this boundary.  A batch is validated on the host
 *     before anything is enqueued: a malformed descriptor is an error code,
 *     never a GPU fault.
 *   - bs_blend_step is asynchronous on the given stream.  A call that needs more
 *     workspace than any call before it on the context (more rows, more partial
 *     softmax states, a longer descriptor) frees and reallocates device memory,
 *     which synchronises the device; calls within the sizes already seen do not,
 *     except that a call waits on the host for the fourth-last call's descriptor
 *     copy (its staging slot).  Calls on one context must not overlap in time on
 *     different streams (they share the workspace).
 */
#ifndef BLENDSTEP_H
#define BLENDSTEP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum bs_status {
  BS_OK = 0,
  BS_EINVAL = -1, /* bad shape, non-monotone CSR, page id out of range, kv_len beyond
                     its pages, node pages not matching a member's table, a page that
                     is written this step while referenced more than once, ... */
  BS_ENOMEM = -2, /* host or device allocation failed */
  BS_EHIP = -3,   /* a HIP runtime call failed */
  BS_EUNSUPPORTED = -4 /* shape outside what the kernels are written for */
} bs_status;

/* Layer shape.  The paper leaves the layer itself open (Section 2.1 names Q/K/V
 * projections, GQA, softmax attention, FFN; Section 4.2 "layer normalization,
 * activation, and position embedding"); the Llama-style choices are:
 * pre-norm RMSNorm (eps inside the root), rotate-half RoPE pairing (i, i+dh/2)
 * with angle pos * rope_theta^(-2i/dh), scale 1/sqrt(dh), SwiGLU, two residuals.
 * Supported: head_dim 64 or 128; page_size 16; n_q_heads a multiple of n_kv_heads
 * with ratio <= 16; d_model, d_ffn, head_dim multiples of 8. */
typedef struct bs_layer_cfg {
  int32_t d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, page_size;
  float rms_eps, rope_theta;
  int32_t max_positions; /* RoPE table length; 0 = 16384 */
} bs_layer_cfg;

/* Weights: device, bf16, caller-owned, "out-features major" like a linear layer's
 * weight matrix (each output feature's d inputs are contiguous):
 *   w_qkv     [(Hq + 2 Hkv) * dh, d]   rows: q heads, then k heads, then v heads
 *   w_o       [d, Hq * dh]
 *   w_gate_up [2 F, d]                 rows: F gate rows, then F up rows
 *   w_down    [d, F]
 *   g_attn, g_ffn [d]                  RMSNorm gains */
typedef struct bs_weights {
  const void *w_qkv, *w_o, *w_gate_up, *w_down, *g_attn, *g_ffn;
} bs_weights;

/* Batch descriptor (Section 4.2: a batch is a chunk of prefill tokens plus the
 * decode requests in flight).  All arrays are HOST int32, caller-owned, and are
 * copied during the call.
 *
 * Sequences [0, n_prefill) are prefill segments (one or more rows, causal among
 * themselves, attending to their cached tokens too); sequences [n_prefill, n_seq)
 * are decode sequences with exactly one row.  kv_len[i] is the attended length
 * AFTER this step's rows are appended: rows of sequence i sit at positions
 * kv_len[i]-q_len[i] .. kv_len[i]-1 and their keys/values are written there.
 * Token t of sequence i lives at (page_ids[page_start[i] + t / page_size],
 * t % page_size).  Shared pages repeat the SAME physical id in every sharer's
 * table.
 *
 * Prefix nodes tell the decode-attention kernel which pages to read once for a
 * whole group: node n owns pages node_page_ids[node_page_start[n] ..
 * node_page_start[n+1]) and is shared by the contiguous run of DECODE sequences
 * [node_seq_first[n], node_seq_first[n] + node_seq_count[n]).  Nodes come in DFS
 * pre-order (parent before child); in every member's page table the pages of
 * the root..leaf path come first, in that order.  seq_leaf_node[i] is the
 * deepest node of sequence i or -1.  Prefill segments may reference shared
 * pages in their tables but are not node members (seq_leaf_node = -1). */
typedef struct bs_batch {
  int32_t n_seq, n_prefill, n_rows;
  const int32_t *row_start;       /* [n_seq + 1] */
  const int32_t *kv_len;          /* [n_seq]     */
  const int32_t *page_start;      /* [n_seq + 1] */
  const int32_t *page_ids;        /* [page_start[n_seq]] */
  int32_t n_nodes;
  const int32_t *node_parent;     /* [n_nodes] -1 for roots */
  const int32_t *node_page_start; /* [n_nodes + 1] */
  const int32_t *node_page_ids;   /* [node_page_start[n_nodes]] */
  const int32_t *node_seq_first;  /* [n_nodes] */
  const int32_t *node_seq_count;  /* [n_nodes] may be 0 (node unused this step) */
  const int32_t *seq_leaf_node;   /* [n_seq] */
} bs_batch;

typedef struct bs_ctx bs_ctx;

/* Flags of bs_blend_step. */
#define BS_FLAG_SERIAL 0u   /* every operator of the step over all rows, one launch after the other */
#define BS_FLAG_OVERLAP 1u  /* memory-bound decode attention co-scheduled with the compute-bound GEMMs
                               of the prefill rows (Section 3.3: overlapped, a step costs the larger of
                               its compute and memory times, not their sum; Section 2.2, operator-level
                               overlapping between parts of a batch; Appendix A.2, backend engine):
                               the decode units of at most 16 query rows form a queue that attention
                               workgroups drain inside the prefill rows' output-projection, gate/up and
                               down-projection launches, on CUs of their own; the decode rows' projection
                               and FFN follow.  Still one stream and no events.  Steps without prefill
                               rows or without such units run the serial schedule.  Results differ from
                               the serial schedule by GEMM tile shapes only (same arithmetic per element). */
#define BS_FLAG_PIPELINE 2u /* bs_blend_layers with BS_FLAG_OVERLAP: the two parts of the batch run one stage
                               apart across the layer boundary (Section 2.2, nano-batches; Appendix A.2):
                               the decode rows finish layer l and enter layer l+1 (norm, QKV, KV append)
                               before the prefill rows' down projection of layer l is launched, and that
                               launch carries the first part of their attention of layer l+1.  Ignored by
                               bs_blend_step and wherever BS_FLAG_OVERLAP would run the serial schedule. */

/* Create a context on `device`; allocates the RoPE table and workspace that
 * grows on demand.  *out is NULL on failure; bs_last_error(NULL) then returns
 * the message.  With device = BS_DEVICE_NONE the context is host-only: it makes
 * no HIP call and serves bs_validate_batch and bs_resolve_rows; the GPU entry
 * points return BS_EINVAL on it. */
#define BS_DEVICE_NONE (-1)
int bs_create(const bs_layer_cfg *cfg, int device, bs_ctx **out);
void bs_destroy(bs_ctx *ctx);
const char *bs_last_error(const bs_ctx *ctx);

/* KV pool layout.  The pool is one device array of n_pages pages; a page holds,
 * per KV head, a K tile [page_size][dh] and a transposed V tile [dh][page_size]:
 *   element index of K(page, head, slot, e) = ((page*2 + 0)*Hkv + head)*page_size*dh + slot*dh + e
 *   element index of V(page, head, slot, e) = ((page*2 + 1)*Hkv + head)*page_size*dh + e*page_size + slot
 * bs_kv_page_bytes returns the bytes of one page.  bs_kv_pack / bs_kv_unpack
 * convert (on `stream`, device to device) between that layout and two plain
 * token-major arrays k, v of shape [n_pages][page_size][Hkv][dh] bf16. */
int64_t bs_kv_page_bytes(const bs_ctx *ctx);
int bs_kv_pack(bs_ctx *ctx, const void *k, const void *v, void *kv_pool, int64_t n_pages, void *stream);
int bs_kv_unpack(bs_ctx *ctx, const void *kv_pool, void *k, void *v, int64_t n_pages, void *stream);

/* One blended step of the layer:
 *   h = rmsnorm(x; g_attn); q,k,v = h W_qkv^T; RoPE on q,k; k,v appended to the pool;
 *   o = causal softmax attention per sequence over its pages; x1 = x + o W_o^T;
 *   y = x1 + (silu(h2 W_gate^T) * (h2 W_up^T)) W_down^T with h2 = rmsnorm(x1; g_ffn).
 * x, y: device bf16 [n_rows, d_model]; y may not alias x.  kv_pool: device,
 * n_pages pages, read and (for this step's rows) written.  stream: a hipStream_t
 * (NULL = the default stream). */
int bs_blend_step(bs_ctx *ctx, const bs_weights *w, const bs_batch *batch,
                  const void *x, void *y, void *kv_pool, int64_t n_pages,
                  void *stream, uint32_t flags);

/* The same step through n_layers layers back to back, as a serving engine runs it
 * (Section 2.2: every decoding step passes through all layers; Appendix A.2: the backend
 * runs whole batches layer after layer): layer l has weights w[l] and its own pool
 * kv_pools[l] (all pools have n_pages pages and share the one descriptor, i.e. the same
 * page table), reads the output of layer l-1 (x for l = 0) and the last layer writes y.
 * The descriptor is validated, planned and uploaded once.  w and kv_pools are HOST arrays
 * of n_layers entries, read during the call. */
int bs_blend_layers(bs_ctx *ctx, int32_t n_layers, const bs_weights *w, const bs_batch *batch,
                    const void *x, void *y, void *const *kv_pools, int64_t n_pages,
                    void *stream, uint32_t flags);

/* Host-only check of a descriptor against a pool of n_pages pages (the same
 * validation bs_blend_step performs); touches no GPU. */
int bs_validate_batch(bs_ctx *ctx, const bs_batch *batch, int64_t n_pages);

/* Host-only page resolution, for tests of the indexing: writes, for every row r
 * of the batch, the physical page and slot its key/value are appended to. */
int bs_resolve_rows(bs_ctx *ctx, const bs_batch *batch, int32_t *page_out, int32_t *slot_out);

/* Per-kernel timing.  With profiling on, bs_blend_step brackets each kernel
 * class with HIP events on the stream it runs on; bs_profile_read waits for the
 * recorded events and returns the accumulated milliseconds and launch count of
 * class `which` since the last reset.  Off by default (events cost time).
 * In the serial schedule a step with prefill and decode rows runs both kinds of
 * attention as one launch, booked under BS_K_ATTN_DECODE (BS_K_ATTN_PREFILL
 * then has no launches). */
enum { BS_K_PREP = 0, BS_K_GEMM_QKV, BS_K_ATTN_PREFILL, BS_K_ATTN_DECODE, BS_K_ATTN_MERGE,
       BS_K_GEMM_O, BS_K_GEMM_GATE_UP, BS_K_GEMM_DOWN,
       BS_K_ATTN_QUEUE_REST,   /* BS_FLAG_OVERLAP: the launch that drains what the carrying GEMMs left of the queue */
       BS_K_GEMM_DECODE_ROWS,  /* BS_FLAG_OVERLAP: output projection, gate/up and down of the decode rows */
       BS_K_COUNT };
int bs_profile_enable(bs_ctx *ctx, int on);
int bs_profile_read(bs_ctx *ctx, int which, double *total_ms, int64_t *launches);
int bs_profile_reset(bs_ctx *ctx);

/* Tuning knob: pages per chunk of decode-attention work (even, 2..64).  Smaller chunks give more
 * parallelism and more partial states to merge.  Default: 64 for private tails and for prefix nodes
 * whose work items carry at most 16 query rows, 32 for nodes with more (every chunk of such a node
 * costs one partial state per member row); a call sets both. */
int bs_set_chunk_pages(bs_ctx *ctx, int32_t pages);

/* Tuning knobs of the BS_FLAG_OVERLAP schedule. */
typedef struct bs_overlap_knobs {
  int32_t head_cus_min;     /* CUs that a carrying GEMM launch gives to attention for its whole duration: */
                            /* chosen per launch between head_cus_min and head_cus_max (multiples of 8,
                               0..192; defaults 0 and 96) so that the tiles fill whole rounds on the rest */
  int32_t tail_workgroups;  /* attention workgroups placed behind the tiles of a carrying launch, which start
                               on the CUs that its last round of tiles leaves idle (0..256; default 208) */
  int32_t close_margin;     /* a carrying launch whose last round of tiles leaves CUs idle stops handing out
                               decode units when all but this many of its tiles have finished (0..256;
                               default 8); one whose last round is at least three quarters full stops as
                               soon as the first tile of that round has finished */
  int32_t min_prefill_rows; /* steps with fewer prefill rows run the serial schedule (default 256) */
  int32_t ride_percent;     /* at most this share of the 16-row units' KV bytes waits for the carrying
                               launches; the rest joins the first attention launch (0..100; -1, the
                               default: what the head CUs are expected to read while the tiles run) */
  int32_t attention_waves;  /* wavefronts of an attention workgroup (of its eight) that take units (1..8;
                               default 2: a CU streams nearly as fast with two as with eight, and a unit
                               is finished sooner) */
  int32_t carry_down;       /* 0 (default): the output projection and gate/up of the prefill rows carry
                               attention and one down projection runs over all rows at the end; 1: the down
                               projection is split into prefill and decode rows too and carries attention */
  int32_t drain_in_last;    /* 1 (default): the last carrying launch goes on until the queue is empty;
                               0: it closes like the others and one more launch drains the queue */
  int32_t head_cus_max;
  int32_t always;           /* 0 (default): a step takes the co-scheduled path only if the cost model behind
                               these choices (whole rounds of tiles at measured per-CU rates, 36 GB/s of KV
                               pages per attention CU, 5.3 TB/s for the whole chip) expects it to be shorter
                               than the serial one; 1: whenever it has prefill rows and 16-row units */
} bs_overlap_knobs;
int bs_set_overlap(bs_ctx *ctx, const bs_overlap_knobs *knobs);
int bs_get_overlap(const bs_ctx *ctx, bs_overlap_knobs *knobs);

/* Where the decode attention of the last BS_FLAG_OVERLAP step ran: key/value bytes of the 16-row units
 * read by [0] the first attention launch (with the prefill rows and the wide items), [1..3] the attention
 * workgroups inside the output-projection, gate/up and down-projection launches of the prefill rows,
 * [4] the launch after them (drain_in_last = 0).  kv_bytes: HOST array of 5.  Synchronises the device.
 * Meaningful only after a step that took the co-scheduled path. */
int bs_overlap_report(bs_ctx *ctx, int64_t *kv_bytes);

/* Timeline of the co-scheduled launches, taken inside the kernels (a kernel trace sees one launch where
 * attention and GEMM workgroups run side by side; this shows what ran when, and on which CU).
 * bs_overlap_trace(ctx, 1) allocates the record buffer (8 MB) and makes every later BS_FLAG_OVERLAP step
 * record; (ctx, 0) frees it.  Both synchronise the device.  bs_overlap_trace_read copies the records of
 * one launch of the last such step (launch 0..2: the output-projection, gate/up and down-projection
 * launches of the prefill rows; 3: the launch that drains the rest of the queue) to the HOST array `out`
 * of cap_records x 4 uint64 and sets *n_records to the number the launch has (8 per workgroup, in grid
 * order; 0 if no timeline was taken or the launch had more than 8192 workgroups).  A record is
 * {begin, end} in ticks of the GPU's constant 100 MHz clock, {kind (1 attention wavefront, 2 GEMM tile;
 * 0 = unused record) | HW_ID << 8 | XCC_ID << 32}, {units | KV tokens << 32} that an attention wavefront
 * served.  Recording costs a few stores per wavefront; a step that records clears the buffer with a memset
 * on the stream, so it is not for steps captured into a graph. */
int bs_overlap_trace(bs_ctx *ctx, int on);
int bs_overlap_trace_read(bs_ctx *ctx, int32_t launch, uint64_t *out, int64_t cap_records, int64_t *n_records);

/* Tuning knob: GEMM tile shape for the calls on this context: 0 = chosen per problem (default), 1 = 256x256,
 * 2 = 160x256 (not for the QKV GEMM), 3 = 128x128, 6 = 256x256 tiles shared between workgroups (one persistent
 * workgroup per CU; the tiles that do not fill a whole round are cut along K into equal ranges).  With 0, GEMMs of at most 256 rows run as one
 * row of 128x256 or 256x128 tiles on a pipeline with its own look-ahead for the weight panel; a
 * forced shape switches that off. */
int bs_set_gemm_tiles(bs_ctx *ctx, int32_t variant);

/* Stand-alone entry points of the individual operators (the same kernels the
 * step launches), for per-kernel parity tests and roofline measurements.
 *   bs_gemm_nt: C[M,N] = A[M,K] * B[N,K]^T, bf16 in, fp32 accumulate, bf16 out;
 *   K a multiple of 8. */
int bs_gemm_nt(bs_ctx *ctx, const void *a, const void *b, void *c,
               int32_t m, int32_t n, int32_t k, void *stream);
/*   bs_attention: attention alone over an already appended pool.  q: device bf16
 *   [n_rows, Hq*dh] (after RoPE); out: device bf16 [n_rows, Hq*dh]. */
int bs_attention(bs_ctx *ctx, const bs_batch *batch, const void *q, void *out,
                 const void *kv_pool, int64_t n_pages, void *stream, uint32_t flags);

/*   bs_attention_noalloc: bs_attention for callers that cannot allocate device memory during the call
 *   (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same
 *   arguments, same kernels, same result; the descriptor and the partial softmax states of the call live
 *   in a 16 MiB array that is part of the library's code object (every GPU the library runs on holds its
 *   own copy until the process ends) instead of the context's growing workspace.  Limits, checked before
 *   anything is enqueued (BS_EINVAL with a message): the planned descriptor at most 1 MiB, the partial
 *   states at most 15 MiB (one state of n_q_heads x (head_dim + 2) floats per sequence and chunk of up to
 *   64 pages along its prefix path and tail), at most 2^15 sequences and prefix nodes, 2^20 pages.  Calls
 *   on one GPU share the array, whatever their context: calls that overlap in time on one GPU race, and
 *   nothing in it survives a call.  Makes no hipMalloc / hipFree (bs_create has made all of them). */
int bs_attention_noalloc(bs_ctx *ctx, const bs_batch *batch, const void *q, void *out,
                         const void *kv_pool, int64_t n_pages, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BLENDSTEP_H */
