// C ABI of the blended decoder-layer step: context, descriptor validation, the
// per-step plan (row tables, decode-attention work items, partial-state slots)
// and the kernel schedule.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/blendstep.h"
#include "attn.hpp"
#include "gemm.hpp"
#include "misc.hpp"

using namespace bs;

// Scratch of bs_attention_noalloc: the descriptor blob and the partial softmax states of one call live
// in this array, which every GPU the library runs on holds from the moment the code object is loaded
// until the process ends.  Host code never uses the array's name as an address: bs_create asks the
// runtime for the device address once per device and keeps it in g_scratch_ptr.
#define BS_NOALLOC_BLOB_BYTES (1u << 20)
#define BS_NOALLOC_SCRATCH_BYTES (16u << 20)
static __device__ __align__(256) unsigned char scratch[BS_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
unsigned char *g_scratch_ptr[MAX_DEVICES] = {nullptr};
std::mutex g_scratch_mutex;

constexpr int RING = 4;
constexpr long TRACE_CAP = 8192;  // workgroups per launch that a timeline can hold
std::string g_create_error;

struct Plan {
  int n_seq = 0, n_prefill = 0, n_rows = 0, n_decode = 0, n_prefill_rows = 0;
  long off_row_start = 0, off_kv_len = 0, off_page_start = 0, off_row_pos = 0, off_row_page = 0, off_row_slot = 0,
       off_part_start = 0, off_pf_work = 0, off_items = 0, off_pages = 0, total_ints = 0;
  long total_node_pages = 0, n_slots = 0;
  int n_pf_work = 0;
  int n_wide = 0, n_narrow = 0;  // decode items with up to 64 / up to 16 query rows (wide ones first)
};

}  // namespace

struct bs_ctx {
  bs_layer_cfg cfg;
  int device = 0;
  std::string err;
  float *rope_cos = nullptr, *rope_sin = nullptr;
  // activations workspace
  int cap_rows = 0, ss2_parts = 0;
  uint16_t *xg = nullptr, *qbuf = nullptr, *attn = nullptr, *xg2 = nullptr, *act = nullptr;
  float *x1 = nullptr, *rstd1 = nullptr, *rstd2 = nullptr, *ss2 = nullptr;
  long cap_slots = 0;
  float *part_acc = nullptr, *part_m = nullptr, *part_l = nullptr;
  uint16_t *hid[2] = {nullptr, nullptr};  // activations between the layers of bs_blend_layers
  float *splitk_ws = nullptr;  // fp32 partial products of the split-K GEMMs (few-row steps)
  size_t cap_splitk = 0;
  // descriptor blob: pinned host ring and one device copy
  long cap_blob = 0;
  int32_t *d_blob = nullptr;
  int32_t *h_blob[RING] = {nullptr, nullptr, nullptr, nullptr};
  long h_cap[RING] = {0, 0, 0, 0};
  hipEvent_t h_ev[RING];
  bool h_ev_live[RING] = {false, false, false, false};
  int ring_pos = 0;
  // host scratch reused across calls
  std::vector<int32_t> refcount, path_pages, path_chunks, members, blob;
  std::vector<DecodeItem> items, items_wide;
  std::vector<int32_t> pf_work;
  std::vector<std::pair<int, std::pair<int, int>>> pf_order;
  unsigned char *scratch_ptr = nullptr;  // this device's copy of the static scratch array
  // co-scheduling of decode attention with the prefill rows' GEMMs (BS_FLAG_OVERLAP)
  float *sk_ws = nullptr;       // partial tiles of the GEMM launches whose workgroups share tiles
  unsigned *sk_cnt = nullptr;   // their arrival counters (zero between launches)
  unsigned *sync_words = nullptr;  // [0..3] queue counters of the launches of a step, [4..6] finished tiles, [8..10] queue position at which each launch closed
  bs_overlap_knobs ov = {0, 208, 8, 256, -1, 2, 0, 1, 96, 0};
  int64_t ov_first_bytes = 0;      // KV bytes of the 16-row units that the last co-scheduled step gave to its first attention launch
  int ov_first_items = 0;          // and their number
  // optional timeline of the co-scheduled launches: TRACE_CAP workgroups of 8 wavefront records per launch
  uint64_t *trace_buf = nullptr;
  long trace_wgs[4] = {0, 0, 0, 0};  // workgroups of the last step's launches
  int n_cu = 256;
  int forced_tiles = 0;            // bs_set_gemm_tiles
  // tunables
  int chunk_pages = 64;       // pages per chunk of decode-attention work: private tails and nodes with few member rows
  int chunk_pages_wide = 32;  // nodes whose items carry more than 16 query rows: four wavefronts share an item, and every
                              // chunk costs one partial state per member row
  // profiling
  bool prof = false;
  struct Span { hipEvent_t a, b; };
  std::vector<Span> spans[BS_K_COUNT];
  std::vector<hipEvent_t> free_events;
  double prof_ms[BS_K_COUNT] = {0};
  int64_t prof_n[BS_K_COUNT] = {0};
};

namespace {

int fail(bs_ctx *ctx, int code, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (ctx) ctx->err = buf; else g_create_error = buf;
  return code;
}

// No exception crosses the C boundary: host allocations (vectors that grow with the batch) can throw.
template <class F>
int guarded(bs_ctx *c, F &&body) {
  try {
    return body();
  } catch (const std::bad_alloc &) {
    return fail(c, BS_ENOMEM, "out of host memory");
  } catch (const std::exception &e) {
    return fail(c, BS_EINVAL, "unexpected exception: %s", e.what());
  } catch (...) {
    return fail(c, BS_EINVAL, "unexpected exception");
  }
}

#define HIP_TRY(ctx, expr)                                                                         \
  do {                                                                                             \
    hipError_t e_ = (expr);                                                                        \
    if (e_ != hipSuccess) return fail(ctx, BS_EHIP, "%s: %s", #expr, hipGetErrorString(e_));        \
  } while (0)

template <class T>
int dev_alloc(bs_ctx *ctx, T **p, size_t count) {
  if (*p) { hipError_t e = hipFree(*p); *p = nullptr; if (e != hipSuccess) return fail(ctx, BS_EHIP, "hipFree: %s", hipGetErrorString(e)); }
  if (count == 0) return BS_OK;
  hipError_t e = hipMalloc(reinterpret_cast<void **>(p), count * sizeof(T));
  if (e != hipSuccess) { *p = nullptr; return fail(ctx, BS_ENOMEM, "hipMalloc of %zu bytes: %s", count * sizeof(T), hipGetErrorString(e)); }
  return BS_OK;
}

int ensure_rows(bs_ctx *c, int rows) {
  if (rows <= c->cap_rows) return BS_OK;
  const int cap = std::max(rows, 256);
  const bs_layer_cfg &g = c->cfg;
  const size_t hd = (size_t)g.n_q_heads * g.head_dim;
  int rc;
  c->cap_rows = 0;
  if ((rc = dev_alloc(c, &c->xg, (size_t)cap * g.d_model))) return rc;
  if ((rc = dev_alloc(c, &c->hid[0], (size_t)cap * g.d_model))) return rc;
  if ((rc = dev_alloc(c, &c->hid[1], (size_t)cap * g.d_model))) return rc;
  if ((rc = dev_alloc(c, &c->qbuf, (size_t)cap * hd))) return rc;
  if ((rc = dev_alloc(c, &c->attn, (size_t)cap * hd))) return rc;
  if ((rc = dev_alloc(c, &c->x1, (size_t)cap * g.d_model))) return rc;
  if ((rc = dev_alloc(c, &c->xg2, (size_t)cap * g.d_model))) return rc;
  if ((rc = dev_alloc(c, &c->act, (size_t)cap * g.d_ffn))) return rc;
  if ((rc = dev_alloc(c, &c->rstd1, (size_t)cap))) return rc;
  if ((rc = dev_alloc(c, &c->rstd2, (size_t)cap))) return rc;
  c->ss2_parts = ((g.d_model + 255) / 256) * 4;  // covers both tile shapes of the projection
  if ((rc = dev_alloc(c, &c->ss2, (size_t)cap * c->ss2_parts))) return rc;
  c->cap_rows = cap;
  return BS_OK;
}

int ensure_slots(bs_ctx *c, long slots) {
  if (slots <= c->cap_slots) return BS_OK;
  const long cap = slots + slots / 4 + 64;
  const size_t hq = c->cfg.n_q_heads;
  int rc;
  c->cap_slots = 0;
  if ((rc = dev_alloc(c, &c->part_acc, (size_t)cap * hq * c->cfg.head_dim))) return rc;
  if ((rc = dev_alloc(c, &c->part_m, (size_t)cap * hq))) return rc;
  if ((rc = dev_alloc(c, &c->part_l, (size_t)cap * hq))) return rc;
  c->cap_slots = cap;
  return BS_OK;
}

int ensure_splitk(bs_ctx *c, size_t floats) {
  if (floats <= c->cap_splitk) return BS_OK;
  c->cap_splitk = 0;
  int rc = dev_alloc(c, &c->splitk_ws, floats);
  if (rc) return rc;
  c->cap_splitk = floats;
  return BS_OK;
}

int ensure_blob_host(bs_ctx *c, long ints, int slot) {
  if (ints > c->h_cap[slot]) {
    const long cap = ints + ints / 4 + 1024;
    if (c->h_blob[slot]) { HIP_TRY(c, hipHostFree(c->h_blob[slot])); c->h_blob[slot] = nullptr; c->h_cap[slot] = 0; }
    hipError_t e = hipHostMalloc(reinterpret_cast<void **>(&c->h_blob[slot]), (size_t)cap * sizeof(int32_t), hipHostMallocDefault);
    if (e != hipSuccess) return fail(c, BS_ENOMEM, "hipHostMalloc: %s", hipGetErrorString(e));
    c->h_cap[slot] = cap;
  }
  return BS_OK;
}

int ensure_blob(bs_ctx *c, long ints, int slot) {
  if (ints > c->cap_blob) {
    const long cap = ints + ints / 4 + 1024;
    c->cap_blob = 0;
    int rc = dev_alloc(c, &c->d_blob, (size_t)cap);
    if (rc) return rc;
    c->cap_blob = cap;
  }
  return ensure_blob_host(c, ints, slot);
}

// ---------------------------------------------------------------------------------
// descriptor validation (host only)
// ---------------------------------------------------------------------------------
int validate(bs_ctx *c, const bs_batch *b, int64_t n_pages) {
  if (!b) return fail(c, BS_EINVAL, "batch is NULL");
  const int ps = c->cfg.page_size;
  if (b->n_seq < 0 || b->n_prefill < 0 || b->n_prefill > b->n_seq || b->n_rows < 0)
    return fail(c, BS_EINVAL, "bad counts: n_seq=%d n_prefill=%d n_rows=%d", b->n_seq, b->n_prefill, b->n_rows);
  if (n_pages < 0 || n_pages > (int64_t)0x7fffffff) return fail(c, BS_EINVAL, "n_pages=%lld out of range", (long long)n_pages);
  if (b->n_seq == 0) {
    if (b->n_rows != 0) return fail(c, BS_EINVAL, "n_rows=%d with no sequences", b->n_rows);
    return BS_OK;
  }
  if (!b->row_start || !b->kv_len || !b->page_start || (!b->page_ids && b->page_start[b->n_seq] > 0))
    return fail(c, BS_EINVAL, "a required array is NULL");
  if (b->row_start[0] != 0 || b->page_start[0] != 0) return fail(c, BS_EINVAL, "CSR arrays must start at 0");
  for (int s = 0; s < b->n_seq; ++s) {
    const int q = b->row_start[s + 1] - b->row_start[s];
    if (q < 1) return fail(c, BS_EINVAL, "sequence %d has %d rows", s, q);
    if (s >= b->n_prefill && q != 1) return fail(c, BS_EINVAL, "decode sequence %d has %d rows (must be 1)", s, q);
    if (b->kv_len[s] < q) return fail(c, BS_EINVAL, "sequence %d: kv_len %d < its %d rows", s, b->kv_len[s], q);
    if (b->kv_len[s] > c->cfg.max_positions)
      return fail(c, BS_EINVAL, "sequence %d: kv_len %d exceeds max_positions %d", s, b->kv_len[s], c->cfg.max_positions);
    const int np = b->page_start[s + 1] - b->page_start[s];
    if (np < 0) return fail(c, BS_EINVAL, "page_start not monotone at sequence %d", s);
    if ((int64_t)np * ps < b->kv_len[s])
      return fail(c, BS_EINVAL, "sequence %d: kv_len %d exceeds its %d pages", s, b->kv_len[s], np);
  }
  if (b->row_start[b->n_seq] != b->n_rows)
    return fail(c, BS_EINVAL, "row_start ends at %d, n_rows is %d", b->row_start[b->n_seq], b->n_rows);
  const int n_tab = b->page_start[b->n_seq];
  c->refcount.assign((size_t)n_pages, 0);
  for (int i = 0; i < n_tab; ++i) {
    const int p = b->page_ids[i];
    if (p < 0 || p >= n_pages) return fail(c, BS_EINVAL, "page_ids[%d]=%d outside the pool of %lld pages", i, p, (long long)n_pages);
    ++c->refcount[p];
  }
  // prefix nodes
  const int nn = b->n_nodes;
  if (nn < 0) return fail(c, BS_EINVAL, "n_nodes=%d", nn);
  c->path_pages.assign((size_t)nn, 0);
  c->members.assign((size_t)nn, 0);
  if (nn > 0) {
    if (!b->node_parent || !b->node_page_start || !b->node_seq_first || !b->node_seq_count || !b->seq_leaf_node)
      return fail(c, BS_EINVAL, "a node array is NULL");
    if (b->node_page_start[0] != 0) return fail(c, BS_EINVAL, "node_page_start must start at 0");
    for (int n = 0; n < nn; ++n) {
      const int par = b->node_parent[n];
      if (par < -1 || par >= n) return fail(c, BS_EINVAL, "node %d: parent %d breaks DFS pre-order", n, par);
      const int np = b->node_page_start[n + 1] - b->node_page_start[n];
      if (np < 0) return fail(c, BS_EINVAL, "node_page_start not monotone at node %d", n);
      const int f = b->node_seq_first[n], cnt = b->node_seq_count[n];
      if (cnt < 0) return fail(c, BS_EINVAL, "node %d: negative member count", n);
      if (cnt > 0 && (f < b->n_prefill || f + cnt > b->n_seq))
        return fail(c, BS_EINVAL, "node %d: members [%d,%d) are not decode sequences", n, f, f + cnt);
      if (par >= 0 && cnt > 0) {
        const int pf = b->node_seq_first[par], pc = b->node_seq_count[par];
        if (f < pf || f + cnt > pf + pc) return fail(c, BS_EINVAL, "node %d: members not inside its parent's run", n);
      }
      c->path_pages[n] = np + (par >= 0 ? c->path_pages[par] : 0);
      for (int i = b->node_page_start[n]; i < b->node_page_start[n + 1]; ++i) {
        const int p = b->node_page_ids[i];
        if (p < 0 || p >= n_pages) return fail(c, BS_EINVAL, "node_page_ids[%d]=%d outside the pool", i, p);
        c->refcount[p] += 2;  // node pages are never writable, even with a single member
      }
    }
  }
  for (int s = 0; s < b->n_seq; ++s) {
    const int leaf = b->seq_leaf_node ? b->seq_leaf_node[s] : -1;
    if (leaf < -1 || leaf >= nn) return fail(c, BS_EINVAL, "sequence %d: leaf node %d out of range", s, leaf);
    const int q = b->row_start[s + 1] - b->row_start[s];
    if (leaf >= 0) {
      if (s < b->n_prefill) return fail(c, BS_EINVAL, "prefill segment %d cannot be a node member", s);
      const int shared = c->path_pages[leaf];
      if ((int64_t)shared * ps > b->kv_len[s] - q)
        return fail(c, BS_EINVAL, "sequence %d: %d shared pages leave no private slot for its new token", s, shared);
      // the path's pages must open the sequence's table, root first
      int node = leaf, end = shared;
      while (node >= 0) {
        const int np = b->node_page_start[node + 1] - b->node_page_start[node];
        const int f = b->node_seq_first[node], cnt = b->node_seq_count[node];
        if (s < f || s >= f + cnt) return fail(c, BS_EINVAL, "sequence %d lies outside the member run of node %d", s, node);
        ++c->members[node];
        const int32_t *tab = b->page_ids + b->page_start[s] + (end - np);
        if (np > 0 && std::memcmp(tab, b->node_page_ids + b->node_page_start[node], (size_t)np * sizeof(int32_t)) != 0)
          return fail(c, BS_EINVAL, "sequence %d: page table does not carry the pages of node %d", s, node);
        end -= np;
        node = b->node_parent[node];
      }
    }
    // pages this step writes must be referenced exactly once
    const int first = (b->kv_len[s] - q) / ps, last = (b->kv_len[s] - 1) / ps;
    for (int pg = first; pg <= last; ++pg) {
      const int p = b->page_ids[b->page_start[s] + pg];
      if (c->refcount[p] != 1)
        return fail(c, BS_EINVAL, "sequence %d appends into page %d, which is referenced more than once", s, p);
    }
  }
  for (int n = 0; n < nn; ++n)
    if (c->members[n] != b->node_seq_count[n])
      return fail(c, BS_EINVAL, "node %d: %d sequences name it, its member run has %d", n, c->members[n], b->node_seq_count[n]);
  return BS_OK;
}

// ---------------------------------------------------------------------------------
// plan: everything the kernels need, packed in one int32 blob
// ---------------------------------------------------------------------------------
int build_plan(bs_ctx *c, const bs_batch *b, Plan &p, bool with_rows) {
  const int ps = c->cfg.page_size;
  const int grp = c->cfg.n_q_heads / c->cfg.n_kv_heads;
  const int ch = c->chunk_pages;
  const int nn = b->n_nodes;
  p.n_seq = b->n_seq; p.n_prefill = b->n_prefill; p.n_rows = b->n_rows; p.n_decode = b->n_seq - b->n_prefill;
  p.n_prefill_rows = b->n_seq ? b->row_start[b->n_prefill] : 0;
  p.total_node_pages = nn > 0 ? b->node_page_start[nn] : 0;
  const int n_tab = b->n_seq ? b->page_start[b->n_seq] : 0;

  // chunk counts along each node's root path (path_pages was filled by validate)
  c->path_chunks.assign((size_t)nn, 0);
  c->items.clear();
  c->items_wide.clear();
  const int max_members = std::max(1, 64 / grp);  // up to 64 query rows per work item
  for (int n = 0; n < nn; ++n) {
    const int par = b->node_parent[n];
    const int np = b->node_page_start[n + 1] - b->node_page_start[n];
    const int above = par >= 0 ? c->path_chunks[par] : 0;
    const int cnt = b->node_seq_count[n];
    const int n_groups = cnt > 0 ? (cnt + max_members - 1) / max_members : 1;
    // the chunk size of a node is one for all its member groups: their partial states share slot numbers
    const int chn = ((cnt + n_groups - 1) / n_groups) * grp > 16 ? c->chunk_pages_wide : ch;
    const int nch = (np + chn - 1) / chn;
    c->path_chunks[n] = above + nch;
    if (cnt <= 0 || np <= 0) continue;
    for (int g = 0; g < n_groups; ++g) {
      const int lo = (int)((long)cnt * g / n_groups), hi = (int)((long)cnt * (g + 1) / n_groups);
      for (int k = 0; k < nch; ++k) {
        DecodeItem it{};
        it.page_off = b->node_page_start[n] + k * chn;
        it.n_tokens = std::min(chn, np - k * chn) * ps;
        it.seq_first = b->node_seq_first[n] + lo;
        it.n_members = hi - lo;
        it.slot_off = above + k;
        ((hi - lo) * grp > 16 ? c->items_wide : c->items).push_back(it);
      }
    }
  }
  // private tails and partial-state slots
  std::vector<int32_t> &blob = c->blob;
  p.off_row_start = 0;
  p.off_kv_len = p.off_row_start + b->n_seq + 1;
  p.off_page_start = p.off_kv_len + b->n_seq;
  p.off_part_start = p.off_page_start + b->n_seq + 1;
  p.off_row_pos = p.off_part_start + b->n_seq + 1;
  p.off_row_page = p.off_row_pos + b->n_rows;
  p.off_row_slot = p.off_row_page + b->n_rows;
  p.off_pf_work = p.off_row_slot + b->n_rows;
  blob.assign((size_t)p.off_pf_work, 0);
  if (b->n_seq) {
    std::memcpy(&blob[p.off_row_start], b->row_start, sizeof(int32_t) * (b->n_seq + 1));
    std::memcpy(&blob[p.off_kv_len], b->kv_len, sizeof(int32_t) * b->n_seq);
    std::memcpy(&blob[p.off_page_start], b->page_start, sizeof(int32_t) * (b->n_seq + 1));
  }
  int32_t *part_start = &blob[p.off_part_start];
  part_start[0] = 0;
  for (int s = 0; s < b->n_seq; ++s) {
    int slots = 0;
    if (s >= b->n_prefill) {
      const int leaf = (nn > 0) ? b->seq_leaf_node[s] : -1;
      const int shared = leaf >= 0 ? c->path_pages[leaf] : 0;
      const int above = leaf >= 0 ? c->path_chunks[leaf] : 0;
      const int tail_tok = b->kv_len[s] - shared * ps;  // >= 1 by validation
      const int tail_pg = (tail_tok + ps - 1) / ps;
      const int nch = (tail_pg + ch - 1) / ch;
      for (int k = 0; k < nch; ++k) {
        DecodeItem it{};
        it.page_off = (int32_t)(p.total_node_pages + b->page_start[s] + shared + k * ch);
        it.n_tokens = std::min(ch * ps, tail_tok - k * ch * ps);
        it.seq_first = s;
        it.n_members = 1;
        it.slot_off = above + k;
        c->items.push_back(it);
      }
      slots = above + nch;
    }
    part_start[s + 1] = part_start[s] + slots;
  }
  p.n_slots = part_start[b->n_seq];
  if (with_rows) {
    for (int s = 0; s < b->n_seq; ++s) {
      const int r0 = b->row_start[s], q = b->row_start[s + 1] - r0, first = b->kv_len[s] - q;
      for (int j = 0; j < q; ++j) {
        const int pos = first + j;
        blob[p.off_row_pos + r0 + j] = pos;
        blob[p.off_row_page + r0 + j] = b->page_ids[b->page_start[s] + pos / ps];
        blob[p.off_row_slot + r0 + j] = pos % ps;
      }
    }
  }
  // prefill work: (sequence, block of 64 query rows), longest contexts first
  c->pf_work.clear();
  std::vector<std::pair<int, std::pair<int, int>>> &order = c->pf_order;
  order.clear();
  for (int s = 0; s < b->n_prefill; ++s) {
    const int q = b->row_start[s + 1] - b->row_start[s];
    for (int k = 0; k * 64 < q; ++k) order.push_back({-(b->kv_len[s] - q + std::min(q, k * 64 + 64)), {s, k}});
  }
  std::stable_sort(order.begin(), order.end(), [](const auto &x, const auto &y) { return x.first < y.first; });
  p.n_pf_work = (int)order.size();
  p.off_items = p.off_pf_work + 2L * p.n_pf_work;
  // longest chunks first: the many short tail chunks then fill the gaps at the end of the launch
  auto longer = [](const DecodeItem &x, const DecodeItem &y) { return x.n_tokens > y.n_tokens; };
  std::stable_sort(c->items.begin(), c->items.end(), longer);
  std::stable_sort(c->items_wide.begin(), c->items_wide.end(), longer);
  p.n_wide = (int)c->items_wide.size();
  p.n_narrow = (int)c->items.size();
  const long n_items = (long)p.n_wide + p.n_narrow;
  p.off_pages = p.off_items + 8 * n_items;
  p.total_ints = p.off_pages + p.total_node_pages + n_tab;
  blob.resize((size_t)p.total_ints);
  for (int i = 0; i < p.n_pf_work; ++i) {
    blob[p.off_pf_work + 2 * i] = order[i].second.first;
    blob[p.off_pf_work + 2 * i + 1] = order[i].second.second;
  }
  if (p.n_wide) std::memcpy(&blob[p.off_items], c->items_wide.data(), sizeof(DecodeItem) * p.n_wide);
  if (p.n_narrow) std::memcpy(&blob[p.off_items + 8L * p.n_wide], c->items.data(), sizeof(DecodeItem) * p.n_narrow);
  if (p.total_node_pages) std::memcpy(&blob[p.off_pages], b->node_page_ids, sizeof(int32_t) * p.total_node_pages);
  if (n_tab) std::memcpy(&blob[p.off_pages + p.total_node_pages], b->page_ids, sizeof(int32_t) * n_tab);
  for (long i = 0; i < n_items; ++i) {  // every item has at least one token, hence one page
    DecodeItem *it = reinterpret_cast<DecodeItem *>(&blob[p.off_items + 8 * i]);
    it->page0 = blob[p.off_pages + it->page_off];
    it->page1 = blob[p.off_pages + it->page_off + (it->n_tokens > ps ? 1 : 0)];
  }
  return BS_OK;
}

// Stages the plan in the pinned ring and copies it to `dst` (the context's descriptor buffer, grown
// on demand, or - no_grow - a buffer of the caller's that is known to be large enough, with the
// staging slots of bs_create, which are).
int upload_plan(bs_ctx *c, const Plan &p, hipStream_t stream, int32_t *dst = nullptr, bool no_grow = false) {
  const int slot = c->ring_pos;
  c->ring_pos = (c->ring_pos + 1) % RING;
  if (c->h_ev_live[slot]) HIP_TRY(c, hipEventSynchronize(c->h_ev[slot]));
  if (no_grow) {
    if (p.total_ints > c->h_cap[slot]) return fail(c, BS_EINVAL, "descriptor of %ld words exceeds the staging slot", p.total_ints);
  } else {
    int rc = ensure_blob(c, p.total_ints, slot);
    if (rc) return rc;
  }
  if (p.total_ints == 0) return BS_OK;
  std::memcpy(c->h_blob[slot], c->blob.data(), sizeof(int32_t) * p.total_ints);
  HIP_TRY(c, hipMemcpyAsync(dst ? dst : c->d_blob, c->h_blob[slot], sizeof(int32_t) * p.total_ints, hipMemcpyHostToDevice, stream));
  HIP_TRY(c, hipEventRecord(c->h_ev[slot], stream));
  c->h_ev_live[slot] = true;
  return BS_OK;
}

// ---------------------------------------------------------------------------------
// profiling spans
// ---------------------------------------------------------------------------------
int span_begin(bs_ctx *c, int which, hipStream_t s, bs_ctx::Span &sp) {
  if (!c->prof) return BS_OK;
  for (hipEvent_t *e : {&sp.a, &sp.b}) {
    if (!c->free_events.empty()) { *e = c->free_events.back(); c->free_events.pop_back(); }
    else HIP_TRY(c, hipEventCreate(e));
  }
  (void)which;
  HIP_TRY(c, hipEventRecord(sp.a, s));
  return BS_OK;
}
int span_end(bs_ctx *c, int which, hipStream_t s, bs_ctx::Span &sp) {
  if (!c->prof) return BS_OK;
  HIP_TRY(c, hipEventRecord(sp.b, s));
  c->spans[which].push_back(sp);
  return BS_OK;
}

#define SPAN(ctx, which, stream, body)                       \
  do {                                                       \
    bs_ctx::Span sp_{};                                      \
    int rc_ = span_begin(ctx, which, stream, sp_);           \
    if (rc_) return rc_;                                     \
    body;                                                    \
    rc_ = span_end(ctx, which, stream, sp_);                 \
    if (rc_) return rc_;                                     \
  } while (0)

AttnShape attn_shape(const bs_ctx *c) {
  AttnShape s;
  s.n_q_heads = c->cfg.n_q_heads; s.n_kv_heads = c->cfg.n_kv_heads; s.head_dim = c->cfg.head_dim; s.page_size = c->cfg.page_size;
  s.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)c->cfg.head_dim));
  return s;
}

PrefillArgs prefill_args(const bs_ctx *c, const Plan &p, const uint16_t *q, uint16_t *out, const uint16_t *pool) {
  PrefillArgs a;
  a.s = attn_shape(c);
  a.work = c->d_blob + p.off_pf_work; a.n_work = p.n_pf_work;
  a.row_start = c->d_blob + p.off_row_start; a.kv_len = c->d_blob + p.off_kv_len;
  a.page_start = c->d_blob + p.off_page_start; a.page_ids = c->d_blob + p.off_pages + p.total_node_pages;
  a.q = q; a.kv_pool = pool; a.out = out;
  return a;
}

DecodeArgs decode_args(const bs_ctx *c, const Plan &p, const uint16_t *q, const uint16_t *pool) {
  DecodeArgs a;
  a.s = attn_shape(c);
  a.items = reinterpret_cast<const DecodeItem *>(c->d_blob + p.off_items);
  a.item_pages = c->d_blob + p.off_pages;
  a.row_base = p.n_prefill_rows - p.n_prefill; a.part_start = c->d_blob + p.off_part_start;
  a.q = q; a.kv_pool = pool;
  a.part_acc = c->part_acc; a.part_m = c->part_m; a.part_l = c->part_l;
  return a;
}

int run_prefill_attn(bs_ctx *c, const Plan &p, const uint16_t *q, uint16_t *out, const uint16_t *pool, hipStream_t st) {
  if (p.n_pf_work == 0) return BS_OK;
  const PrefillArgs a = prefill_args(c, p, q, out, pool);
  SPAN(c, BS_K_ATTN_PREFILL, st, HIP_TRY(c, launch_prefill_attn(a, st)));
  return BS_OK;
}

int run_decode_merge(bs_ctx *c, const Plan &p, uint16_t *out, hipStream_t st) {
  MergeArgs m;
  m.s = attn_shape(c); m.n_prefill = p.n_prefill; m.n_decode = p.n_decode;
  m.row_start = c->d_blob + p.off_row_start; m.part_start = c->d_blob + p.off_part_start;
  m.part_acc = c->part_acc; m.part_m = c->part_m; m.part_l = c->part_l; m.out = out;
  SPAN(c, BS_K_ATTN_MERGE, st, HIP_TRY(c, launch_decode_merge(m, st)));
  return BS_OK;
}

int run_decode_attn(bs_ctx *c, const Plan &p, const uint16_t *q, uint16_t *out, const uint16_t *pool, hipStream_t st) {
  if (p.n_decode == 0) return BS_OK;
  const DecodeArgs a = decode_args(c, p, q, pool);
  SPAN(c, BS_K_ATTN_DECODE, st, HIP_TRY(c, launch_decode_attn(a, p.n_wide, p.n_narrow, st)));
  return run_decode_merge(c, p, out, st);
}

// Attention of a whole step on one stream: prefill and decode rows in one launch where the step
// has both (its time is booked under the decode class), else the launch of the kind it has.
int run_attention(bs_ctx *c, const Plan &p, const uint16_t *q, uint16_t *out, const uint16_t *pool, hipStream_t st) {
  if (p.n_pf_work == 0 || p.n_decode == 0 || !blended_attn_possible(attn_shape(c))) {
    int rc = run_prefill_attn(c, p, q, out, pool, st);
    return rc ? rc : run_decode_attn(c, p, q, out, pool, st);
  }
  const PrefillArgs pf = prefill_args(c, p, q, out, pool);
  const DecodeArgs d = decode_args(c, p, q, pool);
  SPAN(c, BS_K_ATTN_DECODE, st, HIP_TRY(c, launch_blended_attn(d, p.n_wide, p.n_narrow, pf, st)));
  return run_decode_merge(c, p, out, st);
}

// GEMM arguments of the output projection (+ first residual, second norm), of gate/up (+ SwiGLU)
// and of the down projection (+ second residual) for rows [r0, r1)
GemmArgs o_proj_args(bs_ctx *c, const bs_weights *w, const uint16_t *x, int r0, int r1) {
  const bs_layer_cfg &g = c->cfg;
  const int hd = g.n_q_heads * g.head_dim, d = g.d_model;
  GemmArgs o{};
  o.A = c->attn + (size_t)r0 * hd; o.lda = hd; o.B = (const uint16_t *)w->w_o; o.ldb = hd;
  o.M = r1 - r0; o.N = d; o.K = hd;
  o.C32 = c->x1 + (size_t)r0 * d; o.ldc = d; o.resid = x + (size_t)r0 * d; o.ldr = d;
  o.gain = (const uint16_t *)w->g_ffn; o.C_gain = c->xg2 + (size_t)r0 * d;
  o.ss_out = c->ss2 + r0; o.ss_stride = c->cap_rows;
  o.sk_ws = c->sk_ws; o.sk_cnt = c->sk_cnt;
  return o;
}

GemmArgs gate_up_args(bs_ctx *c, const bs_weights *w, int r0, int r1) {
  const bs_layer_cfg &g = c->cfg;
  const int d = g.d_model, f = g.d_ffn;
  GemmArgs u{};
  u.A = c->xg2 + (size_t)r0 * d; u.lda = d; u.B = (const uint16_t *)w->w_gate_up; u.ldb = d;
  u.M = r1 - r0; u.N = f; u.K = d;
  u.C = c->act + (size_t)r0 * f; u.ldc = f;
  u.rstd = c->rstd2 + r0;
  u.sk_ws = c->sk_ws; u.sk_cnt = c->sk_cnt;
  return u;
}

GemmArgs down_args(bs_ctx *c, const bs_weights *w, uint16_t *y, int r0, int r1) {
  const bs_layer_cfg &g = c->cfg;
  const int d = g.d_model, f = g.d_ffn;
  GemmArgs dn{};
  dn.A = c->act + (size_t)r0 * f; dn.lda = f; dn.B = (const uint16_t *)w->w_down; dn.ldb = f;
  dn.M = r1 - r0; dn.N = d; dn.K = f;
  dn.C = y + (size_t)r0 * d; dn.ldc = d; dn.resid32 = c->x1 + (size_t)r0 * d; dn.ldr = d;
  dn.sk_ws = c->sk_ws; dn.sk_cnt = c->sk_cnt;
  return dn;
}

// output projection and gate/up for rows [r0, r1)
int run_o_gate_up(bs_ctx *c, const bs_weights *w, const uint16_t *x, int r0, int r1, hipStream_t st, int k_o = BS_K_GEMM_O,
                  int k_gu = BS_K_GEMM_GATE_UP) {
  const int rows = r1 - r0;
  if (rows <= 0) return BS_OK;
  const bs_layer_cfg &g = c->cfg;
  const int d = g.d_model;
  GemmArgs o = o_proj_args(c, w, x, r0, r1);
  o.k_splits = gemm_splitk_choice(rows, d, o.K, EPI_RESID_NORM, 0);
  if (o.k_splits > 1) {
    int rc = ensure_splitk(c, (size_t)o.k_splits * rows * d);
    if (rc) return rc;
    o.splitk_ws = c->splitk_ws;
    o.rstd_out = c->rstd2 + r0;  // the reduction closes the second norm's statistics itself
    o.rstd_eps = g.rms_eps;
  }
  const int parts = gemm_ss_parts(o, EPI_RESID_NORM, g.head_dim);
  SPAN(c, k_o, st, {
    HIP_TRY(c, launch_gemm(o, EPI_RESID_NORM, g.head_dim, st));
    if (o.k_splits <= 1)
      HIP_TRY(c, launch_rstd_finalize(c->ss2 + r0, parts, c->cap_rows, c->rstd2 + r0, rows, d, g.rms_eps, st));
  });
  const GemmArgs u = gate_up_args(c, w, r0, r1);
  GemmArgs head, tail;
  if (gemm_round_split(u, EPI_SWIGLU, g.head_dim, &head, &tail)) {
    SPAN(c, k_gu, st, HIP_TRY(c, launch_gemm(head, EPI_SWIGLU, g.head_dim, st)));
    SPAN(c, k_gu, st, HIP_TRY(c, launch_gemm(tail, EPI_SWIGLU, g.head_dim, st)));
  } else {
    SPAN(c, k_gu, st, HIP_TRY(c, launch_gemm(u, EPI_SWIGLU, g.head_dim, st)));
  }
  return BS_OK;
}

// down projection and second residual for rows [r0, r1)
int run_down(bs_ctx *c, const bs_weights *w, uint16_t *y, int r0, int r1, hipStream_t st, int k_dn = BS_K_GEMM_DOWN) {
  const int rows = r1 - r0;
  if (rows <= 0) return BS_OK;
  const bs_layer_cfg &g = c->cfg;
  GemmArgs dn = down_args(c, w, y, r0, r1);
  dn.k_splits = gemm_splitk_choice(rows, dn.N, dn.K, EPI_RESID, 0);
  if (dn.k_splits > 1) {
    int rc = ensure_splitk(c, (size_t)dn.k_splits * rows * dn.N);
    if (rc) return rc;
    dn.splitk_ws = c->splitk_ws;
  }
  SPAN(c, k_dn, st, HIP_TRY(c, launch_gemm(dn, EPI_RESID, g.head_dim, st)));
  return BS_OK;
}

// The co-scheduled part of a step (BS_FLAG_OVERLAP; Section 3.3: overlapped, compute-bound and
// memory-bound work cost the larger of their times; Section 2.2, operator-level overlapping
// between the parts of a batch).  The prefill rows and the decode units that carry more
// than 16 query rows (shared prefix nodes) have their attention first, in one launch; the
// 16-row units (private tails: nearly all of the KV bytes) then form a queue that is drained
// by attention workgroups inside the prefill rows' three GEMM launches, on CUs of their own,
// and by one launch over the whole chip for what is left.  The decode rows' output
// projection and FFN follow.  One stream, no events: what overlaps shares a launch.
// Estimated duration of a GEMM launch of M rows on n_cu CUs by whole rounds of tiles (the cost model
// behind the tile choice: a 256x256 tile sustains 5.8 TFLOP/s per CU, a 160x256 tile 4.5, and 128x128
// tiles, two per CU, take three quarters of a 256x256 round for half its work).
double est_gemm_s(int M, int b_rows, int K, int n_cu) {
  if (M <= 0) return 0.0;
  const double big = 2.0 * 256 * 256 * K / 5.8e12, tall = 2.0 * 160 * 256 * K / 4.5e12, small = 0.75 * big;
  auto rounds = [](long tiles, long slots) { return (double)((tiles + slots - 1) / slots); };
  const long tn = (b_rows + 255) / 256;
  const double t_big = rounds((long)((M + 255) / 256) * tn, n_cu) * big;
  const double t_tall = rounds((long)((M + 159) / 160) * tn, n_cu) * tall;
  const double t_small = rounds((long)((M + 127) / 128) * ((b_rows + 127) / 128), 2L * n_cu) * small;
  return std::min(t_big, std::min(t_tall, t_small));
}

// What the co-scheduled schedule would do with a planned step, and what it is expected to gain.
struct CoPlan {
  GemmArgs ga[3];   // output projection, gate/up, down of the prefill rows
  int order[3] = {0, 1, 2};  // the carrying launches in the order of their launch, as indices into ga
  int n_carriers = 0, head[3] = {0, 0, 0}, margin[3] = {0, 0, 0}, n_first = 0;
  int64_t first_bytes = 0;
  double gain_s = 0.0;  // estimated time of the serial schedule minus that of this one
};

// `down_first`: the schedule of a layer after the first in a pipelined chain of layers, where the down
// projection of the previous layer's prefill rows is the first launch that carries this layer's queue.
void plan_coscheduled(bs_ctx *c, const Plan &p, const bs_weights *w, const uint16_t *x, uint16_t *y, CoPlan &cp,
                      bool down_first = false) {
  const bs_layer_cfg &g = c->cfg;
  const bs_overlap_knobs &k = c->ov;
  const int T = p.n_rows, Tp = p.n_prefill_rows;
  const bool carry_down = k.carry_down != 0 || down_first;
  const int n_carriers = carry_down ? 3 : 2;
  cp.n_carriers = n_carriers;
  if (down_first) { cp.order[0] = 2; cp.order[1] = 0; cp.order[2] = 1; }
  GemmArgs (&ga)[3] = cp.ga;
  int (&head)[3] = cp.head;
  int (&margin)[3] = cp.margin;
  double carriers_s = 0.0;

  // The carrying launches: for each, the tile shape and the number of CUs that go to attention for
  // its whole duration.  Measured on MI355X: a CU reads 36 GB/s of KV pages whatever its
  // neighbours do, while the whole chip reads 5.3 TB/s (20.7 GB/s per CU), so a CU that streams
  // pages beside a GEMM shortens the step's attention time by more than it lengthens the GEMM, as
  // long as the tiles still fill whole rounds on the CUs that remain: the choice minimises
  //   rounds(tiles, CUs - head) * tile time  -  head * 36 GB/s * that time / 5.3 TB/s
  // over both tile shapes and head = head_cus_min, +8, ... (a 256x256 tile sustains 5.8 TFLOP/s
  // per CU, a 160x256 tile 4.5), never hiding more than the queue still holds.
  ga[0] = o_proj_args(c, w, x, 0, Tp); ga[1] = gate_up_args(c, w, 0, Tp); ga[2] = down_args(c, w, y, 0, Tp);
  const int epi[3] = {EPI_RESID_NORM, EPI_SWIGLU, EPI_RESID};
  const size_t per_token = (size_t)2 * g.head_dim * 2 * g.n_kv_heads;
  int64_t narrow_bytes = 0;
  for (const DecodeItem &it : c->items) narrow_bytes += (int64_t)it.n_tokens * per_token;
  const double cu_stream = 36e9, chip_stream = 5.3e12;
  double ride_bytes = 0;
  double left = k.ride_percent >= 0 ? narrow_bytes * (k.ride_percent / 100.0) : (double)narrow_bytes;
  for (int i = 0; i < n_carriers; ++i) {
    const int l = cp.order[i];
    double best = 1e300, best_hidden = 0, best_t = 0;
    for (int v = 1; v <= 2; ++v) {  // 256x256, 160x256
      ga[l].tile_variant = v;
      const long tiles = gemm_ride_tiles(ga[l], epi[l]);
      const double tile_s = 2.0 * (v == 1 ? 256 : 160) * 256 * ga[l].K / (v == 1 ? 5.8e12 : 4.5e12);
      for (int h = k.head_cus_min; h <= std::max(k.head_cus_min, k.head_cus_max); h += 8) {
        const long cus = c->n_cu - h;
        if (cus < 8) break;
        const double t = (double)((tiles + cus - 1) / cus) * tile_s;
        const double hidden = std::min(left, h * cu_stream * t);
        const double net = t - hidden / chip_stream;
        if (net < best) { best = net; best_hidden = hidden; best_t = t; head[l] = h; margin[l] = v; }
      }
    }
    ga[l].tile_variant = margin[l];
    left -= best_hidden;
    ride_bytes += best_hidden;
    carriers_s += best_t;
    // When to stop handing out units.  Tiles of one round end within a few microseconds of each
    // other, and a unit once begun is finished: where the last round is (nearly) full, the queue
    // closes as soon as the first tile of that round is done, so the workgroups behind the tiles
    // find it closed; where the last round leaves CUs idle, those workgroups work on them until
    // all but close_margin tiles are done.
    const long tiles = gemm_ride_tiles(ga[l], epi[l]);
    const long cus = c->n_cu - head[l];
    const long in_last = tiles - (tiles - 1) / cus * cus;
    margin[l] = 4 * in_last >= 3 * cus ? (int)in_last - 1 : k.close_margin;
  }

  // The 16-row units are sorted longest first; the first attention launch takes the long ones and
  // the queue what the carrying launches are expected to hide.
  int n_first = 0;
  int64_t first_bytes = 0;
  while (n_first < p.n_narrow && (double)(narrow_bytes - first_bytes) > ride_bytes) {
    first_bytes += (int64_t)c->items[n_first].n_tokens * per_token;
    ++n_first;
  }
  cp.n_first = n_first;
  cp.first_bytes = first_bytes;
  // Serial: the three GEMMs over all rows and every 16-row unit on the whole chip.  Co-scheduled: the
  // carrying launches, the decode rows' GEMMs after them, the units that do not ride on the whole chip,
  // and about 30 us for the extra launches and the units that outlast their tiles.
  const int hd = g.n_q_heads * g.head_dim, dm = g.d_model, f = g.d_ffn, n_cu = c->n_cu;
  double serial_s = est_gemm_s(T, dm, hd, n_cu) + est_gemm_s(T, 2 * f, dm, n_cu) + (double)narrow_bytes / chip_stream;
  double co_s = carriers_s + est_gemm_s(T - Tp, dm, hd, n_cu) + est_gemm_s(T - Tp, 2 * f, dm, n_cu) +
                ((double)narrow_bytes - ride_bytes) / chip_stream + 30e-6;
  if (carry_down) {
    serial_s += est_gemm_s(T, dm, f, n_cu);
    co_s += est_gemm_s(T - Tp, dm, f, n_cu);
  }
  cp.gain_s = serial_s - co_s;
}

int run_coscheduled(bs_ctx *c, const Plan &p, const bs_weights *w, const uint16_t *x, uint16_t *y, uint16_t *pool,
                    hipStream_t st, CoPlan &cp) {
  int rc;
  const bs_layer_cfg &g = c->cfg;
  const bs_overlap_knobs &k = c->ov;
  const int T = p.n_rows, Tp = p.n_prefill_rows, d = g.d_model;
  const DecodeArgs dargs = decode_args(c, p, c->qbuf, pool);
  const bool carry_down = k.carry_down != 0;
  const int n_carriers = cp.n_carriers, n_first = cp.n_first;
  GemmArgs (&ga)[3] = cp.ga;
  const int (&head)[3] = cp.head;
  const int (&margin)[3] = cp.margin;
  const int epi[3] = {EPI_RESID_NORM, EPI_SWIGLU, EPI_RESID};
  const int kclass[3] = {BS_K_GEMM_O, BS_K_GEMM_GATE_UP, BS_K_GEMM_DOWN};
  c->ov_first_bytes = cp.first_bytes;
  c->ov_first_items = n_first;

  // attention of the prefill rows, of the wide decode items and of the 16-row units that do not ride
  if ((p.n_wide > 0 || n_first > 0) && p.n_pf_work > 0 && blended_attn_possible(attn_shape(c))) {
    const PrefillArgs pf = prefill_args(c, p, c->qbuf, c->attn, pool);
    SPAN(c, BS_K_ATTN_DECODE, st, HIP_TRY(c, launch_blended_attn(dargs, p.n_wide, n_first, pf, st)));
  } else {
    if ((rc = run_prefill_attn(c, p, c->qbuf, c->attn, pool, st))) return rc;
    if (p.n_wide > 0 || n_first > 0)
      SPAN(c, BS_K_ATTN_DECODE, st, HIP_TRY(c, launch_decode_attn(dargs, p.n_wide, n_first, st)));
  }

  GemmRide ride{};
  ride.q.d = dargs;
  ride.q.first_item = p.n_wide + n_first;
  ride.q.n_units = (p.n_narrow - n_first) * g.n_kv_heads;
  ride.q.waves = k.attention_waves;
  if (c->trace_buf) HIP_TRY(c, hipMemsetAsync(c->trace_buf, 0, sizeof(uint64_t) * 4 * TRACE_CAP * 8 * TRACE_WORDS, st));
  // timeline records of launch l (grid of `wgs` workgroups), if a timeline is being taken and the grid fits
  auto trace_of = [&](int l, long wgs) -> uint64_t * {
    c->trace_wgs[l] = (c->trace_buf && wgs <= TRACE_CAP) ? wgs : 0;
    return c->trace_wgs[l] ? c->trace_buf + (size_t)l * TRACE_CAP * 8 * TRACE_WORDS : nullptr;
  };
  for (long &n : c->trace_wgs) n = 0;
  for (int l = 0; l < n_carriers; ++l) {
    const bool last = l == n_carriers - 1;
    ride.head = head[l];
    ride.tail = k.tail_workgroups;
    // the last carrying launch never closes the queue when it is to drain it: its attention
    // workgroups (at least eight behind the tiles) then go on until the queue is empty
    ride.close_margin = (last && k.drain_in_last) ? -1 : margin[l];
    if (last && k.drain_in_last) ride.tail = std::max(ride.tail, c->n_cu - ride.head);
    ride.q.ticket = c->sync_words + l;
    ride.ticket_next = c->sync_words + l + 1;
    ride.done = c->sync_words + 4 + l;
    ride.closed_at = c->sync_words + 8 + l;
    ride.q.trace = trace_of(l, ride.head + ride.tail + gemm_ride_tiles(ga[l], epi[l]));
    if (l == 0) {
      const int parts = gemm_ss_parts(ga[0], EPI_RESID_NORM, g.head_dim);
      SPAN(c, kclass[0], st, {
        HIP_TRY(c, launch_gemm_with_attention(ga[0], epi[0], g.head_dim, ride, st));
        HIP_TRY(c, launch_rstd_finalize(c->ss2, parts, c->cap_rows, c->rstd2, Tp, d, g.rms_eps, st));
      });
    } else {
      SPAN(c, kclass[l], st, HIP_TRY(c, launch_gemm_with_attention(ga[l], epi[l], g.head_dim, ride, st)));
    }
  }
  if (!k.drain_in_last) {  // what the carrying launches left of the queue, on the whole chip
    DecodeQueue rest = ride.q;
    rest.ticket = c->sync_words + n_carriers;
    rest.trace = trace_of(3, c->n_cu);
    SPAN(c, BS_K_ATTN_QUEUE_REST, st, HIP_TRY(c, launch_decode_queue(rest, c->n_cu, st)));
  }
  if ((rc = run_decode_merge(c, p, c->attn, st))) return rc;
  if ((rc = run_o_gate_up(c, w, x, Tp, T, st, BS_K_GEMM_DECODE_ROWS, BS_K_GEMM_DECODE_ROWS))) return rc;
  if (carry_down) return run_down(c, w, y, Tp, T, st, BS_K_GEMM_DECODE_ROWS);
  return run_down(c, w, y, 0, T, st);
}

int check_cfg(const bs_layer_cfg *g) {
  if (!g) return fail(nullptr, BS_EINVAL, "cfg is NULL");
  if (g->page_size != 16) return fail(nullptr, BS_EUNSUPPORTED, "page_size %d (only 16)", g->page_size);
  if (g->head_dim != 64 && g->head_dim != 128) return fail(nullptr, BS_EUNSUPPORTED, "head_dim %d (64 or 128)", g->head_dim);
  if (g->n_kv_heads < 1 || g->n_q_heads < 1 || g->n_q_heads % g->n_kv_heads || g->n_q_heads / g->n_kv_heads > 16)
    return fail(nullptr, BS_EUNSUPPORTED, "heads %d/%d", g->n_q_heads, g->n_kv_heads);
  if (g->d_model < 8 || g->d_model % 8 || g->d_ffn < 8 || g->d_ffn % 8)
    return fail(nullptr, BS_EUNSUPPORTED, "d_model %d and d_ffn %d must be multiples of 8", g->d_model, g->d_ffn);
  if (!(g->rms_eps >= 0.f) || !(g->rope_theta > 0.f)) return fail(nullptr, BS_EINVAL, "bad rms_eps or rope_theta");
  return BS_OK;
}

}  // namespace

extern "C" {

int bs_create(const bs_layer_cfg *cfg, int device, bs_ctx **out) {
  if (!out) return fail(nullptr, BS_EINVAL, "out is NULL");
  *out = nullptr;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  int n_dev = 0;
  if (device != BS_DEVICE_NONE && (hipGetDeviceCount(&n_dev) != hipSuccess || device < 0 || device >= n_dev))
    return fail(nullptr, BS_EHIP, "device %d not available (%d visible)", device, n_dev);
  bs_ctx *c = new (std::nothrow) bs_ctx();
  if (!c) return fail(nullptr, BS_ENOMEM, "out of host memory");
  c->cfg = *cfg;
  if (c->cfg.max_positions <= 0) c->cfg.max_positions = 16384;
  c->device = device;
  if (device == BS_DEVICE_NONE) { *out = c; return BS_OK; }  // host-only: validation and indexing
  auto bail = [&](int code) { g_create_error = c->err; bs_destroy(c); return code; };
  if (hipSetDevice(device) != hipSuccess) { c->err = "hipSetDevice failed"; return bail(BS_EHIP); }
  const int half = c->cfg.head_dim / 2;
  if ((rc = dev_alloc(c, &c->rope_cos, (size_t)c->cfg.max_positions * half))) return bail(rc);
  if ((rc = dev_alloc(c, &c->rope_sin, (size_t)c->cfg.max_positions * half))) return bail(rc);
  hipError_t e = launch_rope_table(c->rope_cos, c->rope_sin, c->cfg.max_positions, half, (double)c->cfg.rope_theta, nullptr);
  if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
  if (e != hipSuccess) { c->err = std::string("rope table: ") + hipGetErrorString(e); return bail(BS_EHIP); }
  for (int i = 0; i < RING; ++i)
    if (hipEventCreateWithFlags(&c->h_ev[i], hipEventDisableTiming) != hipSuccess) { c->err = "hipEventCreate failed"; return bail(BS_EHIP); }
  {  // this device's copy of the static scratch array (each GPU holds its own, at its own address)
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (device < MAX_DEVICES && !g_scratch_ptr[device]) {
      void *ptr = nullptr;
      const hipError_t es = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
      if (es != hipSuccess || !ptr) { c->err = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(es); return bail(BS_EHIP); }
      g_scratch_ptr[device] = static_cast<unsigned char *>(ptr);
    }
    c->scratch_ptr = device < MAX_DEVICES ? g_scratch_ptr[device] : nullptr;
  }
  // pinned staging for descriptors up to the size bs_attention_noalloc accepts, and host vectors that
  // such a call then never has to grow
  for (int i = 0; i < RING; ++i)
    if ((rc = ensure_blob_host(c, BS_NOALLOC_BLOB_BYTES / sizeof(int32_t), i))) return bail(rc);
  try {
    c->blob.reserve(BS_NOALLOC_BLOB_BYTES / sizeof(int32_t));
    c->items.reserve(BS_NOALLOC_BLOB_BYTES / sizeof(DecodeItem));
    c->items_wide.reserve(BS_NOALLOC_BLOB_BYTES / sizeof(DecodeItem));
    c->pf_order.reserve(1 << 15);
    c->pf_work.reserve(1 << 16);
    c->refcount.reserve(1 << 20);
    c->path_pages.reserve(1 << 15); c->path_chunks.reserve(1 << 15); c->members.reserve(1 << 15);
  } catch (const std::bad_alloc &) { c->err = "out of host memory"; return bail(BS_ENOMEM); }
  if ((rc = dev_alloc(c, &c->sync_words, 16))) return bail(rc);
  if (hipMemset(c->sync_words, 0, 16 * sizeof(unsigned)) != hipSuccess) { c->err = "hipMemset failed"; return bail(BS_EHIP); }
  if ((rc = dev_alloc(c, &c->sk_ws, gemm_sk_workspace_floats()))) return bail(rc);
  if ((rc = dev_alloc(c, &c->sk_cnt, (size_t)gemm_sk_counters()))) return bail(rc);
  if (hipMemset(c->sk_cnt, 0, gemm_sk_counters() * sizeof(unsigned)) != hipSuccess) { c->err = "hipMemset failed"; return bail(BS_EHIP); }
  {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) { c->err = "hipGetDeviceProperties failed"; return bail(BS_EHIP); }
    c->n_cu = prop.multiProcessorCount;
  }
  *out = c;
  return BS_OK;
}

void bs_destroy(bs_ctx *c) {
  if (!c) return;
  if (c->device == BS_DEVICE_NONE) { delete c; return; }
  (void)hipSetDevice(c->device);
  (void)hipDeviceSynchronize();
  for (void *p : {(void *)c->rope_cos, (void *)c->rope_sin, (void *)c->xg, (void *)c->qbuf, (void *)c->attn, (void *)c->x1,
                  (void *)c->xg2, (void *)c->act, (void *)c->rstd1, (void *)c->rstd2, (void *)c->ss2, (void *)c->part_acc, (void *)c->part_m,
                  (void *)c->part_l, (void *)c->d_blob, (void *)c->splitk_ws, (void *)c->hid[0], (void *)c->hid[1], (void *)c->sync_words, (void *)c->trace_buf, (void *)c->sk_ws, (void *)c->sk_cnt})
    if (p) (void)hipFree(p);
  for (int i = 0; i < RING; ++i) {
    if (c->h_blob[i]) (void)hipHostFree(c->h_blob[i]);
    (void)hipEventDestroy(c->h_ev[i]);
  }
  for (auto &v : c->spans) for (auto &s : v) { (void)hipEventDestroy(s.a); (void)hipEventDestroy(s.b); }
  for (auto e : c->free_events) (void)hipEventDestroy(e);
  delete c;
}

const char *bs_last_error(const bs_ctx *c) { return c ? c->err.c_str() : g_create_error.c_str(); }

int64_t bs_kv_page_bytes(const bs_ctx *c) {
  return c ? (int64_t)2 * c->cfg.n_kv_heads * c->cfg.page_size * c->cfg.head_dim * 2 : 0;
}

int bs_kv_pack(bs_ctx *c, const void *k, const void *v, void *pool, int64_t n_pages, void *stream) {
  return guarded(c, [&]() -> int {
  if (!c) return BS_EINVAL;
  if (c->device == BS_DEVICE_NONE) return fail(c, BS_EINVAL, "host-only context");
  if (!k || !v || !pool || n_pages < 0) return fail(c, BS_EINVAL, "bs_kv_pack: bad argument");
  HIP_TRY(c, launch_kv_pack((const uint16_t *)k, (const uint16_t *)v, (uint16_t *)pool, n_pages, c->cfg.n_kv_heads, c->cfg.head_dim, (hipStream_t)stream));
  return BS_OK;
  });
}

int bs_kv_unpack(bs_ctx *c, const void *pool, void *k, void *v, int64_t n_pages, void *stream) {
  return guarded(c, [&]() -> int {
  if (!c) return BS_EINVAL;
  if (c->device == BS_DEVICE_NONE) return fail(c, BS_EINVAL, "host-only context");
  if (!k || !v || !pool || n_pages < 0) return fail(c, BS_EINVAL, "bs_kv_unpack: bad argument");
  HIP_TRY(c, launch_kv_unpack((const uint16_t *)pool, (uint16_t *)k, (uint16_t *)v, n_pages, c->cfg.n_kv_heads, c->cfg.head_dim, (hipStream_t)stream));
  return BS_OK;
  });
}

int bs_validate_batch(bs_ctx *c, const bs_batch *b, int64_t n_pages) {
  return guarded(c, [&]() -> int {
  if (!c) return BS_EINVAL;
  return validate(c, b, n_pages);
  });
}

int bs_resolve_rows(bs_ctx *c, const bs_batch *b, int32_t *page_out, int32_t *slot_out) {
  return guarded(c, [&]() -> int {
  if (!c) return BS_EINVAL;
  if (!b || !page_out || !slot_out) return fail(c, BS_EINVAL, "bs_resolve_rows: NULL argument");
  // the pool size is not an argument here: take the largest page id named (the arrays it sits in are
  // checked for NULL first; everything else is validate()'s job)
  if (b->n_seq < 0 || b->n_nodes < 0) return fail(c, BS_EINVAL, "bad counts: n_seq=%d n_nodes=%d", b->n_seq, b->n_nodes);
  if (b->n_seq > 0 && (!b->page_start || (!b->page_ids && b->page_start[b->n_seq] > 0)))
    return fail(c, BS_EINVAL, "a required array is NULL");
  if (b->n_nodes > 0 && (!b->node_page_start || (!b->node_page_ids && b->node_page_start[b->n_nodes] > 0)))
    return fail(c, BS_EINVAL, "a node array is NULL");
  int64_t max_page = 0;
  for (int i = 0; b->n_seq > 0 && i < b->page_start[b->n_seq]; ++i) max_page = std::max<int64_t>(max_page, b->page_ids[i]);
  for (int i = 0; b->n_nodes > 0 && i < b->node_page_start[b->n_nodes]; ++i) max_page = std::max<int64_t>(max_page, b->node_page_ids[i]);
  if (max_page >= (int64_t)0x7fffffff) return fail(c, BS_EINVAL, "page id out of range");
  int rc = validate(c, b, max_page + 1);
  if (rc) return rc;
  Plan p;
  if ((rc = build_plan(c, b, p, true))) return rc;
  for (int r = 0; r < b->n_rows; ++r) {
    page_out[r] = c->blob[p.off_row_page + r];
    slot_out[r] = c->blob[p.off_row_slot + r];
  }
  return BS_OK;
  });
}

}  // extern "C"

namespace {

// First norm and fused QKV projection (RoPE, KV append into `pool`) of rows [r0, r1) of x.
// `clear_sync`: the prep kernel also clears the counters of the co-scheduled launches.
int run_prep_qkv(bs_ctx *c, const Plan &p, const bs_weights *w, const uint16_t *x, uint16_t *pool, int r0, int r1,
                 bool clear_sync, hipStream_t st) {
  int rc;
  const bs_layer_cfg &g = c->cfg;
  const int d = g.d_model, rows = r1 - r0, hd = g.n_q_heads * g.head_dim;
  if (rows <= 0) return BS_OK;
  SPAN(c, BS_K_PREP, st, HIP_TRY(c, launch_norm_prep(x + (size_t)r0 * d, (const uint16_t *)w->g_attn, c->xg + (size_t)r0 * d,
                                                     c->rstd1 + r0, rows, d, g.rms_eps, clear_sync ? c->sync_words : nullptr, 16, st)));
  GemmArgs q{};
  q.A = c->xg + (size_t)r0 * d; q.lda = d; q.B = (const uint16_t *)w->w_qkv; q.ldb = d;
  q.M = rows; q.N = (g.n_q_heads + 2 * g.n_kv_heads) * g.head_dim; q.K = d;
  q.rstd = c->rstd1 + r0;
  q.n_q_heads = g.n_q_heads; q.n_kv_heads = g.n_kv_heads;
  q.rope_cos = c->rope_cos; q.rope_sin = c->rope_sin;
  q.row_pos = c->d_blob + p.off_row_pos + r0; q.row_page = c->d_blob + p.off_row_page + r0; q.row_slot = c->d_blob + p.off_row_slot + r0;
  q.q_out = c->qbuf + (size_t)r0 * hd; q.kv_pool = pool;
  q.sk_ws = c->sk_ws; q.sk_cnt = c->sk_cnt;
  q.k_splits = gemm_splitk_choice(q.M, q.N, q.K, EPI_QKV, 0);
  if (q.k_splits > 1) {
    if ((rc = ensure_splitk(c, (size_t)q.k_splits * q.M * q.N))) return rc;
    q.splitk_ws = c->splitk_ws;
  }
  SPAN(c, BS_K_GEMM_QKV, st, HIP_TRY(c, launch_gemm(q, EPI_QKV, g.head_dim, st)));
  return BS_OK;
}

// every kernel of one layer for the planned batch: x -> y, appending to `pool`
int run_layer(bs_ctx *c, const Plan &p, const bs_weights *w, const uint16_t *x, uint16_t *y, uint16_t *pool, hipStream_t st,
              uint32_t flags) {
  int rc;
  const int T = p.n_rows;
  if ((rc = run_prep_qkv(c, p, w, x, pool, 0, T, true, st))) return rc;

  // co-scheduling pays where there are GEMM rows that do not wait for decode attention (the
  // prefill rows) and 16-row decode units to run beside them
  // and where its cost model expects the step to come out shorter than the serial one (knob `always`: regardless)
  if ((flags & BS_FLAG_OVERLAP) && p.n_narrow > 0 && p.n_prefill_rows >= c->ov.min_prefill_rows) {
    CoPlan cp;
    plan_coscheduled(c, p, w, x, y, cp);
    if (c->ov.always || cp.gain_s > 0.0) return run_coscheduled(c, p, w, x, y, pool, st, cp);
  }
  if ((rc = run_attention(c, p, c->qbuf, c->attn, pool, st))) return rc;
  if ((rc = run_o_gate_up(c, w, x, 0, T, st))) return rc;
  return run_down(c, w, y, 0, T, st);
}

// Layers back to back with the two parts of the batch one stage apart (BS_FLAG_PIPELINE; Section 2.2,
// nano-batches: operators of different parts of a batch overlap across the layer boundary;
// Appendix A.2).  The decode rows run ahead of the prefill rows: they finish layer l (their output
// projection, FFN) and enter layer l+1 (norm, QKV, KV append) BEFORE the prefill rows' down projection
// of layer l is launched, so that launch, whose tiles leave CUs idle, already carries the decode
// attention of layer l+1 with its whole queue still to draw from; the prefill rows' output projection
// and gate/up of layer l+1 carry the rest, as in a single co-scheduled layer.  The two parts touch
// disjoint rows of every workspace buffer, and a part is never more than one layer ahead, so the two
// alternating hidden-state buffers suffice.  Same kernels, same arithmetic per row as run_layer.
int run_layers_pipelined(bs_ctx *c, const Plan &p, int n_layers, const bs_weights *w, const uint16_t *x, uint16_t *y,
                         void *const *pools, hipStream_t st, CoPlan &first, CoPlan &later) {
  int rc;
  const bs_layer_cfg &g = c->cfg;
  const bs_overlap_knobs &k = c->ov;
  const int T = p.n_rows, Tp = p.n_prefill_rows, d = g.d_model;
  const int epi[3] = {EPI_RESID_NORM, EPI_SWIGLU, EPI_RESID};
  const int kclass[3] = {BS_K_GEMM_O, BS_K_GEMM_GATE_UP, BS_K_GEMM_DOWN};
  for (long &n : c->trace_wgs) n = 0;

  // launch number `slot` of a layer's carrying launches: GEMM `gi` of `cp` with arguments `a`
  auto carry = [&](const CoPlan &cp, int slot, int gi, GemmArgs a, const DecodeArgs &dargs, bool last) -> int {
    GemmRide ride{};
    ride.q.d = dargs;
    ride.q.first_item = p.n_wide + cp.n_first;
    ride.q.n_units = (p.n_narrow - cp.n_first) * g.n_kv_heads;
    ride.q.waves = k.attention_waves;
    ride.head = cp.head[gi];
    ride.tail = last ? std::max(k.tail_workgroups, c->n_cu - ride.head) : k.tail_workgroups;
    ride.close_margin = last ? -1 : cp.margin[gi];  // the last carrying launch of a layer drains the queue
    ride.q.ticket = c->sync_words + slot;
    ride.ticket_next = c->sync_words + slot + 1;
    ride.done = c->sync_words + 4 + slot;
    ride.closed_at = c->sync_words + 8 + slot;
    a.tile_variant = cp.ga[gi].tile_variant;
    if (gi == 0) {
      const int parts = gemm_ss_parts(a, EPI_RESID_NORM, g.head_dim);
      SPAN(c, kclass[0], st, {
        HIP_TRY(c, launch_gemm_with_attention(a, epi[0], g.head_dim, ride, st));
        HIP_TRY(c, launch_rstd_finalize(c->ss2, parts, c->cap_rows, c->rstd2, Tp, d, g.rms_eps, st));
      });
    } else {
      SPAN(c, kclass[gi], st, HIP_TRY(c, launch_gemm_with_attention(a, epi[gi], g.head_dim, ride, st)));
    }
    return BS_OK;
  };

  const uint16_t *in = x;
  if ((rc = run_prep_qkv(c, p, &w[0], in, (uint16_t *)pools[0], 0, T, true, st))) return rc;
  for (int l = 0; l < n_layers; ++l) {
    const CoPlan &cp = l == 0 ? first : later;
    uint16_t *out = (l == n_layers - 1) ? y : c->hid[l & 1];
    uint16_t *pool = (uint16_t *)pools[l];
    const DecodeArgs dargs = decode_args(c, p, c->qbuf, pool);
    c->ov_first_bytes = cp.first_bytes;
    c->ov_first_items = cp.n_first;
    // attention of the prefill rows, of the wide decode items and of the 16-row units that do not ride
    if ((p.n_wide > 0 || cp.n_first > 0) && p.n_pf_work > 0 && blended_attn_possible(attn_shape(c))) {
      const PrefillArgs pf = prefill_args(c, p, c->qbuf, c->attn, pool);
      SPAN(c, BS_K_ATTN_DECODE, st, HIP_TRY(c, launch_blended_attn(dargs, p.n_wide, cp.n_first, pf, st)));
    } else {
      if ((rc = run_prefill_attn(c, p, c->qbuf, c->attn, pool, st))) return rc;
      if (p.n_wide > 0 || cp.n_first > 0)
        SPAN(c, BS_K_ATTN_DECODE, st, HIP_TRY(c, launch_decode_attn(dargs, p.n_wide, cp.n_first, st)));
    }
    // (in a later layer launch 0 was the previous layer's down projection)
    const int s0 = l == 0 ? 0 : 1;
    if ((rc = carry(cp, s0, 0, o_proj_args(c, &w[l], in, 0, Tp), dargs, false))) return rc;
    if ((rc = carry(cp, s0 + 1, 1, gate_up_args(c, &w[l], 0, Tp), dargs, true))) return rc;
    if ((rc = run_decode_merge(c, p, c->attn, st))) return rc;
    if ((rc = run_o_gate_up(c, &w[l], in, Tp, T, st, BS_K_GEMM_DECODE_ROWS, BS_K_GEMM_DECODE_ROWS))) return rc;
    if (l == n_layers - 1) return run_down(c, &w[l], out, 0, T, st);
    // the decode rows leave this layer and enter the next ...
    if ((rc = run_down(c, &w[l], out, Tp, T, st, BS_K_GEMM_DECODE_ROWS))) return rc;
    if ((rc = run_prep_qkv(c, p, &w[l + 1], out, (uint16_t *)pools[l + 1], Tp, T, true, st))) return rc;
    // ... whose attention starts beside the prefill rows' down projection of this one
    const DecodeArgs next = decode_args(c, p, c->qbuf, (uint16_t *)pools[l + 1]);
    if ((rc = carry(later, 0, 2, down_args(c, &w[l], out, 0, Tp), next, false))) return rc;
    if ((rc = run_prep_qkv(c, p, &w[l + 1], out, (uint16_t *)pools[l + 1], 0, Tp, false, st))) return rc;
    in = out;
  }
  return BS_OK;
}

bool weights_ok(const bs_weights *w) {
  return w && w->w_qkv && w->w_o && w->w_gate_up && w->w_down && w->g_attn && w->g_ffn;
}

}  // namespace

extern "C" {

int bs_blend_step(bs_ctx *c, const bs_weights *w, const bs_batch *b, const void *x_, void *y_, void *pool_,
                  int64_t n_pages, void *stream_, uint32_t flags) {
  return guarded(c, [&]() -> int {
  if (!c) return BS_EINVAL;
  if (c->device == BS_DEVICE_NONE) return fail(c, BS_EINVAL, "host-only context");
  if (!weights_ok(w)) return fail(c, BS_EINVAL, "a weight pointer is NULL");
  int rc = validate(c, b, n_pages);
  if (rc) return rc;
  if (b->n_rows == 0) return BS_OK;
  if (!x_ || !y_ || !pool_ || x_ == y_) return fail(c, BS_EINVAL, "x, y, kv_pool must be distinct non-NULL device pointers");
  HIP_TRY(c, hipSetDevice(c->device));
  gemm_force_variant(c->forced_tiles);
  hipStream_t st = (hipStream_t)stream_;
  Plan p;
  if ((rc = build_plan(c, b, p, true))) return rc;
  if ((rc = ensure_rows(c, p.n_rows))) return rc;
  if ((rc = ensure_slots(c, p.n_slots))) return rc;
  if ((rc = upload_plan(c, p, st))) return rc;
  return run_layer(c, p, w, (const uint16_t *)x_, (uint16_t *)y_, (uint16_t *)pool_, st, flags);
  });
}

int bs_blend_layers(bs_ctx *c, int32_t n_layers, const bs_weights *w, const bs_batch *b, const void *x_, void *y_,
                    void *const *pools, int64_t n_pages, void *stream_, uint32_t flags) {
  return guarded(c, [&]() -> int {
  if (!c) return BS_EINVAL;
  if (c->device == BS_DEVICE_NONE) return fail(c, BS_EINVAL, "host-only context");
  if (n_layers < 1 || !w || !pools) return fail(c, BS_EINVAL, "bs_blend_layers: n_layers %d, weights or pools NULL", n_layers);
  for (int l = 0; l < n_layers; ++l)
    if (!weights_ok(&w[l]) || !pools[l]) return fail(c, BS_EINVAL, "layer %d: a weight or pool pointer is NULL", l);
  int rc = validate(c, b, n_pages);
  if (rc) return rc;
  if (b->n_rows == 0) return BS_OK;
  if (!x_ || !y_ || x_ == y_) return fail(c, BS_EINVAL, "x and y must be distinct non-NULL device pointers");
  HIP_TRY(c, hipSetDevice(c->device));
  gemm_force_variant(c->forced_tiles);
  hipStream_t st = (hipStream_t)stream_;
  Plan p;
  if ((rc = build_plan(c, b, p, true))) return rc;
  if ((rc = ensure_rows(c, p.n_rows))) return rc;
  if ((rc = ensure_slots(c, p.n_slots))) return rc;
  if ((rc = upload_plan(c, p, st))) return rc;
  // one descriptor, validated, planned and uploaded once; activations alternate between two
  // workspace buffers so that neither x nor y is touched before / after its own layer
  const uint16_t *in = (const uint16_t *)x_;
  if ((flags & BS_FLAG_OVERLAP) && (flags & BS_FLAG_PIPELINE) && n_layers > 1 && p.n_narrow > 0 &&
      p.n_prefill_rows >= c->ov.min_prefill_rows && p.n_prefill_rows < p.n_rows) {
    CoPlan first, later;
    plan_coscheduled(c, p, &w[0], in, (uint16_t *)y_, first);
    plan_coscheduled(c, p, &w[0], in, (uint16_t *)y_, later, true);
    if (c->ov.always || first.gain_s > 0.0)
      return run_layers_pipelined(c, p, n_layers, w, in, (uint16_t *)y_, pools, st, first, later);
  }
  for (int l = 0; l < n_layers; ++l) {
    uint16_t *out = (l == n_layers - 1) ? (uint16_t *)y_ : c->hid[l & 1];
    if ((rc = run_layer(c, p, &w[l], in, out, (uint16_t *)pools[l], st, flags))) return rc;
    in = out;
  }
  return BS_OK;
  });
}

int bs_attention(bs_ctx *c, const bs_batch *b, const void *q, void *out, const void *pool, int64_t n_pages,
                 void *stream_, uint32_t flags) {
  return guarded(c, [&]() -> int {
  (void)flags;
  if (!c) return BS_EINVAL;
  if (c->device == BS_DEVICE_NONE) return fail(c, BS_EINVAL, "host-only context");
  int rc = validate(c, b, n_pages);
  if (rc) return rc;
  if (b->n_rows == 0) return BS_OK;
  if (!q || !out || !pool) return fail(c, BS_EINVAL, "bs_attention: NULL pointer");
  HIP_TRY(c, hipSetDevice(c->device));
  hipStream_t st = (hipStream_t)stream_;
  Plan p;
  if ((rc = build_plan(c, b, p, false))) return rc;
  if ((rc = ensure_slots(c, p.n_slots))) return rc;
  if ((rc = upload_plan(c, p, st))) return rc;
  if ((rc = run_attention(c, p, (const uint16_t *)q, (uint16_t *)out, (const uint16_t *)pool, st))) return rc;
  return BS_OK;
  });
}

int bs_attention_noalloc(bs_ctx *c, const bs_batch *b, const void *q, void *out, const void *pool, int64_t n_pages,
                         void *stream_) {
  return guarded(c, [&]() -> int {
  if (!c) return BS_EINVAL;
  if (c->device == BS_DEVICE_NONE) return fail(c, BS_EINVAL, "host-only context");
  if (!c->scratch_ptr) return fail(c, BS_EHIP, "bs_attention_noalloc: no scratch array on device %d", c->device);
  if (n_pages > (1 << 20)) return fail(c, BS_EINVAL, "bs_attention_noalloc: n_pages %lld exceeds the limit of %d", (long long)n_pages, 1 << 20);
  if (b && ((long)b->n_seq > (1 << 15) || (long)b->n_nodes > (1 << 15) || (long)b->n_rows > (1 << 20)))
    return fail(c, BS_EINVAL, "bs_attention_noalloc: more than %d sequences or prefix nodes", 1 << 15);
  int rc = validate(c, b, n_pages);
  if (rc) return rc;
  if (b->n_rows == 0) return BS_OK;
  if (!q || !out || !pool) return fail(c, BS_EINVAL, "bs_attention_noalloc: NULL pointer");
  HIP_TRY(c, hipSetDevice(c->device));
  hipStream_t st = (hipStream_t)stream_;
  Plan p;
  if ((rc = build_plan(c, b, p, false))) return rc;
  // layout of the scratch array: descriptor blob | m | l | acc of the partial states (m and l padded
  // to whole 16-byte units, so that the accumulators after them stay 16-byte aligned)
  const size_t hq = c->cfg.n_q_heads, dh = c->cfg.head_dim;
  const size_t ml_floats = ((size_t)p.n_slots * hq + 3) / 4 * 4;
  const size_t state_bytes = (2 * ml_floats + (size_t)p.n_slots * hq * dh) * sizeof(float);
  if ((size_t)p.total_ints * sizeof(int32_t) > BS_NOALLOC_BLOB_BYTES)
    return fail(c, BS_EINVAL, "bs_attention_noalloc: descriptor of %ld bytes exceeds the limit of %u", p.total_ints * 4L, BS_NOALLOC_BLOB_BYTES);
  if (state_bytes > BS_NOALLOC_SCRATCH_BYTES - BS_NOALLOC_BLOB_BYTES)
    return fail(c, BS_EINVAL, "bs_attention_noalloc: %ld partial softmax states (%zu bytes) exceed the limit of %u bytes",
                p.n_slots, state_bytes, BS_NOALLOC_SCRATCH_BYTES - BS_NOALLOC_BLOB_BYTES);
  // the kernels take their buffers from the context; for this call they are parts of the scratch array
  int32_t *const blob0 = c->d_blob;
  float *const acc0 = c->part_acc, *const m0 = c->part_m, *const l0 = c->part_l;
  unsigned char *ptr = c->scratch_ptr;
  c->d_blob = reinterpret_cast<int32_t *>(ptr);
  c->part_m = reinterpret_cast<float *>(ptr + BS_NOALLOC_BLOB_BYTES);
  c->part_l = c->part_m + ml_floats;
  c->part_acc = c->part_l + ml_floats;
  rc = upload_plan(c, p, st, c->d_blob, true);
  if (!rc) rc = run_attention(c, p, (const uint16_t *)q, (uint16_t *)out, (const uint16_t *)pool, st);
  c->d_blob = blob0;
  c->part_acc = acc0; c->part_m = m0; c->part_l = l0;
  return rc;
  });
}

int bs_gemm_nt(bs_ctx *c, const void *a, const void *b, void *out, int32_t m, int32_t n, int32_t k, void *stream) {
  return guarded(c, [&]() -> int {
  if (!c) return BS_EINVAL;
  if (c->device == BS_DEVICE_NONE) return fail(c, BS_EINVAL, "host-only context");
  if (m < 0 || n < 0 || k < 0 || (k % 8) || (n % 8)) return fail(c, BS_EINVAL, "bs_gemm_nt: m=%d n=%d k=%d (n, k multiples of 8)", m, n, k);
  if (m == 0 || n == 0) return BS_OK;
  if (!a || !b || !out) return fail(c, BS_EINVAL, "bs_gemm_nt: NULL pointer");
  HIP_TRY(c, hipSetDevice(c->device));
  gemm_force_variant(c->forced_tiles);
  GemmArgs g{};
  g.A = (const uint16_t *)a; g.lda = k; g.B = (const uint16_t *)b; g.ldb = k;
  g.M = m; g.N = n; g.K = k; g.C = (uint16_t *)out; g.ldc = n;
  g.sk_ws = c->sk_ws; g.sk_cnt = c->sk_cnt;
  HIP_TRY(c, launch_gemm(g, EPI_PLAIN, c->cfg.head_dim, (hipStream_t)stream));
  return BS_OK;
  });
}

int bs_profile_enable(bs_ctx *c, int on) {
  if (!c) return BS_EINVAL;
  c->prof = on != 0;
  return BS_OK;
}

int bs_profile_reset(bs_ctx *c) {
  return guarded(c, [&]() -> int {
  if (!c) return BS_EINVAL;
  for (int k = 0; k < BS_K_COUNT; ++k) {
    for (auto &s : c->spans[k]) {
      (void)hipEventSynchronize(s.b);
      c->free_events.push_back(s.a);
      c->free_events.push_back(s.b);
    }
    c->spans[k].clear();
    c->prof_ms[k] = 0;
    c->prof_n[k] = 0;
  }
  return BS_OK;
  });
}

int bs_profile_read(bs_ctx *c, int which, double *total_ms, int64_t *launches) {
  return guarded(c, [&]() -> int {
  if (!c) return BS_EINVAL;
  if (which < 0 || which >= BS_K_COUNT) return fail(c, BS_EINVAL, "bs_profile_read: class %d", which);
  for (auto &s : c->spans[which]) {
    HIP_TRY(c, hipEventSynchronize(s.b));
    float ms = 0.f;
    HIP_TRY(c, hipEventElapsedTime(&ms, s.a, s.b));
    c->prof_ms[which] += ms;
    c->prof_n[which] += 1;
    c->free_events.push_back(s.a);
    c->free_events.push_back(s.b);
  }
  c->spans[which].clear();
  if (total_ms) *total_ms = c->prof_ms[which];
  if (launches) *launches = c->prof_n[which];
  return BS_OK;
  });
}

int bs_set_gemm_tiles(bs_ctx *c, int32_t variant) {
  if (!c) return BS_EINVAL;
  if (variant < 0 || (variant > 3 && variant != 6)) return fail(c, BS_EINVAL, "gemm tile variant %d (0..3 or 6)", variant);
  c->forced_tiles = variant;
  return BS_OK;
}

int bs_overlap_trace(bs_ctx *c, int on) {
  return guarded(c, [&]() -> int {
  if (!c) return BS_EINVAL;
  if (c->device == BS_DEVICE_NONE) return fail(c, BS_EINVAL, "host-only context");
  HIP_TRY(c, hipSetDevice(c->device));
  HIP_TRY(c, hipDeviceSynchronize());
  for (long &n : c->trace_wgs) n = 0;
  if (on && !c->trace_buf) return dev_alloc(c, &c->trace_buf, (size_t)4 * TRACE_CAP * 8 * TRACE_WORDS);
  if (!on && c->trace_buf) return dev_alloc(c, &c->trace_buf, 0);
  return BS_OK;
  });
}

int bs_overlap_trace_read(bs_ctx *c, int32_t launch, uint64_t *out, int64_t cap_records, int64_t *n_records) {
  return guarded(c, [&]() -> int {
  if (!c) return BS_EINVAL;
  if (c->device == BS_DEVICE_NONE) return fail(c, BS_EINVAL, "host-only context");
  if (launch < 0 || launch > 3 || !n_records || cap_records < 0 || (cap_records > 0 && !out))
    return fail(c, BS_EINVAL, "bs_overlap_trace_read: bad argument");
  const int64_t n = c->trace_buf ? c->trace_wgs[launch] * 8 : 0;
  *n_records = n;
  if (n == 0 || cap_records == 0) return BS_OK;
  HIP_TRY(c, hipSetDevice(c->device));
  HIP_TRY(c, hipDeviceSynchronize());
  HIP_TRY(c, hipMemcpy(out, c->trace_buf + (size_t)launch * TRACE_CAP * 8 * TRACE_WORDS,
                       sizeof(uint64_t) * TRACE_WORDS * (size_t)std::min(n, cap_records), hipMemcpyDeviceToHost));
  return BS_OK;
  });
}

int bs_overlap_report(bs_ctx *c, int64_t *kv_bytes) {
  return guarded(c, [&]() -> int {
  if (!c) return BS_EINVAL;
  if (c->device == BS_DEVICE_NONE) return fail(c, BS_EINVAL, "host-only context");
  if (!kv_bytes) return fail(c, BS_EINVAL, "bs_overlap_report: NULL argument");
  HIP_TRY(c, hipSetDevice(c->device));
  HIP_TRY(c, hipDeviceSynchronize());
  unsigned words[16];
  HIP_TRY(c, hipMemcpy(words, c->sync_words, sizeof words, hipMemcpyDeviceToHost));
  const int hkv = c->cfg.n_kv_heads;
  const long first = (long)c->ov_first_items * hkv;
  const long n_units = (long)c->items.size() * hkv - first;
  // the queue positions at which the carrying launches closed; a launch that did not close (the one
  // that drains the queue, or a launch that did not run) took everything that was left
  long pos[5] = {0, n_units, n_units, n_units, n_units};
  for (int l = 1; l <= 3; ++l)
    if (words[l - 1] >= DECODE_QUEUE_CLOSED) pos[l] = std::min<long>(words[8 + l - 1], n_units);
  for (int l = 1; l <= 3; ++l) pos[l] = std::max(pos[l], pos[l - 1]);
  const int64_t per_token = (int64_t)2 * c->cfg.head_dim * 2;  // K and V of one token and KV head
  kv_bytes[0] = c->ov_first_bytes;
  for (int l = 0; l < 4; ++l) {
    int64_t tokens = 0;
    for (long u = pos[l]; u < pos[l + 1]; ++u) tokens += c->items[(size_t)((first + u) / hkv)].n_tokens;
    kv_bytes[1 + l] = tokens * per_token;
  }
  return BS_OK;
  });
}

int bs_set_overlap(bs_ctx *c, const bs_overlap_knobs *k) {
  if (!c) return BS_EINVAL;
  if (!k) return fail(c, BS_EINVAL, "bs_set_overlap: NULL argument");
  if (k->head_cus_min < 0 || k->head_cus_min > 192 || k->head_cus_min % 8)
    return fail(c, BS_EINVAL, "head_cus_min %d (a multiple of 8, 0..192)", k->head_cus_min);
  if (k->tail_workgroups < 0 || k->tail_workgroups > 256) return fail(c, BS_EINVAL, "tail_workgroups %d (0..256)", k->tail_workgroups);
  if (k->close_margin < 0 || k->close_margin > 256) return fail(c, BS_EINVAL, "close_margin %d (0..256)", k->close_margin);
  if (k->min_prefill_rows < 1) return fail(c, BS_EINVAL, "min_prefill_rows %d (at least 1)", k->min_prefill_rows);
  if (k->ride_percent < -1 || k->ride_percent > 100) return fail(c, BS_EINVAL, "ride_percent %d (-1 or 0..100)", k->ride_percent);
  if (k->attention_waves < 1 || k->attention_waves > 8) return fail(c, BS_EINVAL, "attention_waves %d (1..8)", k->attention_waves);
  if (k->head_cus_max < 0 || k->head_cus_max > 192 || k->head_cus_max % 8)
    return fail(c, BS_EINVAL, "head_cus_max %d (a multiple of 8, 0..192)", k->head_cus_max);
  c->ov = *k;
  c->ov.carry_down = k->carry_down != 0;
  c->ov.drain_in_last = k->drain_in_last != 0;
  c->ov.always = k->always != 0;
  return BS_OK;
}

int bs_get_overlap(const bs_ctx *c, bs_overlap_knobs *k) {
  if (!c || !k) return BS_EINVAL;
  *k = c->ov;
  return BS_OK;
}

/* Tuning knob used by the benchmark sweeps: pages per decode-attention chunk. */
int bs_set_chunk_pages(bs_ctx *c, int32_t pages) {
  if (!c) return BS_EINVAL;
  if (pages < 2 || pages > 64 || (pages & 1)) return fail(c, BS_EINVAL, "chunk_pages %d (even, 2..64)", pages);
  c->chunk_pages = pages;
  c->chunk_pages_wide = pages;
  return BS_OK;
}

}  // extern "C"
