// Host-side batch builder: resource-aware prefix tree, layer-wise sort, conditional
// node splitting and dual scan of BlendServe (Sections 5.1-5.4, Algorithms 1-3),
// single-step form.
// Plain C++, no GPU calls.  Built with floating-point contraction off: the few
// double-precision expressions are evaluated exactly as written.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <limits>
#include <map>
#include <new>
#include <string>
#include <vector>

#include "../../include/blendstep_builder.h"

namespace {

struct Req {
  std::vector<int32_t> tok;
  int32_t d_est, n_cached;
};

// A trie node while the tree is being grown by insertion.
struct Grow {
  int32_t start = 0, end = 0;        // token depths of the segment
  int32_t owner = -1;                // a request whose prompt spells the segment
  int32_t parent = -1;
  int32_t req = -1;                  // >= 0: a leaf
  std::map<int32_t, int32_t> kids;   // first token of the child's segment -> node
  std::vector<int32_t> ends_here;    // requests whose prompt ends exactly at `end`
};

// The finished tree in DFS pre-order.
struct Node {
  int32_t parent, start, end, req, first_leaf, leaf_count;
  int64_t A, B, n_req, sum_p, sum_d;
  int64_t lo_a, lo_b, hi_a, hi_b;    // (A, B) of the least / most compute-intensive leaf below
  int32_t min_req;
  std::vector<int32_t> kids;
};

}  // namespace

struct bs_builder {
  bs_cost_model cm;
  std::string err;
  std::vector<Req> reqs;
  std::vector<Node> nodes;          // valid after finalize
  std::vector<int32_t> leaf_order;
  std::vector<int32_t> leaf_node;   // request -> node
  std::vector<char> detached;       // request was re-inserted under the root by node splitting
  int mem_model = BS_MEM_EXPANDED;
  bool finalized = false;
};

namespace {

int fail(bs_builder *b, int code, const char *fmt, ...) {
  char buf[400];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (b) b->err = buf;
  return code;
}

// is (A1, B1) strictly more compute-intensive than (A2, B2)?  A/B compared exactly.
int cmp_density(int64_t A1, int64_t B1, int64_t A2, int64_t B2) {
  if (B1 == 0 && B2 == 0) return 0;
  if (B1 == 0) return 1;
  if (B2 == 0) return -1;
  const __int128 l = (__int128)A1 * B2, r = (__int128)A2 * B1;
  return (l > r) - (l < r);
}

double rho_of(const bs_cost_model &cm, int64_t A, int64_t B) {
  if (B == 0) return std::numeric_limits<double>::infinity();
  const double t_comp = (2.0 * (double)cm.p_model) * (double)A / cm.compute;
  const double t_mem = ((double)cm.kv_bytes * (double)B) / (2.0 * cm.bandwidth);
  return t_comp / t_mem;
}

void partition(double rho_rt, double rho_l, double rho_r, double M, double *m_l, double *m_r) {
  const double inf = std::numeric_limits<double>::infinity();
  double ml;
  if (rho_l == rho_r) ml = M;
  else if (rho_l == inf) ml = (rho_rt != inf) ? 0.0 : M;
  else ml = M * ((rho_rt - rho_r) / (rho_l - rho_r));
  ml = std::min(std::max(ml, 0.0), M);
  *m_l = ml;
  *m_r = M - ml;
}

// ---- trie growth: radix insertion ------------------------------------------------------
struct Grower {
  const std::vector<Req> &reqs;
  std::vector<Grow> g;
  explicit Grower(const std::vector<Req> &r) : reqs(r) { g.emplace_back(); }

  int32_t tok_at(const Grow &n, int32_t depth) const { return reqs[n.owner].tok[depth]; }

  void insert(int32_t r) {
    const std::vector<int32_t> &t = reqs[r].tok;
    const int32_t p = (int32_t)t.size();
    int32_t node = 0, depth = 0;
    for (;;) {
      if (g[node].req >= 0) {  // reached a leaf: it becomes an internal node that its request ends at
        g[node].ends_here.push_back(g[node].req);
        g[node].req = -1;
      }
      if (depth == p) { g[node].ends_here.push_back(r); return; }
      auto it = g[node].kids.find(t[depth]);
      if (it == g[node].kids.end()) {
        Grow leaf;
        leaf.start = depth; leaf.end = p; leaf.owner = r; leaf.parent = node; leaf.req = r;
        g.push_back(leaf);
        g[node].kids[t[depth]] = (int32_t)g.size() - 1;
        return;
      }
      const int32_t c = it->second;
      const int32_t len = g[c].end - g[c].start;
      int32_t m = 0;
      while (m < len && depth + m < p && tok_at(g[c], g[c].start + m) == t[depth + m]) ++m;
      if (m == len) { node = c; depth += m; continue; }
      // split c at m: a new internal node takes the matched part
      Grow mid;
      mid.start = g[c].start; mid.end = g[c].start + m; mid.owner = g[c].owner; mid.parent = node;
      g.push_back(mid);
      const int32_t mi = (int32_t)g.size() - 1;
      g[node].kids[t[depth]] = mi;
      g[c].start += m;
      g[c].parent = mi;
      g[mi].kids[tok_at(g[c], g[c].start)] = c;
      node = mi;
      depth += m;
    }
  }
};

struct Tmp {  // unsorted finished tree
  int32_t parent, start, end, req;
  int64_t A = 0, B = 0, n_req = 0, sum_p = 0, sum_d = 0;
  int64_t S = 0, max_d = 0;  // prefix-pages-read-once memory model: loaded tokens (x2) at or below the segment; longest output below
  int64_t lo_a = 0, lo_b = 1, hi_a = 0, hi_b = 1;
  int32_t min_req = 0;
  std::vector<int32_t> kids;
};

// Build the sorted, numbered tree over the requests: the trie of those not detached, the
// detached ones as direct children of the root with their whole prompt as own segment.
void rebuild(bs_builder *b) {
  const int32_t nr = (int32_t)b->reqs.size();
  b->detached.resize(nr, 0);
  Grower gr(b->reqs);
  for (int32_t r = 0; r < nr; ++r)
    if (!b->detached[r]) gr.insert(r);
  // flatten: requests that end at an internal node become leaves with an empty segment
  std::vector<Tmp> t(gr.g.size());
  for (size_t i = 0; i < gr.g.size(); ++i) {
    t[i].parent = gr.g[i].parent; t[i].start = gr.g[i].start; t[i].end = gr.g[i].end; t[i].req = gr.g[i].req;
    for (auto &kv : gr.g[i].kids) t[i].kids.push_back(kv.second);
  }
  for (size_t i = 0; i < gr.g.size(); ++i)
    for (int32_t r : gr.g[i].ends_here) {
      Tmp leaf;
      leaf.parent = (int32_t)i; leaf.start = leaf.end = gr.g[i].end; leaf.req = r;
      t.push_back(leaf);
      t[i].kids.push_back((int32_t)t.size() - 1);
    }
  for (int32_t r = 0; r < nr; ++r)
    if (b->detached[r]) {
      Tmp leaf;
      leaf.parent = 0; leaf.start = 0; leaf.end = (int32_t)b->reqs[r].tok.size(); leaf.req = r;
      t.push_back(leaf);
      t[0].kids.push_back((int32_t)t.size() - 1);
    }
  // bottom-up annotation in reverse creation order is not enough (splits re-parent), so walk explicitly
  std::vector<int32_t> order;  // pre-order
  order.reserve(t.size());
  {
    std::vector<int32_t> st{0};
    while (!st.empty()) {
      const int32_t n = st.back(); st.pop_back();
      order.push_back(n);
      for (int32_t c : t[n].kids) st.push_back(c);
    }
  }
  for (size_t k = order.size(); k-- > 0;) {
    Tmp &n = t[order[k]];
    int64_t below;
    if (n.req >= 0) {
      const Req &r = b->reqs[n.req];
      const int64_t p = (int64_t)r.tok.size(), d = r.d_est;
      n.n_req = 1; n.sum_p = p; n.sum_d = d; n.min_req = n.req;
      n.B = 2 * p * d + d * d;
      n.S = 2 * (int64_t)(n.end - n.start) * d + d * d; n.max_d = d;
      below = (n.end - n.start) + d;
      n.lo_a = n.hi_a = n.start + below; n.lo_b = n.hi_b = n.B;
    } else {
      below = n.end - n.start;
      n.min_req = std::numeric_limits<int32_t>::max();
      bool first = true;
      for (int32_t c : n.kids) {
        const Tmp &ch = t[c];
        if (first || cmp_density(ch.lo_a, ch.lo_b, n.lo_a, n.lo_b) < 0) { n.lo_a = ch.lo_a; n.lo_b = ch.lo_b; }
        if (first || cmp_density(ch.hi_a, ch.hi_b, n.hi_a, n.hi_b) > 0) { n.hi_a = ch.hi_a; n.hi_b = ch.hi_b; }
        first = false;
        n.n_req += ch.n_req; n.sum_p += ch.sum_p; n.sum_d += ch.sum_d; n.B += ch.B;
        n.S += ch.S; n.max_d = std::max(n.max_d, ch.max_d);
        n.min_req = std::min(n.min_req, ch.min_req);
        below += ch.A - ch.start;
      }
      // a shared segment is charged once per step while any request below it decodes
      n.S += 2 * (int64_t)(n.end - n.start) * n.max_d;
      if (b->mem_model == BS_MEM_SHARED) n.B = n.S + 2 * (int64_t)n.start * n.max_d;
    }
    n.A = n.start + below;
  }
  // Algorithm 1: order every node's children by density, compute-intensive first
  for (Tmp &n : t)
    std::sort(n.kids.begin(), n.kids.end(), [&](int32_t x, int32_t y) {
      const int c = cmp_density(t[x].A, t[x].B, t[y].A, t[y].B);
      if (c) return c > 0;
      return t[x].min_req < t[y].min_req;
    });
  // DFS pre-order numbering of the sorted tree
  b->nodes.clear();
  b->leaf_order.clear();
  b->leaf_node.assign(nr, -1);
  std::vector<int32_t> new_id(t.size(), -1);
  struct Frame { int32_t n; size_t next; };
  std::vector<Frame> st;
  auto open = [&](int32_t n, int32_t parent_new) {
    Node out;
    out.parent = parent_new; out.start = t[n].start; out.end = t[n].end; out.req = t[n].req;
    out.first_leaf = (int32_t)b->leaf_order.size(); out.leaf_count = 0;
    out.A = t[n].A; out.B = t[n].B; out.n_req = t[n].n_req; out.sum_p = t[n].sum_p; out.sum_d = t[n].sum_d;
    out.min_req = t[n].min_req;
    out.lo_a = t[n].lo_a; out.lo_b = t[n].lo_b; out.hi_a = t[n].hi_a; out.hi_b = t[n].hi_b;
    new_id[n] = (int32_t)b->nodes.size();
    b->nodes.push_back(out);
    if (t[n].req >= 0) { b->leaf_node[t[n].req] = new_id[n]; b->leaf_order.push_back(t[n].req); }
    st.push_back({n, 0});
  };
  open(0, -1);
  while (!st.empty()) {
    Frame &f = st.back();
    if (f.next < t[f.n].kids.size()) {
      const int32_t c = t[f.n].kids[f.next++];
      const int32_t me = new_id[f.n];
      open(c, me);
      b->nodes[me].kids.push_back(new_id[c]);
    } else {
      Node &nd = b->nodes[new_id[f.n]];
      nd.leaf_count = (int32_t)b->leaf_order.size() - nd.first_leaf;
      st.pop_back();
    }
  }
}

// Indices of a longest non-increasing subsequence of the densities (A[i], B[i]), by patience:
// pile k holds the index of the densest last element of any such subsequence of length k + 1
// seen so far; a new element goes to the first pile whose last element is strictly less dense
// (else it opens a new pile) and remembers the top of the pile before.
std::vector<int32_t> longest_non_increasing(const std::vector<int64_t> &A, const std::vector<int64_t> &B) {
  const int32_t n = (int32_t)A.size();
  std::vector<int32_t> tails, pred(n, -1);
  for (int32_t i = 0; i < n; ++i) {
    int32_t lo = 0, hi = (int32_t)tails.size();
    while (lo < hi) {
      const int32_t mid = (lo + hi) / 2;
      if (cmp_density(A[i], B[i], A[tails[mid]], B[tails[mid]]) > 0) hi = mid; else lo = mid + 1;
    }
    pred[i] = lo > 0 ? tails[lo - 1] : -1;
    if (lo == (int32_t)tails.size()) tails.push_back(i); else tails[lo] = i;
  }
  std::vector<int32_t> out;
  for (int32_t i = tails.empty() ? -1 : tails.back(); i >= 0; i = pred[i]) out.push_back(i);
  std::reverse(out.begin(), out.end());
  return out;
}

struct Pre { int32_t req, cached, chunk; };  // a prefill segment: request, tokens already cached, rows this step
struct Dec { int32_t req, ctx; };            // a decode sequence: request, tokens cached before this step

// The descriptor of an explicit step: the prefill segments in the order given, then the decode
// sequences in leaf order.  Prefix nodes = trie nodes with at least two of the decode sequences
// below them and at least one whole page of their own; pages are numbered afresh, node pages
// first (DFS order), then every sequence's private pages.
// A descriptor in memory that bs_batch_free releases; NULL when memory runs out.
bs_batch_owned *own_batch(int32_t n_pre, int32_t n_dec, const std::vector<int32_t> &row_start, const std::vector<int32_t> &kv_len,
                          const std::vector<int32_t> &page_start, const std::vector<int32_t> &page_ids,
                          const std::vector<int32_t> &o_parent, const std::vector<int32_t> &o_pstart,
                          const std::vector<int32_t> &o_pages, const std::vector<int32_t> &o_first,
                          const std::vector<int32_t> &o_count, const std::vector<int32_t> &seq_leaf,
                          const std::vector<int32_t> &seq_req, int64_t n_pages) {
  bs_batch_owned *o = new (std::nothrow) bs_batch_owned();
  if (!o) return nullptr;
  std::memset(o, 0, sizeof *o);
  bool ok = true;
  auto dup = [&ok](const std::vector<int32_t> &v) -> int32_t * {
    int32_t *p = new (std::nothrow) int32_t[v.size() ? v.size() : 1];
    if (!p) { ok = false; return nullptr; }
    if (!v.empty()) std::memcpy(p, v.data(), v.size() * sizeof(int32_t));
    return p;
  };
  o->batch.n_seq = n_pre + n_dec; o->batch.n_prefill = n_pre; o->batch.n_rows = row_start.back();
  o->batch.row_start = dup(row_start); o->batch.kv_len = dup(kv_len); o->batch.page_start = dup(page_start);
  o->batch.page_ids = dup(page_ids);
  o->batch.n_nodes = (int32_t)o_parent.size();
  o->batch.node_parent = dup(o_parent); o->batch.node_page_start = dup(o_pstart); o->batch.node_page_ids = dup(o_pages);
  o->batch.node_seq_first = dup(o_first); o->batch.node_seq_count = dup(o_count); o->batch.seq_leaf_node = dup(seq_leaf);
  o->seq_request = dup(seq_req);
  o->n_pages = n_pages;
  if (!ok) { bs_batch_free(o); return nullptr; }
  return o;
}

int emit(bs_builder *b, const std::vector<Pre> &pre, std::vector<Dec> dec, bs_batch_owned **out) {
  const std::vector<Node> &nd = b->nodes;
  const int32_t ps = b->cm.page_size;
  std::vector<int32_t> leaf_pos(b->reqs.size(), 0);
  for (size_t i = 0; i < b->leaf_order.size(); ++i) leaf_pos[b->leaf_order[i]] = (int32_t)i;
  std::sort(dec.begin(), dec.end(), [&](const Dec &x, const Dec &y) { return leaf_pos[x.req] < leaf_pos[y.req]; });

  // prefix nodes: internal trie nodes with >= 2 admitted decode members and >= 1 whole new page
  const int32_t n_pre = (int32_t)pre.size(), n_dec = (int32_t)dec.size();
  std::vector<int32_t> mem_count(nd.size(), 0), mem_first(nd.size(), std::numeric_limits<int32_t>::max());
  for (int32_t k = 0; k < n_dec; ++k) {
    int32_t n = nd[b->leaf_node[dec[k].req]].parent;
    while (n >= 0) { ++mem_count[n]; mem_first[n] = std::min(mem_first[n], k); n = nd[n].parent; }
  }
  std::vector<int32_t> node_id(nd.size(), -1), cover(nd.size(), 0);
  std::vector<int32_t> o_parent, o_first, o_count, o_pstart{0}, o_pages;
  int64_t next_page = 0;
  for (size_t n = 0; n < nd.size(); ++n) {
    if (nd[n].req >= 0) continue;
    const int32_t par = nd[n].parent;
    const int32_t above = par >= 0 ? cover[par] : 0;
    const int32_t hi = nd[n].end / ps;
    if (mem_count[n] >= 2 && hi > above) {
      int32_t anc = par;
      while (anc >= 0 && node_id[anc] < 0) anc = nd[anc].parent;
      node_id[n] = (int32_t)o_parent.size();
      o_parent.push_back(anc >= 0 ? node_id[anc] : -1);
      o_first.push_back(n_pre + mem_first[n]);
      o_count.push_back(mem_count[n]);
      for (int32_t k = above; k < hi; ++k) o_pages.push_back((int32_t)next_page++);
      o_pstart.push_back((int32_t)o_pages.size());
      cover[n] = hi;
    } else {
      cover[n] = above;
    }
  }
  std::vector<int32_t> row_start{0}, kv_len, page_start{0}, page_ids, seq_leaf, seq_req;
  for (const Pre &s : pre) {
    const int32_t kv = s.cached + s.chunk;
    const int32_t npg = (kv + ps - 1) / ps;
    for (int32_t k = 0; k < npg; ++k) page_ids.push_back((int32_t)next_page++);
    row_start.push_back(row_start.back() + s.chunk);
    kv_len.push_back(kv); page_start.push_back((int32_t)page_ids.size()); seq_leaf.push_back(-1); seq_req.push_back(s.req);
  }
  std::vector<int32_t> path;
  for (int32_t k = 0; k < n_dec; ++k) {
    const int32_t ri = dec[k].req;
    const int32_t kv = dec[k].ctx + 1;
    int32_t n = nd[b->leaf_node[ri]].parent;
    while (n >= 0 && node_id[n] < 0) n = nd[n].parent;
    const int32_t leaf = n >= 0 ? node_id[n] : -1;
    path.clear();
    for (int32_t q = leaf; q >= 0; q = o_parent[q]) path.push_back(q);
    int32_t shared = 0;
    for (size_t q = path.size(); q-- > 0;) {
      const int32_t id = path[q];
      page_ids.insert(page_ids.end(), o_pages.begin() + o_pstart[id], o_pages.begin() + o_pstart[id + 1]);
      shared += o_pstart[id + 1] - o_pstart[id];
    }
    const int32_t npg = (kv + ps - 1) / ps;
    for (int32_t q = shared; q < npg; ++q) page_ids.push_back((int32_t)next_page++);
    row_start.push_back(row_start.back() + 1);
    kv_len.push_back(kv); page_start.push_back((int32_t)page_ids.size()); seq_leaf.push_back(leaf); seq_req.push_back(ri);
  }

  bs_batch_owned *o = own_batch(n_pre, n_dec, row_start, kv_len, page_start, page_ids, o_parent, o_pstart, o_pages, o_first,
                                o_count, seq_leaf, seq_req, next_page);
  if (!o) return fail(b, BS_ENOMEM, "out of memory");
  *out = o;
  return BS_OK;
}

// Algorithm 3 on the first branching node's leftmost and rightmost subtree
// No exception crosses the C boundary (vectors and maps grow with the pool).
template <class F>
int guarded(bs_builder *b, F &&body) {
  try {
    return body();
  } catch (const std::bad_alloc &) {
    return fail(b, BS_ENOMEM, "out of memory");
  } catch (const std::exception &e) {
    return fail(b, BS_EINVAL, "unexpected exception: %s", e.what());
  } catch (...) {
    return fail(b, BS_EINVAL, "unexpected exception");
  }
}

void scan_budgets(const bs_builder *b, bs_scan_info *out) {
  const bs_cost_model &cm = b->cm;
  const std::vector<Node> &nd = b->nodes;
  int32_t rt = 0;
  while (nd[rt].req < 0 && nd[rt].kids.size() == 1) rt = nd[rt].kids[0];
  int32_t L = rt, R = rt;
  if (nd[rt].req < 0 && nd[rt].kids.size() >= 2) { L = nd[rt].kids.front(); R = nd[rt].kids.back(); }
  bs_scan_info info;
  std::memset(&info, 0, sizeof info);
  info.rho_rt = rho_of(cm, nd[rt].A, nd[rt].B);
  info.rho_l = rho_of(cm, nd[L].A, nd[L].B);
  info.rho_r = rho_of(cm, nd[R].A, nd[R].B);
  partition(info.rho_rt, info.rho_l, info.rho_r, (double)cm.mem_bytes, &info.m_l, &info.m_r);
  auto side = [&](const Node &s, double m, int64_t *n_out, int64_t *c_out) {
    const double p_bar = (double)s.sum_p / (double)s.n_req;
    const double d_bar = (double)s.sum_d / (double)s.n_req;
    int64_t n = (int64_t)std::floor(m / ((p_bar + d_bar / 2.0) * (double)cm.kv_bytes));
    if (n < 1) n = 1;
    *n_out = n;
    *c_out = (d_bar == 0.0) ? -1 : (int64_t)std::floor((double)n * p_bar / d_bar);
  };
  side(nd[L], info.m_l, &info.n_l, &info.c_l);
  side(nd[R], info.m_r, &info.n_r, &info.c_r);
  *out = info;
}

}  // namespace

extern "C" {

int bs_builder_create(const bs_cost_model *cm, bs_builder **out) {
  if (!out) return BS_EINVAL;
  *out = nullptr;
  if (!cm || cm->p_model <= 0 || cm->kv_bytes <= 0 || !(cm->compute > 0) || !(cm->bandwidth > 0) || cm->mem_bytes < 0 ||
      cm->page_size <= 0)
    return BS_EINVAL;
  bs_builder *b = new (std::nothrow) bs_builder();
  if (!b) return BS_ENOMEM;
  b->cm = *cm;
  *out = b;
  return BS_OK;
}

void bs_builder_destroy(bs_builder *b) { delete b; }

const char *bs_builder_last_error(const bs_builder *b) { return b ? b->err.c_str() : "builder is NULL"; }

int bs_builder_add(bs_builder *b, const int32_t *tokens, int32_t n_tokens, int32_t d_est, int32_t n_cached) {
  return guarded(b, [&]() -> int {
  if (!b) return BS_EINVAL;
  if (b->finalized) return fail(b, BS_EINVAL, "requests cannot be added after finalize");
  if (n_tokens < 1 || !tokens) return fail(b, BS_EINVAL, "a request needs at least one prompt token");
  if (d_est < 0 || n_cached < 0) return fail(b, BS_EINVAL, "d_est and n_cached must be >= 0");
  Req r;
  r.tok.assign(tokens, tokens + n_tokens);
  r.d_est = d_est;
  r.n_cached = n_cached;
  b->reqs.push_back(std::move(r));
  return (int)b->reqs.size() - 1;
  });
}

int bs_builder_set_mem_model(bs_builder *b, int mem_model) {
  if (!b) return BS_EINVAL;
  if (b->finalized) return fail(b, BS_EINVAL, "bs_builder_set_mem_model after bs_builder_finalize");
  if (mem_model != BS_MEM_EXPANDED && mem_model != BS_MEM_SHARED) return fail(b, BS_EINVAL, "unknown memory model %d", mem_model);
  b->mem_model = mem_model;
  return BS_OK;
}

int64_t bs_kv_bytes_per_token(int variant, int32_t n_layers, int32_t n_heads, int32_t head_dim, int32_t n_kv_heads,
                              int32_t latent_dim, int32_t rope_dim, int32_t elem_bytes) {
  if (n_layers <= 0 || elem_bytes <= 0) return BS_EINVAL;
  int64_t per_layer;
  switch (variant) {
    case BS_ATTN_MHA:
      if (n_heads <= 0 || head_dim <= 0) return BS_EINVAL;
      per_layer = 2 * (int64_t)n_heads * head_dim;
      break;
    case BS_ATTN_MQA:
      if (head_dim <= 0) return BS_EINVAL;
      per_layer = 2 * (int64_t)head_dim;
      break;
    case BS_ATTN_GQA:
      if (n_heads <= 0 || head_dim <= 0 || n_kv_heads <= 0 || n_heads % n_kv_heads) return BS_EINVAL;
      per_layer = 2 * (int64_t)n_kv_heads * head_dim;
      break;
    case BS_ATTN_MLA:
      if (latent_dim <= 0 || rope_dim < 0) return BS_EINVAL;
      per_layer = (int64_t)latent_dim + rope_dim;
      break;
    default:
      return BS_EINVAL;
  }
  return per_layer * n_layers * elem_bytes;
}

int bs_builder_finalize(bs_builder *b) {
  return guarded(b, [&]() -> int {
  if (!b) return BS_EINVAL;
  if (b->finalized) return BS_OK;
  rebuild(b);
  b->finalized = true;
  return BS_OK;
  });
}

int bs_builder_split(bs_builder *b, int64_t t, int64_t budget_tokens, bs_split_info *info) {
  return guarded(b, [&]() -> int {
  if (!b) return BS_EINVAL;
  if (!b->finalized) return fail(b, BS_EINVAL, "bs_builder_split before bs_builder_finalize");
  if (t < 0) return fail(b, BS_EINVAL, "threshold t must be >= 0");
  if (b->mem_model != BS_MEM_EXPANDED)
    return fail(b, BS_EINVAL, "node splitting is defined for the additive memory model (BS_MEM_EXPANDED) only");
  int64_t spent = 0;
  int32_t rounds = 0, n_split = 0;
  std::vector<int64_t> A, B;
  for (;;) {
    const int32_t n = (int32_t)b->leaf_order.size();
    A.resize(n); B.resize(n);
    for (int32_t i = 0; i < n; ++i) {
      const Node &lf = b->nodes[b->leaf_node[b->leaf_order[i]]];
      A[i] = lf.A; B[i] = lf.B;
    }
    const std::vector<int32_t> keep = longest_non_increasing(A, B);
    if ((int32_t)keep.size() == n) break;  // C1
    std::vector<char> kept(n, 0), movable(n, 0), cand(n, 0);
    for (int32_t i : keep) kept[i] = 1;
    bool any = false;
    // first kind: a leaf that drags a subtree X to the wrong side of the sibling Q next to it
    // while belonging, itself, on the far side of all of Q
    for (int32_t i = 0; i < n; ++i) {
      const Node &lf = b->nodes[b->leaf_node[b->leaf_order[i]]];
      movable[i] = lf.parent != 0;
      if (!movable[i]) continue;
      const int64_t gone_a = lf.A - lf.start, gone_b = lf.B;  // what every ancestor loses with the leaf
      for (int32_t x = lf.parent; x != 0 && !cand[i]; x = b->nodes[x].parent) {
        const Node &X = b->nodes[x];
        const std::vector<int32_t> &sib = b->nodes[X.parent].kids;
        const size_t j = (size_t)(std::find(sib.begin(), sib.end(), x) - sib.begin());
        const int64_t ra = X.A - gone_a, rb = X.B - gone_b;
        if (j > 0) {
          const Node &Q = b->nodes[sib[j - 1]];
          if (cmp_density(ra, rb, Q.A, Q.B) > 0 && cmp_density(lf.A, lf.B, Q.lo_a, Q.lo_b) < 0) cand[i] = 1;
        }
        if (j + 1 < sib.size()) {
          const Node &Q = b->nodes[sib[j + 1]];
          if (cmp_density(ra, rb, Q.A, Q.B) < 0 && cmp_density(lf.A, lf.B, Q.hi_a, Q.hi_b) > 0) cand[i] = 1;
        }
      }
      any = any || cand[i];
    }
    if (!any) {
      // second kind: the leaves outside the longest non-increasing subsequence
      for (int32_t i = 0; i < n; ++i) cand[i] = !kept[i] && movable[i];
      for (int32_t i = 0; i + 1 < n; ++i)
        if (cmp_density(A[i], B[i], A[i + 1], B[i + 1]) < 0 && !cand[i] && !cand[i + 1]) {
          // the outlier of this violation sits under the root already: move its neighbour
          if (!kept[i] && movable[i + 1]) cand[i + 1] = 1;
          else if (!kept[i + 1] && movable[i]) cand[i] = 1;
        }
    }
    std::vector<std::pair<int64_t, int32_t>> todo;  // (cost = shared prefix length, request)
    for (int32_t i = 0; i < n; ++i)
      if (cand[i]) {
        const int32_t r = b->leaf_order[i];
        const int64_t cost = b->nodes[b->leaf_node[r]].start;
        if (cost <= t) todo.emplace_back(cost, r);
      }
    std::sort(todo.begin(), todo.end());
    int32_t took = 0;
    for (const auto &c : todo) {
      if (budget_tokens >= 0 && spent + c.first > budget_tokens) break;
      b->detached[c.second] = 1;
      spent += c.first;
      ++took;
    }
    if (took == 0) break;  // C2
    n_split += took;
    ++rounds;
    rebuild(b);
  }
  if (info) {
    const int32_t n = (int32_t)b->leaf_order.size();
    int32_t mono = 1;
    for (int32_t i = 0; i + 1 < n && mono; ++i) {
      const Node &x = b->nodes[b->leaf_node[b->leaf_order[i]]], &y = b->nodes[b->leaf_node[b->leaf_order[i + 1]]];
      if (cmp_density(x.A, x.B, y.A, y.B) < 0) mono = 0;
    }
    info->n_split = n_split; info->rounds = rounds; info->monotone = mono; info->recompute_tokens = spent;
  }
  return BS_OK;
  });
}

int bs_builder_tree_size(const bs_builder *b, int32_t *n_nodes, int32_t *n_requests) {
  if (!b || !b->finalized) return BS_EINVAL;
  if (n_nodes) *n_nodes = (int32_t)b->nodes.size();
  if (n_requests) *n_requests = (int32_t)b->reqs.size();
  return BS_OK;
}

int bs_builder_tree(const bs_builder *b, int32_t *parent, int32_t *start, int32_t *end, int32_t *req,
                    int32_t *first_leaf, int32_t *leaf_count, int64_t *A, int64_t *B, int32_t *leaf_order) {
  if (!b || !b->finalized) return BS_EINVAL;
  for (size_t i = 0; i < b->nodes.size(); ++i) {
    const Node &n = b->nodes[i];
    if (parent) parent[i] = n.parent;
    if (start) start[i] = n.start;
    if (end) end[i] = n.end;
    if (req) req[i] = n.req;
    if (first_leaf) first_leaf[i] = n.first_leaf;
    if (leaf_count) leaf_count[i] = n.leaf_count;
    if (A) A[i] = n.A;
    if (B) B[i] = n.B;
  }
  if (leaf_order) std::copy(b->leaf_order.begin(), b->leaf_order.end(), leaf_order);
  return BS_OK;
}

int bs_builder_emit(bs_builder *b, int32_t n_pre, const int32_t *pre_req, const int32_t *pre_cached,
                    const int32_t *pre_chunk, int32_t n_dec, const int32_t *dec_req, const int32_t *dec_ctx,
                    bs_batch_owned **out) {
  return guarded(b, [&]() -> int {
  if (!b || !out) return BS_EINVAL;
  *out = nullptr;
  if (!b->finalized) return fail(b, BS_EINVAL, "finalize the builder first");
  if (n_pre < 0 || n_dec < 0 || (n_pre && (!pre_req || !pre_cached || !pre_chunk)) || (n_dec && (!dec_req || !dec_ctx)))
    return fail(b, BS_EINVAL, "bs_builder_emit: bad counts or NULL arrays");
  const int32_t nr = (int32_t)b->reqs.size();
  std::vector<char> seen(nr, 0);
  std::vector<Pre> pre;
  std::vector<Dec> dec;
  for (int32_t i = 0; i < n_pre; ++i) {
    const int32_t r = pre_req[i];
    if (r < 0 || r >= nr || seen[r]) return fail(b, BS_EINVAL, "prefill segment %d: request %d out of range or repeated", i, r);
    seen[r] = 1;
    const int64_t p = (int64_t)b->reqs[r].tok.size();
    if (pre_cached[i] < 0 || pre_chunk[i] < 1 || (int64_t)pre_cached[i] + pre_chunk[i] > p)
      return fail(b, BS_EINVAL, "prefill segment %d: cached %d + chunk %d must lie within the prompt (%lld tokens)", i,
                  pre_cached[i], pre_chunk[i], (long long)p);
    pre.push_back({r, pre_cached[i], pre_chunk[i]});
  }
  for (int32_t i = 0; i < n_dec; ++i) {
    const int32_t r = dec_req[i];
    if (r < 0 || r >= nr || seen[r]) return fail(b, BS_EINVAL, "decode sequence %d: request %d out of range or repeated", i, r);
    seen[r] = 1;
    if (dec_ctx[i] < (int64_t)b->reqs[r].tok.size())
      return fail(b, BS_EINVAL, "decode sequence %d: context %d shorter than the prompt", i, dec_ctx[i]);
    dec.push_back({r, dec_ctx[i]});
  }
  return emit(b, pre, dec, out);
  });
}

void bs_batch_free(bs_batch_owned *o) {
  if (!o) return;
  delete[] o->batch.row_start; delete[] o->batch.kv_len; delete[] o->batch.page_start; delete[] o->batch.page_ids;
  delete[] o->batch.node_parent; delete[] o->batch.node_page_start; delete[] o->batch.node_page_ids;
  delete[] o->batch.node_seq_first; delete[] o->batch.node_seq_count; delete[] o->batch.seq_leaf_node;
  delete[] o->seq_request;
  delete o;
}

int bs_builder_next_batch(bs_builder *b, int64_t prefill_budget, int64_t decode_budget, bs_batch_owned **out) {
  return guarded(b, [&]() -> int {
  if (!b || !out) return BS_EINVAL;
  *out = nullptr;
  if (!b->finalized) return fail(b, BS_EINVAL, "finalize the builder first");
  if (b->reqs.empty()) return fail(b, BS_EINVAL, "no requests");
  bs_scan_info info;
  scan_budgets(b, &info);

  const int64_t INF = (int64_t)1 << 60;
  int64_t n_l = info.n_l, n_r = info.n_r;
  int64_t c_l = info.c_l < 0 ? INF : info.c_l, c_r = info.c_r < 0 ? INF : info.c_r;
  if (prefill_budget > 0 && c_l + c_r > prefill_budget) {
    if (c_l >= INF && c_r >= INF) c_l = prefill_budget / 2;
    else if (c_l >= INF) c_l = std::max<int64_t>(0, prefill_budget - c_r);
    else if (c_r >= INF) c_l = std::min(c_l, prefill_budget);
    else c_l = (int64_t)(((__int128)c_l * prefill_budget) / (c_l + c_r));
    c_r = prefill_budget - c_l;
  }
  if (decode_budget > 0 && n_l + n_r > decode_budget) {
    n_l = (int64_t)(((__int128)n_l * decode_budget) / (n_l + n_r));
    n_r = decode_budget - n_l;
  }

  std::vector<Pre> pre;
  std::vector<int32_t> dec;  // leaf-order positions of admitted decode requests
  const std::vector<int32_t> &order = b->leaf_order;
  auto admit = [&](int32_t pos, bool left) -> bool {
    const int32_t ri = order[pos];
    const Req &r = b->reqs[ri];
    const int32_t p = (int32_t)r.tok.size();
    if (r.n_cached >= p) {
      int64_t &n = left ? n_l : n_r;
      if (n <= 0) return false;
      --n;
      dec.push_back(pos);
      return true;
    }
    int64_t &c = left ? c_l : c_r;
    if (c <= 0) return false;
    const int32_t chunk = (int32_t)std::min<int64_t>(p - r.n_cached, c);
    pre.push_back({ri, r.n_cached, chunk});
    c -= chunk;
    return true;
  };
  int32_t i = 0, j = (int32_t)order.size() - 1;
  bool go_l = true, go_r = true;
  while (i <= j && (go_l || go_r)) {
    if (go_l && i <= j) { if (admit(i, true)) ++i; else go_l = false; }
    if (go_r && i <= j) { if (admit(j, false)) --j; else go_r = false; }
  }
  info.n_prefill = (int32_t)pre.size();
  info.n_decode = (int32_t)dec.size();
  std::vector<Dec> dec_list;
  for (int32_t pos : dec) dec_list.push_back({order[pos], b->reqs[order[pos]].n_cached});
  int rc = emit(b, pre, dec_list, out);
  if (rc) return rc;
  (*out)->info = info;
  return BS_OK;
  });
}

}  // extern "C"

// ---------------------------------------------------------------------------------------------
// Multi-step driver (Section 3.2 and Appendix A.2, batch scheduler: the runtime batch is re-formed
// every iteration; Section 5.3, dual scanner with the memory partition of Algorithm 3; Section 5.4,
// adaptation to misjudged output lengths; Appendix A.2, runtime prefix tree): request state, the
// memory account of the two partitions, the two scanners, and KV pages that keep their physical
// number from the step that first writes them to the step that frees them.
// ---------------------------------------------------------------------------------------------
namespace {

struct Live {
  bool alive = false;
  int32_t side = 0, cached = 0, generated = 0;
  int64_t reserved = 0;
  std::vector<int32_t> pages;  // private pages, logical page shared_hi + k
};

}  // namespace

struct bs_sched {
  const bs_builder *b = nullptr;
  bs_sched_cfg cfg;
  std::string err;
  std::vector<int32_t> d_true, order, pos_in_leaf_order;
  bool two_sided = true;
  int64_t cap[2] = {0, 0}, used[2] = {0, 0}, pre_num = 1, pre_den = 1, p_side[2] = {0, 0};
  int32_t lo = 0, hi = -1, n_live = 0;
  std::vector<Live> live;                  // by request
  std::vector<int32_t> admitted;           // admission order
  std::vector<std::vector<int32_t>> path;  // by request: internal ancestors with a segment, top down
  std::vector<int32_t> shared_hi;          // by request
  // per tree node
  std::vector<int32_t> page_lo, page_hi, ref, done, owner, nside;
  std::vector<std::vector<int32_t>> node_pages;
  std::vector<int32_t> free_pages;         // min-heap
  bs_sched_stats st;
};

namespace {

int sfail(bs_sched *s, int code, const char *fmt, ...) {
  char buf[400];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (s) s->err = buf;
  return code;
}

struct PoolExhausted {};

int32_t take_page(bs_sched *s) {
  if (s->free_pages.empty()) throw PoolExhausted();
  std::pop_heap(s->free_pages.begin(), s->free_pages.end(), std::greater<int32_t>());
  const int32_t p = s->free_pages.back();
  s->free_pages.pop_back();
  return p;
}

void give_page(bs_sched *s, int32_t p) {
  s->free_pages.push_back(p);
  std::push_heap(s->free_pages.begin(), s->free_pages.end(), std::greater<int32_t>());
}

int32_t prompt_len(const bs_sched *s, int32_t r) { return (int32_t)s->b->reqs[r].tok.size(); }

// admission of request r from `side`; false = refused (it waits, or its side's memory is full)
bool try_admit(bs_sched *s, int32_t r, int side, bool borrow) {
  const std::vector<Node> &nd = s->b->nodes;
  const int32_t p = prompt_len(s, r);
  const std::vector<int32_t> &path = s->path[r];
  int32_t cached_pages = 0;
  bool chain = true;
  std::vector<int32_t> mine;
  for (int32_t n : path) {
    const int32_t seg = nd[n].end - nd[n].start;
    if (s->ref[n] > 0 && s->done[n] == seg) {
      if (chain) cached_pages = s->page_hi[n];
    } else if (s->ref[n] > 0 && s->owner[n] >= 0) {
      return false;  // somebody is still computing this segment
    } else {
      mine.push_back(n);
      chain = false;
    }
  }
  const int64_t own = (int64_t)(p - nd[s->b->leaf_node[r]].start) + s->b->reqs[r].d_est;
  int64_t need = own;
  for (int32_t n : path)
    if (s->ref[n] == 0) need += nd[n].end - nd[n].start;
  const bool over = borrow ? (s->used[0] + s->used[1] + need > s->cfg.mem_tokens) : (s->used[side] + need > s->cap[side]);
  if (over && s->n_live > 0) return false;
  Live &lv = s->live[r];
  lv = Live();
  lv.alive = true;
  lv.side = side;
  lv.cached = std::min(16 * cached_pages, p - 1);
  lv.reserved = own;
  s->used[side] += own;
  for (int32_t n : path) {
    if (s->ref[n] == 0) {
      s->used[side] += nd[n].end - nd[n].start;
      s->nside[n] = side; s->done[n] = 0; s->owner[n] = -1;
      s->node_pages[n].clear();
    }
    ++s->ref[n];
  }
  for (int32_t n : mine) s->owner[n] = r;
  s->st.prompt_tokens_skipped += lv.cached;
  ++s->n_live;
  s->admitted.push_back(r);
  return true;
}

void release(bs_sched *s, int32_t r) {
  const std::vector<Node> &nd = s->b->nodes;
  Live &lv = s->live[r];
  s->used[lv.side] -= lv.reserved;
  for (int32_t pg : lv.pages) give_page(s, pg);
  for (int32_t n : s->path[r]) {
    if (--s->ref[n] == 0) {
      s->used[s->nside[n]] -= nd[n].end - nd[n].start;
      s->done[n] = 0; s->owner[n] = -1;
      for (int32_t pg : s->node_pages[n]) give_page(s, pg);
      s->node_pages[n].clear();
    }
  }
  lv = Live();
  --s->n_live;
}

// physical page of logical page j of live request r; allocates up to it if asked
int32_t page_of(bs_sched *s, int32_t r, int32_t j, bool may_allocate) {
  const int32_t sh = s->shared_hi[r];
  std::vector<int32_t> *pages;
  int32_t k;
  if (j < sh) {
    pages = nullptr;
    k = 0;
    for (int32_t n : s->path[r])
      if (s->page_lo[n] <= j && j < s->page_hi[n]) { pages = &s->node_pages[n]; k = j - s->page_lo[n]; break; }
  } else {
    pages = &s->live[r].pages;
    k = j - sh;
  }
  while (may_allocate && (int32_t)pages->size() <= k) pages->push_back(take_page(s));
  return (*pages)[k];
}

void plan(bs_sched *s, std::vector<Pre> &pre, std::vector<Dec> &dec) {
  int64_t budget = s->cfg.token_budget;
  const int32_t n_req = (int32_t)s->live.size();
  for (int32_t k = 0; k < n_req; ++k) {  // leaf order: what the descriptor needs
    const int32_t r = s->b->leaf_order[k];
    const Live &lv = s->live[r];
    if (lv.alive && lv.cached >= prompt_len(s, r)) dec.push_back({r, prompt_len(s, r) + lv.generated - 1});
  }
  budget -= (int64_t)dec.size();
  {
    std::vector<int32_t> keep;
    for (int32_t r : s->admitted)
      if (s->live[r].alive && s->live[r].cached < prompt_len(s, r)) keep.push_back(r);
    s->admitted.swap(keep);
  }
  const int64_t b0 = std::max<int64_t>(0, budget);
  int64_t share[2];
  share[0] = b0 * s->pre_num / s->pre_den;
  if (s->two_sided) {  // neither scanner is starved: room for one average request of its side
    share[0] = std::max(share[0], std::min(s->p_side[0], b0 / 2));
    share[0] = std::min(share[0], b0 - std::min(s->p_side[1], b0 / 2));
  }
  share[1] = b0 - share[0];
  std::vector<int32_t> waiting;
  for (int32_t r : s->admitted) {
    Live &lv = s->live[r];
    const int64_t chunk = std::min<int64_t>(prompt_len(s, r) - lv.cached, share[lv.side]);
    if (chunk <= 0) { waiting.push_back(r); continue; }
    pre.push_back({r, lv.cached, (int32_t)chunk});
    budget -= chunk;
    share[lv.side] -= chunk;
  }
  for (int pass = 0; pass < 2; ++pass) {
    const bool borrow = pass == 1;
    bool is_open[2] = {true, s->two_sided};
    if (borrow) {
      for (int32_t r : waiting) {
        if (budget <= 0) break;
        Live &lv = s->live[r];
        const int64_t chunk = std::min<int64_t>(prompt_len(s, r) - lv.cached, budget);
        pre.push_back({r, lv.cached, (int32_t)chunk});
        budget -= chunk;
      }
      share[0] = share[1] = budget;
    }
    while (budget > 0 && s->lo <= s->hi && (is_open[0] || is_open[1])) {
      bool progressed = false;
      for (int side = 0; side < 2; ++side) {
        if (!is_open[side] || s->lo > s->hi || budget <= 0) continue;
        if (share[side] <= 0) { is_open[side] = false; continue; }
        const int32_t r = side == 0 ? s->order[s->lo] : s->order[s->hi];
        if (!try_admit(s, r, side, borrow)) { is_open[side] = false; continue; }
        if (side == 0) ++s->lo; else --s->hi;
        const Live &lv = s->live[r];
        const int64_t chunk = std::min<int64_t>(std::min<int64_t>(prompt_len(s, r) - lv.cached, budget), share[side]);
        pre.push_back({r, lv.cached, (int32_t)chunk});
        budget -= chunk;
        share[side] -= chunk;
        progressed = true;
      }
      if (!progressed) break;
    }
  }
  int64_t total = (int64_t)dec.size();
  for (const Pre &x : pre) total += x.chunk;
  int64_t extra = total > s->cfg.row_multiple ? total % s->cfg.row_multiple : 0;
  while (extra > 0 && !pre.empty()) {
    const int64_t cut = std::min<int64_t>(extra, pre.back().chunk);
    if (cut == pre.back().chunk) pre.pop_back(); else pre.back().chunk -= (int32_t)cut;
    extra -= cut;
  }
}

bs_batch_owned *emit_step(bs_sched *s, const std::vector<Pre> &pre, const std::vector<Dec> &dec) {
  const std::vector<Node> &nd = s->b->nodes;
  const int32_t n_pre = (int32_t)pre.size(), n_dec = (int32_t)dec.size();
  // pages that this step writes into come into being, in the order of the descriptor
  for (const Pre &x : pre)
    for (int32_t j = x.cached / 16; j <= (x.cached + x.chunk - 1) / 16; ++j) page_of(s, x.req, j, true);
  for (const Dec &x : dec) page_of(s, x.req, x.ctx / 16, true);
  std::vector<int32_t> row_start{0}, kv_len, page_start{0}, page_ids, seq_leaf, seq_req;
  for (const Pre &x : pre) {
    const int32_t kv = x.cached + x.chunk;
    for (int32_t j = 0; j < (kv + 15) / 16; ++j) page_ids.push_back(page_of(s, x.req, j, false));
    row_start.push_back(row_start.back() + x.chunk);
    kv_len.push_back(kv); page_start.push_back((int32_t)page_ids.size()); seq_leaf.push_back(-1); seq_req.push_back(x.req);
  }
  // prefix nodes: segments with at least two decode members in this step and at least one page, in DFS order
  const int32_t n_nodes = (int32_t)nd.size();
  std::vector<int32_t> count(n_nodes, 0), first(n_nodes, -1), id(n_nodes, -1);
  for (int32_t k = 0; k < n_dec; ++k)
    for (int32_t n : s->path[dec[k].req]) {
      if (count[n]++ == 0) first[n] = k;
    }
  std::vector<int32_t> o_parent, o_first, o_count, o_pstart{0}, o_pages;
  for (int32_t n = 0; n < n_nodes; ++n) {  // the nodes are stored in DFS pre-order
    if (nd[n].req >= 0 || count[n] < 2 || s->page_hi[n] <= s->page_lo[n]) continue;
    int32_t anc = nd[n].parent;
    while (anc >= 0 && id[anc] < 0) anc = nd[anc].parent;
    id[n] = (int32_t)o_parent.size();
    o_parent.push_back(anc >= 0 ? id[anc] : -1);
    o_first.push_back(n_pre + first[n]);
    o_count.push_back(count[n]);
    o_pages.insert(o_pages.end(), s->node_pages[n].begin(), s->node_pages[n].end());
    o_pstart.push_back((int32_t)o_pages.size());
  }
  for (const Dec &x : dec) {
    const int32_t kv = x.ctx + 1;
    for (int32_t j = 0; j < (kv + 15) / 16; ++j) page_ids.push_back(page_of(s, x.req, j, false));
    row_start.push_back(row_start.back() + 1);
    int32_t deepest = -1;
    for (int32_t n : s->path[x.req])
      if (id[n] >= 0) deepest = id[n];
    kv_len.push_back(kv); page_start.push_back((int32_t)page_ids.size()); seq_leaf.push_back(deepest); seq_req.push_back(x.req);
  }
  return own_batch(n_pre, n_dec, row_start, kv_len, page_start, page_ids, o_parent, o_pstart, o_pages, o_first, o_count,
                   seq_leaf, seq_req, s->cfg.n_pages);
}

void commit(bs_sched *s, const std::vector<Pre> &pre, const std::vector<Dec> &dec) {
  const std::vector<Node> &nd = s->b->nodes;
  bs_sched_stats &st = s->st;
  int64_t pre_rows = 0;
  for (const Pre &x : pre) pre_rows += x.chunk;
  ++st.steps;
  st.prefill_rows += pre_rows;
  st.decode_rows += (int64_t)dec.size();
  st.rows += pre_rows + (int64_t)dec.size();
  st.peak_tokens = std::max(st.peak_tokens, s->used[0] + s->used[1]);
  st.peak_pages = std::max<int64_t>(st.peak_pages, s->cfg.n_pages - (int64_t)s->free_pages.size());
  for (const Pre &x : pre) {
    Live &lv = s->live[x.req];
    const int32_t lo = x.cached, hi = x.cached + x.chunk;
    for (int32_t n : s->path[x.req]) {
      const int32_t a = nd[n].start, e = nd[n].end;
      if (hi <= a || lo >= e || s->owner[n] != x.req) continue;
      s->done[n] = std::max(s->done[n], std::min(hi, e) - a);
      if (s->done[n] == e - a) s->owner[n] = -1;
    }
    lv.cached = hi;
    if (lv.cached == prompt_len(s, x.req)) {
      lv.generated = 1;
      ++st.tokens_out;
      if (lv.generated >= s->d_true[x.req]) { ++st.finished; release(s, x.req); }
    }
  }
  for (const Dec &x : dec) {
    Live &lv = s->live[x.req];
    ++lv.generated;
    ++st.tokens_out;
    const int64_t d_est = s->b->reqs[x.req].d_est;
    if (lv.generated > d_est) {
      ++lv.reserved;
      ++s->used[lv.side];
      if (s->two_sided && lv.side == 0 && s->cfg.relocate_pct > 0 && (int64_t)lv.generated * 100 >= (int64_t)s->cfg.relocate_pct * d_est) {
        s->used[0] -= lv.reserved;
        s->used[1] += lv.reserved;
        lv.side = 1;
        ++st.relocated;
      }
    }
    if (lv.generated >= s->d_true[x.req]) { ++st.finished; release(s, x.req); }
  }
}

}  // namespace

extern "C" {

int bs_sched_create(const bs_builder *b, const bs_sched_cfg *cfg, const int32_t *d_true, const int32_t *order, bs_sched **out) {
  if (!out) return BS_EINVAL;
  *out = nullptr;
  if (!b || !cfg || !d_true) return BS_EINVAL;
  if (!b->finalized || b->reqs.empty()) return BS_EINVAL;
  if (b->cm.page_size != 16 || cfg->mem_tokens < 1 || cfg->token_budget < 1 || cfg->n_pages < 1 || cfg->relocate_pct < 0 ||
      cfg->row_multiple < 1)
    return BS_EINVAL;
  try {
    bs_sched *s = new bs_sched();
    s->b = b;
    s->cfg = *cfg;
    std::memset(&s->st, 0, sizeof s->st);
    const std::vector<Node> &nd = b->nodes;
    const int32_t n_req = (int32_t)b->reqs.size(), n_nodes = (int32_t)nd.size();
    for (int32_t r = 0; r < n_req; ++r) {
      if (d_true[r] < 1) { delete s; return BS_EINVAL; }
      if (b->reqs[r].tok.empty()) { delete s; return BS_EINVAL; }
    }
    s->d_true.assign(d_true, d_true + n_req);
    s->pos_in_leaf_order.assign(n_req, 0);
    for (int32_t k = 0; k < n_req; ++k) s->pos_in_leaf_order[b->leaf_order[k]] = k;
    s->two_sided = order == nullptr;
    if (order) {
      std::vector<char> seen(n_req, 0);
      for (int32_t k = 0; k < n_req; ++k) {
        if (order[k] < 0 || order[k] >= n_req || seen[order[k]]) { delete s; return BS_EINVAL; }
        seen[order[k]] = 1;
      }
      s->order.assign(order, order + n_req);
      s->cap[0] = cfg->mem_tokens; s->cap[1] = 0;
      s->pre_num = s->pre_den = 1;
    } else {
      s->order = b->leaf_order;
      bs_scan_info info;
      scan_budgets(b, &info);
      const double m = info.m_l + info.m_r;
      const double frac_l = m > 0 ? info.m_l / m : 0.5;
      s->cap[0] = (int64_t)std::floor((double)cfg->mem_tokens * frac_l);
      s->cap[1] = cfg->mem_tokens - s->cap[0];
      if (info.c_l < 0 || info.c_r < 0 || info.c_l + info.c_r == 0) { s->pre_num = 1; s->pre_den = 2; }
      else { s->pre_num = info.c_l; s->pre_den = info.c_l + info.c_r; }
      int32_t rt = 0;
      while (nd[rt].req < 0 && nd[rt].kids.size() == 1) rt = nd[rt].kids[0];
      int32_t L = rt, R = rt;
      if (nd[rt].req < 0 && nd[rt].kids.size() >= 2) { L = nd[rt].kids.front(); R = nd[rt].kids.back(); }
      s->p_side[0] = (nd[L].sum_p + nd[L].n_req - 1) / nd[L].n_req;
      s->p_side[1] = (nd[R].sum_p + nd[R].n_req - 1) / nd[R].n_req;
    }
    s->lo = 0; s->hi = n_req - 1;
    // shareable pages of every internal node (parents come before children in the node array)
    s->page_lo.assign(n_nodes, 0); s->page_hi.assign(n_nodes, 0);
    for (int32_t n = 0; n < n_nodes; ++n) {
      if (nd[n].req >= 0) continue;
      const int32_t above = nd[n].parent >= 0 ? s->page_hi[nd[n].parent] : 0;
      bool ends_here = false;
      for (int32_t c : nd[n].kids)
        if (nd[c].req >= 0 && nd[c].end == nd[n].end) ends_here = true;
      const int32_t hi = (ends_here && nd[n].end > 0) ? (nd[n].end - 1) / 16 : nd[n].end / 16;
      s->page_lo[n] = above;
      s->page_hi[n] = std::max(above, hi);
    }
    s->ref.assign(n_nodes, 0); s->done.assign(n_nodes, 0); s->owner.assign(n_nodes, -1); s->nside.assign(n_nodes, 0);
    s->node_pages.assign(n_nodes, {});
    s->live.assign(n_req, Live());
    s->path.assign(n_req, {});
    s->shared_hi.assign(n_req, 0);
    for (int32_t r = 0; r < n_req; ++r) {
      std::vector<int32_t> &p = s->path[r];
      for (int32_t n = nd[b->leaf_node[r]].parent; n >= 0; n = nd[n].parent)
        if (nd[n].end > nd[n].start) p.push_back(n);
      std::reverse(p.begin(), p.end());
      s->shared_hi[r] = p.empty() ? 0 : s->page_hi[p.back()];
    }
    s->free_pages.resize(cfg->n_pages);
    for (int32_t i = 0; i < cfg->n_pages; ++i) s->free_pages[i] = i;  // ascending: already a min-heap
    *out = s;
    return BS_OK;
  } catch (const std::bad_alloc &) {
    return BS_ENOMEM;
  }
}

void bs_sched_destroy(bs_sched *s) { delete s; }

const char *bs_sched_last_error(const bs_sched *s) { return s ? s->err.c_str() : "scheduler is NULL"; }

int bs_sched_next(bs_sched *s, bs_batch_owned **out) {
  if (!s || !out) return BS_EINVAL;
  *out = nullptr;
  try {
    if (s->n_live == 0 && s->lo > s->hi) return BS_SCHED_DONE;
    std::vector<Pre> pre;
    std::vector<Dec> dec;
    plan(s, pre, dec);
    if (pre.empty() && dec.empty()) return sfail(s, BS_EINVAL, "the driver is stuck: nothing fits the memory of either side");
    bs_batch_owned *o = emit_step(s, pre, dec);
    if (!o) return sfail(s, BS_ENOMEM, "out of memory");
    commit(s, pre, dec);
    *out = o;
    return BS_OK;
  } catch (const PoolExhausted &) {
    return sfail(s, BS_ENOMEM, "the page pool of %d pages is exhausted", s->cfg.n_pages);
  } catch (const std::bad_alloc &) {
    return sfail(s, BS_ENOMEM, "out of memory");
  }
}

int bs_sched_get_stats(const bs_sched *s, bs_sched_stats *out) {
  if (!s || !out) return BS_EINVAL;
  *out = s->st;
  out->mem_left = s->cap[0];
  out->mem_right = s->cap[1];
  return BS_OK;
}

}  // extern "C"
