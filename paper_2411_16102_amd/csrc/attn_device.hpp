// Device code of the decode-attention work unit, shared by the attention kernels and by the
// GEMM launches that carry decode attention on a part of the chip (BlendServe Section 3.3:
// with compute-bound and memory-bound operators overlapped a step costs the larger of the
// two times, not their sum; Section 2.2: operator-level overlapping).
#pragma once
#include "attn.hpp"
#include "common.hpp"

namespace bs {
namespace attn_dev {

constexpr float NEG_BIG = -1.0e30f;
__device__ __forceinline__ u32x4_t ld16(const uint16_t *p) { return *reinterpret_cast<const u32x4_t *>(p); }
__device__ __forceinline__ u32x2_t ld8(const uint16_t *p) { return *reinterpret_cast<const u32x2_t *>(p); }
// KV pages of a 16-row unit are read once per step and by nobody else: their loads can be marked
// non-temporal, so that the caches keep what is read again (GEMM operands of the tiles that run
// beside an attention workgroup, page tables, queries) rather than pages nobody returns to.
// Measured on MI355X: GEMM tiles beside attention workgroups 145 -> 107 us (output projection) and
// 96 -> 83 us (gate/up), a launch of 16-row units alone 5.3 -> 6.0 TB/s; but the launch that mixes
// prefill workgroups, 64-row units and 16-row units loses 3 to 7 % with it (8B and 70B blended
// shapes), so the caller chooses: NT for launches of 16-row units alone and for units that ride
// in a GEMM launch, ordinary loads otherwise.
template <bool NT>
__device__ __forceinline__ u32x4_t ld16_kv(const uint16_t *p) {
  if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
  else return ld16(p);
}
template <bool NT>
__device__ __forceinline__ u32x2_t ld8_kv(const uint16_t *p) {
  if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const u32x2_t *>(p));
  else return ld8(p);
}

// zero the bf16 halves of `v` (tokens t0 .. t0+3) that lie at or beyond `limit`
__device__ __forceinline__ u32x2_t mask_tokens(u32x2_t v, int t0, int limit) {
  if (t0 + 0 >= limit) v.x &= 0xFFFF0000u;
  if (t0 + 1 >= limit) v.x &= 0x0000FFFFu;
  if (t0 + 2 >= limit) v.y &= 0xFFFF0000u;
  if (t0 + 3 >= limit) v.y &= 0x0000FFFFu;
  return v;
}

// ------------------------------------------------------------------------------
// decode attention: one wavefront per (item, KV head), up to 16 * NQB query rows
// ------------------------------------------------------------------------------
// The online softmax keeps a per-row reference exponent m that only moves when a
// new score exceeds it by more than TAU (in log2 units): probabilities are then
// bounded by 2^TAU, which bf16 and the fp32 accumulators hold without loss, and
// the accumulators are rescaled a few times per chunk instead of once per page.
constexpr float TAU = 8.0f;

template <int DH, int NQB, bool NT = false>
__device__ __forceinline__ void decode_unit(const DecodeArgs &a, int item, int kvh, int wave, int lane, uint16_t *q_sh) {
  constexpr int KC = DH / 32;  // 32-wide chunks of the head dimension (QK^T contraction)
  constexpr int DB = DH / 16;  // 16-row blocks of the head dimension (PV output rows)
  const int hkv = a.s.n_kv_heads, hq = a.s.n_q_heads, grp = hq / hkv;
  const DecodeItem it = a.items[item];
  const int n_rows = it.n_members * grp;
  const int n_tok = it.n_tokens;
  const int n_pg = (n_tok + 15) >> 4;
  const int jq = lane & 15, g4 = lane >> 4;
  const size_t tile = (size_t)16 * DH;
  const float sc = a.s.scale_log2e;

  // query fragments: B operand of S^T = K Q^T; lane (jq, g4) holds Q[row 16 qb + jq][32c + 8 g4 ..+7].
  // With four blocks of head dimension 128 they would not fit beside the accumulators
  // and the two K/V register sets, so they stay in LDS (each lane re-reads only what it
  // wrote itself: no barrier is needed) and are fetched again for every pair of pages.
  constexpr bool Q_LDS = NQB > 1 && DH > 64;
  constexpr int QLD = DH + 8;  // padded row: 16-byte reads of 16 consecutive rows spread over all banks
  bf16x8_t qf[Q_LDS ? 1 : NQB][Q_LDS ? 1 : KC];
  uint32_t q_off = (uint32_t)((wave * NQB * 16 + jq) * QLD + 8 * g4);
  bool row_ok[NQB];
  int my_seq[NQB], my_head[NQB], my_part[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int r = qb * 16 + jq;
    row_ok[qb] = r < n_rows;
    my_seq[qb] = it.seq_first + (row_ok[qb] ? r / grp : 0);
    my_head[qb] = kvh * grp + (row_ok[qb] ? r % grp : 0);
    my_part[qb] = a.part_start[my_seq[qb]];  // needed only at the end: asked for now, it costs no wait there
    // a decode sequence has one row, and the decode rows follow the prefill rows in sequence order
    const uint16_t *p = a.q + (size_t)(my_seq[qb] + a.row_base) * (hq * DH) + my_head[qb] * DH + 8 * g4;
#pragma unroll
    for (int c = 0; c < KC; ++c) {
      u32x4_t v = {0u, 0u, 0u, 0u};
      if (row_ok[qb]) v = ld16(p + 32 * c);
      if constexpr (Q_LDS)
        *reinterpret_cast<u32x4_t *>(&q_sh[q_off + qb * 16 * QLD + 32 * c]) = v;
      else
        qf[qb][c] = as_bf16x8(v);
    }
  }
  auto q_frag = [&](int qb, int c) -> bf16x8_t {
    if constexpr (Q_LDS)
      return as_bf16x8(*reinterpret_cast<const u32x4_t *>(&q_sh[q_off + qb * 16 * QLD + 32 * c]));
    else
      return qf[qb][c];
  };

  f32x4_t o[NQB][DB];
  float m[NQB], l[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    m[qb] = NEG_BIG;
    l[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db) o[qb][db] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  }

  // The chunk's page ids sit in one register (lane i holds page i; chunks have at most
  // 64 pages), so the loop never waits on a scalar memory load to form an address.
  const int n_pairs = (n_pg + 1) >> 1;
  const int my_page = a.item_pages[it.page_off + (lane < n_pg ? lane : n_pg - 1)];

  // One pair of pages (32 tokens) per step, two register sets in ping-pong: while one
  // pair is being computed the other pair (16 KB per wavefront) is in flight, and the
  // set just consumed is refilled at once.  Loads are unconditional (past the end they
  // re-read the last pair, whose tokens are then all masked), which keeps the loop
  // straight-line so that every wait covers exactly the loads it needs.  A pair is
  // loaded once and used by all NQB blocks of 16 query rows.
  struct Frags {
    u32x4_t k[2][KC];
    u32x2_t v0[DB], v1[DB];
  };
  auto page_of = [&](int i) -> size_t {
    return (size_t)__builtin_amdgcn_readlane(my_page, i < n_pg ? i : n_pg - 1);
  };
  auto load_pages = [&](size_t p0, size_t p1, Frags &f) {
    const uint16_t *k0 = a.kv_pool + ((p0 * 2 + 0) * hkv + kvh) * tile + jq * DH + 8 * g4;
    const uint16_t *k1 = a.kv_pool + ((p1 * 2 + 0) * hkv + kvh) * tile + jq * DH + 8 * g4;
    const uint16_t *v0 = a.kv_pool + ((p0 * 2 + 1) * hkv + kvh) * tile + jq * 16 + 4 * g4;
    const uint16_t *v1 = a.kv_pool + ((p1 * 2 + 1) * hkv + kvh) * tile + jq * 16 + 4 * g4;
#pragma unroll
    for (int c = 0; c < KC; ++c) {
      f.k[0][c] = ld16_kv<NT>(k0 + 32 * c);
      f.k[1][c] = ld16_kv<NT>(k1 + 32 * c);
    }
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      f.v0[db] = ld8_kv<NT>(v0 + db * 256);
      f.v1[db] = ld8_kv<NT>(v1 + db * 256);
    }
  };
  auto load = [&](int pr, Frags &f) {
    const int i0 = 2 * (pr < n_pairs ? pr : n_pairs - 1);
    load_pages(page_of(i0), page_of(i0 + 1), f);
  };
  auto compute = [&](int pr, Frags &f) {
    const int tb = pr * 32;
    const bool ragged = tb + 32 > n_tok;  // the last pair of a chunk, or a step past the end
    if constexpr (Q_LDS) asm volatile("" : "+v"(q_off));  // keep the query reads inside the loop
    if (ragged) {  // never let stale slots (possibly NaN bit patterns) meet a zero probability
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        f.v0[db] = mask_tokens(f.v0[db], tb + 4 * g4, n_tok);
        f.v1[db] = mask_tokens(f.v1[db], tb + 16 + 4 * g4, n_tok);
      }
    }
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      f32x4_t s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < KC; ++c) {
        const bf16x8_t qv = q_frag(qb, c);
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(f.k[0][c]), qv, s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(f.k[1][c]), qv, s1, 0, 0, 0);
      }
      float sv[8];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        sv[r] = s0[r] * sc;
        sv[4 + r] = s1[r] * sc;
      }
      if (ragged) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (tb + 4 * g4 + r >= n_tok) sv[r] = NEG_BIG;
          if (tb + 16 + 4 * g4 + r >= n_tok) sv[4 + r] = NEG_BIG;
        }
      }
      float mx = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      if (__builtin_amdgcn_ballot_w64(mx > m[qb] + TAU) != 0) {  // wave-uniform: somebody's reference must move
        const float m_new = fmaxf(m[qb], mx);
        const float alpha = fast_exp2(m[qb] - m_new);
        m[qb] = m_new;
        l[qb] *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db) o[qb][db] *= alpha;
      }
      float ps = 0.f;
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        sv[r] = fast_exp2(sv[r] - m[qb]);
        ps += sv[r];
      }
      l[qb] += ps;
      u32x4_t pw;
      pw.x = pack_bf16x2(sv[0], sv[1]);
      pw.y = pack_bf16x2(sv[2], sv[3]);
      pw.z = pack_bf16x2(sv[4], sv[5]);
      pw.w = pack_bf16x2(sv[6], sv[7]);
      const bf16x8_t pf = as_bf16x8(pw);
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        u32x4_t vw;
        vw.x = f.v0[db].x;
        vw.y = f.v0[db].y;
        vw.z = f.v1[db].x;
        vw.w = f.v1[db].y;
        o[qb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vw), pf, o[qb][db], 0, 0, 0);
      }
    }
  };

  // the item names its first two pages itself: the first loads need not wait for the page list
  Frags fa, fb;
  load_pages((size_t)it.page0, (size_t)it.page1, fa);
  load(1, fb);
  for (int pr = 0; pr < n_pairs; pr += 2) {
    compute(pr, fa);
    if constexpr (NQB > 1) __builtin_amdgcn_sched_barrier(0);  // refill only once the set is dead
    load(pr + 2, fa);
    if constexpr (NQB > 1) __builtin_amdgcn_sched_barrier(0);
    compute(pr + 1, fb);
    if constexpr (NQB > 1) __builtin_amdgcn_sched_barrier(0);
    load(pr + 3, fb);
    if constexpr (NQB > 1) __builtin_amdgcn_sched_barrier(0);
  }

  // partial state out: lane (jq, g4) holds, of query row 16 qb + jq, dh = 16 db + 4 g4 .. +3
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    float ls = l[qb];
    ls += __shfl_xor(ls, 16, 64);
    ls += __shfl_xor(ls, 32, 64);
    if (row_ok[qb]) {
      const size_t base = (size_t)(my_part[qb] + it.slot_off) * hq + my_head[qb];
#pragma unroll
      for (int db = 0; db < DB; ++db)
        *reinterpret_cast<f32x4_t *>(a.part_acc + base * DH + 16 * db + 4 * g4) = o[qb][db];
      if (g4 == 0) {
        a.part_m[base] = m[qb];
        a.part_l[base] = ls;
      }
    }
  }
}

// One trace record (see DecodeQueue::trace): when a wavefront began and ended, on which CU, and
// what it did in between.
__device__ __forceinline__ void trace_record(uint64_t *rec, uint64_t t0, int kind, unsigned units, unsigned tokens) {
  // HW_ID (register 4): wave, SIMD, pipe, CU, shader array and engine; XCC_ID (register 20)
  const unsigned hw = __builtin_amdgcn_s_getreg((16 - 1) << 11 | 0 << 6 | 4);
  const unsigned xcc = __builtin_amdgcn_s_getreg((4 - 1) << 11 | 0 << 6 | 20);
  rec[0] = t0;
  rec[1] = wall_clock64();
  rec[2] = (uint64_t)kind | (uint64_t)hw << 8 | (uint64_t)xcc << 32;
  rec[3] = (uint64_t)units | (uint64_t)tokens << 32;
}

// A wavefront that serves a queue of 16-row units: it draws unit numbers from the queue's
// ticket counter until they run out (or until the launch that carries the queue has closed
// the counter by pushing it past every unit number), one memory round trip per unit.
// `rec`: this wavefront's trace record or NULL.
template <int DH>
__device__ __forceinline__ void decode_queue_worker(const DecodeQueue &q, int wave, int lane, uint64_t *rec) {
  const int hkv = q.d.s.n_kv_heads;
  if (wave >= q.waves) return;
  const uint64_t t0 = rec ? wall_clock64() : 0;
  unsigned units = 0, tokens = 0;
  for (;;) {
    unsigned tk = 0;
    if (lane == 0) tk = atomicAdd(q.ticket, 1u);
    tk = (unsigned)__builtin_amdgcn_readfirstlane((int)tk);
    if (tk >= (unsigned)q.n_units) break;
    const int item = q.first_item + (int)tk / hkv;
    decode_unit<DH, 1, true>(q.d, item, (int)tk % hkv, wave, lane, nullptr);
    if (rec) {
      ++units;
      tokens += (unsigned)q.d.items[item].n_tokens;
    }
  }
  if (rec && lane == 0) trace_record(rec, t0, TRACE_ATTENTION, units, tokens);
}

}  // namespace attn_dev
}  // namespace bs
