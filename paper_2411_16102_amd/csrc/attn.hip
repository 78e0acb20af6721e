// Paged attention kernels for gfx950.
//
// KV page layout (per page, per KV head): a K tile [16 slots][dh] and a
// TRANSPOSED V tile [dh][16 slots].  Both contractions then read their MFMA
// operands straight from global memory with the contracted index contiguous:
// scores contract over dh (K rows), outputs contract over tokens (V^T rows).
//
// Both kernels compute transposed products, S^T = K Q^T and O^T = V^T P^T, so that
// a lane owns ONE query row (its accumulator column): the running maximum, the
// running sum and the rescale factor of the online softmax are per-lane scalars,
// and the probabilities leave the score accumulators already in the register
// layout the second MFMA wants for its P^T operand (the token order inside a
// k-group is permuted the same way on the V^T side, which a contraction allows).
//
// Decode attention is prefix-aware (BlendServe Appendix A.2, intra-batch prefix
// sharing; Section 4.1, decode attention is the memory-bound operator whose time
// is the bytes of KV it loads): the pages of a prefix node are read once for all
// member sequences of the node, whose query rows are stacked along the MFMA N
// dimension; every (node chunk | private tail chunk) leaves a partial softmax
// state (m, l, acc) per query row and head, and a second kernel merges a
// sequence's states along its root-to-leaf path.
#include <type_traits>

#include "attn.hpp"
#include "attn_device.hpp"
#include "common.hpp"

namespace bs {
namespace {
using namespace attn_dev;


// One launch for both kinds of item, one wavefront per SIMD (the 16-row items stream as fast
// with one wavefront per SIMD as with two).  Grid order: wide workgroups first, narrow ones
// after, longest first within a kind.  Where the wide workgroups are at least a third of the
// grid, one of them alternates with two narrow ones for as long as both kinds last (what is
// left of the wide kind goes first): a wavefront with 64 query rows spends part of its time
// on arithmetic, and the narrow wavefronts beside it use the bandwidth it leaves (measured:
// -9 % with 1280 wide and 2048 narrow workgroups, +2 % with 390 and 1812, hence the rule).
// The period is odd on purpose: workgroups go to the eight XCDs in turn, and a period of
// four would send every wide workgroup to the same two of them.
template <int DH, bool NT_NARROW>
__device__ __forceinline__ void decode_workgroup(const DecodeArgs &a, int n_wide_units, int n_narrow_units, int b, int wave,
                                                 int lane, uint16_t *q_sh) {
  constexpr int WQB = 4;  // blocks of 16 query rows of a wide item
  const int hkv = a.s.n_kv_heads;
  const int nw = (n_wide_units + 3) >> 2, nn = (n_narrow_units + 3) >> 2;  // workgroups of each kind
  const int mixed = 2 * nw >= nn ? min(nw, nn >> 1) : 0;                   // periods of one wide + two narrow
  const int lead = nw - mixed;                                             // wide workgroups ahead of the mixed part
  bool wide;
  int wg;  // index of this workgroup within its kind
  if (b < lead) {
    wide = true;
    wg = b;
  } else if (b - lead < 3 * mixed) {
    const int per = (b - lead) / 3, pos = (b - lead) % 3;
    wide = pos == 0;
    wg = wide ? lead + per : 2 * per + pos - 1;
  } else {
    wide = false;
    wg = 2 * mixed + (b - lead - 3 * mixed);
  }
  const int unit = wg * 4 + wave;
  if (wide) {
    if (unit < n_wide_units) decode_unit<DH, WQB>(a, unit / hkv, unit % hkv, wave, lane, q_sh);
  } else {
    if (unit < n_narrow_units) decode_unit<DH, 1, NT_NARROW>(a, n_wide_units / hkv + unit / hkv, unit % hkv, wave, lane, q_sh);
  }
}

constexpr int DECODE_Q_LDS(int dh) { return dh > 64 ? 4 * 4 * 16 * (dh + 8) : 8; }  // bf16 elements: queries of four wide units

template <int DH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void decode_attn_kernel(const DecodeArgs a, int n_wide_units, int n_narrow_units) {
  __shared__ __align__(16) uint16_t q_sh[DECODE_Q_LDS(DH)];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // a launch of decode units alone: non-temporal loads for the 16-row units (see ld16_kv)
  decode_workgroup<DH, true>(a, n_wide_units, n_narrow_units, blockIdx.x, wave, threadIdx.x & 63, q_sh);
}

// ------------------------------------------------------------------------------
// merge: dh/4 lanes per (decode sequence, query head), four output elements per lane
//   M = max_p m_p;  w_p = 2^(m_p - M);  out = sum_p w_p acc_p / sum_p w_p l_p
// ------------------------------------------------------------------------------
// A wavefront covers 256/dh heads of one sequence, so its loads of the partial outputs are
// 16 bytes per lane, and the partial states are added four at a time with their loads
// issued together: the kernel is a chain of a few memory round trips, not bandwidth.
template <int DH>
__global__ __launch_bounds__(256) void decode_merge_kernel(const MergeArgs a) {
  constexpr int LPH = DH / 4;    // lanes per head
  constexpr int HPW = 64 / LPH;  // heads per wavefront
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int hq = a.s.n_q_heads;
  const int units_per_seq = (hq + HPW - 1) / HPW;
  const int unit = blockIdx.x * 4 + wave;
  if (unit >= a.n_decode * units_per_seq) return;
  const int seq = a.n_prefill + unit / units_per_seq;
  const int sub = lane / LPH, li = lane % LPH;
  const int head_raw = (unit % units_per_seq) * HPW + sub;
  const bool ok = head_raw < hq;
  const int head = ok ? head_raw : hq - 1;  // lanes past the last head repeat it and store nothing
  const int s0 = a.part_start[seq], n = a.part_start[seq + 1] - s0;
  float mx = NEG_BIG;
  for (int p = li; p < n; p += LPH) mx = fmaxf(mx, a.part_m[(size_t)(s0 + p) * hq + head]);
#pragma unroll
  for (int o = LPH / 2; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  float ls = 0.f;
  for (int p = li; p < n; p += LPH) {
    const size_t b = (size_t)(s0 + p) * hq + head;
    ls += fast_exp2(a.part_m[b] - mx) * a.part_l[b];
  }
#pragma unroll
  for (int o = LPH / 2; o >= 1; o >>= 1) ls += __shfl_xor(ls, o, 64);
  f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
  int p = 0;
  for (; p + 4 <= n; p += 4) {
    float w[4];
    f32x4_t v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const size_t b = (size_t)(s0 + p + u) * hq + head;
      w[u] = a.part_m[b];
      v[u] = *reinterpret_cast<const f32x4_t *>(a.part_acc + b * DH + li * 4);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) acc += fast_exp2(w[u] - mx) * v[u];
  }
  for (; p < n; ++p) {
    const size_t b = (size_t)(s0 + p) * hq + head;
    acc += fast_exp2(a.part_m[b] - mx) * *reinterpret_cast<const f32x4_t *>(a.part_acc + b * DH + li * 4);
  }
  if (!ok) return;
  const float inv = 1.f / ls;
  u32x2_t o2;
  o2.x = pack_bf16x2(acc[0] * inv, acc[1] * inv);
  o2.y = pack_bf16x2(acc[2] * inv, acc[3] * inv);
  *reinterpret_cast<u32x2_t *>(a.out + (size_t)a.row_start[seq] * (hq * DH) + head * DH + li * 4) = o2;
}

// acc *= alpha for an MFMA accumulator that lives in the accumulation registers.  Written out
// by hand so that the only vector-ALU use of the output accumulators inside the block loop
// is this rarely taken path: left to the compiler, the register copies it needs are hoisted
// to the top of every iteration.  The trailing wait states separate the last register write
// from a following MFMA that reads it.
__device__ __forceinline__ void scale_acc(f32x16_t &acc, float alpha) {
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float e = acc[r], t;
    asm(  // not volatile: the compiler must see that it touches no memory
        "v_accvgpr_read_b32 %1, %0\n\t"
        "v_mul_f32 %1, %1, %2\n\t"
        "v_accvgpr_write_b32 %0, %1\n\t"
        "s_nop 3"
        : "+a"(e), "=&v"(t)
        : "v"(alpha));
    acc[r] = e;
  }
}

// ------------------------------------------------------------------------------
// prefill attention: one wavefront per (64 query rows, query head); the
// wavefronts of a workgroup are the heads of one KV group and walk the same pages
// ------------------------------------------------------------------------------
// Two blocks of 32 query rows share every key and value fragment the wavefront loads: the
// operands come straight from global memory (a lane's key fragment is 16 bytes of a
// 256-byte row, so a load instruction touches 32 cache lines), and twice the rows per load
// is half the L1 accesses per MFMA.  The accumulators of 64 rows x dh 128 leave room for
// one wavefront per SIMD only, so vector-ALU and matrix work of a block overlap only as far
// as the instruction order below lets them.  A variant that stages keys and values in LDS
// for eight wavefronts of 32 rows (one workgroup-wide load per block, one barrier per block)
// was measured slower: its wavefronts move in lockstep and the LDS, matrix and
// vector-ALU phases of a block add up instead of overlapping.
template <int DH>
__device__ __forceinline__ void prefill_workgroup(const PrefillArgs &a, int heads_per_wg, int b, int wave, int lane) {
  constexpr int KC = DH / 16;  // k-steps of the 32x32x16 score MFMA
  constexpr int DB = DH / 32;  // 32-row blocks of the output
  constexpr int NQ = 2;        // blocks of 32 query rows per wavefront
  const int hkv = a.s.n_kv_heads, hq = a.s.n_q_heads, grp = hq / hkv;
  const int wg_per_work = hq / heads_per_wg;
  const int w = b / wg_per_work;
  const int seq = a.work[2 * w], qblk = a.work[2 * w + 1];  // block of 64 query rows
  const int head = (b % wg_per_work) * heads_per_wg + wave;
  const int kvh = head / grp;
  const int r0 = a.row_start[seq], q_len = a.row_start[seq + 1] - r0;
  const int kv_len = a.kv_len[seq];
  const int lr = lane & 31, g2 = lane >> 5;
  const size_t tile = (size_t)16 * DH;
  const int32_t *pages = a.page_ids + a.page_start[seq];
  const int n_pg = (kv_len + 15) >> 4;
  const uint32_t v_off = lr * 16 + 4 * g2;  // this lane's element within a value tile [dh][16 tokens]

  int n_q[NQ], my_pos[NQ], last_tb[NQ], first_pos[NQ];
  bf16x8_t qf[NQ][KC];
  f32x16_t o[NQ][DB];
  float m[NQ], l[NQ];
#pragma unroll
  for (int qb = 0; qb < NQ; ++qb) {
    const int row0 = qblk * 64 + qb * 32;
    n_q[qb] = min(32, q_len - row0);                       // <= 0: the block does not exist
    first_pos[qb] = kv_len - q_len + row0;
    my_pos[qb] = min(first_pos[qb] + lr, kv_len - 1);
    last_tb[qb] = n_q[qb] > 0 ? (first_pos[qb] + n_q[qb] - 1) / 32 : -1;  // last block of 32 tokens it attends to
    const bool ok = lr < n_q[qb];
    const uint16_t *p = a.q + (size_t)(r0 + (ok ? row0 + lr : 0)) * (hq * DH) + head * DH + 8 * g2;
#pragma unroll
    for (int c = 0; c < KC; ++c) {
      u32x4_t v = {0u, 0u, 0u, 0u};
      if (ok) v = ld16(p + 16 * c);
      qf[qb][c] = as_bf16x8(v);
    }
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[qb][db][r] = 0.f;
    m[qb] = NEG_BIG;
    l[qb] = 0.f;
  }

  const int n_tb = max(last_tb[0], last_tb[1]) + 1;
  // Software pipeline, one block of 32 tokens deep: while block tb is computed, the values of
  // block tb+1 travel into the second value buffer, its keys into the key registers (as soon
  // as the score MFMAs of block tb have read them) and the page ids of block tb+2 into scalar
  // registers.  Steps past the end re-read the last block (never used).
  struct PagePair { int p0, p1; };
  auto page_pair = [&](int tb) __attribute__((always_inline)) {
    const int t = tb < n_tb ? tb : n_tb - 1;
    PagePair pp;
    pp.p0 = pages[2 * t];
    pp.p1 = (2 * t + 1 < n_pg) ? pages[2 * t + 1] : pp.p0;
    return pp;
  };
  auto load_k = [&](PagePair pp, u32x4_t (&kf)[KC]) __attribute__((always_inline)) {
    const size_t pk = (lr < 16) ? pp.p0 : pp.p1;
    const uint16_t *kp = a.kv_pool + ((pk * 2 + 0) * hkv + kvh) * tile + (lr & 15) * DH + 8 * g2;
#pragma unroll
    for (int c = 0; c < KC; ++c) kf[c] = ld16(kp + 16 * c);
  };
  // values of a block as loaded: [32-row block of dh][16-token half of the block][8 tokens]
  auto load_v = [&](PagePair pp, u32x2_t (&r)[DB][4]) __attribute__((always_inline)) {
    const uint16_t *v0 = a.kv_pool + (((size_t)pp.p0 * 2 + 1) * hkv + kvh) * tile;  // wave-uniform bases,
    const uint16_t *v1 = a.kv_pool + (((size_t)pp.p1 * 2 + 1) * hkv + kvh) * tile;  // lane offset v_off
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      r[db][0] = ld8(v0 + v_off + 512 * db);
      r[db][1] = ld8(v0 + v_off + 512 * db + 8);
      r[db][2] = ld8(v1 + v_off + 512 * db);
      r[db][3] = ld8(v1 + v_off + 512 * db + 8);
    }
  };
  // block tb: keys in kf and values in vr have been requested; `next` holds the pages of block tb+1
  auto block = [&](int tb, u32x4_t (&kf)[KC], u32x2_t (&vr)[DB][4], u32x2_t (&vn)[DB][4], PagePair &next, auto two) __attribute__((always_inline)) {
    const PagePair after = page_pair(tb + 2);
    load_v(next, vn);
    if (tb * 32 + 32 > kv_len) {  // wave-uniform: the block runs past the context
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int h = 0; h < 4; ++h) vr[db][h] = mask_tokens(vr[db][h], tb * 32 + 8 * h + 4 * g2, kv_len);
    }
    u32x4_t va[DB][2];
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      va[db][0] = u32x4_t{vr[db][0].x, vr[db][0].y, vr[db][1].x, vr[db][1].y};
      va[db][1] = u32x4_t{vr[db][2].x, vr[db][2].y, vr[db][3].x, vr[db][3].y};
    }
    // Order of issue: both score products, then softmax of the first query block (its VALU
    // work runs while the matrix pipe is still busy with the second product), its PV product,
    // softmax of the second block under that product, and the second PV product.
    auto scores = [&](int qb) {
      f32x16_t s;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
      for (int c = 0; c < KC; ++c)
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kf[c]), qf[qb][c], s, 0, 0, 0);
      return s;
    };
    // element r of s: token tb*32 + 8*(r/4) + 4*g2 + r%4 against the query at my_pos
    // softmax of one query block in two parts.  `prepare` (mask, running maximum, the rare
    // rescale) branches; `weights` (exponentials, row sums, bf16 packing) does not, so that
    // the scheduler may slide it under the MFMAs of the other query block.
    auto prepare = [&](f32x16_t &s, int qb) __attribute__((always_inline)) {
      if (tb * 32 + 31 > first_pos[qb]) {  // wave-uniform: the block holds tokens some query must not see
        const int lim = my_pos[qb] - tb * 32 - 4 * g2;
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (8 * (r >> 2) + (r & 3) > lim) s[r] = NEG_BIG;
      }
      float mx = fmaxf(s[0], s[1]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) mx = fmaxf(fmaxf(mx, s[r]), s[r + 1]);
      mx *= a.s.scale_log2e;  // the scale is positive: the maximum commutes with it
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      // lazy reference exponent, as in the decode kernel: rescale only when somebody's maximum
      // has grown by more than 2^TAU
      if (__builtin_amdgcn_ballot_w64(mx > m[qb] + TAU) != 0) {
        const float m_new = fmaxf(m[qb], mx);
        const float alpha = fast_exp2(m[qb] - m_new);
        m[qb] = m_new;
        l[qb] *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db) scale_acc(o[qb][db], alpha);
      }
    };
    auto weights = [&](f32x16_t &s, int qb, u32x4_t &pw0, u32x4_t &pw1) __attribute__((always_inline)) {
      const float neg_m = -m[qb];
      float ps = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        s[r] = fast_exp2(__builtin_fmaf(s[r], a.s.scale_log2e, neg_m));
        ps += s[r];
      }
      l[qb] += ps;
      pw0.x = pack_bf16x2(s[0], s[1]);
      pw0.y = pack_bf16x2(s[2], s[3]);
      pw0.z = pack_bf16x2(s[4], s[5]);
      pw0.w = pack_bf16x2(s[6], s[7]);
      pw1.x = pack_bf16x2(s[8], s[9]);
      pw1.y = pack_bf16x2(s[10], s[11]);
      pw1.z = pack_bf16x2(s[12], s[13]);
      pw1.w = pack_bf16x2(s[14], s[15]);
    };
    auto pv = [&](int qb, const u32x4_t &pw0, const u32x4_t &pw1) __attribute__((always_inline)) {
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(va[db][0]), as_bf16x8(pw0), o[qb][db], 0, 0, 0);
        o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(va[db][1]), as_bf16x8(pw1), o[qb][db], 0, 0, 0);
      }
    };
    u32x4_t pa0, pa1, pb0, pb1;
    if constexpr (decltype(two)::value) {  // the second query block exists
      // (past the first block's last position its scores are all masked and add nothing)
      f32x16_t s0 = scores(0);
      f32x16_t s1 = scores(1);
      load_k(next, kf);
      prepare(s0, 0);
      prepare(s1, 1);
      __builtin_amdgcn_sched_barrier(0);
      weights(s0, 0, pa0, pa1);
      __builtin_amdgcn_sched_barrier(0);
      // the first PV product, one MFMA at a time, with the second block's weights in between
      pv(0, pa0, pa1);
      weights(s1, 1, pb0, pb1);
#pragma unroll
      for (int i = 0; i < 2 * DB; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);           // one MFMA
        __builtin_amdgcn_sched_group_barrier(0x002, 56 / (2 * DB), 0);  // its share of the VALU work
      }
      __builtin_amdgcn_sched_barrier(0);
      pv(1, pb0, pb1);
    } else {
      f32x16_t s0 = scores(0);
      load_k(next, kf);
      prepare(s0, 0);
      weights(s0, 0, pa0, pa1);
      pv(0, pa0, pa1);
    }
    next = after;
  };
  u32x4_t kf[KC];
  u32x2_t v_a[DB][4], v_b[DB][4];
  {
    const PagePair first = page_pair(0);
    load_k(first, kf);
    load_v(first, v_a);
  }
  PagePair next = page_pair(1);
  auto run = [&](auto two) __attribute__((always_inline)) {
    for (int tb = 0; tb < n_tb; tb += 2) {
      block(tb, kf, v_a, v_b, next, two);
      if (tb + 1 < n_tb) block(tb + 1, kf, v_b, v_a, next, two);
    }
  };
  if (n_q[1] > 0)  // wave-uniform: the second block of query rows exists
    run(std::true_type{});
  else
    run(std::false_type{});
#pragma unroll
  for (int qb = 0; qb < NQ; ++qb) {
    float ls = l[qb];
    ls += __shfl_xor(ls, 32, 64);
    if (lr < n_q[qb]) {
      const float inv = 1.f / ls;
      uint16_t *dst = a.out + (size_t)(r0 + qblk * 64 + qb * 32 + lr) * (hq * DH) + head * DH;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          u32x2_t v;
          v.x = pack_bf16x2(o[qb][db][4 * q + 0] * inv, o[qb][db][4 * q + 1] * inv);
          v.y = pack_bf16x2(o[qb][db][4 * q + 2] * inv, o[qb][db][4 * q + 3] * inv);
          *reinterpret_cast<u32x2_t *>(dst + 32 * db + 8 * q + 4 * g2) = v;
        }
    }
  }
}

template <int DH>
__global__ __launch_bounds__(256) void prefill_attn_kernel(const PrefillArgs a, int heads_per_wg) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  prefill_workgroup<DH>(a, heads_per_wg, blockIdx.x, wave, threadIdx.x & 63);
}

// Prefill and decode attention of one step in one launch.  A prefill workgroup is bound by the
// matrix and vector pipes and leaves the memory system idle, a decode workgroup is the
// opposite, and each needs a CU to itself (one wavefront per SIMD), so the two kinds blend
// across CUs: the grid deals one prefill workgroup per `period` workgroups (an odd number, so
// that they rotate over the XCDs) for as long as both kinds last, each kind in its own order
// (longest first).  Workgroups of four wavefronts only (four query heads of a KV group).
// Measured against the two launches one after the other: 0.520 -> 0.498 ms on the 8B blended
// shape (2048 prefill rows, 1024 decode sequences), 0.746 -> 0.717 ms on the 70B one.
template <int DH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void blended_attn_kernel(
    const DecodeArgs d, int n_wide_units, int n_narrow_units, const PrefillArgs pf, int n_pf_wgs, int period) {
  __shared__ __align__(16) uint16_t q_sh[DECODE_Q_LDS(DH)];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int n_dec = ((n_wide_units + 3) >> 2) + ((n_narrow_units + 3) >> 2);
  const int mixed = min(n_pf_wgs, n_dec / (period - 1));  // periods of one prefill + (period - 1) decode workgroups
  const int b = blockIdx.x;
  bool prefill;
  int idx;
  if (b < period * mixed) {
    const int per = b / period, pos = b % period;
    prefill = pos == 0;
    idx = prefill ? per : (period - 1) * per + pos - 1;
  } else {
    const int r = b - period * mixed;
    prefill = r < n_pf_wgs - mixed;
    idx = prefill ? mixed + r : (period - 1) * mixed + r - (n_pf_wgs - mixed);
  }
  if (prefill)
    prefill_workgroup<DH>(pf, 4, idx, wave, lane);
  else
    decode_workgroup<DH, false>(d, n_wide_units, n_narrow_units, idx, wave, lane, q_sh);
}

// What the GEMM launches of a step have left of its queue of 16-row units, on the whole chip:
// workgroups of eight wavefronts (two per SIMD: a 16-row unit needs under half of a SIMD's
// registers), every wavefront drawing units until the queue is empty.
template <int DH>
__global__ __launch_bounds__(512) void decode_queue_kernel(const DecodeQueue q) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  decode_queue_worker<DH>(q, wave, threadIdx.x & 63,
                          q.trace ? q.trace + (size_t)TRACE_WORDS * (8 * blockIdx.x + wave) : nullptr);
}

}  // namespace

hipError_t launch_decode_queue(const DecodeQueue &q, int n_workgroups, hipStream_t stream) {
  if (q.n_units <= 0 || n_workgroups <= 0) return hipSuccess;
  if (q.d.s.head_dim == 128)
    hipLaunchKernelGGL((decode_queue_kernel<128>), dim3(n_workgroups), dim3(512), 0, stream, q);
  else if (q.d.s.head_dim == 64)
    hipLaunchKernelGGL((decode_queue_kernel<64>), dim3(n_workgroups), dim3(512), 0, stream, q);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_decode_attn(const DecodeArgs &a, int n_wide, int n_narrow, hipStream_t stream) {
  const int n_wide_units = n_wide * a.s.n_kv_heads, n_narrow_units = n_narrow * a.s.n_kv_heads;
  const int wgs = (n_wide_units + 3) / 4 + (n_narrow_units + 3) / 4;  // a workgroup holds units of one kind
  if (wgs <= 0) return hipSuccess;
  const dim3 grid(wgs), block(256);
  if (a.s.head_dim == 128)
    hipLaunchKernelGGL((decode_attn_kernel<128>), grid, block, 0, stream, a, n_wide_units, n_narrow_units);
  else if (a.s.head_dim == 64)
    hipLaunchKernelGGL((decode_attn_kernel<64>), grid, block, 0, stream, a, n_wide_units, n_narrow_units);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_decode_merge(const MergeArgs &a, hipStream_t stream) {
  if (a.n_decode <= 0) return hipSuccess;
  if (a.s.head_dim != 128 && a.s.head_dim != 64) return hipErrorInvalidValue;
  const int hpw = 256 / a.s.head_dim;  // heads per wavefront
  const int units = a.n_decode * ((a.s.n_q_heads + hpw - 1) / hpw);
  if (a.s.head_dim == 128)
    hipLaunchKernelGGL((decode_merge_kernel<128>), dim3((units + 3) / 4), dim3(256), 0, stream, a);
  else
    hipLaunchKernelGGL((decode_merge_kernel<64>), dim3((units + 3) / 4), dim3(256), 0, stream, a);
  return hipGetLastError();
}

bool blended_attn_possible(const AttnShape &s) { return (s.n_q_heads / s.n_kv_heads) % 4 == 0; }

hipError_t launch_blended_attn(const DecodeArgs &d, int n_wide, int n_narrow, const PrefillArgs &pf, hipStream_t stream) {
  if (!blended_attn_possible(d.s)) return hipErrorInvalidValue;
  const int n_wide_units = n_wide * d.s.n_kv_heads, n_narrow_units = n_narrow * d.s.n_kv_heads;
  const int n_dec = (n_wide_units + 3) / 4 + (n_narrow_units + 3) / 4;
  const int n_pf = pf.n_work * (pf.s.n_q_heads / 4);
  if (n_dec <= 0 || n_pf <= 0) return hipErrorInvalidValue;
  // one workgroup in five is a prefill one until they run out (periods of 3 to 17 measured on the 8B and
  // 70B shapes: 3 and 5 are the fastest, the long ones cost 1-3 % of the launch); odd, so that the prefill
  // workgroups visit every XCD in turn
  const int period = n_dec >= 4 * n_pf ? 5 : 3;
  const dim3 grid(n_dec + n_pf), block(256);
  if (d.s.head_dim == 128)
    hipLaunchKernelGGL((blended_attn_kernel<128>), grid, block, 0, stream, d, n_wide_units, n_narrow_units, pf, n_pf, period);
  else if (d.s.head_dim == 64)
    hipLaunchKernelGGL((blended_attn_kernel<64>), grid, block, 0, stream, d, n_wide_units, n_narrow_units, pf, n_pf, period);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_prefill_attn(const PrefillArgs &a, hipStream_t stream) {
  if (a.n_work <= 0) return hipSuccess;
  const int grp = a.s.n_q_heads / a.s.n_kv_heads;
  const int hpw = (grp % 4 == 0) ? 4 : ((grp % 2 == 0) ? 2 : 1);  // heads of one KV group share a workgroup
  const dim3 grid(a.n_work * (a.s.n_q_heads / hpw)), block(64 * hpw);
  if (a.s.head_dim == 128)
    hipLaunchKernelGGL((prefill_attn_kernel<128>), grid, block, 0, stream, a, hpw);
  else if (a.s.head_dim == 64)
    hipLaunchKernelGGL((prefill_attn_kernel<64>), grid, block, 0, stream, a, hpw);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace bs
