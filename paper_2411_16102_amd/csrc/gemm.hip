// bf16 "NT" GEMM  C[M,N] = A[M,K] * B[N,K]^T  for gfx950, fp32 accumulation on
// v_mfma_f32_16x16x32_bf16, tiles staged through LDS, fused epilogues.  (The chip lowers its
// clock under matrix load; at that limit the 16x16x32 shape, which moves fewer accumulator
// registers per flop, sustains 1.87 PFLOP/s on random operands where 32x32x16 sustains
// 1.7, and this kernel gained 10 to 24 % from the change.)
//
// Operand roles are swapped with respect to the usual picture: the weight rows
// feed the MFMA "A" operand and the activation rows the "B" operand, so an
// accumulator block holds C^T: a lane owns ONE activation row (m = lane % 16) and
// a run of four consecutive output features (n = 4 * (lane / 16) ..).  Every fused epilogue is then
// lane-local: the RMSNorm factor of a row is one scalar per lane, a RoPE pair
// (i, i + dh/2) and a SwiGLU (gate, up) pair sit in two accumulator blocks of the
// same lane, and results leave as 8-byte bf16x4 stores.
//
// Tiles travel global -> LDS directly (global_load_lds_dwordx4), so no VGPRs are spent
// on staging.  A k-tile is BK = 64 wide: a tile row is then one whole 128-byte cache
// line, which the memory pipeline delivers about 1.5 times faster than the two 64-byte
// halves fetched separately (measured: 41 against 26 B/clk/CU into LDS).  LDS is a ring
// of five 32 KB units, one unit holding the activation panel or the weight panel of one
// k-tile, so two and a half k-tiles fit in the 160 KB: while tile kt is multiplied,
// tile kt+1 has landed or is landing and the weight panel of tile kt+2 is in flight.
// (GEMMs of at most 256 rows use a second pipeline, DEEP in the kernel below: one row
// of tiles, a few slots for the activation panel and all other LDS for the weight
// panel, the two kinds of panel requested by different wavefronts.)  Rows are 128 B whose eight 16-byte chunks are XOR-swizzled with
// ((row >> 1) & 7): two consecutive rows fill the 256-byte bank row, so the swizzle
// must change every two rows for the ds_read_b128 of a fragment (16 rows by four chunk
// columns) to be conflict-free.  Waits on the LDS-DMA loads are placed by hand
// (s_waitcnt vmcnt + s_barrier); the compiler does not track them.
#include <algorithm>
#include "gemm.hpp"
#include "attn_device.hpp"
#include "common.hpp"

namespace bs {

// sixteen bytes of zeros: the source of tile chunks that lie beyond K
__device__ __align__(16) uint16_t g_gemm_zero_chunk[8];

namespace {

constexpr int BK = 64;      // k-extent of one k-tile: rows of 128 bytes
constexpr int NU = 5;       // LDS ring, in units of one operand panel of one k-tile
constexpr int XCDS = 8;

struct TileCoord { int tm, tn; };
struct Yes { static constexpr bool value = true; };
struct No { static constexpr bool value = false; };

// Workgroup ids are dealt round-robin to the 8 XCDs; give each XCD a contiguous
// range of tiles and walk that range in groups of GM tile rows, so the tiles in
// flight on one XCD share activation and weight panels in that XCD's L2.
__device__ __forceinline__ TileCoord map_tile(int pid, int n_tiles, int tiles_m, int tiles_n) {
  const int per = n_tiles / XCDS, rem = n_tiles % XCDS;
  const int xcd = pid % XCDS, idx = pid / XCDS;
  const int lin = xcd * per + (xcd < rem ? xcd : rem) + idx;
  constexpr int GM = 4;
  const int group = GM * tiles_n;
  const int g = lin / group;
  const int first_m = g * GM;
  const int gm = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
  const int in = lin - g * group;
  TileCoord t;
  t.tm = first_m + in % gm;
  t.tn = in / gm;
  return t;
}

__device__ __forceinline__ void store_bf16x4(uint16_t *p, float a, float b, float c, float d) {
  u32x2_t v;
  v.x = pack_bf16x2(a, b);
  v.y = pack_bf16x2(c, d);
  *reinterpret_cast<u32x2_t *>(p) = v;
}

// s_waitcnt immediate (gfx9 encoding): wait until at most `vm` vector-memory
// operations are outstanding and, if lgkm0, until all LDS reads have returned
constexpr int waitcnt_imm(int vm, bool lgkm0) {
  return (vm & 0xF) | ((vm >> 4) << 14) | 0x70 | (lgkm0 ? 0 : 0xF00);
}

// Shared tiles.  A launch of G persistent workgroups takes the tiles [0, n_dp) of the launch's
// tile order whole, workgroup w the tiles w, w + G, ...; the k-tiles of the other n_sk tiles
// form one line of n_sk * nk iterations that the first g_sk workgroups cut into equal
// consecutive ranges, so a tile at a cut is computed by two or more workgroups, each over a
// part of K.  Every such workgroup leaves its partial tile in the workspace and counts itself
// in; the one that arrives last adds the parts up (always in the order of their k-ranges,
// its own part re-read like the others, so the sum does not depend on who was last) and runs
// the epilogue.  Nobody waits for anybody.
struct SkPlan {
  int n_dp, n_sk, g_sk, nk;
  float *ws;      // [2 * G][BM * BN]: slot 2 w of workgroup w for its first segment, 2 w + 1 for its last
  unsigned *cnt;  // [n_sk] arrivals at each shared tile; zero between launches
};
struct SkSeg {
  int pid, kt0, kt1;  // tile, k-tiles [kt0, kt1)
  int j;              // index of the tile among the shared ones
  int parts;          // workgroups that hold a part of the tile (1: this one has all of it)
  int w_first;        // the first of them; they are consecutive
  int my_slot;
};
constexpr int SK_SNAP = 4;      // a cut this close to a tile boundary moves onto it
constexpr int SK_MIN_ITERS = 16;  // shortest range worth a workgroup of its own

// first iteration of workgroup w's range (w = g_sk: the end of the line)
__device__ __forceinline__ int sk_bound(const SkPlan &p, int w) {
  const int total = p.n_sk * p.nk;
  int b = (int)((long)total * w / p.g_sk);
  const int r = b % p.nk;
  if (r < SK_SNAP) b -= r;
  else if (p.nk - r < SK_SNAP) b += p.nk - r;
  return b;
}
// the workgroups whose ranges meet shared tile j
__device__ __forceinline__ void sk_tile_span(const SkPlan &p, int j, int *w_first, int *parts) {
  const int lo = j * p.nk, hi = lo + p.nk;
  int w = (int)((long)lo * p.g_sk / (p.n_sk * p.nk));
  while (w + 1 < p.g_sk && sk_bound(p, w + 1) <= lo) ++w;
  while (w > 0 && sk_bound(p, w) > lo) --w;
  int n = 1;
  while (w + n < p.g_sk && sk_bound(p, w + n) < hi) ++n;
  *w_first = w;
  *parts = n;
}

// One workgroup's tile; `bid` is the workgroup's number among the GEMM workgroups of the launch
// (SK: the tile and the k-range come from `seg` instead).
template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int DH, int DEEP = 0, bool SK = false>
__device__ __forceinline__ void gemm_tile(const GemmArgs &a, const int bid, const SkPlan *sp = nullptr, const SkSeg seg = SkSeg{}) {
  static_assert(!SK || (!DEEP && EPI != EPI_PARTIAL), "shared tiles use the five-panel ring and a real epilogue");
  constexpr int NW = WAVES_M * WAVES_N;
  // DEEP: the pipeline for one round of tiles over few rows, where every CU streams a weight
  // panel of its own from HBM; the first half of the wavefronts requests the activation
  // panels, the second half the weight panels (see the pipeline below)
  constexpr int XW = DEEP ? NW / 2 : NW, WW = DEEP ? NW / 2 : NW;  // wavefronts that share the loads of a panel
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  constexpr int MI = WTM / 16, NI = WTN / 16;  // 16x16 accumulator blocks of a wavefront's tile
  constexpr int OUT_BN = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  constexpr int ROWB = BK * 2;                       // bytes of one tile row
  constexpr int UNIT = (BM > BN ? BM : BN) * ROWB;   // one ring unit holds either panel
  constexpr int GA = BM / 8, GB = BN / 8;            // 8-row groups = one 1 KB wavefront load each
  constexpr int LA = (GA + XW - 1) / XW, LB = (GB + WW - 1) / WW;  // loads per thread per panel
  static_assert(!DEEP || NW % 2 == 0, "two halves of the workgroup share the loads");
  static_assert(BK == 64, "swizzle and fragment addressing assume 128-byte tile rows");
  static_assert(WTM % 16 == 0 && WTN % 16 == 0, "tiles are made of 16x16 MFMA blocks");
  static_assert(EPI != EPI_SWIGLU || WTN % 64 == 0, "32 gate rows and their 32 up rows pair up inside a wave");
  static_assert(EPI != EPI_QKV || (WTN % DH == 0 && DH % 64 == 0), "a wave covers whole heads");
  static_assert(2 * LA + 2 * LB < 64, "outstanding loads must fit the vmcnt field");

  extern __shared__ __align__(16) unsigned char smem[];

  const int n_lim = a.n_count ? a.n_begin + a.n_count : a.N;  // end of the output columns of this launch
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (n_lim - a.n_begin + OUT_BN - 1) / OUT_BN;
  // split-K: consecutive workgroups are the k-ranges of one tile
  const int split = (EPI == EPI_PARTIAL) ? bid % a.k_splits : 0;
  const int tile_id = SK ? seg.pid : (EPI == EPI_PARTIAL) ? bid / a.k_splits : bid;
  const TileCoord tc = map_tile(tile_id, tiles_m * tiles_n, tiles_m, tiles_n);
  const int m0 = tc.tm * BM, n0 = a.n_begin + tc.tn * OUT_BN;

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm0 = (wave / WAVES_N) * WTM, wn0 = (wave % WAVES_N) * WTN;
  const int lr = lane & 15, lg = lane >> 4;  // row of a 16-row block; k-chunk of a fragment, feature group of an accumulator

  // ---- global -> LDS, without passing through registers ---------------------------
  // One wavefront load moves 8 tile rows (1 KB): lane i lands at LDS byte 16 i of the
  // group, i.e. row i/8, 16-byte slot i%8, and fetches the chunk that the XOR swizzle
  // assigns to that slot, so the eight lanes of a row cover one whole cache line.  Rows
  // past the matrix edge are clamped to the last row (their accumulators are never
  // stored); chunks past K read a block of zeros instead.
  const int g_row = lane >> 3, g_slot = lane & 7;
  // byte offsets from the matrix base (the host checks that they fit 32 bits): the address
  // of a load is then a uniform 64-bit base, advanced per k-tile by scalar code, plus a
  // per-lane offset that never changes
  uint32_t off_a[LA], off_b[LB];
  int ka[LA], kb[LB];        // element offset of this lane's chunk inside a k-tile
  int dst_a[LA], dst_b[LB];  // LDS byte offset of the group inside a unit
#pragma unroll
  for (int i = 0; i < LA; ++i) {
    // when the groups do not divide over the wavefronts the surplus loads repeat the last
    // group (same bytes to the same place), so every wavefront issues LA loads per panel
    const int grp = (wave % XW + i * XW) < GA ? (wave % XW + i * XW) : GA - 1;
    const int row = grp * 8 + g_row;
    const int chunk = g_slot ^ ((row >> 1) & 7);
    ka[i] = chunk * 8;
    dst_a[i] = grp * 1024;
    int gm = m0 + row;
    gm = gm < a.M ? gm : a.M - 1;
    off_a[i] = (uint32_t)(((size_t)gm * a.lda + chunk * 8) * 2);
  }
#pragma unroll
  for (int i = 0; i < LB; ++i) {
    const int grp = (wave % WW + i * WW) < GB ? (wave % WW + i * WW) : GB - 1;
    const int wr = grp * 8 + g_row;
    const int chunk = g_slot ^ ((wr >> 1) & 7);
    kb[i] = chunk * 8;
    dst_b[i] = grp * 1024;
    int gn;
    if (EPI == EPI_SWIGLU) {
      const int blk = wr >> 5;
      int col = n0 + (blk >> 1) * 32 + (wr & 31);
      col = col < a.N ? col : a.N - 1;
      gn = col + ((blk & 1) ? a.N : 0);
    } else {
      gn = n0 + wr;
      gn = gn < a.N ? gn : a.N - 1;
    }
    off_b[i] = (uint32_t)(((size_t)gn * a.ldb + chunk * 8) * 2);
  }
  // load number i of panel X(kt) / W(kt) into ring slot `slot`; `checked` handles chunks past K
  auto dma_a = [&](int kt, int lds_off, int i, auto checked) {
    const unsigned char *base = reinterpret_cast<const unsigned char *>(a.A) + (size_t)kt * ROWB;
    const void *p = base + off_a[i];
    if constexpr (decltype(checked)::value)
      if (kt * BK + ka[i] >= a.K) p = g_gemm_zero_chunk;
    __builtin_amdgcn_global_load_lds(p, (__attribute__((address_space(3))) void *)(smem + lds_off + dst_a[i]), 16, 0, 0);
  };
  auto dma_b = [&](int kt, int lds_off, int i, auto checked) {
    const unsigned char *base = reinterpret_cast<const unsigned char *>(a.B) + (size_t)kt * ROWB;
    const void *p = base + off_b[i];
    if constexpr (decltype(checked)::value)
      if (kt * BK + kb[i] >= a.K) p = g_gemm_zero_chunk;
    __builtin_amdgcn_global_load_lds(p, (__attribute__((address_space(3))) void *)(smem + lds_off + dst_b[i]), 16, 0, 0);
  };

  f32x4_t acc[NI][MI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) acc[ni][mi] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // fragment addresses: tile row of the lane, chunk 4*ks + lg swizzled by ((row >> 1) & 7)
  const int sw = (lr >> 1) & 7;
  const int xfrag = (wm0 + lr) * ROWB;
  const int wfrag = (wn0 + lr) * ROWB;

  const int nk_all = (a.K + BK - 1) / BK;
  // this workgroup's k-tiles [kt0, kt1): all of them, or one of k_splits nearly equal ranges
  const int kt0 = SK ? seg.kt0 : (EPI == EPI_PARTIAL) ? (int)((long)nk_all * split / a.k_splits) : 0;
  const int kt1 = SK ? seg.kt1 : (EPI == EPI_PARTIAL) ? (int)((long)nk_all * (split + 1) / a.k_splits) : nk_all;
  constexpr int NF = MI + NI;   // fragment reads per 32-wide k-step
  constexpr int NMF = MI * NI;  // MFMAs per 32-wide k-step
  // read number o of k-step ks (32 wide, two per tile) of the panels in ring slots sa, sb
  // (xo, wo: LDS byte offsets of the two panels)
  auto frag = [&](int xo, int wo, int ks, int o, bf16x8_t (&xf)[MI], bf16x8_t (&wf)[NI]) {
    const int ch = ((ks * 4 + lg) ^ sw) << 4;
    if (o < MI)
      xf[o] = as_bf16x8(*reinterpret_cast<const u32x4_t *>(smem + xo + xfrag + o * 16 * ROWB + ch));
    else
      wf[o - MI] = as_bf16x8(*reinterpret_cast<const u32x4_t *>(smem + wo + wfrag + (o - MI) * 16 * ROWB + ch));
  };
  // One k-step: its NMF MFMAs in program order, with the `n_ops` side operations (LDS
  // reads of the next k-step, DMA requests) dealt out behind the first MFMAs, `per` at a
  // time, so that the matrix pipe is never left idle behind a run of memory instructions.
  auto step = [&](const bf16x8_t (&xf)[MI], const bf16x8_t (&wf)[NI], int n_ops, int per, auto &&op) {
#pragma unroll
    for (int j = 0; j < NMF; ++j) {
      const int ni = j / MI, mi = j % MI;
      acc[ni][mi] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[ni], xf[mi], acc[ni][mi], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int q = 0; q < per; ++q)
        if (j * per + q < n_ops) op(j * per + q);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto next_slot = [](int s, int by) { s += by; return s >= NU ? s - NU : s; };
  static_assert(NU == 5, "the pipeline below is written for a ring of five panels");
  // Software pipeline.  Panels are numbered in issue order, W(0) X(0) W(1) X(1) ..., and
  // panel u lives in ring slot u % 5.  Once the last fragments of tile kt are in
  // registers, at the one barrier of the iteration, X(kt+2) and W(kt+3) are requested
  // into the two slots that tile kt frees: the weight panel, which in a layer streams from
  // HBM, gets the two k-tiles of look-ahead, and the activation panel, which the previous
  // kernel has just left in the caches, gets one.  LDS -> registers: the fragments of the next
  // 32-wide k-step are requested while the MFMAs of the current one are issued, across
  // tile boundaries too, so the matrix pipe never waits for a whole LDS read phase.
  // The compiler counts an LDS-DMA load as a pending LDS operation of unknown order, so
  // every wait it places before an MFMA is lgkmcnt(0); waiting explicitly at the start of
  // a k-step, for reads issued during the first MFMAs of the previous one, keeps those
  // waits from covering reads that were only just issued.
  constexpr int LGKM0 = waitcnt_imm(63, true);
  constexpr int PER_F = (NF + NMF - 1) / NMF;  // side operations per MFMA: one is enough where a step has 32 MFMAs
  constexpr int N_P = NF + LB + LA;
  constexpr int PER_P = (N_P + NMF - 1) / NMF;
  (void)N_P; (void)PER_P;
  bf16x8_t xa[MI], wa[NI], xb[MI], wb[NI];
  if constexpr (!DEEP) {
#pragma unroll
    for (int i = 0; i < LB; ++i) dma_b(kt0, 0 * UNIT, i, Yes{});
#pragma unroll
    for (int i = 0; i < LA; ++i) dma_a(kt0, 1 * UNIT, i, Yes{});
#pragma unroll
    for (int i = 0; i < LB; ++i) dma_b(kt0 + 1, 2 * UNIT, i, Yes{});
#pragma unroll
    for (int i = 0; i < LA; ++i) dma_a(kt0 + 1, 3 * UNIT, i, Yes{});
#pragma unroll
    for (int i = 0; i < LB; ++i) dma_b(kt0 + 2, 4 * UNIT, i, Yes{});
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(2 * LB + LA, true));  // tile 0 has landed
    __builtin_amdgcn_s_barrier();
    int sb = 0, sa = 1;  // slots of the tile being multiplied: weights, activations
#pragma unroll
    for (int o = 0; o < NF; ++o) frag(sa * UNIT, sb * UNIT, 0, o, xa, wa);
    auto tile = [&](int kt, auto checked) {
      __builtin_amdgcn_s_waitcnt(LGKM0);
      step(xa, wa, NF, PER_F, [&](int o) { frag(sa * UNIT, sb * UNIT, 1, o, xb, wb); });
      // Every fragment of tile kt is in registers once the LDS reads have returned, and
      // tile kt+1 has landed once this wavefront's loads other than the youngest panel,
      // W(kt+2), are done; after the barrier both hold for every wavefront, so the two
      // slots of tile kt can be refilled and tile kt+1 can be read.
      __builtin_amdgcn_s_waitcnt(waitcnt_imm(LB, true));
      __builtin_amdgcn_s_barrier();
      const int na = next_slot(sa, 2), nb = next_slot(sb, 2);
      step(xb, wb, N_P, PER_P, [&](int o) {
        if (o < NF)
          frag(na * UNIT, nb * UNIT, 0, o, xa, wa);
        else if (o < NF + LA)
          dma_a(kt + 2, sb * UNIT, o - NF, checked);
        else
          dma_b(kt + 3, sa * UNIT, o - NF - LA, checked);
      });
      sa = na;
      sb = nb;
    };
    int kt = kt0;
    const int n_plain = a.K / BK - 3;  // tiles kt for which X(kt+2) and W(kt+3) lie wholly inside K
    for (; kt < n_plain && kt < kt1; ++kt) tile(kt, No{});
    for (; kt < kt1; ++kt) tile(kt, Yes{});
  } else {
    // One round of tiles over few rows: every CU streams a weight panel of its own from HBM,
    // and the ring of five equal slots gives it two k-tiles of look-ahead at most.  Here LDS
    // holds NXS = DEEP + 1 slots for the activation panel (shared by all tiles, served by the
    // L2: NXS - 1 k-tiles of look-ahead) and all the rest, NWS slots, for the weight panel:
    // NWS - 1 k-tiles of look-ahead.  The memory counter of a wavefront retires its loads in
    // order, so a wait for an activation panel would also wait for every weight panel
    // requested before it; the two kinds of request therefore come from different wavefronts:
    // the first half of the workgroup loads activations and waits until its NXS - 2 youngest
    // panels remain, the second half loads weights and waits until its NWS - 2 youngest remain.
    constexpr int NXS = DEEP + 1;  // activation slots
    constexpr int UX = BM * ROWB, UW = BN * ROWB, W_BASE = NXS * UX;
    constexpr int NWS = (160 * 1024 - W_BASE) / UW;
    static_assert(NWS >= 3 && (NWS - 1) * LB < 64 && (NXS - 1) * LA < 64, "slots and the vmcnt field");
    const bool loads_x = wave < XW;  // uniform
    if (loads_x) {
#pragma unroll
      for (int sl = 0; sl < NXS; ++sl)
#pragma unroll
        for (int i = 0; i < LA; ++i) dma_a(kt0 + sl, sl * UX, i, Yes{});
      __builtin_amdgcn_s_waitcnt(waitcnt_imm((NXS - 1) * LA, true));
    } else {
#pragma unroll
      for (int sl = 0; sl < NWS; ++sl)
#pragma unroll
        for (int i = 0; i < LB; ++i) dma_b(kt0 + sl, W_BASE + sl * UW, i, Yes{});
      __builtin_amdgcn_s_waitcnt(waitcnt_imm((NWS - 1) * LB, true));
    }
    __builtin_amdgcn_s_barrier();  // tile 0 has landed
    int xs = 0, ws = 0;            // activation and weight slot numbers of the tile being multiplied
#pragma unroll
    for (int o = 0; o < NF; ++o) frag(xs * UX, W_BASE + ws * UW, 0, o, xa, wa);
    constexpr int N_X = NF + LA, N_W = NF + LB;
    constexpr int PER_X = (N_X + NMF - 1) / NMF, PER_W = (N_W + NMF - 1) / NMF;
    auto tile = [&](int kt, auto checked) {
      const int wo = W_BASE + ws * UW, xo = xs * UX;
      __builtin_amdgcn_s_waitcnt(LGKM0);
      step(xa, wa, NF, PER_F, [&](int o) { frag(xo, wo, 1, o, xb, wb); });
      // after the barrier: every wavefront holds all fragments of tile kt, X(kt+1) has landed
      // (the activation half waited until only X(kt+2) .. X(kt+NXS-1) were outstanding) and so
      // has W(kt+1) (the weight half: only W(kt+2) .. W(kt+NWS-1))
      if (loads_x)
        __builtin_amdgcn_s_waitcnt(waitcnt_imm((NXS - 2) * LA, true));
      else
        __builtin_amdgcn_s_waitcnt(waitcnt_imm((NWS - 2) * LB, true));
      __builtin_amdgcn_s_barrier();
      const int nxs = xs + 1 == NXS ? 0 : xs + 1, nws = ws + 1 == NWS ? 0 : ws + 1;
      const int nxo = nxs * UX;
      const int nwo = W_BASE + nws * UW;
      if (loads_x)
        step(xb, wb, N_X, PER_X, [&](int o) {
          if (o < NF)
            frag(nxo, nwo, 0, o, xa, wa);
          else
            dma_a(kt + NXS, xo, o - NF, checked);
        });
      else
        step(xb, wb, N_W, PER_W, [&](int o) {
          if (o < NF)
            frag(nxo, nwo, 0, o, xa, wa);
          else
            dma_b(kt + NWS, wo, o - NF, checked);
        });
      xs = nxs;
      ws = nws;
    };
    int kt = kt0;
    const int n_plain = a.K / BK - (NWS > NXS ? NWS : NXS);  // tiles kt for which X(kt+NXS) and W(kt+NWS) lie wholly inside K
    for (; kt < n_plain && kt < kt1; ++kt) tile(kt, No{});
    for (; kt < kt1; ++kt) tile(kt, Yes{});
  }
  // drain the look-ahead loads (zeros or clamped rows) before the LDS is released
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, true));
  // the value heads of the fused projection pass through LDS on their way out: nobody may
  // still be reading panels there
  if (EPI == EPI_QKV) __syncthreads();

  if constexpr (SK) {
    if (seg.parts > 1) {
      constexpr int NT = NW * 64;
      constexpr size_t TILE = (size_t)BM * BN;
      // The register image of the accumulators, 16 bytes per thread and block (whoever adds the
      // parts up has the same layout).  The eight XCDs keep L2 caches of their own, so parts
      // written and read with ordinary accesses would need the whole-cache write-back and
      // invalidation of a device-wide fence at every cut (measured: a quarter of a millisecond
      // per launch); the parts travel with the device-scope cache policy instead (sc1: to and
      // from the point where all XCDs agree), which touches nothing else.
      typedef unsigned int u4_t __attribute__((ext_vector_type(4)));
      constexpr int SC1 = 16;
      const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(sp->ws, 0, 0x7fffffff, 0x00020000);
      const unsigned voff = (unsigned)t * 16u;
      {
        const unsigned soff = (unsigned)seg.my_slot * (unsigned)(TILE * 4);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
          for (int mi = 0; mi < MI; ++mi) {
            const f32x4_t c = acc[ni][mi];
            const u4_t v = {__float_as_uint(c[0]), __float_as_uint(c[1]), __float_as_uint(c[2]), __float_as_uint(c[3])};
            __builtin_amdgcn_raw_buffer_store_b128(v, rs, voff + (unsigned)((ni * MI + mi) * NT * 16), soff, SC1);
          }
      }
      __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, true));  // the part has arrived there before the workgroup counts itself in
      __syncthreads();
      volatile unsigned *flag = reinterpret_cast<volatile unsigned *>(smem + NU * UNIT - 16);
      if (t == 0) *flag = atomicAdd(sp->cnt + seg.j, 1u);
      __syncthreads();
      if (*flag + 1u != (unsigned)seg.parts) return;
      if (t == 0) atomicExch(sp->cnt + seg.j, 0u);  // as the next launch expects it
      for (int q = 0; q < seg.parts; ++q) {
        const int w2 = seg.w_first + q;
        const int slot = 2 * w2 + (sk_bound(*sp, w2) / sp->nk == seg.j ? 0 : 1);
        const unsigned soff = (unsigned)slot * (unsigned)(TILE * 4);
        // sixteen blocks at a time: the loads of a batch are all in flight before the first is
        // used (each is a round trip past the L2; the registers of the fragments are free now)
        constexpr int NB = NI * MI, BATCH = NB < 16 ? NB : 16;
        static_assert(NB % BATCH == 0, "whole batches");
#pragma unroll
        for (int b0 = 0; b0 < NB; b0 += BATCH) {
          u4_t v[BATCH];
#pragma unroll
          for (int b = 0; b < BATCH; ++b)
            v[b] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff + (unsigned)((b0 + b) * NT * 16), soff, SC1);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int b = 0; b < BATCH; ++b) {
            const int ni = (b0 + b) / MI, mi = (b0 + b) % MI;
            const f32x4_t c = {__uint_as_float(v[b].x), __uint_as_float(v[b].y), __uint_as_float(v[b].z), __uint_as_float(v[b].w)};
            acc[ni][mi] = q == 0 ? c : acc[ni][mi] + c;
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  }

  // ---- epilogues ---------------------------------------------------------------
  // accumulator element e of block (ni, mi): m = m0 + wm0 + mi*16 + lr,
  // n = n_tile + wn0 + ni*16 + 4*lg + e
  // A tile that lies wholly inside the matrix takes a copy of the epilogue without bounds
  // checks: straight-line code whose loads all go out together; with the checks every
  // block is a basic block of its own and the epilogue becomes a chain of memory round trips.
  auto epilogue = [&](auto checked) {
    constexpr bool CK = decltype(checked)::value;
    float rstd[MI];
    if (EPI == EPI_QKV || EPI == EPI_SWIGLU) {
  #pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const int m = m0 + wm0 + mi * 16 + lr;
        rstd[mi] = (!CK || m < a.M) ? a.rstd[m] : 0.f;
      }
    }

    if (EPI == EPI_PARTIAL) {
      float *ws = a.splitk_ws + (size_t)split * a.M * a.N;
  #pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const int m = m0 + wm0 + mi * 16 + lr;
        if (CK && m >= a.M) continue;
  #pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
          const int n = n0 + wn0 + ni * 16 + 4 * lg;
          if (CK && n >= a.N) continue;
          *reinterpret_cast<f32x4_t *>(ws + (size_t)m * a.N + n) = acc[ni][mi];
        }
      }
    }

    if (EPI == EPI_PLAIN || EPI == EPI_RESID) {
  #pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const int m = m0 + wm0 + mi * 16 + lr;
        if (CK && m >= a.M) continue;
  #pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
          const int n = n0 + wn0 + ni * 16 + 4 * lg;
          if (CK && n >= n_lim) continue;
          float v[4];
  #pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = acc[ni][mi][e];
          if (EPI == EPI_RESID) {
            if (a.resid32) {
              const f32x4_t rr = *reinterpret_cast<const f32x4_t *>(a.resid32 + (size_t)m * a.ldr + n);
  #pragma unroll
              for (int e = 0; e < 4; ++e) v[e] += rr[e];
            } else {
              const u32x2_t rr = *reinterpret_cast<const u32x2_t *>(a.resid + (size_t)m * a.ldr + n);
              v[0] += __uint_as_float(rr.x << 16);
              v[1] += __uint_as_float(rr.x & 0xFFFF0000u);
              v[2] += __uint_as_float(rr.y << 16);
              v[3] += __uint_as_float(rr.y & 0xFFFF0000u);
            }
          }
          store_bf16x4(a.C + (size_t)m * a.ldc + n, v[0], v[1], v[2], v[3]);
        }
      }
    }

    if (EPI == EPI_RESID_NORM) {
  #pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const int m = m0 + wm0 + mi * 16 + lr;
        float ss = 0.f;
        if (!CK || m < a.M) {
  #pragma unroll
          for (int ni = 0; ni < NI; ++ni) {
            const int n = n0 + wn0 + ni * 16 + 4 * lg;
            if (CK && n >= a.N) continue;
            const u32x2_t rr = *reinterpret_cast<const u32x2_t *>(a.resid + (size_t)m * a.ldr + n);
            const u32x2_t gg = *reinterpret_cast<const u32x2_t *>(a.gain + n);
            float v[4], g[4];
            v[0] = acc[ni][mi][0] + __uint_as_float(rr.x << 16);
            v[1] = acc[ni][mi][1] + __uint_as_float(rr.x & 0xFFFF0000u);
            v[2] = acc[ni][mi][2] + __uint_as_float(rr.y << 16);
            v[3] = acc[ni][mi][3] + __uint_as_float(rr.y & 0xFFFF0000u);
            g[0] = __uint_as_float(gg.x << 16);
            g[1] = __uint_as_float(gg.x & 0xFFFF0000u);
            g[2] = __uint_as_float(gg.y << 16);
            g[3] = __uint_as_float(gg.y & 0xFFFF0000u);
  #pragma unroll
            for (int e = 0; e < 4; ++e) ss += v[e] * v[e];
            // x1 stays in fp32 for the second residual add; the next GEMM reads bf16(x1 * gain)
            *reinterpret_cast<f32x4_t *>(a.C32 + (size_t)m * a.ldc + n) = f32x4_t{v[0], v[1], v[2], v[3]};
            store_bf16x4(a.C_gain + (size_t)m * a.ldc + n, v[0] * g[0], v[1] * g[1], v[2] * g[2], v[3] * g[3]);
          }
        }
        // the four lanes that share the row (lg = 0..3) add up: one partial sum per wavefront column
        ss += __shfl_xor(ss, 16, 64);
        ss += __shfl_xor(ss, 32, 64);
        if (lg == 0 && (!CK || m < a.M))
          a.ss_out[(size_t)(tc.tn * WAVES_N + (wave % WAVES_N)) * a.ss_stride + m] = ss;
      }
    }

    if (EPI == EPI_SWIGLU) {
      // the weight tile interleaves 32 gate rows with the matching 32 up rows: blocks 4p, 4p+1 are
      // gate features 32p .. 32p+31 of the wavefront, blocks 4p+2, 4p+3 their up features
  #pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const int m = m0 + wm0 + mi * 16 + lr;
        if (CK && m >= a.M) continue;
        const float s = rstd[mi];
  #pragma unroll
        for (int p = 0; p < NI / 4; ++p)
  #pragma unroll
          for (int h = 0; h < 2; ++h) {
            const int n = n0 + (wn0 >> 1) + p * 32 + h * 16 + 4 * lg;
            if (CK && n >= n_lim) continue;
            float v[4];
  #pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float g = acc[4 * p + h][mi][e] * s;
              const float u = acc[4 * p + 2 + h][mi][e] * s;
              v[e] = g / (1.f + __expf(-g)) * u;
            }
            store_bf16x4(a.C + (size_t)m * a.ldc + n, v[0], v[1], v[2], v[3]);
          }
      }
    }

    if (EPI == EPI_QKV) {
      constexpr int HB = DH / 16, PB = HB / 2, HALF = DH / 2;
      constexpr int FS = (WTM + 4) * 2;  // bytes per feature of a wavefront's transposed block
      static_assert(NW * WTN * FS <= NU * UNIT, "the transposed blocks fit the panel ring");
      const size_t tile_elems = (size_t)16 * DH;  // one K or V tile of a (page, head)
  #pragma unroll
      for (int hh = 0; hh < WTN / DH; ++hh) {
        const int nh = n0 + wn0 + hh * DH;
        if (CK && nh >= a.N) continue;
        const int head = nh / DH;
        const bool is_q = head < a.n_q_heads;
        const bool is_k = !is_q && head < a.n_q_heads + a.n_kv_heads;
  #pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
          const int m = m0 + wm0 + mi * 16 + lr;
          if (CK && m >= a.M) continue;
          const float s = rstd[mi];
          if (is_q || is_k) {
            const int pos = a.row_pos[m];
            uint16_t *dst;
            if (is_q) {
              dst = a.q_out + (size_t)m * (a.n_q_heads * DH) + head * DH;
            } else {
              const size_t page = a.row_page[m];
              dst = a.kv_pool + ((page * 2 + 0) * a.n_kv_heads + (head - a.n_q_heads)) * tile_elems +
                    (size_t)a.row_slot[m] * DH;
            }
  #pragma unroll
            for (int j = 0; j < PB; ++j) {
              const int i = j * 16 + 4 * lg;
              const f32x4_t c4 = *reinterpret_cast<const f32x4_t *>(a.rope_cos + (size_t)pos * HALF + i);
              const f32x4_t s4 = *reinterpret_cast<const f32x4_t *>(a.rope_sin + (size_t)pos * HALF + i);
              float lo[4], hi[4];
  #pragma unroll
              for (int e = 0; e < 4; ++e) {
                const float l = acc[hh * HB + j][mi][e] * s;
                const float h = acc[hh * HB + PB + j][mi][e] * s;
                lo[e] = l * c4[e] - h * s4[e];
                hi[e] = h * c4[e] + l * s4[e];
              }
              store_bf16x4(dst + i, lo[0], lo[1], lo[2], lo[3]);
              store_bf16x4(dst + HALF + i, hi[0], hi[1], hi[2], hi[3]);
            }
          } else {
            // V^T tiles hold, per feature, the 16 slots of a page side by side, while a lane
            // holds four features of one row: the wavefront turns its block round in LDS
            // (feature-major, FS bytes per feature: the row count padded so that neither the
            // 2-byte writes nor the 8-byte reads below collide on banks)
            unsigned char *vt = smem + wave * (WTN * FS) + hh * (DH * FS);
  #pragma unroll
            for (int b = 0; b < HB; ++b)
  #pragma unroll
              for (int e = 0; e < 4; ++e)
                *reinterpret_cast<uint16_t *>(vt + (b * 16 + 4 * lg + e) * FS + (mi * 16 + lr) * 2) =
                    f32_to_bf16(acc[hh * HB + b][mi][e] * s);
          }
        }
        if (!is_q && !is_k) {
          // back out of LDS (written and read by this wavefront only): lane = 4 * feature + quad
          // reads rows 4 quad .. 4 quad + 3 of a 16-row block for one feature.  Inside a prefill
          // segment these are four adjacent slots of one page, and the 64 lanes then cover 512
          // contiguous bytes of the page's V^T tile; they go out as one 8-byte store (or two
          // 4-byte ones) where the address allows.  Rows of different sequences, or on either
          // side of a page boundary, take a 2-byte store each.
          __builtin_amdgcn_wave_barrier();  // the LDS operations of a wavefront complete in order
          const unsigned char *vt = smem + wave * (WTN * FS) + hh * (DH * FS);
          const int vh = head - a.n_q_heads - a.n_kv_heads;
          const int fl = lane >> 2, rq = lane & 3;
  #pragma unroll
          for (int mi = 0; mi < MI; ++mi) {
            const int ml = mi * 16 + rq * 4, mb = m0 + wm0 + ml;
            size_t pg[4];
            int sl[4];
  #pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int m = (!CK || mb + e < a.M) ? mb + e : a.M - 1;
              pg[e] = a.row_page[m];
              sl[e] = a.row_slot[m];
            }
            bool run = !CK || mb + 3 < a.M;
  #pragma unroll
            for (int e = 1; e < 4; ++e) run = run && pg[e] == pg[0] && sl[e] == sl[0] + e;
  #pragma unroll
            for (int b = 0; b < HB; ++b) {
              const int ei = b * 16 + fl;
              const u32x2_t v = *reinterpret_cast<const u32x2_t *>(vt + ei * FS + ml * 2);
              uint16_t *d0 = a.kv_pool + ((pg[0] * 2 + 1) * a.n_kv_heads + vh) * tile_elems + ei * 16 + sl[0];
              if (run && (reinterpret_cast<uintptr_t>(d0) & 7) == 0) {
                *reinterpret_cast<u32x2_t *>(d0) = v;
              } else if (run && (reinterpret_cast<uintptr_t>(d0) & 3) == 0) {
                reinterpret_cast<uint32_t *>(d0)[0] = v.x;
                reinterpret_cast<uint32_t *>(d0)[1] = v.y;
              } else {
                const uint16_t ve[4] = {(uint16_t)(v.x & 0xFFFFu), (uint16_t)(v.x >> 16), (uint16_t)(v.y & 0xFFFFu),
                                        (uint16_t)(v.y >> 16)};
  #pragma unroll
                for (int e = 0; e < 4; ++e)
                  if (!CK || mb + e < a.M)
                    a.kv_pool[((pg[e] * 2 + 1) * a.n_kv_heads + vh) * tile_elems + ei * 16 + sl[e]] = ve[e];
              }
            }
          }
        }
      }
    }
  };
  if (m0 + BM <= a.M && n0 + OUT_BN <= n_lim && (EPI != EPI_QKV || n0 + BN <= a.N))
    epilogue(No{});
  else
    epilogue(Yes{});
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int DH, int DEEP = 0>
__global__ __launch_bounds__(WAVES_M *WAVES_N * 64) void gemm_kernel(const GemmArgs a) {
  gemm_tile<BM, BN, WAVES_M, WAVES_N, EPI, DH, DEEP>(a, (int)blockIdx.x);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int DH>
__global__ __launch_bounds__(WAVES_M *WAVES_N * 64) void gemm_sk_kernel(const GemmArgs a, const SkPlan p) {
  const int w = (int)blockIdx.x, G = (int)gridDim.x;
  int pid = w;
  int i = 0, i1 = 0, j0 = 0;
  if (w < p.g_sk) {
    i = sk_bound(p, w);
    i1 = sk_bound(p, w + 1);
    j0 = i / p.nk;
  }
  bool again = false;
  for (;;) {
    SkSeg s;
    if (pid < p.n_dp) {
      s = SkSeg{pid, 0, p.nk, 0, 1, 0, 0};
      pid += G;
    } else if (i < i1) {
      const int j = i / p.nk, kt0 = i - j * p.nk;
      const int kt1 = (i1 - j * p.nk) < p.nk ? (i1 - j * p.nk) : p.nk;
      s = SkSeg{p.n_dp + j, kt0, kt1, j, 1, 0, 0};
      if (kt0 > 0 || kt1 < p.nk) {
        sk_tile_span(p, j, &s.w_first, &s.parts);
        s.my_slot = 2 * w + (j == j0 ? 0 : 1);
      }
      i = j * p.nk + kt1;
    } else {
      break;
    }
    if (again) __syncthreads();  // the panel ring and the flag word change hands
    again = true;
    gemm_tile<BM, BN, WAVES_M, WAVES_N, EPI, DH, 0, true>(a, 0, &p, s);
  }
}

// A GEMM launch that carries decode attention (Section 3.3: a step whose compute-bound and
// memory-bound operators overlap costs the larger of their times; Section 2.2, operator-level
// overlapping).  Grid: `head` attention workgroups, the GEMM tiles, `tail` attention
// workgroups.  A workgroup of either kind takes a whole CU (the tile all of its LDS, either
// kind half of every SIMD's registers per wavefront), so the two kinds never share one: the
// head workgroups hold their CUs for as long as the GEMM runs and stream KV pages beside it,
// the tail workgroups start on the CUs that the last, partly filled round of tiles leaves
// idle.  The attention wavefronts draw 16-row units from the step's queue; the tile that
// brings the count of finished tiles to `close_at` closes the queue for this launch and
// hands its position to the next one, so nobody starts a unit that would outlast the GEMM
// by more than its own length.  No workgroup ever waits for another.
template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int DH, int ADH>
__global__ __launch_bounds__(WAVES_M *WAVES_N * 64) void gemm_attn_kernel(const GemmArgs a, const GemmRide r, const int n_tiles,
                                                                              const unsigned close_at) {
  static_assert(WAVES_M * WAVES_N == 8, "attention workgroups are written for eight wavefronts");
  const int b = (int)blockIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint64_t *rec = r.q.trace ? r.q.trace + (size_t)TRACE_WORDS * (8 * b + wave) : nullptr;
  if (b < r.head || b >= r.head + n_tiles) {
    attn_dev::decode_queue_worker<ADH>(r.q, wave, threadIdx.x & 63, rec);
    return;
  }
  const uint64_t t0 = rec ? wall_clock64() : 0;
  gemm_tile<BM, BN, WAVES_M, WAVES_N, EPI, DH>(a, b - r.head);
  if (threadIdx.x == 0) {
    const unsigned before = atomicAdd(r.done, 1u);
    if (before + 1 == close_at) {
      const unsigned pos = atomicAdd(r.q.ticket, DECODE_QUEUE_CLOSED);
      const unsigned capped = pos < (unsigned)r.q.n_units ? pos : (unsigned)r.q.n_units;
      atomicExch(r.ticket_next, capped);
      if (r.closed_at) *r.closed_at = capped;
    }
    if (rec) attn_dev::trace_record(rec, t0, TRACE_TILE, before + 1 == close_at ? 1u : 0u, 0u);
  }
}

constexpr int MAX_SPLITS = 8;

// four consecutive columns of one row, summed over the k-ranges in a fixed order; the loads are
// independent of one another and go out together
__device__ __forceinline__ f32x4_t splitk_sum(const float *p, size_t plane, int k_splits) {
  f32x4_t part[MAX_SPLITS];
#pragma unroll
  for (int s = 0; s < MAX_SPLITS; ++s)
    part[s] = s < k_splits ? *reinterpret_cast<const f32x4_t *>(p + s * plane) : f32x4_t{0.f, 0.f, 0.f, 0.f};
  f32x4_t v = part[0];
#pragma unroll
  for (int s = 1; s < MAX_SPLITS; ++s) v += part[s];
  return v;
}

// Second half of a split-K product: adds the k_splits partial rows and applies the epilogue.
// RESID: y = resid + sum, one thread per four columns.
__global__ __launch_bounds__(256) void splitk_reduce_resid_kernel(const GemmArgs a) {
  const int m = blockIdx.x, n = (blockIdx.y * 256 + threadIdx.x) * 4;
  if (n >= a.N) return;
  f32x4_t v = splitk_sum(a.splitk_ws + (size_t)m * a.N + n, (size_t)a.M * a.N, a.k_splits);
  if (a.resid32) {
    v += *reinterpret_cast<const f32x4_t *>(a.resid32 + (size_t)m * a.ldr + n);
  } else {
    const u32x2_t rr = *reinterpret_cast<const u32x2_t *>(a.resid + (size_t)m * a.ldr + n);
    v[0] += __uint_as_float(rr.x << 16);
    v[1] += __uint_as_float(rr.x & 0xFFFF0000u);
    v[2] += __uint_as_float(rr.y << 16);
    v[3] += __uint_as_float(rr.y & 0xFFFF0000u);
  }
  store_bf16x4(a.C + (size_t)m * a.ldc + n, v[0], v[1], v[2], v[3]);
}

// RESID_NORM: x1 = resid + sum in fp32, bf16(x1 * gain), and the row's sum of squares, complete,
// in ss_out slot 0; one workgroup per row.
__global__ __launch_bounds__(256) void splitk_reduce_resid_norm_kernel(const GemmArgs a) {
  const int m = blockIdx.x;
  float ss = 0.f;
  for (int n = threadIdx.x * 4; n < a.N; n += 256 * 4) {
    f32x4_t v = splitk_sum(a.splitk_ws + (size_t)m * a.N + n, (size_t)a.M * a.N, a.k_splits);
    const u32x2_t rr = *reinterpret_cast<const u32x2_t *>(a.resid + (size_t)m * a.ldr + n);
    v[0] += __uint_as_float(rr.x << 16);
    v[1] += __uint_as_float(rr.x & 0xFFFF0000u);
    v[2] += __uint_as_float(rr.y << 16);
    v[3] += __uint_as_float(rr.y & 0xFFFF0000u);
    const u32x2_t gg = *reinterpret_cast<const u32x2_t *>(a.gain + n);
    const float g0 = __uint_as_float(gg.x << 16), g1 = __uint_as_float(gg.x & 0xFFFF0000u);
    const float g2 = __uint_as_float(gg.y << 16), g3 = __uint_as_float(gg.y & 0xFFFF0000u);
    ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
    *reinterpret_cast<f32x4_t *>(a.C32 + (size_t)m * a.ldc + n) = v;
    store_bf16x4(a.C_gain + (size_t)m * a.ldc + n, v[0] * g0, v[1] * g1, v[2] * g2, v[3] * g3);
  }
  __shared__ float part[4];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  if (threadIdx.x == 0) {
    const float row = (part[0] + part[1]) + (part[2] + part[3]);
    a.ss_out[m] = row;
    if (a.rstd_out) a.rstd_out[m] = rsqrtf(row / (float)a.N + a.rstd_eps);
  }
}

// QKV: scale by the row's RMSNorm factor, rotate the q and k heads (pairs i, i + dh/2), store q
// to its buffer, k and v into the row's page slot (v transposed).  One thread per four
// consecutive pairs (q and k heads) or four consecutive v elements.
__global__ __launch_bounds__(256) void splitk_reduce_qkv_kernel(const GemmArgs a, int dh) {
  const int m = blockIdx.x;
  const int item = blockIdx.y * 256 + threadIdx.x;
  const size_t plane = (size_t)a.M * a.N;
  const float *ws = a.splitk_ws + (size_t)m * a.N;
  const float rs = a.rstd[m];
  const int half = dh / 2, q4 = half / 4;
  const size_t page = a.row_page[m];
  const int slot = a.row_slot[m];
  const size_t tile_elems = (size_t)16 * dh;
  const int n_rot = (a.n_q_heads + a.n_kv_heads) * q4;
  if (item < n_rot) {
    const int head = item / q4, i = (item % q4) * 4, pos = a.row_pos[m];
    const f32x4_t l = splitk_sum(ws + head * dh + i, plane, a.k_splits) * rs;
    const f32x4_t h = splitk_sum(ws + head * dh + half + i, plane, a.k_splits) * rs;
    const f32x4_t c = *reinterpret_cast<const f32x4_t *>(a.rope_cos + (size_t)pos * half + i);
    const f32x4_t sn = *reinterpret_cast<const f32x4_t *>(a.rope_sin + (size_t)pos * half + i);
    uint16_t *dst = head < a.n_q_heads
                        ? a.q_out + (size_t)m * (a.n_q_heads * dh) + head * dh
                        : a.kv_pool + ((page * 2 + 0) * a.n_kv_heads + (head - a.n_q_heads)) * tile_elems + (size_t)slot * dh;
    const f32x4_t lo = l * c - h * sn, hi = h * c + l * sn;
    store_bf16x4(dst + i, lo[0], lo[1], lo[2], lo[3]);
    store_bf16x4(dst + half + i, hi[0], hi[1], hi[2], hi[3]);
  } else if (item < n_rot + a.n_kv_heads * (dh / 4)) {
    const int w = (item - n_rot) * 4, head = w / dh, e = w % dh;
    const f32x4_t v = splitk_sum(ws + (a.n_q_heads + a.n_kv_heads) * dh + w, plane, a.k_splits) * rs;
    uint16_t *dst = a.kv_pool + ((page * 2 + 1) * a.n_kv_heads + head) * tile_elems + slot;
#pragma unroll
    for (int j = 0; j < 4; ++j) dst[(e + j) * 16] = f32_to_bf16(v[j]);
  }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int DH, int DEEP = 0>
hipError_t launch_one(const GemmArgs &a, hipStream_t stream) {
  constexpr int OUT_BN = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  constexpr int LDS = DEEP ? 160 * 1024 : NU * (BM > BN ? BM : BN) * BK * 2;
  auto kern = gemm_kernel<BM, BN, WAVES_M, WAVES_N, EPI, DH, DEEP>;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int n_cols = a.n_count ? a.n_count : a.N;
  const int tiles = ((a.M + BM - 1) / BM) * ((n_cols + OUT_BN - 1) / OUT_BN) * (EPI == EPI_PARTIAL ? a.k_splits : 1);
  if (tiles <= 0) return hipSuccess;
  hipLaunchKernelGGL(kern, dim3(tiles), dim3(WAVES_M * WAVES_N * 64), LDS, stream, a);
  return hipGetLastError();
}

constexpr int SK_MAX_G = 256;  // workgroups of a shared-tile launch at most: one per CU

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int DH>
hipError_t launch_sk(const GemmArgs &a, hipStream_t stream) {
  constexpr int OUT_BN = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  constexpr int LDS = NU * (BM > BN ? BM : BN) * BK * 2;
  static_assert(BM == 256 && BN == 256, "the workspace slots are sized for 256x256 tiles");
  if (!a.sk_ws || !a.sk_cnt || a.n_count || a.k_splits > 1) return hipErrorInvalidValue;
  auto kern = gemm_sk_kernel<BM, BN, WAVES_M, WAVES_N, EPI, DH>;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const long tiles = (long)((a.M + BM - 1) / BM) * ((a.N + OUT_BN - 1) / OUT_BN);
  if (tiles <= 0) return hipSuccess;
  const int G = a.n_cu > 0 && a.n_cu < SK_MAX_G ? a.n_cu : SK_MAX_G;
  SkPlan p{};
  p.nk = (a.K + BK - 1) / BK;
  p.ws = a.sk_ws;
  p.cnt = a.sk_cnt;
  if (tiles % G == 0) {
    p.n_dp = (int)tiles;
  } else {
    // (with more than one round the last whole round is shared too: every workgroup then has more
    // than a tile's worth of iterations and at most two cuts)
    p.n_sk = tiles > G ? (int)(tiles % G) + G : (int)tiles;
    p.n_dp = (int)tiles - p.n_sk;
    const long total = (long)p.n_sk * p.nk;
    p.g_sk = (int)std::min<long>(G, std::max<long>(1, total / SK_MIN_ITERS));
    if (total * p.g_sk >= (1L << 31)) return hipErrorInvalidValue;
  }
  const int grid = (int)std::min<long>(G, std::max<long>(p.g_sk, p.n_dp));
  hipLaunchKernelGGL(kern, dim3(grid), dim3(WAVES_M * WAVES_N * 64), LDS, stream, a, p);
  return hipGetLastError();
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int ADH>
hipError_t launch_ride(const GemmArgs &a, const GemmRide &r, hipStream_t stream) {
  constexpr int OUT_BN = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  constexpr int LDS = NU * (BM > BN ? BM : BN) * BK * 2;
  static_assert(LDS == 160 * 1024, "a workgroup of either kind must take the whole LDS of its CU");
  auto kern = gemm_attn_kernel<BM, BN, WAVES_M, WAVES_N, EPI, 64, ADH>;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int tiles = ((a.M + BM - 1) / BM) * ((a.N + OUT_BN - 1) / OUT_BN);
  if (tiles <= 0) return hipErrorInvalidValue;
  // (a negative margin: no tile closes the queue, the launch drains it)
  const int close_at = r.close_margin < 0 ? tiles + 1 : (tiles - r.close_margin > 1 ? tiles - r.close_margin : 1);
  hipLaunchKernelGGL(kern, dim3(r.head + tiles + r.tail), dim3(WAVES_M * WAVES_N * 64), LDS, stream, a, r, tiles,
                     (unsigned)close_at);
  return hipGetLastError();
}

// Tile shapes.  BIG: 256x256, 8 wavefronts.  TALL: 160x256, 8 wavefronts of 80x64: 2560 (and
// 5120) rows by 4096 (8192) columns then make exactly one (four) full rounds of 256
// workgroups where 256x256 tiles leave 38 % (17 %) of the CUs idle.  SMALL: 128x128.
// S128 / S256: 128x256 and 256x128 tiles on the deep weight ring, for at most 128 / 256 rows.
// activation slots of the short-row pipeline, minus one: three slots leave four weight slots of 16 KB
// (256x128) or three of 32 KB (128x256); measured against two slots (six / four weight slots) on the
// 256-row gate/up GEMM of the 8B layer: 0.075 against 0.078 ms, the other GEMMs the same
constexpr int DEEP_X = 2;
enum { V_AUTO = 0, V_BIG = 1, V_TALL = 2, V_SMALL = 3, V_S128 = 4, V_S256 = 5, V_SHARED = 6 };
constexpr int N_CU = 256;

thread_local int g_forced_variant = V_AUTO;  // set by the calling entry point from its context, for the launches of that call

long n_tiles(int m, int n, int bm, int bn) { return (long)((m + bm - 1) / bm) * ((n + bn - 1) / bn); }

// Estimated time of a launch in units of one full round of 256x256 tiles: full rounds of
// workgroups (the 128x128 tile runs two per CU) cost T each; a last, partly filled round costs
// T (a + (1 - a) fill): workgroups that share the chip with fewer others run faster, but not in
// proportion.  T and a were fitted on MI355X to the four GEMM shapes of the 8B layer at 384 to
// 2560 rows (the 160x256 tile: 0.072 ms per full round at K = 4096 where the 256x256 tile takes
// 0.100 and 512 tiles of 128x128 take 0.075).
// few rows: one tile row on the deep weight ring (0 where the rows do not fit one tile, or a shape is forced)
int short_variant(int m) {
  if (g_forced_variant != V_AUTO || m > 256) return 0;
  return m <= 128 ? V_S128 : V_S256;
}

// share_k: the contraction length if the launch may share tiles between workgroups (it has the
// workspace for it and covers all columns), else 0
int choose_variant(int m, int n_b_rows, int epilogue, int dh, int n_cu, int share_k = 0) {
  if (n_cu <= 0) n_cu = N_CU;
  if (g_forced_variant != V_AUTO && !(g_forced_variant == V_TALL && epilogue == EPI_QKV)) return g_forced_variant;
  (void)dh;
  if (const int sv = short_variant(m); sv && (epilogue == EPI_SWIGLU || epilogue == EPI_PLAIN)) {
    // worth it once the single row of tiles fills at least half the chip
    if (2 * n_tiles(m, n_b_rows, sv == V_S128 ? 128 : 256, sv == V_S128 ? 256 : 128) >= n_cu) return sv;
  }
  struct Cand { int v, bm, bn, per_cu; double T, a; };
  const Cand cands[3] = {{V_BIG, 256, 256, 1, 1.00, 0.72}, {V_TALL, 160, 256, 1, 0.76, 0.65}, {V_SMALL, 128, 128, 2, 0.75, 0.60}};
  int best = V_SMALL;
  double best_t = 1e300;
  for (const Cand &c : cands) {
    if (c.v == V_TALL && epilogue == EPI_QKV) continue;  // a wavefront must cover whole heads
    const long tiles = n_tiles(m, n_b_rows, c.bm, c.bn);
    const long slots = (long)n_cu * c.per_cu;
    const long full = tiles / slots, rem = tiles % slots;
    const double t = (double)full * c.T + (rem ? c.T * (c.a + (1.0 - c.a) * (double)rem / (double)slots) : 0.0);
    if (t < best_t) { best_t = t; best = c.v; }
  }
  // Shared 256x256 tiles: the chip's worth of k-tile iterations with nothing idle, 3 % for the
  // persistent loop, and what the cuts cost: a workgroup passes up to two partial tiles through
  // memory, about 0.08 ms per launch whatever its size (measured on the GEMMs of the 8B and 70B
  // layers), i.e. 53 k-tiles' worth of a round.  It pays only where K is long: the down
  // projection of the 70B layer at 5120 rows, 2.5 rounds of 448 k-tiles, 1.92 against 2.11 ms.
  if (share_k >= 4096 && m > 256) {
    const long tiles = n_tiles(m, n_b_rows, 256, 256);
    const long g = std::min<long>(n_cu, N_CU);
    if (tiles % g) {
      const double t = (double)tiles / (double)g * 1.03 + 53.0 / (double)((share_k + BK - 1) / BK);
      if (t < best_t) { best_t = t; best = V_SHARED; }
    }
  }
  return best;
}

template <int EPI, int DH_BIG_M, int DH_BIG_N>
hipError_t launch_variant(const GemmArgs &a, int v, hipStream_t stream) {
  if (v == V_BIG) return launch_one<256, 256, DH_BIG_M, DH_BIG_N, EPI, (DH_BIG_M == 4 ? 128 : 64)>(a, stream);
  if (v == V_SHARED) return launch_sk<256, 256, DH_BIG_M, DH_BIG_N, EPI, (DH_BIG_M == 4 ? 128 : 64)>(a, stream);
  if (v == V_TALL) return launch_one<160, 256, 2, 4, EPI, 64>(a, stream);
  if constexpr (EPI == EPI_SWIGLU || EPI == EPI_PLAIN) {
    if (v == V_S128) return launch_one<128, 256, 2, 4, EPI, 64, DEEP_X>(a, stream);
    if (v == V_S256) return launch_one<256, 128, 4, 2, EPI, 64, DEEP_X>(a, stream);
  }
  return launch_one<128, 128, 2, 2, EPI, 64>(a, stream);
}

}  // namespace

void gemm_force_variant(int v) { g_forced_variant = v; }
size_t gemm_sk_workspace_floats() { return (size_t)2 * SK_MAX_G * 256 * 256; }
int gemm_sk_counters() { return 2 * SK_MAX_G; }

bool gemm_round_split(const GemmArgs &a, int epilogue, int dh, GemmArgs *head, GemmArgs *tail) {
  if (epilogue != EPI_SWIGLU || g_forced_variant != V_AUTO || a.k_splits > 1) return false;
  const int n_cols = a.n_count ? a.n_count : a.N;
  if (choose_variant(a.M, 2 * n_cols, epilogue, dh, a.n_cu) != V_BIG) return false;
  const int n_cu = a.n_cu > 0 ? a.n_cu : N_CU;
  const long tm = (a.M + 255) / 256, tn = (n_cols + 127) / 128;  // a 256x256 tile yields 128 output columns
  const long tiles = tm * tn, full = tiles / n_cu, idle = (full + 1) * n_cu - tiles;
  const long cols_big = full * n_cu / tm;
  if (full < 1 || tiles % n_cu == 0 || idle * 4 <= n_cu || cols_big < 1 || cols_big >= tn) return false;
  *head = a;
  *tail = a;
  head->n_count = (int)cols_big * 128;
  tail->n_begin = a.n_begin + head->n_count;
  tail->n_count = n_cols - head->n_count;
  head->tile_variant = V_BIG;
  tail->tile_variant = V_SMALL;  // two workgroups per CU fill the chip best with what is left of a round
  return true;
}

int gemm_splitk_choice(int M, int N, int K, int epilogue, int n_cu) {
  if (epilogue != EPI_RESID && epilogue != EPI_RESID_NORM && epilogue != EPI_QKV) return 1;
  if (n_cu <= 0) n_cu = N_CU;
  const long by_k = ((K + BK - 1) / BK) / 8;    // at least eight k-tiles per range
  if (const int sv = short_variant(M)) {        // one workgroup per CU, each with a k-range of a one-row tile
    const long tiles = n_tiles(M, N, sv == V_S128 ? 128 : 256, sv == V_S128 ? 256 : 128);
    const long s = std::min((long)MAX_SPLITS, std::min((long)n_cu / tiles, by_k));
    return s >= 2 ? (int)s : 1;
  }
  if (choose_variant(M, N, epilogue, 64, n_cu) != V_SMALL) return 1;  // only where the smallest tile is already in use
  const long tiles = n_tiles(M, N, 128, 128);
  const long room = 2L * n_cu / tiles;          // two 128x128 workgroups fit one CU
  const long s = std::min((long)MAX_SPLITS, std::min(room, by_k));
  return s >= 2 ? (int)s : 1;
}

int gemm_ss_parts(const GemmArgs &a, int epilogue, int dh) {
  if (a.k_splits > 1) return 1;  // the split-K reduction leaves whole row sums
  const int v = a.tile_variant ? a.tile_variant
                               : choose_variant(a.M, a.N, epilogue, dh, a.n_cu, a.sk_ws && a.sk_cnt && !a.n_count ? a.K : 0);
  // partial row sums: one per (column tile, wavefront column)
  return v == V_SMALL ? ((a.N + 127) / 128) * 2 : ((a.N + 255) / 256) * 4;
}

int gemm_ride_variant(int m, int n_b_rows, int n_cu) {
  // the eight-wavefront tiles only: 256x256 or 160x256, by the same cost model of rounds
  struct Cand { int v, bm; double T, a; };
  const Cand cands[2] = {{V_BIG, 256, 1.00, 0.72}, {V_TALL, 160, 0.76, 0.65}};
  if (n_cu <= 0) n_cu = N_CU;
  int best = V_BIG;
  double best_t = 1e300;
  for (const Cand &c : cands) {
    const long tiles = n_tiles(m, n_b_rows, c.bm, 256);
    const long full = tiles / n_cu, rem = tiles % n_cu;
    const double t = (double)full * c.T + (rem ? c.T * (c.a + (1.0 - c.a) * (double)rem / (double)n_cu) : 0.0);
    if (t < best_t) { best_t = t; best = c.v; }
  }
  return best;
}

int gemm_ride_tiles(const GemmArgs &a, int epilogue) {
  const int bm = a.tile_variant == V_TALL ? 160 : 256, out_bn = epilogue == EPI_SWIGLU ? 128 : 256;
  return ((a.M + bm - 1) / bm) * ((a.N + out_bn - 1) / out_bn);
}

hipError_t launch_gemm_with_attention(const GemmArgs &a, int epilogue, int dh, const GemmRide &r, hipStream_t stream) {
  (void)dh;
  if (a.k_splits > 1 || a.n_count || r.head < 0 || r.head % XCDS || r.tail < 0 || !r.done || !r.ticket_next || !r.q.ticket)
    return hipErrorInvalidValue;
  const int b_rows = (epilogue == EPI_SWIGLU) ? 2 * a.N : a.N;
  if ((size_t)a.M * a.lda * 2 >= ((size_t)1 << 32) || (size_t)b_rows * a.ldb * 2 >= ((size_t)1 << 32))
    return hipErrorInvalidValue;
  const int v = a.tile_variant ? a.tile_variant : gemm_ride_variant(a.M, b_rows, N_CU - r.head);
  if (v != V_BIG && v != V_TALL) return hipErrorInvalidValue;
  const int adh = r.q.d.s.head_dim;
  if (adh != 64 && adh != 128) return hipErrorInvalidValue;
#define BS_RIDE(EPI)                                                                                  \
  return v == V_BIG ? (adh == 128 ? launch_ride<256, 256, 2, 4, EPI, 128>(a, r, stream)               \
                                  : launch_ride<256, 256, 2, 4, EPI, 64>(a, r, stream))               \
                    : (adh == 128 ? launch_ride<160, 256, 2, 4, EPI, 128>(a, r, stream)               \
                                  : launch_ride<160, 256, 2, 4, EPI, 64>(a, r, stream))
  switch (epilogue) {
    case EPI_RESID_NORM: BS_RIDE(EPI_RESID_NORM);
    case EPI_SWIGLU: BS_RIDE(EPI_SWIGLU);
    case EPI_RESID: BS_RIDE(EPI_RESID);
    default: return hipErrorInvalidValue;
  }
#undef BS_RIDE
}

hipError_t launch_gemm(const GemmArgs &a, int epilogue, int dh, hipStream_t stream) {
  // the kernels address operand rows with 32-bit byte offsets from the matrix base
  if ((size_t)a.M * a.lda * 2 >= ((size_t)1 << 32) ||
      (size_t)((epilogue == EPI_SWIGLU) ? 2 * a.N : a.N) * a.ldb * 2 >= ((size_t)1 << 32))
    return hipErrorInvalidValue;
  if (a.k_splits > 1) {
    if ((epilogue != EPI_RESID && epilogue != EPI_RESID_NORM && epilogue != EPI_QKV) || !a.splitk_ws || a.N % 4)
      return hipErrorInvalidValue;
    const int sv = short_variant(a.M);
    hipError_t e = sv == V_S128   ? launch_one<128, 256, 2, 4, EPI_PARTIAL, 64, DEEP_X>(a, stream)
                   : sv == V_S256 ? launch_one<256, 128, 4, 2, EPI_PARTIAL, 64, DEEP_X>(a, stream)
                                  : launch_one<128, 128, 2, 2, EPI_PARTIAL, 64>(a, stream);
    if (e != hipSuccess) return e;
    if (epilogue == EPI_QKV) {
      const int items = ((a.n_q_heads + a.n_kv_heads) * (dh / 2) + a.n_kv_heads * dh) / 4;
      hipLaunchKernelGGL(splitk_reduce_qkv_kernel, dim3(a.M, (items + 255) / 256), dim3(256), 0, stream, a, dh);
    } else if (epilogue == EPI_RESID) {
      hipLaunchKernelGGL(splitk_reduce_resid_kernel, dim3(a.M, (a.N / 4 + 255) / 256), dim3(256), 0, stream, a);
    } else {
      hipLaunchKernelGGL(splitk_reduce_resid_norm_kernel, dim3(a.M), dim3(256), 0, stream, a);
    }
    return hipGetLastError();
  }
  if (a.n_count && epilogue != EPI_SWIGLU && epilogue != EPI_PLAIN) return hipErrorInvalidValue;
  const int n_cols = a.n_count ? a.n_count : a.N;
  const int v = a.tile_variant ? a.tile_variant
                               : choose_variant(a.M, (epilogue == EPI_SWIGLU) ? 2 * n_cols : n_cols, epilogue, dh, a.n_cu,
                                                a.sk_ws && a.sk_cnt && !a.n_count ? a.K : 0);
  switch (epilogue) {
    case EPI_PLAIN: return launch_variant<EPI_PLAIN, 2, 4>(a, v, stream);
    case EPI_RESID: return launch_variant<EPI_RESID, 2, 4>(a, v, stream);
    case EPI_RESID_NORM: return launch_variant<EPI_RESID_NORM, 2, 4>(a, v, stream);
    case EPI_SWIGLU: return launch_variant<EPI_SWIGLU, 2, 4>(a, v, stream);
    case EPI_QKV:
      if (dh == 128)
        return v == V_SHARED ? launch_sk<256, 256, 4, 2, EPI_QKV, 128>(a, stream)
               : v == V_BIG  ? launch_one<256, 256, 4, 2, EPI_QKV, 128>(a, stream)
                             : launch_one<128, 128, 4, 1, EPI_QKV, 128>(a, stream);
      if (dh == 64)
        return v == V_SHARED ? launch_sk<256, 256, 2, 4, EPI_QKV, 64>(a, stream)
               : v == V_BIG  ? launch_one<256, 256, 2, 4, EPI_QKV, 64>(a, stream)
                             : launch_one<128, 128, 2, 2, EPI_QKV, 64>(a, stream);
      return hipErrorInvalidValue;
    default:
      return hipErrorInvalidValue;
  }
}

}  // namespace bs
