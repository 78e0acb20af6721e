// bf16 GEMM on the gfx950 matrix cores with the layer's small operators fused
// into the epilogues (BlendServe Section 4.1: the GEMMs - QKV generation, output
// projection, FFN - are the compute-bound operators; Section 4.2: normalisation,
// activation and position embedding are small next to them, so they ride along).
#pragma once
#include <stdint.h>
#include <hip/hip_runtime.h>

#include "attn.hpp"

namespace bs {

enum GemmEpilogue {
  EPI_PLAIN = 0,      // C = A B^T
  EPI_QKV = 1,        // row scale (RMSNorm), RoPE on q and k heads, q to its buffer, k and v into KV pages
  EPI_RESID_NORM = 2, // x1 = resid + A B^T in fp32; also bf16(x1 * gain) and partial row sums of x1^2 for the next norm
  EPI_SWIGLU = 3,     // out = silu(s * gate) * (s * up), s = per-row RMSNorm scale
  EPI_RESID = 4,      // y = resid + A B^T (resid in bf16, or in fp32 when resid32 is set)
  EPI_PARTIAL = 5     // internal: fp32 partial products of one k-range into the split-K workspace
};

struct GemmArgs {
  const uint16_t *A;  // [M, K] bf16 activations, row stride lda
  const uint16_t *B;  // [N, K] bf16 weights (out-features major), row stride ldb
  int M, N, K, lda, ldb;
  int n_cu;           // CUs the launch may use (0 = the whole chip); only steers the tile choice
  int n_begin, n_count;  // output columns [n_begin, n_begin + n_count) only (n_count = 0: all N); SWIGLU and PLAIN
  int tile_variant;      // 0: chosen by the cost model; else that tile shape (set by gemm_round_split for its tail)
  uint16_t *C;        // output [M, ldc] bf16 (PLAIN, RESID*, SWIGLU)
  int ldc;
  const uint16_t *resid;  // [M, ldr] bf16
  const float *resid32;   // [M, ldr] fp32 (EPI_RESID only; takes precedence)
  int ldr;
  // RMSNorm of the A rows, applied as a per-row factor after the contraction
  const float *rstd;     // [M] 1 / sqrt(mean(x^2) + eps) of each row (QKV, SWIGLU)
  int ss_stride;         // row stride of ss_out
  // RESID_NORM extras
  const uint16_t *gain;  // [N] bf16 gain of the next norm
  float *C32;            // [M, ldc] x1 in fp32
  uint16_t *C_gain;      // [M, ldc] bf16(x1 * gain)
  float *ss_out;         // [tiles_n * waves_n][ss_stride] partial row sums of x1^2
  float *rstd_out;       // split-K only (may be NULL): the reduction, which sees whole rows, leaves
  float rstd_eps;        //   1 / sqrt(mean(x1^2) + rstd_eps) of each row here, and no pass over ss_out is needed
  // Split-K (QKV, RESID and RESID_NORM with few tiles): k_splits > 1 cuts K into that many ranges,
  // each (tile, range) is one workgroup that leaves fp32 partial products in splitk_ws
  // [k_splits][M][N]; a second kernel adds them up in a fixed order and applies the epilogue.
  // The caller takes k_splits from gemm_splitk_choice and provides the workspace.
  int k_splits;
  float *splitk_ws;
  // Shared tiles (tile_variant 6, see gemm_sk_kernel): room for the partial tiles, at least
  // gemm_sk_workspace_floats() floats, and gemm_sk_counters() counters that are zero between launches.
  // Launches that use them must not overlap in time.
  float *sk_ws;
  unsigned *sk_cnt;
  // SWIGLU: B holds F gate rows then F up rows; N = F
  // QKV extras
  int n_q_heads, n_kv_heads;
  const float *rope_cos, *rope_sin;  // [max_pos][dh/2]
  const int32_t *row_pos, *row_page, *row_slot;  // [M]
  uint16_t *q_out;    // [M, Hq*dh]
  uint16_t *kv_pool;  // pages: [2][Hkv][...]
};

// Decode attention that shares a GEMM launch (see gemm_attn_kernel in gemm.hip).
struct GemmRide {
  DecodeQueue q;          // the step's queue of 16-row units; q.ticket is this launch's counter
  int head, tail;         // attention workgroups ahead of the tiles (a multiple of 8) and behind them
  unsigned *done;         // tiles of this launch that have finished (zero at launch)
  int close_margin;       // the queue closes for this launch when all but this many tiles have finished (negative: never)
  unsigned *ticket_next;  // where the closing tile leaves the queue position for the next launch
  unsigned *closed_at;    // and a copy that nobody adds to, for the report of where the attention ran (may be NULL)
};
// The GEMM on `n_cu - ride.head` CUs' worth of 256x256 or 160x256 tiles with the attention
// workgroups of `ride` around them.  Epilogues RESID_NORM, SWIGLU and RESID; no split-K.
hipError_t launch_gemm_with_attention(const GemmArgs &a, int epilogue, int dh, const GemmRide &ride, hipStream_t stream);
// tile shape (a value for GemmArgs::tile_variant) that such a launch takes for M rows, `n_b_rows`
// weight rows and `n_cu` CUs left to the tiles
int gemm_ride_variant(int m, int n_b_rows, int n_cu);
// tiles of such a launch (a.tile_variant set)
int gemm_ride_tiles(const GemmArgs &a, int epilogue);

// Picks a tile shape for the problem and launches on `stream`.  dh is the head
// dimension (used by EPI_QKV only).  Returns hipSuccess or the launch error.
hipError_t launch_gemm(const GemmArgs &a, int epilogue, int dh, hipStream_t stream);
// partial-sum slots a RESID_NORM launch over N columns writes
int gemm_ss_parts(const GemmArgs &a, int epilogue, int dh);
// Whole rounds first: when a gate/up GEMM on 256x256 tiles would end with a round that leaves
// more than a quarter of the chip idle, returns true and the two column ranges to launch
// instead: `head` = the tile columns of the whole rounds, `tail` = the rest (whatever tile
// shape suits them).
bool gemm_round_split(const GemmArgs &a, int epilogue, int dh, GemmArgs *head, GemmArgs *tail);
// Number of k-ranges worth using for this problem (1 = no split): only when the tiles would
// leave most of the chip idle and every range keeps at least eight k-tiles.
int gemm_splitk_choice(int M, int N, int K, int epilogue, int n_cu);
void gemm_force_variant(int v);  // 0 = choose by shape, 1 = 256x256, 2 = 160x256, 3 = 128x128 tiles, 6 = shared 256x256 tiles (tuning)
size_t gemm_sk_workspace_floats();
int gemm_sk_counters();

}  // namespace bs
