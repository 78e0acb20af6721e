// Paged attention for the blended step: prefix-aware decode attention (partial
// softmax states per prefix node / private tail, then a merge) and causal
// prefill attention, both on the gfx950 matrix cores.
#pragma once
#include <stdint.h>
#include <hip/hip_runtime.h>

namespace bs {

// One unit of decode-attention work: a run of pages (a chunk of a prefix node,
// or of one sequence's private tail) attended to by the query rows of a
// contiguous run of member sequences.
struct DecodeItem {
  int32_t page_off;   // first page of the chunk in item_pages
  int32_t n_tokens;   // tokens in the chunk (the last page may be partial)
  int32_t seq_first;  // first member sequence
  int32_t n_members;  // member sequences (n_members * group <= 16 * nqb query rows of the launch)
  int32_t slot_off;   // partial-state slot of this chunk inside every member's slot range
  int32_t page0, page1;  // pool pages of the chunk's first two pages (page1 = page0 in a chunk of one page)
  int32_t pad;
};

struct AttnShape {
  int n_q_heads, n_kv_heads, head_dim, page_size;
  float scale_log2e;  // log2(e) / sqrt(dh)
};

struct DecodeArgs {
  AttnShape s;
  const DecodeItem *items;
  const int32_t *item_pages;
  int row_base;               // row of decode sequence s = s + row_base (one row each, after the prefill rows)
  const int32_t *part_start;  // [n_seq + 1] partial-state slots of each sequence
  const uint16_t *q;          // [T, Hq*dh]
  const uint16_t *kv_pool;
  float *part_acc;            // [slots][Hq][dh]
  float *part_m, *part_l;     // [slots][Hq]
};

// The 16-row units of a step as a queue that several launches drain in turn: unit u is
// (item first_item + u / Hkv, KV head u % Hkv); a wavefront takes the next unit by adding one
// to *ticket and stops at the first number >= n_units.  A launch that must hand the rest of
// the queue on (a GEMM launch that carries attention workgroups: when its last tiles finish)
// closes its counter by adding DECODE_QUEUE_CLOSED to it and stores the position it found
// there, capped at n_units, as the start value of the next launch's counter.
constexpr unsigned DECODE_QUEUE_CLOSED = 0x40000000u;
struct DecodeQueue {
  DecodeArgs d;
  int first_item, n_units;
  unsigned *ticket;
  int waves;  // wavefronts of an attention workgroup (of eight) that take units
  // Optional timeline of the launch (NULL: none): record 8 b + w of 4 x uint64 belongs to wavefront
  // w of workgroup b: {begin, end} in ticks of the constant 100 MHz clock, {kind | HW_ID << 8 |
  // XCC_ID << 32}, {units | KV tokens << 32} served in between (tiles: wavefront 0 only).
  uint64_t *trace;
};
enum { TRACE_ATTENTION = 1, TRACE_TILE = 2 };
constexpr int TRACE_WORDS = 4;
// what is left in the queue, on the whole chip: workgroups of eight wavefronts, each drawing units
hipError_t launch_decode_queue(const DecodeQueue &q, int n_workgroups, hipStream_t stream);

// one launch over items [0, n_wide) of up to 64 query rows each, then [n_wide, n_wide + n_narrow) of up to 16
hipError_t launch_decode_attn(const DecodeArgs &a, int n_wide, int n_narrow, hipStream_t stream);

struct MergeArgs {
  AttnShape s;
  int n_prefill, n_decode;
  const int32_t *row_start, *part_start;
  const float *part_acc, *part_m, *part_l;
  uint16_t *out;  // [T, Hq*dh]
};
hipError_t launch_decode_merge(const MergeArgs &a, hipStream_t stream);

struct PrefillArgs {
  AttnShape s;
  const int32_t *work;  // [n_work][2] = (sequence, block of 64 query rows)
  int n_work;
  const int32_t *row_start, *kv_len, *page_start, *page_ids;
  const uint16_t *q;
  const uint16_t *kv_pool;
  uint16_t *out;
};
hipError_t launch_prefill_attn(const PrefillArgs &a, hipStream_t stream);

// both kinds in one launch (prefill workgroups dealt evenly among the decode ones); needs a step with
// prefill work and decode items, and a group size that is a multiple of four
bool blended_attn_possible(const AttnShape &s);
hipError_t launch_blended_attn(const DecodeArgs &d, int n_wide, int n_narrow, const PrefillArgs &pf, hipStream_t stream);

}  // namespace bs
