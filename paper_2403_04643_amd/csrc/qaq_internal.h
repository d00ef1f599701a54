// Internal declarations shared by the host API and the kernel files of libqaq.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "../../include/qaq.h"
#include "../../include/qaq_aux.h"
#include "qaq_layout.h"

#define QAQ_MAX_KV_HEADS 128
#define QAQ_MAX_WINDOW 8
#define QAQ_MAX_THR 256          // threshold table of a call: per KV head, or per (sequence, KV head) where lengths differ
#define QAQ_MAX_RAGGED_BATCH 64  // sequences of a cache whose lengths differ

// What every kernel sees of a cache: raw pointers into the arena plus the shape.
struct QaqView {
  uint8_t* codes[2];
  uint32_t* mm[2];
  uint8_t* perm[2];
  uint8_t* oidx[2];
  uint16_t* oval[2];
  uint8_t* tags[2];
  uint16_t* counts;
  float* vbound;
  float* kthr;
  void* ring;               // score rows of the window: fp32, or (ring_half 1) fp16, or (2) bf16
  int ring_half;
  float* partial;
  long long* statbuf;
  unsigned int* refused;   // per tile side: [0] widenings refused for want of the unquantized copy, [1] widenings served
  uint32_t* todo;          // [B][Hkv][NT][2] list of tile sides a decode-step update hands to the general kernel
  uint32_t* todo_count;    // [2] entries of the list; the two counters serve alternate steps
  int B, Hq, Hkv, D, Tmax, NT, no2, window;
  int has1;                // the width set contains 1: kernels take their five-class variants
  int csr;                 // outliers by thresholds: oidx / oval are per-tile pools in position order, addressed
  uint16_t* ostart[2];     // ... through (first entry, count) per position
  uint8_t* ocnt[2];
  const float* othr;       // [2][Hkv][2] thresholds (lo, hi)
  uint32_t cap[2];
  // Sequences of different lengths: every length the host passes (cached tokens, tokens a window row
  // covers) is that of the longest sequence, and sequence b is shortfall[b] tokens shorter -- a
  // decode step adds one token to every sequence, so the differences stay what the first append made them.
  int ragged;              // 0: all sequences have one length, kernels do not read the table
  int shortfall[QAQ_MAX_RAGGED_BATCH];
};

// tokens of sequence b, given the longest sequence's count
__device__ __forceinline__ int qaq_seq_len(const QaqView& v, int b, int len_longest) {
  return v.ragged ? max(len_longest - v.shortfall[b], 0) : len_longest;
}

__host__ __device__ __forceinline__ size_t qaq_bh(const QaqView& v, int b, int h) { return (size_t)b * v.Hkv + h; }
// The window's rows: value as stored (what the predicted score is taken over), load, store.
// bf16 of a finite float, round to nearest even: the upper 16 bits after adding half an ulp
// (one less on an even upper half)
__device__ __forceinline__ uint16_t qaq_bf16_bits(float s) {
  const uint32_t u = __float_as_uint(s);
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ float qaq_ring_value(const QaqView& v, float s) {
  return v.ring_half == 1 ? __half2float(__float2half_rn(s)) : v.ring_half == 2 ? __uint_as_float((uint32_t)qaq_bf16_bits(s) << 16) : s;
}
__device__ __forceinline__ float qaq_ring_load(const QaqView& v, size_t i) {
  return v.ring_half == 1 ? __half2float(((const __half*)v.ring)[i])
       : v.ring_half == 2 ? __uint_as_float((uint32_t)((const uint16_t*)v.ring)[i] << 16) : ((const float*)v.ring)[i];
}
__device__ __forceinline__ void qaq_ring_store(const QaqView& v, size_t i, float s) {
  if (v.ring_half == 1) ((__half*)v.ring)[i] = __float2half_rn(s);
  else if (v.ring_half == 2) ((uint16_t*)v.ring)[i] = qaq_bf16_bits(s);
  else ((float*)v.ring)[i] = s;
}
// What the value rule is applied to (Section 4.2, the attention window): the largest score of position t
// over this step's row -- the maximum over the G query heads of the KV head, rows row0 .. row0+G-1 of
// `scores`, `stride` floats apart, GB of them loaded at a time, rounded to what the window stores;
// returned in *s_row -- and the window's stored rows other than `skip`.  With GB = 0 there is no row of
// this step (*s_row = 0).
// All loads are issued before the first is used: a loop that folds each value in as it arrives pays one
// memory round trip per row.  For that the loads carry no condition at all (a load under a branch is
// waited for where the branch ends): the row count is a template argument, the row that is left out is
// replaced by another one (read twice, folded once), a query head past the last one reads the last one
// again, and every row of the ring is allocated for every position -- what a row does not cover is left
// out of the maximum, not out of the loads.  ri = index of (sequence, KV head, t) inside a row; bit r of
// `covered` says whether row r covers position t (qaq_rows_covering).
// bit r: window row r holds a score of position t of sequence b (row_len: tokens each row covers, by the
// longest sequence's count).  Constant indices only, so that the table stays where the kernel arguments are.
__device__ __forceinline__ uint32_t qaq_rows_covering(const QaqView& v, const int (&row_len)[QAQ_MAX_WINDOW], int b, int t) {
  uint32_t m = 0u;
#pragma unroll
  for (int r = 0; r < QAQ_MAX_WINDOW; ++r)
    if (t < qaq_seq_len(v, b, row_len[r])) m |= 1u << r;
  return m;
}
template <int W, typename RAW, int GB>
__device__ __forceinline__ float qaq_predicted_w(const QaqView& v, uint32_t covered, int skip, size_t ri, int t,
                                                 const float* scores, size_t row0, int G, size_t stride, float* s_row) {
  const size_t ring_row = (size_t)v.B * v.Hkv * v.Tmax;
  const int other = skip == 0 ? (W > 1 ? 1 : 0) : 0;
  RAW raw[W];
#pragma unroll
  for (int r = 0; r < W; ++r) raw[r] = ((const RAW*)v.ring)[(size_t)(r == skip ? other : r) * ring_row + ri];
  float s = 0.0f;
  if (GB > 0) {
    float x[GB > 0 ? GB : 1];
#pragma unroll
    for (int j = 0; j < GB; ++j) x[j] = scores[(row0 + min(j, G - 1)) * stride + t];
#pragma unroll
    for (int j = 0; j < GB; ++j) s = fmaxf(s, x[j]);         // probabilities: >= 0
    for (int g0 = GB; g0 < G; g0 += GB) {
#pragma unroll
      for (int j = 0; j < GB; ++j) x[j] = scores[(row0 + min(g0 + j, G - 1)) * stride + t];
#pragma unroll
      for (int j = 0; j < GB; ++j) s = fmaxf(s, x[j]);
    }
    s = v.ring_half == 1 ? __half2float(__float2half_rn(s)) : v.ring_half == 2 ? __uint_as_float((uint32_t)qaq_bf16_bits(s) << 16) : s;
  }
  *s_row = s;
  float m = s;
#pragma unroll
  for (int r = 0; r < W; ++r) {
    const float x = sizeof(RAW) == 4 ? __uint_as_float((uint32_t)raw[r])
                  : v.ring_half == 1 ? __half2float(__ushort_as_half((unsigned short)raw[r])) : __uint_as_float((uint32_t)raw[r] << 16);
    if (r != skip && ((covered >> r) & 1u)) m = fmaxf(m, x);
  }
  return m;
}
template <typename RAW, int GB>
__device__ __forceinline__ float qaq_predicted_t(const QaqView& v, uint32_t covered, int skip, size_t ri, int t,
                                                 const float* scores, size_t row0, int G, size_t stride, float* s_row) {
  switch (v.window) {
    case 1: return qaq_predicted_w<1, RAW, GB>(v, covered, skip, ri, t, scores, row0, G, stride, s_row);
    case 2: return qaq_predicted_w<2, RAW, GB>(v, covered, skip, ri, t, scores, row0, G, stride, s_row);
    case 3: return qaq_predicted_w<3, RAW, GB>(v, covered, skip, ri, t, scores, row0, G, stride, s_row);
    case 4: return qaq_predicted_w<4, RAW, GB>(v, covered, skip, ri, t, scores, row0, G, stride, s_row);
    case 5: return qaq_predicted_w<5, RAW, GB>(v, covered, skip, ri, t, scores, row0, G, stride, s_row);
    case 6: return qaq_predicted_w<6, RAW, GB>(v, covered, skip, ri, t, scores, row0, G, stride, s_row);
    case 7: return qaq_predicted_w<7, RAW, GB>(v, covered, skip, ri, t, scores, row0, G, stride, s_row);
    default: return qaq_predicted_w<8, RAW, GB>(v, covered, skip, ri, t, scores, row0, G, stride, s_row);
  }
}
template <bool SCORES>
__device__ __forceinline__ float qaq_predicted(const QaqView& v, uint32_t covered, int skip, size_t ri, int t,
                                               const float* scores, size_t row0, int G, size_t stride, float* s_row) {
  // query heads per batch of loads: none, one (no grouped-query attention), four
  if (!SCORES)
    return v.ring_half ? qaq_predicted_t<uint16_t, 0>(v, covered, skip, ri, t, scores, row0, G, stride, s_row)
                       : qaq_predicted_t<uint32_t, 0>(v, covered, skip, ri, t, scores, row0, G, stride, s_row);
  if (G == 1)
    return v.ring_half ? qaq_predicted_t<uint16_t, 1>(v, covered, skip, ri, t, scores, row0, G, stride, s_row)
                       : qaq_predicted_t<uint32_t, 1>(v, covered, skip, ri, t, scores, row0, G, stride, s_row);
  return v.ring_half ? qaq_predicted_t<uint16_t, 4>(v, covered, skip, ri, t, scores, row0, G, stride, s_row)
                     : qaq_predicted_t<uint32_t, 4>(v, covered, skip, ri, t, scores, row0, G, stride, s_row);
}
__device__ __forceinline__ uint8_t* qaq_tile_codes(const QaqView& v, int side, int b, int h, int tile) {
  return v.codes[side] + ((qaq_bh(v, b, h) * v.NT + tile) * (size_t)v.cap[side]);
}
__device__ __forceinline__ size_t qaq_slot_index(const QaqView& v, int b, int h, int tile, int slot) {
  return qaq_bh(v, b, h) * v.Tmax + (size_t)tile * QAQ_TT + slot;
}
// n_tok: tokens the tile holds (the 1-bit class is what the four stored counts leave of them)
__device__ __forceinline__ QaqCounts qaq_load_counts(const QaqView& v, int side, int b, int h, int tile, int n_tok) {
  const uint16_t* p = v.counts + (((qaq_bh(v, b, h) * v.NT + tile) * 2 + side) * 4);
  QaqCounts c;
  c.n3 = p[QC3]; c.n2 = p[QC2]; c.n4 = p[QC4]; c.n8 = p[QC8];
  c.n1 = n_tok - (c.n3 + c.n2 + c.n4 + c.n8);
  return c;
}

// The window's part of qaq_predicted in a compact form for the general build kernel (no variants by
// row count: always QAQ_MAX_WINDOW loads, a row that does not count replaced by one that does or by row 0):
// the largest stored score of position t over the rows in `covered` other than `skip`, at least `start`.
__device__ __forceinline__ float qaq_window_max_compact(const QaqView& v, uint32_t covered, int skip, size_t ri, float start) {
  const size_t ring_row = (size_t)v.B * v.Hkv * v.Tmax;
  uint32_t raw[QAQ_MAX_WINDOW];
  if (v.ring_half) {
#pragma unroll
    for (int r = 0; r < QAQ_MAX_WINDOW; ++r) raw[r] = ((const uint16_t*)v.ring)[(size_t)(r < v.window && r != skip ? r : 0) * ring_row + ri];
  } else {
#pragma unroll
    for (int r = 0; r < QAQ_MAX_WINDOW; ++r) raw[r] = ((const uint32_t*)v.ring)[(size_t)(r < v.window && r != skip ? r : 0) * ring_row + ri];
  }
  float m = start;
#pragma unroll
  for (int r = 0; r < QAQ_MAX_WINDOW; ++r) {
    const float x = v.ring_half == 1 ? __half2float(__ushort_as_half((unsigned short)raw[r]))
                  : v.ring_half == 2 ? __uint_as_float(raw[r] << 16) : __uint_as_float(raw[r]);
    if (r < v.window && r != skip && ((covered >> r) & 1u)) m = fmaxf(m, x);
  }
  return m;
}

#if defined(__HIPCC__)
// ---- wavefront reductions on the data-parallel-primitive path (no LDS round trips) -----
// One instruction per step: the DPP form of the arithmetic instruction itself (the compiler
// would emit a move with the lane pattern, a NaN-quieting max of each input and the max).
// A VGPR written by a vector instruction needs two wait states before a DPP read.
#define QAQ_DPP_STEP(op, pat) "s_nop 1\n\t" op " %0, %0, %0 " pat "\n\t"
__device__ __forceinline__ float wave_max(float x) {
  asm volatile(QAQ_DPP_STEP("v_max_f32_dpp", "quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf")
               QAQ_DPP_STEP("v_max_f32_dpp", "quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf")
               QAQ_DPP_STEP("v_max_f32_dpp", "row_half_mirror row_mask:0xf bank_mask:0xf")
               QAQ_DPP_STEP("v_max_f32_dpp", "row_mirror row_mask:0xf bank_mask:0xf")
               QAQ_DPP_STEP("v_max_f32_dpp", "row_bcast:15 row_mask:0xa bank_mask:0xf")      // into rows 1 and 3
               QAQ_DPP_STEP("v_max_f32_dpp", "row_bcast:31 row_mask:0xc bank_mask:0xf")      // into rows 2 and 3
               "s_nop 1"
               : "+v"(x));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}
__device__ __forceinline__ float wave_sum(float x) {
  asm volatile(QAQ_DPP_STEP("v_add_f32_dpp", "quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf")
               QAQ_DPP_STEP("v_add_f32_dpp", "quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf")
               QAQ_DPP_STEP("v_add_f32_dpp", "row_half_mirror row_mask:0xf bank_mask:0xf")
               QAQ_DPP_STEP("v_add_f32_dpp", "row_mirror row_mask:0xf bank_mask:0xf")
               QAQ_DPP_STEP("v_add_f32_dpp", "row_bcast:15 row_mask:0xa bank_mask:0xf")
               QAQ_DPP_STEP("v_add_f32_dpp", "row_bcast:31 row_mask:0xc bank_mask:0xf")
               "s_nop 1"
               : "+v"(x));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}
__device__ __forceinline__ float wave_min(float x) {
  asm volatile(QAQ_DPP_STEP("v_min_f32_dpp", "quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf")
               QAQ_DPP_STEP("v_min_f32_dpp", "quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf")
               QAQ_DPP_STEP("v_min_f32_dpp", "row_half_mirror row_mask:0xf bank_mask:0xf")
               QAQ_DPP_STEP("v_min_f32_dpp", "row_mirror row_mask:0xf bank_mask:0xf")
               QAQ_DPP_STEP("v_min_f32_dpp", "row_bcast:15 row_mask:0xa bank_mask:0xf")      // into rows 1 and 3
               QAQ_DPP_STEP("v_min_f32_dpp", "row_bcast:31 row_mask:0xc bank_mask:0xf")      // into rows 2 and 3
               "s_nop 1"
               : "+v"(x));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}
#endif

// What the width rules need (Section 4.1 written as comparisons, Section 4.2 window).
struct QaqRuleArgs {
  int G;                   // query heads per KV head
  const float* scores;     // [B,Hq,score_stride] or null
  int score_stride;
  int new_row;             // ring row that receives `scores` (ignored if null)
  int row_len[QAQ_MAX_WINDOW];  // tokens covered by each ring row, 0 = unused
  int nbits;
  int bit_set[5];
  float tau_k[QAQ_MAX_THR];        // key-rule threshold per KV head; per (sequence, KV head) in a cache with different lengths
  float c_v[QAQ_MAX_RAGGED_BATCH]; // value-rule threshold; per sequence in such a cache, else entry 0
  uint8_t* out_bits[2];    // [B,Hkv,len] or null
};
__device__ __forceinline__ float qaq_tau_k(const QaqRuleArgs& r, const QaqView& v, int b, int h) { return r.tau_k[v.ragged ? b * v.Hkv + h : h]; }
__device__ __forceinline__ float qaq_c_v(const QaqRuleArgs& r, const QaqView& v, int b) { return r.c_v[v.ragged ? b : 0]; }

struct QaqBuildArgs {
  QaqView v;
  int mode;          // 0 = append, 1 = requantize, 2 = decode-step update (append one token, select, requantize),
                     // 3 = append at the widths the rules give from the window as it stands
  QaqRuleArgs rule;  // modes 2 and 3
  int len_before, len_after, tile0, n_new, widest;
  const __half* newx[2];       // append: [B,Hkv,n_new,D]
  const uint8_t* newbits[2];   // append: [B,Hkv,n_new] or null; requantize: [B,Hkv,len] or null
  const __half* orig[2];       // requantize: [B,Hkv,orig_tokens,D] or null
  __half* orig_put[2];         // same buffers when the appended tokens are to be written into them, else null
  int orig_tokens;             // token extent of the unquantized copies (>= len)
  // decode-step update: tile sides the fast kernel leaves to the general one, (unit * NT + tile) * 2 + side
  uint32_t* todo;
  uint32_t* todo_count;        // the counter this step appends through (zero when the step starts)
  uint32_t* todo_count_next;   // the next step's counter (this step clears it)
};

struct QaqSelectArgs {
  QaqView v;
  int len;                 // tokens to select for
  int G;                   // query heads per KV head
  const float* scores;     // [B,Hq,len] or null
  int new_row;             // ring row that receives `scores` (ignored if null)
  int row_len[QAQ_MAX_WINDOW];  // tokens covered by each ring row, 0 = unused
  int nbits;
  int bit_set[5];
  float tau_k[QAQ_MAX_THR];        // as in QaqRuleArgs
  float c_v[QAQ_MAX_RAGGED_BATCH];
  uint8_t* out_bits[2];    // [B,Hkv,len]
};

struct QaqAttnArgs {
  QaqView v;
  int len, G;
  const __half* q;        // [B,Hq,D]
  const __half* k_new;    // [B,Hkv,D] or null
  const __half* v_new;
  void* out;              // [B,Hq,D]
  int out_is_fp32;
  float* scores;          // [B,Hq,len(+1)] or null
  int score_stride;       // len (+1)
  int ntc;                // most tiles any workgroup of the tile kernel gets (set by the launcher)
  int nparts;             // partials per (sequence, query head)
  int len_shortest;       // cached tokens of the shortest sequence (= len unless the sequences differ in length)
  int lds_logits;         // fused form: the head's raw logits fit the workgroup's LDS (set by the launcher); else they wait in the score buffer
  float* partial;         // two-kernel form: [B*Hq][part_stride][D+4] partial results (max, sum, X) of the parts
  int part_stride;        // partials reserved per (sequence, query head)
};

struct QaqPrefillArgs {
  QaqView v;
  int T, n_rows, G;
  const __half* q;        // [B,Hq,n_rows,D]: queries of prompt positions T-n_rows .. T-1
  const __half* k;        // [B,Hkv,T,D]
  float* scores;          // [n_rows][B,Hq,T]
};

struct QaqExportArgs {
  QaqView v;
  int len, side;
  uint8_t* bits;
  uint16_t* minmax;
  uint8_t* oidx;
  uint16_t* oval;
  uint8_t* codes;
};

struct QaqDequantArgs {
  QaqView v;
  int len, t0, t1;
  __half* out[2];
};

// launchers (each returns the hipError_t of the launch)
hipError_t qaq_launch_init(const QaqView& v, hipStream_t s);
hipError_t qaq_launch_build(const QaqBuildArgs& a, int ntiles, hipStream_t s);
// decode-step update (a.mode == 2): the fast kernel where the configuration has one, followed by the
// general kernel on the tile sides it handed over; else the general kernel on every tile side
hipError_t qaq_launch_update(const QaqBuildArgs& a, int ntiles, hipStream_t s);
hipError_t qaq_launch_select(const QaqSelectArgs& a, hipStream_t s);
// ev: NULL, or four events that take the start and the end of the dispatch of the tile kernel
// ([0], [1]) and of the merge kernel ([2], [3], two-kernel form only); *kernels = dispatches
// made (0 for an empty cache without timing, 1 fused, 2 tile + merge)
// static_scratch: the partial results of the two-kernel form go to the library's file-scope device
// array instead of the cache's arena; *too_big is set (and nothing launched) if they do not fit it
hipError_t qaq_launch_attention(const QaqAttnArgs& a, hipStream_t s, hipEvent_t* ev, int* kernels,
                                bool static_scratch = false, bool* too_big = nullptr);
size_t qaq_static_scratch_bytes();
hipError_t qaq_launch_prefill_window(const QaqPrefillArgs& a, hipStream_t s);
hipError_t qaq_launch_export(const QaqExportArgs& a, hipStream_t s);
hipError_t qaq_launch_dequant(const QaqDequantArgs& a, hipStream_t s);
hipError_t qaq_launch_stats(const QaqView& v, int len, hipStream_t s);
