/*
 * libqaq -- measurement and test aids.  Not part of the product interface of qaq.h: the
 * benchmark uses the first two groups, the layout tests the third.  Same conventions as
 * qaq.h (return codes, device / host pointers, `stream`).
 */
#ifndef QAQ_AUX_H
#define QAQ_AUX_H

#include "qaq.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Measurement aid: after qaq_profile_begin(c, n), the next n qaq_decode_attention calls
 * attach HIP events to the start and the end of their kernel dispatches.  qaq_profile_read
 * waits for them and returns, per call, the milliseconds of the kernel that scans the cache
 * (host_ms_tile) and, where the call needed a second kernel to merge partial results, the
 * time from the end of the first to the end of the second (host_ms_merge; 0 for a call that
 * ran as one kernel).  Host arrays of at least n floats.  n = 0 switches it off. */
int qaq_profile_begin(qaq_cache* c, int32_t max_calls);
int qaq_profile_read(qaq_cache* c, float* host_ms_tile, float* host_ms_merge, int32_t* n_calls);

/* Measurement aids: plain streaming kernels over caller-owned device memory, the yardstick
 * for what this GPU sustains on a pure read (16-byte loads, every byte once, a checksum
 * per workgroup written to dev_sink[0..4095] so that the loads are kept) and on a copy.
 * bytes must be a multiple of 16, pointers 16-byte aligned.  Asynchronous on `stream`. */
int qaq_stream_read(const void* dev_src, size_t bytes, uint32_t* dev_sink, void* stream);
int qaq_stream_copy(void* dev_dst, const void* dev_src, size_t bytes, void* stream);

/* Host-only helpers for layout tests (no device access): where the device layout keeps
 * the bf-bit field (bf = 2, 4, 8; 1 = the low bit of a 3-bit token; 0 = the code of a
 * 1-bit token) of token `idx` of its region, channel d, for a tile side with the given
 * class counts: byte offset of the 32-bit word from the start of the tile side, bit
 * position inside it, and the end of the last region.  And the bytes reserved per tile
 * side. */
int qaq_debug_field(int32_t side, int32_t D, int32_t n3, int32_t n2, int32_t n4, int32_t n8, int32_t n1,
                    int32_t bf, int32_t idx, int32_t d, uint32_t* byte_off, int32_t* shift,
                    uint32_t* region_end);
uint32_t qaq_debug_tile_capacity(int32_t side, int32_t D);

#ifdef __cplusplus
}
#endif
#endif /* QAQ_AUX_H */
