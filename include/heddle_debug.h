/*
 * heddle_debug.h - measurement aids of libheddle, apart from the product interface in heddle.h:
 * per-kernel event timers and a plain streaming-read kernel.  A serving engine does not need them;
 * the benchmark and the tests do.
 */
#ifndef HEDDLE_DEBUG_H
#define HEDDLE_DEBUG_H

#include "heddle.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---- kernel timers ------------------------------------------------------------
 * Average duration in microseconds of the dominant kernel of the last
 * `heddle_attn_decode` / `heddle_attn_append` calls, measured with HIP events
 * recorded on the caller's stream around that kernel.  Recording is off by
 * default; heddle_timing_enable(ctx, N) with N >= 1 clears the statistics and
 * records every N-th launch of each kernel (each recorded launch costs two
 * event records, a few microseconds of stream time); 0 turns it off.
 * heddle_timing_read synchronises the recorded events.  which: 0 = split-K
 * decode kernel, 1 = combine kernel, 2 = append attention kernel, 3 = KV write of an
 * append (a decode step's new rows are stored by the launch that uploads its plan),
 * 4 = pack, 5 = unpack, 6 = shared-prefix kernel, 7 = matrix-core kernel for tiles of few rows
 * (short chunks; decode with 8 query heads per kv head or a number of them the
 * split-K kernel is not built for). */
int heddle_timing_enable(heddle_ctx* ctx, int32_t on);
int heddle_timing_read(heddle_ctx* ctx, int32_t which, double* avg_us, int64_t* n_launches);
/* The recorded launches one by one: writes the durations (microseconds) of up to
 * `cap` of them to us_out (HOST, in no particular order once more than 2048 were
 * recorded and old ones overwritten) and the number held to *n_out; cap = 0
 * only counts.  Synchronises the recorded events. */
int heddle_timing_samples(heddle_ctx* ctx, int32_t which, int64_t cap, float* us_out, int64_t* n_out);

/* What the context's scratch holds at the moment, in bytes: out3[0] plan buffer (device),
 * out3[1] split-K partials (device), out3[2] pinned staging ring (host).  A value that
 * changes between two calls means the call in between reallocated (and synchronised):
 * after heddle_ctx_reserve no call within the reserved limits may change them. */
int heddle_ctx_scratch_bytes(const heddle_ctx* ctx, uint64_t* out3 /* HOST [3] */);

/* Streams `bytes` bytes from `src` (DEVICE) through a plain coalesced read kernel
 * and writes one checksum word per workgroup to `sink` (DEVICE, >= 4096 uint32);
 * used to measure the streaming-read ceiling of the device. */
int heddle_stream_read(const void* src, uint64_t bytes, uint32_t* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* HEDDLE_DEBUG_H */
