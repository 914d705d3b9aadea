/*
 * Measurement aids for the benchmark; not part of libbittrain's interface.
 *
 * libbittrain_bench.so is the codec's source compiled once more with per-tile time stamps
 * (-DBT_TIMELINE, so every bt_* call of include/bittrain.h is in it as well) plus the two calls
 * below.  Only bench.py loads it.
 */
#ifndef BITTRAIN_BENCH_AIDS_H
#define BITTRAIN_BENCH_AIDS_H

#include "bittrain.h"

#ifdef __cplusplus
extern "C" {
#endif

/* A plain stream with the traffic shape of the codec kernels and no dependency between
 * workgroups: what the memory system gives that shape at best.  Workgroup t of `tiles` reads
 * read_rows rows of 4 KiB from d_in and writes write_rows rows of 4 KiB to d_out, each contiguous:
 * d_in must hold tiles * read_rows * 4096 bytes and d_out tiles * write_rows * 4096 bytes (at least
 * 16 * tiles bytes when write_rows is 0), both 16-byte aligned.  d_out receives arbitrary bytes.
 * (read_rows, write_rows) is one of (8,4) the compress shape at 50 % zeros, (4,8) the decompress
 * shape, (8,8), (8,0), (0,8); anything else: BT_ERR_SIZE. */
bt_status bt_stream_probe(const void *d_in, void *d_out, uint64_t tiles, int read_rows, int write_rows,
                          bt_stream stream);

/* From this call on, every bt_compress / bt_decompress launch (and their relatives) records into
 * d_buf, for each slot t < tiles, eight uint64 at d_buf[8 * t], times of the 100 MHz device clock:
 * [0] the tile's loads were asked for, [1] its count was published, [2] its prefix was seen,
 * [3] its stores were issued, [5] polls of the wave so far; and the scanner records, for each of its
 * first max_passes passes that consumed counts, two uint64 at d_buf[8 * tiles + 2 * pass]: the
 * clock, and (first slot << 32 | end slot) of the pass.  d_buf is device memory of buf_words uint64
 * (>= 8 * tiles + 2 * max_passes, else BT_ERR_SIZE), 8-byte aligned, zeroed by the caller;
 * d_buf == NULL switches recording off.  This call waits for the device (it copies to device
 * variables), and recording calls must not overlap.  Errors: BT_ERR_ALIGN, BT_ERR_SIZE, BT_ERR_HIP. */
bt_status bt_timeline_set(uint64_t *d_buf, uint64_t buf_words, uint32_t tiles, uint32_t max_passes);

#ifdef __cplusplus
}
#endif
#endif /* BITTRAIN_BENCH_AIDS_H */
