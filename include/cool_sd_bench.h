/*
 * cool_sd_bench.h -- C ABI of libcool_sd_bench.so, the benchmark companion of libcool_sd.so.
 *
 * Built from the same kernels.  It lets a benchmark time the HBM-bound statistics pass of a
 * verify call (softmax statistics of every target and draft row, Algorithm 1's inputs p_i and
 * q_i) on its own, next to a plain streaming read of the same bytes.  Nothing here belongs in a
 * production path, and the product library exports none of it.  Conventions as in cool_sd.h:
 * device pointers, caller-owned buffers, asynchronous on the given stream, negative status on
 * argument errors detected before anything is enqueued, no state kept between calls.
 */
#ifndef COOL_SD_BENCH_H
#define COOL_SD_BENCH_H

#include "cool_sd.h"

#ifdef __cplusplus
extern "C" {
#endif

/* The statistics pass of cool_sd_verify ALONE, with the grid, chunking and load flavour the
 * verify call would choose for these params and pointers (p->flags is ignored): reads every
 * logit once and leaves the chunk statistics in the workspace; writes no output of the method.
 * Arguments as in cool_sd_verify. */
COOL_SD_API int cool_sd_bench_row_stats(const cool_sd_params* p,
                                        const void* target_dev, const void* target_uncond_dev,
                                        const void* draft_dev, const void* draft_uncond_dev,
                                        const int32_t* draft_tokens_dev,
                                        void* workspace_dev, size_t workspace_bytes,
                                        void* hip_stream);

/* A plain streaming read of two device buffers in ONE launch with the launch shape of the
 * row-statistics kernel on short rows (256 threads, 16 bytes per lane and load, 8 KiB per
 * workgroup) and no arithmetic beyond an exclusive-or of the words -- what this GPU delivers for
 * that many bytes in one launch, start-up included.  a_dev / b_dev: 16-byte aligned, sizes
 * multiples of 16 (b_bytes may be 0); workspace_dev: at least 4 bytes per 8 KiB read (rounded up
 * per buffer), receives one word per workgroup. */
COOL_SD_API int cool_sd_bench_read_probe(const void* a_dev, size_t a_bytes, const void* b_dev, size_t b_bytes,
                                         void* workspace_dev, size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* COOL_SD_BENCH_H */
