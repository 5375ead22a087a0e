/*
 * tokencake_kv, measurement helpers.  NOT part of the serving boundary (tokencake_kv.h): these calls exist
 * for the benchmark, the profiles and the parity tests of the kernels' measurement modes.  They keep no
 * bookkeeping: no ownership check, no in-flight marks, no hazards between streams.  The caller holds every
 * block and buffer it names exclusively until the stream it passes has completed.
 */
#ifndef TOKENCAKE_KV_BENCH_H
#define TOKENCAKE_KV_BENCH_H

#include "tokencake_kv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* dst[i] = src[i]: contiguous DEVICE->DEVICE copy with the gather kernel's access width; the
 * "achievable HBM" reference and the calibration kernel for the traffic counters.
 * bytes must be a multiple of 16. */
int tc_copy_contiguous(void *dst, const void *src, uint64_t bytes, void *stream);
/* The same DEVICE->DEVICE copy with every tile staged in LDS: lds_direct_loads = 0 goes through
 * registers into LDS and back, 1 uses LDS-direct loads.  Kept to measure what LDS staging adds to
 * a copy without reuse (on MI355X it is 3 to 10 % slower than the register path).  bytes must be a multiple of 16 384, both
 * pointers 16-B aligned, the ranges must not overlap; TC_ERR_INVAL otherwise. */
int tc_copy_via_lds(void *dst, const void *src, uint64_t bytes, int lds_direct_loads, void *stream);
/* `iters` launches of a[i] = b[i] + s*c[i] over n fp32 (DEVICE): the HBM-streaming neighbour that
 * the copy stream is overlapped with.  n must be a multiple of 4. */
int tc_hbm_stream(float *a, const float *b, const float *c, uint64_t n, float s, uint32_t iters, void *stream);
/* Comparators without a gather kernel: mode 0 = one hipMemcpyAsync per page, mode 1 = one
 * hipMemcpy2DAsync per block.  direction 0 = offload, 1 = upload.  No bookkeeping. */
int tc_naive_transfer(tc_ctx *ctx, const int32_t *block_ids, uint32_t n, void *host_buf, int mode,
                      int direction, void *stream);

/* One-way HBM streams with the copy kernels' tile and workgroup mapping, to measure what the memory system
 * sustains in each direction: tc_hbm_write stores a pattern to `bytes` of DEVICE memory (non-temporal),
 * tc_hbm_read loads `bytes` and stores nothing.  bytes must be a multiple of 4096, pointers 16-B aligned. */
int tc_hbm_write(void *dst, uint64_t bytes, void *stream);
int tc_hbm_read(const void *src, uint64_t bytes, void *stream);
/* The staged path's copy kernel alone, on records the caller keeps in DEVICE memory: direction 0 =
 * gather_pages (dev_records[j] <- block block_ids[j]), 1 = scatter_pages (block block_ids[j] <- dev_records[j]).
 * n at most the blocks of one staging slot's worth is not required: the launch covers all n records.  Lets a
 * profiler see the kernels with the record side in a known cache state (e.g. filled by tc_copy_contiguous,
 * whose non-temporal stores leave it in HBM, as the copy engine does).  The ids go through the context's id
 * ring like a transfer's; TC_ERR_RANGE / TC_ERR_DUP for bad ids, TC_ERR_INVAL if dev_records is not device
 * memory or n exceeds the ring. */
int tc_stage_on_device(tc_ctx *ctx, int direction, const int32_t *block_ids, uint32_t n, void *dev_records,
                       void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TOKENCAKE_KV_BENCH_H */
