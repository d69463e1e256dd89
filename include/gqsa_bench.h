/*
 * gqsa_bench.h -- measuring instruments that ship in libgqsa.so beside the GQSA path: kernels
 * whose numbers the benchmark reports next to the product's (same GPU, same harness).  They are
 * not part of the method and no product call depends on them.
 *
 *   - a dense fp16 GEMV: the FP16 baseline of the paper's end-to-end tables (Tab. 4, Tab. 13).
 *     The dense 4-bit baseline of Tab. 4 / Tab. 10 (Eq. 1-3 with nothing pruned) needs no kernel
 *     of its own: it is gqsa_pack with sparsity 0;
 *   - a read-only streaming kernel: the HBM read rate that is achievable at a given size;
 *   - a copy kernel of exactly known traffic (calibrates the profiler's byte counters);
 *   - an empty launch with the GEMV's geometry (what a launch costs by itself).
 *
 * Same conventions as gqsa.h: C linkage, [device] pointers are plain device addresses, every
 * call only enqueues on `hip_stream` and returns a gqsa_status_t.
 */
#ifndef GQSA_BENCH_H
#define GQSA_BENCH_H

#include "gqsa.h"

#ifdef __cplusplus
extern "C" {
#endif

/* y[batch,N] = W[N,K] x[batch,K], all fp16 [device], fp32 accumulation. */
gqsa_status_t gqsa_dense_f16_gemv(const void* W_dev, const void* x_dev, void* y_dev,
                                  int64_t N, int64_t K, int batch, void* hip_stream);

/* XOR `bytes` (multiple of 16) of device memory into sink_dev[0..n_wg-1] (uint32 each; n_wg =
 * gqsa_stream_read_workgroups() entries must be there, a small buffer writes fewer): a pure read
 * at full width, every workgroup reading its own contiguous share. */
gqsa_status_t gqsa_stream_read(const void* buf_dev, size_t bytes, void* sink_dev, void* hip_stream);
int gqsa_stream_read_workgroups(void);

/* dst[0..bytes) = src[0..bytes), both [device], 16-byte aligned, bytes a multiple of 16: a kernel
 * of exactly known HBM traffic, used to calibrate the profiler's byte counters. */
gqsa_status_t gqsa_copy(void* dst_dev, const void* src_dev, size_t bytes, void* hip_stream);

/* Launch an empty kernel with the GEMV's geometry (n_workgroups x 1024 threads, lds_bytes of
 * LDS): the cost of a launch by itself, for the benchmark report.  sink_dev [device] non-NULL. */
gqsa_status_t gqsa_launch_floor(int n_workgroups, int lds_bytes, void* sink_dev, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* GQSA_BENCH_H */
