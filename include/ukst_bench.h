/*
 * ukst_bench -- measurement helpers of the benchmark, built into a library of their own
 * (libukst_bench.so).  Nothing here is part of the transpose convolution and libukst.so does not
 * contain it: these kernels only measure what the chip sustains, so that a kernel's rate can be
 * printed next to a measured ceiling as well as next to the published peak.
 */
#ifndef UKST_BENCH_H
#define UKST_BENCH_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Enqueues on `stream` one launch of a register-resident loop of independent MFMAs (dtype 1:
 * 32x32x16 bf16, dtype 0: 32x32x2 fp32; `iters` rounds of 4 per wave, two blocks of four waves per
 * compute unit) and returns the floating-point operations that launch performs, or 0 on a bad
 * argument or a failed launch.  The caller times the launch.  `sink` is a DEVICE buffer of at
 * least 64 floats that is practically never written.
 */
double ukst_bench_mfma_ceiling(int dtype, int iters, void* sink, void* stream);

/*
 * Enqueues on `stream` one launch of a plain streaming kernel that reads `read_bytes` from the
 * DEVICE buffer `src` and writes `write_bytes` to the DEVICE buffer `dst` with 16-byte accesses
 * (both sizes multiples of 16, buffers 16-byte aligned; every written value depends on what was
 * read, so neither side can be dropped).  It is the memory traffic of a layer with that much
 * input and output and no arithmetic: the ceiling for that read/write mix.  Returns 0 on
 * success, -1 on a bad argument or a failed launch.  The caller times the launch.
 */
int ukst_bench_stream_ceiling(const void* src, size_t read_bytes, void* dst, size_t write_bytes,
                              void* stream);

#ifdef __cplusplus
}
#endif
#endif /* UKST_BENCH_H */
