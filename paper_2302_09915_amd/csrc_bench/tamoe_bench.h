/*
 * tamoe_bench.h - yardsticks that bench.py times beside the kernels of the path (libtamoe_bench.so).
 * Not part of the product library and not steps of the method: plain memory kernels with none of the
 * method's logic.  All pointers are device memory of the current device; calls only enqueue on
 * `stream` (a hipStream_t passed as void*).  Return 0, 1 (bad argument) or 2 (launch rejected).
 */
#ifndef TAMOE_BENCH_H
#define TAMOE_BENCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { TAMOE_BENCH_OK = 0, TAMOE_BENCH_BAD_ARG = 1, TAMOE_BENCH_HIP_ERROR = 2 };

/*
 * A plain copy of `bytes` bytes (a multiple of 16) from src to dst, both 16-byte aligned, not
 * overlapping, with one 16-byte load and store per lane.  It moves exactly 2*bytes through HBM, so its
 * duration gives the bandwidth a simple streaming kernel reaches on the machine, and hardware byte
 * counters read for it calibrate the same counters read for the kernels of the path.
 */
int tamoe_copy_probe(const void* src, void* dst, size_t bytes, void* stream);

/*
 * The bare memory operations of the scatter and of the combine on caller-given row tables.
 *   mode 1: b[row0[t]][:] = b[row1[t]][:] = a[t][:]      for t < rows   (one read, two writes)
 *   mode 2: b[t][:] = a[row0[t]][:] xor a[row1[t]][:]    for t < rows   (two reads, one write)
 * Rows are row_bytes long (a positive multiple of 1024).  `other_rows` is the number of rows of the
 * matrix that row0/row1 index (b in mode 1, a in mode 2); entries outside [0, other_rows) are skipped.
 * In mode 1 every row number may occur at most once over both tables.  row0, row1: [rows] int32.
 */
int tamoe_mix_probe(const void* a, void* b, const int32_t* row0, const int32_t* row1, int64_t rows,
                    int64_t other_rows, int row_bytes, int mode, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TAMOE_BENCH_H */
