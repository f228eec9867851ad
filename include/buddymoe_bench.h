/* buddymoe_bench.h - measurement aids exported by libbuddymoe.so beside the layer's
 * C ABI (buddymoe.h).  Nothing here is part of the forward pass; the benchmark
 * uses it to quote the HBM read rate a kernel can reach on the device. */
#ifndef BUDDYMOE_BENCH_H
#define BUDDYMOE_BENCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Reads `bytes` bytes (a multiple of 16,
 * device memory, 16-byte aligned) once with the access pattern of the decode
 * weight stream - every wave instruction a contiguous kilobyte, eight in flight
 * per wave, non-temporal - and discards them.  Its throughput is the HBM read
 * rate a kernel can reach on this device, the practical ceiling beside the
 * datasheet figure the roofline fractions are quoted against.  sink: one
 * device uint32 the kernel may write (it keeps the loads alive).  bytes = 0
 * does nothing (src may then be NULL).
 * Returns a bm_status of buddymoe.h: BM_OK, BM_ERR_NULL, BM_ERR_SHAPE (bytes not a
 * multiple of 16) or BM_ERR_HIP. */
int bm_stream_read(const void *src, size_t bytes, uint32_t *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BUDDYMOE_BENCH_H */
