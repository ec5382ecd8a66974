/*
 * zipccl_yardstick.h -- C ABI of libzipccl_yardstick.so: a measurement aid, not part of the codec library.
 *
 * A plain device-to-device copy kernel for gfx950 (16 bytes per lane, one load and one store per thread, the
 * fastest plain form measured).  The benchmark reports its rate as the practical ceiling next to the HBM peak,
 * and counter runs use it to scale FETCH_SIZE / WRITE_SIZE readings.
 *   d_dst / d_src  device, 16-byte aligned; bytes a multiple of 16; asynchronous on `stream` (hipStream_t as void*)
 * Returns 0, 1 for bad arguments, 5 when the launch failed.
 */
#ifndef ZIPCCL_YARDSTICK_H
#define ZIPCCL_YARDSTICK_H
#include <stddef.h>
#ifdef __cplusplus
extern "C" {
#endif
int zipccl_yardstick_copy(void* d_dst, const void* d_src, size_t bytes, void* stream);
#ifdef __cplusplus
}
#endif
#endif
