/*
 * fk_bench - measurement helper of libfk.so, kept apart from the method's interface (fk.h): it is what bench.py
 * times to report the achievable streaming bandwidth of the box beside the nominal HBM peak.
 */
#ifndef FK_BENCH_H
#define FK_BENCH_H

#include "fk.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Reads `bytes` (>= 16; a multiple of 16 is read, a tail below 16 bytes is ignored) of DEVICE memory at `src`
 * (16-byte aligned) with 16-byte non-temporal loads and discards them; `sink` is 4 bytes of device memory that is
 * practically never written.  Buffers from 352 MB on (beyond the Infinity Cache) are read in whole 8 KB chunks per
 * wavefront, smaller ones grid-strided: the fastest shapes of a sweep on MI355X (7.0 TB/s on 4 GB).  One launch on
 * `stream`; FK_ERR_INVALID_ARG on null or misaligned pointers.
 */
fk_status fk_stream_read(const void *src, size_t bytes, void *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FK_BENCH_H */
