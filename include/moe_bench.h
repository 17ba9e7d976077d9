/*
 * moe_bench.h - C ABI of libmoe_bench.so, the measurement helpers of bench.py.  Nothing here is a
 * step of the MoE layer and the product library (moe_janus.h) does not depend on it.
 */
#ifndef MOE_BENCH_H
#define MOE_BENCH_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Streams `bytes` (rounded down to 16) from src_dev with plain coalesced 128-bit loads and
 * discards them, as a grid of `workgroups` workgroups of 256 threads that each keep
 * `loads_in_flight` (1, 2, 4, 8 or 16) independent loads per thread in flight.  Janus Sec. 2.2: the
 * MoE layer is bound by reading the activated experts' weights; bench.py sweeps this probe over
 * launch shapes and reports its best point next to the FFN kernel's rate.
 * sink_dev: 256 bytes of device memory (written practically never).  src_dev 16-byte aligned.
 * Asynchronous on `stream` (a hipStream_t).  Returns 0, -1 (bad argument) or -4 (launch failed). */
int moe_read_probe(const void *src_dev, size_t bytes, void *sink_dev, int workgroups, int loads_in_flight,
                   void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_BENCH_H */
