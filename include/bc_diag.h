/*
 * bc_diag.h - measurement aids around the library of bc.h.  No operation of the paper; built
 * into a library of their own (libbc_diag.so) so that the product library exports only the
 * method.  Used by the benchmark's read-floor workload.
 */
#ifndef BC_DIAG_H
#define BC_DIAG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* `workgroups` workgroups (1..65536) read `bytes` bytes from `src` (device, 16-byte aligned) with
 * coalesced streaming loads, each a contiguous share, and write one word each to
 * sink[workgroups] (device, may be NULL).  With bytes == 0 it is an empty kernel.
 *  mode 0: 16-byte loads into registers, 8 KB in flight per wave, 512 threads per workgroup;
 *          bytes a multiple of 16.
 *  mode 1: LDS-DMA loads of 1 KB per instruction, up to 48 KB in flight per wave, 512 threads per
 *          workgroup; bytes a multiple of 1024.
 * Returns the status codes of bc.h (0 = ok, -1 = bad argument, -6 = launch failure).  Only
 * enqueues work on `stream` (a hipStream_t as void*, NULL = default stream). */
int32_t bc_diag_stream_read(const void *src, size_t bytes, int32_t workgroups, int32_t mode,
                            uint32_t *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BC_DIAG_H */
