/*
 * distattn_probe.h - measurement aids, kept apart from the attention path and built into a library of their
 * own (libdistattn_probe.so); libdistattn.so does not contain them.
 *
 * Section 5.3, Eq. 5 prices attention by bytes of KV cache read; this call measures what a pure read costs on
 * the GPU at hand, the practical ceiling next to the published HBM peak that the MicroAttention kernels are
 * reported against.
 */
#ifndef DISTATTN_PROBE_H
#define DISTATTN_PROBE_H

#include "distattn.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Streams `bytes` of DEVICE memory at `src` once with 16-byte-per-lane loads and discards the data.
 * `workgroups` workgroups of 512 threads walk `segment_bytes` segments round-robin; `variant` picks the loads in
 * flight per wavefront (0: 4, 1: 8, 2: 16, 3: 8 non-temporal, 4: 16 non-temporal).  `sink` is 4 bytes of device
 * memory (never written unless the data sums to a sentinel).  Enqueued on `stream`; no synchronisation.
 * Errors: DA_ERR_INVALID_ARG for null pointers, sizes that are not multiples of 16 bytes or an unknown variant;
 * DA_ERR_HIP if the launch fails.
 */
da_status da_probe_read(const void *src, size_t bytes, size_t segment_bytes, int32_t workgroups, int32_t variant,
                        void *sink, void *stream);

/*
 * Plain copy of `bytes` bytes (a multiple of 16, both pointers 16-byte aligned DEVICE memory, not overlapping):
 * a kernel that reads exactly `bytes` and writes exactly `bytes`, each once.  What a hardware traffic counter
 * reads for it gives the factor by which the same counter's reading for another kernel is scaled.
 * Errors as for da_probe_read.
 */
da_status da_probe_copy(const void *src, void *dst, size_t bytes, void *stream);

/*
 * Streaming reads with small result writes mixed in, the memory pattern of many short requests (Section 5.3: an
 * instance that lends memory hosts many conversations): `workgroups` x 4 wavefronts each read items of
 * `item_bytes` (the K/V of one short request and kv-head) from `src` (`bytes` in all, dealt round-robin) and write
 * `frag_bytes` of result per item into `dst`, after every `burst` items (0 = never; a value >= the items per
 * wavefront = once, at the end), all wavefronts at the same items (`staggered` = 0) or each at a phase of its own.
 * Timed by the caller, it shows what the write pattern costs the read stream.  Sizes are multiples of 16 bytes,
 * pointers 16-byte aligned DEVICE memory, `dst_bytes` >= bytes / item_bytes * frag_bytes.  Errors as for
 * da_probe_read.
 */
da_status da_probe_read_write(const void *src, size_t bytes, void *dst, size_t dst_bytes, size_t item_bytes,
                              size_t frag_bytes, int32_t workgroups, int32_t burst, int32_t staggered, void *sink,
                              void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DISTATTN_PROBE_H */
