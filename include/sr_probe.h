/*
 * sr_probe.h -- streaming probes of libsrdict.so: what the memory system of the
 * GPU delivers for the byte mix of the dictionary-assembly path (section II-A,
 * Eq. 2: L coefficient planes read once per HR pixel, C output planes written)
 * when no arithmetic stands in the way.  They exist for measurement only: the
 * benchmark reports the assembly kernel's time next to theirs, as an empirical
 * ceiling beside the nominal HBM peak.  They compute nothing of the method.
 *
 * Pointers are DEVICE pointers owned by the caller; work is enqueued on
 * `stream` (hipStream_t, NULL = default stream) without synchronising.
 * Returns 0 or a negative sr_status (sr_dict.h): SR_ERR_NULL,
 * SR_ERR_UNSUPPORTED (size or plane count the probe was not built for),
 * SR_ERR_ALIGN (pointer not 16-byte aligned), SR_ERR_LAUNCH.
 */
#ifndef SR_PROBE_H
#define SR_PROBE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Reads `bytes` (a multiple of 16) from `src` once with non-temporal 16-byte
 * loads and folds them into one word; `sink` (>= 4 bytes) is written only if
 * that word has one particular value, so the loads cannot be dropped. */
int sr_probe_read(const void* src, size_t bytes, void* sink, void* stream);

/* The assembly kernel's traffic without its work: for every run of 128 pixels
 * reads the run from each of `planes` fp16 planes of `pixels` elements (as the
 * kernel does: 8 bytes per lane, the two lane halves on different planes) and
 * writes the run to each of `channels` fp32 planes of `pixels` elements.
 * planes must be 72 or 128, 1 <= channels <= 4, pixels a multiple of 128. */
int sr_probe_mix(const void* coeff, int planes, size_t pixels, void* out, int channels, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SR_PROBE_H */
