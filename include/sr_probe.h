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

/* The same bytes in the assembly kernel's own ORDER: persistent workgroups walk 128 x tile_h tiles of a
 * height x width frame as the kernel does (its split of the tiles over the eight XCDs, four wavefronts on
 * rows w, w + 4, ... of a tile), each wavefront reading one row of 128 pixels from every plane and writing
 * it to every output plane; no LDS, no barrier, no arithmetic.  planes 72 or 128, 1 <= channels <= 4,
 * width a multiple of 128, 1 <= tile_h <= 64, height * width < 2^31. */
int sr_probe_mix_tiled(const void* coeff, int planes, int height, int width, int tile_h, void* out, int channels,
                       void* stream);

/* As sr_probe_mix_tiled, for planes of `elem_bytes`-byte coefficients: 2 (the call above) or 1 (the kernel's
 * 8-bit form: 4 bytes per lane and plane, half the read stream for the same writes). */
int sr_probe_mix_tiled_bytes(const void* coeff, int planes, int elem_bytes, int height, int width, int tile_h, void* out,
                             int channels, void* stream);

/* As sr_probe_mix_tiled_bytes, with the assembly kernel's L2 write-back pacing among the requests: pace_us > 0 makes one
 * wavefront per XCD ask its L2 every pace_us microseconds to write its dirty lines back (the kernel's period is 16);
 * 0 = none, 0 <= pace_us <= 1 000 000. */
int sr_probe_mix_tiled_paced(const void* coeff, int planes, int elem_bytes, int height, int width, int tile_h, void* out,
                             int channels, int pace_us, void* stream);

/* A byte mix with NOTHING of the assembly kernel's access pattern in it: one launch of
 * `blocks` workgroups of 256 threads in which every `writer_every`-th workgroup only
 * writes (16-byte stores sweeping `dst`, `write_bytes` in all) and all others only read
 * (16-byte non-temporal loads sweeping `src`, `read_bytes` in all), so that loads and
 * stores never share a wavefront.  writer_every = 0 (with write_bytes = 0): read only;
 * writer_every = 1 (with read_bytes = 0): write only.  `lds_bytes` of dynamic LDS per
 * workgroup are requested but not used: they cap the workgroups resident per CU
 * (more than 80 KB leaves one per CU, so `blocks` <= 256 then counts the CUs in use).
 * nt_store != 0 writes with non-temporal stores.  Sizes are multiples of 16, pointers
 * 16-byte aligned; `sink` as for sr_probe_read. */
int sr_probe_stream(const void* src, size_t read_bytes, void* dst, size_t write_bytes, int blocks,
                    int writer_every, int lds_bytes, int nt_store, void* sink, void* stream);

/* The byte mix of a frame with 72 fp16 coefficient planes and 3 fp32 output planes of
 * `pixels` elements each (a multiple of 128), changing one property of sr_probe_stream's
 * ideal pattern at a time: read_planes != 0 reads 256-byte pieces from each of the 72
 * planes of `src` (8 bytes per lane, as the assembly kernel does) instead of one
 * contiguous sweep; write_planes != 0 writes 512-byte pieces into each of the 3 planes of
 * `dst` (8 bytes per lane) instead of one contiguous sweep; same_wave != 0 lets every
 * wavefront read and write (otherwise every writer_every-th workgroup, >= 2, only writes).
 * read_planes == 2 (with write_planes and same_wave set): 16 bytes per lane both ways,
 * i.e. 512-byte pieces of the coefficient planes and 1 KB pieces of the output planes.
 * plane_pad_bytes (a multiple of 16, plane reads only) is added to the distance between
 * coefficient planes, which shows what the planes' common low address bits cost.
 * pixels is a multiple of 256; src holds 72 * (2 * pixels + plane_pad_bytes) bytes, dst
 * 12 * pixels bytes, both 16-byte aligned. */
int sr_probe_pattern(const void* src, void* dst, size_t pixels, int read_planes, int write_planes, int same_wave,
                     int blocks, int writer_every, size_t plane_pad_bytes, void* sink, void* stream);

/* The assembly kernel's own mix (sr_probe_pattern with read_planes = write_planes =
 * same_wave = 1) under other cache policies: load_policy / store_policy 0 plain, 1
 * non-temporal, 2 agent scope, 3 system scope.  flush_every > 0: one wavefront per XCD also
 * has its L2 write its dirty lines back after every flush_every-th of its runs.  blocks >= 8. */
int sr_probe_policy(const void* src, void* dst, size_t pixels, int load_policy, int store_policy, int flush_every,
                    int blocks, void* sink, void* stream);

/* As sr_probe_policy, with any combination of the three cache-policy bits of a gfx950 global
 * load / store: load_bits, store_bits = sc0 (1) | sc1 (2) | nt (4). */
int sr_probe_policy_bits(const void* src, void* dst, size_t pixels, int load_bits, int store_bits, int blocks,
                         void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SR_PROBE_H */
