/*
 * libfdprobe -- measurement aid of the libfdattn benchmark; not part of the method and
 * not part of libfdattn.so.
 */
#ifndef FDPROBE_H
#define FDPROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Enqueue a plain streaming read of two DEVICE buffers of `bytes_each` bytes each (a
 * multiple of 65536, 16-byte aligned) with the launch geometry of the decode chunk
 * kernel at 256 keys per chunk and no arithmetic.  `sink` is 4 bytes of device memory
 * (practically never written).  `stream` is a hipStream_t passed as void*.  Timing this
 * gives the read rate a kernel of that shape can reach on the device at hand: the
 * "measured ceiling" the benchmark reports next to the published HBM peak.
 * Returns 0, 1 (a pointer is NULL), 2 (size or alignment) or 6 (the launch failed).
 */
int fd_probe_stream_read(const void *a, const void *b, size_t bytes_each, void *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FDPROBE_H */
