/*
 * wcc_probe.h -- C ABI of libwcc_probe.so, a measurement aid that sits beside libwcc and is not
 * part of it: plain streaming kernels of known size, timed by bench.py next to the kernels of
 * the WCC path so that their rates can be placed against what this device's memory system gives
 * to the simplest possible code (and not only against the published peak).
 */
#ifndef WCC_PROBE_H
#define WCC_PROBE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { WCC_PROBE_READ = 0, WCC_PROBE_WRITE = 1, WCC_PROBE_COPY = 2, WCC_PROBE_WRITE8 = 3 };
enum {
  WCC_PROBE_OK = 0,
  WCC_PROBE_ERR_NULL = 1, /* a required pointer is NULL                                   */
  WCC_PROBE_ERR_SIZE = 2, /* bytes not a positive multiple of 16, blocks out of range, or
                             a pointer that is not 16-byte aligned                        */
  WCC_PROBE_ERR_KIND = 3, /* unknown kind                                                 */
  WCC_PROBE_ERR_HIP = 7   /* the HIP runtime reported an error                            */
};

/* One streaming kernel over `bytes` bytes (a multiple of 16, > 0) enqueued on `stream` (a
 * hipStream_t as void*, NULL = the null stream); src and dst are DEVICE pointers owned by the
 * caller, 16-byte aligned.  READ sums src and writes nothing (dst must still point at >= 16
 * writable bytes); WRITE fills dst with the floats 1, 2, 3, 4 repeated; COPY moves src to dst
 * (the two must not overlap); WRITE8 is WRITE with eight stores a thread, a workgroup covering
 * 32 KiB in a row (`blocks` is ignored).  nontemporal != 0: the accesses carry the non-temporal
 * hint.  blocks: workgroups of 256 threads that walk the buffer with a grid stride (0: 8192; at
 * most 2^24).  Nothing is enqueued when a status other than WCC_PROBE_OK is returned. */
int wcc_probe_stream(int kind, const void *src, void *dst, size_t bytes, int nontemporal,
                     int blocks, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* WCC_PROBE_H */
