/*
 * caat_tools.h -- measuring tools that libcaat.so exports next to the method's C ABI (include/caat.h).  They are not
 * part of the method: bench.py binds them to time every launch of a block call and to probe HBM streaming rates.
 */
#ifndef CAAT_TOOLS_H
#define CAAT_TOOLS_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Per-launch timing of the block calls (a host-side measuring tool, not part of the method): while enabled,
 * caat_block_fwd / caat_block_bwd bracket every kernel they enqueue with a pair of HIP events on the caller's
 * stream.  caat_profile_get waits for record `index` (in launch order since the last reset) and returns a
 * static kernel-family name (host pointer to a NUL-terminated string) and the elapsed milliseconds.  Events
 * are created on first use and reused after a reset.  Not thread-safe; off by default.
 */
int caat_profile_enable(int on);
int caat_profile_reset(void);
int caat_profile_count(void);
int caat_profile_get(int index, const char** name, float* ms);

/*
 * HBM streaming probe (a measuring tool, not part of the method): enqueues one kernel that reads `bytes` bytes of
 * the device buffer `src` (16-byte aligned, bytes % 16 == 0) and, for the copy modes, writes them to `dst`.
 *   mode 0: read, every workgroup walks its own contiguous piece, plain loads
 *   mode 1: the same with the non-temporal hint on the loads
 *   mode 2: read, the whole grid sweeps one window (grid-stride), plain loads
 *   mode 3: copy src -> dst, contiguous piece per workgroup, plain loads and stores
 *   mode 4: the same with the non-temporal hint on loads and stores
 * dst may be NULL for the read modes (a result is only stored if the data hash to one particular value, which
 * keeps the loads alive; pass a buffer of at least 16 bytes to be safe).  The caller times it with events on
 * `hip_stream`; bench.py --probe-hbm does.  This is where the cache-policy choices of the streaming kernels
 * (which accesses carry the hint) were measured.
 */
int caat_hbm_probe(const void* src, void* dst, size_t bytes, int mode, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* CAAT_TOOLS_H */
