/*
 * gh_probe.h -- measurement aid, not part of the method: a pure streaming read
 * of device memory in the access shape of the attention kernel (every wave walks
 * its own contiguous share in 16 KiB tiles of whole 128-byte lines, one to three
 * tiles in flight, non-temporal loads), optionally interleaved with record-sized stores.
 * It gives the rate the memory system delivers to this access pattern when no
 * arithmetic, no strip border and no ragged tail is in the way -- the practical
 * ceiling the attention kernel's achieved bandwidth is read against (the
 * roofline itself stays the published 8 TB/s).
 */
#ifndef GH_PROBE_H
#define GH_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { GH_PROBE_STORE_PLAIN = 0, GH_PROBE_STORE_NT = 1, GH_PROBE_STORE_WRITE_THROUGH = 2 } gh_probe_store;

/*
 * Streams `bytes` bytes at `src` (device, 16-byte aligned) once with n_waves
 * waves.  bytes must be a multiple of n_waves * 32 KiB and n_waves a multiple of
 * 4 in [4, 65536].  store_every > 0: after every store_every tiles (an odd number counts as
 * the next even one) a wave writes
 * 4 KiB to its own place in `rec` (device, n_waves * 4 KiB, 16-byte aligned) with
 * the given policy; 0: no stores and rec may be null.  sink: one device word
 * that keeps the loads alive (written only if the data XORs to a magic value).
 * Waves run in workgroups of four; with n_waves <= 1024 every workgroup is placed
 * on a compute unit of its own (one wave per SIMD; it reserves LDS it does not use).
 * Asynchronous on hip_stream.  Returns a gh_status (gh_tier2.h): GH_ERR_NULL,
 * GH_ERR_SHAPE for sizes that do not divide, GH_ERR_UNSUPPORTED for alignment
 * or an unknown policy, GH_ERR_HIP if the launch failed.
 */
int32_t gh_probe_stream_read(const void* src, size_t bytes, int32_t n_waves, int32_t store_every,
                             int32_t store_policy, void* rec, uint32_t* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* GH_PROBE_H */
