/*
 * st_probe.h -- machine probes for the benchmark (libst_probe.so, a library of its own: nothing of
 * the streaming-constrained attention path is in it, and nothing in libst.so needs it).  They
 * measure what this GPU sustains for the access pattern of the decode kernel and for the matrix
 * instruction the prefill kernel lives on, so that a roofline fraction can be read against a
 * measured ceiling and not only against the data-sheet peak.
 *
 * st_probe_paged_read: n_waves one-wave workgroups each read steps_per_wave x 16 KiB from `pool`
 *   (device memory, pool_bytes a power of two >= 4 KiB, 16-byte aligned) as the decode kernel
 *   reads a paged bf16 cache with head_dim 128: four pseudo-random 4 KiB pages per step, 16 loads
 *   of 16 bytes per lane with its per-lane addressing.  `salt` shifts the page choice: give every
 *   launch another one and, with a pool much larger than the caches, nothing is found cached.
 *   Bytes read per launch = n_waves * steps_per_wave * 16384.  sink: device uint32 (practically
 *   never written).
 * st_probe_mfma_bf16: n_workgroups x 4 waves each issue iterations x 8 v_mfma_f32_32x32x16_bf16
 *   on register operands with random mantissas; flop per launch =
 *   n_workgroups * 4 * iterations * 8 * 32768.  sink: device float.
 * Both enqueue one kernel on hip_stream (a hipStream_t as void*) and return 0, or 1 on bad
 * arguments, 6 if the launch failed (the values of st_status in st.h).
 */
#ifndef ST_PROBE_H
#define ST_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

int32_t st_probe_paged_read(const void* pool, size_t pool_bytes, int32_t n_waves, int32_t steps_per_wave,
                            uint32_t salt, uint32_t* sink, void* hip_stream);
int32_t st_probe_mfma_bf16(int32_t n_workgroups, int32_t iterations, float* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ST_PROBE_H */
