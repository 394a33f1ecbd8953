/*
 * parallax_util.h -- measurement helpers that ship in the same library as the Parallax attention
 * entry points of parallax.h but are NOT part of the method: a plain copy kernel (calibrates the
 * hardware byte counters against a known size), plain read kernels (the streaming bandwidth a
 * kernel of a given size can reach on the box: the floor next to the decode numbers) and a
 * register-only matrix loop (the matrix rate the chip sustains). bench.py and the profile runs
 * call them; the attention path does not. Same conventions as parallax.h: device pointers owned
 * by the caller, enqueued on the caller's stream, no synchronisation, validation on the host.
 */
#ifndef PARALLAX_UTIL_H
#define PARALLAX_UTIL_H

#include "parallax.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Plain device-to-device copy kernel (16 bytes per lane, grid-stride). Used to calibrate
 * hardware byte counters and to measure the achievable streaming bandwidth next to the
 * attention kernels. bytes must be a multiple of 16; pointers 16-byte aligned. */
plx_status parallax_util_copy(void *dst, const void *src, size_t bytes, void *hip_stream);

/* Streams `bytes` from src and writes one 16-byte checksum per workgroup to sink
 * (>= 16 * parallax_util_read_sink_slots() bytes): a read-only bandwidth ceiling. */
plx_status parallax_util_read(const void *src, size_t bytes, void *sink, void *hip_stream);
int32_t parallax_util_read_sink_slots(void);

/* Register-only loop of dense bf16 matrix instructions (v_mfma_f32_32x32x16_bf16, eight
 * independent accumulators per wave, no memory or LDS traffic): the matrix throughput the chip
 * sustains on this machine, reported next to the nominal peak. `workgroups` of 4 waves each run
 * `iters` trips of 8 instructions, i.e. workgroups * 4 * iters * 8 * 32768 flops; sink (device,
 * >= workgroups * 1024 bytes, 4-byte aligned) receives one float per lane so that the work
 * cannot be dropped. 1 <= workgroups <= 65536, 1 <= iters <= 2^24. */
plx_status parallax_util_mfma(int32_t workgroups, int32_t iters, void *sink, void *hip_stream);

/* parallax_util_read with a chosen number of workgroups (1 .. parallax_util_read_sink_slots()):
 * 256 is one persistent workgroup per compute unit, 4096 what parallax_util_read launches. Each
 * lane keeps eight 16-byte loads in flight. For finding the best a plain read can do at the byte
 * count of a small decode step, where launch and ramp weigh as much as the stream itself. */
plx_status parallax_util_read_grid(const void *src, size_t bytes, void *sink, int32_t workgroups,
                                   void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PARALLAX_UTIL_H */
