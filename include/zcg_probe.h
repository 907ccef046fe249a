/*
 * zcg_probe -- measurement probes that go with the zcgather library: the link
 * peak (the metric's denominator), the rate and latency of GPU-issued reads of
 * mapped host memory, a known-size copy for calibrating traffic counters, and a
 * compute kernel that stands in for training. Benchmark and test tooling in a
 * shared object of its own (libzcgprobe.so); nothing here is part of the gather.
 *
 * Every call returns 0 or a negative status: ZCGP_EINVAL for a bad argument,
 * ZCGP_EHIP when a HIP runtime call failed (zcgp_last_hip_error() then gives the
 * hipError_t of the calling thread).
 */
#ifndef ZCG_PROBE_H
#define ZCG_PROBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ZCGP_OK 0
#define ZCGP_EINVAL (-1)
#define ZCGP_EHIP (-4)

int zcgp_last_hip_error(void);

/*
 * Link-peak probe: median over `reps` timed pinned host-to-device hipMemcpyAsync
 * copies of `bytes` bytes, after one warm-up, in GB/s (1e9 bytes). The paper
 * quotes its gather against this block-copy rate (Section 4.1, Section 4.2).
 * SYNCHRONOUS; allocates and frees its buffers.
 */
int zcgp_measure_h2d(int64_t bytes, int reps, int device, double* gb_per_s);

/*
 * Round-trip time of one read of mapped host memory from a GPU lane: a single
 * lane follows `hops` (16 .. 2^22) dependent loads through a random cycle laid
 * over a 256 MiB mapped buffer, one slot per page. With the measured request
 * rate this gives the number of reads in flight (Little's law, the sizing
 * argument of Section 3.2.2). SYNCHRONOUS; allocates and frees its buffers.
 */
int zcgp_measure_host_read_latency(int device, int64_t hops, double* microseconds);

/*
 * The rate at which GPU lanes themselves can pull consecutive bytes of mapped
 * host memory into HBM (the ceiling of any zero-copy gather): median over
 * `reps` runs of a plain streaming kernel with the gather's access shape over a
 * fresh mapped buffer of `bytes` bytes (a multiple of 4096), in GB/s (1e9
 * bytes). Compare with zcgp_measure_h2d, the copy engine's rate over the same
 * link. SYNCHRONOUS; allocates and frees its buffers.
 */
int zcgp_measure_host_stream_read(int device, int64_t bytes, int reps, double* gb_per_s);

/*
 * A plain device-to-device copy kernel of exactly `bytes` bytes (a multiple of
 * 16; src_dev, dst_dev device, CALLER-OWNED, 16-byte aligned), asynchronous on
 * `stream`: the known-size reference that hardware traffic counters are scaled by.
 */
int zcgp_device_copy(void* dst_dev, const void* src_dev, int64_t bytes, void* stream);

/*
 * A stand-in for the training kernels the gather overlaps with (Section 3.2.2,
 * Section 4.3): `blocks` blocks of 256 lanes, each lane runs `iters` dependent
 * fused multiply-adds and adds its result into sink_dev[lane id mod 256]
 * (device, 256 floats, CALLER-OWNED). Pure ALU work, asynchronous on `stream`.
 */
int zcgp_synthetic_compute(void* stream, int blocks, int64_t iters, float* sink_dev);

#ifdef __cplusplus
}
#endif
#endif /* ZCG_PROBE_H */
