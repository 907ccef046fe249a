// libzcgprobe: measurement probes around the gather (link peak, shader-issued read rate and
// latency of mapped host memory, a known-size copy, a stand-in compute kernel). Tooling for
// the benchmark and the tests; shares no code with libzcgather.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <utility>
#include <vector>

#include "zcg_probe.h"

namespace {

constexpr int kBlock = 256;
thread_local int t_last_hip = 0;

int fail_hip(hipError_t e) {
  t_last_hip = (int)e;
  (void)hipGetLastError();  // do not leave a sticky error for the caller's next HIP call
  return ZCGP_EHIP;
}

struct DeviceScope {
  int prev = -1;
  hipError_t err;
  explicit DeviceScope(int device) {
    err = hipGetDevice(&prev);
    if (err == hipSuccess && prev != device) err = hipSetDevice(device);
  }
  ~DeviceScope() {
    int cur = -1;
    if (prev >= 0 && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
  }
};

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __align__(64) uint32_t zcgp_dummy_chunk[16];

// ALU-bound stand-in for a training kernel: a chain of dependent FMAs per lane.
__global__ void __launch_bounds__(kBlock)
zcgp_k_synthetic_compute(int64_t iters, float* __restrict__ sink) {
  float a = 1.0f + (float)threadIdx.x * 1e-6f, b = 0.999999f, c = 1e-7f;
  for (int64_t i = 0; i < iters; ++i) a = __builtin_fmaf(a, b, c);
  atomicAdd(&sink[threadIdx.x], a);
}

// One lane follows a chain of dependent loads: next = chain[next * stride].
__global__ void zcgp_k_chase(const uint64_t* __restrict__ chain, int64_t stride_words, int64_t hops,
                             uint64_t* __restrict__ result) {
  uint64_t p = 0;
  for (int64_t i = 0; i < hops; ++i)
    p = *(const volatile uint64_t __attribute__((address_space(1)))*)(chain + p * stride_words);
  *result = p;
}

// Streams n_chunks consecutive 8-byte chunks from src to dst: the gather's own access shape
// (8-byte lanes, two wave passes in flight, non-temporal stores) with nothing to look up.
__global__ void __launch_bounds__(kBlock)
zcgp_k_stream_read(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst, int64_t n_chunks) {
  constexpr int W = 8, U = 2;
  const int64_t lanes = (int64_t)gridDim.x * kBlock;
  const uint8_t* dummy = reinterpret_cast<const uint8_t*>(zcgp_dummy_chunk);
  for (int64_t c0 = (int64_t)blockIdx.x * kBlock + threadIdx.x; c0 < n_chunks; c0 += lanes * U) {
    u32x2 v[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t c = c0 + (int64_t)u * lanes;
      ok[u] = c < n_chunks;
      v[u] = *reinterpret_cast<const u32x2*>(ok[u] ? src + c * W : dummy);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u])
        __builtin_nontemporal_store(v[u], reinterpret_cast<u32x2*>(dst + (c0 + (int64_t)u * lanes) * W));
  }
}

__global__ void __launch_bounds__(kBlock)
zcgp_k_copy(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t n_chunks) {
  const int64_t lanes = (int64_t)gridDim.x * kBlock;
  for (int64_t c = (int64_t)blockIdx.x * kBlock + threadIdx.x; c < n_chunks; c += lanes) dst[c] = src[c];
}

hipError_t launch_stream_read(hipStream_t s, const void* src, void* dst, int64_t bytes, int blocks) {
  zcgp_k_stream_read<<<dim3((unsigned)blocks), dim3(kBlock), 0, s>>>(
      static_cast<const uint8_t*>(src), static_cast<uint8_t*>(dst), bytes / 8);
  return hipGetLastError();
}

}  // namespace

extern "C" {

int zcgp_last_hip_error(void) { return t_last_hip; }

int zcgp_measure_h2d(int64_t bytes, int reps, int device, double* gb_per_s) {
  if (bytes <= 0 || reps < 1 || reps > 1000 || device < 0 || !gb_per_s) return ZCGP_EINVAL;
  *gb_per_s = 0.0;
  DeviceScope scope(device);
  if (scope.err != hipSuccess) return fail_hip(scope.err);
  void *h = nullptr, *d = nullptr;
  hipStream_t s = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  std::vector<float> ms;
  hipError_t e = hipHostMalloc(&h, (size_t)bytes, hipHostMallocDefault);
  if (e == hipSuccess) e = hipMalloc(&d, (size_t)bytes);
  if (e == hipSuccess) e = hipStreamCreate(&s);
  if (e == hipSuccess) e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  if (e == hipSuccess) {
    // touch the pages so the first timed copy does not pay for faults
    for (int64_t i = 0; i < bytes; i += 4096) static_cast<volatile char*>(h)[i] = (char)i;
    e = hipMemcpyAsync(d, h, (size_t)bytes, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
  }
  for (int r = 0; r < reps && e == hipSuccess; ++r) {
    e = hipEventRecord(e0, s);
    if (e == hipSuccess) e = hipMemcpyAsync(d, h, (size_t)bytes, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float t = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&t, e0, e1);
    if (e == hipSuccess) ms.push_back(t);
  }
  if (e1) (void)hipEventDestroy(e1);
  if (e0) (void)hipEventDestroy(e0);
  if (s) (void)hipStreamDestroy(s);
  if (d) (void)hipFree(d);
  if (h) (void)hipHostFree(h);
  if (e != hipSuccess) return fail_hip(e);
  std::sort(ms.begin(), ms.end());
  const double med = ms[ms.size() / 2];
  *gb_per_s = (double)bytes / (med * 1e-3) / 1e9;
  return ZCGP_OK;
}

int zcgp_synthetic_compute(void* stream, int blocks, int64_t iters, float* sink_dev) {
  if (blocks < 1 || blocks > (1 << 20) || iters < 0 || iters > ((int64_t)1 << 32) || !sink_dev)
    return ZCGP_EINVAL;
  zcgp_k_synthetic_compute<<<dim3((unsigned)blocks), dim3(kBlock), 0, static_cast<hipStream_t>(stream)>>>(
      iters, sink_dev);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? ZCGP_OK : fail_hip(e);
}

int zcgp_device_copy(void* dst_dev, const void* src_dev, int64_t bytes, void* stream) {
  if (!dst_dev || !src_dev || bytes <= 0 || bytes % 16 || ((uintptr_t)dst_dev | (uintptr_t)src_dev) % 16)
    return ZCGP_EINVAL;
  const int64_t n_chunks = bytes / 16;
  int64_t blocks = (n_chunks + kBlock - 1) / kBlock;
  if (blocks > 16384) blocks = 16384;
  zcgp_k_copy<<<dim3((unsigned)blocks), dim3(kBlock), 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const u32x4*>(src_dev), static_cast<u32x4*>(dst_dev), n_chunks);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? ZCGP_OK : fail_hip(e);
}

int zcgp_measure_host_read_latency(int device, int64_t hops, double* microseconds) {
  if (device < 0 || hops < 16 || hops > (1 << 22) || !microseconds) return ZCGP_EINVAL;
  *microseconds = 0.0;
  DeviceScope scope(device);
  if (scope.err != hipSuccess) return fail_hip(scope.err);
  // a random cycle over 2^16 slots, one slot per 4 KiB page of a 256 MiB mapped host buffer
  constexpr int64_t kSlots = 1 << 16, kStrideWords = 4096 / 8;
  uint64_t *host = nullptr, *dev_view = nullptr, *result = nullptr;
  hipStream_t s = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  float ms = 0.f;
  hipError_t e = hipHostMalloc(reinterpret_cast<void**>(&host), (size_t)kSlots * 4096,
                               hipHostMallocMapped | hipHostMallocCoherent);
  if (e == hipSuccess) e = hipHostGetDevicePointer(reinterpret_cast<void**>(&dev_view), host, 0);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&result), sizeof(uint64_t));
  if (e == hipSuccess) e = hipStreamCreate(&s);
  if (e == hipSuccess) e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  if (e == hipSuccess) {
    std::vector<uint64_t> perm((size_t)kSlots);
    for (int64_t i = 0; i < kSlots; ++i) perm[(size_t)i] = (uint64_t)i;
    uint64_t x = 0x9E3779B97F4A7C15ull;
    for (int64_t i = kSlots - 1; i > 0; --i) {  // Fisher-Yates with a xorshift stream
      x ^= x << 13; x ^= x >> 7; x ^= x << 17;
      std::swap(perm[(size_t)i], perm[(size_t)(x % (uint64_t)(i + 1))]);
    }
    for (int64_t i = 0; i < kSlots; ++i)  // perm order becomes one cycle through all slots
      host[perm[(size_t)i] * kStrideWords] = perm[(size_t)((i + 1) % kSlots)];
    zcgp_k_chase<<<dim3(1), dim3(1), 0, s>>>(dev_view, kStrideWords, 64, result);  // warm-up
    e = hipGetLastError();
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e == hipSuccess) e = hipEventRecord(e0, s);
    if (e == hipSuccess) {
      zcgp_k_chase<<<dim3(1), dim3(1), 0, s>>>(dev_view, kStrideWords, hops, result);
      e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  }
  if (e1) (void)hipEventDestroy(e1);
  if (e0) (void)hipEventDestroy(e0);
  if (s) (void)hipStreamDestroy(s);
  if (result) (void)hipFree(result);
  if (host) (void)hipHostFree(host);
  if (e != hipSuccess) return fail_hip(e);
  *microseconds = (double)ms * 1e3 / (double)hops;
  return ZCGP_OK;
}

int zcgp_measure_host_stream_read(int device, int64_t bytes, int reps, double* gb_per_s) {
  if (device < 0 || bytes < 4096 || bytes % 4096 || reps < 1 || reps > 1000 || !gb_per_s)
    return ZCGP_EINVAL;
  *gb_per_s = 0.0;
  DeviceScope scope(device);
  if (scope.err != hipSuccess) return fail_hip(scope.err);
  void *host = nullptr, *dev_view = nullptr, *dst = nullptr;
  hipStream_t s = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  std::vector<float> ms;
  hipError_t e = hipHostMalloc(&host, (size_t)bytes, hipHostMallocMapped | hipHostMallocCoherent);
  if (e == hipSuccess) e = hipHostGetDevicePointer(&dev_view, host, 0);
  if (e == hipSuccess) e = hipMalloc(&dst, (size_t)bytes);
  if (e == hipSuccess) e = hipStreamCreate(&s);
  if (e == hipSuccess) e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  if (e == hipSuccess) {
    for (int64_t i = 0; i < bytes; i += 4096) static_cast<volatile char*>(host)[i] = (char)i;
    e = launch_stream_read(s, dev_view, dst, bytes, 2048);  // warm-up
    if (e == hipSuccess) e = hipStreamSynchronize(s);
  }
  for (int r = 0; r < reps && e == hipSuccess; ++r) {
    e = hipEventRecord(e0, s);
    if (e == hipSuccess) e = launch_stream_read(s, dev_view, dst, bytes, 2048);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float t = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&t, e0, e1);
    if (e == hipSuccess) ms.push_back(t);
  }
  if (e1) (void)hipEventDestroy(e1);
  if (e0) (void)hipEventDestroy(e0);
  if (s) (void)hipStreamDestroy(s);
  if (dst) (void)hipFree(dst);
  if (host) (void)hipHostFree(host);
  if (e != hipSuccess) return fail_hip(e);
  std::sort(ms.begin(), ms.end());
  *gb_per_s = (double)bytes / ((double)ms[ms.size() / 2] * 1e-3) / 1e9;
  return ZCGP_OK;
}

}  // extern "C"
