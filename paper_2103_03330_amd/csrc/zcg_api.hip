// C-ABI entry points of libzcgather: table handles, the gather dispatch, the
// index check and the link-peak probe. Kernels live in zcg_kernels.hip, the
// CPU-gather baseline in zcg_cpu_baseline.hip.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <unordered_set>
#include <vector>

#include "zcg_internal.h"

namespace {

std::mutex g_mu;
std::unordered_set<const zcg_table*> g_live;
thread_local int t_last_hip = 0;

int elem_of(int dtype) {
  if (dtype == ZCG_F16) return 2;
  if (dtype == ZCG_F32) return 4;
  if (dtype == ZCG_B8) return 1;
  if (dtype == ZCG_B64) return 8;
  return 0;
}

int check_shape(int64_t n_rows, int64_t dim, int dtype, zcg_table** out, int* elem) {
  if (!out) return ZCG_EINVAL;
  *out = nullptr;
  *elem = elem_of(dtype);
  if (!*elem) return ZCG_EDTYPE;
  if (n_rows <= 0 || dim <= 0) return ZCG_EINVAL;
  if (dim > (INT64_MAX / *elem) || n_rows > INT64_MAX / (dim * *elem)) return ZCG_EINVAL;
  return ZCG_OK;
}

zcg_table* make_handle(int kind, int dtype, int elem, int device, void* host, void* dev,
                       int64_t n_rows, int64_t dim) {
  zcg_table* t = new (std::nothrow) zcg_table;
  if (!t) return nullptr;
  t->kind = kind; t->dtype = dtype; t->elem = elem; t->device = device;
  t->host = host; t->dev = dev; t->n_rows = n_rows; t->dim = dim;
  t->row_bytes = dim * elem;
  std::lock_guard<std::mutex> lk(g_mu);
  g_live.insert(t);
  return t;
}

// Makes `device` current for the lifetime of the object, then restores.
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

}  // namespace

bool zcg_is_live(const zcg_table* t) {
  if (!t) return false;
  std::lock_guard<std::mutex> lk(g_mu);
  return g_live.count(t) != 0;
}

int zcg_fail_hip(hipError_t e) {
  t_last_hip = (int)e;
  (void)hipGetLastError();  // do not leave a sticky error for the caller's next HIP call
  return ZCG_EHIP;
}

extern "C" {

const char* zcg_version(void) { return "0.1"; }

const char* zcg_strerror(int status) {
  switch (status) {
    case ZCG_OK: return "ok";
    case ZCG_EINVAL: return "invalid argument";
    case ZCG_EDTYPE: return "unsupported element type";
    case ZCG_EHANDLE: return "not a live table handle";
    case ZCG_EHIP: return "HIP runtime call failed";
    case ZCG_ENOMEM: return "out of host memory";
    case ZCG_EALIGN: return "pointer not aligned to the element size";
    case ZCG_EALIAS: return "output overlaps the table";
    case ZCG_ERANGE: return "index out of range";
    case ZCG_EBUSY: return "buffer not released by the consumer";
    case ZCG_ETIMEDOUT: return "wait timed out";
    case ZCG_ECLOSED: return "pipeline finished by the producer";
    default: return "unknown status";
  }
}

int zcg_last_hip_error(void) { return t_last_hip; }

int zcg_register_table(void* host_ptr, int64_t n_rows, int64_t dim, int dtype, int device,
                       zcg_table** out) {
  int elem;
  int rc = check_shape(n_rows, dim, dtype, out, &elem);
  if (rc) return rc;
  if (!host_ptr || device < 0) return ZCG_EINVAL;
  if ((uintptr_t)host_ptr % (uintptr_t)elem) return ZCG_EALIGN;
  DeviceScope scope(device);
  if (scope.err != hipSuccess) return zcg_fail_hip(scope.err);
  const size_t bytes = (size_t)(n_rows * dim * elem);
  hipError_t e = hipHostRegister(host_ptr, bytes, hipHostRegisterMapped | hipHostRegisterPortable);
  if (e != hipSuccess) return zcg_fail_hip(e);
  void* dev = nullptr;
  e = hipHostGetDevicePointer(&dev, host_ptr, 0);
  if (e != hipSuccess || !dev) {
    (void)hipHostUnregister(host_ptr);
    return zcg_fail_hip(e != hipSuccess ? e : hipErrorInvalidValue);
  }
  zcg_table* t = make_handle(ZCG_KIND_REGISTERED, dtype, elem, device, host_ptr, dev, n_rows, dim);
  if (!t) {
    (void)hipHostUnregister(host_ptr);
    return ZCG_ENOMEM;
  }
  *out = t;
  return ZCG_OK;
}

int zcg_alloc_table(int64_t n_rows, int64_t dim, int dtype, unsigned flags, int device,
                    zcg_table** out) {
  int elem;
  int rc = check_shape(n_rows, dim, dtype, out, &elem);
  if (rc) return rc;
  if (device < 0 || (flags & ~(ZCG_ALLOC_NONCOHERENT | ZCG_ALLOC_NUMA_USER | ZCG_ALLOC_UNCACHED))) return ZCG_EINVAL;
  DeviceScope scope(device);
  if (scope.err != hipSuccess) return zcg_fail_hip(scope.err);
  unsigned hip_flags = hipHostMallocMapped | hipHostMallocPortable;
  if ((flags & ZCG_ALLOC_NONCOHERENT) && (flags & ZCG_ALLOC_UNCACHED)) return ZCG_EINVAL;
  if (flags & ZCG_ALLOC_UNCACHED) hip_flags |= hipHostMallocUncached;
  else hip_flags |= (flags & ZCG_ALLOC_NONCOHERENT) ? hipHostMallocNonCoherent : hipHostMallocCoherent;
  if (flags & ZCG_ALLOC_NUMA_USER) hip_flags |= hipHostMallocNumaUser;
  void* host = nullptr;
  hipError_t e = hipHostMalloc(&host, (size_t)(n_rows * dim * elem), hip_flags);
  if (e != hipSuccess || !host) return zcg_fail_hip(e != hipSuccess ? e : hipErrorOutOfMemory);
  void* dev = nullptr;
  e = hipHostGetDevicePointer(&dev, host, 0);
  if (e != hipSuccess || !dev) {
    (void)hipHostFree(host);
    return zcg_fail_hip(e != hipSuccess ? e : hipErrorInvalidValue);
  }
  zcg_table* t = make_handle(ZCG_KIND_ALLOCATED, dtype, elem, device, host, dev, n_rows, dim);
  if (!t) {
    (void)hipHostFree(host);
    return ZCG_ENOMEM;
  }
  *out = t;
  return ZCG_OK;
}

int zcg_table_from_device(void* dev_ptr, int64_t n_rows, int64_t dim, int dtype, int device,
                          zcg_table** out) {
  int elem;
  int rc = check_shape(n_rows, dim, dtype, out, &elem);
  if (rc) return rc;
  if (!dev_ptr || device < 0) return ZCG_EINVAL;
  if ((uintptr_t)dev_ptr % (uintptr_t)elem) return ZCG_EALIGN;
  zcg_table* t = make_handle(ZCG_KIND_DEVICE, dtype, elem, device, nullptr, dev_ptr, n_rows, dim);
  if (!t) return ZCG_ENOMEM;
  *out = t;
  return ZCG_OK;
}

void* zcg_table_device_ptr(const zcg_table* t) { return zcg_is_live(t) ? t->dev : nullptr; }
void* zcg_table_host_ptr(const zcg_table* t) { return zcg_is_live(t) ? t->host : nullptr; }
int64_t zcg_table_row_bytes(const zcg_table* t) { return zcg_is_live(t) ? t->row_bytes : 0; }
int64_t zcg_table_n_rows(const zcg_table* t) { return zcg_is_live(t) ? t->n_rows : 0; }

int zcg_unregister_table(zcg_table* t) {
  {
    std::lock_guard<std::mutex> lk(g_mu);
    if (!t || g_live.erase(t) == 0) return ZCG_EHANDLE;
  }
  int rc = ZCG_OK;
  if (t->kind == ZCG_KIND_REGISTERED) {
    hipError_t e = hipHostUnregister(t->host);
    if (e != hipSuccess) rc = zcg_fail_hip(e);
  } else if (t->kind == ZCG_KIND_ALLOCATED) {
    hipError_t e = hipHostFree(t->host);
    if (e != hipSuccess) rc = zcg_fail_hip(e);
  }
  delete t;
  return rc;
}

int zcg_plan_gather(const zcg_table* t, int64_t n_idx, const void* out_dev,
                    const zcg_launch_opts* opts, zcg_plan* plan) {
  if (!zcg_is_live(t)) return ZCG_EHANDLE;
  return zcg_make_plan(t->row_bytes, t->elem, (uintptr_t)t->dev, (uintptr_t)out_dev, n_idx,
                       t->kind != ZCG_KIND_DEVICE, false, opts, plan);
}

static int gather_common(const zcg_table* t, const int64_t* idx_dev, const int64_t* order_dev,
                         int64_t n_idx, void* out_dev, void* stream, const zcg_launch_opts* opts) {
  if (!zcg_is_live(t)) return ZCG_EHANDLE;
  if (n_idx < 0) return ZCG_EINVAL;
  if (n_idx == 0) return ZCG_OK;
  if (!idx_dev || !out_dev) return ZCG_EINVAL;
  if ((uintptr_t)idx_dev % 8 || (uintptr_t)order_dev % 8) return ZCG_EALIGN;
  if (n_idx > INT64_MAX / t->row_bytes) return ZCG_EINVAL;
  const uintptr_t o0 = (uintptr_t)out_dev, o1 = o0 + (uintptr_t)(n_idx * t->row_bytes);
  const uintptr_t t0 = (uintptr_t)t->dev, t1 = t0 + (uintptr_t)(t->n_rows * t->row_bytes);
  if (o0 < t1 && t0 < o1) return ZCG_EALIAS;
  const bool host_resident = t->kind != ZCG_KIND_DEVICE;
  zcg_plan plan;
  int rc = zcg_make_plan(t->row_bytes, t->elem, t0, o0, n_idx, host_resident, order_dev != nullptr, opts,
                         &plan);
  if (rc) return rc;
  if (order_dev && plan.variant == ZCG_VARIANT_NAIVE) return ZCG_EINVAL;
  hipError_t e = zcg_launch_gather(plan, t->dev, idx_dev, order_dev, n_idx, out_dev, t->row_bytes,
                                   t->elem, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ZCG_OK : zcg_fail_hip(e);
}

int zcg_gather_ex(const zcg_table* t, const int64_t* idx_dev, int64_t n_idx, void* out_dev,
                  void* stream, const zcg_launch_opts* opts) {
  return gather_common(t, idx_dev, nullptr, n_idx, out_dev, stream, opts);
}

int zcg_gather_ordered(const zcg_table* t, const int64_t* idx_dev, const int64_t* order_dev,
                       int64_t n_idx, void* out_dev, void* stream, const zcg_launch_opts* opts) {
  if (n_idx > 0 && !order_dev) return ZCG_EINVAL;
  return gather_common(t, idx_dev, order_dev, n_idx, out_dev, stream, opts);
}

int zcg_gather(const zcg_table* t, const int64_t* idx_dev, int64_t n_idx, void* out_dev,
               void* stream) {
  return zcg_gather_ex(t, idx_dev, n_idx, out_dev, stream, nullptr);
}

int zcg_gather_variant(const zcg_table* t, const int64_t* idx_dev, int64_t n_idx, void* out_dev,
                       void* stream, int variant) {
  zcg_launch_opts o = {};
  o.variant = variant;
  return zcg_gather_ex(t, idx_dev, n_idx, out_dev, stream, &o);
}

int zcg_validate_indices(const zcg_table* t, const int64_t* idx_dev, int64_t n_idx, void* stream,
                         int64_t* n_bad_host) {
  if (!zcg_is_live(t)) return ZCG_EHANDLE;
  if (!n_bad_host || n_idx < 0 || (n_idx > 0 && !idx_dev)) return ZCG_EINVAL;
  *n_bad_host = 0;
  if (n_idx == 0) return ZCG_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned long long* d = nullptr;
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&d), sizeof(*d));
  if (e != hipSuccess) return zcg_fail_hip(e);
  unsigned long long h = 0;
  e = hipMemcpyAsync(d, &h, sizeof(h), hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e == hipSuccess) e = zcg_launch_validate(idx_dev, n_idx, t->n_rows, d, s);
  if (e == hipSuccess) e = hipMemcpyAsync(&h, d, sizeof(h), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  (void)hipFree(d);
  if (e != hipSuccess) return zcg_fail_hip(e);
  *n_bad_host = (int64_t)h;
  return ZCG_OK;
}

int zcg_measure_h2d(int64_t bytes, int reps, int device, double* gb_per_s) {
  if (bytes <= 0 || reps < 1 || reps > 1000 || device < 0 || !gb_per_s) return ZCG_EINVAL;
  *gb_per_s = 0.0;
  DeviceScope scope(device);
  if (scope.err != hipSuccess) return zcg_fail_hip(scope.err);
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
  if (e != hipSuccess) return zcg_fail_hip(e);
  std::sort(ms.begin(), ms.end());
  const double med = ms[ms.size() / 2];
  *gb_per_s = (double)bytes / (med * 1e-3) / 1e9;
  return ZCG_OK;
}

int zcg_device_cu_count(int device, int* n_cus) {
  if (device < 0 || !n_cus) return ZCG_EINVAL;
  int v = 0;
  hipError_t e = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, device);
  if (e != hipSuccess) return zcg_fail_hip(e);
  *n_cus = v;
  return ZCG_OK;
}

int zcg_stream_create_cu_mask(int device, const uint32_t* mask_words, int n_words, void** stream) {
  if (device < 0 || !mask_words || n_words < 1 || n_words > 64 || !stream) return ZCG_EINVAL;
  *stream = nullptr;
  int n_cus = 0;
  int rc = zcg_device_cu_count(device, &n_cus);
  if (rc) return rc;
  int enabled = 0;
  for (int i = 0; i < n_cus && i < n_words * 32; ++i) enabled += (mask_words[i / 32] >> (i % 32)) & 1u;
  if (enabled == 0) return ZCG_EINVAL;  // a stream that can run nowhere would hang its first kernel
  DeviceScope scope(device);
  if (scope.err != hipSuccess) return zcg_fail_hip(scope.err);
  hipStream_t s = nullptr;
  hipError_t e = hipExtStreamCreateWithCUMask(&s, (uint32_t)n_words, mask_words);
  if (e != hipSuccess) return zcg_fail_hip(e);
  *stream = s;
  return ZCG_OK;
}

int zcg_stream_destroy(void* stream) {
  if (!stream) return ZCG_EINVAL;
  hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
  if (e == hipSuccess) e = hipStreamDestroy(static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ZCG_OK : zcg_fail_hip(e);
}

int zcg_synthetic_compute(void* stream, int blocks, int64_t iters, float* sink_dev) {
  if (blocks < 1 || blocks > (1 << 20) || iters < 0 || iters > ((int64_t)1 << 32) || !sink_dev)
    return ZCG_EINVAL;
  hipError_t e = zcg_launch_synthetic_compute(static_cast<hipStream_t>(stream), blocks, iters, sink_dev);
  return e == hipSuccess ? ZCG_OK : zcg_fail_hip(e);
}

int zcg_measure_host_read_latency(int device, int64_t hops, double* microseconds) {
  if (device < 0 || hops < 16 || hops > (1 << 22) || !microseconds) return ZCG_EINVAL;
  *microseconds = 0.0;
  DeviceScope scope(device);
  if (scope.err != hipSuccess) return zcg_fail_hip(scope.err);
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
    e = zcg_launch_chase(s, dev_view, kStrideWords, 64, result);  // warm-up
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e == hipSuccess) e = hipEventRecord(e0, s);
    if (e == hipSuccess) e = zcg_launch_chase(s, dev_view, kStrideWords, hops, result);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  }
  if (e1) (void)hipEventDestroy(e1);
  if (e0) (void)hipEventDestroy(e0);
  if (s) (void)hipStreamDestroy(s);
  if (result) (void)hipFree(result);
  if (host) (void)hipHostFree(host);
  if (e != hipSuccess) return zcg_fail_hip(e);
  *microseconds = (double)ms * 1e3 / (double)hops;
  return ZCG_OK;
}

int zcg_measure_host_stream_read(int device, int64_t bytes, int reps, double* gb_per_s) {
  if (device < 0 || bytes < 4096 || bytes % 4096 || reps < 1 || reps > 1000 || !gb_per_s)
    return ZCG_EINVAL;
  *gb_per_s = 0.0;
  DeviceScope scope(device);
  if (scope.err != hipSuccess) return zcg_fail_hip(scope.err);
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
    e = zcg_launch_stream_read(s, dev_view, dst, bytes, 2048);  // warm-up
    if (e == hipSuccess) e = hipStreamSynchronize(s);
  }
  for (int r = 0; r < reps && e == hipSuccess; ++r) {
    e = hipEventRecord(e0, s);
    if (e == hipSuccess) e = zcg_launch_stream_read(s, dev_view, dst, bytes, 2048);
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
  if (e != hipSuccess) return zcg_fail_hip(e);
  std::sort(ms.begin(), ms.end());
  *gb_per_s = (double)bytes / ((double)ms[ms.size() / 2] * 1e-3) / 1e9;
  return ZCG_OK;
}

int zcg_pinned_alloc(int64_t bytes, void** host_ptr) {
  if (bytes <= 0 || !host_ptr) return ZCG_EINVAL;
  *host_ptr = nullptr;
  hipError_t e = hipHostMalloc(host_ptr, (size_t)bytes, hipHostMallocDefault);
  return e == hipSuccess ? ZCG_OK : zcg_fail_hip(e);
}

int zcg_pinned_free(void* host_ptr) {
  if (!host_ptr) return ZCG_EINVAL;
  hipError_t e = hipHostFree(host_ptr);
  return e == hipSuccess ? ZCG_OK : zcg_fail_hip(e);
}

}  // extern "C"
