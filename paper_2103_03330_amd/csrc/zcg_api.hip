// C-ABI entry points of libzcgather: table handles, the gather dispatch, the
// index check and CU-masked streams. Kernels live in zcg_kernels.hip, the launch
// planning in zcg_plan.hip, the order builder in zcg_order.hip, the CPU-gather
// baseline in zcg_cpu_baseline.hip, the pipeline in zcg_pipeline.hip.
#include <hip/hip_runtime.h>

#include <cmath>
#include <mutex>
#include <new>
#include <unordered_set>

#include "zcg_internal.h"

namespace {

std::mutex g_mu;
std::unordered_set<const zcg_table*> g_live;
uint64_t g_next_serial = 1;  // guarded by g_mu
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
                       int64_t n_rows, int64_t dim, const zcg_table* parent = nullptr) {
  zcg_table* t = new (std::nothrow) zcg_table;
  if (!t) return nullptr;
  t->kind = kind; t->dtype = dtype; t->elem = elem; t->device = device;
  t->parent = parent;
  t->parent_serial = parent ? parent->serial : 0;
  t->host_resident = parent ? parent->host_resident : kind != ZCG_KIND_DEVICE;
  t->host = host; t->dev = dev; t->n_rows = n_rows; t->dim = dim;
  t->row_bytes = dim * elem;
  std::lock_guard<std::mutex> lk(g_mu);
  t->serial = g_next_serial++;
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
  if (g_live.count(t) == 0) return false;
  // a view lives only as long as the very table it slices: a later handle that happens to be
  // allocated at the parent's old address has another serial
  return t->kind != ZCG_KIND_VIEW ||
         (g_live.count(t->parent) != 0 && t->parent->serial == t->parent_serial);
}

int zcg_fail_hip(hipError_t e) {
  t_last_hip = (int)e;
  (void)hipGetLastError();  // do not leave a sticky error for the caller's next HIP call
  return ZCG_EHIP;
}

// Rows of at most one line over the host link are bound by the link's request rate (about 320
// requests per microsecond); walked in ascending table order, listed rows that share a line or
// a 256-byte pair of lines share a request. With lambda listed rows per pair on average, a
// fraction 1 - (1 - exp(-lambda)) / lambda of the requests goes away; measured, about 0.6 of
// that is realised (1 M entries over 10 M rows: 32-byte rows 10.9 -> 14.2 GB/s, 64-byte rows
// 21.5 -> 24.4, 128-byte rows 40.7 -> 45.5). Building the order costs about 12 us per 8-bit
// digit of the row number plus 16 ns per 1,000 entries and digit (37 us for 24-bit row numbers
// and short lists, 84 us for 1 M entries). A caller that lends workspace gets the ordered walk
// from AUTO whenever the saving clearly exceeds that cost -- long lists that are dense in their
// table -- and the plain walk otherwise (262,144 entries over 10 M rows: ordering would save
// 4 % and cost 6 %).
bool zcg_order_pays(const zcg_table* t, int64_t n_idx) {
  if (!t->host_resident || t->row_bytes > 128 || n_idx < 32768 || n_idx > (int64_t)UINT32_MAX)
    return false;
  const double lambda = (double)n_idx * 256.0 / ((double)t->row_bytes * (double)t->n_rows);
  const double shared = 1.0 - (1.0 - std::exp(-lambda)) / lambda;
  const double saved_us = 0.6 * shared * (double)n_idx / 320.0;
  int bits = 1;
  while (bits < 63 && ((int64_t)1 << bits) < t->n_rows) ++bits;
  const double build_us = (double)((bits + 7) / 8) * (12.0 + 0.016e-3 * (double)n_idx);
  return saved_us > 1.25 * build_us;
}

extern "C" {

const char* zcg_version(void) { return "0.2"; }

const char* zcg_strerror(int status) {
  switch (status) {
    case ZCG_OK: return "ok";
    case ZCG_EINVAL: return "invalid argument";
    case ZCG_EDTYPE: return "unsupported element type";
    case ZCG_EHANDLE: return "not a live table handle";
    case ZCG_EHIP: return "HIP runtime call failed";
    case ZCG_ENOMEM: return "out of host memory";
    case ZCG_EALIGN: return "pointer not aligned to the element size";
    case ZCG_EALIAS: return "ranges that must be distinct overlap (output, table, list, order or workspace)";
    case ZCG_ERANGE: return "index out of range";
    case ZCG_EBUSY: return "buffer not released by the consumer";
    case ZCG_ETIMEDOUT: return "wait timed out";
    case ZCG_ECLOSED: return "pipeline finished by the producer";
    case ZCG_ECAPACITY: return "input larger than the entry point's fixed capacity";
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

int zcg_table_view(const zcg_table* parent, int64_t byte_offset, int64_t n_rows, int64_t dim,
                   int dtype, zcg_table** out) {
  int elem;
  int rc = check_shape(n_rows, dim, dtype, out, &elem);
  if (rc) return rc;
  if (!zcg_is_live(parent)) return ZCG_EHANDLE;
  if (byte_offset < 0) return ZCG_EINVAL;
  const int64_t parent_bytes = parent->n_rows * parent->row_bytes;
  const int64_t bytes = n_rows * dim * elem;
  if (byte_offset > parent_bytes || bytes > parent_bytes - byte_offset) return ZCG_EINVAL;
  char* dev = static_cast<char*>(parent->dev) + byte_offset;
  if ((uintptr_t)dev % (uintptr_t)elem) return ZCG_EALIGN;
  void* host = parent->host ? static_cast<char*>(parent->host) + byte_offset : nullptr;
  // a view of a view hangs off the same root, so that liveness is one look-up
  const zcg_table* root = parent->kind == ZCG_KIND_VIEW ? parent->parent : parent;
  zcg_table* t = make_handle(ZCG_KIND_VIEW, dtype, elem, parent->device, host, dev, n_rows, dim, root);
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

static bool wants_order(const zcg_table* t, int64_t n_idx, const zcg_launch_opts* opts) {
  if (!opts || !opts->workspace_dev || opts->variant != ZCG_VARIANT_AUTO) return false;
  if ((uintptr_t)opts->workspace_dev % 256) return false;
  const int64_t order_bytes = (n_idx * 8 + 255) / 256 * 256;
  if (opts->workspace_bytes < order_bytes + zcg_order_scratch_bytes(n_idx)) return false;
  return zcg_order_pays(t, n_idx);
}

int zcg_plan_gather(const zcg_table* t, int64_t n_idx, const void* out_dev,
                    const zcg_launch_opts* opts, zcg_plan* plan) {
  if (!zcg_is_live(t)) return ZCG_EHANDLE;
  const bool ordered = n_idx > 0 && wants_order(t, n_idx, opts);
  int rc = zcg_make_plan(t->row_bytes, t->elem, (uintptr_t)t->dev, (uintptr_t)out_dev, n_idx,
                         t->host_resident, ordered, opts, plan);
  if (rc == ZCG_OK) plan->ordered = ordered ? 1 : 0;
  return rc;
}

int zcg_plan_shape(int64_t row_bytes, int elem_bytes, uint64_t table_addr, uint64_t out_addr,
                   int64_t n_rows, int64_t n_idx, int host_resident, const zcg_launch_opts* opts,
                   zcg_plan* plan) {
  if (!plan || n_rows < 1 || row_bytes < 1) return ZCG_EINVAL;
  zcg_table t = {};  // never registered: only the fields the planning reads
  t.kind = host_resident ? ZCG_KIND_ALLOCATED : ZCG_KIND_DEVICE;
  t.host_resident = host_resident != 0;
  t.elem = elem_bytes;
  t.n_rows = n_rows;
  t.row_bytes = row_bytes;
  const bool ordered = n_idx > 0 && wants_order(&t, n_idx, opts);
  int rc = zcg_make_plan(row_bytes, elem_bytes, (uintptr_t)table_addr, (uintptr_t)out_addr, n_idx,
                         t.host_resident, ordered, opts, plan);
  if (rc == ZCG_OK) plan->ordered = ordered ? 1 : 0;
  return rc;
}

static int gather_common(const zcg_table* t, const int64_t* idx_dev, const int64_t* order_dev,
                         int64_t n_idx, void* out_dev, void* stream, const zcg_launch_opts* opts) {
  if (!zcg_is_live(t)) return ZCG_EHANDLE;
  if (n_idx < 0) return ZCG_EINVAL;
  if (opts && (opts->workspace_bytes < 0 || (opts->workspace_bytes > 0 && !opts->workspace_dev)))
    return ZCG_EINVAL;
  if (n_idx == 0) return ZCG_OK;
  if (!idx_dev || !out_dev) return ZCG_EINVAL;
  if ((uintptr_t)idx_dev % 8 || (uintptr_t)order_dev % 8) return ZCG_EALIGN;
  if (n_idx > INT64_MAX / t->row_bytes) return ZCG_EINVAL;
  const uintptr_t o0 = (uintptr_t)out_dev, o1 = o0 + (uintptr_t)(n_idx * t->row_bytes);
  const uintptr_t t0 = (uintptr_t)t->dev, t1 = t0 + (uintptr_t)(t->n_rows * t->row_bytes);
  if (o0 < t1 && t0 < o1) return ZCG_EALIAS;
  {  // the list and a caller's order are read while the output is written
    const uintptr_t i0 = (uintptr_t)idx_dev, r0 = (uintptr_t)order_dev, len = (uintptr_t)(n_idx * 8);
    if (i0 < o1 && o0 < i0 + len) return ZCG_EALIAS;
    if (order_dev && r0 < o1 && o0 < r0 + len) return ZCG_EALIAS;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool build_order = !order_dev && wants_order(t, n_idx, opts);
  if (build_order) {
    // the workspace is written while the list, the table and the output are in use
    const uintptr_t w0 = (uintptr_t)opts->workspace_dev, w1 = w0 + (uintptr_t)opts->workspace_bytes;
    const uintptr_t i0 = (uintptr_t)idx_dev, i1 = i0 + (uintptr_t)(n_idx * 8);
    if ((w0 < o1 && o0 < w1) || (w0 < t1 && t0 < w1) || (w0 < i1 && i0 < w1)) return ZCG_EALIAS;
  }
  // every argument check comes before the first launch
  zcg_plan plan;
  int rc = zcg_make_plan(t->row_bytes, t->elem, t0, o0, n_idx, t->host_resident,
                         order_dev != nullptr || build_order, opts, &plan);
  if (rc) return rc;
  if ((order_dev || build_order) && plan.variant == ZCG_VARIANT_NAIVE) return ZCG_EINVAL;
  if (build_order) {
    // the order lives at the start of the workspace, the builder's scratch behind it
    int64_t* order = static_cast<int64_t*>(opts->workspace_dev);
    char* scratch = static_cast<char*>(opts->workspace_dev) + (n_idx * 8 + 255) / 256 * 256;
    hipError_t e = zcg_order_launch(idx_dev, n_idx, t->n_rows, order, scratch, s);
    if (e != hipSuccess) return zcg_fail_hip(e);
    order_dev = order;
  }
  hipError_t e = zcg_launch_gather(plan, t->dev, idx_dev, order_dev, n_idx, out_dev, t->row_bytes,
                                   t->elem, s);
  return e == hipSuccess ? ZCG_OK : zcg_fail_hip(e);
}

int zcg_gather_workspace_bytes(int64_t n_idx, int64_t* bytes) {
  if (n_idx < 0 || !bytes) return ZCG_EINVAL;
  *bytes = n_idx ? (n_idx * 8 + 255) / 256 * 256 + zcg_order_scratch_bytes(n_idx) : 0;
  return ZCG_OK;
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
