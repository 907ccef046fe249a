// Producer side of the minibatch pipeline (paper Section 3.3): the sampler hands
// over a node-ID list, the producer copies the list to the GPU by DMA, gathers
// the rows into one of a small ring of GPU buffers, and the consumer (training)
// reads that buffer in place. Buffers alternate (ping-pong), and producer and
// consumer meet once per minibatch -- here through HIP events between a gather
// stream owned by the pipeline and the caller's consumer stream, inside one
// process, instead of IPC handles between processes. The paper's queue between
// the producer and the consumer process is the ring itself: a mutex and a
// condition variable let one producer thread and one consumer thread block on
// "a buffer is free" and "a minibatch is ready".
#include <hip/hip_runtime.h>

#include <chrono>
#include <condition_variable>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "zcg_internal.h"

struct zcg_pipeline {
  const zcg_table* table = nullptr;
  int64_t max_rows = 0;
  int n_buffers = 0;
  bool own_stream = false;
  // Rows of at most one line over the host link are bound by the request rate; walked in
  // ascending table order, neighbouring rows share lines and pairs of lines (measured +12 %
  // on 128-byte rows, +30 % on 32-byte rows, order build included, for lists that are dense in
  // the table). The pipeline owns the memory the order builder needs, so it does this by
  // itself for every minibatch where zcg_order_pays says so.
  bool sorts = false;
  int64_t sort_ws_bytes = 0;
  // The list has to cross the link, in the same direction as the gather's reads. Row numbers of
  // a table of at most 2^32 rows are staged as 32-bit values, and one small kernel on the gather
  // stream reads them out of the pinned staging memory (zero-copy, like the gather itself) and
  // writes the int64 list the gather takes: half the bytes and no copy-engine hand-off
  // (measured with nothing else on the GPU: 400-byte rows 1.077 -> 0.972 ms per minibatch of
  // 110 k rows, the kernel alone being 0.947; a million 32- or 128-byte rows: -3 %). Running
  // this on a stream of its own beside the previous gather is no faster, and a third busy
  // stream was seen to land on the consumer stream's hardware queue and serialise the ring.
  bool narrow_lists = false;
  hipStream_t gather_stream = nullptr;
  // A buffer goes FREE -> FILLING (producer is enqueuing into it) -> READY (its
  // gather is enqueued and `gathered` recorded) -> FREE again on release.
  enum State { FREE, FILLING, READY };
  struct Slot {
    void* out = nullptr;            // caller-owned
    int64_t* idx_dev = nullptr;     // library-owned
    int64_t* idx_pinned = nullptr;  // library-owned (holds 32-bit values when the lists are narrow)
    const uint32_t* idx_pinned_dev = nullptr;  // the same memory as the GPU addresses it
    int64_t* order = nullptr;       // library-owned, only when the pipeline sorts (see `sorts`)
    void* sort_ws = nullptr;        // library-owned workspace of the sort
    hipEvent_t gathered = nullptr;  // recorded on the gather stream after the gather
    hipEvent_t released = nullptr;  // recorded on the consumer stream by release()
    State state = FREE;
    bool ever_used = false;    // `gathered` has been recorded at least once
    bool has_release = false;  // `released` was recorded since the last use
    bool delivered = false;    // handed to the consumer by zcg_pipeline_next
    int64_t n_rows = 0;
  };
  std::vector<Slot> slots;
  // guarded by mu
  std::mutex mu;
  std::condition_variable cv;
  int next_fill = 0;     // buffer the next submit uses
  int next_deliver = 0;  // buffer the next zcg_pipeline_next hands out
  int ready_undelivered = 0;
  bool finished = false;
};

namespace {

constexpr int kWidenBlock = 256;

__global__ __launch_bounds__(kWidenBlock) void zcg_k_widen_list(const uint32_t* __restrict__ narrow,
                                                                 int64_t* __restrict__ wide, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * kWidenBlock;
  for (int64_t i = (int64_t)blockIdx.x * kWidenBlock + threadIdx.x; i < n; i += stride)
    wide[i] = (int64_t)narrow[i];
}

void free_slots(zcg_pipeline* p) {
  for (auto& s : p->slots) {
    if (s.gathered) (void)hipEventDestroy(s.gathered);
    if (s.released) (void)hipEventDestroy(s.released);
    if (s.idx_dev) (void)hipFree(s.idx_dev);
    if (s.idx_pinned) (void)hipHostFree(s.idx_pinned);
    if (s.order) (void)hipFree(s.order);
    if (s.sort_ws) (void)hipFree(s.sort_ws);
  }
  if (p->own_stream && p->gather_stream) (void)hipStreamDestroy(p->gather_stream);
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

// Waits on cv until pred() holds; timeout_ms < 0 waits without limit, 0 only tests.
template <class Pred>
bool wait_for(zcg_pipeline* p, std::unique_lock<std::mutex>& lk, int timeout_ms, Pred pred) {
  if (timeout_ms < 0) {
    p->cv.wait(lk, pred);
    return true;
  }
  return p->cv.wait_for(lk, std::chrono::milliseconds(timeout_ms), pred);
}

int submit_impl(zcg_pipeline* p, const int64_t* idx_host, int64_t n_idx, int timeout_ms, int* slot) {
  if (!p || !slot || n_idx < 0 || n_idx > p->max_rows || (n_idx > 0 && !idx_host)) return ZCG_EINVAL;
  if (!zcg_is_live(p->table)) return ZCG_EHANDLE;
  {  // one branch-free pass (vectorises): the smallest and the largest entry decide
    int64_t lo = 0, hi = 0;
    for (int64_t i = 0; i < n_idx; ++i) {
      lo = idx_host[i] < lo ? idx_host[i] : lo;
      hi = idx_host[i] > hi ? idx_host[i] : hi;
    }
    if (lo < 0 || hi >= p->table->n_rows) return ZCG_ERANGE;
  }
  int k;
  bool wait_copy, wait_release;
  {
    std::unique_lock<std::mutex> lk(p->mu);
    if (p->finished) return ZCG_ECLOSED;
    k = p->next_fill;
    auto& s = p->slots[(size_t)k];
    if (s.state == zcg_pipeline::FILLING) return ZCG_EINVAL;  // a second producer thread
    // the consumer still holds this buffer: nothing is enqueued until it lets go
    if (!wait_for(p, lk, timeout_ms, [&] { return s.state == zcg_pipeline::FREE; }))
      return timeout_ms == 0 ? ZCG_EBUSY : ZCG_ETIMEDOUT;
    s.state = zcg_pipeline::FILLING;
    wait_copy = s.ever_used;
    wait_release = s.has_release;
  }
  auto& s = p->slots[(size_t)k];  // FILLING: only this thread touches the slot now
  DeviceScope scope(p->table->device);
  hipError_t e = scope.err;
  // the previous read of this slot's staging memory (list copy or widening kernel) must be over (it is, unless the
  // producer runs a whole ring ahead of the GPU): a host-side wait, taken outside the lock
  if (e == hipSuccess && wait_copy) e = hipEventSynchronize(s.gathered);
  // the consumer's last reads of this buffer: a device-side wait, the host does not block
  if (e == hipSuccess && wait_release) e = hipStreamWaitEvent(p->gather_stream, s.released, 0);
  int rc = ZCG_OK;
  if (e == hipSuccess && n_idx > 0) {
    if (p->narrow_lists) {  // every entry was checked above to lie in [0, n_rows), n_rows <= 2^32
      uint32_t* staged = reinterpret_cast<uint32_t*>(s.idx_pinned);
      for (int64_t i = 0; i < n_idx; ++i) staged[i] = (uint32_t)idx_host[i];
      const int64_t want = (n_idx + kWidenBlock - 1) / kWidenBlock;
      hipLaunchKernelGGL(zcg_k_widen_list, dim3((unsigned)(want < 2048 ? want : 2048)), dim3(kWidenBlock), 0,
                         p->gather_stream, s.idx_pinned_dev, s.idx_dev, n_idx);
      e = hipGetLastError();
    } else {
      std::memcpy(s.idx_pinned, idx_host, (size_t)n_idx * sizeof(int64_t));
      e = hipMemcpyAsync(s.idx_dev, s.idx_pinned, (size_t)n_idx * sizeof(int64_t),
                         hipMemcpyHostToDevice, p->gather_stream);
    }
    if (e == hipSuccess && p->sorts && zcg_order_pays(p->table, n_idx)) {
      rc = zcg_make_order(s.idx_dev, n_idx, p->table->n_rows, s.order, s.sort_ws, p->sort_ws_bytes,
                          p->gather_stream);
      if (rc == ZCG_OK)
        rc = zcg_gather_ordered(p->table, s.idx_dev, s.order, n_idx, s.out, p->gather_stream, nullptr);
    } else if (e == hipSuccess) {
      rc = zcg_gather(p->table, s.idx_dev, n_idx, s.out, p->gather_stream);
    }
  }
  // recorded even after a failure above when possible: whatever did get enqueued must be
  // covered by the event the next use of this slot waits for
  hipError_t e2 = hipEventRecord(s.gathered, p->gather_stream);
  if (e == hipSuccess) e = e2;
  {
    std::lock_guard<std::mutex> lk(p->mu);
    if (e2 == hipSuccess) s.ever_used = true;
    if (e != hipSuccess || rc != ZCG_OK) {
      s.state = zcg_pipeline::FREE;  // has_release stays: the consumer's event still stands
      p->cv.notify_all();
      return e != hipSuccess ? zcg_fail_hip(e) : rc;
    }
    s.has_release = false;
    s.delivered = false;
    s.n_rows = n_idx;
    s.state = zcg_pipeline::READY;
    p->next_fill = (k + 1) % p->n_buffers;
    ++p->ready_undelivered;
    *slot = k;
  }
  p->cv.notify_all();
  return ZCG_OK;
}

}  // namespace

extern "C" {

int zcg_pipeline_create(const zcg_table* t, int64_t max_rows, int n_buffers, void* const* out_bufs,
                        void* gather_stream, zcg_pipeline** out) {
  if (!out) return ZCG_EINVAL;
  *out = nullptr;
  if (!zcg_is_live(t)) return ZCG_EHANDLE;
  if (max_rows < 1 || n_buffers < 1 || n_buffers > 16 || !out_bufs) return ZCG_EINVAL;
  for (int i = 0; i < n_buffers; ++i) {
    if (!out_bufs[i]) return ZCG_EINVAL;
    if ((uintptr_t)out_bufs[i] % (uintptr_t)t->elem) return ZCG_EALIGN;
  }
  DeviceScope scope(t->device);
  if (scope.err != hipSuccess) return zcg_fail_hip(scope.err);
  zcg_pipeline* p = new (std::nothrow) zcg_pipeline;
  if (!p) return ZCG_ENOMEM;
  p->table = t;
  p->max_rows = max_rows;
  p->n_buffers = n_buffers;
  p->slots.resize((size_t)n_buffers);
  p->sorts = t->host_resident && t->row_bytes <= 128 && max_rows <= (int64_t)UINT32_MAX;
  if (p->sorts && zcg_order_workspace_bytes(max_rows, &p->sort_ws_bytes) != ZCG_OK) p->sorts = false;
  p->narrow_lists = t->n_rows <= ((int64_t)1 << 32);
  hipError_t e = hipSuccess;
  if (gather_stream) {
    p->gather_stream = static_cast<hipStream_t>(gather_stream);
  } else {
    e = hipStreamCreateWithFlags(&p->gather_stream, hipStreamNonBlocking);
    p->own_stream = (e == hipSuccess);
  }
  for (int i = 0; i < n_buffers && e == hipSuccess; ++i) {
    auto& s = p->slots[(size_t)i];
    s.out = out_bufs[i];
    e = hipMalloc(reinterpret_cast<void**>(&s.idx_dev), (size_t)max_rows * sizeof(int64_t));
    if (e == hipSuccess)
      e = hipHostMalloc(reinterpret_cast<void**>(&s.idx_pinned), (size_t)max_rows * sizeof(int64_t),
                        hipHostMallocMapped | hipHostMallocPortable);
    if (e == hipSuccess) {
      void* dp = nullptr;
      e = hipHostGetDevicePointer(&dp, s.idx_pinned, 0);
      s.idx_pinned_dev = static_cast<const uint32_t*>(dp);
    }
    if (e == hipSuccess && p->sorts)
      e = hipMalloc(reinterpret_cast<void**>(&s.order), (size_t)max_rows * sizeof(int64_t));
    if (e == hipSuccess && p->sorts) e = hipMalloc(&s.sort_ws, (size_t)p->sort_ws_bytes);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s.gathered, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s.released, hipEventDisableTiming);
  }
  if (e != hipSuccess) {
    free_slots(p);
    delete p;
    return zcg_fail_hip(e);
  }
  *out = p;
  return ZCG_OK;
}

int zcg_pipeline_submit(zcg_pipeline* p, const int64_t* idx_host, int64_t n_idx, int* slot) {
  return submit_impl(p, idx_host, n_idx, 0, slot);
}

int zcg_pipeline_submit_wait(zcg_pipeline* p, const int64_t* idx_host, int64_t n_idx,
                             int timeout_ms, int* slot) {
  return submit_impl(p, idx_host, n_idx, timeout_ms, slot);
}

int zcg_pipeline_finish(zcg_pipeline* p) {
  if (!p) return ZCG_EINVAL;
  {
    std::lock_guard<std::mutex> lk(p->mu);
    p->finished = true;
  }
  p->cv.notify_all();
  return ZCG_OK;
}

int zcg_pipeline_next(zcg_pipeline* p, int timeout_ms, int* slot) {
  if (!p || !slot) return ZCG_EINVAL;
  std::unique_lock<std::mutex> lk(p->mu);
  const bool ok =
      wait_for(p, lk, timeout_ms, [&] { return p->ready_undelivered > 0 || p->finished; });
  if (p->ready_undelivered > 0) {
    *slot = p->next_deliver;
    p->slots[(size_t)*slot].delivered = true;
    p->next_deliver = (p->next_deliver + 1) % p->n_buffers;
    --p->ready_undelivered;
    return ZCG_OK;
  }
  if (p->finished) return ZCG_ECLOSED;
  (void)ok;
  return ZCG_ETIMEDOUT;
}

int zcg_pipeline_acquire(zcg_pipeline* p, int slot, void* consumer_stream, void** out_dev,
                         int64_t* n_rows) {
  if (!p || slot < 0 || slot >= p->n_buffers) return ZCG_EINVAL;
  std::lock_guard<std::mutex> lk(p->mu);
  auto& s = p->slots[(size_t)slot];
  if (s.state != zcg_pipeline::READY) return ZCG_EINVAL;
  hipError_t e = hipStreamWaitEvent(static_cast<hipStream_t>(consumer_stream), s.gathered, 0);
  if (e != hipSuccess) return zcg_fail_hip(e);
  if (out_dev) *out_dev = s.out;
  if (n_rows) *n_rows = s.n_rows;
  return ZCG_OK;
}

int zcg_pipeline_release(zcg_pipeline* p, int slot, void* consumer_stream) {
  if (!p || slot < 0 || slot >= p->n_buffers) return ZCG_EINVAL;
  {
    std::lock_guard<std::mutex> lk(p->mu);
    auto& s = p->slots[(size_t)slot];
    if (s.state != zcg_pipeline::READY) return ZCG_EINVAL;
    hipError_t e = hipEventRecord(s.released, static_cast<hipStream_t>(consumer_stream));
    if (e != hipSuccess) return zcg_fail_hip(e);
    s.has_release = true;
    s.state = zcg_pipeline::FREE;
    if (!s.delivered) {  // the consumer works from submit's slot numbers, not from next()
      --p->ready_undelivered;
      p->next_deliver = (slot + 1) % p->n_buffers;
    }
  }
  p->cv.notify_all();
  return ZCG_OK;
}

int zcg_pipeline_destroy(zcg_pipeline* p) {
  if (!p) return ZCG_EINVAL;
  hipError_t e = hipStreamSynchronize(p->gather_stream);
  free_slots(p);
  delete p;
  return e == hipSuccess ? ZCG_OK : zcg_fail_hip(e);
}

}  // extern "C"
