// Producer side of the minibatch pipeline (paper Section 3.3): the sampler hands
// over a node-ID list, the producer copies the list to the GPU by DMA, gathers
// the rows into one of a small ring of GPU buffers, and the consumer (training)
// reads that buffer in place. Buffers alternate (ping-pong), and producer and
// consumer meet once per minibatch -- here through HIP events between a gather
// stream owned by the pipeline and the caller's consumer stream, inside one
// process, instead of IPC handles between processes.
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>
#include <vector>

#include "zcg_internal.h"

struct zcg_pipeline {
  const zcg_table* table = nullptr;
  int64_t max_rows = 0;
  int n_buffers = 0;
  int next = 0;
  bool own_stream = false;
  hipStream_t gather_stream = nullptr;
  struct Slot {
    void* out = nullptr;            // caller-owned
    int64_t* idx_dev = nullptr;     // library-owned
    int64_t* idx_pinned = nullptr;  // library-owned
    hipEvent_t gathered = nullptr;  // recorded on the gather stream after the gather
    hipEvent_t released = nullptr;  // recorded on the consumer stream by release()
    bool used = false, has_release = false;
    int64_t n_rows = 0;
  };
  std::vector<Slot> slots;
};

namespace {

void free_slots(zcg_pipeline* p) {
  for (auto& s : p->slots) {
    if (s.gathered) (void)hipEventDestroy(s.gathered);
    if (s.released) (void)hipEventDestroy(s.released);
    if (s.idx_dev) (void)hipFree(s.idx_dev);
    if (s.idx_pinned) (void)hipHostFree(s.idx_pinned);
  }
  if (p->own_stream && p->gather_stream) (void)hipStreamDestroy(p->gather_stream);
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
  zcg_pipeline* p = new (std::nothrow) zcg_pipeline;
  if (!p) return ZCG_ENOMEM;
  p->table = t;
  p->max_rows = max_rows;
  p->n_buffers = n_buffers;
  p->slots.resize((size_t)n_buffers);
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
                        hipHostMallocDefault);
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
  if (!p || !slot || n_idx < 0 || n_idx > p->max_rows || (n_idx > 0 && !idx_host)) return ZCG_EINVAL;
  if (!zcg_is_live(p->table)) return ZCG_EHANDLE;
  for (int64_t i = 0; i < n_idx; ++i)
    if (idx_host[i] < 0 || idx_host[i] >= p->table->n_rows) return ZCG_ERANGE;
  const int k = p->next;
  auto& s = p->slots[(size_t)k];
  if (s.used && !s.has_release) return ZCG_EBUSY;  // the consumer still holds this buffer
  hipError_t e = hipSuccess;
  // the previous list copy out of this slot's staging memory must be over (it is, unless the
  // producer runs a whole ring ahead): the only host-side wait, and it is the back-pressure
  if (s.used) e = hipEventSynchronize(s.gathered);
  // the consumer must be done with this buffer: a device-side wait, the host does not block
  if (e == hipSuccess && s.has_release) e = hipStreamWaitEvent(p->gather_stream, s.released, 0);
  if (e != hipSuccess) return zcg_fail_hip(e);
  if (n_idx > 0) {
    std::memcpy(s.idx_pinned, idx_host, (size_t)n_idx * sizeof(int64_t));
    e = hipMemcpyAsync(s.idx_dev, s.idx_pinned, (size_t)n_idx * sizeof(int64_t),
                       hipMemcpyHostToDevice, p->gather_stream);
    if (e != hipSuccess) return zcg_fail_hip(e);
    int rc = zcg_gather(p->table, s.idx_dev, n_idx, s.out, p->gather_stream);
    if (rc) return rc;
  }
  e = hipEventRecord(s.gathered, p->gather_stream);
  if (e != hipSuccess) return zcg_fail_hip(e);
  s.used = true;
  s.has_release = false;
  s.n_rows = n_idx;
  *slot = k;
  p->next = (k + 1) % p->n_buffers;
  return ZCG_OK;
}

int zcg_pipeline_acquire(zcg_pipeline* p, int slot, void* consumer_stream, void** out_dev,
                         int64_t* n_rows) {
  if (!p || slot < 0 || slot >= p->n_buffers || !p->slots[(size_t)slot].used) return ZCG_EINVAL;
  auto& s = p->slots[(size_t)slot];
  hipError_t e = hipStreamWaitEvent(static_cast<hipStream_t>(consumer_stream), s.gathered, 0);
  if (e != hipSuccess) return zcg_fail_hip(e);
  if (out_dev) *out_dev = s.out;
  if (n_rows) *n_rows = s.n_rows;
  return ZCG_OK;
}

int zcg_pipeline_release(zcg_pipeline* p, int slot, void* consumer_stream) {
  if (!p || slot < 0 || slot >= p->n_buffers || !p->slots[(size_t)slot].used) return ZCG_EINVAL;
  auto& s = p->slots[(size_t)slot];
  hipError_t e = hipEventRecord(s.released, static_cast<hipStream_t>(consumer_stream));
  if (e != hipSuccess) return zcg_fail_hip(e);
  s.has_release = true;
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
