// Internal declarations shared by the translation units of libzcgather.
#ifndef ZCG_INTERNAL_H
#define ZCG_INTERNAL_H

#include <hip/hip_runtime_api.h>
#include <stdint.h>

#include "zcgather.h"

// VIEW: a slice of another live table; owns nothing.
enum zcg_kind { ZCG_KIND_REGISTERED = 1, ZCG_KIND_ALLOCATED = 2, ZCG_KIND_DEVICE = 3, ZCG_KIND_VIEW = 4 };

struct zcg_table {
  int kind;
  bool host_resident;       // the rows live in mapped host memory (read over the host link)
  const zcg_table* parent;  // VIEW: the table it slices, else nullptr
  uint64_t serial;          // unique per handle ever made (a freed handle's address may be reused)
  uint64_t parent_serial;   // VIEW: the serial its parent had when the view was made
  int dtype;
  int elem;  // bytes per element
  int device;
  void* host;  // nullptr for device tables
  void* dev;   // address kernels use
  int64_t n_rows;
  int64_t dim;
  int64_t row_bytes;
};

// zcg_api.hip
bool zcg_is_live(const zcg_table* t);
int zcg_fail_hip(hipError_t e);  // records e for zcg_last_hip_error, returns ZCG_EHIP
// whether walking this list in ascending table order saves more link time than building the
// order costs (short host-resident rows, long lists that are dense in the table)
bool zcg_order_pays(const zcg_table* t, int64_t n_idx);

// zcg_plan.hip
int zcg_make_plan(int64_t row_bytes, int elem, uintptr_t table_addr, uintptr_t out_addr,
                  int64_t n_idx, bool host_resident, bool ordered, const zcg_launch_opts* opts,
                  zcg_plan* plan);  // ordered: the rows will be walked in ascending table order
// zcg_kernels.hip
hipError_t zcg_launch_gather(const zcg_plan& plan, const void* table, const int64_t* idx,
                             const int64_t* order, int64_t n_idx, void* out, int64_t row_bytes, int elem,
                             hipStream_t stream);
hipError_t zcg_launch_validate(const int64_t* idx, int64_t n_idx, int64_t n_rows,
                               unsigned long long* n_bad_dev, hipStream_t stream);

// zcg_order.hip: builds the ascending order of an index list with kernel launches only.
// scratch: device, 256-byte aligned, zcg_order_scratch_bytes(n) bytes; n <= UINT32_MAX.
int64_t zcg_order_scratch_bytes(int64_t n_idx);
hipError_t zcg_order_launch(const int64_t* idx, int64_t n, int64_t n_rows, int64_t* order,
                            void* scratch, hipStream_t stream);

#endif
