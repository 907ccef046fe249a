// Processing order for the ordered gather: a permutation `order` of [0, n) such
// that idx[order[k]] ascends with k. Rows are then fetched in ascending table
// order -- neighbouring work items touch neighbouring lines and pages of the host
// table -- while every row still lands at its own position of the output.
// The sort itself is a library primitive (rocPRIM radix sort of (index, position)
// pairs); all memory it needs comes from the caller's workspace.
#include <hip/hip_runtime.h>

#include <cstring>  // rocPRIM's headers use memset without including it

#include <rocprim/rocprim.hpp>

#include "zcg_internal.h"

namespace {

__global__ void __launch_bounds__(256) zcg_k_iota(int64_t* __restrict__ p, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) p[i] = i;
}

constexpr int64_t kAlign = 256;
int64_t round_up(int64_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

hipError_t sort_temp_bytes(int64_t n, size_t* bytes) {
  *bytes = 0;
  return rocprim::radix_sort_pairs(nullptr, *bytes, static_cast<const uint64_t*>(nullptr),
                                   static_cast<uint64_t*>(nullptr),
                                   static_cast<const int64_t*>(nullptr),
                                   static_cast<int64_t*>(nullptr), (size_t)n, 0, 64, nullptr);
}

}  // namespace

extern "C" {

int zcg_order_workspace_bytes(int64_t n_idx, int64_t* bytes) {
  if (n_idx < 0 || !bytes) return ZCG_EINVAL;
  *bytes = 0;
  if (n_idx == 0) return ZCG_OK;
  size_t temp = 0;
  hipError_t e = sort_temp_bytes(n_idx, &temp);
  if (e != hipSuccess) return zcg_fail_hip(e);
  *bytes = 2 * round_up(n_idx * 8) + round_up((int64_t)temp);
  return ZCG_OK;
}

int zcg_make_order(const int64_t* idx_dev, int64_t n_idx, int64_t n_rows, int64_t* order_dev,
                   void* workspace_dev, int64_t workspace_bytes, void* stream) {
  if (n_idx < 0 || n_rows < 1) return ZCG_EINVAL;
  if (n_idx == 0) return ZCG_OK;
  if (!idx_dev || !order_dev || !workspace_dev) return ZCG_EINVAL;
  if (((uintptr_t)idx_dev | (uintptr_t)order_dev) % 8 || (uintptr_t)workspace_dev % kAlign)
    return ZCG_EALIGN;
  size_t temp = 0;
  hipError_t e = sort_temp_bytes(n_idx, &temp);
  if (e != hipSuccess) return zcg_fail_hip(e);
  const int64_t seg = round_up(n_idx * 8);
  if (workspace_bytes < 2 * seg + round_up((int64_t)temp)) return ZCG_EINVAL;
  char* ws = static_cast<char*>(workspace_dev);
  uint64_t* keys_out = reinterpret_cast<uint64_t*>(ws);
  int64_t* iota = reinterpret_cast<int64_t*>(ws + seg);
  void* sort_temp = ws + 2 * seg;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int64_t blocks = (n_idx + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  zcg_k_iota<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(iota, n_idx);
  e = hipGetLastError();
  if (e != hipSuccess) return zcg_fail_hip(e);
  // valid indices are below n_rows: sort only the bits that can differ
  int end_bit = 1;
  while (end_bit < 63 && ((int64_t)1 << end_bit) < n_rows) ++end_bit;
  e = rocprim::radix_sort_pairs(sort_temp, temp, reinterpret_cast<const uint64_t*>(idx_dev),
                                keys_out, static_cast<const int64_t*>(iota), order_dev,
                                (size_t)n_idx, 0, end_bit, s);
  return e == hipSuccess ? ZCG_OK : zcg_fail_hip(e);
}

}  // extern "C"
