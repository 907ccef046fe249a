// Gather kernels for gfx950 and the host-side plan that picks their launch shape.
//
// The work is pure data movement over the host link (table in mapped host
// memory) or HBM (device-resident table): no MFMA, no LDS. What matters is
//  - which bytes one wave-wide load instruction covers (whole, aligned lines
//    of the host-side memory, Section 3.2.1 of the paper),
//  - how many independent loads each lane keeps in flight (the link's latency
//    is microseconds, Section 3.2.2),
//  - coalesced, non-temporal stores of the dense result.
#include <hip/hip_runtime.h>

#include "zcg_internal.h"

namespace {

constexpr int kBlock = 256;  // 4 wavefronts of 64 lanes
constexpr int kWave = 64;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int W> struct vec_of;
template <> struct vec_of<16> { typedef u32x4 type; };
template <> struct vec_of<8> { typedef u32x2 type; };
template <> struct vec_of<4> { typedef uint32_t type; };
template <> struct vec_of<2> { typedef uint16_t type; };

template <int W, bool NT>
__device__ __forceinline__ typename vec_of<W>::type load_chunk(const uint8_t* p) {
  const auto* q = reinterpret_cast<const typename vec_of<W>::type*>(p);
  if constexpr (NT) return __builtin_nontemporal_load(q);
  else return *q;
}

template <int W, bool NT>
__device__ __forceinline__ void store_chunk(uint8_t* p, typename vec_of<W>::type v) {
  auto* q = reinterpret_cast<typename vec_of<W>::type*>(p);
  if constexpr (NT) __builtin_nontemporal_store(v, q);
  else *q = v;
}

// Lanes whose chunk falls outside the row still execute the load, but from this
// device-resident dummy: the load stays unconditional (so the compiler can keep
// U of them in flight without merging values across branches) and no byte
// outside the row is ever requested from the table.
__device__ __align__(16) uint32_t zcg_dummy_chunk[4];

// Rows whose (aligned) span fits one pass of a lane group of 1 << log2_g lanes.
// Lane l of the group owns the W-byte chunk at  floor(row_start, line) + l*W
// and moves it only if it lies inside the row, so a wave's load covers whole
// lines of the source except at the two row ends. With line_mask == 0 the
// chunks start at the row start instead. Each group keeps U rows in flight:
// U index loads, then U table loads, then U stores.
template <int W, int U, bool NTL, bool NTS>
__global__ void __launch_bounds__(kBlock)
zcg_k_rows_narrow(const uint8_t* __restrict__ table, const int64_t* __restrict__ idx,
                  int64_t n_idx, uint8_t* __restrict__ out, int64_t row_bytes, int log2_g,
                  unsigned line_mask) {
  typedef typename vec_of<W>::type vec;
  const unsigned lane = threadIdx.x & ((1u << log2_g) - 1u);
  const int64_t n_groups = ((int64_t)gridDim.x * kBlock) >> log2_g;
  const int64_t group = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> log2_g;
  const int64_t lane_off = (int64_t)lane * W;
  const uint8_t* dummy = reinterpret_cast<const uint8_t*>(zcg_dummy_chunk);

  for (int64_t base = group; base < n_idx; base += n_groups * U) {
    int64_t row_id[U];
    vec v[U];
    int64_t dst[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t r = base + (int64_t)u * n_groups;
      row_id[u] = idx[r < n_idx ? r : n_idx - 1];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t r = base + (int64_t)u * n_groups;
      const uint8_t* src = table + row_id[u] * row_bytes;
      const int64_t off = lane_off - (int64_t)((uintptr_t)src & line_mask);
      const bool ok = (r < n_idx) && (off >= 0) && (off < row_bytes);
      v[u] = load_chunk<W, NTL>(ok ? src + off : dummy);
      dst[u] = ok ? r * row_bytes + off : -1;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (dst[u] >= 0) store_chunk<W, NTS>(out + dst[u], v[u]);
  }
}

// Rows wider than one wave pass: one wavefront per row, walking the aligned
// span in steps of 64*W bytes, U steps in flight.
template <int W, int U, bool NTL, bool NTS>
__global__ void __launch_bounds__(kBlock)
zcg_k_rows_wide(const uint8_t* __restrict__ table, const int64_t* __restrict__ idx, int64_t n_idx,
                uint8_t* __restrict__ out, int64_t row_bytes, unsigned line_mask) {
  typedef typename vec_of<W>::type vec;
  const unsigned lane = threadIdx.x & (kWave - 1);
  const int64_t n_waves = ((int64_t)gridDim.x * kBlock) / kWave;
  const int64_t wave = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / kWave;
  constexpr int64_t kStep = (int64_t)kWave * W;
  const uint8_t* dummy = reinterpret_cast<const uint8_t*>(zcg_dummy_chunk);

  for (int64_t r = wave; r < n_idx; r += n_waves) {
    const uint8_t* src = table + idx[r] * row_bytes;
    const int64_t mis = (int64_t)((uintptr_t)src & line_mask);
    const int64_t span = mis + row_bytes;
    const int64_t src_shift = -mis;                 // chunk c of the span is src[c - mis]
    const int64_t dst_shift = r * row_bytes - mis;  // and lands at out[r*row_bytes + c - mis]
    for (int64_t c0 = (int64_t)lane * W; c0 < span; c0 += kStep * U) {
      vec v[U];
      bool ok[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t c = c0 + (int64_t)u * kStep;
        ok[u] = (c >= mis) && (c < span);
        v[u] = load_chunk<W, NTL>(ok[u] ? src + (src_shift + c) : dummy);
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) store_chunk<W, NTS>(out + (dst_shift + c0 + (int64_t)u * kStep), v[u]);
    }
  }
}

// The baseline mapping: lane i of the flat grid copies element i of the dense
// output, whatever row it falls in and wherever that row starts in the source.
template <typename E, typename I, bool NTL, bool NTS>
__global__ void __launch_bounds__(kBlock)
zcg_k_flat(const E* __restrict__ table, const int64_t* __restrict__ idx, int64_t n_idx,
           E* __restrict__ out, int64_t dim) {
  const I total = (I)(n_idx * dim);
  const I stride = (I)gridDim.x * kBlock;
  const I d = (I)dim;
  for (I i = (I)blockIdx.x * kBlock + threadIdx.x; i < total; i += stride) {
    const I r = i / d;
    const I c = i - r * d;
    const E* s = table + idx[r] * dim + (int64_t)c;
    E v;
    if constexpr (NTL) v = __builtin_nontemporal_load(s); else v = *s;
    if constexpr (NTS) __builtin_nontemporal_store(v, out + (int64_t)i); else out[(int64_t)i] = v;
  }
}

__global__ void __launch_bounds__(kBlock)
zcg_k_validate(const int64_t* __restrict__ idx, int64_t n_idx, int64_t n_rows,
               unsigned long long* __restrict__ n_bad) {
  unsigned long long bad = 0;
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n_idx; i += stride) {
    const int64_t v = idx[i];
    bad += (v < 0 || v >= n_rows) ? 1ull : 0ull;
  }
  if (bad) atomicAdd(n_bad, bad);
}

int floor_pow2_divisor(uint64_t x, int cap) {  // largest power of two <= cap dividing x
  int w = cap;
  while (w > 1 && (x % (uint64_t)w) != 0) w >>= 1;
  return w;
}

template <int W, int U>
hipError_t launch_rows(const zcg_plan& p, const uint8_t* table, const int64_t* idx, int64_t n_idx,
                       uint8_t* out, int64_t row_bytes, hipStream_t s) {
  const unsigned mask = (p.variant == ZCG_VARIANT_ALIGNED) ? (unsigned)(p.line_bytes - 1) : 0u;
  const dim3 grid((unsigned)p.blocks), block(kBlock);
#define ZCG_LAUNCH(NTL, NTS)                                                                    \
  do {                                                                                          \
    if (p.iters == 1)                                                                           \
      zcg_k_rows_narrow<W, U, NTL, NTS><<<grid, block, 0, s>>>(table, idx, n_idx, out,         \
                                                                 row_bytes, p.log2_group, mask); \
    else                                                                                        \
      zcg_k_rows_wide<W, U, NTL, NTS><<<grid, block, 0, s>>>(table, idx, n_idx, out, row_bytes, \
                                                               mask);                           \
  } while (0)
  if (p.nt_loads && p.nt_stores) ZCG_LAUNCH(true, true);
  else if (p.nt_loads) ZCG_LAUNCH(true, false);
  else if (p.nt_stores) ZCG_LAUNCH(false, true);
  else ZCG_LAUNCH(false, false);
#undef ZCG_LAUNCH
  return hipGetLastError();
}

template <int W>
hipError_t launch_rows_u(const zcg_plan& p, const uint8_t* table, const int64_t* idx,
                         int64_t n_idx, uint8_t* out, int64_t row_bytes, hipStream_t s) {
  switch (p.unroll) {
    case 1: return launch_rows<W, 1>(p, table, idx, n_idx, out, row_bytes, s);
    case 2: return launch_rows<W, 2>(p, table, idx, n_idx, out, row_bytes, s);
    case 4: return launch_rows<W, 4>(p, table, idx, n_idx, out, row_bytes, s);
    case 8: return launch_rows<W, 8>(p, table, idx, n_idx, out, row_bytes, s);
    default: return hipErrorInvalidValue;
  }
}

template <typename E>
hipError_t launch_flat(const zcg_plan& p, const void* table, const int64_t* idx, int64_t n_idx,
                       void* out, int64_t dim, hipStream_t s) {
  const dim3 grid((unsigned)p.blocks), block(kBlock);
  const bool small = (n_idx * dim) < ((int64_t)1 << 32) - (int64_t)p.blocks * kBlock;
  const E* t = static_cast<const E*>(table);
  E* o = static_cast<E*>(out);
#define ZCG_LAUNCH(NTL, NTS)                                                               \
  do {                                                                                     \
    if (small) zcg_k_flat<E, uint32_t, NTL, NTS><<<grid, block, 0, s>>>(t, idx, n_idx, o, dim); \
    else zcg_k_flat<E, int64_t, NTL, NTS><<<grid, block, 0, s>>>(t, idx, n_idx, o, dim);   \
  } while (0)
  if (p.nt_loads && p.nt_stores) ZCG_LAUNCH(true, true);
  else if (p.nt_loads) ZCG_LAUNCH(true, false);
  else if (p.nt_stores) ZCG_LAUNCH(false, true);
  else ZCG_LAUNCH(false, false);
#undef ZCG_LAUNCH
  return hipGetLastError();
}

}  // namespace

int zcg_make_plan(int64_t row_bytes, int elem, uintptr_t table_addr, uintptr_t out_addr,
                  int64_t n_idx, bool host_resident, const zcg_launch_opts* opts, zcg_plan* plan) {
  zcg_launch_opts o = {};
  if (opts) o = *opts;
  if (row_bytes <= 0 || (elem != 2 && elem != 4) || row_bytes % elem != 0 || n_idx < 0 || !plan)
    return ZCG_EINVAL;
  if (table_addr % (uintptr_t)elem != 0 || out_addr % (uintptr_t)elem != 0) return ZCG_EALIGN;

  // defaults
  int variant = o.variant;
  int line = o.line_bytes ? o.line_bytes : 128;
  int unroll = o.unroll ? o.unroll : 4;
  int vec_cap = o.vec_bytes ? o.vec_bytes : 16;
  int max_blocks = o.max_blocks ? o.max_blocks : (host_resident ? 2048 : 8192);
  const int ntl = o.nt_loads == 1 ? 1 : 0;                 // default: plain loads
  const int nts = o.nt_stores == 2 ? 0 : 1;                // default: non-temporal stores
  if (variant < 0 || variant >= ZCG_VARIANT_COUNT) return ZCG_EINVAL;
  if (line != 32 && line != 64 && line != 128 && line != 256) return ZCG_EINVAL;
  if (unroll != 1 && unroll != 2 && unroll != 4 && unroll != 8) return ZCG_EINVAL;
  if (vec_cap != 2 && vec_cap != 4 && vec_cap != 8 && vec_cap != 16) return ZCG_EINVAL;
  if (max_blocks < 1 || o.nt_loads < 0 || o.nt_loads > 2 || o.nt_stores < 0 || o.nt_stores > 2)
    return ZCG_EINVAL;
  if (vec_cap < elem) return ZCG_EINVAL;

  // Widest access that keeps every chunk of every row aligned at both ends.
  int w = floor_pow2_divisor((uint64_t)row_bytes, vec_cap);
  w = floor_pow2_divisor((uint64_t)table_addr, w);
  w = floor_pow2_divisor((uint64_t)out_addr, w);

  if (variant == ZCG_VARIANT_AUTO) {
    // Rows shorter than a line, or made of whole lines on a line-aligned base,
    // need no realignment (the paper's applicability rule, end of Section 3.2.1).
    const bool whole_lines = (row_bytes % line == 0) && (table_addr % (uintptr_t)line == 0);
    variant = (row_bytes < line || whole_lines) ? ZCG_VARIANT_ROWVEC : ZCG_VARIANT_ALIGNED;
  }

  plan->variant = variant;
  plan->line_bytes = line;
  plan->unroll = unroll;
  plan->nt_loads = ntl;
  plan->nt_stores = nts;

  int64_t want_blocks;
  if (variant == ZCG_VARIANT_NAIVE) {
    plan->vec_bytes = elem;
    plan->log2_group = 0;
    plan->iters = 1;
    plan->unroll = 1;
    const int64_t total = n_idx * (row_bytes / elem);
    want_blocks = (total + kBlock - 1) / kBlock;
  } else {
    plan->vec_bytes = w;
    const int64_t worst_span = row_bytes + (variant == ZCG_VARIANT_ALIGNED ? line - w : 0);
    const int64_t chunks = (worst_span + w - 1) / w;
    int lg = 0;
    while (lg < 6 && ((int64_t)1 << lg) < chunks) ++lg;
    plan->log2_group = lg;
    plan->iters = (int)((chunks + ((int64_t)1 << lg) - 1) >> lg);
    if (plan->iters == 1) {
      const int64_t groups = (n_idx + unroll - 1) / unroll;
      want_blocks = ((groups << lg) + kBlock - 1) / kBlock;
    } else {
      plan->log2_group = 6;
      want_blocks = (n_idx * kWave + kBlock - 1) / kBlock;
    }
  }
  if (want_blocks < 1) want_blocks = 1;
  plan->blocks = (int)(want_blocks < max_blocks ? want_blocks : max_blocks);
  return ZCG_OK;
}

hipError_t zcg_launch_gather(const zcg_plan& p, const void* table, const int64_t* idx,
                             int64_t n_idx, void* out, int64_t row_bytes, int elem,
                             hipStream_t stream) {
  if (p.variant == ZCG_VARIANT_NAIVE) {
    const int64_t dim = row_bytes / elem;
    return elem == 4 ? launch_flat<uint32_t>(p, table, idx, n_idx, out, dim, stream)
                     : launch_flat<uint16_t>(p, table, idx, n_idx, out, dim, stream);
  }
  const uint8_t* t = static_cast<const uint8_t*>(table);
  uint8_t* o = static_cast<uint8_t*>(out);
  switch (p.vec_bytes) {
    case 16: return launch_rows_u<16>(p, t, idx, n_idx, o, row_bytes, stream);
    case 8: return launch_rows_u<8>(p, t, idx, n_idx, o, row_bytes, stream);
    case 4: return launch_rows_u<4>(p, t, idx, n_idx, o, row_bytes, stream);
    case 2: return launch_rows_u<2>(p, t, idx, n_idx, o, row_bytes, stream);
    default: return hipErrorInvalidValue;
  }
}

hipError_t zcg_launch_validate(const int64_t* idx, int64_t n_idx, int64_t n_rows,
                               unsigned long long* n_bad_dev, hipStream_t stream) {
  int64_t blocks = (n_idx + kBlock - 1) / kBlock;
  if (blocks > 4096) blocks = 4096;
  if (blocks < 1) blocks = 1;
  zcg_k_validate<<<dim3((unsigned)blocks), dim3(kBlock), 0, stream>>>(idx, n_idx, n_rows, n_bad_dev);
  return hipGetLastError();
}
