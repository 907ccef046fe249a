// Gather kernels for gfx950 and their launchers (the launch shape is chosen in zcg_plan.hip).
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
template <> struct vec_of<1> { typedef uint8_t type; };

// Load modes: 0 plain, 1 non-temporal (nt), 2 system scope (sc0 sc1).
template <int W, int LM>
__device__ __forceinline__ typename vec_of<W>::type load_chunk(const uint8_t* p) {
  typedef typename vec_of<W>::type vec;
  const auto* q = reinterpret_cast<const vec*>(p);
  if constexpr (LM == 1) return __builtin_nontemporal_load(q);
  else if constexpr (LM == 2)
    return *(const volatile vec __attribute__((address_space(1)))*)(q);
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
__device__ __align__(64) uint32_t zcg_dummy_chunk[16];

// Rows whose (aligned) span fits one pass of a lane group of 1 << log2_g lanes.
// Lane l of the group owns the W-byte chunk at  floor(row_start, line) + l*W
// and moves it only if it lies inside the row, so a wave's load covers whole
// lines of the source except at the two row ends. With line_mask == 0 the
// chunks start at the row start instead. Each group keeps U rows in flight:
// U index loads, then U table loads, then U stores.
template <int W, int U, int NTL, bool NTS>
__global__ void __launch_bounds__(kBlock)
zcg_k_rows_narrow(const uint8_t* __restrict__ table, const int64_t* __restrict__ idx,
                  const int64_t* __restrict__ order, int64_t n_idx, uint8_t* __restrict__ out,
                  int64_t row_bytes, int log2_g, unsigned line_mask) {
  typedef typename vec_of<W>::type vec;
  const unsigned lane = threadIdx.x & ((1u << log2_g) - 1u);
  const int64_t n_groups = ((int64_t)gridDim.x * kBlock) >> log2_g;
  const int64_t group = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> log2_g;
  const int64_t lane_off = (int64_t)lane * W;
  const uint8_t* dummy = reinterpret_cast<const uint8_t*>(zcg_dummy_chunk);

  for (int64_t base = group; base < n_idx; base += n_groups * U) {
    int64_t pos[U];  // position in the list = output row; work item k handles order[k]
    int64_t row_id[U];
    vec v[U];
    int64_t dst[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t k = base + (int64_t)u * n_groups;
      const int64_t kc = k < n_idx ? k : n_idx - 1;
      pos[u] = order ? order[kc] : kc;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) row_id[u] = idx[pos[u]];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t k = base + (int64_t)u * n_groups;
      const uint8_t* src = table + row_id[u] * row_bytes;
      const int64_t off = lane_off - (int64_t)((uintptr_t)src & line_mask);
      const bool ok = (k < n_idx) && (off >= 0) && (off < row_bytes);
      v[u] = load_chunk<W, NTL>(ok ? src + off : dummy);
      dst[u] = ok ? pos[u] * row_bytes + off : -1;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (dst[u] >= 0) store_chunk<W, NTS>(out + dst[u], v[u]);
  }
}

// Rows wider than one wave pass: one wavefront per row, walking the aligned
// span in steps of 64*W bytes, U steps in flight.
template <int W, int U, int NTL, bool NTS>
__global__ void __launch_bounds__(kBlock)
zcg_k_rows_wide(const uint8_t* __restrict__ table, const int64_t* __restrict__ idx,
                const int64_t* __restrict__ order, int64_t n_idx, uint8_t* __restrict__ out,
                int64_t row_bytes, unsigned line_mask, int64_t splits, int64_t piece_bytes) {
  typedef typename vec_of<W>::type vec;
  const unsigned lane = threadIdx.x & (kWave - 1);
  const int64_t n_waves = ((int64_t)gridDim.x * kBlock) / kWave;
  const int64_t wave = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / kWave;
  constexpr int64_t kStep = (int64_t)kWave * W;
  const uint8_t* dummy = reinterpret_cast<const uint8_t*>(zcg_dummy_chunk);

  // work item k = (row k / splits, piece k % splits); piece_bytes is a multiple of kStep * U
  for (int64_t k = wave; k < n_idx * splits; k += n_waves) {
    int64_t rk = k, piece = 0;
    if (splits > 1) {
      rk = k / splits;
      piece = k - rk * splits;
    }
    const int64_t r = order ? order[rk] : rk;  // position in the list = output row
    const uint8_t* src = table + idx[r] * row_bytes;
    const int64_t mis = (int64_t)((uintptr_t)src & line_mask);
    const int64_t span = mis + row_bytes;
    const int64_t src_shift = -mis;                 // chunk c of the span is src[c - mis]
    const int64_t dst_shift = r * row_bytes - mis;  // and lands at out[r*row_bytes + c - mis]
    const int64_t c_lo = piece * piece_bytes;
    const int64_t c_hi = (splits > 1 && c_lo + piece_bytes < span) ? c_lo + piece_bytes : span;
    for (int64_t c0 = c_lo + (int64_t)lane * W; c0 < c_hi; c0 += kStep * U) {
      vec v[U];
      bool ok[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t c = c0 + (int64_t)u * kStep;
        ok[u] = (c >= mis) && (c < c_hi);
        v[u] = load_chunk<W, NTL>(ok[u] ? src + (src_shift + c) : dummy);
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) store_chunk<W, NTS>(out + (dst_shift + c0 + (int64_t)u * kStep), v[u]);
    }
  }
}

// ---------------------------------------------------------------------------
// Shifted-store kernels: ALIGNED for rows whose size or bases are only WS-byte
// aligned (WS < W). Loads are still W-byte chunks at line-aligned positions
// (always W-aligned, whatever the row start); a chunk that lies fully inside
// the row is written with one W-byte store to a WS-aligned address, the (at
// most two) chunks that straddle a row end are written element by element.
// This is the paper's trade (Section 3.2.1): reads aligned, the misalignment
// moved to the local writes -- at byte granularity instead of element rotation.
// A straddling chunk is loaded whole: up to W-WS bytes next to the row inside
// the same aligned W-byte block are read and dropped.
// ---------------------------------------------------------------------------
template <int W, int WS, bool NT>
__device__ __forceinline__ void store_chunk_unaligned(uint8_t* p, typename vec_of<W>::type v) {
  typedef typename vec_of<W>::type __attribute__((aligned(WS))) uvec;
  auto* q = reinterpret_cast<uvec*>(p);
  if constexpr (NT) __builtin_nontemporal_store(v, q);
  else *q = v;
}

// off = position of the chunk's first byte relative to the row start (may be negative);
// only bytes at positions [lo, hi) of the row are written.
template <int W, int WS, bool NT>
__device__ __forceinline__ void store_shifted(uint8_t* out_row, int64_t off, int64_t lo, int64_t hi,
                                              typename vec_of<W>::type v) {
  if constexpr (W == WS) {
    store_chunk<W, NT>(out_row + off, v);  // chunks are never partial
  } else {
    if (off >= lo && off + W <= hi) {
      store_chunk_unaligned<W, WS, NT>(out_row + off, v);
    } else {
      typedef typename vec_of<WS>::type elem_t;
      elem_t e[W / WS];
      __builtin_memcpy(e, &v, W);
#pragma unroll
      for (int k = 0; k < W / WS; ++k) {
        const int64_t eo = off + (int64_t)k * WS;
        if (eo >= lo && eo < hi) *reinterpret_cast<elem_t*>(out_row + eo) = e[k];
      }
    }
  }
}

template <int W, int WS, int U, bool NTS>
__global__ void __launch_bounds__(kBlock)
zcg_k_rows_narrow_shift(const uint8_t* __restrict__ table, const int64_t* __restrict__ idx,
                        const int64_t* __restrict__ order, int64_t n_idx,
                        uint8_t* __restrict__ out, int64_t row_bytes, int log2_g,
                        unsigned line_mask) {
  typedef typename vec_of<W>::type vec;
  const unsigned lane = threadIdx.x & ((1u << log2_g) - 1u);
  const int64_t n_groups = ((int64_t)gridDim.x * kBlock) >> log2_g;
  const int64_t group = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> log2_g;
  const int64_t lane_off = (int64_t)lane * W;
  const uint8_t* dummy = reinterpret_cast<const uint8_t*>(zcg_dummy_chunk);

  for (int64_t base = group; base < n_idx; base += n_groups * U) {
    int64_t pos[U];
    int64_t row_id[U];
    vec v[U];
    int64_t off[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t k = base + (int64_t)u * n_groups;
      const int64_t kc = k < n_idx ? k : n_idx - 1;
      pos[u] = order ? order[kc] : kc;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) row_id[u] = idx[pos[u]];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t k = base + (int64_t)u * n_groups;
      const uint8_t* src = table + row_id[u] * row_bytes;
      off[u] = lane_off - (int64_t)((uintptr_t)src & line_mask);
      ok[u] = (k < n_idx) && (off[u] > -(int64_t)W) && (off[u] < row_bytes);
      v[u] = load_chunk<W, 0>(ok[u] ? src + off[u] : dummy);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u]) store_shifted<W, WS, NTS>(out + pos[u] * row_bytes, off[u], 0, row_bytes, v[u]);
  }
}

template <int W, int WS, int U, bool NTS>
__global__ void __launch_bounds__(kBlock)
zcg_k_rows_wide_shift(const uint8_t* __restrict__ table, const int64_t* __restrict__ idx,
                      const int64_t* __restrict__ order, int64_t n_idx, uint8_t* __restrict__ out,
                      int64_t row_bytes, unsigned line_mask, int64_t splits, int64_t piece_bytes) {
  typedef typename vec_of<W>::type vec;
  const unsigned lane = threadIdx.x & (kWave - 1);
  const int64_t n_waves = ((int64_t)gridDim.x * kBlock) / kWave;
  const int64_t wave = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / kWave;
  constexpr int64_t kStep = (int64_t)kWave * W;
  const uint8_t* dummy = reinterpret_cast<const uint8_t*>(zcg_dummy_chunk);

  // work item k = (row k / splits, piece k % splits) as in zcg_k_rows_wide
  for (int64_t k = wave; k < n_idx * splits; k += n_waves) {
    int64_t rk = k, piece = 0;
    if (splits > 1) {
      rk = k / splits;
      piece = k - rk * splits;
    }
    const int64_t r = order ? order[rk] : rk;
    const uint8_t* src = table + idx[r] * row_bytes;
    const int64_t mis = (int64_t)((uintptr_t)src & line_mask);
    uint8_t* out_row = out + r * row_bytes;
    // this piece of the line-aligned span, as offsets relative to the row start
    const int64_t off_lo = piece * piece_bytes - mis;
    const int64_t off_hi = (splits > 1 && off_lo + piece_bytes < row_bytes) ? off_lo + piece_bytes
                                                                           : row_bytes;
    // off walks the chunks of the line-aligned span, relative to the row start
    for (int64_t off0 = off_lo + (int64_t)lane * W; off0 < off_hi; off0 += kStep * U) {
      vec v[U];
      bool ok[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t off = off0 + (int64_t)u * kStep;
        ok[u] = (off > -(int64_t)W) && (off < off_hi);
        v[u] = load_chunk<W, 0>(ok[u] ? src + off : dummy);
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) store_shifted<W, WS, NTS>(out_row, off0 + (int64_t)u * kStep, 0, row_bytes, v[u]);
    }
  }
}

// ---------------------------------------------------------------------------
// HALFLINE kernels.
//
// Measured on gfx950: a vector load of mapped host memory always costs whole
// 128-byte lines on the host link, whatever part of the line the wave asks
// for; a load through the scalar data cache costs one 64-byte half line. So a
// row end that occupies at most one half of its line is fetched with a
// wave-uniform 64-byte scalar load (16 SGPRs, then 16 lanes store one dword
// each), and only the rest of the row with whole-line vector loads:
//   head piece: row start S with S mod 128 >= 64  -> bytes [S, next line)
//   tail piece: row end E with (E-1) mod 128 < 64 -> bytes [line of E-1, E)
// A 400-byte row then moves 3 lines + 1 half line (448 bytes) instead of 4
// lines (512 bytes). This is the paper's aim (Section 3.2.1: as few and as full
// link requests as possible for unaligned rows) with this chip's own means.
// A scalar read is a link request of its own, so it pays only where the line it
// replaces would have been a request of its own too (see split_row).
// Rows, table and output of any granularity (1- and 2-byte elements are stored one by one). The scalar cache is
// invalidated at kernel start like the other caches, never written.
// ---------------------------------------------------------------------------
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
typedef const u32x16 __attribute__((address_space(4)))* half_line_ptr;

__device__ __forceinline__ uint64_t uniform_u64(uint64_t x, int src_lane) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, src_lane);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), src_lane);
  return ((uint64_t)hi << 32) | lo;
}

// Where one row's bytes come from. All fields are byte addresses in the table.
struct RowSplit {
  uint64_t vs, ve;           // [vs, ve): moved by vector loads (whole lines except at S / E)
  uint64_t head_addr;        // 64-byte aligned source of the head piece (valid if has_head)
  uint64_t tail_addr;        // 64-byte aligned source of the tail piece (valid if has_tail)
  bool has_head, has_tail;
};

// only_lone: take an end through the scalar path only if the line it sits in would otherwise
// be requested alone. Measured: the link fetches 256-byte aligned pairs of lines as one
// request when a wave asks for both, and a lone line, a pair and a 64-byte scalar read each
// cost one request; so replacing a lone line saves 64 bytes for free, while replacing a line
// whose partner is part of the row turns one request into two.
__device__ __forceinline__ RowSplit split_row(uint64_t S, uint64_t row_bytes, bool only_lone) {
  RowSplit p;
  const uint64_t E = S + row_bytes;
  const uint64_t next_line = (S | 127u) + 1u;
  // first line: alone if it is the upper line of its pair, or the row ends inside it
  const bool head_lone = ((S >> 7) & 1u) != 0u || E <= next_line;
  p.has_head = (S & 127u) >= 64u && (!only_lone || head_lone);
  p.vs = p.has_head ? (E < next_line ? E : next_line) : S;
  p.head_addr = S & ~(uint64_t)63u;
  const uint64_t last_line = (E - 1u) & ~(uint64_t)127u;
  // last line: alone if it is the lower line of its pair, or nothing before it is left to the
  // vector loads
  const bool tail_lone = ((last_line >> 7) & 1u) == 0u || p.vs >= last_line;
  p.has_tail = (p.vs < E) && (((E - 1u) & 127u) < 64u) && (!only_lone || tail_lone);
  p.tail_addr = last_line;
  p.ve = p.has_tail ? (p.vs > last_line ? p.vs : last_line) : E;
  return p;
}

// The head / tail pieces of one row (wave-uniform S, r) travel as two 64-byte scalar reads;
// lanes 0-15 then store the head piece's 16 dwords, lanes 16-31 the tail piece's. Loading and
// storing are separate steps so that a kernel can issue its vector loads in between: the wave
// then waits for one round trip per row, not two.
struct RowPieces {
  u32x16 hv, tv;
};

__device__ __forceinline__ RowPieces load_pieces(const RowSplit& sp) {
  const uint64_t dummy = (uint64_t)(uintptr_t)zcg_dummy_chunk;
  RowPieces q;
  q.hv = *(half_line_ptr)(sp.has_head ? sp.head_addr : dummy);
  q.tv = *(half_line_ptr)(sp.has_tail ? sp.tail_addr : dummy);
  return q;
}

// WS = granularity of rows and bases (the stores' alignment): dwords when it is 4 or more,
// else the dword's 1- or 2-byte elements one by one.
template <int WS>
__device__ __forceinline__ void store_pieces(const RowSplit& sp, const RowPieces& q, uint64_t S,
                                             uint64_t row_bytes, uint8_t* __restrict__ out_row,
                                             unsigned wave_lane) {
  const unsigned k = wave_lane & 15u;
  uint32_t h = 0, t = 0;
#pragma unroll
  for (unsigned j = 0; j < 16; ++j) {
    h = (k == j) ? q.hv[j] : h;
    t = (k == j) ? q.tv[j] : t;
  }
  const bool is_head_lane = wave_lane < 16u;
  const uint64_t a = (is_head_lane ? sp.head_addr : sp.tail_addr) + 4u * k;  // source of my dword
  const uint64_t lo = is_head_lane ? S : sp.ve;
  const uint64_t hi = is_head_lane ? sp.vs : S + row_bytes;
  const bool has = wave_lane < 32u && (is_head_lane ? sp.has_head : sp.has_tail);
  const uint32_t val = is_head_lane ? h : t;
  if constexpr (WS >= 4) {
    if (has && a >= lo && a < hi) *reinterpret_cast<uint32_t*>(out_row + (a - S)) = val;
  } else {
    typedef typename vec_of<WS>::type elem_t;
#pragma unroll
    for (int j = 0; j < 4 / WS; ++j) {
      const uint64_t aj = a + (uint64_t)(j * WS);
      if (has && aj >= lo && aj < hi)
        *reinterpret_cast<elem_t*>(out_row + (aj - S)) = (elem_t)(val >> (8 * j * WS));
    }
  }
}

template <int WS>
__device__ __forceinline__ void move_pieces(const RowSplit& sp, uint64_t S, uint64_t row_bytes,
                                            uint8_t* __restrict__ out_row, unsigned wave_lane) {
  const RowPieces q = load_pieces(sp);
  store_pieces<WS>(sp, q, S, row_bytes, out_row, wave_lane);
}

template <int W, int WS, int U, bool NTS>
__global__ void __launch_bounds__(kBlock)
zcg_k_rows_narrow_half(const uint8_t* __restrict__ table, const int64_t* __restrict__ idx,
                       const int64_t* __restrict__ order, int64_t n_idx, uint8_t* __restrict__ out,
                       int64_t row_bytes, int log2_g, int only_lone) {
  typedef typename vec_of<W>::type vec;
  const unsigned wave_lane = threadIdx.x & (kWave - 1);
  const unsigned lane = threadIdx.x & ((1u << log2_g) - 1u);
  const int groups_per_wave = kWave >> log2_g;
  const int64_t n_groups = ((int64_t)gridDim.x * kBlock) >> log2_g;
  const int64_t wave_group0 = ((int64_t)blockIdx.x * kBlock + (threadIdx.x & ~(kWave - 1))) >> log2_g;
  const int my_group = (int)(wave_lane >> log2_g);
  const int64_t lane_off = (int64_t)lane * W;
  const uint8_t* dummy = reinterpret_cast<const uint8_t*>(zcg_dummy_chunk);

  // wave-uniform trip count: the wave's first group decides
  for (int64_t wbase = wave_group0; wbase < n_idx; wbase += n_groups * U) {
    int64_t row_id[U];
    int64_t out_row[U];  // position in the list = output row
    uint64_t src[U];
    vec v[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t k = wbase + my_group + (int64_t)u * n_groups;
      const int64_t kc = k < n_idx ? k : n_idx - 1;
      out_row[u] = order ? order[kc] : kc;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) row_id[u] = idx[out_row[u]];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t r = wbase + my_group + (int64_t)u * n_groups;
      const uint64_t S = (uint64_t)(uintptr_t)(table + row_id[u] * row_bytes);
      src[u] = S;
      const RowSplit sp = split_row(S, (uint64_t)row_bytes, only_lone != 0);
      const uint64_t a = (S & ~(uint64_t)127u) + (uint64_t)lane_off;  // line-aligned lane mapping
      ok[u] = (r < n_idx) && (a + W > sp.vs) && (a < sp.ve);
      // pointer formed from `table` so that the load stays a global (not flat) access
      v[u] = load_chunk<W, 0>(ok[u] ? table + (a - (uint64_t)(uintptr_t)table) : dummy);
    }
    // row ends through the scalar cache, one row of the wave at a time
#pragma unroll
    for (int u = 0; u < U; ++u) {
      for (int g = 0; g < groups_per_wave; ++g) {
        const int64_t r = wbase + g + (int64_t)u * n_groups;  // uniform
        if (r < n_idx) {
          const uint64_t S = uniform_u64(src[u], g << log2_g);
          const int64_t dst = (int64_t)uniform_u64((uint64_t)out_row[u], g << log2_g);
          const RowSplit sp = split_row(S, (uint64_t)row_bytes, only_lone != 0);
          if (sp.has_head || sp.has_tail)
            move_pieces<WS>(sp, S, (uint64_t)row_bytes, out + dst * row_bytes, wave_lane);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (ok[u]) {
        const RowSplit sp = split_row(src[u], (uint64_t)row_bytes, only_lone != 0);
        const int64_t off = (int64_t)((src[u] & ~(uint64_t)127u) + (uint64_t)lane_off - src[u]);
        store_shifted<W, WS, NTS>(out + out_row[u] * row_bytes, off, (int64_t)(sp.vs - src[u]),
                                  (int64_t)(sp.ve - src[u]), v[u]);
      }
    }
  }
}

template <int W, int WS, int U, bool NTS>
__global__ void __launch_bounds__(kBlock)
zcg_k_rows_wide_half(const uint8_t* __restrict__ table, const int64_t* __restrict__ idx,
                     const int64_t* __restrict__ order, int64_t n_idx, uint8_t* __restrict__ out,
                     int64_t row_bytes, int only_lone) {
  typedef typename vec_of<W>::type vec;
  const unsigned lane = threadIdx.x & (kWave - 1);
  const int64_t n_waves = ((int64_t)gridDim.x * kBlock) / kWave;
  const int64_t wave = ((int64_t)blockIdx.x * kBlock + (threadIdx.x & ~(kWave - 1))) / kWave;
  constexpr int64_t kStep = (int64_t)kWave * W;
  const uint8_t* dummy = reinterpret_cast<const uint8_t*>(zcg_dummy_chunk);

  // the next row's index is fetched while the current row is in flight
  int64_t r_next = 0, row_next = 0;  // output row (position in the list) and table row
  if (wave < n_idx) {
    r_next = order ? order[wave] : wave;
    row_next = idx[r_next];
  }
  for (int64_t k = wave; k < n_idx; k += n_waves) {
    const int64_t r = r_next, row = row_next;
    const int64_t k_next = k + n_waves < n_idx ? k + n_waves : k;
    r_next = order ? order[k_next] : k_next;
    row_next = idx[r_next];
    const uint64_t S = uniform_u64((uint64_t)(uintptr_t)(table + row * row_bytes), 0);
    const RowSplit sp = split_row(S, (uint64_t)row_bytes, only_lone != 0);
    uint8_t* out_row = out + r * row_bytes;
    bool pieces_pending = sp.has_head || sp.has_tail;  // wave-uniform
    const RowPieces q = load_pieces(sp);               // issued now, used after the vector loads
    // passes start on a 256-byte pair boundary, so that the two lines of a pair are always
    // requested by the same batch of loads and travel as one request
    const uint64_t a0 = (sp.vs & ~(uint64_t)255u) + (uint64_t)lane * W;
    for (uint64_t a = a0; a < sp.ve; a += kStep * U) {
      vec v[U];
      bool ok[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint64_t au = a + (uint64_t)u * kStep;
        ok[u] = (au + W > sp.vs) && (au < sp.ve);
        v[u] = load_chunk<W, 0>(ok[u] ? table + (au - (uint64_t)(uintptr_t)table) : dummy);
      }
      if (pieces_pending) {
        store_pieces<WS>(sp, q, S, (uint64_t)row_bytes, out_row, lane);
        pieces_pending = false;
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u])
          store_shifted<W, WS, NTS>(out_row, (int64_t)(a + (uint64_t)u * kStep - S),
                                    (int64_t)(sp.vs - S), (int64_t)(sp.ve - S), v[u]);
    }
    // lanes whose first chunk lies beyond the vector part never entered the loop (all lanes,
    // when the two pieces are the whole row): every lane passes one of the two calls once
    if (pieces_pending) store_pieces<WS>(sp, q, S, (uint64_t)row_bytes, out_row, lane);
  }
}


// The baseline mapping: lane i of the flat grid copies element i of the dense
// output, whatever row it falls in and wherever that row starts in the source.
template <typename E, typename I, int NTL, bool NTS>
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
    if constexpr (NTL == 1) v = __builtin_nontemporal_load(s);
    else if constexpr (NTL == 2) v = *(const volatile E __attribute__((address_space(1)))*)(s);
    else v = *s;
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

// Bytes of a row's line-aligned span that one wavefront takes when p.row_splits wavefronts
// share the row: whole passes of 64 * W * U bytes, so every piece runs the same loop, and
// enough of them to cover the longest span (row_bytes plus less than a line).
inline int64_t piece_bytes_of(const zcg_plan& p, int64_t row_bytes, int W, int U) {
  const int64_t splits = p.row_splits > 1 ? p.row_splits : 1;
  const int64_t pass = (int64_t)kWave * W * U;
  const int64_t per = (row_bytes + p.line_bytes + splits - 1) / splits;
  return (per + pass - 1) / pass * pass;
}

template <int W, int U>
hipError_t launch_rows(const zcg_plan& p, const uint8_t* table, const int64_t* idx, const int64_t* order, int64_t n_idx,
                       uint8_t* out, int64_t row_bytes, hipStream_t s) {
  const unsigned mask = (p.variant == ZCG_VARIANT_ALIGNED) ? (unsigned)(p.line_bytes - 1) : 0u;
  const dim3 grid((unsigned)p.blocks), block(kBlock);
  const int64_t splits = p.row_splits > 1 ? p.row_splits : 1;
  const int64_t piece = piece_bytes_of(p, row_bytes, W, U);
  const int lone = p.half_ends == 2 ? 1 : 0;
  if constexpr (W >= 4) {
    if (p.variant == ZCG_VARIANT_HALFLINE) {
      if (p.iters == 1) {
        if (p.nt_stores)
          zcg_k_rows_narrow_half<W, W, U, true><<<grid, block, 0, s>>>(table, idx, order, n_idx, out,
                                                                     row_bytes, p.log2_group, lone);
        else
          zcg_k_rows_narrow_half<W, W, U, false><<<grid, block, 0, s>>>(table, idx, order, n_idx, out,
                                                                      row_bytes, p.log2_group, lone);
      } else {
        if (p.nt_stores)
          zcg_k_rows_wide_half<W, W, U, true><<<grid, block, 0, s>>>(table, idx, order, n_idx, out, row_bytes, lone);
        else
          zcg_k_rows_wide_half<W, W, U, false><<<grid, block, 0, s>>>(table, idx, order, n_idx, out, row_bytes, lone);
      }
      return hipGetLastError();
    }
  }
#define ZCG_LAUNCH(NTL, NTS)                                                                    \
  do {                                                                                          \
    if (p.iters == 1)                                                                           \
      zcg_k_rows_narrow<W, U, NTL, NTS><<<grid, block, 0, s>>>(table, idx, order, n_idx, out,  \
                                                                 row_bytes, p.log2_group, mask); \
    else                                                                                        \
      zcg_k_rows_wide<W, U, NTL, NTS><<<grid, block, 0, s>>>(table, idx, order, n_idx, out,    \
                                                               row_bytes, mask, splits, piece); \
  } while (0)
  switch (p.nt_loads * 2 + (p.nt_stores ? 1 : 0)) {
    case 0: ZCG_LAUNCH(0, false); break;
    case 1: ZCG_LAUNCH(0, true); break;
    case 2: ZCG_LAUNCH(1, false); break;
    case 3: ZCG_LAUNCH(1, true); break;
    case 4: ZCG_LAUNCH(2, false); break;
    default: ZCG_LAUNCH(2, true); break;
  }
#undef ZCG_LAUNCH
  return hipGetLastError();
}

template <int W>
hipError_t launch_rows_u(const zcg_plan& p, const uint8_t* table, const int64_t* idx,
                         const int64_t* order, int64_t n_idx, uint8_t* out, int64_t row_bytes, hipStream_t s) {
  switch (p.unroll) {
    case 1: return launch_rows<W, 1>(p, table, idx, order, n_idx, out, row_bytes, s);
    case 2: return launch_rows<W, 2>(p, table, idx, order, n_idx, out, row_bytes, s);
    case 4: return launch_rows<W, 4>(p, table, idx, order, n_idx, out, row_bytes, s);
    case 8: return launch_rows<W, 8>(p, table, idx, order, n_idx, out, row_bytes, s);
    default: return hipErrorInvalidValue;
  }
}

template <int W, int WS, int U>
hipError_t launch_shift(const zcg_plan& p, const uint8_t* table, const int64_t* idx, const int64_t* order, int64_t n_idx,
                        uint8_t* out, int64_t row_bytes, hipStream_t s) {
  const unsigned mask = (unsigned)(p.line_bytes - 1);
  const dim3 grid((unsigned)p.blocks), block(kBlock);
  const int64_t splits = p.row_splits > 1 ? p.row_splits : 1;
  const int64_t piece = piece_bytes_of(p, row_bytes, W, U);
  const int lone = p.half_ends == 2 ? 1 : 0;
  {
    if (p.variant == ZCG_VARIANT_HALFLINE) {
      if (p.iters == 1) {
        if (p.nt_stores)
          zcg_k_rows_narrow_half<W, WS, U, true><<<grid, block, 0, s>>>(table, idx, order, n_idx, out,
                                                                         row_bytes, p.log2_group, lone);
        else
          zcg_k_rows_narrow_half<W, WS, U, false><<<grid, block, 0, s>>>(table, idx, order, n_idx, out,
                                                                          row_bytes, p.log2_group, lone);
      } else {
        if (p.nt_stores)
          zcg_k_rows_wide_half<W, WS, U, true><<<grid, block, 0, s>>>(table, idx, order, n_idx, out,
                                                                       row_bytes, lone);
        else
          zcg_k_rows_wide_half<W, WS, U, false><<<grid, block, 0, s>>>(table, idx, order, n_idx, out,
                                                                        row_bytes, lone);
      }
      return hipGetLastError();
    }
  }
  if (p.iters == 1) {
    if (p.nt_stores)
      zcg_k_rows_narrow_shift<W, WS, U, true><<<grid, block, 0, s>>>(table, idx, order, n_idx, out,
                                                                      row_bytes, p.log2_group, mask);
    else
      zcg_k_rows_narrow_shift<W, WS, U, false><<<grid, block, 0, s>>>(table, idx, order, n_idx, out,
                                                                       row_bytes, p.log2_group, mask);
  } else {
    if (p.nt_stores)
      zcg_k_rows_wide_shift<W, WS, U, true><<<grid, block, 0, s>>>(table, idx, order, n_idx, out, row_bytes,
                                                                    mask, splits, piece);
    else
      zcg_k_rows_wide_shift<W, WS, U, false><<<grid, block, 0, s>>>(table, idx, order, n_idx, out,
                                                                     row_bytes, mask, splits, piece);
  }
  return hipGetLastError();
}

template <int W, int WS>
hipError_t launch_shift_u(const zcg_plan& p, const uint8_t* table, const int64_t* idx,
                          const int64_t* order, int64_t n_idx, uint8_t* out, int64_t row_bytes, hipStream_t s) {
  switch (p.unroll) {
    case 1: return launch_shift<W, WS, 1>(p, table, idx, order, n_idx, out, row_bytes, s);
    case 2: return launch_shift<W, WS, 2>(p, table, idx, order, n_idx, out, row_bytes, s);
    case 4: return launch_shift<W, WS, 4>(p, table, idx, order, n_idx, out, row_bytes, s);
    case 8: return launch_shift<W, WS, 8>(p, table, idx, order, n_idx, out, row_bytes, s);
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
  switch (p.nt_loads * 2 + (p.nt_stores ? 1 : 0)) {
    case 0: ZCG_LAUNCH(0, false); break;
    case 1: ZCG_LAUNCH(0, true); break;
    case 2: ZCG_LAUNCH(1, false); break;
    case 3: ZCG_LAUNCH(1, true); break;
    case 4: ZCG_LAUNCH(2, false); break;
    default: ZCG_LAUNCH(2, true); break;
  }
#undef ZCG_LAUNCH
  return hipGetLastError();
}

}  // namespace

hipError_t zcg_launch_gather(const zcg_plan& p, const void* table, const int64_t* idx,
                             const int64_t* order, int64_t n_idx, void* out, int64_t row_bytes,
                             int elem, hipStream_t stream) {
  // the flat kernel has no processing order
  if (order && p.variant == ZCG_VARIANT_NAIVE) return hipErrorInvalidValue;
  if (p.variant == ZCG_VARIANT_NAIVE) {
    const int64_t dim = row_bytes / elem;
    switch (elem) {
      case 8: return launch_flat<uint64_t>(p, table, idx, n_idx, out, dim, stream);
      case 4: return launch_flat<uint32_t>(p, table, idx, n_idx, out, dim, stream);
      case 2: return launch_flat<uint16_t>(p, table, idx, n_idx, out, dim, stream);
      default: return launch_flat<uint8_t>(p, table, idx, n_idx, out, dim, stream);
    }
  }
  const uint8_t* t = static_cast<const uint8_t*>(table);
  uint8_t* o = static_cast<uint8_t*>(out);
  if (p.store_bytes < p.vec_bytes) {
    switch (p.vec_bytes * 100 + p.store_bytes) {
      case 1608: return launch_shift_u<16, 8>(p, t, idx, order, n_idx, o, row_bytes, stream);
      case 1604: return launch_shift_u<16, 4>(p, t, idx, order, n_idx, o, row_bytes, stream);
      case 1602: return launch_shift_u<16, 2>(p, t, idx, order, n_idx, o, row_bytes, stream);
      case 804: return launch_shift_u<8, 4>(p, t, idx, order, n_idx, o, row_bytes, stream);
      case 802: return launch_shift_u<8, 2>(p, t, idx, order, n_idx, o, row_bytes, stream);
      case 1601: return launch_shift_u<16, 1>(p, t, idx, order, n_idx, o, row_bytes, stream);
      case 801: return launch_shift_u<8, 1>(p, t, idx, order, n_idx, o, row_bytes, stream);
      default: return hipErrorInvalidValue;
    }
  }
  switch (p.vec_bytes) {
    case 16: return launch_rows_u<16>(p, t, idx, order, n_idx, o, row_bytes, stream);
    case 8: return launch_rows_u<8>(p, t, idx, order, n_idx, o, row_bytes, stream);
    case 4: return launch_rows_u<4>(p, t, idx, order, n_idx, o, row_bytes, stream);
    case 2: return launch_rows_u<2>(p, t, idx, order, n_idx, o, row_bytes, stream);
    case 1: return launch_rows_u<1>(p, t, idx, order, n_idx, o, row_bytes, stream);
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
