// Processing order for the ordered gather: a permutation `order` of [0, n) such
// that idx[order[k]] ascends with k, equal entries in list order. Rows are then
// fetched in ascending table order -- neighbouring work items touch neighbouring
// lines and pages of the host table, so rows that share a line or a 256-byte pair
// of lines share a link request -- while every row still lands at its own
// position of the output.
//
// The order is built by a least-significant-digit radix sort written for
// wave64: digits of up to 8 bits, and per digit three kernels,
//   count   : every block histograms the digit over its tile of the list,
//   offsets : per bin, an exclusive prefix of the counts over the blocks,
//   scatter : every block recounts its tile per wavefront, turns the counts into
//             output positions (bin base + blocks before + wavefronts before) and
//             moves its elements; inside a wavefront elements are ranked 64 at a
//             time with ballots, so the pass is stable and its result does not
//             depend on scheduling.
// No kernel waits for another block, nothing is cleared with a memory-set, and all
// temporary memory is the caller's (or the static array of the allocation-free
// entry point): the whole build is a chain of plain kernel launches on one stream.
// Between passes an element travels as (32-bit key, 32-bit list position); the
// output array doubles as the second buffer of the ping-pong. Tables of 2^32 rows
// or more carry the position only and look the key up again in the list.
#include <hip/hip_runtime.h>

#include <mutex>

#include "zcg_internal.h"

// Temporary memory of zcg_make_order_static: one array per GPU the library runs on, held until
// the process ends. In host code this name is only a handle for hipGetSymbolAddress, never an
// address to pass on.
constexpr int64_t kStaticMaxIdx = ZCG_STATIC_ORDER_MAX_IDX;
constexpr int64_t kStaticScratchBytes = kStaticMaxIdx * 8 + (1 << 20) + (64 << 10);  // buffer + counts + bin sizes
static __device__ __align__(256) unsigned char zcg_order_static_scratch[kStaticScratchBytes];

namespace {

constexpr int kBlock = 256;      // 4 wavefronts
constexpr int kWave = 64;
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kMaxBins = 256;    // digits of at most 8 bits
constexpr int64_t kAlign = 256;
constexpr int64_t kMaxBlocks = 1024;  // cap on the grid: the per-bin prefix is one block-wide scan

int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// Elements each wavefront owns: 256 (four steps of 64; short stretches mean many wavefronts in
// flight, and a pass is bound by the latency of its dependent steps, not by bytes), more for
// lists beyond 1 M entries so that the grid stays within kMaxBlocks; a multiple of the wave size.
int64_t wave_span(int64_t n) {
  const int64_t need = (n + kMaxBlocks * kWavesPerBlock - 1) / (kMaxBlocks * kWavesPerBlock);
  return need <= 256 ? 256 : round_up(need, kWave);
}
int64_t grid_blocks(int64_t n) {
  const int64_t per_block = wave_span(n) * kWavesPerBlock;
  return (n + per_block - 1) / per_block;
}
// Bytes set aside for the per-bin per-block counts: room for the grid of any list of up to n
// entries (the grid grows with n up to kMaxBlocks and never exceeds it), so that the scratch a
// caller sized for its longest list also fits every shorter one.
int64_t counts_bytes(int64_t n) {
  const int64_t small_grid = (n + 256 * kWavesPerBlock - 1) / (256 * kWavesPerBlock);
  return round_up(kMaxBins * (small_grid < kMaxBlocks ? small_grid : kMaxBlocks) * 4, kAlign);
}

// Where a pass reads its elements from.
enum Src { SRC_LIST = 0,     // the index list itself: key = idx[i], position = i
           SRC_CARRIED = 1,  // (key32[i], pos[i]) written by the previous pass
           SRC_REFETCH = 2   // pos[i] written by the previous pass, key = idx[pos[i]]
};
// What a pass writes.
enum Dst { DST_CARRIED = 0,  // key32 and position
           DST_POS = 1,      // position only (keys of more than 32 bits)
           DST_ORDER = 2     // the final int64 order
};

struct PassIO {
  const int64_t* idx;
  const uint32_t* src_keys;
  const uint32_t* src_pos;
  uint32_t* dst_keys;
  uint32_t* dst_pos;
  int64_t* order;
};

template <int SRC>
__device__ __forceinline__ void fetch(const PassIO& io, int64_t i, uint64_t& key, uint32_t& pos) {
  if constexpr (SRC == SRC_LIST) {
    key = (uint64_t)io.idx[i];
    pos = (uint32_t)i;
  } else if constexpr (SRC == SRC_CARRIED) {
    key = io.src_keys[i];
    pos = io.src_pos[i];
  } else {
    pos = io.src_pos[i];
    key = (uint64_t)io.idx[pos];
  }
}

// Lanes of the wavefront that are active and hold the same digit as this lane (8 ballots).
__device__ __forceinline__ uint64_t same_digit_lanes(unsigned d, bool active) {
  uint64_t m = __ballot(active);
#pragma unroll
  for (int b = 0; b < 8; ++b) {
    const bool bit = (d >> b) & 1u;
    const uint64_t with_bit = __ballot(active && bit);
    m &= bit ? with_bit : ~with_bit;
  }
  return m;
}

// Exclusive prefix sum over the 256 threads of a block; *total (may be null) gets the sum.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wave_sums,
                                                         uint32_t* total) {
  const unsigned lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  uint32_t incl = v;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const uint32_t up = __shfl_up(incl, d, kWave);
    if (lane >= (unsigned)d) incl += up;
  }
  if (lane == kWave - 1) wave_sums[w] = incl;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int k = 0; k < kWavesPerBlock; ++k) {
    const uint32_t s = wave_sums[k];
    before += (unsigned)k < w ? s : 0u;
    all += s;
  }
  if (total) *total = all;
  __syncthreads();  // wave_sums may be reused by the caller
  return before + incl - v;
}

// counts[bin * n_blocks + block] = entries of the block's tile whose digit is `bin`.
template <int SRC>
__global__ void __launch_bounds__(kBlock)
zcg_k_order_count(PassIO io, int64_t n, int64_t span, int shift, unsigned mask,
                  uint32_t* __restrict__ counts) {
  __shared__ uint32_t hist[kMaxBins];
  hist[threadIdx.x] = 0;
  __syncthreads();
  const unsigned lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int64_t begin = ((int64_t)blockIdx.x * kWavesPerBlock + w) * span;
  const int64_t end = begin + span < n ? begin + span : n;
  for (int64_t i = begin + lane; i < end; i += kWave) {
    uint64_t key;
    uint32_t pos;
    fetch<SRC>(io, i, key, pos);
    atomicAdd(&hist[(unsigned)(key >> shift) & mask], 1u);
  }
  __syncthreads();
  if (threadIdx.x <= mask) counts[(int64_t)threadIdx.x * gridDim.x + blockIdx.x] = hist[threadIdx.x];
}

// One block per bin: counts[bin][0..n_blocks) becomes its exclusive prefix over the blocks,
// totals[bin] the bin's size. n_blocks <= kMaxBlocks = 4 entries per thread.
__global__ void __launch_bounds__(kBlock)
zcg_k_order_offsets(uint32_t* __restrict__ counts, uint32_t* __restrict__ totals, int n_blocks) {
  __shared__ uint32_t wave_sums[kWavesPerBlock];
  constexpr int kPer = (int)(kMaxBlocks / kBlock);
  uint32_t* row = counts + (int64_t)blockIdx.x * n_blocks;
  uint32_t v[kPer], sum = 0;
#pragma unroll
  for (int k = 0; k < kPer; ++k) {
    const int j = (int)threadIdx.x * kPer + k;
    v[k] = j < n_blocks ? row[j] : 0u;
    sum += v[k];
  }
  uint32_t total;
  uint32_t run = block_exclusive_scan(sum, wave_sums, &total);
#pragma unroll
  for (int k = 0; k < kPer; ++k) {
    const int j = (int)threadIdx.x * kPer + k;
    if (j < n_blocks) row[j] = run;
    run += v[k];
  }
  if (threadIdx.x == 0) totals[blockIdx.x] = total;
}

template <int SRC, int DST>
__global__ void __launch_bounds__(kBlock)
zcg_k_order_scatter(PassIO io, int64_t n, int64_t span, int shift, unsigned mask,
                    const uint32_t* __restrict__ offsets, const uint32_t* __restrict__ totals) {
  __shared__ uint32_t next[kWavesPerBlock][kMaxBins];  // per wavefront and bin: next output position
  __shared__ uint32_t wave_sums[kWavesPerBlock];
  const unsigned lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const unsigned bin = threadIdx.x;
  const unsigned n_bins = mask + 1u;
#pragma unroll
  for (int k = 0; k < kWavesPerBlock; ++k) next[k][bin] = 0;
  // where each bin starts in the output: exclusive prefix of the bin sizes
  const uint32_t bin_base = block_exclusive_scan(bin < n_bins ? totals[bin] : 0u, wave_sums, nullptr);

  const int64_t begin = ((int64_t)blockIdx.x * kWavesPerBlock + w) * span;
  const int64_t end = begin + span < n ? begin + span : n;
  // 1. every wavefront counts the digits of its own stretch of the tile
  for (int64_t i = begin + lane; i < end; i += kWave) {
    uint64_t key;
    uint32_t pos;
    fetch<SRC>(io, i, key, pos);
    atomicAdd(&next[w][(unsigned)(key >> shift) & mask], 1u);
  }
  __syncthreads();
  // 2. counts -> first output position of (wavefront, bin): the bin's base, the entries of
  //    earlier blocks, the entries of earlier wavefronts of this block
  if (bin < n_bins) {
    uint32_t run = bin_base + offsets[(int64_t)bin * gridDim.x + blockIdx.x];
#pragma unroll
    for (int k = 0; k < kWavesPerBlock; ++k) {
      const uint32_t c = next[k][bin];
      next[k][bin] = run;
      run += c;
    }
  }
  __syncthreads();
  // 3. every wavefront walks its stretch again in list order, 64 entries at a time; entries of
  //    one step with the same digit are ranked by lane, and only this wavefront touches next[w]
  //    (the next step's entry is fetched while this step's is ranked and stored)
  uint64_t key_next = 0;
  uint32_t pos_next = 0;
  if (begin + lane < end) fetch<SRC>(io, begin + lane, key_next, pos_next);
  for (int64_t i0 = begin; i0 < end; i0 += kWave) {
    const int64_t i = i0 + lane;
    const bool active = i < end;
    const uint64_t key = key_next;
    const uint32_t pos = pos_next;
    if (i + kWave < end) fetch<SRC>(io, i + kWave, key_next, pos_next);
    const unsigned d = (unsigned)(key >> shift) & mask;
    const uint64_t peers = same_digit_lanes(d, active);
    const unsigned rank = (unsigned)__popcll(peers & (((uint64_t)1 << lane) - 1u));
    const int leader = __ffsll((unsigned long long)peers) - 1;
    uint32_t first = 0;
    if (active && (int)lane == leader) first = atomicAdd(&next[w][d], (uint32_t)__popcll(peers));
    first = __shfl(first, leader < 0 ? 0 : leader, kWave);
    if (active) {
      const uint32_t at = first + rank;
      if constexpr (DST == DST_ORDER) {
        io.order[at] = (int64_t)pos;
      } else {
        if constexpr (DST == DST_CARRIED) io.dst_keys[at] = (uint32_t)key;
        io.dst_pos[at] = pos;
      }
    }
  }
}

template <int SRC>
hipError_t launch_pass(int dst, const PassIO& io, int64_t n, int64_t span, int shift, unsigned mask,
                       uint32_t* counts, uint32_t* totals, hipStream_t s) {
  const dim3 grid((unsigned)grid_blocks(n)), block(kBlock);
  zcg_k_order_count<SRC><<<grid, block, 0, s>>>(io, n, span, shift, mask, counts);
  zcg_k_order_offsets<<<dim3(mask + 1u), block, 0, s>>>(counts, totals, (int)grid.x);
  switch (dst) {
    case DST_CARRIED:
      zcg_k_order_scatter<SRC, DST_CARRIED><<<grid, block, 0, s>>>(io, n, span, shift, mask, counts, totals);
      break;
    case DST_POS:
      zcg_k_order_scatter<SRC, DST_POS><<<grid, block, 0, s>>>(io, n, span, shift, mask, counts, totals);
      break;
    default:
      zcg_k_order_scatter<SRC, DST_ORDER><<<grid, block, 0, s>>>(io, n, span, shift, mask, counts, totals);
      break;
  }
  return hipGetLastError();
}

}  // namespace

int64_t zcg_order_scratch_bytes(int64_t n_idx) {
  if (n_idx <= 0) return 0;
  // one (key32, position) buffer, the per-bin per-block counts, the bin sizes
  return round_up(n_idx * 8, kAlign) + counts_bytes(n_idx) + round_up(kMaxBins * 4, kAlign);
}

hipError_t zcg_order_launch(const int64_t* idx, int64_t n, int64_t n_rows, int64_t* order,
                            void* scratch, hipStream_t s) {
  // bits that can differ between valid indices, split evenly over digits of at most 8 bits
  int bits = 1;
  while (bits < 63 && ((int64_t)1 << bits) < n_rows) ++bits;
  const int passes = (bits + 7) / 8;
  const bool wide_keys = bits > 32;
  char* ws = static_cast<char*>(scratch);
  uint32_t* buf_a = reinterpret_cast<uint32_t*>(ws);
  uint32_t* counts = reinterpret_cast<uint32_t*>(ws + round_up(n * 8, kAlign));
  uint32_t* totals = counts + counts_bytes(n) / 4;
  uint32_t* buf_o = reinterpret_cast<uint32_t*>(order);  // the output array is the second buffer
  const int64_t span = wave_span(n);

  int shift = 0;
  const uint32_t* src = nullptr;
  for (int p = 0; p < passes; ++p) {
    const int digit_bits = (bits - shift + (passes - p) - 1) / (passes - p);
    const unsigned mask = (1u << digit_bits) - 1u;
    const bool last = p == passes - 1;
    // passes alternate between the two buffers such that the last one reads buffer A
    uint32_t* dst = ((passes - 2 - p) % 2 == 0) ? buf_a : buf_o;
    PassIO io;
    io.idx = idx;
    io.src_keys = src;
    io.src_pos = src ? src + (wide_keys ? 0 : n) : nullptr;
    io.dst_keys = last ? nullptr : dst;
    io.dst_pos = last ? nullptr : dst + (wide_keys ? 0 : n);
    io.order = order;
    const int dst_kind = last ? DST_ORDER : (wide_keys ? DST_POS : DST_CARRIED);
    hipError_t e;
    if (p == 0) e = launch_pass<SRC_LIST>(dst_kind, io, n, span, shift, mask, counts, totals, s);
    else if (wide_keys) e = launch_pass<SRC_REFETCH>(dst_kind, io, n, span, shift, mask, counts, totals, s);
    else e = launch_pass<SRC_CARRIED>(dst_kind, io, n, span, shift, mask, counts, totals, s);
    if (e != hipSuccess) return e;
    src = dst;
    shift += digit_bits;
  }
  return hipSuccess;
}

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
void* g_static_ptr[kMaxDevices] = {};  // device address of the static array, per device

// The array's address on the current device, looked up once per device.
hipError_t static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(g_static_mu);
  if (!g_static_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(zcg_order_static_scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_static_ptr[dev] = p;
  }
  *out = g_static_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" {

int zcg_make_order_static(const int64_t* idx_dev, int64_t n_idx, int64_t n_rows, int64_t* order_dev,
                          void* stream) {
  if (n_idx < 0 || n_rows < 1) return ZCG_EINVAL;
  if (n_idx > kStaticMaxIdx || zcg_order_scratch_bytes(n_idx) > kStaticScratchBytes) return ZCG_ECAPACITY;
  if (n_idx == 0) return ZCG_OK;
  if (!idx_dev || !order_dev) return ZCG_EINVAL;
  if (((uintptr_t)idx_dev | (uintptr_t)order_dev) % 8) return ZCG_EALIGN;
  {
    const uintptr_t i0 = (uintptr_t)idx_dev, o0 = (uintptr_t)order_dev, len = (uintptr_t)(n_idx * 8);
    if (i0 < o0 + len && o0 < i0 + len) return ZCG_EALIAS;  // the order may not overwrite the list
  }
  void* scratch = nullptr;
  hipError_t e = static_scratch(&scratch);
  if (e != hipSuccess) return zcg_fail_hip(e);
  // nothing in the array has to start at zero: every count, prefix and buffer entry a pass
  // reads was written earlier in the same call
  e = zcg_order_launch(idx_dev, n_idx, n_rows, order_dev, scratch, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ZCG_OK : zcg_fail_hip(e);
}

int zcg_order_workspace_bytes(int64_t n_idx, int64_t* bytes) {
  if (n_idx < 0 || !bytes) return ZCG_EINVAL;
  *bytes = zcg_order_scratch_bytes(n_idx);
  return ZCG_OK;
}

int zcg_make_order(const int64_t* idx_dev, int64_t n_idx, int64_t n_rows, int64_t* order_dev,
                   void* workspace_dev, int64_t workspace_bytes, void* stream) {
  if (n_idx < 0 || n_rows < 1 || n_idx > (int64_t)UINT32_MAX) return ZCG_EINVAL;
  if (n_idx == 0) return ZCG_OK;
  if (!idx_dev || !order_dev || !workspace_dev) return ZCG_EINVAL;
  if (((uintptr_t)idx_dev | (uintptr_t)order_dev) % 8 || (uintptr_t)workspace_dev % kAlign)
    return ZCG_EALIGN;
  if (workspace_bytes < zcg_order_scratch_bytes(n_idx)) return ZCG_EINVAL;
  {  // the list is read while the order and the workspace are written, and those two differ
    const uintptr_t i0 = (uintptr_t)idx_dev, o0 = (uintptr_t)order_dev, w0 = (uintptr_t)workspace_dev;
    const uintptr_t len = (uintptr_t)(n_idx * 8), w1 = w0 + (uintptr_t)workspace_bytes;
    if ((i0 < o0 + len && o0 < i0 + len) || (i0 < w1 && w0 < i0 + len) || (o0 < w1 && w0 < o0 + len))
      return ZCG_EALIAS;
  }
  hipError_t e = zcg_order_launch(idx_dev, n_idx, n_rows, order_dev, workspace_dev,
                                  static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ZCG_OK : zcg_fail_hip(e);
}

}  // extern "C"
