// Host-side launch planning for the gather: picks the kernel, the bytes per lane, the lanes per
// row, the passes per row and the grid from the row size, the real addresses and the options.
// The defaults are measured ones (see the comments at each choice).
#include <stdint.h>

#include "zcg_internal.h"

namespace {

constexpr int kBlock = 256;  // 4 wavefronts of 64 lanes, as in the kernels
constexpr int kWave = 64;

int saturate_int(int64_t x) { return x > INT32_MAX ? INT32_MAX : (int)x; }  // passes of absurdly long rows

int floor_pow2_divisor(uint64_t x, int cap) {  // largest power of two <= cap dividing x
  int w = cap;
  while (w > 1 && (x % (uint64_t)w) != 0) w >>= 1;
  return w;
}

}  // namespace

int zcg_make_plan(int64_t row_bytes, int elem, uintptr_t table_addr, uintptr_t out_addr,
                  int64_t n_idx, bool host_resident, bool ordered, const zcg_launch_opts* opts,
                  zcg_plan* plan) {
  zcg_launch_opts o = {};
  if (opts) o = *opts;
  if (row_bytes <= 0 || (elem != 1 && elem != 2 && elem != 4 && elem != 8) || row_bytes % elem != 0 || n_idx < 0 || !plan)
    return ZCG_EINVAL;
  if (n_idx > INT64_MAX / row_bytes) return ZCG_EINVAL;  // the output would not fit an address space
  if (table_addr % (uintptr_t)elem != 0 || out_addr % (uintptr_t)elem != 0) return ZCG_EALIGN;

  // defaults
  int variant = o.variant;
  int line = o.line_bytes ? o.line_bytes : 128;
  int unroll = o.unroll ? o.unroll : (host_resident ? 2 : 4);
  int vec_cap = o.vec_bytes ? o.vec_bytes : 16;
  if (!o.vec_bytes && host_resident) {
    // Measured over the host link: 8-byte lanes (a wave pass = 512 bytes = 4 lines) are as
    // fast or slightly faster than 16-byte lanes for every row longer than a line; rows of
    // at most one line do best with 16-byte lanes.
    const int pref = row_bytes <= 128 ? 16 : 8;
    vec_cap = pref < elem ? elem : pref;
  }
  // HBM-resident tables (measured): a grid large enough for one row per group without
  // striding and non-temporal table loads are worth up to +19 % (1 KiB rows).
  int max_blocks = o.max_blocks ? o.max_blocks
                                : (!host_resident ? 65536 : (row_bytes > 128 ? 2048 : 8192));
  const int ntl = o.nt_loads == 1 ? 1 : (o.nt_loads == 3 ? 2 : (o.nt_loads == 0 && !host_resident ? 1 : 0));
  const int nts = o.nt_stores == 2 ? 0 : 1;                // default: non-temporal stores
  if (variant < 0 || variant >= ZCG_VARIANT_COUNT) return ZCG_EINVAL;
  if (line != 32 && line != 64 && line != 128 && line != 256) return ZCG_EINVAL;
  if (unroll != 1 && unroll != 2 && unroll != 4 && unroll != 8) return ZCG_EINVAL;
  if (vec_cap != 1 && vec_cap != 2 && vec_cap != 4 && vec_cap != 8 && vec_cap != 16)
    return ZCG_EINVAL;
  if (max_blocks < 1 || o.nt_loads < 0 || o.nt_loads > 3 || o.nt_stores < 0 || o.nt_stores > 2)
    return ZCG_EINVAL;
  if (vec_cap < elem || o.shifted_stores < 0 || o.shifted_stores > 2) return ZCG_EINVAL;
  if (o.row_splits < 0 || o.row_splits > 4096) return ZCG_EINVAL;
  if (o.half_ends < 0 || o.half_ends > 2) return ZCG_EINVAL;
  int min_lg = 0;
  if (o.group_lanes) {
    if (o.group_lanes < 1 || o.group_lanes > kWave || (o.group_lanes & (o.group_lanes - 1)))
      return ZCG_EINVAL;
    while ((1 << min_lg) < o.group_lanes) ++min_lg;
  } else if (host_resident) {
    // Measured: over the host link one row per wave-wide load instruction is the
    // fastest and the least sensitive to grid size and unrolling; rows of at most
    // one line do slightly better 16 lanes wide on a larger grid.
    min_lg = row_bytes > 128 ? 6 : 4;
  }

  // Widest access that keeps every chunk of every row aligned at both ends.
  int w = floor_pow2_divisor((uint64_t)row_bytes, vec_cap);
  w = floor_pow2_divisor((uint64_t)table_addr, w);
  w = floor_pow2_divisor((uint64_t)out_addr, w);

  // HALFLINE moves dwords through the scalar path and needs loads of at least 4 bytes: rows and
  // bases 4-byte granular, or less with wide line-aligned loads and element-wise (shifted) stores.
  const bool half_ok = (w >= 4) || (vec_cap >= 8 && o.shifted_stores != 2);
  if (variant == ZCG_VARIANT_HALFLINE && !half_ok) variant = ZCG_VARIANT_ALIGNED;
  if (variant == ZCG_VARIANT_HALFLINE) line = 128;
  if (variant == ZCG_VARIANT_AUTO) {
    // Rows shorter than a line, or made of whole lines on a line-aligned base,
    // need no realignment (the paper's applicability rule, end of Section 3.2.1).
    const bool whole_lines = (row_bytes % line == 0) && (table_addr % (uintptr_t)line == 0);
    // Over the host link whole-line rows that take several passes and do not sit on the 256-byte
    // pair grid (640, 896, 1152 ... bytes) still gain 0.7...1.4 % from passes that start on pair
    // boundaries, which the line-mapped kernels provide.
    const bool off_pair_grid = host_resident && row_bytes > (int64_t)kWave * vec_cap &&
                               (row_bytes % 256 != 0 || table_addr % 256 != 0);
    variant = (row_bytes < line || (whole_lines && !off_pair_grid)) ? ZCG_VARIANT_ROWVEC
                                                                    : ZCG_VARIANT_ALIGNED;
    // Unaligned rows of more than a line over the host link: row ends that fit half a line go
    // through 64-byte scalar reads. From 768 bytes on every such end does (measured +1.3...4 % on
    // 816...2,408-byte rows with 8- or 16-byte lanes: one more request per 6+ lines, 40 wire
    // bytes less; break-even at 720 bytes); on shorter rows only ends whose line would be
    // requested alone anyway, which saves bytes without adding requests (measured +1.5...4 % on
    // 160...720-byte rows, +6 % on sampled minibatches of 400-byte rows; converting every end
    // there loses 1...8 %, as such rows are close to the link's request limit).
    // Rows that tile half lines exactly (16, 32 or 64 bytes on a 64-byte aligned base) over the
    // host link: each is one 64-byte scalar read instead of one lone 128-byte line, the same
    // request count and half the bytes (measured +1...3 % from 110 k rows per call on, -0.5 % at
    // 20 k, where the row-by-row scalar reads of a wave are not hidden yet). Not when the rows are
    // walked in ascending order: neighbouring rows then share whole lines and pairs, which only
    // vector loads coalesce.
    if (variant == ZCG_VARIANT_ROWVEC && host_resident && row_bytes >= 16 && row_bytes <= 64 &&
        64 % row_bytes == 0 && table_addr % 64 == 0 && n_idx >= 65536 && w >= 4 && !ordered)
      variant = ZCG_VARIANT_HALFLINE, line = 128;
    // A short list of long rows is split over several wavefronts per row (below), which the
    // half-line kernel does not do: filling the link matters more there than 64 bytes per row.
    const bool will_split = o.row_splits ? o.row_splits > 1
                                         : (n_idx < 2048 && row_bytes >= (int64_t)8 * kWave * vec_cap * unroll);
    if (variant == ZCG_VARIANT_ALIGNED && host_resident && row_bytes > 128 && !will_split &&
        (w >= 8 || (vec_cap >= 8 && o.shifted_stores != 2)))
      variant = ZCG_VARIANT_HALFLINE, line = 128;
  }

  // The half-line kernels wait for their scalar reads row by row, so they want a wavefront per
  // row rather than a stride (measured on 400-byte rows: 45.6 GB/s with 2048 blocks, 46.4 with
  // 16384 or more; no difference on 2,408-byte rows).
  if (variant == ZCG_VARIANT_HALFLINE && host_resident && !o.max_blocks) max_blocks = 16384;

  plan->variant = variant;
  plan->half_ends = variant != ZCG_VARIANT_HALFLINE ? 0
                    : (o.half_ends ? o.half_ends : (row_bytes >= 768 ? 1 : 2));
  plan->row_splits = 1;
  plan->line_bytes = line;
  plan->unroll = unroll;
  plan->nt_loads = ntl;
  plan->nt_stores = nts;

  int64_t want_blocks;
  if (variant == ZCG_VARIANT_NAIVE) {
    plan->vec_bytes = elem;
    plan->store_bytes = elem;
    plan->log2_group = 0;
    plan->iters = 1;
    plan->unroll = 1;
    const int64_t total = n_idx * (row_bytes / elem);
    want_blocks = (total + kBlock - 1) / kBlock;
  } else {
    // ALIGNED loads sit at line-aligned positions, so they can stay vec_cap wide when the
    // rows or bases are less aligned than that; only the stores drop to w (shifted stores).
    const bool line_mapped = variant == ZCG_VARIANT_ALIGNED || variant == ZCG_VARIANT_HALFLINE;
    int wl = w;
    if (line_mapped && w < vec_cap && vec_cap >= 8 && o.shifted_stores != 2)
      wl = vec_cap;
    plan->vec_bytes = wl;
    plan->store_bytes = w;
    int64_t worst_span = row_bytes + (line_mapped ? line - w : 0);
    int64_t chunks = (worst_span + wl - 1) / wl;
    int lg = 0;
    while (lg < 6 && ((int64_t)1 << lg) < chunks) ++lg;
    if (lg < min_lg) lg = min_lg;
    plan->log2_group = lg;
    plan->iters = saturate_int((chunks + ((int64_t)1 << lg) - 1) >> lg);
    if (plan->iters == 1) {
      const int64_t groups = (n_idx + unroll - 1) / unroll;
      want_blocks = ((groups << lg) + kBlock - 1) / kBlock;
    } else {
      plan->log2_group = 6;
      // Rows that take several passes anyway: over the host link the passes start on a 256-byte
      // boundary, so that the two lines of a 256-byte aligned pair are always requested by the
      // same batch of loads and travel as one request (measured +1...2 % on 1,028...2,408-byte
      // rows; the half-line kernel does the same on its own).
      if (variant == ZCG_VARIANT_ALIGNED && host_resident && !o.line_bytes && line < 256) {
        line = 256;
        plan->line_bytes = line;
        worst_span = row_bytes + line - w;
        chunks = (worst_span + wl - 1) / wl;
        plan->iters = saturate_int((chunks + kWave - 1) / kWave);
      }
      // One wavefront per row keeps only unroll * 64 * vec_bytes bytes of that row in flight
      // (measured: 0.7 GB/s per row over the host link), so a short list of long rows cannot
      // fill the link. Then several wavefronts share a row, each taking a contiguous piece of
      // at least 4 passes, until about 4096 (host) / 16384 (HBM) wavefronts have work.
      int splits = 1;
      if (variant != ZCG_VARIANT_HALFLINE) {
        const int64_t pass = (int64_t)kWave * wl * unroll;
        const int64_t most = (worst_span + pass - 1) / pass;  // pieces of one pass each
        if (o.row_splits) {
          splits = (int)(o.row_splits < most ? o.row_splits : most);
        } else {
          const int64_t target = host_resident ? 4096 : 16384;
          int64_t want = n_idx > 0 ? target / n_idx : 1;
          const int64_t cap = most / 4;
          if (want > cap) want = cap;
          if (want > 4096) want = 4096;
          splits = want > 1 ? (int)want : 1;
        }
      }
      plan->row_splits = splits;
      want_blocks = (n_idx * splits * kWave + kBlock - 1) / kBlock;
    }
  }
  if (want_blocks < 1) want_blocks = 1;
  plan->blocks = (int)(want_blocks < max_blocks ? want_blocks : max_blocks);
  return ZCG_OK;
}
