// Exercises the launch planning (pure host code) under AddressSanitizer / UBSan over a large
// seeded set of shapes, addresses, list lengths and options, including extreme values. Built
// and run by test_sanitizers.py with g++; no GPU and no HIP runtime call is involved.
#include <cstdint>
#include <cstdio>

#include "zcg_internal.h"

static uint64_t mix(uint64_t& s) {
  s += 0x9E3779B97F4A7C15ull;
  uint64_t z = s;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

int main() {
  uint64_t s = 2103;
  const int elems[] = {1, 2, 4, 8, 3, 0};
  const int64_t dims[] = {1, 2, 3, 7, 16, 25, 100, 128, 257, 602, 4099, 70001, 1 << 20, ((int64_t)1 << 40)};
  const int64_t lists[] = {0, 1, 2, 63, 2048, 4097, 110000, 1000000, ((int64_t)1 << 31) + 5, ((int64_t)1 << 45), -1};
  const int picks[] = {0, 1, 2, 3, 4, 5, 8, 16, 32, 64, 128, 256, 4096, 4097, -1, 1 << 30};
  long ok = 0, rejected = 0;
  for (int it = 0; it < 200000; ++it) {
    const int elem = elems[(mix(s) % 16) ? mix(s) % 4 : mix(s) % 6];  // mostly a valid element size
    const int64_t dim = dims[mix(s) % 14];
    const int64_t row_bytes = dim * (elem > 0 ? elem : 1);
    const uintptr_t step = (mix(s) % 8) && elem > 0 ? (uintptr_t)elem : 1;  // mostly element-aligned bases
    const uintptr_t table = (uintptr_t)0x7F0000000000ull + (uintptr_t)(mix(s) % 256) * step;
    const uintptr_t out = (uintptr_t)0x7E0000000000ull + (uintptr_t)(mix(s) % 256) * step;
    const int64_t n_idx = lists[mix(s) % 11];
    zcg_launch_opts o = {};
    // mostly valid values, now and then a wild one
    auto pick = [&](const int* valid, int n_valid) {
      return (mix(s) % 8) ? valid[mix(s) % (uint64_t)n_valid] : picks[mix(s) % 16];
    };
    const int v_variant[] = {0, 1, 2, 3, 4}, v_blocks[] = {0, 1, 7, 300, 16384, 1 << 20};
    const int v_unroll[] = {0, 1, 2, 4, 8}, v_line[] = {0, 32, 64, 128, 256}, v_03[] = {0, 1, 2, 3};
    const int v_02[] = {0, 1, 2}, v_vec[] = {0, 1, 2, 4, 8, 16}, v_lanes[] = {0, 1, 2, 4, 8, 16, 32, 64};
    const int v_splits[] = {0, 1, 2, 5, 64, 4096};
    o.variant = pick(v_variant, 5);
    o.max_blocks = pick(v_blocks, 6);
    o.unroll = pick(v_unroll, 5);
    o.line_bytes = pick(v_line, 5);
    o.nt_loads = pick(v_03, 4);
    o.nt_stores = pick(v_02, 3);
    o.vec_bytes = pick(v_vec, 6);
    o.group_lanes = pick(v_lanes, 8);
    o.shifted_stores = pick(v_02, 3);
    o.row_splits = pick(v_splits, 6);
    o.half_ends = pick(v_02, 3);
    zcg_plan p = {};
    const int rc = zcg_make_plan(row_bytes, elem, table, out, n_idx, (mix(s) & 1) != 0, (mix(s) & 1) != 0,
                                 (mix(s) % 8) ? &o : nullptr, &p);
    if (rc != ZCG_OK) {
      ++rejected;
      continue;
    }
    ++ok;
    if (p.blocks < 1 || p.vec_bytes < 1 || p.vec_bytes > 16 || p.store_bytes < 1 || p.store_bytes > p.vec_bytes ||
        p.log2_group < 0 || p.log2_group > 6 || p.iters < 1 || p.row_splits < 1 || p.row_splits > 4096) {
      std::printf("FAILED: bad plan at iteration %d: row_bytes %lld elem %d n_idx %lld -> variant %d vec %d store %d lg %d "
                  "iters %d blocks %d splits %d\n", it, (long long)row_bytes, elem, (long long)n_idx, p.variant,
                  p.vec_bytes, p.store_bytes, p.log2_group, p.iters, p.blocks, p.row_splits);
      return 1;
    }
  }
  if (zcg_make_plan(400, 4, 0x1000, 0x2000, 10, true, false, nullptr, nullptr) != ZCG_EINVAL) return 1;
  std::printf("plan driver ok: %ld plans, %ld rejected\n", ok, rejected);
  return ok > 50000 && rejected > 20000 ? 0 : 1;
}
