/*
 * CPU oracle for the sparse feature gather. TEST INFRASTRUCTURE ONLY: tests,
 * the smoke check and the benchmark's cpu_baseline leg may call it; the
 * product library never does, and the two share no code.
 *
 * What it computes is the definition the paper's indexing kernel implements
 * (Section 3.2.1, Listing 2: element `o` of output row `i` is element `o` of
 * source row idx_list[i]; the circular-shift stage only changes which thread
 * copies which element, never the result):
 *
 *     out[i, c] = table[idx[i], c]      0 <= i < n_idx, 0 <= c < dim
 *
 * as a byte copy of row_bytes = dim * elem_size bytes per row. No arithmetic
 * touches the payload, so the result is exact for every bit pattern. Output
 * rows follow the order of the index list; duplicate indices give duplicate
 * rows. Indices are int64 and every offset is 64-bit (the listing's `int`
 * offsets overflow on the paper's own largest table; reading: treat the
 * listing as simplified).
 *
 * Parity status: pinned (brute force on tiny inputs, invariants, a closed-form
 * table, numpy.take as an outside opinion) in tests/test_oracle_pins.py.
 */
#include <stddef.h>
#include <stdint.h>

#define ZCG_ORACLE_OK 0
#define ZCG_ORACLE_EINVAL (-1)
#define ZCG_ORACLE_ERANGE (-2)

/*
 * table     : [n_rows x row_bytes] row-major, host memory
 * idx       : n_idx int64 row numbers, each in [0, n_rows)
 * out       : [n_idx x row_bytes], host memory, must not overlap table
 * n_threads : 1 = the single-thread baseline; >1 = static blocks of output rows
 * bad_pos   : if non-NULL receives the position of the first out-of-range index
 * Returns 0; -1 on bad arguments; -2 if any index is out of range (out is then
 * left untouched).
 */
int zcg_oracle_gather(const void* table, int64_t n_rows, int64_t row_bytes, const int64_t* idx,
                      int64_t n_idx, void* out, int n_threads, int64_t* bad_pos) {
  if (n_rows < 0 || row_bytes <= 0 || n_idx < 0) return ZCG_ORACLE_EINVAL;
  if (n_idx > 0 && (!table || !idx || !out)) return ZCG_ORACLE_EINVAL;
  for (int64_t i = 0; i < n_idx; ++i) {
    if (idx[i] < 0 || idx[i] >= n_rows) {
      if (bad_pos) *bad_pos = i;
      return ZCG_ORACLE_ERANGE;
    }
  }
  const unsigned char* src = (const unsigned char*)table;
  unsigned char* dst = (unsigned char*)out;
  if (n_threads < 1) n_threads = 1;
#pragma omp parallel for schedule(static) num_threads(n_threads)
  for (int64_t i = 0; i < n_idx; ++i) {
    const unsigned char* s = src + idx[i] * row_bytes;
    unsigned char* d = dst + i * row_bytes;
    for (int64_t b = 0; b < row_bytes; ++b) d[b] = s[b];
  }
  return ZCG_ORACLE_OK;
}
