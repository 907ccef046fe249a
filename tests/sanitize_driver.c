/* Small driver that exercises the C oracle and the input generators under
 * AddressSanitizer / UBSan (host code only). Built and run by test_sanitizers.py. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int zcg_oracle_gather(const void*, int64_t, int64_t, const int64_t*, int64_t, void*, int, int64_t*);
int zcgw_fill_table(void*, int64_t, int64_t, int, uint64_t, int, int);
int zcgw_uniform_indices(int64_t*, int64_t, int64_t, uint64_t, int);
typedef struct zcgw_graph zcgw_graph;
zcgw_graph* zcgw_graph_create(int64_t, double, double, uint64_t);
void zcgw_graph_destroy(zcgw_graph*);
int64_t zcgw_graph_degree(const zcgw_graph*, int64_t);
int64_t zcgw_sample_minibatch(zcgw_graph*, int64_t, const int32_t*, int, uint64_t, int64_t*, int64_t,
                              int64_t*);

#define CHECK(c) do { if (!(c)) { printf("FAILED: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

int main(void) {
  const int64_t n_rows = 1009, dim = 37, n_idx = 5003;
  for (int elem = 2; elem <= 4; elem += 2) {
    const int64_t rb = dim * elem;
    unsigned char* table = malloc((size_t)(n_rows * rb));
    unsigned char* out = malloc((size_t)(n_idx * rb));
    int64_t* idx = malloc((size_t)n_idx * 8);
    CHECK(table && out && idx);
    CHECK(zcgw_fill_table(table, n_rows, dim, elem, 7, 0, 3) == 0);
    CHECK(zcgw_fill_table(table, n_rows, dim, elem, 7, 1, 2) == 0);
    CHECK(zcgw_uniform_indices(idx, n_idx, n_rows, 3, 4) == 0);
    int64_t bad = -1;
    for (int nt = 1; nt <= 4; nt += 3) {
      CHECK(zcg_oracle_gather(table, n_rows, rb, idx, n_idx, out, nt, &bad) == 0);
      for (int64_t i = 0; i < n_idx; i += 97)
        CHECK(memcmp(out + i * rb, table + idx[i] * rb, (size_t)rb) == 0);
    }
    idx[17] = n_rows;
    CHECK(zcg_oracle_gather(table, n_rows, rb, idx, n_idx, out, 1, &bad) == -2 && bad == 17);
    CHECK(zcg_oracle_gather(table, n_rows, rb, idx, 0, out, 1, &bad) == 0);
    free(table); free(out); free(idx);
  }
  zcgw_graph* g = zcgw_graph_create(20011, 25.0, 2.1, 99);
  CHECK(g);
  const int32_t fan[3] = {10, 5, 3};
  int64_t cap = 64 * 11 * 6 * 4;
  int64_t* list = malloc((size_t)cap * 8);
  int64_t hop_end[4];
  for (uint64_t b = 0; b < 3; ++b) {
    int64_t n = zcgw_sample_minibatch(g, 64, fan, 3, b, list, cap, hop_end);
    CHECK(n >= 64 && n <= cap && hop_end[3] == n);
    for (int64_t i = 0; i < n; ++i) CHECK(list[i] >= 0 && list[i] < 20011);
  }
  CHECK(zcgw_sample_minibatch(g, 64, fan, 3, 0, list, 70, hop_end) == -2);  /* list too small */
  CHECK(zcgw_sample_minibatch(g, 64, fan, 3, 1, list, cap, hop_end) >= 64); /* scratch still clean */
  CHECK(zcgw_graph_degree(g, 20011) == -1);
  free(list);
  zcgw_graph_destroy(g);
  printf("sanitize driver ok\n");
  return 0;
}
