/*
 * Seeded synthetic inputs for the sparse feature gather: feature-table fill,
 * uniform index lists, an implicit power-law (Chung-Lu style) graph and a
 * k-hop uniform neighbor sampler that emits deduplicated int64 node-ID lists.
 *
 * Nothing here gathers rows: this file only produces the inputs that both the
 * CPU oracle and the GPU library are fed (the paper's flow: sampler picks seed
 * nodes, collects fixed fan-out neighbors per hop, and hands the combined ID
 * list to the gather; Sections 2.2 and 3.3).
 *
 * Every generator is counter based (splitmix64 finaliser keyed on position),
 * so values do not depend on thread count or call order and any single value
 * can be recomputed on its own.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ZCGW_GOLDEN 0x9E3779B97F4A7C15ULL

static inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}

/* value of the counter stream `seed` at position `pos` */
static inline uint64_t stream_at(uint64_t seed, uint64_t pos) {
  return mix64(seed + (pos + 1) * ZCGW_GOLDEN);
}

static inline uint64_t key2(uint64_t seed, uint64_t a, uint64_t b) {
  return mix64(mix64(seed ^ mix64(a + ZCGW_GOLDEN)) + b * ZCGW_GOLDEN + 0x632BE59BD9B4E019ULL);
}

/* unbiased-enough range reduction: floor(z * n / 2^64) */
static inline uint64_t scale_to(uint64_t z, uint64_t n) {
  return (uint64_t)(((unsigned __int128)z * n) >> 64);
}

/* exact float -> IEEE half for values (k-1024)/1024, k in [0,2048) */
static inline uint16_t half_from_k11(uint32_t k) {
  int32_t m = (int32_t)k - 1024; /* value = m * 2^-10, |m| <= 1024 */
  if (m == 0) return 0;
  uint16_t sign = 0;
  if (m < 0) { sign = 0x8000; m = -m; }
  int e = 0; /* m = 1.xxx * 2^e */
  while ((m >> (e + 1)) != 0) ++e;
  /* value = m * 2^-10 = 1.xxx * 2^(e-10); half exponent bias 15 */
  uint32_t frac = ((uint32_t)m << (10 - e)) & 0x3FF;
  return (uint16_t)(sign | (uint32_t)((e - 10 + 15) << 10) | frac);
}

/*
 * Fill a row-major [n_rows x dim] table in place.
 *   elem_bytes 4: fp32, 2: fp16, 1: int8, 8: fp64.
 *   mode 0: uniform on [-1,1): fp32 takes the top 24 bits k of the stream value
 *           and stores (k - 2^23) * 2^-23; fp16 takes the top 11 bits k and
 *           stores (k - 2^10) * 2^-10. Both are exactly representable.
 *   mode 1: raw bit patterns (low 32 / 16 bits of the stream value), which
 *           include NaNs, infinities, denormals and negative zero.
 * Element at flat position p = r*dim + c depends only on (seed, p).
 * Returns 0, or -1 on bad arguments.
 */
int zcgw_fill_table(void* dst, int64_t n_rows, int64_t dim, int elem_bytes, uint64_t seed,
                    int mode, int n_threads) {
  if (!dst || n_rows < 0 || dim <= 0 ||
      (elem_bytes != 1 && elem_bytes != 2 && elem_bytes != 4 && elem_bytes != 8) ||
      (mode != 0 && mode != 1))
    return -1;
  const int64_t total = n_rows * dim;
  if (n_threads < 1) n_threads = 1;
  if (elem_bytes == 4) {
    uint32_t* p = (uint32_t*)dst;
#pragma omp parallel for schedule(static) num_threads(n_threads)
    for (int64_t i = 0; i < total; ++i) {
      uint64_t z = stream_at(seed, (uint64_t)i);
      if (mode == 0) {
        float f = (float)((int32_t)(z >> 40) - (1 << 23)) * 0x1p-23f;
        memcpy(&p[i], &f, 4);
      } else {
        p[i] = (uint32_t)z;
      }
    }
  } else if (elem_bytes == 2) {
    uint16_t* p = (uint16_t*)dst;
#pragma omp parallel for schedule(static) num_threads(n_threads)
    for (int64_t i = 0; i < total; ++i) {
      uint64_t z = stream_at(seed, (uint64_t)i);
      p[i] = (mode == 0) ? half_from_k11((uint32_t)(z >> 53)) : (uint16_t)z;
    }
  } else if (elem_bytes == 1) {
    /* mode 0: int8 uniform on [-128, 127] from the top 8 bits; mode 1: the low byte */
    uint8_t* p = (uint8_t*)dst;
#pragma omp parallel for schedule(static) num_threads(n_threads)
    for (int64_t i = 0; i < total; ++i) {
      uint64_t z = stream_at(seed, (uint64_t)i);
      p[i] = (mode == 0) ? (uint8_t)(z >> 56) : (uint8_t)z;
    }
  } else {
    /* mode 0: fp64 (k - 2^52) * 2^-52 from the top 53 bits k; mode 1: all 64 bits */
    uint64_t* p = (uint64_t*)dst;
#pragma omp parallel for schedule(static) num_threads(n_threads)
    for (int64_t i = 0; i < total; ++i) {
      uint64_t z = stream_at(seed, (uint64_t)i);
      if (mode == 0) {
        double f = (double)((int64_t)(z >> 11) - ((int64_t)1 << 52)) * 0x1p-52;
        memcpy(&p[i], &f, 8);
      } else {
        p[i] = z;
      }
    }
  }
  return 0;
}

/* idx[i] uniform in [0, n_rows), duplicates kept; depends only on (seed, i). */
int zcgw_uniform_indices(int64_t* idx, int64_t n_idx, int64_t n_rows, uint64_t seed,
                         int n_threads) {
  if ((!idx && n_idx > 0) || n_idx < 0 || n_rows <= 0) return -1;
  if (n_threads < 1) n_threads = 1;
#pragma omp parallel for schedule(static) num_threads(n_threads)
  for (int64_t i = 0; i < n_idx; ++i)
    idx[i] = (int64_t)scale_to(stream_at(seed, (uint64_t)i), (uint64_t)n_rows);
  return 0;
}

/* ------------------------------------------------------------------------
 * Implicit power-law graph.
 *
 * Nodes are ranked j = 0..n-1 with expected degree w(j) = c * (j + j0)^(-a),
 * a = 1/(gamma-1). c and j0 are solved so that the mean of w is avg_deg and
 * w(0) = min(sqrt(n*avg_deg), n/4). Rank j carries node label
 * (A*j + B) mod n with gcd(A, n) = 1, so hubs are scattered over the table.
 *
 * The neighbor list of node u is never stored: entry `pos` (0 <= pos < deg(u))
 * is a draw, proportional to w, from the counter stream keyed (seed, u, pos):
 * the inverse CDF of the continuous density (x + j0)^(-a) on [0, n), floored
 * to a rank. Lists are fixed per node (the same for every minibatch), directed
 * (u->v does not imply v->u) and may repeat an entry; the marginal frequency
 * with which a node is named as a neighbor is proportional to its weight, as
 * in a materialised Chung-Lu graph.
 * ------------------------------------------------------------------------ */
typedef struct zcgw_graph {
  int64_t n;
  double avg_deg, gamma, a, one_m_a, inv_one_m_a;
  double j0, c, lo, span; /* lo = j0^(1-a); span = (n+j0)^(1-a) - lo */
  uint64_t seed, A, B, Ainv;
  uint64_t* seen; /* n-bit scratch bitmap for dedup, all zero between calls */
} zcgw_graph;

static uint64_t gcd_u64(uint64_t x, uint64_t y) {
  while (y) { uint64_t t = x % y; x = y; y = t; }
  return x;
}

static uint64_t modinv_u64(uint64_t a, uint64_t n) {
  /* extended Euclid on signed 128-bit */
  __int128 t = 0, nt = 1, r = (__int128)n, nr = (__int128)(a % n);
  while (nr != 0) {
    __int128 q = r / nr, tmp;
    tmp = t - q * nt; t = nt; nt = tmp;
    tmp = r - q * nr; r = nr; nr = tmp;
  }
  if (t < 0) t += (__int128)n;
  return (uint64_t)t;
}

static double mean_for_j0(double j0, double n, double a, double wmax) {
  double oma = 1.0 - a;
  return wmax * pow(j0, a) * (pow(n + j0, oma) - pow(j0, oma)) / (oma * n);
}

zcgw_graph* zcgw_graph_create(int64_t n, double avg_deg, double gamma, uint64_t seed) {
  if (n < 4 || avg_deg < 1.0 || gamma <= 2.0 || gamma > 4.0) return NULL;
  zcgw_graph* g = (zcgw_graph*)calloc(1, sizeof(zcgw_graph));
  if (!g) return NULL;
  g->n = n; g->avg_deg = avg_deg; g->gamma = gamma; g->seed = seed;
  g->a = 1.0 / (gamma - 1.0);
  g->one_m_a = 1.0 - g->a;
  g->inv_one_m_a = 1.0 / g->one_m_a;
  double wmax = sqrt((double)n * avg_deg);
  if (wmax > (double)n / 4.0) wmax = (double)n / 4.0;
  if (wmax < avg_deg) wmax = avg_deg;
  /* bisection on log(j0): mean_for_j0 rises from 0 to wmax */
  double lo = log(1e-9), hi = log((double)n * 1e6);
  for (int it = 0; it < 200; ++it) {
    double mid = 0.5 * (lo + hi);
    if (mean_for_j0(exp(mid), (double)n, g->a, wmax) < avg_deg) lo = mid; else hi = mid;
  }
  g->j0 = exp(0.5 * (lo + hi));
  g->c = wmax * pow(g->j0, g->a);
  g->lo = pow(g->j0, g->one_m_a);
  g->span = pow((double)n + g->j0, g->one_m_a) - g->lo;
  uint64_t A = (mix64(seed ^ 0xA5A5A5A5DEADBEEFULL) % (uint64_t)n) | 1ULL;
  while (A < 2 || gcd_u64(A, (uint64_t)n) != 1) { A += 2; if (A >= (uint64_t)n) A = 3; }
  g->A = A;
  g->B = mix64(seed ^ 0x0123456789ABCDEFULL) % (uint64_t)n;
  g->Ainv = modinv_u64(A, (uint64_t)n);
  g->seen = (uint64_t*)calloc((size_t)((n + 63) / 64), sizeof(uint64_t));
  if (!g->seen) { free(g); return NULL; }
  return g;
}

void zcgw_graph_destroy(zcgw_graph* g) {
  if (!g) return;
  free(g->seen);
  free(g);
}

static inline int64_t label_of_rank(const zcgw_graph* g, int64_t j) {
  return (int64_t)(((unsigned __int128)g->A * (uint64_t)j + g->B) % (uint64_t)g->n);
}

static inline int64_t rank_of_label(const zcgw_graph* g, int64_t u) {
  uint64_t d = ((uint64_t)u + (uint64_t)g->n - g->B) % (uint64_t)g->n;
  return (int64_t)(((unsigned __int128)g->Ainv * d) % (uint64_t)g->n);
}

int64_t zcgw_graph_degree(const zcgw_graph* g, int64_t u) {
  if (!g || u < 0 || u >= g->n) return -1;
  double w = g->c * pow((double)rank_of_label(g, u) + g->j0, -g->a);
  int64_t d = (int64_t)llround(w);
  if (d < 1) d = 1;
  if (d > g->n - 1) d = g->n - 1;
  return d;
}

static inline int64_t draw_rank(const zcgw_graph* g, uint64_t z) {
  double u01 = (double)(z >> 11) * 0x1p-53; /* [0,1) */
  double x = pow(g->lo + u01 * g->span, g->inv_one_m_a) - g->j0;
  int64_t j = (int64_t)floor(x);
  if (j < 0) j = 0;
  if (j >= g->n) j = g->n - 1;
  return j;
}

/* entry `pos` of node u's neighbor list; never equal to u */
int64_t zcgw_graph_neighbor(const zcgw_graph* g, int64_t u, int64_t pos) {
  if (!g || u < 0 || u >= g->n || pos < 0) return -1;
  uint64_t k = key2(g->seed, (uint64_t)u, (uint64_t)pos);
  for (int salt = 0; salt < 4; ++salt) {
    int64_t v = label_of_rank(g, draw_rank(g, mix64(k + (uint64_t)salt * ZCGW_GOLDEN)));
    if (v != u) return v;
  }
  return (u + 1) % g->n;
}

void zcgw_graph_params(const zcgw_graph* g, double* out6) {
  out6[0] = g->j0; out6[1] = g->c; out6[2] = g->a;
  out6[3] = (double)g->A; out6[4] = (double)g->B; out6[5] = (double)g->Ainv;
}

static inline int test_and_set(uint64_t* bm, int64_t v) {
  uint64_t bit = 1ULL << (v & 63);
  uint64_t* w = &bm[v >> 6];
  int was = (*w & bit) != 0;
  *w |= bit;
  return was;
}

/*
 * One minibatch: n_seeds distinct uniform seed nodes, then for hop h = 0..n_hops-1
 * every node gathered so far (seeds and all earlier hops) samples
 * min(fanout[h], deg) distinct positions of its neighbor list, uniformly and
 * without replacement (Floyd's method on positions); neighbors not seen before
 * are appended. Output order is first occurrence: seeds, new hop-1 nodes in
 * discovery order, new hop-2 nodes, ... `hop_end[h]` (n_hops+1 entries) gets
 * the list length after the seeds and after each hop.
 * Returns the list length, -1 on bad arguments, -2 if `cap` is too small.
 */
int64_t zcgw_sample_minibatch(zcgw_graph* g, int64_t n_seeds, const int32_t* fanout, int n_hops,
                              uint64_t batch_id, int64_t* out, int64_t cap, int64_t* hop_end) {
  if (!g || !out || !fanout || n_seeds < 1 || n_seeds > g->n || n_hops < 0 || n_hops > 8 ||
      cap < n_seeds)
    return -1;
  for (int h = 0; h < n_hops; ++h)
    if (fanout[h] < 1 || fanout[h] > 64) return -1;
  const uint64_t bkey = mix64(g->seed ^ mix64(batch_id * ZCGW_GOLDEN + 0x5851F42D4C957F2DULL));
  int64_t len = 0, rc = 0;
  uint64_t ctr = 0;
  while (len < n_seeds) {
    int64_t s = (int64_t)scale_to(stream_at(bkey, ctr++), (uint64_t)g->n);
    if (!test_and_set(g->seen, s)) out[len++] = s;
  }
  if (hop_end) hop_end[0] = len;
  for (int h = 0; h < n_hops && rc == 0; ++h) {
    const int64_t frontier_end = len;
    const int f = fanout[h];
    for (int64_t q = 0; q < frontier_end && rc == 0; ++q) {
      const int64_t u = out[q];
      const int64_t deg = zcgw_graph_degree(g, u);
      int64_t pos[64];
      int take;
      if (deg <= f) {
        take = (int)deg;
        for (int t = 0; t < take; ++t) pos[t] = t;
      } else {
        take = 0;
        const uint64_t nkey = key2(bkey, (uint64_t)u, (uint64_t)h);
        for (int64_t t = deg - f; t < deg; ++t) {
          int64_t r = (int64_t)scale_to(stream_at(nkey, (uint64_t)(t - (deg - f))), (uint64_t)(t + 1));
          int dup = 0;
          for (int k = 0; k < take; ++k) if (pos[k] == r) { dup = 1; break; }
          pos[take++] = dup ? t : r;
        }
      }
      for (int t = 0; t < take; ++t) {
        int64_t v = zcgw_graph_neighbor(g, u, pos[t]);
        if (!test_and_set(g->seen, v)) {
          if (len >= cap) {
            g->seen[v >> 6] &= ~(1ULL << (v & 63));
            rc = -2;
            break;
          }
          out[len++] = v;
        }
      }
    }
    if (hop_end) hop_end[h + 1] = len;
  }
  for (int64_t i = 0; i < len; ++i) g->seen[out[i] >> 6] = 0; /* restore all-zero scratch */
  return rc ? rc : len;
}
