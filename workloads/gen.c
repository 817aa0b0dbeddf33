/*
 * Seeded synthetic input generators for the half-precision GNN aggregation
 * kernels: graphs (uniform-random, R-MAT, log-normal degree), CSR assembly,
 * and fp16 tensors (normal / uniform).  This file holds NO arithmetic of the
 * method under test (no SpMM, SDDMM, softmax or segment planning): it only
 * manufactures inputs, which both the GPU library and the CPU oracle consume.
 *
 * Every random number is a pure function of (seed, counter) -- a splitmix64
 * finaliser over seed + (counter+1)*golden -- so results do not depend on the
 * thread count or on the order of evaluation.
 *
 * Graph conventions (paper section 2.1.1, CSR = offset array + column ids):
 * row i = destination vertex, column j = neighbour; duplicate (i,j) draws are
 * kept as separate non-zeros; within a row columns ascend and equal columns
 * keep generation order.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define GOLDEN 0x9E3779B97F4A7C15ULL

static inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}
static inline uint64_t rnd_u64(uint64_t seed, uint64_t ctr) { return mix64(seed + (ctr + 1) * GOLDEN); }
static inline double rnd_unit(uint64_t seed, uint64_t ctr) { /* [0,1) with 53 bits */
  return (double)(rnd_u64(seed, ctr) >> 11) * (1.0 / 9007199254740992.0);
}
static inline double rnd_normal(uint64_t seed, uint64_t i) { /* Box-Muller, one value per counter pair */
  double u1 = rnd_unit(seed, 2 * i), u2 = rnd_unit(seed, 2 * i + 1);
  return sqrt(-2.0 * log(1.0 - u1)) * cos(6.283185307179586476925286766559 * u2);
}

/* exported for tests of the Python twin of the generator */
uint64_t wl_rnd_u64(uint64_t seed, uint64_t ctr) { return rnd_u64(seed, ctr); }

/* double -> IEEE binary16 bits, round to nearest even (input manufacture only) */
static uint16_t to_half_bits(double v) {
  uint64_t b;
  memcpy(&b, &v, 8);
  uint16_t sign = (uint16_t)((b >> 48) & 0x8000u);
  double a = fabs(v);
  if (a != a) return (uint16_t)(sign | 0x7E00u);
  if (a >= 65520.0) return (uint16_t)(sign | 0x7C00u); /* rounds to inf */
  if (a < 5.9604644775390625e-8 * 0.5) return sign;    /* below half of the least subnormal */
  int e;
  double m = frexp(a, &e); /* a = m * 2^e, m in [0.5,1) */
  int exp = e - 1;         /* a = (2m) * 2^exp, 2m in [1,2) */
  if (exp < -14) {         /* subnormal: units of 2^-24 */
    double q = a * 16777216.0;
    double r = nearbyint(q); /* default rounding mode is nearest-even */
    return (uint16_t)(sign | (uint16_t)r);
  }
  double q = (2.0 * m - 1.0) * 1024.0; /* fraction in units of 2^-10 */
  double r = nearbyint(q);
  uint32_t mant = (uint32_t)r;
  uint32_t bexp = (uint32_t)(exp + 15);
  if (mant == 1024u) { mant = 0; bexp += 1; }
  return (uint16_t)(sign | (bexp << 10) | mant);
}

void wl_fill_normal_f16(uint16_t* out, int64_t n, uint64_t seed, double mean, double sd) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) out[i] = to_half_bits(mean + sd * rnd_normal(seed, (uint64_t)i));
}

void wl_fill_uniform_f16(uint16_t* out, int64_t n, uint64_t seed, double lo, double hi) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) out[i] = to_half_bits(lo + (hi - lo) * rnd_unit(seed, (uint64_t)i));
}

void wl_double_to_f16(const double* in, uint16_t* out, int64_t n) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) out[i] = to_half_bits(in[i]);
}

/* n directed edges with both endpoints uniform in [0,V) */
void wl_edges_uniform(int32_t* row, int32_t* col, int64_t n, int32_t V, uint64_t seed) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    row[i] = (int32_t)(rnd_u64(seed, 2 * (uint64_t)i) % (uint64_t)V);
    col[i] = (int32_t)(rnd_u64(seed, 2 * (uint64_t)i + 1) % (uint64_t)V);
  }
}

/* R-MAT: per level pick a quadrant with probabilities (a,b,c,1-a-b-c); quadrant
 * b sets the column bit, c the row bit, d both.  A draw whose endpoints are not
 * below V is rejected and redrawn with the next attempt counter. */
void wl_edges_rmat(int32_t* row, int32_t* col, int64_t n, int32_t scale, double a, double b, double c,
                   int32_t V, uint64_t seed) {
  const double ab = a + b, abc = a + b + c;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    for (uint64_t attempt = 0;; ++attempt) {
      uint64_t key = mix64(seed ^ mix64((uint64_t)i * 4096ULL + attempt + 0x51ULL));
      uint32_t r = 0, cc = 0;
      for (int32_t l = 0; l < scale; ++l) {
        double u = (double)(rnd_u64(key, (uint64_t)l) >> 11) * (1.0 / 9007199254740992.0);
        r <<= 1;
        cc <<= 1;
        if (u < a) {
        } else if (u < ab) {
          cc |= 1u;
        } else if (u < abc) {
          r |= 1u;
        } else {
          r |= 1u;
          cc |= 1u;
        }
      }
      if ((int64_t)r < V && (int64_t)cc < V) {
        row[i] = (int32_t)r;
        col[i] = (int32_t)cc;
        break;
      }
      if (attempt >= 4095) { /* cannot happen for sane V; keep the loop bounded */
        row[i] = (int32_t)(r % (uint32_t)V);
        col[i] = (int32_t)(cc % (uint32_t)V);
        break;
      }
    }
  }
}

/* seeded Fisher-Yates permutation of 0..V-1 */
void wl_permutation(int32_t* perm, int32_t V, uint64_t seed) {
  for (int32_t i = 0; i < V; ++i) perm[i] = i;
  for (int32_t i = V - 1; i > 0; --i) {
    uint64_t j = rnd_u64(seed, (uint64_t)i) % (uint64_t)(i + 1);
    int32_t t = perm[i];
    perm[i] = perm[j];
    perm[j] = t;
  }
}

void wl_relabel(int32_t* ids, int64_t n, const int32_t* perm) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) ids[i] = perm[ids[i]];
}

/* stable counting sort of (row,col) pairs by key; returns 0 on success */
static int counting_pass(const int32_t* key, const int32_t* ra, const int32_t* ca, int32_t* rb, int32_t* cb,
                         int64_t n, int32_t nkeys) {
  int64_t* cnt = (int64_t*)calloc((size_t)nkeys + 1, sizeof(int64_t));
  if (!cnt) return 1;
  for (int64_t i = 0; i < n; ++i) cnt[key[i] + 1]++;
  for (int32_t k = 0; k < nkeys; ++k) cnt[k + 1] += cnt[k];
  for (int64_t i = 0; i < n; ++i) {
    int64_t p = cnt[key[i]]++;
    rb[p] = ra[i];
    cb[p] = ca[i];
  }
  free(cnt);
  return 0;
}

/* COO (generation order) -> CSR with ascending columns inside a row and ties in
 * generation order.  rowptr has nrows+1 entries, col_out n entries. */
int wl_coo_to_csr(const int32_t* row, const int32_t* col, int64_t n, int32_t nrows, int32_t ncols,
                  int32_t* rowptr, int32_t* col_out) {
  int32_t* r1 = (int32_t*)malloc((size_t)(n > 0 ? n : 1) * 4);
  int32_t* c1 = (int32_t*)malloc((size_t)(n > 0 ? n : 1) * 4);
  int32_t* r2 = (int32_t*)malloc((size_t)(n > 0 ? n : 1) * 4);
  if (!r1 || !c1 || !r2) { free(r1); free(c1); free(r2); return 1; }
  int rc = counting_pass(col, row, col, r1, c1, n, ncols);      /* by column */
  if (!rc) rc = counting_pass(r1, r1, c1, r2, col_out, n, nrows); /* then, stably, by row */
  if (!rc) {
    memset(rowptr, 0, ((size_t)nrows + 1) * 4);
    for (int64_t i = 0; i < n; ++i) rowptr[r2[i] + 1]++;
    for (int32_t k = 0; k < nrows; ++k) rowptr[k + 1] += rowptr[k];
  }
  free(r1); free(c1); free(r2);
  return rc;
}

/* log-normal row degrees: d_i proportional to exp(mu + sigma*n_i), rescaled so the
 * degrees sum to total, clipped to [1, dmax]; the rounding remainder is spread one
 * unit at a time over rows 0,1,2,... (cyclically). */
int wl_lognormal_degrees(int32_t* deg, int32_t V, int64_t total, double mu, double sigma, int32_t dmax,
                         uint64_t seed) {
  double* x = (double*)malloc((size_t)V * 8);
  if (!x) return 1;
  double sum = 0.0;
  for (int32_t i = 0; i < V; ++i) { x[i] = exp(mu + sigma * rnd_normal(seed, (uint64_t)i)); sum += x[i]; }
  int64_t have = 0;
  for (int32_t i = 0; i < V; ++i) {
    double d = floor(x[i] * (double)total / sum);
    if (d < 1.0) d = 1.0;
    if (d > (double)dmax) d = (double)dmax;
    deg[i] = (int32_t)d;
    have += deg[i];
  }
  free(x);
  int32_t i = 0;
  int64_t guard = 0;
  while (have != total && guard < (int64_t)V * 100000) {
    if (have < total && deg[i] < dmax) { deg[i]++; have++; }
    else if (have > total && deg[i] > 1) { deg[i]--; have--; }
    i = (i + 1 == V) ? 0 : i + 1;
    ++guard;
  }
  return have == total ? 0 : 2;
}

static int cmp_i32(const void* a, const void* b) {
  int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x > y) - (x < y);
}

/* for every row, deg_i columns drawn uniformly with replacement from [0,ncols), ascending */
void wl_fill_cols_uniform_sorted(const int32_t* rowptr, int32_t* col, int32_t nrows, int32_t ncols, uint64_t seed) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int32_t r = 0; r < nrows; ++r) {
    int64_t b = rowptr[r], e = rowptr[r + 1];
    for (int64_t k = b; k < e; ++k) col[k] = (int32_t)(rnd_u64(seed, (uint64_t)k) % (uint64_t)ncols);
    qsort(col + b, (size_t)(e - b), 4, cmp_i32);
  }
}

/* symmetric-normalised edge values 1/sqrt(deg_i * deg_j): deg_i = stored entries in
 * row i, deg_j = stored entries in column j (GCN's D^-1/2 A D^-1/2, paper Eq. 2,
 * read for a directed multigraph); value formed in fp64 and rounded once to fp16 */
int wl_symnorm_f16(const int32_t* rowptr, const int32_t* col, int32_t nrows, int32_t ncols, uint16_t* w) {
  int64_t n = rowptr[nrows];
  int32_t* cdeg = (int32_t*)calloc((size_t)ncols, 4);
  if (!cdeg) return 1;
  for (int64_t k = 0; k < n; ++k) cdeg[col[k]]++;
#pragma omp parallel for schedule(dynamic, 1024)
  for (int32_t r = 0; r < nrows; ++r) {
    double dr = (double)(rowptr[r + 1] - rowptr[r]);
    for (int64_t k = rowptr[r]; k < rowptr[r + 1]; ++k) w[k] = to_half_bits(1.0 / sqrt(dr * (double)cdeg[col[k]]));
  }
  free(cdeg);
  return 0;
}
