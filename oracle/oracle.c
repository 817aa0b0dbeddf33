/*
 * CPU oracle for the half-precision GNN aggregation path (HalfGNN, HPDC'25).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, single-threaded, fp64.  It shares no
 * code with the GPU library and must never be called from a product path: only
 * the tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * Every value function is the plain definition from the paper written out in
 * fp64 on the fp16 inputs decoded exactly; nothing is blocked, fused or
 * reordered.  The only "algorithm" here is the segment plan (integer work).
 *
 * Conventions (paper section 2.1.1): CSR = offset array `rowptr` [V+1] plus
 * column ids `col` [E]; row i is the destination vertex whose neighbourhood
 * N(i) is the row; edge-level tensors are edge major [E][H]; vertex-level
 * tensors are row major [V][F] with leading dimension ld; head h owns features
 * [h*D, (h+1)*D), D = F/H.  `eid` (may be NULL) maps CSR position k to the slot
 * of the edge tensors that belongs to that non-zero (used for the transposed
 * graph, whose non-zeros are a permutation of the original ones).
 * fp16 tensors travel as uint16_t bit patterns.
 *
 * Parity pins (tests marked "not gpu"): dense brute force, adjoint identity,
 * degree / row-sum invariants, finite differences, a hand-worked 5-vertex
 * example, exhaustive fp16 codec round trip.  No function here is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- fp16 codec (section 2.2: range 2^-14 .. (2-2^-10)*2^15, i.e. max finite 65504) ---- */
double orc_half_to_double(uint16_t h) {
  int sign = (h >> 15) & 1, e = (h >> 10) & 0x1F, m = h & 0x3FF;
  double v;
  if (e == 0) v = ldexp((double)m, -24);
  else if (e == 31) v = m ? NAN : INFINITY;
  else v = ldexp(1.0 + (double)m / 1024.0, e - 15);
  return sign ? -v : v;
}

/* round-to-nearest-even encode; used only by tests (the oracle's outputs stay fp64) */
uint16_t orc_double_to_half(double v) {
  uint16_t sign = signbit(v) ? 0x8000u : 0;
  double a = fabs(v);
  if (isnan(a)) return sign | 0x7E00u;
  if (a >= 65520.0) return sign | 0x7C00u;
  /* quantum of the binade that holds a */
  int e;
  (void)frexp(a, &e);           /* a in [2^(e-1), 2^e) */
  int qexp = (e - 1 < -14 ? -14 : e - 1) - 10;
  double q = ldexp(1.0, qexp);
  double n = rint(a / q);       /* exact scaling by a power of two, then nearest-even */
  double r = n * q;             /* representable in fp16 (or 65536 -> caught above) */
  if (r == 0.0) return sign;
  int e2;
  double m2 = frexp(r, &e2);    /* r = m2 * 2^e2, m2 in [0.5,1) */
  if (e2 - 1 < -14) return sign | (uint16_t)ldexp(r, 24);
  return sign | (uint16_t)(((e2 - 1 + 15) << 10) | ((int)ldexp(m2 * 2.0 - 1.0, 10)));
}

void orc_decode(const uint16_t* in, double* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = orc_half_to_double(in[i]);
}

/* ---- SpMM: Y <- A_w X (section 2.1.2; SpMMve, and SpMMv when w == NULL) ----
 * Y[i,f] = self_coef * self[i,f] + agg_coef * s_i * sum_{k in row i} w[idx(k), f/D] * cs[col[k]] * X[col[k], f]
 * s_i = 1 (reduce 0, sum), 1/max(deg_i,1) (reduce 1, mean = SpMM + degree-norm,
 * section 5.2.2), times row_scale[i] when given.  cs = col_scale (NULL: 1): with
 * row_scale = col_scale = D^-1/2 this is Eq. 2's D^-1/2 A D^-1/2 X.  self (NULL: no
 * self term) with self_coef = 1 + eps, agg_coef = 1 is Eq. 3 (GIN); reduce = mean with
 * agg_coef = lambda is the half-precision form printed after it.
 * sel == NULL: all V rows, out is [V][F]; otherwise out is [nsel][F] for rows sel[].
 * sabs (may be NULL) receives |self term| + |agg_coef s_i| * sum |w cs x| (natural magnitude). */
void orc_spmm(int32_t V, const int32_t* rowptr, const int32_t* col, const int32_t* eid, const uint16_t* w, int32_t H,
              const uint16_t* X, int64_t ldx, int32_t F, int32_t reduce, const double* row_scale,
              const double* col_scale, const uint16_t* self, int64_t ld_self, double self_coef, double agg_coef,
              const int32_t* sel, int32_t nsel, double* out, double* sabs) {
  int32_t D = F / H;
  int32_t nout = sel ? nsel : V;
  for (int32_t o = 0; o < nout; ++o) {
    int32_t i = sel ? sel[o] : o;
    int32_t deg = rowptr[i + 1] - rowptr[i];
    double s = 1.0;
    if (reduce == 1) s = 1.0 / (double)(deg > 1 ? deg : 1);
    if (row_scale) s *= row_scale[i];
    s *= agg_coef;
    for (int32_t f = 0; f < F; ++f) {
      double acc = 0.0, aabs = 0.0;
      for (int32_t k = rowptr[i]; k < rowptr[i + 1]; ++k) {
        int64_t slot = eid ? eid[k] : k;
        double wk = w ? orc_half_to_double(w[slot * H + f / D]) : 1.0;
        if (col_scale) wk *= col_scale[col[k]];
        double t = wk * orc_half_to_double(X[(int64_t)col[k] * ldx + f]);
        acc += t;
        aabs += fabs(t);
      }
      double selfterm = self ? self_coef * orc_half_to_double(self[(int64_t)i * ld_self + f]) : 0.0;
      out[(int64_t)o * F + f] = selfterm + s * acc;
      if (sabs) sabs[(int64_t)o * F + f] = fabs(selfterm) + fabs(s) * aabs;
    }
  }
}

/* ---- backward SpMM in scatter form: dX <- A_w^T dY (section 2.1.2) ----
 * dX[col[k], f] += w[k, f/D] * dY[i, f] over the non-zeros of A itself; needs no
 * transposed graph, so it pins the transpose builder and its edge-id map. */
void orc_spmm_T_scatter(int32_t V, int32_t ncols, const int32_t* rowptr, const int32_t* col, const uint16_t* w,
                        int32_t H, const uint16_t* dY, int64_t ld, int32_t F, double* dX) {
  int32_t D = F / H;
  memset(dX, 0, (size_t)ncols * F * sizeof(double));
  for (int32_t i = 0; i < V; ++i)
    for (int32_t k = rowptr[i]; k < rowptr[i + 1]; ++k)
      for (int32_t f = 0; f < F; ++f) {
        double wk = w ? orc_half_to_double(w[(int64_t)k * H + f / D]) : 1.0;
        dX[(int64_t)col[k] * F + f] += wk * orc_half_to_double(dY[(int64_t)i * ld + f]);
      }
}

/* ---- transposed graph: CSR of A^T, and eid_T[k'] = CSR position in A of the k'-th
 * non-zero of A^T.  Inside a row of A^T (a column j of A) entries keep the order of
 * their positions in A, i.e. ascending source row, ties in storage order. ---- */
void orc_transpose(int32_t V, int32_t ncols, const int32_t* rowptr, const int32_t* col, int32_t* rowptr_T,
                   int32_t* col_T, int32_t* eid_T) {
  int64_t E = rowptr[V];
  int32_t* next = (int32_t*)calloc((size_t)ncols + 1, 4);
  for (int32_t j = 0; j <= ncols; ++j) rowptr_T[j] = 0;
  for (int64_t k = 0; k < E; ++k) rowptr_T[col[k] + 1]++;
  for (int32_t j = 0; j < ncols; ++j) rowptr_T[j + 1] += rowptr_T[j];
  for (int32_t j = 0; j < ncols; ++j) next[j] = rowptr_T[j];
  for (int32_t i = 0; i < V; ++i)
    for (int32_t k = rowptr[i]; k < rowptr[i + 1]; ++k) {
      int32_t p = next[col[k]]++;
      col_T[p] = i;
      eid_T[p] = k;
    }
  free(next);
}

/* ---- CSR from a COO edge list (section 2.1.1: COO holds one (rowID, colID) pair per non-zero, CSR an offset
 * array and the column ids row by row).  The non-zeros of row r are the edges with rowID r in ascending column
 * order, equal columns (duplicate edges) in the order of the list; eid[p] = the list index of the non-zero at
 * CSR position p.  Written as the definition: count per row, deal the edges out in list order, then a stable
 * insertion sort by column inside every row. ---- */
void orc_coo_to_csr(int64_t E, int32_t V, const int32_t* row, const int32_t* col, int32_t* rowptr, int32_t* col_out,
                    int32_t* eid) {
  int32_t* next = (int32_t*)calloc((size_t)V + 1, 4);
  for (int32_t i = 0; i <= V; ++i) rowptr[i] = 0;
  for (int64_t k = 0; k < E; ++k) rowptr[row[k] + 1]++;
  for (int32_t i = 0; i < V; ++i) rowptr[i + 1] += rowptr[i];
  for (int32_t i = 0; i < V; ++i) next[i] = rowptr[i];
  for (int64_t k = 0; k < E; ++k) {
    int32_t p = next[row[k]]++;
    col_out[p] = col[k];
    eid[p] = (int32_t)k;
  }
  for (int32_t i = 0; i < V; ++i)
    for (int32_t p = rowptr[i] + 1; p < rowptr[i + 1]; ++p) {
      int32_t c = col_out[p], e = eid[p], q = p;
      while (q > rowptr[i] && col_out[q - 1] > c) {
        col_out[q] = col_out[q - 1];
        eid[q] = eid[q - 1];
        --q;
      }
      col_out[q] = c;
      eid[q] = e;
    }
  free(next);
}

/* ---- SDDMM: dW_e <- A (.) (dY X^T) (section 2.1.2), per head ----
 * out[k,h] = sum_{d<D} U[i, h*D+d] * Vt[col[k], h*D+d] for every non-zero k of row i. */
void orc_sddmm_dot(int32_t V, const int32_t* rowptr, const int32_t* col, const int32_t* eid, int32_t H, int32_t D,
                   const uint16_t* U, int64_t ldu, const uint16_t* Vt, int64_t ldv, double* out) {
  for (int32_t i = 0; i < V; ++i)
    for (int32_t k = rowptr[i]; k < rowptr[i + 1]; ++k) {
      int64_t slot = eid ? eid[k] : k;
      for (int32_t h = 0; h < H; ++h) {
        double acc = 0.0;
        for (int32_t d = 0; d < D; ++d)
          acc += orc_half_to_double(U[(int64_t)i * ldu + h * D + d]) *
                 orc_half_to_double(Vt[(int64_t)col[k] * ldv + h * D + d]);
        out[slot * H + h] = acc;
      }
    }
}

/* ---- GAT edge score (the "SDDMM variant" of section 3.1.2 that forms e_ij from the
 * features of both end points and trainable vectors):
 * s = a_l[h].feat[i,h] + a_r[h].feat[col[k],h];  e[k,h] = s > 0 ? s : slope*s ---- */
void orc_gat_score(int32_t V, const int32_t* rowptr, const int32_t* col, int32_t H, int32_t D, const uint16_t* feat,
                   int64_t ld, const uint16_t* a_l, const uint16_t* a_r, double slope, double* e) {
  for (int32_t i = 0; i < V; ++i)
    for (int32_t k = rowptr[i]; k < rowptr[i + 1]; ++k)
      for (int32_t h = 0; h < H; ++h) {
        double s = 0.0;
        for (int32_t d = 0; d < D; ++d)
          s += orc_half_to_double(a_l[h * D + d]) * orc_half_to_double(feat[(int64_t)i * ld + h * D + d]);
        for (int32_t d = 0; d < D; ++d)
          s += orc_half_to_double(a_r[h * D + d]) * orc_half_to_double(feat[(int64_t)col[k] * ld + h * D + d]);
        e[(int64_t)k * H + h] = s > 0.0 ? s : slope * s;
      }
}

/* ---- one GAT aggregation, forward, with nothing rounded in between (sections 2.1.1 and
 * 3.1.2: score from both end points, Eq. 1 over the neighbourhood, then the weighted sum
 * of the neighbours' features).  For row i and head h, over the non-zeros k of the row:
 *   s_k   = a_l[h].U[i,h] + a_r[h].Vt[col k,h];   e_k = s_k > 0 ? s_k : slope*s_k
 *   alpha_k = exp(e_k - m) / sum_k exp(e_k - m),   m = max_k e_k
 *   out[i, h*D+d] = sum_k alpha_k * Vt[col k, h*D+d]
 * lse[i,h] = m + log(sum_k exp(e_k - m)) (what a backward pass needs to rebuild alpha);
 * sabs = sum_k alpha_k * |Vt| (magnitude for tolerances).  An empty row gives out = 0,
 * lse = 0.  U is [V][ldu] (row side), Vt is [ncols][ldv] (column side).
 * Optional (NULL to skip): with mu_k = 1 where s_k > 0 and slope elsewhere (the derivative of
 * the LeakyReLU at s_k),  outm[i, h*D+d] = sum_k alpha_k * mu_k * Vt[col k, h*D+d]  and
 * csum[i,h] = sum_k alpha_k * mu_k: what a forward pass can keep so that the gradient of the
 * row-side score term, sum_k ds_k of orc_gat_backward, needs no second pass over the edges. ---- */
void orc_gat_forward(int32_t V, const int32_t* rowptr, const int32_t* col, int32_t H, int32_t D, const uint16_t* U,
                     int64_t ldu, const uint16_t* Vt, int64_t ldv, const uint16_t* a_l, const uint16_t* a_r,
                     double slope, double* out, double* lse, double* sabs, double* outm, double* csum) {
  int32_t F = H * D;
  for (int32_t i = 0; i < V; ++i) {
    int32_t beg = rowptr[i], end = rowptr[i + 1];
    double* e = (double*)malloc(sizeof(double) * (size_t)(end > beg ? end - beg : 1));
    double* mu = (double*)malloc(sizeof(double) * (size_t)(end > beg ? end - beg : 1));
    for (int32_t h = 0; h < H; ++h) {
      double el = 0.0;
      for (int32_t d = 0; d < D; ++d)
        el += orc_half_to_double(a_l[h * D + d]) * orc_half_to_double(U[(int64_t)i * ldu + h * D + d]);
      double m = -INFINITY;
      for (int32_t k = beg; k < end; ++k) {
        double s = el;
        for (int32_t d = 0; d < D; ++d)
          s += orc_half_to_double(a_r[h * D + d]) * orc_half_to_double(Vt[(int64_t)col[k] * ldv + h * D + d]);
        e[k - beg] = s > 0.0 ? s : slope * s;
        mu[k - beg] = s > 0.0 ? 1.0 : slope;
        m = fmax(m, e[k - beg]);
      }
      double z = 0.0;
      for (int32_t k = beg; k < end; ++k) z += exp(e[k - beg] - m);
      for (int32_t d = 0; d < D; ++d) {
        double acc = 0.0, sa = 0.0, accm = 0.0;
        for (int32_t k = beg; k < end; ++k) {
          double alpha = exp(e[k - beg] - m) / z;
          double x = orc_half_to_double(Vt[(int64_t)col[k] * ldv + h * D + d]);
          acc += alpha * x;
          sa += alpha * fabs(x);
          accm += alpha * mu[k - beg] * x;
        }
        out[(int64_t)i * F + h * D + d] = acc;
        if (sabs) sabs[(int64_t)i * F + h * D + d] = sa;
        if (outm) outm[(int64_t)i * F + h * D + d] = accm;
      }
      if (lse) lse[(int64_t)i * H + h] = end > beg ? m + log(z) : 0.0;
      if (csum) {
        double c = 0.0;
        for (int32_t k = beg; k < end; ++k) c += exp(e[k - beg] - m) / z * mu[k - beg];
        csum[(int64_t)i * H + h] = c;
      }
    }
    free(e);
    free(mu);
  }
}

/* ---- backward of that aggregation.  With L = sum_i <dOut_i, out_i>, and e, alpha as in
 * orc_gat_forward (recomputed here from the inputs):
 *   dalpha_k = <dOut[i,h], Vt[col k,h]>              (SDDMM of section 2.1.2)
 *   t        = sum_k alpha_k * dalpha_k              (= <dOut[i,h], out[i,h]>)
 *   ds_k     = alpha_k * (dalpha_k - t) * (s_k > 0 ? 1 : slope)   (Eq. 1 differentiated, LeakyReLU mask)
 *   d_el[i,h] = sum over row i of ds_k,  d_er[j,h] = sum over the non-zeros with column j of ds_k
 *   dV[j, h*D+d] = sum over the non-zeros with column j of alpha_k * dOut[i, h*D+d]
 * dV is the gradient through the aggregated values only; the gradient through the scores
 * reaches the features as d_el * a_l and d_er * a_r (dense, outside this function). ---- */
void orc_gat_backward(int32_t V, int32_t ncols, const int32_t* rowptr, const int32_t* col, int32_t H, int32_t D,
                      const uint16_t* U, int64_t ldu, const uint16_t* Vt, int64_t ldv, const uint16_t* a_l,
                      const uint16_t* a_r, double slope, const uint16_t* dOut, int64_t lddo, double* dV, double* d_el,
                      double* d_er) {
  int32_t F = H * D;
  memset(dV, 0, sizeof(double) * (size_t)ncols * F);
  memset(d_er, 0, sizeof(double) * (size_t)ncols * H);
  for (int32_t i = 0; i < V; ++i) {
    int32_t beg = rowptr[i], end = rowptr[i + 1];
    int32_t n = end - beg;
    double* s = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    double* alpha = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    for (int32_t h = 0; h < H; ++h) {
      d_el[(int64_t)i * H + h] = 0.0;
      if (n == 0) continue;
      double el = 0.0;
      for (int32_t d = 0; d < D; ++d)
        el += orc_half_to_double(a_l[h * D + d]) * orc_half_to_double(U[(int64_t)i * ldu + h * D + d]);
      double m = -INFINITY;
      for (int32_t k = 0; k < n; ++k) {
        double v = el;
        for (int32_t d = 0; d < D; ++d)
          v += orc_half_to_double(a_r[h * D + d]) * orc_half_to_double(Vt[(int64_t)col[beg + k] * ldv + h * D + d]);
        s[k] = v;
        double e = v > 0.0 ? v : slope * v;
        m = fmax(m, e);
      }
      double z = 0.0;
      for (int32_t k = 0; k < n; ++k) z += exp((s[k] > 0.0 ? s[k] : slope * s[k]) - m);
      double t = 0.0;
      for (int32_t k = 0; k < n; ++k) {
        alpha[k] = exp((s[k] > 0.0 ? s[k] : slope * s[k]) - m) / z;
        double da = 0.0;
        for (int32_t d = 0; d < D; ++d)
          da += orc_half_to_double(dOut[(int64_t)i * lddo + h * D + d]) *
                orc_half_to_double(Vt[(int64_t)col[beg + k] * ldv + h * D + d]);
        t += alpha[k] * da;
      }
      for (int32_t k = 0; k < n; ++k) {
        int64_t j = col[beg + k];
        double da = 0.0;
        for (int32_t d = 0; d < D; ++d)
          da += orc_half_to_double(dOut[(int64_t)i * lddo + h * D + d]) * orc_half_to_double(Vt[j * ldv + h * D + d]);
        double ds = alpha[k] * (da - t) * (s[k] > 0.0 ? 1.0 : slope);
        d_el[(int64_t)i * H + h] += ds;
        d_er[j * H + h] += ds;
        for (int32_t d = 0; d < D; ++d)
          dV[j * F + h * D + d] += alpha[k] * orc_half_to_double(dOut[(int64_t)i * lddo + h * D + d]);
      }
    }
    free(s);
    free(alpha);
  }
}

/* ---- edge softmax, Eq. 1: m_i = max_j e_ij; e'_ij = exp(e_ij - m_i);
 * alpha_ij = e'_ij / sum_j e'_ij, over the neighbourhood (CSR row) of i, per head.
 * Input is fp64 (the caller decodes fp16 scores). ---- */
void orc_edge_softmax(int32_t V, const int32_t* rowptr, int32_t H, const double* e, double* alpha) {
  for (int32_t i = 0; i < V; ++i)
    for (int32_t h = 0; h < H; ++h) {
      if (rowptr[i] == rowptr[i + 1]) continue;
      double m = -INFINITY, z = 0.0;
      for (int32_t k = rowptr[i]; k < rowptr[i + 1]; ++k) m = fmax(m, e[(int64_t)k * H + h]);
      for (int32_t k = rowptr[i]; k < rowptr[i + 1]; ++k) z += exp(e[(int64_t)k * H + h] - m);
      for (int32_t k = rowptr[i]; k < rowptr[i + 1]; ++k)
        alpha[(int64_t)k * H + h] = exp(e[(int64_t)k * H + h] - m) / z;
    }
}

/* ---- backward of Eq. 1 (calculus; the paper does not print it):
 * t_i = sum_j alpha_ij dalpha_ij;  de_ij = alpha_ij (dalpha_ij - t_i);
 * with e given, the LeakyReLU of the score is undone too:
 * ds_ij = de_ij * (e_ij > 0 ? 1 : slope). ---- */
void orc_edge_softmax_bwd(int32_t V, const int32_t* rowptr, int32_t H, const double* alpha, const double* dalpha,
                          const double* e, double slope, double* de) {
  for (int32_t i = 0; i < V; ++i)
    for (int32_t h = 0; h < H; ++h) {
      double t = 0.0;
      for (int32_t k = rowptr[i]; k < rowptr[i + 1]; ++k) t += alpha[(int64_t)k * H + h] * dalpha[(int64_t)k * H + h];
      for (int32_t k = rowptr[i]; k < rowptr[i + 1]; ++k) {
        double g = alpha[(int64_t)k * H + h] * (dalpha[(int64_t)k * H + h] - t);
        if (e) g *= (e[(int64_t)k * H + h] > 0.0 ? 1.0 : slope);
        de[(int64_t)k * H + h] = g;
      }
    }
}

/* ---- sums of an edge tensor over rows (d e_l) and over columns (d e_r) ---- */
void orc_edge_rowsum(int32_t V, const int32_t* rowptr, int32_t H, const double* t, double* out) {
  for (int32_t i = 0; i < V; ++i)
    for (int32_t h = 0; h < H; ++h) {
      double acc = 0.0;
      for (int32_t k = rowptr[i]; k < rowptr[i + 1]; ++k) acc += t[(int64_t)k * H + h];
      out[(int64_t)i * H + h] = acc;
    }
}
void orc_edge_colsum(int32_t V, int32_t ncols, const int32_t* rowptr, const int32_t* col, int32_t H, const double* t,
                     double* out) {
  memset(out, 0, (size_t)ncols * H * sizeof(double));
  for (int32_t i = 0; i < V; ++i)
    for (int32_t k = rowptr[i]; k < rowptr[i + 1]; ++k)
      for (int32_t h = 0; h < H; ++h) out[(int64_t)col[k] * H + h] += t[(int64_t)k * H + h];
}

/* ---- an edge tensor in the edge order of the transposed graph: out[k,h] = t[eid[k],h], eid from
 * orc_transpose (section 2.1.2: the backward SpMM walks A^T, whose k-th non-zero is the
 * eid[k]-th non-zero of A).  Values are copied, not converted. ---- */
void orc_edge_gather(int64_t nnz, const int32_t* eid, int32_t H, const uint16_t* t, uint16_t* out) {
  for (int64_t k = 0; k < nnz; ++k)
    for (int32_t h = 0; h < H; ++h) out[k * H + h] = t[(int64_t)eid[k] * H + h];
}

/* ---- the dense side of a layer (section 3.1.3, Eq. 2: the linear layer turns the previous
 * activation into the dense input of the SpMM; section 6: the input width is projected to the
 * intermediate width by a GeMM).  Y[i,f] = sum_k X[i,k] * W[k,f] (trans = 0, W is K x F) or
 * sum_k X[i,k] * W[f,k] (trans = 1, W is F x K: the product with the transposed weight that
 * carries a gradient back through the layer).  sabs = sum_k |X*W| per output, for tolerances. ---- */
void orc_linear(int64_t n, int32_t K, int32_t F, const uint16_t* X, int64_t ldx, const uint16_t* W, int64_t ldw,
                int32_t trans, double* Y, double* sabs) {
  for (int64_t i = 0; i < n; ++i)
    for (int32_t f = 0; f < F; ++f) {
      double acc = 0.0, sa = 0.0;
      for (int32_t k = 0; k < K; ++k) {
        double w = orc_half_to_double(trans ? W[(int64_t)f * ldw + k] : W[(int64_t)k * ldw + f]);
        double t = orc_half_to_double(X[i * ldx + k]) * w;
        acc += t;
        sa += fabs(t);
      }
      Y[i * F + f] = acc;
      if (sabs) sabs[i * F + f] = sa;
    }
}

/* ---- gradient of the weight of that layer: dW[k,f] = sum_i X[i,k] * dY[i,f] (K x F) ---- */
void orc_linear_wgrad(int64_t n, int32_t K, int32_t F, const uint16_t* X, int64_t ldx, const uint16_t* dY, int64_t ldy,
                      double* dW, double* sabs) {
  for (int32_t k = 0; k < K; ++k)
    for (int32_t f = 0; f < F; ++f) {
      double acc = 0.0, sa = 0.0;
      for (int64_t i = 0; i < n; ++i) {
        double t = orc_half_to_double(X[i * ldx + k]) * orc_half_to_double(dY[i * ldy + f]);
        acc += t;
        sa += fabs(t);
      }
      dW[(int64_t)k * F + f] = acc;
      if (sabs) sabs[(int64_t)k * F + f] = sa;
    }
}

/* ---- gradient of the projected features of a GAT layer and of its attention vectors, from what
 * orc_gat_backward leaves (section 2.1.1: the score is a_l.h_i + a_r.h_j, so it reaches the
 * features through both vectors):
 *   dh[i, h*D+d]  = dV[i, h*D+d] + d_el[i,h] * a_l[h*D+d] + d_er[i,h] * a_r[h*D+d]
 *   da_l[h*D+d]   = sum_i d_el[i,h] * hfeat[i, h*D+d],   da_r likewise with d_er. ---- */
void orc_gat_feature_grad(int32_t V, int32_t H, int32_t D, const uint16_t* dV, int64_t lddv, const uint16_t* d_el,
                          const uint16_t* d_er, const uint16_t* a_l, const uint16_t* a_r, const uint16_t* hfeat,
                          int64_t ldh, double* dh, double* da_l, double* da_r, double* sabs_l, double* sabs_r) {
  int32_t F = H * D;
  for (int32_t f = 0; f < F; ++f) da_l[f] = da_r[f] = sabs_l[f] = sabs_r[f] = 0.0;
  for (int32_t i = 0; i < V; ++i)
    for (int32_t f = 0; f < F; ++f) {
      int32_t h = f / D;
      double gl = orc_half_to_double(d_el[(int64_t)i * H + h]), gr = orc_half_to_double(d_er[(int64_t)i * H + h]);
      double x = orc_half_to_double(hfeat[(int64_t)i * ldh + f]);
      dh[(int64_t)i * F + f] = orc_half_to_double(dV[(int64_t)i * lddv + f]) + gl * orc_half_to_double(a_l[f]) +
                               gr * orc_half_to_double(a_r[f]);
      da_l[f] += gl * x;
      da_r[f] += gr * x;
      sabs_l[f] += fabs(gl * x);
      sabs_r[f] += fabs(gr * x);
    }
}

/* ---- segment plan for the discretized SpMM (section 5.2: edges are dealt out in
 * fixed-size batches in storage order, observation rules 1-3).
 * Segment k owns edges [k*S, min(E,(k+1)*S)).  seg_row_lo/hi[k] = row of its first /
 * last edge.  A non-empty row is "split" when its first and last edge fall in different
 * segments; split rows are listed ascending with the first and last segment they touch.
 * Returns the number of split rows.  Arrays must hold nseg (= ceil(E/S)) entries. ---- */
int32_t orc_segment_plan(int32_t V, const int32_t* rowptr, int32_t S, int32_t* seg_row_lo, int32_t* seg_row_hi,
                         int32_t* split_row, int32_t* split_seg_lo, int32_t* split_seg_hi) {
  int64_t E = rowptr[V];
  int64_t nseg = (E + S - 1) / S;
  int32_t r = 0;
  for (int64_t k = 0; k < nseg; ++k) {
    int64_t e0 = k * (int64_t)S, e1 = (e0 + S < E ? e0 + S : E) - 1;
    while (!(rowptr[r] <= e0 && e0 < rowptr[r + 1])) ++r;
    seg_row_lo[k] = r;
    int32_t q = r;
    while (!(rowptr[q] <= e1 && e1 < rowptr[q + 1])) ++q;
    seg_row_hi[k] = q;
  }
  int32_t ns = 0;
  for (int32_t i = 0; i < V; ++i) {
    if (rowptr[i] == rowptr[i + 1]) continue;
    int32_t a = rowptr[i] / S, b = (rowptr[i + 1] - 1) / S;
    if (a != b) {
      split_row[ns] = i;
      split_seg_lo[ns] = a;
      split_seg_hi[ns] = b;
      ++ns;
    }
  }
  return ns;
}

/* ---- neighbour groups of the vertex-parallel variant (section 5.4): every row is cut,
 * from its first non-zero on, into groups of at most ng neighbours; a group never holds
 * non-zeros of two rows, the last group of a row may be shorter, an empty row has none.
 * Groups are listed in row order: grp_row[j] = row, grp_first[j] = CSR position of the
 * group's first non-zero.  Returns the number of groups; with NULL arrays it only counts. ---- */
int64_t orc_neighbor_groups(int32_t V, const int32_t* rowptr, int32_t ng, int32_t* grp_row, int32_t* grp_first) {
  int64_t n = 0;
  for (int32_t i = 0; i < V; ++i)
    for (int32_t k = rowptr[i]; k < rowptr[i + 1]; k += ng) {
      if (grp_row) grp_row[n] = i;
      if (grp_first) grp_first[n] = k;
      ++n;
    }
  return n;
}

/* ---- demonstration helper (tests only): post-reduction scaling in half precision, the
 * scheme section 3.1.3 says overflows.  mode 0: the running sum itself is kept in fp16
 * (every addition rounds to fp16; large sums stall or reach INF).  mode 1: the sum is
 * formed in wide precision and rounded to fp16 once the reduction is over (INF when it
 * exceeds 65504).  Either way the degree-norm divide comes after, on the fp16 value. ---- */
void orc_spmm_naive_fp16(int32_t V, const int32_t* rowptr, const int32_t* col, const uint16_t* X, int64_t ldx,
                         int32_t F, int32_t reduce, int32_t mode, const int32_t* sel, int32_t nsel, uint16_t* out) {
  int32_t nout = sel ? nsel : V;
  for (int32_t o = 0; o < nout; ++o) {
    int32_t i = sel ? sel[o] : o;
    int32_t deg = rowptr[i + 1] - rowptr[i];
    for (int32_t f = 0; f < F; ++f) {
      double acc = 0.0;
      for (int32_t k = rowptr[i]; k < rowptr[i + 1]; ++k) {
        acc += orc_half_to_double(X[(int64_t)col[k] * ldx + f]);
        if (mode == 0) acc = orc_half_to_double(orc_double_to_half(acc));
      }
      acc = orc_half_to_double(orc_double_to_half(acc));
      if (reduce == 1) acc = acc / (double)(deg > 1 ? deg : 1);
      out[(int64_t)o * F + f] = orc_double_to_half(acc);
    }
  }
}

/* ---- discretized reduction scaling as the paper states it (section 5.2.2): reduce a
 * batch of at most S neighbours, scale that partial, round it to fp16 (the stored
 * partial), move to the next batch; the per-row result is the sum of its partials.
 * by_row = 0: batches are the plan's segments (edge ranges [k*S,(k+1)*S) cut at row
 * boundaries), the edge-parallel form.  by_row = 1: batches are the row's own neighbour
 * groups, S neighbours each counted from the start of the row (section 5.4: the
 * vertex-parallel form never splits a row inside a batch).
 * Returns through out the fp64 sum of the fp16-rounded scaled partials and through
 * maxpart the largest |partial| met before rounding (overflow evidence). ---- */
void orc_spmm_discretized(int32_t V, const int32_t* rowptr, const int32_t* col, const int32_t* eid, const uint16_t* w,
                          int32_t H, const uint16_t* X, int64_t ldx, int32_t F, int32_t reduce,
                          const double* row_scale, int32_t S, int32_t by_row, const int32_t* sel, int32_t nsel,
                          double* out, double* maxpart) {
  int32_t D = F / H;
  int32_t nout = sel ? nsel : V;
  double mp = 0.0;
  for (int32_t o = 0; o < nout; ++o) {
    int32_t i = sel ? sel[o] : o;
    int32_t deg = rowptr[i + 1] - rowptr[i];
    double s = 1.0;
    if (reduce == 1) s = 1.0 / (double)(deg > 1 ? deg : 1);
    if (row_scale) s *= row_scale[i];
    for (int32_t f = 0; f < F; ++f) {
      double total = 0.0;
      int32_t k = rowptr[i];
      while (k < rowptr[i + 1]) {
        int32_t kend = by_row ? rowptr[i] + ((k - rowptr[i]) / S + 1) * S : (k / S + 1) * S;
        if (kend > rowptr[i + 1]) kend = rowptr[i + 1];
        double part = 0.0;
        for (; k < kend; ++k) {
          int64_t slot = eid ? eid[k] : k;
          double wk = w ? orc_half_to_double(w[slot * H + f / D]) : 1.0;
          part += wk * orc_half_to_double(X[(int64_t)col[k] * ldx + f]);
        }
        part *= s;
        if (fabs(part) > mp) mp = fabs(part);
        total += orc_half_to_double(orc_double_to_half(part));
      }
      out[(int64_t)o * F + f] = total;
    }
  }
  if (maxpart) *maxpart = mp;
}
