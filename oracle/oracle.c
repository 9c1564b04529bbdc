/*
 * CPU oracle for batched IVF-PQ search and flat exact k-NN.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, obviously-correct
 * statement of what the search path computes, written from the paper
 * ("The Faiss Library", arXiv 2401.08281).  It shares no code with the HIP
 * library; only tests, the smoke check and the bench's cpu_baseline leg may
 * call it.  Nothing here is blocked, fused or reordered beyond what the cited
 * definition states.
 *
 * Conventions
 *   - vectors are rows of row-major fp32 matrices (Sec. 3 Table 1 "notations", App. A.1)
 *   - metric 0 = L2, returned SQUARED (App. A.6 "Faiss metric types": METRIC_L2 is the
 *     squared Euclidean distance); metric 1 = inner product, larger is better
 *     (Sec. 3 "Distance measures": argmin becomes argmax)
 *   - ids are int64, -1 marks an empty result slot (Sec. 6.1: the sign bit is
 *     reserved for invalid ids)
 *   - ties: the smaller index / id wins (the paper leaves ties open)
 *
 * Two arithmetics are used, on purpose:
 *   canon  : fp32, one chain per (vector, candidate) pair in index order,
 *            diff = a-b rounded to fp32, acc = fmaf(diff, diff, acc)
 *            (IP: acc = fmaf(a, b, acc)).  IEEE-defined, so any machine with a
 *            correctly rounded fma reproduces it bit for bit.  It takes every
 *            DECISION that must be bit-exact: list assignment, probe order,
 *            PQ code.
 *   report : fp64 accumulation rounded once to fp32.  It produces every
 *            DISTANCE that is returned and orders the returned neighbours.
 *
 * Build: gcc -O2 -ffp-contract=off -mfma -fopenmp -shared -fPIC oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define OR_METRIC_L2 0
#define OR_METRIC_IP 1

/* ---- canonical fp32 distances ------------------------------------------ */

float or_canon_l2(const float *a, const float *b, int d) {
  float acc = 0.0f;
  for (int t = 0; t < d; ++t) {
    float diff = a[t] - b[t];
    acc = fmaf(diff, diff, acc);
  }
  return acc;
}

float or_canon_ip(const float *a, const float *b, int d) {
  float acc = 0.0f;
  for (int t = 0; t < d; ++t) acc = fmaf(a[t], b[t], acc);
  return acc;
}

static float canon(const float *a, const float *b, int d, int metric) {
  return metric == OR_METRIC_L2 ? or_canon_l2(a, b, d) : or_canon_ip(a, b, d);
}

/* ---- reported fp64 distances ------------------------------------------- */

static float report_dist(const float *q, const double *xd, int d, int metric) {
  double acc = 0.0;
  if (metric == OR_METRIC_L2) {
    for (int t = 0; t < d; ++t) {
      double diff = (double)q[t] - xd[t];
      acc += diff * diff;
    }
  } else {
    for (int t = 0; t < d; ++t) acc += (double)q[t] * xd[t];
  }
  return (float)acc;
}

/* ---- k best of a stream: sorted insertion, best first ------------------- */

/* "a is strictly better than b": smaller distance for L2, larger score for
 * IP; equal values -> smaller id first (Eq. 2: argsort by increasing
 * distance; tie rule is ours). */
static int better(float da, int64_t ia, float db, int64_t ib, int metric) {
  if (da != db) return metric == OR_METRIC_L2 ? (da < db) : (da > db);
  return ia < ib;
}

typedef struct {
  int k, n, metric;
  float *D;
  int64_t *I;
} topk_t;

static void topk_init(topk_t *h, int k, int metric, float *D, int64_t *I) {
  h->k = k; h->n = 0; h->metric = metric; h->D = D; h->I = I;
  for (int j = 0; j < k; ++j) {
    D[j] = metric == OR_METRIC_L2 ? INFINITY : -INFINITY;
    I[j] = -1;
  }
}

static void topk_push(topk_t *h, float dist, int64_t id) {
  if (h->n == h->k && !better(dist, id, h->D[h->k - 1], h->I[h->k - 1], h->metric)) return;
  int j = h->n < h->k ? h->n++ : h->k - 1;
  while (j > 0 && better(dist, id, h->D[j - 1], h->I[j - 1], h->metric)) {
    h->D[j] = h->D[j - 1];
    h->I[j] = h->I[j - 1];
    --j;
  }
  h->D[j] = dist;
  h->I[j] = id;
}

/* ---- O1: flat exact search (Eq. 1, Eq. 2) ------------------------------ */

void or_flat_search(const float *x, int64_t nb, const float *q, int64_t nq, int d, int metric,
                    int k, float *D, int64_t *I) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t a = 0; a < nq; ++a) {
    const float *qa = q + a * d;
    topk_t h;
    topk_init(&h, k, metric, D + a * k, I + a * k);
    for (int64_t i = 0; i < nb; ++i) {
      const float *xi = x + i * d;
      double acc = 0.0;
      if (metric == OR_METRIC_L2) {
        for (int t = 0; t < d; ++t) {
          double diff = (double)qa[t] - (double)xi[t];
          acc += diff * diff;
        }
      } else {
        for (int t = 0; t < d; ++t) acc += (double)qa[t] * (double)xi[t];
      }
      topk_push(&h, (float)acc, i);
    }
  }
}

/* ---- Refinement of a shortlist (Sec. 3.5 "Refining") ------------------
 * A first, approximate search returns kc candidate ids per query; the accurate
 * second stage computes the exact distance (the definition of Eq. 1, as in
 * or_flat_search: fp64 sum, rounded once) between the query and each candidate
 * vector and keeps the k best, best first, ties to the smaller id.  Entries of
 * the shortlist that are not row numbers of x (the -1 of an empty slot) are
 * skipped; every other entry is taken as given. */
void or_refine(const float *x, int64_t nb, const float *q, int64_t nq, int d, int metric,
               const int64_t *cand, int kc, int k, float *D, int64_t *I) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t a = 0; a < nq; ++a) {
    const float *qa = q + a * d;
    topk_t h;
    topk_init(&h, k, metric, D + a * k, I + a * k);
    for (int j = 0; j < kc; ++j) {
      const int64_t i = cand[a * kc + j];
      if (i < 0 || i >= nb) continue;
      const float *xi = x + i * d;
      double acc = 0.0;
      if (metric == OR_METRIC_L2) {
        for (int t = 0; t < d; ++t) {
          double diff = (double)qa[t] - (double)xi[t];
          acc += diff * diff;
        }
      } else {
        for (int t = 0; t < d; ++t) acc += (double)qa[t] * (double)xi[t];
      }
      topk_push(&h, (float)acc, i);
    }
  }
}

/* ---- O2: list assignment; O6: probe selection (Sec. 5.1) --------------- */

/* list(x) = the best centroid under the index metric by canon arithmetic,
 * ties to the smaller list number. */
void or_assign(const float *x, int64_t n, const float *centroids, int nlist, int d, int metric,
               int32_t *list_of) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    int best = 0;
    float bd = canon(x + i * d, centroids, d, metric);
    for (int l = 1; l < nlist; ++l) {
      float dl = canon(x + i * d, centroids + (int64_t)l * d, d, metric);
      if (better(dl, l, bd, best, metric)) { bd = dl; best = l; }
    }
    list_of[i] = best;
  }
}

/* probes(q) = the nprobe best lists by canon arithmetic, best first.
 * cdist receives the canon value of each probe. nprobe <= nlist. */
void or_coarse_probe(const float *q, int64_t nq, const float *centroids, int nlist, int d,
                     int metric, int nprobe, int32_t *probes, float *cdist) {
#pragma omp parallel for schedule(static)
  for (int64_t a = 0; a < nq; ++a) {
    float *Dt = (float *)malloc(sizeof(float) * nprobe);
    int64_t *It = (int64_t *)malloc(sizeof(int64_t) * nprobe);
    topk_t h;
    topk_init(&h, nprobe, metric, Dt, It);
    for (int l = 0; l < nlist; ++l)
      topk_push(&h, canon(q + a * d, centroids + (int64_t)l * d, d, metric), l);
    for (int p = 0; p < nprobe; ++p) {
      probes[a * nprobe + p] = (int32_t)It[p];
      cdist[a * nprobe + p] = Dt[p];
    }
    free(Dt); free(It);
  }
}

/* ---- k-means (Sec. 4.1 "The k-means vector quantizer": Lloyd's two conditions,
 * applied in turn) ------------------------------------------------------------
 * Each of the niter rounds (1) assigns every training vector to its nearest
 * centroid -- canon L2, ties to the smaller centroid number, the rule of
 * or_assign -- and (2) moves every centroid to the mean of the vectors assigned
 * to it: the float64 sum of those vectors, added one after the other in the order
 * of the training set, divided by their number, rounded once to fp32.  A centroid
 * that received no vector keeps its position (the paper does not say; this is the
 * reading taken).  centroids: in = the initial centroids, out = the trained ones.
 * objective[r], if asked for, is the mean over the training vectors of the canon
 * distance to the assigned centroid in round r's step (1), summed in float64 in the
 * order of the vectors.  assign_out, if asked for, receives the assignment of the
 * LAST round's step (1) (the one the returned centroids are the means of). */
void or_kmeans(const float *x, int64_t n, int d, int K, int niter, float *centroids,
               double *objective, int32_t *assign_out) {
  int32_t *a = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
  float *best = (float *)malloc((size_t)(n > 0 ? n : 1) * sizeof(float));
  double *sum = (double *)malloc((size_t)K * d * sizeof(double));
  int64_t *cnt = (int64_t *)malloc((size_t)K * sizeof(int64_t));
  for (int r = 0; r < niter; ++r) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
      int bj = 0;
      float bd = canon(x + i * d, centroids, d, OR_METRIC_L2);
      for (int j = 1; j < K; ++j) {
        float dj = canon(x + i * d, centroids + (int64_t)j * d, d, OR_METRIC_L2);
        if (dj < bd) { bd = dj; bj = j; }
      }
      a[i] = bj;
      best[i] = bd;
    }
    double obj = 0.0;
    for (int64_t i = 0; i < n; ++i) obj += (double)best[i];
    if (objective) objective[r] = n > 0 ? obj / (double)n : 0.0;
    for (int64_t t = 0; t < (int64_t)K * d; ++t) sum[t] = 0.0;
    for (int j = 0; j < K; ++j) cnt[j] = 0;
    for (int64_t i = 0; i < n; ++i) {
      double *sj = sum + (int64_t)a[i] * d;
      for (int t = 0; t < d; ++t) sj[t] += (double)x[i * d + t];
      ++cnt[a[i]];
    }
    for (int j = 0; j < K; ++j) {
      if (cnt[j] == 0) continue;
      for (int t = 0; t < d; ++t)
        centroids[(int64_t)j * d + t] = (float)(sum[(int64_t)j * d + t] / (double)cnt[j]);
    }
  }
  if (assign_out && niter > 0) memcpy(assign_out, a, (size_t)n * sizeof(int32_t));
  free(a); free(best); free(sum); free(cnt);
}

/* ---- O3/O4: residual PQ encoding (Sec. 4.1 "product quantizer", Sec. 5.1
 * "Encoding residuals") ---------------------------------------------------
 * codebooks: [M][K][dsub] fp32, K = 2^nbits, dsub = d / M.
 * codes: n rows of code_size = M*nbits/8 bytes.  nbits = 8: byte m holds
 * c_m.  nbits = 4: byte i holds c_{2i} in its low nibble and c_{2i+1} in its
 * high nibble.
 * The residual is one fp32 subtraction per component; each sub-vector goes to
 * its nearest sub-centroid by canon L2 (a k-means quantizer minimises squared
 * error whatever the search metric is), ties to the smaller code. */
void or_pq_encode(const float *x, int64_t n, int d, const int32_t *list_of,
                  const float *centroids, int M, int nbits, const float *codebooks,
                  uint8_t *codes) {
  const int K = 1 << nbits, dsub = d / M;
  const int code_size = M * nbits / 8;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    float *r = (float *)malloc(sizeof(float) * d);
    const float *c = centroids + (int64_t)list_of[i] * d;
    for (int t = 0; t < d; ++t) r[t] = x[i * d + t] - c[t];
    uint8_t *out = codes + i * code_size;
    memset(out, 0, code_size);
    for (int m = 0; m < M; ++m) {
      const float *Tm = codebooks + (int64_t)m * K * dsub;
      int best = 0;
      float bd = or_canon_l2(r + m * dsub, Tm, dsub);
      for (int j = 1; j < K; ++j) {
        float dj = or_canon_l2(r + m * dsub, Tm + (int64_t)j * dsub, dsub);
        if (dj < bd) { bd = dj; best = j; }
      }
      if (nbits == 8) out[m] = (uint8_t)best;
      else out[m >> 1] |= (uint8_t)(best << ((m & 1) * 4));
    }
    free(r);
  }
}

static int code_at(const uint8_t *code, int m, int nbits) {
  return nbits == 8 ? code[m] : (code[m >> 1] >> ((m & 1) * 4)) & 15;
}

/* Decoder D(C(x)): centroid plus the concatenated sub-codewords
 * (Sec. 4.1: reconstructions of the sub-quantizers are concatenated).
 * Output in fp64: c and T are fp32, their sum is exact in fp64. */
void or_pq_decode(const uint8_t *codes, int64_t n, int d, const int32_t *list_of,
                  const float *centroids, int M, int nbits, const float *codebooks,
                  double *xdec) {
  const int K = 1 << nbits, dsub = d / M;
  const int code_size = M * nbits / 8;
  for (int64_t i = 0; i < n; ++i) {
    const float *c = centroids + (int64_t)list_of[i] * d;
    for (int m = 0; m < M; ++m) {
      int j = code_at(codes + i * code_size, m, nbits);
      const float *T = codebooks + ((int64_t)m * K + j) * dsub;
      for (int u = 0; u < dsub; ++u)
        xdec[i * d + m * dsub + u] = (double)c[m * dsub + u] + (double)T[u];
    }
  }
}

/* ---- stored norms (Sec. 4.3 "Compressed-domain search": with the decomposition
 * ||q - x'||^2 = ||q||^2 + ||x'||^2 - 2 <q, x'> the term ||x'||^2 must be available at
 * search time; it can be stored next to the code as a float32) ---------------------
 * norm(x') for x' = c_list + concat_m T_m[c_m]: every component is one fp32 addition,
 * the squares are accumulated by one fp32 fused-multiply-add chain in dimension order
 * (the arithmetic is fixed so that the stored numbers can be compared bit for bit). */
void or_pq_norms(const uint8_t *codes, int64_t n, int d, const int32_t *list_of,
                 const float *centroids, int M, int nbits, const float *codebooks, float *norms) {
  const int K = 1 << nbits, dsub = d / M;
  const int code_size = M * nbits / 8;
  for (int64_t i = 0; i < n; ++i) {
    const float *c = centroids + (int64_t)list_of[i] * d;
    float acc = 0.0f;
    for (int m = 0; m < M; ++m) {
      int j = code_at(codes + i * code_size, m, nbits);
      const float *T = codebooks + ((int64_t)m * K + j) * dsub;
      for (int u = 0; u < dsub; ++u) {
        float xt = c[m * dsub + u] + T[u];
        acc = fmaf(xt, xt, acc);
      }
    }
    norms[i] = acc;
  }
}

/* ---- O6-O8: IVF-PQ search (Sec. 5.1, Eq. 10 ADC, Eq. 14 LUT) -------------
 * The index is given as plain arrays: list l owns rows
 * [list_offsets[l], list_offsets[l+1]) of `codes` and `ids`.
 *
 * form 0 (the definition): every stored code of every probed list is decoded
 *   to x' = c_l + concat_m T_m[c_m] and the distance ||q - x'||^2 (or <q,x'>)
 *   is evaluated directly on x' in fp64, rounded once to fp32.
 * form 1 (compressed domain): fp32 residual r = q - c_l, table
 *   LUT_m[j] = canon_l2(r_m, T_m[j]) and the distance is sum_m LUT_m[c_m] in
 *   fp32, m ascending; for IP, LUT_m[j] = canon_ip(q_m, T_m[j]) and the
 *   score is canon_ip(q, c_l) + sum_m LUT_m[c_m].
 * form 2 (L2 only; Sec. 4.3, the decomposition ||q - x'||^2 = ||q||^2 + ||x'||^2
 *   - 2 <q, x'> with the norm stored next to the code, norms[s] from or_pq_norms):
 *   ((||q||^2 - 2 <q, c_l>) + norm) + sum_m (-2 <q_m, T_m[c_m]>) in fp32, m ascending,
 *   every inner product a canon_ip chain.
 * form 3 (L2 only; Sec. 4.3 "Compressed-domain search": the table of a (query, list) pair
 *   split into a term that depends on the query alone and one that depends on the list alone,
 *   the latter computed once when the index is built):
 *   |q_m - c_m - t|^2 = |q_m - c_m|^2 + (-2 <q_m, t>) + (|t|^2 + 2 <c_m, t>), hence
 *   LUT_m[j] = A_m[j] + B_{l,m}[j] with A_m[j] = -2 canon_ip(q_m, T_m[j]) (per query) and
 *   B_{l,m}[j] = fma(2, canon_ip(c_{l,m}, T_m[j]), canon_ip(T_m[j], T_m[j])) (per list), and the
 *   distance is canon_l2(q, c_l) + sum_m LUT_m[c_m] in fp32, m ascending.
 * forms 1 to 3 exist to pin the compressed-domain identities against form 0; parity
 * tests of the GPU path use form 0.
 *
 * nscanned[a] (may be NULL) receives the number of codes visited for query a.
 * probes_out (may be NULL) receives the probed lists, best first. */
void or_ivfpq_search(const float *q, int64_t nq, int d, int metric, int coarse_metric, int nlist,
                     const float *centroids, int M, int nbits, const float *codebooks,
                     const int64_t *list_offsets, const uint8_t *codes, const int64_t *ids,
                     const float *norms, int k, int nprobe, int form, float *D, int64_t *I,
                     int64_t *nscanned, int32_t *probes_out) {
  const int K = 1 << nbits, dsub = d / M;
  const int code_size = M * nbits / 8;
  if (nprobe > nlist) nprobe = nlist;
  int32_t *probes = (int32_t *)malloc(sizeof(int32_t) * nq * nprobe);
  float *cdist = (float *)malloc(sizeof(float) * nq * nprobe);
  /* the lists to visit are the nprobe best under the COARSE metric (Sec. 5.1, the figure on
   * maximum inner product search: an inner-product index may assign and probe by L2, the
   * default there, or by inner product); the scores below are under the index metric */
  or_coarse_probe(q, nq, centroids, nlist, d, coarse_metric, nprobe, probes, cdist);
  if (probes_out) memcpy(probes_out, probes, sizeof(int32_t) * nq * nprobe);

#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t a = 0; a < nq; ++a) {
    const float *qa = q + a * d;
    double *xd = (double *)malloc(sizeof(double) * d);
    float *r = (float *)malloc(sizeof(float) * d);
    float *lut = (float *)malloc(sizeof(float) * M * K);
    topk_t h;
    topk_init(&h, k, metric, D + a * k, I + a * k);
    int64_t visited = 0;
    for (int p = 0; p < nprobe; ++p) {
      const int l = probes[a * nprobe + p];
      const float *c = centroids + (int64_t)l * d;
      float bias = 0.0f;
      if (form == 2) {   /* L2 through stored norms: one table per query would do; rebuilt here per list for plainness */
        bias = fmaf(-2.0f, or_canon_ip(qa, c, d), or_canon_ip(qa, qa, d));
        for (int m = 0; m < M; ++m)
          for (int j = 0; j < K; ++j)
            lut[m * K + j] = -2.0f * or_canon_ip(qa + m * dsub, codebooks + ((int64_t)m * K + j) * dsub, dsub);
      }
      if (form == 3) {   /* per-query term + per-list term; both rebuilt here per pair for plainness */
        bias = or_canon_l2(qa, c, d);
        for (int m = 0; m < M; ++m)
          for (int j = 0; j < K; ++j) {
            const float *T = codebooks + ((int64_t)m * K + j) * dsub;
            const float a_mj = -2.0f * or_canon_ip(qa + m * dsub, T, dsub);
            const float b_mj = fmaf(2.0f, or_canon_ip(c + m * dsub, T, dsub), or_canon_ip(T, T, dsub));
            lut[m * K + j] = a_mj + b_mj;
          }
      }
      if (form == 1) {
        if (metric == OR_METRIC_L2) {
          for (int t = 0; t < d; ++t) r[t] = qa[t] - c[t];
          for (int m = 0; m < M; ++m)
            for (int j = 0; j < K; ++j)
              lut[m * K + j] = or_canon_l2(r + m * dsub, codebooks + ((int64_t)m * K + j) * dsub, dsub);
        } else {
          bias = or_canon_ip(qa, c, d);
          for (int m = 0; m < M; ++m)
            for (int j = 0; j < K; ++j)
              lut[m * K + j] = or_canon_ip(qa + m * dsub, codebooks + ((int64_t)m * K + j) * dsub, dsub);
        }
      }
      for (int64_t s = list_offsets[l]; s < list_offsets[l + 1]; ++s) {
        const uint8_t *code = codes + s * code_size;
        float dist;
        if (form == 0) {
          for (int m = 0; m < M; ++m) {
            const float *T = codebooks + ((int64_t)m * K + code_at(code, m, nbits)) * dsub;
            for (int u = 0; u < dsub; ++u) xd[m * dsub + u] = (double)c[m * dsub + u] + (double)T[u];
          }
          dist = report_dist(qa, xd, d, metric);
        } else {
          dist = form == 2 ? bias + norms[s] : bias;
          for (int m = 0; m < M; ++m) dist += lut[m * K + code_at(code, m, nbits)];
        }
        topk_push(&h, dist, ids[s]);
        ++visited;
      }
    }
    if (nscanned) nscanned[a] = visited;
    free(xd); free(r); free(lut);
  }
  free(probes); free(cdist);
}

/* ---- IVF-Flat search (Sec. 5.1 "Inverted files" with vectors stored as they
 * are; App. A.3 lists it among the GPU indexes) ---------------------------------
 * Same two steps as IVF-PQ -- the nprobe best lists by or_coarse_probe, then a
 * selection over the entries of those lists -- but an entry is the vector
 * itself, so its distance is the definition (float64 sum, rounded once), as in
 * or_flat_search.  vecs: [ntotal, d] in list order (list l owns rows
 * list_offsets[l] .. list_offsets[l + 1]). */
void or_ivfflat_search(const float *q, int64_t nq, int d, int metric, int nlist,
                       const float *centroids, const int64_t *list_offsets, const float *vecs,
                       const int64_t *ids, int k, int nprobe, float *D, int64_t *I,
                       int64_t *nscanned, int32_t *probes_out) {
  if (nprobe > nlist) nprobe = nlist;
  int32_t *probes = (int32_t *)malloc(sizeof(int32_t) * nq * nprobe);
  float *cdist = (float *)malloc(sizeof(float) * nq * nprobe);
  or_coarse_probe(q, nq, centroids, nlist, d, metric, nprobe, probes, cdist);
  if (probes_out) memcpy(probes_out, probes, sizeof(int32_t) * nq * nprobe);
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t a = 0; a < nq; ++a) {
    const float *qa = q + a * d;
    topk_t h;
    topk_init(&h, k, metric, D + a * k, I + a * k);
    int64_t visited = 0;
    for (int p = 0; p < nprobe; ++p) {
      const int l = probes[a * nprobe + p];
      for (int64_t s = list_offsets[l]; s < list_offsets[l + 1]; ++s) {
        const float *xs = vecs + s * d;
        double acc = 0.0;
        if (metric == OR_METRIC_L2) {
          for (int t = 0; t < d; ++t) {
            double diff = (double)qa[t] - (double)xs[t];
            acc += diff * diff;
          }
        } else {
          for (int t = 0; t < d; ++t) acc += (double)qa[t] * (double)xs[t];
        }
        topk_push(&h, (float)acc, ids[s]);
        ++visited;
      }
    }
    if (nscanned) nscanned[a] = visited;
  }
  free(probes); free(cdist);
}

/* ---- 8-bit scalar quantizer and IVF-SQ8 (Sec. 4.1 "Scalar quantizers": a uniform
 * quantizer encodes every component on its own; a scale and an offset per dimension
 * determine which values are reconstructed.  App. A.3 lists the IVF index with a scalar
 * quantizer among the GPU indexes) ------------------------------------------------
 * The paper gives no formula; the reading taken: component t is expected in
 * [vmin_t, vmin_t + 256 step_t); that range is cut into 256 cells of width step_t; the
 * code is the number of the cell that holds the component (components outside go to the
 * first / last cell) and the reconstruction is the middle of the cell:
 *     u = (x_t - vmin_t) / step_t          one fp32 subtraction, one fp32 division
 *     code_t = 0 if u < 0, 255 if u >= 256, else the integer part of u
 *     x'_t = fma(code_t + 0.5, step_t, vmin_t)   in fp32
 * The fp32 operations are fixed so that codes can be compared bit for bit. */
void or_sq8_encode(const float *x, int64_t n, int d, const float *vmin, const float *step,
                   uint8_t *codes) {
  for (int64_t i = 0; i < n; ++i)
    for (int t = 0; t < d; ++t) {
      float u = (x[i * d + t] - vmin[t]) / step[t];
      codes[i * d + t] = u < 0.0f ? 0 : (u >= 256.0f ? 255 : (uint8_t)(int)u);
    }
}

void or_sq8_decode(const uint8_t *codes, int64_t n, int d, const float *vmin, const float *step,
                   float *xdec) {
  for (int64_t i = 0; i < n; ++i)
    for (int t = 0; t < d; ++t)
      xdec[i * d + t] = fmaf((float)codes[i * d + t] + 0.5f, step[t], vmin[t]);
}

/* IVF-SQ8 search: the probes of or_coarse_probe, then for every stored code of the probed
 * lists the distance between the query and the code's reconstruction, by the definition
 * (float64 sum over the fp32 reconstruction, rounded once).  The vectors themselves are
 * encoded (no residual). */
void or_ivfsq8_search(const float *q, int64_t nq, int d, int metric, int nlist,
                      const float *centroids, const float *vmin, const float *step,
                      const int64_t *list_offsets, const uint8_t *codes, const int64_t *ids,
                      int k, int nprobe, float *D, int64_t *I, int64_t *nscanned) {
  if (nprobe > nlist) nprobe = nlist;
  int32_t *probes = (int32_t *)malloc(sizeof(int32_t) * nq * nprobe);
  float *cdist = (float *)malloc(sizeof(float) * nq * nprobe);
  or_coarse_probe(q, nq, centroids, nlist, d, metric, nprobe, probes, cdist);
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t a = 0; a < nq; ++a) {
    const float *qa = q + a * d;
    topk_t h;
    topk_init(&h, k, metric, D + a * k, I + a * k);
    int64_t visited = 0;
    for (int p = 0; p < nprobe; ++p) {
      const int l = probes[a * nprobe + p];
      for (int64_t s = list_offsets[l]; s < list_offsets[l + 1]; ++s) {
        const uint8_t *c = codes + s * d;
        double acc = 0.0;
        for (int t = 0; t < d; ++t) {
          double xt = (double)fmaf((float)c[t] + 0.5f, step[t], vmin[t]);
          if (metric == OR_METRIC_L2) { double diff = (double)qa[t] - xt; acc += diff * diff; }
          else acc += (double)qa[t] * xt;
        }
        topk_push(&h, (float)acc, ids[s]);
        ++visited;
      }
    }
    if (nscanned) nscanned[a] = visited;
  }
  free(probes); free(cdist);
}

int or_num_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}
