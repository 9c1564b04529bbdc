/*
 * Sanitizer run of the CPU oracle.  TEST INFRASTRUCTURE ONLY, like oracle.c.
 *
 * Includes oracle.c and calls every entry point on small seeded inputs held in buffers of
 * exactly the documented sizes, so that AddressSanitizer sees any read or write past an end and
 * UndefinedBehaviorSanitizer any shift, overflow or misaligned access.  Shapes are chosen for the
 * corners: k larger than what a query can reach, nprobe = nlist and nprobe > nlist, empty
 * lists, 4-bit and 8-bit codes, both metrics, an inner-product index probed by L2, every table
 * form, one vector, one list.  A few results are checked for order so that the calls cannot be
 * optimised away; the values themselves are the pin tests' business.
 *
 * Build and run (tests/test_oracle_sanitized.py does this):
 *   gcc -O1 -g -ffp-contract=off -mfma -fsanitize=address,undefined -fno-sanitize-recover=all \
 *       oracle/sanitize_check.c -lm -o sanitize_check && ./sanitize_check
 */
#include "oracle.c"

#include <stdio.h>

static uint64_t rng_state = 0x9e3779b97f4a7c15ull;
static double rnd(void) { /* xorshift64*, uniform in [0, 1) */
  rng_state ^= rng_state >> 12;
  rng_state ^= rng_state << 25;
  rng_state ^= rng_state >> 27;
  return (double)((rng_state * 0x2545F4914F6CDD1Dull) >> 11) / 9007199254740992.0;
}
static float *rand_floats(int64_t n, double lo, double hi) {
  float *p = (float *)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
  for (int64_t i = 0; i < n; ++i) p[i] = (float)(lo + (hi - lo) * rnd());
  return p;
}
static int failures = 0;
static void expect(int ok, const char *what) {
  if (!ok) {
    fprintf(stderr, "sanitize_check: %s\n", what);
    ++failures;
  }
}
static int sorted_best_first(const float *D, const int64_t *I, int k, int metric) {
  for (int j = 1; j < k; ++j) {
    if (I[j] < 0) continue; /* empty slots come last */
    if (I[j - 1] < 0) return 0;
    if (metric == OR_METRIC_L2 ? D[j - 1] > D[j] : D[j - 1] < D[j]) return 0;
  }
  return 1;
}

static void check_flat_and_refine(int64_t nb, int64_t nq, int d, int k, int metric) {
  float *x = rand_floats(nb * d, -1, 1), *q = rand_floats(nq * d, -1, 1);
  float *D = (float *)malloc(sizeof(float) * (size_t)(nq * k));
  int64_t *I = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nq * k));
  or_flat_search(x, nb, q, nq, d, metric, k, D, I);
  for (int64_t a = 0; a < nq; ++a) expect(sorted_best_first(D + a * k, I + a * k, k, metric), "flat search order");
  /* second stage on the first stage's ids (some of them -1 when k > nb) */
  const int k2 = k > 2 ? k / 2 : 1;
  float *D2 = (float *)malloc(sizeof(float) * (size_t)(nq * k2));
  int64_t *I2 = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nq * k2));
  or_refine(x, nb, q, nq, d, metric, I, k, k2, D2, I2);
  for (int64_t a = 0; a < nq; ++a) expect(sorted_best_first(D2 + a * k2, I2 + a * k2, k2, metric), "refine order");
  free(x); free(q); free(D); free(I); free(D2); free(I2);
}

static void check_kmeans(int64_t n, int d, int K, int niter) {
  float *x = rand_floats(n * d, 0, 4), *c = rand_floats((int64_t)K * d, 0, 4);
  double *obj = (double *)malloc(sizeof(double) * (size_t)(niter > 0 ? niter : 1));
  int32_t *assign = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
  or_kmeans(x, n, d, K, niter, c, obj, assign);
  for (int it = 1; it < niter; ++it) expect(obj[it] <= obj[it - 1] * (1 + 1e-12), "k-means objective does not grow");
  for (int64_t i = 0; i < n; ++i) expect(assign[i] >= 0 && assign[i] < K, "k-means assignment range");
  free(x); free(c); free(obj); free(assign);
}

/* Builds a small IVF-PQ index the way the add path is defined (assign, encode, group by list
 * keeping the order of arrival) and searches it in every table form. */
static void check_ivfpq(int64_t nb, int64_t nq, int d, int nlist, int M, int nbits, int metric,
                        int coarse_metric, int k, int nprobe, int leave_empty) {
  const int K = 1 << nbits, dsub = d / M, code_size = M * nbits / 8;
  float *x = rand_floats(nb * d, -1, 1), *q = rand_floats(nq * d, -1, 1);
  float *centroids = rand_floats((int64_t)nlist * d, -1, 1);
  if (leave_empty) /* far away: no vector is assigned to the last list under L2 */
    for (int t = 0; t < d; ++t) centroids[(int64_t)(nlist - 1) * d + t] = metric == OR_METRIC_L2 ? 100.f : 0.f;
  float *codebooks = rand_floats((int64_t)M * K * dsub, -0.5, 0.5);
  int32_t *list_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)(nb > 0 ? nb : 1));
  or_assign(x, nb, centroids, nlist, d, coarse_metric, list_of);
  uint8_t *codes = (uint8_t *)malloc((size_t)(nb * code_size > 0 ? nb * code_size : 1));
  or_pq_encode(x, nb, d, list_of, centroids, M, nbits, codebooks, codes);
  double *xdec = (double *)malloc(sizeof(double) * (size_t)(nb * d > 0 ? nb * d : 1));
  or_pq_decode(codes, nb, d, list_of, centroids, M, nbits, codebooks, xdec);
  /* list-contiguous storage */
  int64_t *off = (int64_t *)calloc((size_t)nlist + 1, sizeof(int64_t));
  for (int64_t i = 0; i < nb; ++i) off[list_of[i] + 1]++;
  for (int l = 0; l < nlist; ++l) off[l + 1] += off[l];
  int64_t *fill = (int64_t *)malloc(sizeof(int64_t) * (size_t)nlist);
  memcpy(fill, off, sizeof(int64_t) * (size_t)nlist);
  uint8_t *scodes = (uint8_t *)malloc((size_t)(nb * code_size > 0 ? nb * code_size : 1));
  int64_t *ids = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nb > 0 ? nb : 1));
  int32_t *slist = (int32_t *)malloc(sizeof(int32_t) * (size_t)(nb > 0 ? nb : 1));
  for (int64_t i = 0; i < nb; ++i) {
    const int64_t at = fill[list_of[i]]++;
    memcpy(scodes + at * code_size, codes + i * code_size, (size_t)code_size);
    ids[at] = i;
    slist[at] = list_of[i];
  }
  float *norms = (float *)malloc(sizeof(float) * (size_t)(nb > 0 ? nb : 1));
  or_pq_norms(scodes, nb, d, slist, centroids, M, nbits, codebooks, norms);
  const int npr = nprobe < nlist ? nprobe : nlist;
  float *D = (float *)malloc(sizeof(float) * (size_t)(nq * k));
  int64_t *I = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nq * k));
  int64_t *nscanned = (int64_t *)malloc(sizeof(int64_t) * (size_t)nq);
  int32_t *probes = (int32_t *)malloc(sizeof(int32_t) * (size_t)(nq * npr));
  float *cdist = (float *)malloc(sizeof(float) * (size_t)(nq * npr));
  or_coarse_probe(q, nq, centroids, nlist, d, coarse_metric, npr, probes, cdist); /* (its contract: nprobe <= nlist) */
  for (int form = 0; form <= 3; ++form) {
    if (form == 3 && metric != OR_METRIC_L2) continue; /* the per-list term belongs to L2 */
    or_ivfpq_search(q, nq, d, metric, coarse_metric, nlist, centroids, M, nbits, codebooks, off, scodes,
                    ids, norms, k, nprobe, form, D, I, nscanned, probes);
    for (int64_t a = 0; a < nq; ++a) {
      expect(sorted_best_first(D + a * k, I + a * k, k, metric), "IVF-PQ search order");
      expect(nscanned[a] >= 0 && nscanned[a] <= nb, "IVF-PQ scanned count");
      for (int j = 0; j < k; ++j) expect(I[a * k + j] >= -1 && I[a * k + j] < nb, "IVF-PQ id range");
    }
  }
  free(x); free(q); free(centroids); free(codebooks); free(list_of); free(codes); free(xdec); free(off);
  free(fill); free(scodes); free(ids); free(slist); free(norms); free(D); free(I); free(nscanned);
  free(probes); free(cdist);
}

static void check_ivfflat_and_sq8(int64_t nb, int64_t nq, int d, int nlist, int metric, int k, int nprobe) {
  float *x = rand_floats(nb * d, -1, 1), *q = rand_floats(nq * d, -1, 1);
  float *centroids = rand_floats((int64_t)nlist * d, -1, 1);
  int32_t *list_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)nb);
  or_assign(x, nb, centroids, nlist, d, metric, list_of);
  int64_t *off = (int64_t *)calloc((size_t)nlist + 1, sizeof(int64_t));
  for (int64_t i = 0; i < nb; ++i) off[list_of[i] + 1]++;
  for (int l = 0; l < nlist; ++l) off[l + 1] += off[l];
  int64_t *fill = (int64_t *)malloc(sizeof(int64_t) * (size_t)nlist);
  memcpy(fill, off, sizeof(int64_t) * (size_t)nlist);
  float *vecs = (float *)malloc(sizeof(float) * (size_t)(nb * d));
  int64_t *ids = (int64_t *)malloc(sizeof(int64_t) * (size_t)nb);
  for (int64_t i = 0; i < nb; ++i) {
    const int64_t at = fill[list_of[i]]++;
    memcpy(vecs + at * d, x + i * d, sizeof(float) * (size_t)d);
    ids[at] = i;
  }
  const int npr = nprobe < nlist ? nprobe : nlist;
  float *D = (float *)malloc(sizeof(float) * (size_t)(nq * k));
  int64_t *I = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nq * k));
  int64_t *nscanned = (int64_t *)malloc(sizeof(int64_t) * (size_t)nq);
  int32_t *probes = (int32_t *)malloc(sizeof(int32_t) * (size_t)(nq * npr));
  or_ivfflat_search(q, nq, d, metric, nlist, centroids, off, vecs, ids, k, nprobe, D, I, nscanned, probes);
  for (int64_t a = 0; a < nq; ++a) expect(sorted_best_first(D + a * k, I + a * k, k, metric), "IVF-Flat search order");
  /* 8-bit scalar quantizer over the same lists */
  float *vmin = (float *)malloc(sizeof(float) * (size_t)d), *step = (float *)malloc(sizeof(float) * (size_t)d);
  for (int t = 0; t < d; ++t) { vmin[t] = -1.f; step[t] = 2.f / 256.f; }
  uint8_t *codes = (uint8_t *)malloc((size_t)(nb * d));
  or_sq8_encode(vecs, nb, d, vmin, step, codes);
  float *dec = (float *)malloc(sizeof(float) * (size_t)(nb * d));
  or_sq8_decode(codes, nb, d, vmin, step, dec);
  for (int64_t i = 0; i < nb * d; ++i) expect(fabsf(dec[i] - vecs[i]) <= step[i % d] * 0.5f * 1.0001f, "SQ8 half-cell bound");
  or_ivfsq8_search(q, nq, d, metric, nlist, centroids, vmin, step, off, codes, ids, k, nprobe, D, I, nscanned);
  for (int64_t a = 0; a < nq; ++a) expect(sorted_best_first(D + a * k, I + a * k, k, metric), "IVF-SQ8 search order");
  free(x); free(q); free(centroids); free(list_of); free(off); free(fill); free(vecs); free(ids); free(D);
  free(I); free(nscanned); free(probes); free(vmin); free(step); free(codes); free(dec);
}

int main(void) {
  const float a[5] = {1.f, 2.f, 3.f, 4.f, 5.f}, b[5] = {0.5f, -2.f, 3.25f, 8.f, 1.f};
  expect(or_canon_l2(a, b, 5) == 48.3125f, "canon L2 of an exactly representable case");
  expect(or_canon_ip(a, b, 5) == 43.25f, "canon IP of an exactly representable case");
  for (int metric = 0; metric <= 1; ++metric) {
    check_flat_and_refine(257, 5, 24, 10, metric);
    check_flat_and_refine(7, 3, 5, 12, metric); /* k > nb: padded results */
    check_flat_and_refine(1, 1, 1, 1, metric);
    check_ivfflat_and_sq8(300, 4, 12, 9, metric, 7, 3);
    check_ivfflat_and_sq8(40, 3, 8, 5, metric, 50, 9); /* k beyond the index, nprobe > nlist */
  }
  check_kmeans(500, 6, 7, 4);
  check_kmeans(5, 3, 8, 2); /* more centroids than vectors: empty clusters */
  check_kmeans(64, 4, 1, 1);
  check_ivfpq(400, 5, 16, 11, 4, 8, OR_METRIC_L2, OR_METRIC_L2, 10, 4, 1);
  check_ivfpq(400, 5, 16, 11, 8, 4, OR_METRIC_L2, OR_METRIC_L2, 10, 11, 0); /* 4-bit, all lists */
  check_ivfpq(300, 4, 24, 6, 12, 4, OR_METRIC_IP, OR_METRIC_IP, 5, 3, 0);
  check_ivfpq(300, 4, 24, 6, 3, 8, OR_METRIC_IP, OR_METRIC_L2, 5, 2, 1);  /* IP index probed by L2 */
  check_ivfpq(30, 3, 8, 4, 2, 8, OR_METRIC_L2, OR_METRIC_L2, 64, 9, 0);    /* k beyond the index, nprobe > nlist */
  check_ivfpq(1, 1, 4, 1, 1, 8, OR_METRIC_L2, OR_METRIC_L2, 1, 1, 0);
  expect(or_num_threads() >= 1, "thread count");
  if (failures) {
    fprintf(stderr, "sanitize_check: %d check(s) failed\n", failures);
    return 1;
  }
  printf("sanitize_check: ok\n");
  return 0;
}
