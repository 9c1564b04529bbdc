// Host-side declarations shared by the translation units of libvs.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef unsigned long long u64;
typedef unsigned int u32;

// ---- canon distance tiles (kernels_dist.hip) --------------------------------
// out[a * ldo + b] = canon distance of A row a and B row b.
void launch_canon_matrix(const float* A, int64_t na, const float* B, int64_t nb, int d, int metric,
                         float* out, int64_t ldo, hipStream_t st);
// best[a] = min over b of key(canon(A_a, B_b), b); best must hold KEY_EMPTY on entry.
void launch_canon_argbest(const float* A, int64_t na, const float* B, int64_t nb, int d,
                          int metric, u64* best, hipStream_t st);

// ---- selection (kernels_select.hip) -----------------------------------------
void launch_fill_u64(u64* p, int64_t n, u64 v, hipStream_t st);
// Final outputs of a selection; any member may be null.
struct SelectOut {
  float* val = nullptr;       // [nrows, k] best values
  int64_t* id64 = nullptr;    // [nrows, k] indices as int64
  int32_t* idx32 = nullptr;   // [nrows, k] indices as int32
};
// keys[r][0..k) <- k best of (first ? {} : keys[r][0..k)) U {key(mat[r][c], col_base + c)}.
// When `last`, the result goes to `out` instead (already ordered best first) and keys is
// not written; keys may be null if first && last.
void launch_row_select(const float* mat, int64_t ld, int64_t nrows, int64_t ncols, u32 col_base,
                       int metric, int k, u64* keys, bool first, bool last, const SelectOut& out,
                       hipStream_t st);
// keys -> (value, int64 id); idmap == NULL: id = index, else id = idmap[index]; empty -> (-1, +-inf)
void launch_keys_to_results(const u64* keys, int64_t n, int metric, float* out_dist,
                            int64_t* out_ids, const int64_t* idmap, hipStream_t st);
// keys -> (int32 index, value); used for probes
void launch_keys_to_probes(const u64* keys, int64_t n, int metric, int32_t* out_idx,
                           float* out_val, hipStream_t st);
void launch_keys_to_index32(const u64* keys, int64_t n, int32_t* out_idx, hipStream_t st);

// ---- IVF-PQ (kernels_ivfpq.hip) ----------------------------------------------
struct IvfpqDims {
  int d, metric, nlist, M, nbits, K, dsub, code_size;
};
// tmp_codes[i][m] = PQ code of sub-vector m of the residual of x_i (one byte per m)
void launch_pq_encode(const IvfpqDims& g, const float* x, int64_t n, const int32_t* list_of,
                      const float* centroids, const float* codebooks, uint8_t* tmp_codes,
                      hipStream_t st);
// move old entries to their new offsets and scatter the new ones
// norms / old_norms / tmp_norms: the stored norms of Sec. 4.3's decomposition, or all null
void launch_relayout(const IvfpqDims& g, const uint8_t* old_codes, const int64_t* old_ids,
                     const float* old_norms, int64_t old_total, const int64_t* old_off,
                     const int64_t* new_off, const uint8_t* tmp_codes,
                     const int64_t* new_ids_or_null, int64_t id_base, const float* tmp_norms,
                     const int64_t* dest, const int32_t* new_list_of, int64_t n_new, uint8_t* codes,
                     int64_t* ids, float* norms, hipStream_t st);
// Indexes of the shapes that the bank-private-table scan kernel serves keep the code at position
// p of its list rotated by p bytes (stored byte b = c_{(b + p) mod M}); launch_relayout writes
// that layout, launch_codes_canonical turns a copy back into byte m = c_m.
bool ivfpq_codes_rotated(const IvfpqDims& g);
void launch_codes_canonical(const IvfpqDims& g, const uint8_t* stored, const int64_t* off,
                            int64_t total, uint8_t* out, hipStream_t st);
// tmp_norms[i] = |c_list(i) + decoded code i|^2.  tmp_codes: one byte per (vector, m) as the encoder
// writes them; stored_form: code_size bytes per vector as the lists hold them (4-bit codes packed
// two per byte; byte order canonical, not rotated)
void launch_pq_norms(const IvfpqDims& g, const uint8_t* tmp_codes, int64_t n, const int32_t* list_of,
                     const float* centroids, const float* codebooks, float* tmp_norms,
                     hipStream_t st, bool stored_form = false);
// norms[i] = |row i|^2 (fma chain in dimension order)
void launch_row_norms(const float* x, int64_t n, int d, float* norms, hipStream_t st);
void launch_list_of_storage(const int64_t* off, int nlist, int64_t total, int32_t* list_of,
                            hipStream_t st);
void launch_list_sizes(const int64_t* off, int nlist, int64_t* sizes, hipStream_t st);
// nsplit > 1: partial[q][s][0..k) = k best keys (value, storage position) of the probes handled by
// split s.  nsplit == 1: final results go straight to out_dist / out_ids (ids[position]).
// counter: one 64-bit word of device memory the scan may use to hand out its work items.
int launch_ivfpq_scan(const IvfpqDims& g, const float* q, int64_t nq, const float* centroids,
                      const float* codebooks, const int32_t* probes, const float* cdist,
                      int nprobe, int nsplit, const int64_t* list_off, const uint8_t* codes,
                      const float* norms, const float* cnorm, const float* list_tables,
                      float* query_tables, int64_t ntotal, int k, u64* partial, u64* counter,
                      const int64_t* ids, float* out_dist, int64_t* out_ids, hipStream_t st);
// The wavefront-private scan (one wavefront per (query, probe split); every table form but the
// residual tables) is used while the mean list is at most this long; it needs query_tables:
// ivfpq_query_table_bytes() of device work space.
constexpr int kWaveScanMaxMeanList = 1024;
bool ivfpq_wave_scan_applies(const IvfpqDims& g, int64_t ntotal);
size_t ivfpq_query_table_bytes(const IvfpqDims& g, int64_t nq);
// Slots of n newly assigned vectors in the grown inverted lists, computed on the device:
// dest[i] = slot of vector i (behind its list's old entries, new vectors of a list in batch order),
// new_off [nlist + 1] = offsets of the grown lists.  list_of [n] (n < 2^31), old_off [nlist + 1],
// work: ivf_place_work_bytes(n, nlist) bytes, all device memory.  Returns the device address of a
// flag that is non-zero once the kernels have run if some list_of[i] is outside [0, nlist).
size_t ivf_place_work_bytes(int64_t n, int nlist);
int* launch_ivf_place(const int32_t* list_of, int64_t n, int nlist, const int64_t* old_off, char* work,
                      int64_t* dest, int64_t* new_off, hipStream_t st);
// cdist[a][p] = <q_a, c_{probes[a][p]}> as one fp32 fused-multiply-add chain in dimension order
// (the value the coarse quantizer itself returns under the inner-product metric); probes < 0 are left alone
void launch_probe_inner_products(const float* q, int64_t nq, int d, const float* centroids,
                                 const int32_t* probes, int nprobe, float* cdist, hipStream_t st);
// stats[0] = sum over the n (query, probe) pairs of the probed list's size, stats[1] = pairs whose
// list is not empty, stats[2] = mfma_rows, stats[3] = *fallback_count (0 if null), stats[4] = p_first
// (probes per query that a list-major search scans query-major first; 0: the search is query-major),
// stats[5] = the part of stats[0] that falls on those probes, stats[6] = 0 (set after a list-major
// scan by launch_search_stats_rescan to the number of queries scanned again); device memory,
// written in stream order.
void launch_search_stats(const int32_t* probes, int64_t n, const int64_t* list_off, const int* fallback_count,
                         int64_t mfma_rows, int nprobe, int p_first, long long* stats, hipStream_t st);
void launch_search_stats_rescan(const unsigned* rescan_count, long long* stats, hipStream_t st);
// out [K][M][dsub] = codebooks [M][K][dsub] with the first two axes exchanged.  launch_ivfpq_scan
// expects it directly behind the codebooks it is given (codebooks + M * K * dsub).
void launch_pq_codebooks_by_entry(const IvfpqDims& g, const float* codebooks, float* out, hipStream_t st);
// out [nlist][K][M]: |T_m[j]|^2 + 2 <c_{l,m}, T_m[j]>, the per-list term of the split look-up tables
void launch_pq_list_tables(const IvfpqDims& g, const float* centroids, const float* codebooks, float* out,
                           hipStream_t st);
// List-major L2 scan with residual tables for large batches (shapes of the bank-private kernel).
bool ivfpq_listmajor_shape(const IvfpqDims& g);
size_t ivfpq_listmajor_bytes(const IvfpqDims& g, int64_t nq, int nprobe, int cap);
const unsigned* ivfpq_listmajor_rescan_count(const IvfpqDims& g, int64_t nq, int nprobe, int cap, const char* lm);
int launch_ivfpq_scan_listmajor(int part, const IvfpqDims& g, const float* q, int64_t nq, const float* centroids,
                                const float* codebooks, const int32_t* probes, const float* cdist, int nprobe,
                                int p_first, int cap, const int64_t* list_off, const uint8_t* codes,
                                int64_t ntotal, int k, u64* first, u64* counter, char* lm, const int64_t* ids,
                                float* out_dist, int64_t* out_ids, hipStream_t st);
void launch_ivfpq_merge(const u64* partial, int64_t nq, int nsplit, int k, int metric,
                        const int64_t* ids, float* out_dist, int64_t* out_ids, hipStream_t st);

// ---- MFMA shortlist + exact re-rank (kernels_mfma.hip) --------------------------
// What operand preparation learns about a matrix (device memory).
struct PrepInfo {
  u32 all_int;        // every value is an integer
  u32 all_bf16;       // every value is exactly representable in bf16
  u32 max_norm_bits;  // bits of the largest squared row norm (non-negative float)
  u32 all_nonneg;     // no value is negative
  // Of the column operand of a k-nearest-rows call only, and only where that operand outlives the
  // call (an index's centroids or vectors): bit 0 (calls with k = 1) and bit 1 (k > 1) are set
  // while the sweeps of such calls may use the fp16 heads alone on operands that are not exactly
  // bf16 (one matrix product instead of three, with the wider error bound that goes with it).  A
  // bit is cleared for good by the exact fallback once more than one row in 512 of a call failed
  // the sufficiency test under that bound.
  u32 heads_only;
};
struct MfmaOperand {
  const float* x;             // [n, d] original fp32 rows
  const unsigned short* hi;   // [n, d] bf16 heads
  const unsigned short* lo;   // [n, d] bf16 tails
  const unsigned short* h16;  // [n, d] fp16 heads (written by operand preparation right behind the tails)
  const float* norm;          // [n] squared norms
  const PrepInfo* info;
  int64_t n;
  int known_bf16;             // info->all_bf16 where the host has read it back (0 / 1), else -1
  bool try_heads_only;        // info->heads_only was set when the operand was prepared (it may have been cleared since)
};
bool mfma_knn_supported(int d, int k);
// operand planes hold this many rows (the tail is zero padding)
int64_t mfma_padded_rows(int64_t n);
int mfma_knn_kp(int k);
void launch_prep(const float* x, int64_t n, int d, unsigned short* hi, unsigned short* lo,
                 float* norm, PrepInfo* info, hipStream_t st, bool try_heads_only = false);
// bytes of the shortlist buffer [na, nsplit, kp] and the column split count to use
size_t mfma_knn_shortlist_bytes(int64_t na, int64_t nb, int d, int k, int* nsplit_out);
// (also clears *fb_count, the counter that launch_rerank of the same call adds to)
void launch_mfma_shortlist(const MfmaOperand& A, const MfmaOperand& B, int d, int metric, int k,
                           int nsplit, u64* shortlist, int* fb_count, hipStream_t st);
// exact k best per row of A from the shortlists; rows that cannot be proven exact are
// recomputed over all of B.  fb_count: 1 int, fb_rows: A.n ints, fb_partial:
// mfma_knn_fallback_bytes(...) bytes (device scratch; may be null when that is 0).
size_t mfma_knn_fallback_bytes(int64_t na, int64_t nb, int k);
void launch_rerank(const MfmaOperand& A, const MfmaOperand& B, int d, int metric, int k, int nsplit,
                   const u64* shortlist, float eps_scale, const SelectOut& out, int* fb_count,
                   int* fb_rows, u64* fb_partial, hipStream_t st);
int read_fallback_total(unsigned long long* out);

// ---- kernels_ivfflat.hip -------------------------------------------------------
void launch_ivfflat_relayout(int d, int nlist, const float* old_rows, const int64_t* old_ids,
                             int64_t old_total, const int64_t* old_off, const int64_t* new_off,
                             const float* x, const int64_t* new_ids_or_null, int64_t id_base,
                             const int64_t* dest, int64_t n_new, float* rows, int64_t* ids,
                             hipStream_t st);
size_t ivfflat_scan_lds_bytes(int d, int k);
// canon distance of every stored vector of the probed lists, k best per (query, probe split):
// results to out_dist / out_ids when nsplit == 1, else keys to partial [nq, nsplit, k]
void launch_ivfflat_scan(int d, int metric, const float* q, int64_t nq, const int32_t* probes,
                         int nprobe, int nsplit, const int64_t* list_off, const float* rows, int k,
                         u64* partial, const int64_t* ids, float* out_dist, int64_t* out_ids,
                         hipStream_t st);

// IVF-SQ8 (same file): 8-bit scalar-quantizer codes [n, d]; scan = IVF-Flat over reconstructions
void launch_sq8_encode(const float* x, int64_t n, int d, const float* vmin, const float* step,
                       uint8_t* codes, hipStream_t st);
size_t ivfsq8_scan_lds_bytes(int d, int k);
void launch_ivfsq8_scan(int d, int metric, const float* q, int64_t nq, const float* vmin,
                        const float* step, const int32_t* probes, int nprobe, int nsplit,
                        const int64_t* list_off, const uint8_t* codes, int k, u64* partial,
                        const int64_t* ids, float* out_dist, int64_t* out_ids, hipStream_t st);

// ---- kernels_train.hip ---------------------------------------------------------
// centroids[j] <- mean of the rows x[order[off[j] .. off[j + 1])] (float64 sum in that order, in
// blocks of 4096 rows whose sums are added in block order); a centroid with an empty range keeps
// its value.  `largest` = the largest range's length; `partial` = work space of
// segmented_mean_partial_bytes (may be null when that is 0)
size_t segmented_mean_partial_bytes(int64_t n, int d, int K, int64_t largest);
void launch_segmented_mean(const float* x, int d, const int32_t* order, const int64_t* off, int K,
                           int64_t largest, float* centroids, double* partial, hipStream_t st);
// stable counting sort of the assignment idx [n] by centroid (K <= 16384) and the float64 sum
// of val [n]: order [n], off [K + 1]; scal[0] = largest cluster, scal[1] != 0 if an
// assignment was outside [0, K); partial [256] sums to the sum of val
size_t kmeans_sort_bytes(int64_t n, int K);
void launch_kmeans_sort(const int32_t* idx, const float* val, int64_t n, int K, char* work, int32_t* order,
                        int64_t* off, int64_t** scal_out, double** partial_out, hipStream_t st);
// out[m][i][:] = (x[i] - centroids[list_of[i]])[m * dsub : (m + 1) * dsub], out is [d / dsub][n][dsub]
void launch_residual_slices(const float* x, int64_t n, int d, int dsub, const float* centroids,
                            const int32_t* list_of, float* out, hipStream_t st);

// ---- kernels_refine.hip --------------------------------------------------------
// k best of each query's kc candidates by canon distance to the candidates' rows of x
size_t refine_lds_bytes(int d, int k);   // LDS of one workgroup; the launch needs it to fit
void launch_refine(const float* x, int64_t nb, const float* q, int64_t nq, int d, int metric,
                   const int64_t* cand, int kc, int k, float* out_dist, int64_t* out_ids,
                   hipStream_t st);
