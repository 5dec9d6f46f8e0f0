/*
 * rii.h -- C ABI of the MI355X (gfx950) implementation of the search path of the
 * reconfigurable inverted index ("Rii", Matsui, Hinami, Satoh, ACM MM 2018).
 *
 * The library computes, for a batch of query vectors, product-quantisation asymmetric
 * distances (Sec. 3 of the paper) and the R nearest database items under the three search
 * procedures of Sec. 4.2: PQ-linear-scan over the whole database, PQ-linear-scan over a sorted
 * set of target identifiers (Alg. 1), and the inverted index (Alg. 2), plus the switch between
 * them (Alg. 3).  All online entry points run hand-written HIP kernels; there is no CPU path.
 *
 * Conventions
 *   - Notation follows the paper: D dimension, M sub-spaces, Z = Ks = 256 code words per
 *     sub-space, N database size, K coarse centres / posting lists, R = topk results,
 *     S target identifiers, L number of candidates, theta the switch threshold.
 *   - Identifiers, code values and list numbers are 0-based.  Identifiers are int32
 *     (the paper stores 32-bit identifiers, Sec. 4.1); counts and offsets are int64.
 *   - Every function returns a rii_status (0 = RII_OK, negative = error).  On error nothing
 *     is written to the outputs.  No exception crosses this boundary.
 *   - "host" pointers are ordinary process memory; "device" pointers are HIP device memory
 *     of the current device.  The caller owns every buffer it passes; the index handle owns
 *     only its own device copies.  Arrays are dense, row-major, in the shapes written beside
 *     each argument.
 *   - Online calls are asynchronous on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream); outputs are valid once the stream has been synchronised.  A handle keeps
 *     scratch memory that the online calls reuse, so calls on one handle must be issued on
 *     one stream at a time.  A call that needs more scratch than the handle holds frees and
 *     re-allocates it first, which waits for the device; rii_index_reserve_workspace sizes it
 *     ahead of time.
 *   - Results are ordered by (distance, identifier) ascending; distances are squared
 *     (Eq. (2)), fp32, accumulated over sub-spaces in ascending order.  When fewer than R
 *     candidates exist the tail is filled with identifier -1 and distance +infinity.
 */
#ifndef RII_H
#define RII_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rii_index rii_index_t; /* opaque */

typedef enum {
  RII_OK = 0,
  RII_ERR_INVALID_ARG = -1,  /* NULL required pointer, non-positive count, topk/nprobe out of range */
  RII_ERR_DIM = -2,          /* M does not divide D, or Ks != 256 */
  RII_ERR_NOT_BUILT = -3,    /* inverted-index call on an index without coarse centres / lists */
  RII_ERR_UNSORTED_IDS = -4, /* posting lists or target identifiers violate their precondition */
  RII_ERR_OOM = -5,          /* host or device allocation failed */
  RII_ERR_DEVICE = -6,       /* a HIP call failed */
  RII_ERR_UNSUPPORTED = -7   /* a size beyond what the kernels are built for (see RII_MAX_*) */
} rii_status;

enum { RII_MEM_HOST = 0, RII_MEM_DEVICE = 1 };

#define RII_KS 256          /* Z of the paper: one byte per sub-space (Sec. 3) */
#define RII_MAX_TOPK 1024   /* largest R / nprobe the fused selection handles */
#define RII_MAX_SORT 16384  /* largest K for which rii_coarse_assign can rank all K lists */
#define RII_MAX_M 64        /* largest number of sub-spaces the scan kernels are built for */

/* Human-readable name of a status code. */
const char* rii_status_string(int status);

/* ------------------------------------------------------------------ host, offline ---- */

/* Train the M codebooks of Sec. 3 ("pre-trained code words") by Lloyd's k-means, one
 * sub-space at a time.  The paper does not fix the trainer; this one starts from Ks rows of a
 * seeded permutation of x, runs `iters` assign/update rounds, keeps the previous code word
 * for an empty cell and accumulates means in double precision.
 *   x             host [n][D] fp32, n >= Ks
 *   codebooks_out host [M][Ks][D/M] fp32 (written)
 * Errors: RII_ERR_DIM, RII_ERR_INVALID_ARG (NULL, n < Ks, iters < 0). */
int rii_train_codebooks(const float* x, int64_t n, int D, int M, int Ks, int iters, uint64_t seed,
                        float* codebooks_out);

/* PQ-encode n vectors on the host (Eq. (1)): for each sub-space the index of the nearest code
 * word; squared distances in fp32, coordinates ascending, no fused multiply-add; ties go to
 * the lower index.  Uses all host cores.
 *   codebooks host [M][Ks][D/M], x host [n][D], codes_out host [n][M] uint8 (written) */
int rii_encode(const float* codebooks, int D, int M, int Ks, const float* x, int64_t n, uint8_t* codes_out);

/* ------------------------------------------------------------------ index handle ---- */

/* Create an empty index around the given codebooks (copied to the device).
 *   codebooks host [M][Ks][D/M];  *out receives the handle (destroy with rii_index_destroy). */
int rii_index_create(const float* codebooks, int D, int M, int Ks, rii_index_t** out);

/* Append n PQ codes to the linear code array (the PushBack of Sec. 4.3, "Data addition").
 * New items get identifiers N .. N+n-1.  If posting lists are installed, each new identifier
 * is also pushed to the list of its nearest coarse centre a(n) (Sec. 4.1), keeping every list
 * in ascending identifier order.
 *   codes [n][M] uint8, in host or device memory as `mem` says (RII_MEM_*).
 * Device memory held per code: M bytes, 2 M for M = 32 (which keeps the codes in two layouts, one
 * for sequential and one for gathered scans, unless RII_OPT_GATHER_COPY is 0), plus M + 4 once
 * posting lists are installed (list-ordered copy, identifier); rii_index_info reports the total.
 * Synchronous.  If the codes were stored but re-listing them failed (RII_ERR_OOM, RII_ERR_DEVICE), the
 * index keeps the codes and is left without posting lists. */
int rii_index_add(rii_index_t* index, const uint8_t* codes, int64_t n, int mem);

/* Install coarse centres and posting lists made elsewhere (Sec. 4.1: C and W).
 *   coarse [K][M] uint8 PQ codes; list_offsets [K+1] int64 with list k =
 *   list_ids[list_offsets[k] .. list_offsets[k+1]); list_ids [N] int32, a permutation of
 *   0..N-1, ascending inside each list.  All three in `mem` memory.
 * Also builds the list-ordered copy of the code array that rii_adc_scan_ivf streams.
 * Errors: RII_ERR_INVALID_ARG (K < 1, offsets not 0..N), RII_ERR_UNSORTED_IDS (host inputs
 * only: not a permutation, or a list not ascending).  Synchronous. */
int rii_index_set_lists(rii_index_t* index, const uint8_t* coarse, int K, const int64_t* list_offsets,
                        const int32_t* list_ids, int mem);

/* Given coarse centres, compute a(n) = argmin_k d_S(x_n, c_k) for every stored code on the
 * GPU and build the posting lists W_k = {n : a(n) = k} (Eq. (4)); ties go to the lower k.
 *   coarse host [K][M] uint8.  Synchronous. */
int rii_index_build_lists(rii_index_t* index, const uint8_t* coarse, int K);

/* Reconfigure (Alg. 4): new coarse centres by clustering min(N, 100 K) stored codes directly
 * in code space, then rebuild all posting lists.  The clustering is a stand-in for PQk-means,
 * whose update rule the paper only cites: centres start from K distinct seeded sample codes;
 * each of `iters` rounds assigns the sample by d_S and then sets, per sub-space, the centre's
 * code to the code word minimising the summed d_S to the cell's members; an empty cell keeps
 * its code.  Deterministic for fixed (K, iters, seed).  Synchronous. */
int rii_index_reconfigure(rii_index_t* index, int K, int iters, uint64_t seed);

/* The threshold theta of Alg. 3 (default 0: always the inverted index when lists exist). */
int rii_index_set_threshold(rii_index_t* index, int64_t theta);

/* Options of a handle (rii_index_set_option).  None of them changes any result.
 *   RII_OPT_GATHER_COPY   M = 32 only: 1 (default) keeps the codes a second time as whole 32-byte
 *                         rows, which is what scans over target identifiers gather from (one memory
 *                         line per row); 0 drops that copy (N M bytes less; such scans then gather
 *                         the two halves of a row from the two 16-byte planes the sequential scans
 *                         read).  Must be set before the first rii_index_add. */
enum { RII_OPT_GATHER_COPY = 2 };
int rii_index_set_option(rii_index_t* index, int option, int64_t value);

/* Size the handle's scratch once, so that no later online call has to grow it (growing it frees and
 * allocates device memory, which waits for the device): enough for every online call with at most
 * Q queries, topk results and, for the inverted index, nprobe lists per query (for rii_query:
 * the largest ceil(K L / |S|) any query of a batch can reach, at most K; 0 if the inverted index
 * is not used).  max_targets is accepted for symmetry with the scans and does not change the
 * size.  Call it again after rii_index_add / reconfigure changed N or K.  Synchronous. */
int rii_index_reserve_workspace(rii_index_t* index, int Q, int topk, int64_t max_targets, int nprobe);

/* Choose theta by measurement (Sec. 4.2, "Selection": the threshold is found by running both
 * search methods for several settings when the structure is built and fitting a line).  For
 * target-set sizes |S| = 64, 256, ... up to max_targets (0 = N) this times, on the GPU and for a
 * batch of nq queries (decoded stored codes, seeded choice), the linear scan over S and the
 * inverted index with ceil(K L / |S|) lists, candidate cap L and the target filter; theta is the
 * crossing point of the two timing curves (straight lines in log-log between the bracketing
 * sizes), 0 if the inverted index is never slower, max_targets + 1 if it is never faster.  The
 * value is stored in the index and returned in *theta_out (may be NULL).  It depends on the
 * batch size nq the caller intends to use.  Needs posting lists.  Synchronous. */
int rii_index_calibrate_threshold(rii_index_t* index, int64_t L, int topk, int nq, int64_t max_targets,
                                  uint64_t seed, int64_t* theta_out);

/* info_out[0..7] = N, D, M, Ks, K (0 without lists), theta, bytes of the paper's data
 * structure ((N+K) M + 4 N, Sec. 4.1), device bytes actually held by the handle. */
int rii_index_info(const rii_index_t* index, int64_t* info_out);

/* Copy the coarse centres, posting lists and per-item assignment out of the handle; any
 * output may be NULL.  coarse_out [K][M], list_offsets_out [K+1], list_ids_out [N],
 * assign_out [N] int32, all in `mem` memory.  Synchronous. */
int rii_index_get_lists(const rii_index_t* index, uint8_t* coarse_out, int64_t* list_offsets_out,
                        int32_t* list_ids_out, int32_t* assign_out, int mem);

/* Copy n stored codes starting at identifier `first` out of the handle ([n][M], `mem` memory). */
int rii_index_get_codes(const rii_index_t* index, int64_t first, int64_t n, uint8_t* codes_out, int mem);

void rii_index_destroy(rii_index_t* index);

/* ------------------------------------------------------------------ device, online ---- */

/* Distance tables (Sec. 3, first line of Alg. 1 and Alg. 2):
 * A(m, z) = squared distance between the m-th part of q and code word z of codebook m, fp32,
 * coordinates ascending, no fused multiply-add.
 *   q device [Q][D] fp32;  lut device [Q][M][Ks] fp32 (written). */
int rii_build_lut(const rii_index_t* index, const float* q, int Q, float* lut, void* stream);

/* First block of Alg. 2: d0(k) = sum_m A(m, c_k^m) for the K coarse centres and the nprobe
 * nearest posting lists in (d0, k) order.  nprobe plays the role of ceil(K L / |S|).
 *   lut device [Q][M][Ks]; list_ids device [Q][nprobe] int32 (written);
 *   list_d0 device [Q][nprobe] fp32 or NULL.
 * 1 <= nprobe <= K; nprobe > RII_MAX_TOPK needs K <= RII_MAX_SORT. */
int rii_coarse_assign(const rii_index_t* index, const float* lut, int Q, int nprobe, int32_t* list_ids,
                      float* list_d0, void* stream);

/* Alg. 1 over the whole database (S = {all}): ADC of every stored code (Eq. (2)) and the topk
 * nearest.   ids device [Q][topk] int32, dist device [Q][topk] fp32 (written).
 * 1 <= topk <= RII_MAX_TOPK. */
int rii_adc_scan_linear(const rii_index_t* index, const float* lut, int Q, int topk, int32_t* ids,
                        float* dist, void* stream);

/* Optional check of the precondition the two calls below place on target identifiers (Sec. 4.2:
 * "sorted integers"): inside each query's range strictly increasing and all in [0, N).
 *   target_ids device int32 (may be NULL when every range is empty); target_offsets device [Q+1]
 *   int64, non-decreasing from a non-negative start.
 * Synchronous (waits for the stream).  Returns RII_OK, RII_ERR_UNSORTED_IDS when an identifier
 * breaks the rule, RII_ERR_INVALID_ARG when the offsets do.  Reads nothing beyond
 * target_offsets[Q] identifiers when the offsets are valid. */
int rii_check_target_ids(const rii_index_t* index, const int32_t* target_ids, const int64_t* target_offsets, int Q,
                         void* stream);

/* Alg. 1 over target identifiers: query i scores only the codes whose identifiers are
 * target_ids[target_offsets[i] .. target_offsets[i+1]).
 *   target_ids device int32, strictly increasing inside each query's range, all in [0, N)
 *   (precondition, Sec. 4.2; not checked here, see rii_check_target_ids); target_offsets device
 *   [Q+1] int64;
 *   max_targets: an upper bound on the largest range length (host value; sizes the launch). */
int rii_adc_scan_subset(const rii_index_t* index, const float* lut, int Q, const int32_t* target_ids,
                        const int64_t* target_offsets, int64_t max_targets, int topk, int32_t* ids,
                        float* dist, void* stream);

/* Second block of Alg. 2: visit the given posting lists in the given order, members in stored
 * order, skip identifiers outside the query's target set, score the rest, stop after L
 * candidates, return the topk nearest.
 *   probe_lists device [Q][nprobe] int32 (as written by rii_coarse_assign);
 *   target_ids / target_offsets as in rii_adc_scan_subset, or both NULL for the whole database;
 *   L > 0 caps the number of scored candidates (first L in traversal order), 0 = no cap. */
int rii_adc_scan_ivf(const rii_index_t* index, const float* lut, int Q, const int32_t* probe_lists,
                     int nprobe, const int32_t* target_ids, const int64_t* target_offsets, int64_t L,
                     int topk, int32_t* ids, float* dist, void* stream);

/* PartialSort + Take of Alg. 1 / Alg. 2 on explicit candidates: for segment i =
 * [cand_offsets[i], cand_offsets[i+1]) return the topk smallest by (distance, identifier).
 *   cand_dist device fp32 (any finite values), cand_ids device int32 or NULL (then the
 *   position inside the segment is the identifier); cand_offsets device [Q+1] int64.
 * topk <= RII_MAX_TOPK, or topk <= RII_MAX_SORT when max_segment <= RII_MAX_SORT
 * (max_segment: host upper bound on the segment length, 0 = unknown). */
int rii_topk(const float* cand_dist, const int32_t* cand_ids, const int64_t* cand_offsets, int Q,
             int64_t max_segment, int topk, int32_t* ids, float* dist, void* stream);

/* Alg. 3 for a batch: build the tables, then per query PQ-linear-scan over its target
 * identifiers when |S| < theta, else the inverted index over ceil(K L / |S|) lists (at most
 * K) stopping after L candidates.  target_ids == NULL means the whole database (|S| = N).
 * An index without posting lists always takes the linear scan.
 *   q device [Q][D]; target_ids / target_offsets device (or both NULL); L >= 1;
 *   ids / dist device [Q][topk] (written). */
int rii_query(const rii_index_t* index, const float* q, int Q, int topk, const int32_t* target_ids,
              const int64_t* target_offsets, int64_t max_targets, int64_t L, int32_t* ids, float* dist,
              void* stream);

/* rii_query for callers that cannot allocate device memory while they search: code that runs
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same results and same kernels as rii_query; the scratch (distance tables, per-query plan, probed
 * lists, candidate lists, bounds and counters) is not the handle's but one array of
 * RII_NOALLOC_SCRATCH_BYTES in the library's own device image, which every GPU the library runs
 * on holds until the process ends.  The call makes no hipMalloc / hipFree and no other allocating
 * runtime call.
 *   Returns RII_ERR_UNSUPPORTED when the batch needs more scratch than the array holds (the need
 *   grows with Q (M + topk) and, for the inverted index, Q ceil(K L / |S|)); RII_ERR_INVALID_ARG
 *   when the current device is not the handle's.
 *   All calls on one GPU share that array, which keeps the last call's contents (the kernels
 *   clear what has to start from zero): two calls that overlap on one GPU -- different streams,
 *   different handles, different threads -- race.  Issue them on one stream. */
#define RII_NOALLOC_SCRATCH_BYTES (64 * 1024 * 1024)
int rii_query_noalloc(const rii_index_t* index, const float* q, int Q, int topk, const int32_t* target_ids,
                      const int64_t* target_offsets, int64_t max_targets, int64_t L, int32_t* ids, float* dist,
                      void* stream);

/* ------------------------------------------------------------------ device, offline ---- */

/* Eq. (1) on the GPU, bit-identical to rii_encode.
 *   x device [n][D] fp32; codes_out device [n][M] uint8 (written). */
int rii_encode_device(const rii_index_t* index, const float* x, int64_t n, uint8_t* codes_out, void* stream);

/* Rotation of the OPQ variant (Sec. 4.5): y = R x for every row, applied to database vectors
 * before rii_encode_device and to queries before rii_build_lut / rii_query; everything after it
 * is plain PQ.  The matrix is pre-trained elsewhere.  fp32, inner index ascending, no fused
 * multiply-add (bit-identical on host and GPU, because the result feeds the arg-min of Eq. (1)).
 *   R device [D][D] row-major; x device [n][D]; y device [n][D] (written; must not alias x). */
int rii_rotate(const float* R, int D, const float* x, int64_t n, float* y, void* stream);

/* a(n) of Sec. 4.1 for arbitrary codes under explicit coarse centres.
 *   codes device [n][M]; coarse device [K][M]; assign_out device [n] int32 (written). */
int rii_assign(const rii_index_t* index, const uint8_t* codes, int64_t n, const uint8_t* coarse, int K,
               int32_t* assign_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RII_H */
