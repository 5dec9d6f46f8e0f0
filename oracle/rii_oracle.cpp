// CPU oracle for the Rii search path (product quantisation + ADC + the three search
// algorithms of the paper).  TEST INFRASTRUCTURE ONLY: it exists to check the HIP library and
// to be timed beside it.  It is plain, single-threaded and slow on purpose, shares no code
// with the GPU library, and must never be called by the product path.
//
// Every routine follows the paper's definition step by step:
//   * encode            Sec. 3, Eq. (1): nearest code word per sub-space.
//   * distance table A  Sec. 3: A(m,z) = squared distance between the m-th part of q and the
//                       z-th code word of the m-th codebook.
//   * ADC               Sec. 3, Eq. (2): d_A(q, x)^2 = sum_m A(m, x^m).
//   * PQLinearScan      Sec. 4.2, Alg. 1.
//   * InvertedIndex     Sec. 4.2, Alg. 2, with ceil(K L / |S|) posting lists, capped at K.
//   * Query             Sec. 4.2, Alg. 3 (|S| < theta -> linear scan, else inverted index).
//   * a(n), W_k         Sec. 4.1, Eq. (4): nearest coarse centre under the symmetric distance.
//   * memory model      Sec. 4.1: (N+K) M log2 Z + 32 N bits.
//   * rotation          Sec. 4.5: y = R x before encoding / table building (OPQ variant).
//
// Readings where the paper is silent (all listed in the design document): identifiers are
// 0-based; ties are broken towards the lower index (code word, list number, identifier);
// results are ordered by (distance, identifier); fewer than R candidates -> the tail is
// padded with id -1 / distance +inf; the outer loop of Alg. 2 visits the sorted prefix only.
//
// Precision: the decisions (argmin of Eq. (1), argmin of a(n), ranking) are taken in fp32,
// accumulating in ascending coordinate / sub-space order with no fused multiply-add, which is
// the precision the GPU library takes them in.  The *_f64 entry points evaluate the same
// definitions in double precision and pin the values.
//
// Build: g++ -O2 -ffp-contract=off -shared -fPIC rii_oracle.cpp -o librii_oracle.so

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <utility>
#include <vector>

namespace {

struct Hit {
  float d;
  int32_t id;
};

inline bool hit_less(const Hit& a, const Hit& b) {
  if (a.d != b.d) return a.d < b.d;
  return a.id < b.id;
}

// Squared distance between two Ds-dimensional vectors, coordinates in ascending order.
template <typename T>
T sqdist(const float* a, const float* b, int Ds) {
  T acc = 0;
  for (int j = 0; j < Ds; ++j) {
    T diff = (T)a[j] - (T)b[j];
    T sq = diff * diff;
    acc = acc + sq;
  }
  return acc;
}

// Sec. 3: distance table A in R^{M x Z} for one query.
template <typename T>
void distance_table(const float* cb, int D, int M, int Z, const float* q, T* A) {
  const int Ds = D / M;
  for (int m = 0; m < M; ++m)
    for (int z = 0; z < Z; ++z)
      A[(size_t)m * Z + z] = sqdist<T>(q + m * Ds, cb + ((size_t)m * Z + z) * Ds, Ds);
}

// Eq. (2): sum over the M sub-spaces, m ascending.
template <typename T>
T adc(const T* A, int M, int Z, const uint8_t* code) {
  T d = 0;
  for (int m = 0; m < M; ++m) d = d + A[(size_t)m * Z + code[m]];
  return d;
}

// PartialSort + Take of Alg. 1 / Alg. 2: the R smallest by (distance, id), padded.
void partial_sort_take(std::vector<Hit>& U, int R, int32_t* out_ids, float* out_dist) {
  size_t r = std::min((size_t)R, U.size());
  std::partial_sort(U.begin(), U.begin() + r, U.end(), hit_less);
  for (size_t i = 0; i < r; ++i) {
    out_ids[i] = U[i].id;
    out_dist[i] = U[i].d;
  }
  for (size_t i = r; i < (size_t)R; ++i) {
    out_ids[i] = -1;
    out_dist[i] = std::numeric_limits<float>::infinity();
  }
}

// n in S by binary search on the sorted target identifiers (Sec. 4.2).
bool member(const int32_t* S, int64_t nS, int32_t n) {
  int64_t lo = 0, hi = nS;
  while (lo < hi) {
    int64_t mid = lo + (hi - lo) / 2;
    if (S[mid] < n) lo = mid + 1; else hi = mid;
  }
  return lo < nS && S[lo] == n;
}

}  // namespace

extern "C" {

// Eq. (1).  x [n][D], cb [M][Z][D/M], codes_out [n][M].  Returns 0, or -2 when M does not divide D.
int orc_encode(const float* cb, int D, int M, int Z, const float* x, int64_t n, uint8_t* codes_out) {
  if (M <= 0 || D % M != 0 || Z < 1 || Z > 256) return -2;
  const int Ds = D / M;
  for (int64_t i = 0; i < n; ++i)
    for (int m = 0; m < M; ++m) {
      int best = 0;
      float bestd = sqdist<float>(x + i * D + m * Ds, cb + ((size_t)m * Z) * Ds, Ds);
      for (int z = 1; z < Z; ++z) {
        float d = sqdist<float>(x + i * D + m * Ds, cb + ((size_t)m * Z + z) * Ds, Ds);
        if (d < bestd) { bestd = d; best = z; }
      }
      codes_out[i * M + m] = (uint8_t)best;
    }
  return 0;
}

// Inverse of Eq. (1): concatenate the selected code words.  x_out [n][D].
int orc_decode(const float* cb, int D, int M, int Z, const uint8_t* codes, int64_t n, float* x_out) {
  if (M <= 0 || D % M != 0) return -2;
  const int Ds = D / M;
  for (int64_t i = 0; i < n; ++i)
    for (int m = 0; m < M; ++m)
      std::memcpy(x_out + i * D + m * Ds, cb + ((size_t)m * Z + codes[i * M + m]) * Ds, sizeof(float) * Ds);
  return 0;
}

// Distance table for Q queries.  q [Q][D], lut_out [Q][M][Z].
int orc_lut(const float* cb, int D, int M, int Z, const float* q, int Q, float* lut_out) {
  if (M <= 0 || D % M != 0) return -2;
  for (int i = 0; i < Q; ++i) distance_table<float>(cb, D, M, Z, q + (size_t)i * D, lut_out + (size_t)i * M * Z);
  return 0;
}
int orc_lut_f64(const float* cb, int D, int M, int Z, const float* q, int Q, double* lut_out) {
  if (M <= 0 || D % M != 0) return -2;
  for (int i = 0; i < Q; ++i) distance_table<double>(cb, D, M, Z, q + (size_t)i * D, lut_out + (size_t)i * M * Z);
  return 0;
}

// Eq. (2) for a list of rows (ids == NULL: rows 0..n-1).  One table, dist_out [n].
int orc_adc(const float* lut, int M, int Z, const uint8_t* codes, const int32_t* ids, int64_t n, float* dist_out) {
  for (int64_t i = 0; i < n; ++i) {
    int64_t row = ids ? ids[i] : i;
    dist_out[i] = adc<float>(lut, M, Z, codes + row * M);
  }
  return 0;
}
int orc_adc_f64(const double* lut, int M, int Z, const uint8_t* codes, const int32_t* ids, int64_t n, double* dist_out) {
  for (int64_t i = 0; i < n; ++i) {
    int64_t row = ids ? ids[i] : i;
    dist_out[i] = adc<double>(lut, M, Z, codes + row * M);
  }
  return 0;
}

// Alg. 1 for one query whose table is given.  S == NULL means the whole database.
int orc_linear_scan(const float* lut, int M, int Z, const uint8_t* codes, int64_t N,
                    const int32_t* S, int64_t nS, int R, int32_t* out_ids, float* out_dist) {
  if (R < 1) return -1;
  std::vector<Hit> U;
  int64_t cnt = S ? nS : N;
  U.reserve((size_t)cnt);
  for (int64_t i = 0; i < cnt; ++i) {
    int32_t s = S ? S[i] : (int32_t)i;
    float d = adc<float>(lut, M, Z, codes + (int64_t)s * M);
    U.push_back(Hit{d, s});
  }
  partial_sort_take(U, R, out_ids, out_dist);
  return 0;
}

// Number of posting lists Alg. 2 looks at: ceil(K L / |S|), at most K.
int64_t orc_num_lists(int64_t K, int64_t L, int64_t nS) {
  if (nS <= 0) return K;
  int64_t p = (K * L + nS - 1) / nS;
  if (p > K) p = K;
  if (p < 1) p = 1;
  return p;
}

// First block of Alg. 2: distance of every coarse centre to the query through the table,
// then the P nearest in (d0, k) order.  out_k / out_d0 have P entries.
int orc_coarse_rank(const float* lut, int M, int Z, const uint8_t* coarse, int K, int P,
                    int32_t* out_k, float* out_d0) {
  if (P < 1 || P > K) return -1;
  std::vector<Hit> T;
  T.reserve(K);
  for (int k = 0; k < K; ++k) T.push_back(Hit{adc<float>(lut, M, Z, coarse + (size_t)k * M), k});
  std::partial_sort(T.begin(), T.begin() + P, T.end(), hit_less);
  for (int i = 0; i < P; ++i) {
    out_k[i] = T[i].id;
    if (out_d0) out_d0[i] = T[i].d;
  }
  return 0;
}

// Alg. 2 for one query whose table is given.  P posting lists are visited in (d0, k) order,
// members in stored order; n not in S is skipped (S == NULL: nothing is skipped); with
// Lcap > 0 the traversal stops once Lcap candidates have been scored.  Posting lists are in
// CSR form: list k holds list_ids[list_off[k] .. list_off[k+1]).
int orc_inverted_index(const float* lut, int M, int Z, const uint8_t* codes, int64_t N,
                       const uint8_t* coarse, int K, const int64_t* list_off, const int32_t* list_ids,
                       const int32_t* S, int64_t nS, int P, int64_t Lcap, int R,
                       int32_t* out_ids, float* out_dist, int64_t* scored_out) {
  (void)N;
  if (R < 1 || P < 1 || P > K) return -1;
  std::vector<int32_t> order(P);
  int rc = orc_coarse_rank(lut, M, Z, coarse, K, P, order.data(), nullptr);
  if (rc) return rc;
  std::vector<Hit> U;
  bool full = false;
  for (int i = 0; i < P && !full; ++i) {
    int k = order[i];
    for (int64_t p = list_off[k]; p < list_off[k + 1]; ++p) {
      int32_t n = list_ids[p];
      if (S && !member(S, nS, n)) continue;
      float d = adc<float>(lut, M, Z, codes + (int64_t)n * M);
      U.push_back(Hit{d, n});
      if (Lcap > 0 && (int64_t)U.size() == Lcap) { full = true; break; }
    }
  }
  if (scored_out) *scored_out = (int64_t)U.size();
  partial_sort_take(U, R, out_ids, out_dist);
  return 0;
}

// Alg. 3 for one query vector: builds the table, then branches on |S| < theta.
// S == NULL is the whole database (|S| = N).  The inverted index looks at
// ceil(K L / |S|) lists and stops after L candidates.  mode_out: 0 linear scan, 1 inverted index.
int orc_query(const float* cb, int D, int M, int Z, const float* q,
              const uint8_t* codes, int64_t N, const uint8_t* coarse, int K,
              const int64_t* list_off, const int32_t* list_ids,
              const int32_t* S, int64_t nS, int64_t L, int64_t theta, int R,
              int32_t* out_ids, float* out_dist, int* mode_out) {
  if (M <= 0 || D % M != 0) return -2;
  std::vector<float> A((size_t)M * Z);
  distance_table<float>(cb, D, M, Z, q, A.data());
  int64_t sizeS = S ? nS : N;
  if (sizeS < theta) {
    if (mode_out) *mode_out = 0;
    return orc_linear_scan(A.data(), M, Z, codes, N, S, nS, R, out_ids, out_dist);
  }
  if (mode_out) *mode_out = 1;
  int P = (int)orc_num_lists(K, L, sizeS);
  return orc_inverted_index(A.data(), M, Z, codes, N, coarse, K, list_off, list_ids, S, nS, P, L, R,
                            out_ids, out_dist, nullptr);
}

// Symmetric distance tables: T[m][i][j] = squared distance between code words i and j of
// codebook m (the PQ-code-to-PQ-code distance d_S of Sec. 4.1).  T_out [M][Z][Z].
int orc_sym_table(const float* cb, int D, int M, int Z, float* T_out) {
  if (M <= 0 || D % M != 0) return -2;
  const int Ds = D / M;
  for (int m = 0; m < M; ++m)
    for (int i = 0; i < Z; ++i)
      for (int j = 0; j < Z; ++j)
        T_out[((size_t)m * Z + i) * Z + j] =
            sqdist<float>(cb + ((size_t)m * Z + i) * Ds, cb + ((size_t)m * Z + j) * Ds, Ds);
  return 0;
}

// a(n) = argmin_k d_S(x_n, c_k), lowest k on ties.  assign_out [n].
int orc_assign(const float* T, int M, int Z, const uint8_t* codes, int64_t n,
               const uint8_t* coarse, int K, int32_t* assign_out) {
  for (int64_t i = 0; i < n; ++i) {
    int best = 0;
    float bestd = 0;
    for (int k = 0; k < K; ++k) {
      float d = 0;
      for (int m = 0; m < M; ++m)
        d = d + T[((size_t)m * Z + codes[i * M + m]) * Z + coarse[(size_t)k * M + m]];
      if (k == 0 || d < bestd) { bestd = d; best = k; }
    }
    assign_out[i] = best;
  }
  return 0;
}

// Eq. (4): W_k = { n : a(n) = k }, members ascending, as CSR.  list_off [K+1], list_ids [N].
int orc_build_lists(const int32_t* assign, int64_t N, int K, int64_t* list_off, int32_t* list_ids) {
  std::vector<int64_t> count(K + 1, 0);
  for (int64_t n = 0; n < N; ++n) {
    if (assign[n] < 0 || assign[n] >= K) return -1;
    ++count[assign[n] + 1];
  }
  list_off[0] = 0;
  for (int k = 0; k < K; ++k) list_off[k + 1] = list_off[k] + count[k + 1];
  std::vector<int64_t> cursor(list_off, list_off + K);
  for (int64_t n = 0; n < N; ++n) list_ids[cursor[assign[n]]++] = (int32_t)n;
  return 0;
}

// Sec. 4.5 (OPQ variant): the input vector is first rotated with a pre-trained D x D matrix,
// y = R x; everything after that is plain PQ.  fp32, inner index ascending, no fused
// multiply-add (the rotated vector feeds the arg-min of Eq. (1), so the precision is fixed).
// R [D][D] row-major, x [n][D], y_out [n][D].
int orc_rotate(const float* R, int D, const float* x, int64_t n, float* y_out) {
  for (int64_t i = 0; i < n; ++i)
    for (int r = 0; r < D; ++r) {
      float acc = 0.f;
      for (int c = 0; c < D; ++c) {
        float prod = R[(size_t)r * D + c] * x[i * D + c];
        acc = acc + prod;
      }
      y_out[i * D + r] = acc;
    }
  return 0;
}

// Sec. 4.1: theoretical size of the data structure in bytes for Z = 256.
int64_t orc_index_bytes(int64_t N, int64_t K, int64_t M) { return ((N + K) * M * 8 + 32 * N) / 8; }

}  // extern "C"
