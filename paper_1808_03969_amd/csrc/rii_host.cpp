// Host-side, offline parts of the library: codebook training, PQ encoding on the host, and the
// bookkeeping behind reconfigure (sampling, centre update, posting-list construction).
// None of this is on the query path.

#include <algorithm>
#include <cmath>
#include <cstring>
#include <thread>
#include <unordered_set>

#include "rii_internal.h"

namespace {

int host_threads() {
  unsigned n = std::thread::hardware_concurrency();
  if (n == 0) n = 1;
  if (n > 32) n = 32;
  return (int)n;
}

template <typename F>
void parallel_for(int64_t n, F f) {
  int T = host_threads();
  if (n < 2 * T) T = 1;
  std::vector<std::thread> th;
  int64_t per = (n + T - 1) / T;
  for (int t = 0; t < T; ++t) {
    int64_t a = t * per, b = std::min(n, a + per);
    if (a >= b) break;
    th.emplace_back([=] { f(a, b); });
  }
  for (auto& x : th) x.join();
}

// squared distance, coordinates ascending, one rounding per operation
inline float sqdist32(const float* a, const float* b, int Ds) {
  float acc = 0.f;
  for (int j = 0; j < Ds; ++j) {
    float diff = a[j] - b[j];
    float sq = diff * diff;
    acc = acc + sq;
  }
  return acc;
}

inline int nearest_codeword(const float* xs, const float* cbm, int Ks, int Ds) {
  int best = 0;
  float bestd = sqdist32(xs, cbm, Ds);
  for (int z = 1; z < Ks; ++z) {
    float d = sqdist32(xs, cbm + (size_t)z * Ds, Ds);
    if (d < bestd) { bestd = d; best = z; }
  }
  return best;
}

}  // namespace

namespace rii_host {

uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

std::vector<int64_t> sample_without_replacement(int64_t N, int64_t n, uint64_t seed) {
  std::vector<int64_t> out;
  if (n >= N) {
    out.resize(N);
    for (int64_t i = 0; i < N; ++i) out[i] = i;
    return out;
  }
  // Floyd's algorithm: for j = N-n .. N-1 pick t in [0, j]; insert t, or j when t is taken.
  std::unordered_set<int64_t> seen;
  seen.reserve((size_t)n * 2);
  uint64_t ctr = 0;
  for (int64_t j = N - n; j < N; ++j) {
    uint64_t r = mix64(seed * 0x9E3779B97F4A7C15ull + (++ctr));
    int64_t t = (int64_t)(r % (uint64_t)(j + 1));
    if (!seen.insert(t).second) seen.insert(j);
  }
  out.assign(seen.begin(), seen.end());
  std::sort(out.begin(), out.end());
  return out;
}

void update_centres(const uint8_t* sample, int64_t n, const int32_t* assign, const float* sym, int M, int K,
                    uint8_t* coarse) {
  // members of each cell
  std::vector<int64_t> off(K + 1, 0);
  for (int64_t i = 0; i < n; ++i) ++off[assign[i] + 1];
  for (int k = 0; k < K; ++k) off[k + 1] += off[k];
  std::vector<int64_t> order(n), cur(off.begin(), off.end() - 1);
  for (int64_t i = 0; i < n; ++i) order[cur[assign[i]]++] = i;
  parallel_for(K, [&](int64_t k0, int64_t k1) {
    std::vector<int64_t> hist(256);
    std::vector<double> cost(256);
    for (int64_t k = k0; k < k1; ++k) {
      if (off[k + 1] == off[k]) continue;  // empty cell keeps its code
      for (int m = 0; m < M; ++m) {
        std::fill(hist.begin(), hist.end(), 0);
        for (int64_t p = off[k]; p < off[k + 1]; ++p) ++hist[sample[order[p] * M + m]];
        std::fill(cost.begin(), cost.end(), 0.0);
        for (int zp = 0; zp < 256; ++zp) {
          if (!hist[zp]) continue;
          const float* row = sym + ((size_t)m * 256 + zp) * 256;
          for (int z = 0; z < 256; ++z) cost[z] += (double)hist[zp] * (double)row[z];
        }
        int best = 0;
        for (int z = 1; z < 256; ++z)
          if (cost[z] < cost[best]) best = z;
        coarse[k * M + m] = (uint8_t)best;
      }
    }
  });
}

int build_csr(const int32_t* assign, int64_t N, int K, std::vector<int64_t>& off, std::vector<int32_t>& ids) {
  off.assign(K + 1, 0);
  for (int64_t n = 0; n < N; ++n) {
    if (assign[n] < 0 || assign[n] >= K) return RII_ERR_INVALID_ARG;
    ++off[assign[n] + 1];
  }
  for (int k = 0; k < K; ++k) off[k + 1] += off[k];
  ids.resize(N);
  std::vector<int64_t> cur(off.begin(), off.end() - 1);
  for (int64_t n = 0; n < N; ++n) ids[cur[assign[n]]++] = (int32_t)n;
  return RII_OK;
}

}  // namespace rii_host

extern "C" {

const char* rii_status_string(int status) {
  switch (status) {
    case RII_OK: return "ok";
    case RII_ERR_INVALID_ARG: return "invalid argument";
    case RII_ERR_DIM: return "M must divide D and Ks must be 256";
    case RII_ERR_NOT_BUILT: return "index has no coarse centres / posting lists";
    case RII_ERR_UNSORTED_IDS: return "identifiers not sorted / not a permutation";
    case RII_ERR_OOM: return "out of memory";
    case RII_ERR_DEVICE: return "HIP call failed";
    case RII_ERR_UNSUPPORTED: return "size not supported by the kernels";
    default: return "unknown status";
  }
}

int rii_train_codebooks(const float* x, int64_t n, int D, int M, int Ks, int iters, uint64_t seed,
                        float* codebooks_out) {
  if (M <= 0 || D <= 0 || D % M != 0 || Ks != RII_KS) return RII_ERR_DIM;
  if (!x || !codebooks_out || n < Ks || iters < 0) return RII_ERR_INVALID_ARG;
  const int Ds = D / M;
  // initial code words: Ks rows of a seeded sample of the training set (same rows for every sub-space)
  std::vector<int64_t> pick = rii_host::sample_without_replacement(n, Ks, seed);
  for (int m = 0; m < M; ++m)
    for (int z = 0; z < Ks; ++z)
      std::memcpy(codebooks_out + ((size_t)m * Ks + z) * Ds, x + pick[z] * D + m * Ds, sizeof(float) * Ds);
  parallel_for(M, [&](int64_t m0, int64_t m1) {
    std::vector<int> label(n);
    std::vector<double> sum((size_t)Ks * Ds);
    std::vector<int64_t> cnt(Ks);
    for (int64_t m = m0; m < m1; ++m) {
      float* cbm = codebooks_out + (size_t)m * Ks * Ds;
      for (int it = 0; it < iters; ++it) {
        for (int64_t i = 0; i < n; ++i) label[i] = nearest_codeword(x + i * D + m * Ds, cbm, Ks, Ds);
        std::fill(sum.begin(), sum.end(), 0.0);
        std::fill(cnt.begin(), cnt.end(), 0);
        for (int64_t i = 0; i < n; ++i) {
          ++cnt[label[i]];
          for (int j = 0; j < Ds; ++j) sum[(size_t)label[i] * Ds + j] += x[i * D + m * Ds + j];
        }
        for (int z = 0; z < Ks; ++z)
          if (cnt[z])
            for (int j = 0; j < Ds; ++j) cbm[(size_t)z * Ds + j] = (float)(sum[(size_t)z * Ds + j] / (double)cnt[z]);
      }
    }
  });
  return RII_OK;
}

int rii_encode(const float* codebooks, int D, int M, int Ks, const float* x, int64_t n, uint8_t* codes_out) {
  if (M <= 0 || D <= 0 || D % M != 0 || Ks != RII_KS) return RII_ERR_DIM;
  if (!codebooks || n < 0 || (n > 0 && (!x || !codes_out))) return RII_ERR_INVALID_ARG;
  const int Ds = D / M;
  parallel_for(n, [&](int64_t a, int64_t b) {
    for (int64_t i = a; i < b; ++i)
      for (int m = 0; m < M; ++m)
        codes_out[i * M + m] =
            (uint8_t)nearest_codeword(x + i * D + m * Ds, codebooks + (size_t)m * Ks * Ds, Ks, Ds);
  });
  return RII_OK;
}

}  // extern "C"
