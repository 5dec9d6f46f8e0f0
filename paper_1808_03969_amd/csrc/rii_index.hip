// The index handle: device copies of the Rii data structure (Sec. 4.1: linear code array,
// coarse centres as PQ codes, posting lists of identifiers), data addition and reconfigure
// (Sec. 4.3, Alg. 4).  Everything here is offline and synchronous.

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <unordered_set>
#include <string>
#include <vector>

#include "rii_internal.h"
#include "rii_bench.h"

extern "C" int rii_internal_sym_table(const rii_index* idx, hipStream_t st);
extern "C" int rii_internal_assign(const rii_index* idx, const uint8_t* codes, int64_t n, int64_t rot_base, int64_t plane,
                                   const uint8_t* coarse, int K, int32_t* assign_out, hipStream_t st);
extern "C" int rii_internal_assign_pruned(const rii_index* idx, const uint8_t* codes, int64_t n, int64_t rot_base,
                                          int64_t plane,
                                          const uint8_t* super, int G, const float* radius, const uint8_t* coarse_g,
                                          const int32_t* perm_g, const int32_t* group_off, int32_t* assign_out,
                                          unsigned long long* visited_total, hipStream_t st);
extern "C" int rii_internal_assign_from_lists(const rii_index* idx, int32_t* d_out, hipStream_t st);
extern "C" int rii_internal_spread_ids(int32_t* ids, int64_t* offsets, int nq, int64_t S, int64_t N, hipStream_t st);
extern "C" int rii_internal_copy_rows(const uint8_t* in, int64_t in_rot, int64_t in_plane, const int32_t* ids,
                                      int64_t n, int M, uint8_t* out, int64_t out_rot, int64_t out_plane,
                                      hipStream_t st);

namespace {

constexpr int kCounters = 8;  // entries of rii_index::d_scan_counters (ScanArgs::counters)

// byte distance between the two planes of a stored array of `rows` rows (see rii_index)
int64_t plane_for(int M, int64_t rows) { return M == 32 ? rows * 16 : 0; }

template <typename T>
void free_dev(T*& p) {
  if (p) (void)hipFree(p);
  p = nullptr;
}

void drop_lists(rii_index* idx) {
  free_dev(idx->d_coarse);
  free_dev(idx->d_coarse_st);
  free_dev(idx->d_list_off);
  free_dev(idx->d_list_ids);
  free_dev(idx->d_codes_list);
  idx->h_coarse.clear();
  idx->h_list_off.clear();
  idx->K = 0;
  idx->max_list_len = 0;
}

// Install lists given on the host (already validated) plus the per-item assignment.
int install_lists(rii_index* idx, const uint8_t* coarse, int K, const std::vector<int64_t>& off,
                  const std::vector<int32_t>& ids, const std::vector<int32_t>& assign) {
  const int64_t N = idx->N;
  const int M = idx->M;
  drop_lists(idx);
  RII_HIP(hipMalloc(&idx->d_coarse, (size_t)K * M));
  RII_HIP(hipMalloc(&idx->d_coarse_st, (size_t)K * M));
  RII_HIP(hipMalloc(&idx->d_list_off, (size_t)(K + 1) * 8));
  RII_HIP(hipMalloc(&idx->d_list_ids, std::max<size_t>((size_t)N * 4, 4)));
  RII_HIP(hipMalloc(&idx->d_codes_list, std::max<size_t>((size_t)N * M, 16)));
  RII_HIP(hipMemcpy(idx->d_coarse, coarse, (size_t)K * M, hipMemcpyHostToDevice));
  idx->plane_coarse = plane_for(M, K);
  idx->plane_list = plane_for(M, N);
  int rc = rii_internal_copy_rows(idx->d_coarse, -1, 0, nullptr, K, M, idx->d_coarse_st, 0, idx->plane_coarse, nullptr);
  if (rc) return rc;
  RII_HIP(hipMemcpy(idx->d_list_off, off.data(), (size_t)(K + 1) * 8, hipMemcpyHostToDevice));
  if (N > 0) {
    RII_HIP(hipMemcpy(idx->d_list_ids, ids.data(), (size_t)N * 4, hipMemcpyHostToDevice));
    // row p of the list-ordered copy = code of identifier list_ids[p], stored form (rotated by p)
    rc = rii_internal_copy_rows(idx->d_codes, 0, idx->plane_codes, idx->d_list_ids, N, M, idx->d_codes_list, 0,
                                idx->plane_list, nullptr);
    if (rc) return rc;
  }
  RII_HIP(hipDeviceSynchronize());
  idx->h_coarse.assign(coarse, coarse + (size_t)K * M);
  idx->h_list_off = off;
  idx->K = K;
  idx->max_list_len = 0;
  for (int k = 0; k < K; ++k) idx->max_list_len = std::max(idx->max_list_len, off[k + 1] - off[k]);
  return RII_OK;
}

// Grouping of the coarse centres used to prune the search for a(n) when K is large.
struct CentreGroups {
  int G = 0;
  uint8_t* d_super = nullptr;    // [G][M]
  float* d_radius = nullptr;     // [G]
  uint8_t* d_coarse_g = nullptr; // [K][M] centres, group after group
  int32_t* d_perm_g = nullptr;   // [K] original centre number of each row of d_coarse_g
  int32_t* d_group_off = nullptr;  // [G+1]
  ~CentreGroups() {
    free_dev(d_super); free_dev(d_radius); free_dev(d_coarse_g); free_dev(d_perm_g); free_dev(d_group_off);
  }
};

constexpr int kPruneMinK = 1024;

// Cluster the K coarse codes into G groups in code space (three rounds of the same clustering
// reconfigure uses) and record each group's radius under d_S.
int make_groups(rii_index* idx, const uint8_t* coarse, int K, CentreGroups& g) {
  const int M = idx->M;
  int G = K / 8;
  if (G < 64) G = 64;
  if (G > 2048) G = 2048;
  if (G > K) G = K;
  g.G = G;
  int rc = rii_internal_sym_table(idx, nullptr);
  if (rc) return rc;
  std::vector<float> sym((size_t)M * 256 * 256);
  RII_HIP(hipDeviceSynchronize());
  RII_HIP(hipMemcpy(sym.data(), idx->d_sym, sym.size() * 4, hipMemcpyDeviceToHost));
  // initial super-centres: the first G distinct coarse codes in a fixed pseudo-random order
  std::vector<int> order(K);
  for (int k = 0; k < K; ++k) order[k] = k;
  std::sort(order.begin(), order.end(), [&](int a, int b) {
    uint64_t ha = rii_host::mix64(0x5eedULL + (uint64_t)a), hb = rii_host::mix64(0x5eedULL + (uint64_t)b);
    return ha != hb ? ha < hb : a < b;
  });
  std::vector<uint8_t> super((size_t)G * M);
  {
    std::unordered_set<std::string> seen;
    int got = 0;
    for (int i = 0; i < K && got < G; ++i) {
      std::string key(reinterpret_cast<const char*>(coarse + (size_t)order[i] * M), M);
      if (seen.insert(key).second) std::memcpy(&super[(size_t)got++ * M], key.data(), M);
    }
    for (int i = 0; got < G; ++i, ++got) std::memcpy(&super[(size_t)got * M], coarse + (size_t)order[i % K] * M, M);
  }
  uint8_t* d_coarse = nullptr;
  int32_t* d_ga = nullptr;
  RII_HIP(hipMalloc(&d_coarse, (size_t)K * M));
  RII_HIP(hipMalloc(&d_ga, (size_t)K * 4));
  RII_HIP(hipMalloc(&g.d_super, (size_t)G * M));
  RII_HIP(hipMemcpy(d_coarse, coarse, (size_t)K * M, hipMemcpyHostToDevice));
  std::vector<int32_t> ga(K);
  for (int it = 0; it < 4; ++it) {
    RII_HIP(hipMemcpy(g.d_super, super.data(), super.size(), hipMemcpyHostToDevice));
    rc = rii_assign(idx, d_coarse, K, g.d_super, G, d_ga, nullptr);
    if (rc) break;
    RII_HIP(hipMemcpy(ga.data(), d_ga, (size_t)K * 4, hipMemcpyDeviceToHost));
    if (it < 3) rii_host::update_centres(coarse, K, ga.data(), sym.data(), M, G, super.data());
  }
  (void)hipFree(d_coarse);
  (void)hipFree(d_ga);
  if (rc) return rc;
  std::vector<float> radius(G, 0.f);
  for (int k = 0; k < K; ++k) {
    double d = 0;
    for (int m = 0; m < M; ++m)
      d += sym[((size_t)m * 256 + coarse[(size_t)k * M + m]) * 256 + super[(size_t)ga[k] * M + m]];
    float r = (float)(std::sqrt(d) * 1.000001);
    if (r > radius[ga[k]]) radius[ga[k]] = r;
  }
  std::vector<int64_t> off64;
  std::vector<int32_t> perm;
  rc = rii_host::build_csr(ga.data(), K, G, off64, perm);
  if (rc) return rc;
  std::vector<int32_t> off(off64.begin(), off64.end());
  std::vector<uint8_t> coarse_g((size_t)K * M);
  for (int p = 0; p < K; ++p) std::memcpy(&coarse_g[(size_t)p * M], coarse + (size_t)perm[p] * M, M);
  RII_HIP(hipMalloc(&g.d_radius, (size_t)G * 4));
  RII_HIP(hipMalloc(&g.d_coarse_g, (size_t)K * M));
  RII_HIP(hipMalloc(&g.d_perm_g, (size_t)K * 4));
  RII_HIP(hipMalloc(&g.d_group_off, (size_t)(G + 1) * 4));
  RII_HIP(hipMemcpy(g.d_radius, radius.data(), (size_t)G * 4, hipMemcpyHostToDevice));
  RII_HIP(hipMemcpy(g.d_coarse_g, coarse_g.data(), coarse_g.size(), hipMemcpyHostToDevice));
  RII_HIP(hipMemcpy(g.d_perm_g, perm.data(), (size_t)K * 4, hipMemcpyHostToDevice));
  RII_HIP(hipMemcpy(g.d_group_off, off.data(), (size_t)(G + 1) * 4, hipMemcpyHostToDevice));
  return RII_OK;
}

// a(n) for n device-resident codes `rows` under the host coarse centres `coarse`; the result
// stays on the device (d_out, n entries).  rot_base >= 0: `rows` is the base of a stored array with
// planes `plane` apart and the items are its rows rot_base..; rot_base < 0: plain codes.  Brute
// force for small K, pruned search (same result) for large K.
int assign_rows_dev(rii_index* idx, const uint8_t* rows, int64_t n, int64_t rot_base, int64_t plane,
                    const uint8_t* coarse, int K, int32_t* d_out) {
  if (n == 0) return RII_OK;
  if (K >= kPruneMinK) {
    CentreGroups g;
    int rc = make_groups(idx, coarse, K, g);
    if (rc) return rc;
    rc = rii_internal_assign_pruned(idx, rows, n, rot_base, plane, g.d_super, g.G, g.d_radius, g.d_coarse_g, g.d_perm_g,
                                    g.d_group_off, d_out, nullptr, nullptr);
    if (rc) return rc;
    RII_HIP(hipDeviceSynchronize());
    return RII_OK;
  }
  uint8_t* d_coarse = nullptr;
  RII_HIP(hipMalloc(&d_coarse, (size_t)K * idx->M));
  int rc = RII_OK;
  if (hipMemcpy(d_coarse, coarse, (size_t)K * idx->M, hipMemcpyHostToDevice) != hipSuccess) rc = RII_ERR_DEVICE;
  if (!rc) rc = rii_internal_assign(idx, rows, n, rot_base, plane, d_coarse, K, d_out, nullptr);
  if (!rc && hipDeviceSynchronize() != hipSuccess) rc = RII_ERR_DEVICE;
  (void)hipFree(d_coarse);
  return rc;
}

int assign_stored(rii_index* idx, int64_t first, int64_t n, const uint8_t* coarse, int K, int32_t* assign_host) {
  if (n == 0) return RII_OK;
  int32_t* d_out = nullptr;
  RII_HIP(hipMalloc(&d_out, (size_t)n * 4));
  int rc = assign_rows_dev(idx, idx->d_codes, n, first, idx->plane_codes, coarse, K, d_out);
  if (!rc && hipMemcpy(assign_host, d_out, (size_t)n * 4, hipMemcpyDeviceToHost) != hipSuccess) rc = RII_ERR_DEVICE;
  (void)hipFree(d_out);
  return rc;
}

// helpers of the threshold calibration

struct DevBuf {
  void* p = nullptr;
  ~DevBuf() {
    if (p) (void)hipFree(p);
  }
  int alloc(size_t bytes) {
    if (hipMalloc(&p, bytes ? bytes : 16) == hipSuccess) return RII_OK;
    (void)hipGetLastError();
    return RII_ERR_OOM;
  }
  template <typename T>
  T* as() { return static_cast<T*>(p); }
};

// median of three timed runs of f() in milliseconds (f launches on the default stream)
template <typename F>
int time_ms(F f, double* out) {
  hipEvent_t a, b;
  RII_HIP(hipEventCreate(&a));
  RII_HIP(hipEventCreate(&b));
  float t[3] = {0.f, 0.f, 0.f};
  int rc = f();  // warm-up (also sizes the scratch)
  for (int i = 0; i < 3 && !rc; ++i) {
    RII_HIP(hipEventRecord(a, nullptr));
    rc = f();
    RII_HIP(hipEventRecord(b, nullptr));
    RII_HIP(hipEventSynchronize(b));
    RII_HIP(hipEventElapsedTime(&t[i], a, b));
  }
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  if (rc) return rc;
  std::sort(t, t + 3);
  *out = t[1];
  return RII_OK;
}

}  // namespace

extern "C" {

int rii_index_create(const float* codebooks, int D, int M, int Ks, rii_index_t** out) {
  if (!out) return RII_ERR_INVALID_ARG;
  if (M <= 0 || D <= 0 || D % M != 0 || Ks != RII_KS) return RII_ERR_DIM;
  if (!codebooks) return RII_ERR_INVALID_ARG;
  rii_index* idx = new (std::nothrow) rii_index();
  if (!idx) return RII_ERR_OOM;
  idx->D = D; idx->M = M; idx->Ks = Ks; idx->Ds = D / M;
  if (hipGetDevice(&idx->device) != hipSuccess) {
    (void)hipGetLastError();
    delete idx;
    return RII_ERR_DEVICE;
  }
  size_t bytes = (size_t)M * Ks * idx->Ds * sizeof(float);
  if (hipMalloc(&idx->d_cb, bytes) != hipSuccess ||
      hipMemcpy(idx->d_cb, codebooks, bytes, hipMemcpyHostToDevice) != hipSuccess) {
    (void)hipGetLastError();
    rii_index_destroy(idx);
    return RII_ERR_DEVICE;
  }
  idx->h_cb.assign(codebooks, codebooks + (size_t)M * Ks * idx->Ds);
  *out = idx;
  return RII_OK;
}

void rii_index_destroy(rii_index_t* idx) {
  if (!idx) return;
  drop_lists(idx);
  free_dev(idx->d_cb);
  free_dev(idx->d_sym);
  free_dev(idx->d_codes);
  idx->d_codes_rows = nullptr;  // part of the same allocation
  if (idx->ws) (void)hipFree(idx->ws);
  if (idx->d_scan_counters) (void)hipFree(idx->d_scan_counters);
  delete idx;
}

int rii_index_set_threshold(rii_index_t* idx, int64_t theta) {
  if (!idx) return RII_ERR_INVALID_ARG;
  idx->theta = theta;
  return RII_OK;
}

int rii_index_set_scan_events(rii_index_t* idx, void* start_event, void* stop_event) {
  if (!idx || ((start_event == nullptr) != (stop_event == nullptr))) return RII_ERR_INVALID_ARG;
  if (start_event && !idx->d_scan_counters) {
    RII_HIP(hipMalloc(&idx->d_scan_counters, kCounters * sizeof(unsigned long long)));
    RII_HIP(hipMemset(idx->d_scan_counters, 0, kCounters * sizeof(unsigned long long)));
  }
  idx->ev_start = start_event;
  idx->ev_stop = stop_event;
  return RII_OK;
}

int rii_index_read_scan_counters(rii_index_t* idx, uint64_t* counters_out) {
  if (!idx || !counters_out) return RII_ERR_INVALID_ARG;
  for (int i = 0; i < kCounters; ++i) counters_out[i] = 0;
  if (!idx->d_scan_counters) return RII_OK;
  unsigned long long h[kCounters] = {};
  RII_HIP(hipMemcpy(h, idx->d_scan_counters, sizeof(h), hipMemcpyDeviceToHost));  // waits for earlier work
  RII_HIP(hipMemset(idx->d_scan_counters, 0, sizeof(h)));
  for (int i = 0; i < kCounters; ++i) counters_out[i] = h[i];
  return RII_OK;
}

int rii_index_set_option(rii_index_t* idx, int option, int64_t value) {
  if (!idx) return RII_ERR_INVALID_ARG;
  switch (option) {
    case RII_OPT_GATHER_COPY:
      if (value != 0 && value != 1) return RII_ERR_INVALID_ARG;
      if (idx->cap > 0 && (value != 0) != idx->keep_rows_copy) return RII_ERR_INVALID_ARG;  // layout is fixed once codes are stored
      idx->keep_rows_copy = value != 0;
      return RII_OK;
    default:
      return RII_ERR_INVALID_ARG;
  }
}

// ---- threshold calibration (Sec. 4.2, "Selection")
int rii_index_calibrate_threshold(rii_index_t* idx, int64_t L, int topk, int nq, int64_t max_targets, uint64_t seed,
                                  int64_t* theta_out) {
  if (!idx || L < 1 || topk < 1 || topk > RII_MAX_TOPK || nq < 1 || nq > 1024) return RII_ERR_INVALID_ARG;
  if (idx->K < 1) return RII_ERR_NOT_BUILT;
  if (idx->N < 2 || idx->h_cb.size() != (size_t)idx->M * 256 * idx->Ds) return RII_ERR_INVALID_ARG;
  const int64_t N = idx->N;
  const int M = idx->M, D = idx->D, Ds = idx->Ds, K = idx->K;
  if (L > N) L = N;  // a cap of N or more never cuts anything, and K * L stays far from overflow
  if (max_targets <= 0 || max_targets > N) max_targets = N;
  // queries: decoded stored codes (vectors the index can certainly answer), seeded choice
  std::vector<int64_t> rows = rii_host::sample_without_replacement(N, std::min<int64_t>(nq, N), seed);
  std::vector<float> q((size_t)nq * D);
  {
    std::vector<uint8_t> code(M);
    for (int i = 0; i < nq; ++i) {
      int rc = rii_index_get_codes(idx, rows[i % rows.size()], 1, code.data(), RII_MEM_HOST);
      if (rc) return rc;
      for (int m = 0; m < M; ++m)
        std::memcpy(&q[(size_t)i * D + m * Ds], &idx->h_cb[((size_t)m * 256 + code[m]) * Ds], sizeof(float) * Ds);
    }
  }
  std::vector<int64_t> sizes;
  for (int64_t s = 64; s < max_targets; s *= 4) sizes.push_back(s);
  sizes.push_back(max_targets);
  DevBuf d_q, d_lut, d_tid, d_off, d_probe, d_ids, d_dist;
  int rc = d_q.alloc((size_t)nq * D * 4);
  if (!rc) rc = d_lut.alloc((size_t)nq * M * 256 * 4);
  if (!rc) rc = d_tid.alloc((size_t)nq * max_targets * 4);
  if (!rc) rc = d_off.alloc((size_t)(nq + 1) * 8);
  if (!rc) rc = d_probe.alloc((size_t)nq * K * 4);
  if (!rc) rc = d_ids.alloc((size_t)nq * topk * 4);
  if (!rc) rc = d_dist.alloc((size_t)nq * topk * 4);
  if (rc) return rc;
  RII_HIP(hipMemcpy(d_q.p, q.data(), q.size() * 4, hipMemcpyHostToDevice));
  rc = rii_build_lut(idx, d_q.as<float>(), nq, d_lut.as<float>(), nullptr);
  if (rc) return rc;
  // time both branches of Alg. 3 on every size
  std::vector<double> t_lin(sizes.size()), t_ivf(sizes.size());
  for (size_t g = 0; g < sizes.size(); ++g) {
    const int64_t S = sizes[g];
    rc = rii_internal_spread_ids(d_tid.as<int32_t>(), d_off.as<int64_t>(), nq, S, N, nullptr);
    if (rc) return rc;
    int64_t p64 = ((int64_t)K * L + S - 1) / S;
    const int P = (int)std::min<int64_t>(std::max<int64_t>(p64, 1), K);
    if (P > RII_MAX_TOPK && K > RII_MAX_SORT) return RII_ERR_UNSUPPORTED;
    rc = time_ms([&] {
      return rii_adc_scan_subset(idx, d_lut.as<float>(), nq, d_tid.as<int32_t>(), d_off.as<int64_t>(), S, topk,
                                 d_ids.as<int32_t>(), d_dist.as<float>(), nullptr);
    }, &t_lin[g]);
    if (rc) return rc;
    rc = time_ms([&] {
      int r2 = rii_coarse_assign(idx, d_lut.as<float>(), nq, P, d_probe.as<int32_t>(), nullptr, nullptr);
      if (r2) return r2;
      return rii_adc_scan_ivf(idx, d_lut.as<float>(), nq, d_probe.as<int32_t>(), P, d_tid.as<int32_t>(),
                              d_off.as<int64_t>(), L, topk, d_ids.as<int32_t>(), d_dist.as<float>(), nullptr);
    }, &t_ivf[g]);
    if (rc) return rc;
  }
  // theta = the size from which the inverted index is the faster branch: the crossing point of
  // the two timing curves, each taken as a straight line in (log |S|, log t) between the two
  // grid sizes that bracket the crossing
  int64_t theta;
  size_t g = 0;
  while (g < sizes.size() && t_ivf[g] > t_lin[g]) ++g;
  if (g == 0) {
    theta = 0;                       // the inverted index wins everywhere
  } else if (g == sizes.size()) {
    theta = max_targets + 1;         // the linear scan wins on the whole grid
  } else {
    const double x0 = std::log((double)sizes[g - 1]), x1 = std::log((double)sizes[g]);
    const double a0 = std::log(t_lin[g - 1]) - std::log(t_ivf[g - 1]);  // > 0: linear scan faster... sign below
    const double a1 = std::log(t_lin[g]) - std::log(t_ivf[g]);
    // difference d(x) = log t_lin - log t_ivf is negative at x0 (linear faster) and >= 0 at x1
    double x = a1 == a0 ? x1 : x0 + (0.0 - a0) * (x1 - x0) / (a1 - a0);
    if (x < x0) x = x0;
    if (x > x1) x = x1;
    theta = (int64_t)std::llround(std::exp(x));
  }
  idx->theta = theta;
  if (theta_out) *theta_out = theta;
  return RII_OK;
}

int rii_index_info(const rii_index_t* idx, int64_t* info) {
  if (!idx || !info) return RII_ERR_INVALID_ARG;
  const int64_t N = idx->N, M = idx->M, K = idx->K;
  info[0] = N; info[1] = idx->D; info[2] = M; info[3] = idx->Ks; info[4] = K; info[5] = idx->theta;
  info[6] = (N + K) * M + 4 * N;
  int64_t dev = (int64_t)M * 256 * idx->Ds * 4 + idx->cap * M * (idx->d_codes_rows != idx->d_codes ? 2 : 1) + (int64_t)idx->ws_bytes;
  if (idx->d_sym) dev += M * 256 * 256 * 4;
  if (K > 0) dev += 2 * K * M + (K + 1) * 8 + N * 4 /*ids*/ + N * M /*list-ordered codes*/;
  info[7] = dev;
  return RII_OK;
}

int rii_index_add(rii_index_t* idx, const uint8_t* codes, int64_t n, int mem) {
  if (!idx || n < 0 || (n > 0 && !codes) || (mem != RII_MEM_HOST && mem != RII_MEM_DEVICE)) return RII_ERR_INVALID_ARG;
  if (idx->M % 4 != 0) return RII_ERR_UNSUPPORTED;
  if (n == 0) return RII_OK;
  if (idx->N + n > 2147483647LL) return RII_ERR_UNSUPPORTED;
  const int M = idx->M;
  if (idx->N + n > idx->cap) {
    int64_t ncap = std::max<int64_t>(idx->N + n, idx->cap + idx->cap / 2);
    uint8_t* nb = nullptr;
    // (M = 32 keeps the codes twice, as two planes and -- unless switched off -- as whole rows:
    // one allocation, rows last)
    const bool rows_copy = plane_for(M, 1) && idx->keep_rows_copy;
    const size_t copies = rows_copy ? 2 : 1;
    if (hipMalloc(&nb, copies * (size_t)ncap * M) != hipSuccess) {
      (void)hipGetLastError();
      ncap = idx->N + n;
      RII_HIP(hipMalloc(&nb, copies * (size_t)ncap * M));
    }
    const int64_t nplane = plane_for(M, ncap);
    if (idx->N > 0) {
      if (nplane) {  // each plane holds 16 bytes a row
        RII_HIP(hipMemcpy(nb, idx->d_codes, (size_t)idx->N * 16, hipMemcpyDeviceToDevice));
        RII_HIP(hipMemcpy(nb + nplane, idx->d_codes + idx->plane_codes, (size_t)idx->N * 16, hipMemcpyDeviceToDevice));
        if (rows_copy) RII_HIP(hipMemcpy(nb + (size_t)ncap * M, idx->d_codes_rows, (size_t)idx->N * M, hipMemcpyDeviceToDevice));
      } else {
        RII_HIP(hipMemcpy(nb, idx->d_codes, (size_t)idx->N * M, hipMemcpyDeviceToDevice));
      }
    }
    free_dev(idx->d_codes);
    idx->d_codes = nb;
    idx->cap = ncap;
    idx->plane_codes = nplane;
    idx->d_codes_rows = rows_copy ? nb + (size_t)ncap * M : nb;
    idx->plane_rows = rows_copy ? 0 : nplane;
  }
  {
    // bring the new rows into stored form (row r rotated by r bytes when M is 8, 16 or 32)
    const uint8_t* src = codes;
    uint8_t* stage = nullptr;
    if (mem == RII_MEM_HOST) {
      RII_HIP(hipMalloc(&stage, (size_t)n * M));
      if (hipMemcpy(stage, codes, (size_t)n * M, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(stage);
        return RII_ERR_DEVICE;
      }
      src = stage;
    }
    int rc = rii_internal_copy_rows(src, -1, 0, nullptr, n, M, idx->d_codes, idx->N, idx->plane_codes, nullptr);
    if (!rc && idx->d_codes_rows != idx->d_codes)
      rc = rii_internal_copy_rows(src, -1, 0, nullptr, n, M, idx->d_codes_rows, idx->N, 0, nullptr);
    if (!rc && hipDeviceSynchronize() != hipSuccess) rc = RII_ERR_DEVICE;
    if (stage) (void)hipFree(stage);
    if (rc) return rc;
  }
  const int64_t oldN = idx->N;
  idx->N += n;
  if (idx->K > 0) {
    // push every new identifier to the list of its nearest coarse centre; lists stay ascending
    // because new identifiers are larger than all stored ones
    std::vector<int32_t> assign(idx->N);
    if (oldN > 0) {  // a(n) of the items stored so far, read back from the lists (it is not kept)
      idx->N = oldN;
      DevBuf d_old;
      int rc0 = d_old.alloc((size_t)oldN * 4);
      if (!rc0) rc0 = rii_internal_assign_from_lists(idx, d_old.as<int32_t>(), nullptr);
      if (!rc0 && hipMemcpy(assign.data(), d_old.p, (size_t)oldN * 4, hipMemcpyDeviceToHost) != hipSuccess) rc0 = RII_ERR_DEVICE;
      idx->N = oldN + n;
      if (rc0) {
        (void)hipGetLastError();
        drop_lists(idx);
        return rc0;
      }
    }
    std::vector<uint8_t> coarse = idx->h_coarse;
    const int K = idx->K;
    // (from here on a failure leaves the index without posting lists rather than with lists
    // that are shorter than the code array)
    int rc = assign_stored(idx, oldN, n, coarse.data(), K, assign.data() + oldN);
    std::vector<int64_t> off;
    std::vector<int32_t> ids;
    if (!rc) rc = rii_host::build_csr(assign.data(), idx->N, K, off, ids);
    if (!rc) rc = install_lists(idx, coarse.data(), K, off, ids, assign);
    if (rc) drop_lists(idx);
    return rc;
  }
  return RII_OK;
}

int rii_index_set_lists(rii_index_t* idx, const uint8_t* coarse, int K, const int64_t* list_offsets,
                        const int32_t* list_ids, int mem) {
  if (!idx || !coarse || !list_offsets || K < 1 || (mem != RII_MEM_HOST && mem != RII_MEM_DEVICE))
    return RII_ERR_INVALID_ARG;
  const int64_t N = idx->N;
  if (N > 0 && !list_ids) return RII_ERR_INVALID_ARG;
  std::vector<uint8_t> hc((size_t)K * idx->M);
  std::vector<int64_t> off(K + 1);
  std::vector<int32_t> ids(N);
  hipMemcpyKind kind = mem == RII_MEM_HOST ? hipMemcpyHostToHost : hipMemcpyDeviceToHost;
  RII_HIP(hipMemcpy(hc.data(), coarse, hc.size(), kind));
  RII_HIP(hipMemcpy(off.data(), list_offsets, (size_t)(K + 1) * 8, kind));
  if (N > 0) RII_HIP(hipMemcpy(ids.data(), list_ids, (size_t)N * 4, kind));
  if (off[0] != 0 || off[K] != N) return RII_ERR_INVALID_ARG;
  std::vector<int32_t> assign(N, -1);
  for (int k = 0; k < K; ++k) {
    if (off[k + 1] < off[k]) return RII_ERR_INVALID_ARG;
    for (int64_t p = off[k]; p < off[k + 1]; ++p) {
      int32_t n = ids[p];
      if (n < 0 || n >= N || assign[n] != -1) return RII_ERR_UNSORTED_IDS;
      if (p > off[k] && ids[p - 1] >= n) return RII_ERR_UNSORTED_IDS;
      assign[n] = k;
    }
  }
  return install_lists(idx, hc.data(), K, off, ids, assign);
}

int rii_index_build_lists(rii_index_t* idx, const uint8_t* coarse, int K) {
  if (!idx || !coarse || K < 1) return RII_ERR_INVALID_ARG;
  std::vector<int32_t> assign(idx->N);
  int rc = assign_stored(idx, 0, idx->N, coarse, K, assign.data());
  if (rc) return rc;
  std::vector<int64_t> off;
  std::vector<int32_t> ids;
  rc = rii_host::build_csr(assign.data(), idx->N, K, off, ids);
  if (rc) return rc;
  return install_lists(idx, coarse, K, off, ids, assign);
}

int rii_index_reconfigure(rii_index_t* idx, int K, int iters, uint64_t seed) {
  if (!idx || K < 1 || iters < 0 || idx->N < K) return RII_ERR_INVALID_ARG;
  const int M = idx->M;
  const int64_t N = idx->N;
  // sample of at most min(N, 100 K) stored codes (Sec. 4.3)
  const int64_t ns = std::min<int64_t>(N, (int64_t)100 * K);
  std::vector<int64_t> rows = rii_host::sample_without_replacement(N, ns, seed);
  std::vector<uint8_t> sample((size_t)ns * M);
  {
    // fetch the sampled rows in plain form
    std::vector<int32_t> r32(rows.begin(), rows.end());
    int32_t* d_rows = nullptr;
    uint8_t* d_tmp = nullptr;
    RII_HIP(hipMalloc(&d_rows, (size_t)ns * 4));
    RII_HIP(hipMalloc(&d_tmp, (size_t)ns * M));
    RII_HIP(hipMemcpy(d_rows, r32.data(), (size_t)ns * 4, hipMemcpyHostToDevice));
    int rc = rii_internal_copy_rows(idx->d_codes, 0, idx->plane_codes, d_rows, ns, M, d_tmp, -1, 0, nullptr);
    if (rc) return rc;
    RII_HIP(hipMemcpy(sample.data(), d_tmp, sample.size(), hipMemcpyDeviceToHost));
    (void)hipFree(d_rows);
    (void)hipFree(d_tmp);
  }
  // initial centres: the first K distinct codes of the sample in a seeded order
  std::vector<uint8_t> coarse((size_t)K * M);
  {
    std::vector<int64_t> order(ns);
    for (int64_t i = 0; i < ns; ++i) order[i] = i;
    std::sort(order.begin(), order.end(), [&](int64_t a, int64_t b) {
      uint64_t ha = rii_host::mix64(seed ^ (uint64_t)rows[a] * 0x9E3779B97F4A7C15ull);
      uint64_t hb = rii_host::mix64(seed ^ (uint64_t)rows[b] * 0x9E3779B97F4A7C15ull);
      return ha != hb ? ha < hb : a < b;
    });
    std::unordered_set<std::string> seen;
    int got = 0;
    for (int64_t i = 0; i < ns && got < K; ++i) {
      std::string key(reinterpret_cast<const char*>(&sample[order[i] * M]), M);
      if (seen.insert(key).second) {
        std::memcpy(&coarse[(size_t)got * M], key.data(), M);
        ++got;
      }
    }
    for (int64_t i = 0; got < K; ++i, ++got)  // fewer than K distinct codes: repeat sample rows
      std::memcpy(&coarse[(size_t)got * M], &sample[order[i % ns] * M], M);
  }
  if (iters > 0) {
    int rc = rii_internal_sym_table(idx, nullptr);
    if (rc) return rc;
    std::vector<float> sym((size_t)M * 256 * 256);
    RII_HIP(hipDeviceSynchronize());
    RII_HIP(hipMemcpy(sym.data(), idx->d_sym, sym.size() * 4, hipMemcpyDeviceToHost));
    uint8_t* d_sample = nullptr;
    int32_t* d_assign = nullptr;
    RII_HIP(hipMalloc(&d_sample, (size_t)ns * M));
    RII_HIP(hipMalloc(&d_assign, (size_t)ns * 4));
    RII_HIP(hipMemcpy(d_sample, sample.data(), sample.size(), hipMemcpyHostToDevice));
    std::vector<int32_t> assign(ns);
    for (int it = 0; it < iters; ++it) {
      int rc2 = assign_rows_dev(idx, d_sample, ns, -1, 0, coarse.data(), K, d_assign);
      if (rc2) return rc2;
      RII_HIP(hipMemcpy(assign.data(), d_assign, (size_t)ns * 4, hipMemcpyDeviceToHost));
      rii_host::update_centres(sample.data(), ns, assign.data(), sym.data(), M, K, coarse.data());
    }
    (void)hipFree(d_sample);
    (void)hipFree(d_assign);
  }
  return rii_index_build_lists(idx, coarse.data(), K);
}

int rii_index_get_lists(const rii_index_t* idx, uint8_t* coarse_out, int64_t* list_offsets_out,
                        int32_t* list_ids_out, int32_t* assign_out, int mem) {
  if (!idx || (mem != RII_MEM_HOST && mem != RII_MEM_DEVICE)) return RII_ERR_INVALID_ARG;
  if (idx->K < 1) return RII_ERR_NOT_BUILT;
  hipMemcpyKind kind = mem == RII_MEM_HOST ? hipMemcpyDeviceToHost : hipMemcpyDeviceToDevice;
  if (coarse_out) RII_HIP(hipMemcpy(coarse_out, idx->d_coarse, (size_t)idx->K * idx->M, kind));
  if (list_offsets_out) RII_HIP(hipMemcpy(list_offsets_out, idx->d_list_off, (size_t)(idx->K + 1) * 8, kind));
  if (list_ids_out && idx->N) RII_HIP(hipMemcpy(list_ids_out, idx->d_list_ids, (size_t)idx->N * 4, kind));
  if (assign_out && idx->N) {
    if (mem == RII_MEM_DEVICE) {
      int rc = rii_internal_assign_from_lists(idx, assign_out, nullptr);
      if (rc) return rc;
      RII_HIP(hipDeviceSynchronize());
    } else {
      DevBuf tmp;
      int rc = tmp.alloc((size_t)idx->N * 4);
      if (!rc) rc = rii_internal_assign_from_lists(idx, tmp.as<int32_t>(), nullptr);
      if (rc) return rc;
      RII_HIP(hipMemcpy(assign_out, tmp.p, (size_t)idx->N * 4, hipMemcpyDeviceToHost));
    }
  }
  return RII_OK;
}

int rii_index_get_codes(const rii_index_t* idx, int64_t first, int64_t n, uint8_t* codes_out, int mem) {
  if (!idx || first < 0 || n < 0 || first + n > idx->N || (n > 0 && !codes_out) ||
      (mem != RII_MEM_HOST && mem != RII_MEM_DEVICE))
    return RII_ERR_INVALID_ARG;
  if (n == 0) return RII_OK;
  const int M = idx->M;
  uint8_t* dst = codes_out;
  uint8_t* stage = nullptr;
  if (mem == RII_MEM_HOST) {
    RII_HIP(hipMalloc(&stage, (size_t)n * M));
    dst = stage;
  }
  int rc = rii_internal_copy_rows(idx->d_codes, first, idx->plane_codes, nullptr, n, M, dst, -1, 0, nullptr);  // plain form
  if (!rc && hipDeviceSynchronize() != hipSuccess) rc = RII_ERR_DEVICE;
  if (!rc && stage && hipMemcpy(codes_out, stage, (size_t)n * M, hipMemcpyDeviceToHost) != hipSuccess) rc = RII_ERR_DEVICE;
  if (stage) (void)hipFree(stage);
  return rc;
}

}  // extern "C"
