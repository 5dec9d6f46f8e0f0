// Internal declarations shared by the translation units of the library (not installed).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <vector>

#include "rii.h"

struct rii_index {
  int D = 0, M = 0, Ks = 0, Ds = 0;
  int device = 0;
  int64_t N = 0;         // stored codes
  int64_t cap = 0;       // rows allocated in d_codes
  int K = 0;             // coarse centres (0: no posting lists)
  int64_t theta = 0;     // switch threshold of the query procedure

  float* d_cb = nullptr;          // [M][256][Ds] codebooks
  std::vector<float> h_cb;        // host mirror of the codebooks
  float* d_sym = nullptr;         // [M][256][256] code-word-to-code-word squared distances (lazy)
  // "Stored" code arrays (d_codes, d_codes_list, d_coarse_st) keep row r rotated by r bytes when
  // M is 8, 16 or 32 (stored[r][t] = code[r][(t + r) % M]), plain otherwise; see rii_kernels.hip.
  // For M = 32 a stored array is two planes: bytes 0..15 of every row first (16 bytes a row), then,
  // plane_* bytes further, bytes 16..31 of every row; plane_* is 0 for every other M.  A scan that
  // settles most rows after 16 look-ups then leaves the second plane alone.  Gathered rows (a
  // target set) want whole rows instead, one cache line a row: for M = 32 the codes are kept a
  // second time in that form (d_codes_rows, the tail of d_codes' allocation); for every other M
  // d_codes_rows is d_codes.
  int64_t plane_codes = 0, plane_list = 0, plane_coarse = 0;
  int64_t plane_rows = 0;         // plane distance of d_codes_rows: 0 (whole rows) unless it is d_codes itself
  bool keep_rows_copy = true;     // M = 32: keep the whole-row copy for gathered scans (RII_OPT_GATHER_COPY)
  uint8_t* d_codes = nullptr;     // [cap][M] codes in identifier order (the linear array), stored form
  uint8_t* d_codes_rows = nullptr;  // [cap][M] the same rows, rotated, never split (what the subset scan gathers from)
  uint8_t* d_coarse = nullptr;    // [K][M] coarse centres (PQ codes), plain
  uint8_t* d_coarse_st = nullptr; // [K][M] coarse centres, stored form (what the coarse ranking scans)
  int64_t* d_list_off = nullptr;  // [K+1]
  int32_t* d_list_ids = nullptr;  // [N] identifiers, list after list
  uint8_t* d_codes_list = nullptr;  // [N][M] codes permuted into list order (row p = code of d_list_ids[p]), stored form
  std::vector<uint8_t> h_coarse;    // host mirror of the coarse centres
  std::vector<int64_t> h_list_off;  // host mirror of the list offsets
  int64_t max_list_len = 0;

  // scratch reused by the online calls (grown on demand)
  mutable void* ws = nullptr;
  mutable size_t ws_bytes = 0;

  bool bench_half_table = false;  // set around one launch by rii_bench_scan_linear_half only
  // optional measurement aid: events recorded right before / after the linear-scan kernel
  void* ev_start = nullptr;
  void* ev_stop = nullptr;
  // ... and, while the events are set, device tallies the scan kernels add to (see ScanArgs::counters)
  unsigned long long* d_scan_counters = nullptr;
};

#define RII_HIP(call)                         \
  do {                                        \
    hipError_t e__ = (call);                  \
    if (e__ != hipSuccess) {                  \
      (void)hipGetLastError();                \
      return e__ == hipErrorOutOfMemory ? RII_ERR_OOM : RII_ERR_DEVICE; \
    }                                         \
  } while (0)

// host-side helpers implemented in rii_host.cpp
namespace rii_host {
uint64_t mix64(uint64_t z);
// n distinct values from [0, N), ascending; seeded.
std::vector<int64_t> sample_without_replacement(int64_t N, int64_t n, uint64_t seed);
// one update round of the code-space clustering used by reconfigure (see rii.h)
void update_centres(const uint8_t* sample, int64_t n, const int32_t* assign, const float* sym, int M, int K,
                    uint8_t* coarse);
// stable grouping of identifiers by list number
int build_csr(const int32_t* assign, int64_t N, int K, std::vector<int64_t>& off, std::vector<int32_t>& ids);
}  // namespace rii_host
