// HIP kernels (gfx950), their launchers and the device-side entry points of the library.
// The device code lives in the rii_dev_*.inc files included below; this file holds the host
// side: workspace layout, launch shapes (scan_chunks, plan_batch), dispatch on M and the
// extern "C" entry points.
//
// Data flow of one query batch:
//   k_build_lut              q, code books                        -> A [Q][M][256]       (Sec. 3)
//   k_scan_w4 / k_scan_w     A in LDS, codes streamed             -> top-R per query     (Alg. 1, whole data)
//   k_scan_w<subset>         A in LDS, codes gathered by id       -> top-R per query     (Alg. 1, target ids)
//   k_scan_w4 / k_scan_w     the same over the coarse codes       -> nearest lists       (Alg. 2, first block)
//   k_ivf_w / k_ivf          A in LDS, probed lists streamed      -> top-R per query     (Alg. 2, second block)
//   k_scan + k_select, k_sort_segments: R above the per-wave kernels' reach, explicit candidates
//
// A candidate is one 64-bit key: order-preserving image of the fp32 distance in the high word,
// identifier in the low word.  Comparing keys as unsigned integers is the (distance,
// identifier) order, so selection is exact and deterministic including ties.

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <type_traits>
#include <unordered_map>
#include <vector>

#include "rii_internal.h"
#include "rii_bench.h"

#ifndef RII_SUBSET_GENERATION
#define RII_SUBSET_GENERATION 256
#endif

namespace {

// Device code, in dependency order (textual includes: everything shares this namespace).
#include "rii_dev_common.inc"
#include "rii_dev_adc.inc"
#include "rii_dev_scan_common.inc"
#include "rii_dev_scan_w.inc"
#include "rii_dev_scan_batched.inc"
#include "rii_dev_select.inc"
#include "rii_dev_ivf.inc"
#include "rii_dev_offline.inc"
#include "rii_dev_bench.inc"

// ------------------------------------------------------------------ host helpers
int ensure_ws(const rii_index* idx, size_t bytes) {
  if (idx->ws_bytes >= bytes) return RII_OK;
  if (idx->ws) (void)hipFree(idx->ws);
  idx->ws = nullptr;
  idx->ws_bytes = 0;
  size_t want = bytes + bytes / 4;
  hipError_t e = hipMalloc(&idx->ws, want);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    e = hipMalloc(&idx->ws, bytes);
    want = bytes;
    if (e != hipSuccess) {
      (void)hipGetLastError();
      return RII_ERR_OOM;
    }
  }
  idx->ws_bytes = want;
  return RII_OK;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

constexpr int64_t kBatchChunkBytes = (int64_t)384 << 20;  // rows of a large batch are scanned in chunks of about this size
constexpr int kSubsetGeneration = RII_SUBSET_GENERATION;  // queries per launch of a subset scan with one block per query


bool m_supported(int M) { return M >= 4 && M <= RII_MAX_M && M % 4 == 0; }

// Per (device, kernel): the dynamic LDS size already granted with hipFuncSetAttribute, and whether
// the kernel was checked to have no static LDS.  Looked up on every launch, written once per
// kernel, so that the online calls make no runtime-attribute calls after their first launch.
struct KernelLdsState {
  size_t granted = 0;
  bool at_zero = false;
};
std::mutex g_lds_mutex;
std::unordered_map<uint64_t, KernelLdsState> g_lds_state;

uint64_t lds_key(const void* kern) {
  int dev = 0;
  (void)hipGetDevice(&dev);
  return (uint64_t)reinterpret_cast<uintptr_t>(kern) * 64u + (uint64_t)(dev & 63);
}

// Allow `kern` to be launched with `bytes` of dynamic LDS.  need_zero: the kernel addresses its
// table as "LDS address 0", so it must not have static LDS in front of the dynamic allocation;
// refuse to launch otherwise (checked once per kernel).
int set_lds_impl(const void* kern, size_t bytes, bool need_zero) {
  std::lock_guard<std::mutex> lock(g_lds_mutex);
  KernelLdsState& st = g_lds_state[lds_key(kern)];
  if (need_zero && !st.at_zero) {
    hipFuncAttributes attr{};
    RII_HIP(hipFuncGetAttributes(&attr, kern));
    if (attr.sharedSizeBytes != 0) return RII_ERR_DEVICE;
    st.at_zero = true;
  }
  if (bytes > 48 * 1024 && bytes > st.granted) {
    RII_HIP(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    st.granted = bytes;
  }
  return RII_OK;
}

template <typename Kern>
int set_lds(Kern kern, size_t bytes) { return set_lds_impl(reinterpret_cast<const void*>(kern), bytes, false); }

// set_lds for the kernels whose table must sit at LDS address 0
template <typename Kern>
int set_lds0(Kern kern, size_t bytes) { return set_lds_impl(reinterpret_cast<const void*>(kern), bytes, true); }

#define DISPATCH_M(M, ...)                                  \
  switch (M) {                                              \
    case 8: { constexpr int MT = 8; __VA_ARGS__; } break;   \
    case 16: { constexpr int MT = 16; __VA_ARGS__; } break; \
    case 32: { constexpr int MT = 32; __VA_ARGS__; } break; \
    case 64: { constexpr int MT = 64; __VA_ARGS__; } break; \
    default: { constexpr int MT = 0; __VA_ARGS__; } break;  \
  }

// Split max_rows rows per query into equal chunks (one block each): about kWantBlocks blocks
// in total when the batch is small, never chunks shorter than kMinTiles tiles.
void scan_chunks(int Q, int64_t max_rows, int64_t* nchunks_out, int64_t* chunk_rows_out) {
  const int64_t tile = (int64_t)kScanThreads * kRowsPerLane;
  int64_t want = std::max<int64_t>(1, kWantBlocks / Q);  // rounded down: one block over a full round costs a second round
  int64_t most = std::max<int64_t>(1, (max_rows + kMinTiles * tile - 1) / (kMinTiles * tile));
  int64_t nchunks = std::min<int64_t>(std::min(want, most), 65535);
  int64_t chunk_rows = (max_rows + nchunks - 1) / nchunks;
  chunk_rows = std::max<int64_t>(tile, (chunk_rows + tile - 1) / tile * tile);
  *nchunks_out = std::max<int64_t>(1, (max_rows + chunk_rows - 1) / chunk_rows);
  *chunk_rows_out = chunk_rows;
}

// Launch shape of the batched kernel k_scan_w4 for Q queries over `rows` rows: groups of four
// queries (the last may be short) times row chunks.  Returns false when the kernel does not
// apply or would leave most of the chip idle (then the one-query kernels split the rows).
bool plan_batch(int M, int Q, int64_t rows, int topk, int64_t* nchunks_out, int64_t* chunk_rows_out) {
  *nchunks_out = 1;
  *chunk_rows_out = rows;
  if (!rot_m(M) || topk > kWaveK4 || Q < 4 || rows < 1) return false;
  const int64_t tile = (int64_t)kScanThreads * kRowsPerLane;
  const int64_t groups = (Q + 3) / 4;
  int64_t chunk_rows = (rows + tile - 1) / tile * tile, nchunks = 1;
  if (groups < 2 * kWantBlocks) {  // fewer than two full rounds of blocks from the groups alone
    const int64_t want = (kBatchWantBlocks + groups - 1) / groups;
    const int64_t most = std::max<int64_t>(1, rows / (kBatchMinTiles * tile));
    nchunks = std::min<int64_t>(std::min(want, most), 65535);
    // whole rounds of blocks (one block per CU): a part-filled last round takes as long as a full one
    if (groups * nchunks > kWantBlocks) nchunks = std::max<int64_t>(1, groups * nchunks / kWantBlocks * kWantBlocks / groups);
    chunk_rows = (rows + nchunks - 1) / nchunks;
    chunk_rows = (chunk_rows + tile - 1) / tile * tile;
    nchunks = (rows + chunk_rows - 1) / chunk_rows;
  } else if (rows * M > 2 * kBatchChunkBytes) {
    // A large batch over a large array: the rows are cut into chunks of about kBatchChunkBytes
    // all the same, chunk index slowest, so that the blocks resident at one time read the same
    // part of the array and the memory-side cache serves most of them.  With the abandoning
    // tests after every eight look-ups the kernel had become bound by the delivery of the code
    // bytes (10^4 queries over 10^8 rows of 32 bytes: 640 ms in one piece, 545 ms in nine).
    nchunks = (rows * M + kBatchChunkBytes - 1) / kBatchChunkBytes;
    chunk_rows = (rows + nchunks - 1) / nchunks;
    chunk_rows = (chunk_rows + tile - 1) / tile * tile;
    nchunks = (rows + chunk_rows - 1) / chunk_rows;
  }
  if (groups * nchunks < kWantBlocks / 4) return false;  // (a quarter of the CUs busy with four queries each still wins)
  *nchunks_out = nchunks;
  *chunk_rows_out = chunk_rows;
  return true;
}

// Scan `nrows_max` rows per query (linear: the whole array) and leave per-block partial keys in
// the workspace; then select.  Workspace layout: [tau Q u32][partial Q*nchunks*k u64].
int launch_scan(const rii_index* idx, const uint8_t* codes, int64_t plane, int64_t N, const float* lut, int Q, int mode,
                const int32_t* target_ids, const int64_t* target_offsets, int64_t max_rows, int topk,
                int32_t* ids, float* dist, int out_stride, const int* qmode, int want_mode, void* ws_base,
                hipStream_t st) {
  const int M = idx->M;
  int64_t nchunks, chunk_rows;
  scan_chunks(Q, max_rows, &nchunks, &chunk_rows);

  // workspace: [tau Q][candidate count Q][prepass counter Q][blocks done Q] u32, then
  // [candidates], then [prepass minima]
  // (the four arrays start 256-byte aligned so that, for a single query, the much-read bound
  // does not share a cache line with the counters the blocks update)
  uint8_t* base = static_cast<uint8_t*>(ws_base);
  const size_t cstride = align_up((size_t)Q * 4, 256) / 4;
  uint32_t* tau = reinterpret_cast<uint32_t*>(base);
  uint32_t* cand_cnt = tau + cstride;
  uint32_t* pre_counter = tau + 2 * cstride;
  uint32_t* done_cnt = tau + 3 * cstride;
  uint64_t* partial = reinterpret_cast<uint64_t*>(base + kScanArrays * cstride * 4);

  ScanArgs a{};
  a.codes = codes; a.plane = plane; a.N = N; a.M = M; a.lut = lut;
  a.target_ids = target_ids; a.target_offsets = target_offsets;
  a.chunk_rows = chunk_rows; a.k = topk; a.partial = partial; a.tau_g = tau;
  int64_t bchunks, brows;
  const bool batched = plan_batch(M, Q, max_rows, topk, &bchunks, &brows) && mode == kLinear && !qmode;
  a.cand_cnt = cand_cnt; a.cand_cap = std::max(nchunks, bchunks) * topk;
  a.nq = Q;
  // [prepass minima] follow the candidates
  uint32_t* minima = reinterpret_cast<uint32_t*>(partial + (size_t)Q * a.cand_cap);
  a.done_cnt = done_cnt; a.ids = ids; a.dist = dist; a.out_stride = out_stride;
  a.qmode = qmode; a.want_mode = want_mode;
  dim3 grid((unsigned)nchunks, (unsigned)Q);
  if (Q > 65535) return RII_ERR_UNSUPPORTED;
  const bool timed = mode == kLinear && idx->ev_start && idx->ev_stop && codes == idx->d_codes;
  a.counters = timed ? idx->d_scan_counters : nullptr;
  if (topk <= kWaveK || rot_m(M)) {  // (rotated stored form: k_scan_w up to RII_MAX_TOPK, with a block-level buffer above kWaveK)
    // When a query's rows are split over several blocks, a short first pass over the leading
    // rows seeds the shared bound, so that the main pass starts with few candidates.
    const int64_t tile_rows = (int64_t)kScanThreads * kRowsPerLane;
    const int64_t tiles = (max_rows + tile_rows - 1) / tile_rows;
    int pre_blocks = (int)std::min<int64_t>(kPrepassBlocks, tiles);
    if (Q >= 4) {
      // Many queries: the seeding blocks no longer run side by side, each costs a table fill, and
      // on a small array 256 of them per query would score all of it once more.  A thirty-second
      // of the rows, and never more than 128 blocks, is enough for a useful bound, as long as
      // there are at least topk wave minima.
      const int64_t least = std::min<int64_t>(tiles, (topk + kScanThreads / 64 - 1) / (kScanThreads / 64) + 1);
      pre_blocks = (int)std::max<int64_t>(least, std::min<int64_t>(std::min(pre_blocks, kPrepassBlocks / 2), tiles / 32));
    }
    // The single-query kernel seeds the bound itself when all its blocks run at once and a query
    // has at least topk of them (rotated form only); otherwise a separate pass does it.
    // ... from its blocks' minima (at most 64 kSeedPerLane blocks), or from its waves' when it
    // has fewer than topk blocks but enough waves
    const int waves = kScanThreads / 64;
    const bool resident = nchunks > 1 && rot_m(M) && !batched && (int64_t)Q * nchunks <= kWantBlocks;
    const bool seed_blocks = resident && nchunks >= topk && nchunks <= 64 * kSeedPerLane;
    const bool seed_waves = resident && !seed_blocks && nchunks * waves >= topk && nchunks * waves <= 64 * kSeedPerLane;
    const bool seed_inside = seed_blocks || seed_waves;
    const bool prepass = nchunks > 1 && !seed_inside;
    a.seed_inside = seed_blocks ? 1 : seed_waves ? 2 : 0;
    const int nzero = seed_blocks ? Q * (int)nchunks : seed_waves ? Q * (int)nchunks * waves : 0;
    k_init_scan<<<(std::max(Q, nzero) + 255) / 256, 256, 0, st>>>(tau, Q, (int)cstride, minima, nzero);
    if (timed) RII_HIP(hipEventRecord(static_cast<hipEvent_t>(idx->ev_start), st));
    a.minima = minima;
    a.counter = pre_counter;
    ScanArgs pre = a;
    pre.minima = minima;
    pre.counter = pre_counter;
    dim3 pgrid((unsigned)pre_blocks, (unsigned)Q);
    const size_t ldsw = table_bytes(M) + (size_t)(kScanThreads / 64 + 1) * kWaveCap * 8 + kBlockVarsBytes;
    const size_t lds4 = 65536 + 4 * (size_t)(kScanThreads / 64 + 1) * kWaveCap4 * 8 +
                        (size_t)(kScanThreads / 64) * kRescoreCap * 8 + kBlockVarsBytes;
    const size_t lds2 = 65536 + 2 * (size_t)(kScanThreads / 64 + 1) * kWaveCap * 8 + kBlockVarsBytes;
    if (batched) {
      // Four queries per block with the integer-table filter; the rows are cut into chunks
      // when the groups alone would not fill the chip, and then the bound-seeding pass runs
      // first so that no block starts without a bound.
      ScanArgs a4 = a;
      a4.chunk_rows = brows;
      const dim3 g4((unsigned)((Q + 3) / 4), (unsigned)bchunks);
      // (no seeding pass for a large batch that is chunked for the cache's sake: its first chunk's
      // blocks find their bounds as an unchunked scan does, the later ones read the query's bound)
      const bool pre4 = bchunks > 1 && (Q + 3) / 4 < 2 * kWantBlocks;
      if (pre4) {
        switch (M) {
          case 8: { int rc = set_lds0(k_tau0<8, kLinear>, tau0_lds(M) + kBlockVarsBytes); if (rc) return rc;
                    k_tau0<8, kLinear><<<pgrid, kScanThreads, tau0_lds(M) + kBlockVarsBytes, st>>>(pre); } break;
          case 16: { int rc = set_lds0(k_tau0<16, kLinear>, tau0_lds(M) + kBlockVarsBytes); if (rc) return rc;
                     k_tau0<16, kLinear><<<pgrid, kScanThreads, tau0_lds(M) + kBlockVarsBytes, st>>>(pre); } break;
          default: { int rc = set_lds0(k_tau0<32, kLinear>, tau0_lds(M) + kBlockVarsBytes); if (rc) return rc;
                     k_tau0<32, kLinear><<<pgrid, kScanThreads, tau0_lds(M) + kBlockVarsBytes, st>>>(pre); } break;
        }
      }
      if (idx->bench_half_table) {  // the separately evaluated half-precision table (measurement entry point only)
        switch (M) {
          case 8: { int rc = set_lds0(k_scan_w4<8, true>, lds4); if (rc) return rc;
                    k_scan_w4<8, true><<<g4, kScanThreads, lds4, st>>>(a4); } break;
          case 16: { int rc = set_lds0(k_scan_w4<16, true>, lds4); if (rc) return rc;
                     k_scan_w4<16, true><<<g4, kScanThreads, lds4, st>>>(a4); } break;
          default: { int rc = set_lds0(k_scan_w4<32, true>, lds4); if (rc) return rc;
                     k_scan_w4<32, true><<<g4, kScanThreads, lds4, st>>>(a4); } break;
        }
      } else {
        switch (M) {
          case 8: { int rc = set_lds0(k_scan_w4<8>, lds4); if (rc) return rc;
                    k_scan_w4<8><<<g4, kScanThreads, lds4, st>>>(a4); } break;
          case 16: { int rc = set_lds0(k_scan_w4<16>, lds4); if (rc) return rc;
                     k_scan_w4<16><<<g4, kScanThreads, lds4, st>>>(a4); } break;
          default: { int rc = set_lds0(k_scan_w4<32>, lds4); if (rc) return rc;
                     k_scan_w4<32><<<g4, kScanThreads, lds4, st>>>(a4); } break;
        }
      }
    } else if (mode == kLinear && rot_m(M) && nchunks == 1 && !qmode && Q >= 2 && topk > kWaveK4 && topk <= kWaveK) {
      // Large batch with topk beyond the four-query kernel's reach: two queries per block
      // (k_scan_w2), every block owning its queries' whole scan, and a single-query block for an
      // odd one left over, addressed as query 0 of argument arrays shifted by Q - 1.
      auto shifted = [&](int o) {
        ScanArgs b = a;
        b.lut = lut + (size_t)o * M * 256;
        b.partial = partial + (size_t)o * a.cand_cap;
        b.tau_g = tau + o; b.cand_cnt = cand_cnt + o; b.done_cnt = done_cnt + o;
        b.ids = ids + (size_t)o * out_stride;
        b.dist = dist ? dist + (size_t)o * out_stride : nullptr;
        return b;
      };
      const dim3 g2(1, (unsigned)(Q / 2));
      switch (M) {
        case 8: { int rc = set_lds0(k_scan_w2<8>, lds2); if (rc) return rc;
                  k_scan_w2<8><<<g2, kScanThreads, lds2, st>>>(a); } break;
        case 16: { int rc = set_lds0(k_scan_w2<16>, lds2); if (rc) return rc;
                   k_scan_w2<16><<<g2, kScanThreads, lds2, st>>>(a); } break;
        default: { int rc = set_lds0(k_scan_w2<32>, lds2); if (rc) return rc;
                   k_scan_w2<32><<<g2, kScanThreads, lds2, st>>>(a); } break;
      }
      if (Q & 1) {
        ScanArgs b = shifted(Q - 1);
        switch (M) {
          case 8: { int rc = set_lds0(k_scan_w<8, kLinear>, ldsw); if (rc) return rc;
                    k_scan_w<8, kLinear><<<dim3(1, 1), kScanThreads, ldsw, st>>>(b); } break;
          case 16: { int rc = set_lds0(k_scan_w<16, kLinear>, ldsw); if (rc) return rc;
                     k_scan_w<16, kLinear><<<dim3(1, 1), kScanThreads, ldsw, st>>>(b); } break;
          default: { int rc = set_lds0(k_scan_w<32, kLinear>, ldsw); if (rc) return rc;
                     k_scan_w<32, kLinear><<<dim3(1, 1), kScanThreads, ldsw, st>>>(b); } break;
        }
      }
    } else if (mode == kLinear) {
      DISPATCH_M(M, { int rc = set_lds0(k_scan_w<MT, kLinear>, ldsw); if (rc) return rc;
                      if (prepass) { int rc2 = set_lds0(k_tau0<MT, kLinear>, tau0_lds(M) + kBlockVarsBytes); if (rc2) return rc2; }
                      if (prepass) k_tau0<MT, kLinear><<<pgrid, kScanThreads, tau0_lds(M) + kBlockVarsBytes, st>>>(pre);
                      k_scan_w<MT, kLinear><<<grid, kScanThreads, ldsw, st>>>(a); });
    } else {
      // One block per query and more queries than the chip holds blocks: the queries are launched
      // a chip-load at a time.  Target lists are sorted, so the blocks of one launch walk the code
      // array from its start to its end together, and a memory line that holds rows of several
      // queries' targets is fetched once for all of them while it stays in the memory-side cache
      // (with all queries in one launch the resident blocks are spread over the whole array).
      const int per_launch = nchunks == 1 && Q > kSubsetGeneration ? kSubsetGeneration : Q;
      for (int o = 0; o < Q; o += per_launch) {
        ScanArgs b = a;
        b.lut = lut + (size_t)o * M * 256;
        b.target_offsets = target_offsets + o;
        b.qmode = qmode ? qmode + o : nullptr;
        b.partial = partial + (size_t)o * a.cand_cap;
        b.tau_g = tau + o; b.cand_cnt = cand_cnt + o; b.done_cnt = done_cnt + o;
        b.ids = ids + (size_t)o * out_stride;
        b.dist = dist ? dist + (size_t)o * out_stride : nullptr;
        const dim3 g((unsigned)nchunks, (unsigned)std::min(per_launch, Q - o));
        DISPATCH_M(M, { int rc = set_lds0(k_scan_w<MT, kSubset>, ldsw); if (rc) return rc;
                        if (prepass) { int rc2 = set_lds0(k_tau0<MT, kSubset>, tau0_lds(M) + kBlockVarsBytes); if (rc2) return rc2; }
                        if (prepass) k_tau0<MT, kSubset><<<pgrid, kScanThreads, tau0_lds(M) + kBlockVarsBytes, st>>>(pre);
                        k_scan_w<MT, kSubset><<<g, kScanThreads, ldsw, st>>>(b); });
      }
    }
  } else {
  k_init_scan<<<(Q + 255) / 256, 256, 0, st>>>(tau, Q, (int)cstride, nullptr, 0);
  if (timed) RII_HIP(hipEventRecord(static_cast<hipEvent_t>(idx->ev_start), st));
  const size_t lds = (size_t)M * 1024 + (size_t)kSelCap * 8;
  if (mode == kLinear) {
    DISPATCH_M(M, { int rc = set_lds(k_scan<MT, kLinear>, lds); if (rc) return rc;
                    k_scan<MT, kLinear><<<grid, kScanThreads, lds, st>>>(a); });
  } else {
    DISPATCH_M(M, { int rc = set_lds(k_scan<MT, kSubset>, lds); if (rc) return rc;
                    k_scan<MT, kSubset><<<grid, kScanThreads, lds, st>>>(a); });
  }
  }
  if (timed) RII_HIP(hipEventRecord(static_cast<hipEvent_t>(idx->ev_stop), st));
  if (topk > kWaveK) {
    SelectArgs s{};
    s.keys = partial; s.nkeys = a.cand_cap; s.key_cnt = cand_cnt; s.k = topk; s.out_stride = out_stride;
    s.ids = ids; s.dist = dist; s.qmode = qmode; s.want_mode = want_mode;
    k_select<<<Q, kScanThreads, 0, st>>>(s);
  }
  RII_HIP(hipGetLastError());
  return RII_OK;
}

// Minima of the bound-seeding pass: it only runs when the rows of a query are cut into chunks,
// which launches of kSeedMaxQ or more queries never do, and with four or more queries it has
// at most kPrepassBlocks / 2 blocks per query (see launch_scan).
constexpr int kSeedMaxQ = 2048;
static_assert(kSeedMaxQ >= 8 * kWantBlocks, "batches that are cut into row chunks have fewer than 2 * kWantBlocks groups of four");
size_t minima_bytes(int Q) {
  const size_t blocks = Q < 4 ? kPrepassBlocks : kPrepassBlocks / 2;
  return (size_t)std::min(Q, kSeedMaxQ) * blocks * (kScanThreads / 64) * 4;
}

size_t scan_ws_bytes(int M, int Q, int64_t max_rows, int topk) {
  int64_t nchunks, chunk_rows;
  scan_chunks(Q, max_rows, &nchunks, &chunk_rows);
  int64_t bchunks, brows;
  plan_batch(M, Q, max_rows, topk, &bchunks, &brows);
  const int64_t cap_chunks = std::max(nchunks, bchunks);
  return kScanArrays * align_up((size_t)Q * 4, 256) + (size_t)Q * cap_chunks * topk * 8 + minima_bytes(Q) + 256;
}

// The same for every batch of at most Q queries, at most max_rows rows and at most topk results:
// a bound that grows with each argument (a batch's blocks per query times its queries stay
// below Q + 4 kBatchWantBlocks + kWantBlocks whatever the launch shape is).
size_t scan_ws_bound(int M, int Q, int64_t max_rows, int topk) {
  const size_t big_chunks = (size_t)(max_rows * M / kBatchChunkBytes + 2);  // chunks of a large batch (see plan_batch)
  return kScanArrays * align_up((size_t)Q * 4, 256) +
         ((size_t)Q * big_chunks + 4 * kBatchWantBlocks + kWantBlocks + 8) * topk * 8 +
         std::max(minima_bytes(Q), minima_bytes(std::min(Q, 3))) + 256;
}

}  // namespace

// ====================================================================== entry points
extern "C" {

int rii_build_lut(const rii_index_t* idx, const float* q, int Q, float* lut, void* stream) {
  if (!idx || !q || !lut || Q < 1) return RII_ERR_INVALID_ARG;
  if (Q > 65535) return RII_ERR_UNSUPPORTED;
  hipStream_t st = static_cast<hipStream_t>(stream);
  k_build_lut<<<dim3(idx->M, Q), 256, 0, st>>>(idx->d_cb, q, idx->D, idx->M, idx->Ds, lut);
  RII_HIP(hipGetLastError());
  return RII_OK;
}

int rii_scan_linear_plan(const rii_index_t* idx, int Q, int topk, int* queries_per_block, int64_t* row_chunks) {
  if (!idx || !queries_per_block || !row_chunks || Q < 1 || topk < 1) return RII_ERR_INVALID_ARG;
  if (topk > RII_MAX_TOPK || !m_supported(idx->M) || Q > 65535) return RII_ERR_UNSUPPORTED;
  int64_t nchunks, chunk_rows, bchunks, brows;
  scan_chunks(Q, idx->N, &nchunks, &chunk_rows);
  if (topk <= kWaveK && plan_batch(idx->M, Q, idx->N, topk, &bchunks, &brows)) {
    *queries_per_block = 4;
    *row_chunks = bchunks;
  } else if (topk <= kWaveK && rot_m(idx->M) && nchunks == 1 && Q >= 2 && topk > kWaveK4) {
    *queries_per_block = 2;
    *row_chunks = 1;
  } else {
    *queries_per_block = 1;
    *row_chunks = nchunks;
  }
  return RII_OK;
}

int rii_bench_lds_lookups(int width, int blocks, int threads, int iters, int lds_bytes, uint32_t* sink, void* stream) {
  if ((width != 4 && width != 8 && width != 64) || blocks < 1 || iters < 1 || !sink) return RII_ERR_INVALID_ARG;
  if (threads < 64 || threads > kScanThreads || threads % 64 != 0) return RII_ERR_INVALID_ARG;
  if (lds_bytes < 65536 || lds_bytes > 160 * 1024) return RII_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (width == 64) {
    int rc = set_lds0(k_lds_lookups<64>, (size_t)lds_bytes);
    if (rc) return rc;
    k_lds_lookups<64><<<blocks, threads, (size_t)lds_bytes, st>>>(iters, sink);
  } else if (width == 8) {
    int rc = set_lds0(k_lds_lookups<8>, (size_t)lds_bytes);
    if (rc) return rc;
    k_lds_lookups<8><<<blocks, threads, (size_t)lds_bytes, st>>>(iters, sink);
  } else {
    int rc = set_lds0(k_lds_lookups<4>, (size_t)lds_bytes);
    if (rc) return rc;
    k_lds_lookups<4><<<blocks, threads, (size_t)lds_bytes, st>>>(iters, sink);
  }
  RII_HIP(hipGetLastError());
  return RII_OK;
}

int rii_bench_scan_linear_half(rii_index_t* idx, const float* lut, int Q, int topk, int32_t* ids, float* dist,
                               void* stream) {
  if (!idx) return RII_ERR_INVALID_ARG;
  int qpb = 0;
  int64_t chunks = 0;
  int rc = rii_scan_linear_plan(idx, Q, topk, &qpb, &chunks);
  if (rc) return rc;
  if (qpb != 4) return RII_ERR_UNSUPPORTED;  // only the four-queries-per-block kernel has the variant
  idx->bench_half_table = true;
  rc = rii_adc_scan_linear(idx, lut, Q, topk, ids, dist, stream);
  idx->bench_half_table = false;
  return rc;
}

int rii_bench_lds_reads(int width, int blocks, int threads, int iters, int lds_bytes, uint32_t* sink, void* stream) {
  if ((width != 4 && width != 8 && width != 16) || blocks < 1 || iters < 1 || !sink) return RII_ERR_INVALID_ARG;
  if (threads < 64 || threads > kScanThreads || threads % 64 != 0) return RII_ERR_INVALID_ARG;
  if (lds_bytes < 65536 || lds_bytes > 160 * 1024) return RII_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (width == 4) {
    int rc = set_lds(k_lds_reads<4>, (size_t)lds_bytes);
    if (rc) return rc;
    k_lds_reads<4><<<blocks, threads, (size_t)lds_bytes, st>>>(iters, sink);
  } else if (width == 8) {
    int rc = set_lds(k_lds_reads<8>, (size_t)lds_bytes);
    if (rc) return rc;
    k_lds_reads<8><<<blocks, threads, (size_t)lds_bytes, st>>>(iters, sink);
  } else {
    int rc = set_lds(k_lds_reads<16>, (size_t)lds_bytes);
    if (rc) return rc;
    k_lds_reads<16><<<blocks, threads, (size_t)lds_bytes, st>>>(iters, sink);
  }
  RII_HIP(hipGetLastError());
  return RII_OK;
}

int rii_adc_scan_linear(const rii_index_t* idx, const float* lut, int Q, int topk, int32_t* ids, float* dist,
                        void* stream) {
  if (!idx || !lut || !ids || !dist || Q < 1 || topk < 1) return RII_ERR_INVALID_ARG;
  if (topk > RII_MAX_TOPK || !m_supported(idx->M) || Q > 65535) return RII_ERR_UNSUPPORTED;
  if (idx->N < 1) return RII_ERR_INVALID_ARG;
  int rc = ensure_ws(idx, scan_ws_bytes(idx->M, Q, idx->N, topk));
  if (rc) return rc;
  return launch_scan(idx, idx->d_codes, idx->plane_codes, idx->N, lut, Q, kLinear, nullptr, nullptr, idx->N, topk, ids, dist, topk,
                     nullptr, 0, idx->ws, static_cast<hipStream_t>(stream));
}

int rii_check_target_ids(const rii_index_t* idx, const int32_t* target_ids, const int64_t* target_offsets, int Q,
                         void* stream) {
  if (!idx || !target_offsets || Q < 1) return RII_ERR_INVALID_ARG;
  if (Q > 65535) return RII_ERR_UNSUPPORTED;
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rc = ensure_ws(idx, 256);
  if (rc) return rc;
  uint32_t* flag = static_cast<uint32_t*>(idx->ws);
  RII_HIP(hipMemsetAsync(flag, 0, 4, st));
  k_check_targets<<<Q, 256, 0, st>>>(target_ids, target_offsets, idx->N, flag);
  RII_HIP(hipGetLastError());
  uint32_t h = 0;
  RII_HIP(hipMemcpyAsync(&h, flag, 4, hipMemcpyDeviceToHost, st));
  RII_HIP(hipStreamSynchronize(st));
  if (h & 2u) return RII_ERR_INVALID_ARG;
  return h ? RII_ERR_UNSORTED_IDS : RII_OK;
}

int rii_adc_scan_subset(const rii_index_t* idx, const float* lut, int Q, const int32_t* target_ids,
                        const int64_t* target_offsets, int64_t max_targets, int topk, int32_t* ids, float* dist,
                        void* stream) {
  if (!idx || !lut || !ids || !dist || !target_offsets || Q < 1 || topk < 1 || max_targets < 0)
    return RII_ERR_INVALID_ARG;
  if (!target_ids && max_targets > 0) return RII_ERR_INVALID_ARG;
  if (topk > RII_MAX_TOPK || !m_supported(idx->M) || Q > 65535) return RII_ERR_UNSUPPORTED;
  if (max_targets > idx->N) max_targets = idx->N;
  int64_t rows = std::max<int64_t>(max_targets, 1);
  int rc = ensure_ws(idx, scan_ws_bytes(idx->M, Q, rows, topk));
  if (rc) return rc;
  return launch_scan(idx, idx->d_codes_rows, idx->plane_rows, idx->N, lut, Q, kSubset, target_ids, target_offsets, rows, topk, ids, dist,
                     topk, nullptr, 0, idx->ws, static_cast<hipStream_t>(stream));
}

int rii_topk(const float* cand_dist, const int32_t* cand_ids, const int64_t* cand_offsets, int Q,
             int64_t max_segment, int topk, int32_t* ids, float* dist, void* stream) {
  if (!cand_dist || !cand_offsets || !ids || Q < 1 || topk < 1 || max_segment < 0) return RII_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  SelectArgs s{};
  s.cand_dist = cand_dist; s.cand_ids = cand_ids; s.cand_offsets = cand_offsets;
  s.k = topk; s.out_stride = topk; s.ids = ids; s.dist = dist;
  if (topk <= RII_MAX_TOPK) {
    k_select<<<Q, kScanThreads, 0, st>>>(s);
  } else {
    if (topk > RII_MAX_SORT || max_segment < 1 || max_segment > RII_MAX_SORT) return RII_ERR_UNSUPPORTED;
    size_t lds = (size_t)RII_MAX_SORT * 8;
    int rc = set_lds(k_sort_segments, lds);
    if (rc) return rc;
    k_sort_segments<<<Q, kScanThreads, lds, st>>>(s);
  }
  RII_HIP(hipGetLastError());
  return RII_OK;
}

// coarse ranking into caller buffers; `ws` must hold what coarse_ws_bytes() says
static size_t coarse_ws_bytes(const rii_index* idx, int Q, int nprobe) {
  if (nprobe <= RII_MAX_TOPK) return scan_ws_bytes(idx->M, Q, idx->K, nprobe);
  return align_up((size_t)Q * idx->K * 4, 256) + align_up((size_t)(Q + 1) * 8, 256);
}

static int coarse_rank(const rii_index* idx, const float* lut, int Q, int nprobe, int32_t* list_ids, float* list_d0,
                       int out_stride, const int* qmode, int want_mode, void* ws, hipStream_t st) {
  const int M = idx->M, K = idx->K;
  if (nprobe <= RII_MAX_TOPK) {
    return launch_scan(idx, idx->d_coarse_st, idx->plane_coarse, K, lut, Q, kLinear, nullptr, nullptr, K, nprobe, list_ids, list_d0,
                       out_stride, qmode, want_mode, ws, st);
  }
  if (K > RII_MAX_SORT) return RII_ERR_UNSUPPORTED;
  float* d0 = static_cast<float*>(ws);
  int64_t* off = reinterpret_cast<int64_t*>(static_cast<uint8_t*>(ws) + align_up((size_t)Q * K * 4, 256));
  const size_t lds = (size_t)M * 1024;
  dim3 grid((K + 255) / 256, Q);
  DISPATCH_M(M, { int rc = set_lds(k_adc_all<MT>, lds); if (rc) return rc;
                  k_adc_all<MT><<<grid, 256, lds, st>>>(idx->d_coarse, K, M, lut, d0, qmode, want_mode); });
  k_iota_offsets<<<(Q + 256) / 256, 256, 0, st>>>(off, Q, K);
  SelectArgs s{};
  s.cand_dist = d0; s.cand_offsets = off; s.k = nprobe; s.out_stride = out_stride;
  s.ids = list_ids; s.dist = list_d0; s.qmode = qmode; s.want_mode = want_mode;
  size_t lds2 = (size_t)RII_MAX_SORT * 8;
  int rc = set_lds(k_sort_segments, lds2);
  if (rc) return rc;
  k_sort_segments<<<Q, kScanThreads, lds2, st>>>(s);
  RII_HIP(hipGetLastError());
  return RII_OK;
}

int rii_coarse_assign(const rii_index_t* idx, const float* lut, int Q, int nprobe, int32_t* list_ids, float* list_d0,
                      void* stream) {
  if (!idx || !lut || !list_ids || Q < 1) return RII_ERR_INVALID_ARG;
  if (idx->K < 1) return RII_ERR_NOT_BUILT;
  if (nprobe < 1 || nprobe > idx->K) return RII_ERR_INVALID_ARG;
  if (!m_supported(idx->M) || Q > 65535) return RII_ERR_UNSUPPORTED;
  if (nprobe > RII_MAX_TOPK && idx->K > RII_MAX_SORT) return RII_ERR_UNSUPPORTED;
  int rc = ensure_ws(idx, coarse_ws_bytes(idx, Q, nprobe));
  if (rc) return rc;
  return coarse_rank(idx, lut, Q, nprobe, list_ids, list_d0, nprobe, nullptr, 0, idx->ws,
                     static_cast<hipStream_t>(stream));
}

// Blocks per query of the multi-block inverted-index scan.
static int ivf_split(int Q, int nprobe) {
  int split = (kWantBlocks + Q - 1) / Q;
  if (split > nprobe) split = nprobe;
  return split < 1 ? 1 : split;
}

static size_t ivf_ws_bytes(int Q, int nprobe, int topk) {
  return kScanArrays * align_up((size_t)Q * 4, 256) + (size_t)Q * ivf_split(Q, nprobe) * topk * 8 + 256;
}

static int launch_ivf(const rii_index* idx, const float* lut, int Q, const int32_t* probe, int probe_stride,
                      int nprobe, const int* nprobe_q, const int32_t* target_ids, const int64_t* target_offsets,
                      int64_t L, int topk, int32_t* ids, float* dist, const int* qmode, int want_mode, void* ws,
                      hipStream_t st) {
  const int M = idx->M;
  IvfArgs a{};
  a.codes_list = idx->d_codes_list; a.plane = idx->plane_list; a.list_ids = idx->d_list_ids; a.list_off = idx->d_list_off; a.M = M;
  a.lut = lut; a.probe = probe; a.probe_stride = probe_stride; a.nprobe = nprobe; a.nprobe_q = nprobe_q;
  a.target_ids = target_ids; a.target_offsets = target_offsets; a.Lcap = L; a.k = topk;
  a.ids = ids; a.dist = dist; a.qmode = qmode; a.want_mode = want_mode;
  if ((L == 0 || !target_ids) && topk <= kWaveK && nprobe <= kIvfMaxProbe && ws && Q <= 65535) {
    // no candidate cap, or a cap without a target set: who scores which member does not matter,
    // so the members of the probed lists are dealt to the waves of one or more blocks per query
    const int split = ivf_split(Q, nprobe);
    const size_t cstride = align_up((size_t)Q * 4, 256) / 4;
    uint32_t* tau = static_cast<uint32_t*>(ws);
    a.tau_g = tau; a.cand_cnt = tau + cstride; a.done_cnt = tau + 3 * cstride;
    a.cand = reinterpret_cast<uint64_t*>(static_cast<uint8_t*>(ws) + kScanArrays * cstride * 4);
    a.cand_cap = (int64_t)split * topk;
    k_init_scan<<<(Q + 255) / 256, 256, 0, st>>>(tau, Q, (int)cstride, nullptr, 0);
    const size_t ldsw = ivf_w_lds(M, nprobe);
    dim3 grid((unsigned)split, (unsigned)Q);
    DISPATCH_M(M, { int rc = set_lds0(k_ivf_w<MT>, ldsw); if (rc) return rc;
                    k_ivf_w<MT><<<grid, kScanThreads, ldsw, st>>>(a); });
    RII_HIP(hipGetLastError());
    return RII_OK;
  }
  const size_t lds = ivf_lds_main(M) + kBlockVarsBytes;
  DISPATCH_M(M, { int rc = set_lds(k_ivf<MT>, lds); if (rc) return rc;
                  k_ivf<MT><<<Q, kScanThreads, lds, st>>>(a); });
  RII_HIP(hipGetLastError());
  return RII_OK;
}

int rii_adc_scan_ivf(const rii_index_t* idx, const float* lut, int Q, const int32_t* probe_lists, int nprobe,
                     const int32_t* target_ids, const int64_t* target_offsets, int64_t L, int topk, int32_t* ids,
                     float* dist, void* stream) {
  if (!idx || !lut || !probe_lists || !ids || !dist || Q < 1 || topk < 1 || L < 0) return RII_ERR_INVALID_ARG;
  if (idx->K < 1) return RII_ERR_NOT_BUILT;
  if (nprobe < 1 || nprobe > idx->K) return RII_ERR_INVALID_ARG;
  if ((target_ids == nullptr) != (target_offsets == nullptr)) return RII_ERR_INVALID_ARG;
  if (topk > RII_MAX_TOPK || !m_supported(idx->M)) return RII_ERR_UNSUPPORTED;
  if (L >= idx->N) L = 0;  // such a cap never cuts anything
  void* ws = nullptr;
  if ((L == 0 || !target_ids) && topk <= kWaveK) {
    int rc = ensure_ws(idx, ivf_ws_bytes(Q, nprobe, topk));
    if (rc) return rc;
    ws = idx->ws;
  }
  return launch_ivf(idx, lut, Q, probe_lists, nprobe, nprobe, nullptr, target_ids, target_offsets, L, topk, ids,
                    dist, nullptr, 0, ws, static_cast<hipStream_t>(stream));
}

// Scratch layout of the query procedure: tables, per-query plan, probed lists, then the stage
// scratch that the scan, the coarse ranking and the inverted-index scan use one after the other.
struct QueryPlan {
  int pmax = 1;          // most lists any inverted-index query of the batch can ask for
  int64_t lin_rows = 1;  // most rows any linear-scan query of the batch can have
  size_t lut_b = 0, plan_b = 0, probe_b = 0, ivf_b = 0, total = 0;
};

static int plan_query(const rii_index* idx, int Q, int topk, bool targets, int64_t max_targets, int64_t L,
                      QueryPlan* p) {
  const int M = idx->M, K = idx->K;
  const bool has_lists = K > 0;
  // Largest number of lists any inverted-index query of this batch can ask for: such a query
  // has |S| >= max(theta, 1), and |S| = N when there is no target set.
  p->pmax = 1;
  if (has_lists) {
    int64_t smin = targets ? std::max<int64_t>(idx->theta, 1) : idx->N;
    int64_t pl = ((int64_t)K * L + smin - 1) / smin;
    p->pmax = (int)std::min<int64_t>(pl, K);
    if (p->pmax > RII_MAX_TOPK && K > RII_MAX_SORT) return RII_ERR_UNSUPPORTED;
  }
  // linear-scan queries have |S| < theta (and at most max_targets, N)
  int64_t lin_rows = targets ? std::min<int64_t>(max_targets, idx->N) : idx->N;
  if (has_lists && idx->theta > 0) lin_rows = std::min<int64_t>(lin_rows, idx->theta - 1);
  if (has_lists && idx->theta <= 0) lin_rows = 0;
  if (!targets && has_lists && idx->N >= idx->theta) lin_rows = 0;
  p->lin_rows = std::max<int64_t>(lin_rows, 1);
  p->lut_b = align_up((size_t)Q * M * 256 * 4, 256);
  p->plan_b = align_up((size_t)Q * 4, 256);
  p->probe_b = align_up((size_t)Q * p->pmax * 4, 256);
  const size_t scan_b = align_up(scan_ws_bytes(M, Q, p->lin_rows, topk), 256);
  const size_t coarse_b = has_lists ? align_up(coarse_ws_bytes(idx, Q, p->pmax), 256) : 0;
  p->ivf_b = has_lists && topk <= kWaveK ? align_up(ivf_ws_bytes(Q, p->pmax, topk), 256) : 0;
  p->total = p->lut_b + 2 * p->plan_b + p->probe_b + std::max(std::max(scan_b, coarse_b), p->ivf_b);
  return RII_OK;
}

static int check_query_args(const rii_index_t* idx, const float* q, int Q, int topk, const int32_t* target_ids,
                            const int64_t* target_offsets, int64_t max_targets, int64_t L, const int32_t* ids,
                            const float* dist) {
  if (!idx || !q || !ids || !dist || Q < 1 || topk < 1 || L < 1 || max_targets < 0) return RII_ERR_INVALID_ARG;
  if ((target_ids == nullptr) != (target_offsets == nullptr)) return RII_ERR_INVALID_ARG;
  if (topk > RII_MAX_TOPK || !m_supported(idx->M) || Q > 65535) return RII_ERR_UNSUPPORTED;
  if (idx->N < 1) return RII_ERR_INVALID_ARG;
  return RII_OK;
}

// Alg. 3 with its scratch at `ws` (p.total bytes).
static int run_query(const rii_index* idx, const QueryPlan& p, const float* q, int Q, int topk,
                     const int32_t* target_ids, const int64_t* target_offsets, int64_t L, int32_t* ids, float* dist,
                     void* ws, hipStream_t st) {
  const int M = idx->M, K = idx->K;
  const bool has_lists = K > 0;
  uint8_t* w = static_cast<uint8_t*>(ws);
  float* lut = reinterpret_cast<float*>(w); w += p.lut_b;
  int* qmode = reinterpret_cast<int*>(w); w += p.plan_b;
  int* nprobe_q = reinterpret_cast<int*>(w); w += p.plan_b;
  int32_t* probe = reinterpret_cast<int32_t*>(w); w += p.probe_b;
  void* stage_ws = w;

  k_build_lut<<<dim3(M, Q), 256, 0, st>>>(idx->d_cb, q, idx->D, M, idx->Ds, lut);
  k_plan<<<(Q + 255) / 256, 256, 0, st>>>(target_offsets, idx->N, Q, idx->theta, K, L, p.pmax, qmode, nprobe_q);
  int rc = RII_OK;
  // linear-scan branch (mode 0)
  if (target_ids) {
    rc = launch_scan(idx, idx->d_codes_rows, idx->plane_rows, idx->N, lut, Q, kSubset, target_ids, target_offsets, p.lin_rows, topk,
                     ids, dist, topk, qmode, 0, stage_ws, st);
  } else if (!has_lists || idx->N < idx->theta) {
    rc = launch_scan(idx, idx->d_codes, idx->plane_codes, idx->N, lut, Q, kLinear, nullptr, nullptr, idx->N, topk, ids, dist, topk,
                     qmode, 0, stage_ws, st);
  }
  if (rc) return rc;
  // inverted-index branch (mode 1); the scratch of the scan stage is reused in stream order
  if (has_lists) {
    rc = coarse_rank(idx, lut, Q, p.pmax, probe, nullptr, p.pmax, qmode, 1, stage_ws, st);
    if (rc) return rc;
    rc = launch_ivf(idx, lut, Q, probe, p.pmax, p.pmax, nprobe_q, target_ids, target_offsets, L, topk, ids, dist, qmode,
                    1, p.ivf_b ? stage_ws : nullptr, st);
    if (rc) return rc;
  }
  RII_HIP(hipGetLastError());
  return RII_OK;
}

int rii_query(const rii_index_t* idx, const float* q, int Q, int topk, const int32_t* target_ids,
              const int64_t* target_offsets, int64_t max_targets, int64_t L, int32_t* ids, float* dist,
              void* stream) {
  int rc = check_query_args(idx, q, Q, topk, target_ids, target_offsets, max_targets, L, ids, dist);
  if (rc) return rc;
  // L >= N asks for all K lists and never cuts the candidates: N says the same, and K * L then
  // stays far from overflow here and in k_plan
  if (L > idx->N) L = idx->N;
  QueryPlan p;
  rc = plan_query(idx, Q, topk, target_ids != nullptr, max_targets, L, &p);
  if (rc) return rc;
  rc = ensure_ws(idx, p.total);
  if (rc) return rc;
  return run_query(idx, p, q, Q, topk, target_ids, target_offsets, L, ids, dist, idx->ws, static_cast<hipStream_t>(stream));
}

int rii_index_reserve_workspace(rii_index_t* idx, int Q, int topk, int64_t max_targets, int nprobe) {
  if (!idx || Q < 1 || topk < 1 || max_targets < 0 || nprobe < 0) return RII_ERR_INVALID_ARG;
  if (topk > RII_MAX_TOPK || Q > 65535) return RII_ERR_UNSUPPORTED;
  const int M = idx->M, K = idx->K;
  nprobe = std::min(nprobe, std::max(K, 1));
  // every stage's need, as bounds that grow with Q and topk (so smaller batches fit as well)
  size_t stage = scan_ws_bound(M, Q, idx->N, topk);
  if (K > 0 && nprobe > 0) {
    const size_t coarse = nprobe <= RII_MAX_TOPK ? scan_ws_bound(M, Q, K, nprobe)
                                                 : align_up((size_t)Q * K * 4, 256) + align_up((size_t)(Q + 1) * 8, 256);
    const size_t ivf = kScanArrays * align_up((size_t)Q * 4, 256) + ((size_t)Q + kWantBlocks) * topk * 8 + 256;
    stage = std::max(stage, std::max(coarse, ivf));
  }
  const size_t query = align_up((size_t)Q * M * 256 * 4, 256) + 2 * align_up((size_t)Q * 4, 256) +
                       align_up((size_t)Q * std::max(nprobe, 1) * 4, 256) + align_up(stage, 256);
  return ensure_ws(idx, query);
}

// ---- the query procedure without any allocation ---------------------------------------------
// Scratch of rii_query_noalloc: one array per GPU, in the library's own device image.  In host
// code the array's name only stands for it; its device address is asked for once per device
// (with that device current) and kept.
static __device__ __align__(256) unsigned char scratch[RII_NOALLOC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

static int scratch_of_current_device(void** out) {
  int dev = -1;
  RII_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return RII_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    RII_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return RII_ERR_DEVICE;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return RII_OK;
}

int rii_query_noalloc(const rii_index_t* idx, const float* q, int Q, int topk, const int32_t* target_ids,
                      const int64_t* target_offsets, int64_t max_targets, int64_t L, int32_t* ids, float* dist,
                      void* stream) {
  int rc = check_query_args(idx, q, Q, topk, target_ids, target_offsets, max_targets, L, ids, dist);
  if (rc) return rc;
  if (L > idx->N) L = idx->N;
  int dev = -1;
  RII_HIP(hipGetDevice(&dev));
  if (dev != idx->device) return RII_ERR_INVALID_ARG;  // the handle's arrays live on another GPU
  QueryPlan p;
  rc = plan_query(idx, Q, topk, target_ids != nullptr, max_targets, L, &p);
  if (rc) return rc;
  if (p.total > (size_t)RII_NOALLOC_SCRATCH_BYTES) return RII_ERR_UNSUPPORTED;  // beyond the static scratch
  void* ws = nullptr;
  rc = scratch_of_current_device(&ws);
  if (rc) return rc;
  return run_query(idx, p, q, Q, topk, target_ids, target_offsets, L, ids, dist, ws, static_cast<hipStream_t>(stream));
}

int rii_encode_device(const rii_index_t* idx, const float* x, int64_t n, uint8_t* codes_out, void* stream) {
  if (!idx || n < 0 || (n > 0 && (!x || !codes_out))) return RII_ERR_INVALID_ARG;
  if (n == 0) return RII_OK;
  const int Ds = idx->Ds;
  size_t lds = (size_t)512 * Ds * 4;
  if (lds > 160 * 1024) return RII_ERR_UNSUPPORTED;
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rc = set_lds(k_encode, lds);
  if (rc) return rc;
  const int64_t max_rows = (int64_t)1 << 30;
  for (int64_t r0 = 0; r0 < n; r0 += max_rows) {
    int64_t cnt = std::min(max_rows, n - r0);
    dim3 grid((unsigned)((cnt + 255) / 256), (unsigned)idx->M);
    k_encode<<<grid, 256, lds, st>>>(idx->d_cb, x + r0 * idx->D, cnt, idx->D, idx->M, Ds, codes_out + r0 * idx->M);
  }
  RII_HIP(hipGetLastError());
  return RII_OK;
}

int rii_rotate(const float* R, int D, const float* x, int64_t n, float* y, void* stream) {
  if (!R || D < 1 || n < 0 || (n > 0 && (!x || !y)) || x == y) return RII_ERR_INVALID_ARG;
  if (n == 0) return RII_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int64_t rows_per_launch = (int64_t)65535 * 8;
  for (int64_t r0 = 0; r0 < n; r0 += rows_per_launch) {
    int64_t cnt = std::min(rows_per_launch, n - r0);
    dim3 grid((unsigned)((D + 31) / 32), (unsigned)((cnt + 7) / 8));
    k_rotate<<<grid, 256, 0, st>>>(R, D, x + r0 * D, cnt, y + r0 * D);
  }
  RII_HIP(hipGetLastError());
  return RII_OK;
}

// lazily build the symmetric table
int rii_internal_sym_table(const rii_index* cidx, hipStream_t st) {
  rii_index* idx = const_cast<rii_index*>(cidx);
  if (idx->d_sym) return RII_OK;
  RII_HIP(hipMalloc(&idx->d_sym, (size_t)idx->M * 256 * 256 * 4));
  k_sym_table<<<dim3(256, idx->M), 256, 0, st>>>(idx->d_cb, idx->Ds, idx->d_sym);
  RII_HIP(hipGetLastError());
  return RII_OK;
}

// a(n) by brute force.  rot_base >= 0: `codes` is the base of a stored array (planes `plane`
// apart) and the items are its rows rot_base .. rot_base+n-1; rot_base < 0: n plain codes.
int rii_internal_assign(const rii_index* idx, const uint8_t* codes, int64_t n, int64_t rot_base, int64_t plane,
                        const uint8_t* coarse, int K, int32_t* assign_out, hipStream_t st) {
  if (!m_supported(idx->M)) return RII_ERR_UNSUPPORTED;
  if (n == 0) return RII_OK;
  if (!rot_m(idx->M) && rot_base >= 0) { codes += rot_base * idx->M; rot_base = -1; }
  int rc = rii_internal_sym_table(idx, st);
  if (rc) return rc;
  const int M = idx->M;
  const size_t lds = (size_t)M * 1024;
  int blocks = (int)std::min<int64_t>(n, 256 * 16);
  DISPATCH_M(M, { int rc2 = set_lds(k_assign<MT>, lds); if (rc2) return rc2;
                  k_assign<MT><<<blocks, 256, lds, st>>>(idx->d_sym, codes, n, rot_base, plane, M, coarse, K, assign_out); });
  RII_HIP(hipGetLastError());
  return RII_OK;
}

int rii_assign(const rii_index_t* idx, const uint8_t* codes, int64_t n, const uint8_t* coarse, int K,
               int32_t* assign_out, void* stream) {
  if (!idx || n < 0 || K < 1 || !coarse || (n > 0 && (!codes || !assign_out))) return RII_ERR_INVALID_ARG;
  return rii_internal_assign(idx, codes, n, -1, 0, coarse, K, assign_out, static_cast<hipStream_t>(stream));
}

// a(n) with pruning (see k_assign_pruned); all pointers device.  visited_total may be NULL.
int rii_internal_assign_pruned(const rii_index* idx, const uint8_t* codes, int64_t n, int64_t rot_base, int64_t plane,
                               const uint8_t* super, int G,
                               const float* radius, const uint8_t* coarse_g, const int32_t* perm_g,
                               const int32_t* group_off, int32_t* assign_out, unsigned long long* visited_total,
                               hipStream_t st) {
  if (n == 0) return RII_OK;
  if (!rot_m(idx->M) && rot_base >= 0) { codes += rot_base * idx->M; rot_base = -1; }
  int rc = rii_internal_sym_table(idx, st);
  if (rc) return rc;
  const int M = idx->M;
  const size_t lds = (size_t)M * 1024 + (size_t)G * 4;
  if (lds > 150 * 1024) return RII_ERR_UNSUPPORTED;
  int blocks = (int)std::min<int64_t>(n, 256 * 32);
  DISPATCH_M(M, { int rc2 = set_lds(k_assign_pruned<MT>, lds); if (rc2) return rc2;
                  k_assign_pruned<MT><<<blocks, 256, lds, st>>>(idx->d_sym, codes, n, rot_base, plane, M, super, G, radius,
                                                               coarse_g,
                                                               perm_g, group_off, assign_out, visited_total); });
  RII_HIP(hipGetLastError());
  return RII_OK;
}

// a(n) of every stored item from the installed posting lists (device buffer of N entries)
int rii_internal_assign_from_lists(const rii_index* idx, int32_t* d_out, hipStream_t st) {
  if (idx->N == 0) return RII_OK;
  const int64_t per = (int64_t)1 << 30;
  if (idx->N > per * 2 - 1) return RII_ERR_UNSUPPORTED;
  k_assign_from_lists<<<(unsigned)((idx->N + 255) / 256), 256, 0, st>>>(idx->d_list_off, idx->d_list_ids, idx->K, idx->N, d_out);
  RII_HIP(hipGetLastError());
  return RII_OK;
}

// used by the threshold calibration in rii_index.hip
int rii_internal_spread_ids(int32_t* ids, int64_t* offsets, int nq, int64_t S, int64_t N, hipStream_t st) {
  int64_t total = std::max<int64_t>((int64_t)nq * S, nq + 1);
  k_spread_ids<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(ids, offsets, nq, S, N);
  RII_HIP(hipGetLastError());
  return RII_OK;
}

// used by rii_index.hip: see k_copy_rows.  For M without a stored form the rotation arguments only
// select the first row of the (plain) arrays.
int rii_internal_copy_rows(const uint8_t* in, int64_t in_rot, int64_t in_plane, const int32_t* ids, int64_t n, int M,
                           uint8_t* out, int64_t out_rot, int64_t out_plane, hipStream_t st) {
  if (n == 0) return RII_OK;
  if (!rot_m(M)) {
    if (in_rot > 0) in += in_rot * M;
    if (out_rot > 0) out += out_rot * M;
    in_rot = out_rot = -1;
  }
  const int M4 = M / 4;
  const int64_t per = ((int64_t)1 << 30) / M4;  // rows per launch
  for (int64_t r0 = 0; r0 < n; r0 += per) {
    int64_t cnt = std::min<int64_t>(per, n - r0);
    int64_t dw = cnt * M4;
    // rows r0.. of this call: shift the row bases of stored arrays, the pointers of plain ones
    const bool seq = !ids;  // source rows follow the output rows
    k_copy_rows<<<(unsigned)((dw + 255) / 256), 256, 0, st>>>(
        seq && in_rot < 0 ? in + r0 * M : in, seq && in_rot >= 0 ? in_rot + r0 : in_rot, in_plane,
        ids ? ids + r0 : nullptr, cnt, M, out_rot < 0 ? out + r0 * M : out, out_rot >= 0 ? out_rot + r0 : out_rot,
        out_plane);
  }
  RII_HIP(hipGetLastError());
  return RII_OK;
}

}  // extern "C"
