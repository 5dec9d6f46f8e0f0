// HIP kernels (gfx950) and the device-side entry points of the library.
//
// Data flow of one query batch:
//   k_build_lut        q, codebooks                       -> A [Q][M][256]          (Sec. 3)
//   k_scan<LINEAR>     A in LDS, codes streamed           -> per-block top-R keys   (Alg. 1, whole data)
//   k_scan<SUBSET>     A in LDS, codes gathered by id     -> per-block top-R keys   (Alg. 1, subset)
//   k_ivf              A in LDS, probed lists streamed    -> top-R                  (Alg. 2, second block)
//   k_select           keys / candidates                  -> top-R sorted           (PartialSort + Take)
//
// A candidate is one 64-bit key: order-preserving image of the fp32 distance in the high word,
// identifier in the low word.  Comparing keys as unsigned integers is the (distance,
// identifier) order, so selection is exact and deterministic including ties.

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <vector>

#include "rii_internal.h"

namespace {

// Launch shape of the scan kernels.  The values were chosen by sweeping them on the 100M-code
// configuration (M = 32): one 1024-thread block per CU, 4 rows per lane per tile.
constexpr int kSelCap = 2048;          // keys held per block between compactions (2 * RII_MAX_TOPK)
constexpr int kScanThreads = 1024;
constexpr int kRowsPerLane = 4;        // rows scored per lane per tile
constexpr int kWantBlocks = 256;       // blocks a small batch is split into (the chip has 256 CUs)
constexpr int kMinTiles = 4;           // shortest chunk, in tiles
constexpr int kPrepassBlocks = 256;    // blocks (tiles) of the bound-seeding pass, per query
// Block-shared scalars of the streaming kernels.  They live at the END of the dynamic LDS
// allocation: a kernel with no static __shared__ object gets its dynamic LDS at address 0, and
// then the byte-permuted table address (see adc_row_rot) is the LDS address itself -- with static
// objects in front the compiler has to add their size to every look-up address.
struct BlockVars {
  int total, off, last;
  uint32_t tg;
  int cnt;
  uint32_t tau;
  float red[16];
  float scale[4];
  int wave_cnt[16];
};
constexpr size_t kBlockVarsBytes = 256;
static_assert(sizeof(BlockVars) <= kBlockVarsBytes, "BlockVars must fit its slot");

constexpr uint64_t kKeyMax = ~0ull;
constexpr uint32_t kOrdMax = 0xFFFFFFFFu;
constexpr uint32_t kOrdInf = 0xFF800000u;  // ord_of(+infinity)

// ------------------------------------------------------------------ keys
__device__ __forceinline__ uint32_t ord_of(float d) {
  uint32_t b = __float_as_uint(d);
  return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float float_of_ord(uint32_t o) {
  uint32_t b = o ^ ((o >> 31) ? 0x80000000u : 0xFFFFFFFFu);
  return __uint_as_float(b);
}
__device__ __forceinline__ uint64_t make_key(float d, int32_t id) {
  return ((uint64_t)ord_of(d) << 32) | (uint32_t)id;
}

// ------------------------------------------------------------------ block-level selection
// keys[0..kSelCap) in LDS, *cnt entries used, *tau = largest distance image still of interest.

__device__ __forceinline__ int next_pow2(int v) {
  int p = 2;
  while (p < v) p <<= 1;
  return p;
}

// Ascending bitonic sort of keys[0..n2), n2 a power of two.  Block-wide; ends with a barrier.
// With first_size > 2 the stages below first_size are skipped: the caller guarantees that the
// runs of first_size/2 keys are already sorted, alternately ascending and descending.
__device__ void block_bitonic_sort(uint64_t* keys, int n2, int first_size = 2) {
  const int tid = threadIdx.x, nthr = blockDim.x;
  for (int size = first_size; size <= n2; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int t = tid; t < (n2 >> 1); t += nthr) {
        int i = 2 * t - (t & (stride - 1));
        int j = i + stride;
        bool up = ((i & size) == 0);
        uint64_t a = keys[i], b = keys[j];
        if ((a > b) == up) {
          keys[i] = b;
          keys[j] = a;
        }
      }
      __syncthreads();
    }
  }
}

// Keep the k smallest keys (sorted ascending) and tighten *tau.  Must be entered by all threads
// after a barrier that follows the last push.
__device__ void sel_compact(uint64_t* keys, int* cnt, uint32_t* tau, int k) {
  const int tid = threadIdx.x, nthr = blockDim.x;
  int c = *cnt;
  if (c > kSelCap) c = kSelCap;
  int n2 = next_pow2(c);
  for (int i = c + tid; i < n2; i += nthr) keys[i] = kKeyMax;
  __syncthreads();
  block_bitonic_sort(keys, n2);
  if (tid == 0) {
    *cnt = c < k ? c : k;
    if (c >= k) {
      uint32_t t = (uint32_t)(keys[k - 1] >> 32);
      if (t < *tau) *tau = t;
    }
  }
  __syncthreads();
}

// Offer up to R keys per thread (bit r of `pend` set: key[r] is a candidate).  Block-wide:
// every thread of the block must call it, the same number of times.  Returns true when a
// compaction happened (tau may have changed).
template <int R>
__device__ bool sel_offer(uint64_t* keys, int* cnt, uint32_t* tau, int k, const uint64_t (&key)[R], uint32_t pend) {
  bool compacted = false;
  while (__syncthreads_or((int)pend)) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (pend & (1u << r)) {
        int idx = atomicAdd(cnt, 1);
        if (idx < kSelCap) {
          keys[idx] = key[r];
          pend &= ~(1u << r);
        }
      }
    }
    __syncthreads();
    if (*cnt >= kSelCap) {  // uniform: nobody changes *cnt before the next barrier
      sel_compact(keys, cnt, tau, k);
      compacted = true;
      uint32_t t = *tau;
#pragma unroll
      for (int r = 0; r < R; ++r)
        if ((pend & (1u << r)) && (uint32_t)(key[r] >> 32) > t) pend &= ~(1u << r);
    }
  }
  return compacted;
}

// ------------------------------------------------------------------ distance tables (Sec. 3)
// grid (M, Q), block 256: thread z computes A(m, z) for query blockIdx.y.
__global__ void k_build_lut(const float* __restrict__ cb, const float* __restrict__ q, int D, int M, int Ds,
                            float* __restrict__ lut) {
  const int m = blockIdx.x, z = threadIdx.x;
  const int64_t qi = blockIdx.y;
  const float* qs = q + qi * D + m * Ds;
  const float* c = cb + ((size_t)m * 256 + z) * Ds;
  float acc = 0.f;
  for (int j = 0; j < Ds; ++j) {
    float diff = __fsub_rn(qs[j], c[j]);
    acc = __fadd_rn(acc, __fmul_rn(diff, diff));
  }
  lut[(qi * M + m) * 256 + z] = acc;
}

// ------------------------------------------------------------------ ADC of one row (Eq. 2)
// Loads the M code bytes of one row with the widest aligned loads M allows and sums the M
// table entries in ascending sub-space order.
template <int MT>
__device__ __forceinline__ float adc_row(const float* __restrict__ A, const uint8_t* __restrict__ row, int Mrt) {
  float d = 0.f;
  if constexpr (MT == 0) {
    // run-time M (a multiple of 4)
    const uint32_t* w = reinterpret_cast<const uint32_t*>(row);
    for (int j = 0; j < (Mrt >> 2); ++j) {
      uint32_t v = w[j];
#pragma unroll
      for (int b = 0; b < 4; ++b) d = __fadd_rn(d, A[(4 * j + b) * 256 + ((v >> (8 * b)) & 255u)]);
    }
  } else if constexpr (MT % 16 == 0) {
    uint32_t w[MT / 4];
    const uint4* p = reinterpret_cast<const uint4*>(row);
#pragma unroll
    for (int j = 0; j < MT / 16; ++j) {
      uint4 v = p[j];
      w[4 * j] = v.x; w[4 * j + 1] = v.y; w[4 * j + 2] = v.z; w[4 * j + 3] = v.w;
    }
#pragma unroll
    for (int m = 0; m < MT; ++m) d = __fadd_rn(d, A[m * 256 + ((w[m >> 2] >> (8 * (m & 3))) & 255u)]);
  } else {
    static_assert(MT == 8, "specialised for M = 8, 16, 32, 64");
    uint2 v = *reinterpret_cast<const uint2*>(row);
    uint32_t w[2] = {v.x, v.y};
#pragma unroll
    for (int m = 0; m < 8; ++m) d = __fadd_rn(d, A[m * 256 + ((w[m >> 2] >> (8 * (m & 3))) & 255u)]);
  }
  return d;
}

// ------------------------------------------------------------------ rotated rows (M = 8, 16, 32)
// For these M the stored code arrays keep row r rotated by r bytes: stored[r][t] = code[r][(t + r) % M].
// The table sits in LDS as T[z][s], 64 slots of 4 bytes per code value z, slot s holding
// A[s % M][z].  A lane scoring row r reads slot (r % 32) + t at step t, i.e. sub-space (r + t) % M
// -- exactly the sub-space stored byte t belongs to.  32 consecutive rows (one per lane) hit 32
// different LDS banks at every step whatever the code values are: no bank conflicts, and the byte
// position t is the same in all lanes, so the address is one v_perm_b32 away from the loaded dword
// (row stride 256 bytes puts z into byte 1).
// The sum then runs over the sub-spaces in rotated order; its fp32 rounding differs from the
// ascending-m sum the results are defined with, so it is used as a filter only: a row whose
// rotated sum is not above (1 + kRotEps(M)) * bound has its ascending-m sum recomputed exactly.
__host__ __device__ constexpr bool rot_m(int M) { return M == 8 || M == 16 || M == 32; }

// The look-up table of the streaming kernels sits at LDS address 0 (they have no static
// __shared__ object, and the host side verifies it: see require_table_at_lds_zero), so the
// byte-permuted value IS the LDS address.  Reading through an address-space-3 pointer made from
// that integer keeps the compiler from adding the (zero) address of the dynamic LDS symbol to
// every look-up.
typedef __attribute__((address_space(3))) const float lds_float;
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) const f32x2_t lds_float2;
typedef __attribute__((address_space(3))) const u32x2_t lds_uint2;
__device__ __forceinline__ float lds_read_f32(uint32_t addr) { return *reinterpret_cast<lds_float*>((uintptr_t)addr); }
__device__ __forceinline__ float2 lds_read_f32x2(uint32_t addr) {
  f32x2_t v = *reinterpret_cast<lds_float2*>((uintptr_t)addr);
  return make_float2(v.x, v.y);
}
__device__ __forceinline__ uint2 lds_read_u32x2(uint32_t addr) {
  u32x2_t v = *reinterpret_cast<lds_uint2*>((uintptr_t)addr);
  return make_uint2(v.x, v.y);
}
// LDS bytes of one query's table: 256 x 64 slots in the rotated layout, [M][256] otherwise.
__host__ __device__ constexpr size_t table_bytes(int M) { return rot_m(M) ? (size_t)65536 : (size_t)M * 1024; }
// LDS of the bound-seeding kernel: the table plus, in the rotated layout, the staging copy used to fill it.
__host__ __device__ constexpr size_t tau0_lds(int M) { return table_bytes(M) + (rot_m(M) ? (size_t)M * 1024 : 0); }
// LDS of the single-block inverted-index kernel before its BlockVars: table + max(keys, staging copy).
__host__ __device__ constexpr size_t ivf_lds_main(int M) {
  return table_bytes(M) + ((size_t)2048 * 8 > (rot_m(M) ? (size_t)M * 1024 : 0) ? (size_t)2048 * 8 : (size_t)M * 1024);
}

// Both sums are within (M-1) u / (1 - (M-1) u) of the exact real sum of non-negative terms
// (u = 2^-24), so they differ by less than a factor 1 + (M-1) 2^-23; M 2^-22 leaves room for
// the rounding of the product bound * (1 + eps) itself.
__device__ __forceinline__ float rot_eps(int M) { return (float)M * 2.384185791015625e-07f; }

// Fill T from the query's table A = lut[M][256].  The table is first copied to `stage` (LDS,
// M KB, coalesced reads), then transposed into T along diagonals: lane l of a group of 32 moves
// element (z0 + l, (s0 + l) % 64), so both the read (bank z % 32) and the write (bank s % 32) touch 32
// different banks.  Block-wide; ends with a barrier.  `stage` may be reused afterwards.
template <int MT>
__device__ __forceinline__ void fill_table_rot(float* T, float* stage, const float* __restrict__ lut) {
  for (int i = threadIdx.x; i < MT * 256; i += blockDim.x) stage[i] = lut[i];
  __syncthreads();
  for (int it = threadIdx.x; it < 256 * 64; it += blockDim.x) {
    const int l = it & 31, blk = it >> 5;
    const int s0 = blk & 63, z0 = (blk >> 6) << 5;
    const int z = z0 + l, s = (s0 + l) & 63;
    T[z * 64 + s] = stage[(s & (MT - 1)) * 256 + z];
  }
  __syncthreads();
}

// The MT code bytes of one stored row as MT/4 words (16-byte loads for M >= 16).
template <int MT>
__device__ __forceinline__ void load_row_words(const uint8_t* __restrict__ row, uint32_t (&w)[MT / 4]) {
  if constexpr (MT == 8) {
    uint2 v = *reinterpret_cast<const uint2*>(row);
    w[0] = v.x; w[1] = v.y;
  } else {
    const uint4* p = reinterpret_cast<const uint4*>(row);
#pragma unroll
    for (int j = 0; j < MT / 16; ++j) {
      uint4 v = p[j];
      w[4 * j] = v.x; w[4 * j + 1] = v.y; w[4 * j + 2] = v.z; w[4 * j + 3] = v.w;
    }
  }
}

// Look-ups after which k_scan_w tests whether a whole wavefront can abandon a slice (half-way
// through the row; anywhere between 1/2 and 3/4 measured the same).  With four queries per
// block (k_scan_w4) the test hardly ever succeeds and was measured to cost more than it saves.
template <int MT> constexpr int kAbandonAt = MT / 2;

// One segment of a stored row: kRotSeg<MT> bytes (16, or 8 for M = 8), as words.
template <int MT> constexpr int kRotSeg = MT >= 16 ? 16 : 8;
template <int MT>
__device__ __forceinline__ void load_row_segment(const uint8_t* __restrict__ row, int seg, uint32_t* w) {
  if constexpr (MT == 8) {
    uint2 v = *reinterpret_cast<const uint2*>(row);
    w[0] = v.x; w[1] = v.y;
  } else {
    uint4 v = reinterpret_cast<const uint4*>(row)[seg];
    w[4 * seg] = v.x; w[4 * seg + 1] = v.y; w[4 * seg + 2] = v.z; w[4 * seg + 3] = v.w;
  }
}

// Rotated-order sum for one stored row given as words; lanebase = (row % 32) * 4.  kAtZero: T is
// known to start at LDS address 0 (kernels without static LDS); otherwise T's address is added
// per look-up.
template <int MT, bool kAtZero = true>
__device__ __forceinline__ float adc_words_rot(const float* T, const uint32_t (&w)[MT / 4], uint32_t lanebase) {
  float d = 0.f;
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    // byte 0 <- lanebase, byte 1 <- code byte t, bytes 2,3 <- 0
    uint32_t addr = __builtin_amdgcn_perm(w[t >> 2], lanebase, 0x0c0c0400u | ((uint32_t)(t & 3) << 8));
    if constexpr (kAtZero) d = __fadd_rn(d, lds_read_f32(addr + t * 4));
    else d = __fadd_rn(d, *reinterpret_cast<const float*>(reinterpret_cast<const char*>(T) + addr + t * 4));
  }
  return d;
}

// The two halves of adc_words_rot for the software-pipelined loops: first all LDS addresses of a
// row (after which its code words are dead and the registers can take the next tile's row) ...
template <int MT>
__device__ __forceinline__ void rot_addrs(const uint32_t (&w)[MT / 4], uint32_t lanebase, uint32_t (&addr)[MT]) {
#pragma unroll
  for (int t = 0; t < MT; ++t)
    addr[t] = __builtin_amdgcn_perm(w[t >> 2], lanebase, 0x0c0c0400u | ((uint32_t)(t & 3) << 8));
}
// ... then the look-ups, table at LDS address 0
template <int MT>
__device__ __forceinline__ float rot_sum(const uint32_t (&addr)[MT]) {
  float d = 0.f;
#pragma unroll
  for (int t = 0; t < MT; ++t) d = __fadd_rn(d, lds_read_f32(addr[t] + t * 4));
  return d;
}
// The same with early abandoning: the entries are squared distances (>= 0) and adding one never
// lowers a sum, so a partial sum above the filter bound fb settles the row; when that holds in
// every lane the wave skips the remaining look-ups (the value returned is then only known to
// exceed fb).
template <int MT>
__device__ __forceinline__ float rot_sum_abandon(const uint32_t (&addr)[MT], float fb) {
  float d = 0.f;
#pragma unroll
  for (int t = 0; t < kAbandonAt<MT>; ++t) d = __fadd_rn(d, lds_read_f32(addr[t] + t * 4));
  if (__ballot(d <= fb) == 0ull) return d;
#pragma unroll
  for (int t = kAbandonAt<MT>; t < MT; ++t) d = __fadd_rn(d, lds_read_f32(addr[t] + t * 4));
  return d;
}

template <int MT, bool kAtZero = true>
__device__ __forceinline__ float adc_row_rot(const float* T, const uint8_t* __restrict__ row, uint32_t lanebase) {
  uint32_t w[MT / 4];
  load_row_words<MT>(row, w);
  return adc_words_rot<MT, kAtZero>(T, w, lanebase);
}

// Ascending-m sum for stored row number r (rotated storage), table in the T layout.
template <int MT>
__device__ __forceinline__ float adc_row_exact_rot(const float* T, const uint8_t* __restrict__ row, int64_t r) {
  float d = 0.f;
#pragma unroll 4
  for (int m = 0; m < MT; ++m) d = __fadd_rn(d, T[(int)row[(m - (int)r) & (MT - 1)] * 64 + m]);
  return d;
}

// Ascending-m sum for stored row number r (rotated storage), table in the plain [m][z] layout.
template <int MT>
__device__ __forceinline__ float adc_row_unrot(const float* A, const uint8_t* __restrict__ row, int64_t r) {
  float d = 0.f;
#pragma unroll 4
  for (int m = 0; m < MT; ++m) d = __fadd_rn(d, A[m * 256 + row[(m - (int)r) & (MT - 1)]]);
  return d;
}

// Upper bound, as a float, for the rotated sum of any row whose ascending-m sum has an image <= bound.
__device__ __forceinline__ float rot_filter(uint32_t bound, float eps) {
  if (bound == kOrdMax) return __uint_as_float(0x7F800000u);
  float f = float_of_ord(bound);
  return __fadd_rn(f, __fmul_rn(f, eps));
}

// ------------------------------------------------------------------ scan (Alg. 1)
struct ScanArgs {
  const uint8_t* codes;          // [N][M]
  int64_t N;
  int M;
  const float* lut;              // [Q][M][256]
  const int32_t* target_ids;     // subset mode
  const int64_t* target_offsets; // subset mode, [Q+1]
  int64_t chunk_rows;            // rows (or targets) per block
  int k;
  uint64_t* partial;             // [Q][cand_cap] candidate keys appended by the blocks
  uint32_t* cand_cnt;            // [Q] number of candidates appended
  int64_t cand_cap;              // gridDim.x * k
  uint32_t* tau_g;               // [Q] shared distance bound per query
  const int* qmode;              // optional [Q]; block runs only when qmode[q] == want_mode
  int want_mode;
  uint32_t* done_cnt;            // [Q] blocks finished (the last one selects the result)
  int32_t* ids;                  // result [Q][out_stride] (written by k_scan_w only)
  float* dist;
  int out_stride;
  uint32_t* minima;              // bound-seeding pass: [Q][gridDim.x * waves] smallest distance image per wave
  uint32_t* counter;             // bound-seeding pass: [Q] blocks finished
  int nq;                        // k_scan_w4: queries in the batch (the last group may be short)
  int seed_inside;               // k_scan_w: seed the shared bound inside the kernel (see there)
};

enum { kLinear = 0, kSubset = 1 };

template <int MT, int MODE>
__global__ __launch_bounds__(kScanThreads) void k_scan(ScanArgs a) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int M = MT ? MT : a.M;
  float* A = reinterpret_cast<float*>(smem);
  uint64_t* keys = reinterpret_cast<uint64_t*>(smem + (size_t)M * 1024);
  __shared__ int s_cnt;
  __shared__ uint32_t s_tau;

  const int tid = threadIdx.x;
  const int64_t q = blockIdx.y;
  uint64_t* cand = a.partial + q * a.cand_cap;
  if (a.qmode && a.qmode[q] != a.want_mode) return;

  int64_t nrows;
  const int32_t* tids = nullptr;
  if (MODE == kLinear) {
    nrows = a.N;
  } else {
    int64_t o0 = a.target_offsets[q];
    nrows = a.target_offsets[q + 1] - o0;
    tids = a.target_ids + o0;
  }
  const int64_t r0 = (int64_t)blockIdx.x * a.chunk_rows;
  const int64_t r1 = r0 + a.chunk_rows < nrows ? r0 + a.chunk_rows : nrows;
  if (r0 >= r1) return;

  const float* lut = a.lut + q * M * 256;
  for (int i = tid; i < M * 256; i += blockDim.x) A[i] = lut[i];
  if (tid == 0) {
    s_cnt = 0;
    s_tau = kOrdMax;
  }
  __syncthreads();

  for (int64_t tile = r0; tile < r1; tile += (int64_t)blockDim.x * kRowsPerLane) {
    uint64_t key[kRowsPerLane];
    uint32_t pend = 0;
    uint32_t tau = s_tau;
    uint32_t tg = __hip_atomic_load(a.tau_g + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (tg < tau) tau = tg;
#pragma unroll
    for (int r = 0; r < kRowsPerLane; ++r) {
      int64_t i = tile + (int64_t)r * blockDim.x + tid;
      key[r] = kKeyMax;
      if (i < r1) {
        int32_t id = MODE == kLinear ? (int32_t)i : tids[i];
        float d;
        if constexpr (rot_m(MT)) d = adc_row_unrot<MT>(A, a.codes + (int64_t)id * M, id);
        else d = adc_row<MT>(A, a.codes + (int64_t)id * M, M);
        key[r] = make_key(d, id);
        if ((uint32_t)(key[r] >> 32) <= tau) pend |= 1u << r;
      }
    }
    if (sel_offer<kRowsPerLane>(keys, &s_cnt, &s_tau, a.k, key, pend)) {
      if (tid == 0) atomicMin(a.tau_g + q, s_tau);
    }
  }
  __syncthreads();
  sel_compact(keys, &s_cnt, &s_tau, a.k);
  if (tid == 0) atomicMin(a.tau_g + q, s_tau);
  const int c = s_cnt;
  __shared__ uint32_t s_base;
  if (tid == 0) s_base = c ? atomicAdd(a.cand_cnt + q, (uint32_t)c) : 0u;
  __syncthreads();
  for (int i = tid; i < c; i += blockDim.x) cand[s_base + i] = keys[i];
}

__device__ __forceinline__ void write_result(const uint64_t* keys, int c, int k, int32_t* ids, float* dist);

// ------------------------------------------------------------------ scan with per-wave selection
// For topk <= kWaveK every wavefront keeps its own candidate buffer (kWaveCap keys in LDS) and
// its own distance bound, so the loop over the rows has no block barrier: a wave that has no
// candidate in a tile (the common case once its bound has tightened) just goes on streaming.
// A full buffer is compacted by the wave alone (bitonic sort of its kWaveCap keys).  At the end
// the waves' sorted buffers are merged by the block.
constexpr int kWaveK = 128;
constexpr int kWaveCap = 256;
constexpr int kUnitTiles = 8;  // wave-tiles per unit of rows taken by a wave of k_scan_w
constexpr long long kSeedWaitTicks = 5000;   // longest wait for the seeded bound, in ticks of the 100 MHz clock (50 us)

// Cross-block hand-over without cache-wide fences: the data is written with agent-scope
// atomic stores (which go through to the coherence point), the writer waits for its own stores
// to complete, and only then takes its ticket; the reader uses agent-scope atomic loads.
__device__ __forceinline__ void wait_own_memory_ops() { __builtin_amdgcn_s_waitcnt(0); }

__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  __builtin_amdgcn_wave_barrier();
}

// Ascending bitonic sort of buf[0..n2) by one wavefront (n2 a power of two, at most kWaveCap).
__device__ __forceinline__ void wave_bitonic_sort(uint64_t* buf, int n2, int lane) {
  for (int size = 2; size <= n2; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int t = lane; t < (n2 >> 1); t += 64) {
        int i = 2 * t - (t & (stride - 1));
        int j = i + stride;
        bool up = ((i & size) == 0);
        uint64_t a = buf[i], b = buf[j];
        if ((a > b) == up) {
          buf[i] = b;
          buf[j] = a;
        }
      }
      wave_sync();
    }
  }
}

// Sort the wave's buffer, keep its k smallest keys, tighten the wave's bound.
__device__ __forceinline__ void wave_compact(uint64_t* buf, int& cnt, uint32_t& tau, int k, int lane) {
  int n2 = next_pow2(cnt);
  for (int i = cnt + lane; i < n2; i += 64) buf[i] = kKeyMax;
  wave_sync();
  wave_bitonic_sort(buf, n2, lane);
  if (cnt >= k) {
    cnt = k;
    uint32_t t = (uint32_t)(buf[k - 1] >> 32);
    if (t < tau) tau = t;
  }
}

// `cap` = keys the wave's buffer holds (kWaveCap unless the kernel says otherwise; must exceed k).
template <int R>
__device__ __forceinline__ void wave_offer(uint64_t* buf, int& cnt, uint32_t& tau, int k, const uint64_t (&key)[R],
                                           uint32_t pend, int lane, int cap = kWaveCap) {
#pragma unroll
  for (int r = 0; r < R; ++r) {
    bool p = ((pend >> r) & 1u) && (uint32_t)(key[r] >> 32) <= tau;
    unsigned long long m;
    while ((m = __ballot(p)) != 0ull) {
      const int room = cap - cnt;
      const int rank = __popcll(m & ((1ull << lane) - 1ull));
      const int n = __popcll(m);
      if (p && rank < room) {
        buf[cnt + rank] = key[r];
        p = false;
      }
      cnt += n < room ? n : room;
      if (cnt == cap) {
        wave_sync();
        wave_compact(buf, cnt, tau, k, lane);
        p = p && (uint32_t)(key[r] >> 32) <= tau;
      }
    }
  }
}

// Bound-seeding pass.  Block b of query q scores the b-th tile of the query's rows; every wave
// records the smallest distance among its rows.  The k-th smallest of these minima belongs to
// k different rows, so it bounds the k-th smallest distance of the whole scan from above.  The
// block that finishes last selects it (one wave, bit-by-bit search) and stores it in tau_g.
template <int MT, int MODE>
__global__ __launch_bounds__(kScanThreads) void k_tau0(ScanArgs a) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int M = MT ? MT : a.M;
  float* A = reinterpret_cast<float*>(smem);
  BlockVars* bv = reinterpret_cast<BlockVars*>(smem + tau0_lds(M));
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nwaves = blockDim.x >> 6;
  const int64_t q = blockIdx.y;
  if (a.qmode && a.qmode[q] != a.want_mode) return;
  int64_t nrows;
  const int32_t* tids = nullptr;
  if (MODE == kLinear) {
    nrows = a.N;
  } else {
    int64_t o0 = a.target_offsets[q];
    nrows = a.target_offsets[q + 1] - o0;
    tids = a.target_ids + o0;
  }
  const int G = gridDim.x * nwaves;
  uint32_t* minima = a.minima + q * G;
  const int64_t r0 = (int64_t)blockIdx.x * blockDim.x * kRowsPerLane;
  uint32_t best = kOrdMax;
  if (r0 < nrows) {  // block-uniform
    const float* lut = a.lut + q * M * 256;
    if constexpr (rot_m(MT)) {
      fill_table_rot<MT>(A, A + 256 * 64, lut);
    } else {
      for (int i = tid; i < M * 256; i += blockDim.x) A[i] = lut[i];
      __syncthreads();
    }
#pragma unroll
    for (int r = 0; r < kRowsPerLane; ++r) {
      int64_t i = r0 + (int64_t)r * blockDim.x + tid;
      if (i < nrows) {
        int32_t id = MODE == kLinear ? (int32_t)i : tids[i];
        float d;
        if constexpr (rot_m(MT)) {
          // rotated-order sum, raised so that it bounds the row's ascending-m sum from above
          d = adc_row_rot<MT>(A, a.codes + (int64_t)id * M, ((uint32_t)id & 31u) << 2);
          d = __fadd_rn(d, __fmul_rn(d, rot_eps(MT)));
        } else {
          d = adc_row<MT>(A, a.codes + (int64_t)id * M, M);
        }
        uint32_t o = ord_of(d);
        if (o < best) best = o;
      }
    }
    for (int o = 32; o > 0; o >>= 1) {
      uint32_t other = __shfl_xor(best, o, 64);
      if (other < best) best = other;
    }
  }
  if (lane == 0) __hip_atomic_store(minima + blockIdx.x * nwaves + wave, best, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  wait_own_memory_ops();
  __syncthreads();
  if (tid == 0) bv->last = atomicAdd(a.counter + q, 1u) == gridDim.x - 1;
  __syncthreads();
  if (!bv->last || wave != 0) return;
  // k-th smallest of the G minima, most significant bit first: bit b of the answer is 0 when at
  // least k values lie below (answer | 1 << b).  Each lane keeps its share of the values in registers.
  const int k = a.k;
  if (G < k) return;
  constexpr int kPerLane = kPrepassBlocks * (kScanThreads / 64) / 64;
  uint32_t v[kPerLane];
#pragma unroll
  for (int j = 0; j < kPerLane; ++j) {
    int i = lane + 64 * j;
    v[j] = i < G ? __hip_atomic_load(minima + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : kOrdMax;
  }
  uint32_t ans = 0;
  for (int b = 31; b >= 0; --b) {
    const uint32_t trial = ans | (1u << b);
    int c = 0;
#pragma unroll
    for (int j = 0; j < kPerLane; ++j) c += v[j] < trial;
    for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, 64);
    if (c < k) ans = trial;
  }
  if (lane == 0 && ans != kOrdMax) atomicMin(a.tau_g + q, ans);
}

// The waves of a block hold cnt keys each in their buffers.  Leaves the block's k smallest keys
// (of those not above `bound`), sorted ascending, at (*out)[0..c) and returns c.  Block-wide;
// ends with a barrier.  wbuf = [nwaves][cap] wave buffers followed by one more cap keys.
__device__ int block_collect(uint64_t* wbuf, int nwaves, int cnt, uint32_t tau, uint32_t bound, int k,
                             uint64_t** out, int* s_total, int* s_off, int cap = kWaveCap) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint64_t* buf = wbuf + (size_t)wave * cap;
  uint64_t* small = wbuf + (size_t)nwaves * cap;
  if (tid == 0) {
    *s_total = 0;
    *s_off = 0;
  }
  wave_sync();
  // Fast path: when only a few keys can still matter, gather them and let one wave sort them.
  int nsurv = 0;
  for (int i0 = 0; i0 < cnt; i0 += 64) {
    int i = i0 + lane;
    bool keep = i < cnt && (uint32_t)(buf[i] >> 32) <= bound;
    nsurv += __popcll(__ballot(keep));
  }
  __syncthreads();
  if (lane == 0 && nsurv) atomicAdd(s_total, nsurv);
  __syncthreads();
  const int total = *s_total;
  if (total <= cap) {
    int base = 0;
    if (lane == 0 && nsurv) base = atomicAdd(s_off, nsurv);
    base = __shfl(base, 0, 64);
    for (int i0 = 0; i0 < cnt; i0 += 64) {
      int i = i0 + lane;
      bool keep = i < cnt && (uint32_t)(buf[i] >> 32) <= bound;
      unsigned long long m = __ballot(keep);
      if (keep) small[base + __popcll(m & ((1ull << lane) - 1ull))] = buf[i];
      base += __popcll(m);
    }
    __syncthreads();
    if (wave == 0) {
      int c = total;
      uint32_t t = kOrdMax;
      wave_compact(small, c, t, k, lane);
    }
    __syncthreads();
    *out = small;
    return total < k ? total : k;
  }
  // General path: every wave sorts what it holds and keeps at most k keys; the runs (kp keys
  // each, alternately ascending / descending, padded with the largest key) are packed at the
  // start of the buffer area and merged by the last stages of a block-wide bitonic sort.
  wave_compact(buf, cnt, tau, k, lane);
  if (cnt > k) cnt = k;
  const int kp = next_pow2(k);
  uint64_t mine[kWaveK / 64];
#pragma unroll
  for (int j = 0; j < kWaveK / 64; ++j) {
    int i = lane + 64 * j;
    mine[j] = (i < cnt) ? buf[i] : kKeyMax;
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kWaveK / 64; ++j) {
    int i = lane + 64 * j;
    if (i < kp) wbuf[(size_t)wave * kp + ((wave & 1) ? (kp - 1 - i) : i)] = mine[j];
  }
  __syncthreads();
  block_bitonic_sort(wbuf, nwaves * kp, 2 * kp);
  // the first c <= k keys are real candidates (the padding sorts last)
  if (tid == 0) *s_total = 0;
  __syncthreads();
  if (tid < k && wbuf[tid] != kKeyMax && (tid == k - 1 || wbuf[tid + 1] == kKeyMax)) *s_total = tid + 1;
  __syncthreads();
  *out = wbuf;
  return *s_total;
}

// Append the block's c best keys (sorted, at best[0..c)) to the query's candidate list and, when
// the block holds k of them, tighten the query's shared bound.  Block-wide.
__device__ void publish_block_result(const uint64_t* best, int c, int k, uint64_t* cand, uint32_t* cand_cnt,
                                     uint32_t* tau_g, int* s_off) {
  const int tid = threadIdx.x;
  if (tid == 0) {
    *s_off = c ? (int)atomicAdd(cand_cnt, (uint32_t)c) : 0;
    if (c >= k) atomicMin(tau_g, (uint32_t)(best[k - 1] >> 32));
  }
  __syncthreads();
  for (int i = tid; i < c; i += blockDim.x)
    __hip_atomic_store(cand + (uint32_t)*s_off + i, best[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Every block of a query calls this once after publishing.  The block that arrives last (ticket
// counter) selects the query's k best from the candidate list and writes the result.
// wbuf = [nwaves + 1][kWaveCap] keys of LDS, free for use.
__device__ void finish_query(uint64_t* wbuf, int nwaves, int k, const uint64_t* cand, const uint32_t* cand_cnt,
                             uint32_t* done_cnt, unsigned nblocks, int32_t* ids, float* dist, int* s_total,
                             int* s_off, int* s_last) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint64_t* buf = wbuf + (size_t)wave * kWaveCap;
  wait_own_memory_ops();
  __syncthreads();
  if (tid == 0) *s_last = atomicAdd(done_cnt, 1u) == nblocks - 1;
  __syncthreads();
  if (!*s_last) return;
  const int64_t n = __hip_atomic_load(cand_cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  constexpr int kBatch = 8;  // keys per lane in flight: the loads bypass the caches, so overlap them
  // Pass A: every thread takes the smallest distance image of its strided share of the
  // candidates; the k-th smallest of these per-thread minima (k different candidates) bounds
  // the k-th smallest candidate, and about k candidates lie below it.
  uint32_t tau = kOrdMax;
  if (n > kWaveCap) {
    uint32_t mine = kOrdMax;
    for (int64_t i0 = 0; i0 < n; i0 += (int64_t)blockDim.x * kBatch) {
      uint64_t key[kBatch];
#pragma unroll
      for (int r = 0; r < kBatch; ++r) {
        const int64_t i = i0 + (int64_t)r * blockDim.x + tid;
        key[r] = i < n ? __hip_atomic_load(cand + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : kKeyMax;
      }
#pragma unroll
      for (int r = 0; r < kBatch; ++r) {
        uint32_t o = (uint32_t)(key[r] >> 32);
        if (o < mine) mine = o;
      }
    }
    uint32_t* s_min = reinterpret_cast<uint32_t*>(wbuf);  // [blockDim.x]
    s_min[tid] = mine;
    __syncthreads();
    if ((int)blockDim.x >= k) {  // every wave finds the same value: no broadcast needed
      uint32_t v[kScanThreads / 64];
#pragma unroll
      for (int j = 0; j < kScanThreads / 64; ++j) v[j] = s_min[lane + 64 * j];
      uint32_t ans = 0;
      for (int b = 31; b >= 0; --b) {
        const uint32_t trial = ans | (1u << b);
        int c = 0;
#pragma unroll
        for (int j = 0; j < kScanThreads / 64; ++j) c += v[j] < trial;
        for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, 64);
        if (c < k) ans = trial;
      }
      tau = ans;
    }
    __syncthreads();
  }
  // Pass B: keep what is not above the bound (per-wave buffers as in the scan), then merge.
  int cnt = 0;
  for (int64_t i0 = (int64_t)wave * 64 * kBatch; i0 < n; i0 += (int64_t)nwaves * 64 * kBatch) {
    uint64_t key[kBatch];
    uint32_t pend = 0;
#pragma unroll
    for (int r = 0; r < kBatch; ++r) {
      const int64_t i = i0 + r * 64 + lane;
      key[r] = i < n ? __hip_atomic_load(cand + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : kKeyMax;
    }
#pragma unroll
    for (int r = 0; r < kBatch; ++r)
      if (key[r] != kKeyMax && (uint32_t)(key[r] >> 32) <= tau) pend |= 1u << r;
    if (__ballot(pend != 0) != 0ull) wave_offer<kBatch>(buf, cnt, tau, k, key, pend, lane);
  }
  uint64_t* best;
  const int c = block_collect(wbuf, nwaves, cnt, tau, kOrdMax, k, &best, s_total, s_off);
  write_result(best, c, k, ids, dist);
}

template <int MT, int MODE>
__global__ __launch_bounds__(kScanThreads) void k_scan_w(ScanArgs a) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int M = MT ? MT : a.M;
  float* A = reinterpret_cast<float*>(smem);
  uint64_t* wbuf = reinterpret_cast<uint64_t*>(smem + table_bytes(M));  // [waves + 1][kWaveCap]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nwaves = blockDim.x >> 6;
  BlockVars* bv = reinterpret_cast<BlockVars*>(wbuf + (size_t)(nwaves + 1) * kWaveCap);
  int& s_total = bv->total;
  int& s_off = bv->off;
  int& s_last = bv->last;
  uint32_t& s_tg = bv->tg;
  const int64_t q = blockIdx.y;
  uint64_t* cand = a.partial + q * a.cand_cap;
  if (a.qmode && a.qmode[q] != a.want_mode) return;

  int64_t nrows;
  const int32_t* tids = nullptr;
  if (MODE == kLinear) {
    nrows = a.N;
  } else {
    int64_t o0 = a.target_offsets[q];
    nrows = a.target_offsets[q + 1] - o0;
    tids = a.target_ids + o0;
  }
  uint64_t* buf = wbuf + (size_t)wave * kWaveCap;
  const int k = a.k;
  const float* lut = a.lut + q * M * 256;

  if constexpr (rot_m(MT)) {
    // Rotated stored form.  Every block has its share of the rows (a.chunk_rows of them), cut
    // into units of kUnitTiles wave-tiles (a wave-tile = 64 lanes x kRowsPerLane consecutive
    // 64-row slices); the block's waves take the units one after the other from a counter in
    // LDS, so each wave streams runs of kUnitTiles * 256 consecutive rows, no wave waits for
    // another inside the loop, and the waves of a block finish together.
    // (Handing units out across blocks through counters in global memory, so that fast blocks
    // take work from slow ones, was measured slower: the wait for a counter's value drains the
    // wave's load pipeline.)
    if (nrows > 0) {  // block-uniform
      // The query's shared bound is re-read once per tile by the block's first wave only and
      // passed on through LDS (a plain word, read without synchronisation: a stale value is
      // still a valid bound); thousands of waves polling one address would serialise on it.
      // Its first value is in place before the barriers of the table fill, hence before any
      // wave can read it.
      uint32_t tg = __hip_atomic_load(a.tau_g + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (tid == 0) {
        __hip_atomic_store(&s_tg, tg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        bv->cnt = nwaves;  // units of the share handed out so far (the first one per wave is fixed)
      }
      fill_table_rot<MT>(A, reinterpret_cast<float*>(wbuf), lut);  // the wave buffers are not in use yet
      constexpr int64_t kWaveTile = 64 * kRowsPerLane;
      constexpr int64_t kUnitRows = kUnitTiles * kWaveTile;
      // this block's share (a.chunk_rows is a multiple of the unit; the last share may be short or empty)
      const int64_t share_lo = (int64_t)blockIdx.x * a.chunk_rows;
      const int64_t share_n = share_lo >= nrows ? 0 : (nrows - share_lo < a.chunk_rows ? nrows - share_lo : a.chunk_rows);
      const uint32_t share_units = (uint32_t)((share_n + kUnitRows - 1) / kUnitRows);
      // First row of the next unit for this wave, -1 when the share is used up (wave-uniform).
      // A wave starts with unit number `wave`; further units come from a counter in LDS, so a
      // wave that runs slower than its neighbours simply takes fewer of them (an LDS atomic
      // returns through the LDS queue and leaves the wave's global loads in flight).
      bool first_unit = true;
      auto next_unit = [&]() -> int64_t {
        uint32_t u;
        if (first_unit) {
          first_unit = false;
          u = (uint32_t)wave;
        } else {
          u = lane == 0 ? (uint32_t)atomicAdd(&bv->cnt, 1) : 0u;
          u = (uint32_t)__builtin_amdgcn_readfirstlane((int)u);
        }
        if (u >= share_units) return -1;
        return share_lo + (int64_t)u * kUnitRows;
      };
      int64_t unit_base = next_unit();
      int t_in = 0;
      // first row of the next wave-tile of this wave, -1 when the rows are used up
      auto next_tile = [&]() -> int64_t {
        if (unit_base < 0) return -1;
        const int64_t base = unit_base + (int64_t)t_in * kWaveTile;
        if (++t_in == kUnitTiles) {
          t_in = 0;
          unit_base = next_unit();
        }
        return base < nrows ? base : -1;
      };
      // row (linear) or target (subset) number of slice r of the tile at `base`, clamped to
      // the last one (valid memory; such rows are masked when scored), and its identifier
      auto id_at = [&](int64_t base, int r) -> int32_t {
        int64_t i = base < 0 ? nrows - 1 : base + r * 64 + lane;
        if (i >= nrows) i = nrows - 1;
        return MODE == kLinear ? (int32_t)i : tids[i];
      };
      int cnt = 0;
      uint32_t tau = kOrdMax;
      // Software pipeline over the wave's tiles: the code words of the next tile are requested
      // while the current one is scored.  Per slice, all LDS addresses are formed first; the
      // slice's words are dead from then on and their registers receive the next tile's slice
      // before the look-ups start.  The identifiers of a target list run one more tile ahead.
      int64_t b0 = next_tile(), b1 = next_tile(), b2 = next_tile();
      int32_t rid[kRowsPerLane], rid_n[kRowsPerLane];
      uint32_t w[kRowsPerLane][MT / 4];
#pragma unroll
      for (int r = 0; r < kRowsPerLane; ++r) rid[r] = id_at(b0, r);
#pragma unroll
      for (int r = 0; r < kRowsPerLane; ++r) load_row_words<MT>(a.codes + (int64_t)rid[r] * M, w[r]);
#pragma unroll
      for (int r = 0; r < kRowsPerLane; ++r) rid_n[r] = id_at(b1, r);
      if (a.seed_inside) {  // block-uniform (a launch parameter)
        // Bound seeding without a kernel of its own (used when all blocks of the launch are
        // resident at once and a query has at least k of them).  Every block scores the first
        // tile of each of its waves and records the smallest distance among those rows; the
        // k-th smallest of the blocks' minima belongs to k different rows, so it bounds the k-th
        // smallest distance of the whole scan from above.  The block that arrives last selects
        // it and stores it in tau_g; the others wait for tau_g to change -- for at most
        // kSeedWaitTicks of the 100 MHz clock, after which they go on without a bound (the
        // bound only saves work, results do not depend on it).
        uint32_t best = kOrdMax;
        if (b0 >= 0) {
#pragma unroll
          for (int r = 0; r < kRowsPerLane; ++r) {
            uint32_t addr[MT];
            rot_addrs<MT>(w[r], ((uint32_t)rid[r] & 31u) << 2, addr);
            float d = rot_sum<MT>(addr);
            d = __fadd_rn(d, __fmul_rn(d, rot_eps(MT)));  // not below the row's ascending-m sum
            const uint32_t o = ord_of(d);
            if (b0 + r * 64 + lane < nrows && o < best) best = o;
          }
        }
        for (int o = 32; o > 0; o >>= 1) {
          const uint32_t other = __shfl_xor(best, o, 64);
          if (other < best) best = other;
        }
        uint32_t* s_min = reinterpret_cast<uint32_t*>(bv->red);  // [waves]
        if (lane == 0) s_min[wave] = best;
        __syncthreads();
        if (tid == 0) {
          for (int i = 1; i < nwaves; ++i) best = s_min[i] < best ? s_min[i] : best;
          __hip_atomic_store(a.minima + q * gridDim.x + blockIdx.x, best, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          wait_own_memory_ops();
          s_last = atomicAdd(a.counter + q, 1u) == gridDim.x - 1;
        }
        __syncthreads();
        if (s_last && wave == 0) {
          // k-th smallest of the gridDim.x <= 256 minima, most significant bit first
          uint32_t v[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int i = lane + 64 * j;
            v[j] = i < (int)gridDim.x
                       ? __hip_atomic_load(a.minima + q * gridDim.x + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                       : kOrdMax;
          }
          uint32_t ans = 0;
          for (int b = 31; b >= 0; --b) {
            const uint32_t trial = ans | (1u << b);
            int c = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) c += v[j] < trial;
            for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, 64);
            if (c < k) ans = trial;
          }
          // (fewer than k rows in all first tiles: the image of +infinity still says "seeded"
          // and lets every row through)
          if (lane == 0) atomicMin(a.tau_g + q, ans < kOrdInf ? ans : kOrdInf);
        }
        if (tid == 0) {
          // tau_g leaves kOrdMax exactly once before any wave enters its loop: by that atomicMin
          const long long t0 = wall_clock64();
          uint32_t seen;
          while ((seen = __hip_atomic_load(a.tau_g + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) == kOrdMax &&
                 wall_clock64() - t0 < kSeedWaitTicks)
            __builtin_amdgcn_s_sleep(4);
          __hip_atomic_store(&s_tg, seen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        __syncthreads();
        tg = __hip_atomic_load(&s_tg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
      while (b0 >= 0) {  // wave-uniform
        uint64_t key[kRowsPerLane];
        uint32_t pend = 0;
        uint32_t fresh = kOrdMax;
        if (wave == 0) fresh = __hip_atomic_load(a.tau_g + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t bound = tg < tau ? tg : tau;
        // filter on the conflict-free rotated-order sum; exact ascending-m sum for the few rows that pass
        const float fb = rot_filter(bound, rot_eps(MT));
        int32_t rid_nn[kRowsPerLane];
        uint32_t live = 0, maybe = 0;
#pragma unroll
        for (int r = 0; r < kRowsPerLane; ++r) {
          key[r] = kKeyMax;
          if (b0 + r * 64 + lane < nrows) live |= 1u << r;
          rid_nn[r] = id_at(b2, r);
        }
#pragma unroll
        for (int r = 0; r < kRowsPerLane; ++r) {
          uint32_t addr[MT];
          rot_addrs<MT>(w[r], ((uint32_t)rid[r] & 31u) << 2, addr);
          load_row_words<MT>(a.codes + (int64_t)rid_n[r] * M, w[r]);
          if (rot_sum_abandon<MT>(addr, fb) <= fb) maybe |= 1u << r;
        }
        maybe &= live;
        if (__ballot(maybe != 0) != 0ull) {
#pragma unroll
          for (int r = 0; r < kRowsPerLane; ++r) {
            if (maybe & (1u << r)) {
              float d = adc_row_exact_rot<MT>(A, a.codes + (int64_t)rid[r] * M, rid[r]);
              key[r] = make_key(d, rid[r]);
              if ((uint32_t)(key[r] >> 32) <= bound) pend |= 1u << r;
            }
          }
        }
        if (__ballot(pend != 0) != 0ull) {
          const uint32_t before = tau;
          wave_offer<kRowsPerLane>(buf, cnt, tau, k, key, pend, lane);
          if (tau < before && lane == 0) atomicMin(a.tau_g + q, tau);
        }
        if (tid == 0) __hip_atomic_store(&s_tg, fresh, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        tg = __hip_atomic_load(&s_tg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        b0 = b1; b1 = b2; b2 = next_tile();
#pragma unroll
        for (int r = 0; r < kRowsPerLane; ++r) {
          rid[r] = rid_n[r];
          rid_n[r] = rid_nn[r];
        }
      }
      tg = __hip_atomic_load(a.tau_g + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      // the block's own k best go to the query's candidate list
      const uint32_t bound = tg < tau ? tg : tau;
      uint64_t* best;
      const int c = block_collect(wbuf, nwaves, cnt, tau, bound, k, &best, &s_total, &s_off);
      publish_block_result(best, c, k, cand, a.cand_cnt + q, a.tau_g + q, &s_off);
    }
  } else {
    // Plain stored form (other M): every block takes a fixed share of the rows.
    const int64_t tile_step = (int64_t)blockDim.x * kRowsPerLane;
    const int64_t r0 = (int64_t)blockIdx.x * a.chunk_rows;
    const int64_t r1 = r0 + a.chunk_rows < nrows ? r0 + a.chunk_rows : nrows;
    if (r0 < r1) {  // block-uniform
      uint32_t tg = __hip_atomic_load(a.tau_g + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (tid == 0) __hip_atomic_store(&s_tg, tg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      for (int i = tid; i < M * 256; i += blockDim.x) A[i] = lut[i];
      __syncthreads();  // also orders the first value of s_tg before any wave reads it
      int cnt = 0;
      uint32_t tau = kOrdMax;
      for (int64_t tile = r0; tile < r1; tile += tile_step) {
        uint64_t key[kRowsPerLane];
        uint32_t pend = 0;
        uint32_t fresh = kOrdMax;
        if (wave == 0) fresh = __hip_atomic_load(a.tau_g + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t bound = tg < tau ? tg : tau;
#pragma unroll
        for (int r = 0; r < kRowsPerLane; ++r) {
          // a wave owns 64 consecutive rows of each of the tile's kRowsPerLane slices
          int64_t i = tile + (int64_t)r * blockDim.x + tid;
          key[r] = kKeyMax;
          if (i < r1) {
            int32_t id = MODE == kLinear ? (int32_t)i : tids[i];
            float d = adc_row<MT>(A, a.codes + (int64_t)id * M, M);
            key[r] = make_key(d, id);
            if ((uint32_t)(key[r] >> 32) <= bound) pend |= 1u << r;
          }
        }
        if (__ballot(pend != 0) != 0ull) {
          const uint32_t before = tau;
          wave_offer<kRowsPerLane>(buf, cnt, tau, k, key, pend, lane);
          if (tau < before && lane == 0) atomicMin(a.tau_g + q, tau);
        }
        if (tid == 0) __hip_atomic_store(&s_tg, fresh, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        tg = __hip_atomic_load(&s_tg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
      tg = __hip_atomic_load(a.tau_g + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const uint32_t bound = tg < tau ? tg : tau;
      uint64_t* best;
      const int c = block_collect(wbuf, nwaves, cnt, tau, bound, k, &best, &s_total, &s_off);
      publish_block_result(best, c, k, cand, a.cand_cnt + q, a.tau_g + q, &s_off);
    }
  }
  finish_query(wbuf, nwaves, k, cand, a.cand_cnt + q, a.done_cnt + q, gridDim.x, a.ids + q * a.out_stride,
               a.dist ? a.dist + q * a.out_stride : nullptr, &s_total, &s_off, &s_last);
}

// ------------------------------------------------------------------ two queries per pass
// Whole-database scan for large batches (every block owns its queries' whole scan), M = 8, 16, 32,
// topk <= kWaveK.  A block serves TWO queries: the table holds float2 entries (one float per
// query), T2[z][s] for 32 slots s, slot s holding (A0[s % M][z], A1[s % M][z]), so one 8-byte
// LDS read yields the look-ups of both queries for the same code byte, and the code loads and the
// address arithmetic are shared.  Rows are in the rotated stored form; lane l reads slot
// (l + t) % 32 at step t (the per-step slot offsets sit in registers), which keeps the 32 lanes of
// a half-wave on different slots.  As in k_scan_w the rotated-order sums are a filter and rows
// that pass are re-scored in ascending sub-space order.  Each wave keeps one candidate buffer
// per query; the block's merge result is the query's result (no cross-block stage).
template <int MT>
__device__ __forceinline__ float adc_row_exact_rot2(const float2* T2, const uint8_t* __restrict__ row, int64_t r,
                                                    int which) {
  float d = 0.f;
#pragma unroll 4
  for (int m = 0; m < MT; ++m) {
    float2 v = T2[(int)row[(m - (int)r) & (MT - 1)] * 32 + m];
    d = __fadd_rn(d, which ? v.y : v.x);
  }
  return d;
}

template <int MT>
__global__ __launch_bounds__(kScanThreads) void k_scan_w2(ScanArgs a) {
  static_assert(rot_m(MT), "rotated stored form only");
  extern __shared__ __align__(16) uint8_t smem[];
  float2* T2 = reinterpret_cast<float2*>(smem);                        // [256][32]
  uint64_t* wbuf0 = reinterpret_cast<uint64_t*>(smem + 65536);        // query 0: [waves + 1][kWaveCap]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nwaves = blockDim.x >> 6;
  uint64_t* wbuf1 = wbuf0 + (size_t)(nwaves + 1) * kWaveCap;          // query 1
  BlockVars* bv = reinterpret_cast<BlockVars*>(wbuf1 + (size_t)(nwaves + 1) * kWaveCap);
  int& s_total = bv->total;
  int& s_off = bv->off;
  const int64_t q0 = 2 * (int64_t)blockIdx.y, q1 = q0 + 1;
  const int k = a.k;
  const int64_t nrows = a.N;

  {  // stage both tables ([M][256] each) in the buffer area, then transpose along diagonals
    float* st0 = reinterpret_cast<float*>(wbuf0);
    float* st1 = st0 + MT * 256;
    const float* l0 = a.lut + q0 * MT * 256;
    const float* l1 = a.lut + q1 * MT * 256;
    for (int i = tid; i < MT * 256; i += blockDim.x) {
      st0[i] = l0[i];
      st1[i] = l1[i];
    }
    __syncthreads();
    for (int it = tid; it < 256 * 32; it += blockDim.x) {
      const int l = it & 31, blk = it >> 5;
      const int s0 = blk & 31, z0 = (blk >> 5) << 5;
      const int z = z0 + l, s = (s0 + l) & 31;
      const int src = (s & (MT - 1)) * 256 + z;
      T2[z * 32 + s] = make_float2(st0[src], st1[src]);
    }
    __syncthreads();
  }
  // Slot offset of step t for this lane, ((tid + t) % 32) * 8 (rows are dealt so that row % 32 ==
  // tid % 32): one byte each, four steps to a register; the byte permute that builds an LDS
  // address takes its low byte from here and its second byte from the code word.
  uint32_t lb4[MT / 4];
#pragma unroll
  for (int j = 0; j < MT / 4; ++j) {
    lb4[j] = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) lb4[j] |= ((uint32_t)((tid + 4 * j + b) & 31) * 8u) << (8 * b);
  }

  uint64_t* buf0 = wbuf0 + (size_t)wave * kWaveCap;
  uint64_t* buf1 = wbuf1 + (size_t)wave * kWaveCap;
  int cnt0 = 0, cnt1 = 0;
  uint32_t tau0 = kOrdMax, tau1 = kOrdMax;
  const int64_t tile_step = (int64_t)blockDim.x * kRowsPerLane;
  // row of slot r in the tile at `tile`; past the end: the last row (valid memory, masked later)
  auto row_at = [&](int64_t tile, int r) -> int64_t {
    int64_t i = tile + (int64_t)r * blockDim.x + tid;
    return i < nrows ? i : nrows - 1;
  };
  uint32_t w[kRowsPerLane][MT / 4];
#pragma unroll
  for (int r = 0; r < kRowsPerLane; ++r) load_row_words<MT>(a.codes + row_at(0, r) * MT, w[r]);
  for (int64_t tile = 0; tile < nrows; tile += tile_step) {
    const float fb0 = rot_filter(tau0, rot_eps(MT)), fb1 = rot_filter(tau1, rot_eps(MT));
    uint32_t maybe0 = 0, maybe1 = 0;
    // software pipeline as in k_scan_w, in segments of 16 code bytes: a segment's LDS addresses
    // first, then the request for the same segment of the next tile's row into the registers
    // just freed, then the look-ups
    uint32_t live = 0;
#pragma unroll
    for (int r = 0; r < kRowsPerLane; ++r) {
      if (tile + (int64_t)r * blockDim.x + tid < nrows) live |= 1u << r;
      const uint8_t* next_row = a.codes + row_at(tile + tile_step, r) * MT;
      float d0 = 0.f, d1 = 0.f;
#pragma unroll
      for (int sg = 0; sg < MT / kRotSeg<MT>; ++sg) {
        uint32_t addr[kRotSeg<MT>];
#pragma unroll
        for (int u = 0; u < kRotSeg<MT>; ++u) {
          const int t = sg * kRotSeg<MT> + u;
          addr[u] = __builtin_amdgcn_perm(w[r][t >> 2], lb4[t >> 2], 0x0c0c0400u | ((uint32_t)(t & 3) * 0x0101u));
        }
        load_row_segment<MT>(next_row, sg, w[r]);
#pragma unroll
        for (int u = 0; u < kRotSeg<MT>; ++u) {
          float2 v = lds_read_f32x2(addr[u]);  // T2 is at LDS address 0
          d0 = __fadd_rn(d0, v.x);
          d1 = __fadd_rn(d1, v.y);
        }
      }
      if (d0 <= fb0) maybe0 |= 1u << r;
      if (d1 <= fb1) maybe1 |= 1u << r;
    }
    maybe0 &= live;
    maybe1 &= live;
    if (__ballot((maybe0 | maybe1) != 0) != 0ull) {
      uint64_t key[kRowsPerLane];
      uint32_t pend = 0;
#pragma unroll
      for (int r = 0; r < kRowsPerLane; ++r) {
        key[r] = kKeyMax;
        if (maybe0 & (1u << r)) {
          const int64_t i = tile + (int64_t)r * blockDim.x + tid;
          key[r] = make_key(adc_row_exact_rot2<MT>(T2, a.codes + i * MT, i, 0), (int32_t)i);
          if ((uint32_t)(key[r] >> 32) <= tau0) pend |= 1u << r;
        }
      }
      if (__ballot(pend != 0) != 0ull) wave_offer<kRowsPerLane>(buf0, cnt0, tau0, k, key, pend, lane);
      pend = 0;
#pragma unroll
      for (int r = 0; r < kRowsPerLane; ++r) {
        key[r] = kKeyMax;
        if (maybe1 & (1u << r)) {
          const int64_t i = tile + (int64_t)r * blockDim.x + tid;
          key[r] = make_key(adc_row_exact_rot2<MT>(T2, a.codes + i * MT, i, 1), (int32_t)i);
          if ((uint32_t)(key[r] >> 32) <= tau1) pend |= 1u << r;
        }
      }
      if (__ballot(pend != 0) != 0ull) wave_offer<kRowsPerLane>(buf1, cnt1, tau1, k, key, pend, lane);
    }
  }
  uint64_t* best;
  int c = block_collect(wbuf0, nwaves, cnt0, tau0, tau0, k, &best, &s_total, &s_off);
  write_result(best, c, k, a.ids + q0 * a.out_stride, a.dist ? a.dist + q0 * a.out_stride : nullptr);
  __syncthreads();
  c = block_collect(wbuf1, nwaves, cnt1, tau1, tau1, k, &best, &s_total, &s_off);
  write_result(best, c, k, a.ids + q1 * a.out_stride, a.dist ? a.dist + q1 * a.out_stride : nullptr);
}

// ------------------------------------------------------------------ four queries per pass
// Same setting as k_scan_w2 (whole-database scan, M = 8, 16, 32), four queries per block, with the
// table quantised to 15-bit integers: T4[z][s] for 32 slots, each entry four 16-bit fields (one
// per query) in one 64-bit word, so one 8-byte LDS read serves four look-ups and ONE 64-bit
// integer addition (v_lshl_add_u64, full rate) accumulates all four sums -- per code byte one
// byte permute, one LDS read, one add.  The integer sum is only a FILTER:
//   e(a) = min(cap, floor(a * scale)),  cap = 32767 / M,  scale = cap / (largest entry) (rounded
//   down), so a field never exceeds 32767 and never carries into its neighbour;
//   sum_m e(a_m) <= scale * (1 + 2^-24) * (real sum) <= scale * tau * (1 + (M + 2) 2^-24) for a
//   row whose fp32 ascending-order distance is <= tau, so with
//   fbq = floor(tau * scale * (1 + 1e-5)) + 1 (at most 32767) every such row has sum <= fbq.
//   The test for the four queries is one 64-bit subtraction: with C holding 0x8000 + fbq_j in
//   field j, C - sum has bit 15 of field j set exactly when sum_j <= fbq_j (every field of the
//   difference stays >= 1, so no borrow crosses fields).
// The filter lets through rows up to (M + 1) / scale above the bound (about 3 % of the largest
// table entry at M = 32).  Rows that pass are re-scored from the fp32 table in global memory, in
// ascending sub-space order; results are therefore exactly those of the fp32 kernels.  Each wave
// keeps one candidate buffer of kWaveCap4 keys per query.
// When the batch alone does not give the chip several rounds of blocks, the code array is cut
// into row chunks (grid.y, see plan_batch) and the chunks' results meet in the per-query
// candidate lists as in k_scan_w; k_tau0 seeds the bounds first.
constexpr int kWaveCap4 = 128;
constexpr int kWaveK4 = 100;  // largest topk this kernel takes (must stay below kWaveCap4)
constexpr int kRescoreCap = 128;  // per-wave queue of rows awaiting their exact score
constexpr int kBatchWantBlocks = 1024;  // blocks wanted from a batched launch (four rounds of the chip)
constexpr int kBatchMinTiles = 64;      // never cut the rows into chunks shorter than this many tiles

// ascending-m fp32 sum for stored row r (rotated form), table A = lut[M][256] in global memory
template <int MT>
__device__ __forceinline__ float adc_row_unrot_global(const float* __restrict__ A, const uint8_t* __restrict__ row,
                                                      int64_t r) {
  float d = 0.f;
#pragma unroll 4
  for (int m = 0; m < MT; ++m) d = __fadd_rn(d, A[m * 256 + row[(m - (int)r) & (MT - 1)]]);
  return d;
}

template <int MT>
__global__ __launch_bounds__(kScanThreads) void k_scan_w4(ScanArgs a) {
  static_assert(rot_m(MT), "rotated stored form only");
  extern __shared__ __align__(16) uint8_t smem[];
  // smem[0 .. 65536): T4 [256][32] x 4 halves, at LDS address 0
  uint64_t* wbuf = reinterpret_cast<uint64_t*>(smem + 65536);          // [4][waves + 1][kWaveCap4]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nwaves = blockDim.x >> 6;
  const size_t qstride = (size_t)(nwaves + 1) * kWaveCap4;
  uint64_t* rq = wbuf + 4 * qstride + (size_t)wave * kRescoreCap;      // [waves][kRescoreCap] (query, row)
  BlockVars* bv = reinterpret_cast<BlockVars*>(wbuf + 4 * qstride + (size_t)nwaves * kRescoreCap);
  float* s_red = bv->red;
  float* s_scale = bv->scale;
  int& s_total = bv->total;
  int& s_off = bv->off;
  // grid = (query groups, row chunks), query group fastest: the blocks resident at one time
  // work on the same chunk of the code array, which the memory-side cache can then serve
  const int64_t q0 = 4 * (int64_t)blockIdx.x;
  // a short last group scores its last query again in the unused places and drops the copies
  const int nlive = a.nq - q0 < 4 ? (int)(a.nq - q0) : 4;
  auto qsrc = [&](int j) -> int64_t { return q0 + (j < nlive ? j : nlive - 1); };
  const int k = a.k;
  const int64_t r0 = (int64_t)blockIdx.y * a.chunk_rows;
  const int64_t nrows = r0 + a.chunk_rows < a.N ? r0 + a.chunk_rows : a.N;  // end of this block's rows
  const bool chunked = gridDim.y > 1;

  // tables: one query at a time through a staging copy (the buffer area), quantised and written
  // along diagonals (see fill_table_rot)
  constexpr uint32_t kCap = 32767u / MT;
  if (tid == 0) bv->cnt = nwaves;  // units handed out so far (the first one per wave is fixed); before the barriers below
  {
    float* stage = reinterpret_cast<float*>(wbuf);
    uint16_t* T4q = reinterpret_cast<uint16_t*>(smem);
    for (int j = 0; j < 4; ++j) {
      const float* lut = a.lut + qsrc(j) * MT * 256;
      float mx = 0.f;
      for (int i = tid; i < MT * 256; i += blockDim.x) {
        float v = lut[i];
        stage[i] = v;
        mx = fmaxf(mx, v);
      }
      for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
      if (lane == 0) s_red[wave] = mx;
      __syncthreads();
      if (tid == 0) {
        float m2 = 0.f;
        for (int w = 0; w < nwaves; ++w) m2 = fmaxf(m2, s_red[w]);
        // cap / max, rounded down a little; a table of zeros (or a tiny one) gets scale 0:
        // every entry quantises to 0 and every row goes to the exact re-scoring
        float sc = 0.f;
        if (m2 > 1e-30f) sc = __fmul_rn(__fdiv_rn((float)kCap, m2), 0.999999f);
        if (!(sc < 1e30f)) sc = 0.f;
        s_scale[j] = sc;
      }
      __syncthreads();
      const float sc = s_scale[j];
      for (int it = tid; it < 256 * 32; it += blockDim.x) {
        const int l = it & 31, blk = it >> 5;
        const int s0 = blk & 31, z0 = (blk >> 5) << 5;
        const int z = z0 + l, s = (s0 + l) & 31;
        uint32_t e = (uint32_t)floorf(__fmul_rn(stage[(s & (MT - 1)) * 256 + z], sc));
        T4q[(size_t)(z * 32 + s) * 4 + j] = (uint16_t)(e < kCap ? e : kCap);
      }
      __syncthreads();
    }
  }
  // Slot offset of step t for this lane, ((tid + t) % 32) * 8 (rows are dealt so that row % 32 ==
  // tid % 32): one byte each, four steps to a register; the byte permute that builds an LDS
  // address takes its low byte from here and its second byte from the code word.
  uint32_t lb4[MT / 4];
#pragma unroll
  for (int j = 0; j < MT / 4; ++j) {
    lb4[j] = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) lb4[j] |= ((uint32_t)((tid + 4 * j + b) & 31) * 8u) << (8 * b);
  }
  const float scale0 = s_scale[0], scale1 = s_scale[1], scale2 = s_scale[2], scale3 = s_scale[3];

  int cnt[4] = {0, 0, 0, 0};
  uint32_t tau[4] = {kOrdMax, kOrdMax, kOrdMax, kOrdMax};
  // With several chunks per query, the blocks of earlier chunks have left the query's bound in
  // tau_g; it is read once here (the waves' own bounds take over from there).
  uint32_t tg[4] = {kOrdMax, kOrdMax, kOrdMax, kOrdMax};
  if (chunked) {
#pragma unroll
    for (int j = 0; j < 4; ++j) tg[j] = __hip_atomic_load(a.tau_g + qsrc(j), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  int qn = 0;  // entries in this wave's re-score queue (wave-uniform)
  // Exact ascending-m scores for queue entries [first, first + n), n <= 64, one per lane, from
  // the fp32 tables in global memory; each goes to its query's candidate buffer.
  auto rescore = [&](int first, int n) {
    wave_sync();  // the queue was written by other lanes
    uint64_t key[1] = {kKeyMax};
    int jq = -1;
    if (lane < n) {
      const uint64_t e = rq[first + lane];
      jq = (int)(e >> 32);
      const int64_t i = (int64_t)(uint32_t)e;
      key[0] = make_key(adc_row_unrot_global<MT>(a.lut + qsrc(jq) * MT * 256, a.codes + i * MT, i), (int32_t)i);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t bound = tau[j] < tg[j] ? tau[j] : tg[j];
      const uint32_t pend = (jq == j && (uint32_t)(key[0] >> 32) <= bound) ? 1u : 0u;
      if (__ballot(pend != 0) != 0ull)
        wave_offer<1>(wbuf + j * qstride + (size_t)wave * kWaveCap4, cnt[j], tau[j], k, key, pend, lane, kWaveCap4);
    }
  };
  // The block's rows [r0, nrows) in units of kUnitTiles wave-tiles (a wave-tile = kRowsPerLane
  // slices of 64 consecutive rows), taken by the waves from a counter in LDS as in k_scan_w, so
  // that the waves of a block finish together.  Units and slices start at multiples of 64, so
  // lane l always scores rows with row % 32 == l % 32 (what lb4 assumes).
  constexpr int64_t kWaveTile = 64 * kRowsPerLane;
  constexpr int64_t kUnitRows = kUnitTiles * kWaveTile;
  const uint32_t share_units = (uint32_t)((nrows - r0 + kUnitRows - 1) / kUnitRows);
  bool first_unit = true;
  auto next_unit = [&]() -> int64_t {
    uint32_t u;
    if (first_unit) {
      first_unit = false;
      u = (uint32_t)wave;
    } else {
      u = lane == 0 ? (uint32_t)atomicAdd(&bv->cnt, 1) : 0u;
      u = (uint32_t)__builtin_amdgcn_readfirstlane((int)u);
    }
    return u < share_units ? r0 + (int64_t)u * kUnitRows : -1;
  };
  int64_t unit_base = next_unit();
  int t_in = 0;
  // first row of the wave's next tile, -1 when the rows are used up
  auto next_tile = [&]() -> int64_t {
    if (unit_base < 0) return -1;
    const int64_t base = unit_base + (int64_t)t_in * kWaveTile;
    if (++t_in == kUnitTiles) {
      t_in = 0;
      unit_base = next_unit();
    }
    return base < nrows ? base : -1;
  };
  // row of slice r of the tile at `base`; past the end (or no tile): the last row (valid memory, masked later)
  auto row_at = [&](int64_t base, int r) -> int64_t {
    const int64_t i = base < 0 ? nrows - 1 : base + r * 64 + lane;
    return i < nrows ? i : nrows - 1;
  };
  int64_t tile = next_tile(), tile_next = next_tile();
  uint32_t w[kRowsPerLane][MT / 4];
#pragma unroll
  for (int r = 0; r < kRowsPerLane; ++r) load_row_words<MT>(a.codes + row_at(tile, r) * MT, w[r]);
  for (; tile >= 0; tile = tile_next, tile_next = next_tile()) {  // wave-uniform
    // C: field j = 0x8000 + fbq_j, fbq_j the filter bound of query j in its table's units
    uint64_t C = 0;
    const float scl[4] = {scale0, scale1, scale2, scale3};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t bound = tau[j] < tg[j] ? tau[j] : tg[j];
      uint32_t fbq = 32767u;
      if (bound != kOrdMax) {
        const float x = __fmul_rn(__fmul_rn(float_of_ord(bound), scl[j]), 1.00001f);
        if (x < 32766.f) fbq = (uint32_t)x + 1u;  // x >= 0: distances are sums of squares
      }
      C |= (uint64_t)(0x8000u | fbq) << (16 * j);
    }
    uint32_t maybe[4] = {0, 0, 0, 0};
    // software pipeline as in k_scan_w, in segments of 16 code bytes: a segment's LDS addresses
    // first, then the request for the same segment of the next tile's row into the registers
    // just freed, then the look-ups
    uint32_t live = 0;
    uint32_t plo[kRowsPerLane], phi[kRowsPerLane];
#pragma unroll
    for (int r = 0; r < kRowsPerLane; ++r) {
      if (tile + r * 64 + lane < nrows) live |= 1u << r;
      const uint8_t* next_row = a.codes + row_at(tile_next, r) * MT;
      uint64_t acc = 0;
#pragma unroll
      for (int sg = 0; sg < MT / kRotSeg<MT>; ++sg) {
        uint32_t addr[kRotSeg<MT>];
#pragma unroll
        for (int u = 0; u < kRotSeg<MT>; ++u) {
          const int t = sg * kRotSeg<MT> + u;
          addr[u] = __builtin_amdgcn_perm(w[r][t >> 2], lb4[t >> 2], 0x0c0c0400u | ((uint32_t)(t & 3) * 0x0101u));
        }
        load_row_segment<MT>(next_row, sg, w[r]);
#pragma unroll
        for (int u = 0; u < kRotSeg<MT>; ++u) {
          const uint2 v = lds_read_u32x2(addr[u]);  // T4 is at LDS address 0
          acc += ((uint64_t)v.y << 32) | v.x;       // four 16-bit sums at once
        }
      }
      const uint64_t pass = (C - acc) & 0x8000800080008000ull;
      plo[r] = (uint32_t)pass;
      phi[r] = (uint32_t)(pass >> 32);
    }
    uint32_t any = 0;
#pragma unroll
    for (int r = 0; r < kRowsPerLane; ++r) any |= (live >> r) & 1u ? (plo[r] | phi[r]) : 0u;
    if (__ballot(any != 0) != 0ull) {  // rare: unpack the pass bits per query
#pragma unroll
      for (int r = 0; r < kRowsPerLane; ++r) {
        if (!((live >> r) & 1u)) continue;
        if (plo[r] & 0x00008000u) maybe[0] |= 1u << r;
        if (plo[r] & 0x80000000u) maybe[1] |= 1u << r;
        if (phi[r] & 0x00008000u) maybe[2] |= 1u << r;
        if (phi[r] & 0x80000000u) maybe[3] |= 1u << r;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) maybe[j] = j < nlive ? maybe[j] : 0u;
    }
    // Rows that pass a filter are not re-scored on the spot (one or two lanes busy, the wave
    // waiting on their table reads from global memory) but queued as (query, row); a full
    // wavefront of 64 queued entries is then re-scored at once, one entry per lane.
    if (__ballot((maybe[0] | maybe[1] | maybe[2] | maybe[3]) != 0) != 0ull) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (__ballot(maybe[j] != 0) == 0ull) continue;  // wave-uniform
#pragma unroll
        for (int r = 0; r < kRowsPerLane; ++r) {
          const bool hit = (maybe[j] >> r) & 1u;
          const unsigned long long m = __ballot(hit);
          if (m == 0ull) continue;
          if (hit) {
            const int64_t i = tile + r * 64 + lane;
            rq[qn + __popcll(m & ((1ull << lane) - 1ull))] = ((uint64_t)j << 32) | (uint32_t)i;
          }
          qn += __popcll(m);
          if (qn >= 64) {  // at most 127 entries are ever queued: kRescoreCap holds them
            qn -= 64;
            rescore(qn, 64);
          }
        }
      }
    }
  }
  if (qn > 0) rescore(0, qn);
  if (!chunked) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (j >= nlive) break;  // block-uniform
      uint64_t* best;
      int c = block_collect(wbuf + j * qstride, nwaves, cnt[j], tau[j], tau[j], k, &best, &s_total, &s_off, kWaveCap4);
      write_result(best, c, k, a.ids + (q0 + j) * a.out_stride, a.dist ? a.dist + (q0 + j) * a.out_stride : nullptr);
      __syncthreads();
    }
    return;
  }
  // Several chunks per query: the block's best keys go to each query's candidate list (all four
  // first: the final selection re-uses the whole buffer area), then the block that arrives last
  // for a query selects its result.
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (j >= nlive) break;  // block-uniform
    const uint32_t bound = tau[j] < tg[j] ? tau[j] : tg[j];
    uint64_t* best;
    int c = block_collect(wbuf + j * qstride, nwaves, cnt[j], tau[j], bound, k, &best, &s_total, &s_off, kWaveCap4);
    publish_block_result(best, c, k, a.partial + (q0 + j) * a.cand_cap, a.cand_cnt + q0 + j, a.tau_g + q0 + j, &s_off);
    __syncthreads();
  }
#pragma unroll 1
  for (int j = 0; j < nlive; ++j) {
    finish_query(wbuf, nwaves, k, a.partial + (q0 + j) * a.cand_cap, a.cand_cnt + q0 + j, a.done_cnt + q0 + j,
                 gridDim.y, a.ids + (q0 + j) * a.out_stride, a.dist ? a.dist + (q0 + j) * a.out_stride : nullptr,
                 &s_total, &s_off, &bv->last);
    __syncthreads();
  }
}

// ------------------------------------------------------------------ PartialSort + Take
struct SelectArgs {
  // source A: keys [Q][nkeys] (per-block partial results)
  const uint64_t* keys;
  int64_t nkeys;               // capacity per query
  const uint32_t* key_cnt;     // [Q] keys actually present (NULL: nkeys)
  // source B: explicit candidates in CSR segments
  const float* cand_dist;
  const int32_t* cand_ids;
  const int64_t* cand_offsets;
  int k;
  int out_stride;      // elements between consecutive queries in ids/dist (>= k)
  int32_t* ids;
  float* dist;
  const int* qmode;
  int want_mode;
};

__device__ __forceinline__ void write_result(const uint64_t* keys, int c, int k, int32_t* ids, float* dist) {
  for (int i = threadIdx.x; i < k; i += blockDim.x) {
    if (i < c && keys[i] != kKeyMax) {
      ids[i] = (int32_t)(uint32_t)keys[i];
      if (dist) dist[i] = float_of_ord((uint32_t)(keys[i] >> 32));
    } else {
      ids[i] = -1;
      if (dist) dist[i] = __uint_as_float(0x7F800000u);
    }
  }
}

// one block per query
__global__ __launch_bounds__(kScanThreads) void k_select(SelectArgs a) {
  __shared__ uint64_t keys[kSelCap];
  __shared__ int s_cnt;
  __shared__ uint32_t s_tau;
  const int tid = threadIdx.x;
  const int64_t q = blockIdx.x;
  if (a.qmode && a.qmode[q] != a.want_mode) return;
  if (tid == 0) {
    s_cnt = 0;
    s_tau = kOrdMax;
  }
  __syncthreads();
  int64_t n, base = 0;
  if (a.keys) {
    n = a.nkeys;
    if (a.key_cnt && a.key_cnt[q] < n) n = a.key_cnt[q];
  } else {
    base = a.cand_offsets[q];
    n = a.cand_offsets[q + 1] - base;
  }
  for (int64_t t0 = 0; t0 < n; t0 += blockDim.x) {
    int64_t i = t0 + tid;
    uint64_t key[1] = {kKeyMax};
    uint32_t pend = 0;
    if (i < n) {
      if (a.keys) key[0] = a.keys[q * a.nkeys + i];
      else key[0] = make_key(a.cand_dist[base + i], a.cand_ids ? a.cand_ids[base + i] : (int32_t)i);
      if (key[0] != kKeyMax && (uint32_t)(key[0] >> 32) <= s_tau) pend = 1;
    }
    sel_offer<1>(keys, &s_cnt, &s_tau, a.k, key, pend);
  }
  __syncthreads();
  sel_compact(keys, &s_cnt, &s_tau, a.k);
  write_result(keys, s_cnt, a.k, a.ids + q * a.out_stride, a.dist ? a.dist + q * a.out_stride : nullptr);
}

// Full sort of short segments (<= RII_MAX_SORT candidates) in LDS; one block per query.
__global__ __launch_bounds__(kScanThreads) void k_sort_segments(SelectArgs a) {
  extern __shared__ __align__(16) uint8_t smem[];
  uint64_t* keys = reinterpret_cast<uint64_t*>(smem);
  const int64_t q = blockIdx.x;
  if (a.qmode && a.qmode[q] != a.want_mode) return;
  const int64_t base = a.cand_offsets[q];
  int n = (int)(a.cand_offsets[q + 1] - base);
  if (n > RII_MAX_SORT) n = RII_MAX_SORT;  // guarded by the host; never read past the LDS array
  const int n2 = next_pow2(n);
  for (int i = threadIdx.x; i < n2; i += blockDim.x)
    keys[i] = i < n ? make_key(a.cand_dist[base + i], a.cand_ids ? a.cand_ids[base + i] : i) : kKeyMax;
  __syncthreads();
  block_bitonic_sort(keys, n2);
  write_result(keys, n, a.k, a.ids + q * a.out_stride, a.dist ? a.dist + q * a.out_stride : nullptr);
}

// ------------------------------------------------------------------ plain ADC distances
// dist[q][i] = ADC of row i for i < nrows; grid (ceil(nrows / block), Q).
template <int MT>
__global__ void k_adc_all(const uint8_t* __restrict__ codes, int64_t nrows, int Mrt, const float* __restrict__ lut,
                          float* __restrict__ dist, const int* qmode, int want_mode) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int M = MT ? MT : Mrt;
  float* A = reinterpret_cast<float*>(smem);
  const int64_t q = blockIdx.y;
  if (qmode && qmode[q] != want_mode) return;
  for (int i = threadIdx.x; i < M * 256; i += blockDim.x) A[i] = lut[q * M * 256 + i];
  __syncthreads();
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < nrows) dist[q * nrows + i] = adc_row<MT>(A, codes + i * M, M);
}

// ------------------------------------------------------------------ inverted index (Alg. 2, second block)
struct IvfArgs {
  const uint8_t* codes_list;     // [N][M] in list order
  const int32_t* list_ids;       // [N]
  const int64_t* list_off;       // [K+1]
  int M;
  const float* lut;
  const int32_t* probe;          // [Q][probe_stride]
  int probe_stride;
  int nprobe;                    // uniform number of lists ...
  const int* nprobe_q;           // ... or per query when not NULL
  const int32_t* target_ids;     // optional filter
  const int64_t* target_offsets;
  int64_t Lcap;                  // 0: none
  int k;
  int32_t* ids;
  float* dist;
  const int* qmode;
  int want_mode;
  // multi-block variant (k_ivf_w): per-query shared bound, candidate list and counters
  uint32_t* tau_g;
  uint32_t* cand_cnt;
  uint32_t* done_cnt;
  uint64_t* cand;
  int64_t cand_cap;
};

__device__ __forceinline__ bool is_member(const int32_t* S, int64_t nS, int32_t n) {
  int64_t lo = 0, hi = nS;
  while (lo < hi) {
    int64_t mid = lo + ((hi - lo) >> 1);
    if (S[mid] < n) lo = mid + 1; else hi = mid;
  }
  return lo < nS && S[lo] == n;
}

// Exclusive prefix count of `flag` over the block in thread order, and the block total.
__device__ __forceinline__ int block_rank(bool flag, int* s_wave, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  unsigned long long b = __ballot(flag);
  int within = __popcll(b & ((1ull << lane) - 1ull));
  if (lane == 0) s_wave[wave] = __popcll(b);
  __syncthreads();
  int before = 0, tot = 0;
  for (int w = 0; w < nw; ++w) {
    int c = s_wave[w];
    if (w < wave) before += c;
    tot += c;
  }
  __syncthreads();
  *total = tot;
  return before + within;
}

template <int MT>
__global__ __launch_bounds__(kScanThreads) void k_ivf(IvfArgs a) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int M = MT ? MT : a.M;
  float* A = reinterpret_cast<float*>(smem);
  uint64_t* keys = reinterpret_cast<uint64_t*>(smem + table_bytes(M));
  BlockVars* bv = reinterpret_cast<BlockVars*>(smem + ivf_lds_main(M));
  int& s_cnt = bv->cnt;
  uint32_t& s_tau = bv->tau;
  int* s_wave = bv->wave_cnt;

  const int tid = threadIdx.x;
  const int64_t q = blockIdx.x;
  if (a.qmode && a.qmode[q] != a.want_mode) return;
  if constexpr (rot_m(MT)) fill_table_rot<MT>(A, reinterpret_cast<float*>(keys), a.lut + q * M * 256);
  else for (int i = tid; i < M * 256; i += blockDim.x) A[i] = a.lut[q * M * 256 + i];
  if (tid == 0) {
    s_cnt = 0;
    s_tau = kOrdMax;
  }
  __syncthreads();

  const int32_t* S = nullptr;
  int64_t nS = 0;
  if (a.target_ids) {
    int64_t o0 = a.target_offsets[q];
    S = a.target_ids + o0;
    nS = a.target_offsets[q + 1] - o0;
  }
  const int np = a.nprobe_q ? a.nprobe_q[q] : a.nprobe;
  int64_t taken = 0;
  bool done = false;
  for (int p = 0; p < np && !done; ++p) {
    const int list = a.probe[q * a.probe_stride + p];
    const int64_t b = a.list_off[list], e = a.list_off[list + 1];
    for (int64_t t0 = b; t0 < e && !done; t0 += blockDim.x) {
      const int64_t pos = t0 + tid;
      bool valid = pos < e;
      int32_t id = valid ? a.list_ids[pos] : -1;
      if (valid && S) valid = is_member(S, nS, id);
      if (a.Lcap > 0) {
        int tot;
        int rank = block_rank(valid, s_wave, &tot);
        if (taken + rank >= a.Lcap) valid = false;
        taken += tot;
        if (taken >= a.Lcap) done = true;  // uniform
      }
      uint64_t key[1] = {kKeyMax};
      uint32_t pend = 0;
      if (valid) {
        float d;
        bool maybe = true;
        if constexpr (rot_m(MT)) {
          // the list-ordered copy is rotated by position; filter on the rotated-order sum first
          // (the block-wide vote in sel_offer brings static LDS with it: the table is not at 0)
          d = adc_row_rot<MT, false>(A, a.codes_list + pos * M, ((uint32_t)pos & 31u) << 2);
          maybe = d <= rot_filter(s_tau, rot_eps(MT));
          if (maybe) d = adc_row_exact_rot<MT>(A, a.codes_list + pos * M, pos);
        } else {
          d = adc_row<MT>(A, a.codes_list + pos * M, M);
        }
        if (maybe) {
          key[0] = make_key(d, id);
          if ((uint32_t)(key[0] >> 32) <= s_tau) pend = 1;
        }
      }
      sel_offer<1>(keys, &s_cnt, &s_tau, a.k, key, pend);
    }
  }
  __syncthreads();
  sel_compact(keys, &s_cnt, &s_tau, a.k);
  write_result(keys, s_cnt, a.k, a.ids + q * a.k, a.dist ? a.dist + q * a.k : nullptr);
}

// Inverted-index scan over the concatenation of a query's probed lists, for the two cases in
// which Alg. 2's result does not depend on who scores which member: no candidate cap (every
// member of the probed lists is a candidate), or a cap without a target set (the candidates are
// then simply the first L members in traversal order).  The members are numbered 0 .. total-1
// in traversal order ("virtual" positions; a prefix sum over the list lengths, kept in LDS, maps
// them to positions in the list-ordered arrays), cut into units of kUnitTiles wave-tiles; the
// units are dealt to the query's blocks in turn and taken by a block's waves from a counter in
// LDS -- tiles are full whatever the list lengths are.
// Scoring, software pipeline and selection as in k_scan_w; identifiers are read for every
// member only when a target set has to be tested, otherwise only for the few rows that pass the
// distance filter.
constexpr int kIvfMaxProbe = 4096;  // lists per query this kernel keeps prefix sums for

__host__ __device__ inline size_t ivf_w_lds(int M, int nprobe) {
  return table_bytes(M) + (size_t)(kScanThreads / 64 + 1) * kWaveCap * 8 + (size_t)(2 * nprobe + 2) * 4 +
         kBlockVarsBytes;
}

template <int MT>
__global__ __launch_bounds__(kScanThreads) void k_ivf_w(IvfArgs a) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int M = MT ? MT : a.M;
  float* A = reinterpret_cast<float*>(smem);
  uint64_t* wbuf = reinterpret_cast<uint64_t*>(smem + table_bytes(M));  // [waves + 1][kWaveCap]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nwaves = blockDim.x >> 6;
  uint32_t* s_pref = reinterpret_cast<uint32_t*>(wbuf + (size_t)(nwaves + 1) * kWaveCap);  // [nprobe + 1] (+1 pad)
  uint32_t* s_start = s_pref + a.nprobe + 2;                                               // [nprobe]
  BlockVars* bv = reinterpret_cast<BlockVars*>(s_start + a.nprobe);
  int& s_total = bv->total;
  int& s_off = bv->off;
  int& s_last = bv->last;
  const int64_t q = blockIdx.y;
  if (a.qmode && a.qmode[q] != a.want_mode) return;
  uint64_t* cand = a.cand + q * a.cand_cap;
  const int k = a.k;
  const int np = a.nprobe_q ? a.nprobe_q[q] : a.nprobe;

  // list starts and the running total of list lengths (the lists are disjoint: the total is < 2^31)
  for (int i = tid; i < np; i += blockDim.x) {
    const int list = a.probe[q * a.probe_stride + i];
    const int64_t b = a.list_off[list], e = a.list_off[list + 1];
    s_start[i] = (uint32_t)b;
    s_pref[i + 1] = (uint32_t)(e - b);
  }
  if (tid == 0) {
    s_pref[0] = 0u;
    bv->cnt = nwaves;  // units of this block handed out so far
  }
  __syncthreads();
  if (wave == 0) {
    const int per = (np + 63) / 64;
    const int lo = lane * per < np ? lane * per : np, hi = lo + per < np ? lo + per : np;
    uint32_t sum = 0;
    for (int i = lo; i < hi; ++i) sum += s_pref[i + 1];
    uint32_t incl = sum;
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t t = __shfl_up(incl, o, 64);
      if (lane >= o) incl += t;
    }
    uint32_t run = incl - sum;
    for (int i = lo; i < hi; ++i) {
      run += s_pref[i + 1];
      s_pref[i + 1] = run;
    }
  }
  __syncthreads();
  int64_t total = s_pref[np];
  if (a.Lcap > 0 && total > a.Lcap) total = a.Lcap;  // (only launched without a target set then)

  constexpr int64_t kWaveTile = 64 * kRowsPerLane;
  constexpr int64_t kUnitRows = kUnitTiles * kWaveTile;
  const int64_t nunits = (total + kUnitRows - 1) / kUnitRows;
  if ((int64_t)blockIdx.x < nunits) {  // block-uniform: this block has at least one unit
    const float* lut = a.lut + q * M * 256;
    if constexpr (rot_m(MT)) {
      fill_table_rot<MT>(A, reinterpret_cast<float*>(wbuf), lut);  // the wave buffers are not in use yet
    } else {
      for (int i = tid; i < M * 256; i += blockDim.x) A[i] = lut[i];
      __syncthreads();
    }
    const int32_t* S = nullptr;
    int64_t nS = 0;
    if (a.target_ids) {
      const int64_t o0 = a.target_offsets[q];
      S = a.target_ids + o0;
      nS = a.target_offsets[q + 1] - o0;
    }
    uint64_t* buf = wbuf + (size_t)wave * kWaveCap;
    int cnt = 0;
    uint32_t tau = kOrdMax;
    uint32_t tg = __hip_atomic_load(a.tau_g + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

    // Block b owns the units b, b + gridDim.x, b + 2 gridDim.x, ...; its waves take them one
    // after the other from a counter in LDS (the first one per wave is fixed).
    int64_t unit = (int64_t)blockIdx.x + (int64_t)gridDim.x * wave;
    int t_in = 0;
    int hint = 0;  // a list at or before the one the next tile starts in (wave-uniform)
    // One tile of the wave: virtual base (or -1), positions of its kRowsPerLane slices in the
    // list-ordered arrays (members past the end repeat the last one and are not live).
    struct Tile { int64_t base; uint32_t pos[kRowsPerLane]; uint32_t live; };
    auto next_tile = [&]() -> Tile {
      Tile t;
      t.live = 0;
      if (unit >= nunits || unit * kUnitRows + (int64_t)t_in * kWaveTile >= total) {
        t.base = -1;
#pragma unroll
        for (int r = 0; r < kRowsPerLane; ++r) t.pos[r] = s_start[0];  // any valid position (total > 0 here)
        return t;
      }
      t.base = unit * kUnitRows + (int64_t)t_in * kWaveTile;
      if (t_in == 0) {  // new unit: find the list of its first member, largest p with pref[p] <= base
        int lo = 0, hi = np;  // pref[lo] <= base < pref[hi] (base < total <= pref[np])
        while (hi - lo > 1) {
          const int mid = (lo + hi) >> 1;
          if ((int64_t)s_pref[mid] <= t.base) lo = mid;
          else hi = mid;
        }
        hint = lo;
      }
      int p = hint;
#pragma unroll
      for (int r = 0; r < kRowsPerLane; ++r) {
        int64_t v = t.base + r * 64 + lane;
        if (v < total) t.live |= 1u << r;
        else v = total - 1;
        while ((int64_t)s_pref[p + 1] <= v) ++p;  // ends: v < total <= pref[np]
        t.pos[r] = s_start[p] + (uint32_t)(v - (int64_t)s_pref[p]);
      }
      hint = __shfl(p, 63, 64);  // the last member's list: not after the next tile's first
      if (++t_in == kUnitTiles) {
        t_in = 0;
        int c = lane == 0 ? atomicAdd(&bv->cnt, 1) : 0;
        c = __builtin_amdgcn_readfirstlane(c);
        unit = (int64_t)blockIdx.x + (int64_t)gridDim.x * c;
      }
      return t;
    };

    if constexpr (rot_m(MT)) {
      Tile cur = next_tile(), nxt = next_tile();
      uint32_t w[kRowsPerLane][MT / 4];
      int32_t idc[kRowsPerLane], idn[kRowsPerLane];
#pragma unroll
      for (int r = 0; r < kRowsPerLane; ++r) {
        load_row_words<MT>(a.codes_list + (int64_t)cur.pos[r] * M, w[r]);
        idc[r] = S ? a.list_ids[cur.pos[r]] : 0;
      }
      while (cur.base >= 0) {  // wave-uniform
        const uint32_t bound = tg < tau ? tg : tau;
        const float fb = rot_filter(bound, rot_eps(MT));
        uint64_t key[kRowsPerLane];
        uint32_t maybe = 0, pend = 0;
#pragma unroll
        for (int r = 0; r < kRowsPerLane; ++r) {
          key[r] = kKeyMax;
          uint32_t addr[MT];
          rot_addrs<MT>(w[r], (cur.pos[r] & 31u) << 2, addr);
          load_row_words<MT>(a.codes_list + (int64_t)nxt.pos[r] * M, w[r]);
          idn[r] = S ? a.list_ids[nxt.pos[r]] : 0;
          if (rot_sum_abandon<MT>(addr, fb) <= fb) maybe |= 1u << r;
        }
        maybe &= cur.live;
        if (__ballot(maybe != 0) != 0ull) {
#pragma unroll
          for (int r = 0; r < kRowsPerLane; ++r) {
            if (maybe & (1u << r)) {
              const int32_t id = S ? idc[r] : a.list_ids[cur.pos[r]];
              if (S && !is_member(S, nS, id)) continue;
              const float d = adc_row_exact_rot<MT>(A, a.codes_list + (int64_t)cur.pos[r] * M, cur.pos[r]);
              key[r] = make_key(d, id);
              if ((uint32_t)(key[r] >> 32) <= bound) pend |= 1u << r;
            }
          }
        }
        if (__ballot(pend != 0) != 0ull) {
          const uint32_t before = tau;
          wave_offer<kRowsPerLane>(buf, cnt, tau, k, key, pend, lane);
          if (tau < before && lane == 0) atomicMin(a.tau_g + q, tau);
        }
        cur = nxt;
#pragma unroll
        for (int r = 0; r < kRowsPerLane; ++r) idc[r] = idn[r];
        if (t_in == 0) tg = __hip_atomic_load(a.tau_g + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        nxt = next_tile();
      }
    } else {
      for (Tile cur = next_tile(); cur.base >= 0; cur = next_tile()) {
        const uint32_t bound = tg < tau ? tg : tau;
        uint64_t key[kRowsPerLane];
        uint32_t pend = 0;
#pragma unroll
        for (int r = 0; r < kRowsPerLane; ++r) {
          key[r] = kKeyMax;
          if (cur.live & (1u << r)) {
            const int32_t id = a.list_ids[cur.pos[r]];
            if (S && !is_member(S, nS, id)) continue;
            const float d = adc_row<MT>(A, a.codes_list + (int64_t)cur.pos[r] * M, M);
            key[r] = make_key(d, id);
            if ((uint32_t)(key[r] >> 32) <= bound) pend |= 1u << r;
          }
        }
        if (__ballot(pend != 0) != 0ull) {
          const uint32_t before = tau;
          wave_offer<kRowsPerLane>(buf, cnt, tau, k, key, pend, lane);
          if (tau < before && lane == 0) atomicMin(a.tau_g + q, tau);
        }
        if (t_in == 0) tg = __hip_atomic_load(a.tau_g + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    tg = __hip_atomic_load(a.tau_g + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint64_t* best;
    const int c = block_collect(wbuf, nwaves, cnt, tau, tg < tau ? tg : tau, k, &best, &s_total, &s_off);
    if (gridDim.x == 1) {  // the query's only block: its result is the query's result
      write_result(best, c, k, a.ids + q * a.k, a.dist ? a.dist + q * a.k : nullptr);
      return;
    }
    publish_block_result(best, c, k, cand, a.cand_cnt + q, a.tau_g + q, &s_off);
  }
  finish_query(wbuf, nwaves, k, cand, a.cand_cnt + q, a.done_cnt + q, gridDim.x, a.ids + q * a.k,
               a.dist ? a.dist + q * a.k : nullptr, &s_total, &s_off, &s_last);
}

// ------------------------------------------------------------------ small utility kernels
// tau[q] = largest bound; the kScanArrays - 1 counter arrays that follow it (stride entries apart) = 0
constexpr int kScanArrays = 4;
__global__ void k_init_scan(uint32_t* tau, int Q, int stride) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= Q) return;
  tau[i] = kOrdMax;
#pragma unroll
  for (int j = 1; j < kScanArrays; ++j) tau[j * (size_t)stride + i] = 0u;
}

// Per-query plan of the query procedure (Alg. 3): mode 0 = linear scan, 1 = inverted index;
// number of lists ceil(K L / |S|) capped at K and at pmax.
__global__ void k_plan(const int64_t* target_offsets, int64_t N, int Q, int64_t theta, int K, int64_t L, int pmax,
                       int* qmode, int* nprobe_q) {
  int q = blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= Q) return;
  int64_t sz = target_offsets ? target_offsets[q + 1] - target_offsets[q] : N;
  int mode = (K > 0 && sz >= theta) ? 1 : 0;
  qmode[q] = mode;
  int64_t p = 1;
  if (mode == 1) {
    p = sz > 0 ? ((int64_t)K * L + sz - 1) / sz : K;  // K, L, sz < 2^31: no overflow
    if (p > K) p = K;
    if (p > pmax) p = pmax;
    if (p < 1) p = 1;
  }
  nprobe_q[q] = (int)p;
}

// Segment offsets i * len for i = 0..Q.
__global__ void k_iota_offsets(int64_t* off, int Q, int64_t len) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i <= Q) off[i] = (int64_t)i * len;
}

// Evenly spread, strictly increasing target identifiers for the threshold calibration:
// query i gets ids[i * S + j] = floor((j + i / nq) * N / S), j < S; offsets[i] = i * S.
__global__ void k_spread_ids(int32_t* ids, int64_t* offsets, int nq, int64_t S, int64_t N) {
  int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g <= nq) offsets[g] = g * S;
  if (g >= (int64_t)nq * S) return;
  int64_t i = g / S, j = g - i * S;
  double pos = ((double)j + (double)i / (double)nq) * ((double)N / (double)S);
  int64_t v = (int64_t)pos;
  ids[g] = (int32_t)(v < N ? v : N - 1);
}

// ------------------------------------------------------------------ offline kernels
// Eq. (1): grid (ceil(n / 256), M), block 256; thread = one vector, block = one sub-space.
__global__ void k_encode(const float* __restrict__ cb, const float* __restrict__ x, int64_t n, int D, int M, int Ds,
                         uint8_t* __restrict__ codes) {
  extern __shared__ __align__(16) uint8_t smem[];
  float* c = reinterpret_cast<float*>(smem);        // [256][Ds]
  float* xs = c + 256 * Ds;                          // [Ds][256]
  const int m = blockIdx.y, tid = threadIdx.x;
  for (int i = tid; i < 256 * Ds; i += blockDim.x) c[i] = cb[(size_t)m * 256 * Ds + i];
  const int64_t row = (int64_t)blockIdx.x * blockDim.x + tid;
  if (row < n)
    for (int j = 0; j < Ds; ++j) xs[j * 256 + tid] = x[row * D + m * Ds + j];
  __syncthreads();
  if (row >= n) return;
  int best = 0;
  float bestd = 0.f;
  for (int z = 0; z < 256; ++z) {
    float acc = 0.f;
    for (int j = 0; j < Ds; ++j) {
      float diff = __fsub_rn(xs[j * 256 + tid], c[z * Ds + j]);
      acc = __fadd_rn(acc, __fmul_rn(diff, diff));
    }
    if (z == 0 || acc < bestd) {
      bestd = acc;
      best = z;
    }
  }
  codes[row * M + m] = (uint8_t)best;
}

// Sec. 4.5 (OPQ variant): y = R x per row.  Block = 32 output coordinates x 8 rows; the inner
// index runs in ascending order through 32-wide LDS tiles with one accumulator per output, one
// rounding per operation, so the result is bit-identical to the plain triple loop.
__global__ __launch_bounds__(256) void k_rotate(const float* __restrict__ R, int D, const float* __restrict__ x,
                                                int64_t n, float* __restrict__ y) {
  __shared__ float Rs[32][33];
  __shared__ float Xs[8][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int r = blockIdx.x * 32 + tx;
  const int64_t i = (int64_t)blockIdx.y * 8 + ty;
  float acc = 0.f;
  for (int c0 = 0; c0 < D; c0 += 32) {
    for (int rr = ty; rr < 32; rr += 8) {
      int gr = blockIdx.x * 32 + rr, gc = c0 + tx;
      Rs[rr][tx] = (gr < D && gc < D) ? R[(size_t)gr * D + gc] : 0.f;
    }
    Xs[ty][tx] = (i < n && c0 + tx < D) ? x[i * D + c0 + tx] : 0.f;
    __syncthreads();
    const int cmax = D - c0 < 32 ? D - c0 : 32;
    for (int c = 0; c < cmax; ++c) acc = __fadd_rn(acc, __fmul_rn(Rs[tx][c], Xs[ty][c]));
    __syncthreads();
  }
  if (r < D && i < n) y[i * D + r] = acc;
}

// Symmetric table: sym[m][i][j] = squared distance between code words i and j of codebook m.
// grid (256, M), block 256.
__global__ void k_sym_table(const float* __restrict__ cb, int Ds, float* __restrict__ sym) {
  const int m = blockIdx.y, i = blockIdx.x, j = threadIdx.x;
  const float* a = cb + ((size_t)m * 256 + i) * Ds;
  const float* b = cb + ((size_t)m * 256 + j) * Ds;
  float acc = 0.f;
  for (int t = 0; t < Ds; ++t) {
    float diff = __fsub_rn(a[t], b[t]);
    acc = __fadd_rn(acc, __fmul_rn(diff, diff));
  }
  sym[((size_t)m * 256 + i) * 256 + j] = acc;
}

// a(n): one block per item at a time (grid-stride over items).  The item's M table rows
// sym[m][code_n[m]][.] act as its distance table; the coarse codes are scanned with it and
// the arg-min (lowest k on ties) is reduced over the block.
template <int MT>
__global__ __launch_bounds__(256) void k_assign(const float* __restrict__ sym, const uint8_t* __restrict__ codes,
                                                int64_t n, int64_t rot_base, int Mrt,
                                                const uint8_t* __restrict__ coarse, int K,
                                                int32_t* __restrict__ assign) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int M = MT ? MT : Mrt;
  float* A = reinterpret_cast<float*>(smem);  // [M][256]
  __shared__ uint64_t s_best[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int64_t item = blockIdx.x; item < n; item += gridDim.x) {
    __syncthreads();
    for (int i = tid; i < M * 256; i += blockDim.x) {
      int m = i >> 8, z = i & 255;
      int pos = rot_base >= 0 ? (int)((m - (rot_base + item)) & (M - 1)) : m;  // rotated storage: see adc_row_rot
      A[i] = sym[((size_t)m * 256 + codes[item * M + pos]) * 256 + z];
    }
    __syncthreads();
    uint64_t best = kKeyMax;
    for (int k = tid; k < K; k += blockDim.x) {
      uint64_t key = make_key(adc_row<MT>(A, coarse + (size_t)k * M, M), k);
      if (key < best) best = key;
    }
    for (int o = 32; o > 0; o >>= 1) {
      uint64_t other = __shfl_xor(best, o, 64);
      if (other < best) best = other;
    }
    if (lane == 0) s_best[wave] = best;
    __syncthreads();
    if (tid == 0) {
      uint64_t b = s_best[0];
      for (int w = 1; w < (int)(blockDim.x >> 6); ++w)
        if (s_best[w] < b) b = s_best[w];
      assign[item] = (int32_t)(uint32_t)b;
    }
  }
}

// a(n) with pruning, for large K.  The K centres are grouped around G "super-centres" (PQ codes
// too); coarse_g holds the centres group after group, perm_g their original numbers, radius[j]
// the largest sqrt(d_S) between a member of group j and its super-centre.  d_S is a squared
// Euclidean distance between decoded vectors, so for every member c of group j
//   sqrt(d_S(x, c)) >= sqrt(d_S(x, g_j)) - radius[j]      (triangle inequality).
// A group is skipped only when this bound, shrunk by a rounding margin, still exceeds the best
// distance already found; every centre that could attain the minimum (or tie with it) is
// scored with the exact fp32 sum, so the result equals the brute-force arg-min, ties to lower k.
template <int MT>
__global__ __launch_bounds__(256) void k_assign_pruned(const float* __restrict__ sym, const uint8_t* __restrict__ codes,
                                                       int64_t n, int64_t rot_base, int Mrt,
                                                       const uint8_t* __restrict__ super, int G,
                                                       const float* __restrict__ radius,
                                                       const uint8_t* __restrict__ coarse_g,
                                                       const int32_t* __restrict__ perm_g,
                                                       const int32_t* __restrict__ group_off,
                                                       int32_t* __restrict__ assign, unsigned long long* visited_total) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int M = MT ? MT : Mrt;
  float* A = reinterpret_cast<float*>(smem);           // [M][256]
  float* lb = A + M * 256;                             // [G] lower bound on d_S to any member of group j
  __shared__ uint64_t s_red[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  unsigned long long visited = 0;
  for (int64_t item = blockIdx.x; item < n; item += gridDim.x) {
    __syncthreads();
    for (int i = tid; i < M * 256; i += blockDim.x) {
      int m = i >> 8, z = i & 255;
      int pos = rot_base >= 0 ? (int)((m - (rot_base + item)) & (M - 1)) : m;  // rotated storage: see adc_row_rot
      A[i] = sym[((size_t)m * 256 + codes[item * M + pos]) * 256 + z];
    }
    __syncthreads();
    // distances to the super-centres, bounds, nearest super-centre
    uint64_t near = kKeyMax;
    for (int j = tid; j < G; j += blockDim.x) {
      float d1 = adc_row<MT>(A, super + (size_t)j * M, M);
      float root = __fsqrt_rn(d1) * 0.99999f - radius[j] * 1.00001f;
      root = root > 0.f ? root : 0.f;
      lb[j] = root * root * 0.99999f;
      uint64_t key = make_key(d1, j);
      if (key < near) near = key;
    }
    for (int o = 32; o > 0; o >>= 1) {
      uint64_t other = __shfl_xor(near, o, 64);
      if (other < near) near = other;
    }
    if (lane == 0) s_red[wave] = near;
    __syncthreads();
    near = s_red[0];
    for (int w = 1; w < 4; ++w) if (s_red[w] < near) near = s_red[w];
    const int jstar = (int)(uint32_t)near;
    __syncthreads();
    // exact scores inside the nearest group
    uint64_t best = kKeyMax;
    for (int p = group_off[jstar] + tid; p < group_off[jstar + 1]; p += blockDim.x) {
      uint64_t key = make_key(adc_row<MT>(A, coarse_g + (size_t)p * M, M), perm_g[p]);
      if (key < best) best = key;
    }
    for (int o = 32; o > 0; o >>= 1) {
      uint64_t other = __shfl_xor(best, o, 64);
      if (other < best) best = other;
    }
    if (lane == 0) s_red[wave] = best;
    __syncthreads();
    best = s_red[0];
    for (int w = 1; w < 4; ++w) if (s_red[w] < best) best = s_red[w];
    __syncthreads();
    // every other group whose bound does not exclude it (an empty nearest group leaves best = max: all are visited)
    for (int j = tid; j < G; j += blockDim.x) {
      if (j == jstar) continue;
      float bd = best == kKeyMax ? __uint_as_float(0x7F800000u) : float_of_ord((uint32_t)(best >> 32)) * 1.00001f;
      if (lb[j] > bd) continue;
      for (int p = group_off[j]; p < group_off[j + 1]; ++p) {
        uint64_t key = make_key(adc_row<MT>(A, coarse_g + (size_t)p * M, M), perm_g[p]);
        if (key < best) best = key;
        ++visited;
      }
    }
    for (int o = 32; o > 0; o >>= 1) {
      uint64_t other = __shfl_xor(best, o, 64);
      if (other < best) best = other;
    }
    if (lane == 0) s_red[wave] = best;
    __syncthreads();
    if (tid == 0) {
      uint64_t b = s_red[0];
      for (int w = 1; w < 4; ++w) if (s_red[w] < b) b = s_red[w];
      assign[item] = (int32_t)(uint32_t)b;
    }
  }
  if (visited_total && visited) atomicAdd(visited_total, visited);
}

// General row copy between plain and rotated storage, optionally gathering by identifier:
//   source row of output row i: src = ids ? ids[i] : i;
//   in_rot  >= 0: the source array stores row s rotated by (in_rot + s) bytes, else plain;
//   out_rot >= 0: output row i is stored rotated by (out_rot + i) bytes, else plain.
// One thread per output dword.
__global__ void k_copy_rows(const uint8_t* __restrict__ in, int64_t in_rot, const int32_t* __restrict__ ids,
                            int64_t n, int M, uint8_t* __restrict__ out, int64_t out_rot) {
  const int M4 = M >> 2;
  int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= n * M4) return;
  const int64_t i = g / M4;
  const int w = (int)(g - i * M4);
  const int64_t src = ids ? (int64_t)ids[i] : i;
  const uint8_t* row = in + src * M;
  uint32_t v = 0;
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    int t = 4 * w + b;                                             // output byte position
    int m = out_rot >= 0 ? (int)((t + out_rot + i) & (M - 1)) : t;  // sub-space it holds
    int pos = in_rot >= 0 ? (int)((m - (in_rot + src)) & (M - 1)) : m;
    v |= (uint32_t)row[pos] << (8 * b);
  }
  reinterpret_cast<uint32_t*>(out)[g] = v;
}

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

bool m_supported(int M) { return M >= 4 && M <= RII_MAX_M && M % 4 == 0; }

template <typename Kern>
int set_lds(Kern kern, size_t bytes) {
  if (bytes > 48 * 1024) RII_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  return RII_OK;
}

// The kernels that address their table as "LDS address 0" must not have static LDS in front of
// the dynamic allocation; refuse to launch otherwise.
template <typename Kern>
int require_table_at_lds_zero(Kern kern) {
  hipFuncAttributes attr{};
  RII_HIP(hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(kern)));
  return attr.sharedSizeBytes == 0 ? RII_OK : RII_ERR_DEVICE;
}

// set_lds for the kernels whose table must sit at LDS address 0 (checked once per kernel)
template <typename Kern>
int set_lds0(Kern kern, size_t bytes) {
  static int checked = -1;  // one instance per kernel type and address
  static const void* which = nullptr;
  if (checked < 0 || which != reinterpret_cast<const void*>(kern)) {
    int rc = require_table_at_lds_zero(kern);
    if (rc) return rc;
    checked = 1;
    which = reinterpret_cast<const void*>(kern);
  }
  return set_lds(kern, bytes);
}

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
  int64_t want = (kWantBlocks + Q - 1) / Q;
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
    chunk_rows = (rows + nchunks - 1) / nchunks;
    chunk_rows = (chunk_rows + tile - 1) / tile * tile;
    nchunks = (rows + chunk_rows - 1) / chunk_rows;
  }
  if (groups * nchunks < kWantBlocks) return false;
  *nchunks_out = nchunks;
  *chunk_rows_out = chunk_rows;
  return true;
}

// Scan `nrows_max` rows per query (linear: the whole array) and leave per-block partial keys in
// the workspace; then select.  Workspace layout: [tau Q u32][partial Q*nchunks*k u64].
int launch_scan(const rii_index* idx, const uint8_t* codes, int64_t N, const float* lut, int Q, int mode,
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
  a.codes = codes; a.N = N; a.M = M; a.lut = lut;
  a.target_ids = target_ids; a.target_offsets = target_offsets;
  a.chunk_rows = chunk_rows; a.k = topk; a.partial = partial; a.tau_g = tau;
  int64_t bchunks, brows;
  const bool batched = plan_batch(M, Q, max_rows, topk, &bchunks, &brows) && mode == kLinear && !qmode;
  a.cand_cnt = cand_cnt; a.cand_cap = std::max(nchunks, bchunks) * topk;
  a.nq = Q;
  // [prepass minima] follow the candidates
  uint32_t* minima = reinterpret_cast<uint32_t*>(partial + (size_t)Q * a.cand_cap);
  k_init_scan<<<(Q + 255) / 256, 256, 0, st>>>(tau, Q, (int)cstride);
  a.done_cnt = done_cnt; a.ids = ids; a.dist = dist; a.out_stride = out_stride;
  a.qmode = qmode; a.want_mode = want_mode;
  dim3 grid((unsigned)nchunks, (unsigned)Q);
  if (Q > 65535) return RII_ERR_UNSUPPORTED;
  const bool timed = mode == kLinear && idx->ev_start && idx->ev_stop && codes == idx->d_codes;
  if (timed) RII_HIP(hipEventRecord(static_cast<hipEvent_t>(idx->ev_start), st));
  if (topk <= kWaveK) {
    // When a query's rows are split over several blocks, a short first pass over the leading
    // rows seeds the shared bound, so that the main pass starts with few candidates.
    const int64_t tile_rows = (int64_t)kScanThreads * kRowsPerLane;
    const int pre_blocks = (int)std::min<int64_t>(kPrepassBlocks, (max_rows + tile_rows - 1) / tile_rows);
    // The single-query kernel seeds the bound itself when all its blocks run at once and a query
    // has at least topk of them (rotated form only); otherwise a separate pass does it.
    const bool seed_inside = nchunks > 1 && rot_m(M) && !batched && nchunks >= topk && nchunks <= kPrepassBlocks &&
                             (int64_t)Q * nchunks <= kWantBlocks;
    const bool prepass = nchunks > 1 && !seed_inside;
    a.seed_inside = seed_inside ? 1 : 0;
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
      const bool pre4 = bchunks > 1;
      switch (M) {
        case 8: { int rc = set_lds0(k_scan_w4<8>, lds4); if (rc) return rc;
                  if (pre4) { rc = set_lds0(k_tau0<8, kLinear>, tau0_lds(M) + kBlockVarsBytes); if (rc) return rc;
                              k_tau0<8, kLinear><<<pgrid, kScanThreads, tau0_lds(M) + kBlockVarsBytes, st>>>(pre); }
                  k_scan_w4<8><<<g4, kScanThreads, lds4, st>>>(a4); } break;
        case 16: { int rc = set_lds0(k_scan_w4<16>, lds4); if (rc) return rc;
                   if (pre4) { rc = set_lds0(k_tau0<16, kLinear>, tau0_lds(M) + kBlockVarsBytes); if (rc) return rc;
                               k_tau0<16, kLinear><<<pgrid, kScanThreads, tau0_lds(M) + kBlockVarsBytes, st>>>(pre); }
                   k_scan_w4<16><<<g4, kScanThreads, lds4, st>>>(a4); } break;
        default: { int rc = set_lds0(k_scan_w4<32>, lds4); if (rc) return rc;
                   if (pre4) { rc = set_lds0(k_tau0<32, kLinear>, tau0_lds(M) + kBlockVarsBytes); if (rc) return rc;
                               k_tau0<32, kLinear><<<pgrid, kScanThreads, tau0_lds(M) + kBlockVarsBytes, st>>>(pre); }
                   k_scan_w4<32><<<g4, kScanThreads, lds4, st>>>(a4); } break;
      }
    } else if (mode == kLinear && rot_m(M) && nchunks == 1 && !qmode && Q >= 2) {
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
      DISPATCH_M(M, { int rc = set_lds0(k_scan_w<MT, kSubset>, ldsw); if (rc) return rc;
                      if (prepass) { int rc2 = set_lds0(k_tau0<MT, kSubset>, tau0_lds(M) + kBlockVarsBytes); if (rc2) return rc2; }
                      if (prepass) k_tau0<MT, kSubset><<<pgrid, kScanThreads, tau0_lds(M) + kBlockVarsBytes, st>>>(pre);
                      k_scan_w<MT, kSubset><<<grid, kScanThreads, ldsw, st>>>(a); });
    }
  } else {
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

size_t scan_ws_bytes(int M, int Q, int64_t max_rows, int topk) {
  int64_t nchunks, chunk_rows;
  scan_chunks(Q, max_rows, &nchunks, &chunk_rows);
  int64_t bchunks, brows;
  plan_batch(M, Q, max_rows, topk, &bchunks, &brows);
  const int64_t cap_chunks = std::max(nchunks, bchunks);
  return kScanArrays * align_up((size_t)Q * 4, 256) + (size_t)Q * cap_chunks * topk * 8 +
         (size_t)Q * kPrepassBlocks * (kScanThreads / 64) * 4 + 256;
}

// ------------------------------------------------------------------ LDS look-up ceiling
// The inner loop of the scan kernels with everything else taken away: per look-up one byte
// permute (address), one LDS read, one add per component.  The "code words" are made up in
// registers (a xorshift step per 32 look-ups); lane l uses slot (l + t) % 32 at step t like
// k_scan_w2 / k_scan_w4, so the 32 lanes of a half-wave never share a bank.
template <int WIDTH>
__global__ __launch_bounds__(kScanThreads) void k_lds_lookups(int iters, uint32_t* sink) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int tid = threadIdx.x;
  for (int i = tid; i < 65536 / 4; i += blockDim.x) reinterpret_cast<uint32_t*>(smem)[i] = (uint32_t)i;
  __syncthreads();
  uint32_t lb4[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    lb4[j] = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) lb4[j] |= ((uint32_t)((tid + 4 * j + b) & 31) * 8u) << (8 * b);
  }
  uint32_t w[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) w[j] = (uint32_t)(tid * 8 + j) * 2654435761u + blockIdx.x;
  uint32_t acc0 = 0, acc1 = 0;
  uint64_t acc64 = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int t = 0; t < 32; ++t) {
      const uint32_t addr = __builtin_amdgcn_perm(w[t >> 2], lb4[t >> 2], 0x0c0c0400u | ((uint32_t)(t & 3) * 0x0101u));
      if constexpr (WIDTH == 64) {
        uint2 v = lds_read_u32x2(addr);
        acc64 += ((uint64_t)v.y << 32) | v.x;  // one 64-bit integer add per look-up
      } else if constexpr (WIDTH == 8) {
        uint2 v = lds_read_u32x2(addr);
        acc0 += v.x;
        acc1 += v.y;
      } else {
        acc0 += __float_as_uint(lds_read_f32(addr & ~4u));
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      w[j] ^= w[j] << 13;
      w[j] ^= w[j] >> 17;
      w[j] ^= w[j] << 5;
    }
  }
  acc0 ^= (uint32_t)acc64 ^ (uint32_t)(acc64 >> 32);
  if ((acc0 ^ acc1) == 0x9e3779b9u) sink[0] = acc0;  // practically never: keeps the loop alive
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
  } else if (topk <= kWaveK && rot_m(idx->M) && nchunks == 1 && Q >= 2) {
    *queries_per_block = 2;
    *row_chunks = 1;
  } else {
    *queries_per_block = 1;
    *row_chunks = nchunks;
  }
  return RII_OK;
}

int rii_bench_lds_lookups(int width, int blocks, int iters, int lds_bytes, uint32_t* sink, void* stream) {
  if ((width != 4 && width != 8 && width != 64) || blocks < 1 || iters < 1 || !sink) return RII_ERR_INVALID_ARG;
  if (lds_bytes < 65536 || lds_bytes > 160 * 1024) return RII_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (width == 64) {
    int rc = set_lds0(k_lds_lookups<64>, (size_t)lds_bytes);
    if (rc) return rc;
    k_lds_lookups<64><<<blocks, kScanThreads, (size_t)lds_bytes, st>>>(iters, sink);
  } else if (width == 8) {
    int rc = set_lds0(k_lds_lookups<8>, (size_t)lds_bytes);
    if (rc) return rc;
    k_lds_lookups<8><<<blocks, kScanThreads, (size_t)lds_bytes, st>>>(iters, sink);
  } else {
    int rc = set_lds0(k_lds_lookups<4>, (size_t)lds_bytes);
    if (rc) return rc;
    k_lds_lookups<4><<<blocks, kScanThreads, (size_t)lds_bytes, st>>>(iters, sink);
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
  return launch_scan(idx, idx->d_codes, idx->N, lut, Q, kLinear, nullptr, nullptr, idx->N, topk, ids, dist, topk,
                     nullptr, 0, idx->ws, static_cast<hipStream_t>(stream));
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
  return launch_scan(idx, idx->d_codes, idx->N, lut, Q, kSubset, target_ids, target_offsets, rows, topk, ids, dist,
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
    return launch_scan(idx, idx->d_coarse_st, K, lut, Q, kLinear, nullptr, nullptr, K, nprobe, list_ids, list_d0,
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
  a.codes_list = idx->d_codes_list; a.list_ids = idx->d_list_ids; a.list_off = idx->d_list_off; a.M = M;
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
    k_init_scan<<<(Q + 255) / 256, 256, 0, st>>>(tau, Q, (int)cstride);
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
  void* ws = nullptr;
  if ((L == 0 || !target_ids) && topk <= kWaveK) {
    int rc = ensure_ws(idx, ivf_ws_bytes(Q, nprobe, topk));
    if (rc) return rc;
    ws = idx->ws;
  }
  return launch_ivf(idx, lut, Q, probe_lists, nprobe, nprobe, nullptr, target_ids, target_offsets, L, topk, ids,
                    dist, nullptr, 0, ws, static_cast<hipStream_t>(stream));
}

int rii_query(const rii_index_t* idx, const float* q, int Q, int topk, const int32_t* target_ids,
              const int64_t* target_offsets, int64_t max_targets, int64_t L, int32_t* ids, float* dist,
              void* stream) {
  if (!idx || !q || !ids || !dist || Q < 1 || topk < 1 || L < 1 || max_targets < 0) return RII_ERR_INVALID_ARG;
  if ((target_ids == nullptr) != (target_offsets == nullptr)) return RII_ERR_INVALID_ARG;
  if (topk > RII_MAX_TOPK || !m_supported(idx->M) || Q > 65535) return RII_ERR_UNSUPPORTED;
  if (idx->N < 1) return RII_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int M = idx->M, K = idx->K;
  const bool has_lists = K > 0;
  // Largest number of lists any inverted-index query of this batch can ask for: such a query
  // has |S| >= max(theta, 1), and |S| = N when there is no target set.
  int pmax = 1;
  if (has_lists) {
    int64_t smin = target_ids ? std::max<int64_t>(idx->theta, 1) : idx->N;
    int64_t p = ((int64_t)K * L + smin - 1) / smin;
    pmax = (int)std::min<int64_t>(p, K);
    if (pmax > RII_MAX_TOPK && K > RII_MAX_SORT) return RII_ERR_UNSUPPORTED;
  }
  // linear-scan queries have |S| < theta (and at most max_targets, N)
  int64_t lin_rows = target_ids ? std::min<int64_t>(max_targets, idx->N) : idx->N;
  if (has_lists && idx->theta > 0) lin_rows = std::min<int64_t>(lin_rows, idx->theta - 1);
  if (has_lists && idx->theta <= 0) lin_rows = 0;
  if (!target_ids && has_lists && idx->N >= idx->theta) lin_rows = 0;
  lin_rows = std::max<int64_t>(lin_rows, 1);

  const size_t lut_b = align_up((size_t)Q * M * 256 * 4, 256);
  const size_t plan_b = align_up((size_t)Q * 4, 256);
  const size_t probe_b = align_up((size_t)Q * pmax * 4, 256);
  const size_t scan_b = align_up(scan_ws_bytes(idx->M, Q, lin_rows, topk), 256);
  const size_t coarse_b = has_lists ? align_up(coarse_ws_bytes(idx, Q, pmax), 256) : 0;
  const size_t ivf_b = has_lists && topk <= kWaveK ? align_up(ivf_ws_bytes(Q, pmax, topk), 256) : 0;
  int rc = ensure_ws(idx, lut_b + 2 * plan_b + probe_b + std::max(std::max(scan_b, coarse_b), ivf_b));
  if (rc) return rc;
  uint8_t* w = static_cast<uint8_t*>(idx->ws);
  float* lut = reinterpret_cast<float*>(w); w += lut_b;
  int* qmode = reinterpret_cast<int*>(w); w += plan_b;
  int* nprobe_q = reinterpret_cast<int*>(w); w += plan_b;
  int32_t* probe = reinterpret_cast<int32_t*>(w); w += probe_b;
  void* stage_ws = w;

  k_build_lut<<<dim3(M, Q), 256, 0, st>>>(idx->d_cb, q, idx->D, M, idx->Ds, lut);
  k_plan<<<(Q + 255) / 256, 256, 0, st>>>(target_offsets, idx->N, Q, idx->theta, K, L, pmax, qmode, nprobe_q);
  // linear-scan branch (mode 0)
  if (target_ids) {
    rc = launch_scan(idx, idx->d_codes, idx->N, lut, Q, kSubset, target_ids, target_offsets, lin_rows, topk, ids,
                     dist, topk, qmode, 0, stage_ws, st);
  } else if (!has_lists || idx->N < idx->theta) {
    rc = launch_scan(idx, idx->d_codes, idx->N, lut, Q, kLinear, nullptr, nullptr, idx->N, topk, ids, dist, topk,
                     qmode, 0, stage_ws, st);
  }
  if (rc) return rc;
  // inverted-index branch (mode 1); the scratch of the scan stage is reused in stream order
  if (has_lists) {
    rc = coarse_rank(idx, lut, Q, pmax, probe, nullptr, pmax, qmode, 1, stage_ws, st);
    if (rc) return rc;
    rc = launch_ivf(idx, lut, Q, probe, pmax, pmax, nprobe_q, target_ids, target_offsets, L, topk, ids, dist, qmode,
                    1, ivf_b ? stage_ws : nullptr, st);
    if (rc) return rc;
  }
  RII_HIP(hipGetLastError());
  return RII_OK;
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

// a(n) by brute force.  rot_base >= 0: `codes` are stored rows rot_base .. rot_base+n-1 (rotated
// storage when rot_m(M)); rot_base < 0: plain codes.
int rii_internal_assign(const rii_index* idx, const uint8_t* codes, int64_t n, int64_t rot_base, const uint8_t* coarse,
                        int K, int32_t* assign_out, hipStream_t st) {
  if (!m_supported(idx->M)) return RII_ERR_UNSUPPORTED;
  if (n == 0) return RII_OK;
  if (!rot_m(idx->M)) rot_base = -1;
  int rc = rii_internal_sym_table(idx, st);
  if (rc) return rc;
  const int M = idx->M;
  const size_t lds = (size_t)M * 1024;
  int blocks = (int)std::min<int64_t>(n, 256 * 16);
  DISPATCH_M(M, { int rc2 = set_lds(k_assign<MT>, lds); if (rc2) return rc2;
                  k_assign<MT><<<blocks, 256, lds, st>>>(idx->d_sym, codes, n, rot_base, M, coarse, K, assign_out); });
  RII_HIP(hipGetLastError());
  return RII_OK;
}

int rii_assign(const rii_index_t* idx, const uint8_t* codes, int64_t n, const uint8_t* coarse, int K,
               int32_t* assign_out, void* stream) {
  if (!idx || n < 0 || K < 1 || !coarse || (n > 0 && (!codes || !assign_out))) return RII_ERR_INVALID_ARG;
  return rii_internal_assign(idx, codes, n, -1, coarse, K, assign_out, static_cast<hipStream_t>(stream));
}

// a(n) with pruning (see k_assign_pruned); all pointers device.  visited_total may be NULL.
int rii_internal_assign_pruned(const rii_index* idx, const uint8_t* codes, int64_t n, int64_t rot_base,
                               const uint8_t* super, int G,
                               const float* radius, const uint8_t* coarse_g, const int32_t* perm_g,
                               const int32_t* group_off, int32_t* assign_out, unsigned long long* visited_total,
                               hipStream_t st) {
  if (n == 0) return RII_OK;
  if (!rot_m(idx->M)) rot_base = -1;
  int rc = rii_internal_sym_table(idx, st);
  if (rc) return rc;
  const int M = idx->M;
  const size_t lds = (size_t)M * 1024 + (size_t)G * 4;
  if (lds > 150 * 1024) return RII_ERR_UNSUPPORTED;
  int blocks = (int)std::min<int64_t>(n, 256 * 32);
  DISPATCH_M(M, { int rc2 = set_lds(k_assign_pruned<MT>, lds); if (rc2) return rc2;
                  k_assign_pruned<MT><<<blocks, 256, lds, st>>>(idx->d_sym, codes, n, rot_base, M, super, G, radius, coarse_g,
                                                               perm_g, group_off, assign_out, visited_total); });
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

// used by rii_index.hip: see k_copy_rows.  The rotation arguments are ignored (plain) unless rot_m(M).
int rii_internal_copy_rows(const uint8_t* in, int64_t in_rot, const int32_t* ids, int64_t n, int M, uint8_t* out,
                           int64_t out_rot, hipStream_t st) {
  if (n == 0) return RII_OK;
  if (!rot_m(M)) in_rot = out_rot = -1;
  const int M4 = M / 4;
  const int64_t per = ((int64_t)1 << 30) / M4;  // rows per launch
  for (int64_t r0 = 0; r0 < n; r0 += per) {
    int64_t cnt = std::min<int64_t>(per, n - r0);
    int64_t dw = cnt * M4;
    // rows r0.. of this call: shift the rotation bases and (when not gathering) the source pointer
    k_copy_rows<<<(unsigned)((dw + 255) / 256), 256, 0, st>>>(ids ? in : in + r0 * M,
                                                           in_rot >= 0 && !ids ? in_rot + r0 : in_rot,
                                                           ids ? ids + r0 : nullptr, cnt, M, out + r0 * M,
                                                           out_rot >= 0 ? out_rot + r0 : out_rot);
  }
  RII_HIP(hipGetLastError());
  return RII_OK;
}

}  // extern "C"
