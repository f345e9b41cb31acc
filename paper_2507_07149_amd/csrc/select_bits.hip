// Width selection on the device by rank quantiles of the per-group range.
//
// The benchmark workloads assign widths by ranking the groups by (range, group index),
// range = max - min in binary32, and splitting the ranking into C equal parts: rank r gets
// classes[floor(r*C/G)].  This stands in for the paper's controller (Sec. 3.4.1 chooses widths
// from per-activation importance under memory/time budgets); doing it on the device lets the
// sequence statistics -> widths -> plan -> quantize run without the host touching the data.
//
// No sort is needed.  class(g) = number of thresholds k in 1..C-1 with rank(g) >= R_k,
// R_k = ceil(k*G/C).  For each k a radix select (three passes of histograms over the keys, digits
// of 11, 11 and 10 bits, most significant first) finds T_k, the key at sorted position R_k, and
// E_k, how many keys equal to T_k precede that position.  Then rank(g) >= R_k  iff  key_g > T_k,
// or key_g == T_k and g >= I_k, where I_k is the index of the E_k-th (counting from zero) group
// whose key equals T_k.  Keys are the bit patterns of the ranges, which order like the ranges
// because a range is never negative.
//
// Six launches: zero the counters; write the keys and count their first digit; count the second
// digit; count the third; count the keys equal to T_k per block of 4096 groups and find I_k;
// classify.  What used to be a launch of one workgroup after each counting pass (pick the bin
// that holds the rank, scan the per-block tie counts) is done by the workgroup that finishes
// last, found with a ticket counter.  Everything that crosses workgroups inside a launch goes
// through device-scope atomics (adds, stores, loads), so no cache write-back is needed; what a
// later launch reads is written with ordinary stores.
#include "daf_device.h"
#include "daf_internal.h"

namespace {

using namespace daf;

constexpr int kThreads = 512;
constexpr int kItems = 8;                        // consecutive groups per thread in the ordered passes
constexpr int kBlockGroups = kThreads * kItems;  // 4096
constexpr int kMaxThresholds = 3;                // C <= 4
constexpr int kHistCopies = 2;
constexpr int kBins = 2048;                      // the widest digit has 11 bits
constexpr int kBinsPerThread = kBins / kThreads; // 4
constexpr int kPasses = 3;
constexpr int kLaunchesWithTicket = 4;           // three counting passes and the tie count
constexpr int kTicketLanes = 16;
constexpr unsigned kMaxWorkgroups = 384;         // of the counting launches, see daf_launch_select_bits
static_assert(kBins % kThreads == 0 && kBinsPerThread % 2 == 0, "a thread reads its bins in 8-byte pieces");
constexpr int kLdsCopies0 = 8;                   // copies of a workgroup's own histogram, first pass (one histogram)
constexpr int kLdsCopies = 2;                    // later passes (one histogram per threshold)

__host__ __device__ constexpr int pass_shift(int pass) { return pass == 0 ? 21 : pass == 1 ? 10 : 0; }
__host__ __device__ constexpr int pass_bits(int pass) { return pass == 2 ? 10 : 11; }

struct SelectState {
  uint32_t prefix[kMaxThresholds];      // digits of T_k decided so far
  uint32_t rank[kMaxThresholds];        // rank still to be located inside the prefix bucket; E_k at the end
  uint32_t tie_index[kMaxThresholds];   // I_k
  // Workgroups of a launch that have finished (all zero between launches), in two levels:
  // [1 + r] counts the workgroups whose index is r modulo kTicketLanes, [0] the residues that are
  // complete.  Atomics to one address are served one after the other, about 8 ns each; a single
  // counter drawn by 1024 workgroups that finish together costs as much as a small launch.
  uint32_t ticket[kLaunchesWithTicket][1 + kTicketLanes];
  uint32_t pad[3];
  // kHistCopies copies of the histograms, a workgroup adds to copy (its index mod kHistCopies):
  // atomics to one address are served one after the other at the memory side (about 8 ns each),
  // and with few distinct digits every workgroup hits the same few counters.  One copy is
  // 3 x 2048 counters: the workgroup that picks the bins reads all copies, so there are few.
  uint32_t hist[kHistCopies][kMaxThresholds][kBins];
};
static_assert(offsetof(SelectState, hist) % 16 == 0, "the counters are read and cleared in 8- and 16-byte pieces");

// Ranks to locate, empty prefixes, zeroed counters and tickets.
__global__ __launch_bounds__(kThreads) void k_select_init(SelectState* __restrict__ st, uint32_t r0, uint32_t r1,
                                                          uint32_t r2) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    st->prefix[0] = st->prefix[1] = st->prefix[2] = 0u;
    st->rank[0] = r0;
    st->rank[1] = r1;
    st->rank[2] = r2;
    st->tie_index[0] = st->tie_index[1] = st->tie_index[2] = 0u;
    for (int i = 0; i < kLaunchesWithTicket * (1 + kTicketLanes); ++i) (&st->ticket[0][0])[i] = 0u;
  }
  uint4* h = reinterpret_cast<uint4*>(&st->hist[0][0][0]);
  constexpr int kPieces = kHistCopies * kMaxThresholds * kBins / 4;
  for (int i = blockIdx.x * kThreads + threadIdx.x; i < kPieces; i += gridDim.x * kThreads)
    h[i] = make_uint4(0u, 0u, 0u, 0u);
}

// A workgroup's own histogram in LDS holds COPIES counters per bin, side by side, and a lane adds
// to copy (lane mod COPIES).  The digits of a wave are often few (the leading digit of a range is
// its sign and most of its exponent; ranges of 16-bit tensors have few mantissa bits), and LDS
// atomics of one instruction to one address are served one after the other: the copies divide
// that queue, at no cost in instructions.  (Counting equal digits with ballots first, and adding
// once per distinct digit, took some 40 scalar and vector instructions per call, which was more
// than the queue it avoided.)
template <int COPIES>
__device__ __forceinline__ void hist_add(uint32_t* h, uint32_t digit, bool active) {
  if (active) atomicAdd(&h[digit * COPIES + (threadIdx.x & (COPIES - 1))], 1u);
}
template <int COPIES>
__device__ __forceinline__ uint32_t hist_count(const uint32_t* h, int bin) {
  uint32_t c = 0u;
#pragma unroll
  for (int j = 0; j < COPIES; ++j) c += h[bin * COPIES + j];
  return c;
}

// Exclusive prefix sum of one value per thread over the kThreads threads of a workgroup, and the
// workgroup's total: a DPP scan inside each wave, the wave totals through LDS (two barriers).
__device__ __forceinline__ uint32_t block_exclusive_sum(uint32_t v, uint32_t* wave_tot, uint32_t* total) {
  constexpr int kWaves = kThreads / kWave;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  const uint32_t incl = wave_inclusive_sum(v);
  __syncthreads();                                       // wave_tot may still be read from an earlier call
  if (lane == kWave - 1) wave_tot[wave] = incl;
  __syncthreads();
  uint32_t before = 0u, all = 0u;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const uint32_t t = wave_tot[w];
    before += (w < wave) ? t : 0u;
    all += t;
  }
  *total = all;
  return before + incl - v;
}

// Device-scope accesses for what one workgroup writes and another reads inside a launch.
__device__ __forceinline__ uint64_t coherent_load(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t coherent_load(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void coherent_store(uint32_t* p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// True in every thread of the workgroup that finishes a launch last.  Each thread first waits for
// its own atomics and stores to be acknowledged, so when the last ticket is drawn every
// workgroup's contributions are in place.  The caller zeroes ticket[0] when it is done.
__device__ __forceinline__ bool last_workgroup(uint32_t* ticket, uint32_t* flag) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t r = blockIdx.x % kTicketLanes;
    const uint32_t with_r = (gridDim.x - r + kTicketLanes - 1) / kTicketLanes;
    const uint32_t residues = gridDim.x < (unsigned)kTicketLanes ? gridDim.x : (unsigned)kTicketLanes;
    uint32_t last = 0u;
    if (__hip_atomic_fetch_add(&ticket[1 + r], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == with_r - 1) {
      coherent_store(&ticket[1 + r], 0u);
      last = (__hip_atomic_fetch_add(&ticket[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == residues - 1) ? 1u : 0u;
    }
    *flag = last;
  }
  __syncthreads();
  asm volatile("" ::: "memory");
  return *flag != 0u;
}

// Thresholds whose prefixes are equal so far select inside the same bucket: they share one
// histogram, that of the first of them.
struct Slices {
  int of[kMaxThresholds];
};
__device__ __forceinline__ Slices shared_slices(const uint32_t (&prefix)[kMaxThresholds], int pass) {
  Slices s;
  s.of[0] = 0;
  s.of[1] = (pass == 0 || prefix[1] == prefix[0]) ? 0 : 1;
  s.of[2] = (pass == 0 || prefix[2] == prefix[0]) ? 0 : (prefix[2] == prefix[1]) ? s.of[1] : 2;
  return s;
}

// The end of a counting pass, run by every workgroup after it has added its counts: the one that
// finishes last sums the copies, finds for each threshold the bin whose cumulative count first
// exceeds the rank, extends the prefix by that digit, and leaves counters and ticket zeroed.
template <int PASS>
__device__ __forceinline__ void finish_pass(SelectState* __restrict__ st, int n_thresholds,
                                            const uint32_t (&prefix)[kMaxThresholds], const Slices& slices,
                                            uint32_t* wave_tot, uint32_t* flag) {
  if (!last_workgroup(st->ticket[PASS], flag)) return;
  uint32_t rank[kMaxThresholds];
  for (int k = 0; k < kMaxThresholds; ++k) rank[k] = st->rank[k];
  // The counters come from memory past the caches, a few microseconds per trip: the loads of all
  // histograms in use are issued before any of them is needed.
  uint64_t raw[kMaxThresholds][kHistCopies][kBinsPerThread / 2];
#pragma unroll
  for (int k = 0; k < kMaxThresholds; ++k) {
    const bool used = k < n_thresholds && slices.of[k] == k;
#pragma unroll
    for (int c = 0; c < kHistCopies; ++c) {
      const uint64_t* src = reinterpret_cast<const uint64_t*>(&st->hist[c][k][threadIdx.x * kBinsPerThread]);
#pragma unroll
      for (int i = 0; i < kBinsPerThread / 2; ++i) raw[k][c][i] = used ? coherent_load(src + i) : 0ull;
    }
  }
  uint32_t hs[kMaxThresholds][kBinsPerThread];
#pragma unroll
  for (int k = 0; k < kMaxThresholds; ++k) {
#pragma unroll
    for (int i = 0; i < kBinsPerThread / 2; ++i) {
      uint32_t lo = 0u, hi = 0u;
#pragma unroll
      for (int c = 0; c < kHistCopies; ++c) {
        lo += (uint32_t)raw[k][c][i];
        hi += (uint32_t)(raw[k][c][i] >> 32);
      }
      hs[k][2 * i] = lo;
      hs[k][2 * i + 1] = hi;
    }
  }
#pragma unroll
  for (int k = 0; k < kMaxThresholds; ++k) {
    if (k >= n_thresholds) break;
    uint32_t h[kBinsPerThread];
    uint32_t sum = 0u;
#pragma unroll
    for (int i = 0; i < kBinsPerThread; ++i) {
      h[i] = slices.of[k] == 0 ? hs[0][i] : slices.of[k] == 1 ? hs[1][i] : hs[2][i];
      sum += h[i];
    }
    uint32_t total;
    uint32_t run = block_exclusive_sum(sum, wave_tot, &total);
#pragma unroll
    for (int i = 0; i < kBinsPerThread; ++i) {
      if (run <= rank[k] && rank[k] < run + h[i]) {       // exactly one bin (ranks are < G)
        st->prefix[k] = prefix[k] | ((uint32_t)(threadIdx.x * kBinsPerThread + i) << pass_shift(PASS));
        st->rank[k] = rank[k] - run;
      }
      run += h[i];
    }
  }
  __syncthreads();                                        // every thread has its counts
  uint4* h4 = reinterpret_cast<uint4*>(&st->hist[0][0][0]);
  constexpr int kPieces = kHistCopies * kMaxThresholds * kBins / 4;
  for (int i = threadIdx.x; i < kPieces; i += kThreads) h4[i] = make_uint4(0u, 0u, 0u, 0u);
  if (threadIdx.x == 0) coherent_store(&st->ticket[PASS][0], 0u);
}

// keys[g] = bit pattern of the group's range, and in the same pass the histogram of the keys'
// leading digit (every key counts for every threshold, so one histogram serves all).  A wave
// takes 512 consecutive groups per trip, eight loads of each array in flight per lane.
// FROM_SCALE = false: the range is gmax - gmin.  FROM_SCALE = true: gmin holds the groups' scales of
// an earlier quantize call and prev_bits (or, when null, prev_uniform) the widths it ran with; the
// range is scale * (2^b - 1), Eq. 1 (left) turned round, in binary32.
template <bool FROM_SCALE>
__global__ __launch_bounds__(kThreads) void k_select_keys(const float* __restrict__ gmin, const float* __restrict__ gmax,
                                                          const uint8_t* __restrict__ prev_bits, uint32_t prev_uniform,
                                                          int64_t G, uint32_t* __restrict__ keys,
                                                          SelectState* __restrict__ st, int n_thresholds) {
  constexpr int kLoads = 8;
  __shared__ uint32_t lh[kBins * kLdsCopies0];
  __shared__ uint32_t wave_tot[kThreads / kWave];
  __shared__ uint32_t flag;
  for (int i = threadIdx.x; i < kBins * kLdsCopies0; i += kThreads) lh[i] = 0u;
  __syncthreads();
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t wave_stride = (int64_t)gridDim.x * (kThreads / kWave) * (kWave * kLoads);
  const int64_t first = ((int64_t)blockIdx.x * (kThreads / kWave) + (threadIdx.x >> 6)) * (kWave * kLoads);
  for (int64_t g0 = first; g0 < G; g0 += wave_stride) {
    float lo[kLoads], hi[kLoads];
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
      const int64_t g = g0 + j * kWave + lane;
      lo[j] = (g < G) ? gmin[g] : 0.0f;
      if (FROM_SCALE) {
        const uint32_t b = (prev_bits != nullptr && g < G) ? (uint32_t)prev_bits[g] : prev_uniform;
        hi[j] = (float)((1u << (b & 15u)) - 1u);          // L of the earlier call
      } else {
        hi[j] = (g < G) ? gmax[g] : 0.0f;
      }
    }
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
      const int64_t g = g0 + j * kWave + lane;
      const uint32_t key = f2u(FROM_SCALE ? lo[j] * hi[j] : hi[j] - lo[j]);
      if (g < G) keys[g] = key;
      hist_add<kLdsCopies0>(lh, key >> pass_shift(0), g < G);
    }
  }
  __syncthreads();
  if (n_thresholds > 0) {
    for (int i = threadIdx.x; i < kBins; i += kThreads) {
      const uint32_t c = hist_count<kLdsCopies0>(lh, i);
      if (c) atomicAdd(&st->hist[blockIdx.x % kHistCopies][0][i], c);
    }
  }
  const uint32_t prefix[kMaxThresholds] = {0u, 0u, 0u};
  finish_pass<0>(st, n_thresholds, prefix, shared_slices(prefix, 0), wave_tot, &flag);
}

// Histogram of the PASS-th digit among the keys whose higher digits equal the prefix.
template <int PASS>
__global__ __launch_bounds__(kThreads) void k_select_hist(const uint32_t* __restrict__ keys, int64_t G,
                                                          SelectState* __restrict__ st, int n_thresholds) {
  constexpr int kShift = pass_shift(PASS), kDigitBins = 1 << pass_bits(PASS);
  __shared__ uint32_t lh[kMaxThresholds][kBins * kLdsCopies];
  __shared__ uint32_t wave_tot[kThreads / kWave];
  __shared__ uint32_t flag;
  for (int i = threadIdx.x; i < kMaxThresholds * kBins * kLdsCopies; i += kThreads) (&lh[0][0])[i] = 0u;
  __syncthreads();
  uint32_t prefix[kMaxThresholds];
  for (int k = 0; k < kMaxThresholds; ++k) prefix[k] = st->prefix[k];
  const Slices slices = shared_slices(prefix, PASS);
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  // Sixteen keys per lane and trip: four 16-byte loads issued together (the key array is padded
  // to whole chunks), so that enough bytes are in flight; a wave takes 256 consecutive chunks.
  constexpr int kLoads = 4;
  const int64_t n_chunks = (G + 3) >> 2;
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t wave_stride = stride / kWave * (kWave * kLoads);
  const int64_t first = ((int64_t)blockIdx.x * (kThreads / kWave) + (threadIdx.x >> 6)) * (kWave * kLoads);
  for (int64_t c0 = first; c0 < n_chunks; c0 += wave_stride) {
    uint4 v[kLoads];
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
      const int64_t c = c0 + j * kWave + lane;
      v[j] = make_uint4(0u, 0u, 0u, 0u);
      if (c < n_chunks) v[j] = reinterpret_cast<const uint4*>(keys)[c];
    }
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
      const int64_t c = c0 + j * kWave + lane;
      const uint32_t key4[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool in = c * 4 + e < G;
        const uint32_t key = key4[e];
        const uint32_t digit = (key >> kShift) & (uint32_t)(kDigitBins - 1);
#pragma unroll
        for (int k = 0; k < kMaxThresholds; ++k) {
          if (k >= n_thresholds || slices.of[k] != k) continue;   // counted with an earlier threshold
          hist_add<kLdsCopies>(lh[k], digit, in && (((key ^ prefix[k]) >> (kShift + pass_bits(PASS))) == 0u));
        }
      }
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < n_thresholds * kBins; i += kThreads) {
    const int k = i / kBins;
    const uint32_t c = hist_count<kLdsCopies>(lh[k], i % kBins);
    if (c && slices.of[k] == k) atomicAdd(&(&st->hist[blockIdx.x % kHistCopies][0][0])[i], c);
  }
  finish_pass<PASS>(st, n_thresholds, prefix, slices, wave_tot, &flag);
}

// A thread's kItems consecutive keys: two 16-byte loads (the key array is padded to a multiple
// of four entries and 16-byte aligned, and a thread's first index is a multiple of eight);
// entries at or past G read as 0xFFFFFFFF.
__device__ __forceinline__ void load_keys(const uint32_t* __restrict__ keys, int64_t base, int64_t G,
                                          uint32_t (&key)[kItems]) {
  static_assert(kItems == 8, "two uint4 loads");
  const int64_t padded = (G + 3) & ~(int64_t)3;
  uint4 a = make_uint4(~0u, ~0u, ~0u, ~0u), b = a;
  if (base < padded) a = *reinterpret_cast<const uint4*>(keys + base);
  if (base + 4 < padded) b = *reinterpret_cast<const uint4*>(keys + base + 4);
  key[0] = a.x; key[1] = a.y; key[2] = a.z; key[3] = a.w;
  key[4] = b.x; key[5] = b.y; key[6] = b.z; key[7] = b.w;
#pragma unroll
  for (int i = 0; i < kItems; ++i)
    if (base + i >= G) key[i] = 0xFFFFFFFFu;
}

// Per block of 4096 consecutive groups: how many keys equal each threshold.  The workgroup that
// finishes last then finds, for every threshold with E_k > 0, the block in which the running
// count of equal keys passes E_k, and inside that block the group I_k itself.
__global__ __launch_bounds__(kThreads) void k_select_ties(const uint32_t* __restrict__ keys, int64_t G,
                                                          SelectState* __restrict__ st, int n_thresholds,
                                                          uint32_t* __restrict__ block_ties, int64_t n_blocks) {
  __shared__ uint32_t cnt[kMaxThresholds];
  __shared__ uint32_t wave_tot[kThreads / kWave];
  __shared__ uint32_t flag;
  __shared__ uint32_t found[kMaxThresholds][2];          // block that holds I_k, equal keys still to skip in it
  if (threadIdx.x < 2 * kMaxThresholds) (&found[0][0])[threadIdx.x] = 0u;
  uint32_t T[kMaxThresholds], E[kMaxThresholds];
  for (int k = 0; k < kMaxThresholds; ++k) {
    T[k] = st->prefix[k];
    E[k] = st->rank[k];
  }
  const int64_t ties_stride = (n_blocks + 3) & ~(int64_t)3;      // per threshold; keeps 8-byte loads aligned
  // A workgroup takes every gridDim.x-th block: few workgroups, because each draws a ticket at
  // the end and tickets are served one after the other.
  for (int64_t b = blockIdx.x; b < n_blocks; b += gridDim.x) {
    if (threadIdx.x < kMaxThresholds) cnt[threadIdx.x] = 0u;
    __syncthreads();
    const int64_t base = b * kBlockGroups + (int64_t)threadIdx.x * kItems;
    uint32_t c[kMaxThresholds] = {0u, 0u, 0u};
    uint32_t key[kItems];
    load_keys(keys, base, G, key);
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
      if (base + i < G) {
        for (int k = 0; k < n_thresholds; ++k) c[k] += (key[i] == T[k]) ? 1u : 0u;
      }
    }
    for (int k = 0; k < n_thresholds; ++k)
      if (c[k]) atomicAdd(&cnt[k], c[k]);
    __syncthreads();
    if (threadIdx.x < (unsigned)n_thresholds)
      coherent_store(&block_ties[(int64_t)threadIdx.x * ties_stride + b], cnt[threadIdx.x]);
    __syncthreads();
  }
  if (!last_workgroup(st->ticket[kPasses], &flag)) return;

  // Running count of equal keys over the blocks, 4096 blocks per trip (eight consecutive counts
  // per thread, all thresholds' loads issued together), until the block that holds I_k is found.
  bool wanted[kMaxThresholds];
  uint32_t carry[kMaxThresholds];
#pragma unroll
  for (int k = 0; k < kMaxThresholds; ++k) {
    wanted[k] = k < n_thresholds && E[k] != 0u;           // E_k = 0: every equal key counts, I_k = 0
    carry[k] = 0u;
  }
  for (int64_t t0 = 0; t0 < n_blocks; t0 += kBlockGroups) {
    const int64_t i0 = t0 + (int64_t)threadIdx.x * kItems;
    uint64_t raw[kMaxThresholds][kItems / 2];
#pragma unroll
    for (int k = 0; k < kMaxThresholds; ++k) {
      const uint64_t* src = reinterpret_cast<const uint64_t*>(block_ties + (int64_t)k * ties_stride + i0);
#pragma unroll
      for (int j = 0; j < kItems / 2; ++j)
        raw[k][j] = (wanted[k] && i0 + 2 * j < n_blocks) ? coherent_load(src + j) : 0ull;
    }
#pragma unroll
    for (int k = 0; k < kMaxThresholds; ++k) {
      if (!wanted[k]) continue;
      uint32_t v[kItems];
      uint32_t sum = 0u;
#pragma unroll
      for (int j = 0; j < kItems; ++j) {
        const uint32_t e = (j & 1) ? (uint32_t)(raw[k][j / 2] >> 32) : (uint32_t)raw[k][j / 2];
        v[j] = (i0 + j < n_blocks) ? e : 0u;              // the padding of the array holds no counts
        sum += v[j];
      }
      uint32_t total;
      uint32_t run = carry[k] + block_exclusive_sum(sum, wave_tot, &total);
      if (run <= E[k] && E[k] < run + sum) {              // at most one thread over all trips (E_k < number of equal keys)
#pragma unroll
        for (int j = 0; j < kItems; ++j) {
          if (run <= E[k] && E[k] < run + v[j]) {
            found[k][0] = (uint32_t)(i0 + j);
            found[k][1] = E[k] - run;
          }
          run += v[j];
        }
      }
      carry[k] += total;
    }
  }
  __syncthreads();
  // Inside the found blocks: the thread whose keys hold the wanted equal key writes its index.
  uint32_t fkey[kMaxThresholds][kItems];
  int64_t fbase[kMaxThresholds];
#pragma unroll
  for (int k = 0; k < kMaxThresholds; ++k) {
    fbase[k] = (int64_t)found[k][0] * kBlockGroups + (int64_t)threadIdx.x * kItems;
    if (wanted[k]) load_keys(keys, fbase[k], G, fkey[k]);
  }
#pragma unroll
  for (int k = 0; k < kMaxThresholds; ++k) {
    if (!wanted[k]) continue;
    const uint32_t skip = found[k][1];
    uint32_t mine = 0u;
#pragma unroll
    for (int i = 0; i < kItems; ++i) mine += (fbase[k] + i < G && fkey[k][i] == T[k]) ? 1u : 0u;
    uint32_t total;
    uint32_t before = block_exclusive_sum(mine, wave_tot, &total);
    if (before <= skip && skip < before + mine) {
#pragma unroll
      for (int i = 0; i < kItems; ++i) {
        if (fbase[k] + i < G && fkey[k][i] == T[k]) {
          if (before == skip) st->tie_index[k] = (uint32_t)(fbase[k] + i);
          ++before;
        }
      }
    }
  }
  if (threadIdx.x == 0) coherent_store(&st->ticket[kPasses][0], 0u);
}

__global__ __launch_bounds__(kThreads) void k_select_classify(const uint32_t* __restrict__ keys, int64_t G,
                                                              const SelectState* __restrict__ st, int n_thresholds,
                                                              uint32_t classes_packed, uint8_t* __restrict__ out_bits) {
  const int64_t base = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * kItems;
  uint32_t T[kMaxThresholds], I[kMaxThresholds];
  for (int k = 0; k < kMaxThresholds; ++k) {
    T[k] = st->prefix[k];
    I[k] = st->tie_index[k];
  }
  uint32_t key[kItems];
  load_keys(keys, base, G, key);
  uint8_t w[kItems];
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const uint32_t g = (uint32_t)(base + i);
    uint32_t cls = 0;
    for (int k = 0; k < n_thresholds; ++k)
      if (key[i] > T[k] || (key[i] == T[k] && g >= I[k])) ++cls;
    w[i] = (uint8_t)(classes_packed >> (8u * cls));
  }
  if (base + kItems <= G && (reinterpret_cast<uintptr_t>(out_bits) & 7u) == 0u) {
    const uint2 v = make_uint2((uint32_t)w[0] | ((uint32_t)w[1] << 8) | ((uint32_t)w[2] << 16) | ((uint32_t)w[3] << 24),
                               (uint32_t)w[4] | ((uint32_t)w[5] << 8) | ((uint32_t)w[6] << 16) | ((uint32_t)w[7] << 24));
    *reinterpret_cast<uint2*>(out_bits + base) = v;       // eight widths in one store
  } else {
#pragma unroll
    for (int i = 0; i < kItems; ++i)
      if (base + i < G) out_bits[base + i] = w[i];
  }
}

}  // namespace

int64_t daf_select_bits_workspace_size(int64_t G) {
  const int64_t n_blocks = (G + kBlockGroups - 1) / kBlockGroups;
  return (int64_t)sizeof(SelectState) + ((G + 3) / 4) * 16 + kMaxThresholds * ((n_blocks + 3) / 4) * 16 + 64;
}

hipError_t daf_launch_select_bits(const float* gmin, const float* gmax, const uint8_t* prev_bits, int32_t prev_uniform,
                                  int64_t G, const uint8_t* classes, int n_classes, uint8_t* out_bits, void* workspace,
                                  hipStream_t stream) {
  SelectState* st = static_cast<SelectState*>(workspace);
  uint32_t* keys = reinterpret_cast<uint32_t*>(static_cast<char*>(workspace) + ((sizeof(SelectState) + 15) / 16) * 16);
  uint32_t* block_ties = keys + ((G + 3) / 4) * 4;
  const int64_t n_blocks = (G + kBlockGroups - 1) / kBlockGroups;

  // thresholds R_k = ceil(k*G/C) that some rank can reach (R_k < G); the rest never apply
  uint32_t R[kMaxThresholds] = {0u, 0u, 0u};
  int n_thr = 0;
  for (int k = 1; k < n_classes; ++k) {
    const int64_t r = (k * G + n_classes - 1) / n_classes;
    if (r < G) R[n_thr++] = (uint32_t)r;
  }
  uint32_t packed = 0;
  for (int c = 0; c < n_classes; ++c) packed |= (uint32_t)classes[c] << (8 * c);
  // thresholds skipped because R_k >= G sit at the end (R_k grows with k), so class = number of
  // satisfied thresholds still indexes `classes` correctly.

  // The counting launches take at most kMaxWorkgroups workgroups of 8 waves: each adds its non-zero
  // counts to the shared counters and draws a ticket, and both are served one after the other per
  // address (5.6 M groups: 82 us for the whole selection with 384 workgroups of 512 threads, 84 with
  // 256, 90 with 1024; 94 to 125 with workgroups of 256 threads).
  const unsigned cap = kMaxWorkgroups;
  hipLaunchKernelGGL(k_select_init, dim3(24), dim3(kThreads), 0, stream, st, R[0], R[1], R[2]);
  const unsigned kblocks = (unsigned)((G + 8 * kThreads - 1) / (8 * kThreads));                  // eight keys per thread and trip
  if (gmax != nullptr)
    hipLaunchKernelGGL(k_select_keys<false>, dim3(kblocks < cap ? kblocks : cap), dim3(kThreads), 0, stream, gmin, gmax,
                       nullptr, 0u, G, keys, st, n_thr);
  else
    hipLaunchKernelGGL(k_select_keys<true>, dim3(kblocks < cap ? kblocks : cap), dim3(kThreads), 0, stream, gmin, nullptr,
                       prev_bits, (uint32_t)prev_uniform, G, keys, st, n_thr);
  if (n_thr > 0) {
    const unsigned cblocks = (unsigned)((((G + 3) >> 2) + 4 * kThreads - 1) / (4 * kThreads));   // sixteen keys per thread and trip
    const unsigned hblocks = cblocks < cap ? cblocks : cap;
    hipLaunchKernelGGL(k_select_hist<1>, dim3(hblocks), dim3(kThreads), 0, stream, keys, G, st, n_thr);
    hipLaunchKernelGGL(k_select_hist<2>, dim3(hblocks), dim3(kThreads), 0, stream, keys, G, st, n_thr);
    hipLaunchKernelGGL(k_select_ties, dim3((unsigned)(n_blocks < cap ? n_blocks : cap)), dim3(kThreads), 0, stream, keys,
                       G, st, n_thr, block_ties, n_blocks);
  }
  hipLaunchKernelGGL(k_select_classify, dim3((unsigned)n_blocks), dim3(kThreads), 0, stream, keys, G, st, n_thr, packed,
                     out_bits);
  return hipGetLastError();
}
