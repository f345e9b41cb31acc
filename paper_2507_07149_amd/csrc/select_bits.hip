// Width selection on the device by rank quantiles of the per-group range.
//
// The benchmark workloads assign widths by ranking the groups by (range, group index),
// range = max - min in binary32, and splitting the ranking into C equal parts: rank r gets
// classes[floor(r*C/G)].  This stands in for the paper's controller (Sec. 3.4.1 chooses widths
// from per-activation importance under memory/time budgets); doing it on the device lets the
// sequence statistics -> widths -> plan -> quantize run without the host touching the data.
//
// No sort is needed.  class(g) = number of thresholds k in 1..C-1 with rank(g) >= R_k,
// R_k = ceil(k*G/C).  For each k a radix select (four passes of 8-bit histograms over the keys,
// most significant digit first) finds T_k, the key at sorted position R_k, and E_k, how many
// keys equal to T_k precede that position.  Then rank(g) >= R_k  iff  key_g > T_k, or
// key_g == T_k and (number of h < g with key_h == T_k) >= E_k; the count of earlier equal keys
// comes from a block-wise prefix count.  Keys are the bit patterns of the ranges, which order
// like the ranges because a range is never negative.
#include "daf_device.h"
#include "daf_internal.h"

namespace {

using namespace daf;

constexpr int kThreads = 256;
constexpr int kItems = 8;                        // consecutive groups per thread in the ordered passes
constexpr int kBlockGroups = kThreads * kItems;  // 2048
constexpr int kMaxThresholds = 3;                // C <= 4
constexpr int kHistCopies = 16;

struct SelectState {
  uint32_t prefix[kMaxThresholds];      // digits of T_k decided so far
  uint32_t rank[kMaxThresholds];        // rank still to be located inside the prefix bucket; E_k at the end
  // kHistCopies copies of the histograms, a workgroup adds to copy (its index mod kHistCopies):
  // atomics to one address are served one after the other at the memory side (about 8 ns each),
  // and with few distinct digits every workgroup hits the same few counters.
  uint32_t hist[kHistCopies][kMaxThresholds][256];
};

// One workgroup: ranks to locate, empty prefixes, zeroed counters.
__global__ __launch_bounds__(kThreads) void k_select_init(SelectState* __restrict__ st, uint32_t r0, uint32_t r1,
                                                          uint32_t r2) {
  if (threadIdx.x == 0) {
    st->prefix[0] = st->prefix[1] = st->prefix[2] = 0u;
    st->rank[0] = r0;
    st->rank[1] = r1;
    st->rank[2] = r2;
  }
  for (int i = threadIdx.x; i < kHistCopies * kMaxThresholds * 256; i += kThreads) (&st->hist[0][0][0])[i] = 0u;
}

// Adds one count per active lane to h[digit].  The digits of a wave are often few (the leading
// digit of a range is its sign and most of its exponent), and LDS atomics of one instruction to
// one address are served one after the other: the three most frequent leaders' digits are
// counted with a ballot and added once, whatever is left goes one lane at a time.
__device__ __forceinline__ void wave_hist_add(uint32_t* h, uint32_t digit, bool active) {
  const int lane = threadIdx.x & (kWave - 1);
  uint64_t todo = __builtin_amdgcn_ballot_w64(active);
  for (int round = 0; round < 3 && todo != 0ull; ++round) {
    const int leader = __builtin_ctzll(todo);
    const uint32_t d = (uint32_t)__builtin_amdgcn_readlane((int)digit, leader);
    const uint64_t same = __builtin_amdgcn_ballot_w64(active && digit == d) & todo;
    if (__builtin_popcountll(same) < 4) break;           // spread-out digits: plain atomics are cheaper
    if (lane == leader) atomicAdd(&h[d], (uint32_t)__builtin_popcountll(same));
    todo &= ~same;
  }
  if ((todo >> lane) & 1ull) atomicAdd(&h[digit], 1u);
}

// keys[g] = bit pattern of the group's range, and in the same pass the histogram of the keys'
// leading digit (the first of the four passes: every key counts for every threshold, so one
// histogram is added to the counters of all of them).  A wave takes 512 consecutive groups per trip,
// eight loads of each array in flight per lane.
__global__ __launch_bounds__(kThreads) void k_select_keys(const float* __restrict__ gmin, const float* __restrict__ gmax,
                                                          int64_t G, uint32_t* __restrict__ keys,
                                                          SelectState* __restrict__ st, int n_thresholds) {
  constexpr int kLoads = 8;
  __shared__ uint32_t lh[256];
  for (int i = threadIdx.x; i < 256; i += kThreads) lh[i] = 0u;
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
      hi[j] = (g < G) ? gmax[g] : 0.0f;
    }
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
      const int64_t g = g0 + j * kWave + lane;
      const uint32_t key = f2u(hi[j] - lo[j]);
      if (g < G) keys[g] = key;
      wave_hist_add(lh, key >> 24, g < G);
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < n_thresholds * 256; i += kThreads) {
    const uint32_t c = lh[i & 255];
    if (c) atomicAdd(&(&st->hist[blockIdx.x % kHistCopies][0][0])[i], c);
  }
}

// Histogram of the digit at `shift` among the keys whose higher digits equal the prefix.  In
// the first pass (shift 24) every key counts for every threshold: one histogram serves all.
__global__ __launch_bounds__(kThreads) void k_select_hist(const uint32_t* __restrict__ keys, int64_t G,
                                                          SelectState* __restrict__ st, int n_thresholds, int shift) {
  __shared__ uint32_t lh[kMaxThresholds][256];
  for (int i = threadIdx.x; i < kMaxThresholds * 256; i += kThreads) (&lh[0][0])[i] = 0u;
  __syncthreads();
  uint32_t prefix[kMaxThresholds];
  for (int k = 0; k < kMaxThresholds; ++k) prefix[k] = st->prefix[k];
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  // every lane of a wave makes the same number of trips (the ballots need whole waves); lanes
  // past the end take part with nothing to add
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
        const uint32_t digit = (key >> shift) & 0xFFu;
        if (shift == 24) {
          wave_hist_add(lh[0], digit, in);
        } else {
          for (int k = 0; k < n_thresholds; ++k)
            wave_hist_add(lh[k], digit, in && (((key ^ prefix[k]) >> (shift + 8)) == 0u));
        }
      }
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < n_thresholds * 256; i += kThreads) {
    const uint32_t c = (shift == 24) ? lh[0][i & 255] : (&lh[0][0])[i];
    if (c) atomicAdd(&(&st->hist[blockIdx.x % kHistCopies][0][0])[i], c);
  }
}

// One workgroup: per threshold, the bin whose cumulative count first exceeds the rank.
__global__ __launch_bounds__(256) void k_select_pick(SelectState* __restrict__ st, int n_thresholds, int shift) {
  __shared__ uint32_t cum[256];
  for (int k = 0; k < n_thresholds; ++k) {
    uint32_t h = 0u;
    for (int r = 0; r < kHistCopies; ++r) {
      h += st->hist[r][k][threadIdx.x];
      st->hist[r][k][threadIdx.x] = 0u;                  // ready for the next pass
    }
    cum[threadIdx.x] = h;
    __syncthreads();
    uint32_t acc = h;                                    // inclusive scan over the 256 bins
    for (int o = 1; o < 256; o <<= 1) {
      const uint32_t add = (threadIdx.x >= (unsigned)o) ? cum[threadIdx.x - o] : 0u;
      __syncthreads();
      acc += add;
      cum[threadIdx.x] = acc;
      __syncthreads();
    }
    const uint32_t rank = st->rank[k];
    const uint32_t before = acc - h;
    __syncthreads();
    if (before <= rank && rank < acc) {                  // exactly one bin (ranks are < G)
      st->prefix[k] |= (uint32_t)threadIdx.x << shift;
      st->rank[k] = rank - before;
    }
    __syncthreads();
  }
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

// Per block of 2048 consecutive groups: how many keys equal each threshold.
__global__ __launch_bounds__(kThreads) void k_select_tie_count(const uint32_t* __restrict__ keys, int64_t G,
                                                               const SelectState* __restrict__ st, int n_thresholds,
                                                               uint32_t* __restrict__ block_ties) {
  __shared__ uint32_t cnt[kMaxThresholds];
  if (threadIdx.x < kMaxThresholds) cnt[threadIdx.x] = 0u;
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * kBlockGroups + (int64_t)threadIdx.x * kItems;
  uint32_t c[kMaxThresholds] = {0u, 0u, 0u};
  uint32_t key[kItems];
  load_keys(keys, base, G, key);
  uint32_t T[kMaxThresholds];
  for (int k = 0; k < kMaxThresholds; ++k) T[k] = st->prefix[k];
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    if (base + i < G) {
      for (int k = 0; k < n_thresholds; ++k) c[k] += (key[i] == T[k]) ? 1u : 0u;
    }
  }
  for (int k = 0; k < n_thresholds; ++k)
    if (c[k]) atomicAdd(&cnt[k], c[k]);
  __syncthreads();
  if (threadIdx.x < (unsigned)n_thresholds) block_ties[(int64_t)threadIdx.x * gridDim.x + blockIdx.x] = cnt[threadIdx.x];
}

// One workgroup: exclusive scan of the per-block tie counts, per threshold, in place.  A thread
// takes a run of consecutive entries, the runs' sums are scanned across the workgroup.
__global__ __launch_bounds__(kThreads) void k_select_tie_scan(uint32_t* __restrict__ block_ties, int64_t n_blocks,
                                                              int n_thresholds) {
  __shared__ uint32_t wave_tot[kThreads / kWave];
  const int64_t per = (n_blocks + kThreads - 1) / kThreads;
  const int64_t lo = (int64_t)threadIdx.x * per;
  const int64_t hi = lo + per < n_blocks ? lo + per : n_blocks;
  for (int k = 0; k < n_thresholds; ++k) {
    uint32_t* t = block_ties + (int64_t)k * n_blocks;
    uint32_t sum = 0u;
    for (int64_t i = lo; i < hi; ++i) sum += t[i];
    uint32_t total;
    uint32_t run = block_exclusive_sum(sum, wave_tot, &total);
    for (int64_t i = lo; i < hi; ++i) {
      const uint32_t v = t[i];
      t[i] = run;
      run += v;
    }
  }
}

__global__ __launch_bounds__(kThreads) void k_select_classify(const uint32_t* __restrict__ keys, int64_t G,
                                                              const SelectState* __restrict__ st, int n_thresholds,
                                                              const uint32_t* __restrict__ block_ties,
                                                              uint32_t classes_packed, uint8_t* __restrict__ out_bits) {
  __shared__ uint32_t wave_tot[kThreads / kWave];
  const int64_t base = (int64_t)blockIdx.x * kBlockGroups + (int64_t)threadIdx.x * kItems;
  uint32_t T[kMaxThresholds], E[kMaxThresholds];
  for (int k = 0; k < kMaxThresholds; ++k) {
    T[k] = st->prefix[k];
    E[k] = st->rank[k];
  }
  uint32_t key[kItems];
  uint32_t mine[kMaxThresholds] = {0u, 0u, 0u};          // equal keys among this thread's groups
  load_keys(keys, base, G, key);
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const int64_t g = base + i;
    for (int k = 0; k < n_thresholds; ++k) mine[k] += (g < G && key[i] == T[k]) ? 1u : 0u;
  }
  // exclusive prefix of `mine` over the threads of the block, per threshold
  uint32_t before[kMaxThresholds];
  for (int k = 0; k < n_thresholds; ++k) {
    uint32_t total;
    before[k] = block_ties[(int64_t)k * gridDim.x + blockIdx.x] + block_exclusive_sum(mine[k], wave_tot, &total);
  }
  uint8_t w[kItems];
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    uint32_t cls = 0;
    for (int k = 0; k < n_thresholds; ++k) {
      const bool eq = key[i] == T[k];
      if (key[i] > T[k] || (eq && before[k] >= E[k])) ++cls;
      before[k] += eq ? 1u : 0u;
    }
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
  return (int64_t)sizeof(SelectState) + ((G + 3) / 4) * 16 + kMaxThresholds * n_blocks * 4 + 64;
}

hipError_t daf_launch_select_bits(const float* gmin, const float* gmax, int64_t G, const uint8_t* classes,
                                  int n_classes, uint8_t* out_bits, void* workspace, hipStream_t stream) {
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

  hipLaunchKernelGGL(k_select_init, dim3(1), dim3(kThreads), 0, stream, st, R[0], R[1], R[2]);
  const unsigned kblocks = (unsigned)((G + 8 * kThreads - 1) / (8 * kThreads));                  // eight keys per thread and trip
  hipLaunchKernelGGL(k_select_keys, dim3(kblocks < 1024u ? kblocks : 1024u), dim3(kThreads), 0, stream, gmin, gmax, G,
                     keys, st, n_thr);
  if (n_thr > 0) {
    const unsigned cblocks = (unsigned)((((G + 3) >> 2) + 4 * kThreads - 1) / (4 * kThreads));   // sixteen keys per thread and trip
    const unsigned hblocks = cblocks < 1024u ? cblocks : 1024u;
    for (int shift = 24; shift >= 0; shift -= 8) {
      if (shift != 24)                 // the leading digit was counted while the keys were written
        hipLaunchKernelGGL(k_select_hist, dim3(hblocks), dim3(kThreads), 0, stream, keys, G, st, n_thr, shift);
      hipLaunchKernelGGL(k_select_pick, dim3(1), dim3(256), 0, stream, st, n_thr, shift);
    }
    hipLaunchKernelGGL(k_select_tie_count, dim3((unsigned)n_blocks), dim3(kThreads), 0, stream, keys, G, st, n_thr,
                       block_ties);
    hipLaunchKernelGGL(k_select_tie_scan, dim3(1), dim3(kThreads), 0, stream, block_ties, n_blocks, n_thr);
  }
  hipLaunchKernelGGL(k_select_classify, dim3((unsigned)n_blocks), dim3(kThreads), 0, stream, keys, G, st, n_thr,
                     block_ties, packed, out_bits);
  return hipGetLastError();
}
