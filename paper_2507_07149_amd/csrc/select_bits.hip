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

struct SelectState {
  uint32_t prefix[kMaxThresholds];      // digits of T_k decided so far
  uint32_t rank[kMaxThresholds];        // rank still to be located inside the prefix bucket; E_k at the end
  uint32_t hist[kMaxThresholds][256];
};

__global__ __launch_bounds__(kThreads) void k_select_keys(const float* __restrict__ gmin, const float* __restrict__ gmax,
                                                          int64_t G, uint32_t* __restrict__ keys,
                                                          SelectState* __restrict__ st, uint32_t r0, uint32_t r1,
                                                          uint32_t r2) {
  const int64_t g = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (g < G) keys[g] = f2u(gmax[g] - gmin[g]);
  if (g == 0) {
    st->prefix[0] = st->prefix[1] = st->prefix[2] = 0u;
    st->rank[0] = r0;
    st->rank[1] = r1;
    st->rank[2] = r2;
  }
  if (blockIdx.x == 0) {
    for (int i = threadIdx.x; i < kMaxThresholds * 256; i += kThreads) (&st->hist[0][0])[i] = 0u;
  }
}

// Histogram of the digit at `shift` among the keys whose higher digits equal the prefix.
__global__ __launch_bounds__(kThreads) void k_select_hist(const uint32_t* __restrict__ keys, int64_t G,
                                                          SelectState* __restrict__ st, int n_thresholds, int shift) {
  __shared__ uint32_t lh[kMaxThresholds][256];
  for (int i = threadIdx.x; i < kMaxThresholds * 256; i += kThreads) (&lh[0][0])[i] = 0u;
  __syncthreads();
  uint32_t prefix[kMaxThresholds];
  for (int k = 0; k < kMaxThresholds; ++k) prefix[k] = st->prefix[k];
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t g = (int64_t)blockIdx.x * kThreads + threadIdx.x; g < G; g += stride) {
    const uint32_t key = keys[g];
    const uint32_t digit = (key >> shift) & 0xFFu;
    for (int k = 0; k < n_thresholds; ++k) {
      const bool match = (shift == 24) || (((key ^ prefix[k]) >> (shift + 8)) == 0u);
      if (match) atomicAdd(&lh[k][digit], 1u);
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < n_thresholds * 256; i += kThreads) {
    const uint32_t c = (&lh[0][0])[i];
    if (c) atomicAdd(&(&st->hist[0][0])[i], c);
  }
}

// One workgroup: per threshold, the bin whose cumulative count first exceeds the rank.
__global__ __launch_bounds__(256) void k_select_pick(SelectState* __restrict__ st, int n_thresholds, int shift) {
  __shared__ uint32_t cum[256];
  for (int k = 0; k < n_thresholds; ++k) {
    const uint32_t h = st->hist[k][threadIdx.x];
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
    st->hist[k][threadIdx.x] = 0u;                       // ready for the next pass
    __syncthreads();
  }
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
  for (int i = 0; i < kItems; ++i) {
    const int64_t g = base + i;
    if (g < G) {
      const uint32_t key = keys[g];
      for (int k = 0; k < n_thresholds; ++k) c[k] += (key == st->prefix[k]) ? 1u : 0u;
    }
  }
  for (int k = 0; k < n_thresholds; ++k)
    if (c[k]) atomicAdd(&cnt[k], c[k]);
  __syncthreads();
  if (threadIdx.x < (unsigned)n_thresholds) block_ties[(int64_t)threadIdx.x * gridDim.x + blockIdx.x] = cnt[threadIdx.x];
}

// One workgroup: exclusive scan of the per-block tie counts, per threshold, in place.
__global__ __launch_bounds__(kThreads) void k_select_tie_scan(uint32_t* __restrict__ block_ties, int64_t n_blocks,
                                                              int n_thresholds) {
  __shared__ uint32_t lds[kThreads];
  for (int k = 0; k < n_thresholds; ++k) {
    uint32_t* t = block_ties + (int64_t)k * n_blocks;
    uint32_t carry = 0;
    for (int64_t c = 0; c < n_blocks; c += kThreads) {
      const int64_t i = c + threadIdx.x;
      const uint32_t v = (i < n_blocks) ? t[i] : 0u;
      lds[threadIdx.x] = v;
      __syncthreads();
      uint32_t acc = v;
      for (int o = 1; o < kThreads; o <<= 1) {
        const uint32_t add = (threadIdx.x >= (unsigned)o) ? lds[threadIdx.x - o] : 0u;
        __syncthreads();
        acc += add;
        lds[threadIdx.x] = acc;
        __syncthreads();
      }
      if (i < n_blocks) t[i] = carry + acc - v;
      carry += lds[kThreads - 1];
      __syncthreads();
    }
  }
}

__global__ __launch_bounds__(kThreads) void k_select_classify(const uint32_t* __restrict__ keys, int64_t G,
                                                              const SelectState* __restrict__ st, int n_thresholds,
                                                              const uint32_t* __restrict__ block_ties,
                                                              uint32_t classes_packed, uint8_t* __restrict__ out_bits) {
  __shared__ uint32_t lds[kMaxThresholds][kThreads];
  const int64_t base = (int64_t)blockIdx.x * kBlockGroups + (int64_t)threadIdx.x * kItems;
  uint32_t T[kMaxThresholds], E[kMaxThresholds];
  for (int k = 0; k < kMaxThresholds; ++k) {
    T[k] = st->prefix[k];
    E[k] = st->rank[k];
  }
  uint32_t key[kItems];
  uint32_t mine[kMaxThresholds] = {0u, 0u, 0u};          // equal keys among this thread's groups
  for (int i = 0; i < kItems; ++i) {
    const int64_t g = base + i;
    key[i] = (g < G) ? keys[g] : 0xFFFFFFFFu;
    for (int k = 0; k < n_thresholds; ++k) mine[k] += (g < G && key[i] == T[k]) ? 1u : 0u;
  }
  // exclusive prefix of `mine` over the threads of the block, per threshold
  uint32_t before[kMaxThresholds];
  for (int k = 0; k < n_thresholds; ++k) lds[k][threadIdx.x] = mine[k];
  __syncthreads();
  for (int k = 0; k < n_thresholds; ++k) {
    uint32_t acc = mine[k];
    for (int o = 1; o < kThreads; o <<= 1) {
      const uint32_t add = (threadIdx.x >= (unsigned)o) ? lds[k][threadIdx.x - o] : 0u;
      __syncthreads();
      acc += add;
      lds[k][threadIdx.x] = acc;
      __syncthreads();
    }
    before[k] = block_ties[(int64_t)k * gridDim.x + blockIdx.x] + acc - mine[k];
  }
  for (int i = 0; i < kItems; ++i) {
    const int64_t g = base + i;
    if (g >= G) break;
    uint32_t cls = 0;
    for (int k = 0; k < n_thresholds; ++k) {
      const bool eq = key[i] == T[k];
      if (key[i] > T[k] || (eq && before[k] >= E[k])) ++cls;
      before[k] += eq ? 1u : 0u;
    }
    out_bits[g] = (uint8_t)(classes_packed >> (8u * cls));
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

  const unsigned gblocks = (unsigned)((G + kThreads - 1) / kThreads);
  hipLaunchKernelGGL(k_select_keys, dim3(gblocks), dim3(kThreads), 0, stream, gmin, gmax, G, keys, st, R[0], R[1], R[2]);
  if (n_thr > 0) {
    unsigned hblocks = gblocks < 1024u ? gblocks : 1024u;
    for (int shift = 24; shift >= 0; shift -= 8) {
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
