// Device exclusive prefix scan of per-group packed word counts.
//
// The packed buffer concatenates the groups' codes (paper Sec. 3.3 speaks of packing the
// compressed values together); with a bit width per group the position of group g is the
// sum of the word counts of all groups before it.  Three small kernels: per-block sums, a
// single-block scan of those sums, and a per-block rescan that writes the offsets.
#include "daf_device.h"
#include "daf_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kItems = 8;                          // consecutive groups per thread
constexpr int kBlockGroups = kThreads * kItems;    // 2048

__device__ __forceinline__ uint32_t group_words(uint32_t b, int64_t g, int64_t num_groups, int64_t n,
                                                int32_t gs, int* bad) {
  const bool ok = (b == 1u) | (b == 2u) | (b == 4u) | (b == 8u);
  if (!ok) { *bad = 1; return 0u; }
  const int64_t len = (g == num_groups - 1) ? (n - g * (int64_t)gs) : (int64_t)gs;
  return (uint32_t)((len * b + 31) >> 5);
}

// Sum over a block; result valid in thread 0.
__device__ __forceinline__ unsigned long long block_sum(unsigned long long v, unsigned long long* lds) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) lds[wave] = v;
  __syncthreads();
  return lds[0] + lds[1] + lds[2] + lds[3];
}

__global__ __launch_bounds__(kThreads) void k_plan_block_sums(const uint8_t* __restrict__ bits,
                                                              int64_t num_groups, int64_t n, int32_t gs,
                                                              unsigned long long* __restrict__ block_sums,
                                                              int* __restrict__ bad_flag) {
  __shared__ unsigned long long lds[4];
  const int64_t base = (int64_t)blockIdx.x * kBlockGroups + (int64_t)threadIdx.x * kItems;
  unsigned long long s = 0;
  int bad = 0;
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const int64_t g = base + i;
    if (g < num_groups) s += group_words(bits[g], g, num_groups, n, gs, &bad);
  }
  if (bad) atomicOr(bad_flag, 1);
  const unsigned long long tot = block_sum(s, lds);
  if (threadIdx.x == 0) block_sums[blockIdx.x] = tot;
}

// One block turns block_sums[] into exclusive offsets in place and writes the grand total.
__global__ __launch_bounds__(kThreads) void k_plan_scan_block_sums(unsigned long long* __restrict__ block_sums,
                                                                   int64_t n_blocks,
                                                                   unsigned long long* __restrict__ total) {
  __shared__ unsigned long long lds[kThreads];
  unsigned long long carry = 0;
  for (int64_t c = 0; c < n_blocks; c += kThreads) {
    const int64_t i = c + threadIdx.x;
    const unsigned long long v = (i < n_blocks) ? block_sums[i] : 0ull;
    lds[threadIdx.x] = v;
    __syncthreads();
    // Hillis-Steele inclusive scan over the 256 entries
    unsigned long long acc = v;
    for (int o = 1; o < kThreads; o <<= 1) {
      const unsigned long long add = (threadIdx.x >= (unsigned)o) ? lds[threadIdx.x - o] : 0ull;
      __syncthreads();
      acc += add;
      lds[threadIdx.x] = acc;
      __syncthreads();
    }
    if (i < n_blocks) block_sums[i] = carry + acc - v;
    carry += lds[kThreads - 1];
    __syncthreads();
  }
  if (threadIdx.x == 0) *total = carry;
}

__global__ __launch_bounds__(kThreads) void k_plan_write_offsets(const uint8_t* __restrict__ bits,
                                                                 int64_t num_groups, int64_t n, int32_t gs,
                                                                 const unsigned long long* __restrict__ block_off,
                                                                 uint32_t* __restrict__ off) {
  __shared__ unsigned long long lds[kThreads];
  const int64_t base = (int64_t)blockIdx.x * kBlockGroups + (int64_t)threadIdx.x * kItems;
  uint32_t w[kItems];
  unsigned long long s = 0;
  int bad = 0;
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const int64_t g = base + i;
    w[i] = (g < num_groups) ? group_words(bits[g], g, num_groups, n, gs, &bad) : 0u;
    s += w[i];
  }
  lds[threadIdx.x] = s;
  __syncthreads();
  unsigned long long acc = s;
  for (int o = 1; o < kThreads; o <<= 1) {
    const unsigned long long add = (threadIdx.x >= (unsigned)o) ? lds[threadIdx.x - o] : 0ull;
    __syncthreads();
    acc += add;
    lds[threadIdx.x] = acc;
    __syncthreads();
  }
  unsigned long long run = block_off[blockIdx.x] + acc - s;   // exclusive offset of this thread's first group
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const int64_t g = base + i;
    if (g < num_groups) off[g] = (uint32_t)run;
    run += w[i];
  }
}

}  // namespace

int64_t daf_plan_scan_blocks(int64_t num_groups) { return (num_groups + kBlockGroups - 1) / kBlockGroups; }

hipError_t daf_launch_plan_scan(const uint8_t* d_bits, int64_t num_groups, int64_t n, int32_t group_size,
                                uint32_t* d_off, unsigned long long* d_block_sums, int64_t n_blocks,
                                unsigned long long* d_total, int* d_bad, hipStream_t stream) {
  hipLaunchKernelGGL(k_plan_block_sums, dim3((unsigned)n_blocks), dim3(kThreads), 0, stream, d_bits,
                     num_groups, n, group_size, d_block_sums, d_bad);
  hipLaunchKernelGGL(k_plan_scan_block_sums, dim3(1), dim3(kThreads), 0, stream, d_block_sums, n_blocks,
                     d_total);
  hipLaunchKernelGGL(k_plan_write_offsets, dim3((unsigned)n_blocks), dim3(kThreads), 0, stream, d_bits,
                     num_groups, n, group_size, d_block_sums, d_off);
  return hipGetLastError();
}
