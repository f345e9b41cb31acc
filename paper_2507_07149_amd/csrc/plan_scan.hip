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

// A thread's kItems consecutive widths: one 8-byte load when all of them exist and the array
// is 8-byte aligned (a thread's first index is a multiple of eight), else byte by byte; entries
// at or past num_groups read as 0.
__device__ __forceinline__ void load_widths(const uint8_t* __restrict__ bits, int64_t base, int64_t num_groups,
                                            uint32_t (&b)[kItems]) {
  static_assert(kItems == 8, "one 8-byte load");
  if (base + kItems <= num_groups && (reinterpret_cast<uintptr_t>(bits) & 7u) == 0u) {
    const uint2 v = *reinterpret_cast<const uint2*>(bits + base);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      b[i] = (v.x >> (8 * i)) & 0xFFu;
      b[4 + i] = (v.y >> (8 * i)) & 0xFFu;
    }
  } else {
#pragma unroll
    for (int i = 0; i < kItems; ++i) b[i] = (base + i < num_groups) ? (uint32_t)bits[base + i] : 0u;
  }
}

// Sum over a block; result valid in thread 0.
__device__ __forceinline__ unsigned long long block_sum(unsigned long long v, unsigned long long* lds) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) lds[wave] = v;
  __syncthreads();
  return lds[0] + lds[1] + lds[2] + lds[3];
}

// Widths outside {1,2,4,8} are replaced by 8 in the plan's copy (so that every kernel that reads
// the copy stays inside its buffers whatever the caller passed) and reported: bit 63 of the
// block's sum carries "this block saw an invalid width".
constexpr unsigned long long kBadBit = 1ull << 63;

__global__ __launch_bounds__(kThreads) void k_plan_block_sums(const uint8_t* __restrict__ src_bits,
                                                              uint8_t* __restrict__ plan_bits,
                                                              int64_t num_groups, int64_t n, int32_t gs,
                                                              unsigned long long* __restrict__ block_sums) {
  __shared__ unsigned long long lds[4];
  const int64_t base = (int64_t)blockIdx.x * kBlockGroups + (int64_t)threadIdx.x * kItems;
  unsigned long long s = 0;
  int bad = 0;
  uint32_t b[kItems];
  load_widths(src_bits, base, num_groups, b);
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const int64_t g = base + i;
    if (g < num_groups) {
      int bad_here = 0;
      (void)group_words(b[i], g, num_groups, n, gs, &bad_here);
      if (bad_here) { b[i] = 8u; bad = 1; }
      s += group_words(b[i], g, num_groups, n, gs, &bad_here);
    }
  }
  if (base + kItems <= num_groups && (reinterpret_cast<uintptr_t>(plan_bits) & 7u) == 0u) {
    uint2 v;
    v.x = b[0] | (b[1] << 8) | (b[2] << 16) | (b[3] << 24);
    v.y = b[4] | (b[5] << 8) | (b[6] << 16) | (b[7] << 24);
    *reinterpret_cast<uint2*>(plan_bits + base) = v;
  } else {
#pragma unroll
    for (int i = 0; i < kItems; ++i)
      if (base + i < num_groups) plan_bits[base + i] = (uint8_t)b[i];
  }
  const int any_bad = __syncthreads_or(bad);
  const unsigned long long tot = block_sum(s, lds);      // far below 2^63
  if (threadIdx.x == 0) block_sums[blockIdx.x] = tot | (any_bad ? kBadBit : 0ull);
}

// One block turns block_sums[] into exclusive offsets in place and writes the grand total: a
// thread sums a run of consecutive entries, the 256 run sums are scanned once, the run is
// rewritten.
__global__ __launch_bounds__(kThreads) void k_plan_scan_block_sums(unsigned long long* __restrict__ block_sums,
                                                                   int64_t n_blocks,
                                                                   unsigned long long* __restrict__ total,
                                                                   int* __restrict__ bad_flag) {
  __shared__ unsigned long long lds[kThreads];
  const int64_t per = (n_blocks + kThreads - 1) / kThreads;
  const int64_t lo = (int64_t)threadIdx.x * per;
  const int64_t hi = lo + per < n_blocks ? lo + per : n_blocks;
  unsigned long long sum = 0;
  int bad = 0;
  for (int64_t i = lo; i < hi; ++i) {
    const unsigned long long v = block_sums[i];
    bad |= (v & kBadBit) ? 1 : 0;
    block_sums[i] = v & ~kBadBit;
    sum += v & ~kBadBit;
  }
  const int any_bad = __syncthreads_or(bad);
  if (threadIdx.x == 0) *bad_flag = any_bad;
  lds[threadIdx.x] = sum;
  __syncthreads();
  unsigned long long acc = sum;                          // Hillis-Steele inclusive scan over the 256 run sums
  for (int o = 1; o < kThreads; o <<= 1) {
    const unsigned long long add = (threadIdx.x >= (unsigned)o) ? lds[threadIdx.x - o] : 0ull;
    __syncthreads();
    acc += add;
    lds[threadIdx.x] = acc;
    __syncthreads();
  }
  unsigned long long run = acc - sum;
  for (int64_t i = lo; i < hi; ++i) {
    const unsigned long long v = block_sums[i];
    block_sums[i] = run;
    run += v;
  }
  if (threadIdx.x == kThreads - 1) *total = acc;
}

// Offsets are kept modulo 2^32 (a plan whose total reaches 2^32 words is rejected from the 64-bit
// total, and its offsets are never used), so the scan inside a block runs on 32-bit values: a
// DPP scan inside each wave, the wave totals through LDS.
__global__ __launch_bounds__(kThreads) void k_plan_write_offsets(const uint8_t* __restrict__ bits,
                                                                 int64_t num_groups, int64_t n, int32_t gs,
                                                                 const unsigned long long* __restrict__ block_off,
                                                                 uint32_t* __restrict__ off) {
  __shared__ uint32_t wave_tot[kThreads / daf::kWave];
  const int64_t base = (int64_t)blockIdx.x * kBlockGroups + (int64_t)threadIdx.x * kItems;
  uint32_t b[kItems], w[kItems];
  load_widths(bits, base, num_groups, b);
  uint32_t s = 0;
  int bad = 0;
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const int64_t g = base + i;
    w[i] = (g < num_groups) ? group_words(b[i], g, num_groups, n, gs, &bad) : 0u;
    s += w[i];
  }
  const int lane = threadIdx.x & (daf::kWave - 1), wave = threadIdx.x >> 6;
  const uint32_t incl = daf::wave_inclusive_sum(s);
  if (lane == daf::kWave - 1) wave_tot[wave] = incl;
  __syncthreads();
  uint32_t before = 0u;
#pragma unroll
  for (int v = 0; v < kThreads / daf::kWave; ++v) before += (v < wave) ? wave_tot[v] : 0u;
  uint32_t run = (uint32_t)block_off[blockIdx.x] + before + incl - s;   // offset of this thread's first group
  uint32_t o[kItems];
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    o[i] = run;
    run += w[i];
  }
  if (base + kItems <= num_groups) {                     // two 16-byte stores
    *reinterpret_cast<uint4*>(off + base) = make_uint4(o[0], o[1], o[2], o[3]);
    *reinterpret_cast<uint4*>(off + base + 4) = make_uint4(o[4], o[5], o[6], o[7]);
  } else {
#pragma unroll
    for (int i = 0; i < kItems; ++i)
      if (base + i < num_groups) off[base + i] = o[i];
  }
}

}  // namespace

int64_t daf_plan_scan_blocks(int64_t num_groups) { return (num_groups + kBlockGroups - 1) / kBlockGroups; }

hipError_t daf_launch_plan_scan(const uint8_t* src_bits, uint8_t* plan_bits, int64_t num_groups, int64_t n,
                                int32_t group_size, uint32_t* d_off, unsigned long long* d_block_sums, int64_t n_blocks,
                                unsigned long long* d_total, int* d_bad, hipStream_t stream) {
  hipLaunchKernelGGL(k_plan_block_sums, dim3((unsigned)n_blocks), dim3(kThreads), 0, stream, src_bits, plan_bits,
                     num_groups, n, group_size, d_block_sums);
  hipLaunchKernelGGL(k_plan_scan_block_sums, dim3(1), dim3(kThreads), 0, stream, d_block_sums, n_blocks,
                     d_total, d_bad);
  hipLaunchKernelGGL(k_plan_write_offsets, dim3((unsigned)n_blocks), dim3(kThreads), 0, stream, plan_bits,
                     num_groups, n, group_size, d_block_sums, d_off);
  return hipGetLastError();
}
