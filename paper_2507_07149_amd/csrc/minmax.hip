// Whole-tensor minimum and maximum: the collective reduction of the paper's Sec. 3.2, in the
// two forms it describes.
//
//   two-pass   every workgroup reduces its share (registers -> wave -> LDS) and writes one
//              (min, max) pair to memory; a second, single-workgroup launch reduces the pairs
//              (the paper's "parallel reduction": block results go through DRAM and another
//              kernel is launched).
//   atomic     the same in-workgroup tree, but the workgroup then merges its pair straight into
//              one shared (min, max) in memory with a float atomic minimum/maximum built from
//              integer compare-and-swap (Algorithm 1), so no second launch is needed (the
//              paper's hybrid: tree inside a block, atomics across blocks).  A ticket counter
//              lets the last workgroup publish the result and re-arm the workspace.
//
// Differences from Algorithm 1 as printed: the loop is left as soon as the stored value is
// already <= the candidate (no compare-and-swap is issued for a value that cannot change the
// result), which removes nearly all contention on a GPU with ~2000 resident workgroups: the
// running minimum changes O(log n) times over a kernel.
#include "daf_device.h"
#include "daf_internal.h"

namespace {

using namespace daf;

constexpr int kThreads = 256;
// 16-byte chunks in flight per thread and iteration, and the largest grid, per method (measured
// on a 51 M-element tensor: two-pass 39.6 us with 4 chunks and 2048 workgroups, 34.7 us with 8
// and 1024; the atomic form serialises on its one result, so it takes one workgroup per compute
// unit with more loads in flight each: 166 us with 4 and 2048, 42.6 us with 16 and 256).
constexpr int kUnroll = 8;
constexpr int kMaxBlocks = 1024;
constexpr int kUnrollAtomic = 16;
constexpr int kMaxBlocksAtomic = 256;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct MinMaxWorkspace {          // layout of the caller's workspace
  float cur_min, cur_max;         // atomic method: running result (+inf, -inf when idle)
  unsigned ticket;                // atomic method: workgroups finished (0 when idle)
  unsigned pad;
  float2 partial[kMaxBlocks];     // two-pass method: one pair per workgroup
};

// Float atomic minimum / maximum in the manner of Algorithm 1: the value lives in memory as its
// bit pattern and is replaced with an integer compare-and-swap, retried while another workgroup
// got in between.  The loop is left as soon as the stored value is already at least as good as the
// candidate, so no swap is issued for a value that cannot change the result.
template <bool IS_MIN>
__device__ __forceinline__ void atomic_extremum(float* target, float candidate) {
  unsigned* bits = reinterpret_cast<unsigned*>(target);
  unsigned seen = __atomic_load_n(bits, __ATOMIC_RELAXED);
  while (IS_MIN ? candidate < u2f(seen) : candidate > u2f(seen)) {
    // on failure `seen` receives the value found, and the test above runs again on it
    if (__atomic_compare_exchange_n(bits, &seen, f2u(candidate), false, __ATOMIC_RELAXED, __ATOMIC_RELAXED)) break;
  }
}

// (min, max) of a workgroup's values; valid in thread 0.
__device__ __forceinline__ void block_minmax(float& mn, float& mx, float& mn2, float& mx2, float2* lds) {
  seg_minmax_x2<6>(mn, mx, mn2, mx2);           // complete in lane 63 of every wave
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  if (lane == kWave - 1) lds[wave] = make_float2(vmin(mn, mn2), vmax(mx, mx2));
  __syncthreads();
  if (threadIdx.x == 0) {
    mn = lds[0].x;
    mx = lds[0].y;
    for (int w = 1; w < kThreads / kWave; ++w) {
      mn = vmin(mn, lds[w].x);
      mx = vmax(mx, lds[w].y);
    }
  }
}

template <int DT>
__device__ __forceinline__ void chunk_minmax(const u32x4 v, float& mn, float& mx) {
  const uint4 raw = make_uint4(v.x, v.y, v.z, v.w);
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  float f[kEpl];
#pragma unroll
  for (int e = 0; e < kEpl; ++e) f[e] = chunk_elem<DT>(raw, e);
  if (kEpl == 4) {
    mn = vmin3(mn, vmin3(f[0], f[1], f[2]), f[3]);
    mx = vmax3(mx, vmax3(f[0], f[1], f[2]), f[3]);
  } else {
    mn = vmin3(vmin3(mn, f[0], f[1]), vmin3(f[2], f[3], f[4 % kEpl]), vmin3(f[5 % kEpl], f[6 % kEpl], f[7 % kEpl]));
    mx = vmax3(vmax3(mx, f[0], f[1]), vmax3(f[2], f[3], f[4 % kEpl]), vmax3(f[5 % kEpl], f[6 % kEpl], f[7 % kEpl]));
  }
}

template <int DT, bool ATOMIC>
__global__ __launch_bounds__(kThreads) void k_minmax(const void* __restrict__ x, int64_t n,
                                                     MinMaxWorkspace* __restrict__ ws,
                                                     float* __restrict__ out_minmax) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  constexpr int kU = ATOMIC ? kUnrollAtomic : kUnroll;
  __shared__ float2 lds[kThreads / kWave];
  const u32x4* chunks = static_cast<const u32x4*>(x);
  const int64_t n_chunks = n / kEpl;
  const float first = (DT == kF32) ? static_cast<const float*>(x)[0]
                                   : widen16<DT == kF32 ? kF16 : DT>(static_cast<const uint16_t*>(x)[0]);
  float mn = first, mx = first, mn2 = first, mx2 = first;      // element 0 is a safe identity

  const int64_t stride = (int64_t)gridDim.x * kThreads;
  int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  for (; c + (kU - 1) * stride < n_chunks; c += kU * stride) {
    u32x4 v[kU];
#pragma unroll
    for (int k = 0; k < kU; ++k) v[k] = __builtin_nontemporal_load(&chunks[c + k * stride]);
#pragma unroll
    for (int k = 0; k < kU; k += 2) {
      chunk_minmax<DT>(v[k], mn, mx);
      chunk_minmax<DT>(v[k + 1], mn2, mx2);
    }
  }
  for (; c < n_chunks; c += stride) chunk_minmax<DT>(__builtin_nontemporal_load(&chunks[c]), mn, mx);
  if (blockIdx.x == 0 && threadIdx.x == 0) {                    // the < kEpl elements after the last chunk
    for (int64_t i = n_chunks * kEpl; i < n; ++i) {
      const float v = (DT == kF32) ? static_cast<const float*>(x)[i]
                                   : widen16<DT == kF32 ? kF16 : DT>(static_cast<const uint16_t*>(x)[i]);
      mn = vmin(mn, v);
      mx = vmax(mx, v);
    }
  }
  block_minmax(mn, mx, mn2, mx2, lds);
  if (threadIdx.x != 0) return;

  if (!ATOMIC) {
    ws->partial[blockIdx.x] = make_float2(mn, mx);
    return;
  }
  // All communication between workgroups goes through device-scope atomics on the workspace,
  // which execute at the memory side in the order this thread issues them once each has
  // returned: the compare-and-swap loops above consume their return values, and the wait
  // below covers the path that only loaded.  No plain load or store is shared, so no cache
  // write-back/invalidate (which a full fence would add, per workgroup) is needed; measured,
  // such fences made this kernel 5x slower on 2048 workgroups.
  atomic_extremum<true>(&ws->cur_min, mn);
  atomic_extremum<false>(&ws->cur_max, mx);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  const unsigned ticket = atomicAdd(&ws->ticket, 1u);
  if (ticket == gridDim.x - 1) {                                // every workgroup has merged its pair
    const float rmin = u2f(atomicExch(reinterpret_cast<unsigned*>(&ws->cur_min), 0x7F800000u));   // re-arm: +inf
    const float rmax = u2f(atomicExch(reinterpret_cast<unsigned*>(&ws->cur_max), 0xFF800000u));   // re-arm: -inf
    atomicExch(&ws->ticket, 0u);
    out_minmax[0] = rmin + 0.0f;                                // a zero result is +0
    out_minmax[1] = rmax + 0.0f;
  }
}

__global__ __launch_bounds__(kThreads) void k_minmax_final(const MinMaxWorkspace* __restrict__ ws, int n_partials,
                                                           float* __restrict__ out_minmax) {
  __shared__ float2 lds[kThreads / kWave];
  float mn = ws->partial[0].x, mx = ws->partial[0].y, mn2 = mn, mx2 = mx;
  for (int i = threadIdx.x; i < n_partials; i += kThreads) {
    const float2 p = ws->partial[i];
    mn = vmin(mn, p.x);
    mx = vmax(mx, p.y);
  }
  block_minmax(mn, mx, mn2, mx2, lds);
  if (threadIdx.x == 0) {
    out_minmax[0] = mn + 0.0f;
    out_minmax[1] = mx + 0.0f;
  }
}

__global__ void k_minmax_workspace_init(MinMaxWorkspace* ws) {
  ws->cur_min = u2f(0x7F800000u);
  ws->cur_max = u2f(0xFF800000u);
  ws->ticket = 0u;
  ws->pad = 0u;
}

template <int DT>
hipError_t launch(const void* x, int64_t n, int method, MinMaxWorkspace* ws, float* out, hipStream_t stream) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  const int64_t n_chunks = n / kEpl;
  const int unroll = method == DAF_REDUCE_ATOMIC ? kUnrollAtomic : kUnroll;
  const int cap = method == DAF_REDUCE_ATOMIC ? kMaxBlocksAtomic : kMaxBlocks;
  int64_t blocks = (n_chunks + (int64_t)kThreads * unroll - 1) / ((int64_t)kThreads * unroll);
  if (blocks < 1) blocks = 1;
  if (blocks > cap) blocks = cap;
  if (method == DAF_REDUCE_ATOMIC) {
    hipLaunchKernelGGL((k_minmax<DT, true>), dim3((unsigned)blocks), dim3(kThreads), 0, stream, x, n, ws, out);
    return hipGetLastError();
  }
  hipLaunchKernelGGL((k_minmax<DT, false>), dim3((unsigned)blocks), dim3(kThreads), 0, stream, x, n, ws, out);
  hipLaunchKernelGGL(k_minmax_final, dim3(1), dim3(kThreads), 0, stream, ws, (int)blocks, out);
  return hipGetLastError();
}

}  // namespace

int64_t daf_minmax_workspace_size(void) { return (int64_t)sizeof(MinMaxWorkspace); }

hipError_t daf_launch_minmax_workspace_init(void* workspace, hipStream_t stream) {
  hipLaunchKernelGGL(k_minmax_workspace_init, dim3(1), dim3(1), 0, stream, static_cast<MinMaxWorkspace*>(workspace));
  return hipGetLastError();
}

hipError_t daf_launch_minmax(const void* x, int dtype, int64_t n, int method, void* workspace, float* out_minmax,
                             hipStream_t stream) {
  MinMaxWorkspace* ws = static_cast<MinMaxWorkspace*>(workspace);
  switch (dtype) {
    case daf::kF32:  return launch<daf::kF32>(x, n, method, ws, out_minmax, stream);
    case daf::kF16:  return launch<daf::kF16>(x, n, method, ws, out_minmax, stream);
    case daf::kBF16: return launch<daf::kBF16>(x, n, method, ws, out_minmax, stream);
    default: return hipErrorInvalidValue;
  }
}
