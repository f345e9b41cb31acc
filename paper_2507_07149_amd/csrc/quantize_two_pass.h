// Route "two passes": groups longer than 65536 elements, few long groups, one group per tensor.
#pragma once
#include "quantize_common.h"
#include "quantize_tile.h"

namespace {

// ------------------------------------------------------------------------------------------
// Groups longer than a tile (up to the whole tensor: the paper's per-tensor statistics).
// ------------------------------------------------------------------------------------------
// The group's min/max can no longer be found inside one wave, so the work is split the way
// Sec. 3.2.1 describes: every tile writes its (min, max) to memory, a second small launch
// reduces the pairs of each group, and the quantize pass reads the group's pair back.
// (Merging the tile results with Algorithm 1's atomic minimum instead was measured on the
// whole-tensor reduction: thousands of workgroups hitting one address serialise, and the
// extra launch is cheaper on this GPU.)

constexpr int kBigTile = 4096;   // elements per tile in every max-shape instantiation

template <int DT>
__global__ __launch_bounds__(kThreads) void k_tile_minmax(const void* __restrict__ x, int64_t n_full_tiles,
                                                          int64_t n, float2* __restrict__ partial) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  constexpr int kLoads = kBigTile / (kWave * kEpl);
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t tile = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  float mn, mx;
  if (tile < n_full_tiles) {
    const u32x4* chunks = static_cast<const u32x4*>(x) + tile * (kLoads * kWave);
    u32x4 v[kLoads];
#pragma unroll
    for (int u = 0; u < kLoads; ++u) v[u] = __builtin_nontemporal_load(&chunks[u * kWave + lane]);
    float a[2], b[2];
#pragma unroll
    for (int u = 0; u < kLoads; ++u) {
      const uint4 raw = make_uint4(v[u].x, v[u].y, v[u].z, v[u].w);
      float f[kEpl];
#pragma unroll
      for (int e = 0; e < kEpl; ++e) f[e] = chunk_elem<DT>(raw, e);
      float lo = vmin(vmin3(f[0], f[1], f[2]), f[3]), hi = vmax(vmax3(f[0], f[1], f[2]), f[3]);
      if (kEpl == 8) {
        lo = vmin3(lo, vmin3(f[4 % kEpl], f[5 % kEpl], f[6 % kEpl]), f[7 % kEpl]);
        hi = vmax3(hi, vmax3(f[4 % kEpl], f[5 % kEpl], f[6 % kEpl]), f[7 % kEpl]);
      }
      a[u & 1] = (u < 2) ? lo : vmin(a[u & 1], lo);
      b[u & 1] = (u < 2) ? hi : vmax(b[u & 1], hi);
    }
    seg_minmax_x2<6>(a[0], b[0], a[1], b[1]);
    mn = vmin(a[0], a[1]);
    mx = vmax(b[0], b[1]);
  } else if (tile == n_full_tiles && n_full_tiles * kBigTile < n) {
    // the elements after the last full tile, one wave, element by element
    const int64_t e0 = n_full_tiles * kBigTile;
    mn = mx = load_elem<DT>(x, e0);
    for (int64_t i = e0 + lane; i < n; i += kWave) {
      const float f = load_elem<DT>(x, i);
      mn = vmin(mn, f);
      mx = vmax(mx, f);
    }
    float mn2 = mn, mx2 = mx;
    seg_minmax_x2<6>(mn, mx, mn2, mx2);
  } else {
    return;
  }
  if (lane == kWave - 1) partial[tile] = make_float2(mn, mx);
}

// One workgroup per group: reduce the group's tile pairs (up to N/4096 of them when the whole
// tensor is one group, hence the wide workgroup and several loads in flight per thread).
constexpr int kReduceThreads = 1024;
__global__ __launch_bounds__(kReduceThreads) void k_group_reduce(const float2* __restrict__ partial,
                                                                 int64_t n_partials, int64_t tiles_per_group,
                                                                 float2* __restrict__ stat) {
  __shared__ float2 lds[kReduceThreads / kWave];
  const int64_t g = blockIdx.x;
  const int64_t lo = g * tiles_per_group;
  const int64_t hi = (lo + tiles_per_group < n_partials) ? lo + tiles_per_group : n_partials;
  float mn = partial[lo].x, mx = partial[lo].y, mn2 = mn, mx2 = mx;
  int64_t i = lo + threadIdx.x;
  for (; i + 3 * kReduceThreads < hi; i += 4 * kReduceThreads) {
    const float2 p0 = partial[i], p1 = partial[i + kReduceThreads], p2 = partial[i + 2 * kReduceThreads],
                 p3 = partial[i + 3 * kReduceThreads];
    mn = vmin3(mn, p0.x, p1.x);
    mx = vmax3(mx, p0.y, p1.y);
    mn2 = vmin3(mn2, p2.x, p3.x);
    mx2 = vmax3(mx2, p2.y, p3.y);
  }
  for (; i < hi; i += kReduceThreads) {
    const float2 p = partial[i];
    mn = vmin(mn, p.x);
    mx = vmax(mx, p.y);
  }
  seg_minmax_x2<6>(mn, mx, mn2, mx2);
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  if (lane == kWave - 1) lds[wave] = make_float2(vmin(mn, mn2), vmax(mx, mx2));
  __syncthreads();
  if (threadIdx.x == 0) {
    float2 r = lds[0];
    for (int w = 1; w < kReduceThreads / kWave; ++w) {
      r.x = vmin(r.x, lds[w].x);
      r.y = vmax(r.y, lds[w].y);
    }
    stat[g] = r;
  }
}

// The elements after the last full tile, [e_begin, n): all in group g, whose (min, max) is
// known.  One workgroup, one packed word per thread and iteration.
template <int DT>
__global__ __launch_bounds__(kThreads) void k_quantize_pack_tail_ext(
    const void* __restrict__ x, int64_t e_begin, int64_t n, int64_t g, int64_t group_begin,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, int32_t uniform_bits,
    const float2* __restrict__ ext_stat, uint32_t seed_lo, uint32_t seed_hi, uint32_t* __restrict__ words,
    float* __restrict__ out_min, float* __restrict__ out_scale) {
  const uint32_t b = uniform_bits ? (uint32_t)uniform_bits : (uint32_t)bits[g];
  const uint32_t group_off = uniform_bits ? (uint32_t)((group_begin * uniform_bits) >> 5) : off[g];
  const uint32_t word_base = group_off + (uint32_t)(((e_begin - group_begin) * b) >> 5);
  const float2 st = ext_stat[g];
  const GroupScale s = group_scale(st.x, st.y, b);
  if (threadIdx.x == 0 && e_begin == group_begin) {
    out_min[g] = s.mn;
    out_scale[g] = s.scale;
  }
  const int64_t len = n - e_begin;
  const uint32_t cpw = 32u / b;
  const int64_t n_words = (len * b + 31) >> 5;
  for (int64_t t = threadIdx.x; t < n_words; t += kThreads) {
    uint32_t word = 0;
    uint64_t cur_blk = ~0ull;
    uint4 rnd = make_uint4(0, 0, 0, 0);
    for (uint32_t c = 0; c < cpw; ++c) {
      const int64_t j = t * cpw + c;
      if (j >= len) break;
      const uint64_t i = (uint64_t)(e_begin + j);
      const uint64_t blk = i / kElemsPerPhilox;
      if (blk != cur_blk) {
        rnd = philox_block(blk, seed_lo, seed_hi);
        cur_blk = blk;
      }
      const uint32_t slot = (uint32_t)(i % kElemsPerPhilox);
      const uint32_t rw = (slot < 4) ? rnd.x : (slot < 8) ? rnd.y : (slot < 12) ? rnd.z : rnd.w;
      const uint32_t r = (rw >> (8u * (slot & 3u))) & 0xFFu;
      const int nc = neg_code<true>(load_elem<DT>(x, e_begin + j), s.mn, s.inv, r);
      word |= (uint32_t)(-nc) << (32u - b - c * b);
    }
    words[word_base + t] = word;
  }
}

template <int DT>
hipError_t launch_big(const daf_plan_t* p, const void* x, uint32_t seed_lo, uint32_t seed_hi, uint32_t* out_words,
                      float* out_min, float* out_scale, void* scratch, hipStream_t stream) {
  constexpr int kMaxLog2 = (DT == kF32) ? 10 : 9;                // the shape whose tile is one group
  static_assert(TileShape<DT, kMaxLog2>::kElems == kBigTile && TileShape<DT, kMaxLog2>::kGroups == 1, "shape");
  const int64_t n_full_tiles = p->n / kBigTile;
  const bool tail = n_full_tiles * kBigTile < p->n;
  const int64_t n_partials = n_full_tiles + (tail ? 1 : 0);
  const int64_t tpg = (p->num_groups == 1) ? n_partials : p->group_size / kBigTile;
  float2* partial = reinterpret_cast<float2*>(scratch);        // every entry read below is written first
  float2* stat = partial + n_partials;

  const unsigned blocks1 = (unsigned)((n_partials + kWavesPerBlock - 1) / kWavesPerBlock);
  hipLaunchKernelGGL((k_tile_minmax<DT>), dim3(blocks1), dim3(kThreads), 0, stream, x, n_full_tiles, p->n, partial);
  hipLaunchKernelGGL(k_group_reduce, dim3((unsigned)p->num_groups), dim3(kReduceThreads), 0, stream, partial,
                     n_partials, tpg, stat);
  if (n_full_tiles > 0) {
    const unsigned blocks = (unsigned)((n_full_tiles + kWavesPerBlock - 1) / kWavesPerBlock);
#define DAF_LAUNCH(BITS)                                                                                      \
  hipLaunchKernelGGL((k_quantize_pack_tile<DT, kMaxLog2, BITS, true>), dim3(blocks), dim3(kThreads), 0, stream, \
                     static_cast<const u32x4*>(x), n_full_tiles, p->d_bits, p->d_off, seed_lo, seed_hi,       \
                     out_words, out_min, out_scale, stat, tpg, nullptr, nullptr, (int64_t)0, (int64_t)0, (int64_t)0)
    switch (p->uniform_bits) {
      case 0: DAF_LAUNCH(0); break;
      case 1: DAF_LAUNCH(1); break;
      case 2: DAF_LAUNCH(2); break;
      case 4: DAF_LAUNCH(4); break;
      case 8: DAF_LAUNCH(8); break;
      default: return hipErrorInvalidValue;
    }
#undef DAF_LAUNCH
  }
  if (tail) {
    const int64_t g = p->num_groups - 1;
    hipLaunchKernelGGL((k_quantize_pack_tail_ext<DT>), dim3(1), dim3(kThreads), 0, stream, x,
                       n_full_tiles * kBigTile, p->n, g, g * (int64_t)p->group_size, p->d_bits, p->d_off,
                       p->uniform_bits, stat, seed_lo, seed_hi, out_words, out_min, out_scale);
  }
  return hipGetLastError();
}

}  // namespace
