// Forward-pass side: per-group min/max -> scale -> stochastic-rounding quantization ->
// bit packing, in one pass over the activation (paper Sec. 2.2, Eq. 1; Sec. 3.3; order of
// codes in a word from Algorithm 2).  The kernels, by group size (always a multiple of 32):
//
//   k_quantize_pack_tile   powers of two up to 4096.  One wave owns a tile of 2048 or 4096
//                          consecutive elements (a whole number of groups).  x is read from HBM
//                          once with 16-byte loads and stays in registers between the reduction
//                          and the quantization; random bytes, group statistics and the packed
//                          words are staged in wave-private LDS; the words leave as contiguous
//                          runs.
//   k_quantize_pack_units  other sizes up to 4096: the same, with a tile of as many whole groups
//                          as fit into 128 units of 32 elements.
//   k_quantize_pack_long   4128 ... 65536: one workgroup per group, a slice per wave, (min, max)
//                          exchanged through LDS; x is still read once.
//   two passes             longer groups and per-tensor statistics (k_tile_minmax,
//                          k_group_reduce, then k_quantize_pack_tile with the group's pair).
//   k_quantize_pack_group  one wave (or workgroup) per group, element loads: whatever the others
//                          leave, i.e. the groups after the last full tile and the short last
//                          group.
//
// Rounding arithmetic.  With mn, L = 2^b-1 and inv = L/range of the group, an element maps to
// v = (x-mn)*inv and is rounded up iff r + 1/2 < frac(v)*256 for its random byte r, i.e. iff
// r < T where T = ceil(256*frac(v) - 1/2) counts the bytes that round up.  With the integer
// part folded in, code = floor((ceil(256*v - 1/2) + 255 - r) / 256).  The kernels evaluate the
// negated form, which needs one conversion instruction and one add per element:
//     code = -( (floor((mn-x)*(inv*256) + 1/2) + r) >> 8 )        (arithmetic shift)
// (mn-x)*(inv*256) is -256*v exactly as long as inv*256 does not overflow; groups where it
// would are handled with two multiplications.  floor(w + 1/2) is exact for |w| < 2^16.
// No clamp to L is needed: v <= L*(1+2^-22), so ceil(256*v - 1/2) <= 256*L.
//
// The kernels live in one header per route (quantize_group.h, quantize_tile.h,
// quantize_two_pass.h, quantize_units.h, quantize_long.h, shared pieces in quantize_common.h);
// this file holds the per-group statistics call, the choice of route and the list calls.
#include "quantize_common.h"
#include "quantize_group.h"
#include "quantize_tile.h"
#include "quantize_two_pass.h"
#include "quantize_units.h"
#include "quantize_long.h"

namespace {

// ------------------------------------------------------------------------------------------
// Statistics only: per-group min and max, for a controller that chooses the widths.
// ------------------------------------------------------------------------------------------
// One wave per group, any group size (a multiple of 32 elements, so every group starts on a
// 16-byte boundary): the group's whole 16-byte chunks four per lane at a time, the elements
// after them (the tensor's short last group only) one by one.
template <int DT>
__device__ __forceinline__ void group_minmax_group_body(const void* __restrict__ x, int64_t n, int32_t gs,
                                                        int64_t g_begin, int64_t g_end, float* __restrict__ out_min,
                                                        float* __restrict__ out_max, int64_t wave, int64_t n_waves) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  const int lane = threadIdx.x & (kWave - 1);
  for (int64_t g = g_begin + wave; g < g_end; g += n_waves) {
    const int64_t lo = g * (int64_t)gs;
    const int32_t len = (int32_t)((lo + gs <= n) ? gs : (n - lo));
    const int32_t n_chunks = len / kEpl;
    const u32x4* chunks = static_cast<const u32x4*>(x) + lo / kEpl;
    float mn = load_elem<DT>(x, lo), mx = mn;              // element 0 exists in every group
    for (int32_t c0 = lane; c0 < n_chunks; c0 += 4 * kWave) {
      u32x4 v[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int32_t c = c0 + q * kWave;
        v[q] = __builtin_nontemporal_load(&chunks[c < n_chunks ? c : c0]);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint4 raw = make_uint4(v[q].x, v[q].y, v[q].z, v[q].w);
#pragma unroll
        for (int e = 0; e < kEpl; ++e) {
          const float f = chunk_elem<DT>(raw, e);
          mn = vmin(mn, f);
          mx = vmax(mx, f);
        }
      }
    }
    for (int32_t j = n_chunks * kEpl + lane; j < len; j += kWave) {
      const float f = load_elem<DT>(x, lo + j);
      mn = vmin(mn, f);
      mx = vmax(mx, f);
    }
    float mn2 = mn, mx2 = mx;
    seg_minmax_x2<6>(mn, mx, mn2, mx2);
    if (lane == kWave - 1) {
      out_min[g] = mn + 0.0f;
      out_max[g] = mx + 0.0f;
    }
  }
}

template <int DT>
__global__ __launch_bounds__(kThreads) void k_group_minmax_group(const void* __restrict__ x, int64_t n, int32_t gs,
                                                                 int64_t g_begin, int64_t g_end,
                                                                 float* __restrict__ out_min,
                                                                 float* __restrict__ out_max) {
  group_minmax_group_body<DT>(x, n, gs, g_begin, g_end, out_min, out_max,
                              (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6),
                              (int64_t)gridDim.x * kWavesPerBlock);
}

template <int DT, int LPG_LOG2>
__global__ __launch_bounds__(kThreads) void k_group_minmax_tile(const u32x4* __restrict__ x, int64_t n_tiles,
                                                                float* __restrict__ out_min,
                                                                float* __restrict__ out_max, int64_t n_elems,
                                                                int64_t left_begin, int64_t left_end) {
  using S = TileShape<DT, LPG_LOG2>;
  __shared__ float2 stat_all[kWavesPerBlock][kWave];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // groups left over after the last whole tile: one more workgroup, the first of the grid
  const unsigned first_tile_block = left_end > left_begin ? 1u : 0u;
  if (blockIdx.x < first_tile_block) {
    group_minmax_group_body<DT>(x, n_elems, S::kGroupSize, left_begin, left_end, out_min, out_max, wave_in_block,
                                kWavesPerBlock);
    return;
  }
  const int64_t tile = (int64_t)(blockIdx.x - first_tile_block) * kWavesPerBlock + wave_in_block;
  if (tile >= n_tiles) return;
  float2* stat = stat_all[wave_in_block];
  uint4 raw[S::kLoads];
#pragma unroll
  for (int u = 0; u < S::kLoads; ++u) {
    const u32x4 v = __builtin_nontemporal_load(&x[tile * (S::kLoads * kWave) + u * kWave + lane]);
    raw[u] = make_uint4(v.x, v.y, v.z, v.w);
  }
  float xf[S::kLoads][S::kEpl];
  tile_minmax<DT, LPG_LOG2>(raw, xf, stat, lane);
  wave_lds_sync();
  if (lane < S::kGroups) {
    float2 st = stat[lane * S::kLoadsPerGroup];
#pragma unroll
    for (int j = 1; j < S::kLoadsPerGroup; ++j) {
      const float2 t = stat[lane * S::kLoadsPerGroup + j];
      st.x = vmin(st.x, t.x);
      st.y = vmax(st.y, t.y);
    }
    out_min[tile * S::kGroups + lane] = st.x + 0.0f;
    out_max[tile * S::kGroups + lane] = st.y + 0.0f;
  }
}

__global__ void k_stat_to_outputs(const float2* __restrict__ stat, int64_t num_groups, float* __restrict__ out_min,
                                  float* __restrict__ out_max) {
  const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g < num_groups) {
    out_min[g] = stat[g].x + 0.0f;
    out_max[g] = stat[g].y + 0.0f;
  }
}

// Statistics only, for the group sizes of the unit path (32 * m elements, 3 <= m <= 128, m not a
// power of two): the first steps of k_quantize_pack_units.
template <int DT>
__global__ __launch_bounds__(kThreads) void k_group_minmax_units(const u32x4* __restrict__ x, int64_t n_tiles, int32_t m,
                                                                 int32_t k_full, int32_t k_last, int32_t part_log2,
                                                                 float* __restrict__ out_min,
                                                                 float* __restrict__ out_max, int64_t n_elems,
                                                                 int64_t left_begin, int64_t left_end) {
  using S = UnitShape<DT>;
  __shared__ float2 ustat_all[kWavesPerBlock][S::kUnits];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // the tensor's short last group: one more workgroup, the first of the grid
  const unsigned first_tile_block = left_end > left_begin ? 1u : 0u;
  if (blockIdx.x < first_tile_block) {
    group_minmax_group_body<DT>(x, n_elems, m * 32, left_begin, left_end, out_min, out_max, wave_in_block,
                                kWavesPerBlock);
    return;
  }
  const int64_t tile = (int64_t)(blockIdx.x - first_tile_block) * kWavesPerBlock + wave_in_block;
  if (tile >= n_tiles) return;
  const int k = (tile == n_tiles - 1) ? k_last : k_full;
  const uint32_t n_chunks = ((uint32_t)(k * m)) << S::kLanesLog2;
  const int64_t chunk0 = tile * (int64_t)(((uint32_t)(k_full * m)) << S::kLanesLog2);
  uint4 raw[S::kLoads];
  unit_tile_load<DT>(x, chunk0, n_chunks, lane, raw);
  float xf[S::kLoads][S::kEpl];
  const float2 st = unit_tile_stats<DT>(raw, xf, ustat_all[wave_in_block], k, m, part_log2, lane);
  if (lane < k) {
    out_min[tile * k_full + lane] = st.x + 0.0f;
    out_max[tile * k_full + lane] = st.y + 0.0f;
  }
}

template <int DT>
hipError_t launch_group_minmax(const daf_plan_t* p, const void* x, float* out_min, float* out_max,
                               hipStream_t stream) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  // Groups longer than a tile: tile pairs, then a per-group reduce, unless there are enough
  // groups to fill the device with one wave each (then one launch below does it, 25 % faster).
  if (p->d_big_scratch != nullptr && p->num_groups < 1024) {
    const int64_t n_full_tiles = p->n / kBigTile;
    const int64_t n_partials = n_full_tiles + ((n_full_tiles * kBigTile < p->n) ? 1 : 0);
    const int64_t tpg = (p->num_groups == 1) ? n_partials : p->group_size / kBigTile;
    float2* partial = reinterpret_cast<float2*>(p->d_big_scratch);
    float2* stat = partial + n_partials;
    hipLaunchKernelGGL((k_tile_minmax<DT>), dim3((unsigned)((n_partials + kWavesPerBlock - 1) / kWavesPerBlock)),
                       dim3(kThreads), 0, stream, x, n_full_tiles, p->n, partial);
    hipLaunchKernelGGL(k_group_reduce, dim3((unsigned)p->num_groups), dim3(kReduceThreads), 0, stream, partial,
                       n_partials, tpg, stat);
    hipLaunchKernelGGL(k_stat_to_outputs, dim3((unsigned)((p->num_groups + 255) / 256)), dim3(256), 0, stream, stat,
                       p->num_groups, out_min, out_max);
    return hipGetLastError();
  }
  const int64_t full_groups = p->n / p->group_size;
  int64_t fast_groups = 0;
  const int32_t lpg = p->group_size / kEpl;
  if (p->group_size % kEpl == 0 && lpg >= 4 && (lpg & (lpg - 1)) == 0) {
#define DAF_CASE(LOG2)                                                                                          \
  case (1 << LOG2):                                                                                             \
    if constexpr (TileShape<DT, LOG2>::kValid) {                                                                \
      const int64_t n_tiles = full_groups / TileShape<DT, LOG2>::kGroups;                                       \
      const int64_t left = n_tiles * TileShape<DT, LOG2>::kGroups;                                              \
      if (n_tiles > 0) {                                                                                        \
        hipLaunchKernelGGL((k_group_minmax_tile<DT, LOG2>), dim3((unsigned)((n_tiles + kWavesPerBlock - 1) /    \
                           kWavesPerBlock) + (left < p->num_groups ? 1u : 0u)), dim3(kThreads), 0, stream,      \
                           static_cast<const u32x4*>(x), n_tiles, out_min, out_max, p->n, left, p->num_groups); \
        fast_groups = p->num_groups;        /* the leftover groups ride in the same launch */                   \
      }                                                                                                         \
    }                                                                                                           \
    break;
    switch (lpg) {
      DAF_CASE(2) DAF_CASE(3) DAF_CASE(4) DAF_CASE(5) DAF_CASE(6)
      DAF_CASE(7) DAF_CASE(8) DAF_CASE(9) DAF_CASE(10)
      default: break;
    }
#undef DAF_CASE
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  UnitGeometry ug;
  if (fast_groups == 0 && unit_geometry(p, &ug)) {
    hipLaunchKernelGGL((k_group_minmax_units<DT>), dim3((unsigned)((ug.n_tiles + kWavesPerBlock - 1) / kWavesPerBlock) +
                       (ug.full_groups < p->num_groups ? 1u : 0u)), dim3(kThreads), 0, stream,
                       static_cast<const u32x4*>(x), ug.n_tiles, ug.m, ug.k, ug.k_last, ug.part_log2, out_min, out_max,
                       p->n, ug.full_groups, p->num_groups);
    fast_groups = p->num_groups;            // the short last group rides in the same launch
  }
  const int64_t rest = p->num_groups - fast_groups;
  if (rest > 0) {
    int64_t blocks = (rest + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL((k_group_minmax_group<DT>), dim3((unsigned)blocks), dim3(kThreads), 0, stream, x, p->n,
                       p->group_size, fast_groups, p->num_groups, out_min, out_max);
  }
  return hipGetLastError();
}

// Tiles per tensor on the fast path (0 if the plan is not eligible) and the groups they cover.
template <int DT>
bool tile_geometry(const daf_plan_t* p, int* lpg_log2, int64_t* n_tiles, int64_t* fast_groups) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  *n_tiles = 0;
  *fast_groups = 0;
  if (p->d_big_scratch != nullptr) return false;
  const int32_t lpg = p->group_size / kEpl;
  if (p->group_size % kEpl != 0 || lpg < 4 || (lpg & (lpg - 1)) != 0) return false;
  const int64_t full_groups = p->n / p->group_size;
  bool ok = false;
#define DAF_CASE(LOG2)                                                   \
  case (1 << LOG2):                                                      \
    if constexpr (QTile<DT, LOG2>::kValid) {                             \
      *lpg_log2 = LOG2;                                                  \
      *n_tiles = full_groups / QTile<DT, LOG2>::kGroups;                 \
      *fast_groups = *n_tiles * QTile<DT, LOG2>::kGroups;                \
      ok = *n_tiles > 0;                                                 \
    }                                                                    \
    break;
  switch (lpg) {
    DAF_CASE(2) DAF_CASE(3) DAF_CASE(4) DAF_CASE(5) DAF_CASE(6)
    DAF_CASE(7) DAF_CASE(8) DAF_CASE(9) DAF_CASE(10)
    default: break;
  }
#undef DAF_CASE
  return ok;
}

// Which kernels a plan's quantize call uses for its whole groups (the values of daf_route_t).
template <int DT>
int quantize_route(const daf_plan_t* p) {
  int log2 = 0;
  int64_t n_tiles = 0, fast_groups = 0;
  UnitGeometry ug;
  if (long_applies(p)) return 2;
  if (p->d_big_scratch != nullptr) return 3;
  if (tile_geometry<DT>(p, &log2, &n_tiles, &fast_groups)) return 0;
  if (unit_geometry(p, &ug)) return 1;
  return 4;
}

template <int DT, bool METRICS, bool RELU = false>
hipError_t launch_dtype(const daf_plan_t* p, const void* x, uint64_t seed, uint32_t* out_words, float* out_min,
                        float* out_scale, float* out_metrics, void* out_y, hipStream_t stream,
                        void* big_scratch = nullptr) {
  const uint32_t seed_lo = (uint32_t)seed, seed_hi = (uint32_t)(seed >> 32);
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  const int64_t full_groups = p->n / p->group_size;
  int64_t fast_groups = 0;
  const int route = quantize_route<DT>(p);                  // 0 tile, 1 units, 2 long, 3 two passes, 4 group by group
  if (route == 2) {                     // groups of 4128 .. 65536 elements, one workgroup each
    const hipError_t e = launch_long<DT, RELU, METRICS>(p, x, seed_lo, seed_hi, out_words, out_min, out_scale, out_y,
                                                        out_metrics, &fast_groups, stream);
    if (e != hipSuccess) return e;
  }
  if (route == 3) {                     // statistics first (scratch set up by daf_plan)
    if (METRICS || RELU) return hipErrorNotSupported;
    return launch_big<DT>(p, x, seed_lo, seed_hi, out_words, out_min, out_scale,
                          big_scratch ? big_scratch : p->d_big_scratch, stream);
  }

  // fast path: groups of 4 .. 1024 chunks (a power of two, at most one tile), whole tiles only
  const int32_t lpg = p->group_size / kEpl;
  if (route == 0) {
    int64_t n_tiles = 0;
    hipError_t e = hipSuccess;
#define DAF_CASE(LOG2)                                                                                   \
  case (1 << LOG2):                                                                                      \
    if constexpr (QTile<DT, LOG2>::kValid) {                                                             \
      n_tiles = full_groups / QTile<DT, LOG2>::kGroups;                                                  \
      fast_groups = p->num_groups;          /* the leftover groups ride in the same launch */            \
      if (n_tiles > 0) e = launch_tile<DT, LOG2, METRICS, RELU>(p, x, n_tiles, seed_lo, seed_hi, out_words, \
                                                                out_min, out_scale, out_metrics, out_y,  \
                                                                stream);                                 \
    }                                                                                                    \
    break;
    switch (lpg) {
      DAF_CASE(2) DAF_CASE(3) DAF_CASE(4) DAF_CASE(5) DAF_CASE(6)
      DAF_CASE(7) DAF_CASE(8) DAF_CASE(9) DAF_CASE(10)
      default: break;
    }
#undef DAF_CASE
    if (e != hipSuccess) return e;
  }

  if (route == 1) {
    const hipError_t e = launch_units<DT, RELU, METRICS>(p, x, seed_lo, seed_hi, out_words, out_min, out_scale, out_y,
                                                         out_metrics, &fast_groups, stream);
    if (e != hipSuccess) return e;
  }

  // general path for everything the tiles did not cover
  const int64_t rest = p->num_groups - fast_groups;
  if (rest > 0) {
    if constexpr (!METRICS) {
      if (p->group_size >= 1024) {         // long groups: a workgroup each
        const int64_t blocks = rest < 65536 ? rest : 65536;
        hipLaunchKernelGGL((k_quantize_pack_group<DT, false, RELU, true>), dim3((unsigned)blocks), dim3(kThreads), 0,
                           stream, x, p->n, p->group_size, fast_groups, p->num_groups, p->d_bits, p->d_off,
                           p->uniform_bits, seed_lo, seed_hi, out_words, out_min, out_scale, out_metrics, out_y);
        return hipGetLastError();
      }
    }
    int64_t blocks = (rest + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL((k_quantize_pack_group<DT, METRICS, RELU>), dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                       x, p->n, p->group_size, fast_groups, p->num_groups, p->d_bits, p->d_off, p->uniform_bits,
                       seed_lo, seed_hi, out_words, out_min, out_scale, out_metrics, out_y);
    return hipGetLastError();
  }
  return hipSuccess;
}

template <int DT, int LPG_LOG2>
hipError_t launch_batch_bits(const Batch& batch, int32_t uniform_bits, hipStream_t stream) {
  const int64_t tiles = batch.e[batch.n - 1].tile_end;
  const unsigned blocks = (unsigned)((tiles + kWavesPerBlock - 1) / kWavesPerBlock);
#define DAF_LAUNCH(BITS) \
  hipLaunchKernelGGL((k_quantize_pack_tile_batch<DT, LPG_LOG2, BITS>), dim3(blocks), dim3(kThreads), 0, stream, batch)
  switch (uniform_bits) {
    case 0: DAF_LAUNCH(0); break;
    case 1: DAF_LAUNCH(1); break;
    case 2: DAF_LAUNCH(2); break;
    case 4: DAF_LAUNCH(4); break;
    case 8: DAF_LAUNCH(8); break;
    default: return hipErrorInvalidValue;
  }
#undef DAF_LAUNCH
  return hipGetLastError();
}

template <int DT>
hipError_t launch_batch(const Batch& batch, int lpg_log2, int32_t uniform_bits, hipStream_t stream) {
  switch (lpg_log2) {
#define DAF_CASE(LOG2)                                                                      \
  case LOG2:                                                                                \
    if constexpr (QTile<DT, LOG2>::kValid) return launch_batch_bits<DT, LOG2>(batch, uniform_bits, stream);  \
    break;
    DAF_CASE(2) DAF_CASE(3) DAF_CASE(4) DAF_CASE(5) DAF_CASE(6)
    DAF_CASE(7) DAF_CASE(8) DAF_CASE(9) DAF_CASE(10)
#undef DAF_CASE
    default: break;
  }
  return hipErrorInvalidValue;
}

// Same results as one daf_launch_quantize_pack per item.  Consecutive items whose plans share
// group size and width kind go into one launch for their whole tiles (at most kMaxBatch per
// launch); the groups after an item's last whole tile, and items the fast path does not cover,
// are launched as before.
template <int DT>
hipError_t launch_items(const daf_quantize_item_t* items, int32_t n_items, hipStream_t stream) {
  Batch batch;
  batch.clear();
  UnitBatch ubatch;                    // items of the unit path (group sizes that are not a power of two)
  ubatch.clear();
  int cur_log2 = -1, cur_gs = -1, cur_bits = -1, ucur_bits = -1;
  hipError_t err = hipSuccess;
  auto flush = [&]() {
    if (batch.n > 0 && err == hipSuccess) err = launch_batch<DT>(batch, cur_log2, cur_bits, stream);
    batch.clear();
  };
  GroupBatch gbatch[2];                // leftovers: [0] a wave per group, [1] a workgroup per group
  gbatch[0].n = gbatch[1].n = 0;
  auto gflush = [&](int coop) {
    GroupBatch& gb = gbatch[coop];
    if (gb.n > 0 && err == hipSuccess) {
      if (coop)
        hipLaunchKernelGGL((k_quantize_pack_group_batch<DT, true>), dim3((unsigned)gb.n), dim3(kThreads), 0, stream, gb);
      else
        hipLaunchKernelGGL((k_quantize_pack_group_batch<DT, false>), dim3((unsigned)gb.n), dim3(kThreads), 0, stream, gb);
      err = hipGetLastError();
    }
    gb.n = 0;
  };
  // the groups [g_begin, num_groups) of an item, to be quantized group by group
  auto leftovers = [&](const daf_quantize_item_t& it, int64_t g_begin) {
    const daf_plan_t* p = it.plan;
    if (g_begin >= p->num_groups || err != hipSuccess) return;
    const int coop = p->group_size >= 1024 ? 1 : 0;
    GroupBatch& gb = gbatch[coop];
    if (gb.n == 32) gflush(coop);
    GroupBatchEntry& e = gb.e[gb.n++];
    e.x = it.x;
    e.bits = p->d_bits;
    e.off = p->d_off;
    e.words = it.out_words;
    e.mn = it.out_min;
    e.sc = it.out_scale;
    e.n = p->n;
    e.g_begin = g_begin;
    e.g_end = p->num_groups;
    e.gs = p->group_size;
    e.uniform_bits = p->uniform_bits;
    e.seed_lo = (uint32_t)it.seed;
    e.seed_hi = (uint32_t)(it.seed >> 32);
  };
  LongBatch lbatch;                    // items of the one-workgroup-per-group kernel
  lbatch.n = 0;
  int lcur_bits = -1, lcur_waves = -1;
  auto lflush = [&]() {
    if (lbatch.n > 0 && err == hipSuccess) {
      const unsigned blocks = (unsigned)lbatch.e[lbatch.n - 1].group_end;
      const unsigned lds_bytes = (unsigned)(lcur_waves * (sizeof(LongWaveLds) + sizeof(float4)));
#define DAF_LAUNCH(BITS)                                                                                    \
  hipLaunchKernelGGL((k_quantize_pack_long_batch<DT, BITS>), dim3(blocks), dim3(kWave * lcur_waves), lds_bytes, \
                     stream, lbatch)
      switch (lcur_bits) {
        case 0: DAF_LAUNCH(0); break;
        case 1: DAF_LAUNCH(1); break;
        case 2: DAF_LAUNCH(2); break;
        case 4: DAF_LAUNCH(4); break;
        case 8: DAF_LAUNCH(8); break;
        default: err = hipErrorInvalidValue; break;
      }
#undef DAF_LAUNCH
      if (err == hipSuccess) err = hipGetLastError();
    }
    lbatch.n = 0;
  };
  auto uflush = [&]() {
    if (ubatch.n > 0 && err == hipSuccess) {
      const unsigned blocks = (unsigned)((ubatch.e[ubatch.n - 1].tile_end + kWavesPerBlock - 1) / kWavesPerBlock);
#define DAF_LAUNCH(BITS) \
  hipLaunchKernelGGL((k_quantize_pack_units_batch<DT, BITS>), dim3(blocks), dim3(kThreads), 0, stream, ubatch)
      switch (ucur_bits) {
        case 0: DAF_LAUNCH(0); break;
        case 1: DAF_LAUNCH(1); break;
        case 2: DAF_LAUNCH(2); break;
        case 4: DAF_LAUNCH(4); break;
        case 8: DAF_LAUNCH(8); break;
        default: err = hipErrorInvalidValue; break;
      }
#undef DAF_LAUNCH
      if (err == hipSuccess) err = hipGetLastError();
    }
    ubatch.clear();
  };
  for (int32_t i = 0; i < n_items && err == hipSuccess; ++i) {
    const daf_quantize_item_t& it = items[i];
    const daf_plan_t* p = it.plan;
    int log2 = 0;
    int64_t n_tiles = 0, fast_groups = 0;
    if (long_applies(p)) {
      const int32_t m = p->group_size / 32;
      const int32_t n_waves = (m + 127) / 128;
      const int64_t full_groups = p->n / p->group_size;
      if (lbatch.n == kMaxBatch || (lbatch.n > 0 && (p->uniform_bits != lcur_bits || n_waves != lcur_waves)) ||
          (lbatch.n > 0 && lbatch.e[lbatch.n - 1].group_end + full_groups > 0x7fffffff))
        lflush();
      lcur_bits = p->uniform_bits;
      lcur_waves = n_waves;
      LongBatchEntry& e = lbatch.e[lbatch.n];
      e.x = it.x;
      e.bits = p->d_bits;
      e.off = p->d_off;
      e.words = it.out_words;
      e.mn = it.out_min;
      e.sc = it.out_scale;
      e.group_end = (lbatch.n ? lbatch.e[lbatch.n - 1].group_end : 0) + full_groups;
      e.seed_lo = (uint32_t)it.seed;
      e.seed_hi = (uint32_t)(it.seed >> 32);
      e.m = m;
      e.units_per_wave = (m + n_waves - 1) / n_waves;
      ++lbatch.n;
      leftovers(it, full_groups);                                       // the short last group
      continue;
    }
    UnitGeometry ug;
    if (p->d_big_scratch == nullptr && unit_geometry(p, &ug)) {
      if (ubatch.n == kMaxBatch || (ubatch.n > 0 && p->uniform_bits != ucur_bits) ||
          (ubatch.n > 0 && ubatch.e[ubatch.n - 1].tile_end + ug.n_tiles > 0x7fffffff))
        uflush();
      ucur_bits = p->uniform_bits;
      UnitBatchEntry& e = ubatch.e[ubatch.n];
      e.x = it.x;
      e.bits = p->d_bits;
      e.off = p->d_off;
      e.words = it.out_words;
      e.mn = it.out_min;
      e.sc = it.out_scale;
      e.tile_end = (ubatch.n ? ubatch.e[ubatch.n - 1].tile_end : 0) + ug.n_tiles;
      ubatch.ends[ubatch.n] = (uint32_t)e.tile_end;
      e.seed_lo = (uint32_t)it.seed;
      e.seed_hi = (uint32_t)(it.seed >> 32);
      e.m = ug.m;
      e.k = ug.k;
      e.k_last = ug.k_last;
      e.part_log2 = ug.part_log2;
      e.magic = (65536u + (uint32_t)ug.m - 1u) / (uint32_t)ug.m;
      ++ubatch.n;
      leftovers(it, ug.full_groups);                                    // the short last group
      continue;
    }
    if (!tile_geometry<DT>(p, &log2, &n_tiles, &fast_groups)) {
      flush();
      if (err == hipSuccess)
        err = launch_dtype<DT, false>(p, it.x, it.seed, it.out_words, it.out_min, it.out_scale, nullptr, nullptr, stream);
      continue;
    }
    if (batch.n == kMaxBatch || (batch.n > 0 && (p->group_size != cur_gs || p->uniform_bits != cur_bits)) ||
        (batch.n > 0 && batch.e[batch.n - 1].tile_end + n_tiles > 0x7fffffff))
      flush();
    cur_log2 = log2;
    cur_gs = p->group_size;
    cur_bits = p->uniform_bits;
    BatchEntry& e = batch.e[batch.n];
    e.x = it.x;
    e.bits = p->d_bits;
    e.off = p->d_off;
    e.words = it.out_words;
    e.mn = it.out_min;
    e.sc = it.out_scale;
    e.tile_end = (batch.n ? batch.e[batch.n - 1].tile_end : 0) + n_tiles;
    batch.ends[batch.n] = (uint32_t)e.tile_end;
    e.seed_lo = (uint32_t)it.seed;
    e.seed_hi = (uint32_t)(it.seed >> 32);
    ++batch.n;
    leftovers(it, fast_groups);                                         // groups after the last whole tile
  }
  flush();
  uflush();
  lflush();
  gflush(0);
  gflush(1);
  return err;
}

}  // namespace

// This file is compiled once per element format (-DDAF_DT=0, 1, 2: the three builds run in
// parallel and each holds a third of the kernel instantiations); quantize_dispatch.hip picks
// the build by dtype.
#ifndef DAF_DT
#error "compile with -DDAF_DT=0 (binary32), 1 (binary16) or 2 (bfloat16)"
#endif
#define DAF_DT_NAME_(name, dt) name##_dt##dt
#define DAF_DT_NAME(name, dt) DAF_DT_NAME_(name, dt)

#if DAF_DT == 0
bool daf_quantize_reads_once(const daf_plan_t* plan) { return plan->d_big_scratch == nullptr || long_applies(plan); }
#endif

int DAF_DT_NAME(daf_quantize_route, DAF_DT)(const daf_plan_t* plan) { return quantize_route<DAF_DT>(plan); }

hipError_t DAF_DT_NAME(daf_launch_quantize_pack_batch, DAF_DT)(const daf_quantize_item_t* items, int32_t n_items,
                                                               hipStream_t stream) {
  return launch_items<DAF_DT>(items, n_items, stream);
}

hipError_t DAF_DT_NAME(daf_launch_group_minmax, DAF_DT)(const daf_plan_t* plan, const void* x, float* out_min,
                                                        float* out_max, hipStream_t stream) {
  return launch_group_minmax<DAF_DT>(plan, x, out_min, out_max, stream);
}

hipError_t DAF_DT_NAME(daf_launch_quantize_pack, DAF_DT)(const daf_plan_t* plan, const void* x, uint64_t seed,
                                                         uint32_t* out_words, float* out_min, float* out_scale,
                                                         float* out_metrics, void* out_relu_y, void* big_scratch,
                                                         hipStream_t stream) {
  if (out_metrics && out_relu_y) return hipErrorNotSupported;
  if (out_relu_y)
    return launch_dtype<DAF_DT, false, true>(plan, x, seed, out_words, out_min, out_scale, nullptr, out_relu_y, stream);
  return out_metrics ? launch_dtype<DAF_DT, true>(plan, x, seed, out_words, out_min, out_scale, out_metrics, nullptr, stream)
                     : launch_dtype<DAF_DT, false>(plan, x, seed, out_words, out_min, out_scale, nullptr, nullptr, stream,
                                                   big_scratch);
}
