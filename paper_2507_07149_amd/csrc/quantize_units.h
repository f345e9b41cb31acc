// Route "units": group sizes of 32*m elements, m not a power of two, up to 4096.
#pragma once
#include "quantize_common.h"
#include "quantize_tile.h"

namespace {

// ------------------------------------------------------------------------------------------
// Unit path: one wave per run of whole groups, for group sizes that are a multiple of 32
// elements but not a power of two (a row of a transformer activation: 768, 3072, ...).
// ------------------------------------------------------------------------------------------
// A unit is 32 consecutive elements: an aligned run of 8 lanes (binary32) or 4 lanes (16-bit
// formats) of one load.  A group is m units (3 <= m <= 128), a tile is k = 128 / m whole groups
// (fewer in the tensor's last tile), at most 4096 elements as on the fast path; lane l of load u holds chunk u*64 + l of the tile
// as far as the tile reaches (lanes past its end hold a copy of its last chunk and store
// nothing).  Min and max are reduced to units with DPP, the units of a group are then combined
// by 64 / k lanes (rounded down to a power of two) reading them from LDS.  Everything after
// that is the fast path's: lane g finishes group g, every chunk is quantized against its
// group's entry and staged, the tile's words leave as one run.
template <int DT>
struct UnitShape {
  static constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  static constexpr int kLoads = 4096 / (kWave * kEpl);             // 16 (binary32) or 8 (16-bit)
  static constexpr int kLanesLog2 = (DT == kF32) ? 3 : 2;          // log2 lanes (chunks) per unit
  static constexpr int kUnitsPerLoad = kWave >> kLanesLog2;
  static constexpr int kUnits = kLoads * kUnitsPerLoad;            // 128
  static constexpr int kPhilox = 4096 / kElemsPerPhilox / kWave;   // Philox calls per lane
  static_assert(kUnits == 128 && kLoads % 2 == 0, "unit tile");
};

template <int DT>
struct alignas(16) UnitLds {
  union {
    uint8_t rand_bytes[4096];        // byte e serves tile element e; later the staged words
    uint32_t stage[1024];
  };
  GroupInfo info[kWave];
  float2 ustat[UnitShape<DT>::kUnits];   // (min, max) per unit
};

// All global loads of a unit tile, issued up front: lane l of load u takes chunk u*64 + l,
// lanes past the tile's end a copy of its last chunk.
template <int DT>
__device__ __forceinline__ void unit_tile_load(const u32x4* x, int64_t chunk0, uint32_t n_chunks, int lane,
                                               uint4 (&raw)[UnitShape<DT>::kLoads]) {
#pragma unroll
  for (int u = 0; u < UnitShape<DT>::kLoads; ++u) {
    const uint32_t c = (uint32_t)(u * kWave + lane);
    const uint32_t cc = c < n_chunks ? c : n_chunks - 1u;
    const u32x4 v = __builtin_nontemporal_load(&x[chunk0 + cc]);
    raw[u] = make_uint4(v.x, v.y, v.z, v.w);
  }
}

// RELU variants: every loaded element becomes max(z, +0) and the tile's chunks are written to
// out_y in the layout they were read in (out_y may be the input: a lane overwrites only chunks
// it has loaded, and max(., +0) of an already written chunk is the chunk itself).
template <int DT>
__device__ __forceinline__ void unit_tile_relu(uint4 (&raw)[UnitShape<DT>::kLoads], u32x4* out_y, int64_t chunk0,
                                               uint32_t n_chunks, int lane) {
#pragma unroll
  for (int u = 0; u < UnitShape<DT>::kLoads; ++u) {
    raw[u] = make_uint4(relu_bits<DT>(raw[u].x), relu_bits<DT>(raw[u].y), relu_bits<DT>(raw[u].z),
                        relu_bits<DT>(raw[u].w));
    const uint32_t c = (uint32_t)(u * kWave + lane);
    const u32x4 y = {raw[u].x, raw[u].y, raw[u].z, raw[u].w};
    if (c < n_chunks) out_y[chunk0 + c] = y;
  }
}

// Widens the tile into xf and returns, in lane g < k, the (min, max) of group g of the tile
// (k groups of m units each).  In-lane over the chunk, DPP across the unit's lanes, one pair
// per unit to LDS; then 2^part_log2 lanes share a group's m units and combine.
template <int DT>
__device__ __forceinline__ float2 unit_tile_stats(const uint4 (&raw)[UnitShape<DT>::kLoads],
                                                  float (&xf)[UnitShape<DT>::kLoads][ElemTraits<DT>::kPerLoad],
                                                  float2* ustat, int k, int m, int part_log2, int lane) {
  using S = UnitShape<DT>;
  constexpr int kEpl = S::kEpl;
#pragma unroll
  for (int u = 0; u < S::kLoads; u += 2) {
    float mn[2], mx[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int e = 0; e < kEpl; ++e) xf[u + h][e] = chunk_elem<DT>(raw[u + h], e);
      const float(&v)[kEpl] = xf[u + h];
      if (kEpl == 4) {
        mn[h] = vmin(vmin3(v[0], v[1], v[2]), v[3]);
        mx[h] = vmax(vmax3(v[0], v[1], v[2]), v[3]);
      } else {
        mn[h] = vmin(vmin3(vmin3(vmin3(v[0], v[1], v[2]), v[3], v[4 % kEpl]), v[5 % kEpl], v[6 % kEpl]), v[7 % kEpl]);
        mx[h] = vmax(vmax3(vmax3(vmax3(v[0], v[1], v[2]), v[3], v[4 % kEpl]), v[5 % kEpl], v[6 % kEpl]), v[7 % kEpl]);
      }
    }
    seg_minmax_x2<S::kLanesLog2>(mn[0], mx[0], mn[1], mx[1]);
    if ((lane & ((1 << S::kLanesLog2) - 1)) == (1 << S::kLanesLog2) - 1) {
      ustat[u * S::kUnitsPerLoad + (lane >> S::kLanesLog2)] = make_float2(mn[0], mx[0]);
      ustat[(u + 1) * S::kUnitsPerLoad + (lane >> S::kLanesLog2)] = make_float2(mn[1], mx[1]);
    }
  }
  wave_lds_sync();

  const int part = 1 << part_log2;
  int j = lane >> part_log2;
  j = j < k ? j : k - 1;                                   // idle lanes repeat the last group
  const int p0 = lane & (part - 1);                        // < m: part <= 64 / k <= m
  const float2* us = ustat + j * m;
  float2 st = us[p0];
  for (int i = p0 + part; i < m; i += part) {
    const float2 t = us[i];
    st.x = vmin(st.x, t.x);
    st.y = vmax(st.y, t.y);
  }
  for (int d = 1; d < part; d <<= 1) {
    st.x = vmin(st.x, __shfl_xor(st.x, d));
    st.y = vmax(st.y, __shfl_xor(st.y, d));
  }
  const int src = (lane < k ? lane : k - 1) << part_log2;  // lane g takes group g's pair
  st.x = __shfl(st.x, src);
  st.y = __shfl(st.y, src);
  return st;
}

// METRICS variant of the unit kernel: per-unit partial sums (error, magnitude, rounding variance;
// one writer per entry), combined per group in a fixed order, so the sums do not depend on timing.
struct UnitMetricsLds {
  float gscale[kWave];
  float usum[3][128];
};
struct UnitNoMetricsLds {};

// Sum of a group's m per-unit values, returned in lane g < k for group g (same sharing of the
// units among 2^part_log2 lanes as unit_tile_stats).
__device__ __forceinline__ float unit_group_sum(const float* usum, int k, int m, int part_log2, int lane) {
  const int part = 1 << part_log2;
  int j = lane >> part_log2;
  j = j < k ? j : k - 1;
  const int p0 = lane & (part - 1);
  const float* us = usum + j * m;
  float acc = us[p0];
  for (int i = p0 + part; i < m; i += part) acc += us[i];
  for (int d = 1; d < part; d <<= 1) acc += __shfl_xor(acc, d);
  return __shfl(acc, (lane < k ? lane : k - 1) << part_log2);
}

template <int DT, int B, bool RELU = false, bool METRICS = false>
__device__ __forceinline__ void quantize_pack_units_body(
    typename std::conditional<RELU, const u32x4*, const u32x4* __restrict__>::type x, int64_t tile, int wave_in_block,
    int64_t n_tiles, int32_t m, int32_t k_full, int32_t k_last, uint32_t magic, int32_t part_log2,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, uint32_t seed_lo, uint32_t seed_hi,
    uint32_t* __restrict__ words, float* __restrict__ out_min, float* __restrict__ out_scale, u32x4* out_y,
    float* __restrict__ out_metrics) {
  using S = UnitShape<DT>;
  static_assert(!(RELU && METRICS), "the fused max(z, 0) and the fused metrics are separate variants");
  constexpr int kEpl = S::kEpl;
  constexpr bool kMixed = (B == 0);
  __shared__ UnitLds<DT> lds_all[kWavesPerBlock];
  __shared__ typename std::conditional<METRICS, UnitMetricsLds, UnitNoMetricsLds>::type mlds_all[kWavesPerBlock];

  const int lane = threadIdx.x & (kWave - 1);
  UnitLds<DT>& lds = lds_all[wave_in_block];
  auto& mlds = mlds_all[wave_in_block];
  uint8_t* stage8 = reinterpret_cast<uint8_t*>(lds.stage);

  const int k = (tile == n_tiles - 1) ? k_last : k_full;     // the last tile may hold fewer groups
  const uint32_t units = (uint32_t)(k * m);                  // units of the tile, <= 128
  const uint32_t n_chunks = units << S::kLanesLog2;          // chunks of the tile
  const uint32_t group_chunks = (uint32_t)m << S::kLanesLog2;
  const uint32_t group_words32 = (uint32_t)m;                // words per group and bit of width
  const int64_t g0 = tile * k_full;
  const int64_t chunk0 = tile * (int64_t)(((uint32_t)(k_full * m)) << S::kLanesLog2);

  // 1. all global loads of the tile, issued up front
  uint4 raw[S::kLoads];
  unit_tile_load<DT>(x, chunk0, n_chunks, lane, raw);
  if constexpr (RELU) unit_tile_relu<DT>(raw, out_y, chunk0, n_chunks, lane);

  uint32_t my_b = (uint32_t)B;
  uint32_t tile_base;
  if (kMixed) {
    my_b = (lane < k) ? (uint32_t)bits[g0 + lane] : 1u;
    tile_base = off[g0];
  } else {
    tile_base = (uint32_t)tile * ((uint32_t)(k_full * m) * (uint32_t)B);
  }

  // 2. random bytes of the tile (two Philox blocks per unit)
  {
    const uint64_t blk0 = (uint64_t)tile * (uint64_t)((uint32_t)(k_full * m) * 2u);
    uint4* dst = reinterpret_cast<uint4*>(lds.rand_bytes);
#pragma unroll
    for (int q = 0; q < S::kPhilox; ++q) {
      const uint32_t i = (uint32_t)(q * kWave + lane);
      if (i < units * 2u) dst[i] = philox_block(blk0 + i, seed_lo, seed_hi);
    }
  }

  // 3. + 4a. min/max per unit, then per group: lane g holds group g's pair
  float xf[S::kLoads][kEpl];
  const float2 st = unit_tile_stats<DT>(raw, xf, lds.ustat, k, m, part_log2, lane);

  // 4b. lane g of the wave finishes group g of the tile: scale, reciprocal, place in the run
  bool need_exact2;
  uint32_t tile_words;
  {
    const GroupScale s = group_scale(st.x, st.y, my_b);
    const float invs = s.inv * kScale;
    need_exact2 = __builtin_amdgcn_ballot_w64(!(invs <= 3.402823466e+38f) && lane < k) != 0ull;
    uint32_t woff;
    if (kMixed) {
      const uint32_t w = (lane < k) ? group_words32 * my_b : 0u;
      const uint32_t incl = wave_inclusive_sum(w);
      tile_words = (uint32_t)__builtin_amdgcn_readlane((int)incl, kWave - 1);
      woff = incl - w;
    } else {
      tile_words = units * (uint32_t)B;
      woff = (uint32_t)lane * (group_words32 * (uint32_t)B);
    }
    if (lane < k) {
      out_min[g0 + lane] = s.mn;
      out_scale[g0 + lane] = s.scale;
      GroupInfo gi;
      gi.mn = s.mn;
      gi.invs = need_exact2 ? s.inv : invs;
      const uint32_t lane_bits = (uint32_t)kEpl * my_b;
      const uint32_t swz = (lane_bits <= 8u) ? 3u : (lane_bits == 16u) ? 2u : 0u;
      gi.b = my_b | (swz << 8);
      gi.byte_off = woff * 4u;
      lds.info[lane] = gi;
      if constexpr (METRICS) mlds.gscale[lane] = s.scale;
    }
  }

  // the lane's random bytes, one dword per four elements, out of LDS before it is reused
  uint32_t rnd[S::kLoads][kEpl / 4];
#pragma unroll
  for (int u = 0; u < S::kLoads; ++u) {
    if (kEpl == 4) {
      rnd[u][0] = reinterpret_cast<const uint32_t*>(lds.rand_bytes)[u * kWave + lane];
    } else {
      const uint2 r2 = reinterpret_cast<const uint2*>(lds.rand_bytes)[u * kWave + lane];
      rnd[u][0] = r2.x;
      rnd[u][kEpl / 4 - 1] = r2.y;
    }
  }
  wave_lds_sync();

  // 5. quantize every chunk of the tile and drop its bits at their place in the staged run
#pragma unroll
  for (int u = 0; u < S::kLoads; ++u) {
    const uint32_t c = (uint32_t)(u * kWave + lane);
    if (c < n_chunks) {
      // (24-bit multiplications: every product here is far below 2^24, and the full 32-bit
      // multiplication runs at a quarter of the rate)
      const uint32_t grp = __umul24(c >> S::kLanesLog2, magic) >> 16;   // unit / m
      const uint32_t lig = c - __umul24(grp, group_chunks);            // chunk inside its group
      const GroupInfo gi = lds.info[grp];
      const uint32_t b = kMixed ? (gi.b & 0xFFu) : (uint32_t)B;
      const uint32_t addr = (gi.byte_off + (__umul24(lig, b * (uint32_t)kEpl) >> 3)) ^ (gi.b >> 8);
      uint32_t n0, n1;
      if constexpr (METRICS) {
        const float g_scale = mlds.gscale[grp];
        float err, mag, var, unused = 0.0f;
        if (need_exact2)
          quantize_chunk<DT, true, true>(xf[u], gi.mn, gi.invs, b, rnd[u], n0, n1, g_scale, &err, &mag, &var);
        else
          quantize_chunk<DT, false, true>(xf[u], gi.mn, gi.invs, b, rnd[u], n0, n1, g_scale, &err, &mag, &var);
        seg_sum2<S::kLanesLog2>(err, mag);       // over the unit's lanes (all valid, or none)
        seg_sum2<S::kLanesLog2>(var, unused);
        if ((lane & ((1 << S::kLanesLog2) - 1)) == (1 << S::kLanesLog2) - 1) {
          mlds.usum[0][c >> S::kLanesLog2] = err;
          mlds.usum[1][c >> S::kLanesLog2] = mag;
          mlds.usum[2][c >> S::kLanesLog2] = var;
        }
      } else {
        if (need_exact2) quantize_chunk<DT, true>(xf[u], gi.mn, gi.invs, b, rnd[u], n0, n1);
        else             quantize_chunk<DT, false>(xf[u], gi.mn, gi.invs, b, rnd[u], n0, n1);
      }
      stage_chunk<kEpl>(stage8, addr, b, n0, n1, lane);
    }
  }
  wave_lds_sync();

  // 6. the tile's words are one contiguous run in the packed buffer
  uint32_t* dst = words + tile_base;
  for (uint32_t i = lane; i < tile_words; i += kWave) __builtin_nontemporal_store(lds.stage[i], &dst[i]);
  if constexpr (METRICS) {
    const float err = unit_group_sum(mlds.usum[0], k, m, part_log2, lane);
    const float mag = unit_group_sum(mlds.usum[1], k, m, part_log2, lane);
    const float var = unit_group_sum(mlds.usum[2], k, m, part_log2, lane);
    if (lane < k) {
      const float sc = mlds.gscale[lane];
      float* o = out_metrics + 3 * (g0 + lane);
      o[0] = err;
      o[1] = mag;
      o[2] = (var * 1.52587890625e-05f) * (sc * sc);
    }
  }
}

template <int DT, int B, bool RELU = false, bool METRICS = false>
__global__ __launch_bounds__(kThreads) void k_quantize_pack_units(
    typename std::conditional<RELU, const u32x4*, const u32x4* __restrict__>::type x, int64_t n_tiles, int32_t m,
    int32_t k_full, int32_t k_last, uint32_t magic, int32_t part_log2,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, uint32_t seed_lo, uint32_t seed_hi,
    uint32_t* __restrict__ words, float* __restrict__ out_min, float* __restrict__ out_scale, u32x4* out_y,
    float* __restrict__ out_metrics, int64_t n_elems, int64_t left_begin, int64_t left_end) {
  const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // When the tensor has a short last group the grid has one more workgroup, the first, which
  // quantizes the groups left_begin .. left_end - 1 the general way: no launch of their own, and
  // their chain of dependent loads runs while the tiles stream.
  const unsigned first_tile_block = left_end > left_begin ? 1u : 0u;
  const int64_t tile = (int64_t)(blockIdx.x - first_tile_block) * kWavesPerBlock + wave_in_block;
  if (blockIdx.x < first_tile_block) {
    quantize_pack_group_body<DT, METRICS, RELU, !METRICS>(x, n_elems, m * 32, left_begin, left_end, bits, off, B, seed_lo,
                                                          seed_hi, words, out_min, out_scale, out_metrics, out_y,
                                                          METRICS ? (int64_t)wave_in_block : (int64_t)0,
                                                          METRICS ? (int64_t)kWavesPerBlock : (int64_t)1);
    return;
  }
  if (tile >= n_tiles) return;
  quantize_pack_units_body<DT, B, RELU, METRICS>(x, tile, wave_in_block, n_tiles, m, k_full, k_last, magic, part_log2,
                                                 bits, off, seed_lo, seed_hi, words, out_min, out_scale, out_y,
                                                 out_metrics);
}

// Several tensors in one launch, as k_quantize_pack_tile_batch; the entries may have different
// group sizes (the tile geometry travels with each entry).
struct UnitBatchEntry {
  const void* x;
  const uint8_t* bits;
  const uint32_t* off;
  uint32_t* words;
  float* mn;
  float* sc;
  int64_t tile_end;                                 // tiles of this and all earlier entries
  uint32_t seed_lo, seed_hi;
  int32_t m, k, k_last, part_log2;
  uint32_t magic;
};
struct UnitBatch {
  uint32_t ends[kBatchSlots];                       // e[t].tile_end, 0xFFFFFFFF beyond n
  UnitBatchEntry e[kMaxBatch];
  int32_t n;
  void clear() {
    n = 0;
    for (int i = 0; i < kBatchSlots; ++i) ends[i] = 0xFFFFFFFFu;
  }
};

template <int DT, int B>
__global__ __launch_bounds__(kThreads) void k_quantize_pack_units_batch(const UnitBatch batch) {
  const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t gtile = (int64_t)blockIdx.x * kWavesPerBlock + wave_in_block;
  const int t = batch_entry_of(batch.ends, (uint32_t)gtile);
  if (t >= batch.n) return;
  const UnitBatchEntry& e = batch.e[t];
  const int64_t first = t ? batch.e[t - 1].tile_end : 0;
  quantize_pack_units_body<DT, B>(static_cast<const u32x4*>(e.x), gtile - first, wave_in_block, e.tile_end - first, e.m,
                                  e.k, e.k_last, e.magic, e.part_log2, e.bits, e.off, e.seed_lo, e.seed_hi, e.words,
                                  e.mn, e.sc, nullptr, nullptr);
}

// Geometry of the unit path for a plan, shared by the quantize and the statistics launchers.
struct UnitGeometry {
  int32_t m, k, k_last, part_log2;
  int64_t n_tiles, full_groups;
};
inline bool unit_geometry(const daf_plan_t* p, UnitGeometry* u) {
  const int32_t gs = p->group_size;
  u->m = gs / 32;
  if (gs % 32 != 0 || u->m < 3 || u->m > 128 || (u->m & (u->m - 1)) == 0) return false;
  u->k = 128 / u->m;
  u->full_groups = p->n / gs;
  u->n_tiles = (u->full_groups + u->k - 1) / u->k;                  // the last one may hold fewer groups
  if (u->n_tiles == 0) return false;
  u->k_last = (int32_t)(u->full_groups - (u->n_tiles - 1) * u->k);
  u->part_log2 = 0;
  while ((2 << u->part_log2) * u->k <= kWave) ++u->part_log2;       // largest power of two <= 64 / k
  return true;
}

// Group sizes the unit path takes: 32 * m elements with 3 <= m <= 128 and m not a power of two
// (those are the fast path's).  Returns the groups it covered.
template <int DT, bool RELU, bool METRICS>
hipError_t launch_units(const daf_plan_t* p, const void* x, uint32_t seed_lo, uint32_t seed_hi, uint32_t* out_words,
                        float* out_min, float* out_scale, void* out_y, float* out_metrics, int64_t* covered,
                        hipStream_t stream) {
  *covered = 0;
  UnitGeometry ug;
  if (!unit_geometry(p, &ug)) return hipSuccess;
  const int32_t m = ug.m, k = ug.k, k_last = ug.k_last, part_log2 = ug.part_log2;
  const int64_t n_tiles = ug.n_tiles, full_groups = ug.full_groups;
  const uint32_t magic = (65536u + (uint32_t)m - 1u) / (uint32_t)m;   // floor(u / m) = (u * magic) >> 16 for u < 128
  // one more workgroup for the tensor's short last group, if it has one
  const unsigned blocks = (unsigned)((n_tiles + kWavesPerBlock - 1) / kWavesPerBlock) + (p->num_groups > full_groups ? 1u : 0u);
#define DAF_LAUNCH(BITS)                                                                                       \
  hipLaunchKernelGGL((k_quantize_pack_units<DT, BITS, RELU, METRICS>), dim3(blocks), dim3(kThreads), 0, stream, \
                     static_cast<const u32x4*>(x), n_tiles, m, k, k_last, magic, part_log2, p->d_bits, p->d_off, \
                     seed_lo, seed_hi, out_words, out_min, out_scale, static_cast<u32x4*>(out_y), out_metrics,  \
                     p->n, full_groups, p->num_groups)
  switch (p->uniform_bits) {
    case 0: DAF_LAUNCH(0); break;
    case 1: DAF_LAUNCH(1); break;
    case 2: DAF_LAUNCH(2); break;
    case 4: DAF_LAUNCH(4); break;
    case 8: DAF_LAUNCH(8); break;
    default: return hipErrorInvalidValue;
  }
#undef DAF_LAUNCH
  *covered = p->num_groups;                                 // the short last group included
  return hipGetLastError();
}

}  // namespace
