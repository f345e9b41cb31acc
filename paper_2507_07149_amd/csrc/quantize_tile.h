// Route "tile": group sizes that are a power of two up to 4096, one wave per tile.
#pragma once
#include "quantize_common.h"
#include "quantize_group.h"

namespace {

// ------------------------------------------------------------------------------------------
// Fast path: one wave per tile.
// ------------------------------------------------------------------------------------------
// Lane l of load u holds the 16-byte chunk u*64 + l of the tile.  A group spans
// 2^LPG_LOG2 consecutive chunks: up to 64 neighbouring lanes of one load (LPG_LOG2 <= 6), or
// the whole wave over 2, 4, 8 or 16 consecutive loads (LPG_LOG2 = 7..10).
// DIV = 2: a tile of half the size (2048 elements of a 16-bit format): twice as many, shorter
// waves, for tensors so small that whole-size tiles would leave the last round of waves half
// empty.
template <int DT, int LPG_LOG2, int DIV = 1>
struct TileShape {
  static constexpr int kEpl = ElemTraits<DT>::kPerLoad;            // elements per lane per load
  static constexpr int kLaneLog2 = LPG_LOG2 < 6 ? LPG_LOG2 : 6;    // log2 lanes of a group in one load
  static constexpr int kLpg = 1 << kLaneLog2;                      // lanes per group (in one load)
  static constexpr int kGpl = kWave / kLpg;                        // group segments per load
  static constexpr int kLoadsPerGroup = 1 << (LPG_LOG2 - kLaneLog2);
  static constexpr int kMaxLoads = 4096 / (kWave * kEpl) / DIV;    // 16 (fp32) or 8 (16-bit), over DIV
  static constexpr int kLoads = (kMaxLoads * kGpl <= kWave) ? kMaxLoads : kWave / kGpl;
  static constexpr int kSegments = kLoads * kGpl;                  // (load, lane run) pairs, <= 64
  static constexpr int kGroups = kSegments / kLoadsPerGroup;       // groups per tile
  static constexpr int kElems = kLoads * kWave * kEpl;             // 2048 or 4096
  static constexpr int kGroupSize = (1 << LPG_LOG2) * kEpl;
  static constexpr int kPhilox = kElems / kElemsPerPhilox / kWave; // Philox calls per lane
  static constexpr bool kValid = kLoadsPerGroup <= kLoads && kElems >= kElemsPerPhilox * kWave;
  static_assert(kSegments <= kWave, "tile shape");
};

// The tile the quantize kernels use for a group shape.  binary32 tiles are a quarter of the
// largest size (1024 elements, 4 loads per lane; a half where a group needs more loads): the
// binary32 kernel is bound by memory, and with a third of the registers per wave more waves keep
// loads in flight.  Measured, whole / half / quarter tiles: 40.6 / 37.0 / 35.2 us on a
// 51 M-element tensor, 150 / 141 / 131 us on 205 M elements.  The 16-bit kernels are bound by
// vector instructions and lose to the per-tile overhead of smaller tiles (measured), so they keep
// the whole size.
template <int DT, int LPG_LOG2>
constexpr int tile_div() {
  if (DT != kF32) return 1;
  if (TileShape<DT, LPG_LOG2, 4>::kValid && TileShape<DT, LPG_LOG2, 4>::kElems < TileShape<DT, LPG_LOG2, 2>::kElems) return 4;
  if (TileShape<DT, LPG_LOG2, 2>::kValid && TileShape<DT, LPG_LOG2, 2>::kElems < TileShape<DT, LPG_LOG2, 1>::kElems) return 2;
  return 1;
}
template <int DT, int LPG_LOG2>
using QTile = TileShape<DT, LPG_LOG2, tile_div<DT, LPG_LOG2>()>;

struct alignas(16) GroupInfo {   // what every lane of a group needs for the element map
  float mn;
  float invs;                    // inv*256, or inv on the two-multiplication path
  uint32_t b;                    // width; bits 8..9: byte-address swizzle of the staged run (3, 2 or 0)
  uint32_t byte_off;             // byte offset of the group inside the tile's packed run
};

template <int DT, int LPG_LOG2, int DIV = 1>
struct alignas(16) WaveLds {
  using S = TileShape<DT, LPG_LOG2, DIV>;
  // First the random bytes of the tile (byte e serves tile element e); once every lane has
  // taken its bytes into registers the same memory stages the tile's packed words (at most
  // 8 bits per element, so the run always fits).
  // The staged run starts up to three words in, so that 16-byte pieces of it line up with
  // 16-byte pieces of the packed buffer.
  union {
    uint8_t rand_bytes[S::kElems];
    uint32_t stage[S::kElems / 4 + 4];
  };
  GroupInfo info[kWave];
  float2 stat[kWave];                   // (min, max) per group, written by the group's last lane;
                                        // later (metrics variant) the group's (error, magnitude) sums
  float gscale[kWave];                  // scale per group (metrics variant)
  float gvar[kWave];                    // sum of T*(256-T) per group (metrics variant)
};

// Codes of one 16-byte chunk, accumulated most significant first and NEGATED (the element map
// yields -code): nacc0 = -(elements 0..3), nacc1 = -(elements 4..7) (16-bit inputs only).
//
// METRICS: also returns this lane's share of the group's importance sums (Sec. 3.2 names
// quantization error and tensor magnitude): err += (x - xhat)^2 with xhat = fma(code, scale, mn)
// as the dequantizer computes it, mag += x^2, both in binary32; var = sum of T*(256-T), the
// variance of the stochastic rounding in units of scale^2 / 65536 (exact integer).
template <int DT, bool EXACT2, bool METRICS = false>
__device__ __forceinline__ void quantize_chunk(const float (&xf)[ElemTraits<DT>::kPerLoad], float mn,
                                               float invs, uint32_t b, const uint32_t* rnd,
                                               uint32_t& nacc0, uint32_t& nacc1, float scale = 0.0f,
                                               float* err = nullptr, float* mag = nullptr, float* var = nullptr) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  uint32_t nacc[2] = {0u, 0u};
  float e2 = 0.0f, m2 = 0.0f;
  uint32_t v2 = 0u;
#pragma unroll
  for (int q = 0; q < kEpl / 4; ++q) {
    const uint32_t rw = rnd[q];                 // the random bytes of four consecutive elements
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float xv = xf[q * 4 + e];
      int rt;
      const int nc = neg_code<EXACT2>(xv, mn, invs, (rw >> (8 * e)) & 0xFFu, METRICS ? &rt : nullptr);
      nacc[q] = (nacc[q] << b) + (uint32_t)nc;
      if (METRICS) {
        const float d = xv - __builtin_fmaf((float)(-nc), scale, mn);
        e2 = __builtin_fmaf(d, d, e2);
        m2 = __builtin_fmaf(xv, xv, m2);
        v2 += sr_variance_term(rt);
      }
    }
  }
  nacc0 = nacc[0];
  nacc1 = nacc[1];
  if (METRICS) {
    *err = e2;
    *mag = m2;
    *var = (float)v2;
  }
}

// The same for a chunk of eight binary16 values taken straight from the loaded dwords: min - x is
// one mixed-precision fma per element (the widening conversion disappears into it).
template <bool EXACT2>
__device__ __forceinline__ void quantize_chunk_f16(const uint4& raw, float mn, float invs, uint32_t b,
                                                   const uint32_t* rnd, uint32_t& nacc0, uint32_t& nacc1) {
  const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
  uint32_t nacc[2] = {0u, 0u};
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const uint32_t rw = rnd[q];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t pair = w[q * 2 + (e >> 1)];
      const float d = (e & 1) ? min_minus_half<1>(pair, mn) : min_minus_half<0>(pair, mn);
      nacc[q] = (nacc[q] << b) + (uint32_t)neg_code_of_difference<EXACT2>(d, invs, (rw >> (8 * e)) & 0xFFu);
    }
  }
  nacc0 = nacc[0];
  nacc1 = nacc[1];
}

// binary16 tiles: one [-max : min] dword (two binary16 halves, daf_device.h) per (load, lane run)
// segment in stat[segment].x; nothing is widened.
template <int LPG_LOG2, int DIV>
__device__ __forceinline__ void tile_minmax_f16(const uint4 (&raw)[TileShape<kF16, LPG_LOG2, DIV>::kLoads], float2* stat,
                                                int lane) {
  using S = TileShape<kF16, LPG_LOG2, DIV>;
  static_assert(S::kLoads % 4 == 0, "loads are reduced four at a time");
#pragma unroll
  for (int u = 0; u < S::kLoads; u += 4) {
    uint32_t p[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) p[h] = chunk_stat_f16(raw[u + h]);
    seg_pk_min_x4<S::kLaneLog2>(p[0], p[1], p[2], p[3]);
    if ((lane & (S::kLpg - 1)) == S::kLpg - 1) {
#pragma unroll
      for (int h = 0; h < 4; ++h) stat[(u + h) * S::kGpl + (lane >> S::kLaneLog2)].x = u2f(p[h]);
    }
  }
}

// Widens the tile's chunks into xf and leaves one (min, max) pair per (load, lane run) segment
// in stat[load * runs_per_load + run]; a group's segments are consecutive entries.
template <int DT, int LPG_LOG2, int DIV = 1>
__device__ __forceinline__ void tile_minmax(const uint4 (&raw)[TileShape<DT, LPG_LOG2, DIV>::kLoads],
                                            float (&xf)[TileShape<DT, LPG_LOG2, DIV>::kLoads][ElemTraits<DT>::kPerLoad],
                                            float2* stat, int lane) {
  using S = TileShape<DT, LPG_LOG2, DIV>;
  constexpr int kEpl = S::kEpl;
  static_assert(S::kLoads % 2 == 0, "loads are reduced in pairs");
  if constexpr (DT == kF32 && LPG_LOG2 >= 5 && S::kLoads == 16) {
    // groups of 32 or 64 lanes: all 16 loads are reduced together (transposed reduction)
    float lmn[16], lmx[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
#pragma unroll
      for (int e = 0; e < kEpl; ++e) xf[u][e] = chunk_elem<DT>(raw[u], e);
      lmn[u] = vmin(vmin3(xf[u][0], xf[u][1], xf[u][2]), xf[u][3]);
      lmx[u] = vmax(vmax3(xf[u][0], xf[u][1], xf[u][2]), xf[u][3]);
    }
    float mn[2], mx[2];
    transposed_minmax16<S::kLaneLog2>(lmn, lmx, mn, mx);
    if ((lane & 3) == 0) {
      if (LPG_LOG2 >= 6) {
        stat[(lane >> 2) & 15] = make_float2(mn[0], mx[0]);
      } else {
        const int u = (lane >> 2) & 7, seg = lane >> 5;
        stat[u * 2 + seg] = make_float2(mn[0], mx[0]);
        stat[(u + 8) * 2 + seg] = make_float2(mn[1], mx[1]);
      }
    }
  } else {
    // two loads at a time so that four independent DPP chains interleave
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
      seg_minmax_x2<S::kLaneLog2>(mn[0], mx[0], mn[1], mx[1]);
      if ((lane & (S::kLpg - 1)) == S::kLpg - 1) {
        stat[u * S::kGpl + (lane >> S::kLaneLog2)] = make_float2(mn[0], mx[0]);
        stat[(u + 1) * S::kGpl + (lane >> S::kLaneLog2)] = make_float2(mn[1], mx[1]);
      }
    }
  }
}

// Drops the codes of one chunk (negated accumulators n0, n1 as quantize_chunk returns them) at
// byte address `addr` of the staged word run: a nibble pair, a byte, a halfword or whole words.
template <int EPL>
__device__ __forceinline__ void stage_chunk(uint8_t* stage8, uint32_t addr, uint32_t b, uint32_t n0, uint32_t n1,
                                            int lane);

// The same with `addr` an absolute LDS byte address (the staging area's own address already
// added in, once per group instead of once per store).
template <int EPL>
__device__ __forceinline__ void stage_chunk_at(uint32_t addr, uint32_t b, uint32_t n0, uint32_t n1, int lane) {
  typedef __attribute__((address_space(3))) uint8_t lds_u8;
  stage_chunk<EPL>((uint8_t*)(lds_u8*)(uintptr_t)addr, 0u, b, n0, n1, lane);
}

template <int EPL>
__device__ __forceinline__ void stage_chunk(uint8_t* stage8, uint32_t addr, uint32_t b, uint32_t n0, uint32_t n1,
                                            int lane) {
  if (EPL == 4) {
    const uint32_t acc = 0u - n0;
    if (b == 1u) {           // 4 bits per lane: the even lane takes its odd neighbour's nibble
      const uint32_t nb = dpp<kDppXor1>(acc, acc);
      if ((lane & 1) == 0) stage8[addr] = (uint8_t)((acc << 4) | nb);
    } else if (b == 2u) {
      stage8[addr] = (uint8_t)acc;
    } else if (b == 4u) {
      *reinterpret_cast<uint16_t*>(stage8 + addr) = (uint16_t)acc;
    } else {
      *reinterpret_cast<uint32_t*>(stage8 + addr) = acc;
    }
  } else {
    if (b == 8u) {
      *reinterpret_cast<uint2*>(stage8 + addr) = make_uint2(0u - n0, 0u - n1);
    } else {
      const uint32_t both = 0u - ((n0 << (4u * b)) + n1);
      if (b == 4u) {
        *reinterpret_cast<uint32_t*>(stage8 + addr) = both;
      } else if (b == 2u) {
        *reinterpret_cast<uint16_t*>(stage8 + addr) = (uint16_t)both;
      } else {
        stage8[addr] = (uint8_t)both;
      }
    }
  }
}

// B = 1, 2, 4, 8: every group has that width (offsets are computed).  B = 0: per-group widths
// from `bits`, offsets from `off`.
// One tile per wave; the hardware schedules the waves.  (A looping variant in which a wave
// prefetched its next tile while quantizing the current one was slower: it needs more
// registers, and on this architecture loads and stores share one in-order counter, so waiting
// for a prefetched load also waits for the stores issued after it.)
//
// EXT = true (only with the one-group-per-tile shape): the group is `tiles_per_group` tiles
// long and its (min, max) comes from `ext_stat`, computed by an earlier pass; the tile skips
// the reduction, and the group's first tile stores min and scale.
//
// METRICS = true: additionally writes, per group, the sums (x - xhat)^2 and x^2 over the group
// (binary32, accumulated per lane, then across the group's lanes, then across its loads) and the
// variance of the stochastic rounding, scale^2 * sum p (1 - p).
//
// RELU = true: x holds z; every element becomes max(z, +0) right after the load, the result is
// written to out_y in the same layout (out_y may be x itself: a lane only overwrites chunks it
// has already loaded), and everything else sees y.
template <int DT, int LPG_LOG2, int B, bool EXT = false, bool METRICS = false, bool RELU = false, int DIV = 1>
__device__ __forceinline__ void quantize_pack_tile_body(
    typename std::conditional<RELU, const u32x4*, const u32x4* __restrict__>::type x, int64_t tile, int wave_in_block,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, uint32_t seed_lo, uint32_t seed_hi,
    uint32_t* __restrict__ words, float* __restrict__ out_min, float* __restrict__ out_scale,
    const float2* __restrict__ ext_stat, int64_t tiles_per_group, float* __restrict__ out_metrics,
    u32x4* out_y) {
  using S = TileShape<DT, LPG_LOG2, DIV>;
  static_assert(!EXT || S::kGroups == 1, "external statistics: the tile is part of one group");
  static_assert(!(EXT && METRICS), "metrics are not computed for groups longer than a tile");
  static_assert(!(RELU && (EXT || METRICS)), "the fused max(z, 0) exists for the plain tile kernel only");
  constexpr int kEpl = S::kEpl;
  constexpr bool kMixed = (B == 0);
  constexpr uint32_t kGroupWords32 = S::kGroupSize / 32;      // words per group and bit of width
  __shared__ WaveLds<DT, LPG_LOG2, DIV> lds_all[kWavesPerBlock];

  const int lane = threadIdx.x & (kWave - 1);
  WaveLds<DT, LPG_LOG2, DIV>& lds = lds_all[wave_in_block];
  const uint32_t lane_in_run = (uint32_t)(lane & (S::kLpg - 1));
  // LDS byte address of the staging area (16-byte aligned, so the byte swizzles commute with it)
  const uint32_t stage_base = (uint32_t)reinterpret_cast<uintptr_t>(lds.stage);

  // 1. all global loads of the tile, issued up front
  uint4 raw[S::kLoads];
#pragma unroll
  for (int u = 0; u < S::kLoads; ++u) {
    const u32x4 v = __builtin_nontemporal_load(&x[tile * (S::kLoads * kWave) + u * kWave + lane]);
    raw[u] = make_uint4(v.x, v.y, v.z, v.w);
  }
  if constexpr (RELU) {
#pragma unroll
    for (int u = 0; u < S::kLoads; ++u) {
      raw[u] = make_uint4(relu_bits<DT>(raw[u].x), relu_bits<DT>(raw[u].y), relu_bits<DT>(raw[u].z),
                          relu_bits<DT>(raw[u].w));
      const u32x4 y = {raw[u].x, raw[u].y, raw[u].z, raw[u].w};
      out_y[tile * (S::kLoads * kWave) + u * kWave + lane] = y;    // the next layer reads it soon: cached store
    }
  }

  {
    // first group of the tile, and the tile's position inside it (EXT only)
    const int64_t g0 = EXT ? tile / tiles_per_group : tile * S::kGroups;
    const uint32_t tile_in_group = EXT ? (uint32_t)(tile - g0 * tiles_per_group) : 0u;

    uint32_t my_b = (uint32_t)B;
    uint32_t tile_base;
    if (kMixed) {
      my_b = (lane < S::kGroups) ? (uint32_t)bits[g0 + lane] : 1u;
      tile_base = off[g0];
      if (EXT) tile_base += tile_in_group * (kGroupWords32 * (uint32_t)__builtin_amdgcn_readfirstlane((int)my_b));
    } else {
      tile_base = (uint32_t)tile * (uint32_t)(S::kGroups * kGroupWords32 * B);
    }

    // The run is staged `head` words into the staging area, head = the word index of its first
    // word in the packed buffer modulo 4: 16-byte pieces of the two then coincide.
    const uint32_t head = ((uint32_t)(reinterpret_cast<uintptr_t>(words) >> 2) + tile_base) & 3u;

    // 2. random bytes of the tile (independent of the data; overlaps the loads' latency)
    {
      const uint64_t blk0 = (uint64_t)tile * (S::kElems / kElemsPerPhilox);
      uint4* dst = reinterpret_cast<uint4*>(lds.rand_bytes);
#pragma unroll
      for (int m = 0; m < S::kPhilox; ++m)
        dst[m * kWave + lane] = philox_block(blk0 + (uint64_t)(m * kWave + lane), seed_lo, seed_hi);
    }

    // 3. per-group min/max: in-lane over the chunk, then across the group's lanes.
    //    binary16 tiles stay in their loaded form: packed minimum / maximum on the pairs here, and
    //    the subtraction of step 5 widens on the fly (the metrics variant needs the widened values).
    constexpr bool kPairs16 = (DT == kF16) && !METRICS;
    float xf[kPairs16 ? 1 : S::kLoads][kEpl];
    if constexpr (kPairs16) {
      if constexpr (!EXT) tile_minmax_f16<LPG_LOG2, DIV>(raw, lds.stat, lane);
    } else if constexpr (EXT) {
#pragma unroll
      for (int u = 0; u < S::kLoads; ++u) {
#pragma unroll
        for (int e = 0; e < kEpl; ++e) xf[u][e] = chunk_elem<DT>(raw[u], e);
      }
    } else {
      tile_minmax<DT, LPG_LOG2, DIV>(raw, xf, lds.stat, lane);
    }
    wave_lds_sync();

    // 4. lane g of the wave finishes group g of the tile: scale, reciprocal, place in the run
    bool need_exact2;
    uint32_t tile_words;
    {
      float2 st;
      if constexpr (EXT) {
        st = ext_stat[g0];
      } else if constexpr (kPairs16) {
        uint32_t pk = f2u(lds.stat[(lane & (S::kGroups - 1)) * S::kLoadsPerGroup].x);
#pragma unroll
        for (int j = 1; j < S::kLoadsPerGroup; ++j)
          pk = pk_min_f16(pk, f2u(lds.stat[(lane & (S::kGroups - 1)) * S::kLoadsPerGroup + j].x));
        st = make_float2(stat_f16_min(pk), stat_f16_max(pk));
      } else {
        // the group's (load, lane run) segments are consecutive entries of stat
        st = lds.stat[(lane & (S::kGroups - 1)) * S::kLoadsPerGroup];
#pragma unroll
        for (int j = 1; j < S::kLoadsPerGroup; ++j) {
          const float2 t = lds.stat[(lane & (S::kGroups - 1)) * S::kLoadsPerGroup + j];
          st.x = vmin(st.x, t.x);
          st.y = vmax(st.y, t.y);
        }
      }
      const GroupScale s = group_scale(st.x, st.y, my_b);
      const float invs = s.inv * kScale;
      need_exact2 = __builtin_amdgcn_ballot_w64(!(invs <= 3.402823466e+38f) && lane < S::kGroups) != 0ull;
      uint32_t woff;
      if (kMixed) {
        const uint32_t w = (lane < S::kGroups) ? kGroupWords32 * my_b : 0u;
        const uint32_t incl = wave_inclusive_sum(w);
        tile_words = (uint32_t)__builtin_amdgcn_readlane((int)incl, kWave - 1);
        woff = incl - w;
      } else {
        tile_words = S::kGroups * kGroupWords32 * B;
        woff = (uint32_t)lane * (kGroupWords32 * B);
      }
      if (lane < S::kGroups) {
        if (!EXT || tile_in_group == 0u) {
          if (kMixed) {
            // Streaming stores: with many packed words per tile (wide codes) plain stores
            // of these two small runs slowed the whole kernel down measurably; with the
            // few words of uniform narrow codes they made no difference.
            __builtin_nontemporal_store(s.mn, &out_min[g0 + lane]);
            __builtin_nontemporal_store(s.scale, &out_scale[g0 + lane]);
          } else {
            out_min[g0 + lane] = s.mn;
            out_scale[g0 + lane] = s.scale;
          }
        }
        GroupInfo gi;
        gi.mn = s.mn;
        gi.invs = need_exact2 ? s.inv : invs;
        // A lane's bits are written as a byte (swizzle 3), a halfword (2) or whole words (0).
        const uint32_t lane_bits = (uint32_t)kEpl * my_b;
        const uint32_t swz = (lane_bits <= 8u) ? 3u : (lane_bits == 16u) ? 2u : 0u;
        gi.b = my_b | (swz << 8);
        gi.byte_off = stage_base + (woff + head) * 4u;
        lds.info[lane] = gi;
        if (METRICS) lds.gscale[lane] = s.scale;
      }
      if (METRICS) {
        wave_lds_sync();                       // every lane has read its (min, max) pairs
        lds.stat[lane] = make_float2(0.0f, 0.0f);
        lds.gvar[lane] = 0.0f;
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

    // 5. quantize every chunk and drop its bits at their place in the staged word run.
    //    The staged run is a big-endian bit string per word: byte k of the string lives at
    //    byte address k^3, halfword k at byte address 2k^2.
    //    (One copy of the loop per multiplication variant, chosen once per tile: the variant for
    //    groups whose reciprocal times 256 overflows is rare.)
    auto quantize_tile = [&](auto exact2) {
      constexpr bool kExact2 = decltype(exact2)::value;
#pragma unroll
      for (int u = 0; u < S::kLoads; ++u) {
        const int grp = (u * S::kGpl + (lane >> S::kLaneLog2)) / S::kLoadsPerGroup;
        // position of this lane's chunk among the chunks of its group
        const uint32_t lig = lane_in_run + (uint32_t)(u % S::kLoadsPerGroup) * kWave;
        float g_mn, g_invs;
        uint32_t b, addr;
        if (kMixed) {
          const GroupInfo gi = lds.info[grp];
          g_mn = gi.mn; g_invs = gi.invs; b = gi.b & 0xFFu;
          // byte address of this lane's bits: lig * (kEpl*b) bits = lig*b*kEpl/8 bytes
          addr = (gi.byte_off + ((lig * b * (uint32_t)kEpl) >> 3)) ^ (gi.b >> 8);
        } else {
          const float2 mi = *reinterpret_cast<const float2*>(&lds.info[grp]);
          g_mn = mi.x; g_invs = mi.y; b = B;
          constexpr uint32_t kLaneBits = (uint32_t)kEpl * B;
          constexpr uint32_t kSwz = (kLaneBits <= 8u) ? 3u : (kLaneBits == 16u) ? 2u : 0u;
          addr = (stage_base + head * 4u + (uint32_t)grp * (kGroupWords32 * B * 4u) + ((lig * kLaneBits) >> 3)) ^ kSwz;
        }
        uint32_t n0, n1;
        if constexpr (METRICS) {
          const float g_scale = lds.gscale[grp];
          float err, mag, var, unused = 0.0f;
          quantize_chunk<DT, kExact2, true>(xf[u], g_mn, g_invs, b, rnd[u], n0, n1, g_scale, &err, &mag, &var);
          seg_sum2<S::kLaneLog2>(err, mag);      // over the group's lanes of this load
          seg_sum2<S::kLaneLog2>(var, unused);
          if (lane_in_run == (uint32_t)S::kLpg - 1u) {
            const float2 acc = lds.stat[grp];    // the group's earlier loads (same lane, in order)
            lds.stat[grp] = make_float2(acc.x + err, acc.y + mag);
            lds.gvar[grp] += var;
          }
        } else if constexpr (kPairs16) {
          quantize_chunk_f16<kExact2>(raw[u], g_mn, g_invs, b, rnd[u], n0, n1);
        } else {
          quantize_chunk<DT, kExact2>(xf[u], g_mn, g_invs, b, rnd[u], n0, n1);
        }
        stage_chunk_at<kEpl>(addr, b, n0, n1, lane);
      }
    };
    if (need_exact2) quantize_tile(std::true_type{});
    else             quantize_tile(std::false_type{});
    wave_lds_sync();

    // 6. the tile's words are one contiguous run of the packed buffer; they leave in 16-byte
    //    pieces (single words at a ragged start or end) with streaming stores: the words are read
    //    back by the backward pass, long after they have left the caches (with ordinary stores
    //    the mixed-width kernels ran a tenth slower).
    {
      const uint32_t span = head + tile_words;
      uint32_t* dst = words + tile_base - head;                 // 16-byte aligned
      const uint32_t full_begin = (head + 3u) & ~3u, full_end = span & ~3u;
      for (uint32_t w0 = full_begin + (uint32_t)lane * 4u; w0 < full_end; w0 += kWave * 4u)
        __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(&lds.stage[w0]), reinterpret_cast<u32x4*>(dst + w0));
      // the up to three words before the first and after the last whole piece: lanes 0..3 and 4..7
      const uint32_t w = (lane < 4) ? (uint32_t)lane : full_end + (uint32_t)lane - 4u;
      if (lane < 8 && ((lane < 4) ? (w >= head && w < full_begin) : (w < span)))
        __builtin_nontemporal_store(lds.stage[w], dst + w);
    }
    if (METRICS && lane < S::kGroups) {
      const float sc = lds.gscale[lane];
      float* m = out_metrics + 3 * (g0 + lane);
      m[0] = lds.stat[lane].x;
      m[1] = lds.stat[lane].y;
      m[2] = (lds.gvar[lane] * 1.52587890625e-05f) * (sc * sc);
    }
  }
}

template <int DT, int LPG_LOG2, int B, bool EXT = false, bool METRICS = false, bool RELU = false, int DIV = 1>
__global__ __launch_bounds__(kThreads) void k_quantize_pack_tile(
    typename std::conditional<RELU, const u32x4*, const u32x4* __restrict__>::type x, int64_t n_tiles,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, uint32_t seed_lo, uint32_t seed_hi,
    uint32_t* __restrict__ words, float* __restrict__ out_min, float* __restrict__ out_scale,
    const float2* __restrict__ ext_stat, int64_t tiles_per_group, float* __restrict__ out_metrics,
    u32x4* out_y, int64_t n_elems, int64_t left_begin, int64_t left_end) {
  const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // When groups are left over after the last whole tile (left_begin .. left_end - 1, the tensor's
  // short last group among them) the grid has one more workgroup, the first, which quantizes
  // them the general way: no launch of their own, and they run while the tiles stream.
  const unsigned first_tile_block = (!EXT && left_end > left_begin) ? 1u : 0u;
  if constexpr (!EXT) {
    if (blockIdx.x < first_tile_block) {
      constexpr bool kCoop = !METRICS && TileShape<DT, LPG_LOG2>::kGroupSize >= 1024;
      quantize_pack_group_body<DT, METRICS, RELU, kCoop>(x, n_elems, TileShape<DT, LPG_LOG2>::kGroupSize, left_begin,
                                                         left_end, bits, off, B, seed_lo, seed_hi, words, out_min,
                                                         out_scale, out_metrics, out_y,
                                                         kCoop ? (int64_t)0 : (int64_t)wave_in_block,
                                                         kCoop ? (int64_t)1 : (int64_t)kWavesPerBlock);
      return;
    }
  }
  const int64_t tile = (int64_t)(blockIdx.x - first_tile_block) * kWavesPerBlock + wave_in_block;
  if (tile >= n_tiles) return;
  quantize_pack_tile_body<DT, LPG_LOG2, B, EXT, METRICS, RELU, DIV>(x, tile, wave_in_block, bits, off, seed_lo, seed_hi,
                                                                    words, out_min, out_scale, ext_stat,
                                                                    tiles_per_group, out_metrics, out_y);
}

// Several tensors in one launch (the activations a training step saves, Sec. 3.1): the tiles
// of all of them form one sequence, and a wave finds its tensor by walking the cumulative tile
// counts.  One launch has one ramp at its start and one tail at its end instead of one per
// tensor.  The descriptors travel as kernel arguments.
constexpr int kMaxBatch = 32;
struct BatchEntry {
  const void* x;
  const uint8_t* bits;
  const uint32_t* off;
  uint32_t* words;
  float* mn;
  float* sc;
  int64_t tile_end;                                 // tiles of this and all earlier entries
  uint32_t seed_lo, seed_hi;
};
struct Batch {
  uint32_t ends[kBatchSlots];                       // e[t].tile_end, 0xFFFFFFFF beyond n
  BatchEntry e[kMaxBatch];
  int32_t n;
  void clear() {
    n = 0;
    for (int i = 0; i < kBatchSlots; ++i) ends[i] = 0xFFFFFFFFu;
  }
};
static_assert(kMaxBatch <= kBatchSlots, "one cumulative count per entry");

template <int DT, int LPG_LOG2, int B>
__global__ __launch_bounds__(kThreads) void k_quantize_pack_tile_batch(const Batch batch) {
  const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t gtile = (int64_t)blockIdx.x * kWavesPerBlock + wave_in_block;
  const int t = batch_entry_of(batch.ends, (uint32_t)gtile);
  if (t >= batch.n) return;                          // past the last tile (the grid is whole workgroups)
  const BatchEntry& e = batch.e[t];
  const int64_t tile = gtile - (t ? batch.e[t - 1].tile_end : 0);
  quantize_pack_tile_body<DT, LPG_LOG2, B, false, false, false, tile_div<DT, LPG_LOG2>()>(
      static_cast<const u32x4*>(e.x), tile, wave_in_block, e.bits, e.off, e.seed_lo, e.seed_hi, e.words, e.mn, e.sc,
      nullptr, (int64_t)1, nullptr, nullptr);
}

template <int DT, int LPG_LOG2, bool METRICS, bool RELU>
hipError_t launch_tile(const daf_plan_t* p, const void* x, int64_t n_tiles, uint32_t seed_lo, uint32_t seed_hi,
                       uint32_t* out_words, float* out_min, float* out_scale, float* out_metrics, void* out_y,
                       hipStream_t stream) {
  using S = QTile<DT, LPG_LOG2>;
  const int64_t left = n_tiles * S::kGroups;                         // first group after the whole tiles
#define DAF_LAUNCH(BITS)                                                                                   \
  do {                                                                                                     \
    auto kernel = k_quantize_pack_tile<DT, LPG_LOG2, BITS, false, METRICS, RELU, tile_div<DT, LPG_LOG2>()>; \
    const unsigned blocks = (unsigned)((n_tiles + kWavesPerBlock - 1) / kWavesPerBlock) + (left < p->num_groups ? 1u : 0u); \
    hipLaunchKernelGGL(kernel, dim3(blocks), dim3(kThreads), 0, stream, static_cast<const u32x4*>(x),      \
                       n_tiles, p->d_bits, p->d_off, seed_lo, seed_hi, out_words, out_min, out_scale,      \
                       nullptr, (int64_t)1, out_metrics, static_cast<u32x4*>(out_y), p->n, left,           \
                       p->num_groups);                                                                     \
  } while (0)
  switch (p->uniform_bits) {
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

}  // namespace
