// Route "long": groups of 4128 ... 65536 elements, one workgroup per group.
#pragma once
#include "quantize_common.h"
#include "quantize_units.h"

namespace {

// Long groups, 128 < m <= 2048 units (4096 < group size <= 65536 elements, e.g. a row of
// 11008): one workgroup per group, one wave per slice of at most 128 units.  Every wave keeps
// its slice in registers, the waves exchange their (min, max) through LDS, and each then
// quantizes and writes its part of the group's words: the activation is read once.
struct LongWaveLds {
  union {
    uint8_t rand_bytes[4096];
    uint32_t stage[1024];
  };
};
constexpr int kLongMaxWaves = 16;

template <int DT, int B, bool RELU = false, bool METRICS = false>
__device__ __forceinline__ void quantize_pack_long_body(
    typename std::conditional<RELU, const u32x4*, const u32x4* __restrict__>::type x, int64_t g, int32_t m,
    int32_t units_per_wave, const uint8_t* __restrict__ bits,
    const uint32_t* __restrict__ off, uint32_t seed_lo, uint32_t seed_hi, uint32_t* __restrict__ words,
    float* __restrict__ out_min, float* __restrict__ out_scale, u32x4* out_y, float* __restrict__ out_metrics) {
  using S = UnitShape<DT>;
  static_assert(!(RELU && METRICS), "the fused max(z, 0) and the fused metrics are separate variants");
  constexpr int kEpl = S::kEpl;
  constexpr bool kMixed = (B == 0);
  // n_waves slices, then 16 bytes per wave for its (min, max), then (METRICS) 16 per wave for its sums
  extern __shared__ __align__(16) uint8_t dyn_lds[];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n_waves = (int)(blockDim.x >> 6);
  LongWaveLds& lds = reinterpret_cast<LongWaveLds*>(dyn_lds)[wave];
  float4* wstat = reinterpret_cast<float4*>(dyn_lds + (size_t)n_waves * sizeof(LongWaveLds));   // 16 bytes per wave
  uint8_t* stage8 = reinterpret_cast<uint8_t*>(lds.stage);

  const int32_t unit0 = wave * units_per_wave;               // first unit of this wave's slice
  const uint32_t units = (uint32_t)((m - unit0 < units_per_wave) ? m - unit0 : units_per_wave);   // >= 1
  const uint32_t n_chunks = units << S::kLanesLog2;
  const int64_t first_unit = g * m + unit0;                  // in the tensor
  const int64_t chunk0 = first_unit << S::kLanesLog2;

  // 1. all global loads of the slice, issued up front
  uint4 raw[S::kLoads];
  unit_tile_load<DT>(x, chunk0, n_chunks, lane, raw);
  if constexpr (RELU) unit_tile_relu<DT>(raw, out_y, chunk0, n_chunks, lane);
  const uint32_t b = kMixed ? (uint32_t)bits[g] : (uint32_t)B;
  const uint32_t group_base = kMixed ? off[g] : (uint32_t)g * ((uint32_t)m * (uint32_t)B);

  // 2. random bytes of the slice (two Philox blocks per unit)
  {
    const uint64_t blk0 = (uint64_t)first_unit * 2u;
    uint4* dst = reinterpret_cast<uint4*>(lds.rand_bytes);
#pragma unroll
    for (int q = 0; q < S::kPhilox; ++q) {
      const uint32_t i = (uint32_t)(q * kWave + lane);
      if (i < units * 2u) dst[i] = philox_block(blk0 + i, seed_lo, seed_hi);
    }
  }

  // 3. min/max of the slice, then of the group
  float xf[S::kLoads][kEpl];
  {
    float a[2], c2[2];
#pragma unroll
    for (int u = 0; u < S::kLoads; ++u) {
#pragma unroll
      for (int e = 0; e < kEpl; ++e) xf[u][e] = chunk_elem<DT>(raw[u], e);
      const float(&v)[kEpl] = xf[u];
      float lo = vmin(vmin3(v[0], v[1], v[2]), v[3]), hi = vmax(vmax3(v[0], v[1], v[2]), v[3]);
      if (kEpl == 8) {
        lo = vmin3(lo, vmin3(v[4 % kEpl], v[5 % kEpl], v[6 % kEpl]), v[7 % kEpl]);
        hi = vmax3(hi, vmax3(v[4 % kEpl], v[5 % kEpl], v[6 % kEpl]), v[7 % kEpl]);
      }
      a[u & 1] = (u < 2) ? lo : vmin(a[u & 1], lo);
      c2[u & 1] = (u < 2) ? hi : vmax(c2[u & 1], hi);
    }
    seg_minmax_x2<6>(a[0], c2[0], a[1], c2[1]);
    if (lane == kWave - 1) wstat[wave] = make_float4(vmin(a[0], a[1]), vmax(c2[0], c2[1]), 0.0f, 0.0f);
  }
  __syncthreads();
  float2 st = make_float2(wstat[0].x, wstat[0].y);
  for (int w = 1; w < n_waves; ++w) {
    const float4 t = wstat[w];
    st.x = vmin(st.x, t.x);
    st.y = vmax(st.y, t.y);
  }
  const GroupScale s = group_scale(st.x, st.y, b);
  float invs = s.inv * kScale;
  const bool need_exact2 = !(invs <= 3.402823466e+38f);
  if (need_exact2) invs = s.inv;
  if (threadIdx.x == 0) {
    out_min[g] = s.mn;
    out_scale[g] = s.scale;
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

  // 5. quantize every chunk of the slice and drop its bits at their place in the staged run
  float m_err = 0.0f, m_mag = 0.0f, m_var = 0.0f;            // METRICS: this lane's share of the group's sums
  const uint32_t lane_bits = (uint32_t)kEpl * b;
  const uint32_t swz = (lane_bits <= 8u) ? 3u : (lane_bits == 16u) ? 2u : 0u;
#pragma unroll
  for (int u = 0; u < S::kLoads; ++u) {
    const uint32_t c = (uint32_t)(u * kWave + lane);
    if (c < n_chunks) {
      const uint32_t addr = (__umul24(c, lane_bits) >> 3) ^ swz;
      uint32_t n0, n1;
      if constexpr (METRICS) {
        float err, mag, var;
        if (need_exact2) quantize_chunk<DT, true, true>(xf[u], s.mn, invs, b, rnd[u], n0, n1, s.scale, &err, &mag, &var);
        else             quantize_chunk<DT, false, true>(xf[u], s.mn, invs, b, rnd[u], n0, n1, s.scale, &err, &mag, &var);
        m_err += err;
        m_mag += mag;
        m_var += var;
      } else {
        if (need_exact2) quantize_chunk<DT, true>(xf[u], s.mn, invs, b, rnd[u], n0, n1);
        else             quantize_chunk<DT, false>(xf[u], s.mn, invs, b, rnd[u], n0, n1);
      }
      stage_chunk<kEpl>(stage8, addr, b, n0, n1, lane);
    }
  }
  wave_lds_sync();

  // 6. the slice's words are one contiguous run inside the group's
  uint32_t* dst = words + group_base + (uint32_t)unit0 * b;
  const uint32_t slice_words = units * b;
  for (uint32_t i = lane; i < slice_words; i += kWave) __builtin_nontemporal_store(lds.stage[i], &dst[i]);

  if constexpr (METRICS) {
    // per lane over its chunks, across the wave, then across the waves in a fixed order
    float unused = 0.0f;
    seg_sum2<6>(m_err, m_mag);
    seg_sum2<6>(m_var, unused);
    float4* wsum = wstat + n_waves;
    if (lane == kWave - 1) wsum[wave] = make_float4(m_err, m_mag, m_var, 0.0f);
    __syncthreads();
    if (threadIdx.x == 0) {
      float e = 0.0f, q = 0.0f, v = 0.0f;
      for (int w = 0; w < n_waves; ++w) {
        e += wsum[w].x;
        q += wsum[w].y;
        v += wsum[w].z;
      }
      out_metrics[3 * g] = e;
      out_metrics[3 * g + 1] = q;
      out_metrics[3 * g + 2] = (v * 1.52587890625e-05f) * (s.scale * s.scale);
    }
  }
}

// Takes plans whose groups are 32 * m elements, 128 < m <= 2048, when there are enough groups to
// fill the device with one workgroup each, or when the two-pass route does not apply (groups
// not a whole number of tiles).  Returns the groups it covered (all whole groups, or none).
template <int DT, int B, bool RELU = false, bool METRICS = false>
__global__ __launch_bounds__(kWave * kLongMaxWaves) void k_quantize_pack_long(
    typename std::conditional<RELU, const u32x4*, const u32x4* __restrict__>::type x, int32_t m,
    int32_t units_per_wave, const uint8_t* __restrict__ bits,
    const uint32_t* __restrict__ off, uint32_t seed_lo, uint32_t seed_hi, uint32_t* __restrict__ words,
    float* __restrict__ out_min, float* __restrict__ out_scale, u32x4* out_y, float* __restrict__ out_metrics,
    int64_t n_elems, int64_t full_groups) {
  // When the tensor has a short last group the grid has one more workgroup, the first, which
  // quantizes that group the general way: no launch of its own, and its chain of dependent loads
  // runs while the whole groups stream.
  const unsigned first_group_block = gridDim.x > (unsigned)full_groups ? 1u : 0u;
  if (blockIdx.x < first_group_block) {
    quantize_pack_group_body<DT, METRICS, RELU, !METRICS>(x, n_elems, m * 32, full_groups, full_groups + 1, bits, off, B,
                                                          seed_lo, seed_hi, words, out_min, out_scale, out_metrics, out_y,
                                                          METRICS ? (int64_t)(threadIdx.x >> 6) : (int64_t)0,
                                                          METRICS ? (int64_t)(blockDim.x >> 6) : (int64_t)1);
    return;
  }
  quantize_pack_long_body<DT, B, RELU, METRICS>(x, (int64_t)(blockIdx.x - first_group_block), m, units_per_wave, bits,
                                                off, seed_lo, seed_hi, words, out_min, out_scale, out_y, out_metrics);
}

// Several tensors in one launch: the groups of all entries form one sequence of workgroups.  The
// entries of a launch have the same number of waves per group (the workgroup size).
struct LongBatchEntry {
  const void* x;
  const uint8_t* bits;
  const uint32_t* off;
  uint32_t* words;
  float* mn;
  float* sc;
  int64_t group_end;                                // whole groups of this and all earlier entries
  uint32_t seed_lo, seed_hi;
  int32_t m, units_per_wave;
};
struct LongBatch {
  LongBatchEntry e[kMaxBatch];
  int32_t n;
};

template <int DT, int B>
__global__ __launch_bounds__(kWave * kLongMaxWaves) void k_quantize_pack_long_batch(const LongBatch batch) {
  const int64_t gg = blockIdx.x;                    // < batch.e[batch.n - 1].group_end: the grid is exactly that
  int t = 0;
  while (gg >= batch.e[t].group_end) ++t;           // uniform over the workgroup
  const LongBatchEntry& e = batch.e[t];
  quantize_pack_long_body<DT, B>(static_cast<const u32x4*>(e.x), gg - (t ? batch.e[t - 1].group_end : 0), e.m,
                                 e.units_per_wave, e.bits, e.off, e.seed_lo, e.seed_hi, e.words, e.mn, e.sc, nullptr,
                                 nullptr);
}

inline bool long_applies(const daf_plan_t* p) {
  const int32_t gs = p->group_size;
  const int32_t m = gs / 32;
  if (gs % 32 != 0 || m <= 128 || m > 128 * kLongMaxWaves) return false;
  const int64_t full_groups = p->n / gs;
  if (full_groups == 0 || full_groups >= 0x7fffffff) return false;
  if (p->d_big_scratch != nullptr && full_groups < 256) return false;          // the two-pass route fills the device better
  return true;
}

template <int DT, bool RELU, bool METRICS>
hipError_t launch_long(const daf_plan_t* p, const void* x, uint32_t seed_lo, uint32_t seed_hi, uint32_t* out_words,
                       float* out_min, float* out_scale, void* out_y, float* out_metrics, int64_t* covered,
                       hipStream_t stream) {
  *covered = 0;
  if (!long_applies(p)) return hipSuccess;
  const int32_t gs = p->group_size;
  const int32_t m = gs / 32;
  const int64_t full_groups = p->n / gs;
  const int32_t n_waves = (m + 127) / 128;
  const int32_t units_per_wave = (m + n_waves - 1) / n_waves;
  const unsigned lds_bytes = (unsigned)(n_waves * (sizeof(LongWaveLds) + sizeof(float4) + (METRICS ? sizeof(float4) : 0)));
  const unsigned blocks = (unsigned)full_groups + (p->num_groups > full_groups ? 1u : 0u);   // + the short last group
#define DAF_LAUNCH(BITS)                                                                                          \
  hipLaunchKernelGGL((k_quantize_pack_long<DT, BITS, RELU, METRICS>), dim3(blocks),                               \
                     dim3(kWave * n_waves), lds_bytes, stream, static_cast<const u32x4*>(x), m, units_per_wave,   \
                     p->d_bits, p->d_off, seed_lo, seed_hi, out_words, out_min, out_scale,                        \
                     static_cast<u32x4*>(out_y), out_metrics, p->n, full_groups)
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
