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
#include <type_traits>

#include "daf_device.h"
#include "daf_internal.h"

namespace {

using namespace daf;

constexpr int kWavesPerBlock = 4;
constexpr int kThreads = kWave * kWavesPerBlock;
constexpr float kScale = 256.0f;            // 2^kRandBits
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct GroupScale {
  float mn, scale, inv;
};

// Eq. 1 (left) per group, plus the reciprocal used for the per-element map.
__device__ __forceinline__ GroupScale group_scale(float mn, float mx, uint32_t b) {
  GroupScale s;
  s.mn = mn + 0.0f;                               // a zero minimum is stored as +0
  const float mxc = mx + 0.0f;
  const float L = (float)((1u << b) - 1u);
  const float range = mxc - s.mn;
  s.scale = range / L;
  float inv = 0.0f;
  if (range > 0.0f) {
    inv = L / range;
    if (!(inv <= 3.402823466e+38f)) inv = 0.0f;   // reciprocal overflowed
  }
  s.inv = inv;
  return s;
}

// Negated code of one element.  EXACT2 = false: invs = inv*256 (finite).  EXACT2 = true:
// invs = inv, and the factor 256 is applied to the rounded product.
template <bool EXACT2>
__device__ __forceinline__ int neg_code_of_difference(float d, float invs, uint32_t r) {   // d = mn - x
  float w = d * invs;
  if (EXACT2) w = w * kScale;
  return (round_half_up_to_int(w) + (int)r) >> 8;
}

template <bool EXACT2>
__device__ __forceinline__ int neg_code(float x, float mn, float invs, uint32_t r, int* t_out = nullptr) {
  float w = (mn - x) * invs;
  if (EXACT2) w = w * kScale;
  const int t = round_half_up_to_int(w);            // -(256*floor(v) + T), T = byte values that round up
  if (t_out) *t_out = t;
  return (t + (int)r) >> 8;
}

// T * (256 - T) for the element whose rounded product is t: 65536 * p * (1 - p) with p = T / 256
// the probability of rounding up (T = 256, always up, reads as 0 here: the same product).
__device__ __forceinline__ uint32_t sr_variance_term(int t) {
  const uint32_t T = (uint32_t)(-t) & 255u;
  return T * (256u - T);
}

// max(x, +0) on the raw bits of one 32-bit word (one binary32 value or two 16-bit values):
// a value whose sign bit is set (negative, or -0) is a negative integer and becomes +0, any
// other value is kept; for finite inputs that is x > 0 ? x : +0 exactly.
template <int DT>
__device__ __forceinline__ uint32_t relu_bits(uint32_t w) {
  if (DT == kF32) {
    const int32_t v = (int32_t)w;
    return (uint32_t)(v > 0 ? v : 0);
  }
  typedef short short2v __attribute__((ext_vector_type(2)));
  const short2v v = __builtin_bit_cast(short2v, w);
  const short2v zero = {0, 0};
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(v, zero));
}

// ------------------------------------------------------------------------------------------
// General path: one wave per group.
// ------------------------------------------------------------------------------------------
template <int DT, bool RELU = false>
__device__ __forceinline__ float load_elem(const void* x, int64_t i) {
  float v;
  if (DT == kF32) v = static_cast<const float*>(x)[i];
  else v = widen16<DT == kF32 ? kF16 : DT>(static_cast<const uint16_t*>(x)[i]);
  if (RELU) v = v > 0.0f ? v : 0.0f;
  return v;
}
template <int DT>
__device__ __forceinline__ void store_elem(void* y, int64_t i, float v) {   // v is a value of the format
  if (DT == kF32) static_cast<float*>(y)[i] = v;
  else static_cast<uint16_t*>(y)[i] = (uint16_t)(DT == kBF16 ? f2u(v) >> 16 : narrow16<DT == kF32 ? kF16 : DT>(v));
}

// RELU = true: the input is z, every element is replaced by max(z, +0) before anything else, and
// the result is also written to out_y (which may be the input buffer itself).
//
// COOP = true: the four waves of a workgroup share one group (long groups, of which a call
// usually has one: the tensor's short last group); the loops below then stride by the
// workgroup and the waves exchange their (min, max) through LDS.
// `wave` of `n_waves`: this wave's (COOP: this workgroup's) place among those that share the
// groups g_begin .. g_end - 1.
template <int DT, bool METRICS = false, bool RELU = false, bool COOP = false>
__device__ __forceinline__ void quantize_pack_group_body(
    const void* x, int64_t n, int32_t gs, int64_t g_begin, int64_t g_end,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, int32_t uniform_bits,
    uint32_t seed_lo, uint32_t seed_hi, uint32_t* __restrict__ words, float* __restrict__ out_min,
    float* __restrict__ out_scale, float* __restrict__ out_metrics, void* out_y, int64_t wave, int64_t n_waves) {
  static_assert(!(COOP && METRICS), "the metrics sums are reduced inside one wave");
  const int kStride = COOP ? (int)blockDim.x : kWave;        // threads that share a group (COOP: any workgroup size)
  __shared__ float2 coop_stat[16];
  const int lane = COOP ? (int)threadIdx.x : (int)(threadIdx.x & (kWave - 1));   // index among them
  for (int64_t g = g_begin + wave; g < g_end; g += n_waves) {
    const int64_t lo = g * (int64_t)gs;
    const int32_t len = (int32_t)((lo + gs <= n) ? gs : (n - lo));
    const uint32_t b = uniform_bits ? (uint32_t)uniform_bits : (uint32_t)bits[g];
    const uint32_t woff = uniform_bits ? (uint32_t)(g * (((int64_t)gs * uniform_bits) >> 5)) : off[g];

    float mn = load_elem<DT, RELU>(x, lo), mx = mn;        // element 0 exists in every group
    for (int32_t j0 = lane; j0 < len; j0 += 8 * kStride) {  // eight loads in flight per lane
      float v[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int32_t j = j0 + q * kStride;
        v[q] = load_elem<DT, RELU>(x, lo + (j < len ? j : j0));
      }
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int32_t j = j0 + q * kStride;
        if (RELU && j < len) store_elem<DT>(out_y, lo + j, v[q]);   // every element passes here exactly once
        mn = fminf(mn, v[q]);
        mx = fmaxf(mx, v[q]);
      }
    }
    for (int o = 32; o > 0; o >>= 1) {
      mn = fminf(mn, __shfl_xor(mn, o));
      mx = fmaxf(mx, __shfl_xor(mx, o));
    }
    if (COOP) {
      // (the barrier also orders the y written above before the reads below: in place, a thread
      // re-reads elements that another wave has replaced by max(z, +0))
      if ((threadIdx.x & (kWave - 1)) == 0) coop_stat[threadIdx.x >> 6] = make_float2(mn, mx);
      __syncthreads();
      for (int w = 0; w < (int)(blockDim.x >> 6); ++w) {
        mn = fminf(mn, coop_stat[w].x);
        mx = fmaxf(mx, coop_stat[w].y);
      }
      __syncthreads();                                     // before the next group overwrites the pairs
    }
    const GroupScale s = group_scale(mn, mx, b);
    if (lane == 0) {
      out_min[g] = s.mn;
      out_scale[g] = s.scale;
    }
    const uint32_t cpw = 32u / b;                          // codes per word
    const int32_t n_words = (int32_t)(((int64_t)len * b + 31) >> 5);
    float err = 0.0f, mag = 0.0f;
    uint32_t var_i = 0u;
    // A word's codes are taken 16 elements at a time (one Philox block; a word of 1-bit codes
    // takes two rounds): all loads of a round are issued before any is used, so a lone long
    // group costs one memory latency per round and not one per element.
    const int32_t per_round = (int32_t)(cpw < 16u ? cpw : 16u);
    for (int32_t t = lane; t < n_words; t += kStride) {
      uint32_t word = 0;
      for (int32_t c0 = 0; c0 < (int32_t)cpw; c0 += 16) {
        const int32_t j0 = t * (int32_t)cpw + c0;            // a multiple of per_round
        if (j0 >= len) break;
        const uint64_t i0 = (uint64_t)(lo + j0);
        const uint4 rnd = philox_block(i0 / kElemsPerPhilox, seed_lo, seed_hi);
        const uint32_t slot0 = (uint32_t)(i0 % kElemsPerPhilox);
        float xv[16];
#pragma unroll
        for (int c = 0; c < 16; ++c)
          xv[c] = (c < per_round && j0 + c < len) ? load_elem<DT, RELU>(x, lo + j0 + c) : 0.0f;   // z or y: max(., +0) gives y either way
#pragma unroll
        for (int c = 0; c < 16; ++c) {
          if (c < per_round && j0 + c < len) {
            const uint32_t slot = slot0 + (uint32_t)c;
            const uint32_t rw = (slot < 4) ? rnd.x : (slot < 8) ? rnd.y : (slot < 12) ? rnd.z : rnd.w;
            const uint32_t r = (rw >> (8u * (slot & 3u))) & 0xFFu;
            int rt;
            const int nc = neg_code<true>(xv[c], s.mn, s.inv, r, &rt);
            word |= (uint32_t)(-nc) << (32u - b - (uint32_t)(c0 + c) * b);
            if (METRICS) {
              const float d = xv[c] - __builtin_fmaf((float)(-nc), s.scale, s.mn);
              err = __builtin_fmaf(d, d, err);
              mag = __builtin_fmaf(xv[c], xv[c], mag);
              var_i += sr_variance_term(rt);
            }
          }
        }
      }
      words[woff + t] = word;
    }
    if (METRICS) {
      float var = (float)var_i, unused = 0.0f;
      seg_sum2<6>(err, mag);
      seg_sum2<6>(var, unused);
      if (lane == kWave - 1) {
        out_metrics[3 * g] = err;
        out_metrics[3 * g + 1] = mag;
        out_metrics[3 * g + 2] = (var * 1.52587890625e-05f) * (s.scale * s.scale);
      }
    }
  }
}

template <int DT, bool METRICS = false, bool RELU = false, bool COOP = false>
__global__ __launch_bounds__(kThreads) void k_quantize_pack_group(
    const void* x, int64_t n, int32_t gs, int64_t g_begin, int64_t g_end,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, int32_t uniform_bits,
    uint32_t seed_lo, uint32_t seed_hi, uint32_t* __restrict__ words, float* __restrict__ out_min,
    float* __restrict__ out_scale, float* __restrict__ out_metrics, void* out_y) {
  const int64_t wave = COOP ? (int64_t)blockIdx.x : (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  const int64_t n_waves = COOP ? (int64_t)gridDim.x : (int64_t)gridDim.x * kWavesPerBlock;
  quantize_pack_group_body<DT, METRICS, RELU, COOP>(x, n, gs, g_begin, g_end, bits, off, uniform_bits, seed_lo, seed_hi,
                                                    words, out_min, out_scale, out_metrics, out_y, wave, n_waves);
}

// The leftovers of several tensors in one launch (list calls): one workgroup per entry takes the
// entry's groups g_begin .. g_end - 1, its four waves a group each or (COOP) all four together.
struct GroupBatchEntry {
  const void* x;
  const uint8_t* bits;
  const uint32_t* off;
  uint32_t* words;
  float* mn;
  float* sc;
  int64_t n, g_begin, g_end;
  int32_t gs, uniform_bits;
  uint32_t seed_lo, seed_hi;
};
struct GroupBatch {
  GroupBatchEntry e[32];
  int32_t n;
};

template <int DT, bool COOP>
__global__ __launch_bounds__(kThreads) void k_quantize_pack_group_batch(const GroupBatch batch) {
  const GroupBatchEntry& e = batch.e[blockIdx.x];
  quantize_pack_group_body<DT, false, false, COOP>(e.x, e.n, e.gs, e.g_begin, e.g_end, e.bits, e.off, e.uniform_bits,
                                                   e.seed_lo, e.seed_hi, e.words, e.mn, e.sc, nullptr, nullptr,
                                                   COOP ? (int64_t)0 : (int64_t)(threadIdx.x >> 6),
                                                   COOP ? (int64_t)1 : (int64_t)kWavesPerBlock);
}

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
