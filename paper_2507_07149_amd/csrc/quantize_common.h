// Shared by the quantize kernels of every route: launch shape, Eq. 1 per group (scale and the
// reciprocal used by the element map), the negated element map itself, the fused max(z, 0).
// Included by quantize_pack.hip only (once per element format).
#pragma once
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

}  // namespace
