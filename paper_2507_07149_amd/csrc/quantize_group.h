// Route "group": one wave (or workgroup) per group with element loads: whatever the other routes
// leave over (groups after the last whole tile, the tensor's short last group).
#pragma once
#include "quantize_common.h"

namespace {

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

}  // namespace
