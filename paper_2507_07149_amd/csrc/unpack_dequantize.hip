// Backward-pass side: unpack the codes (the extraction rule of Algorithm 2, for the group's
// own width) and dequantize them to the original precision, xhat = fma(code, scale, min)
// (inverse of Eq. 1; paper Sec. 2.2).  Two kernels:
//
//   k_unpack_dequantize_chunk  the fast path.  A thread produces 16 bytes of output at a time
//                              (4 fp32 or 8 16-bit elements).  Such a chunk never straddles a
//                              group and its bits never straddle a word pair, so it needs one
//                              (or, at 8 bits and 16-bit output, two) packed words.  Covers every
//                              whole chunk of the tensor, for any group size.
//   k_unpack_dequantize_tail   the fewer than 8 elements after the last whole chunk (list calls; a
//                              single-tensor call gives them to one more workgroup of the main launch).
//
// RELU_BWD = true turns both into the backward of y = max(z, 0) whose output y was the saved
// activation: instead of xhat the kernels write grad_z = (xhat > 0) ? grad_y : +0, with xhat
// rounded to the element format first, so the result is what a threshold on the materialised
// xhat would give, and xhat itself never reaches memory.
#include "daf_device.h"
#include "daf_internal.h"

namespace {

using namespace daf;

constexpr int kThreads = 256;
// 16-byte chunks per thread: 8, so that the small dependent loads of eight chunks (widths and
// offsets first, then the words) are in flight together.  Measured with the packed inputs coming
// from HBM, as they do in a backward pass (tensors rotating over more than the memory-side
// cache holds): 1 / 2 / 4 / 8 chunks with one width for all groups take 46.7 / 45.3 / 41.7 /
// 41.9 us on a 51 M-element binary32 tensor.  (With the 14 MB of packed input left in that cache
// by the previous launch, one chunk per thread looks best, 32.5 us: a measurement artefact.)
#ifndef DAF_DEQ_CHUNKS_UNIFORM
#define DAF_DEQ_CHUNKS_UNIFORM 8
#endif
#ifndef DAF_DEQ_CHUNKS_MIXED
#define DAF_DEQ_CHUNKS_MIXED 8
#endif
constexpr int chunks_per_thread(bool mixed) { return mixed ? DAF_DEQ_CHUNKS_MIXED : DAF_DEQ_CHUNKS_UNIFORM; }
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int DT>
__device__ __forceinline__ void store_elem(void* out, int64_t i, float v) {
  if (DT == kF32) static_cast<float*>(out)[i] = v;
  else static_cast<uint16_t*>(out)[i] = (uint16_t)narrow16<DT == kF32 ? kF16 : DT>(v);
}

// Positive in the element format: the pattern read as a signed integer is > 0 (finite values).
template <int DT>
__device__ __forceinline__ uint32_t keep_where_positive(uint32_t xhat_word, uint32_t grad_word) {
  if (DT == kF32) return ((int32_t)xhat_word > 0) ? grad_word : 0u;
  const uint32_t lo = ((int16_t)(uint16_t)(xhat_word & 0xFFFFu) > 0) ? (grad_word & 0xFFFFu) : 0u;
  const uint32_t hi = ((int16_t)(uint16_t)(xhat_word >> 16) > 0) ? (grad_word & 0xFFFF0000u) : 0u;
  return lo | hi;
}

// The last elements of the tensor, [e_begin, n) with n - e_begin < 8: all in the last group.
template <int DT, bool RELU_BWD>
__device__ __forceinline__ void unpack_dequantize_tail_body(
    const uint32_t* __restrict__ words, const float* __restrict__ mn, const float* __restrict__ scale,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, int32_t uniform_bits, int64_t e_begin,
    int64_t n, int32_t gs, void* out, const void* grad) {
  const int64_t i = e_begin + threadIdx.x;
  if (i >= n) return;
  const int64_t g = i / gs;
  const uint32_t b = uniform_bits ? (uint32_t)uniform_bits : (uint32_t)bits[g];
  const uint32_t woff = uniform_bits ? (uint32_t)(g * (((int64_t)gs * uniform_bits) >> 5)) : off[g];
  const uint64_t bitpos = (uint64_t)(i - g * (int64_t)gs) * b;
  const uint32_t w = words[woff + (bitpos >> 5)];
  const uint32_t code = (w >> (32u - b - (uint32_t)(bitpos & 31u))) & ((1u << b) - 1u);
  const float v = __builtin_fmaf((float)code, scale[g], mn[g]);
  if (RELU_BWD) {
    if (DT == kF32) {
      const uint32_t gw = static_cast<const uint32_t*>(grad)[i];
      static_cast<uint32_t*>(out)[i] = keep_where_positive<DT>(f2u(v), gw);
    } else {
      const uint32_t gw = static_cast<const uint16_t*>(grad)[i];
      const uint32_t xh = narrow16<DT == kF32 ? kF16 : DT>(v);
      static_cast<uint16_t*>(out)[i] = (uint16_t)keep_where_positive<DT>(xh, gw);
    }
  } else {
    store_elem<DT>(out, i, v);
  }
}

template <int DT, bool RELU_BWD>
__global__ __launch_bounds__(kWave) void k_unpack_dequantize_tail(
    const uint32_t* __restrict__ words, const float* __restrict__ mn, const float* __restrict__ scale,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, int32_t uniform_bits, int64_t e_begin,
    int64_t n, int32_t gs, void* out, const void* grad) {
  unpack_dequantize_tail_body<DT, RELU_BWD>(words, mn, scale, bits, off, uniform_bits, e_begin, n, gs, out, grad);
}

// The loop over a thread's chunks is split into phases (metadata loads, word loads,
// arithmetic + stores) so that all loads of one phase are in flight together: with per-group
// widths the word address depends on two earlier loads, and a chunk-by-chunk loop would pay
// that latency once per chunk.
template <int DT, bool MIXED, bool RELU_BWD>
__device__ __forceinline__ void unpack_dequantize_block(
    int64_t block, const uint32_t* __restrict__ words, const float* __restrict__ mn, const float* __restrict__ scale,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, int32_t uniform_bits,
    int64_t n_chunks, int32_t gs, int32_t gs_shift, u32x4* out, const u32x4* grad, bool cached) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  constexpr int K = chunks_per_thread(MIXED);
  const int64_t base = block * (kThreads * K) + threadIdx.x;

  int64_t g[K];
  uint32_t b[K], woff[K], bitpos[K];
  float m[K], s[K];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    int64_t c = base + (int64_t)k * kThreads;
    c = (c < n_chunks) ? c : n_chunks - 1;                         // clamp: loads stay in bounds
    const int64_t e0 = c * kEpl;                                   // first element of the chunk
    g[k] = (gs_shift >= 0) ? (e0 >> gs_shift) : (e0 / gs);
    bitpos[k] = (uint32_t)(e0 - g[k] * (int64_t)gs);               // element position in the group
    if (MIXED) {
      b[k] = bits[g[k]];
      woff[k] = off[g[k]];
    } else {
      b[k] = (uint32_t)uniform_bits;
      woff[k] = (uint32_t)g[k] * ((uint32_t)(gs >> 5) * b[k]);
    }
    m[k] = mn[g[k]];
    s[k] = scale[g[k]];
  }
  uint32_t w0[K], w1[K];
  u32x4 gq[RELU_BWD ? K : 1];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    if (RELU_BWD) {                                                // the gradient chunk at the output's place
      int64_t c = base + (int64_t)k * kThreads;
      c = (c < n_chunks) ? c : n_chunks - 1;
      gq[k] = __builtin_nontemporal_load(&grad[c]);
    }
    const uint64_t bit64 = (uint64_t)bitpos[k] * b[k];             // bit position in the group
    bitpos[k] = (uint32_t)bit64 & 31u;                             // ... and in its word
    const uint32_t* wp = words + woff[k] + (uint32_t)(bit64 >> 5);
    w0[k] = wp[0];
    w1[k] = (kEpl == 8 && b[k] == 8u) ? wp[1] : 0u;                // 64 bits only for 8 x 8-bit codes
  }
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int64_t c = base + (int64_t)k * kThreads;
    const uint32_t levels = (1u << b[k]) - 1u;
    float v[kEpl];
    if (kEpl == 8 && b[k] == 8u) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[e] = __builtin_fmaf((float)((w0[k] >> (24 - 8 * e)) & 0xFFu), s[k], m[k]);
        v[kEpl - 4 + e] = __builtin_fmaf((float)((w1[k] >> (24 - 8 * e)) & 0xFFu), s[k], m[k]);
      }
    } else {
      const uint32_t pbits = (uint32_t)kEpl * b[k];                // <= 32 here
      const uint32_t field = w0[k] >> (32u - pbits - bitpos[k]);
#pragma unroll
      for (int e = 0; e < kEpl; ++e) {
        const uint32_t code = (field >> ((uint32_t)(kEpl - 1 - e) * b[k])) & levels;
        v[e] = __builtin_fmaf((float)code, s[k], m[k]);
      }
    }
    u32x4 o;
    if (DT == kF32) {
      o = (u32x4){f2u(v[0]), f2u(v[1]), f2u(v[2]), f2u(v[3])};
    } else {
      constexpr int D = (DT == kF32) ? kF16 : DT;
      uint32_t h[4];
#pragma unroll
      for (int q = 0; q < 4; ++q)
        h[q] = narrow16<D>(v[(2 * q) % kEpl]) | (narrow16<D>(v[(2 * q + 1) % kEpl]) << 16);
      o = (u32x4){h[0], h[1], h[2], h[3]};
    }
    if (RELU_BWD) {
      o = (u32x4){keep_where_positive<DT>(o.x, gq[k].x), keep_where_positive<DT>(o.y, gq[k].y),
                  keep_where_positive<DT>(o.z, gq[k].z), keep_where_positive<DT>(o.w, gq[k].w)};
    }
    if (c < n_chunks) {
      // Streaming by default: the kernel alone is up to 16 % faster.  Cached when the plan asks
      // for it: a memory-bound consumer that reads the output next then finds part of it in
      // the caches.  (The streaming store goes through a pointer the compiler cannot see
      // through: it merges two stores to one address and drops the hint.)
      if (cached) {
        out[c] = o;
      } else {
        __attribute__((address_space(1))) u32x4* q = (__attribute__((address_space(1))) u32x4*)&out[c];
        asm volatile("" : "+v"(q));
        __builtin_nontemporal_store(o, q);
      }
    }
  }
}

template <int DT, bool MIXED, bool RELU_BWD>
__global__ __launch_bounds__(kThreads) void k_unpack_dequantize_chunk(
    const uint32_t* __restrict__ words, const float* __restrict__ mn, const float* __restrict__ scale,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, int32_t uniform_bits,
    int64_t n_chunks, int32_t gs, int32_t gs_shift, u32x4* out, const u32x4* grad, int cached, int64_t n) {
  // When elements are left after the last whole chunk (fewer than 8) the grid has one more
  // workgroup, the first, whose first wave takes them: no launch of their own.
  const unsigned first_chunk_block = n > n_chunks * ElemTraits<DT>::kPerLoad ? 1u : 0u;
  if (blockIdx.x < first_chunk_block) {
    if (threadIdx.x < kWave)
      unpack_dequantize_tail_body<DT, RELU_BWD>(words, mn, scale, bits, off, uniform_bits,
                                                n_chunks * ElemTraits<DT>::kPerLoad, n, gs, out, grad);
    return;
  }
  unpack_dequantize_block<DT, MIXED, RELU_BWD>((int64_t)(blockIdx.x - first_chunk_block), words, mn, scale, bits, off,
                                               uniform_bits, n_chunks, gs, gs_shift, out, grad, cached != 0);
}

// Several tensors in one launch: the blocks of all of them form one sequence and a block finds
// its tensor by walking the cumulative block counts (descriptors travel as kernel arguments).
constexpr int kMaxBatch = 32;
struct BatchEntry {
  const uint32_t* words;
  const float* mn;
  const float* scale;
  const uint8_t* bits;
  const uint32_t* off;
  u32x4* out;
  int64_t n_chunks;
  int64_t block_end;                                // blocks of this and all earlier entries
  int32_t uniform_bits, gs, gs_shift;
  int32_t cached;                                   // the plan's output store policy
};
struct Batch {
  BatchEntry e[kMaxBatch];
  int32_t n;
};

template <int DT, bool MIXED>
__global__ __launch_bounds__(kThreads) void k_unpack_dequantize_chunk_batch(const Batch batch) {
  const int64_t gblock = blockIdx.x;
  // (gblock < the last entry's block_end by the grid size, so t < batch.n)
  const int t = batch_entry_of(batch.e, batch.n, gblock, [](const BatchEntry& b) { return b.block_end; });
  const BatchEntry& e = batch.e[t];
  unpack_dequantize_block<DT, MIXED, false>(gblock - (t ? batch.e[t - 1].block_end : 0), e.words, e.mn, e.scale, e.bits,
                                            e.off, e.uniform_bits, e.n_chunks, e.gs, e.gs_shift, e.out, nullptr,
                                            e.cached != 0);
}

template <int DT, bool RELU_BWD>
hipError_t launch_dtype(const daf_plan_t* p, const uint32_t* words, const float* mn, const float* scale,
                        const uint8_t* d_bits, void* out_x, const void* grad, hipStream_t stream) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  const int64_t n_chunks = p->n / kEpl;                 // a chunk never straddles a group (32 | group size)
  int32_t gs_shift = -1;
  if ((p->group_size & (p->group_size - 1)) == 0) gs_shift = __builtin_ctz((unsigned)p->group_size);
  if (n_chunks > 0) {
    const int64_t per_block = (int64_t)kThreads * chunks_per_thread(p->uniform_bits == 0);
    const unsigned blocks = (unsigned)((n_chunks + per_block - 1) / per_block) + (n_chunks * kEpl < p->n ? 1u : 0u);
    if (p->uniform_bits)
      hipLaunchKernelGGL((k_unpack_dequantize_chunk<DT, false, RELU_BWD>), dim3(blocks), dim3(kThreads), 0, stream,
                         words, mn, scale, nullptr, nullptr, p->uniform_bits, n_chunks, p->group_size, gs_shift,
                         static_cast<u32x4*>(out_x), static_cast<const u32x4*>(grad), p->output_cached, p->n);
    else
      hipLaunchKernelGGL((k_unpack_dequantize_chunk<DT, true, RELU_BWD>), dim3(blocks), dim3(kThreads), 0, stream,
                         words, mn, scale, d_bits, p->d_off, 0, n_chunks, p->group_size, gs_shift,
                         static_cast<u32x4*>(out_x), static_cast<const u32x4*>(grad), p->output_cached, p->n);
    return hipGetLastError();                            // the elements after the last chunk rode along
  }
  if (n_chunks * kEpl < p->n) {
    hipLaunchKernelGGL((k_unpack_dequantize_tail<DT, RELU_BWD>), dim3(1), dim3(kWave), 0, stream, words, mn, scale,
                       d_bits, p->d_off, p->uniform_bits, n_chunks * kEpl, p->n, p->group_size, out_x, grad);
    return hipGetLastError();
  }
  return hipSuccess;
}

// Same results as one daf_launch_unpack_dequantize per item.  Consecutive items of the same
// width kind (one width for all groups, or per-group widths) share a launch for their whole
// chunks (at most kMaxBatch per launch); the few elements after an item's last whole chunk are
// launched as before.
template <int DT>
hipError_t launch_items(const daf_dequantize_item_t* items, int32_t n_items, hipStream_t stream) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  Batch batch;
  batch.n = 0;
  bool cur_mixed = false;
  hipError_t err = hipSuccess;
  auto flush = [&]() {
    if (batch.n > 0 && err == hipSuccess) {
      const unsigned blocks = (unsigned)batch.e[batch.n - 1].block_end;
      if (cur_mixed)
        hipLaunchKernelGGL((k_unpack_dequantize_chunk_batch<DT, true>), dim3(blocks), dim3(kThreads), 0, stream, batch);
      else
        hipLaunchKernelGGL((k_unpack_dequantize_chunk_batch<DT, false>), dim3(blocks), dim3(kThreads), 0, stream, batch);
      err = hipGetLastError();
    }
    batch.n = 0;
  };
  for (int32_t i = 0; i < n_items && err == hipSuccess; ++i) {
    const daf_dequantize_item_t& it = items[i];
    const daf_plan_t* p = it.plan;
    const uint8_t* d_bits = it.bits ? it.bits : p->d_bits;
    const int64_t n_chunks = p->n / kEpl;
    const bool mixed = p->uniform_bits == 0;
    if (n_chunks > 0) {
      const int64_t per_block = (int64_t)kThreads * chunks_per_thread(mixed);
      const int64_t blocks = (n_chunks + per_block - 1) / per_block;
      if (batch.n == kMaxBatch || (batch.n > 0 && mixed != cur_mixed) ||
          (batch.n > 0 && batch.e[batch.n - 1].block_end + blocks > 0x7fffffff))
        flush();
      cur_mixed = mixed;
      BatchEntry& e = batch.e[batch.n];
      e.words = it.words;
      e.mn = it.min;
      e.scale = it.scale;
      e.bits = mixed ? d_bits : nullptr;
      e.off = mixed ? p->d_off : nullptr;
      e.out = static_cast<u32x4*>(it.out_x);
      e.n_chunks = n_chunks;
      e.block_end = (batch.n ? batch.e[batch.n - 1].block_end : 0) + blocks;
      e.uniform_bits = p->uniform_bits;
      e.gs = p->group_size;
      e.gs_shift = ((p->group_size & (p->group_size - 1)) == 0) ? __builtin_ctz((unsigned)p->group_size) : -1;
      e.cached = p->output_cached;
      ++batch.n;
    }
    if (n_chunks * kEpl < p->n && err == hipSuccess) {
      hipLaunchKernelGGL((k_unpack_dequantize_tail<DT, false>), dim3(1), dim3(kWave), 0, stream, it.words, it.min,
                         it.scale, d_bits, p->d_off, p->uniform_bits, n_chunks * kEpl, p->n, p->group_size, it.out_x,
                         nullptr);
      err = hipGetLastError();
    }
  }
  flush();
  return err;
}

}  // namespace

hipError_t daf_launch_unpack_dequantize_batch(const daf_dequantize_item_t* items, int32_t n_items, int dtype,
                                              hipStream_t stream) {
  switch (dtype) {
    case daf::kF32:  return launch_items<daf::kF32>(items, n_items, stream);
    case daf::kF16:  return launch_items<daf::kF16>(items, n_items, stream);
    case daf::kBF16: return launch_items<daf::kBF16>(items, n_items, stream);
    default: return hipErrorInvalidValue;
  }
}

hipError_t daf_launch_unpack_dequantize(const daf_plan_t* plan, const uint32_t* words, const float* mn,
                                        const float* scale, const uint8_t* d_bits, void* out_x, int dtype,
                                        const void* relu_grad_y, hipStream_t stream) {
#define DAF_DT(D)                                                                                        \
  return relu_grad_y ? launch_dtype<D, true>(plan, words, mn, scale, d_bits, out_x, relu_grad_y, stream) \
                     : launch_dtype<D, false>(plan, words, mn, scale, d_bits, out_x, nullptr, stream)
  switch (dtype) {
    case daf::kF32:  DAF_DT(daf::kF32);
    case daf::kF16:  DAF_DT(daf::kF16);
    case daf::kBF16: DAF_DT(daf::kBF16);
    default: return hipErrorInvalidValue;
  }
#undef DAF_DT
}
