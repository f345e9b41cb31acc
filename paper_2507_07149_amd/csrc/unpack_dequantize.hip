// Backward-pass side: unpack the codes (the extraction rule of Algorithm 2, for the group's
// own width) and dequantize them to the original precision, xhat = fma(code, scale, min)
// (inverse of Eq. 1; paper Sec. 2.2).  Two kernels:
//
//   k_unpack_dequantize_tile   group sizes that are a power of two (64 or fewer groups per tile).  One
//                              wave owns a tile of 512 output chunks of 16 bytes: it fetches the
//                              tile's min, scale, widths and its contiguous run of packed words
//                              with coalesced loads into wave-private LDS (one round trip to
//                              memory; two with per-group widths, whose word offsets come from an
//                              in-tile prefix sum), then produces the chunks from LDS.
//   k_unpack_dequantize_chunk  any group size.  A thread produces 16 bytes of output at a time
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

// One 16-byte output chunk (4 binary32 or 8 16-bit elements) from the packed word(s) that hold
// its codes: w0 (and w1 for eight 8-bit codes), the chunk's first bit at `bitpos` of w0, width
// b; xhat = fma(code, scale, min) in binary32, then round-to-nearest-even to the element format.
template <int DT>
__device__ __forceinline__ u32x4 dequantize_chunk(uint32_t w0, uint32_t w1, uint32_t bitpos, uint32_t b, float m,
                                                  float s) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  const uint32_t levels = (1u << b) - 1u;
  float v[kEpl];
  if (kEpl == 8 && b == 8u) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[e] = __builtin_fmaf((float)((w0 >> (24 - 8 * e)) & 0xFFu), s, m);
      v[kEpl - 4 + e] = __builtin_fmaf((float)((w1 >> (24 - 8 * e)) & 0xFFu), s, m);
    }
  } else {
    const uint32_t pbits = (uint32_t)kEpl * b;                     // <= 32 here
    const uint32_t field = w0 >> (32u - pbits - bitpos);
#pragma unroll
    for (int e = 0; e < kEpl; ++e) {
      const uint32_t code = (field >> ((uint32_t)(kEpl - 1 - e) * b)) & levels;
      v[e] = __builtin_fmaf((float)code, s, m);
    }
  }
  if (DT == kF32) return (u32x4){f2u(v[0]), f2u(v[1]), f2u(v[2]), f2u(v[3])};
  constexpr int D = (DT == kF32) ? kF16 : DT;
  uint32_t h[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) h[q] = narrow16<D>(v[(2 * q) % kEpl]) | (narrow16<D>(v[(2 * q + 1) % kEpl]) << 16);
  return (u32x4){h[0], h[1], h[2], h[3]};
}

// Streaming by default: the kernel alone is up to 16 % faster.  Cached when the plan asks for
// it: a memory-bound consumer that reads the output next then finds part of it in the caches.
// (The streaming store goes through a pointer the compiler cannot see through: it merges two
// stores to one address and drops the hint.)
__device__ __forceinline__ void store_chunk(u32x4* out, int64_t c, u32x4 o, bool cached) {
  if (cached) {
    out[c] = o;
  } else {
    __attribute__((address_space(1))) u32x4* q = (__attribute__((address_space(1))) u32x4*)&out[c];
    asm volatile("" : "+v"(q));
    __builtin_nontemporal_store(o, q);
  }
}

// The loop over a thread's chunks is split into phases (metadata loads, word loads,
// arithmetic + stores) so that all loads of one phase are in flight together: with per-group
// widths the word address depends on two earlier loads, and a chunk-by-chunk loop would pay
// that latency once per chunk.
template <int DT, bool MIXED, bool RELU_BWD>
__device__ __forceinline__ void unpack_dequantize_block(
    int64_t block, const uint32_t* __restrict__ words, const float* __restrict__ mn, const float* __restrict__ scale,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, int32_t uniform_bits,
    int64_t n_chunks, int32_t gs, int32_t gs_shift, u32x4* out, const u32x4* grad, bool cached, int64_t chunk0 = 0) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  constexpr int K = chunks_per_thread(MIXED);
  const int64_t base = chunk0 + block * (kThreads * K) + threadIdx.x;   // chunk0: the first chunk this launch covers

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
    u32x4 o = dequantize_chunk<DT>(w0[k], w1[k], bitpos[k], b[k], m[k], s[k]);
    if (RELU_BWD) {
      o = (u32x4){keep_where_positive<DT>(o.x, gq[k].x), keep_where_positive<DT>(o.y, gq[k].y),
                  keep_where_positive<DT>(o.z, gq[k].z), keep_where_positive<DT>(o.w, gq[k].w)};
    }
    if (c < n_chunks) store_chunk(out, c, o, cached);
  }
}

template <int DT, bool MIXED, bool RELU_BWD>
__global__ __launch_bounds__(kThreads) void k_unpack_dequantize_chunk(
    const uint32_t* __restrict__ words, const float* __restrict__ mn, const float* __restrict__ scale,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, int32_t uniform_bits,
    int64_t n_chunks, int32_t gs, int32_t gs_shift, u32x4* out, const u32x4* grad, int cached, int64_t n,
    int64_t chunk0) {
  // Covers the chunks chunk0 .. n_chunks - 1 (chunk0 > 0: the chunks that the tile kernel of a
  // list call left over).
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
                                               uniform_bits, n_chunks, gs, gs_shift, out, grad, cached != 0, chunk0);
}

// ------------------------------------------------------------------------------------------
// Tile path: one wave per tile of 512 output chunks (2048 binary32 or 4096 16-bit elements).
// ------------------------------------------------------------------------------------------
// The chunk kernel below fetches widths, offsets, min, scale and words chunk by chunk: small
// loads that depend on each other, which a backward pass (whose packed input comes from HBM, not
// from a cache) pays in full.  Here the wave reads everything its tile needs with coalesced loads
// issued together: min, scale (and width) of the tile's groups, one offset, and the tile's words,
// which are one contiguous run of the packed buffer.  With per-group widths the run's length and
// the groups' places in it come from a prefix sum over the tile's widths, so the word loads form
// a second round.  The chunks are then produced from wave-private LDS.
// 8 chunks per lane: measured against 4 and 16 with the packed input coming from HBM (38.9 / 38.3 /
// 40.7 us on a 51 M-element binary32 tensor, 168 / 157 / 164 us on the LLM-shaped bfloat16 one;
// only a 50 MB binary16 tensor prefers 16).  Fewer than 8 would make a 1-bit binary32 run
// shorter than one word per lane.
constexpr int kTileChunksPerLane = 8;
constexpr int kTileChunks = kWave * kTileChunksPerLane;           // 512
constexpr int kWavesPerBlock = kThreads / kWave;

struct alignas(16) TileGroup {   // what a chunk needs to know about its group
  float mn, scale;
  uint32_t b;                    // width
  uint32_t woff;                 // first word of the group in the staged run
};

// B = 1, 2, 4, 8: every group has that width.  B = 0: per-group widths and offsets.
template <int DT, int B, int U>
struct alignas(16) TileLds {
  static constexpr int kWords = kWave * U * ElemTraits<DT>::kPerLoad * (B ? B : 8) / 32;     // the run, at most
  uint32_t stage[kWords + 4];
  TileGroup group[kWave];
};

// U = 16-byte chunks per lane: 8; 16 for small tensors with per-group widths (see launch_dtype).
template <int DT, int B, bool RELU_BWD, int U = kTileChunksPerLane>
__device__ __forceinline__ void unpack_dequantize_tile_body(
    int64_t tile, int wave_in_block, const uint32_t* __restrict__ words, const float* __restrict__ mn,
    const float* __restrict__ scale, const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off,
    int32_t gs_log2, u32x4* out, const u32x4* grad, bool cached) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  constexpr int kTileChunks = kWave * U;
  constexpr int kElems = kTileChunks * kEpl;
  constexpr bool kMixed = (B == 0);
  constexpr int kMaxWords = TileLds<DT, B, U>::kWords;
  constexpr int kWordLoads = (kMaxWords + kWave - 1) / kWave;     // per lane
  __shared__ TileLds<DT, B, U> lds_all[kWavesPerBlock];
  TileLds<DT, B, U>& lds = lds_all[wave_in_block];
  const int lane = threadIdx.x & (kWave - 1);
  const int groups = kElems >> gs_log2;                          // 1 .. 64 whole groups per tile
  const int64_t g0 = tile * groups;
  const uint32_t group_words32 = (1u << gs_log2) >> 5;           // words per group and bit of width

  // first trip to memory: the groups' constants (lane g takes group g), the gradient chunks, and with one
  // width for all groups the words as well
  TileGroup mine;
  mine.mn = 0.0f; mine.scale = 0.0f; mine.b = B ? (uint32_t)B : 1u;
  uint32_t tile_base;
  if (lane < groups) {
    mine.mn = mn[g0 + lane];
    mine.scale = scale[g0 + lane];
    if (kMixed) mine.b = bits[g0 + lane];
  }
  if (kMixed) tile_base = off[g0];
  else tile_base = (uint32_t)tile * (uint32_t)(kElems / 32 * B);
  u32x4 gq[RELU_BWD ? U : 1];
  if (RELU_BWD) {
#pragma unroll
    for (int u = 0; u < U; ++u) gq[u] = __builtin_nontemporal_load(&grad[tile * kTileChunks + u * kWave + lane]);
  }
  uint32_t wv[kWordLoads];
  uint32_t tile_words;
  if (!kMixed) {
    tile_words = kMaxWords;
#pragma unroll
    for (int j = 0; j < kWordLoads; ++j) wv[j] = __builtin_nontemporal_load(&words[tile_base + j * kWave + lane]);
    static_assert(kMaxWords % kWave == 0, "every lane loads whole rounds of the run: the run must be a multiple of 64 words");
    mine.woff = (uint32_t)lane * (group_words32 * B);
  } else {
    const uint32_t gw = (lane < groups) ? group_words32 * mine.b : 0u;
    const uint32_t incl = wave_inclusive_sum(gw);
    tile_words = (uint32_t)__builtin_amdgcn_readlane((int)incl, kWave - 1);
    mine.woff = incl - gw;
    // second trip: the run's words (its length is known only now)
#pragma unroll
    for (int j = 0; j < kWordLoads; ++j) {
      const uint32_t i = (uint32_t)(j * kWave + lane);                 // < kWordLoads * 64 = kMaxWords: inside stage
      wv[j] = (i < tile_words) ? __builtin_nontemporal_load(&words[tile_base + i]) : 0u;
    }
  }
#pragma unroll
  for (int j = 0; j < kWordLoads; ++j) lds.stage[j * kWave + lane] = wv[j];
  lds.group[lane] = mine;
  wave_lds_sync();

  // All LDS reads of a phase are issued together (group constants, then words), so that the
  // eight chunks pay the LDS latency twice, not sixteen times.
  const uint32_t pos_mask = (1u << gs_log2) - 1u;
  TileGroup g[U];
  uint32_t w0[U], w1[U], bit[U];
#pragma unroll
  for (int u = 0; u < U; ++u) g[u] = lds.group[((uint32_t)(u * kWave + lane) * kEpl) >> gs_log2];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint32_t e0 = (uint32_t)(u * kWave + lane) * kEpl;     // first element of chunk u*64 + lane of the tile
    const uint32_t b = kMixed ? g[u].b : (uint32_t)B;
    bit[u] = (e0 & pos_mask) * b;                                // bit position in the group (< 2^15)
    const uint32_t widx = g[u].woff + (bit[u] >> 5);
    w0[u] = lds.stage[widx];
    w1[u] = (kEpl == 8 && b == 8u) ? lds.stage[widx + 1] : 0u;
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint32_t b = kMixed ? g[u].b : (uint32_t)B;
    u32x4 o = dequantize_chunk<DT>(w0[u], w1[u], bit[u] & 31u, b, g[u].mn, g[u].scale);
    if (RELU_BWD) {
      o = (u32x4){keep_where_positive<DT>(o.x, gq[u].x), keep_where_positive<DT>(o.y, gq[u].y),
                  keep_where_positive<DT>(o.z, gq[u].z), keep_where_positive<DT>(o.w, gq[u].w)};
    }
    store_chunk(out, tile * kTileChunks + (int64_t)(u * kWave + lane), o, cached);
  }
}

// The whole tiles of one tensor; when chunks (and the fewer than 8 elements after the last whole
// chunk) are left over, the grid has one more workgroup, the first, which takes them the
// chunk kernel's way.
// At most 6 waves per SIMD: the kernels need few registers and would run 8, but the write stream
// then loses locality (the 17-tensor list: 466 us with 8, 409 us with 6, 450 us with 4).
#ifndef DAF_DEQ_TILE_WAVES
#define DAF_DEQ_TILE_WAVES 6
#endif
#define DAF_TILE_WAVES __attribute__((amdgpu_waves_per_eu(1, DAF_DEQ_TILE_WAVES)))
template <int DT, int B, bool RELU_BWD, int U = kTileChunksPerLane>
__global__ __launch_bounds__(kThreads) DAF_TILE_WAVES void k_unpack_dequantize_tile(
    const uint32_t* __restrict__ words, const float* __restrict__ mn, const float* __restrict__ scale,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, int64_t n_tiles, int32_t gs, int32_t gs_log2,
    u32x4* out, const u32x4* grad, int cached, int64_t n_chunks, int64_t n) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  constexpr int kTileChunks = kWave * U;
  static_assert(kTileChunks <= kThreads * chunks_per_thread(B == 0), "the left-over chunks fit one workgroup");
  const bool left = n_tiles * kTileChunks * kEpl < n;
  if (left && blockIdx.x == 0) {
    if (n_tiles * kTileChunks < n_chunks)
      unpack_dequantize_block<DT, B == 0, RELU_BWD>(0, words, mn, scale, bits, off, B, n_chunks, gs, gs_log2, out, grad,
                                                    cached != 0, n_tiles * kTileChunks);
    if (n_chunks * kEpl < n && threadIdx.x < kWave)
      unpack_dequantize_tail_body<DT, RELU_BWD>(words, mn, scale, bits, off, B, n_chunks * kEpl, n, gs, out, grad);
    return;
  }
  const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t tile = (int64_t)(blockIdx.x - (left ? 1u : 0u)) * kWavesPerBlock + wave_in_block;
  if (tile >= n_tiles) return;
  unpack_dequantize_tile_body<DT, B, RELU_BWD, U>(tile, wave_in_block, words, mn, scale, bits, off, gs_log2, out, grad,
                                                  cached != 0);
}

// ---- tiles for group sizes that are not a power of two -------------------------------------
// The same tile, but groups start anywhere in it (the first and the last may continue in the
// neighbouring tiles): lane l holds the constants of group g_first + l, a chunk finds its group
// by dividing its element index by the group size (a multiply-high with a rounded-up
// reciprocal, exact for the few thousand values that occur), and with one width for all groups
// the packed words do not depend on the group size at all: element e sits at bit e * B of the
// stream.  With per-group widths the run starts at the word of the tile's first element inside
// its group and may be one word longer than the tile's bits.
template <int DT, int B>
struct alignas(16) TileLdsAny {
  static constexpr int kWords = TileLds<DT, B, kTileChunksPerLane>::kWords + (B ? 0 : kWave);
  uint32_t stage[kWords + 4];
  TileGroup group[kWave];
};

template <int DT, int B, bool RELU_BWD>
__device__ __forceinline__ void unpack_dequantize_tile_any_body(
    int64_t tile, int wave_in_block, const uint32_t* __restrict__ words, const float* __restrict__ mn,
    const float* __restrict__ scale, const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, int32_t gs,
    uint32_t gs_magic, int64_t G, u32x4* out, const u32x4* grad, bool cached) {
  constexpr int U = kTileChunksPerLane;
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  constexpr int kElems = kTileChunks * kEpl;
  constexpr bool kMixed = (B == 0);
  constexpr int kMaxWords = TileLdsAny<DT, B>::kWords;
  constexpr int kWordLoads = kMaxWords / kWave;
  static_assert(kMaxWords % kWave == 0, "every lane loads whole rounds of the run");
  __shared__ TileLdsAny<DT, B> lds_all[kWavesPerBlock];
  TileLdsAny<DT, B>& lds = lds_all[wave_in_block];
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t e_tile0 = tile * kElems;
  const int64_t g_first = e_tile0 / gs;                          // once per wave
  const uint32_t rem0 = (uint32_t)(e_tile0 - g_first * gs);      // the tile starts this far into its first group
  const int groups = (int)((rem0 + (uint32_t)kElems - 1u) / (uint32_t)gs) + 1;   // at most 64: checked by the launcher

  TileGroup mine;
  mine.mn = 0.0f; mine.scale = 0.0f; mine.b = B ? (uint32_t)B : 1u; mine.woff = 0u;
  uint32_t my_off = 0u;
  if (lane < groups && g_first + lane < G) {
    mine.mn = mn[g_first + lane];
    mine.scale = scale[g_first + lane];
    if (kMixed) {
      mine.b = bits[g_first + lane];
      my_off = off[g_first + lane];
    }
  }
  u32x4 gq[RELU_BWD ? U : 1];
  if (RELU_BWD) {
#pragma unroll
    for (int u = 0; u < U; ++u) gq[u] = __builtin_nontemporal_load(&grad[tile * kTileChunks + u * kWave + lane]);
  }
  uint32_t wv[kWordLoads];
  if (!kMixed) {
    const uint32_t tile_base = (uint32_t)tile * (uint32_t)(kElems / 32 * B);
#pragma unroll
    for (int j = 0; j < kWordLoads; ++j) wv[j] = __builtin_nontemporal_load(&words[tile_base + j * kWave + lane]);
  } else {
    const uint32_t b_first = (uint32_t)__builtin_amdgcn_readlane((int)mine.b, 0);
    const uint32_t off_first = (uint32_t)__builtin_amdgcn_readlane((int)my_off, 0);
    const uint32_t first_word = off_first + ((rem0 * b_first) >> 5);
    const uint32_t e_last = rem0 + (uint32_t)(kElems - kEpl);                     // the tile's last chunk
    const int gl_last = __builtin_amdgcn_readfirstlane((int)__umulhi(e_last, gs_magic));
    const uint32_t b_last = (uint32_t)__builtin_amdgcn_readlane((int)mine.b, gl_last);
    const uint32_t off_last = (uint32_t)__builtin_amdgcn_readlane((int)my_off, gl_last);
    const uint32_t bit_end = (e_last - (uint32_t)gl_last * (uint32_t)gs + (uint32_t)kEpl) * b_last;
    const uint32_t tile_words = off_last + ((bit_end + 31u) >> 5) - first_word;   // <= kMaxWords
    mine.woff = my_off - first_word;                    // modulo 2^32: the first group may start before the run
#pragma unroll
    for (int j = 0; j < kWordLoads; ++j) {
      const uint32_t i = (uint32_t)(j * kWave + lane);
      wv[j] = (i < tile_words) ? __builtin_nontemporal_load(&words[first_word + i]) : 0u;
    }
  }
#pragma unroll
  for (int j = 0; j < kWordLoads; ++j) lds.stage[j * kWave + lane] = wv[j];
  lds.group[lane] = mine;
  wave_lds_sync();

  TileGroup g[U];
  uint32_t w0[U], w1[U], bit[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint32_t e0 = (uint32_t)(u * kWave + lane) * kEpl;     // first element of chunk u*64 + lane of the tile
    const uint32_t gl = __umulhi(rem0 + e0, gs_magic);           // = (rem0 + e0) / gs
    g[u] = lds.group[gl];
    const uint32_t b = kMixed ? g[u].b : (uint32_t)B;
    uint32_t widx;
    if (kMixed) {
      bit[u] = (rem0 + e0 - gl * (uint32_t)gs) * b;              // bit position inside the group
      widx = g[u].woff + (bit[u] >> 5);
    } else {
      bit[u] = e0 * b;                                           // bit position inside the tile's run
      widx = bit[u] >> 5;
    }
    w0[u] = lds.stage[widx];
    w1[u] = (kEpl == 8 && b == 8u) ? lds.stage[widx + 1] : 0u;
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint32_t b = kMixed ? g[u].b : (uint32_t)B;
    u32x4 o = dequantize_chunk<DT>(w0[u], w1[u], bit[u] & 31u, b, g[u].mn, g[u].scale);
    if (RELU_BWD) {
      o = (u32x4){keep_where_positive<DT>(o.x, gq[u].x), keep_where_positive<DT>(o.y, gq[u].y),
                  keep_where_positive<DT>(o.z, gq[u].z), keep_where_positive<DT>(o.w, gq[u].w)};
    }
    store_chunk(out, tile * kTileChunks + (int64_t)(u * kWave + lane), o, cached);
  }
}

template <int DT, int B, bool RELU_BWD>
__global__ __launch_bounds__(kThreads) DAF_TILE_WAVES void k_unpack_dequantize_tile_any(
    const uint32_t* __restrict__ words, const float* __restrict__ mn, const float* __restrict__ scale,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, int64_t n_tiles, int32_t gs, uint32_t gs_magic,
    int64_t G, u32x4* out, const u32x4* grad, int cached, int64_t n_chunks, int64_t n) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  const bool left = n_tiles * kTileChunks * kEpl < n;
  if (left && blockIdx.x == 0) {                       // what the tiles leave over, the chunk kernel's way
    if (n_tiles * kTileChunks < n_chunks)
      unpack_dequantize_block<DT, B == 0, RELU_BWD>(0, words, mn, scale, bits, off, B, n_chunks, gs, -1, out, grad,
                                                    cached != 0, n_tiles * kTileChunks);
    if (n_chunks * kEpl < n && threadIdx.x < kWave)
      unpack_dequantize_tail_body<DT, RELU_BWD>(words, mn, scale, bits, off, B, n_chunks * kEpl, n, gs, out, grad);
    return;
  }
  const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t tile = (int64_t)(blockIdx.x - (left ? 1u : 0u)) * kWavesPerBlock + wave_in_block;
  if (tile >= n_tiles) return;
  unpack_dequantize_tile_any_body<DT, B, RELU_BWD>(tile, wave_in_block, words, mn, scale, bits, off, gs, gs_magic, G, out,
                                                   grad, cached != 0);
}

// Whole tiles of a plan whose group size is not a power of two on that path (0: does not fit).
template <int DT>
int64_t any_tile_path_tiles(const daf_plan_t* p, uint32_t* magic) {
  constexpr int kElems = kTileChunks * ElemTraits<DT>::kPerLoad;
  const int64_t gs = p->group_size;
  if ((gs & (gs - 1)) == 0 || gs < 64 || gs > 32768 || gs % 32 != 0) return 0;
  if ((gs - 1 + kElems - 1) / gs + 1 > kWave) return 0;           // groups that touch one tile
  if (p->num_groups >= ((int64_t)1 << 31)) return 0;
  *magic = (uint32_t)((((uint64_t)1 << 32) + (uint64_t)gs - 1) / (uint64_t)gs);
  return p->n / kElems;
}

// Several tensors in one launch: the tiles of all of them form one sequence.
struct TileBatchEntry {
  const uint32_t* words;
  const float* mn;
  const float* scale;
  const uint8_t* bits;
  const uint32_t* off;
  u32x4* out;
  int64_t tile_end;                                 // tiles of this and all earlier entries
  int32_t gs_log2;
  int32_t cached;                                   // the plan's output store policy
};
constexpr int kMaxTileBatch = kBatchSlots;
struct TileBatch {
  uint32_t ends[kBatchSlots];                       // e[t].tile_end, 0xFFFFFFFF beyond n
  TileBatchEntry e[kMaxTileBatch];
  int32_t n;
};

template <int DT, int B>
__global__ __launch_bounds__(kThreads) DAF_TILE_WAVES void k_unpack_dequantize_tile_batch(const TileBatch batch) {
  const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t gtile = (int64_t)blockIdx.x * kWavesPerBlock + wave_in_block;
  const int t = batch_entry_of(batch.ends, (uint32_t)gtile);
  if (t >= batch.n) return;                          // past the last tile (the grid is whole workgroups)
  const TileBatchEntry e = batch.e[t];               // by value: one scalar load of the whole descriptor
  unpack_dequantize_tile_body<DT, B, false>(gtile - (t ? batch.e[t - 1].tile_end : 0), wave_in_block, e.words, e.mn,
                                            e.scale, e.bits, e.off, e.gs_log2, e.out, nullptr, e.cached != 0);
}

// Whole tiles of a plan on the tile path (0: the plan's group size does not fit it).
template <int DT>
int64_t tile_path_tiles(const daf_plan_t* p, int32_t* gs_log2, int chunks_per_lane = kTileChunksPerLane) {
  const int kElems = kWave * chunks_per_lane * ElemTraits<DT>::kPerLoad;
  const int32_t gs = p->group_size;
  if ((gs & (gs - 1)) != 0 || gs > kElems || kElems / gs > kWave) return 0;
  *gs_log2 = __builtin_ctz((unsigned)gs);
  return p->n / kElems;
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
  uint32_t ends[kBatchSlots];                       // e[t].block_end, 0xFFFFFFFF beyond n
  BatchEntry e[kMaxBatch];
  int32_t n;
};

template <int DT, bool MIXED>
__global__ __launch_bounds__(kThreads) void k_unpack_dequantize_chunk_batch(const Batch batch) {
  const int64_t gblock = blockIdx.x;
  const int t = batch_entry_of(batch.ends, (uint32_t)gblock);   // < batch.n: the grid ends with the last entry's blocks
  const BatchEntry& e = batch.e[t];
  unpack_dequantize_block<DT, MIXED, false>(gblock - (t ? batch.e[t - 1].block_end : 0), e.words, e.mn, e.scale, e.bits,
                                            e.off, e.uniform_bits, e.n_chunks, e.gs, e.gs_shift, e.out, nullptr,
                                            e.cached != 0);
}

// The chunks chunk0 .. of a tensor (and the elements after its last whole chunk) through the chunk kernel.
template <int DT, bool RELU_BWD>
hipError_t launch_chunks(const daf_plan_t* p, const uint32_t* words, const float* mn, const float* scale,
                         const uint8_t* d_bits, void* out_x, const void* grad, int64_t chunk0, hipStream_t stream) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  const int64_t n_chunks = p->n / kEpl;                 // a chunk never straddles a group (32 | group size)
  int32_t gs_shift = -1;
  if ((p->group_size & (p->group_size - 1)) == 0) gs_shift = __builtin_ctz((unsigned)p->group_size);
  if (n_chunks > chunk0) {
    const int64_t per_block = (int64_t)kThreads * chunks_per_thread(p->uniform_bits == 0);
    const unsigned blocks = (unsigned)((n_chunks - chunk0 + per_block - 1) / per_block) + (n_chunks * kEpl < p->n ? 1u : 0u);
    if (p->uniform_bits)
      hipLaunchKernelGGL((k_unpack_dequantize_chunk<DT, false, RELU_BWD>), dim3(blocks), dim3(kThreads), 0, stream,
                         words, mn, scale, nullptr, nullptr, p->uniform_bits, n_chunks, p->group_size, gs_shift,
                         static_cast<u32x4*>(out_x), static_cast<const u32x4*>(grad), p->output_cached, p->n, chunk0);
    else
      hipLaunchKernelGGL((k_unpack_dequantize_chunk<DT, true, RELU_BWD>), dim3(blocks), dim3(kThreads), 0, stream,
                         words, mn, scale, d_bits, p->d_off, 0, n_chunks, p->group_size, gs_shift,
                         static_cast<u32x4*>(out_x), static_cast<const u32x4*>(grad), p->output_cached, p->n, chunk0);
    return hipGetLastError();                            // the elements after the last chunk rode along
  }
  if (n_chunks * kEpl < p->n) {
    hipLaunchKernelGGL((k_unpack_dequantize_tail<DT, RELU_BWD>), dim3(1), dim3(kWave), 0, stream, words, mn, scale,
                       d_bits, p->d_off, p->uniform_bits, n_chunks * kEpl, p->n, p->group_size, out_x, grad);
    return hipGetLastError();
  }
  return hipSuccess;
}

template <int DT, bool RELU_BWD>
hipError_t launch_dtype(const daf_plan_t* p, const uint32_t* words, const float* mn, const float* scale,
                        const uint8_t* d_bits, void* out_x, const void* grad, hipStream_t stream) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  int32_t gs_log2 = 0;
  const int64_t n_tiles = tile_path_tiles<DT>(p, &gs_log2);
  uint32_t magic = 0;
  // (binary32 with 8 bits for every group stays with the chunk kernel: 0.76-0.78 of the memory rate
  // there against 0.70-0.74 through tiles, measured on 2^27 elements with groups of 96 ... 11008)
  const int64_t any_tiles =
      (n_tiles == 0 && !(DT == kF32 && p->uniform_bits == 8)) ? any_tile_path_tiles<DT>(p, &magic) : 0;
  if (any_tiles > 0) {
    const bool left = any_tiles * kTileChunks * kEpl < p->n;
    const unsigned blocks = (unsigned)((any_tiles + kWavesPerBlock - 1) / kWavesPerBlock) + (left ? 1u : 0u);
#define DAF_LAUNCH(BITS)                                                                                          \
  hipLaunchKernelGGL((k_unpack_dequantize_tile_any<DT, BITS, RELU_BWD>), dim3(blocks), dim3(kThreads), 0, stream,  \
                     words, mn, scale, d_bits, p->d_off, any_tiles, p->group_size, magic, p->num_groups,          \
                     static_cast<u32x4*>(out_x), static_cast<const u32x4*>(grad), p->output_cached, p->n / kEpl,  \
                     p->n)
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
  if (n_tiles == 0) return launch_chunks<DT, RELU_BWD>(p, words, mn, scale, d_bits, out_x, grad, 0, stream);
  // A small tensor with per-group widths takes tiles of twice the size: every wave pays two
  // round trips to memory (widths, then words) before it can store anything, and with few
  // waves per SIMD to overlap them fewer, longer waves come out ahead (a 50 MB binary16 tensor:
  // 14.5 -> 12.5 us; the 721 MB bfloat16 one prefers the smaller tile, 157 against 164 us).
  if (p->uniform_bits == 0 && n_tiles <= 8192) {
    int32_t log2_big = 0;
    const int64_t big_tiles = tile_path_tiles<DT>(p, &log2_big, 2 * kTileChunksPerLane);
    if (big_tiles > 0) {
      constexpr int kBig = 2 * kTileChunks;
      const bool left = big_tiles * kBig * kEpl < p->n;
      const unsigned blocks = (unsigned)((big_tiles + kWavesPerBlock - 1) / kWavesPerBlock) + (left ? 1u : 0u);
      hipLaunchKernelGGL((k_unpack_dequantize_tile<DT, 0, RELU_BWD, 2 * kTileChunksPerLane>), dim3(blocks), dim3(kThreads),
                         0, stream, words, mn, scale, d_bits, p->d_off, big_tiles, p->group_size, log2_big,
                         static_cast<u32x4*>(out_x), static_cast<const u32x4*>(grad), p->output_cached, p->n / kEpl,
                         p->n);
      return hipGetLastError();
    }
  }
  const bool left = n_tiles * kTileChunks * kEpl < p->n;
  const unsigned blocks = (unsigned)((n_tiles + kWavesPerBlock - 1) / kWavesPerBlock) + (left ? 1u : 0u);
#define DAF_LAUNCH(BITS)                                                                                      \
  hipLaunchKernelGGL((k_unpack_dequantize_tile<DT, BITS, RELU_BWD>), dim3(blocks), dim3(kThreads), 0, stream,  \
                     words, mn, scale, d_bits, p->d_off, n_tiles, p->group_size, gs_log2,                     \
                     static_cast<u32x4*>(out_x), static_cast<const u32x4*>(grad), p->output_cached,           \
                     p->n / kEpl, p->n)
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

// Same results as one daf_launch_unpack_dequantize per item.  Consecutive items of the same
// width kind (one width for all groups, or per-group widths) share a launch for their whole
// chunks (at most kMaxBatch per launch); the few elements after an item's last whole chunk are
// launched as before.
template <int DT>
hipError_t launch_items(const daf_dequantize_item_t* items, int32_t n_items, hipStream_t stream) {
  constexpr int kEpl = ElemTraits<DT>::kPerLoad;
  Batch batch;
  batch.n = 0;
  for (int i = 0; i < kBatchSlots; ++i) batch.ends[i] = 0xFFFFFFFFu;
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
    for (int i = 0; i < kBatchSlots; ++i) batch.ends[i] = 0xFFFFFFFFu;
  };
  TileBatch tbatch;                    // items on the tile path (group size a power of two)
  tbatch.n = 0;
  for (int i = 0; i < kBatchSlots; ++i) tbatch.ends[i] = 0xFFFFFFFFu;
  int tcur_bits = -1;
  auto tflush = [&]() {
    if (tbatch.n > 0 && err == hipSuccess) {
      const unsigned blocks = (unsigned)((tbatch.e[tbatch.n - 1].tile_end + kWavesPerBlock - 1) / kWavesPerBlock);
#define DAF_LAUNCH(BITS) \
  hipLaunchKernelGGL((k_unpack_dequantize_tile_batch<DT, BITS>), dim3(blocks), dim3(kThreads), 0, stream, tbatch)
      switch (tcur_bits) {
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
    tbatch.n = 0;
    for (int i = 0; i < kBatchSlots; ++i) tbatch.ends[i] = 0xFFFFFFFFu;
  };
  for (int32_t i = 0; i < n_items && err == hipSuccess; ++i) {
    const daf_dequantize_item_t& it = items[i];
    const daf_plan_t* p = it.plan;
    const uint8_t* d_bits = it.bits ? it.bits : p->d_bits;
    const int64_t n_chunks = p->n / kEpl;
    const bool mixed = p->uniform_bits == 0;
    int32_t gs_log2 = 0;
    const int64_t n_tiles = tile_path_tiles<DT>(p, &gs_log2);
    if (n_tiles > 0) {
      if (tbatch.n == kMaxTileBatch || (tbatch.n > 0 && p->uniform_bits != tcur_bits) ||
          (tbatch.n > 0 && tbatch.e[tbatch.n - 1].tile_end + n_tiles > 0x7fffffff))
        tflush();
      tcur_bits = p->uniform_bits;
      TileBatchEntry& e = tbatch.e[tbatch.n];
      e.words = it.words;
      e.mn = it.min;
      e.scale = it.scale;
      e.bits = mixed ? d_bits : nullptr;
      e.off = mixed ? p->d_off : nullptr;
      e.out = static_cast<u32x4*>(it.out_x);
      e.tile_end = (tbatch.n ? tbatch.e[tbatch.n - 1].tile_end : 0) + n_tiles;
      tbatch.ends[tbatch.n] = (uint32_t)e.tile_end;
      e.gs_log2 = gs_log2;
      e.cached = p->output_cached;
      ++tbatch.n;
      if (n_tiles * kTileChunks * kEpl < p->n)          // chunks and elements after the last whole tile
        err = launch_chunks<DT, false>(p, it.words, it.min, it.scale, d_bits, it.out_x, nullptr,
                                       n_tiles * kTileChunks, stream);
      continue;
    }
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
      batch.ends[batch.n] = (uint32_t)e.block_end;
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
  tflush();
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
