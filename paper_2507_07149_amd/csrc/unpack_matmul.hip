// Consumer fusion for a contraction: the weight gradient of y = x W^T,
//     dW[n, k] = sum_m grad_y[m, n] * xhat[m, k],
// computed straight from the packed activation.  Unpacking and dequantization (Algorithm 2,
// inverse of Eq. 1) are the prologue of every tile of the product: xhat goes from registers
// into LDS and from there into the matrix cores, and is never written to HBM (unpacking next
// to the consumer, Sec. 3.3 and Sec. 4.3.1).  This is the one dense contraction on the path,
// so it runs on MFMA (v_mfma_f32_32x32x16 for bf16 / f16, binary32 accumulation).
//
// Both operands have the reduction index m as their slow dimension in memory, while an MFMA
// lane needs 8 consecutive m for one row (of grad_y^T) or one column (of xhat).  The tiles go
// into LDS as they are (row = one m, columns contiguous) and are transposed by the operand
// reads: gfx950's ds_read_b64_tr_b16 hands lane L of each group of 16 lanes the L-th 16-bit
// element of each of the four 32-byte runs addressed by lanes 0-3, 4-7, 8-11 and 12-15.  With
// those four runs on four consecutive rows, a lane receives 4 consecutive m of its column; two
// such loads make one 8-element MFMA operand.  Rows are padded (stride = 64 bytes mod 256) so
// that the four rows of a load fall on different banks.
//
// Work-group tile: 256 (n) x BK (k) outputs, BK = 256 on 8 waves, or 128 or 64 on 4 waves; 32
// values of m per step.  A wave owns 64 (n) x 128 (k) (64 x 64 in the narrowest tile): 2 x 4
// MFMA blocks of 32 x 32, 128 accumulator registers, two waves per SIMD.  The wide n keeps the
// number of times a value of x is dequantized (once per tile of n) low; the wide k keeps the
// number of times a row of grad_y is fetched low.  Two copies of the LDS tiles: while the
// products read one, the next step's tiles are built in the other, next to the MFMA
// instructions; one barrier per step.  Global loads run two steps ahead of their use; the
// per-group constants are fetched once per work-group, six steps ahead, and passed through a
// ring in LDS.
#include "daf_device.h"
#include "daf_internal.h"

namespace {

using namespace daf;

constexpr int kBN = 256;
// The tile is BK = 64, 128 or 256 columns of k wide (a template parameter of the kernel).  Four
// waves side by side along n, each with all the columns of k up to 128; the 256-column tile
// has a second row of four waves for columns 128..255.  ES = bytes per element of grad_y and
// xhat: 2 (bf16, f16; 32 values of m per step) or 4 (binary32; 16 values of m per step, so
// that the LDS tiles have the same size).
template <int BK, int ES>
struct TileB {
  static constexpr int kBM = ES == 2 ? 32 : 16;     // values of m per step
  static constexpr int kThreads = BK > 128 ? 512 : 256;
  static constexpr int kWaveK = BK > 128 ? 128 : BK;        // columns of k per wave
  // Row strides in LDS: 64 bytes mod 256 for the transposing 16-bit reads (four rows of a load on
  // different banks), 128 bytes mod 256 for the plain 32-bit reads (the two rows of a load).
  static constexpr int kPad = ES == 2 ? 64 : 128;
  static constexpr int kRowA = kBN * ES + kPad;     // bytes per row of the grad_y tile in LDS
  static constexpr int kRow = BK * ES + kPad;       // bytes per row of the xhat tile in LDS
  static constexpr int kBufBytes = kBM * (kRowA + kRow);   // one copy of both tiles
  static constexpr int kGyChunks = kBN * ES / 16;   // 16-byte chunks per row of the grad_y tile
  static constexpr int kGyRows = kBM / (kThreads / kGyChunks);   // rows of the grad_y tile per thread: 4 or 2
  static constexpr int kSegs = BK / 8;              // 8-column segments per row
  static constexpr int kRowsPerPass = kThreads / kSegs;    // rows of x the threads cover at once
  static constexpr int kPasses = kBM >= kRowsPerPass ? kBM / kRowsPerPass : 1;   // 1 or 2
  // (binary32 with 64 columns: the threads cover 32 rows at once but a step has 16; the upper
  // half of the threads, whole waves, then has no part in the x tile)
  static constexpr bool kAllThreadsOnX = kBM >= kRowsPerPass;
  static constexpr int kJ = kWaveK / 32;            // MFMA blocks along k per wave
  // Per-group constants of a step (min, scale, width, word offset: 16 bytes per group) go
  // through a ring in LDS: at most BK / 32 groups per row of the tile (groups have >= 32 elements).
  static constexpr int kGroupsPerRow = BK / 32;
  static constexpr int kMetaEntries = kBM * kGroupsPerRow;          // per step
  static constexpr int kMetaRing = BK > 64 ? 8 : 5;                 // steps in the ring (5 is the minimum)
  static_assert(kGyRows >= 2, "tile shape");
};
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

template <int DT>
__device__ __forceinline__ f32x16 mfma_32x32x16(const uint4& a, const uint4& b, f32x16 c) {
  if constexpr (DT == kBF16) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                   0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0,
                                                  0);
  }
}

// binary32: one element of each operand per lane, two values of m per instruction
__device__ __forceinline__ f32x16 mfma_32x32x2(float a, float b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) i16x4 lds_i16x4;

// One MFMA operand: 8 consecutive m of the lane's column, from rows `p` (m .. m+3 across the
// lane groups) and `p + 4 rows`.
__device__ __forceinline__ uint4 operand_tr(const char* p, int row_bytes) {
  const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(p));
  const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(p + 4 * row_bytes));
  const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
  return make_uint4(l2.x, l2.y, h2.x, h2.y);
}

// The width and word offset of the group of a thread's segment, read from the ring one step
// before the words are requested.
template <int P>
struct Addr {
  uint32_t b[P], off[P];
};
// Everything a thread needs to build its share of one step's LDS tiles: 4 rows x 8 columns of
// grad_y, and the words and width of 8 columns of P rows of x.  Nothing here is computed from
// loaded values when it is requested (that would make the requesting step wait for its own loads).
template <int P, int R>
struct Stage {
  uint4 gy[R];
  uint32_t wa[P], wb[P], b[P];                      // the word of codes 0..3, the word of codes 4..7, the width
};

// A load from a block-uniform base plus a 32-bit per-thread byte offset: one address register
// per load instead of a 64-bit pair and the 64-bit arithmetic that makes it.
// A loop-invariant offset is passed through opaque() inside the loop: otherwise its widening to
// 64 bits is moved out of the loop and the scalar-base form of the load can no longer be chosen.
__device__ __forceinline__ uint32_t opaque(uint32_t v) {
  asm volatile("" : "+v"(v));
  return v;
}

template <class T>
__device__ __forceinline__ T load_at(const void* uniform_base, uint32_t byte_off) {
  const char* base = static_cast<const char*>(uniform_base);
  return *reinterpret_cast<const T*>(base + byte_off);
}

template <int I> struct Index { static constexpr int value = I; };
template <int N, int I = 0, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(Index<I>{});
    static_for<N, I + 1>(f);
  }
}

// Two binary32 values rounded to nearest-even in the 16-bit format, lo in bits 0..15 (the same
// patterns the plain dequantize kernel stores; the compiler's conversions are the hardware's
// round-to-nearest-even ones, one instruction per pair for bf16).
template <int DT>
__device__ __forceinline__ uint32_t narrow16_pair(float lo, float hi) {
  if constexpr (DT == kBF16) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
  } else {
    asm("" : "+v"(lo), "+v"(hi));                   // the binary32 values exist before they are rounded again
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    const f16x2 v = {(_Float16)lo, (_Float16)hi};
    return __builtin_bit_cast(uint32_t, v);
  }
}

// PARTIAL_N: N is not a multiple of 256 (see n_valid below); otherwise those checks are compiled out.
// Position in the tile sequence -> tile.  The sequence walks panels of four tile rows (n) column
// by column (k): 32 consecutive positions, which is what runs on one XCD at a time, are a patch of
// about 4 x 8 tiles that shares four panels of grad_y and eight of the packed x in that XCD's
// L2, where a row-major sequence shares one or two and thirty-two.  A bijection on
// [0, tiles_n * tiles_k); the last panel may be lower.
__device__ __forceinline__ void tile_of_position(uint32_t pos, uint32_t tiles_n, uint32_t tiles_k, uint32_t& tn,
                                                 uint32_t& tk) {
  constexpr uint32_t kPanel = 4;
  const uint32_t full = tiles_n / kPanel * kPanel;
  if (pos < full * tiles_k) {
    const uint32_t panel = pos / (kPanel * tiles_k), in = pos - panel * (kPanel * tiles_k);
    tn = panel * kPanel + in % kPanel;
    tk = in / kPanel;
  } else {
    const uint32_t rows = tiles_n - full, in = pos - full * tiles_k;
    tn = full + in % rows;
    tk = in / rows;
  }
}

template <int DT, bool MIXED, int BK, bool PARTIAL_N>
__global__ __launch_bounds__((TileB<BK, (DT == kF32 ? 4 : 2)>::kThreads), (BK > 128 ? 1 : 2)) void k_unpack_matmul(
    const uint32_t* __restrict__ words, const float* __restrict__ mn, const float* __restrict__ scale,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, uint32_t uniform_bits, int32_t gs,
    const void* __restrict__ grad_y, int64_t M, int64_t N, int64_t K, int32_t tiles_n, int32_t tiles_k,
    uint32_t whole, int32_t slices, float* __restrict__ out, float* __restrict__ partial) {
  constexpr int ES = DT == kF32 ? 4 : 2;
  using TB = TileB<BK, ES>;
  constexpr int kBM = TB::kBM, kRowA = TB::kRowA, kRowB = TB::kRow, kBufBytes = TB::kBufBytes, kP = TB::kPasses,
                kJ = TB::kJ, kR = TB::kGyRows;
  // Two copies of: the grad_y tile (kBM rows of kRowA bytes), then the xhat tile (kBM rows of
  // kRowB bytes).  While the products read one copy, the next step's tiles are written into the other.
  __shared__ __attribute__((aligned(16))) char lds[2][kBufBytes];
  // Ring of per-group constants: slot (q mod kMetaRing) holds {min, scale, width, word offset}
  // of the groups of step q, entry = row * kGroupsPerRow + (group - first group of the tile).
  __shared__ uint4 meta[TB::kMetaRing][TB::kMetaEntries];

  const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
  // The first `whole` work-groups take one tile each over all of m and write it to `out`; the
  // tiles after those are each taken by `slices` work-groups, one slice of m each, which write
  // their partial sums to `partial` as compact tiles [slice][tile - whole][256][BK].
  // Consecutive block ids go to different XCDs (each with its own L2).  Give every XCD a
  // contiguous range of the tile sequence (tile_of_position): the tiles resident on an XCD at
  // one time are then a compact patch.
  const uint32_t n_tiles = (uint32_t)tiles_n * (uint32_t)tiles_k;
  const uint32_t bid = blockIdx.x;
  const bool sliced = bid >= whole;
  const uint32_t count = sliced ? n_tiles - whole : whole;       // tiles of this kind
  const uint32_t rel = sliced ? bid - whole : bid;
  const uint32_t slice = sliced ? rel / count : 0u;
  uint32_t ti = rel - slice * count;
  {
    const uint32_t xcd = ti & 7u, idx = ti >> 3;
    const uint32_t base = count / 8u, rem = count & 7u;          // XCD x owns base (+1 if x < rem) tiles
    ti = xcd * base + (xcd < rem ? xcd : rem) + idx;
  }
  const uint32_t tile = sliced ? whole + ti : ti;
  uint32_t tn, tk;
  tile_of_position(tile, (uint32_t)tiles_n, (uint32_t)tiles_k, tn, tk);
  const int64_t n0 = (int64_t)tn * kBN, k0 = (int64_t)tk * BK;
  // The last tile of n may reach past the output (N is a multiple of 64, not of 256): the waves
  // whose 64 columns lie outside take part in the loads and the tile construction but run no
  // products and store nothing; the chunks of grad_y outside are read from column 0 instead.
  const uint32_t n_valid = PARTIAL_N ? (uint32_t)((N - n0) < kBN ? (N - n0) : kBN) : (uint32_t)kBN;
  // The steps of m are dealt out to the slices as evenly as whole steps allow.
  const int all_steps = (int)(M / kBM);
  const int per = sliced ? all_steps / slices : all_steps, extra = sliced ? all_steps % slices : 0;
  const int steps = per + ((int)slice < extra ? 1 : 0);
  const int64_t m_begin = ((int64_t)slice * per + ((int)slice < extra ? (int)slice : extra)) * kBM;

  // Loader roles.  grad_y: thread (cg, rq) owns rows kR*rq .. kR*rq+kR-1 of the step and columns
  // 16 bytes of the 256 columns.  x: thread (co, xr) owns columns 8*co .. 8*co+7 of the BK in row
  // xr (and, for BK = 128, row xr + 16).  Addresses are a block-uniform 64-bit base that
  // advances by a constant per step, plus 32-bit per-thread byte offsets.
  const uint32_t cg = t % (uint32_t)TB::kGyChunks, rq = t / (uint32_t)TB::kGyChunks;
  const uint32_t co = t % (uint32_t)TB::kSegs, xr = t / (uint32_t)TB::kSegs;
  const bool on_x = TB::kAllThreadsOnX || xr < (uint32_t)kBM;          // (uniform per wave)
  const uint32_t row_bytes = (uint32_t)N * (uint32_t)ES;                // bytes per grad_y row
  const uint32_t gpr = (uint32_t)(K / gs);                              // groups per row of x
  const uint32_t k_col = (uint32_t)k0 + 8u * co;
  const uint32_t gk = k_col / (uint32_t)gs;
  const uint32_t in_group = k_col - gk * (uint32_t)gs;                  // multiple of 8
  const uint32_t wpgb = (uint32_t)gs >> 5;                              // words per group and bit of width
  const char* gy_base = reinterpret_cast<const char*>(grad_y) + (m_begin * (int64_t)row_bytes + n0 * ES);
  const uint32_t gy_voff = ((uint32_t)kR * rq) * row_bytes + (cg * (16u / ES) < n_valid ? 16u * cg : 0u);
  const int64_t g_step0 = m_begin * (int64_t)gpr;                        // uniform; + 32*gpr per step

  // The per-group constants are fetched once per work-group and step, one group per thread
  // (threads 0 .. 32 * kGroupsPerRow - 1: whole waves), six steps ahead, and handed to the
  // threads that need them through the ring: four small loads per thread and step of its own
  // would keep the memory pipeline busier than the tiles of grad_y do.
  const uint32_t g_first = (uint32_t)k0 / (uint32_t)gs;
  const uint32_t n_groups = ((uint32_t)k0 + (uint32_t)BK - 1u) / (uint32_t)gs - g_first + 1u;   // <= kGroupsPerRow
  const bool meta_wave = t < (uint32_t)TB::kMetaEntries;
  const uint32_t m_row = t / (uint32_t)TB::kGroupsPerRow, m_j = t % (uint32_t)TB::kGroupsPerRow;
  const bool meta_lane = meta_wave && m_j < n_groups;
  const uint32_t m_goff = m_row * gpr + g_first + m_j;                  // the loader's group, relative to the step's first
  const uint32_t my_entry = xr * (uint32_t)TB::kGroupsPerRow + (gk - g_first);   // the consumer's entry (pass 0)

  const int64_t g_stride = kBM * (int64_t)gpr;                           // groups per step
  const int64_t gy_stride = kBM * (int64_t)row_bytes;                    // bytes of grad_y per step
  // gu: index of the step's first group (uniform)
  auto meta_load = [&](uint4& mv, int64_t gu) __attribute__((always_inline)) {
    if (meta_lane) {
      const uint32_t mo = opaque(m_goff), mo4 = 4u * mo;
      mv.x = __builtin_bit_cast(uint32_t, load_at<float>(mn + gu, mo4));
      mv.y = __builtin_bit_cast(uint32_t, load_at<float>(scale + gu, mo4));
      if (MIXED) {
        mv.z = load_at<uint8_t>(bits + gu, mo);
        mv.w = load_at<uint32_t>(off + gu, mo4);
      } else {
        mv.z = uniform_bits;
        mv.w = ((uint32_t)gu + m_goff) * (wpgb * uniform_bits);
      }
    }
  };
  auto meta_store = [&](const uint4& mv, uint32_t slot) __attribute__((always_inline)) {
    if (meta_lane) meta[slot][t] = mv;
  };
  const uint32_t g_voff = xr * gpr + gk;                                 // the thread's group, relative to the step's first
  auto fetch_addr = [&](Addr<kP>& ad, uint32_t slot, int step) __attribute__((always_inline)) {
    if (!on_x) return;
#pragma unroll
    for (int p = 0; p < kP; ++p) {
      if (MIXED) {
        const uint4* e = &meta[slot][my_entry + (uint32_t)(p * TB::kRowsPerPass * TB::kGroupsPerRow)];
        const uint2 v = *reinterpret_cast<const uint2*>(reinterpret_cast<const char*>(e) + 8);
        ad.b[p] = v.x;
        ad.off[p] = v.y;
      } else {                                      // one width: the offset follows from the group's index
        const uint32_t g = (uint32_t)(g_step0 + (int64_t)step * (kBM * (int64_t)gpr)) + g_voff +
                           (uint32_t)(p * TB::kRowsPerPass) * gpr;
        ad.b[p] = uniform_bits;
        ad.off[p] = g * (wpgb * uniform_bits);
      }
    }
  };
  // gp: the step's rows of grad_y, at the tile's first column (uniform)
  auto fetch_stage = [&](Stage<kP, kR>& f, const Addr<kP>& ad, const char* gp) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < kR; ++r) {
      const u32x4 v = load_at<u32x4>(gp + (int64_t)r * row_bytes, opaque(gy_voff));   // (per load: else rows 1..3 get vector addresses)
      f.gy[r] = make_uint4(v.x, v.y, v.z, v.w);
    }
    if (!on_x) return;
#pragma unroll
    for (int p = 0; p < kP; ++p) {
      // The 8 codes lie in one word, or (8 bits) in two: codes 0..3 in the first, 4..7 in the next.
      const uint32_t wi = ad.off[p] + (__umul24(in_group, ad.b[p]) >> 5);   // (both factors are small)
      f.wa[p] = load_at<uint32_t>(words, 4u * wi);
      f.wb[p] = load_at<uint32_t>(words, 4u * (wi + (ad.b[p] >> 3)));
      f.b[p] = ad.b[p];
    }
  };

  f32x16 acc[2][kJ];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < kJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const uint32_t wn = wave & 3u, wk = wave >> 2;    // (wk = 0 except for the 256-column tile)
  const bool wave_valid = !PARTIAL_N || 64u * wn < n_valid;   // (uniform per wave)
  const uint32_t li = lane & 31u, lg = lane >> 5;
  // Operand reads, 16-bit formats: lane l of 16-lane group G = l / 16 addresses row
  // 8*(l/32) + (l%16)/4 (plus 16 per sub-step, plus 4 for the second half of the operand) and
  // the 4 columns 16*(G%2) + 4*(l%4) .. of its 32-column block; it receives column
  // 16*(G%2) + l%16 = l%32 of the block.  In odd rows of the xhat tile the two 8-byte halves of
  // every 16 bytes are exchanged: the writes of two neighbouring rows (one instruction) then
  // fall on different banks.  binary32: lane l reads the element in row l/32 (plus 2 per pair of
  // m), column l%32 of its block: no transposition is needed with one element per lane.
  const uint32_t tr_row = 8u * lg + ((lane & 15u) >> 2), tr_col = 16u * ((lane >> 4) & 1u) + 4u * (lane & 3u);
  const uint32_t a_read = ES == 2 ? tr_row * (uint32_t)kRowA + (64u * wn + tr_col) * 2u
                                  : lg * (uint32_t)kRowA + (64u * wn + li) * 4u;
  const uint32_t b_read = (uint32_t)(kBM * kRowA) + wk * (uint32_t)(TB::kWaveK * ES) +
                          (ES == 2 ? tr_row * (uint32_t)kRowB + ((tr_col * 2u) ^ (8u * (tr_row & 1u)))
                                   : lg * (uint32_t)kRowB + li * 4u);

  // Half of the work of turning a stage into LDS tiles: half of the thread's grad_y rows
  // (copied as loaded) and half of each of its rows of x.
  const uint32_t a_store = ((uint32_t)kR * rq) * (uint32_t)kRowA + 16u * cg;
  const uint32_t b_store = (uint32_t)(kBM * kRowA) + xr * (uint32_t)kRowB +
                           (ES == 2 ? 16u * co + 8u * (xr & 1u) : 32u * co);
  auto build_half = [&](const Stage<kP, kR>& cur, char* buf, int hs, uint32_t slot) __attribute__((always_inline)) {
#pragma unroll
    for (int rr = 0; rr < kR / 2; ++rr) {
      const int r = (kR / 2) * hs + rr;
      *reinterpret_cast<uint4*>(buf + a_store + (uint32_t)r * kRowA) = cur.gy[r];
    }
    if (!on_x) return;
    // ---- xhat: unpack, dequantize, round to the element format; 4 columns of the row ----
    // Element j of a group has its lowest bit at bit -(j + 1) * b (mod 32) of its word; the
    // bit-field extract takes its offset mod 32, which also covers the second word of 8-bit codes.
#pragma unroll
    for (int p = 0; p < kP; ++p) {
      const uint32_t b = cur.b[p];
      uint32_t w = hs ? cur.wb[p] : cur.wa[p];
      // The word is taken here, after the barrier that ended the step before: moved up into
      // that step, its unpacking would wait for the loads requested last.
      asm volatile("" : "+v"(w));
      const float2 ms = *reinterpret_cast<const float2*>(
          &meta[slot][my_entry + (uint32_t)(p * TB::kRowsPerPass * TB::kGroupsPerRow)]);   // {min, scale}
      uint32_t sh = (uint32_t)__mul24((int)b, -(int)(in_group + 4u * (uint32_t)hs + 1u));
      float v[4];
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) {
        const uint32_t code = __builtin_amdgcn_ubfe(w, sh, b);
        sh -= b;
        v[cc] = __builtin_fmaf((float)code, ms.y, ms.x);
      }
      if constexpr (ES == 2) {
        *reinterpret_cast<uint2*>(buf + ((b_store + (uint32_t)(p * TB::kRowsPerPass * kRowB)) ^ (8u * (uint32_t)hs))) =
            make_uint2(narrow16_pair<DT>(v[0], v[1]), narrow16_pair<DT>(v[2], v[3]));
      } else {
        *reinterpret_cast<float4*>(buf + b_store + (uint32_t)(p * TB::kRowsPerPass * kRowB) + 16u * (uint32_t)hs) =
            make_float4(v[0], v[1], v[2], v[3]);
      }
    }
  };

  // Position in the ring of the step c steps after the one whose position is `at`.
  constexpr uint32_t kRing = (uint32_t)TB::kMetaRing;
  auto ring = [&](uint32_t at, uint32_t c) __attribute__((always_inline)) {
    const uint32_t v = at + c;                      // at < kRing, c <= kRing
    if constexpr ((kRing & (kRing - 1u)) == 0u) return v & (kRing - 1u);
    return v >= kRing ? v - kRing : v;
  };

  // One step: run the products on copy BUF of the tiles while building the next step's tiles
  // (from `next`) in the other copy, then request the loads of the step after that into the
  // registers just consumed.  `at` is the step's position in the ring of group constants.
  uint4 mv;                                         // group constants on their way into the ring
  const char* gy_next;                              // rows of grad_y of the step requested next
  int64_t gu_meta;                                  // first group of the step whose constants are requested next
  auto do_step = [&](auto BUF, Stage<kP, kR>& next, Addr<kP>& ad_use, Addr<kP>& ad_fill, int step, uint32_t& at)
                     __attribute__((always_inline)) {
    constexpr int buf = decltype(BUF)::value;
    // Group constants: those requested one step ago (of step + 5) go into the ring, those of
    // step + 6 are requested; width and offset of step + 4 (stored one step ago) are read.
    if (meta_wave) {
      meta_store(mv, ring(at, 5));
      meta_load(mv, gu_meta);
    }
    if (step + 6 < steps - 1) gu_meta += g_stride;  // (past the end the last step's are requested again)
    fetch_addr(ad_fill, ring(at, 4), min(step + 4, steps - 1));
    const char* a_lds = lds[buf] + a_read;
    const char* b_lds = lds[buf] + b_read;
#pragma unroll
    for (int ss = 0; ss < 2; ++ss) {                // two halves of the step, a half of the next tiles built in each
      if (!wave_valid) {                            // (a wave outside the output only helps to build the tiles)
        build_half(next, lds[buf ^ 1], ss, ring(at, 1));
      } else if constexpr (ES == 2) {
        uint4 a[2], b[kJ];
#pragma unroll
        for (int i = 0; i < 2; ++i) a[i] = operand_tr(a_lds + ss * 16 * kRowA + i * 64, kRowA);
#pragma unroll
        for (int j = 0; j < kJ; ++j) b[j] = operand_tr(b_lds + ss * 16 * kRowB + j * 64, kRowB);
        build_half(next, lds[buf ^ 1], ss, ring(at, 1));
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < kJ; ++j) acc[i][j] = mfma_32x32x16<DT>(a[i], b[j], acc[i][j]);
      } else {
        build_half(next, lds[buf ^ 1], ss, ring(at, 1));
#pragma unroll
        for (int kk = 0; kk < kBM / 4; ++kk) {        // pairs of m in this half
          const int row = ss * (kBM / 2) + 2 * kk;
          float a[2], b[kJ];
#pragma unroll
          for (int i = 0; i < 2; ++i) a[i] = *reinterpret_cast<const float*>(a_lds + row * kRowA + i * 128);
#pragma unroll
          for (int j = 0; j < kJ; ++j) b[j] = *reinterpret_cast<const float*>(b_lds + row * kRowB + j * 128);
#pragma unroll
          for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < kJ; ++j) acc[i][j] = mfma_32x32x2(a[i], b[j], acc[i][j]);
        }
      }
    }
    // Requested unconditionally (past the end the last step is requested again and never
    // used), so that the number of loads in flight is the same in every iteration.
    fetch_stage(next, ad_use, gy_next);
    if (step + 3 < steps - 1) gy_next += gy_stride;
    __syncthreads();                                // the other copies are complete, this one is free
    at = ring(at, 1);
  };

  // Step q lives in stage q % 2 and LDS copy q % 2, its width and offset in ad[q % 2] (read
  // one step before its words are requested), its group constants in ring position q mod kRing.
  // Prologue: group constants of steps 0..4 in the ring, those of step 5 requested; tiles of
  // step 0 built; loads of steps 1 and 2 requested.
  Stage<kP, kR> st[2];
  Addr<kP> ad[2];
  if (meta_wave) {
    uint4 m0[5];                                    // all requested before the first is stored: one load latency
#pragma unroll
    for (int q = 0; q < 5; ++q) {
      m0[q] = make_uint4(0u, 0u, 0u, 0u);
      meta_load(m0[q], g_step0 + (int64_t)min(q, steps - 1) * g_stride);
    }
    meta_load(mv, g_step0 + (int64_t)min(5, steps - 1) * g_stride);
#pragma unroll
    for (int q = 0; q < 5; ++q) meta_store(m0[q], (uint32_t)q);
  }
  gu_meta = g_step0 + (int64_t)min(6, steps - 1) * g_stride;
  __syncthreads();
  fetch_addr(ad[0], 0u, 0);
  fetch_addr(ad[1], 1u, min(1, steps - 1));
  fetch_stage(st[0], ad[0], gy_base);
  fetch_addr(ad[0], 2u, min(2, steps - 1));
  fetch_stage(st[1], ad[1], gy_base + min(1, steps - 1) * gy_stride);
  build_half(st[0], lds[0], 0, 0u);
  build_half(st[0], lds[0], 1, 0u);
  fetch_addr(ad[1], 3u, min(3, steps - 1));
  fetch_stage(st[0], ad[0], gy_base + min(2, steps - 1) * gy_stride);
  gy_next = gy_base + min(3, steps - 1) * gy_stride;
  // Every load has arrived before the loop is entered (once per work-group): the waits at the
  // top of the loop must hold on this path too, and are then the ones its own iterations need.
  __builtin_amdgcn_s_waitcnt(0x0F70);               // vmcnt(0)
  __syncthreads();
  __builtin_amdgcn_sched_barrier(0);

  // In iteration s: products on copy s % 2; tiles of step s+1 (stage (s+1) % 2) into the other
  // copy; then loads of step s+3 into that same stage, with the width and offset in
  // ad[(s+1) % 2] (read in iteration s-1); width and offset of step s+4 into ad[s % 2].
  uint32_t at = 0u;
  int base = 0;
  for (; base + 2 <= steps; base += 2) {
    do_step(Index<0>{}, st[1], ad[1], ad[0], base, at);
    do_step(Index<1>{}, st[0], ad[0], ad[1], base + 1, at);
  }
  if (base < steps) do_step(Index<0>{}, st[1], ad[1], ad[0], base, at);

  // ---- epilogue: register r of a 32 x 32 block is row 8*(r/4) + 4*(lane/32) + r%4, column lane%32 ----
  float* dst = sliced ? partial + ((int64_t)slice * count + ti) * (int64_t)(kBN * BK) : out + n0 * K + k0;
  const int64_t ld = sliced ? BK : K;
  if (!wave_valid) return;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < kJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t n = 64 * wn + 32 * i + 8 * (r >> 2) + 4 * lg + (r & 3);
        const int64_t k = TB::kWaveK * wk + 32 * j + li;
        dst[n * ld + k] = acc[i][j][r];
      }
}

// The sliced tiles: out[tile] = sum over the slices of partial[slice][tile - whole]; one
// work-group per 256 x 16 strip of a tile (bk4 = BK / 4 float4 per row).  A launch adds n
// slices that lie `stride` slices apart, starting at slice blockIdx.y * n * stride, and writes
// the sum over the first of them (TO_OUT = false) or into the output (TO_OUT = true, one group):
// more than 16 slices are added in two levels, 16 at a time and then the 16th ones, so that
// the additions of one output are spread over several work-groups.
template <bool TO_OUT>
__global__ __launch_bounds__(256) void k_sum_slices(float4* __restrict__ partial, uint32_t whole, uint32_t count,
                                                    int32_t slices, int32_t n, int32_t stride, uint32_t tiles_n,
                                                    int32_t tiles_k,
                                                    int32_t bk4, int64_t N, int64_t K, float* __restrict__ out) {
  const uint32_t strips = (uint32_t)(kBN * bk4) / 256u;           // work-groups per tile
  const uint32_t ti = blockIdx.x / strips;
  const uint32_t e = (blockIdx.x - ti * strips) * 256u + threadIdx.x;   // float4 index inside the tile
  const int64_t tile4 = (int64_t)kBN * bk4;
  const uint32_t tile = whole + ti;
  uint32_t tn, tk;
  tile_of_position(tile, tiles_n, (uint32_t)tiles_k, tn, tk);
  const uint32_t row = e / (uint32_t)bk4, col4 = e - row * (uint32_t)bk4;
  if ((int64_t)tn * kBN + row >= N) return;          // rows of the last tile of n past the output
  const int32_t first = (int32_t)blockIdx.y * n * stride;
  float4* p0 = partial + ((int64_t)first * count + ti) * tile4 + e;
  float4 s = *p0;
  for (int32_t j = 1; j < n && first + j * stride < slices; ++j) {
    const float4 v = p0[(int64_t)j * stride * count * tile4];
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  if (TO_OUT) {
    float* dst = out + ((int64_t)tn * kBN + row) * K + (int64_t)tk * (bk4 * 4) + 4 * col4;
    *reinterpret_cast<float4*>(dst) = s;
  } else {
    *p0 = s;
  }
}

}  // namespace

// M is a multiple of 32 for every element format (the 16-bit kernels take 32 values of m per
// step, the binary32 kernel 16); the slicing below counts m in units of 32.
constexpr int kStepM = 32;

// Width of the tile along k.  Each doubling halves the number of times a row of grad_y is
// fetched; the 256-column tile (8 waves, one work-group per CU) is used when the output has
// enough of them to fill the chip without slicing m, else the 128-column one (measured: LLM
// shape 780 -> 860 TFLOP/s with 256 columns, ViT shape 0.30 against 0.29 ms).
static int tile_bk(int64_t N, int64_t K) {
  if (K % 256 == 0 && ((N + kBN - 1) / kBN) * (K / 256) >= 256) return 256;
  return K % 128 == 0 ? 128 : 64;
}

// How the tiles are run.  Work-groups run in rounds of as many as fit on the chip (slots: 1 per
// CU with the 256-column tile, 2 with the 128-column one, 3 with the 64-column one; 256 CUs).
// The tiles of the whole rounds run over all of m; the tiles of a last, partly filled round
// (all tiles, when there is less than one round) may be cut into `slices` slices of m (2 to 16,
// more for outputs of a few tiles; of as equal a number of steps as possible) that run as work-groups of their own
// and leave partial sums: a round of those takes 1/slices of the time, and the partial sums
// (kept below 256 MiB) are written once and read once more at about 4 TB/s.  The cheapest
// choice by that estimate; the per-step times are measured ones.
namespace {
struct Schedule {
  int bk;
  int64_t tiles, whole;    // tiles in all; tiles that run over all of m
  int32_t slices;          // of each other tile (1: there is none)
};
Schedule schedule(int64_t M, int64_t N, int64_t K, int es) {   // es: bytes per element (2 or 4)
  Schedule sc;
  sc.bk = tile_bk(N, K);
  sc.tiles = ((N + kBN - 1) / kBN) * (K / sc.bk);
  const int64_t slots = 256 * (sc.bk == 256 ? 1 : sc.bk == 128 ? 2 : 3);
  const int64_t steps = M / kStepM;
  // one work-group over all of m, per 32 values of m: the 16-bit kernels are bound by instruction
  // issue, the binary32 kernel by its MFMAs (128 per wave of 64 cycles each)
  const double t_all_m = (double)steps * (es == 4 ? 8.0e-6 : sc.bk == 256 ? 1.1e-6 : 1.25e-6);
  const double tile_bytes = (double)kBN * sc.bk * 4.0;
  sc.whole = sc.tiles;
  sc.slices = 1;
  double best_cost = (double)((sc.tiles + slots - 1) / slots) * t_all_m;
  const int64_t whole = sc.tiles / slots * slots, rest = sc.tiles - whole;
  if (rest == 0) return sc;
  // (at most 16 slices, or, for outputs of a few tiles only, as many as fill the chip once)
  const int64_t max_slices = rest * 16 >= slots ? 16 : (slots / rest < 256 ? slots / rest : 256);
  for (int32_t s = 2; s <= max_slices && steps >= 4 * s; ++s) {
    if ((double)s * rest * tile_bytes > 256.0 * 1048576.0) break;
    const double longest = (double)((steps + s - 1) / s) / (double)steps;      // share of m of the longest slice
    const double cost = (double)(whole / slots) * t_all_m + (double)((rest * s + slots - 1) / slots) * t_all_m * longest +
                        (2 * s + 1) * rest * tile_bytes / 4.0e12;
    if (cost < best_cost * 0.98) {                   // (a clear gain only)
      best_cost = cost;
      sc.whole = whole;
      sc.slices = s;
    }
  }
  return sc;
}
}  // namespace

// The number of slices depends on the element format (the binary32 kernel is slower per step,
// so more slices pay off); the workspace is sized for the larger of the two.
int64_t daf_unpack_matmul_workspace_size(int64_t M, int64_t N, int64_t K) {
  int64_t bytes = 0;
  for (int es = 2; es <= 4; es += 2) {
    const Schedule sc = schedule(M, N, K, es);
    const int64_t b = sc.slices > 1 ? (int64_t)sc.slices * (sc.tiles - sc.whole) * kBN * sc.bk * 4 : 0;
    bytes = b > bytes ? b : bytes;
  }
  return bytes;
}

bool daf_unpack_matmul_shape_ok(int64_t M, int64_t N, int64_t K, int32_t gs) {
  // N and K below 2^24: the per-thread parts of the addresses are 32-bit byte offsets.
  // (N a multiple of 64: a wave's 64 columns of n are inside the output or outside it as a whole)
  return M > 0 && N > 0 && K > 0 && M % kStepM == 0 && N % 64 == 0 && K % 64 == 0 && K % gs == 0 &&
         N < (1 << 24) && K < (1 << 24) && ((N + kBN - 1) / kBN) * (K / 64) * 16 < (int64_t)1 << 31;
}

hipError_t daf_launch_unpack_matmul(const daf_plan_t* p, const uint32_t* words, const float* mn, const float* scale,
                                    const uint8_t* d_bits, const void* grad_y, int64_t N, int64_t K, int dtype,
                                    float* out, float* workspace, hipStream_t stream) {
  const int64_t M = p->n / K;
  const Schedule sc = schedule(M, N, K, dtype == daf::kF32 ? 4 : 2);
  const int bk = sc.bk;
  const int32_t tiles_n = (int32_t)((N + kBN - 1) / kBN), tiles_k = (int32_t)(K / bk);
  const int64_t rest = sc.tiles - sc.whole;
  const unsigned blocks = (unsigned)(sc.whole + rest * sc.slices);
  const uint32_t whole = (uint32_t)sc.whole;
  const int32_t slices = sc.slices;
  const void* gy = grad_y;
#define DAF_LAUNCH_P(DT, MIXED, BK, PARTIAL)                                                                               \
  hipLaunchKernelGGL((k_unpack_matmul<DT, MIXED, BK, PARTIAL>), dim3(blocks),                                     \
                     dim3(TileB<BK, DT == daf::kF32 ? 4 : 2>::kThreads), 0, stream, words,                        \
                     mn, scale,                                                                                   \
                     d_bits, p->d_off, (uint32_t)p->uniform_bits, p->group_size, gy, M, N, K, tiles_n, tiles_k,   \
                     whole, slices, out, workspace)
#define DAF_LAUNCH(DT, MIXED, BK)                                                                                 \
  do {                                                                                                            \
    if (N % kBN == 0) DAF_LAUNCH_P(DT, MIXED, BK, false); else DAF_LAUNCH_P(DT, MIXED, BK, true);                 \
  } while (0)
#define DAF_LAUNCH_BK(DT, MIXED)                                                                                  \
  do {                                                                                                            \
    if (bk == 256) DAF_LAUNCH(DT, MIXED, 256);                                                                    \
    else if (bk == 128) DAF_LAUNCH(DT, MIXED, 128);                                                               \
    else DAF_LAUNCH(DT, MIXED, 64);                                                                               \
  } while (0)
  if (dtype == daf::kBF16) {
    if (p->uniform_bits) DAF_LAUNCH_BK(daf::kBF16, false); else DAF_LAUNCH_BK(daf::kBF16, true);
  } else if (dtype == daf::kF16) {
    if (p->uniform_bits) DAF_LAUNCH_BK(daf::kF16, false); else DAF_LAUNCH_BK(daf::kF16, true);
  } else if (dtype == daf::kF32) {
    if (p->uniform_bits) DAF_LAUNCH_BK(daf::kF32, false); else DAF_LAUNCH_BK(daf::kF32, true);
  } else {
    return hipErrorInvalidValue;
  }
#undef DAF_LAUNCH_BK
#undef DAF_LAUNCH
#undef DAF_LAUNCH_P
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || rest == 0) return e;
  const int32_t bk4 = bk / 4;
  const unsigned rblocks = (unsigned)(rest * (kBN * bk4 / 256));
  float4* part = reinterpret_cast<float4*>(workspace);
  int32_t n = slices, stride = 1;
  if (slices > 16) {                                  // first level: every 16 slices into the first of them
    const unsigned chunks = (unsigned)((slices + 15) / 16);
    hipLaunchKernelGGL(k_sum_slices<false>, dim3(rblocks, chunks), dim3(256), 0, stream, part, whole, (uint32_t)rest,
                       slices, 16, 1, (uint32_t)tiles_n, tiles_k, bk4, N, K, out);
    n = (int32_t)chunks;
    stride = 16;
  }
  hipLaunchKernelGGL(k_sum_slices<true>, dim3(rblocks, 1), dim3(256), 0, stream, part, whole, (uint32_t)rest, slices, n,
                     stride, (uint32_t)tiles_n, tiles_k, bk4, N, K, out);
  return hipGetLastError();
}
