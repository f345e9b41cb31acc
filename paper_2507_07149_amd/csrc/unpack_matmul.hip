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
// Work-group tile: 256 (n) x 64 (k) outputs, 32 values of m per step, 4 waves of 64 x 64
// each (2 x 2 MFMA blocks of 32 x 32, 64 accumulator registers).  The wide n keeps the number
// of times a value of x is dequantized (once per tile of n) low; the small wave tile keeps the
// register count low enough for several work-groups per CU, which is what hides the latencies
// of one wave behind the work of another.  Two copies of the LDS tiles: while the products
// read one, the next step's tiles are built in the other, between the MFMA instructions.
#include "daf_device.h"
#include "daf_internal.h"

namespace {

using namespace daf;

constexpr int kBN = 256, kBK = 64, kBM = 32, kThreads = 256;
constexpr int kRowA = kBN * 2 + 64;                 // bytes per row of the grad_y tile in LDS (padded)
constexpr int kRowB = kBK * 2 + 64;                 // bytes per row of the xhat tile in LDS (padded)
constexpr int kBufBytes = kBM * (kRowA + kRowB);    // one copy of both tiles
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

// With per-group widths the address of a row's words depends on off[] and bits[] of its group:
// those are fetched one step before the words are requested.
struct Addr {
  uint32_t b, off;
};
// Everything a thread needs to build its share of one step's LDS tiles: 4 rows x 8 columns of
// grad_y, and the words, width, min and scale of 8 columns of one row of x.
struct Stage {
  uint4 gy[4];
  uint32_t w0, w1, b;                               // code c < 4 is in w0, c >= 4 in w1 (the same word below 8 bits)
  float mn, sc;
};

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

template <int DT, bool MIXED>
__global__ __launch_bounds__(kThreads, 2) void k_unpack_matmul(
    const uint32_t* __restrict__ words, const float* __restrict__ mn, const float* __restrict__ scale,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, uint32_t uniform_bits, int32_t gs,
    const u32x4* __restrict__ grad_y, int64_t M, int64_t N, int64_t K, int32_t tiles_n, int32_t tiles_k,
    int32_t splits, uint32_t total_words, float* __restrict__ out) {
  // Two copies of: the grad_y tile (kBM rows of kRowA bytes), then the xhat tile (kBM rows of
  // kRowB bytes).  While the products read one copy, the next step's tiles are written into the other.
  __shared__ __attribute__((aligned(16))) char lds[2][kBufBytes];

  const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
  // Consecutive block ids go to different XCDs (each with its own L2).  Give every XCD a
  // contiguous range of the tile sequence, and order the sequence in bands of 4 tiles of n, k
  // running inside a band: the ~32 tiles resident on an XCD then form a 4 x 8 patch that reads
  // 4 panels of grad_y and 8 (small) panels of packed words per step instead of all 16 of grad_y.
  const uint32_t n_tiles = (uint32_t)tiles_n * (uint32_t)tiles_k;
  const uint32_t bid = blockIdx.x;
  const uint32_t split = bid / n_tiles;
  uint32_t tile = bid - split * n_tiles;
  {
    const uint32_t xcd = tile & 7u, idx = tile >> 3;
    const uint32_t base = n_tiles / 8u, rem = n_tiles & 7u;       // XCD x owns base (+1 if x < rem) tiles
    tile = xcd * base + (xcd < rem ? xcd : rem) + idx;
  }
  constexpr uint32_t kBand = 1;
  const uint32_t band = tile / (kBand * (uint32_t)tiles_k);
  const uint32_t in_band = tile - band * (kBand * (uint32_t)tiles_k);
  const uint32_t band_h = ((uint32_t)tiles_n - band * kBand) < kBand ? ((uint32_t)tiles_n - band * kBand) : kBand;
  const uint32_t tn = band * kBand + in_band % band_h, tk = in_band / band_h;
  const int64_t n0 = (int64_t)tn * kBN, k0 = (int64_t)tk * kBK;
  const int64_t m_per_split = M / splits;
  const int64_t m_begin = (int64_t)split * m_per_split;
  const int steps = (int)(m_per_split / kBM);

  // Loader roles.  grad_y: thread (cg, rq) owns rows 4*rq .. 4*rq+3 of the step and columns
  // 8*cg .. 8*cg+7 of the 256.  x: thread (co, xr) owns row xr and columns 8*co .. 8*co+7 of the
  // 64: one load instruction each for its words, min, scale (and width, offset) per step.  Addresses are a block-uniform 64-bit base that advances by a
  // constant per step, plus 32-bit per-thread offsets.
  const uint32_t cg = t & 31u, rq = t >> 5;
  const uint32_t co = t & 7u, xr = t >> 3;
  const uint32_t row_chunks = (uint32_t)(N / 8);                        // 16-byte chunks per grad_y row
  const uint32_t gpr = (uint32_t)(K / gs);                              // groups per row of x
  const uint32_t k_col = (uint32_t)k0 + 8u * co;
  const uint32_t gk = k_col / (uint32_t)gs;
  const uint32_t in_group = k_col - gk * (uint32_t)gs;                  // multiple of 8
  const uint32_t wpgb = (uint32_t)gs >> 5;                              // words per group and bit of width
  const u32x4* gy_step = grad_y + m_begin * (int64_t)row_chunks + n0 / 8;   // uniform; + 32 rows per step
  const uint32_t gy_off = (4u * rq) * row_chunks + cg;
  const int64_t g_step0 = m_begin * (int64_t)gpr;                        // uniform; + 32*gpr per step
  const uint32_t g_off = xr * gpr + gk;

  auto fetch_addr = [&](Addr& ad, int step) __attribute__((always_inline)) {
    const int64_t g = g_step0 + (int64_t)step * (kBM * (int64_t)gpr) + g_off;
    if (MIXED) {
      ad.b = bits[g];
      ad.off = off[g];
    } else {
      ad.b = uniform_bits;
      ad.off = (uint32_t)g * (wpgb * uniform_bits);
    }
  };
  auto fetch_stage = [&](Stage& f, const Addr& ad, int step) __attribute__((always_inline)) {
    const u32x4* gp = gy_step + (int64_t)step * (kBM * (int64_t)row_chunks);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const u32x4 v = gp[gy_off + (uint32_t)r * row_chunks];
      f.gy[r] = make_uint4(v.x, v.y, v.z, v.w);
    }
    // The 8 codes lie in two words (8 bits) or in one: one 8-byte load either way.  For a single
    // word the load is the aligned pair that contains it (or, for the last word of a buffer with
    // an odd number of words, the word before it and it).
    const uint32_t wi = ad.off + ((in_group * ad.b) >> 5);
    const bool two = ad.b == 8u;
    const uint32_t ps = two ? wi : (((wi | 1u) < total_words) ? (wi & ~1u) : wi - 1u);
    uint2 pair;
    __builtin_memcpy(&pair, words + ps, 8);
    const uint32_t one = (wi != ps) ? pair.y : pair.x;
    f.w0 = two ? pair.x : one;
    f.w1 = two ? pair.y : one;
    f.b = ad.b;
    const int64_t g = g_step0 + (int64_t)step * (kBM * (int64_t)gpr) + g_off;
    f.mn = mn[g];
    f.sc = scale[g];
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const uint32_t wn = wave;
  const uint32_t li = lane & 31u, lg = lane >> 5;
  // Operand reads: lane l of 16-lane group G = l / 16 addresses row 8*(l/32) + (l%16)/4 (plus 16 per
  // sub-step, plus 4 for the second half of the operand) and the 4 columns 16*(G%2) + 4*(l%4) ..
  // of its 32-column block; it receives column 16*(G%2) + l%16 = l%32 of the block.
  const uint32_t tr_row = 8u * lg + ((lane & 15u) >> 2), tr_col = 16u * ((lane >> 4) & 1u) + 4u * (lane & 3u);
  const uint32_t a_read = tr_row * (uint32_t)kRowA + (64u * wn + tr_col) * 2u;
  const uint32_t b_read = (uint32_t)(kBM * kRowA) + tr_row * (uint32_t)kRowB + tr_col * 2u;

  // Half of the work of turning a stage into LDS tiles: two of the thread's four grad_y rows
  // (copied as loaded) and one of its two rows of x.
  const uint32_t a_store = (4u * rq) * (uint32_t)kRowA + 16u * cg;
  const uint32_t b_store = (uint32_t)(kBM * kRowA) + xr * (uint32_t)kRowB + 16u * co;
  auto build_half = [&](const Stage& cur, char* buf, int hs) __attribute__((always_inline)) {
#pragma unroll
    for (int rr = 0; rr < 2; ++rr) {
      const int r = 2 * hs + rr;
      *reinterpret_cast<uint4*>(buf + a_store + (uint32_t)r * kRowA) = cur.gy[r];
    }
    // ---- xhat: unpack, dequantize, round to the element format; 4 columns = 8 bytes of the row ----
    // Code c sits at bit s0 + (7-c)*b, s0 placing the 8 codes inside their word; for 8-bit codes
    // (two words) the position is taken inside the word, mod 32.
    {
      const uint32_t b = cur.b;
      const uint32_t s0 = (b == 8u) ? 0u : 32u - 8u * b - ((in_group * b) & 31u);
      const uint32_t w = hs ? cur.w1 : cur.w0;
      float v[4];
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) {
        const int c = 4 * hs + cc;
        const uint32_t code = __builtin_amdgcn_ubfe(w, (s0 + (uint32_t)(7 - c) * b) & 31u, b);
        v[cc] = __builtin_fmaf((float)code, cur.sc, cur.mn);
      }
      *reinterpret_cast<uint2*>(buf + b_store + 8u * (uint32_t)hs) =
          make_uint2(narrow16_pair<DT>(v[0], v[1]), narrow16_pair<DT>(v[2], v[3]));
    }
  };

  // One step: run the products on copy BUF of the tiles while building the next step's tiles
  // (from `next`) in the other copy, then request the loads of the step after that into the
  // registers just consumed.
  auto do_step = [&](auto BUF, Stage& next, Addr& ad_use, Addr& ad_fill, int step) __attribute__((always_inline)) {
    constexpr int buf = decltype(BUF)::value;
    // The group addresses of the step after the one requested below go first: when they are
    // needed (one step from now) all of this step's other loads are younger and may stay in flight.
    fetch_addr(ad_fill, min(step + 4, steps - 1));
    const char* a_lds = lds[buf] + a_read;
    const char* b_lds = lds[buf] + b_read;
#pragma unroll
    for (int ss = 0; ss < kBM / 16; ++ss) {
      uint4 a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) a[i] = operand_tr(a_lds + ss * 16 * kRowA + i * 64, kRowA);
#pragma unroll
      for (int j = 0; j < 2; ++j) b[j] = operand_tr(b_lds + ss * 16 * kRowB + j * 64, kRowB);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = mfma_32x32x16<DT>(a[i], b[j], acc[i][j]);
      build_half(next, lds[buf ^ 1], ss);
    }
    // Requested unconditionally (past the end the last step is requested again and never
    // used), so that the number of loads in flight is the same in every iteration.
    fetch_stage(next, ad_use, min(step + 3, steps - 1));
    __syncthreads();                                // the other copy is complete, this one is free
  };

  // Step q lives in stage q % 2 and LDS copy q % 2, its group addresses in ad[q % 2] (requested
  // one step before its words).  Prologue: steps 0..2 requested (step 0 is consumed at once,
  // step 2 takes its registers), addresses of step 3 requested, tiles of step 0 built.
  Stage st[2];
  Addr ad[2];
  fetch_addr(ad[0], 0);
  fetch_stage(st[0], ad[0], 0);
  fetch_addr(ad[1], min(1, steps - 1));
  fetch_stage(st[1], ad[1], min(1, steps - 1));
  build_half(st[0], lds[0], 0);
  build_half(st[0], lds[0], 1);
  fetch_addr(ad[0], min(2, steps - 1));
  fetch_stage(st[0], ad[0], min(2, steps - 1));
  fetch_addr(ad[1], min(3, steps - 1));
  __syncthreads();

  // In iteration s: products on copy s % 2; tiles of step s+1 (stage (s+1) % 2) into the other
  // copy; then loads of step s+3 into that same stage, with the addresses in ad[(s+1) % 2]
  // (requested in iteration s-1); addresses of step s+4 into ad[s % 2].
  // Several steps per trip of the main loop: at a loop header the compiler waits for every load
  // in flight (it does not carry the order of the previous trip's loads across the back edge),
  // so the fewer headers, the fewer full drains of the prefetch.
  constexpr int kTrip = MIXED ? 2 : 8;              // (more would cost the mixed-width kernel a work-group per CU in registers)
  int base = 0;
  for (; base + kTrip <= steps; base += kTrip) {
#pragma unroll
    for (int u = 0; u < kTrip; u += 2) {
      do_step(Index<0>{}, st[1], ad[1], ad[0], base + u);
      do_step(Index<1>{}, st[0], ad[0], ad[1], base + u + 1);
    }
  }
  for (; base + 2 <= steps; base += 2) {
    do_step(Index<0>{}, st[1], ad[1], ad[0], base);
    do_step(Index<1>{}, st[0], ad[0], ad[1], base + 1);
  }
  if (base < steps) do_step(Index<0>{}, st[1], ad[1], ad[0], base);

  // ---- epilogue: register r of a 32 x 32 block is row 8*(r/4) + 4*(lane/32) + r%4, column lane%32 ----
  float* dst = out + (int64_t)split * N * K;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t n = n0 + 64 * wn + 32 * i + 8 * (r >> 2) + 4 * lg + (r & 3);
        const int64_t k = k0 + 32 * j + li;
        dst[n * K + k] = acc[i][j][r];
      }
}

// out[i] = sum over the slabs of part[s][i]
__global__ __launch_bounds__(256) void k_sum_slabs(const float4* __restrict__ part, int64_t n4, int32_t splits,
                                                   float4* __restrict__ out) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) {
    float4 s = part[i];
    for (int32_t p = 1; p < splits; ++p) {
      const float4 v = part[(int64_t)p * n4 + i];
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    out[i] = s;
  }
}

}  // namespace

// Number of slices of m that run as separate work-groups: 1 when the output alone has enough
// tiles to fill the chip, otherwise a power of two (at most 16) that divides M / 64.
int32_t daf_unpack_matmul_splits(int64_t M, int64_t N, int64_t K) {
  const int64_t tiles = (N / kBN) * (K / kBK);
  int32_t s = 1;
  while (s < 16 && tiles * s < 512 && (M / kBM) % (2 * s) == 0) s *= 2;
  return s;
}

bool daf_unpack_matmul_shape_ok(int64_t M, int64_t N, int64_t K, int32_t gs) {
  return M > 0 && N > 0 && K > 0 && M % kBM == 0 && N % kBN == 0 && K % kBK == 0 && K % gs == 0 &&
         (N / kBN) * (K / kBK) * 16 < (int64_t)1 << 31;
}

hipError_t daf_launch_unpack_matmul(const daf_plan_t* p, const uint32_t* words, const float* mn, const float* scale,
                                    const uint8_t* d_bits, const void* grad_y, int64_t N, int64_t K, int dtype,
                                    float* out, float* workspace, hipStream_t stream) {
  const int64_t M = p->n / K;
  const int32_t splits = daf_unpack_matmul_splits(M, N, K);
  const int32_t tiles_n = (int32_t)(N / kBN), tiles_k = (int32_t)(K / kBK);
  const unsigned blocks = (unsigned)((int64_t)tiles_n * tiles_k * splits);
  float* target = splits > 1 ? workspace : out;
  const u32x4* gy = static_cast<const u32x4*>(grad_y);
#define DAF_LAUNCH(DT, MIXED)                                                                                     \
  hipLaunchKernelGGL((k_unpack_matmul<DT, MIXED>), dim3(blocks), dim3(kThreads), 0, stream, words, mn, scale,     \
                     d_bits, p->d_off, (uint32_t)p->uniform_bits, p->group_size, gy, M, N, K, tiles_n, tiles_k,   \
                     splits, (uint32_t)p->total_words, target)
  if (dtype == daf::kBF16) {
    if (p->uniform_bits) DAF_LAUNCH(daf::kBF16, false); else DAF_LAUNCH(daf::kBF16, true);
  } else if (dtype == daf::kF16) {
    if (p->uniform_bits) DAF_LAUNCH(daf::kF16, false); else DAF_LAUNCH(daf::kF16, true);
  } else {
    return hipErrorInvalidValue;
  }
#undef DAF_LAUNCH
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || splits == 1) return e;
  const int64_t n4 = N * K / 4;
  const unsigned rblocks = (unsigned)((n4 + 255) / 256 < 4096 ? (n4 + 255) / 256 : 4096);
  hipLaunchKernelGGL(k_sum_slabs, dim3(rblocks), dim3(256), 0, stream, reinterpret_cast<const float4*>(workspace), n4,
                     splits, reinterpret_cast<float4*>(out));
  return hipGetLastError();
}
