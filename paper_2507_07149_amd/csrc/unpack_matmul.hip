// Consumer fusion for a contraction: the weight gradient of y = x W^T,
//     dW[n, k] = sum_m grad_y[m, n] * xhat[m, k],
// computed straight from the packed activation.  Unpacking and dequantization (Algorithm 2,
// inverse of Eq. 1) are the prologue of every tile of the product: xhat goes from registers
// into LDS and from there into the matrix cores, and is never written to HBM (unpacking next
// to the consumer, Sec. 3.3 and Sec. 4.3.1).  This is the one dense contraction on the path,
// so it runs on MFMA (v_mfma_f32_32x32x16 for bf16 / f16, binary32 accumulation).
//
// Both operands have the reduction index m as their slow dimension in memory, while an MFMA
// lane needs 8 consecutive m for one row (of grad_y^T) or one column (of xhat).  The tiles are
// therefore transposed on their way into LDS: a thread holds 4 rows x 8 columns, pairs rows in
// registers, and writes, per column, 8 bytes = 4 consecutive m.  LDS holds 16-byte units
// (column, 8 consecutive m); unit (c, o) lives at index c*8 + (o ^ s(c)) with
// s(c) = (c & 7) ^ ((c >> 3) & 7), which makes both the transposing writes and the operand
// reads conflict-free.
//
// Work-group tile: 256 (n) x 128 (k) outputs, 64 values of m per step, 4 waves in a 2 x 2
// arrangement of 128 x 64 each (4 x 2 MFMA blocks of 32 x 32, 128 accumulator registers).
#include "daf_device.h"
#include "daf_internal.h"

namespace {

using namespace daf;

constexpr int kBN = 256, kBK = 128, kBM = 64, kThreads = 256;
constexpr int kOct = kBM / 8;                       // 16-byte units per column
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

__device__ __forceinline__ uint32_t lds_unit(uint32_t col, uint32_t oct) {
  return col * (uint32_t)kOct + (oct ^ ((col & 7u) ^ ((col >> 3) & 7u)));
}

// What one thread fetches for one step: 4 rows x 8 columns of each of the two 128-column halves
// of the grad_y tile, and the packed words and group constants of 4 rows x 8 columns of xhat.
struct Fetch {
  uint4 gy[2][4];
  uint32_t w0[4], w1[4], shift[4], b[4];
  float mn[4], sc[4];
};

template <int DT, bool MIXED>
__device__ __forceinline__ void fetch_step(Fetch& f, const u32x4* __restrict__ grad_y, int64_t N8, int64_t m_base,
                                           int64_t n0_8, uint32_t co, const uint32_t* __restrict__ words,
                                           const float* __restrict__ mn, const float* __restrict__ scale,
                                           const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off,
                                           uint32_t uniform_bits, int64_t groups_per_row, int32_t gs,
                                           uint32_t words_per_group_bit, int64_t k_col) {
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int64_t m = m_base + r;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const u32x4 v = grad_y[m * N8 + n0_8 + 16 * h + co];
      f.gy[h][r] = make_uint4(v.x, v.y, v.z, v.w);
    }
    // the 8 codes of row m, columns k_col .. k_col+7: one group, one or two words
    const int64_t gk = k_col / gs;
    const int64_t g = m * groups_per_row + gk;
    const uint32_t in_group = (uint32_t)(k_col - gk * gs);
    uint32_t b, woff;
    if (MIXED) {
      b = bits[g];
      woff = off[g];
    } else {
      b = uniform_bits;
      woff = (uint32_t)g * (words_per_group_bit * b);
    }
    const uint32_t bit = in_group * b;
    const uint32_t* wp = words + woff + (bit >> 5);
    f.w0[r] = wp[0];
    f.w1[r] = (b == 8u) ? wp[1] : 0u;
    f.shift[r] = 32u - 8u * b - (bit & 31u);        // used for b < 8 only
    f.b[r] = b;
    f.mn[r] = mn[g];
    f.sc[r] = scale[g];
  }
}

// 16-bit pattern of xhat for code c (exactly what the plain dequantize kernel stores).
template <int DT>
__device__ __forceinline__ uint32_t xhat16(uint32_t code, float sc, float mn) {
  return narrow16<DT>(__builtin_fmaf((float)code, sc, mn));
}

template <int DT, bool MIXED>
__global__ __launch_bounds__(kThreads, 2) void k_unpack_matmul(
    const uint32_t* __restrict__ words, const float* __restrict__ mn, const float* __restrict__ scale,
    const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, uint32_t uniform_bits, int32_t gs,
    const u32x4* __restrict__ grad_y, int64_t M, int64_t N, int64_t K, int32_t tiles_n, int32_t tiles_k,
    int32_t splits, float* __restrict__ out) {
  __shared__ uint4 a_lds[kBN * kOct];               // grad_y^T: (n, 8 consecutive m)
  __shared__ uint4 b_lds[kBK * kOct];               // xhat^T:   (k, 8 consecutive m)

  const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
  // Consecutive block ids go to different XCDs (each with its own L2).  Give every XCD a
  // contiguous range of tiles, n fastest, so that the tiles resident on one XCD share their
  // xhat panel and a few grad_y panels.
  const uint32_t n_tiles = (uint32_t)tiles_n * (uint32_t)tiles_k;
  const uint32_t per_split = n_tiles;
  const uint32_t bid = blockIdx.x;
  const uint32_t split = bid / per_split;
  uint32_t tile = bid - split * per_split;
  {
    const uint32_t xcd = tile & 7u, idx = tile >> 3;
    const uint32_t base = n_tiles / 8u, rem = n_tiles & 7u;       // XCD x owns base (+1 if x < rem) tiles
    tile = xcd * base + (xcd < rem ? xcd : rem) + idx;
  }
  const uint32_t tn = tile % (uint32_t)tiles_n, tk = tile / (uint32_t)tiles_n;
  const int64_t n0 = (int64_t)tn * kBN, k0 = (int64_t)tk * kBK;
  const int64_t m_per_split = M / splits;
  const int64_t m_begin = (int64_t)split * m_per_split;
  const int steps = (int)(m_per_split / kBM);

  const uint32_t co = t & 15u, rq = t >> 4;         // column octet and row quad of the loader role
  const uint32_t oct = rq >> 1, half = rq & 1u;
  const int64_t N8 = N / 8;
  const int64_t groups_per_row = K / gs;
  const uint32_t wpgb = (uint32_t)gs >> 5;
  const int64_t k_col = k0 + 8 * (int64_t)co;

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  Fetch f;
  fetch_step<DT, MIXED>(f, grad_y, N8, m_begin + 4 * (int64_t)rq, n0 / 8, co, words, mn, scale, bits, off,
                        uniform_bits, groups_per_row, gs, wpgb, k_col);

  const uint32_t wn = wave >> 1, wk = wave & 1u;
  const uint32_t li = lane & 31u, lg = lane >> 5;

  for (int step = 0; step < steps; ++step) {
    __syncthreads();                                // the previous step's operand reads are done

    // ---- grad_y: pair rows, one 8-byte store per column ----
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t r0[4] = {f.gy[h][0].x, f.gy[h][0].y, f.gy[h][0].z, f.gy[h][0].w};
      const uint32_t r1[4] = {f.gy[h][1].x, f.gy[h][1].y, f.gy[h][1].z, f.gy[h][1].w};
      const uint32_t r2[4] = {f.gy[h][2].x, f.gy[h][2].y, f.gy[h][2].z, f.gy[h][2].w};
      const uint32_t r3[4] = {f.gy[h][3].x, f.gy[h][3].y, f.gy[h][3].z, f.gy[h][3].w};
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const int j = c >> 1;
        uint2 v;
        if (c & 1) {
          v.x = (r0[j] >> 16) | (r1[j] & 0xFFFF0000u);
          v.y = (r2[j] >> 16) | (r3[j] & 0xFFFF0000u);
        } else {
          v.x = (r0[j] & 0xFFFFu) | (r1[j] << 16);
          v.y = (r2[j] & 0xFFFFu) | (r3[j] << 16);
        }
        const uint32_t col = 128u * (uint32_t)h + 8u * co + (uint32_t)c;
        reinterpret_cast<uint2*>(a_lds)[lds_unit(col, oct) * 2u + half] = v;
      }
    }
    // ---- xhat: unpack, dequantize, round to the element format, same transposed store ----
    {
      uint32_t xh[4][8];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const uint32_t b = f.b[r];
        if (b == 8u) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            xh[r][e] = xhat16<DT>((f.w0[r] >> (24 - 8 * e)) & 0xFFu, f.sc[r], f.mn[r]);
            xh[r][4 + e] = xhat16<DT>((f.w1[r] >> (24 - 8 * e)) & 0xFFu, f.sc[r], f.mn[r]);
          }
        } else {
          const uint32_t field = f.w0[r] >> f.shift[r];
          const uint32_t levels = (1u << b) - 1u;
#pragma unroll
          for (int e = 0; e < 8; ++e)
            xh[r][e] = xhat16<DT>((field >> ((uint32_t)(7 - e) * b)) & levels, f.sc[r], f.mn[r]);
        }
      }
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        uint2 v;
        v.x = xh[0][c] | (xh[1][c] << 16);
        v.y = xh[2][c] | (xh[3][c] << 16);
        const uint32_t col = 8u * co + (uint32_t)c;
        reinterpret_cast<uint2*>(b_lds)[lds_unit(col, oct) * 2u + half] = v;
      }
    }
    __syncthreads();

    if (step + 1 < steps)                           // next step's loads fly during the products
      fetch_step<DT, MIXED>(f, grad_y, N8, m_begin + (int64_t)(step + 1) * kBM + 4 * (int64_t)rq, n0 / 8, co, words,
                            mn, scale, bits, off, uniform_bits, groups_per_row, gs, wpgb, k_col);

#pragma unroll
    for (int ss = 0; ss < kBM / 16; ++ss) {
      const uint32_t o = 2u * (uint32_t)ss + lg;
      uint4 a[4], b[2];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = a_lds[lds_unit(128u * wn + 32u * (uint32_t)i + li, o)];
#pragma unroll
      for (int j = 0; j < 2; ++j) b[j] = b_lds[lds_unit(64u * wk + 32u * (uint32_t)j + li, o)];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = mfma_32x32x16<DT>(a[i], b[j], acc[i][j]);
    }
  }

  // ---- epilogue: register r of a 32 x 32 block is row 8*(r/4) + 4*(lane/32) + r%4, column lane%32 ----
  float* dst = out + (int64_t)split * N * K;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t n = n0 + 128 * wn + 32 * i + 8 * (r >> 2) + 4 * lg + (r & 3);
        const int64_t k = k0 + 64 * wk + 32 * j + li;
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
                     splits, target)
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
