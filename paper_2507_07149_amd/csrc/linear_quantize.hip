// Producer fusion into a matrix product: y = x W^T of a linear layer, with the quantize+pack of y
// (Sec. 2.2 Eq. 1, Sec. 3.3) as the epilogue of the output tile, so that the activation the
// next layer saves is reduced, quantized and packed inside the kernel that produces it
// (Sec. 3.2.3) and is never read back from memory for that purpose.
//
//   x [M, K], W [N, K], y [M, N], all in one 16-bit format, row-major; products accumulated in
//   binary32 on the matrix cores (v_mfma_f32_32x32x16_bf16 / _f16), y rounded to the format with
//   round-to-nearest-even.  Groups are runs of 32, 64 or 128 consecutive elements of a row of y
//   (the flat grouping of daf_plan with such a group size, N being a multiple of 256), so a
//   group lies inside one wave's 64 x 128 part of the 256 x 256 output tile.
//
// The product is computed transposed (W supplies the rows of each 32 x 32 block, x the columns):
// a lane then holds, for ONE row m of y, four runs of four consecutive n per block, and after
// two half-wave swaps 16 consecutive n: one Philox block, 32 contiguous bytes of y, a whole
// number of packed words for every width but 1 (where the two lanes of a row put their halves
// together).  Minimum and maximum of a group are then a reduction inside a lane plus one
// exchange with the lane 32 away.  The element map, the random bytes and the word layout are
// those of daf_quantize_pack, so words, min and scale equal daf_quantize_pack(y) bit for bit.
#include "quantize_common.h"

namespace {

constexpr int kLinThreads = 512;             // 8 waves: 4 along m x 2 along n
constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kPitch = kBK * 2 + 16;         // bytes per staged row: 16-byte reads of 32 consecutive rows hit distinct banks
constexpr int kOperandBytes = 256 * kPitch;
constexpr int kStageBytes = 2 * kOperandBytes;

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

template <int DT>
__device__ __forceinline__ f32x16 mfma16(const u32x4& a, const u32x4& b, f32x16 c) {
  if constexpr (DT == kBF16) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                   0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0,
                                                  0);
  }
}

// Two binary32 values rounded (nearest even) to the 16-bit format, low half first.
template <int DT>
__device__ __forceinline__ uint32_t round_pair(float lo, float hi) {
  if constexpr (DT == kBF16) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
  } else {
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    const f16x2 v = {(_Float16)lo, (_Float16)hi};
    return __builtin_bit_cast(uint32_t, v);
  }
}

// The value held by the lane 32 away.
__device__ __forceinline__ uint32_t other_half(uint32_t v) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return (threadIdx.x & 32) ? r.x : r.y;
}
__device__ __forceinline__ float both_halves_min(float v) { return vmin(v, u2f(other_half(f2u(v)))); }
__device__ __forceinline__ float both_halves_max(float v) { return vmax(v, u2f(other_half(f2u(v)))); }

// blockIdx -> tile.  Whole rounds of 256 workgroups: the s-th workgroup of die d in round r takes
// position 256 r + 32 d + s; the rest keep their index.  Position -> tile: panels of kPanel tile
// rows, column by column inside a panel (the last panel may be lower).  Both maps are bijections.
struct TileIndex {
  int m, n;
};
__host__ __device__ inline TileIndex tile_of_workgroup(int id, int tiles_m, int tiles_n) {
  constexpr int kDies = 8, kPerDie = 32, kPanel = 4;
  const int total = tiles_m * tiles_n;
  int pos = id;
  if (id < total / (kDies * kPerDie) * (kDies * kPerDie)) {
    const int die = id % kDies, seq = id / kDies;
    pos = (seq / kPerDie) * (kDies * kPerDie) + die * kPerDie + seq % kPerDie;
  }
  const int full = tiles_m / kPanel * kPanel;            // tile rows in whole panels
  TileIndex t;
  if (pos < full * tiles_n) {
    const int panel = pos / (kPanel * tiles_n), in = pos % (kPanel * tiles_n);
    t.m = panel * kPanel + in % kPanel;
    t.n = in / kPanel;
  } else {
    const int rows = tiles_m - full, in = pos - full * tiles_n;
    t.m = full + in % rows;
    t.n = in / rows;
  }
  return t;
}

// A thread's share of one step's tiles: four 16-byte pieces of W and four of x (rows 64 apart).
struct Staged {
  u32x4 w0, w1, w2, w3, x0, x1, x2, x3;
};
__device__ __forceinline__ void fetch(Staged& st, const char* gx, const char* gw, int64_t rows64, int step) {
  const int64_t k_off = (int64_t)step * (kBK * 2);
  st.w0 = *reinterpret_cast<const u32x4*>(gw + k_off);
  st.x0 = *reinterpret_cast<const u32x4*>(gx + k_off);
  st.w1 = *reinterpret_cast<const u32x4*>(gw + rows64 + k_off);
  st.x1 = *reinterpret_cast<const u32x4*>(gx + rows64 + k_off);
  st.w2 = *reinterpret_cast<const u32x4*>(gw + 2 * rows64 + k_off);
  st.x2 = *reinterpret_cast<const u32x4*>(gx + 2 * rows64 + k_off);
  st.w3 = *reinterpret_cast<const u32x4*>(gw + 3 * rows64 + k_off);
  st.x3 = *reinterpret_cast<const u32x4*>(gx + 3 * rows64 + k_off);
}
__device__ __forceinline__ void stash(const Staged& st, char* base) {
  *reinterpret_cast<u32x4*>(base) = st.w0;
  *reinterpret_cast<u32x4*>(base + 64 * kPitch) = st.w1;
  *reinterpret_cast<u32x4*>(base + 128 * kPitch) = st.w2;
  *reinterpret_cast<u32x4*>(base + 192 * kPitch) = st.w3;
  *reinterpret_cast<u32x4*>(base + kOperandBytes) = st.x0;
  *reinterpret_cast<u32x4*>(base + kOperandBytes + 64 * kPitch) = st.x1;
  *reinterpret_cast<u32x4*>(base + kOperandBytes + 128 * kPitch) = st.x2;
  *reinterpret_cast<u32x4*>(base + kOperandBytes + 192 * kPitch) = st.x3;
}

template <int DT, int GS_LOG2, bool MIXED, bool QUANT>
__global__ __launch_bounds__(kLinThreads, 2) void k_linear_quantize_pack(
    const char* __restrict__ x, const char* __restrict__ w, int M, int N, int K, uint32_t seed_lo, uint32_t seed_hi,
    uint32_t uniform_b, const uint8_t* __restrict__ bits, const uint32_t* __restrict__ off, char* __restrict__ y,
    uint32_t* __restrict__ words, float* __restrict__ out_min, float* __restrict__ out_scale) {
  __shared__ __align__(16) char lds[2 * kStageBytes];
  const int t = threadIdx.x, lane = t & (kWave - 1), wave = t >> 6;
  const int wm = wave & 3, wn = wave >> 2;
  const int li = lane & 31, lg = lane >> 5;

  // Workgroups are handed to the eight dies in turn, so the 32 workgroups that run together on one
  // die (32 compute units, one cache) are every eighth one.  They get 32 consecutive positions
  // of an order that walks panels of four tile rows column by column: a patch of about 4 x 8
  // tiles, whose workgroups, moving through k in step, share four slabs of x and eight of W in
  // that cache instead of one and thirty-two.
  const int tiles_n = N / kBN, tiles_m = M / kBM;
  const TileIndex ti = tile_of_workgroup((int)blockIdx.x, tiles_m, tiles_n);
  const int tm = ti.m, tn = ti.n;
  const int64_t m0 = (int64_t)tm * kBM, n0 = (int64_t)tn * kBN;

  // Staging: 2048 16-byte pieces per operand and step of 64 k, four per thread: rows crow + 64 j.
  const int crow = t >> 3, ccol = t & 7;
  const char* gx = x + ((m0 + crow) * K + ccol * 8) * 2;
  const char* gw = w + ((n0 + crow) * K + ccol * 8) * 2;
  const int64_t rows64 = (int64_t)64 * K * 2;
  const int stash_off = crow * kPitch + ccol * 16;
  f32x16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // Step s computes on copy s % 2 of the staged tiles while the registers that hold step s + 1 are
  // written to the other copy and the loads of step s + 2 are issued: one barrier per step.  Past
  // the end the last step is fetched and staged again (unused), which keeps the loop free of
  // branches around the loads.
  const int steps = K / kBK;
  Staged st;
  fetch(st, gx, gw, rows64, 0);
  stash(st, lds + stash_off);
  fetch(st, gx, gw, rows64, steps > 1 ? 1 : 0);
  const int a_off = (wn * 128 + li) * kPitch + lg * 16;
  const int b_off = kOperandBytes + (wm * 64 + li) * kPitch + lg * 16;
  for (int s = 0; s < steps; ++s) {
    __syncthreads();                       // copy s % 2 is complete; nobody reads the other copy any more
    stash(st, lds + ((s + 1) & 1) * kStageBytes + stash_off);
    fetch(st, gx, gw, rows64, s + 2 < steps ? s + 2 : steps - 1);
    const char* base = lds + (s & 1) * kStageBytes;
#pragma unroll
    for (int ks = 0; ks < kBK / 16; ++ks) {
      u32x4 a[4], b[2];
#pragma unroll
      for (int nb = 0; nb < 4; ++nb) a[nb] = *reinterpret_cast<const u32x4*>(base + a_off + nb * 32 * kPitch + ks * 32);
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) b[mb] = *reinterpret_cast<const u32x4*>(base + b_off + mb * 32 * kPitch + ks * 32);
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) acc[mb][nb] = mfma16<DT>(a[nb], b[mb], acc[mb][nb]);
    }
  }

  // ---- epilogue.  Register r of a 32 x 32 block: n = 8*(r/4) + 4*(lane/32) + r%4, m = lane%32. ----
  constexpr int kGs = 1 << GS_LOG2, kBlocksPerGroup = kGs / 32, kGroups = 4 / kBlocksPerGroup;
#pragma unroll
  for (int mb = 0; mb < 2; ++mb) {
    const int64_t m = m0 + wm * 64 + mb * 32 + li;
    const int64_t n_lane = n0 + wn * 128 + lg * 16;             // + 32 nb: this lane's 16 consecutive n of block nb
    float xf[4][16];
    float bmn[4], bmx[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      uint32_t d[4][2];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        d[j][0] = round_pair<DT>(acc[mb][nb][4 * j], acc[mb][nb][4 * j + 1]);
        d[j][1] = round_pair<DT>(acc[mb][nb][4 * j + 2], acc[mb][nb][4 * j + 3]);
      }
      // Lower half-wave: runs j = 0..3 are n 0-3, 8-11, 16-19, 24-27; upper: 4-7, 12-15, 20-23, 28-31.
      // Swapping the upper half of run 0 with the lower half of run 2 (and 1 with 3) leaves n 0-15
      // in the lower half-wave and n 16-31 in the upper one.
      uint32_t yv[8];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const u32x2 r02 = __builtin_amdgcn_permlane32_swap(d[0][h], d[2][h], false, false);
        const u32x2 r13 = __builtin_amdgcn_permlane32_swap(d[1][h], d[3][h], false, false);
        yv[h] = r02.x;
        yv[2 + h] = r02.y;
        yv[4 + h] = r13.x;
        yv[6 + h] = r13.y;
      }
      char* dst = y + (m * N + n_lane + nb * 32) * 2;
      *reinterpret_cast<u32x4*>(dst) = u32x4{yv[0], yv[1], yv[2], yv[3]};
      *reinterpret_cast<u32x4*>(dst + 16) = u32x4{yv[4], yv[5], yv[6], yv[7]};
      float mn = 0.0f, mx = 0.0f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const uint32_t pair = yv[e >> 1];
        const float v = widen16<DT>((e & 1) ? (pair >> 16) : (pair & 0xFFFFu));
        xf[nb][e] = v;
        mn = e == 0 ? v : vmin(mn, v);
        mx = e == 0 ? v : vmax(mx, v);
      }
      bmn[nb] = mn;
      bmx[nb] = mx;
    }
    if (!QUANT) continue;                                        // the product alone
#pragma unroll
    for (int gi = 0; gi < kGroups; ++gi) {
      float mn = bmn[gi * kBlocksPerGroup], mx = bmx[gi * kBlocksPerGroup];
#pragma unroll
      for (int q = 1; q < kBlocksPerGroup; ++q) {
        mn = vmin(mn, bmn[gi * kBlocksPerGroup + q]);
        mx = vmax(mx, bmx[gi * kBlocksPerGroup + q]);
      }
      mn = both_halves_min(mn);
      mx = both_halves_max(mx);
      const int64_t g = (m * N + n0 + wn * 128 + gi * kGs) >> GS_LOG2;
      const uint32_t b = MIXED ? (uint32_t)bits[g] : uniform_b;
      const uint32_t woff = MIXED ? off[g] : (uint32_t)(g * (int64_t)((kGs * uniform_b) >> 5));
      const GroupScale gs = group_scale(mn, mx, b);
      if (lg == 0) {
        out_min[g] = gs.mn;
        out_scale[g] = gs.scale;
      }
      const float invs = gs.inv * kScale;
      const bool exact2 = !(invs <= 3.402823466e+38f);          // the factor 256 is then applied to the rounded product
      const float mult = exact2 ? gs.inv : invs;
#pragma unroll
      for (int q = 0; q < kBlocksPerGroup; ++q) {
        const int nb = gi * kBlocksPerGroup + q;
        const uint32_t e0 = (uint32_t)(q * 32 + lg * 16);       // first of the lane's 16 elements, counted inside the group
        const uint4 rnd4 = philox_block((uint64_t)((m * N + n_lane + nb * 32) >> 4), seed_lo, seed_hi);
        const uint32_t rnd[4] = {rnd4.x, rnd4.y, rnd4.z, rnd4.w};
        uint32_t p[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          uint32_t nacc = 0u;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float wv = (gs.mn - xf[nb][4 * c + e]) * mult;
            const float wv2 = wv * kScale;
            wv = exact2 ? wv2 : wv;
            const int nc = (round_half_up_to_int(wv) + (int)((rnd[c] >> (8 * e)) & 0xFFu)) >> 8;
            nacc = (nacc << b) + (uint32_t)nc;
          }
          p[c] = 0u - nacc;                                      // four codes, first element most significant
        }
        uint32_t* dst = words + woff;
        if (b == 8u) {
#pragma unroll
          for (int c = 0; c < 4; ++c) dst[(e0 >> 2) + c] = p[c];
        } else if (b == 4u) {
          dst[(e0 >> 3)] = (p[0] << 16) | (p[1] & 0xFFFFu);
          dst[(e0 >> 3) + 1] = (p[2] << 16) | (p[3] & 0xFFFFu);
        } else if (b == 2u) {
          dst[e0 >> 4] = (p[0] << 24) | ((p[1] & 0xFFu) << 16) | ((p[2] & 0xFFu) << 8) | (p[3] & 0xFFu);
        } else {
          const uint32_t half = ((p[0] & 0xFu) << 12) | ((p[1] & 0xFu) << 8) | ((p[2] & 0xFu) << 4) | (p[3] & 0xFu);
          const uint32_t upper = other_half(half);               // the lane 32 away runs the same branch: same group, same width
          if (lg == 0) dst[e0 >> 5] = (half << 16) | upper;
        }
      }
    }
  }
}

template <int DT, int GS_LOG2>
hipError_t launch_gs(const daf_plan_t* p, const void* x, const void* w, int M, int N, int K, uint64_t seed, void* y,
                     uint32_t* words, float* mn, float* sc, hipStream_t stream) {
  const unsigned grid = (unsigned)((M / kBM) * (N / kBN));
  const uint32_t lo = (uint32_t)seed, hi = (uint32_t)(seed >> 32);
  if (words == nullptr)
    hipLaunchKernelGGL((k_linear_quantize_pack<DT, GS_LOG2, false, false>), dim3(grid), dim3(kLinThreads), 0, stream,
                       (const char*)x, (const char*)w, M, N, K, lo, hi, 8u, nullptr, nullptr, (char*)y, words, mn, sc);
  else if (p->uniform_bits)
    hipLaunchKernelGGL((k_linear_quantize_pack<DT, GS_LOG2, false, true>), dim3(grid), dim3(kLinThreads), 0, stream,
                       (const char*)x, (const char*)w, M, N, K, lo, hi, (uint32_t)p->uniform_bits, nullptr, nullptr,
                       (char*)y, words, mn, sc);
  else
    hipLaunchKernelGGL((k_linear_quantize_pack<DT, GS_LOG2, true, true>), dim3(grid), dim3(kLinThreads), 0, stream,
                       (const char*)x, (const char*)w, M, N, K, lo, hi, 0u, p->d_bits, p->d_off, (char*)y, words, mn, sc);
  return hipGetLastError();
}

template <int DT>
hipError_t launch_dt(const daf_plan_t* p, const void* x, const void* w, int M, int N, int K, uint64_t seed, void* y,
                     uint32_t* words, float* mn, float* sc, hipStream_t stream) {
  switch (p->group_size) {
    case 32: return launch_gs<DT, 5>(p, x, w, M, N, K, seed, y, words, mn, sc, stream);
    case 64: return launch_gs<DT, 6>(p, x, w, M, N, K, seed, y, words, mn, sc, stream);
    default: return launch_gs<DT, 7>(p, x, w, M, N, K, seed, y, words, mn, sc, stream);
  }
}

}  // namespace

void daf_linear_tile_map(int id, int tiles_m, int tiles_n, int* tm, int* tn) {
  const TileIndex t = tile_of_workgroup(id, tiles_m, tiles_n);
  *tm = t.m;
  *tn = t.n;
}

bool daf_linear_quantize_supported(const daf_plan_t* p, int64_t N, int64_t K, int dtype) {
  if (dtype != DAF_F16 && dtype != DAF_BF16) return false;
  if (p->group_size != 32 && p->group_size != 64 && p->group_size != 128) return false;
  if (N < kBN || N % kBN != 0 || K < kBK || K % kBK != 0 || p->n % N != 0) return false;
  const int64_t M = p->n / N;
  if (M % kBM != 0) return false;
  return M <= (1 << 24) && N <= (1 << 24) && K <= (1 << 24) && (M / kBM) * (N / kBN) < (int64_t)1 << 31;
}

hipError_t daf_launch_linear_quantize_pack(const daf_plan_t* p, const void* x, const void* w, int64_t N, int64_t K,
                                           int dtype, uint64_t seed, void* y, uint32_t* words, float* mn, float* sc,
                                           hipStream_t stream) {
  const int M = (int)(p->n / N);
  if (dtype == DAF_BF16) return launch_dt<kBF16>(p, x, w, M, (int)N, (int)K, seed, y, words, mn, sc, stream);
  return launch_dt<kF16>(p, x, w, M, (int)N, (int)K, seed, y, words, mn, sc, stream);
}
