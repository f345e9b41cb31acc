// Device-side helpers of libdaf: wave-level data movement, Philox4x32-10, exact widening
// and round-to-nearest-even narrowing of the 16-bit float formats.  gfx950 only (wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace daf {

constexpr int kWave = 64;
constexpr int kRandBits = 8;          // random bits per element
constexpr int kElemsPerPhilox = 16;   // 128 / kRandBits

enum : int { kF32 = 0, kF16 = 1, kBF16 = 2 };

template <int DT> struct ElemTraits;
template <> struct ElemTraits<kF32>  { static constexpr int kBytes = 4; static constexpr int kPerLoad = 4; };
template <> struct ElemTraits<kF16>  { static constexpr int kBytes = 2; static constexpr int kPerLoad = 8; };
template <> struct ElemTraits<kBF16> { static constexpr int kBytes = 2; static constexpr int kPerLoad = 8; };

__device__ __forceinline__ float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t f2u(float f) { return __builtin_bit_cast(uint32_t, f); }

// Orders this wave's LDS traffic: everything written before is visible to every lane after.
// A wave executes its LDS instructions in order, so no hardware barrier is needed; this only
// stops the compiler from moving memory operations across the point.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// DPP lane exchange.  Lanes whose row is not in ROW_MASK keep `old`.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ uint32_t dpp(uint32_t old, uint32_t src) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)old, (int)src, CTRL, ROW_MASK, 0xF, false);
}
constexpr int kDppXor1 = 0xB1;          // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;          // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;   // lane i <-> 7-i inside groups of 8
constexpr int kDppMirror = 0x140;       // lane i <-> 15-i inside rows of 16
constexpr int kDppBcast15 = 0x142;      // lane 15 of each row -> every lane of the next row
constexpr int kDppBcast31 = 0x143;      // lane 31 -> every lane of rows 2 and 3
constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;

// Plain min/max instructions.  (fminf/fmaxf would first canonicalise every operand with an
// extra instruction each, to quiet signalling NaNs; inputs here are finite by contract.)
__device__ __forceinline__ float vmin(float a, float b) {
  float r;
  asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float vmax(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float vmin3(float a, float b, float c) {
  float r;
  asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ __forceinline__ float vmax3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// min (a, c) and max (b, d) of two independent value pairs over aligned runs of
// LPG = 2^LPG_LOG2 lanes, one DPP instruction per step and value.  The complete result is
// guaranteed in the LAST lane of each run (for LPG <= 16 every lane of the run has it).
// Four independent chains are interleaved, so an instruction reads a register written four
// instructions earlier, which satisfies the two wait states a DPP read needs after a VALU
// write; the leading s_nop covers whatever the compiler issued just before the block (VALU
// write of an operand, or of EXEC), the trailing one whatever it issues right after.
#define DAF_DPP_X1 "quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf"
#define DAF_DPP_X2 "quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf"
#define DAF_DPP_HM "row_half_mirror row_mask:0xf bank_mask:0xf"
#define DAF_DPP_M "row_mirror row_mask:0xf bank_mask:0xf"
#define DAF_DPP_B15 "row_bcast:15 row_mask:0xa bank_mask:0xf"
#define DAF_DPP_B31 "row_bcast:31 row_mask:0xc bank_mask:0xf"
#define DAF_MM4(CTRL)                          \
  "v_min_f32_dpp %0, %0, %0 " CTRL "\n"        \
  "v_max_f32_dpp %1, %1, %1 " CTRL "\n"        \
  "v_min_f32_dpp %2, %2, %2 " CTRL "\n"        \
  "v_max_f32_dpp %3, %3, %3 " CTRL "\n"
#define DAF_MM4_ASM(BODY) \
  asm("s_nop 4\n" BODY "s_nop 1\n" : "+v"(a), "+v"(b), "+v"(c), "+v"(d))
template <int LPG_LOG2>
__device__ __forceinline__ void seg_minmax_x2(float& a, float& b, float& c, float& d) {
  static_assert(LPG_LOG2 >= 2 && LPG_LOG2 <= 6, "run length 4..64 lanes");
  if constexpr (LPG_LOG2 == 2) {
    DAF_MM4_ASM(DAF_MM4(DAF_DPP_X1) DAF_MM4(DAF_DPP_X2));
  } else if constexpr (LPG_LOG2 == 3) {
    DAF_MM4_ASM(DAF_MM4(DAF_DPP_X1) DAF_MM4(DAF_DPP_X2) DAF_MM4(DAF_DPP_HM));
  } else if constexpr (LPG_LOG2 == 4) {
    DAF_MM4_ASM(DAF_MM4(DAF_DPP_X1) DAF_MM4(DAF_DPP_X2) DAF_MM4(DAF_DPP_HM) DAF_MM4(DAF_DPP_M));
  } else if constexpr (LPG_LOG2 == 5) {
    DAF_MM4_ASM(DAF_MM4(DAF_DPP_X1) DAF_MM4(DAF_DPP_X2) DAF_MM4(DAF_DPP_HM) DAF_MM4(DAF_DPP_M)
                DAF_MM4(DAF_DPP_B15));
  } else {
    DAF_MM4_ASM(DAF_MM4(DAF_DPP_X1) DAF_MM4(DAF_DPP_X2) DAF_MM4(DAF_DPP_HM) DAF_MM4(DAF_DPP_M)
                DAF_MM4(DAF_DPP_B15) DAF_MM4(DAF_DPP_B31));
  }
}
#undef DAF_MM4_ASM
#undef DAF_MM4

// Inclusive prefix sum over the 64 lanes of a wave.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v) {
#define DAF_SCAN(CTRL, MASK) v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, MASK, 0xF, false)
  DAF_SCAN(kDppRowShr1, 0xF);
  DAF_SCAN(kDppRowShr2, 0xF);
  DAF_SCAN(kDppRowShr4, 0xF);
  DAF_SCAN(kDppRowShr8, 0xF);
  DAF_SCAN(kDppBcast15, 0xA);
  DAF_SCAN(kDppBcast31, 0xC);
#undef DAF_SCAN
  return v;
}

// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies and two
// three-way xors; the key advances by the Weyl constants between rounds.
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
  uint32_t r;
  asm("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x96" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

__device__ __forceinline__ uint4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
    const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return make_uint4(c0, c1, c2, c3);
}

// The 16 random bytes of Philox block `blk` under `seed`: byte s serves element 16*blk + s.
__device__ __forceinline__ uint4 philox_block(uint64_t blk, uint32_t seed_lo, uint32_t seed_hi) {
  return philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), 0u, 0u, seed_lo, seed_hi);
}

// floor(x) as a signed integer in one instruction.
__device__ __forceinline__ int floor_to_int(float x) {
  int r;
  asm("v_cvt_flr_i32_f32 %0, %1" : "=v"(r) : "v"(x));
  return r;
}

// ---- 16-bit formats -----------------------------------------------------------------
template <int DT> __device__ __forceinline__ float widen16(uint32_t h16);
template <> __device__ __forceinline__ float widen16<kF16>(uint32_t h16) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)h16);
}
template <> __device__ __forceinline__ float widen16<kBF16>(uint32_t h16) { return u2f(h16 << 16); }

template <int DT> __device__ __forceinline__ uint32_t narrow16(float f);   // finite inputs, RNE
template <> __device__ __forceinline__ uint32_t narrow16<kF16>(float f) {
  // The binary32 value must exist before it is rounded to binary16: without this barrier the
  // compiler merges the producing fma and the conversion into one mixed-precision
  // instruction that rounds the exact result once, which differs in the last bit now and then.
  asm("" : "+v"(f));
  return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
}
template <> __device__ __forceinline__ uint32_t narrow16<kBF16>(float f) {
  const uint32_t u = f2u(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Element e (0-based) of a 16-byte chunk held in four dwords.
template <int DT>
__device__ __forceinline__ float chunk_elem(const uint4& raw, int e) {
  const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
  if (DT == kF32) return u2f(w[e]);
  const uint32_t d = w[e >> 1];
  if (DT == kBF16) return (e & 1) ? u2f(d & 0xFFFF0000u) : u2f(d << 16);
  return widen16<DT == kF32 ? kF16 : DT>((e & 1) ? (d >> 16) : (d & 0xFFFFu));
}

}  // namespace daf
