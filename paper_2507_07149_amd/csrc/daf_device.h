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

// ---- transposed reduction --------------------------------------------------------------
// Reducing 16 registers (one per load) over the lanes of a wave one register at a time costs
// one DPP instruction per register and level.  Reducing them together is cheaper: at a level
// that pairs lane L with lane L^k, two registers A and B are merged into one whose lanes with
// bit k clear hold A reduced over {L, L^k} and whose lanes with bit k set hold B reduced the
// same way, so every level halves the number of live registers.
//
// Levels 4 and 8 (inside a row of 16 lanes): two DPP instructions with complementary bank
// masks write the two lane sets of the merged register.
#define DAF_BANK_PAIR(OP, O, A, B, CTRL_LO, MASK_LO, CTRL_HI, MASK_HI)                          \
  OP " " O ", " A ", " A " " CTRL_LO " row_mask:0xf bank_mask:" MASK_LO "\n"                   \
  OP " " O ", " B ", " B " " CTRL_HI " row_mask:0xf bank_mask:" MASK_HI "\n"
// lanes with bit 2 clear (banks 0, 2) take A from lane+4; lanes with bit 2 set take B from lane-4
#define DAF_X4(OP, O, A, B) DAF_BANK_PAIR(OP, O, A, B, "row_shl:4", "0x5", "row_shr:4", "0xa")
// lanes 0..7 of a row (banks 0, 1) take A from lane+8; lanes 8..15 take B from lane-8
#define DAF_X8(OP, O, A, B) DAF_BANK_PAIR(OP, O, A, B, "row_ror:8", "0x3", "row_ror:8", "0xc")

// in[16] -> out[8] at level 4, or in[8] -> out[4] at level 8 (OP = v_min_f32_dpp / v_max_f32_dpp).
// Instructions of one block are independent of each other (distinct outputs, inputs are
// read-only), so only the block's first DPP read needs the wait states after a VALU write.
#define DAF_DEFINE_BANK_LEVEL(NAME, OP, X)                                                       \
  __device__ __forceinline__ void NAME##_16(const float (&i)[16], float (&o)[8]) {               \
    asm("s_nop 4\n" X(OP, "%0", "%8", "%9") X(OP, "%1", "%10", "%11") X(OP, "%2", "%12", "%13")  \
        X(OP, "%3", "%14", "%15") X(OP, "%4", "%16", "%17") X(OP, "%5", "%18", "%19")            \
        X(OP, "%6", "%20", "%21") X(OP, "%7", "%22", "%23") "s_nop 1\n"                          \
        : "=&v"(o[0]), "=&v"(o[1]), "=&v"(o[2]), "=&v"(o[3]), "=&v"(o[4]), "=&v"(o[5]),          \
          "=&v"(o[6]), "=&v"(o[7])                                                               \
        : "v"(i[0]), "v"(i[1]), "v"(i[2]), "v"(i[3]), "v"(i[4]), "v"(i[5]), "v"(i[6]),           \
          "v"(i[7]), "v"(i[8]), "v"(i[9]), "v"(i[10]), "v"(i[11]), "v"(i[12]), "v"(i[13]),       \
          "v"(i[14]), "v"(i[15]));                                                               \
  }                                                                                              \
  __device__ __forceinline__ void NAME##_8(const float (&i)[8], float (&o)[4]) {                 \
    asm("s_nop 4\n" X(OP, "%0", "%4", "%5") X(OP, "%1", "%6", "%7") X(OP, "%2", "%8", "%9")      \
        X(OP, "%3", "%10", "%11") "s_nop 1\n"                                                    \
        : "=&v"(o[0]), "=&v"(o[1]), "=&v"(o[2]), "=&v"(o[3])                                     \
        : "v"(i[0]), "v"(i[1]), "v"(i[2]), "v"(i[3]), "v"(i[4]), "v"(i[5]), "v"(i[6]),           \
          "v"(i[7]));                                                                            \
  }
DAF_DEFINE_BANK_LEVEL(min_x4, "v_min_f32_dpp", DAF_X4)
DAF_DEFINE_BANK_LEVEL(max_x4, "v_max_f32_dpp", DAF_X4)
DAF_DEFINE_BANK_LEVEL(min_x8, "v_min_f32_dpp", DAF_X8)
DAF_DEFINE_BANK_LEVEL(max_x8, "v_max_f32_dpp", DAF_X8)
#undef DAF_DEFINE_BANK_LEVEL
#undef DAF_X8
#undef DAF_X4
#undef DAF_BANK_PAIR

// Levels 16 and 32 (across rows): the row-swap instructions exchange the odd rows of A with
// the even rows of B (16), or the upper half of A with the lower half of B (32); one min/max
// of the two results then holds A reduced in the lanes with the level's bit clear and B
// reduced in the others.
template <int LEVEL, bool IS_MIN>
__device__ __forceinline__ float merge_rows(float a, float b) {
  typedef unsigned u2 __attribute__((ext_vector_type(2)));
  const u2 r = (LEVEL == 16) ? __builtin_amdgcn_permlane16_swap(f2u(a), f2u(b), false, false)
                             : __builtin_amdgcn_permlane32_swap(f2u(a), f2u(b), false, false);
  return IS_MIN ? vmin(u2f(r.x), u2f(r.y)) : vmax(u2f(r.x), u2f(r.y));
}

// Levels 1 and 2 (inside a quad), one register: afterwards all four lanes of a quad agree.
__device__ __forceinline__ void quad_minmax(float& mn, float& mx) {
  asm("s_nop 4\n"
      "v_min_f32_dpp %0, %0, %0 " DAF_DPP_X1 "\n"
      "v_max_f32_dpp %1, %1, %1 " DAF_DPP_X1 "\n"
      "s_nop 0\n"
      "v_min_f32_dpp %0, %0, %0 " DAF_DPP_X2 "\n"
      "v_max_f32_dpp %1, %1, %1 " DAF_DPP_X2 "\n"
      "s_nop 1\n"
      : "+v"(mn), "+v"(mx));
}

// min/max of 16 per-load values over runs of 32 (LPG_LOG2 = 5) or 64 (6) lanes.
//   LPG_LOG2 = 6: afterwards lane L holds in mn[0]/mx[0] the result of load (L >> 2) & 15.
//   LPG_LOG2 = 5: afterwards lane L holds in mn[r]/mx[r], r = 0, 1, the result of load
//                 8r + ((L >> 2) & 7) for the run L >> 5.
template <int LPG_LOG2>
__device__ __forceinline__ void transposed_minmax16(const float (&mn_in)[16], const float (&mx_in)[16],
                                                    float (&mn)[2], float (&mx)[2]) {
  static_assert(LPG_LOG2 == 5 || LPG_LOG2 == 6, "runs of 32 or 64 lanes");
  float a8[8], b8[8], a4[4], b4[4];
  min_x4_16(mn_in, a8);
  max_x4_16(mx_in, b8);
  min_x8_8(a8, a4);
  max_x8_8(b8, b4);
  float a2[2] = {merge_rows<16, true>(a4[0], a4[1]), merge_rows<16, true>(a4[2], a4[3])};
  float b2[2] = {merge_rows<16, false>(b4[0], b4[1]), merge_rows<16, false>(b4[2], b4[3])};
  if (LPG_LOG2 == 6) {
    mn[0] = merge_rows<32, true>(a2[0], a2[1]);
    mx[0] = merge_rows<32, false>(b2[0], b2[1]);
    quad_minmax(mn[0], mx[0]);
    mn[1] = mn[0];
    mx[1] = mx[0];
  } else {
    mn[0] = a2[0]; mn[1] = a2[1];
    mx[0] = b2[0]; mx[1] = b2[1];
    quad_minmax(mn[0], mx[0]);
    quad_minmax(mn[1], mx[1]);
  }
}

// ---- binary16 pairs: two elements per dword, no widening --------------------------------------
// Minimum / maximum of both halves of three or two dwords (finite inputs; a zero may come out
// with either sign, which the callers' "+ 0.0f" settles).
__device__ __forceinline__ uint32_t pk_min3_f16(uint32_t a, uint32_t b, uint32_t c) {
  uint32_t r;
  asm("v_pk_minimum3_f16 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ __forceinline__ uint32_t pk_max3_f16(uint32_t a, uint32_t b, uint32_t c) {
  uint32_t r;
  asm("v_pk_maximum3_f16 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ __forceinline__ uint32_t pk_min_f16(uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_pk_min_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ uint32_t pk_max_f16(uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// The statistics of the eight binary16 values of a chunk as one dword [-max : min] (two
// binary16 halves), so that a single packed minimum per step reduces both across lanes.
__device__ __forceinline__ uint32_t chunk_stat_f16(const uint4& raw) {
  const uint32_t mn = pk_min_f16(pk_min3_f16(raw.x, raw.y, raw.z), raw.w);
  const uint32_t mx = pk_max_f16(pk_max3_f16(raw.x, raw.y, raw.z), raw.w);
  uint32_t q, r;
  // both halves of q: min of the two halves of mn; both halves of r: -(max of the two halves of mx)
  asm("v_pk_min_f16 %0, %1, %1 op_sel:[0,1] op_sel_hi:[1,0]" : "=v"(q) : "v"(mn));
  asm("v_pk_min_f16 %0, %1, %1 op_sel:[0,1] op_sel_hi:[1,0] neg_lo:[1,1] neg_hi:[1,1]" : "=v"(r) : "v"(mx));
  return __builtin_amdgcn_perm(r, q, 0x07060100u);       // high half from r, low half from q
}
__device__ __forceinline__ float stat_f16_min(uint32_t p) { return (float)__builtin_bit_cast(_Float16, (uint16_t)p); }
__device__ __forceinline__ float stat_f16_max(uint32_t p) {
  return -(float)__builtin_bit_cast(_Float16, (uint16_t)(p >> 16));
}

// Packed minimum of four [-max : min] dwords over aligned runs of 2^LPG_LOG2 lanes; the complete
// result is guaranteed in the LAST lane of each run.  A step moves the partner lane's value with
// a DPP move and merges it with a packed minimum (packed instructions take no DPP operand).
// Four chains are interleaved, so every DPP read of a register comes at least three instructions
// after the write (two wait states are needed); the leading and trailing s_nop cover what the
// compiler puts around the block.  In the row-broadcast steps the lanes outside the row mask keep
// the previous step's partner value in the temporary: a value of their own run, so merging it
// again changes nothing.
#define DAF_PK4(CTRL)                                                                              \
  "v_mov_b32_dpp %4, %0 " CTRL "\n" "v_mov_b32_dpp %5, %1 " CTRL "\n"                              \
  "v_mov_b32_dpp %6, %2 " CTRL "\n" "v_mov_b32_dpp %7, %3 " CTRL "\n"                              \
  "v_pk_min_f16 %0, %0, %4\n" "v_pk_min_f16 %1, %1, %5\n"                                          \
  "v_pk_min_f16 %2, %2, %6\n" "v_pk_min_f16 %3, %3, %7\n"
#define DAF_PK4_ASM(BODY)                                                                          \
  asm("s_nop 4\n" BODY "s_nop 1\n"                                                                 \
      : "+v"(a), "+v"(b), "+v"(c), "+v"(d), "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3))
template <int LPG_LOG2>
__device__ __forceinline__ void seg_pk_min_x4(uint32_t& a, uint32_t& b, uint32_t& c, uint32_t& d) {
  static_assert(LPG_LOG2 >= 2 && LPG_LOG2 <= 6, "run length 4..64 lanes");
  uint32_t t0, t1, t2, t3;
  if constexpr (LPG_LOG2 == 2) {
    DAF_PK4_ASM(DAF_PK4(DAF_DPP_X1) DAF_PK4(DAF_DPP_X2));
  } else if constexpr (LPG_LOG2 == 3) {
    DAF_PK4_ASM(DAF_PK4(DAF_DPP_X1) DAF_PK4(DAF_DPP_X2) DAF_PK4(DAF_DPP_HM));
  } else if constexpr (LPG_LOG2 == 4) {
    DAF_PK4_ASM(DAF_PK4(DAF_DPP_X1) DAF_PK4(DAF_DPP_X2) DAF_PK4(DAF_DPP_HM) DAF_PK4(DAF_DPP_M));
  } else if constexpr (LPG_LOG2 == 5) {
    DAF_PK4_ASM(DAF_PK4(DAF_DPP_X1) DAF_PK4(DAF_DPP_X2) DAF_PK4(DAF_DPP_HM) DAF_PK4(DAF_DPP_M)
                DAF_PK4(DAF_DPP_B15));
  } else {
    DAF_PK4_ASM(DAF_PK4(DAF_DPP_X1) DAF_PK4(DAF_DPP_X2) DAF_PK4(DAF_DPP_HM) DAF_PK4(DAF_DPP_M)
                DAF_PK4(DAF_DPP_B15) DAF_PK4(DAF_DPP_B31));
  }
}
#undef DAF_PK4_ASM
#undef DAF_PK4

// min - x for the low (HI = 0) or high (HI = 1) binary16 half of `pair`, in binary32 with one
// rounding: a mixed-precision fma x * (-1) + min, which is the widened subtraction exactly.
template <int HI>
__device__ __forceinline__ float min_minus_half(uint32_t pair, float mn) {
  float d;
  if (HI) asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(pair), "v"(mn));
  else    asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(pair), "v"(mn));
  return d;
}

// Sums of two values over aligned runs of 2^LPG_LOG2 lanes (complete in the LAST lane of each
// run).  Two chains: an instruction reads the register written two instructions earlier, so one
// s_nop between steps completes the two wait states a DPP read needs.
#define DAF_SUM2(CTRL)                         \
  "v_add_f32_dpp %0, %0, %0 " CTRL "\n"        \
  "v_add_f32_dpp %1, %1, %1 " CTRL "\n"        \
  "s_nop 0\n"
template <int LPG_LOG2>
__device__ __forceinline__ void seg_sum2(float& a, float& b) {
  static_assert(LPG_LOG2 >= 2 && LPG_LOG2 <= 6, "run length 4..64 lanes");
  if constexpr (LPG_LOG2 == 2) {
    asm("s_nop 4\n" DAF_SUM2(DAF_DPP_X1) DAF_SUM2(DAF_DPP_X2) "s_nop 1\n" : "+v"(a), "+v"(b));
  } else if constexpr (LPG_LOG2 == 3) {
    asm("s_nop 4\n" DAF_SUM2(DAF_DPP_X1) DAF_SUM2(DAF_DPP_X2) DAF_SUM2(DAF_DPP_HM) "s_nop 1\n" : "+v"(a), "+v"(b));
  } else if constexpr (LPG_LOG2 == 4) {
    asm("s_nop 4\n" DAF_SUM2(DAF_DPP_X1) DAF_SUM2(DAF_DPP_X2) DAF_SUM2(DAF_DPP_HM) DAF_SUM2(DAF_DPP_M) "s_nop 1\n"
        : "+v"(a), "+v"(b));
  } else if constexpr (LPG_LOG2 == 5) {
    asm("s_nop 4\n" DAF_SUM2(DAF_DPP_X1) DAF_SUM2(DAF_DPP_X2) DAF_SUM2(DAF_DPP_HM) DAF_SUM2(DAF_DPP_M)
        DAF_SUM2(DAF_DPP_B15) "s_nop 1\n" : "+v"(a), "+v"(b));
  } else {
    asm("s_nop 4\n" DAF_SUM2(DAF_DPP_X1) DAF_SUM2(DAF_DPP_X2) DAF_SUM2(DAF_DPP_HM) DAF_SUM2(DAF_DPP_M)
        DAF_SUM2(DAF_DPP_B15) DAF_SUM2(DAF_DPP_B31) "s_nop 1\n" : "+v"(a), "+v"(b));
  }
}
#undef DAF_SUM2

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

// List calls: the units (tiles, blocks) of all tensors of a launch form one sequence, and
// ends[t] holds the number of units of entries 0..t (0xFFFFFFFF in the unused entries).  The
// entry that owns unit `pos` is the number of entries whose cumulative count is <= pos.  The 32
// counts are kernel arguments: they arrive with the wave's first scalar loads, and 32 scalar
// compares find the entry without a trip to memory (a walk over the descriptors costs one
// dependent load per entry; a per-lane load and a ballot one vector round trip, which made a
// short-lived dequantize wave a tenth slower).  `pos` must be wave-uniform.
constexpr int kBatchSlots = 32;
__device__ __forceinline__ int batch_entry_of(const uint32_t (&ends)[kBatchSlots], uint32_t pos) {
  int t = 0;
#pragma unroll
  for (int i = 0; i < kBatchSlots; ++i) t += (ends[i] <= pos) ? 1 : 0;
  return t;
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

// floor(x + 1/2) as a signed integer in one instruction (round to nearest, ties upward).
__device__ __forceinline__ int round_half_up_to_int(float x) {
  int r;
  asm("v_cvt_rpi_i32_f32 %0, %1" : "=v"(r) : "v"(x));
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
