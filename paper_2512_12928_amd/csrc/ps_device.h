// Device-side helpers shared by the gfx950 kernel files: vector types, bf16 packing, addressing of the paged
// cache, cross-lane maxima, the global->LDS load, wait-count encoding, profiling clock records.
#pragma once
#include "ps_internal.h"

namespace ps {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define PS_NEG_INF (-__builtin_inff())
// Online softmax with a lazy reference maximum (prefill work).  Softmax does not care which reference m the exponentials
// are taken against as long as the row sum and the accumulators use the same one: the final division (or the merge, which
// is handed this m) takes the factor out, fp32 has the range, and bf16 has fp32's exponent.  Two uses:
//  * both prefill roles rescale the accumulators (64 multiplications per lane that stand between the output MFMAs of one
//    tile and those of the next) only when some row's tile maximum exceeds its reference by more than PS_RESCALE_SLACK
//    powers of two; until then a row's probabilities are at most 2^PS_RESCALE_SLACK instead of at most 1;
//  * the MFMA waves of fused_kernel do not even take the maximum of a tile unless they have to: on their first tile,
//    while some row has seen no key yet (m = -inf), and on a tile whose row sums say that the reference has fallen too
//    far behind (a row sum beyond PS_ROWSUM_LIMIT, or not a number: the tile is then done once more with its maximum
//    taken, before anything of it has been accumulated).  In between the probabilities are bounded by that limit, and
//    a tile costs 8 three-way maxima and a cross-lane exchange less.  (In the prefill role of attention_kernel the same
//    check cost what the maxima had when made once per half tile, and more when made once per tile with all
//    exponentials ahead of the output MFMAs: that role takes the maximum of every tile.)
#define PS_RESCALE_SLACK 8.f
#define PS_ROWSUM_LIMIT 0x1p40f

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);  // round to nearest even
  return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// Zero the 16-bit elements e (0..3) of v whose token index first+e is >= limit.
__device__ __forceinline__ uint2 zero_from(uint2 v, int first, int limit) {
  uint32_t m0 = (first + 0 < limit ? 0x0000FFFFu : 0u) | (first + 1 < limit ? 0xFFFF0000u : 0u);
  uint32_t m1 = (first + 2 < limit ? 0x0000FFFFu : 0u) | (first + 3 < limit ? 0xFFFF0000u : 0u);
  v.x &= m0;
  v.y &= m1;
  return v;
}

__device__ __forceinline__ const uint16_t* k_slice(const uint16_t* cache, int block, int Hkv, int g) {
  return cache + ((size_t)(block * 2 + 0) * Hkv + g) * kSliceElems;
}
__device__ __forceinline__ const uint16_t* v_slice(const uint16_t* cache, int block, int Hkv, int g) {
  return cache + ((size_t)(block * 2 + 1) * Hkv + g) * kSliceElems;
}

// Profiling only (P.clocks != NULL): the first thread of workgroup `slot` notes the shader-clock counter and
// the constant 100 MHz counter, at its start (at = 0) and at its end (at = 2); the host turns the two
// differences into the shader clock the workgroup ran at.  Decode workgroups use slots [0, kClockSlots),
// prefill workgroups [kClockSlots, 2 * kClockSlots); workgroups beyond that are not recorded.
__device__ __forceinline__ void clock_record(const StepParams& P, int slot, int at) {
  if (P.clocks != nullptr && threadIdx.x == 0 && slot < 2 * kClockSlots) {
    P.clocks[slot * 4 + at] = __builtin_amdgcn_s_memtime();
    P.clocks[slot * 4 + at + 1] = __builtin_amdgcn_s_memrealtime();
  }
}

__device__ __forceinline__ bf16x8 load_stream16(const uint16_t* p) {
  return __builtin_bit_cast(bf16x8, __builtin_nontemporal_load((const u32x4*)p));
}

// Zero the 16-bit elements e (0..7) of v whose token index first+e is >= limit.
__device__ __forceinline__ bf16x8 zero_from8(bf16x8 v, int first, int limit) {
  u32x4 w = __builtin_bit_cast(u32x4, v);
#pragma unroll
  for (int i = 0; i < 4; ++i)
    w[i] &= (first + 2 * i < limit ? 0x0000FFFFu : 0u) | (first + 2 * i + 1 < limit ? 0xFFFF0000u : 0u);
  return __builtin_bit_cast(bf16x8, w);
}

// Sum of the 16 bf16 values in eight registers (each a pair), as fp32: four independent chains of v_dot2c_f32_bf16
// against a pair of ones, then three additions.  The block ends with the wait states the ISA asks for before another
// kind of vector instruction reads a dot product's result.
__device__ __forceinline__ float sum_bf16x16(const uint4& a, const uint4& b) {
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  const uint32_t ones = 0x3F803F80u;
  asm("v_dot2c_f32_bf16 %0, %4, %12\n\tv_dot2c_f32_bf16 %1, %5, %12\n\tv_dot2c_f32_bf16 %2, %6, %12\n\tv_dot2c_f32_bf16 %3, %7, %12\n\t"
      "v_dot2c_f32_bf16 %0, %8, %12\n\tv_dot2c_f32_bf16 %1, %9, %12\n\tv_dot2c_f32_bf16 %2, %10, %12\n\tv_dot2c_f32_bf16 %3, %11, %12\n\t"
      "s_nop 2"
      : "+v"(s0), "+v"(s1), "+v"(s2), "+v"(s3)
      : "v"(a.x), "v"(a.y), "v"(a.z), "v"(a.w), "v"(b.x), "v"(b.y), "v"(b.z), "v"(b.w), "v"(ones));
  return (s0 + s1) + (s2 + s3);
}

// The same for the 8 bf16 values in four registers.
__device__ __forceinline__ float sum_bf16x8(const uint4& a) {
  float s0 = 0.f, s1 = 0.f;
  const uint32_t ones = 0x3F803F80u;
  asm("v_dot2c_f32_bf16 %0, %2, %6\n\tv_dot2c_f32_bf16 %1, %3, %6\n\tv_dot2c_f32_bf16 %0, %4, %6\n\tv_dot2c_f32_bf16 %1, %5, %6\n\t"
      "s_nop 2"
      : "+v"(s0), "+v"(s1)
      : "v"(a.x), "v"(a.y), "v"(a.z), "v"(a.w), "v"(ones));
  return s0 + s1;
}

// max of two that are never NaN (fmaxf wraps NaN-quieting moves around its operands)
__device__ __forceinline__ float max2(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// max over lanes l and l ^ 32 (both lanes get it), on the VALU: v_permlane32_swap exchanges the upper half of its
// first operand with the lower half of its second, so with x in both, one register comes back holding the lower
// half's values in both halves and the other the upper half's.  Written as asm with both registers as outputs: the
// compiler's builtin hands back the first register for either element of its result here, which silently made this
// the lower half's value instead of the maximum.  The swap needs two wait states behind a vector write of its operands.
__device__ __forceinline__ float xor32_max(float x) {
  float a = x, b = x;
  asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  return max2(a, b);
}

// max over lanes l and l ^ 16: v_permlane16_swap exchanges the odd rows (of 16 lanes) of its first operand with the
// even rows of its second.
__device__ __forceinline__ float xor16_max(float x) {
  float a = x, b = x;
  asm("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  return max2(a, b);
}

// s_waitcnt immediate that waits only for vmcnt <= n (gfx9 encoding)
#define PS_VMCNT(n) (((n) & 0xF) | (((n) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

// One lane's 16 bytes at `gptr` -> LDS at lds_base + lane*16 (lds_base wave-uniform).  The LDS
// base travels in M0, which is saved and restored around the load.
__device__ __forceinline__ void load_to_lds16(const void* gptr, uint32_t lds_base) {
  uint32_t saved;
  asm volatile(
      "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
      : "=&s"(saved)
      : "v"(gptr), "s"(lds_base)
      : "memory");
}

// The same with an instruction offset OFF (0 .. 4095 bytes), which the hardware adds to the global address AND to the
// LDS address: lane's 16 bytes at gptr + OFF -> LDS at lds_base + OFF + lane*16.  Several loads off one address
// register pair then cost no vector arithmetic between them.
template <int OFF>
__device__ __forceinline__ void load_to_lds16_off(const void* gptr, uint32_t lds_base) {
  static_assert(OFF >= 0 && OFF < 4096, "13-bit signed instruction offset, used unsigned");
  uint32_t saved;
  asm volatile(
      "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %1, off offset:%3\n\ts_mov_b32 m0, %0"
      : "=&s"(saved)
      : "v"(gptr), "s"(lds_base), "n"(OFF)
      : "memory");
}

// The same addressed by a wave-uniform base (a scalar register pair) plus a 32-bit per-lane byte offset: lane's 16 bytes
// at sbase + voff + OFF -> LDS at lds_base + OFF + lane*16.  Next to busy MFMA waves this form is taken by the memory
// path about three times faster than one with a 64-bit address per lane (one vector register to read instead of two).
template <int OFF>
__device__ __forceinline__ void load_to_lds16_sbase(const void* sbase, uint32_t voff, uint32_t lds_base) {
  static_assert(OFF >= 0 && OFF < 4096, "13-bit signed instruction offset, used unsigned");
  uint32_t saved;
  asm volatile(
      "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\tglobal_load_lds_dwordx4 %1, %2 offset:%4\n\ts_mov_b32 m0, %0"
      : "=&s"(saved)
      : "v"(voff), "s"(sbase), "s"(lds_base), "n"(OFF)
      : "memory");
}

// Largest of the 16 elements a lane holds of a 32x32 MFMA result, without the NaN-quieting moves the compiler wraps
// around fmaxf (the inputs are never NaN: finite scores or -inf).  The ISA asks for 11 wait states between an 8-pass
// MFMA and a vector instruction that reads its result, and the compiler counts none for instructions inside inline asm
// (nor does it keep a separate NOP statement in front of them): with NOPS the block starts with those wait states, so
// it may follow the MFMA at once.
template <bool NOPS>
__device__ __forceinline__ float max16(const f32x16& s) {
  float r;
  if (NOPS)
    asm("s_nop 7\n\ts_nop 3\n\t"
        "v_max3_f32 %0, %1, %2, %3\n\tv_max3_f32 %0, %0, %4, %5\n\tv_max3_f32 %0, %0, %6, %7\n\t"
        "v_max3_f32 %0, %0, %8, %9\n\tv_max3_f32 %0, %0, %10, %11\n\tv_max3_f32 %0, %0, %12, %13\n\t"
        "v_max3_f32 %0, %0, %14, %15\n\tv_max_f32 %0, %0, %16"
        : "=&v"(r)
        : "v"(s[0]), "v"(s[1]), "v"(s[2]), "v"(s[3]), "v"(s[4]), "v"(s[5]), "v"(s[6]), "v"(s[7]), "v"(s[8]), "v"(s[9]),
          "v"(s[10]), "v"(s[11]), "v"(s[12]), "v"(s[13]), "v"(s[14]), "v"(s[15]));
  else
    asm("v_max3_f32 %0, %1, %2, %3\n\tv_max3_f32 %0, %0, %4, %5\n\tv_max3_f32 %0, %0, %6, %7\n\t"
        "v_max3_f32 %0, %0, %8, %9\n\tv_max3_f32 %0, %0, %10, %11\n\tv_max3_f32 %0, %0, %12, %13\n\t"
        "v_max3_f32 %0, %0, %14, %15\n\tv_max_f32 %0, %0, %16"
        : "=&v"(r)
        : "v"(s[0]), "v"(s[1]), "v"(s[2]), "v"(s[3]), "v"(s[4]), "v"(s[5]), "v"(s[6]), "v"(s[7]), "v"(s[8]), "v"(s[9]),
          "v"(s[10]), "v"(s[11]), "v"(s[12]), "v"(s[13]), "v"(s[14]), "v"(s[15]));
  return r;
}
}  // namespace ps
