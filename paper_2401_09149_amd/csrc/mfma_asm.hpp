// Single-instruction assembly wrappers used where the instruction ORDER is part of the design:
// a kernel that runs one wave per SIMD can only overlap its elementwise arithmetic with its
// matrix products if the two are interleaved in program order (one MFMA, then the handful of
// VALU instructions its 32-cycle shadow can hide), and its stationary operands and
// accumulators have to stay in AGPRs without being copied back and forth.  Every statement
// is `asm volatile`, so the compiler keeps them in source order; it still allocates the
// registers and places the LDS waits for their inputs.
//
// Hazards the compiler cannot see inside assembly are handled here by construction:
//  - a VALU instruction may read an MFMA result only 11 wait states after an 8-pass MFMA was
//    issued; the groups that consume a chain's result take a `lead` argument that prepends
//    an s_nop covering that distance, and the kernels place them at least two MFMAs behind
//    the chain's last MFMA anyway;
//  - a non-transcendental VALU instruction needs one wait state after the v_exp_f32 whose
//    result it reads (s_nop 0 in softmax_pair).
#pragma once
#include "attn_common.hpp"

namespace ie {

// acc(VGPR) = A(VGPR) * B(AGPR)
__device__ __forceinline__ void mfma_first_b_agpr(f32x16& acc, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "a"(b));
}
// acc(VGPR) = cin(VGPR) + A(VGPR) * B(AGPR); acc and cin are distinct registers
__device__ __forceinline__ void mfma_first_cin_b_agpr(f32x16& acc, const bf16x8& a, const bf16x8& b, const f32x16& cin) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(acc) : "v"(a), "a"(b), "v"(cin));
}
// acc(VGPR) += A(VGPR) * B(AGPR)
__device__ __forceinline__ void mfma_next_b_agpr(f32x16& acc, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "a"(b));
}
// acc(AGPR) += A(VGPR) * B(VGPR)
__device__ __forceinline__ void mfma_acc_agpr(f32x16& acc, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// The same for compiler-scheduled code, where the instruction in front may be a move INTO the accumulator that the
// compiler placed there (it does not know that the statement reads it as an MFMA's C operand: two wait states).
__device__ __forceinline__ void mfma_acc_agpr_after_moves(f32x16& acc, const bf16x8& a, const bf16x8& b) {
  asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// Pins the compiler's own memory instructions (LDS reads) to this point of the sequence.
__device__ __forceinline__ void asm_fence() { asm volatile("" ::: "memory"); }
__device__ __forceinline__ void mfma_result_fence() { asm volatile("s_nop 15\n\ts_nop 3" ::: "memory"); }

// p0 = exp2(s0*c - l0), p1 = exp2(s1*c - l1), packed = {bf16(p0), bf16(p1)}
template <bool LEAD>
__device__ __forceinline__ void softmax_pair(float& p0, float& p1, uint32_t& packed, float s0, float s1, float c,
                                             float l0, float l1) {
  if (LEAD) asm volatile("s_nop 9");
  asm volatile(
      "v_fma_f32 %0, %3, %5, -%6\n\t"
      "v_fma_f32 %1, %4, %5, -%7\n\t"
      "v_exp_f32 %0, %0\n\t"
      "v_exp_f32 %1, %1\n\t"
      "s_nop 0\n\t"
      "v_cvt_pk_bf16_f32 %2, %0, %1"
      : "=&v"(p0), "=&v"(p1), "=&v"(packed)
      : "v"(s0), "v"(s1), "s"(c), "v"(l0), "v"(l1));
}
// packed = {bf16(p0 * (dp0 - d0)), bf16(p1 * (dp1 - d1))}
template <bool LEAD>
__device__ __forceinline__ void dscore_pair(uint32_t& packed, float p0, float p1, float dp0, float dp1, float d0, float d1) {
  if (LEAD) asm volatile("s_nop 9");
  float t0, t1;
  asm volatile(
      "v_sub_f32 %0, %5, %7\n\t"
      "v_sub_f32 %1, %6, %8\n\t"
      "v_mul_f32 %0, %0, %3\n\t"
      "v_mul_f32 %1, %1, %4\n\t"
      "v_cvt_pk_bf16_f32 %2, %0, %1"
      : "=&v"(t0), "=&v"(t1), "=&v"(packed)
      : "v"(p0), "v"(p1), "v"(dp0), "v"(dp1), "v"(d0), "v"(d1));
}

// Single-element forms, for schedules that give every MFMA at most ~4 VALU slots.
// p = exp2(s*c + nl), nl = -lse*log2(e).  LEAD: the first use of an MFMA chain's result (see file header).
template <bool LEAD>
__device__ __forceinline__ void softmax_elem(float& p, float s, float c, float nl) {
  if (LEAD) asm volatile("s_nop 9");
  asm volatile("v_fma_f32 %0, %1, %2, %3\n\tv_exp_f32 %0, %0" : "=&v"(p) : "v"(s), "s"(c), "v"(nl));
}
// d = p * dp  (the dP chain started from -delta)
template <bool LEAD>
__device__ __forceinline__ void mul_elem(float& d, float p, float dp) {
  if (LEAD) asm volatile("s_nop 9");
  asm volatile("v_mul_f32 %0, %1, %2" : "=v"(d) : "v"(p), "v"(dp));
}
// packed = {bf16(a), bf16(b)}.  When a or b comes from v_exp_f32, at least one other instruction
// must have been issued since (the callers put an MFMA in between).
__device__ __forceinline__ void pack_pair(uint32_t& packed, float a, float b) {
  asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(packed) : "v"(a), "v"(b));
}

// ---- row maximum of a 32x32 C block held as one column per lane (forward softmax) -----------
// t = max(s[0..8]) / t = max(t, s[9..15]): two groups of four instructions
template <bool LEAD>
__device__ __forceinline__ void colmax_lo(float& t, const f32x16& s) {
  if (LEAD) asm volatile("s_nop 9");
  asm volatile(
      "v_max3_f32 %0, %1, %2, %3\n\t"
      "v_max3_f32 %0, %0, %4, %5\n\t"
      "v_max3_f32 %0, %0, %6, %7\n\t"
      "v_max3_f32 %0, %0, %8, %9"
      : "=&v"(t)
      : "v"(s[0]), "v"(s[1]), "v"(s[2]), "v"(s[3]), "v"(s[4]), "v"(s[5]), "v"(s[6]), "v"(s[7]), "v"(s[8]));
}
__device__ __forceinline__ void colmax_hi(float& t, const f32x16& s) {
  asm volatile(
      "v_max3_f32 %0, %0, %1, %2\n\t"
      "v_max3_f32 %0, %0, %3, %4\n\t"
      "v_max3_f32 %0, %0, %5, %6\n\t"
      "v_max_f32 %0, %0, %7"
      : "+v"(t)
      : "v"(s[9]), "v"(s[10]), "v"(s[11]), "v"(s[12]), "v"(s[13]), "v"(s[14]), "v"(s[15]));
}
// t = max(t, t of the lane 32 away): the two half-waves hold the two halves of a column
__device__ __forceinline__ void halfwave_max_asm(float& t) {
  float u;
  asm volatile(
      "v_mov_b32 %1, %0\n\t"
      "s_nop 1\n\t"
      "v_permlane32_swap_b32 %0, %1\n\t"
      "v_max_f32 %0, %0, %1"
      : "+v"(t), "=&v"(u));
}
// One element of the forward softmax, as one block so that the compiler puts nothing between its
// instructions: p = exp2(s*c + negmc); then, with the PREVIOUS elements (whose v_exp_f32 results
// are by now at least one instruction old): l += p_prev, and packed = {bf16(p_prev2), bf16(p_prev)}.
__device__ __forceinline__ void exp_elem(float& p, float s, float c, float negmc) {
  asm volatile("v_fma_f32 %0, %1, %2, %3\n\tv_exp_f32 %0, %0" : "=&v"(p) : "v"(s), "s"(c), "v"(negmc));
}
__device__ __forceinline__ void exp_elem_add(float& p, float s, float c, float negmc, float& l, float p_prev) {
  asm volatile("v_fma_f32 %0, %2, %3, %4\n\tv_exp_f32 %0, %0\n\tv_add_f32 %1, %1, %5"
               : "=&v"(p), "+v"(l)
               : "v"(s), "s"(c), "v"(negmc), "v"(p_prev));
}
__device__ __forceinline__ void exp_elem_add_pack(float& p, float s, float c, float negmc, float& l, float p_prev,
                                                  uint32_t& packed, float p_prev2) {
  asm volatile("v_fma_f32 %0, %3, %4, %5\n\tv_exp_f32 %0, %0\n\tv_add_f32 %1, %1, %6\n\tv_cvt_pk_bf16_f32 %2, %7, %6"
               : "=&v"(p), "+v"(l), "=v"(packed)
               : "v"(s), "s"(c), "v"(negmc), "v"(p_prev), "v"(p_prev2));
}
// Element 2 opens the block's sum: lsum = p0 + p1.
__device__ __forceinline__ void exp_elem_first_sum(float& p, float s, float c, float negmc, float& lsum, float p0, float p1,
                                                   uint32_t& packed) {
  asm volatile("v_fma_f32 %0, %3, %4, %5\n\tv_exp_f32 %0, %0\n\tv_add_f32 %1, %6, %7\n\tv_cvt_pk_bf16_f32 %2, %6, %7"
               : "=&v"(p), "=&v"(lsum), "=v"(packed)
               : "v"(s), "s"(c), "v"(negmc), "v"(p0), "v"(p1));
}
// The last element's sum and pack (one MFMA later).
__device__ __forceinline__ void add_pack(float& l, float p_prev, uint32_t& packed, float p_prev2) {
  asm volatile("v_add_f32 %0, %0, %2\n\tv_cvt_pk_bf16_f32 %1, %3, %2" : "+v"(l), "=v"(packed) : "v"(p_prev), "v"(p_prev2));
}

__device__ __forceinline__ bf16x8 frag_from_words(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  u32x4 w = {a, b, c, d};
  return __builtin_bit_cast(bf16x8, w);
}

}  // namespace ie
