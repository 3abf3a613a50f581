// Decode of one lane's share of a narrow-format group to correctly rounded bf16, shared by the kernels that multiply
// bf16-rounded weights (the LDS-tiled ones).  Device code only.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace ccq {

typedef __attribute__((ext_vector_type(2))) float dec_f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 dec_bf16x2;

// (a & mask) | orv in plain C (no instruction is written as inline assembly: the compiler's hazard recognizer does
// not see those); callers keep mask and orv in registers so that v_and_or_b32 is selected.
__device__ __forceinline__ uint32_t dec_and_or(uint32_t a, uint32_t mask, uint32_t orv) { return (a & mask) | orv; }

__device__ __forceinline__ uint32_t dec_pack_bf16(float lo, float hi) {
  dec_f32x2 v = {lo, hi};
  dec_bf16x2 b = __builtin_convertvector(v, dec_bf16x2);  // round to nearest even
  return __builtin_bit_cast(uint32_t, b);
}

constexpr uint32_t kDecMask2 = 0x03F003F0u;  // bits 4..9 of the mantissas of two fp16 numbers
constexpr uint32_t kDecBase2 = 0x54005400u;  // fp16 64.0 twice
constexpr float kDecBase = 64.f;             // the accumulator offset c0 is -(kDecBase + zp) * scale

typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;

// Sixteen weights of one lane (four stored bytes of a narrow-format group: k = 16 kq .. 16 kq + 15) to correctly
// rounded bf16, eight packed pairs in k order.
//   Code Cluster (Alg. 3): c = round(q alpha + beta) by one FMA against beta + 2^23 (`bem`), the 15-bit code in the
//   low mantissa bits.  Two codes side by side in one register (v_perm), and for each of the four windows of Table 1's
//   shift list [9,6,3,0] one shift and one v_and_or put both codes' state into bits 4..9 of the mantissa of fp16 64.0:
//   two fp16 numbers 64 + state, exact.  The linear map d = (w_uint - zp) s of Alg. 3's last line is then one
//   mixed-precision FMA per weight, fma(64 + state, s, c0) with c0 = -(64 + zp) s: 64 + zp has at most 8 significant
//   bits, s at most 15 (a 4-bit field times an fp16 super scale), so c0 and the result are exact in fp32 and the bf16
//   written is the correctly rounded exact weight.  50 vector instructions per 16 weights (64 with one fp32 number per
//   state, the first version).
__device__ __forceinline__ void decode16_narrow(uint32_t d, float al, float bem, float s, float c0, uint32_t mask2, uint32_t base2, uint32_t (&o)[8]) {
  uint32_t cb[4];
#pragma unroll
  for (int b = 0; b < 4; ++b) cb[b] = __builtin_bit_cast(uint32_t, __builtin_fmaf((float)((d >> (8 * b)) & 0xFFu), al, bem));
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint32_t pr = __builtin_amdgcn_perm(cb[2 * h + 1], cb[2 * h], 0x05040100u);  // code 2h in the low half, code 2h + 1 in the high half
    const f16x2 w0 = __builtin_bit_cast(f16x2, dec_and_or(pr >> 5, mask2, base2));  // window at bit 9: weights 8h + 0 and 8h + 4
    const f16x2 w1 = __builtin_bit_cast(f16x2, dec_and_or(pr >> 2, mask2, base2));  // window at bit 6: weights 8h + 1 and 8h + 5
    const f16x2 w2 = __builtin_bit_cast(f16x2, dec_and_or(pr << 1, mask2, base2));  // window at bit 3: weights 8h + 2 and 8h + 6
    const f16x2 w3 = __builtin_bit_cast(f16x2, dec_and_or(pr << 4, mask2, base2));  // window at bit 0: weights 8h + 3 and 8h + 7
    o[4 * h + 0] = dec_pack_bf16(__builtin_fmaf((float)w0.x, s, c0), __builtin_fmaf((float)w1.x, s, c0));
    o[4 * h + 1] = dec_pack_bf16(__builtin_fmaf((float)w2.x, s, c0), __builtin_fmaf((float)w3.x, s, c0));
    o[4 * h + 2] = dec_pack_bf16(__builtin_fmaf((float)w0.y, s, c0), __builtin_fmaf((float)w1.y, s, c0));
    o[4 * h + 3] = dec_pack_bf16(__builtin_fmaf((float)w2.y, s, c0), __builtin_fmaf((float)w3.y, s, c0));
  }
}

constexpr uint32_t kDecMaskW2 = 0x00F000F0u;  // bits 4..7 of the mantissas of two fp16 numbers (a 4-bit state)

// Six weights of one lane (two stored bytes a, b of a wide-format group: codes of (L=4,N=3,S=2), weights 3 code .. + 2)
// to fp32, in k order.  `pp` holds the two bytes as {0, b, 0, a}.  Table 1's shift list [4, 2, 0] with mask 0xF: the
// window at shift 4 already sits in bits 4..7 of its half, the other two are moved there with one shift each, and one
// v_and_or per window puts both codes' state into the mantissas of two fp16 64.0 (64 + state, exact).  Then Alg. 2's
// last line, d = (w_uint - zp) s, as one mixed-precision FMA per weight with c0 = -(64 + zp) s (exact in fp32: at
// most 8 significant bits times at most 15).  11 vector instructions per 6 weights.
__device__ __forceinline__ void decode6_wide(uint32_t pp, float s, float c0, uint32_t mask2, uint32_t base2, float (&w)[6]) {
  const f16x2 f0 = __builtin_bit_cast(f16x2, dec_and_or(pp, mask2, base2));
  const f16x2 f1 = __builtin_bit_cast(f16x2, dec_and_or(pp << 2, mask2, base2));
  const f16x2 f2 = __builtin_bit_cast(f16x2, dec_and_or(pp << 4, mask2, base2));
  w[0] = __builtin_fmaf((float)f0.x, s, c0);
  w[1] = __builtin_fmaf((float)f1.x, s, c0);
  w[2] = __builtin_fmaf((float)f2.x, s, c0);
  w[3] = __builtin_fmaf((float)f0.y, s, c0);
  w[4] = __builtin_fmaf((float)f1.y, s, c0);
  w[5] = __builtin_fmaf((float)f2.y, s, c0);
}

}  // namespace ccq
