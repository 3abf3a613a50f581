// Dense GEMV on narrow-format weights -- the decode step of generation (one activation row, Alg. 3 fused into the
// contraction; the GEMV operator of the "Inference Performance" section).
//
// A call of this size (19 MB for 8192 x 8192) lasts a few microseconds and is bound by instruction issue, not by
// HBM: what counts is the number of instructions per weight and how early every wavefront has all of its requests
// in flight.  Shape of the kernel:
//   * a workgroup owns one row tile (16 output rows; RT = 1 is what is built) and all of K; its W wavefronts cut K into W shares of TPW
//     k-tiles (4 groups of 64 weights each), so the K reduction stays inside the workgroup (LDS, fixed order);
//   * a wavefront requests its slice of x, its TPW code tiles (one 16-byte nontemporal load per lane and tile:
//     the device order of the code stream is the operand order of the matrix core) and their scales before it does
//     anything else; nothing is requested later and no request sits under a condition;
//   * x is staged once per wavefront in a private LDS region, already permuted into matrix-core operand fragments
//     (no workgroup barrier before the contraction);
//   * decode: the clustered byte q becomes the 15-bit code round(q alpha + beta) with one fused multiply-add against
//     beta + 2^23 (the sum lies in [2^23, 2^24), where fp32 spacing is 1, so the hardware's round-to-nearest-even is
//     the rounding of Eq. 1 and the code sits in the low mantissa bits); two codes are put side by side in one register
//     and each of the four windows of Table 1 (shifts 9, 6, 3, 0, mask 0x3F) is cut out of both with one shift and one
//     and-or into the mantissa of bf16 128.0: the operand is the bf16 integer 128 + state, exactly;
//   * contraction: MFMA 16x16x32 bf16, two per group: lane l = (row n, quarter kq) feeds the eight weights of its quarter
//     as column n of the B operand, and every one of the sixteen rows of the A operand is the one activation row (lane
//     (m, kq) supplies the fragment of quarter kq whatever m is: an LDS broadcast), so every lane receives the whole
//     group's product for its column, the four quarters already added; the accumulator of a group starts at
//     -(128 + zp) sum x, so the group's result is sum (state - zp) x, which is multiplied by the group scale afterwards:
//     the linear map (w_uint - zp) * s of Alg. 3 applied after the contraction.  (The first version used four MFMA
//     4x4x4 per group, each lane multiplying its own 16 weights, and two cross-lane adds at the end: twice the matrix
//     instructions; 8192 x 8192: 6.86 -> 6.65 us, 7.56 -> 7.10 us on a slower box.)
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstddef>
#include <cstdint>
#include <cstdlib>

#include "ccq_internal.h"

namespace ccq {
namespace gemv {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

struct Args {          // 72 bytes: two scalar loads, issued together
  const uint8_t* codes;
  const uint16_t* scales;
  const float* alpha;
  const float* beta;
  const uint16_t* x;
  uint16_t* y;
  const uint16_t* scale_super;   // fp16 [N], compressed scales only
  int32_t tiles;                 // k-tiles per row tile
  float cneg;                    // -(128 + zp)
  int32_t g_last;                // last real group of K (groups past it are padding: their scale is 0, and the
                                 // activations of this group are read in their place)
  int32_t n_last;                // last real output row (rows past it are padding and are not stored)
};

__device__ __forceinline__ uint16_t to_bf16_rne(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);  // NaN stays NaN
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Sum of the eight bf16 values of a fragment in fp32.  (The elements are taken by value first: a bit cast applied
// to an element of an ext-vector lvalue reads element 0.)
__device__ __forceinline__ float frag_sum(const u32x4 o) {
  const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3F803F80u);
  const uint32_t o0 = o.x, o1 = o.y, o2 = o.z, o3 = o.w;
  float s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, o0), ones, 0.f, false);
  s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, o1), ones, s, false);
  s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, o2), ones, s, false);
  s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, o3), ones, s, false);
  return s;
}

// Sum over eight neighbouring lanes (an aligned group of eight), the same in all of them.
__device__ __forceinline__ float group_sum8(float s) {
  s += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, s), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  s += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, s), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  s += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, s), 0x141, 0xF, 0xF, true));  // row_half_mirror: lane 7 - l of its eight
  return s;
}

// Plain C on purpose (no inline assembly: the compiler's hazard recognizer must see the instruction); mask and orv
// are kept in registers by the caller so that a single v_and_or_b32 is selected.
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t orv) { return (a & mask) | orv; }

// The 16 weights of one lane for one group: dword d holds the clustered bytes of codes 4kq .. 4kq+3 of the group.
// Returns, per k-step t (codes 2t, 2t+1), the four registers {state i of code 2t | state i of code 2t+1 << 16} + 128.
__device__ __forceinline__ void decode_dword(uint32_t d, float al, float be_magic, uint32_t c4300, uint32_t mask, u32x4 (&w)[2]) {
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const float fa = __builtin_fmaf((float)((d >> (16 * t)) & 0xFFu), al, be_magic);       // Alg. 3: round(q s_code + zp_code)
    const float fb = __builtin_fmaf((float)((d >> (16 * t + 8)) & 0xFFu), al, be_magic);
    const uint32_t yy = __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, fb), __builtin_bit_cast(uint32_t, fa), 0x05040100u);
    w[t].x = and_or(yy >> 9, mask, c4300);   // Table 1: shifts [9, 6, 3, 0], mask 0x3F, both codes at once
    w[t].y = and_or(yy >> 6, mask, c4300);
    w[t].z = and_or(yy >> 3, mask, c4300);
    w[t].w = and_or(yy, mask, c4300);
  }
}

// RAGGED: the k-tile count is not a multiple of TPW; the last wavefront's share is shorter.  Its requests past the
// last k-tile re-read that tile (a request never sits under a condition) and its loop skips them.
template <int RT, int TPW, int SM, bool RAGGED = false>
__device__ __forceinline__ void rows1_body(const Args& a, const uint32_t rtile0) {
  constexpr int NG = TPW * 4;                         // groups per wavefront
  constexpr int NF = (NG * 8 + 63) / 64;              // x fragments per lane while staging
  constexpr int SH = SM == 0 ? 64 : 16;               // scale halfwords per k-tile and row tile
  constexpr int REGION = NG * 8 * 16 + NG * 4 * 16;   // private LDS bytes per wavefront: fragments, then start-value records
  extern __shared__ __align__(16) unsigned char smem[];
  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t nwaves = blockDim.x >> 6;
  const uint32_t n = lane & 15u, kq = lane >> 4;
  const uint32_t t0 = wave * TPW;                     // first k-tile of this wavefront
  const uint32_t t_last = (uint32_t)a.tiles - 1u;
  // ---- every request, before anything else ------------------------------------------------------------------
  // x: fragment f = (group * 2 + k-step) * 4 + quarter covers elements 64 group + 16 quarter + 8 k-step .. + 7
  u32x4 xv[NF];
#pragma unroll
  for (int i = 0; i < NF; ++i) {
    uint32_t f = lane + 64u * i;
    if (NG * 8 % 64 != 0) f = min(f, (uint32_t)(NG * 8 - 1));
    const uint32_t g = min(t0 * 4u + (f >> 3), (uint32_t)a.g_last);
    const uint32_t off = (g << 6) | ((f & 3u) << 4) | ((f & 4u) << 1);
    xv[i] = *reinterpret_cast<const u32x4*>(a.x + off);
  }
  // per-row parameters next (they are waited for before the first tile: in-order return makes anything requested
  // after the tiles wait for all of them), then the tiles in the order they are consumed
  float al[RT], be_raw[RT];
  uint32_t ssup[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const uint32_t row = min((rtile0 + rt) * 16u + n, (uint32_t)a.n_last);
    al[rt] = a.alpha[row];
    be_raw[rt] = a.beta[row];
    if constexpr (SM == 1) ssup[rt] = a.scale_super[row];
  }
  u32x4 cw[RT][TPW];
  uint32_t sw[RT][TPW][SM == 0 ? 2 : 1];
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const uint32_t ti = RAGGED ? min(t0 + i, t_last) - t0 : (uint32_t)i;
      const uint16_t* sb = a.scales + ((size_t)(rtile0 + rt) * (uint32_t)a.tiles + t0) * SH;
      if constexpr (SM == 0) {
        const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(sb + ti * 64u + n * 4u));
        sw[rt][i][0] = v.x;
        sw[rt][i][1] = v.y;
      } else {
        sw[rt][i][0] = __builtin_nontemporal_load(sb + ti * 16u + n);   // the tile's four 4-bit fields of this row (first line of Alg. 3)
      }
    }
  }
  __builtin_amdgcn_sched_barrier(0);   // keep the (small) scale requests ahead of the code tiles: returns are in order
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const uint32_t ti = RAGGED ? min(t0 + i, t_last) - t0 : (uint32_t)i;
      const uint8_t* cb = a.codes + ((size_t)(rtile0 + rt) * (uint32_t)a.tiles + t0) * 1024u;
      cw[rt][i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(cb + ti * 1024u + lane * 16u));
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  // ---- stage x: permuted fragments and the accumulator start values -(128 + zp) sum x per (group, quarter) ------
  unsigned char* region = smem + (size_t)wave * REGION;
  u32x4* lds_x = reinterpret_cast<u32x4*>(region);
  float* lds_c = reinterpret_cast<float*>(region + NG * 8 * 16);
#pragma unroll
  for (int i = 0; i < NF; ++i) {
    const uint32_t f = lane + 64u * i;
    // the two codes of a k-step cover weights +0..3 and +4..7; their states share registers pairwise, so the
    // k-slots interleave them: {0,4,1,5,2,6,3,7}
    u32x4 o;
    o.x = __builtin_amdgcn_perm(xv[i].z, xv[i].x, 0x05040100u);
    o.y = __builtin_amdgcn_perm(xv[i].z, xv[i].x, 0x07060302u);
    o.z = __builtin_amdgcn_perm(xv[i].w, xv[i].y, 0x05040100u);
    o.w = __builtin_amdgcn_perm(xv[i].w, xv[i].y, 0x07060302u);
    const float s = group_sum8(frag_sum(o));   // the eight fragments of a group sit in eight neighbouring lanes
    if (NG * 8 % 64 == 0 || f < (uint32_t)(NG * 8)) {
      lds_x[f] = o;
      if ((f & 7u) == 0) {
        const float c = a.cneg * s;
        *reinterpret_cast<f32x4*>(lds_c + (f >> 3) * 4u) = f32x4{c, c, c, c};
      }
    }
  }
  __builtin_amdgcn_wave_barrier();
  uint32_t c4300 = 0x43004300u, mask = 0x003F003Fu;
  float magic = 8388608.f;
  asm volatile("" : "+v"(c4300), "+s"(mask), "+v"(magic));   // register values, not literals: v_and_or_b32 gets selected
  float be[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) be[rt] = be_raw[rt] + magic;   // + 2^23: exact, beta is an integer below 2^15

  // ---- contraction ------------------------------------------------------------------------------------------------
  float acc[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) acc[rt] = 0.f;
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    if (RAGGED && t0 + i > t_last) break;   // uniform over the wavefront
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int lg = i * 4 + j;
      const u32x4 x0 = lds_x[(lg * 2 + 0) * 4 + kq];
      const u32x4 x1 = lds_x[(lg * 2 + 1) * 4 + kq];
      const f32x4 cin = *reinterpret_cast<const f32x4*>(lds_c + lg * 4);
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        u32x4 w[2];
        const uint32_t d = j == 0 ? cw[rt][i].x : (j == 1 ? cw[rt][i].y : (j == 2 ? cw[rt][i].z : cw[rt][i].w));
        decode_dword(d, al[rt], be[rt], c4300, mask, w);
        f32x4 p = cin;
        p = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x0), __builtin_bit_cast(bf16x8, w[0]), p, 0, 0, 0);
        p = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x1), __builtin_bit_cast(bf16x8, w[1]), p, 0, 0, 0);
        float s;
        if constexpr (SM == 0) {
          const uint32_t sd = sw[rt][i][j >> 1];
          s = (float)__builtin_bit_cast(_Float16, (uint16_t)((j & 1) ? (sd >> 16) : (sd & 0xFFFFu)));
        } else {
          s = (float)((sw[rt][i][0] >> (4 * j)) & 0xFu);   // the field alone; the row's super scale multiplies the sum once
        }
        acc[rt] = __builtin_fmaf(s, p[0], acc[rt]);
      }
    }
  }
  // ---- the wavefronts of the workgroup (fixed order); the matrix core has added the four quarters of a row ---------
  if (nwaves > 1) {
    __syncthreads();
    float* red = reinterpret_cast<float*>(smem);
    if (wave > 0 && lane < 16u) {
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) red[((wave - 1) * RT + rt) * 16u + lane] = acc[rt];
    }
    __syncthreads();
    if (wave == 0 && lane < 16u) {
      for (uint32_t k = 1; k < nwaves; ++k) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) acc[rt] += red[((k - 1) * RT + rt) * 16u + lane];
      }
    }
  }
  if (wave == 0 && lane < 16u) {
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      float v = acc[rt];
      if constexpr (SM == 1) v *= (float)__builtin_bit_cast(_Float16, (uint16_t)ssup[rt]);
      if ((rtile0 + rt) * 16u + lane <= (uint32_t)a.n_last) a.y[(rtile0 + rt) * 16u + lane] = to_bf16_rne(v);
    }
  }
}

template <int RT, int TPW, int SM>
__global__ void __launch_bounds__(1024) kernel(const Args a) {
  rows1_body<RT, TPW, SM, false>(a, blockIdx.x * RT);
}
template <int TPW, int SM>
__global__ void __launch_bounds__(1024) kernel_unequal(const Args a) {   // the last wavefront's share of K is shorter
  rows1_body<1, TPW, SM, true>(a, blockIdx.x);
}

// ---- two to four activation rows on narrow-format weights -----------------------------------------------------------
// The same kernel with four different rows in the A operand: lane (m, kq) supplies the fragment of row m % 4 (in
// `kernel` all sixteen rows are the same one), so the four accumulator registers of a lane, rows 4 kq .. 4 kq + 3 of its
// column, are the results of rows 0 .. 3.  The weights are streamed and decoded once for all rows; the cost is four
// times the activation staging (LDS: 4 x the fragments) and three more scale multiplies per group.  Rows past M
// repeat row M - 1 and are not stored.
struct Args4 {
  Args a;
  int64_t ldx, ldy;
  int32_t M;
};

// `rows`: NULL (activation row r is row r of x) or the rows' indices in x (the grouped product gathers them).
template <int TPW, int SM, bool RAGGED = false>
__device__ __forceinline__ void rows4_body(const Args& a, const int64_t ldx, const int64_t ldy, const int32_t M, const int32_t* rows, const uint32_t rtile) {
  constexpr int NG = TPW * 4;                             // groups per wavefront
  constexpr int NF = NG * 8 * 4 / 64;                     // staging units (fragment, row) per lane
  constexpr int SH = SM == 0 ? 64 : 16;
  constexpr int REGION = NG * 8 * 16 * 4 + NG * 4 * 16;   // private LDS bytes per wavefront: fragments of four rows, start values
  extern __shared__ __align__(16) unsigned char smem[];
  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t nwaves = blockDim.x >> 6;
  const uint32_t n = lane & 15u, kq = lane >> 4;
  const uint32_t t0 = wave * TPW;
  const uint32_t t_last = (uint32_t)a.tiles - 1u;   // RAGGED: see rows1_body
  // ---- every request, before anything else ------------------------------------------------------------------
  // unit u = lane + 64 i: bits 0-2 = the fragment's (quarter, k-step), bits 3-4 = activation row, the rest = group;
  // a lane stages the same row in all of its units
  const uint32_t sr = min((lane >> 3) & 3u, (uint32_t)M - 1u);
  const size_t xrow = rows ? (size_t)rows[sr] : (size_t)sr;
  u32x4 xv[NF];
#pragma unroll
  for (int i = 0; i < NF; ++i) {
    const uint32_t u = lane + 64u * i;
    const uint32_t f = (u & 7u) | ((u >> 5) << 3);
    const uint32_t g = min(t0 * 4u + (f >> 3), (uint32_t)a.g_last);
    const uint32_t off = (g << 6) | ((f & 3u) << 4) | ((f & 4u) << 1);
    xv[i] = *reinterpret_cast<const u32x4*>(a.x + xrow * (size_t)ldx + off);
  }
  const uint32_t row = min(rtile * 16u + n, (uint32_t)a.n_last);
  const float al = a.alpha[row];
  const float be_raw = a.beta[row];
  uint32_t ssup = 0;
  if constexpr (SM == 1) ssup = a.scale_super[row];
  u32x4 cw[TPW];
  uint32_t sw[TPW][SM == 0 ? 2 : 1];
  const uint16_t* sb = a.scales + ((size_t)rtile * (uint32_t)a.tiles + t0) * SH;
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    const uint32_t ti = RAGGED ? min(t0 + i, t_last) - t0 : (uint32_t)i;
    if constexpr (SM == 0) {
      const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(sb + ti * 64u + n * 4u));
      sw[i][0] = v.x;
      sw[i][1] = v.y;
    } else {
      sw[i][0] = __builtin_nontemporal_load(sb + ti * 16u + n);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  const uint8_t* cb = a.codes + ((size_t)rtile * (uint32_t)a.tiles + t0) * 1024u;
#pragma unroll
  for (int i = 0; i < TPW; ++i)
    cw[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(cb + (RAGGED ? min(t0 + i, t_last) - t0 : (uint32_t)i) * 1024u + lane * 16u));
  __builtin_amdgcn_sched_barrier(0);
  // ---- stage x: fragment f of row r at [f][r], start values -(128 + zp) sum x at [group][quarter][r] ---------------
  unsigned char* region = smem + (size_t)wave * REGION;
  u32x4* lds_x = reinterpret_cast<u32x4*>(region);
  float* lds_c = reinterpret_cast<float*>(region + NG * 8 * 16 * 4);
#pragma unroll
  for (int i = 0; i < NF; ++i) {
    const uint32_t u = lane + 64u * i;
    const uint32_t f = (u & 7u) | ((u >> 5) << 3), r = (u >> 3) & 3u;
    u32x4 o;
    o.x = __builtin_amdgcn_perm(xv[i].z, xv[i].x, 0x05040100u);
    o.y = __builtin_amdgcn_perm(xv[i].z, xv[i].x, 0x07060302u);
    o.z = __builtin_amdgcn_perm(xv[i].w, xv[i].y, 0x05040100u);
    o.w = __builtin_amdgcn_perm(xv[i].w, xv[i].y, 0x07060302u);
    const float s = group_sum8(frag_sum(o));   // the eight fragments of a (group, row) sit in eight neighbouring lanes
    lds_x[f * 4u + r] = o;
    if ((f & 7u) == 0) lds_c[(f >> 3) * 4u + r] = a.cneg * s;
  }
  __builtin_amdgcn_wave_barrier();
  uint32_t c4300 = 0x43004300u, mask = 0x003F003Fu;
  float magic = 8388608.f;
  asm volatile("" : "+v"(c4300), "+s"(mask), "+v"(magic));   // register values, not literals: v_and_or_b32 gets selected
  const float be = be_raw + magic;   // + 2^23: exact, beta is an integer below 2^15

  // ---- contraction ------------------------------------------------------------------------------------------------
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  const uint32_t mr = lane & 3u;   // the activation row this lane supplies: rows 4, 5, ... of the 16-row operand repeat rows 0-3
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    if (RAGGED && t0 + i > t_last) break;   // uniform over the wavefront
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int lg = i * 4 + j;
      const u32x4 x0 = lds_x[((lg * 2 + 0) * 4 + kq) * 4u + mr];
      const u32x4 x1 = lds_x[((lg * 2 + 1) * 4 + kq) * 4u + mr];
      f32x4 p = *reinterpret_cast<const f32x4*>(lds_c + lg * 4);
      u32x4 w[2];
      const uint32_t d = j == 0 ? cw[i].x : (j == 1 ? cw[i].y : (j == 2 ? cw[i].z : cw[i].w));
      decode_dword(d, al, be, c4300, mask, w);
      p = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x0), __builtin_bit_cast(bf16x8, w[0]), p, 0, 0, 0);
      p = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x1), __builtin_bit_cast(bf16x8, w[1]), p, 0, 0, 0);
      float s;
      if constexpr (SM == 0) {
        const uint32_t sd = sw[i][j >> 1];
        s = (float)__builtin_bit_cast(_Float16, (uint16_t)((j & 1) ? (sd >> 16) : (sd & 0xFFFFu)));
      } else {
        s = (float)((sw[i][0] >> (4 * j)) & 0xFu);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[r] = __builtin_fmaf(s, p[r], acc[r]);
    }
  }
  // ---- the wavefronts of the workgroup (fixed order); the matrix core has added the four quarters of a row ---------
  if (nwaves > 1) {
    __syncthreads();
    f32x4* red = reinterpret_cast<f32x4*>(smem);
    if (wave > 0 && lane < 16u) red[(wave - 1) * 16u + lane] = acc;
    __syncthreads();
    if (wave == 0 && lane < 16u) {
      for (uint32_t k = 1; k < nwaves; ++k) acc += red[(k - 1) * 16u + lane];
    }
  }
  if (wave == 0 && lane < 16u && rtile * 16u + lane <= (uint32_t)a.n_last) {
    if constexpr (SM == 1) acc *= (float)__builtin_bit_cast(_Float16, (uint16_t)ssup);
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (r < M) a.y[(size_t)r * (size_t)ldy + rtile * 16u + lane] = to_bf16_rne(acc[r]);
  }
}

template <int TPW, int SM>
__global__ void __launch_bounds__(1024) kernel4(const Args4 aa) {
  rows4_body<TPW, SM, false>(aa.a, aa.ldx, aa.ldy, aa.M, nullptr, blockIdx.x);
}
template <int TPW, int SM>
__global__ void __launch_bounds__(1024) kernel4_unequal(const Args4 aa) {
  rows4_body<TPW, SM, true>(aa.a, aa.ldx, aa.ldy, aa.M, nullptr, blockIdx.x);
}

// ---- grouped product with at most four rows per expert (one or a few tokens' decode step of a mixture of experts:
// the Grouped-GEMM operator of Table 5 with M = 1 and 4) ----------------------------------------------------------------
// Every expert that has rows is a GEMV (or a four-row product) of its own: blockIdx.y picks the expert (from the list
// of experts that have rows, when the host knows it; otherwise every expert, and those without rows leave at once),
// blockIdx.x its row tile; the expert's rows of x are gathered through sorted_rows and its results are rows
// offsets[e] .. offsets[e + 1] - 1 of y.
struct ArgsG {
  Args a;                        // expert 0's arrays; x and y of the whole call
  int64_t ldx, ldy;
  int64_t codes_stride, scales_stride, ab_stride;   // bytes from one expert's arrays to the next (scale_super: ab_stride / 2)
  const int32_t* sorted_rows;
  const int32_t* offsets;
  int32_t n_active;              // > 0: gridDim.y experts are listed in active_ids
  uint16_t active_ids[kMaxActiveList];
};

template <int TPW, int SM, bool FOUR>
__global__ void __launch_bounds__(1024) kernel_grouped(const ArgsG g) {
  uint32_t e = blockIdx.y;
  if (g.n_active > 0) {
    // read straight from the argument segment (a uniform scalar load): indexing the by-value copy with a run-time
    // index would make the compiler keep the whole argument block in scratch memory
    typedef const __attribute__((address_space(4))) uint16_t* KernargU16;
    typedef const __attribute__((address_space(4))) char* KernargBytes;
    KernargBytes args = (KernargBytes)__builtin_amdgcn_kernarg_segment_ptr();
    e = ((KernargU16)(args + offsetof(ArgsG, active_ids)))[blockIdx.y];
  }
  const int32_t p0 = g.offsets[e], Me = g.offsets[e + 1] - p0;
  if (Me <= 0) return;
  Args a = g.a;
  a.codes += (size_t)e * (size_t)g.codes_stride;
  a.scales = reinterpret_cast<const uint16_t*>(reinterpret_cast<const uint8_t*>(a.scales) + (size_t)e * (size_t)g.scales_stride);
  a.alpha = reinterpret_cast<const float*>(reinterpret_cast<const uint8_t*>(a.alpha) + (size_t)e * (size_t)g.ab_stride);
  a.beta = reinterpret_cast<const float*>(reinterpret_cast<const uint8_t*>(a.beta) + (size_t)e * (size_t)g.ab_stride);
  if constexpr (SM == 1)
    a.scale_super = reinterpret_cast<const uint16_t*>(reinterpret_cast<const uint8_t*>(a.scale_super) + (size_t)e * (size_t)(g.ab_stride / 2));
  a.y += (size_t)p0 * (size_t)g.ldy;
  if (FOUR && Me > 1) {   // uniform over the workgroup; an expert with a single row takes the one-row path below
    rows4_body<TPW, SM>(a, g.ldx, g.ldy, min(Me, 4), g.sorted_rows + p0, blockIdx.x);
  } else {
    a.x += (size_t)g.sorted_rows[p0] * (size_t)g.ldx;
    rows1_body<1, TPW, SM>(a, blockIdx.x);
  }
}

// ---- one activation row on wide-format and mixed-format weights ----------------------------------------------------
// The same kernel shape for the (L=4,N=3,S=2) code of Table 1 (Alg. 2) and for a per-group mix of the two formats
// (Sec. 3.3, "Hybrid Bits Mix"): a workgroup owns one row tile and all of K; its first WN wavefronts take shares of
// TPWN narrow k-tiles each, the other WW shares of TPWW wide k-tiles (8 groups of 64 weights, 2816 bytes: three
// 16-byte segments per lane).  With a mix the original group of a packed group (the activation columns to read) comes
// from the group map, which costs one more dependent request at the start.
//   wide decode: lane (row n, quarter kq) holds bytes 6 kq + 2 t, 6 kq + 2 t + 1 of the group in segment t = 0, 1, 2:
//   two 8-bit codes, each three 4-bit states at the shifts [4, 2, 0] with mask 0xF (Table 1); both codes go into one
//   register {0, b, 0, a} and one shift + one and-or cut the same window out of both: bf16 integers 128 + state in
//   k-slots {0,3}, {1,4}, {2,5} of k-step t; slots 6 and 7 are unused and meet zero activations.  Quarter 3 owns
//   bytes 18..21 only: its k-step 1 holds weights {60, 63, 61, -, 62, -} and its k-step 2 nothing (zero activations).
//   With compressed scales (Sec. 3.4) the 4-bit field of a wide group is the low nibble of its byte 21, which the
//   quarter-3 lane of the row holds in segment 1: the other lanes of the row fetch it with ds_bpermute.
struct ArgsNW {
  const uint8_t* codes;
  const uint16_t* scales;
  const float* alpha;
  const float* beta;
  const uint16_t* x;
  uint16_t* y;
  const uint16_t* scale_super;   // fp16 [N], compressed scales only
  const int32_t* meta;           // original group of every packed group (narrow first), or NULL: a single format
  int64_t row_tile_bytes, row_tile_scale_halfs;
  int32_t tiles_n, tiles_w;      // k-tiles per row tile of each format
  int32_t waves_n;               // wavefronts with narrow shares (the first ones)
  int32_t meta_wide;             // entries of the group map that precede the wide groups (narrow groups in whole k-tiles)
  float cneg_n, cneg_w;          // -(128 + zp) per format
  int32_t g_last, n_last;        // last real group of K, last real output row (see Args)
};

__device__ __forceinline__ u32x4 load_chunk16(const uint16_t* p) {   // 16 bytes at 4-byte alignment
  struct __attribute__((packed, aligned(4))) Chunk16 { uint32_t x, y, z, w; };
  const Chunk16 c = *reinterpret_cast<const Chunk16*>(p);
  return u32x4{c.x, c.y, c.z, c.w};
}
// Activation fragment of (quarter kq, k-step t) of a wide group from the 16-byte chunk that starts at element
// min(18 kq + 6 t, 56): k-slots {0, 3, 1, 4, 2, 5, -, -}.
__device__ __forceinline__ u32x4 wide_frag(const u32x4 v, uint32_t kq, int t) {
  u32x4 o = {0u, 0u, 0u, 0u};
  if (kq < 3u || t == 0) {
    o.x = __builtin_amdgcn_perm(v.y, v.x, 0x07060100u);  // elements 0, 3
    o.y = __builtin_amdgcn_perm(v.z, v.x, 0x05040302u);  // 1, 4
    o.z = __builtin_amdgcn_perm(v.z, v.y, 0x07060100u);  // 2, 5
  } else if (t == 1) {                                    // the chunk starts at 56: weights 60, 63 | 61 | 62
    o.x = __builtin_amdgcn_perm(v.w, v.z, 0x07060100u);
    o.y = v.z >> 16;
    o.z = v.w & 0xFFFFu;
  }
  return o;
}

// The same for the hybrid 16-bit word of Sec. 3.2 (which takes the wide kind's place: 8 groups per k-tile, three k-steps
// per group): word 4 t + kq of the group holds weights 7 word .. 7 word + 6 (word 9: weight 63 only), the chunk starts at
// element min(7 word & ~1, 56), k-slots {0, 1, 3, 4, 5, 6, 2, -} (the order in which the decode pairs the states).
__device__ __forceinline__ u32x4 h16_frag(const u32x4 v, uint32_t kq, int t) {
  u32x4 o = {0u, 0u, 0u, 0u};
  const uint32_t word = 4u * t + kq;
  if (word == 9u) {
    o.x = v.w >> 16;                                       // element 63 of the chunk that starts at 56
  } else if (word < 9u) {
    if (word & 1u) {                                       // the word starts at the chunk's second element
      o.x = __builtin_amdgcn_perm(v.y, v.x, 0x05040302u);  // elements 1, 2
      o.y = v.z;                                            // 4, 5
      o.z = v.w;                                            // 6, 7
      o.w = v.y >> 16;                                      // 3
    } else {
      o.x = v.x;                                            // 0, 1
      o.y = __builtin_amdgcn_perm(v.z, v.y, 0x05040302u);  // 3, 4
      o.z = __builtin_amdgcn_perm(v.w, v.z, 0x05040302u);  // 5, 6
      o.w = v.y & 0xFFFFu;                                  // 2
    }
  }
  return o;
}
// First element of the 16-byte chunk that holds the activations of (quarter kq, k-step t) of a group.
template <bool H16>
__device__ __forceinline__ uint32_t chunk_first(uint32_t kq, int t) {
  if constexpr (H16) return min((7u * (4u * t + kq)) & ~1u, 56u);
  else return min(18u * kq + 6u * t, 56u);
}
template <bool H16>
__device__ __forceinline__ u32x4 kind_frag(const u32x4 v, uint32_t kq, int t) {
  if constexpr (H16) return h16_frag(v, kq, t);
  else return wide_frag(v, kq, t);
}
// Weight fragment (k-step t of group j of a k-tile held in `seg`): 8 bf16 integers 128 + state.
//   wide: two 8-bit codes {0, b, 0, a}, windows [4, 2, 0] with mask 0xF of both at once, slots 6 and 7 unused;
//   hybrid word w = (3,3,2) code | (3,4,2) code: seven 3-bit states at the shifts [13, 11, 9, 6, 4, 2, 0], mask 0x7
//   (Table 1).  v = w | w << 18 puts a second copy of the word 18 bits up, so that the state at shift s - 2 of the copy
//   lands 16 bits above the state at shift s: one shift and one and-or cut out two states.
template <bool H16>
__device__ __forceinline__ u32x4 kind_weights(const u32x4 seg, int j, uint32_t mask, uint32_t c4300) {
  const uint32_t d = (j >> 1) == 0 ? seg.x : ((j >> 1) == 1 ? seg.y : ((j >> 1) == 2 ? seg.z : seg.w));
  u32x4 wv;
  if constexpr (H16) {
    const uint32_t w = (j & 1) ? (d >> 16) : (d & 0xFFFFu);
    const uint32_t v = w | (w << 18);
    wv.x = and_or(v >> 13, mask, c4300);  // states 0, 1
    wv.y = and_or(v >> 6, mask, c4300);   // states 3, 4
    wv.z = and_or(v >> 2, mask, c4300);   // states 5, 6
    wv.w = and_or(v >> 9, mask, c4300);   // state 2; the upper half is an unused k-slot (zero activation)
  } else {
    const uint32_t pp = __builtin_amdgcn_perm(0u, d, (j & 1) ? 0x0C030C02u : 0x0C010C00u);  // {0, b, 0, a}
    wv.x = and_or(pp >> 4, mask, c4300);
    wv.y = and_or(pp >> 2, mask, c4300);
    wv.z = and_or(pp, mask, c4300);
    wv.w = pp;                            // unused k-slots (zero activations): any finite value; pp's halves are bf16 numbers below 2^-126, and it is already in a register
  }
  return wv;
}

template <int TPWN, int TPWW, int SM, bool H16>
__device__ __forceinline__ void rows1_nw_body(const ArgsNW& a, const uint32_t rtile) {
  constexpr int NGN = TPWN * 4, NGW = TPWW * 8;                 // groups per narrow / wide share
  constexpr int REGION_N = NGN * 8 * 16 + NGN * 4 * 16;         // private LDS bytes per wavefront: fragments, then start-value records
  constexpr int REGION_W = NGW * 12 * 16 + NGW * 4 * 16;
  extern __shared__ __align__(16) unsigned char smem[];
  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t nwaves = blockDim.x >> 6;
  const uint32_t n = lane & 15u, kq = lane >> 4;
  const uint32_t row = min(rtile * 16u + n, (uint32_t)a.n_last);
  // private regions: the narrow shares' first, then the wide shares'
  const uint32_t wn = TPWN > 0 ? (uint32_t)a.waves_n : 0u;
  unsigned char* region = smem + (wave < wn ? (size_t)wave * REGION_N : (size_t)wn * REGION_N + (size_t)(wave - wn) * REGION_W);
  u32x4* lds_x = reinterpret_cast<u32x4*>(region);
  const uint8_t* code_row = a.codes + (size_t)rtile * (size_t)a.row_tile_bytes;
  const uint16_t* scale_row = a.scales + (size_t)rtile * (size_t)a.row_tile_scale_halfs;
  uint32_t c4300 = 0x43004300u, mask_n = 0x003F003Fu, mask_w = H16 ? 0x00070007u : 0x000F000Fu;
  float magic = 8388608.f;
  asm volatile("" : "+v"(c4300), "+s"(mask_n), "+s"(mask_w), "+v"(magic));   // register values, not literals: v_and_or_b32 gets selected
  uint32_t ssup = 0;
  float acc = 0.f;

  if (TPWN > 0 && wave < wn) {
    // ------------------------------------------------------------------ a share of narrow k-tiles (as in `kernel`)
    constexpr int NF = (NGN * 8 + 63) / 64;
    constexpr int SH = SM == 0 ? 64 : 16;
    const uint32_t t0 = wave * TPWN;
    u32x4 xv[NF > 0 ? NF : 1];
#pragma unroll
    for (int i = 0; i < NF; ++i) {
      uint32_t f = lane + 64u * i;
      if (NGN * 8 % 64 != 0) f = min(f, (uint32_t)(NGN * 8 - 1));
      const uint32_t pg = t0 * 4u + (f >> 3);
      const uint32_t g = a.meta ? (uint32_t)a.meta[pg] : min(pg, (uint32_t)a.g_last);
      const uint32_t off = (g << 6) | ((f & 3u) << 4) | ((f & 4u) << 1);
      xv[i] = *reinterpret_cast<const u32x4*>(a.x + off);
    }
    const float al = a.alpha[row];
    const float be_raw = a.beta[row];
    if constexpr (SM == 1) ssup = a.scale_super[row];
    u32x4 cw[TPWN > 0 ? TPWN : 1];
    uint32_t sw[TPWN > 0 ? TPWN : 1][SM == 0 ? 2 : 1];
#pragma unroll
    for (int i = 0; i < TPWN; ++i) {
      const uint16_t* sb = scale_row + (size_t)t0 * SH;
      if constexpr (SM == 0) {
        const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(sb + i * 64u + n * 4u));
        sw[i][0] = v.x;
        sw[i][1] = v.y;
      } else {
        sw[i][0] = __builtin_nontemporal_load(sb + i * 16u + n);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < TPWN; ++i) cw[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(code_row + (size_t)(t0 + i) * 1024u + lane * 16u));
    __builtin_amdgcn_sched_barrier(0);
    float* lds_c = reinterpret_cast<float*>(region + NGN * 8 * 16);
#pragma unroll
    for (int i = 0; i < NF; ++i) {
      const uint32_t f = lane + 64u * i;
      u32x4 o;
      o.x = __builtin_amdgcn_perm(xv[i].z, xv[i].x, 0x05040100u);
      o.y = __builtin_amdgcn_perm(xv[i].z, xv[i].x, 0x07060302u);
      o.z = __builtin_amdgcn_perm(xv[i].w, xv[i].y, 0x05040100u);
      o.w = __builtin_amdgcn_perm(xv[i].w, xv[i].y, 0x07060302u);
      const float s = group_sum8(frag_sum(o));
      if (NGN * 8 % 64 == 0 || f < (uint32_t)(NGN * 8)) {
        lds_x[f] = o;
        if ((f & 7u) == 0) {
          const float c = a.cneg_n * s;
          *reinterpret_cast<f32x4*>(lds_c + (f >> 3) * 4u) = f32x4{c, c, c, c};
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
    const float be = be_raw + magic;   // + 2^23: exact, beta is an integer below 2^15
#pragma unroll
    for (int i = 0; i < TPWN; ++i) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int lg = i * 4 + j;
        const u32x4 x0 = lds_x[(lg * 2 + 0) * 4 + kq];
        const u32x4 x1 = lds_x[(lg * 2 + 1) * 4 + kq];
        const f32x4 cin = *reinterpret_cast<const f32x4*>(lds_c + lg * 4);
        u32x4 w[2];
        const uint32_t d = j == 0 ? cw[i].x : (j == 1 ? cw[i].y : (j == 2 ? cw[i].z : cw[i].w));
        decode_dword(d, al, be, c4300, mask_n, w);
        f32x4 p = cin;
        p = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x0), __builtin_bit_cast(bf16x8, w[0]), p, 0, 0, 0);
        p = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x1), __builtin_bit_cast(bf16x8, w[1]), p, 0, 0, 0);
        float s;
        if constexpr (SM == 0) {
          const uint32_t sd = sw[i][j >> 1];
          s = (float)__builtin_bit_cast(_Float16, (uint16_t)((j & 1) ? (sd >> 16) : (sd & 0xFFFFu)));
        } else {
          s = (float)((sw[i][0] >> (4 * j)) & 0xFu);
        }
        acc = __builtin_fmaf(s, p[0], acc);
      }
    }
  } else {
    // ------------------------------------------------------------------ a share of wide k-tiles
    const uint32_t t0 = (wave - wn) * TPWW;
    // x: lane p < 4 NGW stages (group p / 4, quarter p % 4): three chunks of 16 bytes, one per k-step
    const uint32_t sp = min(lane, (uint32_t)(4 * NGW - 1));
    const uint32_t slg = sp >> 2, skq = sp & 3u;
    const uint32_t pg = t0 * 8u + slg;
    const uint32_t g = a.meta ? (uint32_t)a.meta[(uint32_t)a.meta_wide + pg] : min(pg, (uint32_t)a.g_last);
    u32x4 xc[3];
#pragma unroll
    for (int t = 0; t < 3; ++t) xc[t] = load_chunk16(a.x + (g << 6) + chunk_first<H16>(skq, t));
    if constexpr (SM == 1) ssup = a.scale_super[row];
    u32x4 cw[TPWW][3];
    u32x4 sw[TPWW];
    const uint16_t* sb = scale_row + (size_t)a.tiles_n * 64u + (size_t)t0 * 128u;   // fp16 scales only: [narrow tiles][wide tiles]
#pragma unroll
    for (int i = 0; i < TPWW; ++i) {
      if constexpr (SM == 0) sw[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(sb + i * 128u + n * 8u));
      else sw[i] = u32x4{0u, 0u, 0u, 0u};
    }
    __builtin_amdgcn_sched_barrier(0);
    constexpr uint32_t kTile = H16 ? 2560u : 2816u, kLast = H16 ? 31u : 47u;
    const uint8_t* cb = code_row + (size_t)a.tiles_n * 1024u + (size_t)t0 * kTile;
#pragma unroll
    for (int i = 0; i < TPWW; ++i) {
      const uint8_t* t = cb + i * kTile + lane * 16u;
      cw[i][0] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t));
      cw[i][1] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t + 1024));
      // the third segment has entries for 48 lanes only (32 for the hybrid word); the lanes above re-read the last entry
      // (their k-slots meet zero activations, and every bit pattern decodes to a finite value)
      cw[i][2] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t + 2048 - (lane > kLast ? (lane - kLast) * 16u : 0u)));
    }
    __builtin_amdgcn_sched_barrier(0);
    float* lds_c = reinterpret_cast<float*>(region + NGW * 12 * 16);
    {
      float sum = 0.f;
      u32x4 o[3];
#pragma unroll
      for (int t = 0; t < 3; ++t) {
        o[t] = kind_frag<H16>(xc[t], skq, t);
        sum += frag_sum(o[t]);
      }
      // the four quarters of a group: neighbouring lanes
      sum += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, sum), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
      sum += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, sum), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
      if (lane < (uint32_t)(4 * NGW)) {
#pragma unroll
        for (int t = 0; t < 3; ++t) lds_x[(slg * 3u + t) * 4u + skq] = o[t];
        if (skq == 0) {
          const float c = a.cneg_w * sum;
          *reinterpret_cast<f32x4*>(lds_c + slg * 4u) = f32x4{c, c, c, c};
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < TPWW; ++i) {
      uint32_t fields[4] = {0u, 0u, 0u, 0u};
      if constexpr (SM == 1) {
        // wide: byte 21 of the group, held by the row's quarter-3 lane in segment 1; hybrid word: word 9 of the group
        // (scale mask 0x1FFF of Table 1), held by the row's quarter-1 lane in segment 2
        const int src = (int)(((H16 ? 16u : 48u) + n) * 4u);
        const u32x4 held = cw[i][H16 ? 2 : 1];
        fields[0] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)held.x);
        fields[1] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)held.y);
        fields[2] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)held.z);
        fields[3] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)held.w);
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int lg = i * 8 + j;
        f32x4 p = *reinterpret_cast<const f32x4*>(lds_c + lg * 4);
#pragma unroll
        for (int t = 0; t < 3; ++t) {
          const u32x4 xf = lds_x[(lg * 3 + t) * 4 + kq];
          const u32x4 wv = kind_weights<H16>(cw[i][t], j, mask_w, c4300);
          p = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xf), __builtin_bit_cast(bf16x8, wv), p, 0, 0, 0);
        }
        float s;
        if constexpr (SM == 0) {
          const uint32_t sd = (j >> 1) == 0 ? sw[i].x : ((j >> 1) == 1 ? sw[i].y : ((j >> 1) == 2 ? sw[i].z : sw[i].w));
          s = (float)__builtin_bit_cast(_Float16, (uint16_t)((j & 1) ? (sd >> 16) : (sd & 0xFFFFu)));
        } else if constexpr (H16) {
          s = (float)((fields[j >> 1] >> (16 * (j & 1))) & 0x1FFFu);    // the field alone; the row's super scale multiplies the sum once
        } else {
          s = (float)((fields[j >> 1] >> (16 * (j & 1) + 8)) & 0xFu);
        }
        acc = __builtin_fmaf(s, p[0], acc);
      }
    }
  }
  // ---- the wavefronts of the workgroup (fixed order); the matrix core has added the four quarters of a row ---------
  if (nwaves > 1) {
    __syncthreads();
    float* red = reinterpret_cast<float*>(smem);
    if (wave > 0 && lane < 16u) red[(wave - 1) * 16u + lane] = acc;
    __syncthreads();
    if (wave == 0 && lane < 16u) {
      for (uint32_t k = 1; k < nwaves; ++k) acc += red[(k - 1) * 16u + lane];
    }
  }
  if (wave == 0 && lane < 16u) {
    float v = acc;
    if constexpr (SM == 1) v *= (float)__builtin_bit_cast(_Float16, (uint16_t)ssup);
    if (rtile * 16u + lane <= (uint32_t)a.n_last) a.y[rtile * 16u + lane] = to_bf16_rne(v);
  }
}

template <int TPWN, int TPWW, int SM, bool H16 = false>
__global__ void __launch_bounds__(1024) kernel_nw(const ArgsNW a) {
  rows1_nw_body<TPWN, TPWW, SM, H16>(a, blockIdx.x);
}

// The grouped product with at most one row per expert on these formats: one such GEMV per expert that has a row (see
// kernel_grouped).  The group map is the same for all experts.
struct ArgsNWG {
  ArgsNW a;                      // expert 0's arrays; x and y of the whole call
  int64_t ldx, ldy;
  int64_t codes_stride, scales_stride, ab_stride;
  const int32_t* sorted_rows;
  const int32_t* offsets;
  int32_t n_active;
  uint16_t active_ids[kMaxActiveList];
};

template <int TPWN, int TPWW, int SM, bool H16 = false>
__global__ void __launch_bounds__(1024) kernel_nw_grouped(const ArgsNWG g) {
  uint32_t e = blockIdx.y;
  if (g.n_active > 0) {
    typedef const __attribute__((address_space(4))) uint16_t* KernargU16;
    typedef const __attribute__((address_space(4))) char* KernargBytes;
    KernargBytes args = (KernargBytes)__builtin_amdgcn_kernarg_segment_ptr();
    e = ((KernargU16)(args + offsetof(ArgsNWG, active_ids)))[blockIdx.y];
  }
  const int32_t p0 = g.offsets[e];
  if (g.offsets[e + 1] <= p0) return;
  ArgsNW a = g.a;
  a.codes += (size_t)e * (size_t)g.codes_stride;
  a.scales = reinterpret_cast<const uint16_t*>(reinterpret_cast<const uint8_t*>(a.scales) + (size_t)e * (size_t)g.scales_stride);
  if constexpr (TPWN > 0) {
    a.alpha = reinterpret_cast<const float*>(reinterpret_cast<const uint8_t*>(a.alpha) + (size_t)e * (size_t)g.ab_stride);
    a.beta = reinterpret_cast<const float*>(reinterpret_cast<const uint8_t*>(a.beta) + (size_t)e * (size_t)g.ab_stride);
  }
  if constexpr (SM == 1)
    a.scale_super = reinterpret_cast<const uint16_t*>(reinterpret_cast<const uint8_t*>(a.scale_super) + (size_t)e * (size_t)(g.ab_stride / 2));
  a.x += (size_t)g.sorted_rows[p0] * (size_t)g.ldx;
  a.y += (size_t)p0 * (size_t)g.ldy;
  rows1_nw_body<TPWN, TPWW, SM, H16>(a, blockIdx.x);
}

// ---- two to sixteen activation rows --------------------------------------------------------------------------------
// Same decode, MFMA 16x16x32 bf16 in place of 4x4x4: lane l owns output row n = l % 16 of its row tile and quarter
// kq = l / 16 of every group (the B operand), the activations are the A operand (row m = l % 16, k-slots of quarter
// kq), and the lane receives rows m = 4 kq .. 4 kq + 3 of column n.  The activation fragments of 16 rows are sixteen
// times those of one row, so they are staged once per workgroup and shared by its NW wavefronts = NW row tiles; K is
// cut into shares of TPW k-tiles across workgroups (gridDim.y), whose fp32 partial tiles are added in index
// order by a second, small kernel (a share that covers all of K writes bf16 results directly).  Letting the share that
// arrives last at a row block add the tiles inside this kernel was measured and is slower on this chip: the shares run
// on different XCDs, whose L2 caches are not coherent with each other, so the partial tiles, the arrival counter and the
// final reads each make a round trip to memory (three dependent ones, 6-8 us at 8192 x 8192 against 3.9 us for the
// second launch).  One workgroup barrier in the whole kernel.
struct Args16 {
  const uint8_t* codes;
  const uint16_t* scales;
  const float* alpha;
  const float* beta;
  const uint16_t* x;
  uint16_t* y;
  const uint16_t* scale_super;
  float* partial;                // fp32 [shares][M][N] when K is cut
  int64_t ldx, ldy;
  int32_t tiles, row_tiles, M, N;   // N: rows of the device layout (a multiple of 16), the stride of the partial tiles
  float cneg;
  int32_t g_last, n_last;           // last real group of K, last real output row (see Args)
};

template <int TPW, int SM, int NW, int MT, bool RAGGED>
__device__ __forceinline__ void rows16_body(const Args16& a) {
  constexpr int MR = 16 * MT;                  // activation rows held: MT tiles of 16 (MT = 2 serves 17..32 rows)
  constexpr int NG = TPW * 4;                  // groups per share
  constexpr int NU = NG * 4 * MR;              // staging units: (group, row, quarter) = 16 consecutive activations
  constexpr int SH = SM == 0 ? 64 : 16;
  extern __shared__ __align__(16) unsigned char smem[];
  u32x4* lds_x = reinterpret_cast<u32x4*>(smem);                       // [group][k-step][quarter][row]
  float* lds_c = reinterpret_cast<float*>(smem + (size_t)NG * 8 * 16 * MR);  // [group][row]
  constexpr uint32_t nthreads = 64u * NW;
  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t n = lane & 15u, kq = lane >> 4;
  const uint32_t t0 = blockIdx.y * TPW;
  const uint32_t t_last = (uint32_t)a.tiles - 1u;   // RAGGED: the last share is shorter; its requests past this tile re-read it
  const uint32_t rtile_raw = blockIdx.x * NW + wave;
  const bool active = rtile_raw < (uint32_t)a.row_tiles;
  const uint32_t rtile = active ? rtile_raw : (uint32_t)a.row_tiles - 1u;   // a ragged last block re-reads the last tile; nothing of it is stored

  // ---- every request, before anything else --------------------------------------------------------------------
  // unit u = (group * 16 + row) * 4 + quarter: the quarters of a (group, row) sit in neighbouring lanes
  constexpr int NUT = (NU + (int)nthreads - 1) / (int)nthreads;   // units per thread
  // (two 16-row tiles: the units go in two rounds through the same registers; the second round's requests wait behind
  // the code tiles', which take longer than anything here)
  constexpr int NUA = MT == 1 ? NUT : (NUT + 1) / 2;                // units per thread and round
  u32x4 xv[NUA][2];
  auto request = [&](int i0) {
#pragma unroll
    for (int i = 0; i < NUA; ++i) {
      uint32_t u = tid + (uint32_t)(i0 + i) * nthreads;
      if (NU % nthreads != 0 || NUT % NUA != 0) u = min(u, (uint32_t)NU - 1u);   // clamped: the request is unconditional
      const uint32_t q = u & 3u, m = (u >> 2) & (uint32_t)(MR - 1), lg = u / (uint32_t)(4 * MR);
      const uint32_t row = min(m, (uint32_t)a.M - 1u);                  // rows past M repeat the last one; never stored
      const uint16_t* p = a.x + (size_t)row * (size_t)a.ldx + ((size_t)min(t0 * 4u + lg, (uint32_t)a.g_last) * 64u + q * 16u);
      xv[i][0] = *reinterpret_cast<const u32x4*>(p);
      xv[i][1] = *reinterpret_cast<const u32x4*>(p + 8);
    }
  };
  request(0);
  const uint32_t prow = min(rtile * 16u + n, (uint32_t)a.n_last);
  const float al = a.alpha[prow];
  const float be_raw = a.beta[prow];
  uint32_t ssup = 0;
  if constexpr (SM == 1) ssup = a.scale_super[prow];
  u32x4 cw[TPW];
  uint32_t sw[TPW][SM == 0 ? 2 : 1];
  const uint16_t* sb = a.scales + ((size_t)rtile * (uint32_t)a.tiles + t0) * SH;
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    const uint32_t ti = RAGGED ? min(t0 + i, t_last) - t0 : (uint32_t)i;
    if constexpr (SM == 0) {
      const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(sb + ti * 64u + n * 4u));
      sw[i][0] = v.x;
      sw[i][1] = v.y;
    } else {
      sw[i][0] = __builtin_nontemporal_load(sb + ti * 16u + n);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  const uint8_t* cb = a.codes + ((size_t)rtile * (uint32_t)a.tiles + t0) * 1024u;
#pragma unroll
  for (int i = 0; i < TPW; ++i)
    cw[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(cb + (RAGGED ? min(t0 + i, t_last) - t0 : (uint32_t)i) * 1024u + lane * 16u));
  __builtin_amdgcn_sched_barrier(0);

  // ---- stage the activations: fragments in k-slot order {0,4,1,5,2,6,3,7} and the start values ----------------------
  auto finish = [&](int i0) {
#pragma unroll
    for (int i = 0; i < NUA; ++i) {
      const uint32_t u = tid + (uint32_t)(i0 + i) * nthreads;
      float s = 0.f;
      u32x4 o[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        o[t].x = __builtin_amdgcn_perm(xv[i][t].z, xv[i][t].x, 0x05040100u);
        o[t].y = __builtin_amdgcn_perm(xv[i][t].z, xv[i][t].x, 0x07060302u);
        o[t].z = __builtin_amdgcn_perm(xv[i][t].w, xv[i][t].y, 0x05040100u);
        o[t].w = __builtin_amdgcn_perm(xv[i][t].w, xv[i][t].y, 0x07060302u);
        s += frag_sum(o[t]);
      }
      // the four quarters of a (group, row): neighbouring lanes
      s += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, s), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
      s += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, s), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
      if ((NU % nthreads == 0 && NUT % NUA == 0) || u < (uint32_t)NU) {
        const uint32_t q = u & 3u, m = (u >> 2) & (uint32_t)(MR - 1), lg = u / (uint32_t)(4 * MR);
        lds_x[((lg * 2u + 0u) * 4u + q) * (uint32_t)MR + m] = o[0];
        lds_x[((lg * 2u + 1u) * 4u + q) * (uint32_t)MR + m] = o[1];
        if (q == 0) lds_c[lg * (uint32_t)MR + m] = a.cneg * s;
      }
    }
  };
  finish(0);
  if constexpr (NUA < NUT) {
    request(NUA);
    finish(NUA);
  }
  __syncthreads();

  uint32_t c4300 = 0x43004300u, mask = 0x003F003Fu;
  float magic = 8388608.f;
  asm volatile("" : "+v"(c4300), "+s"(mask), "+v"(magic));
  const float be = be_raw + magic;   // + 2^23: exact, beta is an integer below 2^15

  // ---- contraction ------------------------------------------------------------------------------------------------
  typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
  f32x4 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    if (RAGGED && t0 + i > t_last) break;   // uniform over the workgroup
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int lg = i * 4 + j;
      u32x4 w[2];
      const uint32_t d = j == 0 ? cw[i].x : (j == 1 ? cw[i].y : (j == 2 ? cw[i].z : cw[i].w));
      decode_dword(d, al, be, c4300, mask, w);
      float sc;
      if constexpr (SM == 0) {
        const uint32_t sd = sw[i][j >> 1];
        sc = (float)__builtin_bit_cast(_Float16, (uint16_t)((j & 1) ? (sd >> 16) : (sd & 0xFFFFu)));
      } else {
        sc = (float)((sw[i][0] >> (4 * j)) & 0xFu);
      }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const u32x4 x0 = lds_x[((lg * 2 + 0) * 4 + kq) * MR + mt * 16 + n];   // here n is the activation row of this lane's A fragment
        const u32x4 x1 = lds_x[((lg * 2 + 1) * 4 + kq) * MR + mt * 16 + n];
        f32x4 p = *reinterpret_cast<const f32x4*>(lds_c + lg * MR + mt * 16 + 4 * kq);
        p = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x0), __builtin_bit_cast(bf16x8, w[0]), p, 0, 0, 0);
        p = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x1), __builtin_bit_cast(bf16x8, w[1]), p, 0, 0, 0);
        acc[mt][0] = __builtin_fmaf(sc, p[0], acc[mt][0]);
        acc[mt][1] = __builtin_fmaf(sc, p[1], acc[mt][1]);
        acc[mt][2] = __builtin_fmaf(sc, p[2], acc[mt][2]);
        acc[mt][3] = __builtin_fmaf(sc, p[3], acc[mt][3]);
      }
    }
    // two tiles: the sums are pinned after every k-tile.  Left alone the compiler moves all scale multiplies to the end
    // of the kernel (behind the wait for the scale loads) and keeps every group's MFMA result live until then: 128
    // registers for those alone, 160 in all and three wavefronts per SIMD.  Pinned per k-tile: 76 registers; per group:
    // 61, but small calls lose the overlap between groups.  With one tile the same pin costs time (config 2 at
    // M = 8 / 16: 11.3 / 11.7 -> 12.3 / 12.9 us): its 100 registers already let every wavefront of such a call be resident
    if constexpr (MT > 1) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) asm volatile("" : "+v"(acc[mt][0]), "+v"(acc[mt][1]), "+v"(acc[mt][2]), "+v"(acc[mt][3]));
    }
  }
  if constexpr (SM == 1) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] *= (float)__builtin_bit_cast(_Float16, (uint16_t)ssup);
  }

  // ---- store: lane (n, kq) holds rows 4 kq .. 4 kq + 3 of column n (of every 16-row tile) ---------------------------------
  const uint32_t col = rtile * 16u + n;
  if (active && col <= (uint32_t)a.n_last) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const uint32_t m = 16u * mt + 4u * kq + r;
        if (m < (uint32_t)a.M) {
          // (nontemporal: the partial tiles are read once, by another kernel; kept out of the L2 they need no write-back
          // when this kernel ends: config 2 at M = 16 12.9 -> 12.1 us)
          if (gridDim.y > 1) __builtin_nontemporal_store(acc[mt][r], &a.partial[((size_t)blockIdx.y * (uint32_t)a.M + m) * (uint32_t)a.N + col]);
          else a.y[(size_t)m * (size_t)a.ldy + col] = to_bf16_rne(acc[mt][r]);
        }
      }
    }
  }
}

template <int TPW, int SM, int NW>
__global__ void __launch_bounds__(64 * NW) kernel16(const Args16 a) {
  rows16_body<TPW, SM, NW, 1, false>(a);
}
template <int TPW, int SM, int NW>
__global__ void __launch_bounds__(64 * NW) kernel16_unequal(const Args16 a) {   // the last share of K is shorter
  rows16_body<TPW, SM, NW, 1, true>(a);
}
// 17..32 rows: two 16-row tiles of activations per workgroup (twice the LDS, two workgroups of eight wavefronts per CU:
// the register budget of four wavefronts per SIMD)
template <int TPW, int SM, int NW>
__global__ void __launch_bounds__(64 * NW, 4) kernel32(const Args16 a) {
  rows16_body<TPW, SM, NW, 2, false>(a);
}
template <int TPW, int SM, int NW>
__global__ void __launch_bounds__(64 * NW, 4) kernel32_unequal(const Args16 a) {
  rows16_body<TPW, SM, NW, 2, true>(a);
}

// ---- two to sixteen activation rows on wide-format and mixed weights ------------------------------------------------
// kernel16 for the (L=4,N=3,S=2) code and for per-group mixes: a workgroup is NW row tiles that share one staged slice
// of the activations; the K shares (gridDim.y) are narrow shares of TPWN k-tiles first, then wide shares of TPWW k-tiles
// of 8 groups.  A wide group is three MFMA 16x16x32 k-steps of 8 k-slots, 6 of them used (see kernel_nw); its
// activation fragments are cut out of three 16-byte chunks per (group, row, quarter).
struct Args16NW {
  const uint8_t* codes;
  const uint16_t* scales;
  const float* alpha;
  const float* beta;
  const uint16_t* x;
  uint16_t* y;
  const uint16_t* scale_super;
  const int32_t* meta;           // original group of every packed group (narrow first), or NULL: a single format
  float* partial;                // fp32 [shares][M][N] when K is cut
  int64_t ldx, ldy;
  int64_t row_tile_bytes, row_tile_scale_halfs;
  int32_t tiles_n, tiles_w, row_tiles, M, N;   // N: rows of the device layout, the stride of the partial tiles
  int32_t shares_n;              // K shares that are narrow (the first ones)
  int32_t meta_wide;             // entries of the group map that precede the wide groups
  float cneg_n, cneg_w;
  int32_t g_last, n_last;
};

template <int TPWN, int TPWW, int SM, int NW, bool H16 = false>
__global__ void __launch_bounds__(64 * NW) kernel16_nw(const Args16NW a) {
  constexpr int NGN = TPWN * 4, NGW = TPWW * 8;
  extern __shared__ __align__(16) unsigned char smem[];
  u32x4* lds_x = reinterpret_cast<u32x4*>(smem);
  constexpr uint32_t nthreads = 64u * NW;
  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t n = lane & 15u, kq = lane >> 4;
  const uint32_t rtile_raw = blockIdx.x * NW + wave;
  const bool active = rtile_raw < (uint32_t)a.row_tiles;
  const uint32_t rtile = active ? rtile_raw : (uint32_t)a.row_tiles - 1u;   // a ragged last block re-reads the last tile; nothing of it is stored
  const uint32_t prow = min(rtile * 16u + n, (uint32_t)a.n_last);
  const uint8_t* code_row = a.codes + (size_t)rtile * (size_t)a.row_tile_bytes;
  const uint16_t* scale_row = a.scales + (size_t)rtile * (size_t)a.row_tile_scale_halfs;
  uint32_t c4300 = 0x43004300u, mask_n = 0x003F003Fu, mask_w = H16 ? 0x00070007u : 0x000F000Fu;
  float magic = 8388608.f;
  asm volatile("" : "+v"(c4300), "+s"(mask_n), "+s"(mask_w), "+v"(magic));
  typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  uint32_t ssup = 0;
  if constexpr (SM == 1) ssup = a.scale_super[prow];
  const uint32_t sn = TPWN > 0 ? (uint32_t)a.shares_n : 0u;

  if (TPWN > 0 && blockIdx.y < sn) {
    // ------------------------------------------------------------------ a narrow share (as in kernel16)
    constexpr int NU = NGN * 4 * 16;
    constexpr int SH = SM == 0 ? 64 : 16;
    constexpr int NUT = NU > 0 ? (NU + (int)nthreads - 1) / (int)nthreads : 1;
    float* lds_c = reinterpret_cast<float*>(smem + (size_t)NGN * 8 * 16 * 16);
    const uint32_t t0 = blockIdx.y * TPWN;
    u32x4 xv[NUT][2];
#pragma unroll
    for (int i = 0; i < NUT; ++i) {
      uint32_t u = tid + (uint32_t)i * nthreads;
      if (NU % nthreads != 0) u = min(u, (uint32_t)NU - 1u);
      const uint32_t q = u & 3u, m = (u >> 2) & 15u, lg = u >> 6;
      const uint32_t row = min(m, (uint32_t)a.M - 1u);
      const uint32_t pg = t0 * 4u + lg;
      const uint32_t g = a.meta ? (uint32_t)a.meta[pg] : min(pg, (uint32_t)a.g_last);
      const uint16_t* p = a.x + (size_t)row * (size_t)a.ldx + ((size_t)g * 64u + q * 16u);
      xv[i][0] = *reinterpret_cast<const u32x4*>(p);
      xv[i][1] = *reinterpret_cast<const u32x4*>(p + 8);
    }
    const float al = a.alpha[prow];
    const float be_raw = a.beta[prow];
    u32x4 cw[TPWN > 0 ? TPWN : 1];
    uint32_t sw[TPWN > 0 ? TPWN : 1][SM == 0 ? 2 : 1];
    const uint16_t* sb = scale_row + (size_t)t0 * SH;
#pragma unroll
    for (int i = 0; i < TPWN; ++i) {
      if constexpr (SM == 0) {
        const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(sb + i * 64u + n * 4u));
        sw[i][0] = v.x;
        sw[i][1] = v.y;
      } else {
        sw[i][0] = __builtin_nontemporal_load(sb + i * 16u + n);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < TPWN; ++i) cw[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(code_row + (size_t)(t0 + i) * 1024u + lane * 16u));
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < NUT; ++i) {
      const uint32_t u = tid + (uint32_t)i * nthreads;
      float s = 0.f;
      u32x4 o[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        o[t].x = __builtin_amdgcn_perm(xv[i][t].z, xv[i][t].x, 0x05040100u);
        o[t].y = __builtin_amdgcn_perm(xv[i][t].z, xv[i][t].x, 0x07060302u);
        o[t].z = __builtin_amdgcn_perm(xv[i][t].w, xv[i][t].y, 0x05040100u);
        o[t].w = __builtin_amdgcn_perm(xv[i][t].w, xv[i][t].y, 0x07060302u);
        s += frag_sum(o[t]);
      }
      s += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, s), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
      s += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, s), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
      if (NU % nthreads == 0 || u < (uint32_t)NU) {
        const uint32_t q = u & 3u, m = (u >> 2) & 15u, lg = u >> 6;
        lds_x[((lg * 2u + 0u) * 4u + q) * 16u + m] = o[0];
        lds_x[((lg * 2u + 1u) * 4u + q) * 16u + m] = o[1];
        if (q == 0) lds_c[lg * 16u + m] = a.cneg_n * s;
      }
    }
    __syncthreads();
    const float be = be_raw + magic;
#pragma unroll
    for (int i = 0; i < TPWN; ++i) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int lg = i * 4 + j;
        const u32x4 x0 = lds_x[((lg * 2 + 0) * 4 + kq) * 16 + n];
        const u32x4 x1 = lds_x[((lg * 2 + 1) * 4 + kq) * 16 + n];
        f32x4 p = *reinterpret_cast<const f32x4*>(lds_c + lg * 16 + 4 * kq);
        u32x4 w[2];
        const uint32_t d = j == 0 ? cw[i].x : (j == 1 ? cw[i].y : (j == 2 ? cw[i].z : cw[i].w));
        decode_dword(d, al, be, c4300, mask_n, w);
        p = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x0), __builtin_bit_cast(bf16x8, w[0]), p, 0, 0, 0);
        p = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x1), __builtin_bit_cast(bf16x8, w[1]), p, 0, 0, 0);
        float sc;
        if constexpr (SM == 0) {
          const uint32_t sd = sw[i][j >> 1];
          sc = (float)__builtin_bit_cast(_Float16, (uint16_t)((j & 1) ? (sd >> 16) : (sd & 0xFFFFu)));
        } else {
          sc = (float)((sw[i][0] >> (4 * j)) & 0xFu);
        }
        acc[0] = __builtin_fmaf(sc, p[0], acc[0]);
        acc[1] = __builtin_fmaf(sc, p[1], acc[1]);
        acc[2] = __builtin_fmaf(sc, p[2], acc[2]);
        acc[3] = __builtin_fmaf(sc, p[3], acc[3]);
      }
    }
  } else {
    // ------------------------------------------------------------------ a wide share
    constexpr int NU = NGW * 4 * 16;                                   // staging units: (group, row, quarter)
    constexpr int NUT = (NU + (int)nthreads - 1) / (int)nthreads;
    float* lds_c = reinterpret_cast<float*>(smem + (size_t)NGW * 12 * 16 * 16);   // [group][row]
    const uint32_t t0 = (blockIdx.y - sn) * TPWW;
    u32x4 xv[NUT][3];
#pragma unroll
    for (int i = 0; i < NUT; ++i) {
      uint32_t u = tid + (uint32_t)i * nthreads;
      if (NU % nthreads != 0) u = min(u, (uint32_t)NU - 1u);
      const uint32_t q = u & 3u, m = (u >> 2) & 15u, lg = u >> 6;
      const uint32_t row = min(m, (uint32_t)a.M - 1u);
      const uint32_t pg = t0 * 8u + lg;
      const uint32_t g = a.meta ? (uint32_t)a.meta[(uint32_t)a.meta_wide + pg] : min(pg, (uint32_t)a.g_last);
      const uint16_t* p = a.x + (size_t)row * (size_t)a.ldx + (size_t)g * 64u;
#pragma unroll
      for (int t = 0; t < 3; ++t) xv[i][t] = load_chunk16(p + chunk_first<H16>(q, t));
    }
    u32x4 cw[TPWW][3];
    u32x4 sw[TPWW];
    const uint16_t* sb = scale_row + (size_t)a.tiles_n * 64u + (size_t)t0 * 128u;   // fp16 scales only
#pragma unroll
    for (int i = 0; i < TPWW; ++i) {
      if constexpr (SM == 0) sw[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(sb + i * 128u + n * 8u));
      else sw[i] = u32x4{0u, 0u, 0u, 0u};
    }
    __builtin_amdgcn_sched_barrier(0);
    constexpr uint32_t kTile = H16 ? 2560u : 2816u, kLast = H16 ? 31u : 47u;
    const uint8_t* cb = code_row + (size_t)a.tiles_n * 1024u + (size_t)t0 * kTile;
#pragma unroll
    for (int i = 0; i < TPWW; ++i) {
      const uint8_t* t = cb + i * kTile + lane * 16u;
      cw[i][0] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t));
      cw[i][1] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t + 1024));
      cw[i][2] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t + 2048 - (lane > kLast ? (lane - kLast) * 16u : 0u)));
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < NUT; ++i) {
      const uint32_t u = tid + (uint32_t)i * nthreads;
      const uint32_t uq = min(u, (uint32_t)NU - 1u) & 3u;
      float s = 0.f;
      u32x4 o[3];
#pragma unroll
      for (int t = 0; t < 3; ++t) {
        o[t] = kind_frag<H16>(xv[i][t], uq, t);
        s += frag_sum(o[t]);
      }
      s += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, s), 0xB1, 0xF, 0xF, true));   // the four quarters of a (group, row): neighbouring lanes
      s += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, s), 0x4E, 0xF, 0xF, true));
      if (NU % nthreads == 0 || u < (uint32_t)NU) {
        const uint32_t q = u & 3u, m = (u >> 2) & 15u, lg = u >> 6;
#pragma unroll
        for (int t = 0; t < 3; ++t) lds_x[((lg * 3u + t) * 4u + q) * 16u + m] = o[t];
        if (q == 0) lds_c[lg * 16u + m] = a.cneg_w * s;
      }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < TPWW; ++i) {
      uint32_t fields[4] = {0u, 0u, 0u, 0u};
      if constexpr (SM == 1) {
        const int src = (int)(((H16 ? 16u : 48u) + n) * 4u);
        const u32x4 held = cw[i][H16 ? 2 : 1];
        fields[0] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)held.x);
        fields[1] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)held.y);
        fields[2] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)held.z);
        fields[3] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)held.w);
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int lg = i * 8 + j;
        f32x4 p = *reinterpret_cast<const f32x4*>(lds_c + lg * 16 + 4 * kq);
#pragma unroll
        for (int t = 0; t < 3; ++t) {
          const u32x4 xf = lds_x[((lg * 3 + t) * 4 + kq) * 16 + n];     // here n is the activation row of this lane's A fragment
          const u32x4 wv = kind_weights<H16>(cw[i][t], j, mask_w, c4300);
          p = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xf), __builtin_bit_cast(bf16x8, wv), p, 0, 0, 0);
        }
        float sc;
        if constexpr (SM == 0) {
          const uint32_t sd = (j >> 1) == 0 ? sw[i].x : ((j >> 1) == 1 ? sw[i].y : ((j >> 1) == 2 ? sw[i].z : sw[i].w));
          sc = (float)__builtin_bit_cast(_Float16, (uint16_t)((j & 1) ? (sd >> 16) : (sd & 0xFFFFu)));
        } else if constexpr (H16) {
          sc = (float)((fields[j >> 1] >> (16 * (j & 1))) & 0x1FFFu);
        } else {
          sc = (float)((fields[j >> 1] >> (16 * (j & 1) + 8)) & 0xFu);
        }
        acc[0] = __builtin_fmaf(sc, p[0], acc[0]);
        acc[1] = __builtin_fmaf(sc, p[1], acc[1]);
        acc[2] = __builtin_fmaf(sc, p[2], acc[2]);
        acc[3] = __builtin_fmaf(sc, p[3], acc[3]);
      }
      // shares of two k-tiles: the sums are pinned after each (see rows16_body; 106 -> 74 registers, four -> six wavefronts
      // per SIMD: all-wide 8192 x 28672 at M = 2 / 8 / 16 30.2 / 32.1 / 35.4 -> 27.7 / 30.0 / 32.2 us, smaller calls unchanged)
      if constexpr (TPWW > 1) asm volatile("" : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]));
    }
  }
  if constexpr (SM == 1) acc *= (float)__builtin_bit_cast(_Float16, (uint16_t)ssup);

  // ---- store: lane (n, kq) holds rows 4 kq .. 4 kq + 3 of column n -------------------------------------------------------
  const uint32_t col = rtile * 16u + n;
  if (active && col <= (uint32_t)a.n_last) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const uint32_t m = 4u * kq + r;
      if (m < (uint32_t)a.M) {
        if (gridDim.y > 1) __builtin_nontemporal_store(acc[r], &a.partial[((size_t)blockIdx.y * (uint32_t)a.M + m) * (uint32_t)a.N + col]);
        else a.y[(size_t)m * (size_t)a.ldy + col] = to_bf16_rne(acc[r]);
      }
    }
  }
}

typedef void (*Kernel)(const Args);

template <int SM, bool RAGGED>
static Kernel pick_tpw(int tpw) {
  if constexpr (RAGGED) {
    switch (tpw) {
      case 2: return kernel_unequal<2, SM>;
      case 3: return kernel_unequal<3, SM>;
      case 4: return kernel_unequal<4, SM>;
      case 6: return kernel_unequal<6, SM>;
      case 7: return kernel_unequal<7, SM>;
      case 8: return kernel_unequal<8, SM>;
      default: return nullptr;
    }
  } else {
    switch (tpw) {
      case 1: return kernel<1, 1, SM>;
      case 2: return kernel<1, 2, SM>;
      case 3: return kernel<1, 3, SM>;
      case 4: return kernel<1, 4, SM>;
      case 6: return kernel<1, 6, SM>;
      case 7: return kernel<1, 7, SM>;
      case 8: return kernel<1, 8, SM>;
      default: return nullptr;
    }
  }
}

}  // namespace gemv

// Shape of a GEMV launch: one row tile per workgroup, W <= 16 wavefronts of TPW k-tiles each (W * TPW = k-tiles of a
// row).  Measured on 1024^2 ... 8192 x 28672: shares of two k-tiles are best as long as the chip can hold all
// wavefronts at once (eight per SIMD = 32 per CU: more wavefronts hide more of the issue latency of a stream that is
// bound by instruction issue); beyond that, longer shares (less set-up per weight) win, and when even shares of two
// leave most of the chip empty, shares of one k-tile do.  Two row tiles per wavefront (shared activation fragments)
// measured slower in every shape and are not built.  false: K does not split that way.
bool gemv1_shape(const Layout& L, int cus, int* tpw_out, int* w_out) {
  if (L.tiles[kWide] != 0 || L.has_map || L.tiles[kNarrow] < 1) return false;
  const int tiles = L.tiles[kNarrow];
  const int64_t waves2 = (int64_t)L.row_tiles * ((tiles + 1) / 2);   // wavefronts with shares of two k-tiles
  int want = 2;
  if (waves2 > (int64_t)32 * cus) want = 4;
  else if (2 * waves2 < (int64_t)3 * cus) want = 1;
  static const int kBuilt[] = {1, 2, 3, 4, 6, 7, 8};
  int best = 0, best_dist = 1 << 30;
  for (int tpw : kBuilt) {
    if (tiles % tpw != 0 || tiles / tpw > 16) continue;
    const int dist = std::abs(tpw - want) * 2 + (tpw < want ? 1 : 0);   // nearest; of two equally near the longer share
    if (dist < best_dist) { best_dist = dist; best = tpw; }
  }
  if (best == 0) {
    // no equal split (43 k-tiles for K = 11008): the shortest built share that needs at most 16 wavefronts, the last
    // of which gets what is left
    for (int tpw : kBuilt) {
      if (tpw >= 2 && (tiles + tpw - 1) / tpw <= 16) { best = tpw; break; }
    }
    if (best == 0) return false;
  }
  *tpw_out = best;
  *w_out = (tiles + best - 1) / best;
  return true;
}

int launch_gemv1(const ccq_weight* w, const Layout& L, const void* x, void* y, void* stream, int tpw, int waves) {
  using namespace gemv;
  if (tpw < 1 || waves < 1 || waves > 16 || waves != (L.tiles[kNarrow] + tpw - 1) / tpw || L.tiles[kWide] != 0 || L.has_map) return CCQ_ERR_UNSUPPORTED;
  if ((int64_t)L.row_tiles * L.tiles[kNarrow] * 1024 >= ((int64_t)1 << 40)) return CCQ_ERR_UNSUPPORTED;
  const bool ragged = waves * tpw != L.tiles[kNarrow];
  Args a;
  a.codes = static_cast<const uint8_t*>(w->codes);
  a.scales = static_cast<const uint16_t*>(w->scales);
  a.alpha = w->code_alpha;
  a.beta = w->code_beta;
  a.x = static_cast<const uint16_t*>(x);
  a.y = static_cast<uint16_t*>(y);
  a.scale_super = static_cast<const uint16_t*>(w->scale_super);
  a.tiles = L.tiles[kNarrow];
  a.cneg = -(128.f + L.zp[kNarrow]);
  a.g_last = L.G - 1;
  a.n_last = L.N - 1;
  const Kernel k = L.scale_mode == 0 ? (ragged ? pick_tpw<0, true>(tpw) : pick_tpw<0, false>(tpw)) : (ragged ? pick_tpw<1, true>(tpw) : pick_tpw<1, false>(tpw));
  if (!k) return CCQ_ERR_UNSUPPORTED;
  const size_t lds = (size_t)waves * (tpw * 4) * (8 * 16 + 4 * 16);   // at most 16 * 32 * 192 bytes = 96 KiB
  if (lds > 48 * 1024 && hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
    (void)hipGetLastError();
    return CCQ_ERR_HIP;
  }
  hipLaunchKernelGGL(k, dim3((unsigned)L.row_tiles), dim3((unsigned)(64 * waves)), lds, static_cast<hipStream_t>(stream), a);
  return hipGetLastError() == hipSuccess ? CCQ_OK : CCQ_ERR_HIP;
}

// Two to four rows: the same shares (of one to four k-tiles), as long as the four rows' fragments of all of K fit the LDS
// of a CU (2304 bytes per k-tile: K <= 16384).  Beyond 35 k-tiles only one workgroup fits a CU and the kernel still
// beats the 16-row one with its second launch (12288 x 4096 at M = 4: 7.8 against 13.1 us; 16384 x 4096: 9.3 against 13.7).
bool gemv4_shape(const Layout& L, int cus, int* tpw_out, int* w_out) {
  if (L.tiles[kWide] != 0 || L.has_map || L.tiles[kNarrow] < 1) return false;
  const int tiles = L.tiles[kNarrow];
  if ((int64_t)tiles * 2304 > 150 * 1024) return false;
  const int64_t waves2 = (int64_t)L.row_tiles * ((tiles + 1) / 2);
  int want = 2;
  if (waves2 > (int64_t)32 * cus) want = 4;
  else if (2 * waves2 < (int64_t)3 * cus) want = 1;
  int best = 0, best_dist = 1 << 30;
  for (int tpw : {1, 2, 3, 4}) {   // the share lengths that are built
    if (tiles % tpw != 0 || tiles / tpw > 16) continue;
    const int dist = std::abs(tpw - want) * 2 + (tpw < want ? 1 : 0);
    if (dist < best_dist) { best_dist = dist; best = tpw; }
  }
  if (best == 0) {   // no equal split: unequal shares, the last one shorter (see gemv1_shape)
    for (int tpw : {2, 3, 4}) {
      if ((tiles + tpw - 1) / tpw <= 16) { best = tpw; break; }
    }
    if (best == 0) return false;
  }
  *tpw_out = best;
  *w_out = (tiles + best - 1) / best;
  return true;
}

int launch_gemv4(const ccq_weight* w, const Layout& L, const void* x, int M, int64_t ldx, void* y, int64_t ldy, void* stream, int tpw, int waves) {
  using namespace gemv;
  if (M < 1 || M > 4 || tpw < 1 || waves < 1 || waves > 16 || waves != (L.tiles[kNarrow] + tpw - 1) / tpw || L.tiles[kWide] != 0 || L.has_map) return CCQ_ERR_UNSUPPORTED;
  const bool ragged = waves * tpw != L.tiles[kNarrow];
  if ((int64_t)L.row_tiles * L.tiles[kNarrow] * 1024 >= ((int64_t)1 << 40)) return CCQ_ERR_UNSUPPORTED;
  Args4 a4;
  Args& a = a4.a;
  a.codes = static_cast<const uint8_t*>(w->codes);
  a.scales = static_cast<const uint16_t*>(w->scales);
  a.alpha = w->code_alpha;
  a.beta = w->code_beta;
  a.x = static_cast<const uint16_t*>(x);
  a.y = static_cast<uint16_t*>(y);
  a.scale_super = static_cast<const uint16_t*>(w->scale_super);
  a.tiles = L.tiles[kNarrow];
  a.cneg = -(128.f + L.zp[kNarrow]);
  a.g_last = L.G - 1;
  a.n_last = L.N - 1;
  a4.ldx = ldx;
  a4.ldy = ldy;
  a4.M = M;
  typedef void (*Kernel4)(const Args4);
  Kernel4 k = nullptr;
  if (ragged) {
    if (L.scale_mode == 0) k = tpw == 2 ? kernel4_unequal<2, 0> : (tpw == 3 ? kernel4_unequal<3, 0> : (tpw == 4 ? kernel4_unequal<4, 0> : nullptr));
    else k = tpw == 2 ? kernel4_unequal<2, 1> : (tpw == 3 ? kernel4_unequal<3, 1> : (tpw == 4 ? kernel4_unequal<4, 1> : nullptr));
  } else if (L.scale_mode == 0) {
    k = tpw == 1 ? kernel4<1, 0> : (tpw == 2 ? kernel4<2, 0> : (tpw == 3 ? kernel4<3, 0> : (tpw == 4 ? kernel4<4, 0> : nullptr)));
  } else {
    k = tpw == 1 ? kernel4<1, 1> : (tpw == 2 ? kernel4<2, 1> : (tpw == 3 ? kernel4<3, 1> : (tpw == 4 ? kernel4<4, 1> : nullptr)));
  }
  if (!k) return CCQ_ERR_UNSUPPORTED;
  const size_t lds = (size_t)waves * tpw * 2304;   // 576 bytes per group: 8 fragments of 4 rows, 16 start values
  if (lds > 160 * 1024) return CCQ_ERR_UNSUPPORTED;
  if (lds > 48 * 1024 && hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
    (void)hipGetLastError();
    return CCQ_ERR_HIP;
  }
  hipLaunchKernelGGL(k, dim3((unsigned)L.row_tiles), dim3((unsigned)(64 * waves)), lds, static_cast<hipStream_t>(stream), a4);
  return hipGetLastError() == hipSuccess ? CCQ_OK : CCQ_ERR_HIP;
}

// Grouped product with at most four rows per expert on narrow-format weights: the one-row or the four-row kernel per
// expert that has rows.  Shares of one to four k-tiles, at most 16 per row tile, chosen as for the dense kernels with
// `experts` (those that have rows, as far as the host knows) times as many row tiles.
bool gemv_grouped_shape(const Layout& L, int cus, int experts, bool four, int* tpw_out, int* w_out) {
  if (L.tiles[kWide] != 0 || L.has_map || L.tiles[kNarrow] < 1) return false;
  const int tiles = L.tiles[kNarrow];
  if (four && (int64_t)tiles * 2304 > 150 * 1024) return false;
  const int64_t waves2 = (int64_t)L.row_tiles * std::max(1, experts) * ((tiles + 1) / 2);
  int want = 2;
  if (waves2 > (int64_t)32 * cus) want = 4;   // also with four rows: shares of two measured 14-30 % slower on 100-224 experts of 1024 x 7168
  else if (2 * waves2 < (int64_t)3 * cus) want = 1;
  int best = 0, best_dist = 1 << 30;
  for (int tpw : {1, 2, 3, 4}) {
    if (tiles % tpw != 0 || tiles / tpw > 16) continue;
    const int dist = std::abs(tpw - want) * 2 + (tpw < want ? 1 : 0);
    if (dist < best_dist) { best_dist = dist; best = tpw; }
  }
  if (best == 0) return false;
  *tpw_out = best;
  *w_out = tiles / best;
  return true;
}

namespace gemv {
typedef void (*KernelG)(const ArgsG);
template <int SM, bool FOUR>
static KernelG pick_grouped(int tpw) {
  switch (tpw) {
    case 1: return kernel_grouped<1, SM, FOUR>;
    case 2: return kernel_grouped<2, SM, FOUR>;
    case 3: return kernel_grouped<3, SM, FOUR>;
    case 4: return kernel_grouped<4, SM, FOUR>;
    default: return nullptr;
  }
}
}  // namespace gemv

int launch_gemv_grouped(const ccq_weight* w0, const Layout& L, int E, int64_t codes_stride, int64_t scales_stride, int64_t ab_stride, const void* x,
                        int64_t ldx, const int32_t* sorted_rows, const int32_t* expert_offsets_dev, void* y, int64_t ldy, int most_rows,
                        int n_active, const uint16_t* active_ids, void* stream) {
  using namespace gemv;
  if (most_rows < 1 || most_rows > 4 || E < 1 || E > 65535 || n_active < 0 || n_active > kMaxActiveList) return CCQ_ERR_UNSUPPORTED;
  if ((int64_t)L.row_tiles * L.tiles[kNarrow] * 1024 >= ((int64_t)1 << 40)) return CCQ_ERR_UNSUPPORTED;
  const bool four = most_rows > 1;
  int tpw = 0, waves = 0;
  if (!gemv_grouped_shape(L, device_cus(), n_active > 0 ? n_active : E, four, &tpw, &waves)) return CCQ_ERR_UNSUPPORTED;
  ArgsG g;
  Args& a = g.a;
  a.codes = static_cast<const uint8_t*>(w0->codes);
  a.scales = static_cast<const uint16_t*>(w0->scales);
  a.alpha = w0->code_alpha;
  a.beta = w0->code_beta;
  a.x = static_cast<const uint16_t*>(x);
  a.y = static_cast<uint16_t*>(y);
  a.scale_super = static_cast<const uint16_t*>(w0->scale_super);
  a.tiles = L.tiles[kNarrow];
  a.cneg = -(128.f + L.zp[kNarrow]);
  a.g_last = L.G - 1;
  a.n_last = L.N - 1;
  g.ldx = ldx;
  g.ldy = ldy;
  g.codes_stride = codes_stride;
  g.scales_stride = scales_stride;
  g.ab_stride = ab_stride;
  g.sorted_rows = sorted_rows;
  g.offsets = expert_offsets_dev;
  g.n_active = n_active;
  for (int i = 0; i < kMaxActiveList; ++i) g.active_ids[i] = i < n_active ? active_ids[i] : (uint16_t)0;
  KernelG k = nullptr;
  if (L.scale_mode == 0) k = four ? pick_grouped<0, true>(tpw) : pick_grouped<0, false>(tpw);
  else k = four ? pick_grouped<1, true>(tpw) : pick_grouped<1, false>(tpw);
  if (!k) return CCQ_ERR_UNSUPPORTED;
  const size_t lds = four ? (size_t)waves * tpw * 2304 : (size_t)waves * (tpw * 4) * (8 * 16 + 4 * 16);
  if (lds > 160 * 1024) return CCQ_ERR_UNSUPPORTED;
  if (lds > 48 * 1024 && hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
    (void)hipGetLastError();
    return CCQ_ERR_HIP;
  }
  hipLaunchKernelGGL(k, dim3((unsigned)L.row_tiles, (unsigned)(n_active > 0 ? n_active : E)), dim3((unsigned)(64 * waves)), lds,
                     static_cast<hipStream_t>(stream), g);
  return hipGetLastError() == hipSuccess ? CCQ_OK : CCQ_ERR_HIP;
}

// Shape of a one-row launch on wide-format or mixed weights: wn wavefronts with shares of tpwn narrow k-tiles, then
// ww wavefronts with shares of tpww wide k-tiles, at most 16 in all; shares of two k-tiles where K splits that way
// (every lane of a wavefront then stages one (group, quarter) of the wide share's activations).  false: no wide
// k-tiles, the hybrid word, or K does not split into at most 16 such shares (the caller uses the general kernel).
bool gemv_nw_shape(const Layout& L, int* tpwn_out, int* tpww_out, int* wn_out, int* ww_out) {
  if (L.tiles[kWide] < 1) return false;   // the hybrid word is a wide kind of its own (never mixed)
  const int tn = L.tiles[kNarrow], tw = L.tiles[kWide];
  if (tn == 0) {
    // shares of one k-tile (512 weights per row, as much as the two narrow k-tiles the narrow kernel prefers) while the
    // chip holds all wavefronts at once (32 per CU); beyond that shares of two (config 3, all wide, 28672 wavefronts of
    // one k-tile: 23.3 us against 21.7 us with shares of two)
    const bool fits = (int64_t)L.row_tiles * tw <= (int64_t)32 * device_cus();
    for (int pw : {fits ? 1 : 2, fits ? 2 : 1}) {
      if (tw % pw != 0 || tw / pw > 16) continue;
      *tpwn_out = 0; *tpww_out = pw; *wn_out = 0; *ww_out = tw / pw;
      return true;
    }
    return false;
  }
  // a mix: shares of about the same length first (one wide k-tile is 144 weights per lane, two narrow ones 128); the
  // short pair while the chip holds all its wavefronts at once (32 per CU), the long one beyond that: less set-up per
  // weight (config 3, 32 of 128 groups wide, N = 28672: 19.7 -> 18.2 us)
  static const int kShort[][2] = {{2, 1}, {4, 2}, {2, 2}, {4, 1}, {1, 1}, {1, 2}};
  static const int kLong[][2] = {{4, 2}, {2, 1}, {2, 2}, {4, 1}, {1, 1}, {1, 2}};
  const bool fits = tn % 2 != 0 || (int64_t)L.row_tiles * (tn / 2 + tw) <= (int64_t)32 * device_cus();
  for (const auto& pr : fits ? kShort : kLong) {
    const int pn = pr[0], pw = pr[1];
    if (tn % pn != 0 || tw % pw != 0 || tn / pn + tw / pw > 16) continue;
    *tpwn_out = pn; *tpww_out = pw; *wn_out = tn / pn; *ww_out = tw / pw;
    return true;
  }
  return false;
}

namespace gemv {
// The dense kernel (GROUPED = false, one ArgsNW argument) or the grouped one (one ArgsNWG argument) of a share shape.
template <int SM, bool GROUPED, int TPWN, int TPWW, bool H16 = false>
static const void* nw_entry() {
  if constexpr (GROUPED) return reinterpret_cast<const void*>(&kernel_nw_grouped<TPWN, TPWW, SM, H16>);
  else return reinterpret_cast<const void*>(&kernel_nw<TPWN, TPWW, SM, H16>);
}
template <int SM, bool GROUPED>
static const void* pick_nw_h16(int tpww) {
  if (tpww == 1) return nw_entry<SM, GROUPED, 0, 1, true>();
  if (tpww == 2) return nw_entry<SM, GROUPED, 0, 2, true>();
  return nullptr;
}
template <int SM, bool GROUPED>
static const void* pick_nw(int tpwn, int tpww) {
  if (tpww == 1) {
    switch (tpwn) {
      case 0: return nw_entry<SM, GROUPED, 0, 1>();
      case 1: return nw_entry<SM, GROUPED, 1, 1>();
      case 2: return nw_entry<SM, GROUPED, 2, 1>();
      case 4: return nw_entry<SM, GROUPED, 4, 1>();
    }
  } else if (tpww == 2) {
    switch (tpwn) {
      case 0: return nw_entry<SM, GROUPED, 0, 2>();
      case 1: return nw_entry<SM, GROUPED, 1, 2>();
      case 2: return nw_entry<SM, GROUPED, 2, 2>();
      case 4: return nw_entry<SM, GROUPED, 4, 2>();
    }
  }
  return nullptr;
}
template <bool GROUPED>
static const void* pick_nw_kernel(const Layout& L, int tpwn, int tpww) {
  if (L.h16) return L.scale_mode == 0 ? pick_nw_h16<0, GROUPED>(tpww) : pick_nw_h16<1, GROUPED>(tpww);
  return L.scale_mode == 0 ? pick_nw<0, GROUPED>(tpwn, tpww) : pick_nw<1, GROUPED>(tpwn, tpww);
}

static void fill_args_nw(ArgsNW& a, const ccq_weight* w, const Layout& L, const void* x, void* y, int wn) {
  a.codes = static_cast<const uint8_t*>(w->codes);
  a.scales = static_cast<const uint16_t*>(w->scales);
  a.alpha = w->code_alpha;
  a.beta = w->code_beta;
  a.x = static_cast<const uint16_t*>(x);
  a.y = static_cast<uint16_t*>(y);
  a.scale_super = static_cast<const uint16_t*>(w->scale_super);
  a.meta = L.has_map ? static_cast<const int32_t*>(w->meta) : nullptr;
  a.row_tile_bytes = L.row_tile_bytes;
  a.row_tile_scale_halfs = L.row_tile_scale_halfs;
  a.tiles_n = L.tiles[kNarrow];
  a.tiles_w = L.tiles[kWide];
  a.waves_n = wn;
  a.meta_wide = L.pgroups[kNarrow];
  a.cneg_n = -(128.f + L.zp[kNarrow]);
  a.cneg_w = -(128.f + L.zp[kWide]);
  a.g_last = L.G - 1;
  a.n_last = L.N - 1;
}

// One launch of a kernel that takes a single by-value argument block.
static int launch_nw(const void* k, void* arg_block, dim3 grid, int tpwn, int tpww, int wn, int ww, void* stream) {
  const size_t region_n = (size_t)tpwn * 4 * (8 * 16 + 4 * 16), region_w = (size_t)tpww * 8 * (12 * 16 + 4 * 16);
  const size_t lds = std::max<size_t>((size_t)wn * region_n + (size_t)ww * region_w, 1024);   // at most 16 * 4 KiB; the K reduction reuses the start
  if (lds > 48 * 1024 && hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
    (void)hipGetLastError();
    return CCQ_ERR_HIP;
  }
  void* params[] = {arg_block};
  if (hipLaunchKernel(k, grid, dim3((unsigned)(64 * (wn + ww))), params, lds, static_cast<hipStream_t>(stream)) != hipSuccess) {
    (void)hipGetLastError();
    return CCQ_ERR_HIP;
  }
  return hipGetLastError() == hipSuccess ? CCQ_OK : CCQ_ERR_HIP;
}
}  // namespace gemv

int launch_gemv_nw(const ccq_weight* w, const Layout& L, const void* x, void* y, void* stream, int tpwn, int tpww, int wn, int ww) {
  using namespace gemv;
  if (ww < 1 || wn < 0 || (L.h16 && wn != 0) || wn + ww > 16 || wn * tpwn != L.tiles[kNarrow] || ww * tpww != L.tiles[kWide]) return CCQ_ERR_UNSUPPORTED;
  if (L.row_tile_bytes * (int64_t)L.row_tiles >= ((int64_t)1 << 40)) return CCQ_ERR_UNSUPPORTED;
  ArgsNW a;
  fill_args_nw(a, w, L, x, y, wn);
  const void* k = pick_nw_kernel<false>(L, tpwn, tpww);
  if (!k) return CCQ_ERR_UNSUPPORTED;
  return launch_nw(k, &a, dim3((unsigned)L.row_tiles), tpwn, tpww, wn, ww, stream);
}

// The grouped product with at most one row per expert on wide-format, mixed and hybrid-word weights: one such GEMV per
// expert that has a row; `active_ids` lists the n_active experts that have one (n_active = 0: the grid covers all E).
int launch_gemv_nw_grouped(const ccq_weight* w0, const Layout& L, int E, int64_t codes_stride, int64_t scales_stride, int64_t ab_stride,
                           const void* x, int64_t ldx, const int32_t* sorted_rows, const int32_t* expert_offsets_dev, void* y, int64_t ldy,
                           int n_active, const uint16_t* active_ids, void* stream) {
  using namespace gemv;
  int tpwn = 0, tpww = 0, wn = 0, ww = 0;
  if (E < 1 || E > 65535 || n_active < 0 || n_active > kMaxActiveList || !gemv_nw_shape(L, &tpwn, &tpww, &wn, &ww)) return CCQ_ERR_UNSUPPORTED;
  if (L.row_tile_bytes * (int64_t)L.row_tiles >= ((int64_t)1 << 40)) return CCQ_ERR_UNSUPPORTED;
  ArgsNWG g;
  fill_args_nw(g.a, w0, L, x, y, wn);
  g.ldx = ldx;
  g.ldy = ldy;
  g.codes_stride = codes_stride;
  g.scales_stride = scales_stride;
  g.ab_stride = ab_stride;
  g.sorted_rows = sorted_rows;
  g.offsets = expert_offsets_dev;
  g.n_active = n_active;
  for (int i = 0; i < kMaxActiveList; ++i) g.active_ids[i] = i < n_active ? active_ids[i] : (uint16_t)0;
  const void* k = pick_nw_kernel<true>(L, tpwn, tpww);
  if (!k) return CCQ_ERR_UNSUPPORTED;
  return launch_nw(k, &g, dim3((unsigned)L.row_tiles, (unsigned)(n_active > 0 ? n_active : E)), tpwn, tpww, wn, ww, stream);
}

// K shares of the 2..16-row kernel on wide-format and mixed weights: narrow shares of tpwn k-tiles, then wide shares of
// tpww, at most min(max_shares, kMaxSplitsK) in all; the longest shares first (the least partial-tile traffic: at
// N = 28672 a share's partial tile is as many bytes as 1/6 of a wide k-tile column block), shorter ones only when the
// long ones leave compute units without a workgroup.  false: no wide k-tiles, the hybrid word, or no such split.
bool gemv16_nw_shape(const Layout& L, int cus, int64_t max_shares, int* tpwn_out, int* tpww_out, int* sn_out, int* sw_out) {
  if (L.tiles[kWide] < 1) return false;   // the hybrid word is a wide kind of its own (never mixed)
  const int tn = L.tiles[kNarrow], tw = L.tiles[kWide], nw = 8;
  const int64_t row_blocks = (L.row_tiles + nw - 1) / nw;
  const int64_t cap = std::min<int64_t>(max_shares, kMaxSplitsK);
  static const int kPairs[][2] = {{4, 2}, {2, 1}, {2, 2}, {4, 1}, {1, 1}, {1, 2}};
  static const int kWideOnly[] = {2, 1};
  bool found = false;
  auto take = [&](int pn, int pw) -> bool {
    const int sn = pn > 0 ? tn / pn : 0, sw = tw / pw;
    if (sn + sw > cap) return false;
    if (found && (int64_t)(*sn_out + *sw_out) >= sn + sw) return false;   // only more shares than what is already held
    *tpwn_out = pn; *tpww_out = pw; *sn_out = sn; *sw_out = sw;
    found = true;
    return row_blocks * (sn + sw) >= cus;   // enough workgroups: stop
  };
  if (tn == 0) {
    for (int pw : kWideOnly) {
      if (tw % pw != 0) continue;
      if (take(0, pw)) break;
    }
  } else {
    for (const auto& pr : kPairs) {
      if (tn % pr[0] != 0 || tw % pr[1] != 0) continue;
      if (take(pr[0], pr[1])) break;
    }
  }
  return found;
}

int launch_gemv16_nw(const ccq_weight* w, const Layout& L, const void* x, int M, int64_t ldx, void* y, int64_t ldy, float* partial, int tpwn,
                     int tpww, int sn, int sw, void* stream) {
  using namespace gemv;
  constexpr int nw = 8;
  if (M < 1 || M > 16 || sw < 1 || sn < 0 || (L.h16 && sn != 0) || sn * tpwn != L.tiles[kNarrow] || sw * tpww != L.tiles[kWide]) return CCQ_ERR_UNSUPPORTED;
  const int S = sn + sw;
  if (S > kMaxSplitsK || (S > 1 && !partial)) return CCQ_ERR_UNSUPPORTED;
  if (L.row_tile_bytes * (int64_t)L.row_tiles >= ((int64_t)1 << 40)) return CCQ_ERR_UNSUPPORTED;
  Args16NW a;
  a.codes = static_cast<const uint8_t*>(w->codes);
  a.scales = static_cast<const uint16_t*>(w->scales);
  a.alpha = w->code_alpha;
  a.beta = w->code_beta;
  a.x = static_cast<const uint16_t*>(x);
  a.y = static_cast<uint16_t*>(y);
  a.scale_super = static_cast<const uint16_t*>(w->scale_super);
  a.meta = L.has_map ? static_cast<const int32_t*>(w->meta) : nullptr;
  a.partial = partial;
  a.ldx = ldx;
  a.ldy = ldy;
  a.row_tile_bytes = L.row_tile_bytes;
  a.row_tile_scale_halfs = L.row_tile_scale_halfs;
  a.tiles_n = L.tiles[kNarrow];
  a.tiles_w = L.tiles[kWide];
  a.row_tiles = L.row_tiles;
  a.M = M;
  a.N = L.Npad;
  a.shares_n = sn;
  a.meta_wide = L.pgroups[kNarrow];
  a.cneg_n = -(128.f + L.zp[kNarrow]);
  a.cneg_w = -(128.f + L.zp[kWide]);
  a.g_last = L.G - 1;
  a.n_last = L.N - 1;
  typedef void (*Kernel16NW)(const Args16NW);
  Kernel16NW k = nullptr;
  const int key = tpwn * 10 + tpww;
  if (L.h16) {
    if (L.scale_mode == 0) k = tpww == 1 ? kernel16_nw<0, 1, 0, nw, true> : (tpww == 2 ? kernel16_nw<0, 2, 0, nw, true> : nullptr);
    else k = tpww == 1 ? kernel16_nw<0, 1, 1, nw, true> : (tpww == 2 ? kernel16_nw<0, 2, 1, nw, true> : nullptr);
  } else if (L.scale_mode == 0) {
    switch (key) {
      case 1: k = kernel16_nw<0, 1, 0, nw>; break;
      case 2: k = kernel16_nw<0, 2, 0, nw>; break;
      case 11: k = kernel16_nw<1, 1, 0, nw>; break;
      case 12: k = kernel16_nw<1, 2, 0, nw>; break;
      case 21: k = kernel16_nw<2, 1, 0, nw>; break;
      case 22: k = kernel16_nw<2, 2, 0, nw>; break;
      case 41: k = kernel16_nw<4, 1, 0, nw>; break;
      case 42: k = kernel16_nw<4, 2, 0, nw>; break;
    }
  } else {
    switch (key) {
      case 1: k = kernel16_nw<0, 1, 1, nw>; break;
      case 2: k = kernel16_nw<0, 2, 1, nw>; break;
      case 11: k = kernel16_nw<1, 1, 1, nw>; break;
      case 12: k = kernel16_nw<1, 2, 1, nw>; break;
      case 21: k = kernel16_nw<2, 1, 1, nw>; break;
      case 22: k = kernel16_nw<2, 2, 1, nw>; break;
      case 41: k = kernel16_nw<4, 1, 1, nw>; break;
      case 42: k = kernel16_nw<4, 2, 1, nw>; break;
    }
  }
  if (!k) return CCQ_ERR_UNSUPPORTED;
  const size_t lds_n = (size_t)(tpwn * 4) * (8 * 16 * 16 + 16 * 4), lds_w = (size_t)(tpww * 8) * (12 * 16 * 16 + 16 * 4);
  const size_t lds = std::max(lds_n, lds_w);   // at most 16 groups x 3136 bytes = 49 KiB
  if (lds > 48 * 1024 && hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
    (void)hipGetLastError();
    return CCQ_ERR_HIP;
  }
  const dim3 grid((unsigned)((L.row_tiles + nw - 1) / nw), (unsigned)S);
  hipLaunchKernelGGL(k, grid, dim3((unsigned)(64 * nw)), lds, static_cast<hipStream_t>(stream), a);
  return hipGetLastError() == hipSuccess ? CCQ_OK : CCQ_ERR_HIP;
}

// Shares of K for the 2..16-row kernel: shares of four k-tiles (the least partial-tile traffic) unless that leaves
// compute units without a workgroup, then shorter ones -- but never more shares than `max_shares` (what the caller's
// workspace holds).  false: K does not split into at most min(max_shares, kMaxSplitsK) shares of 1, 2 or 4 k-tiles.
bool gemv16_shape(const Layout& L, int cus, int64_t max_shares, int* tpw_out, int* nw_out) {
  if (L.tiles[kWide] != 0 || L.has_map || L.tiles[kNarrow] < 1) return false;
  const int tiles = L.tiles[kNarrow], nw = 8;
  const int64_t row_blocks = (L.row_tiles + nw - 1) / nw;
  const int64_t cap = std::min<int64_t>(max_shares, kMaxSplitsK);
  int pick = 0;
  for (int tpw : {4, 2, 1}) {
    if (tiles % tpw != 0 || tiles / tpw > cap) continue;
    pick = tpw;                                   // the shortest share that qualifies, unless a longer one fills the chip
    if (row_blocks * (tiles / tpw) >= cus) break;
  }
  if (pick == 0 || tiles / pick > 16) {
    // no equal split, or only one into many short shares (43 k-tiles for K = 11008): unequal shares, the last one
    // shorter -- fewer partial tiles than 43 shares of one k-tile would write
    int unequal = 0;
    for (int tpw : {4, 2}) {
      const int shares = (tiles + tpw - 1) / tpw;
      if (shares > cap) continue;
      unequal = tpw;
      if (row_blocks * shares >= cus) break;
    }
    if (unequal != 0) pick = unequal;
  }
  if (pick == 0) return false;
  *tpw_out = pick;
  *nw_out = nw;
  return true;
}

// Two to 32 rows (beyond 16: two 16-row tiles of activations per workgroup, nw = 8), narrow format, dense.  nw = 8 or 16 wavefronts (row tiles) per workgroup share one staged slice of the
// activations; S = tiles / tpw <= 32 shares of K across workgroups (S > 1 needs `partial`, fp32 [S][M][N], and a pass of
// launch_reduce_splits afterwards).
int launch_gemv16(const ccq_weight* w, const Layout& L, const void* x, int M, int64_t ldx, void* y, int64_t ldy, float* partial, int tpw,
                  int nw, void* stream) {
  using namespace gemv;
  if (M < 1 || M > 32 || L.tiles[kWide] != 0 || L.has_map || L.tiles[kNarrow] < 1) return CCQ_ERR_UNSUPPORTED;
  if (tpw < 1 || nw < 1 || nw > 16) return CCQ_ERR_UNSUPPORTED;
  const int mt = M > 16 ? 2 : 1;   // 16-row tiles of activations held by a workgroup
  const int S = (L.tiles[kNarrow] + tpw - 1) / tpw;
  const bool ragged = L.tiles[kNarrow] % tpw != 0;   // the last share is shorter
  if (S > kMaxSplitsK || (S > 1 && !partial)) return CCQ_ERR_UNSUPPORTED;
  if ((int64_t)L.row_tiles * L.tiles[kNarrow] * 1024 >= ((int64_t)1 << 40)) return CCQ_ERR_UNSUPPORTED;
  Args16 a;
  a.codes = static_cast<const uint8_t*>(w->codes);
  a.scales = static_cast<const uint16_t*>(w->scales);
  a.alpha = w->code_alpha;
  a.beta = w->code_beta;
  a.x = static_cast<const uint16_t*>(x);
  a.y = static_cast<uint16_t*>(y);
  a.scale_super = static_cast<const uint16_t*>(w->scale_super);
  a.partial = partial;
  a.ldx = ldx;
  a.ldy = ldy;
  a.tiles = L.tiles[kNarrow];
  a.row_tiles = L.row_tiles;
  a.M = M;
  a.N = L.Npad;
  a.cneg = -(128.f + L.zp[kNarrow]);
  a.g_last = L.G - 1;
  a.n_last = L.N - 1;
  typedef void (*Kernel16)(const Args16);
  Kernel16 k = nullptr;
  const int key = (ragged ? 10000 : 0) + (mt - 1) * 1000 + tpw * 100 + nw;
  if (L.scale_mode == 0) {
    switch (key) {
      case 11208: k = kernel32_unequal<2, 0, 8>; break;
      case 11408: k = kernel32_unequal<4, 0, 8>; break;
      case 10208: k = kernel16_unequal<2, 0, 8>; break;
      case 10408: k = kernel16_unequal<4, 0, 8>; break;
      case 1108: k = kernel32<1, 0, 8>; break;
      case 1208: k = kernel32<2, 0, 8>; break;
      case 1408: k = kernel32<4, 0, 8>; break;
      case 108: k = kernel16<1, 0, 8>; break;
      case 116: k = kernel16<1, 0, 16>; break;
      case 208: k = kernel16<2, 0, 8>; break;
      case 216: k = kernel16<2, 0, 16>; break;
      case 408: k = kernel16<4, 0, 8>; break;
      case 416: k = kernel16<4, 0, 16>; break;
    }
  } else {
    switch (key) {
      case 11208: k = kernel32_unequal<2, 1, 8>; break;
      case 11408: k = kernel32_unequal<4, 1, 8>; break;
      case 10208: k = kernel16_unequal<2, 1, 8>; break;
      case 10408: k = kernel16_unequal<4, 1, 8>; break;
      case 1108: k = kernel32<1, 1, 8>; break;
      case 1208: k = kernel32<2, 1, 8>; break;
      case 1408: k = kernel32<4, 1, 8>; break;
      case 108: k = kernel16<1, 1, 8>; break;
      case 116: k = kernel16<1, 1, 16>; break;
      case 208: k = kernel16<2, 1, 8>; break;
      case 216: k = kernel16<2, 1, 16>; break;
      case 408: k = kernel16<4, 1, 8>; break;
      case 416: k = kernel16<4, 1, 16>; break;
    }
  }
  if (!k) return CCQ_ERR_UNSUPPORTED;
  const size_t lds = (size_t)(tpw * 4) * (8 * 16 * 16 + 16 * 4) * mt;
  if (lds > 48 * 1024 && hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
    (void)hipGetLastError();
    return CCQ_ERR_HIP;
  }
  const dim3 grid((unsigned)((L.row_tiles + nw - 1) / nw), (unsigned)S);
  hipLaunchKernelGGL(k, grid, dim3((unsigned)(64 * nw)), lds, static_cast<hipStream_t>(stream), a);
  return hipGetLastError() == hipSuccess ? CCQ_OK : CCQ_ERR_HIP;
}

// Compute units of the current device, looked up once per device.
int device_cus() {
  static std::atomic<int> cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
    (void)hipGetLastError();
    return 256;
  }
  int c = cached[dev].load(std::memory_order_relaxed);
  if (c <= 0) {
    if (hipDeviceGetAttribute(&c, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || c <= 0) {
      (void)hipGetLastError();
      c = 256;
    }
    cached[dev].store(c, std::memory_order_relaxed);
  }
  return c;
}

}  // namespace ccq
