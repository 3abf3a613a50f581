// Skinny fused dequantize-and-multiply (M <= 64 rows per pass) and its grouped
// (mixture-of-experts) form, for gfx950.
//
// One wavefront owns 16 (or 32) output rows and a range of k-tiles.  It streams
// the packed code bytes with 128-bit loads, cuts the overlapping states out of
// each code with shifts (Sec. 3.1 "Bitshift Decoding", Table 1 shift lists
// [9,6,3,0] / [4,2,0]), and feeds them to the matrix cores as bf16 integers:
// OR-ing a state s into the mantissa of bf16 128.0 (0x4300) gives exactly
// 128 + s.  The contraction of one 64-weight group therefore yields
//     sum_k (128 + s_k) x_k ,
// and starting the accumulator at  -(128 + zp) * sum_k x_k  turns it into
//     sum_k (s_k - zp) x_k ,
// which is multiplied by the group's fp16 scale afterwards -- the linear map
// d = (w_uint - zp) * s of Alg. 2 / Alg. 3 applied after the contraction
// instead of per weight.  For the Code Cluster format the stored byte q is
// first expanded to the 15-bit code c = round(q*alpha + beta) (Alg. 3) with a
// single fused multiply-add against beta + 2^23: the sum lies in [2^23, 2^24)
// where fp32 has unit spacing, so the hardware's round-to-nearest-even *is* the
// rounding of Eq. 1 and c appears in the low mantissa bits.
//
// MFMA 16x16x32 bf16 operand layout (lane l, quarter kq = l / 16):
//   A (activations): row m = l % 16, k-slots 8kq .. 8kq+7
//   B (weights)    : column n = l % 16, k-slots 8kq .. 8kq+7
//   C/D            : rows m = 4kq .. 4kq+3, column n = l % 16
// so all four accumulator values of a lane share the output row n of W and one
// group scale serves them.
//
// With a single activation row (M = 1) the 16x16x32 shape would spend 15/16 of the matrix-core time
// on rows that do not exist, and that instruction runs at half the rate of the 32x32x16 shape on
// this chip.  The M = 1 path uses MFMA 4x4x4 bf16 instead (16 independent 4x4 blocks per wavefront,
// block = lane / 4): lane l still owns row n = l % 16 and quarter kq = l / 16, feeds 4 weights per
// instruction as column l % 4 of its block, and receives in accumulator element 0 the partial sum of
// its own row over its own quarter; the four quarters are added across lanes at the end.
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstring>

#include <algorithm>
#include <type_traits>

#include "ccq_internal.h"

namespace ccq {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;

struct SkinnyArgs {
  const uint8_t* codes;
  const uint16_t* scales;
  const float* alpha;
  const float* beta;
  const int32_t* meta;
  const uint16_t* scale_super;  // fp16 [N] per expert, compressed scales only
  const uint16_t* x;
  uint16_t* y;
  float* partial;
  const int32_t* sorted_rows;
  const int32_t* expert_offsets;
  int64_t ldx, ldy, codes_stride, scales_stride, ab_stride;
  int64_t row_tile_bytes, row_tile_scale_halfs;
  int32_t M;          // rows (dense) or total rows P (grouped)
  int32_t N;          // rows of the device layout (a multiple of 16): the row stride of `partial`
  int32_t row_tiles;
  int32_t tiles[2];   // k-tiles per kind
  int32_t groups_narrow;  // narrow entries of the group map (whole k-tiles), the offset of the wide ones
  int32_t g_last;     // last real group of K: groups past it pad a k-tile (zero scale) and read this group's activations
  int32_t n_last;     // last real output row: rows past it pad a row tile, take its parameters and are not stored
  int32_t KC[2];      // k-tiles per wavefront per staged chunk, per kind
  int32_t SG[2];      // groups of a k-tile staged at a time (= groups per tile unless LDS is tight; then KC = 1)
  int32_t WR, WK, S;
  int32_t inv_WR;     // ceil(2^16 / WR): wave / WR without a division
  // K partition without divisions: workgroup `split` of S owns tiles [A, B) with A = split*sq + min(split, sr),
  // B - A = sq + (split < sr); its WK wavefronts cut that range the same way with (wq, wr)[B - A - sq].
  int32_t sq[2], sr[2];
  int32_t wq[2][2], wrem[2][2];
  int32_t frag_cap;   // 16-byte fragments the LDS staging area holds (per wavefront when one row is held); the start values follow it
  int32_t cneg_cap;   // floats of start values per wavefront (one held row only; multiple of 4)
  float cneg[2];      // -(128 + zp) per kind
  int32_t n_active;   // > 0: gridDim.z experts are listed in active_ids (the others have no rows)
  uint16_t active_ids[kMaxActiveList];
};

// KIND = format (bit 0: kNarrow / kWide) | scale mode << 1 (bit 1: 0 fp16 group scales, 1 the compressed
// scales of Sec. 3.4: a 4-bit field per group times a per-row super scale) | hybrid word << 2 (bit 2, on top
// of kWide: the second kind is the 16-bit word of Sec. 3.2 that holds a (3,3,2) and a (3,4,2) code, which
// shares the wide kind's shape: 8 groups per k-tile, three k-steps per group, three segments per tile).
constexpr int kScale4 = 2;
constexpr int kH16 = 4;
template <int KIND> struct Traits;
template <> struct Traits<kNarrow> {
  static constexpr int GPT = kNarrowGroupsPerTile, T = 2, SEGS = 1, TILE_BYTES = kNarrowTileBytes, SCALE_HALFS = kNarrowTileScaleHalfs;
};
template <> struct Traits<kWide> {
  static constexpr int GPT = kWideGroupsPerTile, T = 3, SEGS = 3, TILE_BYTES = kWideTileBytes, SCALE_HALFS = kWideTileScaleHalfs;
};
template <> struct Traits<kNarrow | kScale4> : Traits<kNarrow> {
  static constexpr int SCALE_HALFS = kNarrowTileScaleHalfs4;
};
template <> struct Traits<kWide | kScale4> : Traits<kWide> {
  static constexpr int SCALE_HALFS = 0;
};
template <> struct Traits<kWide | kH16> : Traits<kWide> {
  static constexpr int TILE_BYTES = kH16TileBytes;
};
template <> struct Traits<kWide | kH16 | kScale4> : Traits<kWide | kH16> {
  static constexpr int SCALE_HALFS = 0;
};
// activation index inside a group for k-slot i (0..6) of a hybrid word: the decode pairs the states at
// shifts (13,11), (6,4), (2,0) and leaves the one at shift 9 alone, i.e. weights {0,1}, {3,4}, {5,6}, {2}
__device__ __forceinline__ int h16_slot_weight(int i) { return i < 2 ? i : (i < 6 ? i + 1 : 2); }

// Activation fragments of the wide and hybrid-word kinds: the k-slots of (quarter kq, k-step t) of a group
// are six or seven consecutive activations, so one 16-byte load (4-byte aligned; never past the group's own
// 64 elements) fetches them and a few byte permutes put them into slot order.
//   wide:   codes 6kq+2t and 6kq+2t+1, weights 18kq+6t+{0..5}, slots {0,3,1,4,2,5,-,-}; code 21 carries weight
//           63 only (quarter 3: k-step 1 holds {60,63,61,-,62,-}, k-step 2 nothing)
//   hybrid: word 4t+kq, weights 7 word+{0..6}, slots {0,1,3,4,5,6,2,-}; word 9 carries weight 63 only
struct __attribute__((packed, aligned(4))) Chunk16 {  // 16 bytes at 4-byte alignment
  uint32_t x, y, z, w;
};
__device__ __forceinline__ uint4 load_chunk16(const uint16_t* p) {
  const Chunk16 c = *reinterpret_cast<const Chunk16*>(p);
  return uint4{c.x, c.y, c.z, c.w};
}
template <int KIND>
__device__ __forceinline__ int frag_first_element(int kq, int t) {
  if constexpr ((KIND & kH16) != 0) return min((7 * (4 * t + kq)) & ~1, 56);
  else return min(18 * kq + 6 * t, 56);
}
template <int KIND>
__device__ __forceinline__ uint4 frag_from_chunk(const uint4 v, int kq, int t) {
  uint4 o = {0u, 0u, 0u, 0u};
  if constexpr ((KIND & kH16) != 0) {
    const int word = 4 * t + kq;
    if (word == 9) {
      o.x = v.w >> 16;  // element 63 of the chunk that starts at 56
    } else if (word < 9) {
      if (word & 1) {   // the word starts at the chunk's second element
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
  } else {
    if (kq < 3 || t == 0) {
      o.x = __builtin_amdgcn_perm(v.y, v.x, 0x07060100u);  // elements 0, 3
      o.y = __builtin_amdgcn_perm(v.z, v.x, 0x05040302u);  // 1, 4
      o.z = __builtin_amdgcn_perm(v.z, v.y, 0x07060100u);  // 2, 5
    } else if (t == 1) {  // chunk starts at 56: weights 60, 63 | 61 | 62
      o.x = __builtin_amdgcn_perm(v.w, v.z, 0x07060100u);
      o.y = v.z >> 16;
      o.z = v.w & 0xFFFFu;
    }
  }
  return o;
}

// k-tiles [A, B) of kind `kind` that workgroup `split` owns.
__device__ __forceinline__ void split_range(const SkinnyArgs& a, int kind, int split, int& A, int& B) {
  const int q = a.sq[kind], r = a.sr[kind];
  A = split * q + min(split, r);
  B = A + q + (split < r ? 1 : 0);
}
// The part [k0, k1) of that range that wavefront wk of WK owns.
__device__ __forceinline__ void wave_range(const SkinnyArgs& a, int kind, int split, int A, int wk, int& k0, int& k1) {
  const int v = split < a.sr[kind] ? 1 : 0;
  const int q = a.wq[kind][v], r = a.wrem[kind][v];
  k0 = A + wk * q + min(wk, r);
  k1 = k0 + q + (wk < r ? 1 : 0);
}

template <int KIND> struct TileRegs {
  u32x4 c[Traits<KIND>::SEGS];
  uint32_t s[Traits<KIND>::GPT / 2];
};

// (a & mask) | orv.  Plain C on purpose: an instruction written as inline assembly is invisible to the
// compiler's hazard recognizer, and a hand-written v_and_or_b32 whose result fed an MFMA one instruction
// later gave wrong results on the device.  The callers keep mask and orv in registers (not literals) so
// that the compiler can still select the single v_and_or_b32.
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t orv) { return (a & mask) | orv; }

__device__ __forceinline__ uint32_t dword_of(const u32x4& v, int j) {
  return j == 0 ? v.x : (j == 1 ? v.y : (j == 2 ? v.z : v.w));
}

template <int KIND>
__device__ __forceinline__ void load_tile(TileRegs<KIND>& r, const uint8_t* codes_kind, const uint16_t* scales_kind, int kt, int lane) {
  using TR = Traits<KIND>;
  const uint8_t* t = codes_kind + (int64_t)kt * TR::TILE_BYTES + lane * 16;
  r.c[0] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t));
  if constexpr ((KIND & 1) == kWide) {
    r.c[1] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t + 1024));
    // the third segment has entries for 48 lanes only (32 for the hybrid word); the lanes above re-read the last
    // entry (their k-slots are staged as zero activations, and every bit pattern decodes to a finite value)
    constexpr int last = (KIND & kH16) ? 31 : 47;
    r.c[2] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t + 2048 - (lane > last ? (lane - last) * 16 : 0)));
  }
  if constexpr (KIND == kNarrow) {
    const uint2 v = *reinterpret_cast<const uint2*>(scales_kind + (int64_t)kt * TR::SCALE_HALFS + (lane & 15) * TR::GPT);
    r.s[0] = v.x; r.s[1] = v.y;
  } else if constexpr (KIND == kWide || KIND == (kWide | kH16)) {
    const uint4 v = *reinterpret_cast<const uint4*>(scales_kind + (int64_t)kt * TR::SCALE_HALFS + (lane & 15) * TR::GPT);
    r.s[0] = v.x; r.s[1] = v.y; r.s[2] = v.z; r.s[3] = v.w;
  } else if constexpr (KIND == (kNarrow | kScale4)) {
    r.s[0] = scales_kind[(int64_t)kt * TR::SCALE_HALFS + (lane & 15)];  // the tile's four 4-bit fields of this row
  }
  // wide format with compressed scales: the fields sit in the code stream (see tile_scale_fields)
}

// Compressed scales of a wide k-tile: the field of group j is the low nibble of the group's last code byte
// (byte 21), which quarter 3 of the row holds in segment 1, halfword j, high byte.  Every lane fetches
// the four dwords of its row's quarter-3 lane.
template <int KIND>
__device__ __forceinline__ void tile_scale_fields(uint32_t (&f)[4], const TileRegs<KIND>& r, int lane) {
  if constexpr (KIND == (kWide | kScale4)) {
    const int src = (48 + (lane & 15)) * 4;
    f[0] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)r.c[1].x);
    f[1] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)r.c[1].y);
    f[2] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)r.c[1].z);
    f[3] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)r.c[1].w);
  } else if constexpr (KIND == (kWide | kH16 | kScale4)) {
    // hybrid word: the field of group j is the low 13 bits of the group's last word (word 9, scale mask
    // 0x1FFF of Table 1), which quarter 1 of the row holds in segment 2, halfword j
    const int src = (16 + (lane & 15)) * 4;
    f[0] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)r.c[2].x);
    f[1] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)r.c[2].y);
    f[2] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)r.c[2].z);
    f[3] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)r.c[2].w);
  }
}

// Constants of the decode, held in registers: bf16 128.0 twice, and the two-halfword state masks of
// the narrow (0x3F) and wide (0xF) formats (Table 1).
struct DecodeConsts {
  uint32_t c4300;
  uint32_t mask[3];  // narrow, wide, hybrid word
  float ssup[2];  // per-row super scale of each row tile the wavefront owns (compressed scales only)
};

// Weight fragment (8 bf16 integers 128 + state) of group j, k-step t.
template <int KIND>
__device__ __forceinline__ bf16x8 decode_frag(const TileRegs<KIND>& r, int j, int t, float al, float be_magic, uint32_t c4300, uint32_t mask) {
  uint4 o;
  if constexpr ((KIND & 1) == kNarrow) {
    // two clustered bytes -> two 15-bit codes (Alg. 3), side by side in one register
    const uint32_t d = dword_of(r.c[0], j);
    const float fa = __builtin_fmaf((float)((d >> (16 * t)) & 0xFFu), al, be_magic);
    const float fb = __builtin_fmaf((float)((d >> (16 * t + 8)) & 0xFFu), al, be_magic);
    const uint32_t yy = __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, fb), __builtin_bit_cast(uint32_t, fa), 0x05040100u);
    // states by the shift list [9,6,3,0], mask 0x3F (Table 1), for both codes at once
    o.x = and_or(yy >> 9, mask, c4300);
    o.y = and_or(yy >> 6, mask, c4300);
    o.z = and_or(yy >> 3, mask, c4300);
    o.w = and_or(yy, mask, c4300);
  } else if constexpr ((KIND & kH16) != 0) {
    // one 16-bit word w = (3,3,2) code | (3,4,2) code: seven 3-bit states at the shifts [13,11,9,6,4,2,0],
    // mask 0x7 (Table 1).  v = w | w << 18 puts a second copy of the word 18 bits up, so that the state
    // at shift s - 2 of the copy lands 16 bits above the state at shift s: one shift and one and-or cut
    // out two states.  (Bits 14 and 15 of the copy fall off the register; no state of the copy that is
    // used reaches them.)
    const uint32_t d = dword_of(r.c[t], j >> 1);
    const uint32_t w = (j & 1) ? (d >> 16) : (d & 0xFFFFu);
    const uint32_t v = w | (w << 18);
    o.x = and_or(v >> 13, mask, c4300);  // states 0, 1
    o.y = and_or(v >> 6, mask, c4300);   // states 3, 4
    o.z = and_or(v >> 2, mask, c4300);   // states 5, 6
    o.w = and_or(v >> 9, mask, c4300);   // state 2; the upper half is an unused k-slot (zero activation)
  } else {
    // two 8-bit codes of (L=4,N=3,S=2); shift list [4,2,0], mask 0xF (Table 1)
    const uint32_t d = dword_of(r.c[t], j >> 1);
    const uint32_t p = __builtin_amdgcn_perm(0u, d, (j & 1) ? 0x0C030C02u : 0x0C010C00u);  // {0,b,0,a}
    o.x = and_or(p >> 4, mask, c4300);
    o.y = and_or(p >> 2, mask, c4300);
    o.z = and_or(p, mask, c4300);
    o.w = p;      // unused k-slots (their activations are staged as zero): any finite pair; p is already in a register (bf16 values below 2^-126)
  }
  return __builtin_bit_cast(bf16x8, o);
}

// Scale of group j of the tile.  fp16 group scales; or, with compressed scales (Alg. 2 / Alg. 3, first line: field
// times the row's super scale), the field alone: the super scale is the same for every group of a row, so the
// kernels accumulate sum_g field_g * (group result) and multiply by it once, before the store.  For one-hot
// activations that is the same single rounding of field * s_super * (state - zp) as scaling group by group.
template <int KIND>
__device__ __forceinline__ float group_scale(const TileRegs<KIND>& r, const uint32_t (&fields)[4], int j) {
  if constexpr ((KIND & kScale4) == 0) {
    const uint32_t d = r.s[j >> 1];
    const uint16_t h = (uint16_t)((j & 1) ? (d >> 16) : (d & 0xFFFFu));
    return (float)__builtin_bit_cast(_Float16, h);
  } else if constexpr ((KIND & 1) == kNarrow) {
    return (float)((r.s[0] >> (4 * j)) & 0xFu);
  } else if constexpr ((KIND & kH16) != 0) {
    return (float)((fields[j >> 1] >> (16 * (j & 1))) & 0x1FFFu);
  } else {
    return (float)((fields[j >> 1] >> (16 * (j & 1) + 8)) & 0xFu);
  }
}

// Sum of the eight bf16 values of a fragment in fp32: four two-element dot products against (1, 1).
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ __forceinline__ float frag_sum(const uint4 o) {
  const bf16x2_t ones = __builtin_bit_cast(bf16x2_t, 0x3F803F80u);
  float sum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, o.x), ones, 0.f, false);
  sum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, o.y), ones, sum, false);
  sum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, o.z), ones, sum, false);
  sum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, o.w), ones, sum, false);
  return sum;
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);  // NaN stays NaN
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Stage the activations of `ng` packed groups as A-operand fragments and compute
// each group's accumulator start value  cneg * sum_k x[m][k].  Local group lg is
// packed group  pg0 + (lg / sg) * GPT + j0 + lg % sg  of the kind: with sg = GPT,
// j0 = 0 that is a run of whole k-tiles, otherwise groups j0..j0+sg-1 of
// consecutive k-tiles.
//   lds_x    : fragments, index ((lg*T + t)*4 + kq)*MRT + m, 16 bytes each
//   lds_cneg : fp32, index lg*(MT*16) + m
template <int KIND, int MT, int MR, bool META>
__device__ void stage_chunk(uint4* lds_x, float* lds_cneg, const SkinnyArgs& a, const uint16_t* x, int row_base, int rows_valid, int pg0,
                            int ng, int sg, int j0, int tid, int nthreads) {
  using TR = Traits<KIND>;
  constexpr int MRT = (MT == 1) ? MR : MT * 16;
  constexpr int U = 4;  // fragments requested per thread before the first is used
  const int nfrag = ng * TR::T * 4 * MRT;
  const int meta_base = ((KIND & 1) == kWide) ? a.groups_narrow : 0;
  // the workgroup size is a multiple of MRT, so a thread stages the same activation row every time
  const int m = tid % MRT;
  const bool row_ok = m < rows_valid;
  const uint16_t* xrow = x;
  if (row_ok) xrow = x + (a.sorted_rows ? (int64_t)a.sorted_rows[row_base + m] : (int64_t)(row_base + m)) * a.ldx;
  for (int f0 = tid; f0 < nfrag; f0 += nthreads * U) {
    uint4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int f = min(f0 + u * nthreads, nfrag - 1);  // clamped: the request is unconditional
      const int kq = (f / MRT) & 3;
      const int t = (f / (MRT * 4)) % TR::T;
      const int lg = f / (MRT * 4 * TR::T);
      const int pg = pg0 + (lg / sg) * TR::GPT + j0 + lg % sg;
      const int g = META ? a.meta[meta_base + pg] : min(pg, a.g_last);  // a group map exists only for mixed formats
      const uint16_t* xr = xrow + (int64_t)g * kGroup;
      if constexpr ((KIND & 1) == kNarrow) {
        v[u] = *reinterpret_cast<const uint4*>(xr + 16 * kq + 8 * t);
      } else {
        v[u] = load_chunk16(xr + frag_first_element<KIND>(kq, t));
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int f = f0 + u * nthreads;
      if (f < nfrag) {
        uint4 o = {0u, 0u, 0u, 0u};
        if (row_ok) {
          if constexpr ((KIND & 1) == kNarrow) {
            // the two codes of a k-step cover weights 16kq+8t+{0..3} and +{4..7}; slots
            // interleave them: {0,4,1,5,2,6,3,7}
            o.x = __builtin_amdgcn_perm(v[u].z, v[u].x, 0x05040100u);
            o.y = __builtin_amdgcn_perm(v[u].z, v[u].x, 0x07060302u);
            o.z = __builtin_amdgcn_perm(v[u].w, v[u].y, 0x05040100u);
            o.w = __builtin_amdgcn_perm(v[u].w, v[u].y, 0x07060302u);
          } else {
            o = frag_from_chunk<KIND>(v[u], (f / MRT) & 3, (f / (MRT * 4)) % TR::T);
          }
        }
        lds_x[f] = o;
      }
    }
  }
  __syncthreads();
  // start values for the rows that are really held; rows beyond them are never stored
  const int ncneg = ng * MRT;
  const float factor = a.cneg[KIND & 1];
  for (int i = tid; i < ncneg; i += nthreads) {
    const int m = i % MRT;
    const int lg = i / MRT;
    float sum = 0.f;
#pragma unroll
    for (int tk = 0; tk < TR::T * 4; ++tk) {
      const uint4 v = lds_x[(lg * TR::T * 4 + tk) * MRT + m];
      sum += frag_sum(v);
    }
    lds_cneg[lg * (MT * 16) + m] = factor * sum;
  }
  __syncthreads();
}

// Activation fragments and accumulator start values of one group, read from LDS.
template <int KIND, int MT, int MR>
struct GroupOperands {
  uint4 x[Traits<KIND>::T][MT];
  f32x4 cin[MT];
};

// Rows of the product are independent: an activation lane of a row that is not held only feeds a row
// of the product that is never stored.  With a single held row (MR = 1, MFMA 4x4x4) every lane of a
// 4x4 block reads the same fragment (an LDS broadcast, no lane masking): the four rows of the block's
// product are then equal and row 0 is the one that is used.  With up to four held rows (MR = 4) lane
// l of a block supplies row l % 4, and the block's product holds the four rows' results of each column.
template <int KIND, int MT, int MR>
__device__ __forceinline__ void read_group_operands(GroupOperands<KIND, MT, MR>& g, int lg, const uint4* lds_x, const float* lds_cneg, int lane) {
  using TR = Traits<KIND>;
  constexpr int MRT = (MT == 1) ? MR : MT * 16;
  const int kq = lane >> 4, m = lane & 15;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    // one held row: a 16-byte record per group and quarter whose first float is the start value; the other three
    // are never written and feed accumulator elements that are never read
    if constexpr (MR == 1) g.cin[mt] = *reinterpret_cast<const f32x4*>(lds_cneg + (lg * 4 + kq) * 4);
    else if constexpr (MR == 4) g.cin[mt] = *reinterpret_cast<const f32x4*>(lds_cneg + (lg * 4 + kq) * 4);  // the four held rows
    else g.cin[mt] = *reinterpret_cast<const f32x4*>(lds_cneg + (lg * MT + mt) * 16 + 4 * kq);
  }
#pragma unroll
  for (int t = 0; t < TR::T; ++t) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      if constexpr (MR == 16) g.x[t][mt] = lds_x[((lg * TR::T + t) * 4 + kq) * MRT + mt * 16 + m];
      else if constexpr (MR == 4) g.x[t][mt] = lds_x[((lg * TR::T + t) * 4 + kq) * 4 + (lane & 3)];  // row lane % 4 of the 4x4 block
      else g.x[t][mt] = lds_x[(lg * TR::T + t) * 4 + kq];
    }
  }
}

template <int KIND, int MT, int MR, int RT, int J0, int NJ>
__device__ __forceinline__ void process_tile(const TileRegs<KIND> (&r)[RT], int lg0, const uint4* lds_x, const float* lds_cneg, const float (&al)[RT],
                                             const float (&be)[RT], f32x4 (&acc)[RT][MT], int lane, DecodeConsts dc) {
  using TR = Traits<KIND>;
  GroupOperands<KIND, MT, MR> cur;
  uint32_t fields[RT][4];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) tile_scale_fields<KIND>(fields[rt], r[rt], lane);
#pragma unroll
  for (int j = J0; j < J0 + NJ; ++j) {
    const int lg = lg0 + (j - J0);
    read_group_operands<KIND, MT, MR>(cur, lg, lds_x, lds_cneg, lane);
    f32x4 P[RT][MT];
#pragma unroll
    for (int t = 0; t < TR::T; ++t) {
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        const bf16x8 wf = decode_frag<KIND>(r[rt], j, t, al[rt], be[rt], dc.c4300, dc.mask[(KIND & kH16) ? 2 : (KIND & 1)]);
        if constexpr (MR <= 4) {
          // two 4x4x4 steps: k-slots 0..3 and 4..7 of the fragment
          const u32x4 wv = __builtin_bit_cast(u32x4, wf);
          const uint4 xv = cur.x[t][0];
          f32x4 p = t == 0 ? cur.cin[0] : P[rt][0];
          p = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(bf16x4, u32x2{xv.x, xv.y}), __builtin_bit_cast(bf16x4, u32x2{wv.x, wv.y}), p, 0, 0, 0);
          p = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(bf16x4, u32x2{xv.z, xv.w}), __builtin_bit_cast(bf16x4, u32x2{wv.z, wv.w}), p, 0, 0, 0);
          P[rt][0] = p;
        } else {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            P[rt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, cur.x[t][mt]), wf, t == 0 ? cur.cin[mt] : P[rt][mt], 0, 0, 0);
        }
      }
    }
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const float s = group_scale<KIND>(r[rt], fields[rt], j);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        acc[rt][mt][0] = __builtin_fmaf(s, P[rt][mt][0], acc[rt][mt][0]);
        if (MR > 1) {
          acc[rt][mt][1] = __builtin_fmaf(s, P[rt][mt][1], acc[rt][mt][1]);
          acc[rt][mt][2] = __builtin_fmaf(s, P[rt][mt][2], acc[rt][mt][2]);
          acc[rt][mt][3] = __builtin_fmaf(s, P[rt][mt][3], acc[rt][mt][3]);
        }
      }
    }
  }
}

// Code Cluster offset plus 2^23 (exact: beta is an integer below 2^15).  The constant is made opaque so that
// the addition stays where it is written, below the first requests for code tiles: hoisted to the load of
// beta it would make everything after it wait for that load.
template <int RT>
__device__ __forceinline__ void add_code_magic(float (&be)[RT], const float (&be_raw)[RT]) {
  float magic = 8388608.f;
  asm volatile("" : "+v"(magic));
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) be[rt] = be_raw[rt] + magic;
}

// All k-tiles of one kind that belong to this workgroup, chunk by chunk: the
// activations of a chunk (KC k-tiles for each of the WK wavefronts along K) are
// staged in LDS, then every wavefront walks its own tiles with a register ring
// of D tiles in flight.
template <int KIND, int MT, int MR, int RT, bool META>
__device__ void run_kind_tiles(const SkinnyArgs& a, const uint8_t* (&codes_rt)[RT], const uint16_t* (&scales_rt)[RT], bool active,
                               const float (&al)[RT], const float (&be_raw)[RT], f32x4 (&acc)[RT][MT], uint4* lds_x, float* lds_cneg,
                               const uint16_t* x, int row_base, int rows_valid, int split, int wk, int lane, int tid, int nthreads,
                               DecodeConsts dc) {
  using TR = Traits<KIND>;
  // tiles in flight per wavefront: as many as the register budget of the instantiation allows (a refill is
  // requested one tile's work before it is needed, far less than a memory latency, so depth is what keeps
  // the memory system busy)
  constexpr int D = ((KIND & 1) == kNarrow) ? (MT == 1 ? (RT == 1 ? 8 : 4) : (RT == 1 ? 4 : 2)) : (RT == 1 ? 2 : 1);
  int A, B;
  split_range(a, KIND & 1, split, A, B);
  const int KC = a.KC[KIND & 1], CH = KC * a.WK;
  for (int c0 = A; c0 < B; c0 += CH) {
    const int cend = min(c0 + CH, B);
    const int k0 = min(c0 + wk * KC, cend), k1 = min(k0 + KC, cend);
    // Register ring of D tiles.  All loads inside the steady loop are unconditional (a load under a
    // branch would have to be waited for at once); only the last group of tiles is processed without
    // prefetching, and a ragged last group re-reads its last tile.
    TileRegs<KIND> buf[D][RT];
    const int n = k1 - k0, ngroups = (n + D - 1) / D;
    if (active && n > 0) {
#pragma unroll
      for (int i = 0; i < D; ++i) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) load_tile<KIND>(buf[i][rt], codes_rt[rt], scales_rt[rt], k0 + min(i, n - 1), lane);
      }
    }
    __syncthreads();  // the previous chunk's fragments are no longer read
    stage_chunk<KIND, MT, MR, META>(lds_x, lds_cneg, a, x, row_base, rows_valid, c0 * TR::GPT, (cend - c0) * TR::GPT, TR::GPT, 0, tid, nthreads);
    float be[RT];
    add_code_magic<RT>(be, be_raw);
    if (active && n > 0) {
      for (int j = 0; j + 1 < ngroups; ++j) {
#pragma unroll
        for (int i = 0; i < D; ++i) {
          process_tile<KIND, MT, MR, RT, 0, TR::GPT>(buf[i], (k0 + j * D + i - c0) * TR::GPT, lds_x, lds_cneg, al, be, acc, lane, dc);
#pragma unroll
          for (int rt = 0; rt < RT; ++rt)
            load_tile<KIND>(buf[i][rt], codes_rt[rt], scales_rt[rt], k0 + min((j + 1) * D + i, n - 1), lane);
        }
      }
      const int jl = ngroups - 1;
#pragma unroll
      for (int i = 0; i < D; ++i) {
        if (jl * D + i < n)
          process_tile<KIND, MT, MR, RT, 0, TR::GPT>(buf[i], (k0 + jl * D + i - c0) * TR::GPT, lds_x, lds_cneg, al, be, acc, lane, dc);
      }
    }
  }
}

// When many activation rows are held, the fragments of a whole k-tile do not fit
// in LDS next to other workgroups: every wavefront along K then owns one k-tile
// per step and its groups are staged SG at a time.
template <int KIND, int MT, int MR, int RT, int SG, int J0, bool META>
struct SubSteps {
  static __device__ __forceinline__ void run(const SkinnyArgs& a, const TileRegs<KIND> (&r)[RT], bool has, const float (&al)[RT],
                                             const float (&be)[RT], f32x4 (&acc)[RT][MT], uint4* lds_x, float* lds_cneg, const uint16_t* x,
                                             int row_base, int rows_valid, int c0, int ntiles, int wk, int lane, int tid, int nthreads,
                                             DecodeConsts dc) {
    using TR = Traits<KIND>;
    if constexpr (J0 < TR::GPT) {
      __syncthreads();  // the previous step's fragments are no longer read
      stage_chunk<KIND, MT, MR, META>(lds_x, lds_cneg, a, x, row_base, rows_valid, c0 * TR::GPT, ntiles * SG, SG, J0, tid, nthreads);
      if (has) process_tile<KIND, MT, MR, RT, J0, SG>(r, wk * SG, lds_x, lds_cneg, al, be, acc, lane, dc);
      SubSteps<KIND, MT, MR, RT, SG, J0 + SG, META>::run(a, r, has, al, be, acc, lds_x, lds_cneg, x, row_base, rows_valid, c0, ntiles, wk, lane, tid,
                                                   nthreads, dc);
    }
  }
};

template <int KIND, int MT, int MR, int RT, int SG, bool META>
__device__ void run_kind_groups(const SkinnyArgs& a, const uint8_t* (&codes_rt)[RT], const uint16_t* (&scales_rt)[RT], bool active,
                                const float (&al)[RT], const float (&be_raw)[RT], f32x4 (&acc)[RT][MT], uint4* lds_x, float* lds_cneg,
                                const uint16_t* x, int row_base, int rows_valid, int split, int wk, int lane, int tid, int nthreads,
                                DecodeConsts dc) {
  using TR = Traits<KIND>;
  const int tiles = a.tiles[KIND & 1];
  int A, B;
  split_range(a, KIND & 1, split, A, B);
  TileRegs<KIND> cur[RT], nxt[RT];
  if (active && A + wk < B) {
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) load_tile<KIND>(cur[rt], codes_rt[rt], scales_rt[rt], A + wk, lane);
  }
  float be[RT];
  add_code_magic<RT>(be, be_raw);
  for (int c0 = A; c0 < B; c0 += a.WK) {
    const int ntiles = min(a.WK, B - c0);
    const bool has = active && wk < ntiles;
    const bool has_next = active && c0 + a.WK + wk < B;
    if (has_next) {
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) load_tile<KIND>(nxt[rt], codes_rt[rt], scales_rt[rt], c0 + a.WK + wk, lane);
    }
    SubSteps<KIND, MT, MR, RT, SG, 0, META>::run(a, cur, has, al, be, acc, lds_x, lds_cneg, x, row_base, rows_valid, c0, ntiles, wk, lane, tid, nthreads,
                                           dc);
    if (has_next) {
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) cur[rt] = nxt[rt];
    }
  }
}

// ---- one held row (M = 1): wavefront-private staging ------------------------
// Every wavefront stages the activations of its own k-tiles in a private LDS
// region, so no workgroup barrier is needed before the contraction and the
// wavefronts of a workgroup drift apart instead of waiting for each other.
//   lds_x   : fragments, index (lg*T + t)*4 + kq, 16 bytes each
//   lds_cneg: one float per group and quarter, index lg*4 + kq
template <int KIND, bool META>
__device__ __forceinline__ void stage_private(uint4* lds_x, float* lds_cneg, const SkinnyArgs& a, const uint16_t* xr, int pg0, int ng, int lane) {
  using TR = Traits<KIND>;
  const int meta_base = ((KIND & 1) == kWide) ? a.groups_narrow : 0;
  const int nfrag = ng * TR::T * 4;
  for (int f = lane; f < nfrag; f += 64) {
    const int kq = f & 3;
    const int t = (f >> 2) % TR::T;
    const int lg = f / (4 * TR::T);
    const int pg = pg0 + lg;
    const int g = META ? a.meta[meta_base + pg] : min(pg, a.g_last);  // a group map exists only for mixed formats
    const uint16_t* xg = xr + (int64_t)g * kGroup;
    uint4 o = {0u, 0u, 0u, 0u};
    if constexpr ((KIND & 1) == kNarrow) {
      const uint4 v = *reinterpret_cast<const uint4*>(xg + 16 * kq + 8 * t);
      o.x = __builtin_amdgcn_perm(v.z, v.x, 0x05040100u);
      o.y = __builtin_amdgcn_perm(v.z, v.x, 0x07060302u);
      o.z = __builtin_amdgcn_perm(v.w, v.y, 0x05040100u);
      o.w = __builtin_amdgcn_perm(v.w, v.y, 0x07060302u);
    } else {
      o = frag_from_chunk<KIND>(load_chunk16(xg + frag_first_element<KIND>(kq, t)), kq, t);
    }
    lds_x[f] = o;
    if constexpr ((KIND & 1) == kNarrow) {
      // the two fragments of a quarter (k-steps 0 and 1) sit 4 lanes apart: add them with one DPP step
      float sum = frag_sum(o);
      sum += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, sum), 0x104, 0xF, 0xF, true));  // + lane 4 up: the other k-step
      if ((f & 4) == 0) lds_cneg[(lg * 4 + kq) * 4] = a.cneg[KIND & 1] * sum;
    }
  }
  if constexpr ((KIND & 1) == kWide) {
    // three fragments per quarter: one lane per (group, quarter) adds them up from LDS (same wavefront: LDS
    // operations stay in order)
    __builtin_amdgcn_wave_barrier();
    for (int e = lane; e < ng * 4; e += 64) {
      const int lg = e >> 2, kq = e & 3;
      float sum = 0.f;
#pragma unroll
      for (int t = 0; t < TR::T; ++t) {
        const uint4 v = lds_x[(lg * TR::T + t) * 4 + kq];
        sum += frag_sum(v);
      }
      lds_cneg[e * 4] = a.cneg[KIND & 1] * sum;
    }
  }
  __builtin_amdgcn_wave_barrier();
}

// Narrow format, one held row: the same staging in two halves, so that the activation requests can
// go out before the (much slower) code tiles are requested and the conversion to fragments overlaps the
// tiles' flight.  A lane holds up to kPrivFrags fragments of a chunk (6 KiB region / 16 bytes / 64 lanes).
constexpr int kPrivFrags = 6;
template <bool META>
__device__ __forceinline__ void stage_private_request(uint4 (&v)[kPrivFrags], const int32_t* meta, const uint16_t* xr, int pg0, int ng, int g_last, int lane) {
  const int nfrag = ng * 8;
#pragma unroll
  for (int i = 0; i < kPrivFrags; ++i) {
    if (64 * i >= nfrag) break;  // wavefront-uniform
    const int f = min(lane + 64 * i, nfrag - 1);
    const int pg = pg0 + (f >> 3);
    const uint32_t g = META ? (uint32_t)meta[pg] : (uint32_t)min(pg, g_last);
    // element offset: group * 64 + quarter (f & 3) * 16 + k-step ((f >> 2) & 1) * 8, in 32-bit arithmetic (K < 2^31)
    const uint32_t off = (g << 6) | ((uint32_t)(f & 3) << 4) | ((uint32_t)(f & 4) << 1);
    v[i] = *reinterpret_cast<const uint4*>(xr + off);
  }
}
__device__ __forceinline__ void stage_private_finish(const uint4 (&v)[kPrivFrags], uint4* lds_x, float* lds_cneg, float cneg, int ng, int lane) {
  const int nfrag = ng * 8;
#pragma unroll
  for (int i = 0; i < kPrivFrags; ++i) {
    if (64 * i >= nfrag) break;  // wavefront-uniform
    const int f = lane + 64 * i;
    if (f < nfrag) {
      uint4 o;
      o.x = __builtin_amdgcn_perm(v[i].z, v[i].x, 0x05040100u);
      o.y = __builtin_amdgcn_perm(v[i].z, v[i].x, 0x07060302u);
      o.z = __builtin_amdgcn_perm(v[i].w, v[i].y, 0x05040100u);
      o.w = __builtin_amdgcn_perm(v[i].w, v[i].y, 0x07060302u);
      lds_x[f] = o;
      float sum = frag_sum(o);
      sum += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, sum), 0x104, 0xF, 0xF, true));  // + lane 4 up: the other k-step
      if ((f & 4) == 0) lds_cneg[((f >> 3) * 4 + (f & 3)) * 4] = cneg * sum;
    }
  }
  __builtin_amdgcn_wave_barrier();
}

// One held row.  The whole matrix is only a few microseconds of memory traffic, so the depth of the
// register ring decides how much of it is in flight: D tiles per wavefront are requested up front
// (8 for the narrow format: with ~8 k-tiles per wavefront that is all of them), each refilled as soon as
// it has been consumed.
template <int KIND, int RT, bool META>
__device__ void run_kind_private(const SkinnyArgs& a, const uint8_t* (&codes_rt)[RT], const uint16_t* (&scales_rt)[RT], bool active,
                                 const float (&al)[RT], const float (&be_raw)[RT], f32x4 (&acc)[RT][1], uint4* lds_x, float* lds_cneg,
                                 const uint16_t* xr, int split, int wk, int lane, DecodeConsts dc) {
  using TR = Traits<KIND>;
  constexpr int D = ((KIND & 1) == kNarrow) ? (RT == 1 ? 8 : 4) : (RT == 1 ? 2 : 1);
  if (!active) return;
  int A, B;
  split_range(a, KIND & 1, split, A, B);
  int k0, k1;
  wave_range(a, KIND & 1, split, A, wk, k0, k1);
  const int CT = a.KC[KIND & 1];  // k-tiles the private region holds
  for (int c0 = k0; c0 < k1; c0 += CT) {
    const int cend = min(c0 + CT, k1);
    TileRegs<KIND> buf[D][RT];
    const int n = cend - c0, ngroups = (n + D - 1) / D;
    uint4 xv[kPrivFrags];
    if constexpr ((KIND & 1) == kNarrow) stage_private_request<META>(xv, a.meta, xr, c0 * TR::GPT, n * TR::GPT, a.g_last, lane);
#pragma unroll
    for (int i = 0; i < D; ++i) {
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) load_tile<KIND>(buf[i][rt], codes_rt[rt], scales_rt[rt], c0 + min(i, n - 1), lane);
    }
    if constexpr ((KIND & 1) == kNarrow) stage_private_finish(xv, lds_x, lds_cneg, a.cneg[kNarrow], n * TR::GPT, lane);
    else stage_private<KIND, META>(lds_x, lds_cneg, a, xr, c0 * TR::GPT, n * TR::GPT, lane);
    // the Code Cluster offset plus 2^23 (exact: beta is an integer below 2^15); added only here so that
    // nothing above waits for the per-row parameters to arrive
    float be[RT];
    add_code_magic<RT>(be, be_raw);
    for (int j = 0; j + 1 < ngroups; ++j) {
#pragma unroll
      for (int i = 0; i < D; ++i) {
        process_tile<KIND, 1, 1, RT, 0, TR::GPT>(buf[i], (j * D + i) * TR::GPT, lds_x, lds_cneg, al, be, acc, lane, dc);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) load_tile<KIND>(buf[i][rt], codes_rt[rt], scales_rt[rt], c0 + min((j + 1) * D + i, n - 1), lane);
      }
    }
    const int jl = ngroups - 1;
#pragma unroll
    for (int i = 0; i < D; ++i) {
      if (jl * D + i < n) process_tile<KIND, 1, 1, RT, 0, TR::GPT>(buf[i], (jl * D + i) * TR::GPT, lds_x, lds_cneg, al, be, acc, lane, dc);
    }
    __builtin_amdgcn_wave_barrier();  // the region is rewritten by the next chunk
  }
}

template <int KIND, int MT, int MR, int RT, bool META>
__device__ __forceinline__ void run_kind(const SkinnyArgs& a, const uint8_t* (&codes_rt)[RT], const uint16_t* (&scales_rt)[RT], bool active,
                                         const float (&al)[RT], const float (&be)[RT], f32x4 (&acc)[RT][MT], uint4* lds_x, float* lds_cneg,
                                         const uint16_t* x, int row_base, int rows_valid, int split, int wk, int lane, int tid, int nthreads,
                                         DecodeConsts dc) {
  using TR = Traits<KIND>;
  if constexpr (MT >= 2) {
    const int sg = a.SG[KIND & 1];
    if (sg != TR::GPT) {
      if (sg == 1)
        run_kind_groups<KIND, MT, MR, RT, 1, META>(a, codes_rt, scales_rt, active, al, be, acc, lds_x, lds_cneg, x, row_base, rows_valid, split, wk, lane,
                                             tid, nthreads, dc);
      else if (sg == 2)
        run_kind_groups<KIND, MT, MR, RT, 2, META>(a, codes_rt, scales_rt, active, al, be, acc, lds_x, lds_cneg, x, row_base, rows_valid, split, wk, lane,
                                             tid, nthreads, dc);
      else
        run_kind_groups<KIND, MT, MR, RT, 4, META>(a, codes_rt, scales_rt, active, al, be, acc, lds_x, lds_cneg, x, row_base, rows_valid, split, wk, lane,
                                             tid, nthreads, dc);
      return;
    }
  }
  run_kind_tiles<KIND, MT, MR, RT, META>(a, codes_rt, scales_rt, active, al, be, acc, lds_x, lds_cneg, x, row_base, rows_valid, split, wk, lane, tid,
                                   nthreads, dc);
}

// Threads a workgroup of ccq_skinny_kernel may have (the register budget per lane follows from it).  The wide
// format with compressed scales holds the tile's scale fields besides its eight code registers and does not fit
// the 128 registers of a 1024-thread workgroup.
constexpr int skinny_max_threads(int MT, int MR, int FM, int SM) {
  return MT == 4 ? 256 : ((MT == 2 || MR == 1 || (FM == 2 && SM == 1)) ? 512 : 1024);
}

// FM: formats present (1 narrow, 2 wide, 3 both, 4 the hybrid word in place of the wide kind).
// SM: scale mode (0 fp16 group scales, 1 compressed scales)
template <int MT, int MR, int RT, int FM, int SM>
__global__ void __launch_bounds__(skinny_max_threads(MT, MR, FM, SM)) ccq_skinny_kernel(const SkinnyArgs a) {
  constexpr int KN = kNarrow | (SM << 1), KW = kWide | (SM << 1) | (FM == 4 ? kH16 : 0);
  constexpr bool HAS_N = FM == 1 || FM == 3, HAS_W = FM >= 2;
  extern __shared__ __align__(16) unsigned char smem[];
  // Fetch the whole argument block now, in one batch of scalar loads: left to itself the compiler loads it
  // piecemeal behind the early branches, four dependent round trips (about 2.5 us) before the first request
  // for weights goes out.
  asm volatile("" ::"s"(a.codes), "s"(a.scales), "s"(a.alpha), "s"(a.beta), "s"(a.meta), "s"(a.scale_super), "s"(a.x), "s"(a.y), "s"(a.partial), "s"(a.sorted_rows),
               "s"(a.expert_offsets), "s"(a.ldx), "s"(a.ldy), "s"(a.codes_stride), "s"(a.scales_stride), "s"(a.ab_stride), "s"(a.row_tile_bytes),
               "s"(a.row_tile_scale_halfs), "s"(a.M), "s"(a.N), "s"(a.row_tiles), "s"(a.tiles[0]), "s"(a.tiles[1]), "s"(a.WR), "s"(a.WK),
               "s"(a.S), "s"(a.inv_WR));
  const int tid = threadIdx.x, nthreads = blockDim.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps tile indices and base pointers in scalar registers
  const int wk = (wave * a.inv_WR) >> 16, wr = wave - wk * a.WR;
  const int split = blockIdx.y;
  int e = blockIdx.z;
  if (a.n_active > 0) {
    // read straight from the argument segment (a uniform scalar load): indexing the by-value copy with a run-time
    // index would make the compiler keep the whole argument block in scratch memory
    typedef const __attribute__((address_space(4))) uint16_t* KernargU16;
    typedef const __attribute__((address_space(4))) char* KernargBytes;
    KernargBytes args = (KernargBytes)__builtin_amdgcn_kernarg_segment_ptr();
    e = ((KernargU16)(args + offsetof(SkinnyArgs, active_ids)))[blockIdx.z];
  }

  int off0 = 0, Me = a.M;
  if (a.expert_offsets) {
    off0 = a.expert_offsets[e];
    Me = a.expert_offsets[e + 1] - off0;
  }
  if (Me <= 0) return;

  const uint8_t* codes = a.codes + (int64_t)e * a.codes_stride;
  const uint16_t* scales = reinterpret_cast<const uint16_t*>(reinterpret_cast<const uint8_t*>(a.scales) + (int64_t)e * a.scales_stride);
  const float* alpha = a.alpha ? reinterpret_cast<const float*>(reinterpret_cast<const uint8_t*>(a.alpha) + (int64_t)e * a.ab_stride) : nullptr;
  const float* beta = a.beta ? reinterpret_cast<const float*>(reinterpret_cast<const uint8_t*>(a.beta) + (int64_t)e * a.ab_stride) : nullptr;

  const int rtile0 = (blockIdx.x * a.WR + wr) * RT;
  const bool active = rtile0 < a.row_tiles;
  const uint8_t* codes_n[RT];
  const uint8_t* codes_w[RT];
  const uint16_t* scales_n[RT];
  const uint16_t* scales_w[RT];
  float al[RT], be[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int rtile = min(rtile0 + rt, a.row_tiles - 1);  // a ragged last pair re-reads the last tile; its result is not stored
    codes_n[rt] = codes + (int64_t)rtile * a.row_tile_bytes;
    codes_w[rt] = codes_n[rt] + (int64_t)a.tiles[kNarrow] * kNarrowTileBytes;
    scales_n[rt] = scales + (int64_t)rtile * a.row_tile_scale_halfs;
    scales_w[rt] = scales_n[rt] + (int64_t)a.tiles[kNarrow] * Traits<KN>::SCALE_HALFS;
    al[rt] = 0.f;
    be[rt] = 0.f;
    if (HAS_N && active) {
      al[rt] = alpha[min(rtile * 16 + (lane & 15), a.n_last)];
      be[rt] = beta[min(rtile * 16 + (lane & 15), a.n_last)];
    }
    // + 2^23 (exact: beta is an integer below 2^15), which puts the rounded code into the low mantissa bits, is
    // added later, after the first tiles have been requested: nothing before that waits for these two loads
  }

  uint4* lds_x = reinterpret_cast<uint4*>(smem);
  const int frag_cap = a.frag_cap;
  float* lds_cneg = reinterpret_cast<float*>(smem + (size_t)frag_cap * 16);
  // the compiler must see these as register values, not literals, to select v_and_or_b32
  DecodeConsts dc = {0x43004300u, {0x003F003Fu, 0x000F000Fu, 0x00070007u}, {0.f, 0.f}};
  asm volatile("" : "+v"(dc.c4300), "+s"(dc.mask[0]), "+s"(dc.mask[1]), "+s"(dc.mask[2]));
  if constexpr (SM == 1) {
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int rtile = min(rtile0 + rt, a.row_tiles - 1);
      // expert e's super scales: half the byte stride of alpha / beta (fp16 against fp32)
      const uint16_t* ssup = reinterpret_cast<const uint16_t*>(reinterpret_cast<const uint8_t*>(a.scale_super) + (int64_t)e * (a.ab_stride / 2));
      dc.ssup[rt] = (float)__builtin_bit_cast(_Float16, ssup[min(rtile * 16 + (lane & 15), a.n_last)]);
    }
  }

  for (int m0 = 0; m0 < Me; m0 += MT * 16) {
    const int rows_valid = min(MT * 16, Me - m0);
    f32x4 acc[RT][MT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[rt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    if constexpr (MR == 1) {
      // one held row: private staging region of this wavefront (fragments, then start values)
      uint4* my_x = lds_x + (size_t)wave * (a.frag_cap + a.cneg_cap / 4);
      float* my_cneg = reinterpret_cast<float*>(my_x + a.frag_cap);
      const uint16_t* xr = a.x + (a.sorted_rows ? (int64_t)a.sorted_rows[off0 + m0] : (int64_t)(off0 + m0)) * a.ldx;
      if constexpr (HAS_N) run_kind_private<KN, RT, FM == 3>(a, codes_n, scales_n, active, al, be, acc, my_x, my_cneg, xr, split, wk, lane, dc);
      if constexpr (HAS_W) run_kind_private<KW, RT, FM == 3>(a, codes_w, scales_w, active, al, be, acc, my_x, my_cneg, xr, split, wk, lane, dc);
    } else {
      if constexpr (HAS_N)
        run_kind<KN, MT, MR, RT, FM == 3>(a, codes_n, scales_n, active, al, be, acc, lds_x, lds_cneg, a.x, off0 + m0, rows_valid, split, wk, lane, tid,
                                      nthreads, dc);
      if constexpr (HAS_W)
        run_kind<KW, MT, MR, RT, FM == 3>(a, codes_w, scales_w, active, al, be, acc, lds_x, lds_cneg, a.x, off0 + m0, rows_valid, split, wk, lane, tid,
                                    nthreads, dc);
    }

    if constexpr (MR == 1) {
      // every lane holds the partial sum of its row over its own quarter: add the four quarters (fixed order)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        float v = acc[rt][0][0];
        v += __shfl_xor(v, 16);
        v += __shfl_xor(v, 32);
        acc[rt][0][0] = v;
      }
    }
    // ---- reduce the K-splits of this workgroup through LDS (fixed order) ----
    if (a.WK > 1) {
      __syncthreads();
      if constexpr (MR == 1) {
        // one held row: only element 0 of lanes 0..15 carries a result
        float* red = reinterpret_cast<float*>(smem);
        if (wk > 0 && lane < 16) {
#pragma unroll
          for (int rt = 0; rt < RT; ++rt) red[(((wk - 1) * a.WR + wr) * RT + rt) * 16 + lane] = acc[rt][0][0];
        }
        __syncthreads();
        if (wk == 0 && lane < 16) {
          for (int k = 1; k < a.WK; ++k) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) acc[rt][0][0] += red[(((k - 1) * a.WR + wr) * RT + rt) * 16 + lane];
          }
        }
      } else {
        f32x4* red = reinterpret_cast<f32x4*>(smem);
        if (wk > 0) {
#pragma unroll
          for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) red[((((wk - 1) * a.WR + wr) * RT + rt) * MT + mt) * 64 + lane] = acc[rt][mt];
        }
        __syncthreads();
        if (wk == 0) {
          for (int k = 1; k < a.WK; ++k) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
              for (int mt = 0; mt < MT; ++mt) {
                const f32x4 v = red[((((k - 1) * a.WR + wr) * RT + rt) * MT + mt) * 64 + lane];
                acc[rt][mt] += v;
              }
          }
        }
      }
    }

    // ---- store: bf16 result, or fp32 partials when K is also split over workgroups ----
    if (wk == 0 && active) {
      const int kq = lane >> 4;
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        if (rtile0 + rt >= a.row_tiles) continue;
        if constexpr (SM == 1) acc[rt][0] *= dc.ssup[rt];  // compressed scales: the row's super scale, once (see group_scale)
        if constexpr (SM == 1 && MT > 1) {
#pragma unroll
          for (int mt = 1; mt < MT; ++mt) acc[rt][mt] *= dc.ssup[rt];
        }
        const int n = (rtile0 + rt) * 16 + (lane & 15);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
          for (int r = 0; r < (MR == 1 ? 1 : 4); ++r) {
            const int m = mt * 16 + 4 * kq + r;
            if (m < rows_valid && n <= a.n_last) {
              const int64_t prow = (int64_t)off0 + m0 + m;
              if (a.S > 1) __builtin_nontemporal_store(acc[rt][mt][r], &a.partial[((int64_t)split * a.M + prow) * a.N + n]);
              else a.y[prow * a.ldy + n] = f32_to_bf16_rne(acc[rt][mt][r]);
            }
          }
        }
      }
    }
    if (m0 + MT * 16 < Me) __syncthreads();
  }
}

// y[p][n] = bf16( sum_s partial[s][p][n] ), splits added in index order.  `partial` rows hold Npad (a multiple of 16)
// floats of which the first N are results.  Four consecutive columns per thread (partial and y rows are 16-byte
// aligned); all S requests of a thread go out before the first add.
template <int SMAX>
__global__ void __launch_bounds__(256) ccq_reduce_splits_kernel(const float* partial, uint16_t* y, int64_t ldy, int rows, int N, int Npad, int S) {
  const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  const int64_t total = (int64_t)rows * Npad;
  if (i >= total) return;
  // the requests first (every quad below `total` exists, padded columns included); the row and column of the quad are
  // worked out while they are on their way
  f32x4 v[SMAX];
#pragma unroll
  for (int s = 0; s < SMAX; ++s) v[s] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(partial + (int64_t)min(s, S - 1) * total + i));
  __builtin_amdgcn_sched_barrier(0);
  int64_t p, n;
  if (total < ((int64_t)1 << 31)) {
    p = (uint32_t)i / (uint32_t)Npad;
    n = (uint32_t)i % (uint32_t)Npad;
  } else {
    p = i / Npad;
    n = i % Npad;
  }
  if (n >= N) return;
  f32x4 sum = v[0];
#pragma unroll
  for (int s = 1; s < SMAX; ++s)
    if (s < S) sum += v[s];
  uint16_t* dst = y + p * ldy + n;
  if (n + 4 <= N) {
    uint2 o;
    o.x = (uint32_t)f32_to_bf16_rne(sum[0]) | ((uint32_t)f32_to_bf16_rne(sum[1]) << 16);
    o.y = (uint32_t)f32_to_bf16_rne(sum[2]) | ((uint32_t)f32_to_bf16_rne(sum[3]) << 16);
    *reinterpret_cast<uint2*>(dst) = o;
  } else {
    // the last, partly real quad of a row whose length is not a multiple of four: columns from N on are not touched
#pragma unroll
    for (int c = 0; c < 3; ++c)
      if (n + c < N) dst[c] = f32_to_bf16_rne(sum[c]);
  }
}

// ---- 17 to 128 activation rows, dense: the per-row-tile contraction fed by a per-group activation tile ------
// With several 16-row activation tiles held, staging whole k-tiles of activations (above) exposes a memory
// latency, a gather and two barriers per chunk.  Here a workgroup of NW = four or eight wavefronts (as many 16-row
// weight tiles; the first four wavefronts copy the activations) walks K one 64-weight group per step: the 16 MT x 64 activation tile of the step after next is requested, the
// one of the next step is written to the other LDS buffer as MFMA A fragments (already in k-slot order) together
// with the accumulator start values -(128 + zp) sum_k x (the lanes that hold one row's fragments sit side by
// side, so the sum is a few lane shuffles), and the current one is multiplied.  The weights never pass through LDS
// and are decoded exactly as in the kernels above (bf16 integers, scale applied after the group's contraction),
// so the results are those of the per-row-tile kernel, not bf16-rounded weights.
struct RowsArgs {
  const uint8_t* codes;
  const uint16_t* scales;
  const float* alpha;
  const float* beta;
  const int32_t* meta;
  const uint16_t* scale_super;
  const uint16_t* x;
  uint16_t* y;
  float* partial;
  int64_t ldx, ldy;
  int64_t row_tile_bytes, row_tile_scale_halfs;
  int32_t M, N, row_tiles, m_blocks;  // N: rows of the device layout, the row stride of `partial`
  int32_t tiles[2];
  int32_t groups_narrow;
  int32_t g_last, n_last;  // last real group of K and last real output row (see SkinnyArgs)
  int32_t sq[2], sr[2];  // K shares, as in SkinnyArgs
  float cneg[2];
};

template <int MT, int FM, int SM, int NW>
__global__ void __launch_bounds__(64 * NW, 8 / NW) ccq_rows_kernel(const RowsArgs a) {
  constexpr int KN = kNarrow | (SM << 1), KW = kWide | (SM << 1) | (FM == 4 ? kH16 : 0);
  constexpr bool HAS_N = FM == 1 || FM == 3, HAS_W = FM >= 2, META = FM == 3;
  constexpr int MRT = 16 * MT;
  constexpr int RS = HAS_W ? 13 : 9;  // 16-byte fragments per LDS row: 8 or 12, plus one of padding (odd: conflict-free)
  constexpr int NPN = (MRT + 31) / 32, NPW = MRT / 16;  // staging passes: 8 lanes per row (narrow), 16 lanes per row (wide kinds)
  constexpr int NP = HAS_W ? NPW : NPN;
  extern __shared__ __align__(16) unsigned char smem[];
  uint4* As = reinterpret_cast<uint4*>(smem);                          // [2][MRT][RS]
  float* Cn = reinterpret_cast<float*>(smem + (size_t)2 * MRT * RS * 16);  // [2][MRT]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m_block = blockIdx.x % a.m_blocks, n_block = blockIdx.x / a.m_blocks;
  const int split = blockIdx.y;
  const int m0 = m_block * MRT;
  const int kq = lane >> 4, nl = lane & 15;

  int tA[2], tB[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    tA[k] = split * a.sq[k] + min(split, a.sr[k]);
    tB[k] = tA[k] + a.sq[k] + (split < a.sr[k] ? 1 : 0);
  }

  const int rtile_raw = n_block * NW + wave;
  const bool stager = wave < 4;  // the first four wavefronts copy the activation tile (wave-uniform)
  const bool active = rtile_raw < a.row_tiles;
  const int rtile = min(rtile_raw, a.row_tiles - 1);  // a ragged last block re-decodes the last tile; nothing of it is stored
  const uint8_t* codes_n = a.codes + (int64_t)rtile * a.row_tile_bytes;
  const uint8_t* codes_w = codes_n + (int64_t)a.tiles[kNarrow] * kNarrowTileBytes;
  const uint16_t* scales_n = a.scales + (int64_t)rtile * a.row_tile_scale_halfs;
  const uint16_t* scales_w = scales_n + (int64_t)a.tiles[kNarrow] * Traits<KN>::SCALE_HALFS;
  float al = 0.f, be_raw = 0.f;
  if constexpr (HAS_N) {
    al = a.alpha[min(rtile * 16 + nl, a.n_last)];
    be_raw = a.beta[min(rtile * 16 + nl, a.n_last)];
  }
  DecodeConsts dc = {0x43004300u, {0x003F003Fu, 0x000F000Fu, 0x00070007u}, {0.f, 0.f}};
  float magic = 8388608.f;
  asm volatile("" : "+v"(dc.c4300), "+s"(dc.mask[0]), "+s"(dc.mask[1]), "+s"(dc.mask[2]), "+v"(magic));
  if constexpr (SM == 1) dc.ssup[0] = (float)__builtin_bit_cast(_Float16, a.scale_super[min(rtile * 16 + nl, a.n_last)]);

  // ---- activation staging: thread -> (row, fragment) -------------------------------------------------------
  // narrow: 8 lanes per row, lane c holds elements 8c .. 8c+7 = fragment (quarter c / 2, k-step c % 2);
  // wide kinds: 16 lanes per row, lane c < 12 holds fragment (quarter c % 4, k-step c / 4), the others nothing
  const uint16_t* xrow[NP];
  bool xvalid[NP];
  auto rows_of = [&](int lpr, int u) -> int { return tid / lpr + u * (256 / lpr); };
  auto request = [&](uint4 (&v)[NP], int kind, int g) {
    if (HAS_N && (!HAS_W || kind == kNarrow)) {
#pragma unroll
      for (int u = 0; u < NPN; ++u) v[u] = *reinterpret_cast<const uint4*>(xrow[u] + (int64_t)g * kGroup + (tid & 7) * 8);
    } else {
      const int c = min(tid & 15, 11);
#pragma unroll
      for (int u = 0; u < NPW; ++u) v[u] = load_chunk16(xrow[u] + (int64_t)g * kGroup + frag_first_element<KW>(c & 3, c >> 2));
    }
  };
  // xrow / xvalid depend on the lanes-per-row of the kind; a mixed matrix switches once, from narrow to wide
  auto set_rows = [&](int lpr) {
#pragma unroll
    for (int u = 0; u < NP; ++u) {
      const int m = rows_of(lpr, u);
      xvalid[u] = m < MRT && m0 + m < a.M;
      xrow[u] = a.x + (int64_t)min(m0 + min(m, MRT - 1), a.M - 1) * a.ldx;
    }
  };
  auto commit = [&](int buf, const uint4 (&v)[NP], int kind) {
    uint4* dst = As + (size_t)buf * MRT * RS;
    float* cn = Cn + buf * MRT;
    if (HAS_N && (!HAS_W || kind == kNarrow)) {
      const int c = tid & 7;
#pragma unroll
      for (int u = 0; u < NPN; ++u) {
        const int m = rows_of(8, u);
        uint4 o = {0u, 0u, 0u, 0u};
        if (xvalid[u]) {
          o.x = __builtin_amdgcn_perm(v[u].z, v[u].x, 0x05040100u);
          o.y = __builtin_amdgcn_perm(v[u].z, v[u].x, 0x07060302u);
          o.z = __builtin_amdgcn_perm(v[u].w, v[u].y, 0x05040100u);
          o.w = __builtin_amdgcn_perm(v[u].w, v[u].y, 0x07060302u);
        }
        if (m < MRT) dst[m * RS + (c & 1) * 4 + (c >> 1)] = o;  // with 16 rows held half of the threads have no row
        float sum = frag_sum(o);
        sum += __shfl_xor(sum, 1);
        sum += __shfl_xor(sum, 2);
        sum += __shfl_xor(sum, 4);
        if (c == 0 && m < MRT) cn[m] = a.cneg[kNarrow] * sum;
      }
    } else {
      const int c = tid & 15;
#pragma unroll
      for (int u = 0; u < NPW; ++u) {
        const int m = rows_of(16, u);
        uint4 o = {0u, 0u, 0u, 0u};
        if (xvalid[u] && c < 12) o = frag_from_chunk<KW>(v[u], c & 3, c >> 2);
        if (c < 12) dst[m * RS + c] = o;
        float sum = frag_sum(o);
        sum += __shfl_xor(sum, 1);
        sum += __shfl_xor(sum, 2);
        sum += __shfl_xor(sum, 4);
        sum += __shfl_xor(sum, 8);
        if (c == 0) cn[m] = a.cneg[kWide] * sum;
      }
    }
  };

  f32x4 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // group j of the held k-tile against the activation tile in LDS buffer `buf`
  auto contract = [&](auto kind_c, const auto& r, const uint32_t (&fields)[4], int buf, int j, float be) {
    constexpr int KIND = decltype(kind_c)::value;
    using TR = Traits<KIND>;
    const uint4* src = As + (size_t)buf * MRT * RS;
    const float* cn = Cn + buf * MRT;
    f32x4 P[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) P[mt] = *reinterpret_cast<const f32x4*>(cn + mt * 16 + 4 * kq);
#pragma unroll
    for (int t = 0; t < TR::T; ++t) {
      const bf16x8 wf = decode_frag<KIND>(r, j, t, al, be, dc.c4300, dc.mask[(KIND & kH16) ? 2 : (KIND & 1)]);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const uint4 xa = src[(mt * 16 + nl) * RS + t * 4 + kq];
        P[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xa), wf, P[mt], 0, 0, 0);
      }
    }
    const float s = group_scale<KIND>(r, fields, j);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[mt][e] = __builtin_fmaf(s, P[mt][e], acc[mt][e]);
    }
  };
  auto lds_barrier = [&]() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  };

  // steps of this share: the groups of its narrow k-tiles, then those of its wide ones
  const int nsN = HAS_N ? (tB[kNarrow] - tA[kNarrow]) * kNarrowGroupsPerTile : 0;
  const int nsW = HAS_W ? (tB[kWide] - tA[kWide]) * kWideGroupsPerTile : 0;
  const int nsteps = nsN + nsW;
  auto kind_of = [&](int s) -> int { return (HAS_N && (!HAS_W || s < nsN)) ? kNarrow : kWide; };
  auto group_of = [&](int s) -> int {  // original group (activation columns) of step s
    s = min(s, nsteps - 1);
    const int pg = s < nsN ? tA[kNarrow] * kNarrowGroupsPerTile + s : a.groups_narrow + tA[kWide] * kWideGroupsPerTile + (s - nsN);
    if constexpr (META) return a.meta[pg];
    return min(s < nsN ? pg : pg - a.groups_narrow, a.g_last);
  };

  uint4 areg[2][NP];
  int s = 0;
  set_rows(kind_of(0) == kNarrow ? 8 : 16);
  if (stager) request(areg[0], kind_of(0), group_of(0));
  if (HAS_N && HAS_W && nsN == 1) set_rows(16);  // not reachable: narrow groups come in k-tiles of four
  if (stager) {
    request(areg[1], kind_of(min(1, nsteps - 1)), group_of(1));
    commit(0, areg[0], kind_of(0));
  }
  lds_barrier();
  const float be = be_raw + magic;  // Code Cluster offset + 2^23 (exact: beta is an integer below 2^15)
  const uint32_t nofields[4] = {0u, 0u, 0u, 0u};

  // one step: request the tile of step s + 2, multiply step s, write the tile of step s + 1
  auto step = [&](auto JC, auto&& multiply_this) {
    constexpr int J = decltype(JC)::value;
    const int s2 = min(s + 2, nsteps - 1), s1 = min(s + 1, nsteps - 1);
    // areg[J ^ 1] holds step s + 1, requested one step ago; areg[J] (step s, already in LDS) is free for step s + 2
    if (HAS_N && HAS_W && kind_of(s2) != kind_of(s1)) {
      // the request two steps ahead is the first of the other kind: it needs that kind's row assignment, and the
      // commit below still needs the old one -- commit first
      multiply_this(J);
      if (stager) commit(J ^ 1, areg[J ^ 1], kind_of(s1));
      set_rows(16);
      if (stager) request(areg[J], kind_of(s2), group_of(s + 2));
    } else {
      if (stager) request(areg[J], kind_of(s2), group_of(s + 2));
      multiply_this(J);
      if (stager) commit(J ^ 1, areg[J ^ 1], kind_of(s1));
    }
    lds_barrier();
    ++s;
  };
  using J0 = std::integral_constant<int, 0>;
  using J1 = std::integral_constant<int, 1>;

  if constexpr (HAS_N) {
    TileRegs<KN> cur, nxt;
    load_tile<KN>(cur, codes_n, scales_n, tA[kNarrow], lane);
    for (int t = tA[kNarrow]; t < tB[kNarrow]; ++t) {
      load_tile<KN>(nxt, codes_n, scales_n, min(t + 1, a.tiles[kNarrow] - 1), lane);
      step(J0{}, [&](int buf) { contract(std::integral_constant<int, KN>{}, cur, nofields, buf, 0, be); });
      step(J1{}, [&](int buf) { contract(std::integral_constant<int, KN>{}, cur, nofields, buf, 1, be); });
      step(J0{}, [&](int buf) { contract(std::integral_constant<int, KN>{}, cur, nofields, buf, 2, be); });
      step(J1{}, [&](int buf) { contract(std::integral_constant<int, KN>{}, cur, nofields, buf, 3, be); });
      cur = nxt;
    }
  }
  if constexpr (HAS_W) {
    TileRegs<KW> cur, nxt;
    load_tile<KW>(cur, codes_w, scales_w, tA[kWide], lane);
    for (int t = tA[kWide]; t < tB[kWide]; ++t) {
      load_tile<KW>(nxt, codes_w, scales_w, min(t + 1, a.tiles[kWide] - 1), lane);
      uint32_t fields[4] = {0u, 0u, 0u, 0u};
      tile_scale_fields<KW>(fields, cur, lane);
      step(J0{}, [&](int buf) { contract(std::integral_constant<int, KW>{}, cur, fields, buf, 0, be); });
      step(J1{}, [&](int buf) { contract(std::integral_constant<int, KW>{}, cur, fields, buf, 1, be); });
      step(J0{}, [&](int buf) { contract(std::integral_constant<int, KW>{}, cur, fields, buf, 2, be); });
      step(J1{}, [&](int buf) { contract(std::integral_constant<int, KW>{}, cur, fields, buf, 3, be); });
      step(J0{}, [&](int buf) { contract(std::integral_constant<int, KW>{}, cur, fields, buf, 4, be); });
      step(J1{}, [&](int buf) { contract(std::integral_constant<int, KW>{}, cur, fields, buf, 5, be); });
      step(J0{}, [&](int buf) { contract(std::integral_constant<int, KW>{}, cur, fields, buf, 6, be); });
      step(J1{}, [&](int buf) { contract(std::integral_constant<int, KW>{}, cur, fields, buf, 7, be); });
      cur = nxt;
    }
  }

  if (active && rtile * 16 + nl <= a.n_last) {
    const int n = rtile * 16 + nl;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      if constexpr (SM == 1) acc[mt] *= dc.ssup[0];  // compressed scales: the row's super scale, once (see group_scale)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int m = m0 + mt * 16 + 4 * kq + e;
        if (m < a.M) {
          if (gridDim.y > 1) __builtin_nontemporal_store(acc[mt][e], &a.partial[((int64_t)split * a.M + m) * a.N + n]);
          else a.y[(int64_t)m * a.ldy + n] = f32_to_bf16_rne(acc[mt][e]);
        }
      }
    }
  }
}

// Wavefronts (16-row weight tiles) per workgroup of ccq_rows_kernel: eight share one activation tile when there are
// enough row tiles to fill the chip with such workgroups (6-9 % faster than four: half the activation traffic;
// sixteen gain on 8192 rows and lose on 28672), else four.
static int rows_waves(const Layout& L, int M) {
  (void)M;
  return L.row_tiles >= 2 * device_cus() ? 8 : 4;
}

// K shares for ccq_rows_kernel: about four wavefronts per SIMD, at least one k-tile of every format per share.
int rows_splits(const Layout& L, int M) {
  const int mrt = M > 32 ? 64 : (M > 16 ? 32 : 16);
  const int nw = rows_waves(L, M);
  const int64_t blocks = (int64_t)((M + mrt - 1) / mrt) * ((L.row_tiles + nw - 1) / nw);
  const int min_tiles = std::min(L.tiles[kNarrow] > 0 ? L.tiles[kNarrow] : 1 << 30, L.tiles[kWide] > 0 ? L.tiles[kWide] : 1 << 30);
  int64_t s = std::max<int64_t>(1, (16 * (int64_t)device_cus() / nw) / std::max<int64_t>(1, blocks));  // 16 wavefronts per CU: four per SIMD
  s = std::min<int64_t>(s, 8);
  s = std::min<int64_t>(s, std::max(1, min_tiles));
  return (int)s;
}

int launch_rows(const ccq_weight* w, const Layout& L, const void* x, int M, int64_t ldx, void* y, int64_t ldy, float* partial, int S,
                void* stream) {
  RowsArgs a;
  a.codes = static_cast<const uint8_t*>(w->codes);
  a.scales = static_cast<const uint16_t*>(w->scales);
  a.alpha = w->code_alpha;
  a.beta = w->code_beta;
  a.meta = static_cast<const int32_t*>(w->meta);
  a.scale_super = static_cast<const uint16_t*>(w->scale_super);
  a.x = static_cast<const uint16_t*>(x);
  a.y = static_cast<uint16_t*>(y);
  a.partial = partial;
  a.ldx = ldx;
  a.ldy = ldy;
  a.row_tile_bytes = L.row_tile_bytes;
  a.row_tile_scale_halfs = L.row_tile_scale_halfs;
  a.M = M;
  a.N = L.Npad;
  a.g_last = L.G - 1;
  a.n_last = L.N - 1;
  a.row_tiles = L.row_tiles;
  const int mt = M > 32 ? 4 : (M > 16 ? 2 : 1);
  a.m_blocks = (M + 16 * mt - 1) / (16 * mt);
  a.groups_narrow = L.pgroups[kNarrow];
  for (int k = 0; k < 2; ++k) {
    a.tiles[k] = L.tiles[k];
    a.sq[k] = L.tiles[k] / S;
    a.sr[k] = L.tiles[k] % S;
    a.cneg[k] = -(128.f + L.zp[k]);
    if (L.tiles[k] > 0 && a.sq[k] == 0) return CCQ_ERR_BAD_PARAM;  // every share needs a k-tile of every format present
  }
  const int fm = L.h16 ? 4 : (L.tiles[kNarrow] > 0 ? 1 : 0) | (L.tiles[kWide] > 0 ? 2 : 0);
  // built where it is the fastest path: 16 held rows on the wide and hybrid-word formats, 32 on the narrow one
  typedef void (*RowsKernel)(const RowsArgs);
  RowsKernel kern = nullptr;
  const bool cs = L.scale_mode == 1;
  const int nw = rows_waves(L, M);
  if (nw == 8) {
    if (mt == 1 && fm == 2) kern = cs ? ccq_rows_kernel<1, 2, 1, 8> : ccq_rows_kernel<1, 2, 0, 8>;
    else if (mt == 1 && fm == 4) kern = cs ? ccq_rows_kernel<1, 4, 1, 8> : ccq_rows_kernel<1, 4, 0, 8>;
    else if (mt == 2 && fm == 1) kern = cs ? ccq_rows_kernel<2, 1, 1, 8> : ccq_rows_kernel<2, 1, 0, 8>;
  } else {
    if (mt == 1 && fm == 2) kern = cs ? ccq_rows_kernel<1, 2, 1, 4> : ccq_rows_kernel<1, 2, 0, 4>;
    else if (mt == 1 && fm == 4) kern = cs ? ccq_rows_kernel<1, 4, 1, 4> : ccq_rows_kernel<1, 4, 0, 4>;
    else if (mt == 2 && fm == 1) kern = cs ? ccq_rows_kernel<2, 1, 1, 4> : ccq_rows_kernel<2, 1, 0, 4>;
  }
  if (!kern) return CCQ_ERR_UNSUPPORTED;
  const int rs = fm == 1 ? 9 : 13;
  const size_t lds = (size_t)2 * 16 * mt * rs * 16 + (size_t)2 * 16 * mt * 4;
  const int n_blocks = (L.row_tiles + nw - 1) / nw;
  dim3 grid((unsigned)(a.m_blocks * n_blocks), (unsigned)S), block((unsigned)(64 * nw));
  hipLaunchKernelGGL(kern, grid, block, lds, static_cast<hipStream_t>(stream), a);
  if (hipGetLastError() != hipSuccess) return CCQ_ERR_HIP;
  return CCQ_OK;
}

// ---------------------------------------------------------------------------

typedef void (*SkinnyKernel)(const SkinnyArgs);

template <int MT, int MR, int RT, int SM>
static SkinnyKernel pick_fm(int fm) {
  switch (fm) {
    case 1: return ccq_skinny_kernel<MT, MR, RT, 1, SM>;
    case 2: return ccq_skinny_kernel<MT, MR, RT, 2, SM>;
    case 4: return ccq_skinny_kernel<MT, MR, RT, 4, SM>;
    default: return ccq_skinny_kernel<MT, MR, RT, 3, SM>;
  }
}

// Two row tiles per wavefront are built for the narrow format only: with the wide format the
// register file does not hold both tiles' code registers and the compiler would spill to scratch.
template <int MT, int MR, int SM>
static SkinnyKernel pick_rt(int rt, int fm) {
  if (rt == 2) return ccq_skinny_kernel<MT, MR, 2, 1, SM>;
  return pick_fm<MT, MR, 1, SM>(fm);
}

// Compressed scales (sm = 1) are built for up to 16 held rows (the launcher never asks for more).
static SkinnyKernel pick_kernel(int mt, int mr, int rt, int fm, int sm) {
  if (sm == 1) {
    if (mt != 1) return nullptr;
    if (mr == 1) return pick_rt<1, 1, 1>(rt, fm);
    return pick_rt<1, 16, 1>(rt, fm);
  }
  if (mt == 1) {
    if (mr == 1) return pick_rt<1, 1, 0>(rt, fm);
    return pick_rt<1, 16, 0>(rt, fm);
  }
  if (mt == 2) return pick_rt<2, 16, 0>(rt, fm);
  return pick_fm<4, 16, 1, 0>(fm);
}

int launch_skinny(const SkinnyCall& c) {
  const Layout& L = c.L;
  const Decomp& d = c.d;
  // compressed scales are built for one 16-row activation tile held at a time: more rows are walked 16 at a time
  const int rows = std::min(std::max(c.m_tile_hint, 1), L.scale_mode == 1 ? 16 : kMaxSkinnyM);
  int mt = (rows + 15) / 16;
  if (mt == 3) mt = 4;
  const int mr = (mt == 1 && rows == 1) ? 1 : 16;  // rows of the first activation tile that are staged
  const int mrt = mt == 1 ? mr : mt * 16;
  const int fm = L.h16 ? 4 : (L.tiles[kNarrow] > 0 ? 1 : 0) | (L.tiles[kWide] > 0 ? 2 : 0);
  if (64 * d.WR * d.WK > skinny_max_threads(mt, mr, fm, L.scale_mode)) return CCQ_ERR_BAD_PARAM;  // more threads than the kernel is built for
  if (d.RT == 2 && (mt == 4 || fm != 1)) return CCQ_ERR_BAD_PARAM;  // two row tiles per wavefront: narrow format, at most 32 held rows

  SkinnyArgs a;
  a.codes = static_cast<const uint8_t*>(c.w->codes);
  a.scales = static_cast<const uint16_t*>(c.w->scales);
  a.alpha = c.w->code_alpha;
  a.beta = c.w->code_beta;
  a.meta = static_cast<const int32_t*>(c.w->meta);
  a.scale_super = static_cast<const uint16_t*>(c.w->scale_super);
  a.x = static_cast<const uint16_t*>(c.x);
  a.y = static_cast<uint16_t*>(c.y);
  a.partial = c.partial;
  a.sorted_rows = c.sorted_rows;
  a.expert_offsets = c.expert_offsets;
  a.ldx = c.ldx;
  a.ldy = c.ldy;
  a.codes_stride = c.codes_stride;
  a.scales_stride = c.scales_stride;
  a.ab_stride = c.ab_stride;
  a.row_tile_bytes = L.row_tile_bytes;
  a.row_tile_scale_halfs = L.row_tile_scale_halfs;
  a.M = c.M;
  a.N = L.Npad;
  a.g_last = L.G - 1;
  a.n_last = L.N - 1;
  a.row_tiles = L.row_tiles;
  a.tiles[0] = L.tiles[0];
  a.tiles[1] = L.tiles[1];
  a.groups_narrow = L.pgroups[kNarrow];
  a.WR = d.WR;
  a.WK = d.WK;
  a.S = d.S;
  a.inv_WR = (65536 + d.WR - 1) / d.WR;
  for (int k = 0; k < 2; ++k) {
    a.sq[k] = L.tiles[k] / d.S;
    a.sr[k] = L.tiles[k] % d.S;
    for (int v = 0; v < 2; ++v) {
      a.wq[k][v] = (a.sq[k] + v) / d.WK;
      a.wrem[k][v] = (a.sq[k] + v) % d.WK;
    }
  }
  a.cneg[0] = -(128.f + L.zp[0]);
  a.cneg[1] = -(128.f + L.zp[1]);
  a.n_active = c.n_active;
  std::memcpy(a.active_ids, c.active_ids, sizeof(a.active_ids));

  // chunk sizes: as many k-tiles per wavefront as fit the staging budget; if not even one tile per
  // wavefront fits, the groups of a tile are staged a few at a time.  Up to 16 held rows the budget is
  // 36 KiB, so that four workgroups share a CU and one workgroup's staging (barrier, gather, barrier)
  // is covered by the others' contraction.
  const int64_t budget = (mt == 1 ? 36 : 56) * 1024;
  int64_t frag_cap = 0, cneg_cap = 0;
  for (int k = 0; k < 2; ++k) {
    a.KC[k] = 1;
    const int gpt = k == kNarrow ? kNarrowGroupsPerTile : kWideGroupsPerTile, T = k == kNarrow ? 2 : 3;
    a.SG[k] = gpt;
    if (L.tiles[k] == 0) continue;
    const int64_t per_group = (int64_t)T * 4 * mrt * 16 + (int64_t)mt * 16 * 4;
    const int wg_tiles = (L.tiles[k] + d.S - 1) / d.S;             // most k-tiles a workgroup owns
    const int want = (wg_tiles + d.WK - 1) / d.WK;                 // per wavefront if staged at once
    const int64_t fit = budget / (per_group * gpt * d.WK);
    int64_t groups_staged;
    if (fit >= 1 || mt < 2) {
      a.KC[k] = (int)std::max<int64_t>(1, std::min<int64_t>(want, fit));
      groups_staged = (int64_t)a.KC[k] * d.WK * gpt;
    } else {
      int sg = gpt / 2;
      while (sg > 1 && per_group * sg * d.WK > budget) sg /= 2;
      a.SG[k] = sg;
      groups_staged = (int64_t)sg * d.WK;
    }
    frag_cap = std::max<int64_t>(frag_cap, groups_staged * T * 4 * mrt);
    cneg_cap = std::max<int64_t>(cneg_cap, groups_staged * mt * 16);
  }
  a.frag_cap = (int)frag_cap;
  a.cneg_cap = 0;
  int64_t lds = frag_cap * 16 + cneg_cap * 4;
  if (mr == 1 && mt == 1) {
    // one held row: every wavefront has a private region for up to KC k-tiles (about 6 KiB)
    const int waves = d.WR * d.WK;
    int64_t pf = 0, pc = 0;
    for (int k = 0; k < 2; ++k) {
      if (L.tiles[k] == 0) continue;
      const int gpt = k == kNarrow ? kNarrowGroupsPerTile : kWideGroupsPerTile, T = k == kNarrow ? 2 : 3;
      const int per_wave = ((L.tiles[k] + d.S - 1) / d.S + d.WK - 1) / d.WK;
      const int fit = std::max(1, (6 * 1024) / (gpt * T * 4 * 16));
      a.KC[k] = std::max(1, std::min(per_wave, fit));
      a.SG[k] = gpt;
      pf = std::max<int64_t>(pf, (int64_t)a.KC[k] * gpt * T * 4);
      pc = std::max<int64_t>(pc, (int64_t)a.KC[k] * gpt * 16);  // one 16-byte record per group and quarter
    }
    a.frag_cap = (int)pf;
    a.cneg_cap = (int)pc;
    lds = (int64_t)waves * (pf * 16 + pc * 4);
  }
  if (d.WK > 1) lds = std::max<int64_t>(lds, (int64_t)(d.WK - 1) * d.WR * d.RT * mt * 64 * 16);
  if (lds > 150 * 1024) return CCQ_ERR_BAD_PARAM;

  SkinnyKernel kern = pick_kernel(mt, mr, d.RT, fm, L.scale_mode);
  if (!kern) return CCQ_ERR_UNSUPPORTED;
  hipStream_t stream = static_cast<hipStream_t>(c.stream);
  if (lds > 48 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
      (void)hipGetLastError();
      return CCQ_ERR_HIP;
    }
  }
  const int row_blocks = (L.row_tiles + d.WR * d.RT - 1) / (d.WR * d.RT);
  dim3 grid((unsigned)row_blocks, (unsigned)d.S, (unsigned)(c.n_active > 0 ? c.n_active : c.E));
  dim3 block((unsigned)(64 * d.WR * d.WK));
  hipLaunchKernelGGL(kern, grid, block, (size_t)lds, stream, a);
  if (hipGetLastError() != hipSuccess) return CCQ_ERR_HIP;
  if (d.S > 1) return launch_reduce_splits(c.partial, c.y, c.ldy, c.M, L.N, L.Npad, d.S, c.stream);
  return CCQ_OK;
}

int launch_reduce_splits(const float* partial, void* y, int64_t ldy, int rows, int N, int Npad, int S, void* stream) {
  const int64_t total = (int64_t)rows * Npad;  // a multiple of 16
  // small calls: workgroups of one or two wavefronts, so that every CU gets some of this short, latency-bound pass
  // (config 2 at M = 8 / 16: 11.2 / 11.5 -> 10.7 / 11.2 us per step with 64 threads against 256)
  const int64_t quads = total / 4, cus = device_cus();
  const int threads = quads >= 512 * cus ? 256 : (quads >= 256 * cus ? 128 : 64);
  const dim3 grid((unsigned)((quads + threads - 1) / threads)), block(threads);
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint16_t* yy = static_cast<uint16_t*>(y);
  if (S <= 4) hipLaunchKernelGGL(ccq_reduce_splits_kernel<4>, grid, block, 0, st, partial, yy, ldy, rows, N, Npad, S);
  else if (S <= 8) hipLaunchKernelGGL(ccq_reduce_splits_kernel<8>, grid, block, 0, st, partial, yy, ldy, rows, N, Npad, S);
  else hipLaunchKernelGGL(ccq_reduce_splits_kernel<kMaxSplitsK>, grid, block, 0, st, partial, yy, ldy, rows, N, Npad, S);
  if (hipGetLastError() != hipSuccess) return CCQ_ERR_HIP;
  return CCQ_OK;
}

}  // namespace ccq
