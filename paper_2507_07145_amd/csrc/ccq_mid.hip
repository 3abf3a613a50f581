// Fused dequantize-and-multiply for a few dozen activation rows (about 17 to 128), any mix of the
// narrow (L=6,N=4,S=3 + Code Cluster) and wide (L=4,N=3,S=2) formats, gfx950.
//
// With that many rows the per-row-tile kernel re-stages the activations far too often, and the
// 256-row kernel wastes three quarters of its tile.  Here a workgroup owns a 64 x BN tile of the
// output (BN = 128) and a contiguous share of K (grid.y = S shares; fp32 partial tiles go to the
// workspace and are added in index order by the reduction kernel when S > 1).  K is walked one
// 64-weight group per step; per step the workgroup
//   - copies the 64 x 64 activation tile of that group's columns to LDS,
//   - decodes the BN x 64 weight tile to bf16 in LDS: window extraction by the shift lists
//     [9,6,3,0] / [4,2,0] and masks 0x3F / 0xF of Table 1 straight into the mantissa of fp32 128.0,
//     then d = (w_uint - zp) * s (Alg. 2 / Alg. 3, last line) as fma(128 + state, s, -(128 + zp) s),
//     which is exact in fp32, so the stored value is the correctly rounded bf16 of the exact weight,
//   - multiplies the two tiles with MFMA 32x32x16 bf16 (fp32 accumulators).
// The hybrid 16-bit word of Sec. 3.2 (a (3,3,2) and a (3,4,2) code side by side, seven weights per
// word, ten words per group) takes the place of the wide format when it is used: its weights are kept
// in LDS word by word, eight bf16 slots per word (seven weights and one unused slot, 80 slots per
// group), and the activation tile is scattered into the same slot order, so that a decoded word is one
// 16-byte LDS write and a group is five MFMA k-steps instead of four.
// The decode is the bound (about 4 vector instructions per weight, shared by 64 rows), so the
// kernel is kept small enough (55 KiB of LDS, < 128 registers) for two workgroups per CU, whose
// vector and matrix phases overlap.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

#include "ccq_decode.h"
#include "ccq_internal.h"

namespace ccq {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

struct MidArgs {
  const uint8_t* codes;
  const uint16_t* scales;
  const float* alpha;
  const float* beta;
  const int32_t* meta;
  const uint16_t* scale_super;  // fp16 [N], compressed scales only
  const uint16_t* x;
  uint16_t* y;
  float* partial;
  int64_t ldx, ldy;
  int64_t row_tile_bytes, row_tile_scale_halfs;
  int32_t M, N, row_tiles, m_blocks;  // N: rows of the device layout (a multiple of 16), the row stride of `partial`
  int32_t tiles[2];       // k-tiles per kind
  int32_t groups_narrow;  // narrow entries of the group map (whole k-tiles), the offset of the wide ones
  int32_t g_last;         // last real group of K: groups past it pad a k-tile (zero scale) and read this group's activations
  int32_t n_last;         // last real output row: rows past it pad a row tile, take its parameters and are not stored
  int32_t sq[2], sr[2];   // K shares: share `split` owns tiles [split*sq + min(split, sr), +sq + (split < sr)) of each kind
  float zp[2];
  // grouped calls (narrow-format kernel only): blockIdx.z = expert; its rows are output rows [offsets[e], offsets[e+1]),
  // activation row sorted_rows[p] for output row p; expert e's arrays start e * stride bytes after expert 0's
  const int32_t* sorted_rows;
  const int32_t* expert_offsets;
  int64_t codes_stride, scales_stride, ab_stride;
};

constexpr int kMidBM = 64;
constexpr int kMidBN = 128;
constexpr int kMidRow = 64 + 8;     // bf16 elements per padded LDS row (144 bytes)
constexpr int kMidRowH16 = 80 + 8;  // the same for the hybrid word: ten words of eight slots (176 bytes)

__device__ __forceinline__ uint32_t and_or_m(uint32_t a, uint32_t mask, uint32_t orv) { return (a & mask) | orv; }

__device__ __forceinline__ uint32_t pack_bf16_m(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);  // round to nearest even
  return __builtin_bit_cast(uint32_t, b);
}

__device__ __forceinline__ uint32_t dword_sel(const u32x4& v, int j) { return j == 0 ? v.x : (j == 1 ? v.y : (j == 2 ? v.z : v.w)); }

// FM: formats present (1 narrow, 2 wide, 3 both, 4 the hybrid word; a group map exists only for 3).  SM: scale mode (0 fp16 group
// scales; 1 the compressed scales of Sec. 3.4: group scale = 4-bit field * per-row super scale, first line of
// Alg. 2 / Alg. 3; the field of a narrow group comes from the packed scale array, that of a wide group from the
// spare low nibble of the group's last code byte).
// Wavefronts per workgroup (kMidWaves): eight; each decodes one of the block's eight 16-row weight tiles and multiplies 32
// activation rows with 32 columns (wavefronts 0-3 the first 32 rows, 4-7 the others).  With four (two weight tiles and a
// 64 x 32 wave tile each: twice the work per wavefront, half the wavefronts per SIMD, 150-178 registers instead of
// 100-119) the same code measured slower on the same box: 8192 x 8192 at M = 64 wide 28.1 -> 24.9 us, a 3:1 mix
// 46.1 -> 35.2, hybrid word 35.0 -> 31.2; 8192 x 28672: 2-6 % less; M = 2048: 2-4 % less.
constexpr int kMidWaves = 8;
template <int FM, int SM, bool GROUPED>
__global__ void __launch_bounds__(64 * kMidWaves) ccq_mid_kernel(const MidArgs a) {
  constexpr int NWV = kMidWaves;
  constexpr int kMidRTW = 8 / NWV;   // 16-row weight tiles per wavefront
  constexpr int NT = 64 * NWV;       // threads
  constexpr int AI = 8 / NWV;        // 32-row accumulator tiles per wavefront
  constexpr bool HAS_N = FM == 1 || FM == 3, HAS_W = FM >= 2, META = FM == 3, H16 = FM == 4;
  constexpr int ROW = H16 ? kMidRowH16 : kMidRow;
  constexpr int WTILE = H16 ? kH16TileBytes : kWideTileBytes;
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* As = reinterpret_cast<uint16_t*>(smem);   // [2][kMidBM][ROW]
  uint16_t* Bs = As + 2 * kMidBM * ROW;               // [2][kMidBN][ROW]
  int32_t* lds_meta = reinterpret_cast<int32_t*>(Bs + 2 * kMidBN * ROW);  // original group of each step of this share (META only)

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m_block = blockIdx.x % a.m_blocks, n_block = blockIdx.x / a.m_blocks;
  const int split = blockIdx.y;
  const int m0 = m_block * kMidBM, n0 = n_block * kMidBN;
  const int kq = lane >> 4, nl = lane & 15;
  // rows of this block's matrix: all M (dense), or the expert's (grouped; row_off = its first output row)
  int Me = a.M, row_off = 0;
  int64_t e_codes = 0, e_scales = 0, e_ab = 0;
  if constexpr (GROUPED) {
    const int e = blockIdx.z;
    row_off = a.expert_offsets[e];
    Me = a.expert_offsets[e + 1] - row_off;
    if (m0 >= Me) return;  // uniform: before any barrier
    e_codes = e * a.codes_stride;
    e_scales = e * a.scales_stride;
    e_ab = e * a.ab_stride;
  }

  // this share's k-tiles of each kind, and its steps (one 64-weight group each): narrow first, then wide
  int tA[2], tB[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    tA[k] = split * a.sq[k] + min(split, a.sr[k]);
    tB[k] = tA[k] + a.sq[k] + (split < a.sr[k] ? 1 : 0);
  }
  const int nsN = HAS_N ? (tB[kNarrow] - tA[kNarrow]) * kNarrowGroupsPerTile : 0;
  const int nsW = HAS_W ? (tB[kWide] - tA[kWide]) * kWideGroupsPerTile : 0;
  const int nsteps = nsN + nsW;  // even: both factors are

  if constexpr (META) {
    for (int s = tid; s < nsteps; s += NT) {
      const int pg = s < nsN ? tA[kNarrow] * kNarrowGroupsPerTile + s : a.groups_narrow + tA[kWide] * kWideGroupsPerTile + (s - nsN);
      lds_meta[s] = a.meta[pg];
    }
    __syncthreads();
  }
  // original group (activation columns 64 g .. 64 g + 63) of step s
  auto group_of = [&](int s) -> int {
    s = min(s, nsteps - 1);
    if constexpr (META) return lds_meta[s];
    return min(s < nsN ? tA[kNarrow] * kNarrowGroupsPerTile + s : tA[kWide] * kWideGroupsPerTile + (s - nsN), a.g_last);
  };

  // per-wavefront weight rows: row tiles n0/16 + wave*RTW + i, lane (nl, kq)
  const uint8_t* code_base[kMidRTW];
  const uint16_t* scale_base[kMidRTW];
  float al[kMidRTW], be[kMidRTW], ssup[kMidRTW];
#pragma unroll
  for (int i = 0; i < kMidRTW; ++i) {
    const int rtile = min(n0 / 16 + wave * kMidRTW + i, a.row_tiles - 1);  // ragged last block: re-decode the last tile, never stored
    code_base[i] = a.codes + e_codes + (int64_t)rtile * a.row_tile_bytes;
    scale_base[i] = reinterpret_cast<const uint16_t*>(reinterpret_cast<const uint8_t*>(a.scales) + e_scales) + (int64_t)rtile * a.row_tile_scale_halfs;
    al[i] = 0.f;
    be[i] = 0.f;
    ssup[i] = 0.f;
    // expert e's super scales: half the byte stride of alpha / beta (fp16 against fp32)
    if constexpr (SM == 1)
      ssup[i] = (float)__builtin_bit_cast(_Float16, reinterpret_cast<const uint16_t*>(reinterpret_cast<const uint8_t*>(a.scale_super) + e_ab / 2)[min(rtile * 16 + nl, a.n_last)]);
    if constexpr (HAS_N) {
      al[i] = reinterpret_cast<const float*>(reinterpret_cast<const uint8_t*>(a.alpha) + e_ab)[min(rtile * 16 + nl, a.n_last)];
      be[i] = reinterpret_cast<const float*>(reinterpret_cast<const uint8_t*>(a.beta) + e_ab)[min(rtile * 16 + nl, a.n_last)];
    }
  }
  const int64_t wide_code_off = (int64_t)a.tiles[kNarrow] * kNarrowTileBytes;
  const int64_t wide_scale_off = (int64_t)a.tiles[kNarrow] * kNarrowTileScaleHalfs;
  uint32_t c43 = 0x43000000u, mask2 = kDecMask2, base2 = kDecBase2, mask_w = 0x00070000u, mask_w2 = kDecMaskW2;  // mask_w: the hybrid word's 3-bit states
  float magic = 8388608.f;
  asm volatile("" : "+v"(c43), "+s"(mask2), "+v"(base2), "+s"(mask_w), "+s"(mask_w2), "+v"(magic));

  // code tiles in registers: the one being decoded and the next one of the same kind
  u32x4 cn[kMidRTW], cn_next[kMidRTW];
  uint2 sn[kMidRTW], sn_next[kMidRTW];
  u32x4 cw[kMidRTW][3], cw_next[kMidRTW][3];
  uint4 sw[kMidRTW], sw_next[kMidRTW];
  auto load_narrow = [&](u32x4 (&c)[kMidRTW], uint2 (&sc)[kMidRTW], int kt) {
    kt = min(kt, a.tiles[kNarrow] - 1);
#pragma unroll
    for (int i = 0; i < kMidRTW; ++i) {
      c[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(code_base[i] + (int64_t)kt * kNarrowTileBytes + lane * 16));
      if constexpr (SM == 0) sc[i] = *reinterpret_cast<const uint2*>(scale_base[i] + (int64_t)kt * kNarrowTileScaleHalfs + nl * 4);
      else sc[i] = uint2{(uint32_t)scale_base[i][(int64_t)kt * kNarrowTileScaleHalfs4 + nl], 0u};  // the tile's four 4-bit fields
    }
  };
  auto load_wide = [&](u32x4 (&c)[kMidRTW][3], uint4 (&sc)[kMidRTW], int kt) {
    kt = min(kt, a.tiles[kWide] - 1);
#pragma unroll
    for (int i = 0; i < kMidRTW; ++i) {
      const uint8_t* t = code_base[i] + wide_code_off + (int64_t)kt * WTILE + lane * 16;
      c[i][0] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t));
      c[i][1] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t + 1024));
      // the third segment has entries for 48 lanes only (32 for the hybrid word); the lanes above re-read the
      // last entry (what they decode from it lands in the padding columns of the LDS row, or is not written)
      constexpr int last = H16 ? 31 : 47;
      c[i][2] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t + 2048 - (lane > last ? (lane - last) * 16 : 0)));
      if constexpr (SM == 0) sc[i] = *reinterpret_cast<const uint4*>(scale_base[i] + wide_scale_off + (int64_t)kt * kWideTileScaleHalfs + nl * 8);
      else sc[i] = uint4{0u, 0u, 0u, 0u};  // the fields sit in the code stream
    }
  };

  // activation copy: 2 chunks of 16 bytes per thread and step; rows past M re-read row M-1 (their
  // products land in accumulator rows that are never stored)
  constexpr int XC = 512 / NT;   // 16-byte chunks of the activation tile per thread
  const uint16_t* xrow[XC];
  int a_lds_off[XC];
#pragma unroll
  for (int i = 0; i < XC; ++i) {
    const int c = tid + NT * i, row = c >> 3, col = c & 7;
    int64_t xr = row_off + min(m0 + row, Me - 1);
    if constexpr (GROUPED) {
      if (a.sorted_rows) xr = a.sorted_rows[xr];
    }
    xrow[i] = a.x + xr * a.ldx + col * 8;
    a_lds_off[i] = row * ROW + (H16 ? 0 : col * 8);
  }
  // hybrid word: element e of a group sits in slot 8 (e / 7) + e % 7 (weight 63, alone in the last word, in
  // slot 72); the unused slots are cleared once and never written again
  int a_slot[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int e = (tid & 7) * 8 + j;
    a_slot[j] = H16 ? (e == 63 ? 72 : 8 * (e / 7) + e % 7) : 0;
  }
  if constexpr (H16) {
    for (int i = tid; i < 2 * kMidBM * ROW / 8; i += NT) reinterpret_cast<u32x4*>(As)[i] = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();
  }
  auto load_a = [&](u32x4 (&dst)[XC], int s) {
    const int64_t off = (int64_t)group_of(s) * kGroup;
#pragma unroll
    for (int i = 0; i < XC; ++i) dst[i] = *reinterpret_cast<const u32x4*>(xrow[i] + off);
  };
  auto store_a = [&](int buf, const u32x4 (&src)[XC]) {
    uint16_t* dst = As + buf * kMidBM * ROW;
    if constexpr (H16) {
#pragma unroll
      for (int i = 0; i < XC; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const uint32_t d = src[i][q];
          dst[a_lds_off[i] + a_slot[2 * q]] = (uint16_t)(d & 0xFFFFu);
          dst[a_lds_off[i] + a_slot[2 * q + 1]] = (uint16_t)(d >> 16);
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < XC; ++i) *reinterpret_cast<u32x4*>(dst + a_lds_off[i]) = src[i];
    }
  };

  // decode group j of the held narrow k-tile: 16 weights per lane (k = 16 kq .. 16 kq + 15)
  auto decode_narrow = [&](int buf, int j) {
    uint16_t* dst = Bs + buf * kMidBN * ROW;
#pragma unroll
    for (int i = 0; i < kMidRTW; ++i) {
      const uint32_t d = dword_sel(cn[i], j);
      float s;
      if constexpr (SM == 0) {
        const uint32_t sd = (j >> 1) ? sn[i].y : sn[i].x;
        s = (float)__builtin_bit_cast(_Float16, (uint16_t)((j & 1) ? (sd >> 16) : (sd & 0xFFFFu)));
      } else {
        s = (float)((sn[i].x >> (4 * j)) & 0xFu) * ssup[i];  // (s_q >> s_shift) & s_mask times s_super: exact
      }
      const float c0 = -(kDecBase + a.zp[kNarrow]) * s;  // exact: 8-bit times at most 15-bit significand
      const float bem = be[i] + magic;                    // + 2^23: exact, beta is an integer below 2^15
      uint32_t o[8];
      decode16_narrow(d, al[i], bem, s, c0, mask2, base2, o);
      uint16_t* p = dst + ((wave * kMidRTW + i) * 16 + nl) * ROW + kq * 16;
      *reinterpret_cast<u32x4*>(p) = u32x4{o[0], o[1], o[2], o[3]};
      *reinterpret_cast<u32x4*>(p + 8) = u32x4{o[4], o[5], o[6], o[7]};
    }
  };
  // decode group j of the held wide k-tile: canonical bytes 6 kq .. 6 kq + 5 of the group, 3 weights each
  // (k = 18 kq .. 18 kq + 17).  Quarter 3 owns bytes 18..21 only (weights 54..63); what it writes beyond
  // column 63 falls into the padding of its own LDS row.
  auto decode_wide = [&](int buf, int j) {
    uint16_t* dst = Bs + buf * kMidBN * ROW;
    if constexpr (H16) {
      // words kq, 4 + kq and (kq < 2) 8 + kq of group j: seven 3-bit states at the shifts [13,11,9,6,4,2,0]
      // (Table 1), each moved to bit 16, the lowest integer bit of fp32 128.0
#pragma unroll
      for (int i = 0; i < kMidRTW; ++i) {
        float s;
        if constexpr (SM == 0) {
          const uint32_t sd = dword_sel(u32x4{sw[i].x, sw[i].y, sw[i].z, sw[i].w}, j >> 1);
          s = (float)__builtin_bit_cast(_Float16, (uint16_t)((j & 1) ? (sd >> 16) : (sd & 0xFFFFu)));
        } else {
          // Alg. 2 with the scale mask 0x1FFF of Table 1: the low 13 bits of the group's last word (word 9), which
          // quarter 1 of the row holds in segment 2, halfword j
          const uint32_t q1 = (uint32_t)__builtin_amdgcn_ds_bpermute((16 + nl) * 4, (int)dword_sel(cw[i][2], j >> 1));
          s = (float)((q1 >> (16 * (j & 1))) & 0x1FFFu) * ssup[i];  // exact: 13-bit integer times 11-bit significand
        }
        const float c0 = -(128.f + a.zp[kWide]) * s;
        const float zoff = 128.f + a.zp[kWide];
        uint16_t* row = dst + ((wave * kMidRTW + i) * 16 + nl) * ROW;
#pragma unroll
        for (int t = 0; t < 3; ++t) {
          const uint32_t dd = dword_sel(cw[i][t], j >> 1);
          const uint32_t w = (j & 1) ? (dd >> 16) : (dd & 0xFFFFu);
          // With fp16 group scales (128 + zp) s is exact and one fused multiply-add gives the exactly rounded
          // weight.  A 13-bit field times an 11-bit super scale fills all 24 bits of s, so there the offset is
          // taken off first (exact) and the product (state - zp) s is rounded once to fp32.
          auto value = [&](uint32_t shifted) -> float {
            const float st = __builtin_bit_cast(float, and_or_m(shifted, mask_w, c43));  // 128 + state
            if constexpr (SM == 0) return __builtin_fmaf(st, s, c0);
            else return (st - zoff) * s;
          };
          const float f0 = value(w << 3), f1 = value(w << 5), f2 = value(w << 7), f3 = value(w << 10);
          const float f4 = value(w << 12), f5 = value(w << 14), f6 = value(w << 16);
          // the eighth slot of a word meets a zero activation; any finite value will do
          const u32x4 o = {pack_bf16_m(f0, f1), pack_bf16_m(f2, f3), pack_bf16_m(f4, f5), pack_bf16_m(f6, f6)};
          if (t < 2 || kq < 2) *reinterpret_cast<u32x4*>(row + (4 * t + kq) * 8) = o;
        }
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < kMidRTW; ++i) {
      float s;
      if constexpr (SM == 0) {
        const uint32_t sd = dword_sel(u32x4{sw[i].x, sw[i].y, sw[i].z, sw[i].w}, j >> 1);
        s = (float)__builtin_bit_cast(_Float16, (uint16_t)((j & 1) ? (sd >> 16) : (sd & 0xFFFFu)));
      } else {
        // Alg. 2: the low nibble of the group's last code byte (byte 21), which quarter 3 of the row holds in
        // segment 1, halfword j, high byte
        const uint32_t own = dword_sel(cw[i][1], j >> 1);
        const uint32_t q3 = (uint32_t)__builtin_amdgcn_ds_bpermute((48 + nl) * 4, (int)own);
        s = (float)((q3 >> (16 * (j & 1) + 8)) & 0xFu) * ssup[i];
      }
      const float c0 = -(kDecBase + a.zp[kWide]) * s;
      float w[18];
#pragma unroll
      for (int t = 0; t < 3; ++t) {
        const uint32_t dd = dword_sel(cw[i][t], j >> 1);
        const uint32_t pp = __builtin_amdgcn_perm(0u, dd, (j & 1) ? 0x0C030C02u : 0x0C010C00u);  // two codes, low byte first: {0, b, 0, a}
        float w6[6];
        decode6_wide(pp, s, c0, mask_w2, base2, w6);
#pragma unroll
        for (int e = 0; e < 6; ++e) w[6 * t + e] = w6[e];
      }
      uint32_t* p = reinterpret_cast<uint32_t*>(dst + ((wave * kMidRTW + i) * 16 + nl) * ROW + kq * 18);
#pragma unroll
      for (int q = 0; q < 9; ++q) p[q] = pack_bf16_m(w[2 * q], w[2 * q + 1]);
    }
  };

  f32x16 acc[AI];
#pragma unroll
  for (int i = 0; i < AI; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  const int wcol = wave & 3, wrow = wave >> 2;   // this wavefront's 32 columns; its half of the rows (eight wavefronts)
  const int a_frag_off = (wrow * 32 + (lane & 31)) * ROW + (lane >> 5) * 8;
  const int b_frag_off = (wcol * 32 + (lane & 31)) * ROW + (lane >> 5) * 8;
  auto multiply = [&](int buf) {
    const uint16_t* Ab = As + buf * kMidBM * ROW + a_frag_off;
    const uint16_t* Bb = Bs + buf * kMidBN * ROW + b_frag_off;
#pragma unroll
    for (int kk = 0; kk < (H16 ? 5 : 4); ++kk) {  // 16 k-slots per MFMA: 64 weights, or ten words of eight slots
      const bf16x8 bfr = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Bb + kk * 16));
#pragma unroll
      for (int i = 0; i < AI; ++i) {
        const bf16x8 af = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Ab + i * 32 * ROW + kk * 16));
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfr, acc[i], 0, 0, 0);
      }
    }
  };
  auto lds_barrier = [&]() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  };

  // Every share holds at least two k-tiles of each format present (the launcher sees to it).  All global
  // loads below are unconditional and sit at fixed places of straight-line loop bodies: a request under a
  // condition makes the compiler wait for every outstanding load at the next use of any of them.
  {
    // activation chunks of step s live in register set s & 3, requested four steps ahead of their use: a
    // step is far shorter than a memory latency
    u32x4 areg[4][XC];
    int s = 0;  // step counter of this share: narrow steps first, then wide ones
    if constexpr (HAS_N) load_narrow(cn, sn, tA[kNarrow]);
    if constexpr (HAS_W) load_wide(cw, sw, tA[kWide]);
    load_a(areg[0], 0);
    load_a(areg[1], 1);
    load_a(areg[2], 2);
    load_a(areg[3], 3);
    store_a(0, areg[0]);
    if constexpr (HAS_N) decode_narrow(0, 0);
    else decode_wide(0, 0);
    lds_barrier();
    // one step (J = s & 3): LDS buffer J & 1 is multiplied while step s + 1 is written to the other buffer
    // and the activations of step s + 4 are requested
    auto step = [&](auto JC, auto&& decode_next) {
      constexpr int J = decltype(JC)::value;
      constexpr int P = J & 1;
      load_a(areg[J], s + 4);
      multiply(P);
      store_a(P ^ 1, areg[(J + 1) & 3]);
      decode_next(P ^ 1);
      lds_barrier();
      ++s;
    };
    using J0 = std::integral_constant<int, 0>;
    using J1 = std::integral_constant<int, 1>;
    using J2 = std::integral_constant<int, 2>;
    using J3 = std::integral_constant<int, 3>;
    if constexpr (HAS_N) {
      for (int t = tA[kNarrow]; t < tB[kNarrow]; ++t) {
        load_narrow(cn_next, sn_next, t + 1);
        step(J0{}, [&](int nb) { decode_narrow(nb, 1); });
        step(J1{}, [&](int nb) { decode_narrow(nb, 2); });
        step(J2{}, [&](int nb) { decode_narrow(nb, 3); });
        step(J3{}, [&](int nb) {
#pragma unroll
          for (int i = 0; i < kMidRTW; ++i) { cn[i] = cn_next[i]; sn[i] = sn_next[i]; }
          if (t + 1 < tB[kNarrow]) decode_narrow(nb, 0);
          else if constexpr (HAS_W) decode_wide(nb, 0);
        });
      }
    }
    if constexpr (HAS_W) {
      for (int t = tA[kWide]; t < tB[kWide]; ++t) {
        load_wide(cw_next, sw_next, t + 1);
        step(J0{}, [&](int nb) { decode_wide(nb, 1); });
        step(J1{}, [&](int nb) { decode_wide(nb, 2); });
        step(J2{}, [&](int nb) { decode_wide(nb, 3); });
        step(J3{}, [&](int nb) { decode_wide(nb, 4); });
        step(J0{}, [&](int nb) { decode_wide(nb, 5); });
        step(J1{}, [&](int nb) { decode_wide(nb, 6); });
        step(J2{}, [&](int nb) { decode_wide(nb, 7); });
        step(J3{}, [&](int nb) {
#pragma unroll
          for (int i = 0; i < kMidRTW; ++i) {
#pragma unroll
            for (int tt = 0; tt < 3; ++tt) cw[i][tt] = cw_next[i][tt];
            sw[i] = sw_next[i];
          }
          if (t + 1 < tB[kWide]) decode_wide(nb, 0);
        });
      }
    }
  }

  // epilogue: D[row][col], row = 8*(r/4) + 4*(lane/32) + r%4, col = lane%32
  const int n = n0 + wcol * 32 + (lane & 31);
#pragma unroll
  for (int i = 0; i < AI; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + (wrow + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      const float val = acc[i][r];  // by value: bit-casting the element lvalue itself reads element 0
      if (m < Me && n <= a.n_last) {
        if (gridDim.y > 1) __builtin_nontemporal_store(val, &a.partial[((int64_t)split * a.M + row_off + m) * a.N + n]);
        else a.y[(int64_t)(row_off + m) * a.ldy + n] = (uint16_t)(pack_bf16_m(val, 0.f) & 0xFFFFu);
      }
    }
  }
}

// ---- narrow format: the same tile with the decoded weights kept in registers ----------------------------
// A wavefront multiplies exactly the 32 columns it decodes, so the decoded tile need not pass through LDS: MFMA
// 32x32x16 wants lane l to hold column l % 32 and eight k-slots of half l / 32, while the code stream gives lane l
// row l % 16 of both of the wavefront's row tiles and quarter l / 16 of every group.  The *codes* (2 bits per
// weight) are exchanged between lanes instead of the decoded weights: lane (half h, tile ti, row nl) fetches the
// dwords of quarters 2h and 2h+1 of its own column from lanes nl + 16 (2h + q) with ds_bpermute, once per k-tile,
// and then decodes 32 weights of one column per group: k-slots 8 kk .. 8 kk + 7 of MFMA step kk are weights
// 32 h + 8 kk .. of the group, which is also how the activation fragment is read.  Only the activation tile
// lives in LDS (18 KiB).
template <int SM, bool GROUPED>
__global__ void __launch_bounds__(256) ccq_midr_narrow_kernel(const MidArgs a) {
  constexpr int ROW = kMidRow;
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* As = reinterpret_cast<uint16_t*>(smem);  // [2][kMidBM][ROW]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m_block = blockIdx.x % a.m_blocks, n_block = blockIdx.x / a.m_blocks;
  const int split = blockIdx.y;
  const int m0 = m_block * kMidBM, n0 = n_block * kMidBN;
  // rows of this block's matrix: all M (dense), or the expert's (grouped; row_off = its first output row)
  int Me = a.M, row_off = 0;
  int64_t e_codes = 0, e_scales = 0, e_ab = 0;
  if constexpr (GROUPED) {
    const int e = blockIdx.z;
    row_off = a.expert_offsets[e];
    Me = a.expert_offsets[e + 1] - row_off;
    if (m0 >= Me) return;  // uniform: before any barrier
    e_codes = e * a.codes_stride;
    e_scales = e * a.scales_stride;
    e_ab = e * a.ab_stride;
  }
  const int nl = lane & 15;
  const int ti = (lane >> 4) & 1, h = lane >> 5;  // the column this lane multiplies: row tile ti of the wavefront, row nl; k half h

  const int tA = split * a.sq[kNarrow] + min(split, a.sr[kNarrow]);
  const int tB = tA + a.sq[kNarrow] + (split < a.sr[kNarrow] ? 1 : 0);
  const int nsteps = (tB - tA) * kNarrowGroupsPerTile;

  const uint8_t* code_base[2];
  const uint16_t* scale_base[2];
  float al_t = 0.f, be_t = 0.f, ssup_t = 0.f;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int rtile = min(n0 / 16 + wave * 2 + i, a.row_tiles - 1);  // ragged last block: re-decode the last tile, never stored
    code_base[i] = a.codes + e_codes + (int64_t)rtile * a.row_tile_bytes;
    scale_base[i] = reinterpret_cast<const uint16_t*>(reinterpret_cast<const uint8_t*>(a.scales) + e_scales) + (int64_t)rtile * a.row_tile_scale_halfs;
  }
  {
    const int rtile = min(n0 / 16 + wave * 2 + ti, a.row_tiles - 1);
    al_t = reinterpret_cast<const float*>(reinterpret_cast<const uint8_t*>(a.alpha) + e_ab)[min(rtile * 16 + nl, a.n_last)];
    be_t = reinterpret_cast<const float*>(reinterpret_cast<const uint8_t*>(a.beta) + e_ab)[min(rtile * 16 + nl, a.n_last)];
    // expert e's super scales: half the byte stride of alpha / beta (fp16 against fp32)
    if constexpr (SM == 1)
      ssup_t = (float)__builtin_bit_cast(_Float16, reinterpret_cast<const uint16_t*>(reinterpret_cast<const uint8_t*>(a.scale_super) + e_ab / 2)[min(rtile * 16 + nl, a.n_last)]);
  }
  uint32_t mask2 = kDecMask2, base2 = kDecBase2;
  float magic = 8388608.f;
  asm volatile("" : "+s"(mask2), "+v"(base2), "+v"(magic));

  // raw code tiles as loaded (lane = row nl, quarter lane / 16, both row tiles), and the exchanged ones (this lane's
  // column: ex[q] = the four groups' dwords of quarter 2h + q)
  u32x4 craw[2], craw_next[2];
  uint2 sraw[2], sraw_next[2];
  u32x4 ex[2];
  uint2 s_t;
  auto load_codes = [&](u32x4 (&c)[2], uint2 (&sc)[2], int kt) {
    kt = min(kt, a.tiles[kNarrow] - 1);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      c[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(code_base[i] + (int64_t)kt * kNarrowTileBytes + lane * 16));
      if constexpr (SM == 0) sc[i] = *reinterpret_cast<const uint2*>(scale_base[i] + (int64_t)kt * kNarrowTileScaleHalfs + nl * 4);
      else sc[i] = uint2{(uint32_t)scale_base[i][(int64_t)kt * kNarrowTileScaleHalfs4 + nl], 0u};
    }
  };
  auto exchange = [&]() {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int src = (nl + 16 * (2 * h + q)) * 4;
      u32x4 r;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const uint32_t r0 = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)craw[0][d]);
        const uint32_t r1 = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)craw[1][d]);
        r[d] = ti ? r1 : r0;
      }
      ex[q] = r;
    }
    s_t = ti ? sraw[1] : sraw[0];  // every quarter-lane of a row holds the row's scales
  };

  const uint16_t* xrow[2];
  int a_lds_off[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = tid + 256 * i, row = c >> 3, col = c & 7;
    int64_t xr = row_off + min(m0 + row, Me - 1);  // rows past the end re-read the last row; their products are never stored
    if constexpr (GROUPED) {
      if (a.sorted_rows) xr = a.sorted_rows[xr];
    }
    xrow[i] = a.x + xr * a.ldx + col * 8;
    a_lds_off[i] = row * ROW + col * 8;
  }
  auto load_a = [&](u32x4 (&dst)[2], int s) {
    const int64_t off = (int64_t)min(tA * kNarrowGroupsPerTile + min(s, nsteps - 1), a.g_last) * kGroup;
#pragma unroll
    for (int i = 0; i < 2; ++i) dst[i] = *reinterpret_cast<const u32x4*>(xrow[i] + off);
  };
  auto store_a = [&](int buf, const u32x4 (&src)[2]) {
    uint16_t* dst = As + buf * kMidBM * ROW;
#pragma unroll
    for (int i = 0; i < 2; ++i) *reinterpret_cast<u32x4*>(dst + a_lds_off[i]) = src[i];
  };

  // group j of the held k-tile: 32 weights of this lane's column, as four MFMA B fragments
  auto decode = [&](u32x4 (&bf)[4], int j) {
    float s;
    if constexpr (SM == 0) {
      const uint32_t sd = (j >> 1) ? s_t.y : s_t.x;
      s = (float)__builtin_bit_cast(_Float16, (uint16_t)((j & 1) ? (sd >> 16) : (sd & 0xFFFFu)));
    } else {
      s = (float)((s_t.x >> (4 * j)) & 0xFu) * ssup_t;
    }
    const float c0 = -(kDecBase + a.zp[kNarrow]) * s;
    const float bem = be_t + magic;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const uint32_t d = dword_sel(ex[q], j);
      uint32_t o[8];
      decode16_narrow(d, al_t, bem, s, c0, mask2, base2, o);
      bf[2 * q] = u32x4{o[0], o[1], o[2], o[3]};
      bf[2 * q + 1] = u32x4{o[4], o[5], o[6], o[7]};
    }
  };

  f32x16 acc[2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  const int a_frag_off = (lane & 31) * ROW + h * 32;
  auto multiply = [&](int buf, const u32x4 (&bf)[4]) {
    const uint16_t* Ab = As + buf * kMidBM * ROW + a_frag_off;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const bf16x8 af = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Ab + i * 32 * ROW + kk * 8));
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, __builtin_bit_cast(bf16x8, bf[kk]), acc[i], 0, 0, 0);
      }
    }
  };
  auto lds_barrier = [&]() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  };

  {
    u32x4 areg[4][2];
    u32x4 bcur[4], bnext[4];
    int s = 0;
    load_codes(craw, sraw, tA);
    load_a(areg[0], 0);
    load_a(areg[1], 1);
    load_a(areg[2], 2);
    load_a(areg[3], 3);
    store_a(0, areg[0]);
    exchange();
    decode(bcur, 0);
    lds_barrier();
    // one step (J = s & 3): the activation tile of step s is multiplied with the fragments decoded during the previous
    // step, while the fragments of step s + 1 are decoded and its activation tile goes to the other LDS buffer
    auto step = [&](auto JC, auto&& prepare_next) {
      constexpr int J = decltype(JC)::value;
      constexpr int P = J & 1;
      load_a(areg[J], s + 4);
      prepare_next();
      multiply(P, bcur);
      store_a(P ^ 1, areg[(J + 1) & 3]);
#pragma unroll
      for (int k = 0; k < 4; ++k) bcur[k] = bnext[k];
      lds_barrier();
      ++s;
    };
    using J0 = std::integral_constant<int, 0>;
    using J1 = std::integral_constant<int, 1>;
    using J2 = std::integral_constant<int, 2>;
    using J3 = std::integral_constant<int, 3>;
    for (int t = tA; t < tB; ++t) {
      load_codes(craw_next, sraw_next, t + 1);
      step(J0{}, [&]() { decode(bnext, 1); });
      step(J1{}, [&]() { decode(bnext, 2); });
      step(J2{}, [&]() { decode(bnext, 3); });
      step(J3{}, [&]() {
#pragma unroll
        for (int i = 0; i < 2; ++i) { craw[i] = craw_next[i]; sraw[i] = sraw_next[i]; }
        exchange();
        decode(bnext, 0);  // of the next k-tile (a repeat of the last one after the last: not used)
      });
    }
  }

  const int n = n0 + wave * 32 + (lane & 31);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      const float val = acc[i][r];
      if (m < Me && n <= a.n_last) {
        if (gridDim.y > 1) __builtin_nontemporal_store(val, &a.partial[((int64_t)split * a.M + row_off + m) * a.N + n]);
        else a.y[(int64_t)(row_off + m) * a.ldy + n] = (uint16_t)(pack_bf16_m(val, 0.f) & 0xFFFFu);
      }
    }
  }
}

// K shares for the mid-M kernel.  The kernel is bound by instruction issue, and a second workgroup on a CU
// adds only about 15 %, while every share costs a pass of fp32 partial tiles through memory (written, then
// read by the reduction): aim at one workgroup per CU, at least two k-tiles of every format per share.
int mid_splits(const Layout& L, int M) {
  const int64_t blocks = (int64_t)((M + kMidBM - 1) / kMidBM) * ((L.N + kMidBN - 1) / kMidBN);
  const int min_tiles = std::min(L.tiles[kNarrow] > 0 ? L.tiles[kNarrow] : 1 << 30, L.tiles[kWide] > 0 ? L.tiles[kWide] : 1 << 30);
  // one workgroup per CU, or two when the weights have wide-format groups and there are at least 128 blocks: that
  // kernel moves more through LDS per MFMA and gains from a second workgroup on the CU (config 3, M = 64: 84 -> 75 us),
  // the register-decode kernel for the narrow format does not
  const int64_t cus = device_cus();
  const int64_t target = (L.tiles[kWide] > 0 && 2 * blocks >= cus) ? 2 * cus : cus;
  int64_t s = std::max<int64_t>(1, target / std::max<int64_t>(1, blocks));
  s = std::min<int64_t>(s, 8);
  s = std::min<int64_t>(s, std::max(1, min_tiles / 2));
  return (int)s;
}

int launch_mid(const ccq_weight* w, const Layout& L, const void* x, int M, int64_t ldx, void* y, int64_t ldy, float* partial, int S,
               void* stream) {
  MidArgs a;
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
  a.m_blocks = (M + kMidBM - 1) / kMidBM;
  a.tiles[0] = L.tiles[0];
  a.tiles[1] = L.tiles[1];
  a.groups_narrow = L.pgroups[kNarrow];
  a.sorted_rows = nullptr;
  a.expert_offsets = nullptr;
  a.codes_stride = a.scales_stride = a.ab_stride = 0;
  for (int k = 0; k < 2; ++k) {
    a.sq[k] = L.tiles[k] / S;
    a.sr[k] = L.tiles[k] % S;
    a.zp[k] = L.zp[k];
  }
  const int n_blocks = (L.N + kMidBN - 1) / kMidBN;
  const int fm = L.h16 ? 4 : (L.tiles[kNarrow] > 0 ? 1 : 0) | (L.tiles[kWide] > 0 ? 2 : 0);
  const int max_steps = ((L.tiles[kNarrow] + S - 1) / S) * kNarrowGroupsPerTile + ((L.tiles[kWide] + S - 1) / S) * kWideGroupsPerTile;
  if (fm == 1) {  // narrow format only: decoded weights stay in registers
    const size_t lds_r = (size_t)2 * kMidBM * kMidRow * 2;
    dim3 grid_r((unsigned)(a.m_blocks * n_blocks), (unsigned)S), block_r(256);
    if (L.scale_mode == 0) hipLaunchKernelGGL((ccq_midr_narrow_kernel<0, false>), grid_r, block_r, lds_r, static_cast<hipStream_t>(stream), a);
    else hipLaunchKernelGGL((ccq_midr_narrow_kernel<1, false>), grid_r, block_r, lds_r, static_cast<hipStream_t>(stream), a);
    if (hipGetLastError() != hipSuccess) return CCQ_ERR_HIP;
    return CCQ_OK;
  }
  const size_t lds = (size_t)2 * (kMidBM + kMidBN) * (fm == 4 ? kMidRowH16 : kMidRow) * 2 + (fm == 3 ? (size_t)max_steps * 4 : 0);
  if (lds > (fm == 4 ? 72 : 64) * 1024) return CCQ_ERR_UNSUPPORTED;
  typedef void (*MidKernel)(const MidArgs);
  const MidKernel table[2][4] = {{ccq_mid_kernel<1, 0, false>, ccq_mid_kernel<2, 0, false>, ccq_mid_kernel<3, 0, false>, ccq_mid_kernel<4, 0, false>},
                                 {ccq_mid_kernel<1, 1, false>, ccq_mid_kernel<2, 1, false>, ccq_mid_kernel<3, 1, false>, ccq_mid_kernel<4, 1, false>}};
  const MidKernel kern = table[L.scale_mode][fm - 1];
  if (!kern) return CCQ_ERR_UNSUPPORTED;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
    (void)hipGetLastError();
    return CCQ_ERR_HIP;
  }
  dim3 grid((unsigned)(a.m_blocks * n_blocks), (unsigned)S), block(64 * kMidWaves);
  hipLaunchKernelGGL(kern, grid, block, lds, static_cast<hipStream_t>(stream), a);
  if (hipGetLastError() != hipSuccess) return CCQ_ERR_HIP;
  return CCQ_OK;
}

// Grouped GEMM with many rows per expert: the 64-row kernel (register-decode variant for the narrow format) over
// (row block of the expert, column block, expert); blocks past an expert's rows return at once.  `most_rows` = the
// largest row count of an expert (from the host copy of the offsets); K is not cut (no workspace).
int launch_mid_grouped(const ccq_weight* w0, const Layout& L, int E, int64_t codes_stride, int64_t scales_stride, int64_t ab_stride, const void* x,
                       int64_t ldx, const int32_t* sorted_rows, int P, const int32_t* expert_offsets, int most_rows, void* y, int64_t ldy,
                       void* stream) {
  if (E < 1 || E > 65535 || most_rows < 1) return CCQ_ERR_UNSUPPORTED;
  MidArgs a;
  a.codes = static_cast<const uint8_t*>(w0->codes);
  a.scales = static_cast<const uint16_t*>(w0->scales);
  a.alpha = w0->code_alpha;
  a.beta = w0->code_beta;
  a.meta = static_cast<const int32_t*>(w0->meta);
  a.scale_super = static_cast<const uint16_t*>(w0->scale_super);
  a.x = static_cast<const uint16_t*>(x);
  a.y = static_cast<uint16_t*>(y);
  a.partial = nullptr;
  a.ldx = ldx;
  a.ldy = ldy;
  a.row_tile_bytes = L.row_tile_bytes;
  a.row_tile_scale_halfs = L.row_tile_scale_halfs;
  a.M = P;
  a.N = L.Npad;
  a.g_last = L.G - 1;
  a.n_last = L.N - 1;
  a.row_tiles = L.row_tiles;
  a.m_blocks = (most_rows + kMidBM - 1) / kMidBM;
  a.tiles[0] = L.tiles[0];
  a.tiles[1] = L.tiles[1];
  a.groups_narrow = L.pgroups[kNarrow];
  for (int k = 0; k < 2; ++k) {
    a.sq[k] = L.tiles[k];
    a.sr[k] = 0;
    a.zp[k] = L.zp[k];
  }
  a.sorted_rows = sorted_rows;
  a.expert_offsets = expert_offsets;
  a.codes_stride = codes_stride;
  a.scales_stride = scales_stride;
  a.ab_stride = ab_stride;
  const int n_blocks = (L.N + kMidBN - 1) / kMidBN;
  dim3 grid((unsigned)(a.m_blocks * n_blocks), 1u, (unsigned)E), block(256);
  const int fm = L.h16 ? 4 : (L.tiles[kNarrow] > 0 ? 1 : 0) | (L.tiles[kWide] > 0 ? 2 : 0);
  if (fm == 1) {  // narrow format only: decoded weights stay in registers
    const size_t lds_r = (size_t)2 * kMidBM * kMidRow * 2;
    if (L.scale_mode == 0) hipLaunchKernelGGL((ccq_midr_narrow_kernel<0, true>), grid, block, lds_r, static_cast<hipStream_t>(stream), a);
    else hipLaunchKernelGGL((ccq_midr_narrow_kernel<1, true>), grid, block, lds_r, static_cast<hipStream_t>(stream), a);
    if (hipGetLastError() != hipSuccess) return CCQ_ERR_HIP;
    return CCQ_OK;
  }
  const int max_steps = L.tiles[kNarrow] * kNarrowGroupsPerTile + L.tiles[kWide] * kWideGroupsPerTile;
  const size_t lds = (size_t)2 * (kMidBM + kMidBN) * (fm == 4 ? kMidRowH16 : kMidRow) * 2 + (fm == 3 ? (size_t)max_steps * 4 : 0);
  if (lds > (fm == 4 ? 72 : 64) * 1024) return CCQ_ERR_UNSUPPORTED;
  typedef void (*MidKernel)(const MidArgs);
  const MidKernel table[2][3] = {{ccq_mid_kernel<2, 0, true>, ccq_mid_kernel<3, 0, true>, ccq_mid_kernel<4, 0, true>},
                                 {ccq_mid_kernel<2, 1, true>, ccq_mid_kernel<3, 1, true>, ccq_mid_kernel<4, 1, true>}};
  const MidKernel kern = table[L.scale_mode][fm - 2];
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
    (void)hipGetLastError();
    return CCQ_ERR_HIP;
  }
  hipLaunchKernelGGL(kern, grid, dim3(64 * kMidWaves), lds, static_cast<hipStream_t>(stream), a);
  if (hipGetLastError() != hipSuccess) return CCQ_ERR_HIP;
  return CCQ_OK;
}

}  // namespace ccq
