// Prefill (large M) fused dequantize-and-multiply for the narrow format
// (L=6,N=4,S=3 + Code Cluster), gfx950.
//
// This is the one place where the work is a dense contraction: a workgroup owns
// a 256 x BN tile of the output, walks K in steps of one 64-weight group, and per
// step
//   - copies the 256 x 64 activation tile to LDS,
//   - decodes the BN x 64 weight tile to bf16 in LDS: the stored byte q becomes
//     the 15-bit code c = round(q*alpha + beta) (Alg. 3) with one FMA against
//     beta + 2^23, the four states are cut out by the shift list [9,6,3,0] and mask
//     0x3F (Table 1), two codes at a time, into the mantissas of two fp16 64.0, and
//     one mixed-precision FMA applies d = (w_uint - zp) * s (Alg. 3, last line):
//     fma(64 + state, s, -(64 + zp) s) is exact in fp32, so the value written is the
//     correctly rounded bf16 of the exact weight (decode16_narrow, ccq_decode.h),
//   - multiplies the two tiles with MFMA 32x32x16 bf16 (fp32 accumulators).
// LDS tiles are double buffered; rows are padded by 16 bytes so that operand
// reads (16 bytes per lane, 32 consecutive rows) spread over all banks.
//
// Workgroup-to-tile map: consecutive workgroup ids walk the M blocks first; with
// 8 M blocks (M = 2048) every XCD keeps one 256-row slab of the activations in its
// own L2 and streams the (small) code bytes.
//
// Two kernels share this design: ccq_prefill8_kernel (BN = 192 or 128, eight wavefronts, two per
// SIMD) when that block width divides N, and ccq_prefill_kernel<4> (BN = 256, four wavefronts) otherwise.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "ccq_decode.h"
#include "ccq_internal.h"

namespace ccq {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

struct PrefillArgs {
  const uint8_t* codes;
  const uint16_t* scales;
  const float* alpha;
  const float* beta;
  const uint16_t* scale_super;  // fp16 [N], compressed scales only
  const uint16_t* x;
  uint16_t* y;
  int64_t ldx, ldy;
  int64_t row_tile_bytes, row_tile_scale_halfs;
  int32_t M, N, K;               // K: columns of the device layout (whole k-tiles of 256)
  int32_t g_last;                // last real group of K: groups past it pad a k-tile (zero scale) and read this group's activations
  int32_t row_tiles;
  int32_t m_blocks;
  float zp;
};

constexpr int kBM = 256;          // output rows (activation rows) per workgroup
constexpr int kBK = 64;           // one group per step
constexpr int kLdsRow = kBK + 8;  // bf16 elements per padded LDS row (144 bytes)

// (a & mask) | orv in plain C (no instruction is written as inline assembly: the compiler's hazard
// recognizer does not see those); mask and orv are kept in registers so v_and_or_b32 is selected.
__device__ __forceinline__ uint32_t and_or_p(uint32_t a, uint32_t mask, uint32_t orv) { return (a & mask) | orv; }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);  // round to nearest even
  return __builtin_bit_cast(uint32_t, b);
}

// RTW = 16-row weight tiles decoded per wavefront per step; BN = 64 * RTW.
// SM: scale mode (0 fp16 group scales; 1 the compressed scales of Sec. 3.4: 4-bit field * per-row super scale).
template <int RTW, int SM>
__global__ void __launch_bounds__(256) ccq_prefill_kernel(const PrefillArgs a) {
  constexpr int BN = 64 * RTW;
  constexpr int NT = BN / 64;  // 32-wide MFMA column tiles per wavefront (wave tile is 128 x BN/2)
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* As = reinterpret_cast<uint16_t*>(smem);                          // [2][kBM][kLdsRow]
  uint16_t* Bs = As + 2 * kBM * kLdsRow;                                     // [2][BN][kLdsRow]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: tile base pointers stay in scalar registers
  const int wm = wave >> 1, wn = wave & 1;
  const int m_block = blockIdx.x % a.m_blocks, n_block = blockIdx.x / a.m_blocks;
  const int m0 = m_block * kBM, n0 = n_block * BN;
  const int kq = lane >> 4, nl = lane & 15;

  // per-thread weight rows: tiles rt = wave*RTW + i of this block, row nl, quarter kq
  const uint8_t* code_ptr[RTW];
  const uint16_t* scale_ptr[RTW];
  float al[RTW], be[RTW], ssup[RTW];
#pragma unroll
  for (int i = 0; i < RTW; ++i) {
    int rtile = n0 / 16 + wave * RTW + i;
    rtile = min(rtile, a.row_tiles - 1);  // ragged last block: re-decode the last tile, never stored
    code_ptr[i] = a.codes + (int64_t)rtile * a.row_tile_bytes;                 // + lane * 16 at the load
    scale_ptr[i] = a.scales + (int64_t)rtile * a.row_tile_scale_halfs;         // + nl * 4 (or + nl) at the load
    const int prow = min(rtile * 16 + nl, a.N - 1);  // rows that pad the last tile take the last row's parameters; never stored
    al[i] = a.alpha[prow];
    be[i] = a.beta[prow] + 8388608.f;
    ssup[i] = 0.f;
    if constexpr (SM == 1) ssup[i] = (float)__builtin_bit_cast(_Float16, a.scale_super[prow]);
  }
  uint32_t base2 = kDecBase2, mask2 = kDecMask2;
  asm volatile("" : "+v"(base2), "+s"(mask2));
  const float neg_off = -(kDecBase + a.zp);
  const uint32_t lane_code_off = lane * 16, lane_scale_off = nl * 4;

  // activation copy: 8 chunks of 16 bytes per thread and step; rows past M re-read row M-1 (their
  // products land in accumulator rows that are never stored)
  // (32-bit byte offsets from the uniform base; the launcher checks that the tile fits 2^31 bytes)
  uint32_t xoff[8];
  int a_lds_off[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int c = tid + 256 * i, row = c >> 3, col = c & 7;
    xoff[i] = (uint32_t)(((int64_t)min(m0 + row, a.M - 1) * a.ldx + col * 8) * 2);
    a_lds_off[i] = row * kLdsRow + col * 8;
  }

  f32x16 acc[4][NT];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nsteps = a.K / kBK;       // a multiple of 4 (narrow k-tiles span 4 groups)
  const int ntiles = nsteps >> 2;
  // Activation chunks in registers on their way to LDS: two sets (step s in set s & 1, requested two
  // steps ahead of its multiplication).  AD = 1 keeps a single set, refilled as soon as its chunks have
  // been written to LDS, should registers ever be short.
  constexpr int AD = 2;
  u32x4 areg[AD][8];
  u32x4 creg[RTW], cnext[RTW];        // codes of the k-tile being decoded / of the next one
  uint2 sreg[RTW], snext[RTW];

  auto load_a = [&](u32x4 (&dst)[8], int step) {
    const char* base = reinterpret_cast<const char*>(a.x + (int64_t)min(step, a.g_last) * kBK);
#pragma unroll
    for (int i = 0; i < 8; ++i) dst[i] = *reinterpret_cast<const u32x4*>(base + xoff[i]);
  };
  auto load_codes = [&](u32x4 (&c)[RTW], uint2 (&sc)[RTW], int kt) {
    kt = min(kt, ntiles - 1);
#pragma unroll
    for (int i = 0; i < RTW; ++i) {
      c[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(code_ptr[i] + (int64_t)kt * kNarrowTileBytes + lane_code_off));
      if constexpr (SM == 0) sc[i] = *reinterpret_cast<const uint2*>(scale_ptr[i] + (int64_t)kt * kNarrowTileScaleHalfs + lane_scale_off);
      else sc[i] = uint2{(uint32_t)scale_ptr[i][(int64_t)kt * kNarrowTileScaleHalfs4 + nl], 0u};  // the tile's four 4-bit fields
    }
  };
  auto store_a = [&](int buf, const u32x4 (&src)[8], int i0, int i1) {
    uint16_t* dst = As + buf * kBM * kLdsRow;
#pragma unroll
    for (int i = i0; i < i1; ++i) *reinterpret_cast<u32x4*>(dst + a_lds_off[i]) = src[i];
  };
  // decode group j (0..3) of row tile i of the held k-tile into LDS buffer `buf`
  auto decode_b = [&](int buf, int j, int i) {
    uint16_t* dst = Bs + buf * BN * kLdsRow;
    const uint32_t d = j == 0 ? creg[i].x : (j == 1 ? creg[i].y : (j == 2 ? creg[i].z : creg[i].w));
    float s;
    if constexpr (SM == 0) {
      const uint32_t sw = (j >> 1) ? sreg[i].y : sreg[i].x;
      s = (float)__builtin_bit_cast(_Float16, (uint16_t)((j & 1) ? (sw >> 16) : (sw & 0xFFFFu)));
    } else {
      s = (float)((sreg[i].x >> (4 * j)) & 0xFu) * ssup[i];  // (s_q >> s_shift) & s_mask times s_super (Alg. 3): exact
    }
    const float c0 = neg_off * s;  // exact: 8-bit times at most 15-bit significand
    uint32_t o[8];
    decode16_narrow(d, al[i], be[i], s, c0, mask2, base2, o);
    uint16_t* p = dst + ((wave * RTW + i) * 16 + nl) * kLdsRow + kq * 16;
    *reinterpret_cast<u32x4*>(p) = u32x4{o[0], o[1], o[2], o[3]};
    *reinterpret_cast<u32x4*>(p + 8) = u32x4{o[4], o[5], o[6], o[7]};
  };

  // MFMA operand fragments, double buffered in registers: while the 4 x NT products of one
  // 16-wide k slice run, the fragments of the next slice are on their way from LDS.
  bf16x8 af[2][4], bfr[2][NT];
  const int a_frag_off = (wm * 128 + (lane & 31)) * kLdsRow + (lane >> 5) * 8;
  const int b_frag_off = (wn * (BN / 2) + (lane & 31)) * kLdsRow + (lane >> 5) * 8;
  auto load_frags = [&](int par, int buf, int kk) {
    const uint16_t* Ab = As + buf * kBM * kLdsRow + a_frag_off + kk * 16;
    const uint16_t* Bb = Bs + buf * BN * kLdsRow + b_frag_off + kk * 16;
#pragma unroll
    for (int i = 0; i < 4; ++i) af[par][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Ab + i * 32 * kLdsRow));
#pragma unroll
    for (int j = 0; j < NT; ++j) bfr[par][j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Bb + j * 32 * kLdsRow));
  };
  auto mfma_rows = [&](int par, int i0, int i1) {
#pragma unroll
    for (int i = i0; i < i1; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[par][i], bfr[par][j], acc[i][j], 0, 0, 0);
  };
  // Workgroup barrier that orders LDS traffic only: global loads issued for later steps stay in
  // flight across it.
  auto lds_barrier = [&]() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  };

  // prologue: steps 0 and 1 of the activations and k-tile 0 of the codes are fetched; step 0 goes to
  // LDS buffer 0
  load_a(areg[0], 0);
  load_codes(creg, sreg, 0);
  if constexpr (AD == 2) load_a(areg[1], 1);
  store_a(0, areg[0], 0, 8);
  if constexpr (AD == 1) load_a(areg[0], 1);
#pragma unroll
  for (int i = 0; i < RTW; ++i) decode_b(0, 0, i);
  lds_barrier();
  load_frags(0, 0, 0);

  // One step (J = step & 3).  While buffer J&1 is multiplied, step + 1 is written to the other
  // buffer (activation chunks fetched a step earlier, weight group J+1 of the held k-tile), the
  // activations of step + 2 and, once per k-tile, the codes of the next k-tile are requested.
  // Everything is unconditional: past the end, loads re-read the last step and the extra LDS
  // contents are never multiplied.
  auto body = [&](int step, auto JC) {
    constexpr int J = decltype(JC)::value;
    constexpr int buf = J & 1;
    if constexpr (AD == 2) load_a(areg[J & 1], step + 2);
    if constexpr (J == 1) load_codes(cnext, snext, (step >> 2) + 1);
    __builtin_amdgcn_sched_barrier(0);  // the requests go out first: nothing below may move above them
    if constexpr (J == 3) {
#pragma unroll
      for (int i = 0; i < RTW; ++i) { creg[i] = cnext[i]; sreg[i] = snext[i]; }
    }
    constexpr int jn = (J + 1) & 3;
    // slice 0
    load_frags(1, buf, 1);
    mfma_rows(0, 0, 4);
    store_a(buf ^ 1, areg[(J + 1) & (AD - 1)], 0, 4);
    decode_b(buf ^ 1, jn, 0);
    // slice 1
    load_frags(0, buf, 2);
    mfma_rows(1, 0, 4);
    store_a(buf ^ 1, areg[(J + 1) & (AD - 1)], 4, 8);
    if constexpr (AD == 1) load_a(areg[0], step + 2);
    decode_b(buf ^ 1, jn, 1);
    // slice 2 and the first half of slice 3
    load_frags(1, buf, 3);
    mfma_rows(0, 0, 4);
#pragma unroll
    for (int i = 2; i < RTW; ++i) decode_b(buf ^ 1, jn, i);
    mfma_rows(1, 0, 2);
    // issue order inside this region: one MFMA, a few vector ALU instructions, one LDS access
#pragma unroll
    for (int i = 0; i < 14 * NT; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);
      __builtin_amdgcn_sched_group_barrier(0x080, 1, 0);
    }
    lds_barrier();
    // rest of slice 3, with the first fragments of the next step
    load_frags(0, buf ^ 1, 0);
    mfma_rows(1, 2, 4);
  };
  for (int step = 0; step < nsteps; step += 4) {
    body(step, std::integral_constant<int, 0>{});
    body(step + 1, std::integral_constant<int, 1>{});
    body(step + 2, std::integral_constant<int, 2>{});
    body(step + 3, std::integral_constant<int, 3>{});
  }

  // epilogue: D[row][col], row = 8*(r/4) + 4*(lane/32) + r%4, col = lane%32.  One store writes two
  // 64-byte row segments; blocks that lie fully inside the output take the path without per-element tests.
  const bool inside = (m0 + kBM <= a.M) && (n0 + BN <= a.N);
  uint16_t* ybase = a.y + (int64_t)(m0 + wm * 128 + 4 * (lane >> 5)) * a.ldy + (n0 + wn * (BN / 2) + (lane & 31));
  const int mlim = a.M - (m0 + wm * 128 + 4 * (lane >> 5));        // rows of this lane's row set that exist
  const int nlim = a.N - (n0 + wn * (BN / 2) + (lane & 31));        // columns likewise
  // (the test of `inside` sits inside the tile loop: around it, the compiler moves all 16 NT x 4 accumulator
  // reads above the branch and runs out of registers)
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      uint32_t bits[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float val = acc[i][j][r];  // by value: bit-casting the element lvalue itself reads element 0
        bits[r] = pack_bf16(val, 0.f);   // round to nearest even
      }
      uint16_t* dst = ybase + (int64_t)(i * 32) * a.ldy + j * 32;
      if (inside) {
#pragma unroll
        for (int r = 0; r < 16; ++r) dst[(int64_t)(8 * (r >> 2) + (r & 3)) * a.ldy] = (uint16_t)bits[r];
      } else if (j * 32 < nlim) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int mrel = i * 32 + 8 * (r >> 2) + (r & 3);
          if (mrel < mlim) dst[(int64_t)(8 * (r >> 2) + (r & 3)) * a.ldy] = (uint16_t)bits[r];
        }
      }
    }
  }
}

// The same tile with eight wavefronts (two per SIMD): a single wavefront cannot issue its LDS and
// global-memory instructions underneath its own MFMAs (each costs it several issue slots), a second
// one on the SIMD fills those slots.  Wave grid 4 (M) x 2 (N), wave tile 64 x 32 NT, BN = 64 NT
// (NT = 3: 192 columns, NT = 2: 128).  Every wavefront decodes row tile `wave` of the block; with 192
// columns wavefronts 0-3 decode row tiles 8-11 as well (their SIMD partners, wavefronts 4-7, have one
// tile each, so every SIMD carries the same work).
template <int NT, int SM>
__global__ void __launch_bounds__(512) ccq_prefill8_kernel(const PrefillArgs a) {
  constexpr int BN = 64 * NT;
  constexpr int kExtra = BN / 16 - 8;  // wavefronts that own a second row tile (4 or 0)
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* As = reinterpret_cast<uint16_t*>(smem);                          // [2][kBM][kLdsRow]
  uint16_t* Bs = As + 2 * kBM * kLdsRow;                                     // [2][BN][kLdsRow]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int m_block = blockIdx.x % a.m_blocks, n_block = blockIdx.x / a.m_blocks;
  const int m0 = m_block * kBM, n0 = n_block * BN;
  const int kq = lane >> 4, nl = lane & 15;
  const bool has_extra = kExtra > 0 && wave < kExtra;

  // row tiles of this wavefront: slot 0 = tile `wave`, slot 1 = tile 8 + wave (wavefronts 0-3 only)
  const uint8_t* code_ptr[2];
  const uint16_t* scale_ptr[2];
  float al[2], be[2], ssup[2];
  int tile_in_block[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    tile_in_block[i] = (i == 0 || kExtra == 0) ? wave : 8 + (wave & (kExtra > 0 ? kExtra - 1 : 0));
    int rtile = n0 / 16 + tile_in_block[i];
    rtile = min(rtile, a.row_tiles - 1);  // ragged last block: re-decode the last tile, never stored
    code_ptr[i] = a.codes + (int64_t)rtile * a.row_tile_bytes;
    scale_ptr[i] = a.scales + (int64_t)rtile * a.row_tile_scale_halfs;
    const int prow = min(rtile * 16 + nl, a.N - 1);  // rows that pad the last tile take the last row's parameters; never stored
    al[i] = a.alpha[prow];
    be[i] = a.beta[prow] + 8388608.f;
    ssup[i] = 0.f;
    if constexpr (SM == 1) ssup[i] = (float)__builtin_bit_cast(_Float16, a.scale_super[prow]);
  }
  uint32_t base2 = kDecBase2, mask2 = kDecMask2;
  asm volatile("" : "+v"(base2), "+s"(mask2));
  const float neg_off = -(kDecBase + a.zp);
  const uint32_t lane_code_off = lane * 16, lane_scale_off = nl * 4;

  // activation copy: 4 chunks of 16 bytes per thread and step (rows past M re-read row M-1)
  uint32_t xoff[4];
  int a_lds_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + 512 * i, row = c >> 3, col = c & 7;
    xoff[i] = (uint32_t)(((int64_t)min(m0 + row, a.M - 1) * a.ldx + col * 8) * 2);
    a_lds_off[i] = row * kLdsRow + col * 8;
  }

  f32x16 acc[2][NT];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nsteps = a.K / kBK;
  const int ntiles = nsteps >> 2;
  u32x4 areg[4];  // activation chunks of the next step on their way to LDS
  u32x4 creg[2], cnext[2];
  uint2 sreg[2], snext[2];

  auto load_a = [&](u32x4 (&dst)[4], int step) {
    const char* base = reinterpret_cast<const char*>(a.x + (int64_t)min(step, a.g_last) * kBK);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint32_t off = xoff[i];
      asm volatile("" : "+v"(off));  // keeps the zero extension next to the load: uniform base + 32-bit lane offset
      dst[i] = *reinterpret_cast<const u32x4*>(base + off);
    }
  };
  auto load_codes_slot = [&](u32x4& c, uint2& sc, int kt, int i) {
    c = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(code_ptr[i] + (int64_t)kt * kNarrowTileBytes + lane_code_off));
    if constexpr (SM == 0) sc = *reinterpret_cast<const uint2*>(scale_ptr[i] + (int64_t)kt * kNarrowTileScaleHalfs + lane_scale_off);
    else sc = uint2{(uint32_t)scale_ptr[i][(int64_t)kt * kNarrowTileScaleHalfs4 + nl], 0u};
  };
  auto load_codes = [&](u32x4 (&c)[2], uint2 (&sc)[2], int kt) {
    kt = min(kt, ntiles - 1);
    load_codes_slot(c[0], sc[0], kt, 0);
    if (has_extra) load_codes_slot(c[1], sc[1], kt, 1);
  };
  auto store_a = [&](int buf, const u32x4 (&src)[4], int i0, int i1) {
    uint16_t* dst = As + buf * kBM * kLdsRow;
#pragma unroll
    for (int i = i0; i < i1; ++i) *reinterpret_cast<u32x4*>(dst + a_lds_off[i]) = src[i];
  };
  // decode group j (0..3) of row-tile slot i of the held k-tile into LDS buffer `buf`
  auto decode_b = [&](int buf, int j, int i) {
    uint16_t* dst = Bs + buf * BN * kLdsRow;
    const uint32_t d = j == 0 ? creg[i].x : (j == 1 ? creg[i].y : (j == 2 ? creg[i].z : creg[i].w));
    float s;
    if constexpr (SM == 0) {
      const uint32_t sw = (j >> 1) ? sreg[i].y : sreg[i].x;
      s = (float)__builtin_bit_cast(_Float16, (uint16_t)((j & 1) ? (sw >> 16) : (sw & 0xFFFFu)));
    } else {
      s = (float)((sreg[i].x >> (4 * j)) & 0xFu) * ssup[i];
    }
    const float c0 = neg_off * s;  // exact: 8-bit times at most 15-bit significand
    uint32_t o[8];
    decode16_narrow(d, al[i], be[i], s, c0, mask2, base2, o);
    uint16_t* p = dst + (tile_in_block[i] * 16 + nl) * kLdsRow + kq * 16;
    *reinterpret_cast<u32x4*>(p) = u32x4{o[0], o[1], o[2], o[3]};
    *reinterpret_cast<u32x4*>(p + 8) = u32x4{o[4], o[5], o[6], o[7]};
  };

  bf16x8 af[2][2], bfr[2][NT];
  const int a_frag_off = (wm * 64 + (lane & 31)) * kLdsRow + (lane >> 5) * 8;
  const int b_frag_off = (wn * (BN / 2) + (lane & 31)) * kLdsRow + (lane >> 5) * 8;
  auto load_frags = [&](int par, int buf, int kk) {
    const uint16_t* Ab = As + buf * kBM * kLdsRow + a_frag_off + kk * 16;
    const uint16_t* Bb = Bs + buf * BN * kLdsRow + b_frag_off + kk * 16;
#pragma unroll
    for (int i = 0; i < 2; ++i) af[par][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Ab + i * 32 * kLdsRow));
#pragma unroll
    for (int j = 0; j < NT; ++j) bfr[par][j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Bb + j * 32 * kLdsRow));
  };
  auto mfma_rows = [&](int par, int i0, int i1) {
#pragma unroll
    for (int i = i0; i < i1; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[par][i], bfr[par][j], acc[i][j], 0, 0, 0);
  };
  auto lds_barrier = [&]() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  };

  load_a(areg, 0);
  load_codes(creg, sreg, 0);
  store_a(0, areg, 0, 4);
  load_a(areg, 1);
  decode_b(0, 0, 0);
  if (has_extra) decode_b(0, 0, 1);
  lds_barrier();
  load_frags(0, 0, 0);

  // One step (J = step & 3): buffer J&1 is multiplied while step + 1 is written to the other buffer.
  // HEAVY wavefronts (those with a second row tile) decode it inside the same stream, with more vector
  // instructions between two MFMAs; the two kinds run separate copies of the loop.
  auto body = [&](int step, auto JC, auto HC) {
    constexpr int J = decltype(JC)::value;
    constexpr bool HEAVY = decltype(HC)::value;
    constexpr int buf = J & 1;
    constexpr int jn = (J + 1) & 3;
    if constexpr (J == 1) {
      const int kt = min((step >> 2) + 1, ntiles - 1);
      load_codes_slot(cnext[0], snext[0], kt, 0);
      if constexpr (HEAVY) load_codes_slot(cnext[1], snext[1], kt, 1);
    }
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (J == 3) {
      creg[0] = cnext[0]; sreg[0] = snext[0];
      if constexpr (HEAVY) { creg[1] = cnext[1]; sreg[1] = snext[1]; }
    }
    // Program order: all fragment reads of this step first, the LDS writes of step + 1 last (the compiler
    // keeps LDS reads behind earlier LDS writes, so a write waiting for its decode would hold them back);
    // the issue order below spreads the decode arithmetic under the MFMAs all the same.
    load_frags(1, buf, 1);
    mfma_rows(0, 0, 2);
    load_frags(0, buf, 2);
    mfma_rows(1, 0, 2);
    load_frags(1, buf, 3);
    mfma_rows(0, 0, 2);
    mfma_rows(1, 0, 1);
    store_a(buf ^ 1, areg, 0, 4);
    load_a(areg, step + 2);
    decode_b(buf ^ 1, jn, 0);
    if constexpr (HEAVY) decode_b(buf ^ 1, jn, 1);
    // issue order inside this region: one MFMA, a few vector ALU instructions, one LDS access
#pragma unroll
    for (int i = 0; i < 7 * NT; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, HEAVY ? 7 : (NT == 2 ? 5 : 4), 0);
      __builtin_amdgcn_sched_group_barrier(0x080, 1, 0);
    }
    lds_barrier();
    load_frags(0, buf ^ 1, 0);
    mfma_rows(1, 1, 2);
  };
  bool heavy_loop = false;
  if constexpr (kExtra > 0) heavy_loop = has_extra;
  if (heavy_loop) {
    if constexpr (kExtra > 0) {
      for (int step = 0; step < nsteps; step += 4) {
        body(step, std::integral_constant<int, 0>{}, std::true_type{});
        body(step + 1, std::integral_constant<int, 1>{}, std::true_type{});
        body(step + 2, std::integral_constant<int, 2>{}, std::true_type{});
        body(step + 3, std::integral_constant<int, 3>{}, std::true_type{});
      }
    }
  } else {
    for (int step = 0; step < nsteps; step += 4) {
      body(step, std::integral_constant<int, 0>{}, std::false_type{});
      body(step + 1, std::integral_constant<int, 1>{}, std::false_type{});
      body(step + 2, std::integral_constant<int, 2>{}, std::false_type{});
      body(step + 3, std::integral_constant<int, 3>{}, std::false_type{});
    }
  }

  const bool inside = (m0 + kBM <= a.M) && (n0 + BN <= a.N);
  uint16_t* ybase = a.y + (int64_t)(m0 + wm * 64 + 4 * (lane >> 5)) * a.ldy + (n0 + wn * (BN / 2) + (lane & 31));
  const int mlim = a.M - (m0 + wm * 64 + 4 * (lane >> 5));
  const int nlim = a.N - (n0 + wn * (BN / 2) + (lane & 31));
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      uint32_t bits[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float val = acc[i][j][r];
        bits[r] = pack_bf16(val, 0.f);
      }
      uint16_t* dst = ybase + (int64_t)(i * 32) * a.ldy + j * 32;
      if (inside) {
#pragma unroll
        for (int r = 0; r < 16; ++r) dst[(int64_t)(8 * (r >> 2) + (r & 3)) * a.ldy] = (uint16_t)bits[r];
      } else if (j * 32 < nlim) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int mrel = i * 32 + 8 * (r >> 2) + (r & 3);
          if (mrel < mlim) dst[(int64_t)(8 * (r >> 2) + (r & 3)) * a.ldy] = (uint16_t)bits[r];
        }
      }
    }
  }
}

// Column blocks: 192 (eight wavefronts) when they tile N exactly; else 128 (eight wavefronts) when those tile N
// and fit one round of 256 workgroups; else 256 (four wavefronts, ragged last block allowed).
int prefill_block_cols(const Layout& L, int M) {
  const int64_t m_blocks = (M + kBM - 1) / kBM;
  if (L.N % 192 == 0) return 192;
  if (L.N % 128 == 0 && m_blocks * (L.N / 128) <= 256) return 128;
  return 256;
}

int launch_prefill(const ccq_weight* w, const Layout& L, const void* x, int M, int64_t ldx, void* y, int64_t ldy, void* stream) {
  PrefillArgs a;
  a.codes = static_cast<const uint8_t*>(w->codes);
  a.scales = static_cast<const uint16_t*>(w->scales);
  a.alpha = w->code_alpha;
  a.beta = w->code_beta;
  a.scale_super = static_cast<const uint16_t*>(w->scale_super);
  a.x = static_cast<const uint16_t*>(x);
  a.y = static_cast<uint16_t*>(y);
  a.ldx = ldx;
  a.ldy = ldy;
  a.row_tile_bytes = L.row_tile_bytes;
  a.row_tile_scale_halfs = L.row_tile_scale_halfs;
  a.M = M;
  a.N = L.N;
  a.K = L.tiles[kNarrow] * kNarrowGroupsPerTile * kGroup;
  a.g_last = L.G - 1;
  a.row_tiles = L.row_tiles;
  a.m_blocks = (M + kBM - 1) / kBM;
  a.zp = L.zp[kNarrow];
  if (((int64_t)M * ldx + L.K) * 2 >= (int64_t)1 << 31) return CCQ_ERR_UNSUPPORTED;  // activation offsets are 32-bit
  const int BN = prefill_block_cols(L, M);
  const int n_blocks = (L.N + BN - 1) / BN;
  const size_t lds = (size_t)2 * (kBM + BN) * kLdsRow * 2;
  typedef void (*PrefillKernel)(const PrefillArgs);
  const PrefillKernel table[2][3] = {{ccq_prefill8_kernel<2, 0>, ccq_prefill8_kernel<3, 0>, ccq_prefill_kernel<4, 0>},
                                     {ccq_prefill8_kernel<2, 1>, ccq_prefill8_kernel<3, 1>, ccq_prefill_kernel<4, 1>}};
  const PrefillKernel kern = table[L.scale_mode][BN == 128 ? 0 : (BN == 192 ? 1 : 2)];
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
    (void)hipGetLastError();
    return CCQ_ERR_HIP;
  }
  dim3 grid((unsigned)(a.m_blocks * n_blocks)), block(BN == 256 ? 256 : 512);
  hipLaunchKernelGGL(kern, grid, block, lds, static_cast<hipStream_t>(stream), a);
  if (hipGetLastError() != hipSuccess) return CCQ_ERR_HIP;
  return CCQ_OK;
}

}  // namespace ccq
