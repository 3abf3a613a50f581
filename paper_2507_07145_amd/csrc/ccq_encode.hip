// The offline quantizer of CCQ on the GPU (gfx950): Alg. 1 (group scale, nearest codeword of the
// convolutional codebook for every N-vector), the least-squares scale of Eq. 4 ("Scale Optimization"),
// and the Code Cluster map of Sec. 3.3 / Eq. 1, for the narrow (L=6,N=4,S=3 + Code Cluster) and the wide
// (L=4,N=3,S=2) formats.  Output goes straight into the device layout that ccq_gemm reads.
//
// The codebook is never built.  A code is a path through the state graph (first state, then S fresh
// bits per step), so the nearest codeword is a shortest path: 2^L lanes of a wavefront hold the 2^L
// states, one step takes the best of the 2^S predecessors of every state (lane shuffles), and the final
// answer is the best of the 2^L end states.  Ties go to the numerically lowest code at every
// comparison, which is what an exhaustive scan over all 2^T codes in ascending order returns.
//
// Every decision (an argmin, a kept-or-rejected scale) is taken in fp64 with separate multiplies and adds
// in a fixed order -- squared errors of a vector are added left to right, the sums of Eq. 4 and of the
// group error run over the 64 weights in index order -- so that the result does not depend on how the
// work is spread over lanes.  Contraction into fused multiply-adds is switched off for this file.
#include <hip/hip_runtime.h>

#include <cmath>

#include "ccq_internal.h"

#pragma clang fp contract(off)

namespace ccq {

struct EncArgs {
  const float* W;       // fp32 [N][ldw]
  int64_t ldw;
  int32_t N, G;        // rows; groups per row (all kinds)
  // the groups of the kind this launch works on (all of them unless the matrix mixes formats): GK groups per row,
  // the p-th of them is original group meta[mbase + p] (p itself without a map), entry pbase + p of a row in the
  // per-(row, group) workspace arrays, and sits at packed position p of the kind's k-tiles, which start
  // kind_code_off bytes / kind_scale_off halfwords into a row tile.  (The map holds whole k-tiles per kind, the
  // workspace arrays only the real groups: with a ragged last narrow tile mbase > pbase for the wide kind.)
  int32_t GK, pbase, mbase;
  const int32_t* meta;
  int64_t kind_code_off, kind_scale_off;
  double zp;
  uint8_t* codes;       // device order
  uint16_t* scales;     // device order, fp16 bits
  float* alpha;
  float* beta;
  uint16_t* rowcodes;   // workspace: the unclustered codes, [N][G][16] (narrow format only)
  uint16_t* rowscale;   // workspace: fp16 bits of the group scales after the first pass, [N][G]
  // compressed scales (Sec. 3.4) only:
  uint16_t* canon_scales;  // workspace: final fp16 group scales, [N][G] (not in device order); NULL = fp16 scales are the output
  uint8_t* fields;         // workspace: the 4-bit field of every group, [N][G]
  uint16_t* ssup;          // output: fp16 super scale per output channel, [N]
  double field_max;        // largest value of a scale field: 15, or 8191 for the hybrid word
  int64_t row_tile_bytes, row_tile_scale_halfs;
};

// ---- fp16 rounding of a non-negative finite double (11-bit significand, minimum normal exponent -14,
// subnormals with quantum 2^-24, round to nearest even), as a double; overflow gives +inf
__device__ __forceinline__ double fp16_round(double x) {
  if (x == 0.0) return 0.0;
  int e;
  (void)frexp(x, &e);  // x = f * 2^e, f in [0.5, 1)
  int q = e - 11;
  if (q < -24) q = -24;
  const double r = nearbyint(ldexp(x, -q));
  const double y = ldexp(r, q);
  return y > 65504.0 ? INFINITY : y;
}
// the scale that is stored: fp16-rounded, and the smallest normal fp16 number when that would be 0 or inf
__device__ __forceinline__ double fp16_scale(double s) {
  const double r = fp16_round(s);
  return (!(r > 0.0) || isinf(r)) ? 0x1p-14 : r;
}
// bit pattern of a non-negative double that is exactly an fp16 number
__device__ __forceinline__ uint16_t fp16_bits(double y) {
  if (y == 0.0) return 0;
  int e;
  const double f = frexp(y, &e);
  const int E = e - 1;
  if (E < -14) return (uint16_t)ldexp(y, 24);
  const uint16_t m = (uint16_t)ldexp(f, 11) & 0x3FFu;
  return (uint16_t)(((E + 15) << 10) | m);
}
__device__ __forceinline__ double fp16_value(uint16_t h) {
  const int e = (h >> 10) & 0x1F, m = h & 0x3FF;
  return e == 0 ? ldexp((double)m, -24) : ldexp((double)(m | 0x400), e - 25);
}

// (row, group) of a wavefront: n = row, p = position among the row's groups of this kind, g = original group
// (activation columns 64 g ..), widx = index into the per-(row, group) workspace arrays that span all kinds
struct GroupId {
  int n, p, g;
  int64_t widx;
};
__device__ __forceinline__ bool group_id(const EncArgs& a, int64_t gidx, GroupId& id) {
  if (gidx >= (int64_t)a.N * a.GK) return false;
  id.n = (int)(gidx / a.GK);
  id.p = (int)(gidx % a.GK);
  id.g = a.meta ? a.meta[a.mbase + id.p] : id.p;
  id.widx = (int64_t)id.n * a.G + a.pbase + id.p;
  return true;
}

__device__ __forceinline__ double sqerr(double v, double s, double lv) {
  const double d = v - s * lv;
  return d * d;
}

// Nearest codeword of one N-vector (Alg. 1, the argmin), by the 2^L lanes lane & ~(2^L - 1) .. of the
// wavefront; every lane of that set returns the code.  v[] must be the same in all lanes of the set.
template <int L, int NV, int S>
__device__ __forceinline__ uint32_t nearest_code(const double (&v)[NV], double s, double zp, int lane) {
  constexpr int NS = 1 << L, NT = 1 << S;
  const int st = lane & (NS - 1), base = lane & ~(NS - 1);
  const double lv = (double)st - zp;  // the state's value in the integer domain
  double cost = sqerr(v[0], s, lv);
  uint32_t pre = (uint32_t)st;  // code prefix of the best path that ends in this state
#pragma unroll
  for (int i = 1; i < NV; ++i) {
    const double e = sqerr(v[i], s, lv);
    double best = INFINITY;
    uint32_t bcode = 0xFFFFFFFFu;
#pragma unroll
    for (int h = 0; h < NT; ++h) {
      const int p = base | (h << (L - S)) | (st >> S);  // the predecessors of st: p << S | t = st (mod 2^L)
      const double cp = __shfl(cost, p);
      const uint32_t pp = (uint32_t)__shfl((int)pre, p);
      const double c = cp + e;
      const uint32_t code = (pp << S) | (uint32_t)(st & (NT - 1));
      if (c < best || (c == best && code < bcode)) { best = c; bcode = code; }
    }
    cost = best;
    pre = bcode;
  }
#pragma unroll
  for (int off = NS / 2; off >= 1; off >>= 1) {
    const double oc = __shfl_xor(cost, off);
    const uint32_t op = (uint32_t)__shfl_xor((int)pre, off);
    if (oc < cost || (oc == cost && op < pre)) { cost = oc; pre = op; }
  }
  return pre;
}

// All vectors of the 64-weight group held one weight per lane; lane j returns code j of the group.
template <int L, int NV, int S>
__device__ __forceinline__ uint32_t search_group(double w, double s, double zp, int lane) {
  constexpr int NS = 1 << L, VPW = 64 / NS, CPG = (kGroup + NV - 1) / NV;
  uint32_t mine = 0;
  for (int j0 = 0; j0 < CPG; j0 += VPW) {
    const int j = min(j0 + lane / NS, CPG - 1);
    double v[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int idx = NV * j + i;
      const double val = __shfl(w, min(idx, kGroup - 1));
      v[i] = idx < kGroup ? val : 0.0;  // zero-padded tail (Sec. 3.1)
    }
    const uint32_t code = nearest_code<L, NV, S>(v, s, zp, lane);
#pragma unroll
    for (int sg = 0; sg < VPW; ++sg) {
      const uint32_t c = (uint32_t)__shfl((int)code, sg * NS);
      if (lane == j0 + sg && j0 + sg < CPG) mine = c;
    }
  }
  return mine;
}

// Eq. 4: S = sum(W Wq) / sum(Wq^2), sums in index order; `fallback` when the denominator is zero.
__device__ __forceinline__ double refit_scale(double w, double wq, double fallback) {
  double num = 0.0, den = 0.0;
  for (int i = 0; i < kGroup; ++i) {
    const double wi = __shfl(w, i), qi = __shfl(wq, i);
    num += wi * qi;
    den += qi * qi;
  }
  return den > 0.0 ? num / den : fallback;
}
__device__ __forceinline__ double group_error(double w, double wq, double s) {
  double e = 0.0;
  for (int i = 0; i < kGroup; ++i) {
    const double wi = __shfl(w, i), qi = __shfl(wq, i);
    const double d = wi - qi * s;
    e += d * d;
  }
  return e;
}

__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmax(v, __shfl_xor(v, off));
  return v;
}

// First pass, one wavefront per (row, group): scale = absmax / (2^(L-1) - 1), search, Eq. 4 refit (kept
// when the error does not grow), fp16 rounding, search again with the stored scale.  An all-zero group
// gets scale 0 and codes 0.  Without Code Cluster this is the final result and is written in device
// order; with it the codes and scales go to the workspace for the next two passes.
template <int L, int NV, int S, bool CLUSTER>
__global__ void __launch_bounds__(256) ccq_encode_groups_kernel(const EncArgs a) {
  constexpr int NS = 1 << L, CPG = (kGroup + NV - 1) / NV;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t gidx = (int64_t)blockIdx.x * 4 + wave;
  GroupId id;
  if (!group_id(a, gidx, id)) return;
  const int n = id.n, gi = id.p;
  const double w = (double)a.W[(int64_t)n * a.ldw + (int64_t)id.g * kGroup + lane];
  const double amax = wave_max(fabs(w));
  uint32_t code = 0;
  double s = 0.0;
  if (amax != 0.0) {
    const double qmax = (double)((1 << (L - 1)) - 1);
    const double s0 = amax / qmax;
    code = search_group<L, NV, S>(w, s0, a.zp, lane);
    const uint32_t cj = (uint32_t)__shfl((int)code, lane / NV);
    const double wq = (double)((cj >> ((NV - 1 - lane % NV) * S)) & (NS - 1)) - a.zp;
    double s1 = refit_scale(w, wq, s0);
    if (!(s1 > 0.0) || group_error(w, wq, s1) > group_error(w, wq, s0)) s1 = s0;
    s = fp16_scale(s1);
    code = search_group<L, NV, S>(w, s, a.zp, lane);
  }
  if constexpr (CLUSTER) {
    if (lane < CPG) a.rowcodes[gidx * CPG + lane] = (uint16_t)code;
    if (lane == 0) a.rowscale[gidx] = fp16_bits(s);
  } else {
    // wide format: one byte per code; byte c of the group is segment (c % 6) / 2, quarter c / 6, byte c % 2
    // of halfword (group within the k-tile of 8)
    const int r = n % kRowsPerTile;
    if (lane < CPG) {
      const int kq = lane / 6, rem = lane % 6;
      a.codes[(int64_t)(n / kRowsPerTile) * a.row_tile_bytes + a.kind_code_off + (int64_t)(gi / kWideGroupsPerTile) * kWideTileBytes + (rem / 2) * 1024 +
              (kq * 16 + r) * 16 + (gi % kWideGroupsPerTile) * 2 + (rem % 2)] = (uint8_t)code;
    }
    if (lane == 0) {
      if (a.canon_scales) a.canon_scales[id.widx] = fp16_bits(s);
      else
        a.scales[(int64_t)(n / kRowsPerTile) * a.row_tile_scale_halfs + a.kind_scale_off + (int64_t)(gi / kWideGroupsPerTile) * kWideTileScaleHalfs +
                 r * kWideGroupsPerTile + gi % kWideGroupsPerTile] = fp16_bits(s);
    }
  }
}

// Second pass (Sec. 3.3, Eq. 1), one workgroup per output channel: beta = smallest code of the row,
// alpha = (largest - smallest) / 255 (1 when they are equal).
__global__ void __launch_bounds__(256) ccq_encode_cluster_kernel(const EncArgs a) {
  __shared__ uint32_t smin[256], smax[256];
  const int n = blockIdx.x, per_row = a.GK * 16;
  uint32_t lo = 0xFFFFFFFFu, hi = 0;
  for (int i = threadIdx.x; i < per_row; i += 256) {
    const uint32_t c = a.rowcodes[(int64_t)n * per_row + i];
    lo = min(lo, c);
    hi = max(hi, c);
  }
  smin[threadIdx.x] = lo;
  smax[threadIdx.x] = hi;
  __syncthreads();
  for (int off = 128; off >= 1; off >>= 1) {
    if ((int)threadIdx.x < off) {
      smin[threadIdx.x] = min(smin[threadIdx.x], smin[threadIdx.x + off]);
      smax[threadIdx.x] = max(smax[threadIdx.x], smax[threadIdx.x + off]);
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const uint32_t cmin = smin[0], cmax = smax[0];
    a.beta[n] = (float)cmin;
    a.alpha[n] = cmax > cmin ? (float)((double)(cmax - cmin) / 255.0) : 1.0f;
  }
}

// Third pass (narrow format), one wavefront per (row, group): every vector is searched again over the
// 256 codes round(q alpha + beta) the row's map can reach (never worse than rounding the unconstrained
// code by Eq. 1, which is one of the candidates), then one more Eq. 4 refit with the final codes, kept
// when the error does not grow.  Bytes and fp16 scales are written in device order.
__global__ void __launch_bounds__(256) ccq_encode_finish_narrow_kernel(const EncArgs a) {
  __shared__ uint32_t reach[4][256];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t gidx = (int64_t)blockIdx.x * 4 + wave;
  GroupId id;
  if (!group_id(a, gidx, id)) return;
  const int n = id.n, gi = id.p;
  const double al = (double)a.alpha[n], be = (double)a.beta[n];
  uint32_t mycodes[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int q = lane + 64 * t;
    // exact: an 8-bit integer times a 24-bit significand plus an integer below 2^15 fits a double
    mycodes[t] = (uint32_t)nearbyint((double)q * al + be);
    reach[wave][q] = mycodes[t];
  }
  __builtin_amdgcn_wave_barrier();
  const double w = (double)a.W[(int64_t)n * a.ldw + (int64_t)id.g * kGroup + lane];
  double s = fp16_value(a.rowscale[gidx]);
  uint32_t myq = 0;
  for (int j = 0; j < 16; ++j) {
    double v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = __shfl(w, 4 * j + i);
    double best = INFINITY;
    uint32_t bq = 0xFFFFFFFFu;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const uint32_t c = mycodes[t];
      double cost = sqerr(v[0], s, (double)((c >> 9) & 63u) - a.zp);
      cost = cost + sqerr(v[1], s, (double)((c >> 6) & 63u) - a.zp);
      cost = cost + sqerr(v[2], s, (double)((c >> 3) & 63u) - a.zp);
      cost = cost + sqerr(v[3], s, (double)(c & 63u) - a.zp);
      if (cost < best) { best = cost; bq = (uint32_t)(lane + 64 * t); }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const double oc = __shfl_xor(best, off);
      const uint32_t oq = (uint32_t)__shfl_xor((int)bq, off);
      if (oc < best || (oc == best && oq < bq)) { best = oc; bq = oq; }
    }
    if (lane == j) myq = bq;
  }
  const uint32_t qsel = (uint32_t)__shfl((int)myq, lane >> 2);
  const uint32_t c = reach[wave][qsel];
  const double wq = (double)((c >> (9 - 3 * (lane & 3))) & 63u) - a.zp;
  const double s2 = refit_scale(w, wq, s);
  const double s2h = s2 > 0.0 ? fp16_scale(s2) : s;
  if (group_error(w, wq, s2h) <= group_error(w, wq, s)) s = s2h;
  // narrow k-tile: byte 4 kq + b of group j of the tile sits at (kq * 16 + row) * 16 + 4 j + b
  const int r = n % kRowsPerTile;
  if (lane < 16)
    a.codes[(int64_t)(n / kRowsPerTile) * a.row_tile_bytes + a.kind_code_off + (int64_t)(gi / kNarrowGroupsPerTile) * kNarrowTileBytes + ((lane >> 2) * 16 + r) * 16 +
            (gi % kNarrowGroupsPerTile) * 4 + (lane & 3)] = (uint8_t)myq;
  if (lane == 0) {
    if (a.canon_scales) a.canon_scales[id.widx] = fp16_bits(s);
    else
      a.scales[(int64_t)(n / kRowsPerTile) * a.row_tile_scale_halfs + a.kind_scale_off + (int64_t)(gi / kNarrowGroupsPerTile) * kNarrowTileScaleHalfs +
               r * kNarrowGroupsPerTile + gi % kNarrowGroupsPerTile] = fp16_bits(s);
  }
}

// ---- Sec. 3.4 "Scale Compression", encoder side ------------------------------------------------------
// Channel-wise super scale: the largest group scale of the row / the largest field value, rounded to fp16.  (fp16 bit patterns of
// non-negative numbers order like the numbers.)
__global__ void __launch_bounds__(256) ccq_encode_super_kernel(const EncArgs a) {
  __shared__ uint32_t smax[256];
  const int n = blockIdx.x;
  uint32_t hi = 0;
  for (int i = threadIdx.x; i < a.G; i += 256) hi = max(hi, (uint32_t)a.canon_scales[(int64_t)n * a.G + i]);
  smax[threadIdx.x] = hi;
  __syncthreads();
  for (int off = 128; off >= 1; off >>= 1) {
    if ((int)threadIdx.x < off) smax[threadIdx.x] = max(smax[threadIdx.x], smax[threadIdx.x + off]);
    __syncthreads();
  }
  if (threadIdx.x == 0) a.ssup[n] = fp16_bits(fp16_round(fp16_value((uint16_t)smax[0]) / a.field_max));
}

// One wavefront per (row, group): the group scale becomes the nearest multiple field * s_super, field in 1..15 (0 only
// when the scale or the super scale is 0); because the scale that is stored has changed, the group's codes are
// searched again with it -- over all codes (wide format) or over the 256 codes the row's Code Cluster map reaches
// (narrow format).  The field goes into the spare low nibble of the wide group's last byte, or to the workspace
// for the packing pass.
template <bool NARROW>
__global__ void __launch_bounds__(256) ccq_encode_compress_kernel(const EncArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t gidx = (int64_t)blockIdx.x * 4 + wave;
  GroupId id;
  if (!group_id(a, gidx, id)) return;
  const int n = id.n, gi = id.p;
  const double s = fp16_value(a.canon_scales[id.widx]), ssup = fp16_value(a.ssup[n]);
  int k = 0;
  if (ssup > 0.0 && s > 0.0) {
    const double kr = nearbyint(s / ssup);
    k = kr < 1.0 ? 1 : (kr > 15.0 ? 15 : (int)kr);
  }
  const double se = (double)k * ssup;  // the scale the decoder will use
  const double w = (double)a.W[(int64_t)n * a.ldw + (int64_t)id.g * kGroup + lane];
  const int r = n % kRowsPerTile;
  if constexpr (NARROW) {
    if (se > 0.0) {
      const double al = (double)a.alpha[n], be = (double)a.beta[n];
      uint32_t mycodes[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) mycodes[t] = (uint32_t)nearbyint((double)(lane + 64 * t) * al + be);
      uint32_t myq = 0;
      for (int j = 0; j < 16; ++j) {
        double v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = __shfl(w, 4 * j + i);
        double best = INFINITY;
        uint32_t bq = 0xFFFFFFFFu;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const uint32_t c = mycodes[t];
          double cost = sqerr(v[0], se, (double)((c >> 9) & 63u) - a.zp);
          cost = cost + sqerr(v[1], se, (double)((c >> 6) & 63u) - a.zp);
          cost = cost + sqerr(v[2], se, (double)((c >> 3) & 63u) - a.zp);
          cost = cost + sqerr(v[3], se, (double)(c & 63u) - a.zp);
          if (cost < best) { best = cost; bq = (uint32_t)(lane + 64 * t); }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
          const double oc = __shfl_xor(best, off);
          const uint32_t oq = (uint32_t)__shfl_xor((int)bq, off);
          if (oc < best || (oc == best && oq < bq)) { best = oc; bq = oq; }
        }
        if (lane == j) myq = bq;
      }
      if (lane < 16)
        a.codes[(int64_t)(n / kRowsPerTile) * a.row_tile_bytes + a.kind_code_off + (int64_t)(gi / kNarrowGroupsPerTile) * kNarrowTileBytes + ((lane >> 2) * 16 + r) * 16 +
                (gi % kNarrowGroupsPerTile) * 4 + (lane & 3)] = (uint8_t)myq;
    }
    if (lane == 0) a.fields[gidx] = (uint8_t)k;
  } else {
    uint32_t code = 0;
    if (se > 0.0) code = search_group<4, 3, 2>(w, se, a.zp, lane);
    if (lane < 22) {
      const int kq = lane / 6, rem = lane % 6;
      uint8_t* p = a.codes + (int64_t)(n / kRowsPerTile) * a.row_tile_bytes + a.kind_code_off + (int64_t)(gi / kWideGroupsPerTile) * kWideTileBytes + (rem / 2) * 1024 +
                   (kq * 16 + r) * 16 + (gi % kWideGroupsPerTile) * 2 + (rem % 2);
      uint32_t byte = se > 0.0 ? code : (uint32_t)*p;  // an all-zero group keeps its codes
      if (lane == 21) byte = (byte & 0xF0u) | (uint32_t)k;
      if (se > 0.0 || lane == 21) *p = (uint8_t)byte;
    }
  }
}

// ---- the hybrid 16-bit word (Sec. 3.2): a (3,3,2) code on weights 7j..7j+2 and a (3,4,2) code on weights 7j+3..7j+6
// of word j, searched independently (their bits do not overlap); ten words per group, the last one zero-padded ----

// Lane j (j < 10) returns word j of the group held one weight per lane.
__device__ __forceinline__ uint32_t search_h16(double w, double s, double zp, int lane) {
  uint32_t mine = 0;
  for (int j0 = 0; j0 < 10; j0 += 8) {
    const int j = min(j0 + (lane >> 3), 9);
    double va[3], vb[4];
#pragma unroll
    for (int i = 0; i < 7; ++i) {
      const int idx = 7 * j + i;
      const double val = __shfl(w, min(idx, kGroup - 1));
      const double v = idx < kGroup ? val : 0.0;
      if (i < 3) va[i] = v;
      else vb[i - 3] = v;
    }
    const uint32_t ca = nearest_code<3, 3, 2>(va, s, zp, lane);
    const uint32_t cb = nearest_code<3, 4, 2>(vb, s, zp, lane);
    const uint32_t word = (ca << 9) | cb;
#pragma unroll
    for (int sg = 0; sg < 8; ++sg) {
      const uint32_t c = (uint32_t)__shfl((int)word, sg * 8);
      if (lane == j0 + sg && j0 + sg < 10) mine = c;
    }
  }
  return mine;
}

// word j of group gi, row n, in the hybrid-word k-tile: segment j / 4, lane (j % 4) * 16 + row, halfword gi % 8
__device__ __forceinline__ uint16_t* h16_word_ptr(const EncArgs& a, int n, int gi, int j) {
  return reinterpret_cast<uint16_t*>(a.codes + (int64_t)(n / kRowsPerTile) * a.row_tile_bytes + a.kind_code_off + (int64_t)(gi / kWideGroupsPerTile) * kH16TileBytes +
                                     (j >> 2) * 1024 + ((j & 3) * 16 + n % kRowsPerTile) * 16 + (gi % kWideGroupsPerTile) * 2);
}

// One wavefront per (row, group): Alg. 1 with the Eq. 4 refit as for the other formats; 2^(L-1) - 1 = 3.
__global__ void __launch_bounds__(256) ccq_encode_h16_kernel(const EncArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t gidx = (int64_t)blockIdx.x * 4 + wave;
  GroupId id;
  if (!group_id(a, gidx, id)) return;
  const int n = id.n, gi = id.p;
  const double w = (double)a.W[(int64_t)n * a.ldw + (int64_t)id.g * kGroup + lane];
  const double amax = wave_max(fabs(w));
  uint32_t word = 0;
  double s = 0.0;
  if (amax != 0.0) {
    const double s0 = amax / 3.0;
    word = search_h16(w, s0, a.zp, lane);
    const uint32_t wj = (uint32_t)__shfl((int)word, lane / 7);
    const int i = lane % 7;
    const int shift = i < 3 ? 13 - 2 * i : 12 - 2 * i;  // Table 1: [13,11,9,6,4,2,0]
    const double wq = (double)((wj >> shift) & 7u) - a.zp;
    double s1 = refit_scale(w, wq, s0);
    if (!(s1 > 0.0) || group_error(w, wq, s1) > group_error(w, wq, s0)) s1 = s0;
    s = fp16_scale(s1);
    word = search_h16(w, s, a.zp, lane);
  }
  if (lane < 10) *h16_word_ptr(a, n, gi, lane) = (uint16_t)word;
  if (lane == 0) {
    if (a.canon_scales) a.canon_scales[id.widx] = fp16_bits(s);
    else
      a.scales[(int64_t)(n / kRowsPerTile) * a.row_tile_scale_halfs + a.kind_scale_off + (int64_t)(gi / kWideGroupsPerTile) * kWideTileScaleHalfs +
               (n % kRowsPerTile) * kWideGroupsPerTile + gi % kWideGroupsPerTile] = fp16_bits(s);
  }
}

// Compressed scales of the hybrid word: 13-bit field in the low bits of the group's last word (scale mask 0x1FFF of
// Table 1), words searched again with the scale that is stored.
__global__ void __launch_bounds__(256) ccq_encode_h16_compress_kernel(const EncArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t gidx = (int64_t)blockIdx.x * 4 + wave;
  GroupId id;
  if (!group_id(a, gidx, id)) return;
  const int n = id.n, gi = id.p;
  const double s = fp16_value(a.canon_scales[id.widx]), ssup = fp16_value(a.ssup[n]);
  int k = 0;
  if (ssup > 0.0 && s > 0.0) {
    const double kr = nearbyint(s / ssup);
    k = kr < 1.0 ? 1 : (kr > 8191.0 ? 8191 : (int)kr);
  }
  const double se = (double)k * ssup;
  const double w = (double)a.W[(int64_t)n * a.ldw + (int64_t)id.g * kGroup + lane];
  uint32_t word = 0;
  if (se > 0.0) word = search_h16(w, se, a.zp, lane);
  if (lane < 10) {
    uint16_t* p = h16_word_ptr(a, n, gi, lane);
    uint32_t v = se > 0.0 ? word : (uint32_t)*p;  // an all-zero group keeps its words
    if (lane == 9) v = (v & 0xE000u) | (uint32_t)k;
    if (se > 0.0 || lane == 9) *p = (uint16_t)v;
  }
}

// Narrow format: the four 4-bit fields of a k-tile's groups into one 16-bit word per row (group j in bits 4j..4j+3).
__global__ void __launch_bounds__(256) ccq_encode_pack_fields_kernel(const EncArgs a) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int tiles = (a.GK + kNarrowGroupsPerTile - 1) / kNarrowGroupsPerTile;
  if (i >= (int64_t)a.N * tiles) return;
  const int n = (int)(i / tiles), t = (int)(i % tiles);
  const uint8_t* f = a.fields + (int64_t)n * a.GK;
  uint32_t word = 0;  // groups that pad the last k-tile keep field 0: scale 0
#pragma unroll
  for (int j = 0; j < kNarrowGroupsPerTile; ++j) {
    const int p = t * kNarrowGroupsPerTile + j;
    if (p < a.GK) word |= (uint32_t)f[p] << (4 * j);
  }
  a.scales[(int64_t)(n / kRowsPerTile) * a.row_tile_scale_halfs + a.kind_scale_off + (int64_t)t * kNarrowTileScaleHalfs4 + n % kRowsPerTile] = (uint16_t)word;
}

// Clears `n16` 16-byte units (a kernel, not a memset node: the call may be recorded into a graph).
__global__ void __launch_bounds__(256) ccq_encode_clear_kernel(uint4* p, int64_t n16) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) p[i] = uint4{0u, 0u, 0u, 0u};
}

static int64_t round16(int64_t v) { return (v + 15) / 16 * 16; }

// workspace: [unclustered codes and first-pass scales (narrow)] [final fp16 scales, fields (compressed scales)]
int64_t encode_workspace_bytes(const Layout& L) {
  const int64_t groups = (int64_t)L.N * L.G, narrow = (int64_t)L.N * L.groups[kNarrow];
  int64_t need = 0;
  if (narrow > 0) need += round16(narrow * 16 * 2) + round16(narrow * 2);
  if (L.scale_mode == 1) need += round16(groups * 2) + round16(narrow);
  return need;
}

int launch_encode(const Layout& L, const float* W, int64_t ldw, void* codes, void* scales, float* alpha, float* beta, void* scale_super,
                  const int32_t* meta, void* workspace, void* stream) {
  const int64_t groups = (int64_t)L.N * L.G, narrow = (int64_t)L.N * L.groups[kNarrow];
  EncArgs a;
  a.field_max = L.h16 ? 8191.0 : 15.0;
  a.W = W;
  a.ldw = ldw;
  a.N = L.N;
  a.G = L.G;
  a.meta = L.has_map ? meta : nullptr;
  a.codes = static_cast<uint8_t*>(codes);
  a.scales = static_cast<uint16_t*>(scales);
  a.alpha = alpha;
  a.beta = beta;
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  a.rowcodes = nullptr;
  a.rowscale = nullptr;
  if (narrow > 0) {
    a.rowcodes = reinterpret_cast<uint16_t*>(ws);
    ws += round16(narrow * 16 * 2);
    a.rowscale = reinterpret_cast<uint16_t*>(ws);
    ws += round16(narrow * 2);
  }
  a.canon_scales = nullptr;
  a.fields = nullptr;
  a.ssup = static_cast<uint16_t*>(scale_super);
  if (L.scale_mode == 1) {
    a.canon_scales = reinterpret_cast<uint16_t*>(ws);
    ws += round16(groups * 2);
    a.fields = ws;
  }
  a.row_tile_bytes = L.row_tile_bytes;
  a.row_tile_scale_halfs = L.row_tile_scale_halfs;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const dim3 block(256);
  if (L.padded()) {
    // rows that pad the last row tile and groups that pad the last k-tile of a kind are written by no kernel below:
    // zero codes and zero scales (both arrays are whole 16-byte units: a row tile's share of either is)
    const int64_t code16 = L.row_tile_bytes * L.row_tiles / 16, scale16 = L.row_tile_scale_halfs * L.row_tiles / 8;
    if (code16 > 0) hipLaunchKernelGGL(ccq_encode_clear_kernel, dim3((unsigned)((code16 + 255) / 256)), block, 0, st, reinterpret_cast<uint4*>(codes), code16);
    if (scale16 > 0 && scales)
      hipLaunchKernelGGL(ccq_encode_clear_kernel, dim3((unsigned)((scale16 + 255) / 256)), block, 0, st, reinterpret_cast<uint4*>(scales), scale16);
  }
  // the narrow groups of every row, then the wide ones (or the hybrid words, which never mix)
  EncArgs an = a, aw = a;
  an.GK = L.groups[kNarrow];
  an.pbase = 0;
  an.mbase = 0;
  an.kind_code_off = 0;
  an.kind_scale_off = 0;
  an.zp = (double)L.zp[kNarrow];
  aw.GK = L.groups[kWide];
  aw.pbase = L.groups[kNarrow];
  aw.mbase = L.pgroups[kNarrow];
  aw.kind_code_off = (int64_t)L.tiles[kNarrow] * kNarrowTileBytes;
  aw.kind_scale_off = L.scale_mode == 1 ? 0 : (int64_t)L.tiles[kNarrow] * kNarrowTileScaleHalfs;
  aw.zp = (double)L.zp[kWide];
  const dim3 grid_n((unsigned)((narrow + 3) / 4)), grid_w((unsigned)(((int64_t)L.N * L.groups[kWide] + 3) / 4));
  if (an.GK > 0) {
    hipLaunchKernelGGL((ccq_encode_groups_kernel<6, 4, 3, true>), grid_n, block, 0, st, an);
    hipLaunchKernelGGL(ccq_encode_cluster_kernel, dim3((unsigned)L.N), block, 0, st, an);
    hipLaunchKernelGGL(ccq_encode_finish_narrow_kernel, grid_n, block, 0, st, an);
  }
  if (aw.GK > 0) {
    if (L.h16) hipLaunchKernelGGL(ccq_encode_h16_kernel, grid_w, block, 0, st, aw);
    else hipLaunchKernelGGL((ccq_encode_groups_kernel<4, 3, 2, false>), grid_w, block, 0, st, aw);
  }
  if (L.scale_mode == 1) {
    hipLaunchKernelGGL(ccq_encode_super_kernel, dim3((unsigned)L.N), block, 0, st, a);
    if (an.GK > 0) {
      hipLaunchKernelGGL(ccq_encode_compress_kernel<true>, grid_n, block, 0, st, an);
      const int64_t words = (int64_t)L.N * L.tiles[kNarrow];
      hipLaunchKernelGGL(ccq_encode_pack_fields_kernel, dim3((unsigned)((words + 255) / 256)), block, 0, st, an);
    }
    if (aw.GK > 0) {
      if (L.h16) hipLaunchKernelGGL(ccq_encode_h16_compress_kernel, grid_w, block, 0, st, aw);
      else hipLaunchKernelGGL(ccq_encode_compress_kernel<false>, grid_w, block, 0, st, aw);
    }
  }
  if (hipGetLastError() != hipSuccess) return CCQ_ERR_HIP;
  return CCQ_OK;
}

}  // namespace ccq
