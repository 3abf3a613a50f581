// Host layer of libccq: descriptor validation, layout accounting (Eq. 5 of the
// CCQ paper), canonical -> device order permutations, argument checks and
// dispatch to the kernel launchers.  No device code in this file.
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

#include "ccq_internal.h"

namespace ccq {

static bool is_narrow(const ccq_code& c) { return c.L == 6 && c.N == 4 && c.S == 3 && c.code_cluster == 1; }
static bool is_wide(const ccq_code& c) { return c.L == 4 && c.N == 3 && c.S == 2 && c.code_cluster == 0; }
// the two halves of the hybrid word of Sec. 3.2: (3,3,2) in the top 7 bits, (3,4,2) in the low 9 bits
static bool is_h16(const ccq_weight* w) {
  return w->n_formats == 2 && !w->group_fmt && w->fmt[0].L == 3 && w->fmt[0].N == 3 && w->fmt[0].S == 2 && w->fmt[0].code_cluster == 0 &&
         w->fmt[1].L == 3 && w->fmt[1].N == 4 && w->fmt[1].S == 2 && w->fmt[1].code_cluster == 0;
}

static int ceil_div_i(int a, int b) { return (a + b - 1) / b; }

int make_layout(const ccq_weight* w, Layout* out) {
  if (!w || !out) return CCQ_ERR_NULL;
  if (w->K <= 0 || w->N <= 0 || w->n_formats < 1 || w->n_formats > 2) return CCQ_ERR_BAD_PARAM;
  if (w->group != kGroup) return w->group > 0 ? CCQ_ERR_UNSUPPORTED : CCQ_ERR_BAD_PARAM;
  if (w->K % kGroup != 0) return CCQ_ERR_BAD_PARAM;
  if (w->scale_mode != 0 && w->scale_mode != 1) return CCQ_ERR_UNSUPPORTED;
  if (w->n_formats == 1 && w->group_fmt) return CCQ_ERR_BAD_PARAM;
  Layout L;
  L.scale_mode = w->scale_mode;
  L.K = w->K;
  L.N = w->N;
  L.G = w->K / kGroup;
  if (is_h16(w)) {
    // one zero-point for the seven states of a word
    const float zp = w->fmt[0].zp;
    if (w->fmt[1].zp != zp) return CCQ_ERR_UNSUPPORTED;
    if (!(zp * 2.0f == std::floor(zp * 2.0f)) || zp < 0.f || zp > 64.f) return CCQ_ERR_BAD_PARAM;
    L.h16 = true;
    L.kind_of_fmt[0] = L.kind_of_fmt[1] = kWide;
    L.zp[kWide] = zp;
    L.groups[kWide] = L.G;
    L.tiles[kWide] = ceil_div_i(L.G, kWideGroupsPerTile);
    L.pgroups[kWide] = L.tiles[kWide] * kWideGroupsPerTile;
    L.row_tile_bytes = (int64_t)L.tiles[kWide] * kH16TileBytes;
    L.row_tile_scale_halfs = L.scale_mode == 1 ? 0 : (int64_t)L.tiles[kWide] * kWideTileScaleHalfs;  // mode 1: the fields sit in the words
    L.row_tiles = ceil_div_i(w->N, kRowsPerTile);
    L.Npad = L.row_tiles * kRowsPerTile;
    if (L.row_tile_bytes * (int64_t)L.row_tiles >= (int64_t)1 << 40) return CCQ_ERR_BAD_PARAM;
    *out = L;
    return CCQ_OK;
  }
  for (int f = 0; f < w->n_formats; ++f) {
    const ccq_code& c = w->fmt[f];
    if (c.L < 1 || c.N < 1 || c.S < 1 || c.S > c.L || c.L > 16) return CCQ_ERR_BAD_PARAM;
    float twice = c.zp * 2.0f;
    if (!(twice == std::floor(twice)) || c.zp < 0.f || c.zp > 64.f) return CCQ_ERR_BAD_PARAM;
    if (is_narrow(c)) L.kind_of_fmt[f] = kNarrow;
    else if (is_wide(c)) L.kind_of_fmt[f] = kWide;
    else return CCQ_ERR_UNSUPPORTED;
    L.zp[L.kind_of_fmt[f]] = c.zp;
  }
  if (w->n_formats == 2 && L.kind_of_fmt[0] == L.kind_of_fmt[1]) return CCQ_ERR_BAD_PARAM;
  L.has_map = w->group_fmt != nullptr;
  if (w->n_formats == 2 && !w->group_fmt) return CCQ_ERR_NULL;
  for (int g = 0; g < L.G; ++g) {
    int f = w->group_fmt ? w->group_fmt[g] : 0;
    if (f < 0 || f >= w->n_formats) return CCQ_ERR_BAD_PARAM;
    L.groups[L.kind_of_fmt[f]]++;
  }
  // whole k-tiles and whole row tiles in the device layout: what is missing is padding (zero codes, zero scales)
  L.tiles[kNarrow] = ceil_div_i(L.groups[kNarrow], kNarrowGroupsPerTile);
  L.tiles[kWide] = ceil_div_i(L.groups[kWide], kWideGroupsPerTile);
  L.pgroups[kNarrow] = L.tiles[kNarrow] * kNarrowGroupsPerTile;
  L.pgroups[kWide] = L.tiles[kWide] * kWideGroupsPerTile;
  L.row_tile_bytes = (int64_t)L.tiles[kNarrow] * kNarrowTileBytes + (int64_t)L.tiles[kWide] * kWideTileBytes;
  L.row_tile_scale_halfs = L.scale_mode == 1
                               ? (int64_t)L.tiles[kNarrow] * kNarrowTileScaleHalfs4
                               : (int64_t)L.tiles[kNarrow] * kNarrowTileScaleHalfs + (int64_t)L.tiles[kWide] * kWideTileScaleHalfs;
  L.row_tiles = ceil_div_i(w->N, kRowsPerTile);
  L.Npad = L.row_tiles * kRowsPerTile;
  if (L.row_tile_bytes * (int64_t)L.row_tiles >= (int64_t)1 << 40) return CCQ_ERR_BAD_PARAM;
  *out = L;
  return CCQ_OK;
}

// ---- launch decomposition ---------------------------------------------------

bool decomp_ok(const Layout& L, const Decomp& d) {
  (void)L;
  if (d.RT < 1 || d.RT > 2) return false;
  if (d.WR < 1 || d.WK < 1 || d.WR * d.WK > 16) return false;
  if (d.S < 1 || d.S > kMaxSplitsK) return false;
  return true;
}

static int ceil_div(int a, int b) { return (a + b - 1) / b; }

Decomp choose_decomp(const Layout& L, int M, int experts, int rows_total) {
  (void)rows_total;
  Decomp d;
  const int64_t cus = device_cus();
  const int nt = L.tiles[kNarrow] + L.tiles[kWide];  // k-tiles per row tile
  const int64_t units = (int64_t)L.row_tiles * experts;  // row tiles over all experts
  if (M == 1) {
    // GEMV, bound by the vector ALU: a workgroup is one group of wavefronts that split K among
    // themselves (reduced in LDS, no workspace pass); every wavefront gets about 8 k-tiles so that its
    // set-up cost is amortised, and two row tiles when there are plenty of rows (narrow format only).
    d.RT = (units >= 4 * cus && L.tiles[kWide] == 0) ? 2 : 1;
    d.WR = 1;
    d.WK = std::max(1, std::min(8, nt / (L.tiles[kNarrow] > 0 ? 8 : 4)));  // wide k-tiles are 2.75 times the bytes of narrow ones
    d.S = 1;
  } else {
    // two row tiles per wavefront only for the narrow format with at most 32 held rows (register budget)
    d.RT = (L.row_tiles >= 2 && M <= 32 && L.tiles[kWide] == 0) ? 2 : 1;
    // wavefronts side by side that share one staged activation chunk: four, or eight for mixed formats with many
    // rows, whose staging (a gather through the group map, one row tile per wavefront) is the larger part of the
    // work (config 3, M = 16: 61 -> 42 us; 8192 x 8192 mixed: 21.8 -> 18.8 us; 4096 x 4096 is better off with four)
    // -- and for grouped calls on long rows of narrow-format weights (config 4, K = 7168: 108 -> 96 us; with K = 2048
    // four are better)
    const bool mixed_many_rows = L.tiles[kNarrow] > 0 && L.tiles[kWide] > 0 && L.row_tiles >= 2 * cus && M <= 16;
    const bool grouped_long_k = experts > 1 && L.tiles[kWide] == 0 && L.tiles[kNarrow] >= 24 && M <= 32;
    const int wr_max = (mixed_many_rows || grouped_long_k) ? 8 : 4;
    d.WR = (int)std::min<int64_t>(wr_max, std::max(1, L.row_tiles / d.RT));
    d.WK = 1;
    int64_t row_blocks = (int64_t)ceil_div(L.row_tiles, d.RT * d.WR) * experts;
    // workgroups wanted: two per CU for the narrow format, four for the wide kinds, whose per-chunk staging is longer
    // than the contraction it feeds and is best hidden by other workgroups of the same CU
    const int64_t want_blocks = (L.tiles[kNarrow] > 0 ? 2 : 4) * cus;
    int s = (int)std::max<int64_t>(1, want_blocks / std::max<int64_t>(1, row_blocks));
    s = std::min(s, std::max(1, nt / 2));
    if (M > 16) s = std::min(s, 2);
    d.S = std::min(s, kMaxSplitsK);
  }
  return d;
}

}  // namespace ccq

using namespace ccq;

// Which kernel a dense call of M rows uses when no launch shape is given.
enum DensePath { kPathGemv, kPathGemv16, kPathGemv16NW, kPathSkinny, kPathRows, kPathMid, kPathPrefill };
static DensePath dense_path(const Layout& L, int M) {
  const bool narrow_only = L.tiles[kWide] == 0, wide_only = L.tiles[kNarrow] == 0;
  if (narrow_only && !L.has_map && M < kMidMinM) {
    // one row: the GEMV kernel; two to four: its four-row variant where K splits into its shares and fits its LDS; up to sixteen: the
    // 16-row kernel (each falls back to the per-row-tile kernel if K does not split its way)
    int tpw = 0, nw = 0;
    if (M == 1 || (M <= kGemvMaxM && gemv4_shape(L, 256, &tpw, &nw))) return kPathGemv;
    if (gemv16_shape(L, 256, kMaxSplitsK, &tpw, &nw)) return kPathGemv16;
  }
  // two to sixteen rows on wide-format and mixed weights: the 16-row kernel for those formats, where K splits its way
  if (!narrow_only && M >= 2 && M < kMidMinM) {
    int tpwn = 0, tpww = 0, sn = 0, sw = 0;
    if (gemv16_nw_shape(L, 256, kMaxSplitsK, &tpwn, &tpww, &sn, &sw)) return kPathGemv16NW;
  }
  // per-group activation tiles with the weights in registers: measured faster than its neighbours for 2-16 rows on the
  // wide and hybrid-word formats (whose whole-k-tile staging is the costliest) and for 17-32 rows on the narrow one
  if (wide_only && M >= 2 && M < kMidMinM) return kPathRows;
  if (M < kMidMinM) return kPathSkinny;
  if (narrow_only && M <= 32) {
    // 17..32 rows: the 16-row kernel holding two 16-row tiles of activations, where K splits its way
    int tpw = 0, nw = 0;
    if (!L.has_map && gemv16_shape(L, 256, kMaxSplitsK, &tpw, &nw)) return kPathGemv16;
    return kPathRows;
  }
  if (narrow_only && M > 128) {
    // 256-row tiles pay off once they fill enough of the chip.  Both kernels are bound by the same two things (matrix
    // core time, and the vector work of decoding a weight tile once per row block of the output), so their times
    // are compared in units of one output element per round of workgroups over the chip's CUs; the relative costs
    // per element are ratios measured between the kernels, not times: the 256-row kernel costs 1.0 with 192-column
    // blocks and 1.22 with 128 or 256 columns, up to 40 % more when more than half of the CUs are busy (the clock
    // sinks under a full matrix load); the 64-row kernel, which decodes every weight tile four times as often,
    // costs 2.4 and about 0.4 of a round in fixed set-up.
    const int64_t cus = device_cus();
    const int bn = prefill_block_cols(L, M);
    const int64_t wg_p = (int64_t)ceil_div(M, 256) * ceil_div(L.N, bn);
    const int64_t rounds_p = (wg_p + cus - 1) / cus;
    const double fill = (double)wg_p / (double)(rounds_p * cus);
    const double t_p = (double)rounds_p * 256.0 * bn * (bn == 192 ? 1.0 : 1.22) * (1.0 + 0.8 * std::max(0.0, fill - 0.5));
    const int64_t wg_m = (int64_t)ceil_div(M, 64) * ceil_div(L.N, 128);
    const double rounds_m = std::max(1.0, (double)wg_m / (double)cus);   // its workgroups are short: partial rounds overlap
    const double t_m = (rounds_m + 0.42) * 64.0 * 128.0 * 2.4;
    return t_p <= t_m ? kPathPrefill : kPathMid;
  }
  return kPathMid;
}

// Workspace the per-row-tile kernel needs for M rows in the library's own decomposition: it walks the rows in
// passes of kMaxSkinnyM and a last, shorter one.
static int64_t skinny_need(const Layout& L, int M) {
  int64_t need = 0;
  for (int mc : {M >= kMaxSkinnyM ? kMaxSkinnyM : 0, M % kMaxSkinnyM}) {
    if (mc == 0) continue;
    const Decomp d = choose_decomp(L, mc, 1, mc);
    if (d.S > 1) need = std::max(need, (int64_t)d.S * mc * L.Npad * 4);
  }
  return need;
}

// Workspace one dense call of exactly M rows needs (fp32 partial tiles of the K shares) on the kernel the library
// picks for it.
static int64_t dense_need(const Layout& L, int M) {
  if (M <= 0) return 0;
  switch (dense_path(L, M)) {
    case kPathGemv: {
      int tpw = 0, waves = 0;
      // whether K splits does not depend on the chip
      if (M == 1 ? gemv1_shape(L, 256, &tpw, &waves) : gemv4_shape(L, 256, &tpw, &waves)) return 0;
      return skinny_need(L, M);
    }
    case kPathGemv16: {
      int tpw = 0, nw = 0;
      if (!gemv16_shape(L, device_cus(), kMaxSplitsK, &tpw, &nw)) return skinny_need(L, M);
      const int S = (L.tiles[kNarrow] + tpw - 1) / tpw;
      return S > 1 ? (int64_t)S * M * L.Npad * 4 : 0;
    }
    case kPathGemv16NW: {
      int tpwn = 0, tpww = 0, sn = 0, sw = 0;
      if (!gemv16_nw_shape(L, device_cus(), kMaxSplitsK, &tpwn, &tpww, &sn, &sw)) return skinny_need(L, M);
      return sn + sw > 1 ? (int64_t)(sn + sw) * M * L.Npad * 4 : 0;
    }
    case kPathRows: {
      const int S = rows_splits(L, M);
      return S > 1 ? (int64_t)S * M * L.Npad * 4 : 0;
    }
    case kPathMid:
    case kPathPrefill: {  // the 256-row kernel needs none; where it does not apply the 64-row kernel runs
      const int S = mid_splits(L, M);
      return S > 1 ? (int64_t)S * M * L.Npad * 4 : 0;
    }
    default:
      return skinny_need(L, M);
  }
}

// The largest need over 1..M_max rows.  Between two multiples of 16 the kernel choice and the number of K shares
// do not change (they depend on the row count through its 16-, 32-, 64- and 256-row blocks and the thresholds 1,
// 4, 16, 32, 128), and with both fixed the need grows with the row count: only those row counts are looked at.
// K is cut only while the row and column blocks do not fill the chip, which bounds the row counts that matter.
static int64_t dense_workspace_bytes(const Layout& L, int M_max) {
  int64_t need = 0;
  const int cap = std::min(M_max, 4096);
  for (int m : {1, 2, 4}) if (m <= M_max) need = std::max(need, dense_need(L, m));
  for (int m = 16; m <= cap; m += 16) need = std::max(need, dense_need(L, m));
  need = std::max(need, dense_need(L, std::min(M_max, cap)));
  if (M_max > cap) need = std::max(need, dense_need(L, M_max));
  return need;
}

extern "C" int ccq_pack_info(const ccq_weight* w, int32_t M_max, ccq_info* out) {
  if (!w || !out) return CCQ_ERR_NULL;
  if (M_max < 0) return CCQ_ERR_BAD_PARAM;
  Layout L;
  int rc = make_layout(w, &L);
  if (rc != CCQ_OK) return rc;
  ccq_info info;
  std::memset(&info, 0, sizeof(info));
  info.bytes_per_group[0] = info.bytes_per_group[1] = 0;
  for (int f = 0; f < w->n_formats; ++f)
    info.bytes_per_group[f] = L.h16 ? kH16GroupBytes : (L.kind_of_fmt[f] == kNarrow ? kNarrowGroupBytes : kWideGroupBytes);
  for (int f = 0; f < w->n_formats; ++f) info.groups[f] = L.groups[L.kind_of_fmt[f]];
  info.row_tile_bytes = L.row_tile_bytes;
  info.code_bytes = L.row_tile_bytes * L.row_tiles;
  info.scale_bytes = L.row_tile_scale_halfs * L.row_tiles * 2;
  info.meta_bytes = (int64_t)(L.pgroups[kNarrow] + L.pgroups[kWide]) * 4;
  info.align = 16;
  info.workspace_bytes = dense_workspace_bytes(L, M_max);
  info.padded_N = L.Npad;
  for (int f = 0; f < w->n_formats; ++f) info.padded_groups[f] = L.pgroups[L.kind_of_fmt[f]];
  // Eq. 5: stored code bits per weight; a narrow group holds 64/4 one-byte codes
  // (g = 0 mod N: scale bits come on top), a wide group ceil(64/3) = 22 one-byte
  // codes (g = 1 mod N: the spare bits of the last code are part of the count).
  // The accounting is that of the canonical arrays (what the method stores); the padding of the device layout
  // (whole row tiles and k-tiles) is reported separately.
  const double weights = (double)L.N * (double)L.K;
  const int64_t canon_row = L.h16 ? (int64_t)L.G * kH16GroupBytes : (int64_t)L.groups[kNarrow] * kNarrowGroupBytes + (int64_t)L.groups[kWide] * kWideGroupBytes;
  info.canonical_code_bytes = canon_row * L.N;
  const double canon_scale_bytes =
      L.scale_mode == 0 ? 2.0 * (double)L.G * (double)L.N : (double)((L.groups[kNarrow] + 1) / 2) * (double)L.N;
  info.code_bpw = 8.0 * (double)info.canonical_code_bytes / weights;
  const double ab_bytes = (L.groups[kNarrow] > 0 ? 8.0 * (double)L.N : 0.0) + (L.scale_mode == 1 ? 2.0 * (double)L.N : 0.0);
  info.total_bpw = 8.0 * ((double)info.canonical_code_bytes + canon_scale_bytes + ab_bytes) / weights;
  *out = info;
  return CCQ_OK;
}

// packed index of every group: narrow groups first (k order), then wide
static void packed_order(const ccq_weight* w, const Layout& L, std::vector<int>& pos_in_kind, std::vector<int>& kind) {
  pos_in_kind.resize(L.G);
  kind.resize(L.G);
  int cnt[2] = {0, 0};
  for (int g = 0; g < L.G; ++g) {
    int k = group_kind(w, L, g);
    kind[g] = k;
    pos_in_kind[g] = cnt[k]++;
  }
}

extern "C" int ccq_pack_codes(const ccq_weight* w, const uint8_t* src, void* out_v) {
  if (!w || !src || !out_v) return CCQ_ERR_NULL;
  Layout L;
  int rc = make_layout(w, &L);
  if (rc != CCQ_OK) return rc;
  uint8_t* out = static_cast<uint8_t*>(out_v);
  std::memset(out, 0, (size_t)(L.row_tile_bytes * L.row_tiles));   // padded rows and groups: zero codes
  if (L.h16) {
    for (int n = 0; n < L.N; ++n) {
      const uint8_t* row = src + (int64_t)n * L.G * kH16GroupBytes;
      uint8_t* tile_row = out + (int64_t)(n / kRowsPerTile) * L.row_tile_bytes;
      const int r = n % kRowsPerTile;
      for (int g = 0; g < L.G; ++g) {
        uint8_t* tile = tile_row + (int64_t)(g / kWideGroupsPerTile) * kH16TileBytes;
        const int j = g % kWideGroupsPerTile;
        for (int word = 0; word < 10; ++word) {
          const int t = word / 4, kq = word % 4;
          for (int b = 0; b < 2; ++b) tile[t * 1024 + (kq * 16 + r) * 16 + j * 2 + b] = row[(int64_t)g * kH16GroupBytes + 2 * word + b];
        }
      }
    }
    return CCQ_OK;
  }
  std::vector<int> pos, kind;
  packed_order(w, L, pos, kind);
  std::vector<int64_t> goff(L.G);  // canonical byte offset of each group inside a row
  int64_t row_bytes = 0;
  for (int g = 0; g < L.G; ++g) {
    goff[g] = row_bytes;
    row_bytes += kind[g] == kNarrow ? kNarrowGroupBytes : kWideGroupBytes;
  }
  const int64_t wide_base = (int64_t)L.tiles[kNarrow] * kNarrowTileBytes;
  for (int n = 0; n < L.N; ++n) {
    const uint8_t* row = src + (int64_t)n * row_bytes;
    uint8_t* tile_row = out + (int64_t)(n / kRowsPerTile) * L.row_tile_bytes;
    const int r = n % kRowsPerTile;
    for (int g = 0; g < L.G; ++g) {
      const uint8_t* gb = row + goff[g];
      if (kind[g] == kNarrow) {
        uint8_t* tile = tile_row + (int64_t)(pos[g] / kNarrowGroupsPerTile) * kNarrowTileBytes;
        const int j = pos[g] % kNarrowGroupsPerTile;
        for (int kq = 0; kq < 4; ++kq)
          for (int b = 0; b < 4; ++b) tile[(kq * 16 + r) * 16 + j * 4 + b] = gb[4 * kq + b];
      } else {
        uint8_t* tile = tile_row + wide_base + (int64_t)(pos[g] / kWideGroupsPerTile) * kWideTileBytes;
        const int j = pos[g] % kWideGroupsPerTile;
        for (int kq = 0; kq < 4; ++kq)
          for (int t = 0; t < 3; ++t) {
            if (kq == 3 && t == 2) continue;  // quarter 3 owns bytes 18..21 only
            for (int b = 0; b < 2; ++b) tile[t * 1024 + (kq * 16 + r) * 16 + j * 2 + b] = gb[6 * kq + 2 * t + b];
          }
      }
    }
  }
  return CCQ_OK;
}

extern "C" int ccq_pack_scales4(const ccq_weight* w, const uint8_t* src, void* out_v) {
  if (!w || !src || !out_v) return CCQ_ERR_NULL;
  Layout L;
  int rc = make_layout(w, &L);
  if (rc != CCQ_OK) return rc;
  if (L.scale_mode != 1) return CCQ_ERR_BAD_PARAM;
  uint16_t* out = static_cast<uint16_t*>(out_v);
  const int64_t src_row_bytes = (L.groups[kNarrow] + 1) / 2;
  std::memset(out, 0, (size_t)(L.row_tile_scale_halfs * L.row_tiles * 2));
  for (int n = 0; n < L.N; ++n) {
    uint16_t* tile_row = out + (int64_t)(n / kRowsPerTile) * L.row_tile_scale_halfs;
    const int r = n % kRowsPerTile;
    for (int p = 0; p < L.groups[kNarrow]; ++p) {  // p-th narrow-format group of the row, k order
      const uint32_t field = (src[(int64_t)n * src_row_bytes + p / 2] >> (4 * (p % 2))) & 0xFu;  // (s_q >> s_shift) & s_mask, Alg. 3
      tile_row[(int64_t)(p / 4) * kNarrowTileScaleHalfs4 + r] |= (uint16_t)(field << (4 * (p % 4)));
    }
  }
  return CCQ_OK;
}

extern "C" int ccq_pack_scales(const ccq_weight* w, const uint16_t* src, void* out_v) {
  if (!w || !src || !out_v) return CCQ_ERR_NULL;
  Layout L;
  int rc = make_layout(w, &L);
  if (rc != CCQ_OK) return rc;
  if (L.scale_mode != 0) return CCQ_ERR_BAD_PARAM;
  uint16_t* out = static_cast<uint16_t*>(out_v);
  std::memset(out, 0, (size_t)(L.row_tile_scale_halfs * L.row_tiles * 2));   // padded rows and groups: scale 0
  std::vector<int> pos, kind;
  packed_order(w, L, pos, kind);
  const int64_t wide_base = (int64_t)L.tiles[kNarrow] * kNarrowTileScaleHalfs;
  for (int n = 0; n < L.N; ++n) {
    uint16_t* tile_row = out + (int64_t)(n / kRowsPerTile) * L.row_tile_scale_halfs;
    const int r = n % kRowsPerTile;
    for (int g = 0; g < L.G; ++g) {
      uint16_t v = src[(int64_t)n * L.G + g];
      if (kind[g] == kNarrow)
        tile_row[(int64_t)(pos[g] / 4) * kNarrowTileScaleHalfs + r * 4 + pos[g] % 4] = v;
      else
        tile_row[wide_base + (int64_t)(pos[g] / 8) * kWideTileScaleHalfs + r * 8 + pos[g] % 8] = v;
    }
  }
  return CCQ_OK;
}

extern "C" int ccq_pack_meta(const ccq_weight* w, void* out_v) {
  if (!w || !out_v) return CCQ_ERR_NULL;
  Layout L;
  int rc = make_layout(w, &L);
  if (rc != CCQ_OK) return rc;
  int32_t* out = static_cast<int32_t*>(out_v);
  std::vector<int> pos, kind;
  packed_order(w, L, pos, kind);
  // padded positions name the last real group: its activations are read in place of theirs (their scale is 0)
  for (int i = 0; i < L.pgroups[kNarrow] + L.pgroups[kWide]; ++i) out[i] = L.G - 1;
  for (int g = 0; g < L.G; ++g) out[(kind[g] == kNarrow ? 0 : L.pgroups[kNarrow]) + pos[g]] = g;
  return CCQ_OK;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static int check_weight_ptrs(const ccq_weight* w, const Layout& L) {
  if (!w->codes) return CCQ_ERR_NULL;
  if (!w->scales && (L.scale_mode == 0 || L.groups[kNarrow] > 0)) return CCQ_ERR_NULL;
  if (L.scale_mode == 1 && !w->scale_super) return CCQ_ERR_NULL;
  if (L.groups[kNarrow] > 0 && (!w->code_alpha || !w->code_beta)) return CCQ_ERR_NULL;
  if (L.has_map && !w->meta) return CCQ_ERR_NULL;
  if (!aligned16(w->codes) || !aligned16(w->scales) || !aligned16(w->code_alpha) || !aligned16(w->code_beta) || !aligned16(w->meta) ||
      (L.scale_mode == 1 && !aligned16(w->scale_super)))
    return CCQ_ERR_ALIGN;
  return CCQ_OK;
}

namespace ccq {

static bool is_explicit(const ccq_launch* l) { return l && (l->rows_per_wave_tiles || l->waves_rows || l->waves_k || l->splits_k); }

// Decomposition of one pass of mc rows of the per-row-tile kernel.
static int pass_decomp(const Layout& L, int mc, const ccq_launch* launch, Decomp* d) {
  if (is_explicit(launch)) {
    d->RT = launch->rows_per_wave_tiles ? launch->rows_per_wave_tiles : 1;
    d->WR = launch->waves_rows ? launch->waves_rows : 1;
    d->WK = launch->waves_k ? launch->waves_k : 1;
    d->S = launch->splits_k ? launch->splits_k : 1;
    if (!decomp_ok(L, *d)) return CCQ_ERR_BAD_PARAM;
  } else {
    *d = choose_decomp(L, mc, 1, mc);
  }
  return CCQ_OK;
}

// Everything is checked before the first launch: arguments, the decomposition of every pass and the workspace
// each of them needs.  After that only a failing HIP launch (CCQ_ERR_HIP) can end a call part-way.
int gemm_dispatch(const ccq_weight* w, const void* x, int32_t M, int64_t ldx, void* y, int64_t ldy, void* workspace,
                  int64_t workspace_bytes, void* stream, const ccq_launch* launch) {
  if (!w) return CCQ_ERR_NULL;
  Layout L;
  int rc = make_layout(w, &L);
  if (rc != CCQ_OK) return rc;
  if (M < 0 || workspace_bytes < 0) return CCQ_ERR_BAD_PARAM;
  if (M == 0) return CCQ_OK;
  if (!x || !y) return CCQ_ERR_NULL;
  rc = check_weight_ptrs(w, L);
  if (rc != CCQ_OK) return rc;
  if (ldx < L.K || ldy < L.N) return CCQ_ERR_BAD_PARAM;
  if (!aligned16(x) || !aligned16(y) || !aligned16(workspace) || ldx % 8 != 0 || ldy % 8 != 0) return CCQ_ERR_ALIGN;
  const int64_t have = workspace ? workspace_bytes : 0;

  const bool explicit_launch = is_explicit(launch);
  // the passes of the per-row-tile kernel (the explicit path, and what the other paths fall back to)
  int64_t need_passes = 0;
  for (int mc : {M >= kMaxSkinnyM ? kMaxSkinnyM : 0, M % kMaxSkinnyM}) {
    if (mc == 0) continue;
    Decomp d;
    rc = pass_decomp(L, mc, launch, &d);
    if (rc != CCQ_OK) return rc;
    if (d.S > 1) need_passes = std::max(need_passes, (int64_t)d.S * mc * L.Npad * 4);
  }
  if (!explicit_launch && dense_path(L, M) != kPathGemv16 && dense_path(L, M) != kPathGemv16NW && have < dense_need(L, M)) return CCQ_ERR_WORKSPACE;

  if (!explicit_launch) {
    const DensePath path = dense_path(L, M);
    // many rows, narrow format only: the 256-row LDS-tiled MFMA kernel
    if (path == kPathPrefill) {
      rc = launch_prefill(w, L, x, M, ldx, y, ldy, stream);
      if (rc != CCQ_ERR_UNSUPPORTED) return rc;
    }
    if (path == kPathGemv16) {
      // as many shares of K as the chip wants and the workspace holds (a smaller workspace only means longer shares)
      int tpw = 0, nw = 0;
      const int64_t plane = (int64_t)M * L.Npad * 4;
      if (gemv16_shape(L, device_cus(), std::max<int64_t>(1, have / plane), &tpw, &nw)) {
        const int S = (L.tiles[kNarrow] + tpw - 1) / tpw;
        float* partial = S > 1 ? static_cast<float*>(workspace) : nullptr;
        rc = launch_gemv16(w, L, x, M, ldx, y, ldy, partial, tpw, nw, stream);
        if (rc == CCQ_OK && S > 1) rc = launch_reduce_splits(partial, y, ldy, M, L.N, L.Npad, S, stream);
        if (rc != CCQ_ERR_UNSUPPORTED) return rc;
      }
    }
    if (path == kPathGemv16NW) {
      // the same on wide-format and mixed weights
      int tpwn = 0, tpww = 0, sn = 0, sw = 0;
      const int64_t plane = (int64_t)M * L.Npad * 4;
      if (gemv16_nw_shape(L, device_cus(), std::max<int64_t>(1, have / plane), &tpwn, &tpww, &sn, &sw)) {
        const int S = sn + sw;
        float* partial = S > 1 ? static_cast<float*>(workspace) : nullptr;
        rc = launch_gemv16_nw(w, L, x, M, ldx, y, ldy, partial, tpwn, tpww, sn, sw, stream);
        if (rc == CCQ_OK && S > 1) rc = launch_reduce_splits(partial, y, ldy, M, L.N, L.Npad, S, stream);
        if (rc != CCQ_ERR_UNSUPPORTED) return rc;
      }
    }
    if (path == kPathRows) {
      const int S = rows_splits(L, M);
      float* partial = S > 1 ? static_cast<float*>(workspace) : nullptr;
      rc = launch_rows(w, L, x, M, ldx, y, ldy, partial, S, stream);
      if (rc == CCQ_OK && S > 1) rc = launch_reduce_splits(partial, y, ldy, M, L.N, L.Npad, S, stream);
      return rc;
    }
    // a few dozen rows (or many rows on wide / mixed formats): the 64-row LDS-tiled kernel
    if (path == kPathMid || path == kPathPrefill) {
      const int S = mid_splits(L, M);
      float* partial = S > 1 ? static_cast<float*>(workspace) : nullptr;
      rc = launch_mid(w, L, x, M, ldx, y, ldy, partial, S, stream);
      if (rc == CCQ_OK && S > 1) rc = launch_reduce_splits(partial, y, ldy, M, L.N, L.Npad, S, stream);
      if (rc != CCQ_ERR_UNSUPPORTED) return rc;
    }
    // one to four rows, narrow format only: the lean GEMV kernel (same arithmetic as the general path)
    if (path == kPathGemv) {
      int tpw = 0, waves = 0;
      if (M == 1 && gemv1_shape(L, device_cus(), &tpw, &waves)) {
        rc = launch_gemv1(w, L, x, y, stream, tpw, waves);
        if (rc != CCQ_ERR_UNSUPPORTED) return rc;
      }
      if (M > 1 && gemv4_shape(L, device_cus(), &tpw, &waves)) {
        rc = launch_gemv4(w, L, x, M, ldx, y, ldy, stream, tpw, waves);
        if (rc != CCQ_ERR_UNSUPPORTED) return rc;
      }
    }
  }

  // one row on wide-format or mixed weights: the one-row kernel for those formats
  if (!explicit_launch && M == 1) {
    int tpwn = 0, tpww = 0, wn = 0, ww = 0;
    if (gemv_nw_shape(L, &tpwn, &tpww, &wn, &ww)) {
      rc = launch_gemv_nw(w, L, x, y, stream, tpwn, tpww, wn, ww);
      if (rc != CCQ_ERR_UNSUPPORTED) return rc;
    }
  }

  // otherwise rows are processed in passes of at most kMaxSkinnyM (nothing has been enqueued when control gets here)
  if (have < need_passes) return CCQ_ERR_WORKSPACE;
  for (int m0 = 0; m0 < M; m0 += kMaxSkinnyM) {
    const int mc = std::min(kMaxSkinnyM, M - m0);
    SkinnyCall c;
    c.w = w;
    c.L = L;
    rc = pass_decomp(L, mc, launch, &c.d);
    if (rc != CCQ_OK) return rc;
    if (c.d.S > 1) c.partial = static_cast<float*>(workspace);
    c.E = 1;
    c.x = static_cast<const uint16_t*>(x) + (int64_t)m0 * ldx;
    c.ldx = ldx;
    c.y = static_cast<uint16_t*>(y) + (int64_t)m0 * ldy;
    c.ldy = ldy;
    c.M = mc;
    c.m_tile_hint = mc;
    c.stream = stream;
    rc = launch_skinny(c);
    if (rc != CCQ_OK) return rc;
  }
  return CCQ_OK;
}

int64_t gemm_workspace_need(const ccq_weight* w, int32_t M) {
  Layout L;
  if (!w || M < 0 || make_layout(w, &L) != CCQ_OK) return -1;
  return dense_need(L, M);
}

}  // namespace ccq

extern "C" int64_t ccq_gemm_workspace_bytes(const ccq_weight* w, int32_t M) { return ccq::gemm_workspace_need(w, M); }

extern "C" int ccq_gemm(const ccq_weight* w, const void* x, int32_t M, int64_t ldx, void* y, int64_t ldy, void* workspace,
                        int64_t workspace_bytes, void* hip_stream) {
  return gemm_dispatch(w, x, M, ldx, y, ldy, workspace, workspace_bytes, hip_stream, nullptr);
}

extern "C" int ccq_gemm_ex(const ccq_weight* w, const void* x, int32_t M, int64_t ldx, void* y, int64_t ldy, void* workspace,
                           int64_t workspace_bytes, void* hip_stream, const ccq_launch* launch) {
  return gemm_dispatch(w, x, M, ldx, y, ldy, workspace, workspace_bytes, hip_stream, launch);
}

static int grouped_tile_rows(int E, int P) {
  // rows one pass holds: twice the mean rows per expert, rounded up to 16, at most 64
  int64_t mean2 = E > 0 ? (2 * (int64_t)P + E - 1) / E : 0;
  int rows = (int)std::min<int64_t>(kMaxSkinnyM, std::max<int64_t>(16, ((mean2 + 15) / 16) * 16));
  return rows;
}

// Launch shape of a grouped call.  `active` = experts that have rows (known only when the caller passes the
// host copy of the offsets; otherwise all E are assumed busy).  With few active experts -- a decode step routes
// a handful of tokens to 8 of 256 experts -- the row blocks alone cannot fill the chip, so K is cut into more
// shares, as many as the workspace the caller brought allows.
static Decomp grouped_decomp(const Layout& L, int E, int P, int active, int64_t workspace_bytes) {
  Decomp d = choose_decomp(L, grouped_tile_rows(E, P), std::max(1, active), P);
  const int64_t per_share = (int64_t)P * L.Npad * 4;
  if (d.S > 1 && per_share > 0) d.S = (int)std::max<int64_t>(1, std::min<int64_t>(d.S, workspace_bytes / per_share));
  return d;
}

// Recommended workspace: room for the K shares a call with few active experts would like (at most 64 MiB); a
// smaller workspace, down to none, only means fewer shares.
extern "C" int64_t ccq_grouped_workspace_bytes(const ccq_weight* w0, int32_t E, int32_t P) {
  Layout L;
  if (make_layout(w0, &L) != CCQ_OK || E <= 0 || P < 0) return -1;
  if (P == 0) return 0;
  const int active_min = std::max(1, std::min(E, (P + kMaxSkinnyM - 1) / kMaxSkinnyM));
  Decomp d = choose_decomp(L, grouped_tile_rows(E, P), active_min, P);
  const int64_t want = d.S > 1 ? (int64_t)d.S * P * L.Npad * 4 : 0;
  return std::min<int64_t>(want, (int64_t)64 << 20);
}

extern "C" int ccq_grouped_gemm(const ccq_weight* w0, int32_t E, int64_t codes_stride, int64_t scales_stride, int64_t ab_stride,
                                const void* x, int32_t T, int64_t ldx, const int32_t* sorted_rows, int32_t P,
                                const int32_t* expert_offsets_dev, const int32_t* expert_offsets_host, void* y, int64_t ldy,
                                void* workspace, int64_t workspace_bytes, void* hip_stream) {
  if (!w0) return CCQ_ERR_NULL;
  Layout L;
  int rc = make_layout(w0, &L);
  if (rc != CCQ_OK) return rc;
  if (E <= 0 || P < 0 || T < 0 || workspace_bytes < 0) return CCQ_ERR_BAD_PARAM;
  if (expert_offsets_host) {
    if (expert_offsets_host[0] != 0 || expert_offsets_host[E] != P) return CCQ_ERR_ROUTING;
    for (int e = 0; e < E; ++e)
      if (expert_offsets_host[e + 1] < expert_offsets_host[e]) return CCQ_ERR_ROUTING;
  }
  if (P == 0) return CCQ_OK;
  if (T == 0) return CCQ_ERR_ROUTING;
  if (!x || !y || !sorted_rows || !expert_offsets_dev) return CCQ_ERR_NULL;
  rc = check_weight_ptrs(w0, L);
  if (rc != CCQ_OK) return rc;
  if (ldx < L.K || ldy < L.N) return CCQ_ERR_BAD_PARAM;
  if (E > 1) {
    const int64_t code_bytes = L.row_tile_bytes * L.row_tiles, scale_bytes = L.row_tile_scale_halfs * L.row_tiles * 2;
    if (codes_stride < code_bytes || scales_stride < scale_bytes) return CCQ_ERR_BAD_PARAM;
    if ((L.groups[kNarrow] > 0 || L.scale_mode == 1) && ab_stride < (int64_t)L.N * 4) return CCQ_ERR_BAD_PARAM;
    if (codes_stride % 16 || scales_stride % 16 || ab_stride % 16) return CCQ_ERR_ALIGN;
  }
  if (!aligned16(x) || !aligned16(y) || !aligned16(workspace) || !aligned16(sorted_rows) || !aligned16(expert_offsets_dev) ||
      ldx % 8 != 0 || ldy % 8 != 0)
    return CCQ_ERR_ALIGN;
  SkinnyCall c;
  c.w = w0;
  c.L = L;
  c.m_tile_hint = grouped_tile_rows(E, P);
  int active = E, most_rows = P;
  if (expert_offsets_host) {
    active = 0;
    most_rows = 0;
    for (int e = 0; e < E; ++e) {
      const int rows = expert_offsets_host[e + 1] - expert_offsets_host[e];
      active += rows > 0 ? 1 : 0;
      most_rows = std::max(most_rows, rows);
    }
  }
  if (expert_offsets_host && active < E && active <= kMaxActiveList && E <= 65536) {
    // launch over the experts that have rows only
    c.n_active = active;
    int k = 0;
    for (int e = 0; e < E; ++e)
      if (expert_offsets_host[e + 1] > expert_offsets_host[e]) c.active_ids[k++] = (uint16_t)e;
  }
  if (expert_offsets_host && most_rows > 32) {
    // many rows per expert (a prefill-sized routing): the 64-row kernel, one grid over (row block, column block,
    // expert); on narrow-format weights measured 2.2-2.4 times faster than 64-row passes of the per-row-tile kernel
    // from 33 rows on, slower below
    rc = launch_mid_grouped(w0, L, E, codes_stride, scales_stride, ab_stride, x, ldx, sorted_rows, P, expert_offsets_dev, most_rows, y, ldy,
                            hip_stream);
    if (rc != CCQ_ERR_UNSUPPORTED) return rc;
  }
  const int with_rows = expert_offsets_host ? active : std::min(E, P);   // experts that have rows (without the host copy: at most P)
  if (most_rows <= kGemvMaxM &&
      (c.n_active > 0 || (int64_t)(E - with_rows) * L.row_tiles <= std::max<int64_t>(64 * (int64_t)device_cus(), (int64_t)with_rows * L.row_tiles / 2))) {
    // one or a few tokens' decode step: every expert that has rows is a GEMV (or a four-row product) of its own.  (Not
    // when the grid would have to span many more experts without rows than with: dispatching their workgroups costs
    // more than it saves.  Letting experts with more rows take one pass over their weights per four rows measured
    // slower than the per-row-tile kernel once most experts need the four-row body: 181 against 150 us on 224 experts
    // of 1024 x 7168 with 512 rows.)
    rc = launch_gemv_grouped(w0, L, E, codes_stride, scales_stride, ab_stride, x, ldx, sorted_rows, expert_offsets_dev, y, ldy, most_rows,
                             c.n_active, c.active_ids, hip_stream);
    if (rc != CCQ_ERR_UNSUPPORTED) return rc;
    if (most_rows == 1) {   // the same on the wide, mixed and hybrid-word formats, one row per expert only
      rc = launch_gemv_nw_grouped(w0, L, E, codes_stride, scales_stride, ab_stride, x, ldx, sorted_rows, expert_offsets_dev, y, ldy, c.n_active,
                                  c.active_ids, hip_stream);
      if (rc != CCQ_ERR_UNSUPPORTED) return rc;
    }
  }
  if (most_rows == 1) {
    // no expert has more than one row (on formats or shapes the kernel above is not built for): the
    // one-held-row kernel (wavefront-private staging, no 16-row activation tile)
    c.m_tile_hint = 1;
    c.d = choose_decomp(L, 1, std::max(1, active), P);
    // the grid spans all E experts and most of them have no row: beyond about 64 workgroups per CU the dispatch of the
    // empty ones shows, and fewer, larger workgroups (several row tiles side by side, at most 512 threads) are faster
    const int wr_max = std::max(1, std::min(std::min(4, 8 / c.d.WK), L.row_tiles / c.d.RT));
    while (c.d.WR * 2 <= wr_max && (int64_t)ceil_div(L.row_tiles, c.d.RT * c.d.WR) * (c.n_active > 0 ? c.n_active : E) > 64 * (int64_t)device_cus()) c.d.WR *= 2;
  } else {
    c.d = grouped_decomp(L, E, P, active, workspace ? workspace_bytes : 0);
  }
  if (c.d.S > 1) c.partial = static_cast<float*>(workspace);
  c.E = E;
  c.codes_stride = codes_stride;
  c.scales_stride = scales_stride;
  c.ab_stride = ab_stride;
  c.x = x;
  c.ldx = ldx;
  c.y = y;
  c.ldy = ldy;
  c.M = P;
  c.sorted_rows = sorted_rows;
  c.expert_offsets = expert_offsets_dev;
  c.stream = hip_stream;
  return launch_skinny(c);
}

// The GPU quantizer is built for every layout the multiply kernels read.
static int encode_layout(const ccq_weight* w, Layout* L) { return make_layout(w, L); }

extern "C" int64_t ccq_quantize_workspace_bytes(const ccq_weight* w) {
  Layout L;
  if (!w || encode_layout(w, &L) != CCQ_OK) return -1;
  return encode_workspace_bytes(L);
}

extern "C" int ccq_quantize(const ccq_weight* w, const float* W, int64_t ldw, void* codes_out, void* scales_out, float* alpha_out,
                            float* beta_out, void* scale_super_out, void* workspace, int64_t workspace_bytes, void* hip_stream) {
  if (!w) return CCQ_ERR_NULL;
  Layout L;
  int rc = encode_layout(w, &L);
  if (rc != CCQ_OK) return rc;
  const bool cluster = L.groups[kNarrow] > 0;
  if (!W || !codes_out) return CCQ_ERR_NULL;
  if (!scales_out && (L.scale_mode == 0 || cluster)) return CCQ_ERR_NULL;  // wide groups keep compressed scales in the code stream
  if (cluster && (!alpha_out || !beta_out)) return CCQ_ERR_NULL;
  if (L.scale_mode == 1 && !scale_super_out) return CCQ_ERR_NULL;
  if (L.has_map && !w->meta) return CCQ_ERR_NULL;
  if (!aligned16(w->meta)) return CCQ_ERR_ALIGN;
  if (ldw < L.K) return CCQ_ERR_BAD_PARAM;
  if (!aligned16(W) || !aligned16(codes_out) || !aligned16(scales_out) || !aligned16(alpha_out) || !aligned16(beta_out) || !aligned16(scale_super_out) ||
      !aligned16(workspace) || ldw % 4 != 0)
    return CCQ_ERR_ALIGN;
  const int64_t need = encode_workspace_bytes(L);
  if (need > 0 && (!workspace || workspace_bytes < need)) return CCQ_ERR_WORKSPACE;
  return launch_encode(L, W, ldw, codes_out, scales_out, alpha_out, beta_out, scale_super_out, static_cast<const int32_t*>(w->meta),
                       need > 0 ? workspace : nullptr, hip_stream);
}

extern "C" const char* ccq_status_string(int status) {
  switch (status) {
    case CCQ_OK: return "CCQ_OK";
    case CCQ_ERR_NULL: return "CCQ_ERR_NULL";
    case CCQ_ERR_BAD_PARAM: return "CCQ_ERR_BAD_PARAM";
    case CCQ_ERR_UNSUPPORTED: return "CCQ_ERR_UNSUPPORTED";
    case CCQ_ERR_ALIGN: return "CCQ_ERR_ALIGN";
    case CCQ_ERR_WORKSPACE: return "CCQ_ERR_WORKSPACE";
    case CCQ_ERR_ROUTING: return "CCQ_ERR_ROUTING";
    case CCQ_ERR_HIP: return "CCQ_ERR_HIP";
    default: return "CCQ_ERR_UNKNOWN";
  }
}
