// Internal declarations shared by the host layer and the kernel launchers of
// libccq.  Nothing here is part of the public C ABI (include/ccq.h).
#pragma once
#include <cstdint>

#include "ccq.h"

namespace ccq {

// ---- device layout of the packed code stream ------------------------------
// Output rows are cut into tiles of 16; K is cut into k-tiles.  A k-tile of the
// narrow format spans 4 groups (256 weights), one of the wide format 8 groups
// (512 weights).  Inside a row tile all narrow k-tiles come first (k order),
// then all wide k-tiles.  Lane l of a wavefront owns output row (l % 16) and
// quarter kq = l / 16 of every group.
//
//   narrow k-tile (1024 B): lane l reads bytes [16 l, 16 l + 16): dword j is
//     group j of the tile, holding that group's canonical bytes 4kq..4kq+3
//     (the codes of weights 16kq..16kq+15).
//   wide k-tile (2816 B): three segments t = 0,1,2 of 1024, 1024, 768 bytes;
//     lane l reads 16 bytes of segment t: halfword j is group j of the tile,
//     holding canonical bytes 6kq+2t, 6kq+2t+1 of the group (quarter 3 has only
//     bytes 18..21, so segment 2 has no entries for lanes 48..63).
//   hybrid-word k-tile (2560 B; Sec. 3.2, one (3,3,2) and one (3,4,2) code in a 16-bit word, ten
//     words per group): takes the place of the wide kind.  Three segments t = 0,1,2 of 1024, 1024,
//     512 bytes; halfword j of lane l's 16 bytes of segment t is word 4t + kq of group j (words 8
//     and 9 only: segment 2 has no entries for lanes 32..63).
constexpr int kGroup = 64;
constexpr int kRowsPerTile = 16;
constexpr int kNarrowGroupsPerTile = 4;
constexpr int kWideGroupsPerTile = 8;
constexpr int kNarrowTileBytes = 1024;
constexpr int kWideTileBytes = 2816;
constexpr int kNarrowGroupBytes = 16;
constexpr int kWideGroupBytes = 22;
constexpr int kH16TileBytes = 2560;
constexpr int kH16GroupBytes = 20;
// fp16 scales: per row tile, per k-tile, [row 0..15][group of the tile]
constexpr int kNarrowTileScaleHalfs = 16 * 4;
constexpr int kWideTileScaleHalfs = 16 * 8;
// compressed scales (Sec. 3.4): per narrow k-tile one 16-bit word per row, holding the four 4-bit
// fields of the tile's groups (group j in bits 4j..4j+3); wide groups keep theirs in the code stream
constexpr int kNarrowTileScaleHalfs4 = 16;

constexpr int kMaxSkinnyM = 64;   // rows one pass of the skinny kernel holds
constexpr int kMaxSplitsK = 32;

enum Kind : int { kNarrow = 0, kWide = 1 };

// A validated view of a ccq_weight.  The device layout holds whole row tiles and whole k-tiles: a matrix whose
// N is not a multiple of 16, or whose groups of a kind do not fill their last k-tile, is padded by the pack routines
// with rows and groups of zero codes and zero scales (they decode to zeros); the kernels never store the padded
// rows and read the activations of the last real group in place of a padded group's.
struct Layout {
  int K = 0, N = 0, G = 0;      // as given: N output rows, G = K / 64 groups
  int Npad = 0;                 // N rounded up to whole row tiles
  int groups[2] = {0, 0};       // groups per kind, as given
  int pgroups[2] = {0, 0};      // groups per kind in the device layout (whole k-tiles)
  int tiles[2] = {0, 0};        // k-tiles per kind
  int kind_of_fmt[2] = {0, 0};  // descriptor format index -> Kind
  float zp[2] = {0.f, 0.f};     // zero-point per kind
  bool has_map = false;         // group_fmt given
  bool h16 = false;             // the second kind is the hybrid 16-bit word of Sec. 3.2 (then there are no narrow groups)
  int scale_mode = 0;           // 0 fp16 group scales, 1 4-bit fields times a per-row super scale
  int64_t row_tile_bytes = 0;
  int64_t row_tile_scale_halfs = 0;
  int row_tiles = 0;
  bool padded() const { return Npad != N || pgroups[0] != groups[0] || pgroups[1] != groups[1]; }
};

// Validates the shape/format part of a descriptor (no pointer checks).
int make_layout(const ccq_weight* w, Layout* out);
// Kind of group g.
inline int group_kind(const ccq_weight* w, const Layout& L, int g) {
  return L.kind_of_fmt[w->group_fmt ? w->group_fmt[g] : 0];
}

// Launch decomposition of the skinny kernel.
struct Decomp {
  int RT = 1;  // 16-row tiles per wavefront
  int WR = 1;  // wavefronts along rows per workgroup
  int WK = 1;  // wavefronts along K per workgroup
  int S = 1;   // workgroups along K
};
Decomp choose_decomp(const Layout& L, int M, int experts, int rows_total);
bool decomp_ok(const Layout& L, const Decomp& d);

// Kernel launchers (ccq_skinny.hip).  All pointers DEVICE unless noted.
// Grouped calls whose host copy of the offsets shows at most this many experts with rows launch a grid over those
// experts only; their ids travel in the kernel arguments.
constexpr int kMaxActiveList = 128;

struct SkinnyCall {
  const ccq_weight* w = nullptr;  // HOST descriptor of expert 0
  Layout L;
  Decomp d;
  int E = 1;
  int64_t codes_stride = 0, scales_stride = 0, ab_stride = 0;
  const void* x = nullptr;
  int64_t ldx = 0;
  void* y = nullptr;
  int64_t ldy = 0;
  int M = 0;                            // rows (dense) / P total rows (grouped)
  int m_tile_hint = 0;                  // rows one pass should hold (<= 64)
  const int32_t* sorted_rows = nullptr; // grouped only
  const int32_t* expert_offsets = nullptr;
  float* partial = nullptr;             // fp32 [S][M][N] when S > 1
  void* stream = nullptr;
  int n_active = 0;                     // > 0: the grid's z extent; block z works on expert active_ids[z]
  uint16_t active_ids[kMaxActiveList] = {};
};
int launch_skinny(const SkinnyCall& c);

constexpr int kGemvMaxM = 4;       // rows of the four-row kernel

// One activation row on narrow-format weights (ccq_gemv.hip): shape of the launch for a chip of `cus` compute units
// (false when K does not split into at most 16 shares of a built length, the last one possibly shorter), and the
// launcher; the same for two to four rows (gemv4: equal shares only, and false when the four rows' activation fragments
// of all of K do not fit the LDS twice), and for one row on wide-format and mixed weights (gemv_nw).
bool gemv1_shape(const Layout& L, int cus, int* tpw_out, int* w_out);
int launch_gemv1(const ccq_weight* w, const Layout& L, const void* x, void* y, void* stream, int tpw, int waves);
bool gemv4_shape(const Layout& L, int cus, int* tpw_out, int* w_out);
int launch_gemv4(const ccq_weight* w, const Layout& L, const void* x, int M, int64_t ldx, void* y, int64_t ldy, void* stream, int tpw, int waves);
// Grouped product with at most `most_rows` <= 4 rows per expert on narrow-format weights: one GEMV (or four-row
// product) per expert; `active_ids` lists the n_active experts that have rows (n_active = 0: the grid covers all E).
bool gemv_grouped_shape(const Layout& L, int cus, int experts, bool four, int* tpw_out, int* w_out);
int launch_gemv_grouped(const ccq_weight* w0, const Layout& L, int E, int64_t codes_stride, int64_t scales_stride, int64_t ab_stride, const void* x,
                        int64_t ldx, const int32_t* sorted_rows, const int32_t* expert_offsets_dev, void* y, int64_t ldy, int most_rows,
                        int n_active, const uint16_t* active_ids, void* stream);
bool gemv_nw_shape(const Layout& L, int* tpwn_out, int* tpww_out, int* wn_out, int* ww_out);
int launch_gemv_nw(const ccq_weight* w, const Layout& L, const void* x, void* y, void* stream, int tpwn, int tpww, int wn, int ww);
int launch_gemv_nw_grouped(const ccq_weight* w0, const Layout& L, int E, int64_t codes_stride, int64_t scales_stride, int64_t ab_stride,
                           const void* x, int64_t ldx, const int32_t* sorted_rows, const int32_t* expert_offsets_dev, void* y, int64_t ldy,
                           int n_active, const uint16_t* active_ids, void* stream);
int device_cus();  // compute units of the current device (cached per device)
// Two to sixteen rows on narrow-format weights (ccq_gemv.hip): K is cut into tiles / tpw shares across workgroups; with
// more than one share the fp32 partial tiles go to `partial` ([shares][M][N]) and launch_reduce_splits adds them.
bool gemv16_shape(const Layout& L, int cus, int64_t max_shares, int* tpw_out, int* nw_out);
bool gemv16_nw_shape(const Layout& L, int cus, int64_t max_shares, int* tpwn_out, int* tpww_out, int* sn_out, int* sw_out);
int launch_gemv16_nw(const ccq_weight* w, const Layout& L, const void* x, int M, int64_t ldx, void* y, int64_t ldy, float* partial, int tpwn,
                     int tpww, int sn, int sw, void* stream);
int launch_gemv16(const ccq_weight* w, const Layout& L, const void* x, int M, int64_t ldx, void* y, int64_t ldy, float* partial, int tpw,
                  int nw, void* stream);

// Kernel for a few dozen to a few hundred rows, any format mix (ccq_mid.hip): 64-row tiles, K cut into S
// shares whose fp32 partial tiles go to `partial` ([S][M][N]) when S > 1 (then call launch_reduce_splits).
constexpr int kMidMinM = 17;
int launch_mid_grouped(const ccq_weight* w0, const Layout& L, int E, int64_t codes_stride, int64_t scales_stride, int64_t ab_stride, const void* x,
                       int64_t ldx, const int32_t* sorted_rows, int P, const int32_t* expert_offsets, int most_rows, void* y, int64_t ldy,
                       void* stream);
int mid_splits(const Layout& L, int M);
int launch_mid(const ccq_weight* w, const Layout& L, const void* x, int M, int64_t ldx, void* y, int64_t ldy, float* partial, int S,
               void* stream);
// y[m][n] = bf16(sum_s partial[s][m][n]), shares added in index order (ccq_skinny.hip).
int launch_reduce_splits(const float* partial, void* y, int64_t ldy, int rows, int N, int Npad, int S, void* stream);

// Per-group activation tiles, weights in registers (ccq_skinny.hip).  Built for up to 16 rows on wide-only and
// hybrid-word layouts and for 17-32 rows on narrow-only ones; CCQ_ERR_UNSUPPORTED otherwise.
int rows_splits(const Layout& L, int M);
int launch_rows(const ccq_weight* w, const Layout& L, const void* x, int M, int64_t ldx, void* y, int64_t ldy, float* partial, int S,
                void* stream);

// The dispatcher behind ccq_gemm / ccq_gemm_ex (ccq_host.cpp) and the workspace a call of exactly M rows needs.
int gemm_dispatch(const ccq_weight* w, const void* x, int32_t M, int64_t ldx, void* y, int64_t ldy, void* workspace,
                  int64_t workspace_bytes, void* stream, const ccq_launch* launch);
int64_t gemm_workspace_need(const ccq_weight* w, int32_t M);

// Large-M kernel for narrow-format weights (ccq_prefill.hip).
int prefill_block_cols(const Layout& L, int M);  // column-block width launch_prefill uses: 128, 192 or 256
int launch_prefill(const ccq_weight* w, const Layout& L, const void* x, int M, int64_t ldx, void* y, int64_t ldy, void* stream);

// The quantizer (ccq_encode.hip): every layout the multiply kernels read, fp16 or compressed group scales.
int64_t encode_workspace_bytes(const Layout& L);
int launch_encode(const Layout& L, const float* W, int64_t ldw, void* codes, void* scales, float* alpha, float* beta, void* scale_super,
                  const int32_t* meta, void* workspace, void* stream);

}  // namespace ccq
