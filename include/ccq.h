/*
 * libccq -- fused dequantize-and-multiply for Convolutional Code Quantization
 * (CCQ, arXiv 2507.07145) on AMD MI355X (gfx950).
 *
 * The library computes  y = x * W_dq^T  where W_dq is never materialised in
 * memory: the packed convolutional-code bitstream is streamed from HBM, the
 * overlapping L-bit states are cut out of each code with bit shifts (Sec. 3.1
 * "Bitshift Decoding", Table 1), mapped to values by the linear rule
 * (state - zp) * scale (Alg. 2 / Alg. 3, last line of the loop) and contracted
 * against bf16 activations with fp32 accumulation.  No codebook is stored or
 * looked up.
 *
 * Supported code configurations (Table 1):
 *   narrow  (L=6,N=4,S=3) with Code Cluster: one byte per 4 weights (2.0 bpw);
 *           the byte q is first expanded to the 15-bit code
 *           c = round(q * code_alpha[n] + code_beta[n])   (Alg. 3, Eq. 1)
 *   wide    (L=4,N=3,S=2): 22 bytes per 64 weights (2.75 bpw), Alg. 2.
 *   hybrid  (L=3,N=3,S=2) and (L=3,N=4,S=2) side by side in one little-endian
 *           16-bit word (Sec. 3.2 "Hybrid Encoding", Table 1 row 2): seven
 *           3-bit states per word at the shifts [13,11,9,6,4,2,0]; a 64-weight
 *           group is 10 words (20 bytes, 2.5 bpw), the last of which carries
 *           weight 63 in its top state and 13 unused bits.  Selected by
 *           n_formats = 2, fmt[0] = (3,3,2), fmt[1] = (3,4,2), both with the
 *           same zp and code_cluster = 0, group_fmt = NULL.  With scale_mode 1
 *           the 13 unused bits hold the scale field (scale mask 0x1FFF of
 *           Table 1; Alg. 2: s = (last word & 0x1FFF) * scale_super[n]) and
 *           `scales` is not used.
 * A weight matrix uses the narrow format, the wide format, a per-group mix of
 * those two (group_fmt), all rows sharing the same map, or the hybrid word.
 * Group size is 64 along K (K a multiple of 64; N, K and the group map are otherwise free) and scales are fp16, one
 * per (row, group), unless scale_mode says otherwise.
 *
 * Conventions
 *   - Every pointer is marked HOST or DEVICE.  The caller owns all buffers; the
 *     library never allocates or frees device memory and never synchronises
 *     (the host-side ccq_pack_* routines use temporary host memory of their
 *     own).  DEVICE pointers must be 16-byte aligned.
 *   - ccq_gemm / ccq_grouped_gemm enqueue work on `hip_stream` (a hipStream_t
 *     passed as void*, NULL = the default stream) and return immediately.
 *   - Return value: CCQ_OK or a negative ccq_status.  Arguments, launch shapes
 *     and workspace sizes are all checked before the first launch: on any
 *     error other than CCQ_ERR_HIP nothing has been enqueued (CCQ_ERR_HIP
 *     reports a HIP launch that failed, possibly after earlier launches of
 *     the same call).
 *   - "Canonical" order is the paper's: row n of W_q is the concatenation over
 *     groups (k order) of the group's codes, code j covering weights N*j..N*j+N-1
 *     of the group (Alg. 2/3: q_w = W_q[idx / p_w]); the first state of a code
 *     sits in its most significant bits (Sec. 3.1, the 00->01->10 = 0010
 *     example).  The kernels read a permuted "device" order of the same bytes,
 *     produced by the ccq_pack_* host routines below; it stores the same bytes, plus
 *     zero padding up to whole tiles (see ccq_info).
 */
#ifndef CCQ_H
#define CCQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CCQ_OK = 0,
  CCQ_ERR_NULL = -1,        /* a required pointer is NULL                    */
  CCQ_ERR_BAD_PARAM = -2,   /* inconsistent sizes / values                   */
  CCQ_ERR_UNSUPPORTED = -3, /* valid CCQ, but not built into the kernels     */
  CCQ_ERR_ALIGN = -4,       /* DEVICE pointer or leading dim not aligned     */
  CCQ_ERR_WORKSPACE = -5,   /* workspace missing or too small                */
  CCQ_ERR_ROUTING = -6,     /* expert offsets not monotone / out of range    */
  CCQ_ERR_HIP = -7          /* a HIP runtime call failed                     */
} ccq_status;

/* A convolutional-code configuration, Sec. 3.1: L bits per state, N states per
 * code, S transition bits between adjacent states; T = L + (N-1)*S code bits. */
typedef struct {
  int32_t L, N, S;
  int32_t code_cluster; /* 1: the stored code is the 8-bit clustered value (Sec. 3.3) */
  float zp;             /* weight zero-point of Alg. 2/3; a multiple of 0.5  */
} ccq_code;

/* One quantized weight matrix W[N][K] (N output channels, K input channels). */
typedef struct {
  int32_t K, N;
  int32_t group;            /* weights per scale along K; must be 64         */
  int32_t n_formats;        /* 1 or 2                                        */
  ccq_code fmt[2];          /* fmt[0] = narrow (6,4,3)+cluster or wide; with 2 formats fmt[0] narrow, fmt[1] wide,
                               or the two halves (3,3,2), (3,4,2) of the hybrid word                  */
  const uint8_t *group_fmt; /* HOST, K/group entries in {0,1} selecting fmt[] per group; NULL = all fmt[0]
                               (must be NULL for the hybrid word, whose two codes share every word) */
  const void *codes;        /* DEVICE, packed codes in device order (ccq_pack_codes)   */
  const void *scales;       /* DEVICE.  scale_mode 0: fp16 group scales in device order (ccq_pack_scales).
                               scale_mode 1: the packed 4-bit scale fields s_q of the narrow-format
                               groups in device order (ccq_pack_scales4); may be NULL when there are
                               no narrow-format groups (a wide-format group carries its field in the
                               spare low nibble of its last code byte, a hybrid-word group in the low
                               13 bits of its last word, Sec. 3.4)                        */
  const float *code_alpha;  /* DEVICE, fp32[N]: Code Cluster scale s_code, >= 0        */
  const float *code_beta;   /* DEVICE, fp32[N]: Code Cluster zero-point zp_code, an
                               integer value >= 0 with round(255*alpha + beta) <= 2^15 - 1,
                               i.e. every byte expands to a 15-bit code (the kernels
                               rely on it; device data is not checked)                 */
  const void *meta;         /* DEVICE, group map in device order (ccq_pack_meta); may be NULL when group_fmt is NULL */
  int32_t scale_mode;       /* 0 = fp16 group scales; 1 = compressed scales of Sec. 3.4: group scale =
                               4-bit (hybrid word: 13-bit) field * scale_super[n] (first line of Alg. 2 / Alg. 3).  Mode 1 is
                               built in every entry point; the per-row-tile kernel then holds 16 rows at
                               a time whatever launch shape is asked for                              */
  const void *scale_super;  /* DEVICE, fp16[N]: per-output-channel super scale s_super (scale_mode 1) */
} ccq_weight;

/* Sizes of the device layout and the accounting of Eq. 5.  The device layout holds whole tiles of 16 output rows and
 * whole k-tiles (4 narrow-format groups, 8 wide-format or hybrid-word groups): any N >= 1, any K that is a multiple of
 * 64 and any group map are accepted, and what does not fill its last tile is padded by the ccq_pack_* routines with
 * zero codes and zero scales (padded weights decode to zeros and padded rows are never stored).  code_bytes,
 * scale_bytes and meta_bytes are the sizes of the device arrays, padding included; the bits-per-weight fields count
 * what the method stores (the canonical arrays). */
typedef struct {
  int64_t code_bytes;       /* bytes of the packed code stream in device order           */
  int64_t scale_bytes;      /* bytes of the `scales` array (fp16 scales, or packed 4-bit fields)      */
  int64_t meta_bytes;       /* bytes ccq_pack_meta writes                                */
  int64_t workspace_bytes;  /* workspace ccq_gemm may need for M <= M_max                */
  int64_t row_tile_bytes;   /* code bytes of one tile of 16 output rows (all of K)       */
  int32_t bytes_per_group[2]; /* code bytes per 64-weight group, per format (16 / 22)    */
  int32_t groups[2];        /* number of groups along K in each format                   */
  int32_t align;            /* required alignment of DEVICE pointers (16)                */
  double code_bpw;          /* code bits per weight: exactly 2.0 narrow, 2.75 wide       */
  double total_bpw;         /* + scales (+ super scales) + per-row alpha/beta                        */
  int64_t canonical_code_bytes; /* bytes of the canonical code array the pack routine reads (= code_bytes without padding) */
  int32_t padded_N;         /* rows of the device layout: N rounded up to a multiple of 16            */
  int32_t padded_groups[2]; /* groups of each format in the device layout (whole k-tiles)             */
} ccq_info;

/* Validate a descriptor (DEVICE pointers may be NULL here) and report the
 * layout sizes, the bits-per-weight accounting of Eq. 5 and the workspace
 * ccq_gemm needs for up to M_max activation rows.  Pure host code. */
int ccq_pack_info(const ccq_weight *w, int32_t M_max, ccq_info *out);

/* Host-side permutations from canonical order to device order.
 *   ccq_pack_codes : canonical_codes HOST uint8 [N][row bytes] (canonical_code_bytes in all) -> out HOST [code_bytes]
 *   ccq_pack_scales: canonical fp16 bits HOST [N][K/64]         -> out HOST [scale_bytes/2]  (scale_mode 0)
 *   ccq_pack_meta  : group_fmt                                  -> out HOST [meta_bytes]
 * Byte values are copied, never altered.  The caller uploads the results. */
int ccq_pack_codes(const ccq_weight *w, const uint8_t *canonical_codes, void *out);
int ccq_pack_scales(const ccq_weight *w, const uint16_t *canonical_scales, void *out);
int ccq_pack_meta(const ccq_weight *w, void *out);
/* scale_mode 1: canonical s_q HOST uint8 [N][ceil(narrow groups / 2)] (the p-th narrow-format group of a row,
 * in k order, in byte p/2 at s_shift = 4*(p%2), Alg. 3) -> out HOST [scale_bytes]. */
int ccq_pack_scales4(const ccq_weight *w, const uint8_t *canonical_sq, void *out);

/* y[m][n] = sum_k x[m][k] * W_dq[n][k]   (the W2A16 GEMV / GEMM of the
 * "Inference Performance" section; Alg. 2/3 fused into the contraction).
 *   x DEVICE bf16 [M][ldx], y DEVICE bf16 [M][ldy] (round to nearest even),
 *   fp32 accumulation.  ldx >= K, ldy >= N, in elements, multiples of 8; columns N.. of y are not written.
 *   The per-row arrays of the descriptor (code_alpha, code_beta, scale_super) hold N entries: no padding.
 *   M = 0 is a no-op.  workspace DEVICE, workspace_bytes >= the value
 *   ccq_pack_info reports for M_max >= M (may be NULL if that value is 0). */
int ccq_gemm(const ccq_weight *w, const void *x, int32_t M, int64_t ldx, void *y, int64_t ldy,
             void *workspace, int64_t workspace_bytes, void *hip_stream);

/* Workspace bytes ccq_gemm needs for exactly M rows (<= the ccq_pack_info figure for any M_max >= M);
 * -1 for an invalid descriptor.  Pure host code. */
int64_t ccq_gemm_workspace_bytes(const ccq_weight *w, int32_t M);

/* ccq_gemm for callers that cannot allocate device memory or bring a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results as ccq_gemm (bit for
 * bit), without the workspace: the fp32 partial tiles of the K shares live in a device array that belongs to the
 * library (ccq_gemm_static_max_workspace() bytes, 8 MiB, held on every GPU the library has run on until the
 * process ends).  A call that would need more (ccq_gemm_workspace_bytes(w, M) tells) returns CCQ_ERR_WORKSPACE and
 * enqueues nothing.  No hipMalloc, hipFree or other allocating call is made.  All calls on one GPU share the
 * array: calls that may overlap on one GPU (different streams, concurrent graph launches) race on it and
 * must be ordered by the caller; calls on one stream are ordered by the stream. */
int ccq_gemm_static(const ccq_weight *w, const void *x, int32_t M, int64_t ldx, void *y, int64_t ldy, void *hip_stream);
int64_t ccq_gemm_static_max_workspace(void);

/* Explicit launch shape for ccq_gemm_ex (0 = let the library choose).  */
typedef struct {
  int32_t rows_per_wave_tiles; /* 16-row tiles each wavefront owns: 1 or 2      */
  int32_t waves_rows;          /* wavefronts of a workgroup along the rows       */
  int32_t waves_k;             /* wavefronts of a workgroup along K (reduced in LDS) */
  int32_t splits_k;            /* workgroups along K (reduced through workspace) */
} ccq_launch;

/* ccq_gemm with a caller-chosen decomposition (tuning and tests). */
int ccq_gemm_ex(const ccq_weight *w, const void *x, int32_t M, int64_t ldx, void *y, int64_t ldy,
                void *workspace, int64_t workspace_bytes, void *hip_stream, const ccq_launch *launch);

/* Grouped GEMM for mixture-of-experts layers (the Grouped-GEMM operator of the
 * "Inference Performance" section).  All E experts share one shape and format:
 * `w0` describes expert 0 and expert e's DEVICE arrays start
 * e * {codes,scales,ab}_stride bytes after expert 0's (ab_stride for code_alpha
 * and code_beta; with scale_mode 1 it must be given, at least 4 N, also for
 * weights without Code Cluster, and expert e's scale_super starts e * ab_stride / 2
 * bytes after expert 0's: fp16 where alpha and beta are fp32).
 *   Output row p in [expert_offsets[e], expert_offsets[e+1]) is
 *       y[p][:] = x[sorted_rows[p]][:] * W_dq(e)^T.
 *   x DEVICE bf16 [T][ldx]; sorted_rows DEVICE int32 [P], values in [0,T);
 *   expert_offsets_dev DEVICE int32 [E+1] with [0] = 0, monotone, [E] = P;
 *   expert_offsets_host HOST copy of the same, or NULL: when given it is
 *   validated (CCQ_ERR_ROUTING) and shapes the launch -- it must equal the
 *   device array: experts it shows as empty may not be visited at all, and
 *   with at most one row per expert the one-row kernel runs, with more than
 *   32 rows on an expert the 64-row kernel; device data is
 *   never read back.  A call captured into a HIP graph that is replayed
 *   with other routings must pass NULL here: the launch recorded with a
 *   host copy is tied to that routing (its busy experts, their row counts);
 *   y DEVICE bf16 [P][ldy].  An expert with no rows writes nothing.
 *   The top-k combine and any activation function stay with the caller. */
int ccq_grouped_gemm(const ccq_weight *w0, int32_t E, int64_t codes_stride, int64_t scales_stride,
                     int64_t ab_stride, const void *x, int32_t T, int64_t ldx,
                     const int32_t *sorted_rows, int32_t P, const int32_t *expert_offsets_dev,
                     const int32_t *expert_offsets_host, void *y, int64_t ldy, void *workspace,
                     int64_t workspace_bytes, void *hip_stream);

/* Recommended workspace for P output rows (at most 64 MiB).  ccq_grouped_gemm works with any smaller
 * workspace, down to none: it only cuts K into fewer shares, which matters when few experts have rows
 * (pass expert_offsets_host so that the library can see that). */
int64_t ccq_grouped_workspace_bytes(const ccq_weight *w0, int32_t E, int32_t P);

/* The offline quantizer on the GPU: Alg. 1 (group scale absmax / (2^(L-1) - 1), nearest codeword of the
 * convolutional codebook for every N-vector, ties to the lowest code), the least-squares scale of Eq. 4
 * (kept when the group's squared error does not grow; the scale is then rounded to fp16 and the search run
 * again with the stored value), and for the narrow format the Code Cluster map of Sec. 3.3 / Eq. 1 per
 * output channel (beta = smallest 15-bit code of the row, alpha = (largest - smallest) / 255; every vector is
 * searched again over the 256 codes round(q alpha + beta), then Eq. 4 once more).  An all-zero group gets
 * scale 0.  With scale_mode 1 the scales are then compressed (Sec. 3.4): per output channel s_super =
 * fp16(largest group scale / 15), every group scale becomes the nearest multiple field * s_super with the
 * field in 1..15 (0 for an all-zero group), and every group's codes are searched once more with the scale
 * that is stored.  All decisions are taken in fp64.
 *   w: shape and format (any the multiply entry points accept: narrow, wide, a per-group mix, the hybrid
 *      word whose two codes are searched independently and whose field is 13 bits; either scale mode).  Of its
 *      DEVICE pointers only `meta` is read, and only for a per-group mix (ccq_pack_meta).
 *   W DEVICE fp32 [N][ldw], ldw >= K, a multiple of 4.
 *   codes_out DEVICE [code_bytes], scales_out DEVICE [scale_bytes] (sizes from ccq_pack_info), both in
 *   device order, padding included (written as zeros): what ccq_gemm reads (scale_mode 1: scales_out receives the packed fields of the narrow-format
 *   groups and may be NULL when there are none).  alpha_out, beta_out DEVICE fp32 [N], needed when there are
 *   narrow-format groups (may be NULL otherwise).  scale_super_out DEVICE fp16 [N], scale_mode 1 only.  workspace DEVICE, at least ccq_quantize_workspace_bytes(w) bytes (-1: not built).
 *   Enqueues on hip_stream and returns; nothing is allocated.  W must be finite (NaN or infinity in a
 *   group gives unspecified codes and scale for that group). */
int64_t ccq_quantize_workspace_bytes(const ccq_weight *w);
int ccq_quantize(const ccq_weight *w, const float *W, int64_t ldw, void *codes_out, void *scales_out,
                 float *alpha_out, float *beta_out, void *scale_super_out, void *workspace,
                 int64_t workspace_bytes, void *hip_stream);

/* Ceiling probes (measurement only; not on the hot path).  The "Inference Performance" section
 * calls the operator memory-bound; these two kernels show what the memory system and the matrix cores deliver
 * when nothing else is asked of them, so that a kernel's rate can be set against an achievable figure as well
 * as against the published peak.
 *   ccq_probe_stream_read: reads src DEVICE [bytes] (a multiple of 16) once with 16-byte nontemporal loads,
 *     loads_per_thread (1, 2, 4 or 8) requests in flight per thread, block_threads (a multiple of 64, at most
 *     512) threads per workgroup; sink DEVICE, at least 4 bytes (written with probability 2^-32 per thread).
 *   ccq_probe_mfma_bf16: `workgroups` workgroups of four wavefronts, each issuing iters x 4 independent
 *     32x32x16 bf16 MFMAs on operands DEVICE bf16 [8][64][8] (read once); sink DEVICE fp32 [workgroups * 256];
 *     *flop_out (HOST, may be NULL) receives the floating-point operations of the launch.
 * Both enqueue one kernel on hip_stream and return a ccq_status. */
int ccq_probe_stream_read(const void *src, int64_t bytes, int32_t loads_per_thread, int32_t block_threads, void *sink,
                          void *hip_stream);
int ccq_probe_mfma_bf16(const void *operands, int32_t workgroups, int32_t iters, void *sink, void *hip_stream, double *flop_out);

/* Human-readable name of a status code. */
const char *ccq_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* CCQ_H */
