/*
 * CCQ CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of Convolutional Code
 * Quantization (arXiv 2507.07145) used to check the GPU library.  Only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may load it;
 * the product path never does.  It shares no code, header, table or constant
 * with the HIP library.
 *
 * What is written out here, with the passage of the paper each part follows:
 *   cco_states            Sec. 3.1 "Definition of Convolutional Code Codebook"
 *                         (code -> N overlapping L-bit states), Table 1 shifts
 *   cco_bpw               Eq. 5 (equivalent bits per weight)
 *   cco_cluster_expand    Alg. 3, the round(q*s_code + zp_code) step; Eq. 1
 *   cco_decode            Alg. 2 / Alg. 3 weight part, group-wise, Sec. 3.1
 *                         "Group-wise Quantization" (zero-padded tail vector)
 *   cco_search_brute      Alg. 1, the argmin over all 2^T codebook rows
 *   cco_search_viterbi    the same argmin as a dynamic program over the state
 *                         graph of Fig. 1 (must return the identical code)
 *   cco_refit_scale       Eq. 4 (closed-form least-squares scale)
 *   cco_quantize          Alg. 1 + Sec. 3.3 Code Cluster + Sec. 3.4 scale step
 *   cco_h16_*             Sec. 3.2 "Hybrid Encoding": (3,3,2) and (3,4,2) side by side in
 *                         one 16-bit word, seven weights per word (Table 1 row 2)
 *   cco_expand_scales     Sec. 3.4 "Scale Compression": s = (4-bit field) * s_super,
 *                         first line of Alg. 2 and of Alg. 3
 *   cco_compress_scales   the encoder side of the same (channel-wise super scale)
 *   cco_matmul            y = x W^T in fp64 (the definition of the GEMM)
 *
 * Parity pins (tests/test_oracle_*.py): the (L=2,N=3,S=1) worked example of
 * Sec. 3.1, the bpw figures 2.66/2.28/2.75/2.5/2.0/2.06 printed in Sec. 3.1-3.4,
 * Table 1's shift lists, the S=L special case (plain packed RTN), closed forms
 * of the Code Cluster map, brute force vs dynamic program, numpy least squares
 * for Eq. 4.  Model-level accuracy (Tables 2-3) is parity unpinned: it needs
 * the paper's models and datasets.
 *
 * Canonical ("paper order") storage of a quantized matrix W[N_out][K]:
 *   row n = concatenation over groups g = 0..K/group-1 (k order) of the
 *   group's stored codes; code j of a group covers weights N*j .. N*j+N-1 of
 *   that group (Alg. 2/3: q_w = W_q[idx / p_w]).  A stored code is one byte
 *   when Code Cluster is on (the clustered 8-bit value), else ceil(T/8) bytes
 *   little-endian.  Scales are IEEE fp16 bit patterns [N_out][K/group].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define CCO_MAX_N 16 /* vector dimension (states per code) limit           */
#define CCO_MAX_L 8  /* state bits limit for the dynamic program's tables   */

typedef struct {
  int32_t L, N, S;      /* state bits, states per code, transition bits      */
  int32_t code_cluster; /* 1: stored value is the 8-bit clustered code       */
  double zp;            /* weight zero-point: value = (state - zp) * scale   */
} cco_code;

/* ---------- small number-format helpers (IEEE, written out) -------------- */

double cco_fp16_to_double(uint16_t h) {
  int sign = (h >> 15) & 1, e = (h >> 10) & 0x1F, m = h & 0x3FF;
  double v;
  if (e == 0) v = ldexp((double)m, -24);
  else if (e == 31) v = m ? NAN : INFINITY;
  else v = ldexp((double)(m | 0x400), e - 25);
  return sign ? -v : v;
}

double cco_bf16_to_double(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* round-to-nearest-even of a finite double to a p-bit-significand binary
 * format with minimum normal exponent emin (value = m * 2^e, |m| < 2^p). */
static double round_to_format(double x, int p, int emin, double maxfinite) {
  if (x == 0.0 || isnan(x) || isinf(x)) return x;
  int e;
  (void)frexp(fabs(x), &e); /* |x| = f * 2^e, f in [0.5,1) */
  int q = e - p;            /* quantum exponent so that |x|/2^q in [2^(p-1),2^p) */
  if (q < emin - (p - 1)) q = emin - (p - 1); /* subnormal range: fixed quantum */
  double scaled = ldexp(x, -q);
  double r = nearbyint(scaled); /* default rounding mode: nearest even */
  double y = ldexp(r, q);
  if (fabs(y) > maxfinite) return x > 0 ? INFINITY : -INFINITY;
  return y;
}

uint16_t cco_double_to_bf16(double x) {
  /* bfloat16: 8-bit significand, fp32 exponent range */
  double y = round_to_format(x, 8, -126, 3.3895313892515355e38);
  float f = (float)y; /* exact: y is representable */
  uint32_t u;
  memcpy(&u, &f, 4);
  return (uint16_t)(u >> 16);
}

uint16_t cco_double_to_fp16(double x) {
  double y = round_to_format(x, 11, -14, 65504.0);
  if (isnan(y)) return 0x7E00;
  uint16_t sign = signbit(y) ? 0x8000 : 0;
  double a = fabs(y);
  if (isinf(a)) return sign | 0x7C00;
  if (a == 0.0) return sign;
  int e;
  double f = frexp(a, &e); /* a = f*2^e, f in [0.5,1) -> 1.xxx * 2^(e-1) */
  int E = e - 1;
  if (E < -14) { /* subnormal: a = m * 2^-24 */
    return sign | (uint16_t)ldexp(a, 24);
  }
  uint16_t m = (uint16_t)(ldexp(f, 11)) & 0x3FF;
  return sign | (uint16_t)((E + 15) << 10) | m;
}

void cco_double_to_bf16_array(int64_t n, const double *in, uint16_t *out) {
  for (int64_t i = 0; i < n; ++i) out[i] = cco_double_to_bf16(in[i]);
}

void cco_fp16_to_double_array(int64_t n, const uint16_t *in, double *out) {
  for (int64_t i = 0; i < n; ++i) out[i] = cco_fp16_to_double(in[i]);
}

/* ---------- Sec. 3.1: code -> states ------------------------------------- */

int cco_T(int L, int N, int S) { return L + (N - 1) * S; }

/* State i of a code is the L-bit window that starts (N-1-i)*S bits above the
 * least significant bit: the first state sits in the most significant bits and
 * each following state re-uses the low L-S bits of its predecessor and appends
 * S fresh transition bits (the (2,3,1) example: states 00,01,10 <-> 0010). */
void cco_states(uint32_t code, int L, int N, int S, uint32_t *st) {
  uint32_t mask = (1u << L) - 1u;
  for (int i = 0; i < N; ++i) st[i] = (code >> ((N - 1 - i) * S)) & mask;
}

/* ---------- Eq. 5: equivalent bits per weight ---------------------------- */

/* T_store is the stored bits per code (T, or 8 under Code Cluster).  When the
 * group is not a multiple of N the last code's spare bits hold the scale and
 * nothing is added; otherwise scale_bits are added per group. */
double cco_bpw(int T_store, int g, int N, int scale_bits) {
  if (g % N != 0) return (double)T_store * (double)((g + N - 1) / N) / (double)g;
  return (double)T_store * (double)(g / N) / (double)g + (double)scale_bits / (double)g;
}

int cco_codes_per_group(int g, int N) { return (g + N - 1) / N; }

int cco_code_bytes(const cco_code *f) {
  if (f->code_cluster) return 1;
  return (cco_T(f->L, f->N, f->S) + 7) / 8;
}

int cco_group_bytes(const cco_code *f, int g) {
  return cco_codes_per_group(g, f->N) * cco_code_bytes(f);
}

/* ---------- Alg. 3 / Eq. 1: Code Cluster expansion ----------------------- */

/* c = round(q * alpha + beta), ties to even, evaluated in exact arithmetic:
 * alpha is split into a 24-bit integer times a power of two, beta must be a
 * non-negative integer.  Returns 0xFFFFFFFF for inputs outside that domain. */
uint32_t cco_cluster_expand(uint32_t q, float alpha, float beta) {
  if (!(alpha >= 0.0f) || !(beta >= 0.0f) || beta != floorf(beta) || beta > 1.0e9f || isinf(alpha))
    return 0xFFFFFFFFu;
  uint64_t B = (uint64_t)beta;
  if (alpha == 0.0f || q == 0) return (uint32_t)B;
  int e;
  float m = frexpf(alpha, &e);             /* alpha = m * 2^e, m in [0.5,1) */
  uint64_t A = (uint64_t)ldexpf(m, 24);    /* exact 24-bit integer          */
  int E = e - 24;                          /* alpha = A * 2^E               */
  uint64_t num = (uint64_t)q * A;          /* < 2^32                        */
  if (E >= 0) {
    if (E > 20) return 0xFFFFFFFFu;
    return (uint32_t)(B + (num << E));
  }
  int sh = -E;
  if (sh >= 40) return (uint32_t)B;        /* q*alpha < 2^-8: rounds to 0   */
  uint64_t whole = num >> sh, rem = num & ((1ull << sh) - 1ull), half = 1ull << (sh - 1);
  uint64_t c = B + whole;
  if (rem > half || (rem == half && (c & 1ull))) c += 1;
  return (uint32_t)c;
}

/* ---------- Alg. 2 / Alg. 3: group-wise decode --------------------------- */

static uint32_t load_code(const uint8_t *p, int nbytes) {
  uint32_t c = 0;
  for (int b = 0; b < nbytes; ++b) c |= (uint32_t)p[b] << (8 * b);
  return c;
}

static void store_code(uint8_t *p, int nbytes, uint32_t c) {
  for (int b = 0; b < nbytes; ++b) p[b] = (uint8_t)(c >> (8 * b));
}

/* Row stride in bytes of the canonical layout. */
int64_t cco_row_bytes(int K, int g, const cco_code fmt[2], const uint8_t *group_fmt) {
  int64_t total = 0;
  for (int gi = 0; gi < K / g; ++gi) total += cco_group_bytes(&fmt[group_fmt ? group_fmt[gi] : 0], g);
  return total;
}

/* Decode the whole matrix to fp64 with the group scales given as fp64:
 * W[n][k] = (state - zp) * scale[n][k/g].  group_fmt may be NULL. */
int cco_decode_f64scales(int K, int Nrows, int g, const cco_code fmt[2], const uint8_t *group_fmt,
                         const uint8_t *codes, const double *scales, const float *alpha,
                         const float *beta, double *W) {
  if (K <= 0 || Nrows <= 0 || g <= 0 || K % g != 0) return -2;
  int G = K / g;
  int64_t row_bytes = cco_row_bytes(K, g, fmt, group_fmt);
  int status = 0;
#pragma omp parallel for schedule(static)
  for (int n = 0; n < Nrows; ++n) {
    const uint8_t *p = codes + (int64_t)n * row_bytes;
    for (int gi = 0; gi < G; ++gi) {
      const cco_code *f = &fmt[group_fmt ? group_fmt[gi] : 0];
      int cb = cco_code_bytes(f), T = cco_T(f->L, f->N, f->S);
      double s = scales[(int64_t)n * G + gi];
      for (int idx = 0; idx < g; ++idx) {
        int j = idx / f->N, i = idx % f->N; /* Alg. 2/3: code index, shift index */
        uint32_t c = load_code(p + (int64_t)j * cb, cb);
        if (f->code_cluster) {
          c = cco_cluster_expand(c, alpha[n], beta[n]);
          if (c == 0xFFFFFFFFu || c >= (1u << T)) {
#pragma omp atomic write
            status = -3;
            c = 0;
          }
        } else {
          c &= (T >= 32) ? 0xFFFFFFFFu : ((1u << T) - 1u);
        }
        uint32_t st = (c >> ((f->N - 1 - i) * f->S)) & ((1u << f->L) - 1u);
        W[(int64_t)n * K + (int64_t)gi * g + idx] = ((double)st - f->zp) * s;
      }
      p += cco_group_bytes(f, g);
    }
  }
  return status;
}

/* The same with fp16 group scales.  The value is exact (a <=7-bit integer or
 * half-integer times an 11-bit significand), so no rounding mode is involved. */
int cco_decode(int K, int Nrows, int g, const cco_code fmt[2], const uint8_t *group_fmt,
               const uint8_t *codes, const uint16_t *scales_fp16, const float *alpha,
               const float *beta, double *W) {
  if (K <= 0 || Nrows <= 0 || g <= 0 || K % g != 0) return -2;
  int64_t n = (int64_t)Nrows * (K / g);
  double *sc = (double *)malloc(sizeof(double) * (size_t)n);
  if (!sc) return -4;
  for (int64_t i = 0; i < n; ++i) sc[i] = cco_fp16_to_double(scales_fp16[i]);
  int rc = cco_decode_f64scales(K, Nrows, g, fmt, group_fmt, codes, sc, alpha, beta, W);
  free(sc);
  return rc;
}

/* ---------- Sec. 3.4 Scale Compression ----------------------------------- */

/* Spare low bits of a group's last stored code: when g is not a multiple of N
 * the last code carries only g mod N states, in its top bits. */
int cco_spare_bits(const cco_code *f, int g) {
  int r = g % f->N;
  if (r == 0 || f->code_cluster) return 0;
  return (f->N - r) * f->S;
}

/* Bytes of the packed 4-bit scale array s_q per row: one nibble for every group
 * that has no spare bits of its own. */
int64_t cco_sq_row_bytes(int K, int g, const cco_code fmt[2], const uint8_t *group_fmt) {
  int64_t cnt = 0;
  for (int gi = 0; gi < K / g; ++gi)
    if (cco_spare_bits(&fmt[group_fmt ? group_fmt[gi] : 0], g) < 4) ++cnt;
  return (cnt + 1) / 2;
}

/* scales[n][gi] = (4-bit field) * s_super[n]   (first line of Alg. 2 / Alg. 3;
 * s_mask = 0xF).  Exact: a 4-bit integer times an 11-bit significand. */
int cco_expand_scales(int K, int Nrows, int g, const cco_code fmt[2], const uint8_t *group_fmt,
                      const uint8_t *codes, const uint8_t *sq_packed, const uint16_t *s_super_fp16,
                      double *scales) {
  if (K <= 0 || Nrows <= 0 || g <= 0 || K % g != 0) return -2;
  int G = K / g;
  int64_t row_bytes = cco_row_bytes(K, g, fmt, group_fmt);
  int64_t sq_bytes = cco_sq_row_bytes(K, g, fmt, group_fmt);
  for (int n = 0; n < Nrows; ++n) {
    const uint8_t *p = codes + (int64_t)n * row_bytes;
    double ssup = cco_fp16_to_double(s_super_fp16[n]);
    int64_t pidx = 0; /* index among the groups that use s_q */
    for (int gi = 0; gi < G; ++gi) {
      const cco_code *f = &fmt[group_fmt ? group_fmt[gi] : 0];
      int gb = cco_group_bytes(f, g);
      uint32_t field;
      if (cco_spare_bits(f, g) >= 4) {
        field = p[gb - 1] & 0xFu; /* Alg. 2: s_uint = the last value of W_q, s_mask = 0xF */
      } else {
        uint32_t sq = sq_packed[(int64_t)n * sq_bytes + pidx / 2];
        field = (sq >> (4 * (pidx % 2))) & 0xFu; /* Alg. 3: (s_q >> s_shift) & s_mask */
        ++pidx;
      }
      scales[(int64_t)n * G + gi] = (double)field * ssup;
      p += gb;
    }
  }
  return 0;
}

/* ---------- the GEMM definition ------------------------------------------ */

/* Y[m][n] = sum_k x[m][k] * W[n][k]; x is bf16 bits, everything in fp64. */
void cco_matmul(int M, int K, int Nrows, const uint16_t *x_bf16, int64_t ldx, const double *W,
                double *Y) {
  double *xd = (double *)malloc(sizeof(double) * (size_t)M * (size_t)K);
  for (int m = 0; m < M; ++m)
    for (int k = 0; k < K; ++k) xd[(int64_t)m * K + k] = cco_bf16_to_double(x_bf16[(int64_t)m * ldx + k]);
#pragma omp parallel for schedule(static)
  for (int n = 0; n < Nrows; ++n) {
    const double *w = W + (int64_t)n * K;
    for (int m = 0; m < M; ++m) {
      const double *xr = xd + (int64_t)m * K;
      double acc = 0.0;
      for (int k = 0; k < K; ++k) acc += xr[k] * w[k];
      Y[(int64_t)m * Nrows + n] = acc;
    }
  }
  free(xd);
}

int cco_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---------- Alg. 1: code search ------------------------------------------ */

static inline double sqerr(double v, double s, double zp, uint32_t st) {
  double d = v - s * ((double)st - zp);
  return d * d;
}

/* Exhaustive argmin over all 2^T codes; squared errors are added left to
 * right; ties go to the lowest code.  v has N entries (zero padded). */
uint32_t cco_search_brute(const double *v, double s, double zp, int L, int N, int S) {
  int T = cco_T(L, N, S);
  uint32_t best = 0, st[CCO_MAX_N];
  double bestc = INFINITY;
  for (uint32_t c = 0; c < (1u << T); ++c) {
    cco_states(c, L, N, S, st);
    double cost = sqerr(v[0], s, zp, st[0]);
    for (int i = 1; i < N; ++i) cost = cost + sqerr(v[i], s, zp, st[i]);
    if (cost < bestc) { bestc = cost; best = c; }
  }
  return best;
}

/* The same argmin as a shortest path through the state graph: a path's code
 * is its first state followed by the transition bits, so comparing code
 * prefixes numerically reproduces the lowest-code tie rule. */
uint32_t cco_search_viterbi(const double *v, double s, double zp, int L, int N, int S) {
  enum { MAXST = 1 << CCO_MAX_L };
  int ns = 1 << L, nt = 1 << S;
  uint32_t mask = (uint32_t)ns - 1u;
  double cost[MAXST], ncost[MAXST];
  uint32_t pre[MAXST], npre[MAXST];
  for (int st = 0; st < ns; ++st) { cost[st] = sqerr(v[0], s, zp, (uint32_t)st); pre[st] = (uint32_t)st; }
  for (int i = 1; i < N; ++i) {
    for (int st = 0; st < ns; ++st) { ncost[st] = INFINITY; npre[st] = 0xFFFFFFFFu; }
    for (int p = 0; p < ns; ++p) {
      for (int t = 0; t < nt; ++t) {
        uint32_t nx = (((uint32_t)p << S) | (uint32_t)t) & mask;
        double c = cost[p] + sqerr(v[i], s, zp, nx);
        uint32_t code = (pre[p] << S) | (uint32_t)t;
        if (c < ncost[nx] || (c == ncost[nx] && code < npre[nx])) { ncost[nx] = c; npre[nx] = code; }
      }
    }
    memcpy(cost, ncost, sizeof(double) * (size_t)ns);
    memcpy(pre, npre, sizeof(uint32_t) * (size_t)ns);
  }
  uint32_t best = 0xFFFFFFFFu;
  double bestc = INFINITY;
  for (int st = 0; st < ns; ++st)
    if (cost[st] < bestc || (cost[st] == bestc && pre[st] < best)) { bestc = cost[st]; best = pre[st]; }
  return best;
}

/* ---------- Eq. 4: least-squares scale ----------------------------------- */

/* S = sum(W * Wq) / sum(Wq^2) over the g real weights of a group, Wq being
 * the decoded integer-domain values (state - zp).  Returns fallback when the
 * denominator is zero. */
double cco_refit_scale(const double *w, const double *wq, int g, double fallback) {
  double num = 0.0, den = 0.0;
  for (int i = 0; i < g; ++i) { num += w[i] * wq[i]; den += wq[i] * wq[i]; }
  return den > 0.0 ? num / den : fallback;
}

static double group_error(const double *w, const double *wq, int g, double s) {
  double e = 0.0;
  for (int i = 0; i < g; ++i) { double d = w[i] - wq[i] * s; e += d * d; }
  return e;
}

/* decoded integer-domain values of one group from its (unclustered) codes */
static void group_wq(const uint32_t *codes, const cco_code *f, int g, double *wq) {
  uint32_t st[CCO_MAX_N];
  for (int idx = 0; idx < g; ++idx) {
    cco_states(codes[idx / f->N], f->L, f->N, f->S, st);
    wq[idx] = (double)st[idx % f->N] - f->zp;
  }
}

static void search_group(const double *w, int g, const cco_code *f, double s, int method, uint32_t *codes) {
  int cpg = cco_codes_per_group(g, f->N);
  double v[CCO_MAX_N];
  for (int j = 0; j < cpg; ++j) {
    for (int i = 0; i < f->N; ++i) { int idx = j * f->N + i; v[i] = idx < g ? w[idx] : 0.0; }
    codes[j] = method == 0 ? cco_search_brute(v, s, f->zp, f->L, f->N, f->S)
                           : cco_search_viterbi(v, s, f->zp, f->L, f->N, f->S);
  }
}

static double fp16_scale(double s) {
  uint16_t h = cco_double_to_fp16(s);
  double r = cco_fp16_to_double(h);
  if (!(r > 0.0) || isinf(r)) r = cco_fp16_to_double(0x0400); /* smallest normal */
  return r;
}

/* ---------- Alg. 1 + Sec. 3.3 + Sec. 3.4: the offline quantizer ---------- */

/* Quantize W (fp32 [Nrows][K]) into the canonical layout.
 *   method 0 = exhaustive search, 1 = dynamic program (identical results).
 *   cluster_research 1 = after Eq. 1 re-search each vector over the 256
 *   reachable clustered codes (never worse than plain Eq. 1 rounding);
 *   0 = plain Eq. 1 rounding of the unconstrained codes.
 * Outputs: codes (row stride cco_row_bytes), scales fp16 [Nrows][K/g],
 * alpha/beta [Nrows] (written only when a format uses Code Cluster).
 * Steps per group (an all-zero group just gets scale 0): scale =
 * absmax/(2^(L-1)-1); search; Eq. 4 refit (kept when
 * the error does not grow); scale rounded to fp16; search again with the
 * stored scale.  Per row with Code Cluster: beta = min code, alpha =
 * (max-min)/255, q = round((c-beta)/alpha) (Eq. 1), optional re-search, then
 * one more Eq. 4 refit with the final codes. */
int cco_quantize(int K, int Nrows, int g, const cco_code fmt[2], const uint8_t *group_fmt,
                 const float *W, int method, int cluster_research, uint8_t *codes,
                 uint16_t *scales_fp16, float *alpha, float *beta) {
  if (K <= 0 || Nrows <= 0 || g <= 0 || K % g != 0) return -2;
  for (int t = 0; t < 2; ++t) {
    const cco_code *f = &fmt[t];
    if (f->L < 1 || f->L > CCO_MAX_L || f->N < 1 || f->N > CCO_MAX_N || f->S < 1 || f->S > f->L) return -2;
    if (cco_T(f->L, f->N, f->S) > 24) return -2;
    if (f->code_cluster && g % f->N != 0) return -2;
    if (!group_fmt) break;
  }
  int G = K / g;
  int64_t row_bytes = cco_row_bytes(K, g, fmt, group_fmt);
  int maxcpg = g; /* N >= 1 */
#pragma omp parallel
  {
    uint32_t *rowcodes = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)G * (size_t)maxcpg);
    double *rowscale = (double *)malloc(sizeof(double) * (size_t)G);
    double *w = (double *)malloc(sizeof(double) * (size_t)g);
    double *wq = (double *)malloc(sizeof(double) * (size_t)g);
    uint32_t(*reach)[CCO_MAX_N] = malloc(sizeof(uint32_t[CCO_MAX_N]) * 256);
#pragma omp for schedule(dynamic, 4)
    for (int n = 0; n < Nrows; ++n) {
      /* pass 1: unconstrained codes and fp16 scales for every group */
      for (int gi = 0; gi < G; ++gi) {
        const cco_code *f = &fmt[group_fmt ? group_fmt[gi] : 0];
        uint32_t *gc = rowcodes + (size_t)gi * (size_t)maxcpg;
        double amax = 0.0;
        for (int i = 0; i < g; ++i) {
          w[i] = (double)W[(int64_t)n * K + (int64_t)gi * g + i];
          if (fabs(w[i]) > amax) amax = fabs(w[i]);
        }
        if (amax == 0.0) { /* an all-zero group: scale 0 reproduces it exactly whatever the codes (Alg. 1 is silent here) */
          for (int j = 0; j < cco_codes_per_group(g, f->N); ++j) gc[j] = 0;
          rowscale[gi] = 0.0;
          continue;
        }
        double qmax = (double)((1 << (f->L - 1)) - 1);
        if (qmax < 1.0) qmax = 1.0;
        double s0 = amax / qmax;
        search_group(w, g, f, s0, method, gc);
        group_wq(gc, f, g, wq);
        double s1 = cco_refit_scale(w, wq, g, s0);
        if (!(s1 > 0.0) || group_error(w, wq, g, s1) > group_error(w, wq, g, s0)) s1 = s0;
        double s = fp16_scale(s1);
        search_group(w, g, f, s, method, gc);
        rowscale[gi] = s;
      }
      /* pass 2: Code Cluster along the output channel (Sec. 3.3, Eq. 1) */
      int any_cluster = 0;
      uint32_t cmin = 0xFFFFFFFFu, cmax = 0;
      for (int gi = 0; gi < G; ++gi) {
        const cco_code *f = &fmt[group_fmt ? group_fmt[gi] : 0];
        if (!f->code_cluster) continue;
        any_cluster = 1;
        int cpg = cco_codes_per_group(g, f->N);
        for (int j = 0; j < cpg; ++j) {
          uint32_t c = rowcodes[(size_t)gi * (size_t)maxcpg + (size_t)j];
          if (c < cmin) cmin = c;
          if (c > cmax) cmax = c;
        }
      }
      float a = 1.0f, b = 0.0f;
      if (any_cluster) {
        b = (float)cmin;
        a = cmax > cmin ? (float)((double)(cmax - cmin) / 255.0) : 1.0f;
        alpha[n] = a;
        beta[n] = b;
      }
      /* pass 3: emit bytes */
      uint8_t *p = codes + (int64_t)n * row_bytes;
      for (int gi = 0; gi < G; ++gi) {
        const cco_code *f = &fmt[group_fmt ? group_fmt[gi] : 0];
        uint32_t *gc = rowcodes + (size_t)gi * (size_t)maxcpg;
        int cpg = cco_codes_per_group(g, f->N), cb = cco_code_bytes(f);
        double s = rowscale[gi];
        if (f->code_cluster) {
          for (int i = 0; i < g; ++i) w[i] = (double)W[(int64_t)n * K + (int64_t)gi * g + i];
          for (int q = 0; q < 256; ++q) cco_states(cco_cluster_expand((uint32_t)q, a, b), f->L, f->N, f->S, reach[q]);
          for (int j = 0; j < cpg; ++j) {
            double qr = nearbyint(((double)gc[j] - (double)b) / (double)a); /* Eq. 1 */
            int q0 = qr < 0.0 ? 0 : (qr > 255.0 ? 255 : (int)qr);
            int qbest = q0;
            if (cluster_research) {
              double bestc = INFINITY;
              for (int q = 0; q < 256; ++q) {
                double cost = sqerr(w[j * f->N], s, f->zp, reach[q][0]);
                for (int i = 1; i < f->N; ++i) cost = cost + sqerr(w[j * f->N + i], s, f->zp, reach[q][i]);
                if (cost < bestc) { bestc = cost; qbest = q; }
              }
            }
            p[j] = (uint8_t)qbest;
            for (int i = 0; i < f->N; ++i) wq[j * f->N + i] = (double)reach[qbest][i] - f->zp;
          }
          double s2 = cco_refit_scale(w, wq, g, s);
          double s2h = s2 > 0.0 ? fp16_scale(s2) : s;
          if (group_error(w, wq, g, s2h) <= group_error(w, wq, g, s)) s = s2h;
        } else {
          for (int j = 0; j < cpg; ++j) store_code(p + (int64_t)j * cb, cb, gc[j]);
        }
        scales_fp16[(int64_t)n * G + gi] = cco_double_to_fp16(s);
        p += cco_group_bytes(f, g);
      }
    }
    free(rowcodes); free(rowscale); free(w); free(wq); free(reach);
  }
  return 0;
}

/* Sec. 3.4 Scale Compression, encoder side.  Input: a matrix already quantized
 * by cco_quantize (codes, fp16 group scales, alpha/beta).  Per row: super scale
 * = fp16(max group scale / 15); every group scale becomes the nearest multiple
 * k * s_super, k in 1..15 (0 only for an all-zero group); because the scale that
 * is stored has changed, the codes of every group are searched again with it
 * (over all codes, or over the 256 reachable ones under the row's Code Cluster
 * map).  The 4-bit fields go to the spare nibble of the group's last byte or to
 * sq_packed (see cco_expand_scales). */
int cco_compress_scales(int K, int Nrows, int g, const cco_code fmt[2], const uint8_t *group_fmt,
                        const float *W, int method, uint8_t *codes, const uint16_t *scales_fp16,
                        const float *alpha, const float *beta, uint8_t *sq_packed,
                        uint16_t *s_super_fp16) {
  if (K <= 0 || Nrows <= 0 || g <= 0 || K % g != 0) return -2;
  int G = K / g;
  int64_t row_bytes = cco_row_bytes(K, g, fmt, group_fmt);
  int64_t sq_bytes = cco_sq_row_bytes(K, g, fmt, group_fmt);
  memset(sq_packed, 0, (size_t)(sq_bytes * Nrows));
#pragma omp parallel
  {
    double *w = (double *)malloc(sizeof(double) * (size_t)g);
    uint32_t *gc = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)g);
    uint32_t(*reach)[CCO_MAX_N] = malloc(sizeof(uint32_t[CCO_MAX_N]) * 256);
#pragma omp for schedule(dynamic, 4)
    for (int n = 0; n < Nrows; ++n) {
      double smax = 0.0;
      for (int gi = 0; gi < G; ++gi) {
        double s = cco_fp16_to_double(scales_fp16[(int64_t)n * G + gi]);
        if (s > smax) smax = s;
      }
      uint16_t sup_bits = cco_double_to_fp16(smax / 15.0);
      double ssup = cco_fp16_to_double(sup_bits);
      s_super_fp16[n] = sup_bits;
      uint8_t *p = codes + (int64_t)n * row_bytes;
      int64_t pidx = 0;
      for (int gi = 0; gi < G; ++gi) {
        const cco_code *f = &fmt[group_fmt ? group_fmt[gi] : 0];
        int gb = cco_group_bytes(f, g), cb = cco_code_bytes(f), cpg = cco_codes_per_group(g, f->N);
        double s = cco_fp16_to_double(scales_fp16[(int64_t)n * G + gi]);
        int k = 0;
        if (ssup > 0.0 && s > 0.0) {
          double kr = nearbyint(s / ssup);
          k = kr < 1.0 ? 1 : (kr > 15.0 ? 15 : (int)kr);
        }
        double se = (double)k * ssup; /* the scale the decoder will use */
        for (int i = 0; i < g; ++i) w[i] = (double)W[(int64_t)n * K + (int64_t)gi * g + i];
        if (se > 0.0) {
          if (f->code_cluster) {
            for (int q = 0; q < 256; ++q) cco_states(cco_cluster_expand((uint32_t)q, alpha[n], beta[n]), f->L, f->N, f->S, reach[q]);
            for (int j = 0; j < cpg; ++j) {
              double bestc = INFINITY;
              int qbest = 0;
              for (int q = 0; q < 256; ++q) {
                double cost = sqerr(w[j * f->N], se, f->zp, reach[q][0]);
                for (int i = 1; i < f->N; ++i) cost = cost + sqerr(w[j * f->N + i], se, f->zp, reach[q][i]);
                if (cost < bestc) { bestc = cost; qbest = q; }
              }
              p[j] = (uint8_t)qbest;
            }
          } else {
            search_group(w, g, f, se, method, gc);
            for (int j = 0; j < cpg; ++j) store_code(p + (int64_t)j * cb, cb, gc[j]);
          }
        }
        if (cco_spare_bits(f, g) >= 4) {
          p[gb - 1] = (uint8_t)((p[gb - 1] & 0xF0u) | (uint32_t)k);
        } else {
          sq_packed[(int64_t)n * sq_bytes + pidx / 2] |= (uint8_t)(k << (4 * (pidx % 2)));
          ++pidx;
        }
        p += gb;
      }
    }
    free(w); free(gc); free(reach);
  }
  return 0;
}

/* ---------- Sec. 3.2 Hybrid Encoding: the 16-bit word ---------------------- */

/* One little-endian uint16 holds a (L=3,N=3,S=2) code in its top 7 bits and a
 * (L=3,N=4,S=2) code in its low 9 bits: seven 3-bit states.  Written out from
 * the two code definitions; Table 1's shift list [13,11,9,6,4,2,0] with mask
 * 0x7 is what this must reproduce (pinned in the tests). */
void cco_h16_states(uint32_t word, uint32_t st[7]) {
  cco_states((word >> 9) & 0x7Fu, 3, 3, 2, st);
  cco_states(word & 0x1FFu, 3, 4, 2, st + 3);
}

int cco_h16_words_per_group(int g) { return (g + 6) / 7; }

/* W[n][k] = (state - zp) * scale[n][k/g], fp16 group scales.  A group stores
 * ceil(g/7) words; the last word of a 64-weight group carries weight 63 in its
 * first state and 13 spare bits (Sec. 3.4), which are ignored here. */
int cco_h16_decode(int K, int Nrows, int g, double zp, const uint8_t *codes, const uint16_t *scales_fp16, double *W) {
  if (K <= 0 || Nrows <= 0 || g <= 0 || K % g != 0) return -2;
  int G = K / g, wpg = cco_h16_words_per_group(g);
#pragma omp parallel for schedule(static)
  for (int n = 0; n < Nrows; ++n) {
    const uint8_t *p = codes + (int64_t)n * G * wpg * 2;
    for (int gi = 0; gi < G; ++gi) {
      double s = cco_fp16_to_double(scales_fp16[(int64_t)n * G + gi]);
      for (int idx = 0; idx < g; ++idx) {
        uint32_t st[7];
        cco_h16_states(load_code(p + (int64_t)(idx / 7) * 2, 2), st); /* Alg. 2: q_w = W_q[idx / p_w], p_w = 7 */
        W[(int64_t)n * K + (int64_t)gi * g + idx] = ((double)st[idx % 7] - zp) * s;
      }
      p += wpg * 2;
    }
  }
  return 0;
}

/* Alg. 1 for the hybrid word: the two codes of a word are searched independently
 * (their bits do not overlap), group scale as in cco_quantize:
 * absmax/(2^(L-1)-1), search, Eq. 4 refit kept when the error does not grow,
 * fp16 rounding, search again with the stored scale.  method as in cco_quantize. */
int cco_h16_quantize(int K, int Nrows, int g, double zp, const float *W, int method, uint8_t *codes, uint16_t *scales_fp16) {
  if (K <= 0 || Nrows <= 0 || g <= 0 || K % g != 0) return -2;
  int G = K / g, wpg = cco_h16_words_per_group(g);
#pragma omp parallel
  {
    double *w = (double *)malloc(sizeof(double) * (size_t)(wpg * 7));
    double *wq = (double *)malloc(sizeof(double) * (size_t)(wpg * 7));
    uint32_t *words = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)wpg);
#pragma omp for schedule(dynamic, 4)
    for (int n = 0; n < Nrows; ++n) {
      for (int gi = 0; gi < G; ++gi) {
        double amax = 0.0;
        for (int i = 0; i < wpg * 7; ++i) {
          w[i] = i < g ? (double)W[(int64_t)n * K + (int64_t)gi * g + i] : 0.0; /* zero-padded tail (Sec. 3.1) */
          if (fabs(w[i]) > amax) amax = fabs(w[i]);
        }
        double s = 0.0;
        for (int j = 0; j < wpg; ++j) words[j] = 0;
        if (amax > 0.0) {
          double s0 = amax / 3.0; /* 2^(L-1) - 1 with L = 3 */
          for (int pass = 0; pass < 2; ++pass) {
            double sc = pass == 0 ? s0 : s;
            for (int j = 0; j < wpg; ++j) {
              uint32_t a = method == 0 ? cco_search_brute(w + 7 * j, sc, zp, 3, 3, 2) : cco_search_viterbi(w + 7 * j, sc, zp, 3, 3, 2);
              uint32_t b = method == 0 ? cco_search_brute(w + 7 * j + 3, sc, zp, 3, 4, 2) : cco_search_viterbi(w + 7 * j + 3, sc, zp, 3, 4, 2);
              words[j] = (a << 9) | b;
            }
            if (pass == 0) {
              for (int j = 0; j < wpg; ++j) {
                uint32_t st[7];
                cco_h16_states(words[j], st);
                for (int i = 0; i < 7; ++i) wq[7 * j + i] = (double)st[i] - zp;
              }
              double s1 = cco_refit_scale(w, wq, g, s0);
              if (!(s1 > 0.0) || group_error(w, wq, g, s1) > group_error(w, wq, g, s0)) s1 = s0;
              s = fp16_scale(s1);
            }
          }
        }
        uint8_t *p = codes + ((int64_t)n * G + gi) * wpg * 2;
        for (int j = 0; j < wpg; ++j) store_code(p + 2 * j, 2, words[j]);
        scales_fp16[(int64_t)n * G + gi] = cco_double_to_fp16(s);
      }
    }
    free(w); free(wq); free(words);
  }
  return 0;
}

/* ---------- Sec. 3.4 on the hybrid word: the 13 spare bits hold the scale --- */

/* Alg. 2, first lines, with Table 1's scale mask 0x1FFF: s_uint is the group's
 * last word, s = (s_uint & 0x1FFF) * s_super[n].  Needs a full last word, i.e.
 * g = 64 (g mod 7 = 1: the last word carries one weight and 13 spare bits). */
int cco_h16_expand_scales(int K, int Nrows, int g, const uint8_t *codes, const uint16_t *s_super_fp16, double *scales) {
  if (K <= 0 || Nrows <= 0 || g <= 0 || K % g != 0 || g % 7 != 1) return -2;
  int G = K / g, wpg = cco_h16_words_per_group(g);
  for (int n = 0; n < Nrows; ++n) {
    double ssup = cco_fp16_to_double(s_super_fp16[n]);
    for (int gi = 0; gi < G; ++gi) {
      uint32_t s_uint = load_code(codes + (((int64_t)n * G + gi) * wpg + (wpg - 1)) * 2, 2);
      scales[(int64_t)n * G + gi] = (double)(s_uint & 0x1FFFu) * ssup;
    }
  }
  return 0;
}

int cco_h16_decode_cs(int K, int Nrows, int g, double zp, const uint8_t *codes, const uint16_t *s_super_fp16, double *W) {
  if (K <= 0 || Nrows <= 0 || g <= 0 || K % g != 0 || g % 7 != 1) return -2;
  int G = K / g, wpg = cco_h16_words_per_group(g);
  double *sc = (double *)malloc(sizeof(double) * (size_t)Nrows * (size_t)G);
  int rc = cco_h16_expand_scales(K, Nrows, g, codes, s_super_fp16, sc);
  if (rc == 0) {
#pragma omp parallel for schedule(static)
    for (int n = 0; n < Nrows; ++n)
      for (int gi = 0; gi < G; ++gi)
        for (int idx = 0; idx < g; ++idx) {
          uint32_t st[7];
          cco_h16_states(load_code(codes + (((int64_t)n * G + gi) * wpg + idx / 7) * 2, 2), st);
          W[(int64_t)n * K + (int64_t)gi * g + idx] = ((double)st[idx % 7] - zp) * sc[(int64_t)n * G + gi];
        }
  }
  free(sc);
  return rc;
}

/* Encoder side: channel-wise super scale = largest group scale of the row / 8191
 * (fp16), field = nearest multiple clipped to 1..8191 (0 for an all-zero group),
 * codes searched again with the scale the decoder will use, field written into
 * the low 13 bits of the group's last word. */
int cco_h16_compress_scales(int K, int Nrows, int g, double zp, const float *W, int method, uint8_t *codes,
                            const uint16_t *scales_fp16, uint16_t *s_super_fp16) {
  if (K <= 0 || Nrows <= 0 || g <= 0 || K % g != 0 || g % 7 != 1) return -2;
  int G = K / g, wpg = cco_h16_words_per_group(g);
#pragma omp parallel
  {
    double *w = (double *)malloc(sizeof(double) * (size_t)(wpg * 7));
#pragma omp for schedule(dynamic, 4)
    for (int n = 0; n < Nrows; ++n) {
      double smax = 0.0;
      for (int gi = 0; gi < G; ++gi) {
        double s = cco_fp16_to_double(scales_fp16[(int64_t)n * G + gi]);
        if (s > smax) smax = s;
      }
      uint16_t sup_bits = cco_double_to_fp16(smax / 8191.0);
      double ssup = cco_fp16_to_double(sup_bits);
      s_super_fp16[n] = sup_bits;
      for (int gi = 0; gi < G; ++gi) {
        uint8_t *p = codes + ((int64_t)n * G + gi) * wpg * 2;
        double s = cco_fp16_to_double(scales_fp16[(int64_t)n * G + gi]);
        int k = 0;
        if (ssup > 0.0 && s > 0.0) {
          double kr = nearbyint(s / ssup);
          k = kr < 1.0 ? 1 : (kr > 8191.0 ? 8191 : (int)kr);
        }
        double se = (double)k * ssup;
        for (int i = 0; i < wpg * 7; ++i) w[i] = i < g ? (double)W[(int64_t)n * K + (int64_t)gi * g + i] : 0.0;
        for (int j = 0; j < wpg; ++j) {
          uint32_t word = load_code(p + 2 * j, 2);
          if (se > 0.0) {
            uint32_t a = method == 0 ? cco_search_brute(w + 7 * j, se, zp, 3, 3, 2) : cco_search_viterbi(w + 7 * j, se, zp, 3, 3, 2);
            uint32_t b = method == 0 ? cco_search_brute(w + 7 * j + 3, se, zp, 3, 4, 2) : cco_search_viterbi(w + 7 * j + 3, se, zp, 3, 4, 2);
            word = (a << 9) | b;
          }
          if (j == wpg - 1) word = (word & 0xE000u) | (uint32_t)k;
          store_code(p + 2 * j, 2, word);
        }
      }
    }
    free(w);
  }
  return 0;
}
