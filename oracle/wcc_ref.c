/*
 * wcc_ref.c -- plain CPU oracle for the Wavelet Compressed Convolution forward
 * path.  TEST INFRASTRUCTURE ONLY: nothing on the product path may link, load
 * or call this file; it shares no code with the HIP library.
 *
 * It follows the explicit WCC algorithm (appendix "Explicit WCC algorithm",
 * Alg. 1) step by step in fp64, with the symmetric signed quantiser of
 * Eq. (quantoperator)/(quantweights) inserted between the joint shrinkage and
 * the 1x1 convolution as the section "Joint hard shrinkage" describes.
 *
 * Readings taken where the paper is silent:
 *   - Haar step: the four 2x2 stride-2 kernels of Eq. (HaarKernel), factor 1/2,
 *     applied as a cross-correlation to the block [[a,b],[c,d]] (a top-left).
 *   - Coefficient order: the concatenation of Eq. (wavelet_transform)
 *     generalised to d levels:  [y1^d | y2^d | y3^d | y4^d | y2^(d-1) | ... | y4^1],
 *     each band row-major.  The position of a coefficient in this vector is its
 *     "linear index" q.
 *   - Channel norm: L1.  Ties: larger norm first, then lower q.
 *   - k = ceil(gamma * n_w * n_h) with gamma = num/den evaluated in integers.
 *   - Quantiser: signed, b = 8, so q_{b-1} has 2^(b-1)-1 = 127 levels a side;
 *     round = round-half-to-even.  The integer code is decided in fp32
 *     (u = c/alpha; clip; rint(127*u)), the precision the GPU library uses for
 *     that decision; everything else is fp64.
 *   - alpha: caller's value if > 0, else the largest kept |coefficient| of the
 *     whole call.
 *
 * Parity pins (tests/test_oracle_pins.py): orthonormality of the explicit
 * transform matrix, Parseval, perfect reconstruction, hand values of
 * Eq. (HaarKernel), keep-ratio-1 == direct 1x1 convolution, the commutation
 * identity of the section "Equivalence of the convolutions", brute-force top-k,
 * quantiser closed-form properties, the BOPs example of the appendix on bit
 * operations; the depthwise 3x3 convolution against a library correlation and shifted
 * impulses, the block of Eq. (inverted) at keep ratio 1 against its dense definition.  Numeric WCC outputs on the paper's datasets: parity unpinned
 * (the paper prints none).
 *
 * Loops marked with an OpenMP pragma run over independent outputs; the
 * arithmetic and its order inside one output element never depend on the
 * thread count.
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#if FLT_EVAL_METHOD != 0
#error "float expressions must be evaluated in float (the code decision is specified in fp32)"
#endif

int wcc_ref_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void wcc_ref_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* k = ceil(num * N / den): the size of the index set I of Alg. 1, gamma = num/den. */
int64_t wcc_ref_k(int64_t N, int64_t num, int64_t den) {
  return (num * N + den - 1) / den;
}

/* Offset of band j (0 = y1 .. 3 = y4) of level l inside the concatenated
 * vector of a d-level transform of an H x W plane.  y1 exists only for l = d. */
static int64_t band_offset(int64_t H, int64_t W, int l, int j) {
  int64_t nl = (H >> l) * (W >> l);
  return (int64_t)j * nl;
}

/* ---- Haar analysis, one plane (Eq. HaarKernel, Eq. wavelet_transform) ---- */
static void haar_fwd_plane(const double *x, int64_t H, int64_t W, int d, double *y,
                           double *ll /* scratch H*W */, double *nxt /* scratch H*W */) {
  memcpy(ll, x, sizeof(double) * (size_t)(H * W));
  int64_t h = H, w = W; /* size of the current low-pass image (row stride w) */
  for (int l = 1; l <= d; ++l) {
    int64_t h2 = h / 2, w2 = w / 2;
    double *y2 = y + band_offset(H, W, l, 1);
    double *y3 = y + band_offset(H, W, l, 2);
    double *y4 = y + band_offset(H, W, l, 3);
    for (int64_t r = 0; r < h2; ++r) {
      for (int64_t c = 0; c < w2; ++c) {
        double a = ll[(2 * r) * w + 2 * c], b = ll[(2 * r) * w + 2 * c + 1];
        double cc = ll[(2 * r + 1) * w + 2 * c], dd = ll[(2 * r + 1) * w + 2 * c + 1];
        nxt[r * w2 + c] = 0.5 * (a + b + cc + dd);
        y2[r * w2 + c] = 0.5 * (a - b + cc - dd);
        y3[r * w2 + c] = 0.5 * (a + b - cc - dd);
        y4[r * w2 + c] = 0.5 * (a - b - cc + dd);
      }
    }
    h = h2;
    w = w2;
    memcpy(ll, nxt, sizeof(double) * (size_t)(h * w));
  }
  memcpy(y, ll, sizeof(double) * (size_t)(h * w)); /* y1^d */
}

/* ---- Haar synthesis, one plane (transposed convolution, levels reversed) ---- */
static void haar_inv_plane(const double *y, int64_t H, int64_t W, int d,
                           double *x, double *ll /* scratch H*W */, double *tmp /* scratch H*W */) {
  int64_t h = H >> d, w = W >> d;
  memcpy(ll, y, sizeof(double) * (size_t)(h * w));
  for (int l = d; l >= 1; --l) {
    const double *y2 = y + band_offset(H, W, l, 1);
    const double *y3 = y + band_offset(H, W, l, 2);
    const double *y4 = y + band_offset(H, W, l, 3);
    int64_t w_out = 2 * w;
    for (int64_t r = 0; r < h; ++r) {
      for (int64_t c = 0; c < w; ++c) {
        double v1 = ll[r * w + c], v2 = y2[r * w + c], v3 = y3[r * w + c], v4 = y4[r * w + c];
        tmp[(2 * r) * w_out + 2 * c] = 0.5 * (v1 + v2 + v3 + v4);
        tmp[(2 * r) * w_out + 2 * c + 1] = 0.5 * (v1 - v2 + v3 - v4);
        tmp[(2 * r + 1) * w_out + 2 * c] = 0.5 * (v1 + v2 - v3 - v4);
        tmp[(2 * r + 1) * w_out + 2 * c + 1] = 0.5 * (v1 - v2 - v3 + v4);
      }
    }
    h *= 2;
    w *= 2;
    memcpy(ll, tmp, sizeof(double) * (size_t)(h * w));
  }
  memcpy(x, ll, sizeof(double) * (size_t)(H * W));
}

/* planes = B*C independent channels; x, y: [planes, H*W]. Returns 0 or -1. */
int wcc_ref_haar_fwd(const double *x, int64_t planes, int64_t H, int64_t W, int d, double *y) {
  if (d < 1 || H % (1 << d) || W % (1 << d)) return -1;
  int fail = 0;
#pragma omp parallel
  {
    double *ll = (double *)malloc(sizeof(double) * (size_t)(H * W));
    double *nxt = (double *)malloc(sizeof(double) * (size_t)(H * W));
    if (!ll || !nxt) {
#pragma omp atomic write
      fail = 1;
    }
#pragma omp for schedule(static)
    for (int64_t p = 0; p < planes; ++p)
      if (ll && nxt) haar_fwd_plane(x + p * H * W, H, W, d, y + p * H * W, ll, nxt);
    free(ll);
    free(nxt);
  }
  return fail ? -1 : 0;
}

int wcc_ref_haar_inv(const double *y, int64_t planes, int64_t H, int64_t W, int d, double *x) {
  if (d < 1 || H % (1 << d) || W % (1 << d)) return -1;
  int fail = 0;
#pragma omp parallel
  {
    double *ll = (double *)malloc(sizeof(double) * (size_t)(H * W));
    double *tmp = (double *)malloc(sizeof(double) * (size_t)(H * W));
    if (!ll || !tmp) {
#pragma omp atomic write
      fail = 1;
    }
#pragma omp for schedule(static)
    for (int64_t p = 0; p < planes; ++p)
      if (ll && tmp) haar_inv_plane(y + p * H * W, H, W, d, x + p * H * W, ll, tmp);
    free(ll);
    free(tmp);
  }
  return fail ? -1 : 0;
}

/* ---- channel norm (Alg. 1: one norm per position, taken over the channels) ---- */
/* coef [B, C, N] -> norm [B, N], L1, channels added in increasing order. */
void wcc_ref_channel_norm(const double *coef, int64_t B, int64_t C, int64_t N, double *norm) {
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < B; ++b) {
    double *s = norm + b * N;
    for (int64_t q = 0; q < N; ++q) s[q] = 0.0;
    for (int64_t c = 0; c < C; ++c) {
      const double *v = coef + (b * C + c) * N;
      for (int64_t q = 0; q < N; ++q) s[q] += fabs(v[q]);
    }
  }
}

/* The other common reading of the norm Alg. 1 leaves unnamed: Euclidean.  The square root is
 * left out (it does not change the order of non-negative numbers):
 * coef [B, C, N] -> norm [B, N] = sum_c coef^2, channels added in increasing order. */
void wcc_ref_channel_norm_sq(const double *coef, int64_t B, int64_t C, int64_t N, double *norm) {
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < B; ++b) {
    double *s = norm + b * N;
    for (int64_t q = 0; q < N; ++q) s[q] = 0.0;
    for (int64_t c = 0; c < C; ++c) {
      const double *v = coef + (b * C + c) * N;
      for (int64_t q = 0; q < N; ++q) s[q] += v[q] * v[q];
    }
  }
}

/* ---- joint top-k (Alg. 1: index set I) by a full sort ---- */
typedef struct {
  double s;
  int64_t q;
} keyed;

static int cmp_norm_desc_index_asc(const void *pa, const void *pb) {
  const keyed *a = (const keyed *)pa, *b = (const keyed *)pb;
  if (a->s > b->s) return -1;
  if (a->s < b->s) return 1;
  if (a->q < b->q) return -1;
  if (a->q > b->q) return 1;
  return 0;
}

static int cmp_i64(const void *pa, const void *pb) {
  int64_t a = *(const int64_t *)pa, b = *(const int64_t *)pb;
  return (a > b) - (a < b);
}

/* norm [B, N] -> idx [B, k], ascending per sample. Returns 0 or -1. */
int wcc_ref_topk(const double *norm, int64_t B, int64_t N, int64_t k, int64_t *idx) {
  if (k < 1 || k > N) return -1;
  int fail = 0;
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < B; ++b) {
    keyed *a = (keyed *)malloc(sizeof(keyed) * (size_t)N);
    if (!a) {
#pragma omp atomic write
      fail = 1;
      continue;
    }
    for (int64_t q = 0; q < N; ++q) {
      a[q].s = norm[b * N + q];
      a[q].q = q;
    }
    qsort(a, (size_t)N, sizeof(keyed), cmp_norm_desc_index_asc);
    for (int64_t j = 0; j < k; ++j) idx[b * k + j] = a[j].q;
    qsort(idx + b * k, (size_t)k, sizeof(int64_t), cmp_i64);
    free(a);
  }
  return fail ? -1 : 0;
}

/* ---- shrinkage T: xc[b,c,j] = coef[b,c,idx[b,j]] ---- */
void wcc_ref_gather(const double *coef, const int64_t *idx, int64_t B, int64_t C, int64_t N,
                    int64_t k, double *xc) {
#pragma omp parallel for schedule(static)
  for (int64_t p = 0; p < B * C; ++p) {
    int64_t b = p / C;
    for (int64_t j = 0; j < k; ++j) xc[p * k + j] = coef[p * N + idx[b * k + j]];
  }
}

/* ---- T^T: z[b,c,idx[b,j]] = yc[b,c,j], zero elsewhere ---- */
void wcc_ref_scatter(const double *yc, const int64_t *idx, int64_t B, int64_t C, int64_t N,
                     int64_t k, double *z) {
#pragma omp parallel for schedule(static)
  for (int64_t p = 0; p < B * C; ++p) {
    int64_t b = p / C;
    for (int64_t q = 0; q < N; ++q) z[p * N + q] = 0.0;
    for (int64_t j = 0; j < k; ++j) z[p * N + idx[b * k + j]] = yc[p * k + j];
  }
}

/* ---- signed uniform quantiser (Eq. quantoperator, Eq. quantweights) ---- */
/* Largest |v| over n values. */
double wcc_ref_absmax(const double *v, int64_t n) {
  double m = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    double a = fabs(v[i]);
    if (a > m) m = a;
  }
  return m;
}

/* codes[i] = round((2^(bits-1)-1) * clip(v[i]/alpha, -1, 1)), the integer inside
 * q_{b-1}; the quantised value is alpha * codes[i] / (2^(bits-1)-1).
 * The code is decided in fp32, operation by operation.  alpha == 0: all codes 0. */
void wcc_ref_quant_codes(const double *v, int64_t n, double alpha, int bits, double *codes) {
  const float levels = (float)((1 << (bits - 1)) - 1);
  const float a = (float)alpha;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    if (!(a > 0.0f)) {
      codes[i] = 0.0;
      continue;
    }
    float t = (float)v[i] / a;          /* scale */
    if (t > 1.0f) t = 1.0f;             /* clip  */
    if (t < -1.0f) t = -1.0f;
    float m = levels * t;
    codes[i] = (double)nearbyintf(m);   /* round (half to even) */
  }
}

/* ---- 1x1 convolution on the compressed signal:  y_i = sum_j k_ij x_j ---- */
/* w [C_out, C_in]; xc [B, C_in, k]; yc [B, C_out, k];
 * out_scale [C_out] multiplies row o of the result (NULL: 1). */
void wcc_ref_pointwise(const double *w, const double *out_scale, const double *xc, int64_t B,
                       int64_t C_in, int64_t C_out, int64_t k, double *yc) {
#pragma omp parallel for schedule(static)
  for (int64_t p = 0; p < B * C_out; ++p) {
    int64_t b = p / C_out, o = p % C_out;
    double *y = yc + p * k;
    for (int64_t j = 0; j < k; ++j) y[j] = 0.0;
    for (int64_t c = 0; c < C_in; ++c) {
      const double kij = w[o * C_in + c];
      const double *xv = xc + (b * C_in + c) * k;
      for (int64_t j = 0; j < k; ++j) y[j] += kij * xv[j];
    }
    if (out_scale)
      for (int64_t j = 0; j < k; ++j) y[j] *= out_scale[o];
  }
}

/* ---- the whole layer (Alg. 1 with the quantiser) ----
 * x [B,C_in,H,W]; w [C_out,C_in] (numbers the stored weights stand for);
 * w_scale [C_out] or NULL; act_bits 0 (none) or 2..16; alpha_in <= 0: max|kept c|.
 * Outputs: y [B,C_out,H,W]; idx_out [B,k] (nullable); alpha_out (nullable).
 * Returns 0, or -1 on bad arguments / out of memory. */
int wcc_ref_forward(const double *x, const double *w, const double *w_scale, int64_t B,
                    int64_t C_in, int64_t C_out, int64_t H, int64_t W, int d, int64_t keep_num,
                    int64_t keep_den, int act_bits, double alpha_in, double *y, int64_t *idx_out,
                    double *alpha_out) {
  const int64_t N = H * W, k = wcc_ref_k(N, keep_num, keep_den);
  if (d < 1 || H % (1 << d) || W % (1 << d) || k < 1 || k > N) return -1;
  int rc = -1;
  double *coef = (double *)malloc(sizeof(double) * (size_t)(B * C_in * N));
  double *norm = (double *)malloc(sizeof(double) * (size_t)(B * N));
  int64_t *idx = (int64_t *)malloc(sizeof(int64_t) * (size_t)(B * k));
  double *xc = (double *)malloc(sizeof(double) * (size_t)(B * C_in * k));
  double *yc = (double *)malloc(sizeof(double) * (size_t)(B * C_out * k));
  double *z = (double *)malloc(sizeof(double) * (size_t)(B * C_out * N));
  double *scale = (double *)malloc(sizeof(double) * (size_t)C_out);
  if (!coef || !norm || !idx || !xc || !yc || !z || !scale) goto done;

  if (wcc_ref_haar_fwd(x, B * C_in, H, W, d, coef)) goto done; /* X_wt            */
  wcc_ref_channel_norm(coef, B, C_in, N, norm);                 /* channel norms   */
  if (wcc_ref_topk(norm, B, N, k, idx)) goto done;              /* I               */
  wcc_ref_gather(coef, idx, B, C_in, N, k, xc);                 /* X_wt[I]         */
  double alpha = 0.0, sx = 1.0;
  if (act_bits > 0) {
    alpha = alpha_in > 0.0 ? alpha_in : wcc_ref_absmax(xc, B * C_in * k);
    /* alpha enters the code decision as an fp32 number */
    alpha = (double)(float)alpha;
    wcc_ref_quant_codes(xc, B * C_in * k, alpha, act_bits, xc); /* integer codes   */
    sx = alpha / (double)((1 << (act_bits - 1)) - 1);
  }
  for (int64_t o = 0; o < C_out; ++o) scale[o] = sx * (w_scale ? w_scale[o] : 1.0);
  wcc_ref_pointwise(w, scale, xc, B, C_in, C_out, k, yc);       /* Y_wt            */
  wcc_ref_scatter(yc, idx, B, C_out, N, k, z);                  /* Y^0[I] = Y_wt   */
  if (wcc_ref_haar_inv(z, B * C_out, H, W, d, y)) goto done;    /* inverse levels  */
  if (idx_out) memcpy(idx_out, idx, sizeof(int64_t) * (size_t)(B * k));
  if (alpha_out) *alpha_out = alpha;
  rc = 0;
done:
  free(coef); free(norm); free(idx); free(xc); free(yc); free(z); free(scale);
  return rc;
}

/* ---- depthwise 3x3 convolution: the K_dw of the inverted residual block (appendix
 * "Inference times", Eq. (inverted)) ----
 * y[p][r][c] = sum_{i,j = 0..2} w[p % C][i][j] * x[p][r + i - 1][c + j - 1], terms outside the
 * plane are zero.  Readings (the paper only names the operator): cross-correlation as in the
 * Haar kernels, stride 1, zero padding 1 -- the residual of Eq. (inverted) needs equal sizes --
 * no bias.  x, y [planes, H, W]; w [C, 3, 3]; plane p uses channel p % C.  Returns 0 or -1. */
int wcc_ref_depthwise3x3(const double *x, const double *w, int64_t planes, int64_t C, int64_t H,
                         int64_t W, double *y) {
  if (planes < 0 || C < 1 || H < 1 || W < 1) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t p = 0; p < planes; ++p) {
    const double *xp = x + p * H * W, *wp = w + (p % C) * 9;
    double *yp = y + p * H * W;
    for (int64_t r = 0; r < H; ++r)
      for (int64_t c = 0; c < W; ++c) {
        double acc = 0.0;
        for (int i = 0; i < 3; ++i)
          for (int j = 0; j < 3; ++j) {
            const int64_t rr = r + i - 1, cc = c + j - 1;
            if (rr >= 0 && rr < H && cc >= 0 && cc < W) acc += wp[i * 3 + j] * xp[rr * W + cc];
          }
        yp[r * W + c] = acc;
      }
  }
  return 0;
}

/* ---- cost model (appendix on bit operations) ---- */
int64_t wcc_ref_conv_mac(int64_t C_in, int64_t C_out, int64_t N_W, int64_t N_H, int64_t K_W,
                         int64_t K_H, int64_t S_W, int64_t S_H) {
  return C_in * C_out * N_W * N_H * K_W * K_H / (S_W * S_H);
}

int64_t wcc_ref_conv_bops(int64_t mac, int64_t b_w, int64_t b_a) { return mac * b_w * b_a; }

/* sum_{l=1..L} 4 * C * N_W * N_H / 4^(l-1) * b_a */
int64_t wcc_ref_haar_bops(int64_t C, int64_t N_W, int64_t N_H, int L, int64_t b_a) {
  int64_t total = 0, n = N_W * N_H;
  for (int l = 1; l <= L; ++l) {
    total += 4 * C * n * b_a;
    n /= 4;
  }
  return total;
}
