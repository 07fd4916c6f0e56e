/*
 * sanitize_main.c -- runs the CPU oracle (wcc_ref.c) as a stand-alone program so that it can be
 * built with gcc's address and undefined-behaviour sanitizers.  TEST INFRASTRUCTURE ONLY.
 *
 * usage: sanitize_main <input file> <output file>
 * input  (host byte order): ten int64 -- B, C_in, C_out, H, W, levels, keep_num, keep_den,
 *        act_bits, has_scale -- then doubles: x [B,C_in,H,W], w [C_out,C_in],
 *        w_scale [C_out] (if has_scale), w_dw [C_in,3,3], alpha_in.
 * output: doubles y [B,C_out,H,W]; int64 idx [B,k]; double alpha; doubles: coef [B,C_in,N]
 *        (transform of x), back [B,C_in,H,W] (its inverse), dw [B,C_in,H,W] (K_dw x).
 * It contains no arithmetic of the method: it reads, calls and writes.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int64_t wcc_ref_k(int64_t N, int64_t num, int64_t den);
int wcc_ref_haar_fwd(const double *x, int64_t planes, int64_t H, int64_t W, int d, double *y);
int wcc_ref_haar_inv(const double *y, int64_t planes, int64_t H, int64_t W, int d, double *x);
int wcc_ref_forward(const double *x, const double *w, const double *w_scale, int64_t B,
                    int64_t C_in, int64_t C_out, int64_t H, int64_t W, int d, int64_t keep_num,
                    int64_t keep_den, int act_bits, double alpha_in, double *y, int64_t *idx_out,
                    double *alpha_out);
int wcc_ref_depthwise3x3(const double *x, const double *w, int64_t planes, int64_t C, int64_t H,
                         int64_t W, double *y);

static double *read_doubles(FILE *f, size_t n) {
  double *p = (double *)malloc(sizeof(double) * (n ? n : 1));
  if (!p || fread(p, sizeof(double), n, f) != n) { fprintf(stderr, "short input\n"); exit(2); }
  return p;
}

int main(int argc, char **argv) {
  if (argc != 3) { fprintf(stderr, "usage: %s <in> <out>\n", argv[0]); return 2; }
  FILE *f = fopen(argv[1], "rb");
  if (!f) { perror(argv[1]); return 2; }
  int64_t h[10];
  if (fread(h, sizeof(int64_t), 10, f) != 10) { fprintf(stderr, "short header\n"); return 2; }
  const int64_t B = h[0], Ci = h[1], Co = h[2], H = h[3], W = h[4], N = H * W;
  const int d = (int)h[5], bits = (int)h[8];
  double *x = read_doubles(f, (size_t)(B * Ci * N));
  double *w = read_doubles(f, (size_t)(Co * Ci));
  double *sc = h[9] ? read_doubles(f, (size_t)Co) : NULL;
  double *wdw = read_doubles(f, (size_t)(Ci * 9));
  double *alpha_in = read_doubles(f, 1);
  fclose(f);

  const int64_t k = wcc_ref_k(N, h[6], h[7]);
  double *y = (double *)malloc(sizeof(double) * (size_t)(B * Co * N));
  int64_t *idx = (int64_t *)malloc(sizeof(int64_t) * (size_t)(B * (k > 0 ? k : 1)));
  double *coef = (double *)malloc(sizeof(double) * (size_t)(B * Ci * N));
  double *back = (double *)malloc(sizeof(double) * (size_t)(B * Ci * N));
  double *dw = (double *)malloc(sizeof(double) * (size_t)(B * Ci * N));
  double alpha = 0.0;
  if (!y || !idx || !coef || !back || !dw) return 2;
  if (wcc_ref_forward(x, w, sc, B, Ci, Co, H, W, d, h[6], h[7], bits, alpha_in[0], y, idx, &alpha)) return 3;
  if (wcc_ref_haar_fwd(x, B * Ci, H, W, d, coef)) return 3;
  if (wcc_ref_haar_inv(coef, B * Ci, H, W, d, back)) return 3;
  if (wcc_ref_depthwise3x3(x, wdw, B * Ci, Ci, H, W, dw)) return 3;

  f = fopen(argv[2], "wb");
  if (!f) { perror(argv[2]); return 2; }
  fwrite(y, sizeof(double), (size_t)(B * Co * N), f);
  fwrite(idx, sizeof(int64_t), (size_t)(B * k), f);
  fwrite(&alpha, sizeof(double), 1, f);
  fwrite(coef, sizeof(double), (size_t)(B * Ci * N), f);
  fwrite(back, sizeof(double), (size_t)(B * Ci * N), f);
  fwrite(dw, sizeof(double), (size_t)(B * Ci * N), f);
  fclose(f);
  free(x); free(w); free(sc); free(wdw); free(alpha_in);
  free(y); free(idx); free(coef); free(back); free(dw);
  return 0;
}
