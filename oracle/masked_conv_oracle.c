/*
 * CPU oracle for the masked (semi-structured activation sparse) convolution.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP
 * library is checked against.  It shares no code with the HIP path; nothing in the
 * product may call it (only tests, the smoke check and the benchmark's cpu_baseline leg).
 *
 * What it computes (paper Sec. 3, Fig. 1-2; Sec. 3.2; App. A, Alg. 2):
 *   the convolution is a product of the lowered activation matrix (one row per output
 *   position, all kh*kw*Cin window entries) with the filter matrix; a binary mask over
 *   output positions removes whole rows of the lowered matrix.  A removed row is skipped
 *   and its output position holds zeros for every output channel (Alg. 2, post-process
 *   branch for mask == 0); a kept row holds the ordinary convolution result (Alg. 2,
 *   copy branch).  Masking one window does not touch the input pixels seen by the
 *   neighbouring windows (Fig. 2).
 *
 * The result has a plain definition, so the oracle is that definition written out:
 * a direct loop nest over (n, oy, ox, co, ky, kx, ci), double accumulation, no lowering
 * matrix, no blocking.  Readings taken where the paper is silent:
 *   - mask value 1 keeps the position, 0 drops it (Alg. 1 getMask, Alg. 2 both functions);
 *     the mask is indexed row-major, position = oy*Wo + ox (+ n*Ho*Wo for a per-row mask);
 *   - a dropped position is +0.0 in every channel: no bias, no activation (Alg. 2 memset);
 *   - bias and ReLU act on kept positions only, after the contraction;
 *   - zero padding, cross-correlation (no kernel flip),
 *     Ho = floor((H + 2*pad - dil*(kh-1) - 1)/stride) + 1;
 *   - the number of rows that run is output_size - sparsity*output_size (Sec. 3.2),
 *     rounded half up to an integer.
 *
 * Parity pins: tests/test_oracle_pins.py (library conv2d at sparsity 0, explicit
 * im2col + matmul + Alg. 2 expansion, closed forms, linearity, Fig. 2 locality,
 * kept-count goldens).
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* parameter vector layout (int32), shared with oracle.py */
enum {
  P_N = 0, P_CIN, P_H, P_W, P_COUT, P_KH, P_KW, P_SH, P_SW, P_PH, P_PW, P_DH, P_DW,
  P_NCHW,        /* 0: x[N,H,W,C], w[O,kh,kw,I], y[N,Ho,Wo,O]; 1: x[N,C,H,W], w[O,I,kh,kw], y[N,O,Ho,Wo] */
  P_HAS_BIAS, P_RELU,
  P_MASK_SPATIAL, /* 0: mask[N*Ho*Wo]; 1: mask[Ho*Wo] shared by every image */
  P_COUNT
};

int oc_param_count(void) { return P_COUNT; }

/* threads the parallel loops will use (reported beside timings) */
int oc_num_threads(void) { return omp_get_max_threads(); }

/* output extent of one spatial axis */
int oc_out_size(int in, int k, int stride, int pad, int dil) {
  int eff = in + 2 * pad - dil * (k - 1) - 1;
  if (eff < 0) return 0;
  return eff / stride + 1;
}

/* rows that remain in the contraction: output_size - sparsity*output_size (Sec. 3.2), half up */
int64_t oc_kept_count(double sparsity, int64_t output_size) {
  return (int64_t)floor((1.0 - sparsity) * (double)output_size + 0.5);
}

/* Alg. 2, indirection init: visit output positions in ascending order and append the
 * position to the list only where the mask is 1.  Returns the list length, or -1 when a
 * mask byte is neither 0 nor 1. */
int64_t oc_compact_rows(const uint8_t* mask, int64_t m, int32_t* row_idx) {
  int64_t index = 0;
  for (int64_t r = 0; r < m; ++r) {
    if (mask[r] > 1) return -1;
    if (mask[r] == 1) row_idx[index++] = (int32_t)r;
  }
  return index;
}

typedef struct {
  int n, cin, h, w, cout, kh, kw, sh, sw, ph, pw, dh, dw, nchw, has_bias, relu, mask_spatial;
  int ho, wo;
  int64_t xs_n, xs_c, xs_h, xs_w;     /* element strides of x */
  int64_t ws_o, ws_i, ws_ky, ws_kx;   /* element strides of w */
  int64_t ys_n, ys_c, ys_h, ys_w;     /* element strides of y */
} geom;

static int make_geom(const int32_t* p, geom* g) {
  g->n = p[P_N]; g->cin = p[P_CIN]; g->h = p[P_H]; g->w = p[P_W]; g->cout = p[P_COUT];
  g->kh = p[P_KH]; g->kw = p[P_KW]; g->sh = p[P_SH]; g->sw = p[P_SW];
  g->ph = p[P_PH]; g->pw = p[P_PW]; g->dh = p[P_DH]; g->dw = p[P_DW];
  g->nchw = p[P_NCHW]; g->has_bias = p[P_HAS_BIAS]; g->relu = p[P_RELU];
  g->mask_spatial = p[P_MASK_SPATIAL];
  if (g->n < 1 || g->cin < 1 || g->h < 1 || g->w < 1 || g->cout < 1 || g->kh < 1 || g->kw < 1 ||
      g->sh < 1 || g->sw < 1 || g->ph < 0 || g->pw < 0 || g->dh < 1 || g->dw < 1)
    return -1;
  g->ho = oc_out_size(g->h, g->kh, g->sh, g->ph, g->dh);
  g->wo = oc_out_size(g->w, g->kw, g->sw, g->pw, g->dw);
  if (g->ho < 1 || g->wo < 1) return -1;
  if (g->nchw) {
    g->xs_w = 1; g->xs_h = g->w; g->xs_c = (int64_t)g->h * g->w; g->xs_n = g->xs_c * g->cin;
    g->ws_kx = 1; g->ws_ky = g->kw; g->ws_i = (int64_t)g->kh * g->kw; g->ws_o = g->ws_i * g->cin;
    g->ys_w = 1; g->ys_h = g->wo; g->ys_c = (int64_t)g->ho * g->wo; g->ys_n = g->ys_c * g->cout;
  } else {
    g->xs_c = 1; g->xs_w = g->cin; g->xs_h = (int64_t)g->w * g->cin; g->xs_n = g->xs_h * g->h;
    g->ws_i = 1; g->ws_kx = g->cin; g->ws_ky = (int64_t)g->kw * g->cin; g->ws_o = g->ws_ky * g->kh;
    g->ys_c = 1; g->ys_w = g->cout; g->ys_h = (int64_t)g->wo * g->cout; g->ys_n = g->ys_h * g->ho;
  }
  return 0;
}

/* One output position: every output channel.  out/absum are strided by ostride. */
static void one_position(const geom* g, const float* x, const float* w, const float* bias,
                         int keep, int n, int oy, int ox, float* out, double* absum, int64_t ostride) {
  for (int co = 0; co < g->cout; ++co) {
    if (!keep) {
      out[co * ostride] = 0.0f;                 /* Alg. 2: memset of the whole channel vector */
      if (absum) absum[co * ostride] = 0.0;
      continue;
    }
    double acc = 0.0, mag = 0.0;
    for (int ky = 0; ky < g->kh; ++ky) {
      int iy = oy * g->sh - g->ph + ky * g->dh;
      if (iy < 0 || iy >= g->h) continue;       /* zero padding */
      for (int kx = 0; kx < g->kw; ++kx) {
        int ix = ox * g->sw - g->pw + kx * g->dw;
        if (ix < 0 || ix >= g->w) continue;
        for (int ci = 0; ci < g->cin; ++ci) {
          double xv = (double)x[n * g->xs_n + ci * g->xs_c + iy * g->xs_h + ix * g->xs_w];
          double wv = (double)w[co * g->ws_o + ci * g->ws_i + ky * g->ws_ky + kx * g->ws_kx];
          acc += xv * wv;
          mag += fabs(xv * wv);
        }
      }
    }
    if (g->has_bias) { acc += (double)bias[co]; mag += fabs((double)bias[co]); }
    if (g->relu && acc < 0.0) acc = 0.0;
    out[co * ostride] = (float)acc;
    if (absum) absum[co * ostride] = mag;
  }
}

static int mask_at(const geom* g, const uint8_t* mask, int n, int oy, int ox) {
  int64_t pos = (int64_t)oy * g->wo + ox;
  if (!g->mask_spatial) pos += (int64_t)n * g->ho * g->wo;
  return mask[pos];
}

/* Whole layer.  y has the dense output layout; absum (optional, same layout, double) receives
 * sum|x*w| + |bias| per element, the scale against which rounding error is judged.
 * Returns 0, -1 for bad geometry, -2 for a mask byte that is neither 0 nor 1. */
int oc_masked_conv2d(const int32_t* p, const float* x, const float* w, const float* bias,
                     const uint8_t* mask, float* y, double* absum) {
  geom g;
  if (make_geom(p, &g)) return -1;
  int64_t mlen = g.mask_spatial ? (int64_t)g.ho * g.wo : (int64_t)g.n * g.ho * g.wo;
  for (int64_t i = 0; i < mlen; ++i) if (mask[i] > 1) return -2;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < g.n; ++n) {
    for (int oy = 0; oy < g.ho; ++oy) {
      for (int ox = 0; ox < g.wo; ++ox) {
        int64_t off = n * g.ys_n + oy * g.ys_h + ox * g.ys_w;
        one_position(&g, x, w, bias, mask_at(&g, mask, n, oy, ox), n, oy, ox,
                     y + off, absum ? absum + off : NULL, g.ys_c);
      }
    }
  }
  return 0;
}

/* Backward pass of the masked convolution (Alg. 1: backward(model) follows maskedForward(model, mask)).
 * The forward pass is y[r,co] = mask[r] ? act(sum_k A[r,k] w[co,k] + bias[co]) : 0 with A the lowered
 * activations (Sec. 3), so with the upstream gradient dy and
 *     g[r,co] = dy[r,co]   if mask[r] == 1 and (no ReLU or y[r,co] > 0),   0 otherwise
 * the chain rule gives
 *     db[co]   = sum_r g[r,co]
 *     dw[co,k] = sum_r g[r,co] * A[r,k]                (a contraction over the kept rows only)
 *     dx[pixel] = sum over the windows (r, tap) that contain the pixel of sum_co g[r,co] * w[co,tap,ci]
 * The ReLU gate is read from the forward output y the caller passes (the stored values, so that both
 * sides of a comparison gate on the same numbers).  Plain loop nest, double accumulation, one thread.
 * dx and dw have the layouts of x and w; dx_abs / dw_abs (optional) receive the sums of the absolute
 * values of the terms, the scale against which rounding error is judged.  Returns 0, -1, -2 like the
 * forward function. */
int oc_masked_conv2d_backward(const int32_t* p, const float* x, const float* w, const float* y, const float* dy,
                              const uint8_t* mask, double* dx, double* dw, double* db, double* dx_abs,
                              double* dw_abs) {
  geom g;
  if (make_geom(p, &g)) return -1;
  int64_t mlen = g.mask_spatial ? (int64_t)g.ho * g.wo : (int64_t)g.n * g.ho * g.wo;
  for (int64_t i = 0; i < mlen; ++i) if (mask[i] > 1) return -2;
  const int64_t nx = (int64_t)g.n * g.cin * g.h * g.w, nw = (int64_t)g.cout * g.cin * g.kh * g.kw;
  for (int64_t i = 0; i < nx; ++i) { dx[i] = 0.0; if (dx_abs) dx_abs[i] = 0.0; }
  for (int64_t i = 0; i < nw; ++i) { dw[i] = 0.0; if (dw_abs) dw_abs[i] = 0.0; }
  for (int co = 0; co < g.cout; ++co) db[co] = 0.0;
  for (int n = 0; n < g.n; ++n)
    for (int oy = 0; oy < g.ho; ++oy)
      for (int ox = 0; ox < g.wo; ++ox) {
        if (!mask_at(&g, mask, n, oy, ox)) continue;            /* a dropped row has no gradient */
        for (int co = 0; co < g.cout; ++co) {
          int64_t yo = n * g.ys_n + co * g.ys_c + oy * g.ys_h + ox * g.ys_w;
          if (g.relu && !(y[yo] > 0.0f)) continue;               /* ReLU gate */
          double gv = (double)dy[yo];
          db[co] += gv;
          for (int ky = 0; ky < g.kh; ++ky) {
            int iy = oy * g.sh - g.ph + ky * g.dh;
            if (iy < 0 || iy >= g.h) continue;
            for (int kx = 0; kx < g.kw; ++kx) {
              int ix = ox * g.sw - g.pw + kx * g.dw;
              if (ix < 0 || ix >= g.w) continue;
              for (int ci = 0; ci < g.cin; ++ci) {
                int64_t xo = n * g.xs_n + ci * g.xs_c + iy * g.xs_h + ix * g.xs_w;
                int64_t wo = co * g.ws_o + ci * g.ws_i + ky * g.ws_ky + kx * g.ws_kx;
                dw[wo] += gv * (double)x[xo];
                dx[xo] += gv * (double)w[wo];
                if (dw_abs) dw_abs[wo] += fabs(gv * (double)x[xo]);
                if (dx_abs) dx_abs[xo] += fabs(gv * (double)w[wo]);
              }
            }
          }
        }
      }
  return 0;
}

/* Selected output positions only (row r = (n*Ho + oy)*Wo + ox); y_rows is [nrows][Cout]
 * regardless of layout.  Used to spot-check layers too large to evaluate in full. */
int oc_masked_conv2d_rows(const int32_t* p, const float* x, const float* w, const float* bias,
                          const uint8_t* mask, const int64_t* rows, int64_t nrows,
                          float* y_rows, double* absum_rows) {
  geom g;
  if (make_geom(p, &g)) return -1;
  int64_t m = (int64_t)g.n * g.ho * g.wo;
  for (int64_t i = 0; i < nrows; ++i) if (rows[i] < 0 || rows[i] >= m) return -3;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < nrows; ++i) {
    int64_t r = rows[i];
    int ox = (int)(r % g.wo);
    int oy = (int)((r / g.wo) % g.ho);
    int n = (int)(r / ((int64_t)g.wo * g.ho));
    one_position(&g, x, w, bias, mask_at(&g, mask, n, oy, ox), n, oy, ox,
                 y_rows + i * g.cout, absum_rows ? absum_rows + i * g.cout : NULL, 1);
  }
  return 0;
}

/* ------------------------------------------------------------------------------------------
 * Storage rounding between layers of a network run (activations are stored in the layer dtype).
 * ------------------------------------------------------------------------------------------ */
void oc_round_bf16(float* a, int64_t count) {
  for (int64_t i = 0; i < count; ++i) {
    uint32_t u; memcpy(&u, &a[i], 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) { u |= 0x00400000u; u &= 0xffff0000u; }   /* NaN stays NaN */
    else { uint32_t lsb = (u >> 16) & 1u; u += 0x7fffu + lsb; u &= 0xffff0000u; }   /* nearest, ties to even */
    memcpy(&a[i], &u, 4);
  }
}

/* nearest binary16 value (ties to even): 11 significant bits, exponent floor -14, overflow to inf */
void oc_round_f16(float* a, int64_t count) {
  for (int64_t i = 0; i < count; ++i) {
    double v = (double)a[i];
    if (v == 0.0 || isnan(v) || isinf(v)) continue;
    int e;
    (void)frexp(fabs(v), &e);            /* |v| = f * 2^e, f in [0.5, 1) */
    int exp2 = e - 1;                    /* |v| in [2^exp2, 2^(exp2+1)) */
    if (exp2 < -14) exp2 = -14;          /* subnormal range shares the quantum of 2^-14 */
    double quantum = ldexp(1.0, exp2 - 10);
    double r = nearbyint(v / quantum) * quantum;   /* default rounding mode: ties to even */
    if (fabs(r) >= 65520.0) r = v > 0 ? INFINITY : -INFINITY;
    a[i] = (float)r;
  }
}

/* ------------------------------------------------------------------------------------------
 * The two glue operators of the ResNet-style test network (NHWC float tensors).
 * ------------------------------------------------------------------------------------------ */

/* max pooling, window k, stride s, padding p (padded positions never win) */
int oc_maxpool2d_nhwc(const float* x, int n, int h, int w, int c, int k, int s, int p, float* y) {
  int ho = oc_out_size(h, k, s, p, 1), wo = oc_out_size(w, k, s, p, 1);
  if (ho < 1 || wo < 1) return -1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int b = 0; b < n; ++b)
    for (int oy = 0; oy < ho; ++oy)
      for (int ox = 0; ox < wo; ++ox)
        for (int ch = 0; ch < c; ++ch) {
          float best = -INFINITY;
          for (int ky = 0; ky < k; ++ky) {
            int iy = oy * s - p + ky;
            if (iy < 0 || iy >= h) continue;
            for (int kx = 0; kx < k; ++kx) {
              int ix = ox * s - p + kx;
              if (ix < 0 || ix >= w) continue;
              float v = x[(((int64_t)b * h + iy) * w + ix) * c + ch];
              if (v > best) best = v;
            }
          }
          y[(((int64_t)b * ho + oy) * wo + ox) * c + ch] = best;
        }
  return 0;
}

/* residual join: y = max(a + b, 0) */
void oc_add_relu(const float* a, const float* b, int64_t count, float* y) {
  for (int64_t i = 0; i < count; ++i) {
    float v = a[i] + b[i];
    y[i] = v > 0.0f ? v : 0.0f;
  }
}
