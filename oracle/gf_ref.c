/*
 * gf_ref.c -- plain CPU oracle (see gf_ref.h).  TEST INFRASTRUCTURE ONLY.
 *
 * Loops are written in the order of the paper's index notation; there is no
 * blocking, fusion or reordering.  The only parallelism is an OpenMP pragma on
 * an outermost loop whose iterations write disjoint outputs.
 */
#include "gf_ref.h"

#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { REF_OK = 0, REF_NULL = 1, REF_BAD_DESC = 2, REF_SHAPE = 3 };

static int cdiv(int a, int b) { return (a + b - 1) / b; }
static int imin(int a, int b) { return a < b ? a : b; }

int gf_ref_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

static int check_desc(const gf_ref_desc* d) {
  if (!d) return REF_NULL;
  if (d->N < 1 || d->C_in < 1 || d->C_out < 1 || d->H_in < 1 || d->W_in < 1) return REF_BAD_DESC;
  if (d->K_h < 1 || d->K_w < 1 || d->stride < 1 || d->pad < 0 || d->dilation < 1) return REF_BAD_DESC;
  if (d->groups < 1 || d->C_in % d->groups || d->C_out % d->groups) return REF_BAD_DESC;
  if (d->r < 1) return REF_BAD_DESC;
  return REF_OK;
}

/* H_y = floor((H_x + 2p - d(K-1) - 1)/s) + 1; patch grid ceil(H_y/r) (Sec. 3.3). */
int gf_ref_out_shape(const gf_ref_desc* d, int* H_out, int* W_out, int* H_p, int* W_p) {
  int rc = check_desc(d);
  if (rc) return rc;
  int eh = d->H_in + 2 * d->pad - d->dilation * (d->K_h - 1) - 1;
  int ew = d->W_in + 2 * d->pad - d->dilation * (d->K_w - 1) - 1;
  if (eh < 0 || ew < 0) return REF_SHAPE;
  int Hy = eh / d->stride + 1, Wy = ew / d->stride + 1;
  int Hp = cdiv(Hy, d->r), Wp = cdiv(Wy, d->r);
  if (d->r > 1) {
    /* the input-side grid (patch r*s on x) must be the same grid */
    int rx = d->r * d->stride;
    if (cdiv(d->H_in, rx) != Hp || cdiv(d->W_in, rx) != Wp) return REF_SHAPE;
  }
  if (H_out) *H_out = Hy;
  if (W_out) *W_out = Wy;
  if (H_p) *H_p = Hp;
  if (W_p) *W_p = Wp;
  return REF_OK;
}

/* Patch reduction of a stack of planes: out[plane,hp,wp] = sum (or mean) of
 * in[plane, hp*q .. hp*q+q-1, wp*q .. wp*q+q-1] restricted to the plane. */
static void patch_reduce(const double* in, double* out, long planes, int H, int W, int q,
                         int mean) {
  int Hp = cdiv(H, q), Wp = cdiv(W, q);
#pragma omp parallel for schedule(static)
  for (long pl = 0; pl < planes; ++pl) {
    const double* src = in + (size_t)pl * H * W;
    double* dst = out + (size_t)pl * Hp * Wp;
    for (int hp = 0; hp < Hp; ++hp)
      for (int wp = 0; wp < Wp; ++wp) {
        int ch = imin(q, H - hp * q), cw = imin(q, W - wp * q);
        double acc = 0.0;
        for (int i = 0; i < ch; ++i)
          for (int j = 0; j < cw; ++j) acc += src[(size_t)(hp * q + i) * W + (wp * q + j)];
        dst[(size_t)hp * Wp + wp] = mean ? acc / (double)(ch * cw) : acc;
      }
  }
}

int gf_ref_filter_grad(const gf_ref_desc* d, const double* g_y, double* gy_u) {
  int Hy, Wy, Hp, Wp;
  int rc = gf_ref_out_shape(d, &Hy, &Wy, &Hp, &Wp);
  if (rc) return rc;
  if (!g_y || !gy_u) return REF_NULL;
  patch_reduce(g_y, gy_u, (long)d->N * d->C_out, Hy, Wy, d->r, 1);
  return REF_OK;
}

int gf_ref_filter_snr(const gf_ref_desc* d, const double* g_y, double* energy, double* noise) {
  int Hy, Wy, Hp, Wp;
  int rc = gf_ref_out_shape(d, &Hy, &Wy, &Hp, &Wp);
  if (rc) return rc;
  if (!g_y || !energy || !noise) return REF_NULL;
  long planes = (long)d->N * d->C_out;
  double* gy_u = (double*)malloc(sizeof(double) * (size_t)planes * Hp * Wp);
  if (!gy_u) return REF_NULL;
  patch_reduce(g_y, gy_u, planes, Hy, Wy, d->r, 1);
  double e = 0.0, v = 0.0;
  for (long pl = 0; pl < planes; ++pl)
    for (int h = 0; h < Hy; ++h)
      for (int w = 0; w < Wy; ++w) {
        double g = g_y[((size_t)pl * Hy + h) * Wy + w];
        double m = gy_u[((size_t)pl * Hp + h / d->r) * Wp + w / d->r]; /* the value g~_y has at (h, w) */
        e += g * g;
        v += (g - m) * (g - m);
      }
  free(gy_u);
  *energy = e;
  *noise = v;
  return REF_OK;
}

int gf_ref_pool_activation(const gf_ref_desc* d, const double* x, double* x_u) {
  int rc = gf_ref_out_shape(d, 0, 0, 0, 0);
  if (rc) return rc;
  if (!x || !x_u) return REF_NULL;
  /* r == 1: exact BP needs x itself (patch 1 even when the layer is strided) */
  int q = d->r == 1 ? 1 : d->r * d->stride;
  patch_reduce(x, x_u, (long)d->N * d->C_in, d->H_in, d->W_in, q, 0);
  return REF_OK;
}

int gf_ref_pool_activation_mask(const gf_ref_desc* d, const double* x, double hi, double* x_u, double* m_u) {
  int rc = gf_ref_pool_activation(d, x, x_u);
  if (rc) return rc;
  if (!m_u) return REF_NULL;
  size_t total = (size_t)d->N * d->C_in * d->H_in * d->W_in;
  double* pass = (double*)malloc(sizeof(double) * total);
  if (!pass) return REF_NULL;
  for (size_t e = 0; e < total; ++e) pass[e] = (x[e] > 0.0 && x[e] < hi) ? 1.0 : 0.0;
  int q = d->r == 1 ? 1 : d->r * d->stride;
  patch_reduce(pass, m_u, (long)d->N * d->C_in, d->H_in, d->W_in, q, 1);   /* mean over in-bounds pixels */
  free(pass);
  return REF_OK;
}

int gf_ref_kernel_sum(const gf_ref_desc* d, const double* w, double* w_sum) {
  int rc = check_desc(d);
  if (rc) return rc;
  if (!w || !w_sum) return REF_NULL;
  int Cg = d->C_in / d->groups, KK = d->K_h * d->K_w;
  for (long e = 0; e < (long)d->C_out * Cg; ++e) {
    double acc = 0.0;
    for (int t = 0; t < KK; ++t) acc += w[(size_t)e * KK + t];
    w_sum[e] = acc;
  }
  return REF_OK;
}

int gf_ref_conv_fwd(const gf_ref_desc* d, const double* x, const double* w, double* y) {
  int Hy, Wy;
  int rc = check_desc(d);
  if (rc) return rc;
  {
    gf_ref_desc e = *d;
    e.r = 1;
    rc = gf_ref_out_shape(&e, &Hy, &Wy, 0, 0);
    if (rc) return rc;
  }
  if (!x || !w || !y) return REF_NULL;
  int Cg = d->C_in / d->groups, Og = d->C_out / d->groups;
  int s = d->stride, p = d->pad, dl = d->dilation;
#pragma omp parallel for schedule(static) collapse(2)
  for (int n = 0; n < d->N; ++n)
    for (int co = 0; co < d->C_out; ++co) {
      int g = co / Og;
      for (int i = 0; i < Hy; ++i)
        for (int j = 0; j < Wy; ++j) {
          double acc = 0.0;
          for (int cl = 0; cl < Cg; ++cl) {
            int ci = g * Cg + cl;
            for (int u = 0; u < d->K_h; ++u)
              for (int v = 0; v < d->K_w; ++v) {
                int h = i * s - p + u * dl, ww = j * s - p + v * dl;
                if (h < 0 || h >= d->H_in || ww < 0 || ww >= d->W_in) continue;
                acc += w[(((size_t)co * Cg + cl) * d->K_h + u) * d->K_w + v] *
                       x[(((size_t)n * d->C_in + ci) * d->H_in + h) * d->W_in + ww];
              }
          }
          y[(((size_t)n * d->C_out + co) * Hy + i) * Wy + j] = acc;
        }
    }
  return REF_OK;
}

/* g_theta[c_o,c_i',u,v] = sum_{n,i,j} x[n,c_i,i s - p + u d, j s - p + v d] g_y[n,c_o,i,j] */
static void exact_wgrad(const gf_ref_desc* d, int Hy, int Wy, const double* x, const double* g_y,
                        double* g_w) {
  int Cg = d->C_in / d->groups, Og = d->C_out / d->groups;
  int s = d->stride, p = d->pad, dl = d->dilation;
#pragma omp parallel for schedule(static)
  for (int co = 0; co < d->C_out; ++co) {
    int g = co / Og;
    for (int cl = 0; cl < Cg; ++cl) {
      int ci = g * Cg + cl;
      for (int u = 0; u < d->K_h; ++u)
        for (int v = 0; v < d->K_w; ++v) {
          double acc = 0.0;
          for (int n = 0; n < d->N; ++n)
            for (int i = 0; i < Hy; ++i)
              for (int j = 0; j < Wy; ++j) {
                int h = i * s - p + u * dl, ww = j * s - p + v * dl;
                if (h < 0 || h >= d->H_in || ww < 0 || ww >= d->W_in) continue;
                acc += x[(((size_t)n * d->C_in + ci) * d->H_in + h) * d->W_in + ww] *
                       g_y[(((size_t)n * d->C_out + co) * Hy + i) * Wy + j];
              }
          g_w[(((size_t)co * Cg + cl) * d->K_h + u) * d->K_w + v] = acc;
        }
    }
  }
}

/* g_x = g_y convolved with the rotated kernel, written as the transpose of the
 * forward index map: every forward term y[i,j] += theta[u,v] x[h,w] sends
 * g_y[i,j] theta[u,v] back to g_x[h,w]. */
static void exact_dgrad(const gf_ref_desc* d, int Hy, int Wy, const double* w, const double* g_y,
                        double* g_x) {
  int Cg = d->C_in / d->groups, Og = d->C_out / d->groups;
  int s = d->stride, p = d->pad, dl = d->dilation;
  size_t per_n = (size_t)d->C_in * d->H_in * d->W_in;
#pragma omp parallel for schedule(static)
  for (int n = 0; n < d->N; ++n) {
    double* gxn = g_x + (size_t)n * per_n;
    memset(gxn, 0, per_n * sizeof(double));
    for (int co = 0; co < d->C_out; ++co) {
      int g = co / Og;
      for (int cl = 0; cl < Cg; ++cl) {
        int ci = g * Cg + cl;
        for (int i = 0; i < Hy; ++i)
          for (int j = 0; j < Wy; ++j) {
            double gy = g_y[(((size_t)n * d->C_out + co) * Hy + i) * Wy + j];
            for (int u = 0; u < d->K_h; ++u)
              for (int v = 0; v < d->K_w; ++v) {
                int h = i * s - p + u * dl, ww = j * s - p + v * dl;
                if (h < 0 || h >= d->H_in || ww < 0 || ww >= d->W_in) continue;
                gxn[((size_t)ci * d->H_in + h) * d->W_in + ww] +=
                    w[(((size_t)co * Cg + cl) * d->K_h + u) * d->K_w + v] * gy;
              }
          }
      }
    }
  }
}

int gf_ref_bwd_exact(const gf_ref_desc* d, const double* x, const double* w, const double* g_y,
                     double* g_w, double* g_x) {
  int Hy, Wy;
  int rc = check_desc(d);
  if (rc) return rc;
  {
    gf_ref_desc e = *d;
    e.r = 1;
    rc = gf_ref_out_shape(&e, &Hy, &Wy, 0, 0);
    if (rc) return rc;
  }
  if (!g_y) return REF_NULL;
  if (g_w) {
    if (!x) return REF_NULL;
    exact_wgrad(d, Hy, Wy, x, g_y, g_w);
  }
  if (g_x) {
    if (!w) return REF_NULL;
    exact_dgrad(d, Hy, Wy, w, g_y, g_x);
  }
  return REF_OK;
}

int gf_ref_bwd_weight(const gf_ref_desc* d, const double* x_u, const double* gy_u, double* g_w) {
  int Hy, Wy, Hp, Wp;
  int rc = gf_ref_out_shape(d, &Hy, &Wy, &Hp, &Wp);
  if (rc) return rc;
  if (!x_u || !gy_u || !g_w) return REF_NULL;
  if (d->r == 1) { /* vanilla BP: x_u is x, gy_u is g_y */
    exact_wgrad(d, Hy, Wy, x_u, gy_u, g_w);
    return REF_OK;
  }
  int Cg = d->C_in / d->groups, Og = d->C_out / d->groups, KK = d->K_h * d->K_w;
  size_t P = (size_t)Hp * Wp;
  double inv_s2 = 1.0 / ((double)d->stride * d->stride);
#pragma omp parallel for schedule(static)
  for (int co = 0; co < d->C_out; ++co) {
    int g = co / Og;
    for (int cl = 0; cl < Cg; ++cl) {
      int ci = g * Cg + cl;
      double acc = 0.0;
      for (int n = 0; n < d->N; ++n)
        for (size_t q = 0; q < P; ++q)
          acc += x_u[((size_t)n * d->C_in + ci) * P + q] * gy_u[((size_t)n * d->C_out + co) * P + q];
      acc *= inv_s2;
      for (int t = 0; t < KK; ++t) g_w[((size_t)co * Cg + cl) * KK + t] = acc;
    }
  }
  return REF_OK;
}

int gf_ref_bwd_input(const gf_ref_desc* d, const double* gy_u, const double* w, double* g_x,
                     int reduced_out) {
  int Hy, Wy, Hp, Wp;
  int rc = gf_ref_out_shape(d, &Hy, &Wy, &Hp, &Wp);
  if (rc) return rc;
  if (!gy_u || !w || !g_x) return REF_NULL;
  if (d->r == 1) { /* vanilla BP; a 1x1 patch grid is the full map either way */
    exact_dgrad(d, Hy, Wy, w, gy_u, g_x);
    return REF_OK;
  }
  int Cg = d->C_in / d->groups, Og = d->C_out / d->groups, KK = d->K_h * d->K_w;
  int rx = d->r * d->stride;
  size_t P = (size_t)Hp * Wp;
  double inv_s2 = 1.0 / ((double)d->stride * d->stride);
#pragma omp parallel for schedule(static) collapse(2)
  for (int n = 0; n < d->N; ++n)
    for (int ci = 0; ci < d->C_in; ++ci) {
      int g = ci / Cg, cl = ci % Cg;
      for (int hp = 0; hp < Hp; ++hp)
        for (int wp = 0; wp < Wp; ++wp) {
          double acc = 0.0;
          for (int ol = 0; ol < Og; ++ol) {
            int co = g * Og + ol;
            double wsum = 0.0; /* text after Eq. (3): spatial sum of the kernel */
            for (int t = 0; t < KK; ++t) wsum += w[((size_t)co * Cg + cl) * KK + t];
            acc += gy_u[((size_t)n * d->C_out + co) * P + (size_t)hp * Wp + wp] * wsum;
          }
          acc *= inv_s2;
          if (reduced_out) {
            g_x[((size_t)n * d->C_in + ci) * P + (size_t)hp * Wp + wp] = acc;
          } else {
            int h1 = imin((hp + 1) * rx, d->H_in), w1 = imin((wp + 1) * rx, d->W_in);
            for (int h = hp * rx; h < h1; ++h)
              for (int ww = wp * rx; ww < w1; ++ww)
                g_x[(((size_t)n * d->C_in + ci) * d->H_in + h) * d->W_in + ww] = acc;
          }
        }
    }
  return REF_OK;
}

int gf_ref_quantize_q8(const double* v, long n, float inv_delta, signed char* q) {
  if (!v || !q) return REF_NULL;
  if (!(inv_delta > 0.0f)) return REF_BAD_DESC;
  for (long i = 0; i < n; ++i) {
    float t = (float)v[i] * inv_delta; /* binary32 product */
    float r = rintf(t);                /* round half to even (default rounding mode) */
    if (r > 127.0f) r = 127.0f;
    if (!(r >= -127.0f)) r = -127.0f; /* also a NaN: it is clipped like minus infinity */
    q[i] = (signed char)r;
  }
  return REF_OK;
}

int gf_ref_bwd_weight_q8(const gf_ref_desc* d, const signed char* x_q, const signed char* gy_q, long long* acc) {
  int Hy, Wy, Hp, Wp;
  int rc = gf_ref_out_shape(d, &Hy, &Wy, &Hp, &Wp);
  if (rc) return rc;
  if (!x_q || !gy_q || !acc) return REF_NULL;
  if (d->r == 1) return REF_BAD_DESC; /* codes are defined for the reduced maps only */
  int Cg = d->C_in / d->groups, Og = d->C_out / d->groups;
  size_t P = (size_t)Hp * Wp;
  for (int co = 0; co < d->C_out; ++co) {
    int g = co / Og;
    for (int cl = 0; cl < Cg; ++cl) {
      int ci = g * Cg + cl;
      long long a = 0;
      for (int n = 0; n < d->N; ++n)
        for (size_t q = 0; q < P; ++q)
          a += (long long)x_q[((size_t)n * d->C_in + ci) * P + q] * (long long)gy_q[((size_t)n * d->C_out + co) * P + q];
      acc[(size_t)co * Cg + cl] = a;
    }
  }
  return REF_OK;
}

int gf_ref_bwd_input_q8(const gf_ref_desc* d, const signed char* gy_q, const signed char* w_q, long long* acc) {
  int Hy, Wy, Hp, Wp;
  int rc = gf_ref_out_shape(d, &Hy, &Wy, &Hp, &Wp);
  if (rc) return rc;
  if (!gy_q || !w_q || !acc) return REF_NULL;
  if (d->r == 1) return REF_BAD_DESC;
  int Cg = d->C_in / d->groups, Og = d->C_out / d->groups;
  size_t P = (size_t)Hp * Wp;
  for (int n = 0; n < d->N; ++n)
    for (int ci = 0; ci < d->C_in; ++ci) {
      int g = ci / Cg, cl = ci % Cg;
      for (size_t q = 0; q < P; ++q) {
        long long a = 0;
        for (int ol = 0; ol < Og; ++ol) {
          int co = g * Og + ol;
          a += (long long)gy_q[((size_t)n * d->C_out + co) * P + q] * (long long)w_q[(size_t)co * Cg + cl];
        }
        acc[((size_t)n * d->C_in + ci) * P + q] = a;
      }
    }
  return REF_OK;
}

int gf_ref_cost_model(const gf_ref_desc* d, gf_ref_cost* out) {
  int Hy, Wy, Hp, Wp;
  int rc = gf_ref_out_shape(d, &Hy, &Wy, &Hp, &Wp);
  if (rc) return rc;
  if (!out) return REF_NULL;
  double Cx = d->C_in, Cy = d->C_out, KK = (double)d->K_h * d->K_w;
  int rx = d->r == 1 ? 1 : d->r * d->stride; /* r == 1 is vanilla BP: x itself is stored */
  out->flops_exact_gx = 2.0 * Cx * Cy * (double)Wy * Hy * KK;
  out->flops_gf_gx = (double)Hp * Wp * Cx * (2.0 * Cy - 1.0);
  out->flops_gf_min = 2.0 * Cx * Cy - Cx;
  out->overhead_fwd = 1.0 / (2.0 * Cy * KK);
  out->overhead_bwd = ((double)d->r * d->r - 1.0) / (2.0 * Cx);
  out->act_elems_exact = Cx * (double)d->H_in * d->W_in;
  out->act_elems_gf = Cx * (double)cdiv(d->H_in, rx) * cdiv(d->W_in, rx);
  return REF_OK;
}
