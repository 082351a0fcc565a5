/*
 * gf_ref.h -- plain CPU oracle for gradient-filtered convolution backward.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, obviously-correct statement of
 * what the GPU library must compute.  Only the test-suite, the smoke check and
 * the benchmark's cpu_baseline leg may call it; the product path never does.
 * It shares no code, header, table or helper with the HIP library.
 *
 * Every tensor is a contiguous NCHW array of double on the host.  Every
 * accumulation is fp64.  Functions return 0 on success, a positive code on a
 * rejected descriptor (1 = null pointer, 2 = bad descriptor, 3 = shape rule).
 *
 * Notation follows the paper's symbol table: x [N,C_x,H_x,W_x] layer input,
 * theta [C_y, C_x/groups, K_h, K_w] kernel, g_y [N,C_y,H_y,W_y] output
 * gradient, r patch size.  "u" tensors hold one value per r x r patch
 * (Supp. B "Gradient Filtering": the matrix of unique values).
 *
 * Readings of the paper taken here (the paper is silent or garbled on them):
 *   - patch limits: the r x r patch that contains the pixel (prose of Sec. 3.3),
 *     not the literal floor/ceil summation bounds of Eq. (2);
 *   - ragged last patch (r does not divide H_y): average / sum over the
 *     in-bounds pixels only, grid ceil(H_y/r) x ceil(W_y/r) (Sec. 3.3);
 *   - stride s > 1: a stride-s layer is a stride-1 layer followed by
 *     subsampling; filtering the zero-inserted gradient with patch r*s gives
 *     input-side patch r_x = r*s and a factor 1/s^2 in both gradients;
 *   - dilation does not enter the filtered formulas (every tap reads its own
 *     padded patch, Supp. B "Boundary Elements");
 *   - groups: the channel sum of Eq. (3) runs over the group of c_i only;
 *   - r == 1 is DEFINED as exact back-propagation (Sec. 4.2: a 1x1 patch means
 *     vanilla BP): the "u" tensors are then the full maps and the weight /
 *     input gradient entries evaluate the exact K x K contractions.
 */
#ifndef GF_REF_H
#define GF_REF_H

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gf_ref_desc {
  int N, C_in, C_out, H_in, W_in;
  int K_h, K_w, stride, pad, dilation, groups;
  int r;
} gf_ref_desc;

/* Closed forms of Sec. 3.2 / Sec. 4.2 / Sec. 4.3, per image unless noted. */
typedef struct gf_ref_cost {
  double flops_exact_gx;   /* Eq. (1): 2 C_x C_y W_y H_y W_th H_th              */
  double flops_gf_gx;      /* Eq. (12) leading term: ceil(H_y/r)ceil(W_y/r) C_x (2 C_y - 1) */
  double flops_gf_min;     /* Eq. (13) leading term: 2 C_x C_y - C_x            */
  double overhead_fwd;     /* Sec. 4.2 "Overhead": 1 / (2 C_o W_th H_th)        */
  double overhead_bwd;     /* Sec. 4.2 "Overhead": (r^2 - 1) / (2 C_x)          */
  double act_elems_exact;  /* Sec. 4.3: C_x H_x W_x stored values per image      */
  double act_elems_gf;     /* Sec. 4.3: C_x ceil(H_x/r_x) ceil(W_x/r_x)          */
} gf_ref_cost;

int gf_ref_out_shape(const gf_ref_desc* d, int* H_out, int* W_out, int* H_p, int* W_p);

/* S1, Eq. (2): gy_u[n,c,hp,wp] = mean of g_y over the patch.  [N,C_out,H_p,W_p] */
int gf_ref_filter_grad(const gf_ref_desc* d, const double* g_y, double* gy_u);
/* Noise of the filter, first line of Eq. (8) taken in the pixel domain (per patch the DFT keeps
 * sums of squares up to the common factor r^2, so the ratio is the same):
 *   *energy = sum g_y^2,  *noise = sum (g_y - its patch mean)^2,  SNR = energy / noise.   */
int gf_ref_filter_snr(const gf_ref_desc* d, const double* g_y, double* energy, double* noise);
/* S0, text after Eq. (5): x_u[n,c,hp,wp] = sum of x over the r_x x r_x patch.
 * [N,C_in,H_p,W_p]; with r == 1 it is a copy of x, [N,C_in,H_in,W_in].          */
int gf_ref_pool_activation(const gf_ref_desc* d, const double* x, double* x_u);
/* S0 for a layer whose input is the output of a ReLU (hi = +inf) or of a clipped ReLU
 * (0 < x < hi passes the gradient): beside x_u, m_u[n,c,hp,wp] = the fraction of the patch's
 * in-bounds pixels through which that non-linearity passes a gradient.  With the upper layer's
 * input gradient constant on every patch (Eq. 3), the gradient filter of the layer below
 * (Eq. 2, patch r_x) applied to the masked gradient returns that constant times m_u.        */
int gf_ref_pool_activation_mask(const gf_ref_desc* d, const double* x, double hi, double* x_u, double* m_u);
/* S2, text after Eq. (3): w_sum[c_o,c_i'] = sum over taps.  [C_out, C_in/groups] */
int gf_ref_kernel_sum(const gf_ref_desc* d, const double* w, double* w_sum);
/* S3, Eq. (5): Frobenius inner product of x_u and gy_u over (n, patch), scaled
 * 1/s^2, written to every tap.  g_w [C_out, C_in/groups, K_h, K_w].             */
int gf_ref_bwd_weight(const gf_ref_desc* d, const double* x_u, const double* gy_u, double* g_w);
/* S4, Eq. (3): channel sum of gy_u times w_sum, scaled 1/s^2, then every pixel
 * of the input-side patch takes its patch's value.  g_x [N,C_in,H_in,W_in], or
 * [N,C_in,H_p,W_p] when reduced_out != 0.                                        */
int gf_ref_bwd_input(const gf_ref_desc* d, const double* gy_u, const double* w, double* g_x,
                     int reduced_out);
/* Sec. 3.1: exact g_theta (Frobenius inner product) and g_x (convolution with
 * the rotated kernel), zero padding; either output may be NULL.                 */
int gf_ref_bwd_exact(const gf_ref_desc* d, const double* x, const double* w, const double* g_y,
                     double* g_w, double* g_x);
/* Forward convolution y = conv(x, theta) (Sec. 3.1), used to pin the backward. */
int gf_ref_conv_fwd(const gf_ref_desc* d, const double* x, const double* w, double* y);

/* ---- gradient filtering on 8-bit codes (Supp. H combines the method with 8-bit gradient
 * quantisation but fixes no quantiser; reading taken here: one step size per tensor, symmetric
 * signed codes, round half to even, clipped to +-127 -- the per-tensor scheme of the 8-bit training
 * methods the supplement cites, without their stochastic rounding).  The reduced maps gy_u, x_u and
 * the kernel sum are held as codes; Eq. 5 and Eq. 3 are then integer contractions, exact, and the
 * caller scales the integer once by the product of the two step sizes (and 1/s^2). ---- */
/* q[i] = clip(round_half_even((float)v[i] * inv_delta), -127, 127); the product and the rounding are
 * taken in binary32, the precision in which the GPU kernels take the same decision.  A NaN gets
 * the code -127 (it fails every comparison of the clip, like minus infinity). */
int gf_ref_quantize_q8(const double* v, long n, float inv_delta, signed char* q);
/* Eq. 5 on codes: acc[c_o, c_i'] = sum over (n, patch) of x_q * gy_q.  [C_out, C_in/groups], exact. */
int gf_ref_bwd_weight_q8(const gf_ref_desc* d, const signed char* x_q, const signed char* gy_q, long long* acc);
/* Eq. 3 on codes: acc[n, c_i, patch] = sum over the group's c_o of gy_q * w_q, w_q [C_out, C_in/groups]
 * the codes of the kernel sum.  [N, C_in, H_p, W_p], exact. */
int gf_ref_bwd_input_q8(const gf_ref_desc* d, const signed char* gy_q, const signed char* w_q, long long* acc);

int gf_ref_cost_model(const gf_ref_desc* d, gf_ref_cost* out);

/* Number of threads the OpenMP build will use (1 when built without OpenMP). */
int gf_ref_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif /* GF_REF_H */
