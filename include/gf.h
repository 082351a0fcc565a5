/*
 * gf.h -- C ABI of libgf: gradient-filtered convolution backward on AMD MI355X
 * (gfx950), after "Efficient On-device Training via Gradient Filtering"
 * (arXiv 2301.00330).
 *
 * The method (Sec. 3): the output gradient g_y of a conv layer is replaced by
 * its r x r patch averages (Eq. 2) and only one value per patch is kept; the
 * stored forward input x is replaced by its patch sums (text after Eq. 5); the
 * kernel theta by its spatial sum (text after Eq. 3).  The layer's gradients
 * then are two small channel contractions on maps that are r^2 smaller:
 *   g_x~[n,ci,h,w]     = 1/s^2 * sum_co gy_u[n,co,h/r_x,w/r_x] * sum_uv theta[co,ci,u,v]   (Eq. 3)
 *   g_th~[co,ci,u,v]   = 1/s^2 * sum_{n,patch} x_u[n,ci,patch] * gy_u[n,co,patch]          (Eq. 5)
 *
 * Conventions common to every entry point
 *  - Tensors are contiguous NCHW (the paper's index order x[n,c,h,w],
 *    theta[co,ci,u,v]), element type desc->dtype (fp32, or bf16 stored as the
 *    upper 16 bits of an fp32, rounded to nearest even).  Weight gradients are
 *    always fp32.  Accumulation is always fp32.  Rounding points with bf16
 *    storage: the reduced maps x_u and gy_u are rounded once when they are formed
 *    (also inside gf_conv_bwd_filtered, where gy_u never leaves the chip for some
 *    layers); for dense layers with a kernel larger than 1x1 the kernel sum is
 *    rounded once before Eq. 3 (depthwise layers keep it in fp32); g_x is rounded
 *    once when it is stored.
 *  - Every tensor / workspace pointer is a DEVICE pointer, 16-byte aligned,
 *    owned by the caller; the library never allocates, frees or keeps one.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue work on it: they never synchronise and never throw.
 *    The device that owns the stream and the pointers must be the calling
 *    thread's current device.  The library keeps no state, so calls from
 *    several threads or on several streams need no locking as long as their
 *    outputs and workspaces do not overlap; every call may be stream-captured.
 *  - The return value is a gf_status.  Descriptor, pointer, shape and workspace
 *    errors are detected on the host BEFORE anything is enqueued, so a failed
 *    call has no effect on the device.  GF_ERR_DEVICE reports a failed launch.
 *  - Shapes: with (H_y, W_y, H_p, W_p) from gf_out_shape,
 *      x    [N, C_in,  H_in, W_in]        g_y  [N, C_out, H_y, W_y]
 *      w    [C_out, C_in/groups, K_h, K_w] g_w  same shape as w, fp32
 *      x_u  [N, C_in,  H_p, W_p]          gy_u [N, C_out, H_p, W_p]
 *      g_x  [N, C_in,  H_in, W_in]  (or [N, C_in, H_p, W_p] with reduced_out)
 *    The patch grid is H_p = ceil(H_y / r) (Sec. 3.3); a ragged last patch
 *    averages / sums its in-bounds pixels only.  On the input side the patch is
 *    r_x = r * stride, and the layer must satisfy ceil(H_in / r_x) == H_p
 *    (true for every "same"-padded layer), else GF_ERR_SHAPE.
 *  - r == 1 means vanilla back-propagation (Sec. 4.2): x_u and gy_u are then
 *    the full maps x and g_y (x_u is [N, C_in, H_in, W_in]), the two reduction
 *    entries are plain copies, and gf_conv_bwd_weight / gf_conv_bwd_input /
 *    gf_conv_bwd_filtered / gf_conv_bwd_chained evaluate the exact K_h x K_w
 *    contractions of Sec. 3.1.
 *  - Dilation only affects H_y and the exact entry: the filtered formulas read
 *    the tap's own padded patch wherever it lands (Supp. B "Boundary Elements").
 *  - Results are deterministic: no floating-point atomics, so two calls on the
 *    same inputs give bit-identical outputs.
 */
#ifndef GF_H
#define GF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum gf_status {
  GF_OK = 0,
  GF_ERR_NULL = 1,        /* a required pointer is NULL                              */
  GF_ERR_BAD_DESC = 2,    /* non-positive size, r < 1, groups not dividing channels,
                             unknown dtype, wrong struct_size                        */
  GF_ERR_SHAPE = 3,       /* kernel larger than the padded input, or the patch grids
                             of x and g_y differ                                     */
  GF_ERR_UNSUPPORTED = 4, /* legal but not implemented (e.g. a misaligned pointer,
                             more than 2^31 - 2^20 elements in one tensor)           */
  GF_ERR_WORKSPACE = 5,   /* ws is NULL or smaller than gf_workspace_bytes says      */
  GF_ERR_DEVICE = 6       /* the HIP runtime refused a launch                        */
} gf_status;

typedef enum gf_dtype { GF_F32 = 0, GF_BF16 = 1 } gf_dtype;

typedef enum gf_op {
  GF_OP_BWD_WEIGHT = 0,
  GF_OP_BWD_INPUT = 1,
  GF_OP_BWD_EXACT = 2,
  GF_OP_BWD_FILTERED = 3,
  GF_OP_BWD_CHAINED = 4,
  GF_OP_FILTER_SNR = 5,
  GF_OP_BWD_WEIGHT_Q8 = 6,
  GF_OP_BWD_INPUT_Q8 = 7,
  GF_OP_BWD_FILTERED_Q8 = 8,
  GF_OP_BWD_UNIQUE = 9
} gf_op;

/* Plain-old-data layer descriptor in the paper's symbols (Table of symbols,
 * Sec. 3); set struct_size = sizeof(gf_conv_desc). */
typedef struct gf_conv_desc {
  uint32_t struct_size;
  int32_t N, C_in, C_out, H_in, W_in; /* x: [N, C_in, H_in, W_in]                   */
  int32_t K_h, K_w, stride, pad, dilation, groups;
  int32_t r;                          /* patch size on g_y; 1 = vanilla BP          */
  int32_t dtype;                      /* gf_dtype of x, w, g_y, g_x, x_u, gy_u      */
} gf_conv_desc;

/* Closed forms of the paper for one layer (host only). FLOPs and stored
 * activation counts are per image; the byte counts are this library's
 * algorithmic HBM traffic for the whole batch (each tensor read or written
 * once by the step that owns it). */
typedef struct gf_cost {
  double flops_exact_gx;  /* Eq. (1)                                                */
  double flops_gf_gx;     /* Eq. (12), leading term                                 */
  double flops_gf_min;    /* Eq. (13), leading term                                 */
  double overhead_fwd;    /* Sec. 4.2 "Overhead": 1 / (2 C_o W_th H_th)             */
  double overhead_bwd;    /* Sec. 4.2 "Overhead": (r^2 - 1) / (2 C_x)               */
  double act_elems_exact; /* Sec. 4.3: stored values of x per image                 */
  double act_elems_gf;    /* Sec. 4.3: stored values of x_u per image               */
  double bytes_pool;      /* gf_pool_activation: read x, write x_u                  */
  double bytes_filter;    /* gf_filter_grad: read g_y, write gy_u                   */
  double bytes_bwd_weight;/* read x_u and gy_u, write g_w                           */
  double bytes_bwd_input; /* read gy_u and w, write g_x (full resolution)           */
  double bytes_exact;     /* read x, w, g_y; write g_w and g_x                      */
  double flops_bwd_weight;/* 2 N P C_out C_in/groups                                */
  double flops_bwd_input; /* 2 N P C_out C_in/groups                                */
  double flops_exact;     /* 4 N C_out (C_in/groups) K_h K_w H_y W_y                */
} gf_cost;

/* Output map and patch grid of the layer (Sec. 3.3).  Any out pointer may be
 * NULL.  Host only. */
gf_status gf_out_shape(const gf_conv_desc* desc, int32_t* H_y, int32_t* W_y, int32_t* H_p,
                       int32_t* W_p);

/* Scratch bytes `op` needs for this layer (may be 0).  Host only. */
gf_status gf_workspace_bytes(const gf_conv_desc* desc, int op, size_t* bytes);

/* Forward-time pooling of the activation (text after Eq. 5; Fig. 2(a) lower
 * half): x_u = sum of x over each r_x x r_x patch.  x_u is what a training
 * loop keeps for the backward pass instead of x (Sec. 4.3). */
gf_status gf_pool_activation(const gf_conv_desc* desc, const void* x, void* x_u, void* stream);

/* gf_pool_activation for `count` layers in ONE launch (a training step that holds the inputs of several
 * layers, e.g. a recomputed block, pools them together: the small tensors of a network's tail are a few
 * microseconds of work each and a launch costs as much).  descs: HOST array of `count` descriptors; x, x_u:
 * HOST arrays of `count` device pointers.  Every x_u[i] is bit-identical to what gf_pool_activation writes
 * for descs[i].  All layers must share one dtype (else GF_ERR_UNSUPPORTED); layers with r == 1 are copied.
 * count < 1 or > 4096: GF_ERR_BAD_DESC.  Nothing is enqueued unless every layer passes validation. */
gf_status gf_pool_activation_batch(int32_t count, const gf_conv_desc* descs, const void* const* x,
                                   void* const* x_u, void* stream);

/* The same for a layer whose input x is the output of a ReLU (hi = +infinity) or of a clipped
 * ReLU (hi = 6 for ReLU6), for chains of filtered layers (see gf_conv_bwd_chained): beside x_u
 * it writes m_u [N, C_in, H_p, W_p] (storage type), the share of each patch's in-bounds pixels
 * with 0 < x < hi, i.e. the patch average of the gradient mask of that non-linearity.  Eq. 2
 * of the layer below, applied to this layer's patch-constant input gradient (Eq. 3) times the
 * mask, is that gradient's one value per patch times m_u.  hi <= 0 or NaN: GF_ERR_BAD_DESC.
 * With r == 1, x_u is a copy of x and m_u the mask itself, [N, C_in, H_in, W_in]. */
gf_status gf_pool_activation_mask(const gf_conv_desc* desc, const void* x, float hi, void* x_u, void* m_u,
                                  void* stream);

/* The gradient filter (Eq. 2): gy_u = mean of g_y over each r x r patch, one
 * value per patch (the matrix of unique values, Sec. 3.3). */
gf_status gf_filter_grad(const gf_conv_desc* desc, const void* g_y, void* gy_u, void* stream);

/* The gradient filter together with its noise figures (Sec. 3.4, first line of Eq. 8 read in the
 * pixel domain by Parseval; Fig. 5 plots accuracy against this ratio): beside gy_u the call
 * writes, to two doubles in device memory,
 *   stats[0] = sum over the tensor of g_y^2                      (energy of the signal)
 *   stats[1] = sum of (g_y - mean of its patch)^2                (energy the filter removes)
 * so that SNR = stats[0] / stats[1].  The means are the unrounded fp32 patch means; partial
 * sums are added in a fixed order (deterministic).  ws: gf_workspace_bytes(GF_OP_FILTER_SNR). */
gf_status gf_filter_grad_snr(const gf_conv_desc* desc, const void* g_y, void* gy_u, double* stats,
                             void* ws, size_t ws_bytes, void* stream);

/* Filtered weight gradient (Eq. 5): the Frobenius inner product of x_u and gy_u
 * over (n, patch) for every (c_o, c_i) pair of a group, scaled by 1/stride^2 and
 * written to all K_h*K_w taps (they are bit-identical).  g_w is fp32. */
gf_status gf_conv_bwd_weight(const gf_conv_desc* desc, const void* x_u, const void* gy_u,
                             float* g_w, void* ws, size_t ws_bytes, void* stream);

/* Filtered input gradient (Eq. 3): sum over the group's c_o of gy_u times the
 * spatial sum of the kernel, scaled by 1/stride^2; every pixel of an input-side
 * patch receives its patch's value (bit-identical), or, with reduced_out != 0,
 * only the one value per patch is written ([N, C_in, H_p, W_p]). */
gf_status gf_conv_bwd_input(const gf_conv_desc* desc, const void* gy_u, const void* w, void* g_x,
                            int reduced_out, void* ws, size_t ws_bytes, void* stream);

/* The whole backward of one layer under gradient filtering in one call (lower half
 * of Fig. 2(a)): the gradient filter on g_y (Eq. 2), then the weight gradient
 * (Eq. 5) from the stored x_u and the input gradient (Eq. 3) from w.  Same results
 * as gf_filter_grad + gf_conv_bwd_weight + gf_conv_bwd_input: gy_u and g_x bit for
 * bit, g_w up to the order of the fp32 partial sums.  For depthwise layers and for
 * pointwise stride-1 layers with at most 32 input channels it is a single pass over
 * g_y; other dense layers run the filter and then both contractions in one launch;
 * the remaining layers run the three steps back to back.
 * gy_u may be NULL if the caller does not want the filtered gradient itself.  With r == 1, x_u is x and
 * the call is vanilla back-propagation. */
gf_status gf_conv_bwd_filtered(const gf_conv_desc* desc, const void* g_y, const void* x_u,
                               const void* w, void* gy_u, float* g_w, void* g_x, void* ws,
                               size_t ws_bytes, void* stream);

/* gf_conv_bwd_filtered for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * minus the workspace, same kernels, same results bit for bit.  The scratch (partial weight
 * gradients, kernel sums, gy_u when the caller passes none) lives in a static device array of
 * GF_STATIC_SCRATCH_BYTES inside the library; every GPU the library runs on holds its own copy
 * until the process ends.  A layer whose gf_workspace_bytes(GF_OP_BWD_FILTERED) exceeds that size
 * is rejected with GF_ERR_WORKSPACE before anything is enqueued.  The call allocates nothing and
 * frees nothing; the first call on a device looks the array's address up once (make that call
 * outside a stream capture).  All calls on one GPU share the one array and it keeps the last
 * call's contents: calls that overlap in time on the same GPU (different streams or threads)
 * race -- serialise them or use gf_conv_bwd_filtered with workspaces of their own.  Nothing in
 * the array has to start at zero. */
#define GF_STATIC_SCRATCH_BYTES (64u << 20)
gf_status gf_conv_bwd_filtered_static(const gf_conv_desc* desc, const void* g_y, const void* x_u,
                                      const void* w, void* gy_u, float* g_w, void* g_x, void* stream);

/* Backward of one layer inside a chain of gradient-filtered layers with nothing but
 * convolutions between them.  The input gradient of Eq. 3 is constant on every
 * input-side patch, so the filter of the layer below (Eq. 2, patch size r * stride of
 * this layer) would return exactly the one value per patch that this layer computed:
 * such layers can hand each other reduced maps only.  gy_u [N, C_out, H_p, W_p] is the
 * incoming filtered gradient (from gf_filter_grad at the top of the chain, else the
 * g_x of the layer above); the call computes g_w (Eq. 5) and g_x (Eq. 3), with
 * reduced_out != 0 as the reduced map [N, C_in, H_p, W_p] to pass on, else at full
 * resolution.  Same results as gf_conv_bwd_weight + gf_conv_bwd_input (g_x bit for
 * bit, g_w up to the order of the fp32 partial sums); fewer launches, and neither the
 * full-resolution write nor the next layer's read of it.  mask_u (NULL: none) is the m_u of
 * gf_pool_activation_mask for this layer's input: with a (clipped) ReLU below this layer the
 * reduced g_x is multiplied by it (product formed in fp32, rounded once), which is what the
 * filter of the layer below would return for the masked gradient.  It needs reduced_out != 0
 * (or r == 1, where it is the full mask); else GF_ERR_UNSUPPORTED. */
gf_status gf_conv_bwd_chained(const gf_conv_desc* desc, const void* gy_u, const void* x_u,
                              const void* w, float* g_w, void* g_x, int reduced_out, const void* mask_u,
                              void* ws, size_t ws_bytes, void* stream);

/* ---- Gradient filtering on signed 8-bit codes.  Supp. H combines the method with 8-bit
 * gradient quantisation and fixes no quantiser; the reading taken here is the per-tensor scheme
 * of the 8-bit training methods it cites, without their stochastic rounding: a tensor v is held
 * as codes q = clip(round_half_even(v * inv_delta), -127, 127) with ONE step size delta = 1 /
 * inv_delta that the caller chooses (e.g. a running max|v| / 127).  The reduced maps and the
 * kernel sum are held as codes, Eq. 5 and Eq. 3 become integer contractions, which are exact,
 * and the integer is scaled once: `scale` is the product of the two step sizes, the library
 * multiplies by 1/stride^2.  Codes are int8 tensors in the layout of the map they stand for,
 * 16-byte aligned.  r == 1 (no reduced maps) and inv_delta <= 0: GF_ERR_UNSUPPORTED /
 * GF_ERR_BAD_DESC.  The product and the rounding of the code are taken in fp32; a NaN gets the
 * code -127. ---- */

/* S1 with code output: gy_q [N, C_out, H_p, W_p] = codes of the r x r patch means of g_y (Eq. 2). */
gf_status gf_filter_grad_q8(const gf_conv_desc* desc, const void* g_y, float inv_delta, int8_t* gy_q,
                            void* stream);

/* S0 with code output: x_q [N, C_in, H_p, W_p] = codes of the r_x x r_x patch sums of x. */
gf_status gf_pool_activation_q8(const gf_conv_desc* desc, const void* x, float inv_delta, int8_t* x_q,
                                void* stream);

/* gf_pool_activation_q8 for `count` layers (1 ... 4096) in one launch; host arrays as in
 * gf_pool_activation_batch plus one step-size reciprocal per layer.  All layers must have the same
 * dtype (else GF_ERR_UNSUPPORTED).  x_q[i] is bit-identical to gf_pool_activation_q8's. */
gf_status gf_pool_activation_batch_q8(int32_t count, const gf_conv_desc* descs, const void* const* x,
                                      const float* inv_delta, int8_t* const* x_q, void* stream);

/* S2 with code output: w_q [C_out, C_in/groups] = codes of the spatial kernel sums (text after Eq. 3). */
gf_status gf_kernel_sum_q8(const gf_conv_desc* desc, const void* w, float inv_delta, int8_t* w_q,
                           void* stream);

/* Eq. 5 on codes: g_w[c_o, c_i, all taps] = float(sum over (n, patch) of x_q * gy_q) * scale / stride^2,
 * the integer sum exact (64 bits), converted and scaled in fp32.  ws: GF_OP_BWD_WEIGHT_Q8. */
gf_status gf_conv_bwd_weight_q8(const gf_conv_desc* desc, const int8_t* x_q, const int8_t* gy_q, float scale,
                                float* g_w, void* ws, size_t ws_bytes, void* stream);

/* Eq. 3 on codes: g_x = float(sum over the group's c_o of gy_q * w_q) * scale / stride^2, rounded once
 * to the storage type; every pixel of an input-side patch receives its patch's value, or, with
 * reduced_out != 0, one value per patch is written ([N, C_in, H_p, W_p]).  ws: GF_OP_BWD_INPUT_Q8. */
gf_status gf_conv_bwd_input_q8(const gf_conv_desc* desc, const int8_t* gy_q, const int8_t* w_q, float scale,
                               void* g_x, int reduced_out, void* ws, size_t ws_bytes, void* stream);

/* The backward of a layer on codes in one call: gy_q = codes of the patch means of g_y (step size
 * 1 / inv_delta_gy), w_q = codes of the kernel sums of w (1 / inv_delta_w), then Eq. 5 on x_q and gy_q
 * (scale_w = step of x_q times step of gy_q) and Eq. 3 on gy_q and w_q (scale_x = step of gy_q times
 * step of w_q) at full resolution -- the results of gf_filter_grad_q8, gf_kernel_sum_q8,
 * gf_conv_bwd_weight_q8 and gf_conv_bwd_input_q8 called one after the other, bit for bit, in fewer
 * launches (the kernel sums ride along with the filter launch).  x_q comes from gf_pool_activation_q8
 * at forward time.  gy_q may be NULL (the codes then live in the workspace only).
 * ws: gf_workspace_bytes(GF_OP_BWD_FILTERED_Q8). */
gf_status gf_conv_bwd_filtered_q8(const gf_conv_desc* desc, const void* g_y, float inv_delta_gy,
                                  const int8_t* x_q, const void* w, float inv_delta_w, float scale_w,
                                  float scale_x, int8_t* gy_q, float* g_w, void* g_x, void* ws,
                                  size_t ws_bytes, void* stream);

/* Vanilla back-propagation of the layer (Sec. 3.1): g_w = g_y (F) x and
 * g_x = g_y (*) rot180(w), zero padding, with stride, dilation and groups.
 * The reference the filtered path approximates and the speed-up denominator.
 * g_w or g_x may be NULL to skip that gradient (x resp. w may then be NULL). */
gf_status gf_conv_bwd_exact(const gf_conv_desc* desc, const void* x, const void* w,
                            const void* g_y, float* g_w, void* g_x, void* ws, size_t ws_bytes,
                            void* stream);

/* Closed forms of Sec. 3.2, 4.2, 4.3 plus the byte / FLOP model.  Host only. */
/* "Fewer unique elements" alone (Sec. 4.2, the middle cost line of Fig. 3): the gradient map is
 * replaced by its one value per patch, the K x K kernel is kept, and the backward runs on the r^2
 * times smaller maps as it stands -- vanilla BP (Sec. 3.1) of the same kernel, padding and dilation on
 * the patch grid, with x_u (patch sums, gf_pool_activation) for x and gy_u (patch means,
 * gf_filter_grad) for g_y:
 *   g_w[c_o, c_i, u, v] = sum over (n, patch) of x_u[n, c_i, patch + tap (u, v)] * gy_u[n, c_o, patch]
 *   g_x[n, c_i, pixel]  = sum over (c_o, u, v) of w[c_o, c_i, u, v] * gy_u[n, c_o, patch(pixel) - tap (u, v)]
 * every pixel of a patch receiving its patch's value, or, with reduced_out != 0, one value per patch
 * ([N, C_in, H_p, W_p]).  For 1 x 1 kernels this is gf_conv_bwd_weight / gf_conv_bwd_input; with r == 1
 * it is gf_conv_bwd_exact.  Stride-1 layers whose padding keeps the map size (2 pad = dilation (K - 1))
 * only: GF_ERR_UNSUPPORTED for stride > 1, GF_ERR_SHAPE otherwise.  g_w or g_x may be NULL.
 * ws: gf_workspace_bytes(GF_OP_BWD_UNIQUE). */
gf_status gf_conv_bwd_unique(const gf_conv_desc* desc, const void* gy_u, const void* x_u, const void* w,
                             float* g_w, void* g_x, int reduced_out, void* ws, size_t ws_bytes,
                             void* stream);

gf_status gf_cost_model(const gf_conv_desc* desc, gf_cost* out);

const char* gf_status_string(int status);

/* Tracing aid (process-wide; NULL removes it): `fn` is called on the calling thread right before
 * (phase 0) and right after (phase 1) every kernel any entry point enqueues, with the kernel's name
 * and the stream, e.g. to record events around each launch or to list the launches of a call.  The
 * observer must not call into this library.  Not meant to stay set in production loops. */
typedef void (*gf_launch_observer_fn)(void* user, const char* kernel, int phase, void* stream);
void gf_set_launch_observer(gf_launch_observer_fn fn, void* user);

/* Library version: major * 10000 + minor * 100 + patch. */
int gf_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GF_H */
