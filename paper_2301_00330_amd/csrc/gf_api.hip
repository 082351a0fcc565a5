// C ABI of libgf: validation, workspace planning and dispatch.  Every check
// happens on the host before anything is enqueued.
#include <string.h>

#include <atomic>
#include <mutex>
#include <vector>

#include "gf_internal.h"

namespace gf {

gf_status make_geom(const gf_conv_desc* d, Geom* o) {
  if (!d) return GF_ERR_NULL;
  if (d->struct_size != sizeof(gf_conv_desc)) return GF_ERR_BAD_DESC;
  if (d->N < 1 || d->C_in < 1 || d->C_out < 1 || d->H_in < 1 || d->W_in < 1) return GF_ERR_BAD_DESC;
  if (d->K_h < 1 || d->K_w < 1 || d->stride < 1 || d->pad < 0 || d->dilation < 1)
    return GF_ERR_BAD_DESC;
  if (d->groups < 1 || d->C_in % d->groups || d->C_out % d->groups) return GF_ERR_BAD_DESC;
  if (d->r < 1) return GF_ERR_BAD_DESC;
  if (d->dtype != GF_F32 && d->dtype != GF_BF16) return GF_ERR_BAD_DESC;
  // 32-bit element indexing inside the kernels; the margin keeps the index of the last block's
  // last lane, which may point past the end before it is checked, below 2^31 as well.  Every
  // extent is bounded on its own first, so none of the products below can wrap 64 bits.
  const long lim = (1L << 31) - (1L << 20);
  if (d->N > lim || d->C_in > lim || d->C_out > lim || d->H_in > lim || d->W_in > lim || d->K_h > lim ||
      d->K_w > lim || d->pad > (1 << 30) || d->dilation > (1 << 30))
    return GF_ERR_UNSUPPORTED;
  if ((long)d->H_in * d->W_in > lim || (long)d->K_h * d->K_w > lim) return GF_ERR_UNSUPPORTED;
  Geom g;
  g.N = d->N; g.Ci = d->C_in; g.Co = d->C_out; g.H = d->H_in; g.W = d->W_in;
  g.Kh = d->K_h; g.Kw = d->K_w; g.s = d->stride; g.p = d->pad; g.dl = d->dilation;
  g.g = d->groups; g.r = d->r;
  const long eh = (long)g.H + 2L * g.p - (long)g.dl * (g.Kh - 1) - 1;
  const long ew = (long)g.W + 2L * g.p - (long)g.dl * (g.Kw - 1) - 1;
  if (eh < 0 || ew < 0) return GF_ERR_SHAPE;
  g.Hy = (int)(eh / g.s) + 1;
  g.Wy = (int)(ew / g.s) + 1;
  g.Hp = cdiv(g.Hy, g.r);
  g.Wp = cdiv(g.Wy, g.r);
  g.rx = g.r == 1 ? 1 : g.r * g.s;
  if (g.r > 1 && (cdiv(g.H, g.rx) != g.Hp || cdiv(g.W, g.rx) != g.Wp)) return GF_ERR_SHAPE;
  g.Cg = g.Ci / g.g;
  g.Og = g.Co / g.g;
  // element counts, factor by factor with an early exit (each partial product stays below 2^62)
  const long hw = (long)g.H * g.W, hwy = (long)g.Hy * g.Wy, kk = (long)g.Kh * g.Kw;
  if (hwy > lim || hw * g.Ci > lim || hwy * g.Co > lim || kk * g.Cg > lim) return GF_ERR_UNSUPPORTED;
  if (hw * g.Ci * g.N > lim || hwy * g.Co * g.N > lim || kk * g.Cg * g.Co > lim) return GF_ERR_UNSUPPORTED;
  g.KK = g.Kh * g.Kw;
  g.P = g.Hp * g.Wp;
  g.dtype = d->dtype;
  g.b = d->dtype == GF_BF16 ? 2 : 4;
  // grid dimensions y (group x channel tile) and z (image) are limited to 65535
  if (g.N > 65535 || (long)g.g * cdiv(g.Cg > g.Og ? g.Cg : g.Og, 16) > 65535) return GF_ERR_UNSUPPORTED;
  *o = g;
  return GF_OK;
}

static std::atomic<gf_launch_observer_fn> g_observer{nullptr};
static std::atomic<void*> g_observer_user{nullptr};

void observe_launch(const char* kernel_expr, int phase, hipStream_t st) {
  const gf_launch_observer_fn fn = g_observer.load(std::memory_order_relaxed);
  if (!fn) return;
  // the launch site's kernel expression, e.g. "(wgrad_mfma_k<T, TM, TN, WM, WN, true>)": keep the name
  char name[64];
  const char* p = kernel_expr;
  while (*p == '(' || *p == ' ') ++p;
  size_t n = 0;
  while (p[n] && p[n] != '<' && p[n] != ')' && p[n] != ' ' && n + 1 < sizeof(name)) { name[n] = p[n]; ++n; }
  name[n] = 0;
  fn(g_observer_user.load(std::memory_order_relaxed), name, phase, static_cast<void*>(st));
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static gf_status dev(hipError_t e) { return e == hipSuccess ? GF_OK : GF_ERR_DEVICE; }

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// layout of the fused call's workspace: [gy_u when the caller passes none][weight ws][input ws]
static size_t ws_filtered(const Geom& g, bool own_gyu, size_t* off_w, size_t* off_i) {
  if (g.r == 1) {
    if (off_w) *off_w = 0;
    if (off_i) *off_i = 0;
    return ws_exact(g, true, true);
  }
  if (dense_ok(g)) {
    if (off_w) *off_w = 0;
    if (off_i) *off_i = 0;
    return ws_dense(g, true, true);
  }
  int nz = 0;
  if (dw_fused_ok(g, &nz)) {
    if (off_w) *off_w = 0;
    if (off_i) *off_i = 0;
    return (size_t)nz * g.Ci * sizeof(float);
  }
  if (onepass_ok(g, &nz)) {
    if (off_w) *off_w = 0;
    if (off_i) *off_i = 0;
    return (size_t)nz * g.Co * g.Ci * sizeof(float);
  }
  size_t o = own_gyu ? align256((size_t)g.N * g.Co * g.P * g.b) : 0;
  if (off_w) *off_w = o;
  o += align256(ws_bwd_weight(g));
  if (off_i) *off_i = o;
  return o + ws_bwd_input(g, false);
}

// chained entry: [weight-gradient workspace][input-gradient workspace]
static size_t ws_chained(const Geom& g, size_t* off_i) {
  if (g.r == 1) {
    if (off_i) *off_i = 0;
    return ws_exact(g, true, true);
  }
  if (dense_ok(g)) {
    if (off_i) *off_i = 0;
    return ws_dense(g, true, true);
  }
  const size_t o = align256(ws_bwd_weight(g));
  if (off_i) *off_i = o;
  const size_t a = ws_bwd_input(g, true), b = ws_bwd_input(g, false);
  return o + (a > b ? a : b);
}

// one-call backward on codes: [gy_q if the caller keeps none][w_q][weight-gradient slabs][input-gradient map]
static size_t ws_filtered_q8(const Geom& g, bool own_gyq, size_t* off_wq, size_t* off_w, size_t* off_i) {
  size_t o = own_gyq ? align256((size_t)g.N * g.Co * g.P) : 0;
  if (off_wq) *off_wq = o;
  o += align256((size_t)g.Co * g.Cg);
  if (off_w) *off_w = o;
  o += align256(ws_bwd_weight_q8(g));
  if (off_i) *off_i = o;
  return o + ws_bwd_input_q8(g, false);
}

// The layer of gf_conv_bwd_unique on its patch grid: the same kernel, padding, dilation and groups on
// [N, C, H_p, W_p] maps, r = 1.  GF_ERR_SHAPE unless the padding keeps the map size.
static gf_status unique_geom(const Geom& g, Geom* red) {
  gf_conv_desc d;
  d.struct_size = sizeof(gf_conv_desc);
  d.N = g.N; d.C_in = g.Ci; d.C_out = g.Co; d.H_in = g.Hp; d.W_in = g.Wp;
  d.K_h = g.Kh; d.K_w = g.Kw; d.stride = 1; d.pad = g.p; d.dilation = g.dl; d.groups = g.g; d.r = 1;
  d.dtype = (gf_dtype)g.dtype;
  gf_status rc = make_geom(&d, red);
  if (rc) return rc;
  return (red->Hy == g.Hp && red->Wy == g.Wp) ? GF_OK : GF_ERR_SHAPE;
}

// [vanilla BP on the patch grid][the reduced g_x when full resolution is asked for]
static size_t ws_unique(const Geom& g, const Geom& red, bool want_gw, bool want_gx, bool reduced_out, size_t* off_red) {
  size_t o = align256(ws_exact(red, want_gw, want_gx));
  if (off_red) *off_red = o;
  if (want_gx && !reduced_out) o += (size_t)g.N * g.Ci * g.P * g.b;
  return o;
}

static size_t ws_need(const Geom& g, int op, bool reduced_out) {
  switch (op) {
    case GF_OP_BWD_UNIQUE: {
      Geom red;
      if (g.r == 1 || g.s != 1 || unique_geom(g, &red) != GF_OK) return ws_exact(g, true, true);
      return ws_unique(g, red, true, true, false, nullptr);
    }
    case GF_OP_BWD_FILTERED:
      return ws_filtered(g, true, nullptr, nullptr);
    case GF_OP_BWD_CHAINED:
      return ws_chained(g, nullptr);
    case GF_OP_FILTER_SNR:
      return (size_t)patch_reduce_max_blocks((long)g.N * g.Co, g.Hy, g.Wy, g.r) * 2 * sizeof(float);
    case GF_OP_BWD_WEIGHT_Q8:
      return ws_bwd_weight_q8(g);
    case GF_OP_BWD_INPUT_Q8:
      return ws_bwd_input_q8(g, reduced_out);
    case GF_OP_BWD_FILTERED_Q8:
      return ws_filtered_q8(g, true, nullptr, nullptr, nullptr);
    case GF_OP_BWD_WEIGHT:
      return g.r == 1 ? ws_exact(g, true, false) : dense_ok(g) ? ws_dense(g, true, false) : ws_bwd_weight(g);
    case GF_OP_BWD_INPUT:
      return g.r == 1 ? ws_exact(g, false, true) : dense_ok(g) ? ws_dense(g, false, true) : ws_bwd_input(g, reduced_out);
    default:
      return ws_exact(g, true, true);
  }
}

static gf_status check_ws(size_t need, const void* ws, size_t ws_bytes) {
  if (need == 0) return GF_OK;
  if (!ws || ws_bytes < need) return GF_ERR_WORKSPACE;
  if (!aligned16(ws)) return GF_ERR_UNSUPPORTED;
  return GF_OK;
}

}  // namespace gf

using namespace gf;

extern "C" {

int gf_version(void) { return 210; }

void gf_set_launch_observer(gf_launch_observer_fn fn, void* user) {
  g_observer.store(nullptr, std::memory_order_relaxed);
  g_observer_user.store(user, std::memory_order_relaxed);
  g_observer.store(fn, std::memory_order_release);
}

const char* gf_status_string(int s) {
  switch (s) {
    case GF_OK: return "GF_OK";
    case GF_ERR_NULL: return "GF_ERR_NULL: a required pointer is NULL";
    case GF_ERR_BAD_DESC: return "GF_ERR_BAD_DESC: invalid layer descriptor";
    case GF_ERR_SHAPE: return "GF_ERR_SHAPE: kernel exceeds padded input or patch grids of x and g_y differ";
    case GF_ERR_UNSUPPORTED: return "GF_ERR_UNSUPPORTED: misaligned pointer or tensor too large";
    case GF_ERR_WORKSPACE:
      return "GF_ERR_WORKSPACE: workspace missing or too small (static variant: the layer needs more than "
             "GF_STATIC_SCRATCH_BYTES)";
    case GF_ERR_DEVICE: return "GF_ERR_DEVICE: HIP launch failed";
    default: return "GF_ERR_?: unknown status";
  }
}

gf_status gf_out_shape(const gf_conv_desc* desc, int32_t* H_y, int32_t* W_y, int32_t* H_p,
                       int32_t* W_p) {
  Geom g;
  gf_status rc = make_geom(desc, &g);
  if (rc) return rc;
  if (H_y) *H_y = g.Hy;
  if (W_y) *W_y = g.Wy;
  if (H_p) *H_p = g.Hp;
  if (W_p) *W_p = g.Wp;
  return GF_OK;
}

gf_status gf_workspace_bytes(const gf_conv_desc* desc, int op, size_t* bytes) {
  if (op != GF_OP_BWD_WEIGHT && op != GF_OP_BWD_INPUT && op != GF_OP_BWD_EXACT &&
      op != GF_OP_BWD_FILTERED && op != GF_OP_BWD_CHAINED && op != GF_OP_FILTER_SNR &&
      op != GF_OP_BWD_WEIGHT_Q8 && op != GF_OP_BWD_INPUT_Q8 && op != GF_OP_BWD_FILTERED_Q8 &&
      op != GF_OP_BWD_UNIQUE)
    return GF_ERR_BAD_DESC;
  if (!desc) return GF_ERR_NULL;
  gf_conv_desc d1;
  if (desc->struct_size != sizeof(gf_conv_desc)) return GF_ERR_BAD_DESC;
  memcpy(&d1, desc, sizeof(d1));
  if (d1.r < 1) return GF_ERR_BAD_DESC;
  if (op == GF_OP_BWD_EXACT) d1.r = 1;  // the exact entry ignores the patch size
  Geom g;
  gf_status rc = make_geom(&d1, &g);
  if (rc) return rc;
  if (!bytes) return GF_ERR_NULL;
  // the full-resolution form of the input gradient needs at least as much as the reduced one
  *bytes = ws_need(g, op, false);
  return GF_OK;
}

gf_status gf_pool_activation(const gf_conv_desc* desc, const void* x, void* x_u, void* stream) {
  Geom g;
  gf_status rc = make_geom(desc, &g);
  if (rc) return rc;
  if (!x || !x_u) return GF_ERR_NULL;
  if (!aligned16(x) || !aligned16(x_u)) return GF_ERR_UNSUPPORTED;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const long planes = (long)g.N * g.Ci;
  if (g.r == 1)
    return dev(hipMemcpyAsync(x_u, x, (size_t)planes * g.H * g.W * g.b, hipMemcpyDeviceToDevice, st));
  return dev(launch_patch_reduce(x, x_u, planes, g.H, g.W, g.rx, false, g.dtype, st));
}

gf_status gf_pool_activation_batch(int32_t count, const gf_conv_desc* descs, const void* const* x, void* const* x_u,
                                   void* stream) {
  if (count < 1 || count > 4096) return GF_ERR_BAD_DESC;
  if (!descs || !x || !x_u) return GF_ERR_NULL;
  // every layer is validated before anything is enqueued
  std::vector<Geom> gs((size_t)count);
  for (int i = 0; i < count; ++i) {
    gf_status rc = make_geom(&descs[i], &gs[i]);
    if (rc) return rc;
    if (!x[i] || !x_u[i]) return GF_ERR_NULL;
    if (!aligned16(x[i]) || !aligned16(x_u[i])) return GF_ERR_UNSUPPORTED;
    if (gs[i].dtype != gs[0].dtype) return GF_ERR_UNSUPPORTED;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  std::vector<PoolJob> jobs;
  jobs.reserve((size_t)count);
  for (int i = 0; i < count; ++i) {
    const Geom& g = gs[i];
    const long planes = (long)g.N * g.Ci;
    if (g.r == 1) {   // vanilla BP keeps x itself
      gf_status rc = dev(hipMemcpyAsync(x_u[i], x[i], (size_t)planes * g.H * g.W * g.b, hipMemcpyDeviceToDevice, st));
      if (rc) return rc;
      continue;
    }
    jobs.push_back(PoolJob{x[i], x_u[i], planes, g.H, g.W, g.rx, 0.f});
  }
  if (jobs.empty()) return GF_OK;
  return dev(launch_pool_batch(jobs.data(), (int)jobs.size(), gs[0].dtype, st));
}

gf_status gf_filter_grad(const gf_conv_desc* desc, const void* g_y, void* gy_u, void* stream) {
  Geom g;
  gf_status rc = make_geom(desc, &g);
  if (rc) return rc;
  if (!g_y || !gy_u) return GF_ERR_NULL;
  if (!aligned16(g_y) || !aligned16(gy_u)) return GF_ERR_UNSUPPORTED;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const long planes = (long)g.N * g.Co;
  if (g.r == 1)
    return dev(hipMemcpyAsync(gy_u, g_y, (size_t)planes * g.Hy * g.Wy * g.b, hipMemcpyDeviceToDevice, st));
  return dev(launch_patch_reduce(g_y, gy_u, planes, g.Hy, g.Wy, g.r, true, g.dtype, st));
}

// descriptor and step-size checks common to the entry points on 8-bit codes
static gf_status q8_geom(const gf_conv_desc* desc, float factor, Geom* g) {
  gf_status rc = make_geom(desc, g);
  if (rc) return rc;
  if (!(factor > 0.f) || factor > 3.0e38f) return GF_ERR_BAD_DESC;   // also rejects NaN and infinity
  if (!q8_shape_ok(*g)) return GF_ERR_UNSUPPORTED;
  return GF_OK;
}

gf_status gf_filter_grad_q8(const gf_conv_desc* desc, const void* g_y, float inv_delta, int8_t* gy_q,
                            void* stream) {
  Geom g;
  gf_status rc = q8_geom(desc, inv_delta, &g);
  if (rc) return rc;
  if (!g_y || !gy_q) return GF_ERR_NULL;
  if (!aligned16(g_y) || !aligned16(gy_q)) return GF_ERR_UNSUPPORTED;
  return dev(launch_patch_reduce_q8(g_y, gy_q, (long)g.N * g.Co, g.Hy, g.Wy, g.r, true, inv_delta, g.dtype,
                                    static_cast<hipStream_t>(stream)));
}

gf_status gf_pool_activation_q8(const gf_conv_desc* desc, const void* x, float inv_delta, int8_t* x_q,
                                void* stream) {
  Geom g;
  gf_status rc = q8_geom(desc, inv_delta, &g);
  if (rc) return rc;
  if (!x || !x_q) return GF_ERR_NULL;
  if (!aligned16(x) || !aligned16(x_q)) return GF_ERR_UNSUPPORTED;
  return dev(launch_patch_reduce_q8(x, x_q, (long)g.N * g.Ci, g.H, g.W, g.rx, false, inv_delta, g.dtype,
                                    static_cast<hipStream_t>(stream)));
}

gf_status gf_pool_activation_batch_q8(int32_t count, const gf_conv_desc* descs, const void* const* x,
                                      const float* inv_delta, int8_t* const* x_q, void* stream) {
  if (count < 1 || count > 4096) return GF_ERR_BAD_DESC;
  if (!descs || !x || !inv_delta || !x_q) return GF_ERR_NULL;
  // every layer is validated before anything is enqueued
  std::vector<PoolJob> jobs((size_t)count);
  int dtype = GF_F32;
  for (int i = 0; i < count; ++i) {
    Geom g;
    gf_status rc = q8_geom(&descs[i], inv_delta[i], &g);
    if (rc) return rc;
    if (!x[i] || !x_q[i]) return GF_ERR_NULL;
    if (!aligned16(x[i]) || !aligned16(x_q[i])) return GF_ERR_UNSUPPORTED;
    if (i == 0) dtype = g.dtype;
    if (g.dtype != dtype) return GF_ERR_UNSUPPORTED;
    jobs[(size_t)i] = PoolJob{x[i], x_q[i], (long)g.N * g.Ci, g.H, g.W, g.rx, inv_delta[i]};
  }
  return dev(launch_pool_batch(jobs.data(), count, dtype, static_cast<hipStream_t>(stream)));
}

gf_status gf_kernel_sum_q8(const gf_conv_desc* desc, const void* w, float inv_delta, int8_t* w_q,
                           void* stream) {
  Geom g;
  gf_status rc = q8_geom(desc, inv_delta, &g);
  if (rc) return rc;
  if (!w || !w_q) return GF_ERR_NULL;
  if (!aligned16(w) || !aligned16(w_q)) return GF_ERR_UNSUPPORTED;
  return dev(launch_kernel_sum_q8(g, w, inv_delta, w_q, static_cast<hipStream_t>(stream)));
}

gf_status gf_conv_bwd_weight_q8(const gf_conv_desc* desc, const int8_t* x_q, const int8_t* gy_q, float scale,
                                float* g_w, void* ws, size_t ws_bytes, void* stream) {
  Geom g;
  gf_status rc = q8_geom(desc, scale, &g);
  if (rc) return rc;
  if (!x_q || !gy_q || !g_w) return GF_ERR_NULL;
  if (!aligned16(x_q) || !aligned16(gy_q) || !aligned16(g_w)) return GF_ERR_UNSUPPORTED;
  rc = check_ws(ws_bwd_weight_q8(g), ws, ws_bytes);
  if (rc) return rc;
  return dev(launch_bwd_weight_q8(g, x_q, gy_q, scale, g_w, ws, static_cast<hipStream_t>(stream)));
}

gf_status gf_conv_bwd_input_q8(const gf_conv_desc* desc, const int8_t* gy_q, const int8_t* w_q, float scale,
                               void* g_x, int reduced_out, void* ws, size_t ws_bytes, void* stream) {
  Geom g;
  gf_status rc = q8_geom(desc, scale, &g);
  if (rc) return rc;
  if (!gy_q || !w_q || !g_x) return GF_ERR_NULL;
  if (!aligned16(gy_q) || !aligned16(w_q) || !aligned16(g_x)) return GF_ERR_UNSUPPORTED;
  rc = check_ws(ws_bwd_input_q8(g, reduced_out != 0), ws, ws_bytes);
  if (rc) return rc;
  return dev(launch_bwd_input_q8(g, gy_q, w_q, scale, g_x, reduced_out != 0, ws, static_cast<hipStream_t>(stream)));
}

gf_status gf_conv_bwd_weight(const gf_conv_desc* desc, const void* x_u, const void* gy_u,
                             float* g_w, void* ws, size_t ws_bytes, void* stream) {
  Geom g;
  gf_status rc = make_geom(desc, &g);
  if (rc) return rc;
  if (!x_u || !gy_u || !g_w) return GF_ERR_NULL;
  if (!aligned16(x_u) || !aligned16(gy_u) || !aligned16(g_w)) return GF_ERR_UNSUPPORTED;
  rc = check_ws(ws_need(g, GF_OP_BWD_WEIGHT, false), ws, ws_bytes);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (g.r == 1) return dev(launch_exact_wgrad(g, x_u, gy_u, g_w, ws, st));
  if (dense_ok(g)) return dev(launch_dense(g, gy_u, false, x_u, nullptr, nullptr, g_w, nullptr, false, nullptr, ws, st));
  return dev(launch_gf_bwd_weight(g, x_u, gy_u, g_w, ws, st));
}

gf_status gf_conv_bwd_input(const gf_conv_desc* desc, const void* gy_u, const void* w, void* g_x,
                            int reduced_out, void* ws, size_t ws_bytes, void* stream) {
  Geom g;
  gf_status rc = make_geom(desc, &g);
  if (rc) return rc;
  if (!gy_u || !w || !g_x) return GF_ERR_NULL;
  if (!aligned16(gy_u) || !aligned16(w) || !aligned16(g_x)) return GF_ERR_UNSUPPORTED;
  rc = check_ws(ws_need(g, GF_OP_BWD_INPUT, reduced_out != 0), ws, ws_bytes);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (g.r == 1) return dev(launch_exact_dgrad(g, w, gy_u, g_x, ws, st));
  if (dense_ok(g))
    return dev(launch_dense(g, gy_u, false, nullptr, w, nullptr, nullptr, g_x, reduced_out != 0, nullptr, ws, st));
  return dev(launch_gf_bwd_input(g, gy_u, w, g_x, reduced_out != 0, ws, st));
}

// file-scope scratch of gf_conv_bwd_filtered_static: each GPU the library runs on holds its own copy
// at its own address until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the device address it returns is what launches and copies are given.
static __device__ __align__(256) unsigned char scratch[GF_STATIC_SCRATCH_BYTES];

static constexpr int kMaxDevices = 64;
static std::mutex scratch_mu;
static void* scratch_ptr[kMaxDevices];   // per device, filled on the first call with that device current

static gf_status static_scratch(void** out) {
  int devid = -1;
  if (hipGetDevice(&devid) != hipSuccess || devid < 0 || devid >= kMaxDevices) return GF_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(scratch_mu);
  if (!scratch_ptr[devid]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return GF_ERR_DEVICE;
    scratch_ptr[devid] = p;
  }
  *out = scratch_ptr[devid];
  return GF_OK;
}

static gf_status filtered_body(const gf_conv_desc* desc, const void* g_y, const void* x_u, const void* w,
                               void* gy_u, float* g_w, void* g_x, void* ws, size_t ws_bytes, bool ws_static,
                               void* stream);

gf_status gf_conv_bwd_filtered(const gf_conv_desc* desc, const void* g_y, const void* x_u,
                               const void* w, void* gy_u, float* g_w, void* g_x, void* ws,
                               size_t ws_bytes, void* stream) {
  return filtered_body(desc, g_y, x_u, w, gy_u, g_w, g_x, ws, ws_bytes, false, stream);
}

gf_status gf_conv_bwd_filtered_static(const gf_conv_desc* desc, const void* g_y, const void* x_u,
                                      const void* w, void* gy_u, float* g_w, void* g_x, void* stream) {
  return filtered_body(desc, g_y, x_u, w, gy_u, g_w, g_x, nullptr, GF_STATIC_SCRATCH_BYTES, true, stream);
}

static gf_status filtered_body(const gf_conv_desc* desc, const void* g_y, const void* x_u, const void* w,
                               void* gy_u, float* g_w, void* g_x, void* ws, size_t ws_bytes, bool ws_static,
                               void* stream) {
  Geom g;
  gf_status rc = make_geom(desc, &g);
  if (rc) return rc;
  if (!g_y || !x_u || !w || !g_w || !g_x) return GF_ERR_NULL;
  if (!aligned16(g_y) || !aligned16(x_u) || !aligned16(w) || !aligned16(gy_u) || !aligned16(g_w) ||
      !aligned16(g_x))
    return GF_ERR_UNSUPPORTED;
  size_t off_w = 0, off_i = 0;
  const size_t need = ws_filtered(g, gy_u == nullptr, &off_w, &off_i);
  if (ws_static) {  // the library's own scratch: size check first, then this device's address of it
    if (need > ws_bytes) return GF_ERR_WORKSPACE;
    rc = static_scratch(&ws);
    if (rc) return rc;
  }
  rc = check_ws(need, ws, ws_bytes);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* wsb = static_cast<char*>(ws);
  if (g.r == 1) {  // vanilla BP: x_u is x, the filtered gradient is g_y itself
    if (gy_u) {
      rc = dev(hipMemcpyAsync(gy_u, g_y, (size_t)g.N * g.Co * g.Hy * g.Wy * g.b,
                              hipMemcpyDeviceToDevice, st));
      if (rc) return rc;
    }
    if (implicit_ok(g)) return dev(launch_implicit(g, x_u, w, g_y, g_w, g_x, ws, st));
    rc = dev(launch_exact_wgrad(g, x_u, g_y, g_w, ws, st));
    if (rc) return rc;
    return dev(launch_exact_dgrad(g, w, g_y, g_x, ws, st));
  }
  if (dense_ok(g))  // small maps: filter + relayout, then both contractions with their slab sums
    return dev(launch_dense(g, g_y, true, x_u, w, gy_u, g_w, g_x, false, nullptr, ws, st));
  int nz = 0;
  if (dw_fused_ok(g, &nz)) {
    float* part = static_cast<float*>(ws);
    rc = dev(launch_dw_fused(g, g_y, x_u, w, gy_u, g_x, part, st));
    if (rc) return rc;
    return dev(launch_finalize(part, g_w, g.Ci, nz, g.KK, 1.f / ((float)g.s * (float)g.s), st));
  }
  if (onepass_ok(g, &nz)) {  // pointwise with few input channels: g_y is read once
    float* part = static_cast<float*>(ws);
    rc = dev(launch_onepass(g, g_y, x_u, w, gy_u, g_x, part, st));
    if (rc) return rc;
    return dev(launch_finalize(part, g_w, g.Co * g.Ci, nz, g.KK, 1.f, st));
  }
  void* gyu = gy_u ? gy_u : static_cast<void*>(wsb);
  const bool merged = mfma_s3s4_ok(g);
  // the kernel sums (S2) ride along with the filter launch when the merged launch needs them
  KsumJob ksum = {w, wsb + off_i, g.Co * g.Ci, g.KK};
  const bool ride = merged && g.KK > 1;
  rc = dev(launch_patch_reduce(g_y, gyu, (long)g.N * g.Co, g.Hy, g.Wy, g.r, true, g.dtype, st,
                               ride ? &ksum : nullptr));
  if (rc) return rc;
  if (merged) {  // dense: weight and input gradient share one launch
    float* part = reinterpret_cast<float*>(wsb + off_w);
    int nzs = 0;
    rc = dev(launch_mfma_s3s4(g, x_u, gyu, w, wsb + off_i, part, &nzs, g_x, st, ride));
    if (rc) return rc;
    return dev(launch_finalize(part, g_w, g.Co * g.Ci, nzs, g.KK, 1.f / ((float)g.s * (float)g.s), st));
  }
  rc = dev(launch_gf_bwd_weight(g, x_u, gyu, g_w, wsb + off_w, st));
  if (rc) return rc;
  return dev(launch_gf_bwd_input(g, gyu, w, g_x, false, wsb + off_i, st));
}

gf_status gf_pool_activation_mask(const gf_conv_desc* desc, const void* x, float hi, void* x_u, void* m_u,
                                  void* stream) {
  Geom g;
  gf_status rc = make_geom(desc, &g);
  if (rc) return rc;
  if (!x || !x_u || !m_u) return GF_ERR_NULL;
  if (!aligned16(x) || !aligned16(x_u) || !aligned16(m_u)) return GF_ERR_UNSUPPORTED;
  if (!(hi > 0.f)) return GF_ERR_BAD_DESC;
  // r == 1: patches of one pixel (x_u is x, m_u the mask itself)
  return dev(launch_pool_mask(x, x_u, m_u, (long)g.N * g.Ci, g.H, g.W, g.rx, hi, g.dtype,
                              static_cast<hipStream_t>(stream)));
}

gf_status gf_filter_grad_snr(const gf_conv_desc* desc, const void* g_y, void* gy_u, double* stats,
                             void* ws, size_t ws_bytes, void* stream) {
  Geom g;
  gf_status rc = make_geom(desc, &g);
  if (rc) return rc;
  if (!g_y || !gy_u || !stats) return GF_ERR_NULL;
  if (!aligned16(g_y) || !aligned16(gy_u) || !aligned16(stats)) return GF_ERR_UNSUPPORTED;
  rc = check_ws(ws_need(g, GF_OP_FILTER_SNR, false), ws, ws_bytes);
  if (rc) return rc;
  return dev(launch_filter_stats(g_y, gy_u, (long)g.N * g.Co, g.Hy, g.Wy, g.r, g.dtype,
                                 static_cast<float*>(ws), stats, static_cast<hipStream_t>(stream)));
}

// *mask_done: the launches have already multiplied the reduced g_x by mask_u
static gf_status chained_body(const Geom& g, const void* gy_u, const void* x_u, const void* w, float* g_w,
                              void* g_x, int reduced_out, const void* mask_u, bool* mask_done, void* ws,
                              size_t ws_bytes, void* stream);

gf_status gf_conv_bwd_chained(const gf_conv_desc* desc, const void* gy_u, const void* x_u,
                              const void* w, float* g_w, void* g_x, int reduced_out, const void* mask_u,
                              void* ws, size_t ws_bytes, void* stream) {
  Geom g;
  gf_status rc = make_geom(desc, &g);
  if (rc) return rc;
  if (!gy_u || !x_u || !w || !g_w || !g_x) return GF_ERR_NULL;
  if (!aligned16(gy_u) || !aligned16(x_u) || !aligned16(w) || !aligned16(g_w) || !aligned16(g_x) ||
      !aligned16(mask_u))
    return GF_ERR_UNSUPPORTED;
  // the mask fraction exists on the patch grid only: a full-resolution g_x cannot take it
  if (mask_u && g.r > 1 && !reduced_out) return GF_ERR_UNSUPPORTED;
  bool mask_done = false;
  rc = chained_body(g, gy_u, x_u, w, g_w, g_x, reduced_out, mask_u, &mask_done, ws, ws_bytes, stream);
  if (rc || !mask_u || mask_done) return rc;
  const long n = g.r == 1 ? (long)g.N * g.Ci * g.H * g.W : (long)g.N * g.Ci * g.P;
  return dev(launch_mask_mul(g_x, mask_u, n, g.dtype, static_cast<hipStream_t>(stream)));
}

static gf_status chained_body(const Geom& g, const void* gy_u, const void* x_u, const void* w, float* g_w,
                              void* g_x, int reduced_out, const void* mask_u, bool* mask_done, void* ws,
                              size_t ws_bytes, void* stream) {
  gf_status rc;
  size_t off_i = 0;
  rc = check_ws(ws_chained(g, &off_i), ws, ws_bytes);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* wsb = static_cast<char*>(ws);
  const float scale = 1.f / ((float)g.s * (float)g.s);
  if (g.r == 1) {  // the maps are the full maps: vanilla BP
    if (implicit_ok(g)) return dev(launch_implicit(g, x_u, w, gy_u, g_w, g_x, ws, st));
    rc = dev(launch_exact_wgrad(g, x_u, gy_u, g_w, ws, st));
    if (rc) return rc;
    return dev(launch_exact_dgrad(g, w, gy_u, g_x, ws, st));
  }
  if (dense_ok(g)) {
    *mask_done = reduced_out != 0;
    return dev(launch_dense(g, gy_u, false, x_u, w, nullptr, g_w, g_x, reduced_out != 0,
                            reduced_out ? mask_u : nullptr, ws, st));
  }
  if (reduced_out && is_depthwise_layer(g)) {  // one pass over gy_u and x_u
    float* part = reinterpret_cast<float*>(wsb);
    rc = dev(launch_dw_chain(g, x_u, gy_u, w, part, g_x, mask_u, st));
    *mask_done = true;
    if (rc) return rc;
    return dev(launch_finalize(part, g_w, g.Ci, g.N, g.KK, scale, st));
  }
  if (mfma_s3s4_ok(g, reduced_out != 0)) {  // dense: both contractions in one launch
    float* part = reinterpret_cast<float*>(wsb);
    int nzs = 0;
    rc = dev(launch_mfma_s3s4(g, x_u, gy_u, w, wsb + off_i, part, &nzs, g_x, st, false, reduced_out != 0,
                              reduced_out ? mask_u : nullptr));
    *mask_done = reduced_out != 0;
    if (rc) return rc;
    return dev(launch_finalize(part, g_w, g.Co * g.Ci, nzs, g.KK, scale, st));
  }
  rc = dev(launch_gf_bwd_weight(g, x_u, gy_u, g_w, wsb, st));
  if (rc) return rc;
  return dev(launch_gf_bwd_input(g, gy_u, w, g_x, reduced_out != 0, wsb + off_i, st));
}

gf_status gf_conv_bwd_filtered_q8(const gf_conv_desc* desc, const void* g_y, float inv_delta_gy,
                                  const int8_t* x_q, const void* w, float inv_delta_w, float scale_w,
                                  float scale_x, int8_t* gy_q, float* g_w, void* g_x, void* ws,
                                  size_t ws_bytes, void* stream) {
  Geom g;
  gf_status rc = q8_geom(desc, inv_delta_gy, &g);
  if (rc) return rc;
  for (float f : {inv_delta_w, scale_w, scale_x})
    if (!(f > 0.f) || f > 3.0e38f) return GF_ERR_BAD_DESC;
  if (!g_y || !x_q || !w || !g_w || !g_x) return GF_ERR_NULL;
  if (!aligned16(g_y) || !aligned16(x_q) || !aligned16(w) || !aligned16(gy_q) || !aligned16(g_w) || !aligned16(g_x))
    return GF_ERR_UNSUPPORTED;
  size_t off_wq = 0, off_w = 0, off_i = 0;
  rc = check_ws(ws_filtered_q8(g, gy_q == nullptr, &off_wq, &off_w, &off_i), ws, ws_bytes);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* wsb = static_cast<char*>(ws);
  int8_t* gq = gy_q ? gy_q : reinterpret_cast<int8_t*>(wsb);
  int8_t* wq = reinterpret_cast<int8_t*>(wsb + off_wq);
  // the codes of the kernel sums ride along with the filter launch
  KsumJob ksum = {w, wq, g.Co * g.Cg, g.KK, inv_delta_w};
  rc = dev(launch_patch_reduce_q8(g_y, gq, (long)g.N * g.Co, g.Hy, g.Wy, g.r, true, inv_delta_gy, g.dtype, st, &ksum));
  if (rc) return rc;
  rc = dev(launch_bwd_weight_q8(g, x_q, gq, scale_w, g_w, wsb + off_w, st));
  if (rc) return rc;
  return dev(launch_bwd_input_q8(g, gq, wq, scale_x, g_x, false, wsb + off_i, st));
}

gf_status gf_conv_bwd_exact(const gf_conv_desc* desc, const void* x, const void* w,
                            const void* g_y, float* g_w, void* g_x, void* ws, size_t ws_bytes,
                            void* stream) {
  if (!desc) return GF_ERR_NULL;
  gf_conv_desc d1;
  if (desc->struct_size != sizeof(gf_conv_desc)) return GF_ERR_BAD_DESC;
  memcpy(&d1, desc, sizeof(d1));
  if (d1.r < 1) return GF_ERR_BAD_DESC;
  d1.r = 1;  // the exact entry ignores the patch size
  Geom g;
  gf_status rc = make_geom(&d1, &g);
  if (rc) return rc;
  if (!g_y || (!g_w && !g_x)) return GF_ERR_NULL;
  if ((g_w && !x) || (g_x && !w)) return GF_ERR_NULL;
  if (!aligned16(g_y) || !aligned16(x) || !aligned16(w) || !aligned16(g_w) || !aligned16(g_x))
    return GF_ERR_UNSUPPORTED;
  rc = check_ws(ws_exact(g, g_w != nullptr, g_x != nullptr), ws, ws_bytes);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (implicit_ok(g)) return dev(launch_implicit(g, x, w, g_y, g_w, g_x, ws, st));
  if (g_w) {
    rc = dev(launch_exact_wgrad(g, x, g_y, g_w, ws, st));
    if (rc) return rc;
  }
  if (g_x) rc = dev(launch_exact_dgrad(g, w, g_y, g_x, ws, st));
  return rc;
}

gf_status gf_conv_bwd_unique(const gf_conv_desc* desc, const void* gy_u, const void* x_u, const void* w,
                             float* g_w, void* g_x, int reduced_out, void* ws, size_t ws_bytes,
                             void* stream) {
  Geom g;
  gf_status rc = make_geom(desc, &g);
  if (rc) return rc;
  if (g.r == 1)   // no reduced maps: x_u is x, gy_u is g_y
    return gf_conv_bwd_exact(desc, x_u, w, gy_u, g_w, g_x, ws, ws_bytes, stream);
  if (g.s != 1) return GF_ERR_UNSUPPORTED;
  Geom red;
  rc = unique_geom(g, &red);
  if (rc) return rc;
  if (!gy_u || (!g_w && !g_x)) return GF_ERR_NULL;
  if ((g_w && !x_u) || (g_x && !w)) return GF_ERR_NULL;
  if (!aligned16(gy_u) || !aligned16(x_u) || !aligned16(w) || !aligned16(g_w) || !aligned16(g_x))
    return GF_ERR_UNSUPPORTED;
  size_t off_red = 0;
  const bool full = g_x && !reduced_out;
  rc = check_ws(ws_unique(g, red, g_w != nullptr, g_x != nullptr, reduced_out != 0, &off_red), ws, ws_bytes);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* wsb = static_cast<char*>(ws);
  void* gxu = full ? static_cast<void*>(wsb + off_red) : g_x;
  if (implicit_ok(red)) {
    rc = dev(launch_implicit(red, x_u, w, gy_u, g_w, gxu, ws, st));
  } else {
    if (g_w) rc = dev(launch_exact_wgrad(red, x_u, gy_u, g_w, ws, st));
    if (!rc && g_x) rc = dev(launch_exact_dgrad(red, w, gy_u, gxu, ws, st));
  }
  if (rc || !full) return rc;
  return dev(launch_replicate(g, gxu, g_x, st));
}

gf_status gf_cost_model(const gf_conv_desc* desc, gf_cost* out) {
  Geom g;
  gf_status rc = make_geom(desc, &g);
  if (rc) return rc;
  if (!out) return GF_ERR_NULL;
  const double Cx = g.Ci, Cy = g.Co, KK = g.KK, b = g.b;
  const double HWx = (double)g.H * g.W, HWy = (double)g.Hy * g.Wy, P = g.P, N = g.N;
  const double wel = Cy * g.Cg * KK;
  out->flops_exact_gx = 2.0 * Cx * Cy * HWy * KK;
  out->flops_gf_gx = P * Cx * (2.0 * Cy - 1.0);
  out->flops_gf_min = 2.0 * Cx * Cy - Cx;
  out->overhead_fwd = 1.0 / (2.0 * Cy * KK);
  out->overhead_bwd = ((double)g.r * g.r - 1.0) / (2.0 * Cx);
  out->act_elems_exact = Cx * HWx;
  const double Px = g.r == 1 ? HWx : P;  // x_u keeps x's resolution for r == 1
  out->act_elems_gf = Cx * Px;
  out->bytes_pool = b * N * Cx * (HWx + Px);
  out->bytes_filter = b * N * Cy * (HWy + P);
  out->bytes_bwd_weight = b * N * (Cx * Px + Cy * P) + 4.0 * wel;
  out->bytes_bwd_input = b * N * Cy * P + b * wel + b * N * Cx * HWx;
  out->bytes_exact = b * N * (Cx * HWx + Cy * HWy) + b * wel + 4.0 * wel + b * N * Cx * HWx;
  out->flops_bwd_weight = 2.0 * N * P * Cy * g.Cg;
  out->flops_bwd_input = 2.0 * N * P * Cy * g.Cg;
  out->flops_exact = 4.0 * N * Cy * g.Cg * KK * HWy;
  return GF_OK;
}

}  // extern "C"
