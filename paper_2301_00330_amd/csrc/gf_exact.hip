// Vanilla back-propagation of a conv layer (Sec. 3.1): g_theta = g_y (F) x and
// g_x = g_y (*) rot180(theta), with stride, zero padding, dilation and groups.
//  * dense layers whose tap offsets are constant in flattened pixels ("same"-size stride 1,
//    "same"-padded strided layers) are handed to the implicit-GEMM kernels (gf_implicit.hip);
//  * other dense layers: the shifted operand is written once per tap to a column tensor in
//    the workspace and the MFMA GEMMs of the filtered path do the contractions;
//  * depthwise layers whose planes fit LDS: plane-staged kernels (gf_dwexact.hip);
//  * other grouped layers: shape-generic direct kernels, one lane per g_x element
//    (gather over the taps that reach it) and one block per weight-gradient element.
#include "gf_internal.h"

namespace gf {

namespace {

constexpr int kThreads = 256;

struct ExactArgs {
  const void* x;
  const void* w;
  const void* gy;
  void* gx;
  float* gw;
  int N, Ci, Co, H, W, Kh, Kw, s, p, dl, Cg, Og, Hy, Wy;
  int total;
};

template <class T>
__global__ __launch_bounds__(kThreads) void exact_dgrad_k(ExactArgs a) {
  const T* w = static_cast<const T*>(a.w);
  const T* gy = static_cast<const T*>(a.gy);
  T* gx = static_cast<T*>(a.gx);
  for (long e = (long)blockIdx.x * kThreads + threadIdx.x; e < a.total; e += (long)gridDim.x * kThreads) {
    int t = (int)e;
    const int ww = t % a.W; t /= a.W;
    const int h = t % a.H; t /= a.H;
    const int ci = t % a.Ci;
    const int n = t / a.Ci;
    const int grp = ci / a.Cg, cl = ci - grp * a.Cg;
    float acc = 0.f;
    for (int u = 0; u < a.Kh; ++u) {
      const int nh = h + a.p - u * a.dl;
      if (nh < 0 || nh % a.s) continue;
      const int i = nh / a.s;
      if (i >= a.Hy) continue;
      for (int v = 0; v < a.Kw; ++v) {
        const int nw = ww + a.p - v * a.dl;
        if (nw < 0 || nw % a.s) continue;
        const int j = nw / a.s;
        if (j >= a.Wy) continue;
        for (int ol = 0; ol < a.Og; ++ol) {
          const int co = grp * a.Og + ol;
          acc += to_f32(w[(((long)co * a.Cg + cl) * a.Kh + u) * a.Kw + v]) *
                 to_f32(gy[(((long)n * a.Co + co) * a.Hy + i) * a.Wy + j]);
        }
      }
    }
    gx[e] = from_f32<T>(acc);
  }
}

// one block per (co, cl, u, v); lanes stride over (n, i, j); fixed-order tree sum
template <class T>
__global__ __launch_bounds__(kThreads) void exact_wgrad_k(ExactArgs a) {
  __shared__ float red[kThreads / 64];
  const T* x = static_cast<const T*>(a.x);
  const T* gy = static_cast<const T*>(a.gy);
  int t = blockIdx.x;
  const int v = t % a.Kw; t /= a.Kw;
  const int u = t % a.Kh; t /= a.Kh;
  const int cl = t % a.Cg;
  const int co = t / a.Cg;
  const int ci = (co / a.Og) * a.Cg + cl;
  const int HWy = a.Hy * a.Wy;
  const int cnt = a.N * HWy;
  float acc = 0.f;
  for (int e = threadIdx.x; e < cnt; e += kThreads) {
    const int n = e / HWy;
    const int rem = e - n * HWy;
    const int i = rem / a.Wy, j = rem - i * a.Wy;
    const int h = i * a.s - a.p + u * a.dl, ww = j * a.s - a.p + v * a.dl;
    if (h < 0 || h >= a.H || ww < 0 || ww >= a.W) continue;
    acc += to_f32(x[(((long)n * a.Ci + ci) * a.H + h) * a.W + ww]) *
           to_f32(gy[((long)n * a.Co + co) * HWy + rem]);
  }
  for (int m = 32; m > 0; m >>= 1) acc += __shfl_xor(acc, m, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    float s = 0.f;
    for (int k = 0; k < kThreads / 64; ++k) s += red[k];
    a.gw[blockIdx.x] = s;
  }
}

// ---------------------------------------------------------------------------
// Dense layers: the K x K contractions as GEMMs on the MFMA kernels of the filtered path.
// The shifted operand is written out once per tap ("column" tensor in the workspace):
//   weight gradient: xcol[n, ci*KK + t, (i,j)] = x[n, ci, i s - p + u d, j s - p + v d]
//                    g_theta[co, ci, t] = sum_{n,(i,j)} g_y[n, co, (i,j)] * xcol[n, ci*KK + t, (i,j)]
//   input gradient:  gcol[n, co*KK + t, (h,w)] = g_y[n, co, (h + p - u d)/s, (w + p - v d)/s]
//                    g_x[n, ci, (h,w)] = sum_{co,t} theta[co, ci, t] * gcol[n, co*KK + t, (h,w)]
// (zero where the source index is out of range or not divisible by the stride).
// ---------------------------------------------------------------------------
struct ColArgs {
  const void* src;
  void* dst;
  int C, Hs, Ws;      // source tensor [N, C, Hs, Ws]
  int Ho, Wo;         // positions of the column tensor
  int Kh, Kw, s, p, dl;
  int gather_input;   // 1: x -> xcol (forward index map), 0: g_y -> gcol (transposed map)
  long total;         // N * C * KK * Ho * Wo
};

template <class T>
__global__ __launch_bounds__(kThreads) void im2col_k(ColArgs a) {
  constexpr int VE = 16 / (int)sizeof(T);
  const T* src = static_cast<const T*>(a.src);
  T* dst = static_cast<T*>(a.dst);
  const uint32_t HWo = (uint32_t)(a.Ho * a.Wo), KK = (uint32_t)(a.Kh * a.Kw);
  const uint32_t total = (uint32_t)a.total;   // < 2^31 (checked on the host)
  for (uint32_t e0 = (blockIdx.x * kThreads + threadIdx.x) * VE; e0 < total;
       e0 += gridDim.x * kThreads * VE) {
    // decode the first element; the following ones advance the position incrementally
    uint32_t o = e0 % HWo;
    uint32_t row = e0 / HWo;                  // (n * C + c) * KK + t
    uint32_t t = row % KK;
    uint32_t plane = row / KK;                // n * C + c
    int u = (int)(t / a.Kw), vv = (int)(t - (t / a.Kw) * a.Kw);
    int oh = (int)(o / a.Wo), ow = (int)(o - (o / a.Wo) * a.Wo);
    T vals[VE];
#pragma unroll
    for (int k = 0; k < VE; ++k) {
      float v = 0.f;
      if (e0 + k < total) {
        int sh, sw;
        bool ok = true;
        if (a.gather_input) {
          sh = oh * a.s - a.p + u * a.dl;
          sw = ow * a.s - a.p + vv * a.dl;
        } else {
          const int nh = oh + a.p - u * a.dl, nw = ow + a.p - vv * a.dl;
          ok = nh >= 0 && nw >= 0 && nh % a.s == 0 && nw % a.s == 0;
          sh = nh / a.s;
          sw = nw / a.s;
        }
        if (ok && sh >= 0 && sh < a.Hs && sw >= 0 && sw < a.Ws)
          v = to_f32(src[((long)plane * a.Hs + sh) * a.Ws + sw]);
      }
      vals[k] = from_f32<T>(v);
      if (++ow == a.Wo) {
        ow = 0;
        if (++oh == a.Ho) {
          oh = 0;
          if (++vv == a.Kw) {
            vv = 0;
            if (++u == a.Kh) { u = 0; ++plane; }
          }
        }
      }
    }
    if (e0 + VE <= total) {
      *reinterpret_cast<uint4*>(dst + e0) = *reinterpret_cast<const uint4*>(vals);
    } else {
      for (int k = 0; e0 + k < total; ++k) dst[e0 + k] = vals[k];
    }
  }
}

// Stride-1 layers with W_o a multiple of the vector length: a 16-byte vector of the column tensor
// is 8 (4) consecutive pixels of one source row, shifted by the tap offset and clipped at the row
// ends.  One index decode per vector, FastDiv instead of divisions.
struct ColRowsArgs {
  const void* src;
  void* dst;
  int Hs, Ws, Ho, Wo, Kw;
  int dh0, dw0, dstep;   // source row = oh + dh0 + u * dstep, source col = ow + dw0 + v * dstep
  int vpr;               // vectors per column-tensor row of Wo pixels
  uint32_t total_vec;
  FastDiv d_vpr, d_ho, d_kk, d_kw;
};

template <class T>
__global__ __launch_bounds__(kThreads) void im2col_rows_k(ColRowsArgs a) {
  constexpr int VE = 16 / (int)sizeof(T);
  const T* src = static_cast<const T*>(a.src);
  T* dst = static_cast<T*>(a.dst);
  for (uint32_t vi = blockIdx.x * kThreads + threadIdx.x; vi < a.total_vec; vi += gridDim.x * kThreads) {
    const uint32_t rowid = a.d_vpr.div(vi);            // ((plane * KK + t) * Ho + oh)
    const int ow0 = (int)(vi - rowid * a.vpr) * VE;
    const uint32_t pt = a.d_ho.div(rowid);             // plane * KK + t
    const int oh = (int)(rowid - pt * a.Ho);
    const uint32_t plane = a.d_kk.div(pt);
    const int t = (int)(pt - plane * a.d_kk.d);
    const int u = (int)a.d_kw.div((uint32_t)t), v = t - u * a.Kw;
    const int sh = oh + a.dh0 + u * a.dstep;
    const int sw0 = ow0 + a.dw0 + v * a.dstep;
    const bool row_ok = sh >= 0 && sh < a.Hs;
    const T* p = src + ((long)plane * a.Hs + (row_ok ? sh : 0)) * a.Ws;
    T vals[VE];
#pragma unroll
    for (int e = 0; e < VE; ++e) {
      const int sw = sw0 + e;
      const bool ok = row_ok && sw >= 0 && sw < a.Ws;
      const T val = p[ok ? sw : 0];
      vals[e] = ok ? val : from_f32<T>(0.f);
    }
    *reinterpret_cast<uint4*>(dst + (long)vi * VE) = *reinterpret_cast<const uint4*>(vals);
  }
}

// wt[(co*KK + t), ci] = w[co, ci, t]
template <class T>
__global__ __launch_bounds__(kThreads) void permute_w_k(const T* w, T* wt, int Co, int Ci, int KK) {
  const int e = blockIdx.x * kThreads + threadIdx.x;
  if (e >= Co * Ci * KK) return;
  const int ci = e % Ci;
  const int row = e / Ci;
  const int t = row % KK, co = row / KK;
  wt[e] = w[((long)co * Ci + ci) * KK + t];
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// dense layers whose column tensors stay below 2^31 elements go through the GEMM path
bool gemm_path(const Geom& g) {
  if (g.g != 1) return false;
  const long lim = 2147483647L;
  return (long)g.N * g.Ci * g.KK * g.Hy * g.Wy < lim && (long)g.N * g.Co * g.KK * g.H * g.W < lim &&
         (long)g.Co * g.KK <= 65535L * 16 && (long)g.Ci * g.KK <= 65535L * 16;
}

bool pointwise_plain(const Geom& g) { return g.KK == 1 && g.s == 1 && g.p == 0; }

Geom wgrad_geom(const Geom& g) {  // Ci*KK "input channels", one "patch" per output pixel
  Geom q = g;
  q.Ci = g.Ci * g.KK; q.Cg = q.Ci; q.KK = 1; q.Kh = q.Kw = 1;
  q.P = g.Hy * g.Wy; q.Hp = g.Hy; q.Wp = g.Wy; q.r = 2; q.s = 1;
  return q;
}

Geom dgrad_geom(const Geom& g) {  // Co*KK "output channels", one "patch" per input pixel
  Geom q = g;
  q.Co = g.Co * g.KK; q.Og = q.Co; q.KK = 1; q.Kh = q.Kw = 1;
  q.P = g.H * g.W; q.Hp = g.H; q.Wp = g.W; q.r = 2; q.s = 1; q.rx = 1;
  return q;
}

size_t col_bytes(const Geom& g, bool want_gw, bool want_gx) {
  if (pointwise_plain(g)) return 0;
  size_t a = want_gw ? (size_t)g.N * g.Ci * g.KK * g.Hy * g.Wy * g.b : 0;
  size_t c = want_gx ? (size_t)g.N * g.Co * g.KK * g.H * g.W * g.b : 0;
  return align256(a > c ? a : c);
}

size_t aux_bytes(const Geom& g, bool want_gw, bool want_gx) {
  size_t a = 0, c = 0;
  if (want_gw) {
    const Geom q = wgrad_geom(g);
    a = (size_t)mfma_wgrad_splits(q, nullptr) * q.Co * q.Ci * sizeof(float);
  }
  if (want_gx) c = pointwise_plain(g) ? 0 : (size_t)g.Co * g.KK * g.Ci * g.b;
  return align256(a > c ? a : c);
}

template <class T>
hipError_t launch_col(const Geom& g, const void* src, void* dst, bool gather_input, hipStream_t st) {
  ColArgs a;
  a.src = src; a.dst = dst;
  a.Kh = g.Kh; a.Kw = g.Kw; a.s = g.s; a.p = g.p; a.dl = g.dl;
  a.gather_input = gather_input ? 1 : 0;
  if (gather_input) { a.C = g.Ci; a.Hs = g.H; a.Ws = g.W; a.Ho = g.Hy; a.Wo = g.Wy; }
  else { a.C = g.Co; a.Hs = g.Hy; a.Ws = g.Wy; a.Ho = g.H; a.Wo = g.W; }
  a.total = (long)g.N * a.C * g.KK * a.Ho * a.Wo;
  constexpr int VE = 16 / (int)sizeof(T);
  if (g.s == 1 && a.Wo % VE == 0) {
    ColRowsArgs r;
    r.src = src; r.dst = dst; r.Hs = a.Hs; r.Ws = a.Ws; r.Ho = a.Ho; r.Wo = a.Wo; r.Kw = g.Kw;
    // forward map: source = o - p + tap * d;  transposed map: source = o + p - tap * d
    r.dh0 = gather_input ? -g.p : g.p;
    r.dw0 = r.dh0;
    r.dstep = gather_input ? g.dl : -g.dl;
    r.vpr = a.Wo / VE;
    r.total_vec = (uint32_t)(a.total / VE);
    r.d_vpr = FastDiv((uint32_t)r.vpr);
    r.d_ho = FastDiv((uint32_t)a.Ho);
    r.d_kk = FastDiv((uint32_t)g.KK);
    r.d_kw = FastDiv((uint32_t)g.Kw);
    long nb = ((long)r.total_vec + kThreads - 1) / kThreads;
    if (nb > (1 << 20)) nb = 1 << 20;
    GF_LAUNCH(im2col_rows_k<T>, dim3((int)nb), dim3(kThreads), 0, st, r);
    return hipGetLastError();
  }
  long blocks = (a.total / VE + kThreads - 1) / kThreads;
  if (blocks > (1 << 20)) blocks = 1 << 20;
  if (blocks < 1) blocks = 1;
  GF_LAUNCH(im2col_k<T>, dim3((int)blocks), dim3(kThreads), 0, st, a);
  return hipGetLastError();
}

ExactArgs make_args(const Geom& g) {
  ExactArgs a = {};
  a.N = g.N; a.Ci = g.Ci; a.Co = g.Co; a.H = g.H; a.W = g.W; a.Kh = g.Kh; a.Kw = g.Kw;
  a.s = g.s; a.p = g.p; a.dl = g.dl; a.Cg = g.Cg; a.Og = g.Og; a.Hy = g.Hy; a.Wy = g.Wy;
  return a;
}

}  // namespace

size_t ws_exact(const Geom& g, bool want_gw, bool want_gx) {
  if (implicit_ok(g)) return ws_implicit(g, want_gw, want_gx);
  if (!gemm_path(g)) return want_gw && dw_exact_wgrad_ok(g) ? ws_dw_exact_wgrad(g) : 0;
  return col_bytes(g, want_gw, want_gx) + aux_bytes(g, want_gw, want_gx);
}

hipError_t launch_exact_wgrad(const Geom& g, const void* x, const void* g_y, float* g_w, void* ws,
                              hipStream_t st) {
  if (implicit_ok(g)) return launch_implicit(g, x, nullptr, g_y, g_w, nullptr, ws, st);
  if (gemm_path(g)) {
    const void* xcol = x;
    char* wsb = static_cast<char*>(ws);
    // the workspace may have been sized for both gradients: the aux region follows the larger
    // column tensor; the partial slabs are placed right behind this call's own column tensor
    size_t off = 0;
    if (!pointwise_plain(g)) {
      hipError_t e = g.dtype == GF_BF16 ? launch_col<bf16_t>(g, x, ws, true, st)
                                        : launch_col<float>(g, x, ws, true, st);
      if (e != hipSuccess) return e;
      xcol = ws;
      off = align256((size_t)g.N * g.Ci * g.KK * g.Hy * g.Wy * g.b);
    }
    const Geom q = wgrad_geom(g);
    float* part = reinterpret_cast<float*>(wsb + off);
    int nz = 0;
    hipError_t e = launch_mfma_wgrad(q, xcol, g_y, part, &nz, st);
    if (e != hipSuccess) return e;
    return launch_finalize(part, g_w, q.Co * q.Ci, nz, 1, 1.f, st);
  }
  if (dw_exact_wgrad_ok(g)) return launch_dw_exact_wgrad(g, x, g_y, g_w, ws, st);
  ExactArgs a = make_args(g);
  a.x = x;
  a.gy = g_y;
  a.gw = g_w;
  const int blocks = g.Co * g.Cg * g.KK;
  if (g.dtype == GF_BF16)
    GF_LAUNCH(exact_wgrad_k<bf16_t>, dim3(blocks), dim3(kThreads), 0, st, a);
  else
    GF_LAUNCH(exact_wgrad_k<float>, dim3(blocks), dim3(kThreads), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_exact_dgrad(const Geom& g, const void* w, const void* g_y, void* g_x, void* ws,
                              hipStream_t st) {
  if (implicit_ok(g)) return launch_implicit(g, nullptr, w, g_y, nullptr, g_x, ws, st);
  if (gemm_path(g)) {
    const Geom q = dgrad_geom(g);
    if (pointwise_plain(g)) return launch_mfma_dgrad(q, g_y, w, nullptr, g_x, nullptr, st);
    char* wsb = static_cast<char*>(ws);
    hipError_t e = g.dtype == GF_BF16 ? launch_col<bf16_t>(g, g_y, ws, false, st)
                                      : launch_col<float>(g, g_y, ws, false, st);
    if (e != hipSuccess) return e;
    void* wt = wsb + align256((size_t)g.N * g.Co * g.KK * g.H * g.W * g.b);
    const int tot = g.Co * g.Ci * g.KK;
    if (g.dtype == GF_BF16)
      GF_LAUNCH(permute_w_k<bf16_t>, dim3(cdiv(tot, kThreads)), dim3(kThreads), 0, st,
                         static_cast<const bf16_t*>(w), static_cast<bf16_t*>(wt), g.Co, g.Ci, g.KK);
    else
      GF_LAUNCH(permute_w_k<float>, dim3(cdiv(tot, kThreads)), dim3(kThreads), 0, st,
                         static_cast<const float*>(w), static_cast<float*>(wt), g.Co, g.Ci, g.KK);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_mfma_dgrad(q, ws, wt, nullptr, g_x, nullptr, st);
  }
  if (dw_exact_dgrad_ok(g)) return launch_dw_exact_dgrad(g, w, g_y, g_x, st);
  ExactArgs a = make_args(g);
  a.w = w;
  a.gy = g_y;
  a.gx = g_x;
  a.total = g.N * g.Ci * g.H * g.W;
  int blocks = cdiv(a.total, kThreads);
  if (blocks > 1 << 20) blocks = 1 << 20;
  if (g.dtype == GF_BF16)
    GF_LAUNCH(exact_dgrad_k<bf16_t>, dim3(blocks), dim3(kThreads), 0, st, a);
  else
    GF_LAUNCH(exact_dgrad_k<float>, dim3(blocks), dim3(kThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace gf
