// Vanilla back-propagation of a conv layer (Sec. 3.1): g_theta = g_y (F) x and
// g_x = g_y (*) rot180(theta), with stride, zero padding, dilation and groups.
// Shape-generic direct kernels: one lane per g_x element (gather over the taps
// that reach it) and one block per weight-gradient element.
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

ExactArgs make_args(const Geom& g) {
  ExactArgs a = {};
  a.N = g.N; a.Ci = g.Ci; a.Co = g.Co; a.H = g.H; a.W = g.W; a.Kh = g.Kh; a.Kw = g.Kw;
  a.s = g.s; a.p = g.p; a.dl = g.dl; a.Cg = g.Cg; a.Og = g.Og; a.Hy = g.Hy; a.Wy = g.Wy;
  return a;
}

}  // namespace

size_t ws_exact(const Geom&, bool, bool) { return 0; }

hipError_t launch_exact_wgrad(const Geom& g, const void* x, const void* g_y, float* g_w, void*,
                              hipStream_t st) {
  ExactArgs a = make_args(g);
  a.x = x;
  a.gy = g_y;
  a.gw = g_w;
  const int blocks = g.Co * g.Cg * g.KK;
  if (g.dtype == GF_BF16)
    hipLaunchKernelGGL(exact_wgrad_k<bf16_t>, dim3(blocks), dim3(kThreads), 0, st, a);
  else
    hipLaunchKernelGGL(exact_wgrad_k<float>, dim3(blocks), dim3(kThreads), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_exact_dgrad(const Geom& g, const void* w, const void* g_y, void* g_x, void*,
                              hipStream_t st) {
  ExactArgs a = make_args(g);
  a.w = w;
  a.gy = g_y;
  a.gx = g_x;
  a.total = g.N * g.Ci * g.H * g.W;
  int blocks = cdiv(a.total, kThreads);
  if (blocks > 1 << 20) blocks = 1 << 20;
  if (g.dtype == GF_BF16)
    hipLaunchKernelGGL(exact_dgrad_k<bf16_t>, dim3(blocks), dim3(kThreads), 0, st, a);
  else
    hipLaunchKernelGGL(exact_dgrad_k<float>, dim3(blocks), dim3(kThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace gf
