// Vanilla back-propagation (Sec. 3.1) of depthwise layers: every (image, channel) plane is a
// small 2-D problem of its own, so a block stages a run of whole planes in LDS with coalesced
// 16-byte loads (NCHW planes of consecutive channels are one contiguous stream) and all tap
// arithmetic runs from LDS.  Both kernels move each tensor through HBM once.
//   input gradient   g_x[h, w]  = sum_taps theta[c, u, v] * g_y[(h + p - u d) / s, (w + p - v d) / s]
//   weight gradient  g_theta[c, u, v] = sum_{n, i, j} x[i s - p + u d, j s - p + v d] * g_y[i, j]
// The weight gradient is formed per plane (fixed-order sums) and the planes of a channel are
// added over n by the finalize kernel.
#include "gf_internal.h"

namespace gf {

namespace {

constexpr int kThreads = 256;
constexpr int kLdsBudget = 56 * 1024;

struct DwExactArgs {
  const void* x;
  const void* w;
  const void* gy;
  void* gx;
  float* part;   // [N, C, K * K]
  int C, H, W, Hy, Wy, K, s, p, dl;
  int planes, ppb;
  // stride-1 kernels: the staged operand sits in a zero frame of `halo` pixels (PH x PW per plane)
  int halo, PH, PW;
  FastDiv d_hw, d_w, d_hwy, d_wy, d_c;
};

// copy elements [e0, e1) of a tensor to LDS with 16-byte loads; returns the LDS pointer of
// element e0 (the image starts `shift` bytes into `buf`, which needs (e1 - e0) * sizeof(T) + 32 bytes)
template <class T>
__device__ __forceinline__ T* stage_run(const void* base, long e0, long e1, unsigned char* buf, int tid) {
  const long byte0 = e0 * (long)sizeof(T), byte1 = e1 * (long)sizeof(T);
  const long a0 = byte0 & ~15L;   // the tensor base is 16-byte aligned
  const int span = (int)(byte1 - a0);
  const int nvec = span >> 4;
  const uint4* src = reinterpret_cast<const uint4*>(static_cast<const unsigned char*>(base) + a0);
  uint4* dst = reinterpret_cast<uint4*>(buf);
  for (int v = tid; v < nvec; v += 4 * kThreads) {
    // four loads in flight per lane; past-the-end indices are clamped and rewritten
    uint4 rg[4];
    int idx[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) idx[k] = min(v + k * kThreads, nvec - 1);
#pragma unroll
    for (int k = 0; k < 4; ++k) rg[k] = load_stream16(src + idx[k]);
#pragma unroll
    for (int k = 0; k < 4; ++k) dst[idx[k]] = rg[k];
  }
  const int tail0 = nvec << 4;   // fewer than 16 trailing bytes: the run ends where the tensor ends
  const int ntail = (span - tail0) / (int)sizeof(T);
  if (tid < ntail)
    reinterpret_cast<T*>(buf + tail0)[tid] =
        reinterpret_cast<const T*>(reinterpret_cast<const unsigned char*>(src) + tail0)[tid];
  return reinterpret_cast<T*>(buf + (int)(byte0 - a0));
}

// The same run of whole planes [pl0, pl0 + npl) of an [*, H, W] tensor, but laid out in LDS as
// [npl][PH][PW] with the plane at row `top`, column `left` of a zero frame, so that the tap loops
// need no bounds checks.  `buf` must have been cleared (the frame) before the call.
template <class T>
__device__ __forceinline__ void stage_padded(const void* base, int pl0, int npl, int H, int W, int top, int left,
                                             int PH, int PW, const FastDiv& d_hw, const FastDiv& d_w, T* buf,
                                             int tid) {
  constexpr int VE = 16 / (int)sizeof(T);
  const int HW = H * W;
  const long e0 = (long)pl0 * HW, e1 = e0 + (long)npl * HW;
  const long byte0 = e0 * (long)sizeof(T), byte1 = e1 * (long)sizeof(T);
  const long a0 = byte0 & ~15L;
  const int lead = (int)((byte0 - a0) / (long)sizeof(T));   // elements of the first vector that precede the run
  const int nvec = (int)((byte1 - a0) >> 4);                // whole vectors that end inside the run
  const uint4* src = reinterpret_cast<const uint4*>(static_cast<const unsigned char*>(base) + a0);
  const int count = npl * HW;
  auto put = [&](int e, T val) {   // e: element index relative to the run
    const int pl = (int)d_hw.div((uint32_t)e);
    const int rem = e - pl * HW;
    const int h = (int)d_w.div((uint32_t)rem);
    buf[(pl * PH + h + top) * PW + rem - h * W + left] = val;
  };
  for (int v = tid; v < nvec; v += 4 * kThreads) {
    uint4 rg[4];
    int idx[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) idx[k] = min(v + k * kThreads, nvec - 1);
#pragma unroll
    for (int k = 0; k < 4; ++k) rg[k] = load_stream16(src + idx[k]);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (v + k * kThreads >= nvec) continue;
      const T* el = reinterpret_cast<const T*>(&rg[k]);
#pragma unroll
      for (int i = 0; i < VE; ++i) {
        const int e = idx[k] * VE + i - lead;
        if (e >= 0) put(e, el[i]);
      }
    }
  }
  // elements behind the last whole vector (the run ends where the tensor may end)
  const int tail0 = nvec * VE - lead;
  if (tid < count - tail0 && tail0 + tid >= 0) put(tail0 + tid, static_cast<const T*>(base)[e0 + tail0 + tid]);
}

// ---------------------------------------------------------------------------
// input gradient: the block's planes one after the other (WAVE: small planes, a wave per plane);
// the K x K taps of the plane's channel sit in registers, K and the stride S are compile-time
// (S = 0: any stride, with divisions)
// ---------------------------------------------------------------------------
template <class T, int K, int S, bool WAVE>
__global__ __launch_bounds__(kThreads) void dw_exact_dgrad_k(DwExactArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int pl0 = blockIdx.x * a.ppb;
  const int npl = min(a.ppb, a.planes - pl0);
  const int HW = a.H * a.W, HWy = a.Hy * a.Wy;
  const int in_bytes = ((a.ppb * HWy * (int)sizeof(T) + 32) + 15) & ~15;
  const T* gys = stage_run<T>(a.gy, (long)pl0 * HWy, (long)(pl0 + npl) * HWy, smem, tid);
  // the g_x image of the same planes, laid out as in memory (16-byte phase of its first element kept)
  const long obyte0 = (long)pl0 * HW * (long)sizeof(T);
  const long oa0 = obyte0 & ~15L;
  const int oshift = (int)(obyte0 - oa0);
  T* gxs = reinterpret_cast<T*>(smem + in_bytes + oshift);
  const T* w = static_cast<const T*>(a.w);
  __syncthreads();
  const int first = WAVE ? wave : 0, step = WAVE ? kThreads / 64 : 1;
  const int t0 = WAVE ? lane : tid, tstep = WAVE ? 64 : kThreads;
  const int s = S ? S : a.s;
  for (int pl = first; pl < npl; pl += step) {
    const int gpl = pl0 + pl;
    const int c = gpl - (int)a.d_c.div((uint32_t)gpl) * a.C;
    float wk[K * K];
#pragma unroll
    for (int t = 0; t < K * K; ++t) wk[t] = to_f32(w[(long)c * (K * K) + t]);
    const T* src = gys + pl * HWy;
    T* dst = gxs + pl * HW;
    for (int e = t0; e < HW; e += tstep) {
      const int h = (int)a.d_w.div((uint32_t)e);
      const int ww = e - h * a.W;
      int ri[K], cj[K];   // source row offset / column per tap, -1 where the tap does not reach a g_y pixel
#pragma unroll
      for (int u = 0; u < K; ++u) {
        const int nh = h + a.p - u * a.dl;
        const int i = S == 1 ? nh : nh / s;
        ri[u] = (nh >= 0 && i * s == nh && i < a.Hy) ? i * a.Wy : -1;
        const int nw = ww + a.p - u * a.dl;
        const int j = S == 1 ? nw : nw / s;
        cj[u] = (nw >= 0 && j * s == nw && j < a.Wy) ? j : -1;
      }
      float acc = 0.f;
#pragma unroll
      for (int u = 0; u < K; ++u)
#pragma unroll
        for (int v = 0; v < K; ++v) {
          const bool ok = (ri[u] | cj[v]) >= 0;
          const float g = to_f32(src[ok ? ri[u] + cj[v] : 0]);
          acc += ok ? wk[u * K + v] * g : 0.f;
        }
      dst[e] = from_f32<T>(acc);
    }
  }
  __syncthreads();
  // store the image: whole 16-byte vectors, then the partial vectors at both ends, which the
  // neighbouring blocks share, element by element
  T* out = static_cast<T*>(a.gx);
  const long e0 = (long)pl0 * HW;
  const int span = oshift + npl * HW * (int)sizeof(T);
  const int nvec = span >> 4;
  unsigned char* img = smem + in_bytes;
  unsigned char* dstb = reinterpret_cast<unsigned char*>(out) + oa0;
  for (int v = tid + (oshift ? 1 : 0); v < nvec; v += kThreads)
    store_stream16(dstb + ((long)v << 4), *reinterpret_cast<const uint4*>(img + (v << 4)));
  if (oshift) {
    const int nhead = min((16 - oshift) / (int)sizeof(T), npl * HW);
    if (tid < nhead) out[e0 + tid] = gxs[tid];
  }
  {
    const int tail0 = nvec << 4;
    const int ntail = (span - tail0) / (int)sizeof(T);
    const int efirst = (tail0 - oshift) / (int)sizeof(T);
    if (tid < ntail && efirst + tid >= 0) out[e0 + efirst + tid] = gxs[efirst + tid];
  }
}

// stride 1: g_y staged in a zero frame, no bounds checks in the tap loop
template <class T, int K, bool WAVE>
__global__ __launch_bounds__(kThreads) void dw_exact_dgrad_s1_k(DwExactArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int pl0 = blockIdx.x * a.ppb;
  const int npl = min(a.ppb, a.planes - pl0);
  const int HW = a.H * a.W;
  const int pad_elems = a.ppb * a.PH * a.PW;
  const int in_bytes = (pad_elems * (int)sizeof(T) + 15) & ~15;
  T* gys = reinterpret_cast<T*>(smem);
  for (int i = tid; i < (in_bytes >> 4); i += kThreads) reinterpret_cast<uint4*>(smem)[i] = make_uint4(0, 0, 0, 0);
  __syncthreads();
  stage_padded<T>(a.gy, pl0, npl, a.Hy, a.Wy, a.halo, a.halo, a.PH, a.PW, a.d_hwy, a.d_wy, gys, tid);
  const long obyte0 = (long)pl0 * HW * (long)sizeof(T);
  const long oa0 = obyte0 & ~15L;
  const int oshift = (int)(obyte0 - oa0);
  T* gxs = reinterpret_cast<T*>(smem + in_bytes + oshift);
  const T* w = static_cast<const T*>(a.w);
  __syncthreads();
  const int first = WAVE ? wave : 0, step = WAVE ? kThreads / 64 : 1;
  const int t0 = WAVE ? lane : tid, tstep = WAVE ? 64 : kThreads;
  int off[K * K];   // tap (u, v) reads g_y[h + p - u d][w + p - v d]
#pragma unroll
  for (int u = 0; u < K; ++u)
#pragma unroll
    for (int v = 0; v < K; ++v) off[u * K + v] = (a.p + a.halo - u * a.dl) * a.PW + a.p + a.halo - v * a.dl;
  for (int pl = first; pl < npl; pl += step) {
    const int gpl = pl0 + pl;
    const int c = gpl - (int)a.d_c.div((uint32_t)gpl) * a.C;
    float wk[K * K];
#pragma unroll
    for (int t = 0; t < K * K; ++t) wk[t] = to_f32(w[(long)c * (K * K) + t]);
    const T* src = gys + pl * a.PH * a.PW;
    T* dst = gxs + pl * HW;
    for (int e = t0; e < HW; e += tstep) {
      const int h = (int)a.d_w.div((uint32_t)e);
      const int ww = e - h * a.W;
      const T* q = src + h * a.PW + ww;
      float acc = 0.f;
#pragma unroll
      for (int t = 0; t < K * K; ++t) acc += wk[t] * to_f32(q[off[t]]);
      dst[e] = from_f32<T>(acc);
    }
  }
  __syncthreads();
  T* out = static_cast<T*>(a.gx);
  const long e0 = (long)pl0 * HW;
  const int span = oshift + npl * HW * (int)sizeof(T);
  const int nvec = span >> 4;
  unsigned char* img = smem + in_bytes;
  unsigned char* dstb = reinterpret_cast<unsigned char*>(out) + oa0;
  for (int v = tid + (oshift ? 1 : 0); v < nvec; v += kThreads)
    store_stream16(dstb + ((long)v << 4), *reinterpret_cast<const uint4*>(img + (v << 4)));
  if (oshift) {
    const int nhead = min((16 - oshift) / (int)sizeof(T), npl * HW);
    if (tid < nhead) out[e0 + tid] = gxs[tid];
  }
  {
    const int tail0 = nvec << 4;
    const int ntail = (span - tail0) / (int)sizeof(T);
    const int efirst = (tail0 - oshift) / (int)sizeof(T);
    if (tid < ntail && efirst + tid >= 0) out[e0 + efirst + tid] = gxs[efirst + tid];
  }
}

// stride 1: x staged in a zero frame of p pixels, no bounds checks in the tap loop
template <class T, int K, bool WAVE>
__global__ __launch_bounds__(kThreads) void dw_exact_wgrad_s1_k(DwExactArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ float red[kThreads / 64][K * K];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int pl0 = blockIdx.x * a.ppb;
  const int npl = min(a.ppb, a.planes - pl0);
  const int HWy = a.Hy * a.Wy;
  const int pad_elems = a.ppb * a.PH * a.PW;
  const int x_bytes = (pad_elems * (int)sizeof(T) + 15) & ~15;
  T* xs = reinterpret_cast<T*>(smem);
  for (int i = tid; i < (x_bytes >> 4); i += kThreads) reinterpret_cast<uint4*>(smem)[i] = make_uint4(0, 0, 0, 0);
  __syncthreads();
  stage_padded<T>(a.x, pl0, npl, a.H, a.W, a.halo, a.halo, a.PH, a.PW, a.d_hw, a.d_w, xs, tid);
  const T* gys = stage_run<T>(a.gy, (long)pl0 * HWy, (long)(pl0 + npl) * HWy, smem + x_bytes, tid);
  __syncthreads();
  const int first = WAVE ? wave : 0, step = WAVE ? kThreads / 64 : 1;
  const int t0 = WAVE ? lane : tid, tstep = WAVE ? 64 : kThreads;
  int off[K * K];   // tap (u, v) of output (i, j) reads x[i - p + u d][j - p + v d]; the frame is p wide
#pragma unroll
  for (int u = 0; u < K; ++u)
#pragma unroll
    for (int v = 0; v < K; ++v) off[u * K + v] = (u * a.dl) * a.PW + v * a.dl;
  for (int pl = first; pl < npl; pl += step) {
    const T* xp = xs + pl * a.PH * a.PW;
    const T* gp = gys + pl * HWy;
    float acc[K * K];
#pragma unroll
    for (int t = 0; t < K * K; ++t) acc[t] = 0.f;
    for (int e = t0; e < HWy; e += tstep) {
      const int i = (int)a.d_wy.div((uint32_t)e);
      const int j = e - i * a.Wy;
      const float g = to_f32(gp[e]);
      const T* q = xp + i * a.PW + j;
#pragma unroll
      for (int t = 0; t < K * K; ++t) acc[t] += to_f32(q[off[t]]) * g;
    }
#pragma unroll
    for (int t = 0; t < K * K; ++t)
      for (int m = 32; m > 0; m >>= 1) acc[t] += __shfl_xor(acc[t], m, 64);
    float* dst = a.part + (long)(pl0 + pl) * (K * K);
    if constexpr (WAVE) {
      if (lane == 0) {
#pragma unroll
        for (int t = 0; t < K * K; ++t) dst[t] = acc[t];
      }
    } else {
      if (lane == 0) {
#pragma unroll
        for (int t = 0; t < K * K; ++t) red[wave][t] = acc[t];
      }
      __syncthreads();
      if (tid < K * K) {
        float sm = 0.f;
        for (int k = 0; k < kThreads / 64; ++k) sm += red[k][tid];
        dst[tid] = sm;
      }
      __syncthreads();
    }
  }
}

// ---------------------------------------------------------------------------
// weight gradient: K x K accumulators per lane, one plane after the other; WAVE: small planes,
// every wave owns whole planes (no block barrier in the reduction)
// ---------------------------------------------------------------------------
template <class T, int K, bool WAVE>
__global__ __launch_bounds__(kThreads) void dw_exact_wgrad_k(DwExactArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ float red[kThreads / 64][K * K];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int pl0 = blockIdx.x * a.ppb;
  const int npl = min(a.ppb, a.planes - pl0);
  const int HW = a.H * a.W, HWy = a.Hy * a.Wy;
  const int x_bytes = ((a.ppb * HW * (int)sizeof(T) + 32) + 15) & ~15;
  const T* xs = stage_run<T>(a.x, (long)pl0 * HW, (long)(pl0 + npl) * HW, smem, tid);
  const T* gys = stage_run<T>(a.gy, (long)pl0 * HWy, (long)(pl0 + npl) * HWy, smem + x_bytes, tid);
  __syncthreads();
  const int first = WAVE ? wave : 0, step = WAVE ? kThreads / 64 : 1;
  const int t0 = WAVE ? lane : tid, tstep = WAVE ? 64 : kThreads;
  for (int pl = first; pl < npl; pl += step) {
    const T* xp = xs + pl * HW;
    const T* gp = gys + pl * HWy;
    float acc[K * K];
#pragma unroll
    for (int t = 0; t < K * K; ++t) acc[t] = 0.f;
    for (int e = t0; e < HWy; e += tstep) {
      const int i = (int)a.d_wy.div((uint32_t)e);
      const int j = e - i * a.Wy;
      const float g = to_f32(gp[e]);
      const int hb = i * a.s - a.p, wb = j * a.s - a.p;
#pragma unroll
      for (int u = 0; u < K; ++u) {
        const int h = hb + u * a.dl;
        const bool okh = h >= 0 && h < a.H;
#pragma unroll
        for (int v = 0; v < K; ++v) {
          const int ww = wb + v * a.dl;
          const bool ok = okh && ww >= 0 && ww < a.W;
          const float xv = to_f32(xp[ok ? h * a.W + ww : 0]);
          acc[u * K + v] += ok ? xv * g : 0.f;
        }
      }
    }
#pragma unroll
    for (int t = 0; t < K * K; ++t)
      for (int m = 32; m > 0; m >>= 1) acc[t] += __shfl_xor(acc[t], m, 64);
    float* dst = a.part + (long)(pl0 + pl) * (K * K);
    if constexpr (WAVE) {
      if (lane == 0) {
#pragma unroll
        for (int t = 0; t < K * K; ++t) dst[t] = acc[t];
      }
    } else {
      if (lane == 0) {
#pragma unroll
        for (int t = 0; t < K * K; ++t) red[wave][t] = acc[t];
      }
      __syncthreads();
      if (tid < K * K) {
        float s = 0.f;
        for (int k = 0; k < kThreads / 64; ++k) s += red[k][tid];
        dst[tid] = s;
      }
      __syncthreads();
    }
  }
}

bool shape_ok(const Geom& g) {
  if (g.Cg != 1 || g.Og != 1 || g.Ci != g.Co) return false;   // depthwise
  if (g.Kh != g.Kw) return false;
  return true;
}

// planes per block: as many as fit the budget, few enough for ~1024 blocks
int planes_per_block(const Geom& g, long per_plane) {
  long ppb = (kLdsBudget - 96) / per_plane;
  const long planes = (long)g.N * g.Ci;
  if (ppb > planes / 1024) ppb = planes / 1024;
  if (ppb < 1) ppb = 1;
  if (ppb > 64) ppb = 64;
  return (int)ppb;
}

DwExactArgs make_args(const Geom& g) {
  DwExactArgs a = {};
  a.C = g.Ci; a.H = g.H; a.W = g.W; a.Hy = g.Hy; a.Wy = g.Wy; a.K = g.Kh; a.s = g.s; a.p = g.p; a.dl = g.dl;
  a.planes = g.N * g.Ci;
  a.d_hw = FastDiv((uint32_t)(g.H * g.W));
  a.d_w = FastDiv((uint32_t)g.W);
  a.d_hwy = FastDiv((uint32_t)(g.Hy * g.Wy));
  a.d_wy = FastDiv((uint32_t)g.Wy);
  a.d_c = FastDiv((uint32_t)g.Ci);
  return a;
}

}  // namespace

// LDS bytes per plane of the two kernels (stride 1: the staged operand carries its zero frame)
static int dgrad_halo(const Geom& g) { const int h = (g.Kh - 1) * g.dl - g.p; return g.s == 1 && h > 0 ? h : 0; }
static long dgrad_per_plane(const Geom& g) {
  const int h = dgrad_halo(g);
  return ((long)(g.Hy + 2 * h) * (g.Wy + 2 * h) + (long)g.H * g.W) * g.b;
}
static long wgrad_per_plane(const Geom& g) {
  const int h = g.s == 1 ? g.p : 0;
  return ((long)(g.H + 2 * h) * (g.W + 2 * h) + (long)g.Hy * g.Wy) * g.b;
}

bool dw_exact_dgrad_ok(const Geom& g) {
  if (!shape_ok(g) || (g.Kh != 3 && g.Kh != 5 && g.Kh != 7)) return false;
  return dgrad_per_plane(g) + 96 <= kLdsBudget;
}

bool dw_exact_wgrad_ok(const Geom& g) {
  if (!shape_ok(g) || (g.Kh != 3 && g.Kh != 5)) return false;
  return wgrad_per_plane(g) + 96 <= kLdsBudget;
}

size_t ws_dw_exact_wgrad(const Geom& g) { return (size_t)g.N * g.Ci * g.KK * sizeof(float); }

template <class T, int K, int S>
static hipError_t dgrad_launch_s(DwExactArgs& a, bool wave, size_t lds, hipStream_t st) {
  const dim3 grid(cdiv(a.planes, a.ppb)), block(kThreads);
  if constexpr (S == 1) {
    if (wave) GF_LAUNCH((dw_exact_dgrad_s1_k<T, K, true>), grid, block, lds, st, a);
    else GF_LAUNCH((dw_exact_dgrad_s1_k<T, K, false>), grid, block, lds, st, a);
  } else {
    if (wave) GF_LAUNCH((dw_exact_dgrad_k<T, K, S, true>), grid, block, lds, st, a);
    else GF_LAUNCH((dw_exact_dgrad_k<T, K, S, false>), grid, block, lds, st, a);
  }
  return hipGetLastError();
}

template <class T, int K>
static hipError_t dgrad_launch_k(DwExactArgs& a, bool wave, size_t lds, hipStream_t st) {
  if (a.s == 1) return dgrad_launch_s<T, K, 1>(a, wave, lds, st);
  if (a.s == 2) return dgrad_launch_s<T, K, 2>(a, wave, lds, st);
  return dgrad_launch_s<T, K, 0>(a, wave, lds, st);
}

template <class T>
static hipError_t dgrad_launch_t(DwExactArgs& a, bool wave, size_t lds, hipStream_t st) {
  if (a.K == 3) return dgrad_launch_k<T, 3>(a, wave, lds, st);
  if (a.K == 5) return dgrad_launch_k<T, 5>(a, wave, lds, st);
  return dgrad_launch_k<T, 7>(a, wave, lds, st);
}

hipError_t launch_dw_exact_dgrad(const Geom& g, const void* w, const void* g_y, void* g_x, hipStream_t st) {
  DwExactArgs a = make_args(g);
  a.w = w; a.gy = g_y; a.gx = g_x;
  a.ppb = planes_per_block(g, dgrad_per_plane(g));
  const bool wave = g.H * g.W <= 256 && a.ppb >= 4;
  a.halo = dgrad_halo(g);
  a.PH = g.Hy + 2 * a.halo;
  a.PW = g.Wy + 2 * a.halo;
  const int in_bytes = g.s == 1 ? ((a.ppb * a.PH * a.PW * g.b + 15) & ~15)
                                : (((a.ppb * g.Hy * g.Wy * g.b + 32) + 15) & ~15);
  const int out_bytes = ((a.ppb * g.H * g.W * g.b + 32) + 15) & ~15;
  const size_t lds = (size_t)in_bytes + out_bytes;
  if (g.dtype == GF_BF16) return dgrad_launch_t<bf16_t>(a, wave, lds, st);
  return dgrad_launch_t<float>(a, wave, lds, st);
}

template <class T, int K>
static hipError_t wgrad_launch(DwExactArgs& a, bool wave, size_t lds, hipStream_t st) {
  const dim3 grid(cdiv(a.planes, a.ppb)), block(kThreads);
  if (a.s == 1) {
    if (wave) GF_LAUNCH((dw_exact_wgrad_s1_k<T, K, true>), grid, block, lds, st, a);
    else GF_LAUNCH((dw_exact_wgrad_s1_k<T, K, false>), grid, block, lds, st, a);
  } else {
    if (wave) GF_LAUNCH((dw_exact_wgrad_k<T, K, true>), grid, block, lds, st, a);
    else GF_LAUNCH((dw_exact_wgrad_k<T, K, false>), grid, block, lds, st, a);
  }
  return hipGetLastError();
}

hipError_t launch_dw_exact_wgrad(const Geom& g, const void* x, const void* g_y, float* g_w, void* ws,
                                 hipStream_t st) {
  DwExactArgs a = make_args(g);
  a.x = x; a.gy = g_y; a.part = static_cast<float*>(ws);
  a.ppb = planes_per_block(g, wgrad_per_plane(g));
  const bool wave = g.Hy * g.Wy <= 256 && a.ppb >= 4;
  a.halo = g.s == 1 ? g.p : 0;
  a.PH = g.H + 2 * a.halo;
  a.PW = g.W + 2 * a.halo;
  const int x_bytes = g.s == 1 ? ((a.ppb * a.PH * a.PW * g.b + 15) & ~15)
                               : (((a.ppb * g.H * g.W * g.b + 32) + 15) & ~15);
  const int y_bytes = ((a.ppb * g.Hy * g.Wy * g.b + 32) + 15) & ~15;
  const size_t lds = (size_t)x_bytes + y_bytes;
  hipError_t e;
  if (g.dtype == GF_BF16)
    e = g.Kh == 3 ? wgrad_launch<bf16_t, 3>(a, wave, lds, st) : wgrad_launch<bf16_t, 5>(a, wave, lds, st);
  else
    e = g.Kh == 3 ? wgrad_launch<float, 3>(a, wave, lds, st) : wgrad_launch<float, 5>(a, wave, lds, st);
  if (e != hipSuccess) return e;
  // g_theta[c, t] = sum over n of part[n, c, t]
  return launch_finalize(a.part, g_w, g.Ci * g.KK, g.N, 1, 1.f, st);
}

}  // namespace gf
