// Filtered backward from the reduced maps: kernel spatial sum (text after
// Eq. 3), weight gradient (Eq. 5) and input gradient (Eq. 3).
//
// This file holds the shape-generic kernels (any groups, any P, fp32 FMA with
// LDS tiling) and the depthwise kernels.  Reductions over the batch are done in
// two deterministic stages (partials in the workspace, then a fixed-order sum),
// never with floating-point atomics.
#include "gf_internal.h"

namespace gf {

namespace {

constexpr int kThreads = 256;

// ---------------------------------------------------------------------------
// S2: wsum[pair] = sum_t w[pair, t]
// ---------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(kThreads) void kernel_sum_k(const T* w, float* wsum, int pairs, int KK) {
  const int e = blockIdx.x * kThreads + threadIdx.x;
  if (e >= pairs) return;
  wsum[e] = kernel_sum_of(w, e, KK);
}

// ---------------------------------------------------------------------------
// finalize a two-stage reduction: g_w[pair, all taps] = scale * sum_z part[z, pair]
// ---------------------------------------------------------------------------
// 16 outputs per block, G lanes per output: lane zg sums slabs zg, zg + G, ... (all
// loads in flight together), then one lane adds the G sums in index order.
template <int G>
__global__ __launch_bounds__(kThreads) void finalize_gw_k(const float* part, float* g_w, int pairs,
                                                         int nz, int KK, float scale) {
  constexpr int OUT = kThreads / G;
  __shared__ float red[G][OUT + 1];
  const int o = threadIdx.x % OUT, zg = threadIdx.x / OUT;
  const int e = blockIdx.x * OUT + o;
  float acc = 0.f;
  if (e < pairs) {
    int z = zg;
    for (; z + 3 * G < nz; z += 4 * G) {
      const float v0 = part[(long)z * pairs + e], v1 = part[(long)(z + G) * pairs + e];
      const float v2 = part[(long)(z + 2 * G) * pairs + e], v3 = part[(long)(z + 3 * G) * pairs + e];
      acc += v0; acc += v1; acc += v2; acc += v3;
    }
    for (; z < nz; z += G) acc += part[(long)z * pairs + e];
  }
  red[zg][o] = acc;
  __syncthreads();
  if (zg == 0 && e < pairs) {
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < G; ++k) s += red[k][o];
    s *= scale;
    for (int t = 0; t < KK; ++t) g_w[(long)e * KK + t] = s;
  }
}

hipError_t launch_finalize_impl(const float* part, float* g_w, int pairs, int nz, int KK, float scale,
                                hipStream_t st) {
  if (nz >= 32)
    GF_LAUNCH(finalize_gw_k<16>, dim3(cdiv(pairs, kThreads / 16)), dim3(kThreads), 0, st, part, g_w, pairs, nz, KK, scale);
  else if (nz >= 8)
    GF_LAUNCH(finalize_gw_k<4>, dim3(cdiv(pairs, kThreads / 4)), dim3(kThreads), 0, st, part, g_w, pairs, nz, KK, scale);
  else
    GF_LAUNCH(finalize_gw_k<1>, dim3(cdiv(pairs, kThreads)), dim3(kThreads), 0, st, part, g_w, pairs, nz, KK, scale);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// S3 depthwise, stage 1: part[plane] = <x_u[plane, :], gy_u[plane, :]>,
// L lanes per plane (L a power of two <= 64), xor-shuffle reduction.
// ---------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(kThreads) void dw_dot_k(const T* xu, const T* gyu, float* part,
                                                    int planes, int P, int L) {
  const int gid = blockIdx.x * kThreads + threadIdx.x;
  const int plane = gid / L;
  const int lane = gid - plane * L;
  float acc = 0.f;
  if (plane < planes) {
    const T* a = xu + (long)plane * P;
    const T* b = gyu + (long)plane * P;
    for (int p = lane; p < P; p += L) acc += to_f32(a[p]) * to_f32(b[p]);
  }
  for (int m = L >> 1; m > 0; m >>= 1) acc += __shfl_xor(acc, m, 64);
  if (plane < planes && lane == 0) part[plane] = acc;
}

// Same with 16-byte loads (P a multiple of the vector length): L lanes per plane,
// each lane takes vectors lane, lane + L, ... of both operands.
template <class T>
__global__ __launch_bounds__(kThreads) void dw_dot_vec_k(const T* xu, const T* gyu, float* part,
                                                        int planes, int nvec, int L) {
  constexpr int VE = Vec16<T>::N;
  const int gid = blockIdx.x * kThreads + threadIdx.x;
  const int plane = gid / L;
  const int lane = gid - plane * L;
  float acc = 0.f;
  if (plane < planes) {
    const uint4* a = reinterpret_cast<const uint4*>(xu + (long)plane * nvec * VE);
    const uint4* b = reinterpret_cast<const uint4*>(gyu + (long)plane * nvec * VE);
    for (int v = lane; v < nvec; v += 2 * L) {
      const bool two = v + L < nvec;
      const uint4 a0 = a[v], b0 = b[v];
      const uint4 a1 = two ? a[v + L] : make_uint4(0, 0, 0, 0);
      const uint4 b1 = two ? b[v + L] : make_uint4(0, 0, 0, 0);
      float fa[VE], fb[VE];
      Vec16<T>::unpack(a0, fa);
      Vec16<T>::unpack(b0, fb);
#pragma unroll
      for (int e = 0; e < VE; ++e) acc += fa[e] * fb[e];
      Vec16<T>::unpack(a1, fa);
      Vec16<T>::unpack(b1, fb);
#pragma unroll
      for (int e = 0; e < VE; ++e) acc += fa[e] * fb[e];
    }
  }
  for (int m = L >> 1; m > 0; m >>= 1) acc += __shfl_xor(acc, m, 64);
  if (plane < planes && lane == 0) part[plane] = acc;
}

// ---------------------------------------------------------------------------
// Depthwise layer inside a chain of filtered layers: the weight-gradient partial of a plane
// (as dw_dot_k) and, in the same pass over gy_u, the reduced input gradient
// gxu[plane, p] = gy_u[plane, p] * (scalar * kernel sum of the plane's channel)   (Eq. 3).
// ---------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(kThreads) void dw_chain_k(const T* xu, const T* gyu, const T* w, float* part,
                                                      T* gxu, const T* mask, int planes, int P, int L, int C,
                                                      int KK, float scalar) {
  const int gid = blockIdx.x * kThreads + threadIdx.x;
  const int plane = gid / L;
  const int lane = gid - plane * L;
  float acc = 0.f;
  if (plane < planes) {
    const T* a = xu + (long)plane * P;
    const T* b = gyu + (long)plane * P;
    T* o = gxu + (long)plane * P;
    const T* mk = mask ? mask + (long)plane * P : nullptr;
    const float sc = scalar * kernel_sum_of(w, plane % C, KK);
    for (int p = lane; p < P; p += L) {
      const float gv = to_f32(b[p]);
      acc += to_f32(a[p]) * gv;
      T v = from_f32<T>(gv * sc);
      if (mk) v = from_f32<T>(to_f32(v) * to_f32(mk[p]));   // the rounded value times the mask fraction
      o[p] = v;
    }
  }
  for (int m = L >> 1; m > 0; m >>= 1) acc += __shfl_xor(acc, m, 64);
  if (plane < planes && lane == 0) part[plane] = acc;
}

// ---------------------------------------------------------------------------
// S3 generic: part[z, co, cl] = sum_{n in slab z} sum_p gy_u[n,co,p] * x_u[n,ci,p]
// 64 x 64 output tile per block, 4 x 4 per lane, K chunks of 16 patches.
// ---------------------------------------------------------------------------
struct WgradArgs {
  const void* xu;
  const void* gyu;
  float* part;
  int N, Ci, Co, Cg, Og, P;
  int tiles_co;  // per group
  int n_per_z;
};

template <class T>
__global__ __launch_bounds__(kThreads) void gf_wgrad_tile_k(WgradArgs a) {
  __shared__ float As[16][65];  // [k][co]
  __shared__ float Bs[16][65];  // [k][cl]
  const T* xu = static_cast<const T*>(a.xu);
  const T* gyu = static_cast<const T*>(a.gyu);
  const int tid = threadIdx.x;
  const int grp = blockIdx.y / a.tiles_co;
  const int ol0 = (blockIdx.y - grp * a.tiles_co) * 64;  // first c_o of the tile, local to the group
  const int cl0 = blockIdx.x * 64;
  const int n0 = blockIdx.z * a.n_per_z;
  const int n1 = min(n0 + a.n_per_z, a.N);
  const int ty = tid >> 4, tx = tid & 15;
  float acc[4][4] = {};
  for (int n = n0; n < n1; ++n) {
    const T* ga = gyu + ((long)n * a.Co + grp * a.Og) * a.P;
    const T* gb = xu + ((long)n * a.Ci + grp * a.Cg) * a.P;
    for (int p0 = 0; p0 < a.P; p0 += 16) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int e = tid + i * kThreads;
        const int row = e >> 4, k = e & 15;
        const bool kin = p0 + k < a.P;
        As[k][row] = (kin && ol0 + row < a.Og) ? to_f32(ga[(long)(ol0 + row) * a.P + p0 + k]) : 0.f;
        Bs[k][row] = (kin && cl0 + row < a.Cg) ? to_f32(gb[(long)(cl0 + row) * a.P + p0 + k]) : 0.f;
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        float av[4], bv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) av[i] = As[k][ty * 4 + i];
#pragma unroll
        for (int j = 0; j < 4; ++j) bv[j] = Bs[k][tx * 4 + j];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] += av[i] * bv[j];
      }
      __syncthreads();
    }
  }
  float* dst = a.part + (long)blockIdx.z * a.Co * a.Cg;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int ol = ol0 + ty * 4 + i;
    if (ol >= a.Og) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int cl = cl0 + tx * 4 + j;
      if (cl < a.Cg) dst[(long)(grp * a.Og + ol) * a.Cg + cl] = acc[i][j];
    }
  }
}

// ---------------------------------------------------------------------------
// S4 generic, reduced map: dst[n, ci, p] = scale * sum_ol wsum[co, cl] * gy_u[n, co, p]
// 64 (ci) x 64 (p) tile per block, K chunks of 16 output channels.
// ---------------------------------------------------------------------------
struct DgradArgs {
  const void* gyu;
  const float* wsum;
  void* dst;
  int N, Ci, Co, Cg, Og, P;
  int tiles_ci;  // per group
  float scale;
};

template <class T, class D>
__global__ __launch_bounds__(kThreads) void gf_dgrad_tile_k(DgradArgs a) {
  __shared__ float As[16][65];  // [k = ol][cl]
  __shared__ float Bs[16][65];  // [k = ol][p]
  const T* gyu = static_cast<const T*>(a.gyu);
  D* dst = static_cast<D*>(a.dst);
  const int tid = threadIdx.x;
  const int n = blockIdx.z;
  const int grp = blockIdx.y / a.tiles_ci;
  const int cl0 = (blockIdx.y - grp * a.tiles_ci) * 64;
  const int p0 = blockIdx.x * 64;
  const int ty = tid >> 4, tx = tid & 15;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < a.Og; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + i * kThreads;
      const int k = e >> 6, col = e & 63;
      const bool kin = k0 + k < a.Og;
      const int co = grp * a.Og + k0 + k;
      As[k][col] = (kin && cl0 + col < a.Cg) ? a.wsum[(long)co * a.Cg + cl0 + col] : 0.f;
      Bs[k][col] = (kin && p0 + col < a.P) ? to_f32(gyu[((long)n * a.Co + co) * a.P + p0 + col]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) bv[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += av[i] * bv[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int cl = cl0 + ty * 4 + i;
    if (cl >= a.Cg) continue;
    const int ci = grp * a.Cg + cl;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int p = p0 + tx * 4 + j;
      if (p < a.P) dst[((long)n * a.Ci + ci) * a.P + p] = from_f32<D>(acc[i][j] * a.scale);
    }
  }
}

// ---------------------------------------------------------------------------
// Expansion to full resolution: out[plane, h, w] = f(src[plane, h/rx, w/rx]),
// f(v) = v * chscale[plane % C] * scalar (chscale may be null).  Each lane
// produces one 16-byte run of consecutive output elements; the run may cross
// rows and planes, so indices are advanced element by element.
// ---------------------------------------------------------------------------
struct ExpandArgs {
  const void* src;
  void* out;
  const float* chscale;
  float scalar;
  int C, H, W, rx, Hp, Wp;
  int total;  // planes * H * W
  FastDiv d_hw, d_w, d_rx, d_c, d_p;
};

template <class T, class S>
__global__ __launch_bounds__(kThreads) void expand_k(ExpandArgs a) {
  constexpr int V = 16 / (int)sizeof(T);
  const S* src = static_cast<const S*>(a.src);
  T* out = static_cast<T*>(a.out);
  const int e0 = (blockIdx.x * kThreads + threadIdx.x) * V;
  if (e0 >= a.total) return;
  const int HW = a.H * a.W;
  int plane = (int)a.d_hw.div((uint32_t)e0);
  int rem = e0 - plane * HW;
  int h = (int)a.d_w.div((uint32_t)rem);
  int w = rem - h * a.W;
  int hp = (int)a.d_rx.div((uint32_t)h), hr = h - hp * a.rx;
  int wp = (int)a.d_rx.div((uint32_t)w), wr = w - wp * a.rx;
  const int P = a.Hp * a.Wp;
  // source index and channel of every element first, then all loads together (a load inside
  // the stepping loop would be waited for before the next one is issued)
  int sidx[V], chan[V];
  const int last = a.total - 1 - e0;  // elements past the end repeat the last valid one
  int c = plane - (int)a.d_c.div((uint32_t)plane) * a.C;
#pragma unroll
  for (int k = 0; k < V; ++k) {
    if (k <= last) {
      sidx[k] = plane * P + hp * a.Wp + wp;
      chan[k] = c;
    } else {
      sidx[k] = sidx[k > 0 ? k - 1 : 0];
      chan[k] = chan[k > 0 ? k - 1 : 0];
    }
    // advance one output element
    ++w;
    if (++wr == a.rx) { wr = 0; ++wp; }
    if (w == a.W) {
      w = 0; wp = 0; wr = 0;
      ++h;
      if (++hr == a.rx) { hr = 0; ++hp; }
      if (h == a.H) {
        h = 0; hp = 0; hr = 0;
        ++plane;
        if (++c == a.C) c = 0;
      }
    }
  }
  S sv[V];
  float scv[V];
#pragma unroll
  for (int k = 0; k < V; ++k) sv[k] = src[sidx[k]];
#pragma unroll
  for (int k = 0; k < V; ++k) scv[k] = a.chscale ? a.chscale[chan[k]] : 1.f;
  T vals[V];
#pragma unroll
  for (int k = 0; k < V; ++k) vals[k] = from_f32<T>(to_f32(sv[k]) * (a.scalar * scv[k]));
  if (e0 + V <= a.total) {
    *reinterpret_cast<uint4*>(out + e0) = *reinterpret_cast<const uint4*>(vals);
  } else {
    for (int k = 0; e0 + k < a.total; ++k) out[e0 + k] = vals[k];
  }
}

// The same for small or unaligned maps, through LDS: a block writes 8192 consecutive output
// elements, which belong to a few whole or partial planes; their scaled source values
// (planes * P of them, at most kExpandLdsMax) are first loaded with coalesced reads, then every
// lane gathers its 16-byte run from LDS.  Same arithmetic as expand_k: src * (scalar * chscale).
constexpr int kExpandLdsMax = 4096;
constexpr int kExpandPerBlock = kThreads * 32;

template <class T, class S>
__global__ __launch_bounds__(kThreads) void expand_lds_k(ExpandArgs a) {
  constexpr int V = 16 / (int)sizeof(T);
  constexpr int PER = kExpandPerBlock / (kThreads * V);  // 16-byte runs per lane
  __shared__ float sval[kExpandLdsMax];
  const S* src = static_cast<const S*>(a.src);
  T* out = static_cast<T*>(a.out);
  const int HW = a.H * a.W, P = a.Hp * a.Wp;
  const int b0 = blockIdx.x * kExpandPerBlock;
  const int b1 = min(b0 + kExpandPerBlock, a.total);
  const int plane0 = (int)a.d_hw.div((uint32_t)b0);
  const int plane1 = (int)a.d_hw.div((uint32_t)(b1 - 1));
  const int nsrc = (plane1 - plane0 + 1) * P;
  for (int i = threadIdx.x; i < nsrc; i += kThreads) {
    const int pl = plane0 + (int)a.d_p.div((uint32_t)i);
    const int c = pl - (int)a.d_c.div((uint32_t)pl) * a.C;
    const float sc = a.scalar * (a.chscale ? a.chscale[c] : 1.f);
    sval[i] = to_f32(src[(long)plane0 * P + i]) * sc;
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < PER; ++it) {
    const int e0 = b0 + (it * kThreads + threadIdx.x) * V;
    if (e0 >= b1) break;
    int plane = (int)a.d_hw.div((uint32_t)e0);
    int rem = e0 - plane * HW;
    int h = (int)a.d_w.div((uint32_t)rem);
    int w = rem - h * a.W;
    int hp = (int)a.d_rx.div((uint32_t)h), hr = h - hp * a.rx;
    int wp = (int)a.d_rx.div((uint32_t)w), wr = w - wp * a.rx;
    int base = (plane - plane0) * P;
    T vals[V];
#pragma unroll
    for (int k = 0; k < V; ++k) {
      vals[k] = from_f32<T>(sval[min(base + hp * a.Wp + wp, nsrc - 1)]);
      ++w;
      if (++wr == a.rx) { wr = 0; ++wp; }
      if (w == a.W) {
        w = 0; wp = 0; wr = 0;
        ++h;
        if (++hr == a.rx) { hr = 0; ++hp; }
        if (h == a.H) { h = 0; hp = 0; hr = 0; base += P; }
      }
    }
    if (e0 + V <= a.total) {
      *reinterpret_cast<uint4*>(out + e0) = *reinterpret_cast<const uint4*>(vals);
    } else {
      for (int k = 0; e0 + k < a.total; ++k) out[e0 + k] = vals[k];
    }
  }
}

// Fast path: rows are 16-byte multiples, r_x is a power of two that divides W.
// One lane per (patch row, 16-byte column vector): it reads the few source values
// the vector needs once, builds the vector, and stores it to the r_x output rows.
// With `wdw` set the per-channel scale is the depthwise kernel sum, formed here
// (text after Eq. 3) instead of in a launch of its own.
struct ExpandRowsArgs {
  const void* src;
  void* out;
  const float* chscale;  // per channel, or null
  const void* wdw;       // depthwise weights [C, KK], or null
  int KK;
  float scalar;
  int C, H, W, Hp, Wp;
  int vpr;               // 16-byte vectors per output row
  int total_items;       // planes * Hp * vpr
  FastDiv d_vpr, d_hp, d_c;
};

template <class T, class S, int RX>
__global__ __launch_bounds__(kThreads) void expand_rows_k(ExpandRowsArgs a) {
  constexpr int VE = Vec16<T>::N;
  constexpr int NS = VE >= RX ? VE / RX : 1;  // source values per output vector
  const int t = blockIdx.x * kThreads + threadIdx.x;
  if (t >= a.total_items) return;
  const S* src = static_cast<const S*>(a.src);
  T* out = static_cast<T*>(a.out);
  const int s = (int)a.d_vpr.div((uint32_t)t);   // strip = plane * Hp + hp
  const int v = t - s * a.vpr;
  const int pl = (int)a.d_hp.div((uint32_t)s);
  const int hp = s - pl * a.Hp;
  float sc = a.scalar;
  if (a.chscale || a.wdw) {
    const int c = pl - (int)a.d_c.div((uint32_t)pl) * a.C;
    if (a.wdw) {
      sc *= kernel_sum_of(static_cast<const T*>(a.wdw), c, a.KK);
    } else {
      sc *= a.chscale[c];
    }
  }
  const int wp0 = VE >= RX ? v * NS : (v * VE) / RX;
  const S* sp = src + (long)s * a.Wp + wp0;
  float f[VE];
#pragma unroll
  for (int k = 0; k < NS; ++k) {
    const float val = to_f32(sp[k]) * sc;
#pragma unroll
    for (int j = 0; j < VE / NS; ++j) f[k * (VE / NS) + j] = val;
  }
  // round once, then replicate the rounded bits
  const uint4 vec = Vec16<T>::pack(f);
  const int rows = min(RX, a.H - hp * RX);
  T* dst = out + ((long)pl * a.H + (long)hp * RX) * a.W + v * VE;
  for (int i = 0; i < rows; ++i) *reinterpret_cast<uint4*>(dst + (long)i * a.W) = vec;
}

template <class T, class S, int RX>
hipError_t launch_expand_rows(ExpandRowsArgs& a, hipStream_t st) {
  GF_LAUNCH((expand_rows_k<T, S, RX>), dim3(cdiv(a.total_items, kThreads)), dim3(kThreads),
                     0, st, a);
  return hipGetLastError();
}

// The same for planes small enough to stage, without per-channel factors: a block owns a run of
// whole consecutive planes (contiguous in the output), builds their pixels in LDS -- every patch
// value times `scalar`, rounded once to the storage type, written to its r_x x r_x pixels -- and
// streams the run out with 16-byte vectors.  The planes per block are a multiple of the smallest
// count whose bytes are a multiple of 16, so every run starts on a 16-byte boundary; only the
// last block can end with a partial vector.
struct ExpandPlanesArgs {
  const void* src;   // [planes, P]
  void* out;         // [planes, H, W]
  float scalar;
  int planes, ppb, H, W, Wp, P, rx;
  FastDiv d_p, d_wp;
};

template <class T, class S>
__global__ __launch_bounds__(kThreads) void expand_planes_k(ExpandPlanesArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  T* img = reinterpret_cast<T*>(smem);
  const int tid = threadIdx.x;
  const int pl0 = blockIdx.x * a.ppb;
  const int np = min(a.ppb, a.planes - pl0);
  const int HW = a.H * a.W;
  const S* src = static_cast<const S*>(a.src) + (long)pl0 * a.P;
  for (int i = tid; i < np * a.P; i += kThreads) {
    const int pl = (int)a.d_p.div((uint32_t)i);
    const int pp = i - pl * a.P;
    const int hp = (int)a.d_wp.div((uint32_t)pp);
    const int wp = pp - hp * a.Wp;
    const T v = from_f32<T>(to_f32(src[i]) * a.scalar);
    const int h1 = min(a.H, (hp + 1) * a.rx), w1 = min(a.W, (wp + 1) * a.rx);
    for (int h = hp * a.rx; h < h1; ++h)
      for (int w = wp * a.rx; w < w1; ++w) img[pl * HW + h * a.W + w] = v;
  }
  __syncthreads();
  T* out = static_cast<T*>(a.out) + (long)pl0 * HW;
  const int nelem = np * HW;
  constexpr int VE = 16 / (int)sizeof(T);
  const int nvec = nelem / VE;
  for (int v = tid; v < nvec; v += kThreads)
    store_stream16(out + (long)v * VE, *reinterpret_cast<const uint4*>(smem + ((long)v << 4)));
  for (int e = nvec * VE + tid; e < nelem; e += kThreads) out[e] = img[e];
}

constexpr int kExpandPlanesLds = 32 * 1024;

// planes per block of expand_planes_k, 0 if the planes are too large to stage
static int expand_planes_per_block(long planes, int H, int W, int elem_bytes) {
  const long plane_bytes = (long)H * W * elem_bytes;
  long gcd = 16, r = plane_bytes % 16;
  while (r) { const long t = gcd % r; gcd = r; r = t; }
  const long align = 16 / gcd;                                // planes whose bytes are a multiple of 16
  if (align * plane_bytes > kExpandPlanesLds) return 0;
  long ppb = (kExpandPlanesLds / (align * plane_bytes)) * align;
  while (ppb > align && planes / ppb < 1024) ppb -= align;    // enough blocks for the chip
  return (int)ppb;
}

template <class T, class S>
hipError_t launch_expand(const S* src, T* out, const float* chscale, float scalar, long planes,
                         int C, int H, int W, int rx, int Hp, int Wp, hipStream_t st,
                         const void* wdw = nullptr, int KK = 0, float* wsum_scratch = nullptr) {
  constexpr int VEC = 16 / (int)sizeof(T);
  const bool pow2 = rx == 2 || rx == 4 || rx == 8 || rx == 16;
  if (pow2 && W % VEC == 0 && W % rx == 0 && planes * Hp * (W / VEC) < 2147483647L) {
    ExpandRowsArgs e;
    e.src = src; e.out = out; e.chscale = wdw ? nullptr : chscale; e.wdw = wdw; e.KK = KK;
    e.scalar = scalar; e.C = C; e.H = H; e.W = W; e.Hp = Hp; e.Wp = Wp;
    e.vpr = W / VEC;
    e.total_items = (int)(planes * Hp * e.vpr);
    e.d_vpr = FastDiv((uint32_t)e.vpr);
    e.d_hp = FastDiv((uint32_t)Hp);
    e.d_c = FastDiv((uint32_t)C);
    if (rx == 2) return launch_expand_rows<T, S, 2>(e, st);
    if (rx == 4) return launch_expand_rows<T, S, 4>(e, st);
    if (rx == 8) return launch_expand_rows<T, S, 8>(e, st);
    return launch_expand_rows<T, S, 16>(e, st);
  }
  if (!wdw && !chscale) {
    const int ppb = expand_planes_per_block(planes, H, W, (int)sizeof(T));
    if (ppb > 0) {
      ExpandPlanesArgs e;
      e.src = src; e.out = out; e.scalar = scalar;
      e.planes = (int)planes; e.ppb = ppb; e.H = H; e.W = W; e.Wp = Wp; e.P = Hp * Wp; e.rx = rx;
      e.d_p = FastDiv((uint32_t)(Hp * Wp));
      e.d_wp = FastDiv((uint32_t)Wp);
      GF_LAUNCH((expand_planes_k<T, S>), dim3(cdiv(planes, ppb)), dim3(kThreads),
                         (size_t)ppb * H * W * sizeof(T), st, e);
      return hipGetLastError();
    }
  }
  if (wdw) {  // generic path wants the per-channel sums in memory
    hipError_t err = launch_kernel_sum(wdw, wsum_scratch, C, KK, sizeof(T) == 2 ? GF_BF16 : GF_F32, st);
    if (err != hipSuccess) return err;
    chscale = wsum_scratch;
  }
  ExpandArgs a;
  a.src = src;
  a.out = out;
  a.chscale = chscale;
  a.scalar = scalar;
  a.C = C;
  a.H = H;
  a.W = W;
  a.rx = rx;
  a.Hp = Hp;
  a.Wp = Wp;
  a.total = (int)(planes * H * W);
  a.d_hw = FastDiv((uint32_t)(H * W));
  a.d_w = FastDiv((uint32_t)W);
  a.d_rx = FastDiv((uint32_t)rx);
  a.d_c = FastDiv((uint32_t)C);
  a.d_p = FastDiv((uint32_t)(Hp * Wp));
  // planes a block of kExpandPerBlock outputs can touch, times the values per plane
  if (((long)kExpandPerBlock / (H * W) + 2) * Hp * Wp <= kExpandLdsMax) {
    GF_LAUNCH((expand_lds_k<T, S>), dim3(cdiv(a.total, kExpandPerBlock)), dim3(kThreads), 0, st, a);
    return hipGetLastError();
  }
  constexpr int V = 16 / (int)sizeof(T);
  const int blocks = cdiv(cdiv(a.total, V), kThreads);
  GF_LAUNCH((expand_k<T, S>), dim3(blocks), dim3(kThreads), 0, st, a);
  return hipGetLastError();
}

int dw_lanes(int P) {
  int L = 1;
  while (L < P && L < 64) L <<= 1;
  return L;
}

bool is_depthwise(const Geom& g) { return g.Cg == 1 && g.Og == 1; }

int wgrad_splits(const Geom& g) {
  // enough blocks to cover the chip: tiles * splits >= ~512, at most one image per split
  const int tiles = g.g * cdiv(g.Og, 64) * cdiv(g.Cg, 64);
  int z = cdiv(512, tiles);
  if (z > g.N) z = g.N;
  if (z < 1) z = 1;
  const int n_per_z = cdiv(g.N, z);
  return cdiv(g.N, n_per_z);
}

}  // namespace

bool is_depthwise_layer(const Geom& g) { return is_depthwise(g); }

hipError_t launch_finalize(const float* part, float* g_w, int pairs, int nz, int KK, float scale,
                           hipStream_t st) {
  return launch_finalize_impl(part, g_w, pairs, nz, KK, scale, st);
}

hipError_t launch_kernel_sum(const void* w, float* wsum, long pairs, int KK, int dtype,
                             hipStream_t st) {
  const int blocks = cdiv(pairs, kThreads);
  if (dtype == GF_BF16)
    GF_LAUNCH(kernel_sum_k<bf16_t>, dim3(blocks), dim3(kThreads), 0, st,
                       static_cast<const bf16_t*>(w), wsum, (int)pairs, KK);
  else
    GF_LAUNCH(kernel_sum_k<float>, dim3(blocks), dim3(kThreads), 0, st,
                       static_cast<const float*>(w), wsum, (int)pairs, KK);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// S3
// ---------------------------------------------------------------------------
size_t ws_bwd_weight(const Geom& g) {
  if (is_depthwise(g)) return (size_t)g.N * g.Ci * sizeof(float);
  if (g.g == 1) return (size_t)mfma_wgrad_splits(g, nullptr) * g.Co * g.Ci * sizeof(float);
  return (size_t)wgrad_splits(g) * g.Co * g.Cg * sizeof(float);
}

hipError_t launch_gf_bwd_weight(const Geom& g, const void* x_u, const void* gy_u, float* g_w,
                                void* ws, hipStream_t st) {
  float* part = static_cast<float*>(ws);
  const float scale = 1.f / ((float)g.s * (float)g.s);
  const int pairs = g.Co * g.Cg;
  int nz;
  if (is_depthwise(g)) {
    const int planes = g.N * g.Ci;
    const int VE = 16 / g.b;
    if (g.P % VE == 0) {
      const int nvec = g.P / VE;
      const int L = dw_lanes(cdiv(nvec, 2));
      const int blocks = cdiv((long)planes * L, kThreads);
      if (g.dtype == GF_BF16)
        GF_LAUNCH(dw_dot_vec_k<bf16_t>, dim3(blocks), dim3(kThreads), 0, st,
                           static_cast<const bf16_t*>(x_u), static_cast<const bf16_t*>(gy_u), part,
                           planes, nvec, L);
      else
        GF_LAUNCH(dw_dot_vec_k<float>, dim3(blocks), dim3(kThreads), 0, st,
                           static_cast<const float*>(x_u), static_cast<const float*>(gy_u), part,
                           planes, nvec, L);
    } else {
    const int L = dw_lanes(g.P);
    const int blocks = cdiv((long)planes * L, kThreads);
    if (g.dtype == GF_BF16)
      GF_LAUNCH(dw_dot_k<bf16_t>, dim3(blocks), dim3(kThreads), 0, st,
                         static_cast<const bf16_t*>(x_u), static_cast<const bf16_t*>(gy_u), part,
                         planes, g.P, L);
    else
      GF_LAUNCH(dw_dot_k<float>, dim3(blocks), dim3(kThreads), 0, st,
                         static_cast<const float*>(x_u), static_cast<const float*>(gy_u), part,
                         planes, g.P, L);
    }
    nz = g.N;
  } else if (g.g == 1) {
    hipError_t e = launch_mfma_wgrad(g, x_u, gy_u, part, &nz, st);
    if (e != hipSuccess) return e;
  } else {
    WgradArgs a;
    a.xu = x_u;
    a.gyu = gy_u;
    a.part = part;
    a.N = g.N;
    a.Ci = g.Ci;
    a.Co = g.Co;
    a.Cg = g.Cg;
    a.Og = g.Og;
    a.P = g.P;
    a.tiles_co = cdiv(g.Og, 64);
    nz = wgrad_splits(g);
    a.n_per_z = cdiv(g.N, nz);
    dim3 grid(cdiv(g.Cg, 64), g.g * a.tiles_co, nz);
    if (g.dtype == GF_BF16)
      GF_LAUNCH(gf_wgrad_tile_k<bf16_t>, grid, dim3(kThreads), 0, st, a);
    else
      GF_LAUNCH(gf_wgrad_tile_k<float>, grid, dim3(kThreads), 0, st, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_finalize_impl(part, g_w, pairs, nz, g.KK, scale, st);
}

// ---------------------------------------------------------------------------
// S2 + S4
// ---------------------------------------------------------------------------
static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

size_t ws_bwd_input(const Geom& g, bool reduced_out) {
  size_t wsum = align256((size_t)g.Co * g.Cg * sizeof(float));
  if (is_depthwise(g) || reduced_out) return wsum;
  if (g.g == 1) return wsum + (size_t)g.N * g.Ci * g.P * g.b;
  return wsum + (size_t)g.N * g.Ci * g.P * sizeof(float);
}

template <class T>
static hipError_t bwd_input_t(const Geom& g, const T* gy_u, const T* w, T* g_x, bool reduced_out,
                              void* ws, hipStream_t st) {
  float* wsum = static_cast<float*>(ws);
  const float scale = 1.f / ((float)g.s * (float)g.s);
  const long planes = (long)g.N * g.Ci;
  hipError_t e;
  if (is_depthwise(g)) {
    if (reduced_out)
      return launch_expand<T, T>(gy_u, g_x, nullptr, scale, planes, g.Ci, g.Hp, g.Wp, 1, g.Hp, g.Wp, st,
                                 w, g.KK, wsum);
    return launch_expand<T, T>(gy_u, g_x, nullptr, scale, planes, g.Ci, g.H, g.W, g.rx, g.Hp, g.Wp, st,
                               w, g.KK, wsum);
  }
  if (g.g == 1) {  // dense: MFMA GEMM to the reduced map (storage type), then replicate
    if (reduced_out) return launch_mfma_dgrad(g, gy_u, w, ws, g_x, nullptr, st);
    if (mfma_dgrad_writes_full(g)) return launch_mfma_dgrad(g, gy_u, w, ws, nullptr, g_x, st);
    T* redt = reinterpret_cast<T*>(static_cast<char*>(ws) + align256((size_t)g.Co * g.Cg * sizeof(float)));
    e = launch_mfma_dgrad(g, gy_u, w, ws, redt, nullptr, st);
    if (e != hipSuccess) return e;
    return launch_expand<T, T>(redt, g_x, nullptr, 1.f, planes, g.Ci, g.H, g.W, g.rx, g.Hp, g.Wp, st);
  }
  e = launch_kernel_sum(w, wsum, (long)g.Co * g.Cg, g.KK, g.dtype, st);
  if (e != hipSuccess) return e;
  DgradArgs a;
  a.gyu = gy_u;
  a.wsum = wsum;
  a.N = g.N;
  a.Ci = g.Ci;
  a.Co = g.Co;
  a.Cg = g.Cg;
  a.Og = g.Og;
  a.P = g.P;
  a.tiles_ci = cdiv(g.Cg, 64);
  a.scale = scale;
  dim3 grid(cdiv(g.P, 64), g.g * a.tiles_ci, g.N);
  if (reduced_out) {
    a.dst = g_x;
    GF_LAUNCH((gf_dgrad_tile_k<T, T>), grid, dim3(kThreads), 0, st, a);
    return hipGetLastError();
  }
  float* red = reinterpret_cast<float*>(static_cast<char*>(ws) +
                                        align256((size_t)g.Co * g.Cg * sizeof(float)));
  a.dst = red;
  GF_LAUNCH((gf_dgrad_tile_k<T, float>), grid, dim3(kThreads), 0, st, a);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_expand<T, float>(red, g_x, nullptr, 1.f, planes, g.Ci, g.H, g.W, g.rx, g.Hp, g.Wp, st);
}

hipError_t launch_expand_f32(const Geom& g, const float* red, void* g_x, hipStream_t st) {
  const long planes = (long)g.N * g.Ci;
  if (g.dtype == GF_BF16)
    return launch_expand<bf16_t, float>(red, static_cast<bf16_t*>(g_x), nullptr, 1.f, planes, g.Ci, g.H, g.W, g.rx,
                                        g.Hp, g.Wp, st);
  return launch_expand<float, float>(red, static_cast<float*>(g_x), nullptr, 1.f, planes, g.Ci, g.H, g.W, g.rx, g.Hp,
                                     g.Wp, st);
}

// g_x[n, c, h, w] = red[n, c, h / r_x, w / r_x]: a reduced map in the storage type to full resolution
hipError_t launch_replicate(const Geom& g, const void* red, void* g_x, hipStream_t st) {
  const long planes = (long)g.N * g.Ci;
  if (g.dtype == GF_BF16)
    return launch_expand<bf16_t, bf16_t>(static_cast<const bf16_t*>(red), static_cast<bf16_t*>(g_x), nullptr, 1.f,
                                         planes, g.Ci, g.H, g.W, g.rx, g.Hp, g.Wp, st);
  return launch_expand<float, float>(static_cast<const float*>(red), static_cast<float*>(g_x), nullptr, 1.f, planes,
                                     g.Ci, g.H, g.W, g.rx, g.Hp, g.Wp, st);
}

hipError_t launch_gf_bwd_input(const Geom& g, const void* gy_u, const void* w, void* g_x,
                               bool reduced_out, void* ws, hipStream_t st) {
  if (g.dtype == GF_BF16)
    return bwd_input_t<bf16_t>(g, static_cast<const bf16_t*>(gy_u), static_cast<const bf16_t*>(w),
                               static_cast<bf16_t*>(g_x), reduced_out, ws, st);
  return bwd_input_t<float>(g, static_cast<const float*>(gy_u), static_cast<const float*>(w),
                            static_cast<float*>(g_x), reduced_out, ws, st);
}

// Depthwise layer of a chain: partial dot products [N, C] and the reduced input gradient in one
// launch (then launch_finalize with nz = N).
hipError_t launch_dw_chain(const Geom& g, const void* x_u, const void* gy_u, const void* w, float* part,
                           void* g_xu, const void* mask_u, hipStream_t st) {
  const int planes = g.N * g.Ci;
  const int L = dw_lanes(g.P);
  const int blocks = cdiv((long)planes * L, kThreads);
  const float scalar = 1.f / ((float)g.s * (float)g.s);
  if (g.dtype == GF_BF16)
    GF_LAUNCH(dw_chain_k<bf16_t>, dim3(blocks), dim3(kThreads), 0, st, static_cast<const bf16_t*>(x_u),
                       static_cast<const bf16_t*>(gy_u), static_cast<const bf16_t*>(w), part,
                       static_cast<bf16_t*>(g_xu), static_cast<const bf16_t*>(mask_u), planes, g.P, L, g.Ci, g.KK,
                       scalar);
  else
    GF_LAUNCH(dw_chain_k<float>, dim3(blocks), dim3(kThreads), 0, st, static_cast<const float*>(x_u),
                       static_cast<const float*>(gy_u), static_cast<const float*>(w), part,
                       static_cast<float*>(g_xu), static_cast<const float*>(mask_u), planes, g.P, L, g.Ci, g.KK,
                       scalar);
  return hipGetLastError();
}

}  // namespace gf
