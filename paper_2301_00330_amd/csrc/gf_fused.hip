// One launch for the whole filtered backward of a depthwise layer:
// gradient filter (Eq. 2), weight gradient (Eq. 5) and input gradient (Eq. 3).
// g_y is read once; the patch means are rounded to the storage type exactly as the
// stand-alone filter stores them, multiplied with x_u for the weight-gradient
// partial, scaled by the kernel sum (text after Eq. 3, formed in the kernel) and
// written back over the same pixel positions as g_x.  Two stride-1 variants mirror the two
// patch-reduction kernels: register rows for 16-byte-aligned maps, LDS-staged
// flat planes for small or ragged maps.  Strided layers use a third, LDS-staged variant
// with separate images of the g_y run and of the (s^2 times larger) g_x run.
#include "gf_internal.h"

namespace gf {

namespace {

constexpr int kThreads = 256;
constexpr int kLdsBudget = 40 * 1024;

struct DwFusedArgs {
  const void* gy;
  const void* xu;
  const void* w;
  void* gyu;    // nullable
  void* gx;
  float* part;  // [N * cpp, C] partial dot products
  int C, H, W, Hp, Wp, P, KK, q;
  int planes;
  float scale;
  // rows variant
  int ipr, ipp, cpp;  // items per row / per plane, chunks per plane
  FastDiv d_ipr, d_cpp, d_c;
  // LDS variants
  int ppb;            // planes per block
  FastDiv d_wp, d_p;
  // strided LDS variant: g_y is [planes, Hy, Wy], patches q on g_y and qx = q * stride on g_x
  int Hy, Wy, qx;
};

// fixed-order block sum of one float per lane; result valid in lane 0 of the block
__device__ __forceinline__ float block_sum(float v, float* red) {
  for (int m = 32; m > 0; m >>= 1) v += __shfl_xor(v, m, 64);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  float s = 0.f;
  if (threadIdx.x == 0)
    for (int k = 0; k < (int)(blockDim.x >> 6); ++k) s += red[k];
  __syncthreads();
  return s;
}

constexpr int kMaxRowsThreads = 512;

// Blocks of the rows variant: a plane's items are cut into `cpp` equal chunks of at most 512 and
// a block has just enough waves for one chunk (a fixed 256 would leave a quarter of the lanes
// idle on a 56 x 56 plane, which has 392 items).
inline int rows_chunks(int ipp, int* nthreads) {
  const int cpp = cdiv(ipp, kMaxRowsThreads);
  *nthreads = 64 * cdiv(cdiv(ipp, cpp), 64);
  return cpp;
}

// ---------------------------------------------------------------------------
// rows variant: W % max(VE, Q) == 0, rows 16-byte multiples, stride 1
// block = (U consecutive planes, one chunk of 256 items); lane u-th item belongs to plane u
// ---------------------------------------------------------------------------
template <class T, int Q, int U>
__global__ __launch_bounds__(kMaxRowsThreads) void dw_fused_rows_k(DwFusedArgs a) {
  constexpr int VE = Vec16<T>::N;
  constexpr int IW = VE > Q ? VE : Q;
  constexpr int VW = IW / VE;
  constexpr int NOUT = IW / Q;
  __shared__ float red[kMaxRowsThreads / 64];
  const T* gy = static_cast<const T*>(a.gy);
  const T* xu = static_cast<const T*>(a.xu);
  const T* w = static_cast<const T*>(a.w);
  T* gx = static_cast<T*>(a.gx);
  T* gyu = static_cast<T*>(a.gyu);
  const int pg = (int)a.d_cpp.div(blockIdx.x);
  const int chunk = blockIdx.x - pg * a.cpp;
  const int item = chunk * (int)blockDim.x + threadIdx.x;
  const bool item_ok = item < a.ipp;
  const int itc = min(item, a.ipp - 1);
  const int hp = (int)a.d_ipr.div((uint32_t)itc);
  const int col = itc - hp * a.ipr;
  const int rows = min(Q, a.H - hp * Q);

  uint4 v[U][Q][VW];
  T xv[U][NOUT];
  float sc[U];
  int plane[U];
  // kernel sums first: their loads retire before the wide ones issued after them
#pragma unroll
  for (int u = 0; u < U; ++u) {
    plane[u] = pg * U + u;
    const int pc = min(plane[u], a.planes - 1);
    const int c = pc - (int)a.d_c.div((uint32_t)pc) * a.C;
    sc[u] = kernel_sum_of(w, c, a.KK) * a.scale;
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int pc = min(plane[u], a.planes - 1);
    const T* p = gy + ((long)pc * a.H + (long)hp * Q) * a.W + col * IW;
#pragma unroll
    for (int i = 0; i < Q; ++i) {
      const int ri = min(i, rows - 1);
#pragma unroll
      for (int k = 0; k < VW; ++k)
        v[u][i][k] = *reinterpret_cast<const uint4*>(p + (long)ri * a.W + k * VE);
    }
    const T* xp = xu + (long)pc * a.P + hp * a.Wp + col * NOUT;
#pragma unroll
    for (int o = 0; o < NOUT; ++o) xv[u][o] = xp[o];
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const bool ok = item_ok && plane[u] < a.planes;
    float colsum[IW];
#pragma unroll
    for (int e = 0; e < IW; ++e) colsum[e] = 0.f;
#pragma unroll
    for (int i = 0; i < Q; ++i)
#pragma unroll
      for (int k = 0; k < VW; ++k) {
        float f[VE];
        Vec16<T>::unpack(v[u][i][k], f);
        const bool keep = i < rows;
#pragma unroll
        for (int e = 0; e < VE; ++e) colsum[k * VE + e] += keep ? f[e] : 0.f;
      }
    const float den = (float)(rows * Q);
    float dot = 0.f;
    float outv[IW];
    T means[NOUT];
#pragma unroll
    for (int o = 0; o < NOUT; ++o) {
      float acc = 0.f;
#pragma unroll
      for (int j = 0; j < Q; ++j) acc += colsum[o * Q + j];
      means[o] = from_f32<T>(acc / den);           // the value the filter stores
      const float m = to_f32(means[o]);
      dot += m * to_f32(xv[u][o]);
      const float g = to_f32(from_f32<T>(m * sc[u]));  // rounded once, then replicated
#pragma unroll
      for (int j = 0; j < Q; ++j) outv[o * Q + j] = g;
    }
    if (!ok) dot = 0.f;
    if (ok) {
      if (gyu) {
        T* dst = gyu + (long)plane[u] * a.P + hp * a.Wp + col * NOUT;
#pragma unroll
        for (int o = 0; o < NOUT; ++o) dst[o] = means[o];
      }
      T* dst = gx + ((long)plane[u] * a.H + (long)hp * Q) * a.W + col * IW;
#pragma unroll
      for (int k = 0; k < VW; ++k) {
        const uint4 vec = Vec16<T>::pack(outv + k * VE);
        for (int i = 0; i < rows; ++i) *reinterpret_cast<uint4*>(dst + (long)i * a.W + k * VE) = vec;
      }
    }
    const float s = block_sum(dot, red);
    if (threadIdx.x == 0 && plane[u] < a.planes) {
      const int n = (int)a.d_c.div((uint32_t)plane[u]);
      const int c = plane[u] - n * a.C;
      a.part[((long)n * a.cpp + chunk) * a.C + c] = s;
    }
  }
}

// A block's run of g_y (nvec 16-byte vectors) and the x_u values of its patches (nout elements, as
// floats into xs) go to LDS together: the first round of both is in flight before anything is waited
// for.  (With x_u read inside the patch loop every pass over the patches paid a global load's
// latency: 120 planes of 7x7, eight passes -- 19.5 us for a launch that moves 56 MB.)
template <class T>
__device__ __forceinline__ void stage_run_and_xu(const uint4* src_, uint4* dst_, int nvec, const T* xu, float* xs,
                                                 int nout, int tid) {
  constexpr int NV = 8;
  const u32x4_t* src = reinterpret_cast<const u32x4_t*>(src_);
  u32x4_t* dst = reinterpret_cast<u32x4_t*>(dst_);
  // first round of both (a run shorter than one vector is copied by element by the caller)
  const bool has_vec = nvec > 0;
  u32x4_t rg[NV];
  T xr[NV];
  if (has_vec) {
#pragma unroll
    for (int k = 0; k < NV; ++k) rg[k] = src[min(tid + k * kThreads, nvec - 1)];
  }
#pragma unroll
  for (int k = 0; k < NV; ++k) xr[k] = xu[min(tid + k * kThreads, nout - 1)];
  if (has_vec) {
#pragma unroll
    for (int k = 0; k < NV; ++k) dst[min(tid + k * kThreads, nvec - 1)] = rg[k];
  }
#pragma unroll
  for (int k = 0; k < NV; ++k) xs[min(tid + k * kThreads, nout - 1)] = to_f32(xr[k]);
  // what is left of longer runs
  for (int v = tid + NV * kThreads; v < nvec; v += NV * kThreads) {
#pragma unroll
    for (int k = 0; k < NV; ++k) rg[k] = src[min(v + k * kThreads, nvec - 1)];
#pragma unroll
    for (int k = 0; k < NV; ++k) dst[min(v + k * kThreads, nvec - 1)] = rg[k];
  }
  for (int lo = tid + NV * kThreads; lo < nout; lo += NV * kThreads) {
#pragma unroll
    for (int k = 0; k < NV; ++k) xr[k] = xu[min(lo + k * kThreads, nout - 1)];
#pragma unroll
    for (int k = 0; k < NV; ++k) xs[min(lo + k * kThreads, nout - 1)] = to_f32(xr[k]);
  }
}

// ---------------------------------------------------------------------------
// LDS variant: any map whose planes fit the staging buffer, stride 1.
// A block owns ppb whole planes: the flat run of g_y is loaded into LDS, every lane
// reduces one patch and overwrites that patch in LDS with the input-gradient value,
// the run is then stored to g_x with the same coalesced vectors.
// ---------------------------------------------------------------------------
template <class T, int QT>
__global__ __launch_bounds__(kThreads) void dw_fused_lds_k(DwFusedArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x;
  const int HW = a.H * a.W;
  const int pl0 = blockIdx.x * a.ppb;
  const int np = min(a.ppb, a.planes - pl0);
  const long byte0 = (long)pl0 * HW * (long)sizeof(T);
  const long byte1 = byte0 + (long)np * HW * (long)sizeof(T);
  const long a0 = byte0 & ~15L;
  const int span = (int)(byte1 - a0);
  const int nvec = span >> 4;
  const int shift = (int)(byte0 - a0);
  // layout: [run bytes, 16-aligned][prods: ppb * P floats][sc: ppb floats]
  const int run_bytes = ((a.ppb * HW * (int)sizeof(T) + 32) + 15) & ~15;
  float* prods = reinterpret_cast<float*>(smem + run_bytes);
  float* scs = prods + a.ppb * a.P;
  const uint4* src = reinterpret_cast<const uint4*>(static_cast<const unsigned char*>(a.gy) + a0);
  uint4* lds4 = reinterpret_cast<uint4*>(smem);
  const T* xu = static_cast<const T*>(a.xu) + (long)pl0 * a.P;
  const int nout = np * a.P;
  stage_run_and_xu<T>(src, lds4, nvec, xu, prods, nout, tid);
  {
    const int tail0 = nvec << 4;
    const int ntail = (span - tail0) / (int)sizeof(T);
    if (tid < ntail)
      reinterpret_cast<T*>(smem + tail0)[tid] =
          reinterpret_cast<const T*>(reinterpret_cast<const unsigned char*>(src) + tail0)[tid];
  }
  if (tid < np) {
    const int pl = pl0 + tid;
    const int c = pl - (int)a.d_c.div((uint32_t)pl) * a.C;
    scs[tid] = kernel_sum_of(static_cast<const T*>(a.w), c, a.KK) * a.scale;
  }
  __syncthreads();
  T* lds = reinterpret_cast<T*>(smem + shift);  // lds[e], e relative to the first plane
  T* gyu = a.gyu ? static_cast<T*>(a.gyu) + (long)pl0 * a.P : nullptr;
  const int q = QT ? QT : a.q;
  constexpr int UQ = QT ? QT : 1;  // unroll count of the q x q loops (1: run-time q, no unrolling)
  for (int lo = tid; lo < nout; lo += kThreads) {
    const int lp = (int)a.d_p.div((uint32_t)lo);  // local plane
    const int pp = lo - lp * a.P;
    const int hp = (int)a.d_wp.div((uint32_t)pp);
    const int wp = pp - hp * a.Wp;
    const int ch = min(q, a.H - hp * q);
    const int cw = min(q, a.W - wp * q);
    const int base = lp * HW + hp * q * a.W + wp * q;
    const float xval = prods[lo];
    float acc = 0.f;
#pragma unroll UQ
    for (int i = 0; i < q; ++i)
#pragma unroll UQ
      for (int j = 0; j < q; ++j) {
        const bool ok = i < ch && j < cw;
        const float val = to_f32(lds[base + (ok ? i * a.W + j : 0)]);
        acc += ok ? val : 0.f;
      }
    const T mean = from_f32<T>(acc / (float)(ch * cw));
    const float m = to_f32(mean);
    if (gyu) gyu[lo] = mean;
    prods[lo] = m * xval;
    const T g = from_f32<T>(m * scs[lp]);
#pragma unroll UQ
    for (int i = 0; i < q; ++i)
#pragma unroll UQ
      for (int j = 0; j < q; ++j)
        if (i < ch && j < cw) lds[base + i * a.W + j] = g;
  }
  __syncthreads();
  // store the run: whole vectors strictly inside [byte0, byte1), head and tail by element
  T* out = static_cast<T*>(a.gx);
  unsigned char* dstb = static_cast<unsigned char*>(a.gx) + a0;
  const int v0 = shift ? 1 : 0;  // the first vector is shared with the previous block's planes
  for (int v = tid + v0; v < nvec; v += kThreads)
    *reinterpret_cast<uint4*>(dstb + ((long)v << 4)) = lds4[v];
  if (shift) {
    const int nhead = (16 - shift) / (int)sizeof(T);  // elements of this block in vector 0
    if (tid < nhead && tid < np * HW) out[(long)pl0 * HW + tid] = lds[tid];
  }
  {
    const int tail0 = nvec << 4;
    const int ntail = (span - tail0) / (int)sizeof(T);
    const int efirst = (tail0 - shift) / (int)sizeof(T);
    if (tid < ntail && efirst + tid >= 0) out[(long)pl0 * HW + efirst + tid] = lds[efirst + tid];
  }
  // per-plane dot product in fixed order
  if (tid < np) {
    float s = 0.f;
    const float* pr = prods + tid * a.P;
    for (int k = 0; k < a.P; ++k) s += pr[k];
    a.part[pl0 + tid] = s;
  }
}

// ---------------------------------------------------------------------------
// Strided LDS variant.  A block owns ppb whole planes: the flat run of g_y ([Hy, Wy] per plane)
// is loaded into LDS, every lane reduces one q x q patch (in-bounds pixels only) and writes
// the input-gradient value to the patch's qx x qx pixels of an LDS image of the g_x run
// ([H, W] per plane), which is then stored with coalesced vectors.
// ---------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(kThreads) void dw_fused_strided_k(DwFusedArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x;
  const int HW = a.H * a.W, HWy = a.Hy * a.Wy;
  const int pl0 = blockIdx.x * a.ppb;
  const int np = min(a.ppb, a.planes - pl0);
  // layout: [g_y run, 16-aligned][g_x run, 16-aligned][prods: ppb * P floats][sc: ppb floats]
  const int in_bytes = ((a.ppb * HWy * (int)sizeof(T) + 32) + 15) & ~15;
  const int out_bytes = ((a.ppb * HW * (int)sizeof(T) + 32) + 15) & ~15;
  unsigned char* obuf = smem + in_bytes;
  float* prods = reinterpret_cast<float*>(obuf + out_bytes);
  float* scs = prods + a.ppb * a.P;
  // ---- load the g_y run
  const long ib0 = (long)pl0 * HWy * (long)sizeof(T);
  const long ia0 = ib0 & ~15L;
  const int ispan = (int)(ib0 + (long)np * HWy * (long)sizeof(T) - ia0);
  const int invec = ispan >> 4;
  const int ishift = (int)(ib0 - ia0);
  const uint4* src = reinterpret_cast<const uint4*>(static_cast<const unsigned char*>(a.gy) + ia0);
  uint4* in4 = reinterpret_cast<uint4*>(smem);
  const T* xu = static_cast<const T*>(a.xu) + (long)pl0 * a.P;
  const int nout = np * a.P;
  stage_run_and_xu<T>(src, in4, invec, xu, prods, nout, tid);
  {
    const int tail0 = invec << 4;
    const int ntail = (ispan - tail0) / (int)sizeof(T);
    if (tid < ntail)
      reinterpret_cast<T*>(smem + tail0)[tid] =
          reinterpret_cast<const T*>(reinterpret_cast<const unsigned char*>(src) + tail0)[tid];
  }
  if (tid < np) {
    const int pl = pl0 + tid;
    const int c = pl - (int)a.d_c.div((uint32_t)pl) * a.C;
    scs[tid] = kernel_sum_of(static_cast<const T*>(a.w), c, a.KK) * a.scale;
  }
  __syncthreads();
  // ---- patch means, products with x_u, replicated values into the g_x image
  const long ob0 = (long)pl0 * HW * (long)sizeof(T);
  const long oa0 = ob0 & ~15L;
  const int oshift = (int)(ob0 - oa0);
  const int ospan = oshift + np * HW * (int)sizeof(T);
  const T* lin = reinterpret_cast<const T*>(smem + ishift);   // lin[e], e relative to the first g_y plane
  T* lout = reinterpret_cast<T*>(obuf + oshift);              // lout[e], e relative to the first g_x plane
  T* gyu = a.gyu ? static_cast<T*>(a.gyu) + (long)pl0 * a.P : nullptr;
  const int q = a.q, qx = a.qx;
  for (int lo = tid; lo < nout; lo += kThreads) {
    const int lp = (int)a.d_p.div((uint32_t)lo);  // local plane
    const int pp = lo - lp * a.P;
    const int hp = (int)a.d_wp.div((uint32_t)pp);
    const int wp = pp - hp * a.Wp;
    const int ch = min(q, a.Hy - hp * q);
    const int cw = min(q, a.Wy - wp * q);
    const int base = lp * HWy + hp * q * a.Wy + wp * q;
    const float xval = prods[lo];
    float acc = 0.f;
    for (int i = 0; i < ch; ++i)
      for (int j = 0; j < cw; ++j) acc += to_f32(lin[base + i * a.Wy + j]);
    const T mean = from_f32<T>(acc / (float)(ch * cw));
    const float m = to_f32(mean);
    if (gyu) gyu[lo] = mean;
    prods[lo] = m * xval;
    const T g = from_f32<T>(m * scs[lp]);
    const int oh = min(qx, a.H - hp * qx), ow = min(qx, a.W - wp * qx);
    const int obase = lp * HW + hp * qx * a.W + wp * qx;
    for (int i = 0; i < oh; ++i)
      for (int j = 0; j < ow; ++j) lout[obase + i * a.W + j] = g;
  }
  __syncthreads();
  // ---- store the g_x run: whole vectors strictly inside it, head and tail by element
  T* out = static_cast<T*>(a.gx);
  unsigned char* dstb = static_cast<unsigned char*>(a.gx) + oa0;
  const uint4* o4 = reinterpret_cast<const uint4*>(obuf);
  const int onvec = ospan >> 4;
  const int v0 = oshift ? 1 : 0;  // the first vector is shared with the previous block's planes
  for (int v = tid + v0; v < onvec; v += kThreads) *reinterpret_cast<uint4*>(dstb + ((long)v << 4)) = o4[v];
  if (oshift) {
    const int nhead = (16 - oshift) / (int)sizeof(T);  // elements of this block in vector 0
    if (tid < nhead && tid < np * HW) out[(long)pl0 * HW + tid] = lout[tid];
  }
  {
    const int tail0 = onvec << 4;
    const int ntail = (ospan - tail0) / (int)sizeof(T);
    const int efirst = (tail0 - oshift) / (int)sizeof(T);
    if (tid < ntail && efirst + tid >= 0) out[(long)pl0 * HW + efirst + tid] = lout[efirst + tid];
  }
  // per-plane dot product in fixed order
  if (tid < np) {
    float s = 0.f;
    const float* pr = prods + tid * a.P;
    for (int k = 0; k < a.P; ++k) s += pr[k];
    a.part[pl0 + tid] = s;
  }
}

template <class T>
bool rows_variant_ok(const Geom& g) {
  constexpr int VE = Vec16<T>::N;
  const int q = g.r;
  if (q != 2 && q != 4 && q != 8) return false;
  const int IW = VE > q ? VE : q;
  return g.W % IW == 0 && (g.W * (int)sizeof(T)) % 16 == 0;
}

template <class T>
int lds_planes_per_block(const Geom& g) {
  const long per_plane = (long)g.H * g.W * sizeof(T) + (long)g.P * 4 + 4;
  long ppb = (kLdsBudget - 64) / per_plane;
  const long planes = (long)g.N * g.Ci;
  if (ppb > planes / 3072) ppb = planes / 3072;  // ~12 blocks per CU when the tensor allows: rounds of blocks overlap loads and stores
  if (ppb > kThreads) ppb = kThreads;
  const long fit = (64 * 1024 - 64) / per_plane;
  if (ppb < 1) ppb = fit >= 1 ? 1 : 0;
  return (int)ppb;
}

template <class T>
int strided_planes_per_block(const Geom& g) {
  const long per_plane = ((long)g.H * g.W + (long)g.Hy * g.Wy) * sizeof(T) + (long)g.P * 4 + 4;
  long ppb = (kLdsBudget - 128) / per_plane;
  const long planes = (long)g.N * g.Ci;
  if (ppb > planes / 3072) ppb = planes / 3072;  // ~12 blocks per CU when the tensor allows: rounds of blocks overlap loads and stores
  if (ppb > kThreads) ppb = kThreads;
  const long fit = (64 * 1024 - 128) / per_plane;
  if (ppb < 1) ppb = fit >= 1 ? 1 : 0;
  return (int)ppb;
}

}  // namespace

// shapes the fused depthwise launch handles; *nz = number of partial slabs per channel
bool dw_fused_ok(const Geom& g, int* nz) {
  if (!(g.Cg == 1 && g.Og == 1) || g.r < 2) return false;
  if (g.s != 1) {  // strided: whole planes of g_y and g_x side by side in LDS
    const int ppb = g.dtype == GF_BF16 ? strided_planes_per_block<bf16_t>(g) : strided_planes_per_block<float>(g);
    if (ppb < 1) return false;
    if (nz) *nz = g.N;
    return true;
  }
  if (g.Hy != g.H || g.Wy != g.W) return false;
  const bool rows = g.dtype == GF_BF16 ? rows_variant_ok<bf16_t>(g) : rows_variant_ok<float>(g);
  if (rows) {
    const int VE = 16 / g.b;
    const int IW = VE > g.r ? VE : g.r;
    const int ipp = g.Hp * (g.W / IW);
    int nthreads;
    if (nz) *nz = g.N * rows_chunks(ipp, &nthreads);
    return true;
  }
  const int ppb = g.dtype == GF_BF16 ? lds_planes_per_block<bf16_t>(g) : lds_planes_per_block<float>(g);
  if (ppb < 1) return false;
  if (nz) *nz = g.N;
  return true;
}

template <class T>
static hipError_t dw_fused_t(const Geom& g, const void* g_y, const void* x_u, const void* w, void* gy_u,
                             void* g_x, float* part, hipStream_t st) {
  DwFusedArgs a = {};
  a.gy = g_y; a.xu = x_u; a.w = w; a.gyu = gy_u; a.gx = g_x; a.part = part;
  a.C = g.Ci; a.H = g.H; a.W = g.W; a.Hp = g.Hp; a.Wp = g.Wp; a.P = g.P; a.KK = g.KK; a.q = g.r;
  a.planes = g.N * g.Ci;
  a.scale = 1.f / ((float)g.s * (float)g.s);
  a.d_c = FastDiv((uint32_t)g.Ci);
  if (g.s != 1) {
    a.Hy = g.Hy; a.Wy = g.Wy; a.qx = g.rx;
    a.ppb = strided_planes_per_block<T>(g);
    a.d_wp = FastDiv((uint32_t)g.Wp);
    a.d_p = FastDiv((uint32_t)g.P);
    const int in_bytes = ((a.ppb * g.Hy * g.Wy * (int)sizeof(T) + 32) + 15) & ~15;
    const int out_bytes = ((a.ppb * g.H * g.W * (int)sizeof(T) + 32) + 15) & ~15;
    const size_t lds = (size_t)in_bytes + out_bytes + (size_t)a.ppb * g.P * 4 + (size_t)a.ppb * 4;
    GF_LAUNCH(dw_fused_strided_k<T>, dim3(cdiv(a.planes, a.ppb)), dim3(kThreads), lds, st, a);
    return hipGetLastError();
  }
  if (rows_variant_ok<T>(g)) {
    constexpr int VE = Vec16<T>::N;
    const int IW = VE > g.r ? VE : g.r;
    a.ipr = g.W / IW;
    a.ipp = g.Hp * a.ipr;
    int nthreads;
    a.cpp = rows_chunks(a.ipp, &nthreads);
    a.d_ipr = FastDiv((uint32_t)a.ipr);
    a.d_cpp = FastDiv((uint32_t)a.cpp);
    const dim3 grid(a.planes * a.cpp), block(nthreads);
    if (g.r == 8) GF_LAUNCH((dw_fused_rows_k<T, 8, 1>), grid, block, 0, st, a);
    else if (g.r == 2) GF_LAUNCH((dw_fused_rows_k<T, 2, 1>), grid, block, 0, st, a);
    else GF_LAUNCH((dw_fused_rows_k<T, 4, 1>), grid, block, 0, st, a);
    return hipGetLastError();
  }
  a.ppb = lds_planes_per_block<T>(g);
  a.d_wp = FastDiv((uint32_t)g.Wp);
  a.d_p = FastDiv((uint32_t)g.P);
  const int run_bytes = ((a.ppb * g.H * g.W * (int)sizeof(T) + 32) + 15) & ~15;
  const size_t lds = (size_t)run_bytes + (size_t)a.ppb * g.P * 4 + (size_t)a.ppb * 4;
  const int blocks = cdiv(a.planes, a.ppb);
  if (g.r == 2) GF_LAUNCH((dw_fused_lds_k<T, 2>), dim3(blocks), dim3(kThreads), lds, st, a);
  else if (g.r == 4) GF_LAUNCH((dw_fused_lds_k<T, 4>), dim3(blocks), dim3(kThreads), lds, st, a);
  else GF_LAUNCH((dw_fused_lds_k<T, 0>), dim3(blocks), dim3(kThreads), lds, st, a);
  return hipGetLastError();
}

hipError_t launch_dw_fused(const Geom& g, const void* g_y, const void* x_u, const void* w, void* gy_u,
                           void* g_x, float* part, hipStream_t st) {
  if (g.dtype == GF_BF16) return dw_fused_t<bf16_t>(g, g_y, x_u, w, gy_u, g_x, part, st);
  return dw_fused_t<float>(g, g_y, x_u, w, gy_u, g_x, part, st);
}

}  // namespace gf
