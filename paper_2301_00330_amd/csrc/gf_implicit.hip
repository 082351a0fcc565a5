// Vanilla back-propagation (Sec. 3.1) of dense convolutions as implicit GEMMs on the MFMA cores
// of gfx950:
//
//   weight gradient  g_th[co, ci, t] = sum_{n, k} g_y[n, co, k] * xs[n, ci, k + dW(t)]      (k: output pixel)
//   input gradient   g_x[n, ci, j]   = sum_{t, co} th[co, ci, t] * g_y[n, co, j + dD(t)]   (j: input pixel)
//
// Stride 1, output map as wide as the input map ("same" padding): the pixel a tap reads is
// the flattened pixel index plus a constant,
//   dW(t) = (u d - p) W + (v d - p),   dD(t) = (p - u d) W_y + (p - v d),   t = (u, v),
// wherever the tap stays inside the image; where it leaves it the factor is a zero of the
// padding.  So no column tensor is built: the shifted operand is read straight from the
// tensor with 16-byte loads at 2- or 4-byte alignment, and a byte table [tap][8 pixels] says
// which of the eight elements are padding.  Planes are addressed as if they held 8 *
// ceil(HW / 8) pixels, so that a vector never straddles two images; the surplus positions
// are masked like padding.
//
// Stride s > 1: x is first split into its s x s phase planes xq[a, b][n, ci, i, j] =
// x[n, ci, s i + a, s j + b], stored with the row pitch W_y of the output map.  Tap (u, v) of
// output pixel (i, j) reads x[s i + u d - p, s j + v d - p], which is one fixed phase plane at
// (i, j) plus a constant: the same kernels run with a per-tap offset that includes the phase
// plane.  The input gradient is computed phase by phase (each phase of g_x receives the taps
// whose parity matches, so no multiplication is wasted on the zeros of a zero-inserted g_y)
// into phase planes that one more pass interleaves into g_x.
//
// Tiles: 256-lane blocks of 2 x 2 waves, each wave TM x TN MFMA tiles of 16 x 16
// (v_mfma_f32_16x16x32_bf16 / v_mfma_f32_16x16x4_f32); operands are staged through LDS one
// K chunk ahead of the arithmetic.  These GEMMs are small for the chip (a few hundred tiles),
// so what limits them is the bytes a compute unit has in flight: chunks are 256 bytes of K
// per row where registers allow it.
#include "gf_internal.h"
#include "gf_mma.h"

namespace gf {

namespace {

constexpr int kThreads = 256;
constexpr double kPlainWgradMinFlops = 6e9;  // below, the 64 x 64 tiles of the S3 kernel (merged with S4 in one launch) are faster

// AND words of an element mask (bit e keeps element e), computed once for masks shared by
// many vectors
template <class T>
__device__ __forceinline__ void expand_mask(uint32_t m, uint32_t (&w)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (sizeof(T) == 4) {
      w[i] = (uint32_t)((int)(m << (31 - i)) >> 31);
    } else {
      const uint32_t lo = (uint32_t)((int)(m << (31 - 2 * i)) >> 31), hi = (uint32_t)((int)(m << (30 - 2 * i)) >> 31);
      w[i] = (lo & 0xffffu) | (hi & 0xffff0000u);
    }
  }
}
__device__ __forceinline__ uint4 and4(const uint4& v, const uint32_t (&w)[4]) {
  return make_uint4(v.x & w[0], v.y & w[1], v.z & w[2], v.w & w[3]);
}

// mask bits of the vector that starts at pixel q (a multiple of VE) from the table byte of
// its group of eight pixels
template <class T>
__device__ __forceinline__ uint32_t vec_mask(uint32_t byte, int q) {
  return sizeof(T) == 2 ? byte : (byte >> (q & 4)) & 0xfu;
}

// ---------------------------------------------------------------------------
// Set-up.  With e = u d - p, f = v d - p (tap offsets on the input side) and, for stride s,
// a = e mod s, b = f mod s (the phase plane the tap reads), Hq = ceil(H / s), Wq = W_y:
//   tapw[t]        = phase(a, b) * N Ci Hq Wq + floor(e / s) * Wq + floor(f / s)
//   tabw[t][k / 8] bit i: output pixel k + i exists and tap t of it reads inside the image
//   per phase ph = (a, b) of g_x, the taps with (a + p - u d) and (b + p - v d) divisible by s:
//   tapd[ph][kk]   = {t, ((a + p - u d) / s) * W_y + (b + p - v d) / s},  ntap[ph] of them
//   tabd[ph][t][j / 8] bit i: position j + i of the phase plane exists and that tap reaches it
//                             from an output pixel inside the map
// ---------------------------------------------------------------------------
struct PrepArgs {
  uint8_t* tabw;
  uint8_t* tabd;
  int* tapw;    // [KK]
  int2* tapd;   // [s*s][KK]
  int* ntap;    // [s*s]
  int N, Ci, H, W, Hy, Wy, Hq, Wq, Kw, KK, s, d, p, nvw, nvd;
};

__device__ __forceinline__ int floor_div(int a, int b) { return (a >= 0) ? a / b : -((-a + b - 1) / b); }

__device__ __forceinline__ void prep_tables(const PrepArgs& a, int block) {
  const int e0 = block * kThreads + threadIdx.x;
  const int nph = a.s * a.s;
  const int nmax = a.nvw > a.nvd * nph ? a.nvw : a.nvd * nph;
  if (block == 0 && (int)threadIdx.x < nph) {  // tap list of one phase of g_x
    const int ph = threadIdx.x, pa = ph / a.s, pb = ph - pa * a.s;
    int cnt = 0;
    for (int t = 0; t < a.KK; ++t) {
      const int u = t / a.Kw, v = t - u * a.Kw;
      const int ea = pa + a.p - u * a.d, eb = pb + a.p - v * a.d;
      const int qa = floor_div(ea, a.s), qb = floor_div(eb, a.s);
      if (qa * a.s == ea && qb * a.s == eb) a.tapd[ph * a.KK + cnt++] = make_int2(t, qa * a.Wy + qb);
    }
    a.ntap[ph] = cnt;
  }
  if (e0 >= a.KK * nmax) return;
  const int t = e0 / nmax, g = e0 - t * nmax;
  const int u = t / a.Kw, v = t - u * a.Kw;
  const int e = u * a.d - a.p, f = v * a.d - a.p;
  if (g == 0) {
    const int qe = floor_div(e, a.s), qf = floor_div(f, a.s);
    const int ph = (e - qe * a.s) * a.s + (f - qf * a.s);
    a.tapw[t] = ph * (a.N * a.Ci * a.Hq * a.Wq) + qe * a.Wq + qf;
  }
  if (g < a.nvw) {
    uint32_t m = 0;
    for (int i = 0; i < 8; ++i) {
      const int k = g * 8 + i;
      if (k >= a.Hy * a.Wy) break;
      const int hy = k / a.Wy, wy = k - hy * a.Wy;
      const int hs = hy * a.s + e, ws = wy * a.s + f;
      if (hs >= 0 && hs < a.H && ws >= 0 && ws < a.W) m |= 1u << i;
    }
    a.tabw[t * a.nvw + g] = (uint8_t)m;
  }
  if (g < a.nvd * nph) {
    const int ph = g / a.nvd, gg = g - ph * a.nvd;
    const int pa = ph / a.s, pb = ph - pa * a.s;
    const int ea = pa + a.p - u * a.d, eb = pb + a.p - v * a.d;
    const int qa = floor_div(ea, a.s), qb = floor_div(eb, a.s);
    uint32_t m = 0;
    if (qa * a.s == ea && qb * a.s == eb) {
      for (int i = 0; i < 8; ++i) {
        const int j = gg * 8 + i;
        if (j >= a.Hq * a.Wq) break;
        const int h = j / a.Wq, w = j - h * a.Wq;
        const int hs = h + qa, ws = w + qb;
        if (hs >= 0 && hs < a.Hy && ws >= 0 && ws < a.Wy) m |= 1u << i;
      }
    }
    a.tabd[(ph * a.KK + t) * a.nvd + gg] = (uint8_t)m;
  }
}

// One set-up launch.  Blocks [0, tab_blocks): tables and tap lists.  Then w_blocks blocks write the
// kernel tap-major with c_o contiguous, wt[(t * Ci + ci) * Co + co] = w[(co * Ci + ci) * KK + t]
// (input gradient only).  Then the phase planes of x (weight gradient of a strided layer only).
template <class T>
__global__ __launch_bounds__(kThreads) void prep_k(PrepArgs a, int tab_blocks, int w_blocks, const T* w, T* wt,
                                                  int Co, const T* x, T* xq) {
  int b = blockIdx.x;
  if (b < tab_blocks) {
    prep_tables(a, b);
    return;
  }
  b -= tab_blocks;
  if (b < w_blocks) {
    const int e = b * kThreads + threadIdx.x;
    if (e >= Co * a.Ci * a.KK) return;
    const int co = e % Co;
    const int row = e / Co;
    const int ci = row % a.Ci, t = row / a.Ci;
    wt[e] = w[((long)co * a.Ci + ci) * a.KK + t];
    return;
  }
  b -= w_blocks;
  const int PQ = a.Hq * a.Wq;
  const int total = a.s * a.s * a.N * a.Ci * PQ;
  const int e = b * kThreads + threadIdx.x;
  if (e >= total) return;
  const int pos = e % PQ, plane = e / PQ;        // plane = (ph * N + n) * Ci + ci
  const int i = pos / a.Wq, j = pos - i * a.Wq;
  const int nc = plane % (a.N * a.Ci), ph = plane / (a.N * a.Ci);
  const int h = i * a.s + ph / a.s, ww = j * a.s + ph % a.s;
  const bool ok = h < a.H && ww < a.W;
  const T val = x[((long)nc * a.H + (ok ? h : 0)) * a.W + (ok ? ww : 0)];
  xq[e] = ok ? val : from_f32<T>(0.f);
}

// g_x[n, ci, h, w] = gxq[phase(h mod s, w mod s)][n, ci, h / s, w / s]
template <class T>
__global__ __launch_bounds__(kThreads) void interleave_k(const T* gxq, T* gx, int NC, int H, int W, int Hq,
                                                        int Wq, int s) {
  const int e = blockIdx.x * kThreads + threadIdx.x;
  if (e >= NC * H * W) return;
  const int w = e % W, r = e / W;
  const int h = r % H, nc = r / H;
  const int ph = (h % s) * s + (w % s);
  gx[e] = gxq[((long)ph * NC + nc) * (Hq * Wq) + (h / s) * Wq + (w / s)];
}

// ---------------------------------------------------------------------------
// weight gradient: part[z][t][co][ci] = sum over the K chunks of slab z
// ---------------------------------------------------------------------------
struct XWgradArgs {
  const void* gy;
  const void* x;
  float* part;
  const uint8_t* tab;
  const int* tapw;        // per tap: offset of the element of the x operand that output pixel 0 reads
  int N, Ci, Co, KK;
  int HW, HWy, HWyp, nv;  // plane of the x operand (a phase plane for strided layers), plane of g_y
  int nchunks, chunks_per_z, nz;
  int tx, tiles, R;       // c_i tiles, c_i tiles * c_o tiles, tiles * KK
  int xcd_slabs;          // 1: slab z runs on XCD z % 8
  int inner_ok;           // 1: a shifted vector of an inner image (0 < n < N - 1) stays inside the tensors
  int total_x, total_gy;
  FastDiv d_hwyp, d_r, d_tiles, d_tx;
};

// KV = 16-byte vectors of K per staged row.  One-dimensional grid.  The hardware hands
// consecutive blocks to the eight XCDs in turn; with eight or more K slabs block L works on
// slab (L % 8) + 8 * (..), so that all taps and tiles of a slab share one XCD's L2 and each
// XCD touches an eighth of x and g_y.
template <class T, int TM, int TN, int KV>
__global__ __launch_bounds__(kThreads) void xwgrad_k(XWgradArgs a) {
  constexpr int WM = 2, WN = 2;
  constexpr int BM = WM * TM * 16, BN = WN * TN * 16;
  constexpr int VE = Mma<T>::VE, KSTEP = Mma<T>::KSTEP, BK = KV * VE;
  constexpr int RB = KV * 16 + 16;                 // staged row: data + 16 bytes pad
  constexpr int RPP = kThreads / KV;               // rows per pass of the block
  constexpr int LA = BM / RPP, LB = BN / RPP;      // 16-byte loads per lane and chunk
  constexpr uint32_t FULL = Mma<T>::FULL;
  __shared__ __attribute__((aligned(16))) unsigned char As[BM * RB];
  __shared__ __attribute__((aligned(16))) unsigned char Bs[BN * RB];
  const T* gy = static_cast<const T*>(a.gy);
  const T* x = static_cast<const T*>(a.x);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  int z, rest;
  if (a.xcd_slabs) {
    const int L = blockIdx.x, idx = L >> 3;
    const int zl = (int)a.d_r.div((uint32_t)idx);
    z = (L & 7) + 8 * zl;
    rest = idx - zl * a.R;
  } else {
    z = (int)a.d_r.div(blockIdx.x);
    rest = (int)blockIdx.x - z * a.R;
  }
  if (z >= a.nz) return;  // uniform for the block
  const int t = (int)a.d_tiles.div((uint32_t)rest), tile = rest - t * a.tiles;
  const int by = (int)a.d_tx.div((uint32_t)tile), bx = tile - by * a.tx;
  const int delta = a.tapw ? a.tapw[t] : 0;  // no tables: plain contraction of two maps of the same size
  const int m0 = by * BM, n0 = bx * BN;
  const int kc0 = z * a.chunks_per_z;
  const int kc1 = min(kc0 + a.chunks_per_z, a.nchunks);
  const int vi = tid % KV, row0 = tid / KV;  // this lane's vector of the chunk, first tile row
  const bool rows_full = m0 + BM <= a.Co && n0 + BN <= a.Ci;
  const int coHWy = a.Co * a.HWy, ciHW = a.Ci * a.HW;

  int rowa[LA], rowb[LB];  // element offsets of this lane's rows inside an image
#pragma unroll
  for (int i = 0; i < LA; ++i) rowa[i] = min(m0 + row0 + RPP * i, a.Co - 1) * a.HWy;
#pragma unroll
  for (int i = 0; i < LB; ++i) rowb[i] = min(n0 + row0 + RPP * i, a.Ci - 1) * a.HW + delta;

  uint4 ra[LA], rb[LB];
  uint32_t ma = 0, mb = 0;  // element masks of the fetched chunk (the same for every row)
  uint32_t off = 0;         // bit i / bit 16 + i: load i of A / B had to be moved into the tensor
  auto fetch = [&](int kc) {
    const int kq = kc * BK + vi * VE;
    const int n = (int)a.d_hwyp.div((uint32_t)kq);
    const int q = kq - n * a.HWyp;
    const bool img = n < a.N;
    const int nn = min(n, a.N - 1);
    const int rem = a.HWy - q;
    ma = (!img || rem <= 0) ? 0u : (rem >= VE ? FULL : (1u << rem) - 1u);
    mb = a.tab ? (img ? vec_mask<T>(a.tab[t * a.nv + (q >> 3)], q) : 0u) : ma;
    const int basea = nn * coHWy + q, baseb = nn * ciHW + q;
    off = 0;
    if (a.inner_ok && nn > 0 && nn < a.N - 1) {  // inner images: a shifted vector cannot leave the tensors
#pragma unroll
      for (int i = 0; i < LA; ++i) ra[i] = load_vec<T>(gy + (basea + rowa[i]));
#pragma unroll
      for (int i = 0; i < LB; ++i) rb[i] = load_vec<T>(x + (baseb + rowb[i]));
    } else {
#pragma unroll
      for (int i = 0; i < LA; ++i) {
        const int o = basea + rowa[i];
        const int oc = min(o, a.total_gy - VE);   // o >= 0 always
        off |= (o != oc) ? 1u << i : 0u;
        ra[i] = load_vec<T>(gy + oc);
      }
#pragma unroll
      for (int i = 0; i < LB; ++i) {
        const int o = baseb + rowb[i];
        const int oc = min(max(o, 0), a.total_x - VE);
        off |= (o != oc) ? 0x10000u << i : 0u;
        rb[i] = load_vec<T>(x + oc);
      }
    }
  };
  auto stage = [&](int kc) {
    if (off) {  // first or last rows of the tensors only: shift the moved vectors back
      const int kq = kc * BK + vi * VE;
      const int n = (int)a.d_hwyp.div((uint32_t)kq);
      const int q = kq - n * a.HWyp;
      const int nn = min(n, a.N - 1);
      const int basea = nn * coHWy + q, baseb = nn * ciHW + q;
#pragma unroll
      for (int i = 0; i < LA; ++i) {
        const int o = basea + rowa[i];
        ra[i] = realign<T>(ra[i], min(max(o - min(o, a.total_gy - VE), -VE), VE));
      }
#pragma unroll
      for (int i = 0; i < LB; ++i) {
        const int o = baseb + rowb[i];
        rb[i] = realign<T>(rb[i], min(max(o - min(max(o, 0), a.total_x - VE), -VE), VE));
      }
    }
    uint32_t wa[4], wb[4];
    expand_mask<T>(ma, wa);
    expand_mask<T>(mb, wb);
    if (rows_full) {
#pragma unroll
      for (int i = 0; i < LA; ++i) *reinterpret_cast<uint4*>(As + (row0 + RPP * i) * RB + vi * 16) = and4(ra[i], wa);
#pragma unroll
      for (int i = 0; i < LB; ++i) *reinterpret_cast<uint4*>(Bs + (row0 + RPP * i) * RB + vi * 16) = and4(rb[i], wb);
    } else {
#pragma unroll
      for (int i = 0; i < LA; ++i) {
        const int row = row0 + RPP * i;
        *reinterpret_cast<uint4*>(As + row * RB + vi * 16) = m0 + row < a.Co ? and4(ra[i], wa) : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < LB; ++i) {
        const int row = row0 + RPP * i;
        *reinterpret_cast<uint4*>(Bs + row * RB + vi * 16) = n0 + row < a.Ci ? and4(rb[i], wb) : make_uint4(0, 0, 0, 0);
      }
    }
  };

  // bf16 with an even number of 16-row blocks per wave in both directions: 32 x 32 x 16 MFMAs
  constexpr bool BIG = sizeof(T) == 2 && TM % 2 == 0 && TN % 2 == 0;
  f32x4 acc[TM][TN];
  f32x16 acc32[BIG ? TM / 2 : 1][BIG ? TN / 2 : 1];
  if constexpr (BIG) {
#pragma unroll
    for (int i = 0; i < TM / 2; ++i)
#pragma unroll
      for (int j = 0; j < TN / 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc32[i][j][e] = 0.f;
  } else {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  if (kc0 < kc1) fetch(kc0);
  const int r = lane & 15, kg = lane >> 4;
  for (int kc = kc0; kc < kc1; ++kc) {
    stage(kc);
    __syncthreads();
    if (kc + 1 < kc1) fetch(kc + 1);
    if constexpr (BIG) {
      const int r32 = lane & 31, kh = lane >> 5;
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        uint4 fa[TM / 2], fb[TN / 2];
#pragma unroll
        for (int i = 0; i < TM / 2; ++i)
          fa[i] = *reinterpret_cast<const uint4*>(As + ((wm * TM + 2 * i) * 16 + r32) * RB + ks * 32 + kh * 16);
#pragma unroll
        for (int j = 0; j < TN / 2; ++j)
          fb[j] = *reinterpret_cast<const uint4*>(Bs + ((wn * TN + 2 * j) * 16 + r32) * RB + ks * 32 + kh * 16);
#pragma unroll
        for (int i = 0; i < TM / 2; ++i)
#pragma unroll
          for (int j = 0; j < TN / 2; ++j) acc32[i][j] = mma32(fa[i], fb[j], acc32[i][j]);
      }
    } else
#pragma unroll
    for (int ks = 0; ks < BK / KSTEP; ++ks) {
      if constexpr (sizeof(T) == 2) {
        uint4 fa[TM], fb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
          fa[i] = *reinterpret_cast<const uint4*>(As + ((wm * TM + i) * 16 + r) * RB + ks * 64 + kg * 16);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          fb[j] = *reinterpret_cast<const uint4*>(Bs + ((wn * TN + j) * 16 + r) * RB + ks * 64 + kg * 16);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j] = mma16(fa[i], fb[j], acc[i][j]);
      } else {
        float fa[TM], fb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
          fa[i] = *reinterpret_cast<const float*>(As + ((wm * TM + i) * 16 + r) * RB + (ks * 4 + kg) * 4);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          fb[j] = *reinterpret_cast<const float*>(Bs + ((wn * TN + j) * 16 + r) * RB + (ks * 4 + kg) * 4);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j] = mma16(fa[i], fb[j], acc[i][j]);
      }
    }
    __syncthreads();
  }
  float* dst = a.part + ((long)z * a.KK + t) * a.Co * a.Ci;
  if constexpr (BIG) {  // element v: row 8 * (v / 4) + 4 * (lane / 32) + v % 4, column lane % 32 of a 32 x 32 tile
#pragma unroll
    for (int i = 0; i < TM / 2; ++i)
#pragma unroll
      for (int j = 0; j < TN / 2; ++j) {
        const int ci = n0 + (wn * TN + 2 * j) * 16 + (lane & 31);
#pragma unroll
        for (int vv = 0; vv < 16; ++vv) {
          const int co = m0 + (wm * TM + 2 * i) * 16 + 8 * (vv >> 2) + 4 * (lane >> 5) + (vv & 3);
          if (co < a.Co && ci < a.Ci) dst[(long)co * a.Ci + ci] = acc32[i][j][vv];
        }
      }
    return;
  }
  // D[i = 4 * (lane / 16) + v][j = lane % 16] of every 16 x 16 tile
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int ci = n0 + (wn * TN + j) * 16 + (lane & 15);
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) {
        const int co = m0 + (wm * TM + i) * 16 + 4 * (lane >> 4) + vv;
        if (co < a.Co && ci < a.Ci) dst[(long)co * a.Ci + ci] = acc[i][j][vv];
      }
    }
}

// g_w[co, ci, t] = sum_z part[z][t][co][ci].  A block owns kThreads / G consecutive (co, ci) pairs of
// one tap; lane (g, e) adds the slabs z = g, g + G, ... of pair e (four loads in flight, consecutive
// lanes on consecutive pairs), the G partial sums of a pair are then added in index order: the
// result does not depend on scheduling.  G = 1 for large outputs, more lanes per pair for small
// outputs with many slabs (a single lane would walk hundreds of slabs one latency at a time).
template <int G>
__global__ __launch_bounds__(kThreads) void xfinalize_k(const float* part, float* g_w, int pairs, int KK,
                                                       int nz) {
  constexpr int OPB = kThreads / G;
  __shared__ float red[G][OPB];
  const int g = threadIdx.x / OPB, el = threadIdx.x - g * OPB;
  const int e = blockIdx.x * OPB + el;
  const int t = blockIdx.y;
  const float* p = part + (long)t * pairs + min(e, pairs - 1);
  const long zs = (long)KK * pairs;
  float s = 0.f;
  int z = g;
  for (; z + 3 * G < nz; z += 4 * G) {
    const float v0 = p[z * zs], v1 = p[(z + G) * zs], v2 = p[(z + 2 * G) * zs], v3 = p[(z + 3 * G) * zs];
    s += v0; s += v1; s += v2; s += v3;
  }
  for (; z < nz; z += G) s += p[z * zs];
  if constexpr (G == 1) {
    if (e < pairs) g_w[(long)e * KK + t] = s;
  } else {
    red[g][el] = s;
    __syncthreads();
    if (g == 0 && e < pairs) {
      float sum = 0.f;
#pragma unroll
      for (int k = 0; k < G; ++k) sum += red[k][el];
      g_w[(long)e * KK + t] = sum;
    }
  }
}

// ---------------------------------------------------------------------------
// input gradient: g_x[n, ci, j] = sum over (t, co) of wt[t][ci][co] * g_y[n, co, j + dD(t)]
// The kernel tile is K-major in LDS (rows c_i, 16-byte fragments); the g_y tile is K-strided
// (rows of k, or of k-pairs for bf16, so that a lane picks up its k-values with 32-bit reads).
// ---------------------------------------------------------------------------
struct XDgradArgs {
  const void* gy;
  const void* wt;   // [KK][Ci][Co]
  void* gx;         // g_x, or its phase planes [s*s][N][Ci][HW] for a strided layer
  const uint8_t* tab;
  const int2* tapd; // [phase][KK]: {tap, offset of the g_y element that position 0 reads}
  const int* ntap;  // [phase]
  int N, Ci, Co, KK;
  int HW, HWp, HWy, nv, Jp;  // plane of the output (a phase plane for strided layers), plane of g_y
  int total_gy;
  int inner_ok;   // 1: a shifted vector of an inner image (0 < n < N - 1) stays inside g_y
  FastDiv d_hwp, d_nck;  // d_nck: by the number of K chunks per tap of the launched tile shape
};

template <class T, int BM, int BN, int KV>
constexpr int xdgrad_smem_bytes() {
  constexpr int VE = 16 / (int)sizeof(T);
  constexpr int RPS = sizeof(T) == 2 ? 2 : 1;
  constexpr int SC = BN + VE;
  constexpr int tile = BM * (KV * 16 + 16) + (KV * VE / RPS) * (BN + 4) * 4;
  constexpr int out = (BM / 2) * SC * (int)sizeof(T);
  return tile > out ? tile : out;
}

// DEPTH = K chunks a lane keeps in flight in registers (two measured no faster than one: the
// loop is bound by LDS traffic, not by the latency of the global loads)
template <class T, int TM, int TN, int KV, int DEPTH>
__global__ __launch_bounds__(kThreads) void xdgrad_k(XDgradArgs a) {
  constexpr int WM = 2, WN = 2;
  constexpr int BM = WM * TM * 16, BN = WN * TN * 16;
  constexpr int VE = Mma<T>::VE, KSTEP = Mma<T>::KSTEP, BK = KV * VE;
  constexpr int RPS = sizeof(T) == 2 ? 2 : 1;    // k rows per word row of the g_y tile
  constexpr int KP = BK / RPS;                   // word rows of the g_y tile
  constexpr int RB = KV * 16 + 16;               // bytes of one kernel-tile row
  constexpr int RPP = kThreads / KV;             // kernel-tile rows per pass
  constexpr int LA = BM / RPP;                   // kernel vectors per lane and chunk
  constexpr int SB = BN + 4;                     // word stride of the g_y tile
  constexpr int VPB = BN / VE;                   // vectors per k row
  constexpr int PB = KP * VPB / kThreads;        // word-row slots per lane
  constexpr int WSTEP = kThreads / VPB;          // word rows between a lane's slots
  constexpr int SC = BN + VE;                    // element stride of the output staging tile
  static_assert(kThreads % VPB == 0 && PB >= 1 && PB * RPS <= 16 && LA >= 1, "slot layout");
  __shared__ __attribute__((aligned(16))) unsigned char smem[xdgrad_smem_bytes<T, BM, BN, KV>()];
  unsigned char* As = smem;
  uint32_t* Bs = reinterpret_cast<uint32_t*>(smem + BM * RB);
  const T* gy = static_cast<const T*>(a.gy);
  const T* wt = static_cast<const T*>(a.wt);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int m0 = blockIdx.y * BM;
  const int j0 = blockIdx.x * BN;

  // this lane's column vector of the g_y tile
  const int vib = tid % VPB, wrb0 = tid / VPB;
  const int jq = j0 + vib * VE;
  const int nimg = (int)a.d_hwp.div((uint32_t)jq);
  const int q = jq - nimg * a.HWp;
  const bool img = nimg < a.N;
  const int nn = min(nimg, a.N - 1);
  const bool inner = a.inner_ok && nn > 0 && nn < a.N - 1;  // a shifted vector cannot leave the tensor
  const int colbase = nn * a.Co * a.HWy + q;
  // and its vector of the kernel tile
  const int via = tid % KV, rowa0 = tid / KV;
  const bool rows_full = m0 + BM <= a.Ci;
  const int nck = (a.Co + BK - 1) / BK;
  const int cico = a.Ci * a.Co;

  int rowa[LA];
#pragma unroll
  for (int i = 0; i < LA; ++i) rowa[i] = min(m0 + rowa0 + RPP * i, a.Ci - 1) * a.Co + via * VE;

  const int ph = blockIdx.z;                     // phase of g_x (0 for stride 1)
  const int2* taps = a.tapd + ph * a.KK;
  const int ntap = a.ntap[ph];
  const uint8_t* tab = a.tab + (long)ph * a.KK * a.nv;

  struct Regs {
    uint4 ra[LA], rb[PB * RPS];
    uint32_t mb, off;
  };
  Regs regs[DEPTH];
  const int iters = ntap * nck;
  auto fetch = [&](Regs& g, int it) {
    const int kk = (int)a.d_nck.div((uint32_t)it);
    const int k0 = (it - kk * nck) * BK;
    const int2 ti = taps[kk];
    const int t = ti.x;
    const int cb = colbase + ti.y;
    g.mb = img ? vec_mask<T>(tab[t * a.nv + (q >> 3)], q) : 0u;
    g.off = 0;
    const bool kfull = k0 + BK <= a.Co;
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const int kv = min(k0 + via * VE, a.Co - VE) - via * VE;  // keeps the vector inside its row
      g.ra[i] = *reinterpret_cast<const uint4*>(wt + ((long)t * cico + rowa[i] + kv));
    }
    if (inner && kfull) {
#pragma unroll
      for (int i = 0; i < PB; ++i)
#pragma unroll
        for (int h = 0; h < RPS; ++h)
          g.rb[i * RPS + h] = load_vec<T>(gy + (cb + (k0 + (wrb0 + i * WSTEP) * RPS + h) * a.HWy));
    } else {
#pragma unroll
      for (int i = 0; i < PB; ++i)
#pragma unroll
        for (int h = 0; h < RPS; ++h) {
          const int k = min(k0 + (wrb0 + i * WSTEP) * RPS + h, a.Co - 1);
          const int o = cb + k * a.HWy;
          const int oc = min(max(o, 0), a.total_gy - VE);
          g.off |= (o != oc) ? 1u << (i * RPS + h) : 0u;
          g.rb[i * RPS + h] = load_vec<T>(gy + oc);
        }
    }
  };
  // word c of a bf16 word row = (row k col c) | (row k + 1 col c) << 16
  auto put = [&](uint32_t* d, const uint4& lo, const uint4& hi) {
    if constexpr (sizeof(T) == 4) {
      *reinterpret_cast<uint4*>(d) = lo;
    } else {
      uint4 o0, o1;
      o0.x = (lo.x & 0xffffu) | (hi.x << 16); o0.y = (lo.x >> 16) | (hi.x & 0xffff0000u);
      o0.z = (lo.y & 0xffffu) | (hi.y << 16); o0.w = (lo.y >> 16) | (hi.y & 0xffff0000u);
      o1.x = (lo.z & 0xffffu) | (hi.z << 16); o1.y = (lo.z >> 16) | (hi.z & 0xffff0000u);
      o1.z = (lo.w & 0xffffu) | (hi.w << 16); o1.w = (lo.w >> 16) | (hi.w & 0xffff0000u);
      *reinterpret_cast<uint4*>(d) = o0;
      *reinterpret_cast<uint4*>(d + 4) = o1;
    }
  };
  auto stage = [&](Regs& g, int it) {
    const int kk = (int)a.d_nck.div((uint32_t)it);
    const int k0 = (it - kk * nck) * BK;
    if (g.off) {  // first or last rows of g_y only: shift the moved vectors back
      const int cb = colbase + taps[kk].y;
#pragma unroll
      for (int i = 0; i < PB; ++i)
#pragma unroll
        for (int h = 0; h < RPS; ++h) {
          const int k = min(k0 + (wrb0 + i * WSTEP) * RPS + h, a.Co - 1);
          const int o = cb + k * a.HWy;
          g.rb[i * RPS + h] = realign<T>(g.rb[i * RPS + h], min(max(o - min(max(o, 0), a.total_gy - VE), -VE), VE));
        }
    }
    const bool kfull = k0 + BK <= a.Co;
    if (rows_full && kfull) {
#pragma unroll
      for (int i = 0; i < LA; ++i) *reinterpret_cast<uint4*>(As + (rowa0 + RPP * i) * RB + via * 16) = g.ra[i];
    } else {
      const bool kok = k0 + via * VE < a.Co;   // C_o is a multiple of VE: a vector is in or out
#pragma unroll
      for (int i = 0; i < LA; ++i) {
        const int row = rowa0 + RPP * i;
        *reinterpret_cast<uint4*>(As + row * RB + via * 16) = (kok && m0 + row < a.Ci) ? g.ra[i] : make_uint4(0, 0, 0, 0);
      }
    }
    uint32_t wb[4];
    expand_mask<T>(g.mb, wb);
    if (kfull) {
#pragma unroll
      for (int i = 0; i < PB; ++i)
        put(Bs + (wrb0 + i * WSTEP) * SB + vib * VE, and4(g.rb[i * RPS], wb), and4(g.rb[i * RPS + RPS - 1], wb));
    } else {
#pragma unroll
      for (int i = 0; i < PB; ++i) {
        const int wr = wrb0 + i * WSTEP;
        uint4 val[2];
#pragma unroll
        for (int h = 0; h < RPS; ++h)
          val[h] = k0 + wr * RPS + h < a.Co ? and4(g.rb[i * RPS + h], wb) : make_uint4(0, 0, 0, 0);
        put(Bs + wr * SB + vib * VE, val[0], val[RPS - 1]);
      }
    }
  };

  // bf16 with an even number of 16-row blocks per wave in both directions: 32 x 32 x 16 MFMAs
  constexpr bool BIG = sizeof(T) == 2 && TM % 2 == 0 && TN % 2 == 0;
  f32x4 acc[TM][TN];
  f32x16 acc32[BIG ? TM / 2 : 1][BIG ? TN / 2 : 1];
  if constexpr (BIG) {
#pragma unroll
    for (int i = 0; i < TM / 2; ++i)
#pragma unroll
      for (int j = 0; j < TN / 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc32[i][j][e] = 0.f;
  } else {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

#pragma unroll
  for (int dd = 0; dd < DEPTH; ++dd)
    if (dd < iters) fetch(regs[dd], dd);
  const int r = lane & 15, kg = lane >> 4;
  for (int it0 = 0; it0 < iters; it0 += DEPTH) {
#pragma unroll
    for (int dd = 0; dd < DEPTH; ++dd) {
      const int it = it0 + dd;
      if (it >= iters) break;  // uniform
      stage(regs[dd], it);
      __syncthreads();
      if (it + DEPTH < iters) fetch(regs[dd], it + DEPTH);
      if constexpr (BIG) {
        const int r32 = lane & 31, kh = lane >> 5;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {  // 16 k = 8 pair rows per MFMA
          uint4 fa[TM / 2], fb[TN / 2];
#pragma unroll
          for (int i = 0; i < TM / 2; ++i)
            fa[i] = *reinterpret_cast<const uint4*>(As + ((wm * TM + 2 * i) * 16 + r32) * RB + ks * 32 + kh * 16);
#pragma unroll
          for (int j = 0; j < TN / 2; ++j) {
            const uint32_t* p = Bs + (ks * 8 + kh * 4) * SB + (wn * TN + 2 * j) * 16 + r32;
            fb[j] = make_uint4(p[0], p[SB], p[2 * SB], p[3 * SB]);
          }
#pragma unroll
          for (int i = 0; i < TM / 2; ++i)
#pragma unroll
            for (int j = 0; j < TN / 2; ++j) acc32[i][j] = mma32(fa[i], fb[j], acc32[i][j]);
        }
      } else if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (int ks = 0; ks < BK / KSTEP; ++ks) {  // 32 k = 16 pair rows per MFMA
          uint4 fa[TM], fb[TN];
#pragma unroll
          for (int i = 0; i < TM; ++i)
            fa[i] = *reinterpret_cast<const uint4*>(As + ((wm * TM + i) * 16 + r) * RB + ks * 64 + kg * 16);
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            const uint32_t* p = Bs + (ks * 16 + kg * 4) * SB + (wn * TN + j) * 16 + r;
            fb[j] = make_uint4(p[0], p[SB], p[2 * SB], p[3 * SB]);
          }
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = mma16(fa[i], fb[j], acc[i][j]);
        }
      } else {
#pragma unroll
        for (int ks = 0; ks < BK / KSTEP; ++ks) {  // 4 k per MFMA
          float fa[TM], fb[TN];
#pragma unroll
          for (int i = 0; i < TM; ++i)
            fa[i] = *reinterpret_cast<const float*>(As + ((wm * TM + i) * 16 + r) * RB + (ks * 4 + kg) * 4);
#pragma unroll
          for (int j = 0; j < TN; ++j) fb[j] = __uint_as_float(Bs[(ks * 4 + kg) * SB + (wn * TN + j) * 16 + r]);
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = mma16(fa[i], fb[j], acc[i][j]);
        }
      }
      __syncthreads();
    }
  }

  // the two wave rows of the tile go out one after the other through an LDS tile of BM / 2
  // rows (rounded once to the storage type), as 16-byte runs of pixels
  T* Cs = reinterpret_cast<T*>(smem);
  T* out = static_cast<T*>(a.gx) + (long)ph * a.N * a.Ci * a.HW;
  constexpr int HM = BM / 2;
  for (int half = 0; half < 2; ++half) {
    if (wm == half) {
      if constexpr (BIG) {
#pragma unroll
        for (int i = 0; i < TM / 2; ++i)
#pragma unroll
          for (int j = 0; j < TN / 2; ++j)
#pragma unroll
            for (int vv = 0; vv < 16; ++vv) {
              const int row = i * 32 + 8 * (vv >> 2) + 4 * (lane >> 5) + (vv & 3);
              const int col = (wn * TN + 2 * j) * 16 + (lane & 31);
              Cs[row * SC + col] = from_f32<T>(acc32[i][j][vv]);
            }
      } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int vv = 0; vv < 4; ++vv) {
              const int row = i * 16 + 4 * (lane >> 4) + vv;
              const int col = (wn * TN + j) * 16 + (lane & 15);
              Cs[row * SC + col] = from_f32<T>(acc[i][j][vv]);
            }
      }
    }
    __syncthreads();
    for (int s = tid; s < HM * VPB; s += kThreads) {
      const int row = s / VPB, vi = s - row * VPB;
      const int ci = m0 + half * HM + row;
      const int jj = j0 + vi * VE;
      const int n = (int)a.d_hwp.div((uint32_t)jj);
      const int qq = jj - n * a.HWp;
      if (ci >= a.Ci || n >= a.N || qq >= a.HW) continue;
      T* d = out + ((long)n * a.Ci + ci) * a.HW + qq;
      const T* src = Cs + row * SC + vi * VE;
      if (qq + VE <= a.HW) {
        const uint4 val = *reinterpret_cast<const uint4*>(src);
        Unal<T> o;
        o.w[0] = val.x; o.w[1] = val.y; o.w[2] = val.z; o.w[3] = val.w;
        *reinterpret_cast<Unal<T>*>(d) = o;
      } else {
        for (int e = 0; qq + e < a.HW; ++e) d[e] = src[e];
      }
    }
    __syncthreads();
  }
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

int up8(int v) { return (v + 7) / 8 * 8; }

// Geometry of the implicit GEMMs: PQ = plane of the x operand / of the g_x output (the phase
// plane Hq x Wq for strided layers, the image itself for stride 1), PY = plane of g_y.
struct XGeo {
  int s, nph, Hq, Wq, PQ, PY;
};

XGeo make_xgeo(const Geom& g) {
  XGeo q;
  q.s = g.s;
  q.nph = g.s * g.s;
  q.Hq = g.s == 1 ? g.H : (g.H + g.s - 1) / g.s;
  q.Wq = g.s == 1 ? g.W : g.Wy;
  q.PQ = q.Hq * q.Wq;
  q.PY = g.Hy * g.Wy;
  return q;
}

// largest |tap offset| in flattened pixels of a plane of pitch Wq
long max_shift(const Geom& g, const XGeo& q) {
  const long a = g.p, b = (long)g.dl * ((g.Kh > g.Kw ? g.Kh : g.Kw) - 1) - g.p;
  return ((a > b ? a : b) / g.s + 1) * (q.Wq + 1);
}

// one image holds more elements than a tap reaches: then only the first and the last image
// of a tensor need clamped loads
bool inner_images_safe(const Geom& g, const XGeo& q) {
  long skew = (long)q.PQ - q.PY;  // the planes of the two operands may differ in height
  if (skew < 0) skew = -skew;
  const long need = max_shift(g, q) + 16 + skew;
  return (long)g.Ci * q.PQ >= need && (long)g.Co * q.PY >= need;
}

struct XPlan {
  size_t off_tabw, off_tabd, off_taps, off_wt, off_xq, off_gxq, off_part, total;
  int nvw, nvd, nz, chunks_per_z, nchunks, bm, bn, kv;
};

// workspace layout, tile shape of the weight-gradient block and its number of K slabs
template <class T>
XPlan make_plan(const Geom& g, bool want_gw, bool want_gx) {
  const XGeo q = make_xgeo(g);
  XPlan p = {};
  p.nvw = up8(q.PY) / 8;
  p.nvd = up8(q.PQ) / 8;
  size_t off = 0;
  p.off_tabw = off; off += align256((size_t)g.KK * p.nvw);
  p.off_tabd = off; off += align256((size_t)q.nph * g.KK * p.nvd);
  p.off_taps = off; off += align256(sizeof(int) * ((size_t)g.KK + 2 * (size_t)q.nph * g.KK + q.nph));
  p.off_wt = off;
  if (want_gx) off += align256((size_t)g.KK * g.Co * g.Ci * g.b);
  p.off_xq = off;
  if (want_gw && g.s > 1) off += align256((size_t)q.nph * g.N * g.Ci * q.PQ * g.b);
  p.off_gxq = off;
  if (want_gx && g.s > 1) off += align256((size_t)q.nph * g.N * g.Ci * q.PQ * g.b);
  p.off_part = off;
  if (want_gw) {
    const bool small = g.Co <= 64 || g.Ci <= 64;   // 64 x 64 tiles for few channels
    p.bm = small ? 64 : 128;
    p.bn = small ? 64 : 128;
    p.kv = 16;   // 256 bytes of K per staged row (128 measured 5-15 % slower)
    const int bk = p.kv * Mma<T>::VE;
    p.nchunks = cdiv((long)g.N * up8(q.PY), bk);
    const long tiles = (long)cdiv(g.Co, p.bm) * cdiv(g.Ci, p.bn) * g.KK;
    const long slots = small ? 1024 : 512;      // blocks the chip holds at once
    long nz = slots / tiles;
    const long most = p.nchunks / 2 > 0 ? p.nchunks / 2 : 1;  // at least two chunks per block
    if (nz > most) nz = most;
    if (nz < 1) nz = 1;
    p.chunks_per_z = cdiv(p.nchunks, nz);
    p.nz = cdiv(p.nchunks, p.chunks_per_z);
    off += align256((size_t)p.nz * g.KK * g.Co * g.Ci * sizeof(float));
  }
  p.total = off;
  return p;
}

struct XTaps {
  int* tapw;
  int2* tapd;
  int* ntap;
};

XTaps taps_of(const Geom& g, const XGeo& q, const XPlan& p, char* ws) {
  XTaps t;
  int* base = reinterpret_cast<int*>(ws + p.off_taps);
  t.tapd = reinterpret_cast<int2*>(base);            // 8-byte aligned: first in the region
  t.tapw = base + 2 * q.nph * g.KK;
  t.ntap = t.tapw + g.KK;
  return t;
}

template <class T>
hipError_t launch_prep(const Geom& g, const XGeo& q, const XPlan& p, char* ws, const void* x, const void* w,
                       bool want_gw, bool want_gx, hipStream_t st) {
  const XTaps tp = taps_of(g, q, p, ws);
  PrepArgs a;
  a.tabw = reinterpret_cast<uint8_t*>(ws + p.off_tabw);
  a.tabd = reinterpret_cast<uint8_t*>(ws + p.off_tabd);
  a.tapw = tp.tapw; a.tapd = tp.tapd; a.ntap = tp.ntap;
  a.N = g.N; a.Ci = g.Ci; a.H = g.H; a.W = g.W; a.Hy = g.Hy; a.Wy = g.Wy; a.Hq = q.Hq; a.Wq = q.Wq;
  a.Kw = g.Kw; a.KK = g.KK; a.s = g.s; a.d = g.dl; a.p = g.p; a.nvw = p.nvw; a.nvd = p.nvd;
  const int nmax = p.nvw > p.nvd * q.nph ? p.nvw : p.nvd * q.nph;
  const int tab_blocks = cdiv((long)g.KK * nmax, kThreads);
  const int w_blocks = want_gx ? cdiv((long)g.Co * g.Ci * g.KK, kThreads) : 0;
  const int x_blocks = (want_gw && g.s > 1) ? cdiv((long)q.nph * g.N * g.Ci * q.PQ, kThreads) : 0;
  GF_LAUNCH(prep_k<T>, dim3(tab_blocks + w_blocks + x_blocks), dim3(kThreads), 0, st, a, tab_blocks,
                     w_blocks, static_cast<const T*>(w), reinterpret_cast<T*>(ws + p.off_wt), g.Co,
                     static_cast<const T*>(x), reinterpret_cast<T*>(ws + p.off_xq));
  return hipGetLastError();
}

template <class T>
hipError_t wgrad_t(const Geom& g, const XGeo& q, const XPlan& p, const void* x, const void* g_y, float* g_w,
                   char* wsb, hipStream_t st) {
  XWgradArgs a;
  a.gy = g_y;
  a.x = g.s > 1 ? static_cast<const void*>(wsb + p.off_xq) : x;
  a.part = reinterpret_cast<float*>(wsb + p.off_part);
  a.tab = reinterpret_cast<const uint8_t*>(wsb + p.off_tabw);
  a.tapw = taps_of(g, q, p, wsb).tapw;
  a.N = g.N; a.Ci = g.Ci; a.Co = g.Co; a.KK = g.KK;
  a.HW = q.PQ; a.HWy = q.PY; a.HWyp = up8(q.PY); a.nv = p.nvw;
  a.nchunks = p.nchunks; a.chunks_per_z = p.chunks_per_z; a.nz = p.nz;
  a.tx = cdiv(g.Ci, p.bn);
  a.tiles = a.tx * cdiv(g.Co, p.bm);
  a.R = a.tiles * g.KK;
  a.xcd_slabs = p.nz >= 8 ? 1 : 0;
  a.inner_ok = inner_images_safe(g, q) ? 1 : 0;
  a.total_x = q.nph * g.N * g.Ci * q.PQ;
  a.total_gy = g.N * g.Co * q.PY;
  a.d_hwyp = FastDiv((uint32_t)a.HWyp);
  a.d_r = FastDiv((uint32_t)a.R);
  a.d_tiles = FastDiv((uint32_t)a.tiles);
  a.d_tx = FastDiv((uint32_t)a.tx);
  const dim3 grid(a.xcd_slabs ? 8 * a.R * cdiv(p.nz, 8) : a.R * p.nz);
  if (p.bm == 64)
    GF_LAUNCH((xwgrad_k<T, 2, 2, 16>), grid, dim3(kThreads), 0, st, a);
  else
    GF_LAUNCH((xwgrad_k<T, 4, 4, 16>), grid, dim3(kThreads), 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int pairs = g.Co * g.Ci;
  // lanes per output: enough blocks for the chip when the output is small and the slabs are many
  const long outs = (long)pairs * g.KK;
  if (outs <= 16384 && p.nz >= 64)
    GF_LAUNCH(xfinalize_k<16>, dim3(cdiv(pairs, kThreads / 16), g.KK), dim3(kThreads), 0, st, a.part, g_w,
                       pairs, g.KK, p.nz);
  else if (outs <= 131072 && p.nz >= 16)
    GF_LAUNCH(xfinalize_k<4>, dim3(cdiv(pairs, kThreads / 4), g.KK), dim3(kThreads), 0, st, a.part, g_w,
                       pairs, g.KK, p.nz);
  else
    GF_LAUNCH(xfinalize_k<1>, dim3(cdiv(pairs, kThreads), g.KK), dim3(kThreads), 0, st, a.part, g_w, pairs,
                       g.KK, p.nz);
  return hipGetLastError();
}

template <class T>
hipError_t dgrad_t(const Geom& g, const XGeo& q, const XPlan& p, const void* g_y, void* g_x, char* wsb,
                   hipStream_t st) {
  const XTaps tp = taps_of(g, q, p, wsb);
  XDgradArgs a;
  a.gy = g_y; a.wt = wsb + p.off_wt;
  a.gx = g.s > 1 ? static_cast<void*>(wsb + p.off_gxq) : g_x;
  a.tab = reinterpret_cast<const uint8_t*>(wsb + p.off_tabd);
  a.tapd = tp.tapd; a.ntap = tp.ntap;
  a.N = g.N; a.Ci = g.Ci; a.Co = g.Co; a.KK = g.KK;
  a.HW = q.PQ; a.HWp = up8(q.PQ); a.HWy = q.PY; a.nv = p.nvd;
  a.Jp = g.N * a.HWp;
  a.total_gy = g.N * g.Co * q.PY;
  a.inner_ok = inner_images_safe(g, q) ? 1 : 0;
  a.d_hwp = FastDiv((uint32_t)a.HWp);
  // tile shape: 128 x 128 when that still gives about two blocks per compute unit, else narrower
  const long t128 = (long)cdiv(a.Jp, 128) * cdiv(g.Ci, 128) * q.nph;
  constexpr int VE = Mma<T>::VE;
  if (g.Ci > 64 && t128 >= 400) {
    a.d_nck = FastDiv((uint32_t)cdiv(g.Co, 8 * VE));
    GF_LAUNCH((xdgrad_k<T, 4, 4, 8, 1>), dim3(cdiv(a.Jp, 128), cdiv(g.Ci, 128), q.nph), dim3(kThreads), 0, st, a);
  } else if (g.Ci > 64) {
    a.d_nck = FastDiv((uint32_t)cdiv(g.Co, 16 * VE));
    GF_LAUNCH((xdgrad_k<T, 4, 2, 16, 1>), dim3(cdiv(a.Jp, 64), cdiv(g.Ci, 128), q.nph), dim3(kThreads), 0, st, a);
  } else {
    a.d_nck = FastDiv((uint32_t)cdiv(g.Co, 16 * VE));
    GF_LAUNCH((xdgrad_k<T, 2, 2, 16, 1>), dim3(cdiv(a.Jp, 64), cdiv(g.Ci, 64), q.nph), dim3(kThreads), 0, st, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || g.s == 1) return e;
  const long tot = (long)g.N * g.Ci * g.H * g.W;
  GF_LAUNCH(interleave_k<T>, dim3(cdiv(tot, kThreads)), dim3(kThreads), 0, st,
                     reinterpret_cast<const T*>(wsb + p.off_gxq), static_cast<T*>(g_x), g.N * g.Ci, g.H, g.W,
                     q.Hq, q.Wq, g.s);
  return hipGetLastError();
}

template <class T>
hipError_t implicit_t(const Geom& g, const void* x, const void* w, const void* g_y, float* g_w, void* g_x,
                      void* ws, hipStream_t st) {
  const XGeo q = make_xgeo(g);
  const XPlan p = make_plan<T>(g, g_w != nullptr, g_x != nullptr);
  char* wsb = static_cast<char*>(ws);
  hipError_t e = launch_prep<T>(g, q, p, wsb, x, w, g_w != nullptr, g_x != nullptr, st);
  if (e != hipSuccess) return e;
  if (g_w) {
    e = wgrad_t<T>(g, q, p, x, g_y, g_w, wsb, st);
    if (e != hipSuccess) return e;
  }
  if (g_x) e = dgrad_t<T>(g, q, p, g_y, g_x, wsb, st);
  return e;
}

// K slabs of the plain contraction part[z][co][ci] = sum_{n, p} a[n, co, p] * b[n, ci, p] over maps of P pixels
template <class T>
void plain_plan(const Geom& g, int* nz, int* chunks_per_z, int* nchunks) {
  const int bk = 16 * Mma<T>::VE;
  *nchunks = cdiv((long)g.N * up8(g.P), bk);
  const long tiles = (long)cdiv(g.Co, 128) * cdiv(g.Ci, 128);
  long z = 512 / tiles;
  const long most = *nchunks / 2 > 0 ? *nchunks / 2 : 1;
  if (z > most) z = most;
  if (z < 1) z = 1;
  *chunks_per_z = cdiv(*nchunks, z);
  *nz = cdiv(*nchunks, *chunks_per_z);
}

template <class T>
hipError_t plain_wgrad_t(const Geom& g, const void* x_u, const void* gy_u, float* part, int* nz_out,
                         hipStream_t st) {
  XWgradArgs a;
  a.gy = gy_u; a.x = x_u; a.part = part;
  a.tab = nullptr; a.tapw = nullptr;
  a.N = g.N; a.Ci = g.Ci; a.Co = g.Co; a.KK = 1;
  a.HW = g.P; a.HWy = g.P; a.HWyp = up8(g.P); a.nv = 0;
  plain_plan<T>(g, &a.nz, &a.chunks_per_z, &a.nchunks);
  a.tx = cdiv(g.Ci, 128);
  a.tiles = a.tx * cdiv(g.Co, 128);
  a.R = a.tiles;
  a.xcd_slabs = a.nz >= 8 ? 1 : 0;
  a.inner_ok = ((long)g.Ci * g.P >= 16 && (long)g.Co * g.P >= 16) ? 1 : 0;
  a.total_x = g.N * g.Ci * g.P;
  a.total_gy = g.N * g.Co * g.P;
  a.d_hwyp = FastDiv((uint32_t)a.HWyp);
  a.d_r = FastDiv((uint32_t)a.R);
  a.d_tiles = FastDiv((uint32_t)a.tiles);
  a.d_tx = FastDiv((uint32_t)a.tx);
  *nz_out = a.nz;
  const dim3 grid(a.xcd_slabs ? 8 * a.R * cdiv(a.nz, 8) : a.R * a.nz);
  GF_LAUNCH((xwgrad_k<T, 4, 4, 16>), grid, dim3(kThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace

// The filtered weight gradient (Eq. 5) of a large dense layer is the same contraction with one
// tap and no padding: these are the 128 x 128 tiles of the exact weight gradient on x_u and gy_u.
bool plain_wgrad_ok(const Geom& g) {
  const long lim = 2147483647L;
  if (g.g != 1 || g.Co < 128 || g.Ci < 128) return false;
  if ((long)g.N * g.Ci * g.P + 1024 >= lim || (long)g.N * g.Co * g.P + 1024 >= lim) return false;
  if ((long)g.N * up8(g.P) + 1024 >= lim || (long)g.N * g.Ci * g.P < 16 || (long)g.N * g.Co * g.P < 16) return false;
  return 2.0 * g.Co * g.Ci * g.N * g.P >= kPlainWgradMinFlops;
}

int plain_wgrad_splits(const Geom& g) {
  int nz, cpz, nch;
  if (g.dtype == GF_BF16) plain_plan<bf16_t>(g, &nz, &cpz, &nch); else plain_plan<float>(g, &nz, &cpz, &nch);
  return nz;
}

hipError_t launch_plain_wgrad(const Geom& g, const void* x_u, const void* gy_u, float* part, int* nz_out,
                              hipStream_t st) {
  return g.dtype == GF_BF16 ? plain_wgrad_t<bf16_t>(g, x_u, gy_u, part, nz_out, st)
                            : plain_wgrad_t<float>(g, x_u, gy_u, part, nz_out, st);
}

// Dense layers with channel counts that are multiples of the vector length, whose tap offsets
// are constant in flattened pixels: stride 1 with W_y == W, or stride s with ceil(W / s) <= W_y
// (phase planes of pitch W_y); every index (plus the largest tap offset) below 2^31.
bool implicit_ok(const Geom& g) {
  const int ve = 16 / g.b;
  if (g.g != 1 || g.KK > 1024 || g.s > 4) return false;
  if (g.s == 1 ? g.Wy != g.W : (g.W + g.s - 1) / g.s > g.Wy) return false;
  if (g.Ci % ve != 0 || g.Co % ve != 0) return false;
  const XGeo q = make_xgeo(g);
  const long lim = 2147483647L;
  const long pqp = up8(q.PQ), pyp = up8(q.PY);
  const long reach = max_shift(g, q) + 1024;
  const long tx = (long)q.nph * g.N * g.Ci * q.PQ, ty = (long)g.N * g.Co * q.PY;
  if (tx < ve || ty < ve) return false;
  if (tx + reach + pqp >= lim || ty + reach + pyp >= lim) return false;
  if ((long)g.N * g.Ci * g.H * g.W >= lim) return false;
  if ((long)g.N * pqp + 1024 >= lim || (long)g.N * pyp + 1024 >= lim) return false;
  if ((long)g.KK * g.Co * g.Ci >= lim) return false;
  if (cdiv(g.Ci, 64) > 65535 || cdiv(g.Co, 64) > 65535) return false;
  if ((long)cdiv(g.Ci, 64) * cdiv(g.Co, 64) * g.KK * 8 * 130 >= lim) return false;  // one-dimensional grid
  return true;
}

size_t ws_implicit(const Geom& g, bool want_gw, bool want_gx) {
  return g.dtype == GF_BF16 ? make_plan<bf16_t>(g, want_gw, want_gx).total : make_plan<float>(g, want_gw, want_gx).total;
}

// g_w and / or g_x (either may be null): one set-up launch, then the GEMM launches
hipError_t launch_implicit(const Geom& g, const void* x, const void* w, const void* g_y, float* g_w, void* g_x,
                           void* ws, hipStream_t st) {
  return g.dtype == GF_BF16 ? implicit_t<bf16_t>(g, x, w, g_y, g_w, g_x, ws, st)
                            : implicit_t<float>(g, x, w, g_y, g_w, g_x, ws, st);
}

}  // namespace gf
