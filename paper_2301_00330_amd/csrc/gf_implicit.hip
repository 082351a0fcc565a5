// Vanilla back-propagation (Sec. 3.1) of dense stride-1 convolutions whose output map is as
// wide as the input map ("same" padding), as implicit GEMMs on the MFMA cores of gfx950:
//
//   weight gradient  g_th[co, ci, t] = sum_{n, k} g_y[n, co, k] * x[n, ci, k + dW(t)]      (k: output pixel)
//   input gradient   g_x[n, ci, j]   = sum_{t, co} th[co, ci, t] * g_y[n, co, j + dD(t)]   (j: input pixel)
//
// For such layers the pixel a tap reads is the flattened pixel index plus a constant,
//   dW(t) = (u d - p) W + (v d - p),   dD(t) = (p - u d) W_y + (p - v d),   t = (u, v),
// wherever the tap stays inside the image; where it leaves it the factor is a zero of the
// padding.  So no column tensor is built: the shifted operand is read straight from the
// tensor with 16-byte loads at 2- or 4-byte alignment, and a byte table [tap][8 pixels] says
// which of the eight elements are padding.  Planes are addressed as if they held HWp = 8 *
// ceil(HW / 8) pixels, so that a vector never straddles two images; the surplus positions
// are masked like padding.
//
// Tiles: 256-lane blocks of 2 x 2 waves, each wave TM x TN MFMA tiles of 16 x 16
// (v_mfma_f32_16x16x32_bf16 / v_mfma_f32_16x16x4_f32); operands are staged through LDS one
// K chunk ahead of the arithmetic.  These GEMMs are small for the chip (a few hundred tiles),
// so what limits them is the bytes a compute unit has in flight: chunks are 256 bytes of K
// per row where registers allow it.
#include "gf_internal.h"

namespace gf {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;

template <class T> struct Mma;
template <> struct Mma<bf16_t> {
  static constexpr int KSTEP = 32, VE = 8;   // k per MFMA, elements per 16-byte vector
  static constexpr uint32_t FULL = 0xffu;
};
template <> struct Mma<float> {
  static constexpr int KSTEP = 4, VE = 4;
  static constexpr uint32_t FULL = 0xfu;
};

__device__ __forceinline__ f32x4 mma16(const uint4& a, const uint4& b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mma16(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// 16 bytes at the natural alignment of one element
template <class T> struct Unal;
template <> struct __attribute__((packed, aligned(2))) Unal<bf16_t> { uint32_t w[4]; };
template <> struct __attribute__((packed, aligned(4))) Unal<float> { uint32_t w[4]; };

// Elements o .. o + VE - 1 of a tensor of `total` (>= VE) elements.  The load is clamped into
// the tensor; `sh` tells realign() by how many elements the data is off.  Elements whose own
// address lies outside the tensor come out as zeros after realign().
template <class T>
__device__ __forceinline__ uint4 load_clamped(const T* base, int total, int o, int& sh) {
  constexpr int VE = Mma<T>::VE;
  const int oc = min(max(o, 0), total - VE);
  sh = min(max(o - oc, -VE), VE);
  const Unal<T> v = *reinterpret_cast<const Unal<T>*>(base + oc);
  return make_uint4(v.w[0], v.w[1], v.w[2], v.w[3]);
}

template <class T>
__device__ __forceinline__ uint4 load_vec(const T* p) {
  const Unal<T> v = *reinterpret_cast<const Unal<T>*>(p);
  return make_uint4(v.w[0], v.w[1], v.w[2], v.w[3]);
}

template <class T>
__device__ __forceinline__ uint4 realign(const uint4& v, int sh) {  // out[e] = in[e + sh]
  constexpr int VE = Mma<T>::VE;
  if (sh == 0) return v;
  if (sh >= VE || sh <= -VE) return make_uint4(0, 0, 0, 0);
  uint64_t lo = (uint64_t)v.x | ((uint64_t)v.y << 32), hi = (uint64_t)v.z | ((uint64_t)v.w << 32);
  int bits = sh * 8 * (int)sizeof(T);  // 0 < |bits| < 128
  if (bits > 0) {
    if (bits >= 64) { lo = hi >> (bits - 64); hi = 0; }
    else { lo = (lo >> bits) | (hi << (64 - bits)); hi >>= bits; }
  } else {
    bits = -bits;
    if (bits >= 64) { hi = lo << (bits - 64); lo = 0; }
    else { hi = (hi << bits) | (lo >> (64 - bits)); lo <<= bits; }
  }
  return make_uint4((uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32));
}

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
// Padding tables.  tabw[t][k / 8] bit e: output pixel k + e exists and tap t of it reads an
// input pixel inside the image (weight gradient); tabd[t][j / 8] bit e: input pixel j + e
// exists and tap t reaches it from an output pixel inside the map (input gradient).
// ---------------------------------------------------------------------------
struct TabArgs {
  uint8_t* tabw;
  uint8_t* tabd;
  int H, W, Hy, Wy, Kw, KK, d, p, nvw, nvd;
};

__device__ __forceinline__ void pad_table_body(const TabArgs& a, int block) {
  const int e0 = block * kThreads + threadIdx.x;
  const int nmax = a.nvw > a.nvd ? a.nvw : a.nvd;
  if (e0 >= a.KK * nmax) return;
  const int t = e0 / nmax, g = e0 - t * nmax;
  const int u = t / a.Kw, v = t - u * a.Kw;
  if (g < a.nvw) {
    uint32_t m = 0;
    for (int e = 0; e < 8; ++e) {
      const int k = g * 8 + e;
      if (k >= a.Hy * a.Wy) break;
      const int hy = k / a.Wy, wy = k - hy * a.Wy;
      const int hs = hy + u * a.d - a.p, ws = wy + v * a.d - a.p;
      if (hs >= 0 && hs < a.H && ws >= 0 && ws < a.W) m |= 1u << e;
    }
    a.tabw[t * a.nvw + g] = (uint8_t)m;
  }
  if (g < a.nvd) {
    uint32_t m = 0;
    for (int e = 0; e < 8; ++e) {
      const int j = g * 8 + e;
      if (j >= a.H * a.W) break;
      const int h = j / a.W, w = j - h * a.W;
      const int hs = h + a.p - u * a.d, ws = w + a.p - v * a.d;
      if (hs >= 0 && hs < a.Hy && ws >= 0 && ws < a.Wy) m |= 1u << e;
    }
    a.tabd[t * a.nvd + g] = (uint8_t)m;
  }
}

// One set-up launch: the first `tab_blocks` blocks fill the padding tables, the others write the
// kernel tap-major with c_o contiguous, wt[(t * Ci + ci) * Co + co] = w[(co * Ci + ci) * KK + t]
// (only when the input gradient is wanted: wt != null).
template <class T>
__global__ __launch_bounds__(kThreads) void prep_k(TabArgs tab, int tab_blocks, const T* w, T* wt, int Co,
                                                  int Ci, int KK) {
  if ((int)blockIdx.x < tab_blocks) {
    pad_table_body(tab, blockIdx.x);
    return;
  }
  const int e = ((int)blockIdx.x - tab_blocks) * kThreads + threadIdx.x;
  if (e >= Co * Ci * KK) return;
  const int co = e % Co;
  const int row = e / Co;
  const int ci = row % Ci, t = row / Ci;
  wt[e] = w[((long)co * Ci + ci) * KK + t];
}

// ---------------------------------------------------------------------------
// weight gradient: part[z][t][co][ci] = sum over the K chunks of slab z
// ---------------------------------------------------------------------------
struct XWgradArgs {
  const void* gy;
  const void* x;
  float* part;
  const uint8_t* tab;
  int N, Ci, Co, KK, Kw, W, d, p;
  int HW, HWy, HWyp, nv;
  int nchunks, chunks_per_z, nz;
  int tx, tiles, R;       // c_i tiles, c_i tiles * c_o tiles, tiles * KK
  int xcd_slabs;          // 1: slab z runs on XCD z % 8
  int inner_ok;           // 1: a shifted vector of an inner image (0 < n < N - 1) stays inside the tensors
  int total_x, total_gy;
  FastDiv d_hwyp, d_r, d_tiles, d_tx, d_kw;
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
  const int u = (int)a.d_kw.div((uint32_t)t), v = t - u * a.Kw;
  const int delta = (u * a.d - a.p) * a.W + (v * a.d - a.p);
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
    mb = img ? vec_mask<T>(a.tab[t * a.nv + (q >> 3)], q) : 0u;
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

  f32x4 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  if (kc0 < kc1) fetch(kc0);
  const int r = lane & 15, kg = lane >> 4;
  for (int kc = kc0; kc < kc1; ++kc) {
    stage(kc);
    __syncthreads();
    if (kc + 1 < kc1) fetch(kc + 1);
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
  // D[i = 4 * (lane / 16) + v][j = lane % 16] of every 16 x 16 tile
  float* dst = a.part + ((long)z * a.KK + t) * a.Co * a.Ci;
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

// g_w[co, ci, t] = sum_z part[z][t][co][ci], slabs added in index order; one lane per (t, co, ci)
__global__ __launch_bounds__(kThreads) void xfinalize_k(const float* part, float* g_w, int pairs, int KK,
                                                       int nz) {
  const int e = blockIdx.x * kThreads + threadIdx.x;
  const int t = blockIdx.y;
  if (e >= pairs) return;
  const float* p = part + (long)t * pairs + e;
  const long zs = (long)KK * pairs;
  float s = 0.f;
  int z = 0;
  for (; z + 3 < nz; z += 4) {
    const float v0 = p[z * zs], v1 = p[(z + 1) * zs], v2 = p[(z + 2) * zs], v3 = p[(z + 3) * zs];
    s += v0; s += v1; s += v2; s += v3;
  }
  for (; z < nz; ++z) s += p[z * zs];
  g_w[(long)e * KK + t] = s;
}

// ---------------------------------------------------------------------------
// input gradient: g_x[n, ci, j] = sum over (t, co) of wt[t][ci][co] * g_y[n, co, j + dD(t)]
// The kernel tile is K-major in LDS (rows c_i, 16-byte fragments); the g_y tile is K-strided
// (rows of k, or of k-pairs for bf16, so that a lane picks up its k-values with 32-bit reads).
// ---------------------------------------------------------------------------
struct XDgradArgs {
  const void* gy;
  const void* wt;   // [KK][Ci][Co]
  void* gx;
  const uint8_t* tab;
  int N, Ci, Co, KK, Kw, Wy, d, p;
  int HW, HWp, HWy, nv, Jp;
  int total_gy;
  int inner_ok;   // 1: a shifted vector of an inner image (0 < n < N - 1) stays inside g_y
  FastDiv d_hwp;
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

template <class T, int TM, int TN, int KV>
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
  constexpr uint32_t FULL = Mma<T>::FULL;
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

  uint4 ra[LA], rb[PB * RPS];
  uint32_t mb = 0, off = 0;
  auto tap_delta = [&](int t) {
    const int u = t / a.Kw, v = t - u * a.Kw;
    return (a.p - u * a.d) * a.Wy + (a.p - v * a.d);
  };
  auto fetch = [&](int t, int k0) {
    const int cb = colbase + tap_delta(t);
    mb = img ? vec_mask<T>(a.tab[t * a.nv + (q >> 3)], q) : 0u;
    off = 0;
    const bool kfull = k0 + BK <= a.Co;
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const int kv = min(k0 + via * VE, a.Co - VE) - via * VE;  // keeps the vector inside its row
      ra[i] = *reinterpret_cast<const uint4*>(wt + ((long)t * cico + rowa[i] + kv));
    }
    if (inner && kfull) {
#pragma unroll
      for (int i = 0; i < PB; ++i)
#pragma unroll
        for (int h = 0; h < RPS; ++h)
          rb[i * RPS + h] = load_vec<T>(gy + (cb + (k0 + (wrb0 + i * WSTEP) * RPS + h) * a.HWy));
    } else {
#pragma unroll
      for (int i = 0; i < PB; ++i)
#pragma unroll
        for (int h = 0; h < RPS; ++h) {
          const int k = min(k0 + (wrb0 + i * WSTEP) * RPS + h, a.Co - 1);
          const int o = cb + k * a.HWy;
          const int oc = min(max(o, 0), a.total_gy - VE);
          off |= (o != oc) ? 1u << (i * RPS + h) : 0u;
          rb[i * RPS + h] = load_vec<T>(gy + oc);
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
  auto stage = [&](int t, int k0) {
    if (off) {  // first or last rows of g_y only: shift the moved vectors back
      const int cb = colbase + tap_delta(t);
#pragma unroll
      for (int i = 0; i < PB; ++i)
#pragma unroll
        for (int h = 0; h < RPS; ++h) {
          const int k = min(k0 + (wrb0 + i * WSTEP) * RPS + h, a.Co - 1);
          const int o = cb + k * a.HWy;
          rb[i * RPS + h] = realign<T>(rb[i * RPS + h], min(max(o - min(max(o, 0), a.total_gy - VE), -VE), VE));
        }
    }
    const bool kfull = k0 + BK <= a.Co;
    if (rows_full && kfull) {
#pragma unroll
      for (int i = 0; i < LA; ++i) *reinterpret_cast<uint4*>(As + (rowa0 + RPP * i) * RB + via * 16) = ra[i];
    } else {
      const bool kok = k0 + via * VE < a.Co;   // C_o is a multiple of VE: a vector is in or out
#pragma unroll
      for (int i = 0; i < LA; ++i) {
        const int row = rowa0 + RPP * i;
        *reinterpret_cast<uint4*>(As + row * RB + via * 16) = (kok && m0 + row < a.Ci) ? ra[i] : make_uint4(0, 0, 0, 0);
      }
    }
    uint32_t wb[4];
    expand_mask<T>(mb, wb);
    if (kfull) {
#pragma unroll
      for (int i = 0; i < PB; ++i)
        put(Bs + (wrb0 + i * WSTEP) * SB + vib * VE, and4(rb[i * RPS], wb), and4(rb[i * RPS + RPS - 1], wb));
    } else {
#pragma unroll
      for (int i = 0; i < PB; ++i) {
        const int wr = wrb0 + i * WSTEP;
        uint4 val[2];
#pragma unroll
        for (int h = 0; h < RPS; ++h)
          val[h] = k0 + wr * RPS + h < a.Co ? and4(rb[i * RPS + h], wb) : make_uint4(0, 0, 0, 0);
        put(Bs + wr * SB + vib * VE, val[0], val[RPS - 1]);
      }
    }
  };

  f32x4 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  fetch(0, 0);
  const int r = lane & 15, kg = lane >> 4;
  for (int t = 0; t < a.KK; ++t)
    for (int c = 0; c < nck; ++c) {
      stage(t, c * BK);
      __syncthreads();
      if (c + 1 < nck) fetch(t, (c + 1) * BK);
      else if (t + 1 < a.KK) fetch(t + 1, 0);
      if constexpr (sizeof(T) == 2) {
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

  // the two wave rows of the tile go out one after the other through an LDS tile of BM / 2
  // rows (rounded once to the storage type), as 16-byte runs of pixels
  T* Cs = reinterpret_cast<T*>(smem);
  T* out = static_cast<T*>(a.gx);
  constexpr int HM = BM / 2;
  for (int half = 0; half < 2; ++half) {
    if (wm == half) {
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

// largest |tap offset| in flattened pixels
long max_shift(const Geom& g) {
  const long a = g.p, b = (long)g.dl * ((g.Kh > g.Kw ? g.Kh : g.Kw) - 1) - g.p;
  return (a > b ? a : b) * (g.W + 1);
}

// one image holds more elements than a tap reaches: then only the first and the last image
// of a tensor need clamped loads
bool inner_images_safe(const Geom& g) {
  long skew = (long)g.H * g.W - (long)g.Hy * g.Wy;  // the planes of x and g_y may differ in height
  if (skew < 0) skew = -skew;
  const long need = max_shift(g) + 16 + skew;
  return (long)g.Ci * g.H * g.W >= need && (long)g.Co * g.Hy * g.Wy >= need;
}

int hwp_of(int hw) { return (hw + 7) / 8 * 8; }

struct XPlan {
  size_t off_tabw, off_tabd, off_wp, off_part, total;
  int nvw, nvd, nz, chunks_per_z, nchunks, bm, bn, kv;
};

// workspace layout, tile shape of the weight-gradient block and its number of K slabs
template <class T>
XPlan make_plan(const Geom& g, bool want_gw, bool want_gx) {
  XPlan p = {};
  p.nvw = hwp_of(g.Hy * g.Wy) / 8;
  p.nvd = hwp_of(g.H * g.W) / 8;
  size_t off = 0;
  p.off_tabw = off; off += align256((size_t)g.KK * p.nvw);
  p.off_tabd = off; off += align256((size_t)g.KK * p.nvd);
  p.off_wp = off;
  if (want_gx) off += align256((size_t)g.KK * g.Co * g.Ci * g.b);
  p.off_part = off;
  if (want_gw) {
    const bool small = g.Co <= 64 || g.Ci <= 64;   // 64 x 64 tiles for few channels
    p.bm = small ? 64 : 128;
    p.bn = small ? 64 : 128;
    p.kv = 16;
    const int bk = p.kv * Mma<T>::VE;
    p.nchunks = cdiv((long)g.N * hwp_of(g.Hy * g.Wy), bk);
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

template <class T>
hipError_t launch_prep(const Geom& g, const XPlan& p, char* ws, const void* w, bool want_gx, hipStream_t st) {
  TabArgs t;
  t.tabw = reinterpret_cast<uint8_t*>(ws + p.off_tabw);
  t.tabd = reinterpret_cast<uint8_t*>(ws + p.off_tabd);
  t.H = g.H; t.W = g.W; t.Hy = g.Hy; t.Wy = g.Wy; t.Kw = g.Kw; t.KK = g.KK; t.d = g.dl; t.p = g.p;
  t.nvw = p.nvw; t.nvd = p.nvd;
  const int nmax = p.nvw > p.nvd ? p.nvw : p.nvd;
  const int tab_blocks = cdiv((long)g.KK * nmax, kThreads);
  const int w_blocks = want_gx ? cdiv((long)g.Co * g.Ci * g.KK, kThreads) : 0;
  hipLaunchKernelGGL(prep_k<T>, dim3(tab_blocks + w_blocks), dim3(kThreads), 0, st, t, tab_blocks,
                     static_cast<const T*>(w), reinterpret_cast<T*>(ws + p.off_wp), g.Co, g.Ci, g.KK);
  return hipGetLastError();
}

template <class T>
hipError_t wgrad_t(const Geom& g, const XPlan& p, const void* x, const void* g_y, float* g_w, char* wsb,
                   hipStream_t st) {
  XWgradArgs a;
  a.gy = g_y; a.x = x;
  a.part = reinterpret_cast<float*>(wsb + p.off_part);
  a.tab = reinterpret_cast<const uint8_t*>(wsb + p.off_tabw);
  a.N = g.N; a.Ci = g.Ci; a.Co = g.Co; a.KK = g.KK; a.Kw = g.Kw; a.W = g.W; a.d = g.dl; a.p = g.p;
  a.HW = g.H * g.W; a.HWy = g.Hy * g.Wy; a.HWyp = hwp_of(a.HWy); a.nv = p.nvw;
  a.nchunks = p.nchunks; a.chunks_per_z = p.chunks_per_z; a.nz = p.nz;
  a.tx = cdiv(g.Ci, p.bn);
  a.tiles = a.tx * cdiv(g.Co, p.bm);
  a.R = a.tiles * g.KK;
  a.xcd_slabs = p.nz >= 8 ? 1 : 0;
  a.inner_ok = inner_images_safe(g) ? 1 : 0;
  a.total_x = g.N * g.Ci * a.HW;
  a.total_gy = g.N * g.Co * a.HWy;
  a.d_hwyp = FastDiv((uint32_t)a.HWyp);
  a.d_r = FastDiv((uint32_t)a.R);
  a.d_tiles = FastDiv((uint32_t)a.tiles);
  a.d_tx = FastDiv((uint32_t)a.tx);
  a.d_kw = FastDiv((uint32_t)g.Kw);
  const dim3 grid(a.xcd_slabs ? 8 * a.R * cdiv(p.nz, 8) : a.R * p.nz);
  if (p.bm == 64)
    hipLaunchKernelGGL((xwgrad_k<T, 2, 2, 16>), grid, dim3(kThreads), 0, st, a);
  else
    hipLaunchKernelGGL((xwgrad_k<T, 4, 4, 16>), grid, dim3(kThreads), 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int pairs = g.Co * g.Ci;
  hipLaunchKernelGGL(xfinalize_k, dim3(cdiv(pairs, kThreads), g.KK), dim3(kThreads), 0, st, a.part, g_w, pairs,
                     g.KK, p.nz);
  return hipGetLastError();
}

template <class T>
hipError_t dgrad_t(const Geom& g, const XPlan& p, const void* g_y, void* g_x, char* wsb, hipStream_t st) {
  XDgradArgs a;
  a.gy = g_y; a.wt = wsb + p.off_wp; a.gx = g_x;
  a.tab = reinterpret_cast<const uint8_t*>(wsb + p.off_tabd);
  a.N = g.N; a.Ci = g.Ci; a.Co = g.Co; a.KK = g.KK; a.Kw = g.Kw; a.Wy = g.Wy; a.d = g.dl; a.p = g.p;
  a.HW = g.H * g.W; a.HWp = hwp_of(a.HW); a.HWy = g.Hy * g.Wy; a.nv = p.nvd;
  a.Jp = g.N * a.HWp;
  a.total_gy = g.N * g.Co * a.HWy;
  a.inner_ok = inner_images_safe(g) ? 1 : 0;
  a.d_hwp = FastDiv((uint32_t)a.HWp);
  // tile shape: 128 x 128 when that still gives about two blocks per compute unit, else narrower
  const long t128 = (long)cdiv(a.Jp, 128) * cdiv(g.Ci, 128);
  if (g.Ci > 64 && t128 >= 400) {
    hipLaunchKernelGGL((xdgrad_k<T, 4, 4, 8>), dim3(cdiv(a.Jp, 128), cdiv(g.Ci, 128)), dim3(kThreads), 0, st, a);
  } else if (g.Ci > 64) {
    hipLaunchKernelGGL((xdgrad_k<T, 4, 2, 16>), dim3(cdiv(a.Jp, 64), cdiv(g.Ci, 128)), dim3(kThreads), 0, st, a);
  } else {
    hipLaunchKernelGGL((xdgrad_k<T, 2, 2, 16>), dim3(cdiv(a.Jp, 64), cdiv(g.Ci, 64)), dim3(kThreads), 0, st, a);
  }
  return hipGetLastError();
}

template <class T>
hipError_t implicit_t(const Geom& g, const void* x, const void* w, const void* g_y, float* g_w, void* g_x,
                      void* ws, hipStream_t st) {
  const XPlan p = make_plan<T>(g, g_w != nullptr, g_x != nullptr);
  char* wsb = static_cast<char*>(ws);
  hipError_t e = launch_prep<T>(g, p, wsb, w, g_x != nullptr, st);
  if (e != hipSuccess) return e;
  if (g_w) {
    e = wgrad_t<T>(g, p, x, g_y, g_w, wsb, st);
    if (e != hipSuccess) return e;
  }
  if (g_x) e = dgrad_t<T>(g, p, g_y, g_x, wsb, st);
  return e;
}

}  // namespace

// dense stride-1 layers with W_y == W, channel counts that are multiples of the vector length,
// a kernel larger than 1 x 1 and every index (plus the largest tap offset) below 2^31
bool implicit_ok(const Geom& g) {
  const int ve = 16 / g.b;
  if (g.g != 1 || g.s != 1 || g.Wy != g.W || g.KK > 1024) return false;
  if (g.Ci % ve != 0 || g.Co % ve != 0) return false;
  const long lim = 2147483647L;
  const long hwp = hwp_of(g.H * g.W), hwyp = hwp_of(g.Hy * g.Wy);
  const long reach = max_shift(g) + 1024;
  const long tx = (long)g.N * g.Ci * g.H * g.W, ty = (long)g.N * g.Co * g.Hy * g.Wy;
  if (tx < ve || ty < ve) return false;
  if (tx + reach + hwp >= lim || ty + reach + hwyp >= lim) return false;
  if ((long)g.N * hwp + 1024 >= lim || (long)g.N * hwyp + 1024 >= lim) return false;
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
