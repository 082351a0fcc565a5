// Dense-channel (groups == 1) contractions of the filtered backward on the MFMA
// matrix cores of gfx950:
//
//   weight gradient (Eq. 5):  g_th~[co, ci] = sum_j gy_u[co, j] * x_u[ci, j],   j = (n, patch)
//   input gradient  (Eq. 3):  g_x~u[ci, j]  = sum_co wsum[co, ci] * gy_u[co, j]
//
// Both are skinny, bandwidth-bound GEMMs, so the kernels are built around
// 128-byte coalesced row segments staged through LDS and register-prefetched one
// K chunk ahead; the tile shapes are picked on the host for 64-wide wavefronts
// (16x16 MFMA tiles, TM x TN of them per wave, WM x WN waves per 256-lane block).
//
// bf16 uses v_mfma_f32_16x16x32_bf16 (8 k-values per lane), fp32 uses
// v_mfma_f32_16x16x4_f32 (1 k-value per lane).  In the weight gradient both
// operands are K-contiguous in memory and go to LDS as they are.  In the input
// gradient both are K-strided; fp32 still needs no reshuffle (one value per lane)
// while bf16 rows are interleaved in k-pairs on the way into LDS so that a lane
// picks up its 8 k-values with four 32-bit reads.
#include "gf_internal.h"
#include "gf_mma.h"

namespace gf {

namespace {

constexpr int kThreads = 256;
constexpr int kRowBytes = 128 + 16;  // one staged row: 128 data bytes + 16 pad (K-major tiles)

template <class T> __device__ __forceinline__ uint32_t bits_of(T v);
template <> __device__ __forceinline__ uint32_t bits_of<float>(float v) { return __float_as_uint(v); }
template <> __device__ __forceinline__ uint32_t bits_of<bf16_t>(bf16_t v) {
  return (uint32_t)__builtin_bit_cast(uint16_t, v);
}

// 16 bytes (VE elements) of row `base` starting at flat column j = (n, p), where a
// row of image n starts at base + n * img_stride.  Zero beyond jtot.
template <class T, bool VEC>
__device__ __forceinline__ uint4 load_cols(const T* base, long img_stride, int j, int jtot, int P,
                                           const FastDiv& d_p) {
  constexpr int VE = Mma<T>::VE;
  if (VEC) {  // unconditional load of a clamped column (keeps a lane's loads in flight together)
    const int jc = min(j, jtot - VE);
    const int n = (int)d_p.div((uint32_t)jc);
    const int p = jc - n * P;
    const uint4 v = *reinterpret_cast<const uint4*>(base + (long)n * img_stride + p);
    return j < jtot ? v : make_uint4(0, 0, 0, 0);
  }
  if (P >= VE) {
    // Branch-free, with element-aligned 16-byte loads that are always issued (so that a lane's loads
    // stay in flight together): the part of the vector that lies in image n comes from a load
    // pulled back into that image and shifted; the part that lies in image n + 1 (only when the
    // vector crosses the boundary) from a load at the start of the next image, shifted the other
    // way; elements past jtot are cleared.
    const int jc = min(j, jtot - 1);
    const int n = (int)d_p.div((uint32_t)jc);
    const int p = jc - n * P;
    const int pa = min(p, P - VE);
    const int k1 = min(VE, P - p);                         // elements that belong to image n
    const int nlast = (int)d_p.div((uint32_t)(jtot - 1));  // last image this row holds columns of
    const uint4 va = load_vec<T>(base + (long)n * img_stride + pa);
    const uint4 vb = load_vec<T>(base + (long)min(n + 1, nlast) * img_stride);
    const uint4 a = realign<T>(va, p - pa);
    const uint4 b = realign<T>(vb, -k1);
    uint4 v = make_uint4(a.x | b.x, a.y | b.y, a.z | b.z, a.w | b.w);
    const int keep = jtot - j;                             // elements of the vector before jtot
    if (keep < VE) v = keep <= 0 ? make_uint4(0, 0, 0, 0) : realign<T>(realign<T>(v, -(VE - keep)), VE - keep);
    return v;
  }
  uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
  for (int e = 0; e < VE; ++e) {
    const int jj = j + e;
    if (jj < jtot) {
      const int n = (int)d_p.div((uint32_t)jj);
      const int p = jj - n * P;
      const uint32_t b = bits_of<T>(base[(long)n * img_stride + p]);
      if (sizeof(T) == 4) w[e & 3] = b; else w[e >> 1] |= b << ((e & 1) * 16);
    }
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// ---------------------------------------------------------------------------
// weight gradient: part[z, co, ci] = sum over the K chunks of slab z
// ---------------------------------------------------------------------------
struct WgradMfmaArgs {
  const void* gyu;
  const void* xu;
  float* part;
  int Ci, Co, P, Ktot;
  int nchunks, chunks_per_z;
  FastDiv d_p;
  // flat mode (P not a multiple of the vector length, P <= BK): a K chunk is G whole images,
  // the tile rows of one image are one contiguous, 16-byte aligned block that is loaded with
  // vectors and scattered to the [row][k] tile element by element
  int flat, G, N;
};

template <class T>
__device__ __forceinline__ uint32_t elem_bits(const uint4& v, int e) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  if (sizeof(T) == 4) return w[e & 3];
  return (w[e >> 1] >> ((e & 1) * 16)) & 0xffffu;
}

// vectors of the image blocks [rows r0 .. r0+ROWS) x P of images kc*G .. kc*G+G-1
template <class T, int ROWS, int NREG = ROWS / 32>
__device__ __forceinline__ void flat_fetch(uint4* rg, const T* base, int C, int r0, int kc, int P,
                                           int G, int N, int tid) {
  constexpr int VE = Mma<T>::VE;
  const int vpi = ROWS * P / VE;
  const int valid_vec = (min(ROWS, C - r0) * P + VE - 1) / VE;
#pragma unroll
  for (int i = 0; i < NREG; ++i) {
    const int s = tid + i * kThreads;
    const int g = s / vpi, vidx = s - g * vpi;
    const int n = kc * G + g;
    const bool ok = g < G && n < N && vidx < valid_vec;
    const uint4 v = *reinterpret_cast<const uint4*>(base + ((long)min(n, N - 1) * C + r0) * P +
                                                    (long)min(vidx, valid_vec - 1) * VE);
    rg[i] = ok ? v : make_uint4(0, 0, 0, 0);
  }
}

// scatter them into the K-major tile: element (row, p) of image g goes to k = g * P + p
template <class T, int ROWS>
__device__ __forceinline__ void flat_stage_kmajor(unsigned char* tile, const uint4* rg, int C, int r0,
                                                  int P, int G, const FastDiv& d_p, int tid) {
  constexpr int VE = Mma<T>::VE;
  const int vpi = ROWS * P / VE;
  const int valid = min(ROWS, C - r0) * P;
#pragma unroll
  for (int i = 0; i < ROWS / 32; ++i) {
    const int s = tid + i * kThreads;
    const int g = s / vpi, vidx = s - g * vpi;
    if (g >= G) continue;
    int f = vidx * VE;
    int row = (int)d_p.div((uint32_t)f);
    int p = f - row * P;
#pragma unroll
    for (int e = 0; e < VE; ++e) {
      if (f < valid) {
        unsigned char* d = tile + row * kRowBytes + (g * P + p) * (int)sizeof(T);
        if (sizeof(T) == 4) *reinterpret_cast<uint32_t*>(d) = elem_bits<T>(rg[i], e);
        else *reinterpret_cast<uint16_t*>(d) = (uint16_t)elem_bits<T>(rg[i], e);
      }
      ++f;
      if (++p == P) { p = 0; ++row; }
    }
  }
}

// scatter image blocks [ROWS k-rows x P] into the K-strided tile of the input-gradient GEMM:
// element (k, p) of image g goes to column g * P + p; fp32 one k per word row, bf16 a k-pair
// per word row.  Every position of the block is written (zeros past the valid rows), because
// the previous chunk may have left data there.
template <class T, int ROWS, int NREG, int STRIDE>
__device__ __forceinline__ void flat_stage_kstrided(uint32_t* tile, const uint4* rg, int C, int r0,
                                                    int P, int G, const FastDiv& d_p, int tid) {
  constexpr int VE = Mma<T>::VE;
  const int vpi = ROWS * P / VE;
  const int valid = min(ROWS, C - r0) * P;
#pragma unroll
  for (int i = 0; i < NREG; ++i) {
    const int s = tid + i * kThreads;
    const int g = s / vpi, vidx = s - g * vpi;
    if (g >= G) continue;
    int f = vidx * VE;
    int k = (int)d_p.div((uint32_t)f);
    int p = f - k * P;
#pragma unroll
    for (int e = 0; e < VE; ++e) {
      const uint32_t b = f < valid ? elem_bits<T>(rg[i], e) : 0u;
      const int col = g * P + p;
      if (sizeof(T) == 4) tile[k * STRIDE + col] = b;
      else reinterpret_cast<uint16_t*>(tile)[((k >> 1) * STRIDE + col) * 2 + (k & 1)] = (uint16_t)b;
      ++f;
      if (++p == P) { p = 0; ++k; }
    }
  }
}

// block (bx, by, bz) = (c_i tile, c_o tile, K slab); As / Bs: LDS tiles of BM resp. BN staged rows
template <class T, int TM, int TN, int WM, int WN, bool VEC>
__device__ __forceinline__ void wgrad_body(const WgradMfmaArgs& a, int bx, int by, int bz,
                                           unsigned char* As, unsigned char* Bs) {
  constexpr int BM = WM * TM * 16, BN = WN * TN * 16;
  constexpr int BK = Mma<T>::BK, VE = Mma<T>::VE, KSTEP = Mma<T>::KSTEP;
  constexpr int LA = BM / 32, LB = BN / 32;  // 16-byte loads per lane and chunk
  static_assert(WM * WN == 4 && BM % 32 == 0 && BN % 32 == 0, "tile shape");
  const T* gyu = static_cast<const T*>(a.gyu);
  const T* xu = static_cast<const T*>(a.xu);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int m0 = by * BM, n0 = bx * BN;
  const int kc0 = bz * a.chunks_per_z;
  const int kc1 = min(kc0 + a.chunks_per_z, a.nchunks);

  uint4 ra[LA], rb[LB];
  const bool flat = !VEC && a.flat;
  if (flat) {  // pad columns and rows past the channel count are never written: clear them once
    for (int i = tid; i < BM * kRowBytes / 4; i += kThreads) reinterpret_cast<uint32_t*>(As)[i] = 0u;
    for (int i = tid; i < BN * kRowBytes / 4; i += kThreads) reinterpret_cast<uint32_t*>(Bs)[i] = 0u;
    __syncthreads();
  }
  auto fetch = [&](int kc) {
    if (flat) {
      flat_fetch<T, BM>(ra, gyu, a.Co, m0, kc, a.P, a.G, a.N, tid);
      flat_fetch<T, BN>(rb, xu, a.Ci, n0, kc, a.P, a.G, a.N, tid);
      return;
    }
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const int s = tid + i * kThreads, row = s >> 3, vi = s & 7;
      const int co = m0 + row;
      const uint4 v = load_cols<T, VEC>(gyu + (long)min(co, a.Co - 1) * a.P, (long)a.Co * a.P,
                                        kc * BK + vi * VE, a.Ktot, a.P, a.d_p);
      ra[i] = co < a.Co ? v : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
      const int s = tid + i * kThreads, row = s >> 3, vi = s & 7;
      const int ci = n0 + row;
      const uint4 v = load_cols<T, VEC>(xu + (long)min(ci, a.Ci - 1) * a.P, (long)a.Ci * a.P,
                                        kc * BK + vi * VE, a.Ktot, a.P, a.d_p);
      rb[i] = ci < a.Ci ? v : make_uint4(0, 0, 0, 0);
    }
  };
  auto stage = [&]() {
    if (flat) {
      flat_stage_kmajor<T, BM>(As, ra, a.Co, m0, a.P, a.G, a.d_p, tid);
      flat_stage_kmajor<T, BN>(Bs, rb, a.Ci, n0, a.P, a.G, a.d_p, tid);
      return;
    }
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const int s = tid + i * kThreads;
      *reinterpret_cast<uint4*>(As + (s >> 3) * kRowBytes + (s & 7) * 16) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
      const int s = tid + i * kThreads;
      *reinterpret_cast<uint4*>(Bs + (s >> 3) * kRowBytes + (s & 7) * 16) = rb[i];
    }
  };

  f32x4 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  if (kc0 < kc1) fetch(kc0);
  for (int kc = kc0; kc < kc1; ++kc) {
    stage();
    __syncthreads();
    if (kc + 1 < kc1) fetch(kc + 1);
    const int r = lane & 15, kg = lane >> 4;
#pragma unroll
    for (int ks = 0; ks < BK / KSTEP; ++ks) {
      if constexpr (sizeof(T) == 2) {
        uint4 fa[TM], fb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
          fa[i] = *reinterpret_cast<const uint4*>(As + ((wm * TM + i) * 16 + r) * kRowBytes + ks * 64 + kg * 16);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          fb[j] = *reinterpret_cast<const uint4*>(Bs + ((wn * TN + j) * 16 + r) * kRowBytes + ks * 64 + kg * 16);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j] = mma16(fa[i], fb[j], acc[i][j]);
      } else {
        float fa[TM], fb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
          fa[i] = *reinterpret_cast<const float*>(As + ((wm * TM + i) * 16 + r) * kRowBytes + (ks * 4 + kg) * 4);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          fb[j] = *reinterpret_cast<const float*>(Bs + ((wn * TN + j) * 16 + r) * kRowBytes + (ks * 4 + kg) * 4);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j] = mma16(fa[i], fb[j], acc[i][j]);
      }
    }
    __syncthreads();
  }
  // D[i = 4 * (lane / 16) + v][j = lane % 16] of every 16 x 16 tile
  float* dst = a.part + (long)bz * a.Co * a.Ci;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int ci = n0 + (wn * TN + j) * 16 + (lane & 15);
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int co = m0 + (wm * TM + i) * 16 + 4 * (lane >> 4) + v;
        if (co < a.Co && ci < a.Ci) dst[(long)co * a.Ci + ci] = acc[i][j][v];
      }
    }
}

template <class T, int TM, int TN, int WM, int WN, bool VEC>
__global__ __launch_bounds__(kThreads) void wgrad_mfma_k(WgradMfmaArgs a) {
  constexpr int BM = WM * TM * 16, BN = WN * TN * 16;
  __shared__ __attribute__((aligned(16))) unsigned char As[BM * kRowBytes];
  __shared__ __attribute__((aligned(16))) unsigned char Bs[BN * kRowBytes];
  wgrad_body<T, TM, TN, WM, WN, VEC>(a, blockIdx.x, blockIdx.y, blockIdx.z, As, Bs);
}

// ---------------------------------------------------------------------------
// input gradient, reduced map: dst[n, ci, p] = scale * sum_co wt[co, ci] * gy_u[n, co, p]
// ---------------------------------------------------------------------------
struct DgradMfmaArgs {
  const void* gyu;
  const void* wt;   // [Co][Ci] in the storage type: the 1x1 kernel itself or the rounded kernel sum
  void* dst;        // [N, Ci, P] in the storage type
  const void* mask; // nullable, [N, Ci, P]: the reduced map is multiplied by it (rounded value times mask, rounded)
  int Ci, Co, P, Jtot;
  float scale;
  FastDiv d_p;
  // full-resolution store (Eq. 3 broadcast): every patch value goes to its rx x rx pixels
  void* full;       // [N, Ci, H, W], or null to write the reduced map to dst
  int H, W, Wp, rx;
  FastDiv d_wp;
  // plane mode (small or unaligned maps): a tile's columns are `ipt` whole images, so the
  // full-resolution output of a tile row range is one contiguous run of planes per image
  int planes_mode, ipt, cols_per_tile, rows_per_pass;
  // patch-row mode of the full-resolution store: a tile's columns are `prt` whole patch rows, so
  // the rx * prt pixel rows it produces for one c_i are one contiguous run of memory
  int prt;
  // operand loading when P is not a multiple of the vector length: veca = the kernel matrix can
  // still be read with vectors; flatb = gy_u is read as whole-image blocks (column tiles are
  // `ipt` whole images) and scattered into the tile
  int veca, flatb, N;
};

constexpr int kPlaneStageBytes = 16 * 1024;

// rows k (c_o) x columns mn, LDS tile of 32 word-rows: fp32 one k per row, bf16 a k-pair per row
template <class T, int BMN, bool VEC, int NT = kThreads, class RowPtr>
__device__ __forceinline__ void dgrad_fetch(uint4* rg, int tid, int k0, int Ktot, RowPtr&& load_row) {
  constexpr int VE = Mma<T>::VE;
  constexpr int VPR = BMN / VE;                      // vectors per k row
  constexpr int ROWS_PER_SLOT = sizeof(T) == 2 ? 2 : 1;
  constexpr int SLOTS = 32 * VPR;                    // 32 word-rows
  constexpr int PER = (SLOTS + NT - 1) / NT;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int s = tid + i * NT;
    if (SLOTS % NT != 0 && s >= SLOTS) break;
    const int wr = s / VPR, vi = s - wr * VPR;
#pragma unroll
    for (int q = 0; q < ROWS_PER_SLOT; ++q) {
      const int k = k0 + wr * ROWS_PER_SLOT + q;
      const uint4 v = load_row(min(k, Ktot - 1), vi * VE);
      rg[i * ROWS_PER_SLOT + q] = k < Ktot ? v : make_uint4(0, 0, 0, 0);
    }
  }
}

template <class T, int BMN, int STRIDE, int NT = kThreads>
__device__ __forceinline__ void dgrad_stage(uint32_t* tile, const uint4* rg, int tid) {
  constexpr int VE = Mma<T>::VE;
  constexpr int VPR = BMN / VE;
  constexpr int SLOTS = 32 * VPR;
  constexpr int PER = (SLOTS + NT - 1) / NT;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int s = tid + i * NT;
    if (SLOTS % NT != 0 && s >= SLOTS) break;
    const int wr = s / VPR, vi = s - wr * VPR;
    uint32_t* d = tile + wr * STRIDE + vi * VE;
    if constexpr (sizeof(T) == 4) {
      *reinterpret_cast<uint4*>(d) = rg[i];
    } else {
      const uint4 lo = rg[2 * i], hi = rg[2 * i + 1];  // rows k and k + 1, eight columns each
      uint4 o0, o1;                                    // word c = (row k col c) | (row k+1 col c) << 16
      o0.x = (lo.x & 0xffffu) | (hi.x << 16); o0.y = (lo.x >> 16) | (hi.x & 0xffff0000u);
      o0.z = (lo.y & 0xffffu) | (hi.y << 16); o0.w = (lo.y >> 16) | (hi.y & 0xffff0000u);
      o1.x = (lo.z & 0xffffu) | (hi.z << 16); o1.y = (lo.z >> 16) | (hi.z & 0xffff0000u);
      o1.z = (lo.w & 0xffffu) | (hi.w << 16); o1.w = (lo.w >> 16) | (hi.w & 0xffff0000u);
      *reinterpret_cast<uint4*>(d) = o0;
      *reinterpret_cast<uint4*>(d + 4) = o1;
    }
  }
}

// LDS words the input-gradient block needs for its operand tiles / output tile
template <class T, int BM, int BN>
constexpr int dgrad_smem_words() {
  constexpr int SC = BN + 16 / (int)sizeof(T);
  constexpr int tile = 32 * (BM + 4 + BN + 4);
  constexpr int out = (BM * SC * (int)sizeof(T) + 3) / 4;
  return tile > out ? tile : out;
}

template <class T, int BM, int BN, bool VEC>
__device__ __forceinline__ void dgrad_epilogue(const DgradMfmaArgs& a, const T* Cs, unsigned char* Es,
                                               int bx, int m0, int j0, int jend, int tid);

// block (bx, by) = (column tile, c_i tile); smem: dgrad_smem_words() words; Es: plane staging
// buffer (only touched in plane mode)
template <class T, int TM, int TN, int WM, int WN, bool VEC>
__device__ __forceinline__ void dgrad_body(const DgradMfmaArgs& a, int bx, int by, uint32_t* smem,
                                           unsigned char* Es) {
  constexpr int BM = WM * TM * 16, BN = WN * TN * 16;
  constexpr int BK = Mma<T>::BK, VE = Mma<T>::VE;
  constexpr int SA = BM + 4, SB = BN + 4;  // word strides of the two tiles (multiples of 4)
  constexpr int RPS = sizeof(T) == 2 ? 2 : 1;
  constexpr int PA = (32 * BM / VE + kThreads - 1) / kThreads * RPS;
  constexpr int PB = (32 * BN / VE + kThreads - 1) / kThreads * RPS;
  constexpr int SC = BN + 16 / (int)sizeof(T);  // element stride of the output staging tile
  uint32_t* As = smem;
  uint32_t* Bs = smem + 32 * SA;
  const T* gyu = static_cast<const T*>(a.gyu);
  const T* wt = static_cast<const T*>(a.wt);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int m0 = by * BM;  // first c_i
  const int j0 = bx * a.cols_per_tile;  // first flat column (n, p)
  const int jend = min(a.Jtot, j0 + a.cols_per_tile);

  auto load_a = [&](int k, int col) -> uint4 {  // wt[k][m0 + col ..]
    const int ci = m0 + col;
    if (VEC || a.veca) {
      const uint4 v = *reinterpret_cast<const uint4*>(wt + (long)k * a.Ci + min(ci, a.Ci - VE));
      return ci < a.Ci ? v : make_uint4(0, 0, 0, 0);
    }
    uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
    for (int e = 0; e < VE; ++e)
      if (ci + e < a.Ci) {
        const uint32_t b = bits_of<T>(wt[(long)k * a.Ci + ci + e]);
        if (sizeof(T) == 4) w[e & 3] = b; else w[e >> 1] |= b << ((e & 1) * 16);
      }
    return make_uint4(w[0], w[1], w[2], w[3]);
  };
  auto load_b = [&](int k, int col) -> uint4 {  // gy_u[n, k, p] for flat column j0 + col
    return load_cols<T, VEC>(gyu + (long)k * a.P, (long)a.Co * a.P, j0 + col, jend, a.P, a.d_p);
  };

  f32x4 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  uint4 ra[PA], rb[PB];
  const bool flatb = !VEC && a.flatb;
  if (flatb) {  // columns past the tile's images are never written: clear the tile once
    for (int i = tid; i < 32 * SB; i += kThreads) Bs[i] = 0u;
    __syncthreads();
  }
  auto fetch_b = [&](int k0) {
    if (flatb) flat_fetch<T, BK, PB>(rb, gyu, a.Co, k0, bx, a.P, a.ipt, a.N, tid);
    else dgrad_fetch<T, BN, VEC>(rb, tid, k0, a.Co, load_b);
  };
  dgrad_fetch<T, BM, VEC>(ra, tid, 0, a.Co, load_a);
  fetch_b(0);
  const int r = lane & 15, kg = lane >> 4;
  for (int k0 = 0; k0 < a.Co; k0 += BK) {
    dgrad_stage<T, BM, SA>(As, ra, tid);
    if (flatb) flat_stage_kstrided<T, BK, PB, SB>(Bs, rb, a.Co, k0, a.P, a.ipt, a.d_p, tid);
    else dgrad_stage<T, BN, SB>(Bs, rb, tid);
    __syncthreads();
    if (k0 + BK < a.Co) {
      dgrad_fetch<T, BM, VEC>(ra, tid, k0 + BK, a.Co, load_a);
      fetch_b(k0 + BK);
    }
    if constexpr (sizeof(T) == 2) {
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {  // 32 k = 16 pair rows per MFMA
        uint4 fa[TM], fb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const uint32_t* p = As + (ks * 16 + kg * 4) * SA + (wm * TM + i) * 16 + r;
          fa[i] = make_uint4(p[0], p[SA], p[2 * SA], p[3 * SA]);
        }
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
      for (int ks = 0; ks < 8; ++ks) {  // 4 k per MFMA
        float fa[TM], fb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[i] = __uint_as_float(As[(ks * 4 + kg) * SA + (wm * TM + i) * 16 + r]);
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
  // stage the output tile in LDS (rounded once), then store 16-byte runs along j
  T* Cs = reinterpret_cast<T*>(smem);
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = (wm * TM + i) * 16 + 4 * (lane >> 4) + v;
        const int col = (wn * TN + j) * 16 + (lane & 15);
        Cs[row * SC + col] = from_f32<T>(acc[i][j][v] * a.scale);
      }
  __syncthreads();
  dgrad_epilogue<T, BM, BN, VEC>(a, Cs, Es, bx, m0, j0, jend, tid);
}

template <class T, int TM, int TN, int WM, int WN, bool VEC>
__global__ __launch_bounds__(kThreads) void dgrad_mfma_k(DgradMfmaArgs a) {
  constexpr int BM = WM * TM * 16, BN = WN * TN * 16;
  __shared__ __attribute__((aligned(16))) uint32_t smem[dgrad_smem_words<T, BM, BN>()];
  __shared__ __attribute__((aligned(16))) unsigned char Es[kPlaneStageBytes];
  dgrad_body<T, TM, TN, WM, WN, VEC>(a, blockIdx.x, blockIdx.y, smem, Es);
}

// Store the finished tile Cs[BM][SC] (already rounded to the storage type): as the reduced map,
// as 16-byte pixel runs at full resolution, or plane by plane through the LDS image Es.
template <class T, int BM, int BN, bool VEC>
__device__ __forceinline__ void dgrad_epilogue(const DgradMfmaArgs& a, const T* Cs, unsigned char* Es,
                                               int bx, int m0, int j0, int jend, int tid) {
  constexpr int VE = Mma<T>::VE;
  constexpr int SC = BN + 16 / (int)sizeof(T);
  if (a.planes_mode) {
    // Every image of the tile, `rows_per_pass` channel rows at a time: replicate the patch
    // values into an LDS image of the output run (rows are consecutive planes, so the run is
    // contiguous in memory), then store it with 16-byte vectors; the partial vectors at both
    // ends, which neighbouring tiles share, go out element by element.
    T* out = static_cast<T*>(a.full);
    const int HW = a.H * a.W, rx = a.rx;
    const int n0 = bx * a.ipt;
    const int nimg = (jend - j0) / a.P;
    const int rows_valid = min(BM, a.Ci - m0);
    for (int il = 0; il < nimg; ++il)
      for (int r0 = 0; r0 < rows_valid; r0 += a.rows_per_pass) {
        const int nr = min(a.rows_per_pass, rows_valid - r0);
        const long e0 = (((long)(n0 + il) * a.Ci + m0 + r0)) * HW;   // first element of the run
        const long byte0 = e0 * (long)sizeof(T);
        const long a0 = byte0 & ~15L;
        const int shift = (int)(byte0 - a0);
        const int span = shift + nr * HW * (int)sizeof(T);
        T* img = reinterpret_cast<T*>(Es + shift);
        for (int it = tid; it < nr * a.P; it += kThreads) {
          const int rl = (int)a.d_p.div((uint32_t)it);
          const int pp = it - rl * a.P;
          const int hp = (int)a.d_wp.div((uint32_t)pp);
          const int wp = pp - hp * a.Wp;
          const T val = Cs[(r0 + rl) * SC + il * a.P + pp];
          const int h1 = min(a.H, (hp + 1) * rx), w1 = min(a.W, (wp + 1) * rx);
          for (int h = hp * rx; h < h1; ++h)
            for (int ww = wp * rx; ww < w1; ++ww) img[rl * HW + h * a.W + ww] = val;
        }
        __syncthreads();
        const int nvec = span >> 4;
        unsigned char* dstb = reinterpret_cast<unsigned char*>(out) + a0;
        for (int v = tid + (shift ? 1 : 0); v < nvec; v += kThreads)
          *reinterpret_cast<uint4*>(dstb + ((long)v << 4)) = *reinterpret_cast<const uint4*>(Es + (v << 4));
        if (shift) {
          const int nhead = min((16 - shift) / (int)sizeof(T), nr * HW);
          if (tid < nhead) out[e0 + tid] = img[tid];
        }
        {
          const int tail0 = nvec << 4;
          const int ntail = (span - tail0) / (int)sizeof(T);
          const int efirst = (tail0 - shift) / (int)sizeof(T);
          if (tid < ntail && efirst + tid >= 0) out[e0 + efirst + tid] = img[efirst + tid];
        }
        __syncthreads();
      }
    return;
  }
  if (a.full && a.prt > 0) {
    // lane = one 16-byte vector of the contiguous run (prt patch rows x rx pixel rows x W pixels)
    // that a c_i row of the tile owns; consecutive lanes store consecutive vectors, `rpp` rows
    // of c_i per pass.  (host: W == Wp * rx, W % VE == 0, rx a power of two, ipr <= kThreads)
    T* out = static_cast<T*>(a.full);
    const int rx = a.rx, sh = 31 - __builtin_clz(rx);
    const int vpr = a.W / VE;                 // vectors per pixel row
    const int ipr = a.prt * rx * vpr;         // vectors per c_i row of the tile
    const int rpp = kThreads / ipr;
    const int rl = tid / ipr, slot = tid - rl * ipr;
    const int pr = slot / (rx * vpr), rem = slot - pr * rx * vpr;
    const int i = rem / vpr, vv = rem - i * vpr;
    const int gr = bx * a.prt + pr;           // patch row counted over the whole batch
    const int Hp = a.P / a.Wp;
    const int n = gr / Hp, hp = gr - n * Hp;
    const int h = hp * rx + i;
    if (rl >= rpp || pr * a.Wp >= jend - j0 || h >= a.H) return;
    const T* src = Cs + pr * a.Wp;
    T* d = out + (((long)n * a.Ci + m0) * a.H + h) * a.W + vv * VE;
    const int rows_valid = min(BM, a.Ci - m0);
    for (int row = rl; row < rows_valid; row += rpp) {
      T vals[VE];
#pragma unroll
      for (int e = 0; e < VE; ++e) vals[e] = src[row * SC + ((vv * VE + e) >> sh)];
      store_stream16(d + (long)row * a.H * a.W, *reinterpret_cast<const uint4*>(vals));
    }
    return;
  }
  if (a.full) {
    // one item = (row ci, one 16-byte run of output pixels): the few patch values the run needs
    // are read from LDS once and the same vector is stored to the rx pixel rows of the patch row
    // (host guarantees rx | VE or VE | rx, W == Wp * rx, W % VE == 0, Wp * rx % VE == 0)
    T* out = static_cast<T*>(a.full);
    const int rx = a.rx;
    const int vprow = BN * rx / VE;          // vectors per tile row
    const int vshift = 31 - __builtin_clz(vprow);  // BN, rx, VE are powers of two
    for (int s = tid; s < BM * vprow; s += kThreads) {
      const int row = s >> vshift;
      const int ov = s & (vprow - 1);
      const int q0 = ov * VE;                // first output pixel of the run, tile-relative
      const int col = q0 / rx;               // first patch column of the run
      const int ci = m0 + row, j = j0 + col;
      if (ci >= a.Ci || j >= jend) continue;
      const int n = (int)a.d_p.div((uint32_t)j);
      const int p = j - n * a.P;
      const int hp = (int)a.d_wp.div((uint32_t)p);
      const int wp = p - hp * a.Wp;
      T vals[VE];
      const T* src = Cs + row * SC + col;
      if (rx >= VE) {
#pragma unroll
        for (int e = 0; e < VE; ++e) vals[e] = src[0];
      } else {
#pragma unroll
        for (int e = 0; e < VE; ++e) vals[e] = src[e / rx];
      }
      const uint4 vec = *reinterpret_cast<const uint4*>(vals);
      const int h0 = hp * rx;
      const int nrows = min(rx, a.H - h0);
      T* d = out + (((long)n * a.Ci + ci) * a.H + h0) * a.W + wp * rx + (q0 - col * rx);
      for (int i = 0; i < nrows; ++i) *reinterpret_cast<uint4*>(d + (long)i * a.W) = vec;
    }
    return;
  }
  T* dst = static_cast<T*>(a.dst);
  constexpr int VPR = BN / VE;
  for (int s = tid; s < BM * VPR; s += kThreads) {
    const int row = s / VPR, vi = s - row * VPR;
    const int ci = m0 + row, j = j0 + vi * VE;
    if (ci >= a.Ci || j >= jend) continue;
    const T* mask = static_cast<const T*>(a.mask);
    if (VEC) {
      const int n = (int)a.d_p.div((uint32_t)j);
      const int p = j - n * a.P;
      const long o = ((long)n * a.Ci + ci) * a.P + p;
      uint4 v = *reinterpret_cast<const uint4*>(Cs + row * SC + vi * VE);
      if (mask) {
        float f[VE], m[VE];
        Vec16<T>::unpack(v, f);
        Vec16<T>::unpack(*reinterpret_cast<const uint4*>(mask + o), m);
#pragma unroll
        for (int e = 0; e < VE; ++e) f[e] *= m[e];
        v = Vec16<T>::pack(f);
      }
      *reinterpret_cast<uint4*>(dst + o) = v;
    } else {
      for (int e = 0; e < VE && j + e < jend; ++e) {
        const int n = (int)a.d_p.div((uint32_t)(j + e));
        const int p = j + e - n * a.P;
        const long o = ((long)n * a.Ci + ci) * a.P + p;
        T v = Cs[row * SC + vi * VE + e];
        if (mask) v = from_f32<T>(to_f32(v) * to_f32(mask[o]));
        dst[o] = v;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Same contraction for layers whose GEMM has few output tiles but a long K = C_y (small maps,
// many channels): a 32 x BN tile per block, and the four waves split K among themselves.
// Each wave stages its own chunks in a private LDS tile (no block barrier inside the K loop),
// the four accumulators are added in fixed order through LDS at the end.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int BN>
constexpr int ksplit_smem_words() { return 4 * 32 * (32 + 4 + BN + 4); }

// block (bx, by) = (column tile, 32-row c_i tile); smem: ksplit_smem_words<BN>() words
template <class T, int BN, bool VEC>
__device__ __forceinline__ void dgrad_ksplit_body(const DgradMfmaArgs& a, int bx, int by, uint32_t* smem,
                                                  unsigned char* Es) {
  constexpr int BM = 32, TM = 2, TN = BN / 16;
  constexpr int BK = Mma<T>::BK, VE = Mma<T>::VE;
  constexpr int SA = BM + 4, SB = BN + 4;
  constexpr int RPS = sizeof(T) == 2 ? 2 : 1;
  constexpr int PA = (32 * BM / VE + 63) / 64 * RPS;
  constexpr int PB = (32 * BN / VE + 63) / 64 * RPS;
  constexpr int SC = BN + 16 / (int)sizeof(T);
  constexpr int kWaveWords = 32 * (SA + SB);
  constexpr int kSumWords = 4 * BM * BN;                       // the four fp32 accumulator tiles
  constexpr int kOutWords = (BM * SC * (int)sizeof(T) + 3) / 4;
  static_assert(kSumWords + kOutWords <= 4 * kWaveWords, "reduction buffers fit the staging tiles");
  static_assert(4 * kWaveWords == ksplit_smem_words<BN>(), "smem size");
  const T* gyu = static_cast<const T*>(a.gyu);
  const T* wt = static_cast<const T*>(a.wt);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint32_t* As = smem + wave * kWaveWords;
  uint32_t* Bs = As + 32 * SA;
  const int m0 = by * BM;
  const int j0 = bx * a.cols_per_tile;
  const int jend = min(a.Jtot, j0 + a.cols_per_tile);

  auto load_a = [&](int k, int col) -> uint4 {
    const int ci = m0 + col;
    if (VEC) {
      const uint4 v = *reinterpret_cast<const uint4*>(wt + (long)k * a.Ci + min(ci, a.Ci - VE));
      return ci < a.Ci ? v : make_uint4(0, 0, 0, 0);
    }
    uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
    for (int e = 0; e < VE; ++e)
      if (ci + e < a.Ci) {
        const uint32_t b = bits_of<T>(wt[(long)k * a.Ci + ci + e]);
        if (sizeof(T) == 4) w[e & 3] = b; else w[e >> 1] |= b << ((e & 1) * 16);
      }
    return make_uint4(w[0], w[1], w[2], w[3]);
  };
  auto load_b = [&](int k, int col) -> uint4 {
    return load_cols<T, VEC>(gyu + (long)k * a.P, (long)a.Co * a.P, j0 + col, jend, a.P, a.d_p);
  };

  f32x4 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // this wave's K range, whole chunks
  const int nch = (a.Co + BK - 1) / BK;
  const int cpw = (nch + 3) / 4;
  const int kbeg = min(a.Co, wave * cpw * BK);
  const int kend = min(a.Co, kbeg + cpw * BK);
  uint4 ra[PA], rb[PB];
  if (kbeg < kend) {
    dgrad_fetch<T, BM, VEC, 64>(ra, lane, kbeg, kend, load_a);
    dgrad_fetch<T, BN, VEC, 64>(rb, lane, kbeg, kend, load_b);
  }
  const int r = lane & 15, kg = lane >> 4;
  for (int k0 = kbeg; k0 < kend; k0 += BK) {
    dgrad_stage<T, BM, SA, 64>(As, ra, lane);
    dgrad_stage<T, BN, SB, 64>(Bs, rb, lane);
    wave_sync();
    if (k0 + BK < kend) {
      dgrad_fetch<T, BM, VEC, 64>(ra, lane, k0 + BK, kend, load_a);
      dgrad_fetch<T, BN, VEC, 64>(rb, lane, k0 + BK, kend, load_b);
    }
    if constexpr (sizeof(T) == 2) {
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        uint4 fa[TM], fb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const uint32_t* p = As + (ks * 16 + kg * 4) * SA + i * 16 + r;
          fa[i] = make_uint4(p[0], p[SA], p[2 * SA], p[3 * SA]);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const uint32_t* p = Bs + (ks * 16 + kg * 4) * SB + j * 16 + r;
          fb[j] = make_uint4(p[0], p[SB], p[2 * SB], p[3 * SB]);
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j] = mma16(fa[i], fb[j], acc[i][j]);
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        float fa[TM], fb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[i] = __uint_as_float(As[(ks * 4 + kg) * SA + i * 16 + r]);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[j] = __uint_as_float(Bs[(ks * 4 + kg) * SB + j * 16 + r]);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j] = mma16(fa[i], fb[j], acc[i][j]);
      }
    }
    wave_sync();
  }
  __syncthreads();  // every wave is done with its staging tile: reuse the memory
  float* Rs = reinterpret_cast<float*>(smem);               // [4][BM][BN]
  T* Cs = reinterpret_cast<T*>(smem + kSumWords);           // [BM][SC]
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        Rs[(wave * BM + i * 16 + 4 * kg + v) * BN + j * 16 + r] = acc[i][j][v];
  __syncthreads();
  for (int e = tid; e < BM * BN; e += kThreads) {
    const float s = ((Rs[e] + Rs[BM * BN + e]) + Rs[2 * BM * BN + e]) + Rs[3 * BM * BN + e];
    Cs[(e / BN) * SC + (e % BN)] = from_f32<T>(s * a.scale);
  }
  __syncthreads();
  dgrad_epilogue<T, BM, BN, VEC>(a, Cs, Es, bx, m0, j0, jend, tid);
}

template <class T, int BN, bool VEC>
__global__ __launch_bounds__(kThreads) void dgrad_ksplit_k(DgradMfmaArgs a) {
  __shared__ __attribute__((aligned(16))) uint32_t smem[ksplit_smem_words<BN>()];
  __shared__ __attribute__((aligned(16))) unsigned char Es[kPlaneStageBytes];
  dgrad_ksplit_body<T, BN, VEC>(a, blockIdx.x, blockIdx.y, smem, Es);
}

// ---------------------------------------------------------------------------
// Weight and input gradient of one layer in ONE launch: both only depend on gy_u, so the
// first `nw` blocks of the grid run weight-gradient tiles and the rest input-gradient tiles.
// The short, latency-bound K loops of the former overlap with the store-bound epilogues of
// the latter, and one launch ramp is saved.
// ---------------------------------------------------------------------------
struct S3S4Grid {
  int nw, wgx, wgy, dgx;
};

// VEC: vector loads of every operand (else the image-block loaders); PLANES: the input
// gradient stores whole planes through the LDS staging buffer (small / unaligned maps)
template <class T, int WTM, int WTN, int WWM, int WWN, int DTM, int DTN, int DWM, int DWN, bool VEC,
          bool PLANES>
__global__ __launch_bounds__(kThreads) void s3s4_mfma_k(WgradMfmaArgs wa, DgradMfmaArgs da, S3S4Grid g) {
  constexpr int WBM = WWM * WTM * 16, WBN = WWN * WTN * 16;
  constexpr int DBM = DWM * DTM * 16, DBN = DWN * DTN * 16;
  constexpr int kWBytes = (WBM + WBN) * kRowBytes;
  constexpr int kDBytes = dgrad_smem_words<T, DBM, DBN>() * 4;
  __shared__ __attribute__((aligned(16))) unsigned char smem[kWBytes > kDBytes ? kWBytes : kDBytes];
  __shared__ __attribute__((aligned(16))) unsigned char Es[PLANES ? kPlaneStageBytes : 16];
  const int b = blockIdx.x;
  if (b < g.nw) {
    const int bx = b % g.wgx;
    const int t = b / g.wgx;
    wgrad_body<T, WTM, WTN, WWM, WWN, VEC>(wa, bx, t % g.wgy, t / g.wgy, smem, smem + WBM * kRowBytes);
  } else {
    const int q = b - g.nw;
    dgrad_body<T, DTM, DTN, DWM, DWN, VEC>(da, q % g.dgx, q / g.dgx, reinterpret_cast<uint32_t*>(smem), Es);
  }
}

// the same with the K-split input-gradient block
template <class T, int WTM, int WTN, int WWM, int WWN, int BN>
__global__ __launch_bounds__(kThreads) void s3s4_ksplit_k(WgradMfmaArgs wa, DgradMfmaArgs da, S3S4Grid g) {
  constexpr int WBM = WWM * WTM * 16, WBN = WWN * WTN * 16;
  constexpr int kWBytes = (WBM + WBN) * kRowBytes;
  constexpr int kDBytes = ksplit_smem_words<BN>() * 4;
  __shared__ __attribute__((aligned(16))) unsigned char smem[kWBytes > kDBytes ? kWBytes : kDBytes];
  __shared__ __attribute__((aligned(16))) unsigned char Es[kPlaneStageBytes];
  const int b = blockIdx.x;
  if (b < g.nw) {
    const int bx = b % g.wgx;
    const int t = b / g.wgx;
    wgrad_body<T, WTM, WTN, WWM, WWN, true>(wa, bx, t % g.wgy, t / g.wgy, smem, smem + WBM * kRowBytes);
  } else {
    const int q = b - g.nw;
    dgrad_ksplit_body<T, BN, true>(da, q % g.dgx, q / g.dgx, reinterpret_cast<uint32_t*>(smem), Es);
  }
}

// kernel sum rounded to the storage type, [Co][Ci] (text after Eq. 3)
template <class T>
__global__ __launch_bounds__(kThreads) void kernel_sum_t_k(const T* w, T* wsum, int pairs, int KK) {
  const int e = blockIdx.x * kThreads + threadIdx.x;
  if (e >= pairs) return;
  wsum[e] = from_f32<T>(kernel_sum_of(w, e, KK));
}

template <class T, int TM, int TN, int WM, int WN>
hipError_t wgrad_launch(WgradMfmaArgs& a, int nz, bool vec, hipStream_t st) {
  constexpr int BM = WM * TM * 16, BN = WN * TN * 16;
  dim3 grid(cdiv(a.Ci, BN), cdiv(a.Co, BM), nz);
  if (vec)
    GF_LAUNCH((wgrad_mfma_k<T, TM, TN, WM, WN, true>), grid, dim3(kThreads), 0, st, a);
  else
    GF_LAUNCH((wgrad_mfma_k<T, TM, TN, WM, WN, false>), grid, dim3(kThreads), 0, st, a);
  return hipGetLastError();
}

// Column tiles of the input-gradient GEMM when neither whole images nor image blocks are used:
// whole patch rows if the full-resolution store can use them (see DgradMfmaArgs::prt), else BN.
template <class T>
void dgrad_column_tiles(DgradMfmaArgs& a, int BN, int BM) {
  constexpr int VE = Mma<T>::VE;
  a.prt = 0;
  a.cols_per_tile = BN;
  if (!a.full || a.Wp > BN) return;
  const int per_patch_row = a.rx * (a.W / VE);   // vectors of one patch row of one c_i
  if (per_patch_row > kThreads) return;
  int prt = BN / a.Wp;
  if (prt > kThreads / per_patch_row) prt = kThreads / per_patch_row;
  // small problems: rather more, narrower tiles than a chip that is mostly idle
  const long patch_rows = (long)a.Jtot / a.Wp;
  const long want = patch_rows * cdiv(a.Ci, BM) / 128;
  if (want < prt) prt = want < 1 ? 1 : (int)want;
  int up = prt;   // tiles start on vector boundaries of gy_u: the nearest count of patch rows that does
  while (up <= BN / a.Wp && up <= kThreads / per_patch_row && (up * a.Wp) % VE != 0) ++up;
  if (up <= BN / a.Wp && up <= kThreads / per_patch_row) prt = up;
  else
    while (prt > 0 && (prt * a.Wp) % VE != 0) --prt;
  if (prt < 1) return;
  a.prt = prt;
  a.cols_per_tile = prt * a.Wp;
}

template <class T, int TM, int TN, int WM, int WN>
hipError_t dgrad_launch(DgradMfmaArgs& a, bool vec, hipStream_t st) {
  constexpr int BM = WM * TM * 16, BN = WN * TN * 16;
  if (!a.planes_mode && !a.flatb) dgrad_column_tiles<T>(a, BN, BM);
  dim3 grid(cdiv(a.Jtot, a.cols_per_tile), cdiv(a.Ci, BM), 1);
  if (vec)
    GF_LAUNCH((dgrad_mfma_k<T, TM, TN, WM, WN, true>), grid, dim3(kThreads), 0, st, a);
  else
    GF_LAUNCH((dgrad_mfma_k<T, TM, TN, WM, WN, false>), grid, dim3(kThreads), 0, st, a);
  return hipGetLastError();
}

// tile shape of the weight-gradient GEMM: 0 = 64x64, 1 = 128 (co) x 32 (ci), 2 = 32 x 128,
// 4 = 256 x 64.  The last one is for a second operand too large for the caches (the column
// tensors of exact BP): every row tile re-reads it from HBM, so all 256 rows go into one tile.
// (A 128 x 128 tile with 4 x 4 MFMA tiles per wave was measured no faster than 64 x 64.)
constexpr long kHugeOperandBytes = 96L << 20;

int wgrad_shape(const Geom& g) {
  if (g.Ci <= 32 && g.Co > 64) return 1;
  if (g.Co <= 32 && g.Ci > 64) return 2;
  if (g.Co >= 256 && g.Ci >= 256 && g.P % (16 / g.b) == 0 &&
      (long)g.N * g.P * g.Ci * g.b >= kHugeOperandBytes)
    return 4;
  return 0;
}

void wgrad_tile(int shape, int* bm, int* bn) {
  *bm = shape == 1 ? 128 : shape == 2 ? 32 : shape == 4 ? 256 : 64;
  *bn = shape == 1 ? 32 : shape == 2 ? 128 : 64;
}

}  // namespace

// flat mode of the weight-gradient GEMM (see WgradMfmaArgs): G images per K chunk
bool wgrad_flat(const Geom& g, int* G) {
  const int VE = 16 / g.b, BK = g.dtype == GF_BF16 ? 64 : 32;
  if (g.P % VE == 0 || g.P > BK) return false;
  if (((long)g.Co * g.P * g.b) % 16 != 0 || ((long)g.Ci * g.P * g.b) % 16 != 0) return false;
  if (G) *G = BK / g.P;
  return true;
}

int wgrad_chunks(const Geom& g) {
  int G = 1;
  if (wgrad_flat(g, &G)) return cdiv(g.N, G);
  return cdiv((long)g.N * g.P, g.dtype == GF_BF16 ? 64 : 32);
}

// K slabs of the weight-gradient GEMM: enough for ~1024 blocks, but at least four staged
// chunks per block so that the partial slabs stay small next to the operands (measured:
// one chunk per block is slower on the 144 x 24 x 25088 and 512 x 512 x 1024 problems).
int mfma_wgrad_splits(const Geom& g, int* chunks_per_z) {
  const int nchunks = wgrad_chunks(g);
  if (plain_wgrad_ok(g)) {
    if (chunks_per_z) *chunks_per_z = 0;
    return plain_wgrad_splits(g);
  }
  int bm, bn;
  wgrad_tile(wgrad_shape(g), &bm, &bn);
  const int tiles = cdiv(g.Co, bm) * cdiv(g.Ci, bn);
  int nz = cdiv(1024, tiles);
  if (nz > cdiv(nchunks, 4)) nz = cdiv(nchunks, 4);
  // ... unless that leaves most of the chip idle (short K, few tiles): then fewer chunks per block
  const int fill = cdiv(256, tiles);
  if (nz < fill) nz = fill < nchunks ? fill : nchunks;
  if (nz < 1) nz = 1;
  const int cpz = cdiv(nchunks, nz);
  if (chunks_per_z) *chunks_per_z = cpz;
  return cdiv(nchunks, cpz);
}

template <class T>
static hipError_t wgrad_t(const Geom& g, const void* x_u, const void* gy_u, float* part, int* nz_out,
                          hipStream_t st) {
  WgradMfmaArgs a;
  a.gyu = gy_u;
  a.xu = x_u;
  a.part = part;
  a.Ci = g.Ci;
  a.Co = g.Co;
  a.P = g.P;
  a.Ktot = g.N * g.P;
  a.nchunks = wgrad_chunks(g);
  a.N = g.N;
  a.G = 1;
  a.flat = wgrad_flat(g, &a.G) ? 1 : 0;
  const int nz = mfma_wgrad_splits(g, &a.chunks_per_z);
  a.d_p = FastDiv((uint32_t)g.P);
  *nz_out = nz;
  const bool vec = g.P % Mma<T>::VE == 0;
  switch (wgrad_shape(g)) {
    case 1: return wgrad_launch<T, 2, 2, 4, 1>(a, nz, vec, st);
    case 2: return wgrad_launch<T, 2, 2, 1, 4>(a, nz, vec, st);
    case 4: return wgrad_launch<T, 4, 4, 4, 1>(a, nz, vec, st);
    default: return wgrad_launch<T, 2, 2, 2, 2>(a, nz, vec, st);
  }
}

hipError_t launch_mfma_wgrad(const Geom& g, const void* x_u, const void* gy_u, float* part,
                             int* nz_out, hipStream_t st) {
  if (plain_wgrad_ok(g)) return launch_plain_wgrad(g, x_u, gy_u, part, nz_out, st);
  if (g.dtype == GF_BF16) return wgrad_t<bf16_t>(g, x_u, gy_u, part, nz_out, st);
  return wgrad_t<float>(g, x_u, gy_u, part, nz_out, st);
}

template <class T, int BN>
hipError_t dgrad_ksplit_launch(DgradMfmaArgs& a, bool vec, hipStream_t st) {
  if (!a.planes_mode) dgrad_column_tiles<T>(a, BN, 32);
  dim3 grid(cdiv(a.Jtot, a.cols_per_tile), cdiv(a.Ci, 32), 1);
  if (vec)
    GF_LAUNCH((dgrad_ksplit_k<T, BN, true>), grid, dim3(kThreads), 0, st, a);
  else
    GF_LAUNCH((dgrad_ksplit_k<T, BN, false>), grid, dim3(kThreads), 0, st, a);
  return hipGetLastError();
}

template <class T>
static bool dgrad_full_ok(const Geom& g) {
  constexpr int VE = Mma<T>::VE;
  const int rx = g.rx;
  if (rx != 2 && rx != 4 && rx != 8) return false;
  if (g.Ci % VE != 0) return false;                     // vector loads of the kernel matrix
  // (P need not be a vector multiple: gy_u is then read with element-aligned 16-byte loads)
  if (g.W != g.Wp * rx || g.W % VE != 0) return false;  // no ragged patch columns, aligned rows
  if (rx < VE && g.Wp % (VE / rx) != 0) return false;   // a pixel run never leaves its patch row
  return true;
}

// plane mode: whole images fit the 64-column tile and one plane fits the staging buffer
static bool dgrad_planes_ok(const Geom& g) {
  return g.P <= 64 && (long)g.H * g.W * g.b + 32 <= kPlaneStageBytes;
}

bool mfma_dgrad_writes_full(const Geom& g) {
  const bool runs = g.dtype == GF_BF16 ? dgrad_full_ok<bf16_t>(g) : dgrad_full_ok<float>(g);
  return runs || dgrad_planes_ok(g);
}

// images per column tile when tiles are whole images: as many as fit, but few enough to
// leave ~512 blocks for the chip (small maps with a small batch would otherwise run on a
// handful of CUs)
static int images_per_tile(const Geom& g, int bn, int bm) {
  int ipt = bn / g.P;
  while (ipt > 1 && (long)cdiv(g.N, ipt) * cdiv(g.Ci, bm) < 512) --ipt;
  return ipt;
}

// S2 when the kernel is larger than 1x1: its spatial sum, rounded to the storage type
template <class T>
static hipError_t kernel_sum_if_needed(const Geom& g, const void* w, void* wsum_t, const T** wt,
                                       hipStream_t st) {
  *wt = static_cast<const T*>(w);
  if (g.KK == 1) return hipSuccess;
  const int pairs = g.Co * g.Ci;
  GF_LAUNCH(kernel_sum_t_k<T>, dim3(cdiv(pairs, kThreads)), dim3(kThreads), 0, st,
                     static_cast<const T*>(w), static_cast<T*>(wsum_t), pairs, g.KK);
  *wt = static_cast<const T*>(wsum_t);
  return hipGetLastError();
}

template <class T>
static bool dgrad_wants_ksplit(const Geom& g, bool planes) {
  const bool vec = g.P % Mma<T>::VE == 0 && g.Ci % Mma<T>::VE == 0;
  const long tiles64 = (long)cdiv((long)g.N * g.P, planes ? (64 / g.P) * g.P : 64) * cdiv(g.Ci, 64);
  return vec && g.Co >= 512 && tiles64 < 512;
}

template <class T>
static hipError_t dgrad_t(const Geom& g, const void* gy_u, const void* w, void* wsum_t, void* dst,
                          void* full, hipStream_t st) {
  const T* wt = nullptr;
  hipError_t e0 = kernel_sum_if_needed<T>(g, w, wsum_t, &wt, st);
  if (e0 != hipSuccess) return e0;
  DgradMfmaArgs a;
  a.gyu = gy_u;
  a.wt = wt;
  a.dst = dst;
  a.mask = nullptr;
  a.Ci = g.Ci;
  a.Co = g.Co;
  a.P = g.P;
  a.Jtot = g.N * g.P;
  a.scale = 1.f / ((float)g.s * (float)g.s);
  a.d_p = FastDiv((uint32_t)g.P);
  a.full = full;
  a.H = g.H;
  a.W = g.W;
  a.Wp = g.Wp;
  a.rx = g.rx;
  a.d_wp = FastDiv((uint32_t)g.Wp);
  a.planes_mode = 0;
  a.prt = 0;
  a.ipt = 0;
  a.cols_per_tile = 0;
  a.rows_per_pass = 0;
  a.N = g.N;
  a.veca = g.Ci % Mma<T>::VE == 0;
  a.flatb = 0;
  const bool vec = g.P % Mma<T>::VE == 0 && g.Ci % Mma<T>::VE == 0;
  // P not a multiple of the vector length: whole-image column tiles, gy_u read as image blocks
  const bool flatb = g.P % Mma<T>::VE != 0 && g.P <= 64 && ((long)g.Co * g.P * sizeof(T)) % 16 == 0;
  const bool planes = full && !dgrad_full_ok<T>(g);
  // few 64 x 64 tiles and a long K: let the four waves of a block split K instead
  // (measured: pays from K = 512 up; at K = 320 .. 576 with many tiles it is slower)
  const bool ksplit = dgrad_wants_ksplit<T>(g, planes);
  if (planes) {  // small / unaligned maps: whole images per column tile
    const int bn = (ksplit && g.P <= 32) ? 32 : 64;
    a.planes_mode = 1;
    a.ipt = images_per_tile(g, bn, ksplit ? 32 : 64);
    a.cols_per_tile = a.ipt * g.P;
    a.rows_per_pass = (kPlaneStageBytes - 32) / (g.H * g.W * (int)sizeof(T));
    if (ksplit) return bn == 32 ? dgrad_ksplit_launch<T, 32>(a, vec, st) : dgrad_ksplit_launch<T, 64>(a, vec, st);
    a.flatb = flatb ? 1 : 0;
    return dgrad_launch<T, 2, 2, 2, 2>(a, vec, st);
  }
  if (flatb) {  // reduced map out, whole-image column tiles
    a.flatb = 1;
    a.planes_mode = 0;
    a.ipt = images_per_tile(g, 64, 64);
    a.cols_per_tile = a.ipt * g.P;
    return dgrad_launch<T, 2, 2, 2, 2>(a, false, st);
  }
  if (ksplit) return dgrad_ksplit_launch<T, 64>(a, vec, st);
  // many tiles: 128 x 128 halves the operand re-reads from L2, which bound the 64 x 64 tiling
  if (vec && g.Ci >= 256 && (long)cdiv(a.Jtot, 128) * cdiv(g.Ci, 128) >= 512)
    return dgrad_launch<T, 4, 4, 2, 2>(a, vec, st);
  if (g.Ci <= 32) return dgrad_launch<T, 2, 2, 1, 4>(a, vec, st);
  if (vec && g.Ci >= 256 && !full && (long)g.N * g.P * g.Co * g.b >= kHugeOperandBytes)
    return dgrad_launch<T, 4, 4, 4, 1>(a, vec, st);  // huge gy_u (column tensor): read it once
  return dgrad_launch<T, 2, 2, 2, 2>(a, vec, st);
}

// both gradients in one launch: every shape the 64 x 64 (or 32 x 128) input-gradient block handles
// without splitting K among its waves
template <class T>
static bool s3s4_ok(const Geom& g, bool reduced) {
  constexpr int VE = Mma<T>::VE;
  if (g.g != 1 || g.Ci % VE != 0) return false;
  if (wgrad_shape(g) == 4 || plain_wgrad_ok(g)) return false;
  if (reduced) {  // reduced map out: vector columns, element-aligned vectors, or image blocks on both sides
    if (g.P % VE == 0 || g.P > 64) return true;
    return wgrad_flat(g, nullptr) && g.P <= 64 && ((long)g.Co * g.P * sizeof(T)) % 16 == 0;
  }
  const bool runs = dgrad_full_ok<T>(g);
  if (!runs && !dgrad_planes_ok(g)) return false;
  if (g.P % VE != 0) {
    if (runs) return g.P >= VE;   // element-aligned vector loads of gy_u, pixel-run / patch-row store
    // plane mode: image-block loaders on both sides
    if (!wgrad_flat(g, nullptr)) return false;
    if (g.P > 64 || ((long)g.Co * g.P * sizeof(T)) % 16 != 0) return false;
  }
  return true;
}

bool mfma_s3s4_ok(const Geom& g, bool reduced) {
  return g.dtype == GF_BF16 ? s3s4_ok<bf16_t>(g, reduced) : s3s4_ok<float>(g, reduced);
}

template <class T, int WTM, int WTN, int WWM, int WWN>
static hipError_t s3s4_launch(const Geom& g, WgradMfmaArgs& wa, DgradMfmaArgs& da, int nz, hipStream_t st) {
  constexpr int WBM = WWM * WTM * 16, WBN = WWN * WTN * 16;
  S3S4Grid gr;
  gr.wgx = cdiv(g.Ci, WBN);
  gr.wgy = cdiv(g.Co, WBM);
  gr.nw = gr.wgx * gr.wgy * nz;
  const bool vec = g.P % Mma<T>::VE == 0;
  if (dgrad_wants_ksplit<T>(g, da.planes_mode != 0)) {  // K-split block, 32 rows of c_i
    const int bn = (da.planes_mode && g.P <= 32) ? 32 : 64;
    if (da.planes_mode) {
      da.ipt = images_per_tile(g, bn, 32);
      da.cols_per_tile = da.ipt * g.P;
    } else {
      dgrad_column_tiles<T>(da, bn, 32);
    }
    gr.dgx = cdiv(da.Jtot, da.cols_per_tile);
    const int grid = gr.nw + gr.dgx * cdiv(g.Ci, 32);
    if (bn == 32)
      GF_LAUNCH((s3s4_ksplit_k<T, WTM, WTN, WWM, WWN, 32>), dim3(grid), dim3(kThreads), 0, st, wa, da, gr);
    else
      GF_LAUNCH((s3s4_ksplit_k<T, WTM, WTN, WWM, WWN, 64>), dim3(grid), dim3(kThreads), 0, st, wa, da, gr);
    return hipGetLastError();
  }
  if (da.planes_mode || da.flatb) {  // column tiles of whole images
    gr.dgx = cdiv(da.Jtot, da.cols_per_tile);
    const int grid = gr.nw + gr.dgx * cdiv(g.Ci, 64);
    if (vec)
      GF_LAUNCH((s3s4_mfma_k<T, WTM, WTN, WWM, WWN, 2, 2, 2, 2, true, true>), dim3(grid), dim3(kThreads), 0, st, wa, da, gr);
    else
      GF_LAUNCH((s3s4_mfma_k<T, WTM, WTN, WWM, WWN, 2, 2, 2, 2, false, true>), dim3(grid), dim3(kThreads), 0, st, wa, da, gr);
    return hipGetLastError();
  }
  dgrad_column_tiles<T>(da, g.Ci <= 32 ? 128 : 64, g.Ci <= 32 ? 32 : 64);
  gr.dgx = cdiv(da.Jtot, da.cols_per_tile);
  const int nd = gr.dgx * cdiv(g.Ci, g.Ci <= 32 ? 32 : 64);
  const dim3 grid(gr.nw + nd), block(kThreads);
  if (g.Ci <= 32) {
    if (vec) GF_LAUNCH((s3s4_mfma_k<T, WTM, WTN, WWM, WWN, 2, 2, 1, 4, true, false>), grid, block, 0, st, wa, da, gr);
    else GF_LAUNCH((s3s4_mfma_k<T, WTM, WTN, WWM, WWN, 2, 2, 1, 4, false, false>), grid, block, 0, st, wa, da, gr);
  } else {
    if (vec) GF_LAUNCH((s3s4_mfma_k<T, WTM, WTN, WWM, WWN, 2, 2, 2, 2, true, false>), grid, block, 0, st, wa, da, gr);
    else GF_LAUNCH((s3s4_mfma_k<T, WTM, WTN, WWM, WWN, 2, 2, 2, 2, false, false>), grid, block, 0, st, wa, da, gr);
  }
  return hipGetLastError();
}

template <class T>
static hipError_t s3s4_t(const Geom& g, const void* x_u, const void* gy_u, const void* w, void* wsum_t,
                         float* part, int* nz_out, void* g_x, hipStream_t st, bool wsum_ready, bool reduced,
                         const void* mask_u) {
  const T* wt = nullptr;
  if (wsum_ready && g.KK > 1) {
    wt = static_cast<const T*>(wsum_t);  // formed by an earlier launch of the same call
  } else {
    hipError_t e = kernel_sum_if_needed<T>(g, w, wsum_t, &wt, st);
    if (e != hipSuccess) return e;
  }
  WgradMfmaArgs wa;
  wa.gyu = gy_u; wa.xu = x_u; wa.part = part;
  wa.Ci = g.Ci; wa.Co = g.Co; wa.P = g.P; wa.Ktot = g.N * g.P;
  wa.nchunks = wgrad_chunks(g);
  wa.N = g.N; wa.G = 1;
  wa.flat = wgrad_flat(g, &wa.G) ? 1 : 0;
  const int nz = mfma_wgrad_splits(g, &wa.chunks_per_z);
  wa.d_p = FastDiv((uint32_t)g.P);
  *nz_out = nz;
  DgradMfmaArgs da;
  da.gyu = gy_u; da.wt = wt; da.dst = nullptr; da.mask = nullptr;
  da.Ci = g.Ci; da.Co = g.Co; da.P = g.P; da.Jtot = g.N * g.P;
  da.scale = 1.f / ((float)g.s * (float)g.s);
  da.d_p = FastDiv((uint32_t)g.P);
  da.full = g_x; da.H = g.H; da.W = g.W; da.Wp = g.Wp; da.rx = g.rx;
  da.d_wp = FastDiv((uint32_t)g.Wp);
  da.planes_mode = 0; da.prt = 0; da.ipt = 0; da.cols_per_tile = 0; da.rows_per_pass = 0;
  da.N = g.N; da.veca = 1; da.flatb = 0;
  if (reduced) {  // reduced map out, as in dgrad_t
    da.dst = g_x;
    da.mask = mask_u;
    da.full = nullptr;
    if (g.P % Mma<T>::VE != 0 && g.P <= 64) {
      da.flatb = 1;
      da.ipt = images_per_tile(g, 64, 64);
      da.cols_per_tile = da.ipt * g.P;
    }
  } else if (!dgrad_full_ok<T>(g)) {  // plane mode, as in dgrad_t
    da.planes_mode = 1;
    da.ipt = images_per_tile(g, 64, 64);
    da.cols_per_tile = da.ipt * g.P;
    da.rows_per_pass = (kPlaneStageBytes - 32) / (g.H * g.W * (int)sizeof(T));
    da.flatb = g.P % Mma<T>::VE != 0 ? 1 : 0;
  }
  switch (wgrad_shape(g)) {
    case 1: return s3s4_launch<T, 2, 2, 4, 1>(g, wa, da, nz, st);
    case 2: return s3s4_launch<T, 2, 2, 1, 4>(g, wa, da, nz, st);
    default: return s3s4_launch<T, 2, 2, 2, 2>(g, wa, da, nz, st);
  }
}

hipError_t launch_mfma_s3s4(const Geom& g, const void* x_u, const void* gy_u, const void* w,
                            void* wsum_t, float* part, int* nz_out, void* g_x, hipStream_t st,
                            bool wsum_ready, bool reduced, const void* mask_u) {
  if (g.dtype == GF_BF16)
    return s3s4_t<bf16_t>(g, x_u, gy_u, w, wsum_t, part, nz_out, g_x, st, wsum_ready, reduced, mask_u);
  return s3s4_t<float>(g, x_u, gy_u, w, wsum_t, part, nz_out, g_x, st, wsum_ready, reduced, mask_u);
}

hipError_t launch_mfma_dgrad(const Geom& g, const void* gy_u, const void* w, void* wsum_t, void* dst,
                             void* full, hipStream_t st) {
  if (g.dtype == GF_BF16) return dgrad_t<bf16_t>(g, gy_u, w, wsum_t, dst, full, st);
  return dgrad_t<float>(g, gy_u, w, wsum_t, dst, full, st);
}

}  // namespace gf
