// Gradient filtering on signed 8-bit codes (Supp. H combines the method with 8-bit gradient
// quantisation).  The reduced maps gy_u and x_u and the kernel sum are held as codes with one step
// size per tensor (round half to even, clipped to +-127); Eq. 5 and Eq. 3 then are integer
// contractions, which are exact, and the integer is scaled once by the product of the two step
// sizes and 1/s^2.
//
//  * kernel_sum_q8_k   -- codes of the spatial kernel sum (text after Eq. 3)
//  * q8_wgrad_mfma_k   -- Eq. 5 for dense layers with at least 16 channels on both sides:
//                         v_mfma_i32_16x16x64_i8 on 64 x 64 tiles, K = (n, patch) split into slabs,
//                         int32 partial slabs (a slab holds few enough products not to overflow),
//                         q8_finalize_k adds them in 64 bits and scales
//  * q8_wgrad_pair_k   -- Eq. 5 for every other layer (groups, depthwise, tiny planes): one
//                         block per (c_o, c_i) pair, v_dot4_i32_i8 on 32-bit words where the plane
//                         allows it, 64-bit sums
//  * q8_dgrad_mfma_k   -- Eq. 3 for dense layers with many channels on both sides: the same MFMA after
//                         a transposing LDS staging (K = c_o is contiguous in neither operand)
//  * q8_dgrad_tile_k   -- Eq. 3 for planes that are multiples of four codes: a lane owns four patches
//                         of four (or one) input channels and walks the group's c_o; stores the
//                         full-resolution pixel runs itself where the patch rows allow
//  * q8_dgrad_k        -- Eq. 3 for the other planes: one lane per (n, c_i, patch)
//    all three write the reduced map (storage type), or, where they cannot store full resolution
//    themselves, an fp32 map that the expansion kernels of the floating-point path replicate
#include "gf_internal.h"

namespace gf {

namespace {

constexpr int kThreads = 256;
constexpr int kRowBytes = 128 + 16;  // one staged row: 128 codes (K) + pad
typedef int i32x4 __attribute__((ext_vector_type(4)));

template <class T>
__global__ __launch_bounds__(kThreads) void kernel_sum_q8_k(const T* w, int8_t* w_q, int pairs, int KK, float inv) {
  const int e = blockIdx.x * kThreads + threadIdx.x;
  if (e < pairs) w_q[e] = q8_code(kernel_sum_of(w, e, KK), inv);
}

// ---------------------------------------------------------------------------
// Eq. 5, dense: part[z, co, ci] = sum over the K chunks of slab z of gy_q * x_q
// ---------------------------------------------------------------------------
struct Q8WgradArgs {
  const int8_t* gyq;
  const int8_t* xq;
  int* part;
  int Ci, Co, P, Ktot;
  int nchunks, chunks_per_z;
  FastDiv d_p;
};

// 16 codes of row `base` (one channel of every image, images img_stride apart) from flat column
// k = (n, p), k a multiple of 16 (a vector never leaves its image because 16 | P); zero beyond ktot
__device__ __forceinline__ uint4 load_codes(const int8_t* base, long img_stride, int k, int ktot, int P,
                                            const FastDiv& d_p) {
  const int kc = min(k, ktot - 16);
  const int n = (int)d_p.div((uint32_t)kc);
  const int p = kc - n * P;
  const uint4 v = *reinterpret_cast<const uint4*>(base + (long)n * img_stride + p);
  return k < ktot ? v : make_uint4(0, 0, 0, 0);
}

// 16 bytes from an address of any alignment
struct __attribute__((packed, aligned(1))) Unal16 { uint32_t w[4]; };
__device__ __forceinline__ uint4 load16_any(const int8_t* p) {
  const Unal16 v = *reinterpret_cast<const Unal16*>(p);
  return make_uint4(v.w[0], v.w[1], v.w[2], v.w[3]);
}

// out byte e = in byte e + sh, zero where e + sh falls outside 0 .. 15
__device__ __forceinline__ uint4 shift_bytes(const uint4& v, int sh) {
  if (sh == 0) return v;
  if (sh >= 16 || sh <= -16) return make_uint4(0, 0, 0, 0);
  uint64_t lo = (uint64_t)v.x | ((uint64_t)v.y << 32), hi = (uint64_t)v.z | ((uint64_t)v.w << 32);
  int bits = sh * 8;   // 0 < |bits| < 128
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

// The same for planes of any size.  P >= 16: the run k .. k + 15 may start anywhere in image n and
// may continue in image n + 1.  Branch-free, both loads always issued: the part that lies in image
// n comes from a load pulled back into that image and shifted, the part in image n + 1 from a load
// at the start of the next image shifted the other way; codes at and beyond ktot are cleared.
__device__ __forceinline__ uint4 load_codes_any(const int8_t* base, long img_stride, int k, int ktot, int P,
                                                const FastDiv& d_p) {
  if (P < 16) {   // planes smaller than a run (2 x 2, 3 x 3 patch grids): the run is gathered code by code
    uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int kk = min(k + e, ktot - 1);
      const int n = (int)d_p.div((uint32_t)kk);
      const uint32_t c = (uint32_t)(uint8_t)base[(long)n * img_stride + (kk - n * P)];
      w[e >> 2] |= (k + e < ktot ? c : 0u) << (8 * (e & 3));
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
  }
  const int kc = min(k, ktot - 1);
  const int n = (int)d_p.div((uint32_t)kc);
  const int p = kc - n * P;
  const int pa = min(p, P - 16);
  const int k1 = min(16, P - p);                         // codes of the run that belong to image n
  const int nlast = (int)d_p.div((uint32_t)(ktot - 1));
  const uint4 va = load16_any(base + (long)n * img_stride + pa);
  const uint4 vb = load16_any(base + (long)min(n + 1, nlast) * img_stride);
  const uint4 x = shift_bytes(va, p - pa);
  const uint4 y = shift_bytes(vb, -k1);
  uint4 v = make_uint4(x.x | y.x, x.y | y.y, x.z | y.z, x.w | y.w);
  const int keep = ktot - k;                             // codes of the run before ktot
  if (keep < 16) v = keep <= 0 ? make_uint4(0, 0, 0, 0) : shift_bytes(shift_bytes(v, -(16 - keep)), 16 - keep);
  return v;
}

template <bool VEC>
__device__ __forceinline__ uint4 load_codes_t(const int8_t* base, long img_stride, int k, int ktot, int P,
                                              const FastDiv& d_p) {
  if (VEC) return load_codes(base, img_stride, k, ktot, P, d_p);
  return load_codes_any(base, img_stride, k, ktot, P, d_p);
}

// VEC: 16 | P (aligned vector loads); else planes of any size >= 16 through load_codes_any
template <bool VEC>
__global__ __launch_bounds__(kThreads) void q8_wgrad_mfma_k(Q8WgradArgs a) {
  constexpr int BM = 64, BN = 64, BK = 128;
  __shared__ __attribute__((aligned(16))) unsigned char As[BM * kRowBytes];
  __shared__ __attribute__((aligned(16))) unsigned char Bs[BN * kRowBytes];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int kc0 = blockIdx.z * a.chunks_per_z;
  const int kc1 = min(kc0 + a.chunks_per_z, a.nchunks);
  uint4 ra[2], rb[2];
  auto fetch = [&](int kc) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int s = tid + i * kThreads, row = s >> 3, vi = s & 7;
      const int co = m0 + row, ci = n0 + row;
      const uint4 va = load_codes_t<VEC>(a.gyq + (long)min(co, a.Co - 1) * a.P, (long)a.Co * a.P, kc * BK + vi * 16,
                                         a.Ktot, a.P, a.d_p);
      const uint4 vb = load_codes_t<VEC>(a.xq + (long)min(ci, a.Ci - 1) * a.P, (long)a.Ci * a.P, kc * BK + vi * 16,
                                         a.Ktot, a.P, a.d_p);
      ra[i] = co < a.Co ? va : make_uint4(0, 0, 0, 0);
      rb[i] = ci < a.Ci ? vb : make_uint4(0, 0, 0, 0);
    }
  };
  i32x4 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = i32x4{0, 0, 0, 0};
  if (kc0 < kc1) fetch(kc0);
  const int r = lane & 15, kg = lane >> 4;
  for (int kc = kc0; kc < kc1; ++kc) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int s = tid + i * kThreads;
      *reinterpret_cast<uint4*>(As + (s >> 3) * kRowBytes + (s & 7) * 16) = ra[i];
      *reinterpret_cast<uint4*>(Bs + (s >> 3) * kRowBytes + (s & 7) * 16) = rb[i];
    }
    __syncthreads();
    if (kc + 1 < kc1) fetch(kc + 1);
    // A: lane holds row lane % 16, k = 16 * (lane / 16) .. + 15 of the 64-wide k-step; B alike
#pragma unroll
    for (int ks = 0; ks < BK / 64; ++ks) {
      i32x4 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i)
        fa[i] = *reinterpret_cast<const i32x4*>(As + ((wm * 2 + i) * 16 + r) * kRowBytes + ks * 64 + kg * 16);
#pragma unroll
      for (int j = 0; j < 2; ++j)
        fb[j] = *reinterpret_cast<const i32x4*>(Bs + ((wn * 2 + j) * 16 + r) * kRowBytes + ks * 64 + kg * 16);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }
  // D[i = 4 * (lane / 16) + v][j = lane % 16] of every 16 x 16 tile
  int* dst = a.part + (long)blockIdx.z * a.Co * a.Ci;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int ci = n0 + (wn * 2 + j) * 16 + (lane & 15);
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int co = m0 + (wm * 2 + i) * 16 + 4 * (lane >> 4) + v;
        if (co < a.Co && ci < a.Ci) dst[(long)co * a.Ci + ci] = acc[i][j][v];
      }
    }
}

// g_w[pair, all taps] = float(sum over the slabs, 64 bits) * scale; 16 lanes share an output
// (each takes every 16th slab, four loads in flight), then a shuffle tree
__global__ __launch_bounds__(kThreads) void q8_finalize_k(const int* part, float* g_w, int pairs, int nz, int KK,
                                                         float scale) {
  const int sub = threadIdx.x & 15;
  const int e = blockIdx.x * (kThreads / 16) + (threadIdx.x >> 4);
  const int ec = min(e, pairs - 1);
  long long s = 0;
  int z = sub;
  for (; z + 48 < nz; z += 64) {
    const int v0 = part[(long)z * pairs + ec], v1 = part[(long)(z + 16) * pairs + ec];
    const int v2 = part[(long)(z + 32) * pairs + ec], v3 = part[(long)(z + 48) * pairs + ec];
    s += ((long long)v0 + v1) + ((long long)v2 + v3);
  }
  for (; z < nz; z += 16) s += part[(long)z * pairs + ec];
  for (int m = 8; m > 0; m >>= 1) s += __shfl_xor(s, m, 64);
  if (e >= pairs) return;
  const float v = (float)s * scale;
  for (int t = sub; t < KK; t += 16) g_w[(long)e * KK + t] = v;
}

// ---------------------------------------------------------------------------
// Eq. 5, any layer: block = one (c_o, c_i') pair
// ---------------------------------------------------------------------------
struct Q8PairArgs {
  const int8_t* gyq;
  const int8_t* xq;
  float* g_w;
  int N, Ci, Co, Cg, Og, P, KK;
  float scale;
  FastDiv d_per;   // words (P / 4) or codes (P) per plane
};

// V4: the plane is a multiple of four codes, so rows are read as 32-bit words and multiplied with
// v_dot4_i32_i8.  A lane adds at most 1024 words into an int32 before it moves on to 64 bits.
template <bool V4>
__global__ __launch_bounds__(kThreads) void q8_wgrad_pair_k(Q8PairArgs a) {
  __shared__ long long red[kThreads / 64];
  const int pair = blockIdx.x;
  const int co = pair / a.Cg, cl = pair - co * a.Cg;
  const int ci = (co / a.Og) * a.Cg + cl;
  const int8_t* gbase = a.gyq + (long)co * a.P;
  const int8_t* xbase = a.xq + (long)ci * a.P;
  const long gs = (long)a.Co * a.P, xs = (long)a.Ci * a.P;   // image strides
  const int per = V4 ? a.P / 4 : a.P;                        // words / codes per plane
  const int tot = a.N * per;                                 // < 2^31 (host)
  long long s = 0;
  int i = threadIdx.x;
  while (i < tot) {
    int acc = 0;
#pragma unroll 4
    for (int u = 0; u < 1024; ++u) {
      if (i >= tot) break;
      const int n = (int)a.d_per.div((uint32_t)i);
      const int q = i - n * per;
      if (V4) {
        const int gv = reinterpret_cast<const int*>(gbase + n * gs)[q];
        const int xv = reinterpret_cast<const int*>(xbase + n * xs)[q];
        acc = __builtin_amdgcn_sdot4(gv, xv, acc, false);
      } else {
        acc += (int)gbase[n * gs + q] * (int)xbase[n * xs + q];
      }
      i += kThreads;
    }
    s += acc;
  }
  for (int m = 32; m > 0; m >>= 1) s += __shfl_xor(s, m, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    long long t = 0;
    for (int k = 0; k < kThreads / 64; ++k) t += red[k];
    const float v = (float)t * a.scale;
    for (int k = 0; k < a.KK; ++k) a.g_w[(long)pair * a.KK + k] = v;
  }
}

// ---------------------------------------------------------------------------
// Eq. 3: dst[n, ci, p] = float(sum over the group's c_o of gy_q[n, co, p] * w_q[co, cl]) * scale
// ---------------------------------------------------------------------------
struct Q8DgradArgs {
  const int8_t* gyq;
  const int8_t* wq;
  void* dst;
  int N, Ci, Co, Cg, Og, P;
  long total;   // N * Ci * P
  float scale;
  FastDiv d_p, d_ci;
};

template <class D>
__global__ __launch_bounds__(kThreads) void q8_dgrad_k(Q8DgradArgs a) {
  const long e = (long)blockIdx.x * kThreads + threadIdx.x;
  if (e >= a.total) return;
  const int plane = (int)a.d_p.div((uint32_t)e);   // n * Ci + ci   (total < 2^31, checked on the host)
  const int p = (int)e - plane * a.P;
  const int n = (int)a.d_ci.div((uint32_t)plane);
  const int ci = plane - n * a.Ci;
  const int grp = ci / a.Cg, cl = ci - grp * a.Cg;
  const int8_t* gp = a.gyq + ((long)n * a.Co + (long)grp * a.Og) * a.P + p;
  const int8_t* wp = a.wq + (long)grp * a.Og * a.Cg + cl;
  int acc = 0;   // Og * 127^2 < 2^31 for Og <= 133 000 (checked on the host)
  for (int ol = 0; ol < a.Og; ++ol) acc += (int)gp[(long)ol * a.P] * (int)wp[(long)ol * a.Cg];
  static_cast<D*>(a.dst)[e] = from_f32<D>((float)acc * a.scale);
}

// The same for planes that are multiples of four codes: a lane owns four patches of CT input
// channels (CT = 4 needs group widths that are multiples of four; CT = 1 is for layers with so few
// input channels that 4 x 4 tiles would leave most of the chip idle).  Per c_o it reads one word of
// gy_q (four patches) and one word (or one code) of w_q and adds the 4 CT products.
struct Q8DgradTileArgs {
  const int8_t* gyq;
  const int8_t* wq;
  void* dst;
  int N, Ci, Co, Cg, Og, P;
  int total;   // N * (Ci / CT) * (P / 4)
  float scale;
  FastDiv d_p4, d_ct;
  // full-resolution store (RX > 0): the four patches of a lane lie in one patch row (4 | W_p)
  int H, W, Wq;   // Wq = W_p / 4
  FastDiv d_wq;
};

__device__ __forceinline__ int code_of(int word, int k) { return (int)(int8_t)(word >> (8 * k)); }

// SPLIT (1 or 4) neighbouring lanes share a tile and take every SPLIT-th c_o (integer sums, so the
// order does not matter); it shortens the chain of dependent loads when the tiles are few.
// RX > 0: instead of the reduced map, every pixel of the RX x RX input-side patches receives its
// patch's value (rounded once to the storage type, then replicated), as 16-byte runs of pixels.
template <class D, int CT, int SPLIT, int RX>
__global__ __launch_bounds__(kThreads) void q8_dgrad_tile_k(Q8DgradTileArgs a) {
  const int lane_id = blockIdx.x * kThreads + threadIdx.x;
  if (lane_id >= a.total * SPLIT) return;
  const int e = lane_id / SPLIT, sub = lane_id - e * SPLIT;
  const int P4 = a.P >> 2, CN = a.Ci / CT;
  const int planes = (int)a.d_p4.div((uint32_t)e);   // n * CN + c
  const int q = e - planes * P4;
  const int n = (int)a.d_ct.div((uint32_t)planes);
  const int ci0 = (planes - n * CN) * CT;
  const int grp = ci0 / a.Cg, cl0 = ci0 - grp * a.Cg;   // CT | Cg: the lane's channels share a group
  const int8_t* gp = a.gyq + ((long)n * a.Co + (long)grp * a.Og) * a.P + 4 * q;
  const int8_t* wp = a.wq + (long)grp * a.Og * a.Cg + cl0;
  int acc[CT][4];
#pragma unroll
  for (int i = 0; i < CT; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0;
#pragma unroll 4
  for (int ol = sub; ol < a.Og; ol += SPLIT) {
    const int gv = *reinterpret_cast<const int*>(gp + (long)ol * a.P);
    int gc[4], wc[CT];
#pragma unroll
    for (int k = 0; k < 4; ++k) gc[k] = code_of(gv, k);
    if constexpr (CT == 4) {
      const int wv = *reinterpret_cast<const int*>(wp + (long)ol * a.Cg);
#pragma unroll
      for (int k = 0; k < 4; ++k) wc[k] = code_of(wv, k);
    } else {
      wc[0] = (int)wp[(long)ol * a.Cg];
    }
#pragma unroll
    for (int i = 0; i < CT; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] += wc[i] * gc[j];
  }
  if constexpr (SPLIT > 1) {
#pragma unroll
    for (int i = 0; i < CT; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        for (int m = SPLIT >> 1; m > 0; m >>= 1) acc[i][j] += __shfl_xor(acc[i][j], m, 64);
    if (sub != 0) return;
  }
#pragma unroll
  for (int i = 0; i < CT; ++i) {
    D v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = from_f32<D>((float)acc[i][j] * a.scale);
    if constexpr (RX == 0) {
      D* d = static_cast<D*>(a.dst) + ((long)n * a.Ci + ci0 + i) * a.P + 4 * q;
      if constexpr (sizeof(D) == 4) *reinterpret_cast<uint4*>(d) = *reinterpret_cast<const uint4*>(v);
      else *reinterpret_cast<uint2*>(d) = *reinterpret_cast<const uint2*>(v);
    } else {
      constexpr int VE = 16 / (int)sizeof(D);     // pixels per 16-byte run
      constexpr int NV = 4 * RX / VE;             // runs per pixel row of the lane's four patches
      const int hp = (int)a.d_wq.div((uint32_t)q);
      const int wq = q - hp * a.Wq;
      const int h0 = hp * RX, rows = min(RX, a.H - h0);
      __attribute__((aligned(16))) D px[4 * RX];
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int k = 0; k < RX; ++k) px[j * RX + k] = v[j];
      D* d = static_cast<D*>(a.dst) + (((long)n * a.Ci + ci0 + i) * a.H + h0) * a.W + wq * 4 * RX;
      // one run per lane and row: a wave's store covers whole lines, which is what the streaming
      // store wants; with several runs per lane each instruction writes parts of lines (plain stores)
      for (int row = 0; row < rows; ++row)
#pragma unroll
        for (int k = 0; k < NV; ++k) {
          if constexpr (NV == 1) store_stream16(d + (long)row * a.W, *reinterpret_cast<const uint4*>(px));
          else *reinterpret_cast<uint4*>(d + (long)row * a.W + k * VE) = *reinterpret_cast<const uint4*>(px + k * VE);
        }
    }
  }
}

// ---------------------------------------------------------------------------
// Eq. 3 on the int8 matrix cores, dense layers with many channels on both sides:
//   dst[n, ci, p] = float(sum_co w_q[co, ci] * gy_q[n, co, p]) * scale     (reduced map)
// M = c_i, N = (n, p), K = c_o.  Neither operand has K contiguous in memory (w_q is [c_o][c_i],
// gy_q is [n][c_o][p]), so a block reads 16-byte runs along c_i resp. p and writes them to LDS
// transposed, byte by byte, as K-major rows; the MFMA fragments are then the same 16-byte reads
// as in the weight gradient.  64 x 64 tiles, K chunks of 64.  (host: 16 | P, 16 | C_i)
// ---------------------------------------------------------------------------
struct Q8DgradMfmaArgs {
  const int8_t* gyq;
  const int8_t* wq;
  void* dst;
  int Ci, Co, P, Jtot;
  float scale;
  FastDiv d_p;
  int H, W, Wp;    // full-resolution store (RX > 0)
  FastDiv d_wp;
};

// RX == 0: dst is the reduced map.  RX > 0: dst is g_x at full resolution; the tile is rounded to
// the storage type in LDS and every lane stores the 16-byte pixel runs of four neighbouring patches
// of one c_i (host: 4 | W_p, W == W_p * RX).
template <class D, int RX, bool VEC>
__global__ __launch_bounds__(kThreads) void q8_dgrad_mfma_k(Q8DgradMfmaArgs a) {
  constexpr int BK = 64, kRow = BK + 16;   // staged row: 64 codes of K + pad
  __shared__ __attribute__((aligned(16))) unsigned char As[64 * kRow];
  __shared__ __attribute__((aligned(16))) unsigned char Bs[64 * kRow];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
  const int k = tid >> 2, vi = tid & 3;          // this lane's K row and 16-wide column group of a chunk
  // the lane's 16 columns (n, p .. p + 15) do not depend on the chunk
  const int j = j0 + vi * 16;
  const int ci = m0 + vi * 16;
  const int8_t* wcol = a.wq + min(ci, a.Ci - 16);
  auto fetch = [&](int k0, uint4* ra, uint4* rb) {
    const int co = k0 + k;
    const int cc = min(co, a.Co - 1);
    const uint4 va = *reinterpret_cast<const uint4*>(wcol + (long)cc * a.Ci);
    const uint4 vb = load_codes_t<VEC>(a.gyq + (long)cc * a.P, (long)a.Co * a.P, j, a.Jtot, a.P, a.d_p);
    *ra = (co < a.Co && ci < a.Ci) ? va : make_uint4(0, 0, 0, 0);
    *rb = co < a.Co ? vb : make_uint4(0, 0, 0, 0);
  };
  i32x4 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) acc[i][jj] = i32x4{0, 0, 0, 0};
  uint4 ra, rb;
  fetch(0, &ra, &rb);
  const int r = lane & 15, kg = lane >> 4;
  for (int k0 = 0; k0 < a.Co; k0 += BK) {
    {  // transposed staging: code e of the run goes to row (vi * 16 + e), column k
      const uint32_t wa[4] = {ra.x, ra.y, ra.z, ra.w}, wb[4] = {rb.x, rb.y, rb.z, rb.w};
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        As[(vi * 16 + e) * kRow + k] = (unsigned char)(wa[e >> 2] >> (8 * (e & 3)));
        Bs[(vi * 16 + e) * kRow + k] = (unsigned char)(wb[e >> 2] >> (8 * (e & 3)));
      }
    }
    __syncthreads();
    if (k0 + BK < a.Co) fetch(k0 + BK, &ra, &rb);
    i32x4 fa[2], fb[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
      fa[i] = *reinterpret_cast<const i32x4*>(As + ((wm * 2 + i) * 16 + r) * kRow + kg * 16);
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
      fb[jj] = *reinterpret_cast<const i32x4*>(Bs + ((wn * 2 + jj) * 16 + r) * kRow + kg * 16);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
        acc[i][jj] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[i], fb[jj], acc[i][jj], 0, 0, 0);
    __syncthreads();
  }
  // D[row = 4 * (lane / 16) + v][col = lane % 16]: rows are c_i, columns (n, p)
  D* dst = static_cast<D*>(a.dst);
  if constexpr (RX == 0) {
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
      const int col = j0 + (wn * 2 + jj) * 16 + (lane & 15);
      if (col >= a.Jtot) continue;
      const int nn = (int)a.d_p.div((uint32_t)col);
      const long base = (long)nn * a.Ci * a.P + (col - nn * a.P);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int row = m0 + (wm * 2 + i) * 16 + 4 * (lane >> 4) + v;
          if (row < a.Ci) dst[base + (long)row * a.P] = from_f32<D>((float)acc[i][jj][v] * a.scale);
        }
    }
  } else {
    constexpr int SC = 64 + 16 / (int)sizeof(D);   // row stride of the staged tile, in elements
    __shared__ __attribute__((aligned(16))) D Cs[64 * SC];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          Cs[((wm * 2 + i) * 16 + 4 * (lane >> 4) + v) * SC + (wn * 2 + jj) * 16 + (lane & 15)] =
              from_f32<D>((float)acc[i][jj][v] * a.scale);
    __syncthreads();
    constexpr int VE = 16 / (int)sizeof(D), NV = 4 * RX / VE;
    for (int it = tid; it < 64 * 16; it += kThreads) {
      const int cl = it >> 4, quad = it & 15;          // 16 lanes = the 64 patches of one c_i row
      const int cc = m0 + cl, jq = j0 + 4 * quad;
      if (cc >= a.Ci || jq >= a.Jtot) continue;
      const int nn = (int)a.d_p.div((uint32_t)jq);
      const int p = jq - nn * a.P;
      const int hp = (int)a.d_wp.div((uint32_t)p);
      const int wp0 = p - hp * a.Wp;                   // a multiple of four: the four patches share a row
      const int h0 = hp * RX, rows = min(RX, a.H - h0);
      __attribute__((aligned(16))) D px[4 * RX];
#pragma unroll
      for (int jx = 0; jx < 4; ++jx)
#pragma unroll
        for (int kx = 0; kx < RX; ++kx) px[jx * RX + kx] = Cs[cl * SC + 4 * quad + jx];
      D* d = dst + (((long)nn * a.Ci + cc) * a.H + h0) * a.W + wp0 * RX;
      for (int row = 0; row < rows; ++row)
#pragma unroll
        for (int kx = 0; kx < NV; ++kx) {
          if constexpr (NV == 1) store_stream16(d + (long)row * a.W, *reinterpret_cast<const uint4*>(px));
          else *reinterpret_cast<uint4*>(d + (long)row * a.W + kx * VE) = *reinterpret_cast<const uint4*>(px + kx * VE);
        }
    }
  }
}

static bool q8_dgrad_mfma_ok(const Geom& g) {
  return g.g == 1 && g.Ci % 16 == 0 && g.Ci >= 64 && g.Co >= 64;
}

// rx: 0 = reduced map, 2 / 4 = full resolution written by the kernel (see q8_dgrad_full_ok)
template <class D>
static hipError_t q8_dgrad_mfma_launch(const Geom& g, const int8_t* gy_q, const int8_t* w_q, float fscale, void* dst,
                                       int rx, hipStream_t st) {
  Q8DgradMfmaArgs a;
  a.gyq = gy_q; a.wq = w_q; a.dst = dst;
  a.Ci = g.Ci; a.Co = g.Co; a.P = g.P; a.Jtot = g.N * g.P;
  a.scale = fscale;
  a.d_p = FastDiv((uint32_t)g.P);
  a.H = g.H; a.W = g.W; a.Wp = g.Wp;
  a.d_wp = FastDiv((uint32_t)g.Wp);
  const dim3 grid(cdiv(a.Jtot, 64), cdiv(g.Ci, 64)), block(kThreads);
  if (g.P % 16 == 0) {
    if (rx == 2) GF_LAUNCH((q8_dgrad_mfma_k<D, 2, true>), grid, block, 0, st, a);
    else if (rx == 4) GF_LAUNCH((q8_dgrad_mfma_k<D, 4, true>), grid, block, 0, st, a);
    else GF_LAUNCH((q8_dgrad_mfma_k<D, 0, true>), grid, block, 0, st, a);
  } else {
    if (rx == 2) GF_LAUNCH((q8_dgrad_mfma_k<D, 2, false>), grid, block, 0, st, a);
    else if (rx == 4) GF_LAUNCH((q8_dgrad_mfma_k<D, 4, false>), grid, block, 0, st, a);
    else GF_LAUNCH((q8_dgrad_mfma_k<D, 0, false>), grid, block, 0, st, a);
  }
  return hipGetLastError();
}

template <class D, int RX>
static hipError_t q8_tile_launch(Q8DgradTileArgs& a, int ct, bool split, hipStream_t st) {
  const dim3 block(kThreads), grid(cdiv((long)a.total * (split ? 4 : 1), kThreads));
  if (ct == 4 && split) GF_LAUNCH((q8_dgrad_tile_k<D, 4, 4, RX>), grid, block, 0, st, a);
  else if (ct == 4) GF_LAUNCH((q8_dgrad_tile_k<D, 4, 1, RX>), grid, block, 0, st, a);
  else if (split) GF_LAUNCH((q8_dgrad_tile_k<D, 1, 4, RX>), grid, block, 0, st, a);
  else GF_LAUNCH((q8_dgrad_tile_k<D, 1, 1, RX>), grid, block, 0, st, a);
  return hipGetLastError();
}

// the tile kernel can store full resolution itself when a lane's four patches share a patch row and
// the pixel runs are whole 16-byte vectors
static bool q8_dgrad_full_ok(const Geom& g) {
  return g.P % 4 == 0 && g.Wp % 4 == 0 && (g.rx == 2 || g.rx == 4) && g.W == g.Wp * g.rx;
}

// full: dst is g_x at full resolution (only when q8_dgrad_full_ok), else the reduced map
template <class D>
static hipError_t q8_dgrad_launch(const Geom& g, const int8_t* gy_q, const int8_t* w_q, float fscale, void* dst,
                                  bool full, hipStream_t st) {
  if (g.P % 4 == 0) {
    // 4 x 4 tiles (fewest instructions per product) where the group width allows; when they are too
    // few to fill the chip and the channel sum is long, four lanes share a tile
    const int ct = g.Cg % 4 == 0 ? 4 : 1;
    Q8DgradTileArgs a;
    a.gyq = gy_q; a.wq = w_q; a.dst = dst;
    a.N = g.N; a.Ci = g.Ci; a.Co = g.Co; a.Cg = g.Cg; a.Og = g.Og; a.P = g.P;
    a.total = (int)((long)g.N * (g.Ci / ct) * (g.P / 4));
    a.scale = fscale;
    a.d_p4 = FastDiv((uint32_t)(g.P / 4));
    a.d_ct = FastDiv((uint32_t)(g.Ci / ct));
    a.H = g.H; a.W = g.W; a.Wq = g.Wp / 4 > 0 ? g.Wp / 4 : 1;
    a.d_wq = FastDiv((uint32_t)a.Wq);
    const bool split = g.Og >= 32 && a.total < 128 * 1024;
    if (full && g.rx == 2) return q8_tile_launch<D, 2>(a, ct, split, st);
    if (full) return q8_tile_launch<D, 4>(a, ct, split, st);
    return q8_tile_launch<D, 0>(a, ct, split, st);
  }
  Q8DgradArgs a;
  a.gyq = gy_q; a.wq = w_q; a.dst = dst;
  a.N = g.N; a.Ci = g.Ci; a.Co = g.Co; a.Cg = g.Cg; a.Og = g.Og; a.P = g.P;
  a.total = (long)g.N * g.Ci * g.P;
  a.scale = fscale;
  a.d_p = FastDiv((uint32_t)g.P);
  a.d_ci = FastDiv((uint32_t)g.Ci);
  GF_LAUNCH(q8_dgrad_k<D>, dim3(cdiv(a.total, kThreads)), dim3(kThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace

// most products an int32 sum can take: 127^2 * n < 2^31
constexpr long kMaxTerms32 = 133000;

hipError_t launch_kernel_sum_q8(const Geom& g, const void* w, float inv_delta, int8_t* w_q, hipStream_t st) {
  const int pairs = g.Co * g.Cg;
  const dim3 grid(cdiv(pairs, kThreads)), block(kThreads);
  if (g.dtype == GF_BF16)
    GF_LAUNCH(kernel_sum_q8_k<bf16_t>, grid, block, 0, st, static_cast<const bf16_t*>(w), w_q, pairs, g.KK, inv_delta);
  else
    GF_LAUNCH(kernel_sum_q8_k<float>, grid, block, 0, st, static_cast<const float*>(w), w_q, pairs, g.KK, inv_delta);
  return hipGetLastError();
}

static bool q8_wgrad_mfma_ok(const Geom& g) { return g.g == 1 && g.Co >= 16 && g.Ci >= 16; }

// K slabs of the MFMA kernel: ~1024 blocks, at least two chunks per block, and few enough
// products per slab for the int32 partial sums
static int q8_wgrad_splits(const Geom& g, int* chunks_per_z) {
  const int nchunks = cdiv((long)g.N * g.P, 128);
  const int tiles = cdiv(g.Co, 64) * cdiv(g.Ci, 64);
  int nz = cdiv(1024, tiles);
  if (nz > cdiv(nchunks, 2)) nz = cdiv(nchunks, 2);
  if (nz < 1) nz = 1;
  int cpz = cdiv(nchunks, nz);
  if ((long)cpz * 128 > kMaxTerms32) cpz = (int)(kMaxTerms32 / 128);
  *chunks_per_z = cpz;
  return cdiv(nchunks, cpz);
}

size_t ws_bwd_weight_q8(const Geom& g) {
  if (!q8_wgrad_mfma_ok(g)) return 0;
  int cpz;
  return (size_t)q8_wgrad_splits(g, &cpz) * g.Co * g.Ci * sizeof(int);
}

hipError_t launch_bwd_weight_q8(const Geom& g, const int8_t* x_q, const int8_t* gy_q, float scale, float* g_w,
                                void* ws, hipStream_t st) {
  const float fscale = scale / ((float)g.s * (float)g.s);
  if (q8_wgrad_mfma_ok(g)) {
    Q8WgradArgs a;
    a.gyq = gy_q; a.xq = x_q; a.part = static_cast<int*>(ws);
    a.Ci = g.Ci; a.Co = g.Co; a.P = g.P; a.Ktot = g.N * g.P;
    a.nchunks = cdiv((long)g.N * g.P, 128);
    const int nz = q8_wgrad_splits(g, &a.chunks_per_z);
    a.d_p = FastDiv((uint32_t)g.P);
    const dim3 grid(cdiv(g.Ci, 64), cdiv(g.Co, 64), nz);
    if (g.P % 16 == 0) GF_LAUNCH(q8_wgrad_mfma_k<true>, grid, dim3(kThreads), 0, st, a);
    else GF_LAUNCH(q8_wgrad_mfma_k<false>, grid, dim3(kThreads), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int pairs = g.Co * g.Ci;
    GF_LAUNCH(q8_finalize_k, dim3(cdiv(pairs, kThreads / 16)), dim3(kThreads), 0, st, a.part, g_w, pairs, nz,
                       g.KK, fscale);
    return hipGetLastError();
  }
  Q8PairArgs a;
  a.gyq = gy_q; a.xq = x_q; a.g_w = g_w;
  a.N = g.N; a.Ci = g.Ci; a.Co = g.Co; a.Cg = g.Cg; a.Og = g.Og; a.P = g.P; a.KK = g.KK;
  a.scale = fscale;
  const bool v4 = g.P % 4 == 0;
  a.d_per = FastDiv((uint32_t)(v4 ? g.P / 4 : g.P));
  if (v4) GF_LAUNCH(q8_wgrad_pair_k<true>, dim3(g.Co * g.Cg), dim3(kThreads), 0, st, a);
  else GF_LAUNCH(q8_wgrad_pair_k<false>, dim3(g.Co * g.Cg), dim3(kThreads), 0, st, a);
  return hipGetLastError();
}

// the input gradient at full resolution goes through an fp32 reduced map in the workspace
size_t ws_bwd_input_q8(const Geom& g, bool reduced_out) {
  if (reduced_out || q8_dgrad_full_ok(g)) return 0;
  return (size_t)g.N * g.Ci * g.P * sizeof(float);
}

bool q8_shape_ok(const Geom& g) {
  // 64-bit sums where they are long; the int32 sums of q8_dgrad_k and q8_wgrad_pair_k stay in range
  return g.r > 1 && g.Og <= kMaxTerms32 && (long)(g.P / kThreads + 1) <= kMaxTerms32;
}

hipError_t launch_bwd_input_q8(const Geom& g, const int8_t* gy_q, const int8_t* w_q, float scale, void* g_x,
                               bool reduced_out, void* ws, hipStream_t st) {
  const float fscale = scale / ((float)g.s * (float)g.s);
  if (q8_dgrad_mfma_ok(g)) {   // many channels on both sides: matrix cores
    if (reduced_out || q8_dgrad_full_ok(g)) {
      const int rx = reduced_out ? 0 : g.rx;
      return g.dtype == GF_BF16 ? q8_dgrad_mfma_launch<bf16_t>(g, gy_q, w_q, fscale, g_x, rx, st)
                                : q8_dgrad_mfma_launch<float>(g, gy_q, w_q, fscale, g_x, rx, st);
    }
    hipError_t e = q8_dgrad_mfma_launch<float>(g, gy_q, w_q, fscale, ws, 0, st);
    if (e != hipSuccess) return e;
    return launch_expand_f32(g, static_cast<const float*>(ws), g_x, st);
  }
  if (reduced_out || q8_dgrad_full_ok(g))
    return g.dtype == GF_BF16 ? q8_dgrad_launch<bf16_t>(g, gy_q, w_q, fscale, g_x, !reduced_out, st)
                              : q8_dgrad_launch<float>(g, gy_q, w_q, fscale, g_x, !reduced_out, st);
  hipError_t e = q8_dgrad_launch<float>(g, gy_q, w_q, fscale, ws, false, st);
  if (e != hipSuccess) return e;
  return launch_expand_f32(g, static_cast<const float*>(ws), g_x, st);
}

}  // namespace gf
