// Dense layers (groups == 1) on small maps -- the 7x7 / 14x14 tails of ResNet and MobileNetV2 --
// in TWO launches per layer:
//
//   1. dense_prep_k: the gradient filter (Eq. 2) over runs of whole planes staged in LDS; the patch
//      means leave the block three times over: in the caller's layout [N, C_y, P] (if wanted), as
//      GYT [C_y][J] (row = output channel, J = N * P columns) and as GYN [J][C_y] (row = patch).
//      Extra blocks at the head of the grid relay x_u to XUT [C_x][J], form the kernel sums
//      (text after Eq. 3) as WT [C_x][C_y], clear the K padding of all four matrices and zero the
//      tickets of launch 2.  With these layouts both contractions are plain "NT" products of
//      matrices with K contiguous and padded to whole chunks.  The four matrices are stored
//      blocked: [64-row tile][K chunk][64 rows][128 bytes], so the operand tile a block needs
//      for one chunk is ONE contiguous 8 KB run (a row-major matrix would make it 64 pieces of
//      128 bytes, 8 KB apart: measured three to five times slower):
//        weight gradient (Eq. 5):  g_th~[co][ci] = sum_j  GYT[co][j]  * XUT[ci][j]
//        input gradient  (Eq. 3):  g_x~u[ci][j]  = sum_co WT[ci][co]  * GYN[j][co]
//      so neither the patch count of a plane (49, 16, 4 ...) nor image boundaries show up in the
//      operand loaders any more.
//   2. dense_gemm_k: one grid whose blocks are (tile, K slab) pairs of the two products.  Operands
//      go global -> registers (three chunks ahead) -> LDS -> 16-byte fragment reads ->
//      v_mfma_f32_32x32x16_bf16.  fp32 operands are split on their way into LDS into three bf16
//      terms each (x = t0 + t1 + t2 exactly) and a product is accumulated from the six term products
//      of order <= 2 in fp32: six bf16 matrix instructions cost 6/16 of the fp32 ones they replace,
//      and the result is as close to the fp64 reference as that of v_mfma_f32_16x16x4_f32 (measured
//      rms error 2 - 3.5e-7 of the rms gradient either way; 244 -> 222 us for the seven layers of the
//      MobileNetV2 tail).  A slab's partial tile goes
//      to the workspace; the block that takes the last ticket of a tile adds the slabs in slab
//      order (so the result does not depend on which block that is) and runs the epilogue:
//      scale and replicate to the K_h x K_w taps, or round once and write whole planes of g_x
//      (a lane forms 16 bytes of the run at a time, every pixel taking its patch's value).
//      No separate slab-sum launch, no float atomics.
//
// Blocks are numbered so that the blocks one XCD receives (block index mod 8) share operands:
// a K slab of the weight gradient, a group of images of the input gradient.
#include "gf_internal.h"
#include "gf_mma.h"
#include <algorithm>

namespace gf {

bool patch_reduce_uses_rows(int dtype, long planes, int H, int W, int q);  // gf_reduce.hip

namespace {

constexpr int kT = 256;
constexpr int kPitch = 128 + 16;       // bytes of one staged operand row
constexpr int kTile = 64;              // block tile (rows and columns)
constexpr int kPrepInBytes = 24 * 1024;

template <class T> struct El;
template <> struct El<float> { static constexpr int KB = 32, VE = 4; };    // elements per 128-byte chunk / 16-byte vector
template <> struct El<bf16_t> { static constexpr int KB = 64, VE = 8; };

// element (row, k) of a blocked matrix with `chunks` K chunks of KB elements
template <int KB>
__device__ __forceinline__ long blk(int row, int k, int chunks) {
  return ((long)(row >> 6) * chunks + k / KB) * (64 * KB) + (row & 63) * KB + k % KB;
}

// ---------------------------------------------------------------------------
// launch 1: filter + relayout
// ---------------------------------------------------------------------------
struct PrepArgs {
  const void* in;      // [planes][H][W]: g_y, or gy_u itself with q = 1
  int planes, C, H, W, q, Hp, Wp, P, mean, vfirst, R;
  int pw_log;          // log2 of the patch count padded to a power of two (lanes per plane slot)
  long total_in;       // planes * H * W
  FastDiv d_p, d_wp, d_c;
  void* gyu;           // nullable [planes][P]
  void* gyt;           // nullable, blocked [C][kpj]
  void* gyn;           // nullable, blocked [64 * column tiles][kpc]: row 64 * (n / ipt) + (n % ipt) * P + p, so
                       // that a column tile of the input gradient (ipt whole images) is one 64-row tile
  int ipt, gyn_rows;
  FastDiv d_ipt;
  int J, kpj, kpc;     // J = N * P; K extents padded to whole chunks: columns [J, kpj) resp. [Co, kpc) are zeroed
  int chj, chc;        // chunks per row: kpj / KB, kpc / KB
  // side jobs
  const void* xu;      // nullable [N][Ci][P] -> xut, blocked [Ci][kpj]
  void* xut;
  int Ci, nxu;         // nxu = N * Ci * P
  FastDiv d_cip;       // / (Ci * P)
  int relay_t, N;      // relay_t: x_u goes through LDS in pieces of 8 images x 8 channels (16-byte loads and stores)
  FastDiv d_nvi;       // / (8 * P / VE), the vectors of one image's piece
  const void* w;       // nullable [Co][Ci][KK] -> wt, blocked [Ci][kpc], kernel sums rounded to the storage type
  void* wt;
  int Co, KK;
  int* tickets;
  int ntickets;
  int blk_w0, blk_pad0, blk_red0;   // block ranges: [x_u relay | kernel sums | padding and tickets | filter runs]
};

template <class T>
__device__ __forceinline__ void prep_side_jobs(const PrepArgs& a, unsigned char* smem) {
  constexpr int KB = El<T>::KB;
  const int b = blockIdx.x, tid = threadIdx.x;
  T* xut = static_cast<T*>(a.xut);
  T* wt = static_cast<T*>(a.wt);
  if (b < a.blk_w0) {   // x_u [n][ci][p] -> XUT [ci][n * P + p]
    // a few hundred blocks that each walk their share (a block costs about the same whatever it moves);
    // 16-byte pieces where the patches of a plane are a whole number of vectors
    constexpr int VE = El<T>::VE;
    const T* xu = static_cast<const T*>(a.xu);
    if (a.relay_t) {
      // The patches of a plane are no whole number of vectors (7 x 7 patches): a piece of 8 images x 8 channels
      // is read with 16-byte loads (the 8 planes of an image are one aligned run), laid out in LDS as 8 rows
      // [c][n * P + p], and every row leaves as 16-byte stores -- it is a run of 8 P columns of XUT that starts
      // on a vector boundary.  (Element by element this relay took 18 us for 14.5 MB.)
      T* rows = reinterpret_cast<T*>(smem);
      const int pitch = 8 * a.P + VE;
      const int nvi = 8 * a.P / VE, nv = 8 * nvi;
      const int cgroups = a.Ci >> 3, items = (a.N >> 3) * cgroups;
      for (int item = b; item < items; item += a.blk_w0) {
        const int ng = item / cgroups, n0 = ng * 8, ci0 = (item - ng * cgroups) * 8;
        __syncthreads();   // the rows of the previous piece have been stored
        for (int v0 = tid; v0 < nv; v0 += 4 * kT) {
          u32x4_t r[4];
          int n[4], kk[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const int idx = min(v0 + k * kT, nv - 1);
            n[k] = (int)a.d_nvi.div((uint32_t)idx);
            kk[k] = idx - n[k] * nvi;
            r[k] = *reinterpret_cast<const u32x4_t*>(xu + ((long)(n0 + n[k]) * a.Ci + ci0) * a.P + kk[k] * VE);
          }
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            if (v0 + k * kT >= nv) continue;
            const T* el = reinterpret_cast<const T*>(&r[k]);
#pragma unroll
            for (int j = 0; j < VE; ++j) {
              const int e = kk[k] * VE + j;
              const int cl = (int)a.d_p.div((uint32_t)e);
              rows[cl * pitch + n[k] * a.P + e - cl * a.P] = el[j];
            }
          }
        }
        __syncthreads();
        for (int v = tid; v < nv; v += kT) {
          const int cl = (int)a.d_nvi.div((uint32_t)v), kk = v - cl * nvi;
          *reinterpret_cast<u32x4_t*>(xut + blk<KB>(ci0 + cl, n0 * a.P + kk * VE, a.chj)) =
              *reinterpret_cast<const u32x4_t*>(rows + cl * pitch + kk * VE);
        }
      }
      return;
    }
    const int step = a.blk_w0 * kT;
    // eight loads of a lane are in flight together (one at a time, the walk paid a memory latency per step:
    // 18 us for the 14.5 MB of the 576-channel 14 x 14 layer)
    constexpr int NB = 8;
    auto dest = [&](int e) __attribute__((always_inline)) {
      const int n = (int)a.d_cip.div((uint32_t)e);
      const int rem = e - n * a.Ci * a.P;
      const int ci = (int)a.d_p.div((uint32_t)rem);
      return blk<KB>(ci, n * a.P + rem - ci * a.P, a.chj);
    };
    if (a.P % VE == 0) {
      const int nv = a.nxu / VE;
      for (int v0 = b * kT + tid; v0 < nv; v0 += NB * step) {
        u32x4_t r[NB];
#pragma unroll
        for (int k = 0; k < NB; ++k) r[k] = *reinterpret_cast<const u32x4_t*>(xu + (long)min(v0 + k * step, nv - 1) * VE);
#pragma unroll
        for (int k = 0; k < NB; ++k)
          if (v0 + k * step < nv) *reinterpret_cast<u32x4_t*>(xut + dest((v0 + k * step) * VE)) = r[k];
      }
      return;
    }
    for (int e0 = b * kT + tid; e0 < a.nxu; e0 += NB * step) {
      T r[NB];
#pragma unroll
      for (int k = 0; k < NB; ++k) r[k] = xu[min(e0 + k * step, a.nxu - 1)];
#pragma unroll
      for (int k = 0; k < NB; ++k)
        if (e0 + k * step < a.nxu) xut[dest(e0 + k * step)] = r[k];
    }
    return;
  }
  if (b < a.blk_pad0) {  // WT [ci][co] = spatial sum of theta[co][ci], rounded once (1x1: theta itself)
    // 32 x 32 tiles through LDS: reads run along c_i (the kernels of one c_o are contiguous), writes along c_o
    __shared__ float tile[32][33];
    const T* w = static_cast<const T*>(a.w);
    const int tb = b - a.blk_w0;
    const int tiles_ci = (a.Ci + 31) / 32;
    const int co0 = (tb / tiles_ci) * 32, ci0 = (tb % tiles_ci) * 32;
    const int c = tid & 31, r8 = tid >> 5;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int co = co0 + r8 + 8 * k, ci = ci0 + c;
      float v = 0.f;
      if (co < a.Co && ci < a.Ci) {
        const long pair = (long)co * a.Ci + ci;
        v = a.KK == 1 ? to_f32(w[pair]) : to_f32(from_f32<T>(kernel_sum_of(w, pair, a.KK)));
      }
      tile[r8 + 8 * k][c] = v;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int ci = ci0 + r8 + 8 * k, co = co0 + c;
      if (co < a.Co && ci < a.Ci) wt[blk<KB>(ci, co, a.chc)] = from_f32<T>(tile[c][r8 + 8 * k]);
    }
    return;
  }
  // K padding of the four matrices, tickets
  const int padj = a.kpj - a.J, padc = a.kpc - a.Co;
  const int lane0 = (b - a.blk_pad0) * kT + tid, step = (a.blk_red0 - a.blk_pad0) * kT;
  const T zero = from_f32<T>(0.f);
  if (padj > 0) {
    if (a.gyt)
      for (int e = lane0; e < a.C * padj; e += step) static_cast<T*>(a.gyt)[blk<KB>(e / padj, a.J + e % padj, a.chj)] = zero;
    if (a.xut)
      for (int e = lane0; e < a.Ci * padj; e += step) xut[blk<KB>(e / padj, a.J + e % padj, a.chj)] = zero;
  }
  if (padc > 0) {
    if (a.gyn)
      for (int e = lane0; e < a.gyn_rows * padc; e += step) static_cast<T*>(a.gyn)[blk<KB>(e / padc, a.Co + e % padc, a.chc)] = zero;
    if (a.wt)
      for (int e = lane0; e < a.Ci * padc; e += step) wt[blk<KB>(e / padc, a.Co + e % padc, a.chc)] = zero;
  }
  for (int e = lane0; e < a.ntickets; e += step) a.tickets[e] = 0;
}

template <class T>
__global__ __launch_bounds__(kT) void dense_prep_k(PrepArgs a) {
  // side jobs first: their blocks start first and overlap with the filter blocks
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  if ((int)blockIdx.x < a.blk_red0) { prep_side_jobs<T>(a, smem); return; }
  constexpr int VE = El<T>::VE;
  constexpr int MAXV = kPrepInBytes / 16 / kT;   // 16-byte vectors of a run per lane
  const int tid = threadIdx.x;
  const int HW = a.H * a.W;
  T* lin = reinterpret_cast<T*>(smem);
  T* lout = lin + ((a.R * HW + VE - 1) / VE) * VE;   // [planes of the run][P + 1]
  const int PP = a.P + 1;
  const int q = a.q;
  const int nruns = (a.planes + a.R - 1) / a.R;
  const int stride = (int)gridDim.x - a.blk_red0;
  // A block walks runs of R whole planes (contiguous, 16-byte aligned starts: R is a multiple of 8);
  // the next run's loads are in flight while the current one is reduced and written.
  u32x4_t v[MAXV];
  auto prefetch = [&](int run) __attribute__((always_inline)) {
    const int pl0 = run * a.R;
    const int nvec = min(a.R, a.planes - pl0) * HW / VE;
    const u32x4_t* src = reinterpret_cast<const u32x4_t*>(static_cast<const T*>(a.in) + (long)pl0 * HW);
    if (nvec == 0) return;   // a tensor shorter than one vector: its elements are copied one by one below
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
      const int k = tid + i * kT;
      v[i] = __builtin_nontemporal_load(src + min(k, nvec - 1));   // clamped: always issued
    }
  };
  // patch of this lane: tx = patch index (padded to a power of two), ty = plane slot
  const int tx = tid & ((1 << a.pw_log) - 1), ty = tid >> a.pw_log;
  const int txc = min(tx, a.P - 1);
  const int hp = (int)a.d_wp.div((uint32_t)txc), wp = txc - hp * a.Wp;
  const int ch = min(q, a.H - hp * q), cw = min(q, a.W - wp * q);
  const int poff = hp * q * a.W + wp * q;
  const int cnt = ch * cw;
  const bool cnt_pow2 = (cnt & (cnt - 1)) == 0;
  const float inv_cnt = 1.f / (float)cnt;
  int run = (int)blockIdx.x - a.blk_red0;
  if (run < nruns) prefetch(run);
  for (; run < nruns; run += stride) {
    const int pl0 = run * a.R;
    const int npl = min(a.R, a.planes - pl0);
    const int nel = npl * HW, nvec = nel / VE;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
      const int k = tid + i * kT;
      if (k < nvec) reinterpret_cast<u32x4_t*>(lin)[k] = v[i];
    }
    {  // fewer than 16 trailing bytes (only where the tensor ends)
      const T* src = static_cast<const T*>(a.in) + (long)pl0 * HW;
      for (int e = nvec * VE + tid; e < nel; e += kT) lin[e] = src[e];
    }
    if (run + stride < nruns) prefetch(run + stride);
    __syncthreads();
    // first plane of the run as (image, channel); the run's planes follow in channel order
    const int n0 = (int)a.d_c.div((uint32_t)pl0), c0 = pl0 - n0 * a.C;
    // lane = (plane slot, patch): the patch geometry is fixed per lane (no divisions inside the loops).  The
    // lane that forms a mean also stores it in the caller's layout and as GYT; GYN goes through LDS.
    if (tx < a.P) {
      const int slots = kT >> a.pw_log;
      auto emit = [&](int pl, float acc) __attribute__((always_inline)) {
        // a power-of-two count divides exactly either way; anything else takes the true quotient
        if (a.mean) acc = cnt_pow2 ? acc * inv_cnt : acc / (float)(ch * cw);
        const T val = from_f32<T>(acc);
        lout[pl * PP + tx] = val;
        if (a.gyu) static_cast<T*>(a.gyu)[((long)pl0 + pl) * a.P + tx] = val;   // caller's layout: one contiguous run
        if (a.gyt) {                                                           // row = channel, runs of P along j
          int n = n0, c = c0 + pl;
          while (c >= a.C) { c -= a.C; ++n; }
          static_cast<T*>(a.gyt)[blk<El<T>::KB>(c, n * a.P + tx, a.chj)] = val;
        }
      };
      if (q == 2) {
        // the four values of a patch are read at offsets clamped into the patch and the ones past a ragged
        // edge are left out of the sum; two planes per pass, so eight LDS reads are in flight (with loops
        // over the true extent every read waited for the one before: 2.7 us for 24 planes of 14 x 14)
        const bool wide = cw > 1, tall = ch > 1;
        const int o01 = wide ? 1 : 0, o10 = tall ? a.W : 0, o11 = o10 + o01;
        for (int pl = ty; pl < npl; pl += 2 * slots) {
          const bool two = pl + slots < npl;
          const T* b0 = lin + pl * HW + poff;
          const T* b1 = lin + (two ? pl + slots : pl) * HW + poff;
          const float v[2][4] = {{to_f32(b0[0]), to_f32(b0[o01]), to_f32(b0[o10]), to_f32(b0[o11])},
                                 {to_f32(b1[0]), to_f32(b1[o01]), to_f32(b1[o10]), to_f32(b1[o11])}};
          float acc[2];
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            if (a.vfirst) {   // the order of the register kernel of gf_filter_grad: columns first, then across
              float c0s = 0.f + v[u][0], c1s = 0.f + v[u][1];
              c0s = tall ? c0s + v[u][2] : c0s;
              c1s = tall ? c1s + v[u][3] : c1s;
              acc[u] = 0.f + c0s;
              acc[u] = wide ? acc[u] + c1s : acc[u];
            } else {          // the order of its LDS kernel: row by row
              acc[u] = 0.f + v[u][0];
              acc[u] = wide ? acc[u] + v[u][1] : acc[u];
              acc[u] = tall ? acc[u] + v[u][2] : acc[u];
              acc[u] = (tall && wide) ? acc[u] + v[u][3] : acc[u];
            }
          }
          emit(pl, acc[0]);
          if (two) emit(pl + slots, acc[1]);
        }
      } else {
        for (int pl = ty; pl < npl; pl += slots) {
          const T* base = lin + pl * HW + poff;
          float acc = 0.f;
          if (a.vfirst) {
            for (int j = 0; j < cw; ++j) {
              float col = 0.f;
              for (int i = 0; i < ch; ++i) col += to_f32(base[i * a.W + j]);
              acc += col;
            }
          } else {
            for (int i = 0; i < ch; ++i)
              for (int j = 0; j < cw; ++j) acc += to_f32(base[i * a.W + j]);
          }
          emit(pl, acc);
        }
      }
    }
    __syncthreads();
    if (a.gyn) {   // row = (n, p), consecutive lanes = consecutive channels (32 plane slots x 8 patches per pass)
      T* d = static_cast<T*>(a.gyn);
      for (int pl = tid & 31; pl < npl; pl += 32) {
        int n = n0, c = c0 + pl;
        while (c >= a.C) { c -= a.C; ++n; }
        const int tn = (int)a.d_ipt.div((uint32_t)n);
        const int row0 = 64 * tn + (n - tn * a.ipt) * a.P;
        T r[8];   // at most 64 patches per plane: eight per lane, read together
#pragma unroll
        for (int k = 0; k < 8; ++k) r[k] = lout[pl * PP + min((tid >> 5) + 8 * k, a.P - 1)];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int pch = (tid >> 5) + 8 * k;
          if (pch < a.P) d[blk<El<T>::KB>(row0 + pch, c, a.chc)] = r[k];
        }
      }
    }
    __syncthreads();   // lin and lout are rewritten by the next run
  }
}

// ---------------------------------------------------------------------------
// launch 2: both products, split over K slabs, finished by the last block of each tile
// ---------------------------------------------------------------------------
struct GemmArgs {
  int Ci, Co, N, P, J, KK;
  // weight gradient: C[co][ci], K = j
  const void* gyt;     // blocked (see the head of the file)
  const void* xut;
  float* g_w;
  float wscale;
  float* partW;
  int* tickW;
  int w_tm, w_tn, w_nz, w_cpz, w_chunks, nW, nW8;
  // input gradient: C[ci][j], K = co; a column tile holds `ipt` whole images
  const void* wt;
  const void* gyn;
  void* out;           // [N, Ci, H, W], or [N, Ci, P] with `reduced`
  const void* mask;    // nullable [N, Ci, P] (reduced only)
  int reduced;
  float dscale;
  float* partD;
  int* tickD;
  int d_tm, d_tn, d_nz, d_cpz, d_chunks, nD, nD8;
  int ipt, H, W, Wp, rx, HW;
  FastDiv d_p, d_kk, d_w, d_rx, d_hw;
};

// Accumulators of a wave: one 32 x 32 tile of v_mfma_f32_32x32x16_bf16 (fp32 operands enter it as three
// bf16 terms each, see below); row of the tile that element v of lane `lane` holds (the column is lane % 32)
typedef f32x16 acc_t;
constexpr int kBase = 32, kNV = 16;
__device__ __forceinline__ int acc_row(int lane, int v) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

// Four fp32 values as three bf16 terms, x = t0 + t1 + t2 exactly: every term is the nearest bf16 of what the
// earlier ones leave (|t1| <= 2^-8 |x|, |t2| <= 2^-16 |x|), both remainders are exact in fp32, and the second
// has at most 8 significant bits.  A product x y is taken as the six term products of order <= 2; the three
// that are dropped stay below 2^-23 |x y| (2^-24 at most and 2^-27 rms over random operands): the size of one
// rounding of the fp32 accumulation.  One packed
// conversion per pair of values and term, two shifts / masks and two subtractions per pair and remainder.
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void split3(const u32x4_t& v, uint2 (&t)[3]) {
  f32x2_t a = {__uint_as_float(v.x), __uint_as_float(v.y)}, b = {__uint_as_float(v.z), __uint_as_float(v.w)};
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    // one packed conversion per pair (round to nearest even)
    const uint32_t pa = __builtin_bit_cast(uint32_t, __builtin_convertvector(a, bf16x2_t));
    const uint32_t pb = __builtin_bit_cast(uint32_t, __builtin_convertvector(b, bf16x2_t));
    t[k] = make_uint2(pa, pb);
    if (k < 2) {
      a.x -= bf_lo(pa); a.y -= bf_hi(pa);
      b.x -= bf_lo(pb); b.y -= bf_hi(pb);
    }
  }
}
constexpr int kPitchS = 64 + 16;             // bytes of one staged row of one term (32 k as bf16)
constexpr int kTermBytes = kTile * kPitchS;  // one term of an operand tile

// Barrier between the waves of a block that orders LDS traffic only.  __syncthreads() also waits
// for every global load in flight (its fence covers all address spaces), which would end the
// prefetch of the next chunk at every barrier: measured 1.7 us per chunk instead of 0.4.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// acc += A[rows of tile ta][chunks kc0 .. kc1) * B[rows of tile tb][same chunks]^T for blocked operands with
// `chunks` chunks per row; every wave owns one 32 x 32 quadrant of the 64 x 64 tile.
template <class T>
__device__ __forceinline__ void mainloop(const T* A, int ta, const T* B, int tb, int chunks, int kc0, int kc1,
                                         unsigned char* As, unsigned char* Bs,
                                         acc_t& acc) {
  constexpr int KB = El<T>::KB, VE = El<T>::VE;
  constexpr bool SPLIT = sizeof(T) == 4;   // fp32 operands: three bf16 terms each, six products
  constexpr int LV = kTile * 8 / kT;   // 16-byte vectors per lane, operand and chunk
  static_assert(2 * kBase == kTile, "tile shape");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  // the tile of one chunk is 8 KB of consecutive memory in the order of the LDS tile
  const T* pa = A + (long)ta * chunks * (64 * KB) + tid * VE;
  const T* pb = B + (long)tb * chunks * (64 * KB) + tid * VE;
  // A global load takes 1.5 - 2 us here, four chunks of fp32 MFMA work (a block alone on its CU runs
  // the loop at latency / chunks in flight), so three chunks are kept in flight in registers beside the
  // one in LDS; four register sets with fixed roles per step (arrays indexed at run time, or arrays of
  // HIP's uint4 class handed to a lambda, would live in scratch memory).
  u32x4_t a0[LV], b0[LV], a1[LV], b1[LV], a2[LV], b2[LV], a3[LV], b3[LV];
  auto fetch = [&](u32x4_t (&qa)[LV], u32x4_t (&qb)[LV], int kc) __attribute__((always_inline)) {
    const long off = (long)min(kc, kc1 - 1) * (64 * KB);   // past the end: the last chunk again (never staged)
#pragma unroll
    for (int i = 0; i < LV; ++i) {
      qa[i] = *reinterpret_cast<const u32x4_t*>(pa + off + i * (kT * VE));
      qb[i] = *reinterpret_cast<const u32x4_t*>(pb + off + i * (kT * VE));
    }
  };
  // chunk kc: registers (ca, cb) -> LDS, the load of chunk kc + 3 into (na, nb), then the MFMAs
  auto step = [&](u32x4_t (&ca)[LV], u32x4_t (&cb)[LV], u32x4_t (&na)[LV], u32x4_t (&nb)[LV], int kc, bool more)
                  __attribute__((always_inline)) {
    if constexpr (SPLIT) {   // a vector of four k becomes 8 bytes in each of the three term tiles
#pragma unroll
      for (int i = 0; i < LV; ++i) {
        const int s = tid + i * kT;
        uint2 sa[3], sb[3];
        split3(ca[i], sa);
        split3(cb[i], sb);
#pragma unroll
        for (int t = 0; t < 3; ++t) {
          *reinterpret_cast<uint2*>(As + t * kTermBytes + (s >> 3) * kPitchS + (s & 7) * 8) = sa[t];
          *reinterpret_cast<uint2*>(Bs + t * kTermBytes + (s >> 3) * kPitchS + (s & 7) * 8) = sb[t];
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < LV; ++i) {
        const int s = tid + i * kT;
        *reinterpret_cast<u32x4_t*>(As + (s >> 3) * kPitch + (s & 7) * 16) = ca[i];
        *reinterpret_cast<u32x4_t*>(Bs + (s >> 3) * kPitch + (s & 7) * 16) = cb[i];
      }
    }
    lds_barrier();
    if (more) fetch(na, nb, kc + 3);
    if constexpr (SPLIT) {
      const int r = lane & 31, kg = lane >> 5;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {   // 16 k per MFMA, 32 per chunk
        uint4 fa[3], fb[3];
#pragma unroll
        for (int t = 0; t < 3; ++t) {
          fa[t] = *reinterpret_cast<const uint4*>(As + t * kTermBytes + (wm * 32 + r) * kPitchS + ks * 32 + kg * 16);
          fb[t] = *reinterpret_cast<const uint4*>(Bs + t * kTermBytes + (wn * 32 + r) * kPitchS + ks * 32 + kg * 16);
        }
        // smallest products first
        acc = mma32(fa[2], fb[0], acc);
        acc = mma32(fa[0], fb[2], acc);
        acc = mma32(fa[1], fb[1], acc);
        acc = mma32(fa[1], fb[0], acc);
        acc = mma32(fa[0], fb[1], acc);
        acc = mma32(fa[0], fb[0], acc);
      }
    } else {
      const int r = lane & 31, kg = lane >> 5;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {   // 16 k per MFMA, 64 per chunk
        const uint4 fa = *reinterpret_cast<const uint4*>(As + (wm * 32 + r) * kPitch + ks * 32 + kg * 16);
        const uint4 fb = *reinterpret_cast<const uint4*>(Bs + (wn * 32 + r) * kPitch + ks * 32 + kg * 16);
        acc = mma32(fa, fb, acc);
      }
    }
    lds_barrier();
  };
  fetch(a0, b0, kc0);
  fetch(a1, b1, kc0 + 1);
  fetch(a2, b2, kc0 + 2);
  // whole rounds of four steps without a branch inside (the compiler then knows how many loads are in
  // flight at every wait; with conditional steps it drains all of them at the loop head), then the
  // at most three chunks that are left, already on their way
  int kc = kc0;
  for (; kc + 4 <= kc1; kc += 4) {
    step(a0, b0, a3, b3, kc, true);
    step(a1, b1, a0, b0, kc + 1, true);
    step(a2, b2, a1, b1, kc + 2, true);
    step(a3, b3, a2, b2, kc + 3, true);
  }
  if (kc < kc1) step(a0, b0, a3, b3, kc, false);
  if (kc + 1 < kc1) step(a1, b1, a0, b0, kc + 1, false);
  if (kc + 2 < kc1) step(a2, b2, a1, b1, kc + 2, false);
}

// Slab data crosses XCDs inside one launch.  Every XCD has an L2 of its own, and a device-wide
// release / acquire fence writes back resp. invalidates that whole L2, which every block of the grid
// would pay (measured: 5 - 8 x the run time of the whole launch).  The slabs therefore move with
// relaxed device-scope atomic stores and loads, which go through to the memory side and never
// leave a stale or dirty line in an L2; the ticket is a device-scope atomic as well, and the
// stores of a block are complete (workgroup-scope release + barrier) before its ticket is taken.
__device__ __forceinline__ void slab_store(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float slab_load(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The partial tile of this block goes to its slab in the workspace in the order the lanes hold it
// (element e of lane t at slab[e * 256 + t]: every store and load is one contiguous 1 KB run per
// wave), then the ticket.  The block that arrives last -- all slabs of the tile are complete by
// then -- returns true with acc = slab 0 + slab 1 + ... in slab order, whichever block it is.
__device__ __forceinline__ bool reduce_slabs(acc_t& acc, float* slabs, int z, int* ticket, int nz, int* s_flag) {
  constexpr int NE = kNV;   // 16 floats per lane
  const int tid = threadIdx.x;
  float* mine = slabs + (long)z * kTile * kTile + tid;
#pragma unroll
  for (int v = 0; v < NE; ++v) slab_store(mine + v * kT, acc[v]);
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // this wave's stores have completed ...
  __syncthreads();                                          // ... and so have the other waves'
  if (tid == 0) *s_flag = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == nz - 1;
  __syncthreads();
  if (*s_flag == 0) return false;
  // four slabs' loads in flight at a time, additions in slab order
  constexpr int ZB = 4;
  float s[NE];
#pragma unroll
  for (int e = 0; e < NE; ++e) s[e] = 0.f;
  const float* p0 = slabs + tid;
  for (int z0 = 0; z0 < nz; z0 += ZB) {
    float t[ZB][NE];
#pragma unroll
    for (int zz = 0; zz < ZB; ++zz)
#pragma unroll
      for (int e = 0; e < NE; ++e)
        t[zz][e] = slab_load(p0 + (long)min(z0 + zz, nz - 1) * kTile * kTile + e * kT);   // clamped: always issued
#pragma unroll
    for (int zz = 0; zz < ZB; ++zz)
#pragma unroll
      for (int e = 0; e < NE; ++e)
        if (z0 + zz < nz) s[e] += t[zz][e];
  }
#pragma unroll
  for (int v = 0; v < NE; ++v) acc[v] = s[v];
  return true;
}

// the finished tile from the registers into Cs[kTile][kTile + 1]
__device__ __forceinline__ void gather_tile(const acc_t& acc, float* Cs) {
  constexpr int SC = kTile + 1;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
  for (int v = 0; v < kNV; ++v)
    Cs[(wm * kBase + acc_row(lane, v)) * SC + wn * kBase + (lane & (kBase - 1))] = acc[v];
}

template <class T>
__device__ __forceinline__ void wgrad_block(const GemmArgs& a, int L, unsigned char* smem, int* s_flag) {
  acc_t acc;
#pragma unroll
  for (int v = 0; v < kNV; ++v) acc[v] = 0.f;
  const int tiles = a.w_tm * a.w_tn;
  const int z = L / tiles, t = L - z * tiles;
  const int tmi = t / a.w_tn, tni = t - tmi * a.w_tn;
  const int m0 = tmi * kTile, n0 = tni * kTile;
  const int kc0 = z * a.w_cpz, kc1 = min(kc0 + a.w_cpz, a.w_chunks);
  mainloop<T>(static_cast<const T*>(a.gyt), tmi, static_cast<const T*>(a.xut), tni, a.w_chunks, kc0, kc1,
                         smem, smem + (sizeof(T) == 4 ? 3 * kTermBytes : kTile * kPitch), acc);
  if (a.w_nz > 1 &&
      !reduce_slabs(acc, a.partW + (long)t * a.w_nz * kTile * kTile, z, a.tickW + t, a.w_nz, s_flag))
    return;
  constexpr int SC = kTile + 1;
  float* Cs = reinterpret_cast<float*>(smem);
  const int tid = threadIdx.x;
  const int ncol = min(kTile, a.Ci - n0);
  const int run = ncol * a.KK;   // one c_o row of the tile is one contiguous run of g_w
  __syncthreads();
  gather_tile(acc, Cs);
  __syncthreads();
  const int nr = min(kTile, a.Co - m0);
  // All rows in one flat loop of 16-byte stores (a row of the tile is ncol * KK floats, a multiple of 8, and starts
  // on a 16-byte boundary: C_x and n0 are multiples of 8); row and position advance without a division.  Row by
  // row with one float per lane, a 1 x 1 layer kept 64 of 256 lanes busy for 64 passes: 6 - 7 us per tile, 12.6 us
  // with 3 x 3 taps, on the critical path of the launch.
  const int rv = run >> 2, total = nr * rv;          // vectors per row, vectors of the tile
  const int dq = kT / rv, dm = kT - dq * rv;
  int row = tid / rv, rr = tid - row * rv;
#pragma unroll 4
  for (int v = tid; v < total; v += kT) {
    f32x4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = Cs[row * SC + (int)a.d_kk.div((uint32_t)(rr * 4 + j))] * a.wscale;
    *reinterpret_cast<f32x4*>(a.g_w + ((long)(m0 + row) * a.Ci + n0) * a.KK + rr * 4) = o;
    rr += dm; row += dq;
    if (rr >= rv) { rr -= rv; ++row; }
  }
}

template <class T>
__device__ __forceinline__ void dgrad_block(const GemmArgs& a, int L, unsigned char* smem, int* s_flag) {
  acc_t acc;
#pragma unroll
  for (int v = 0; v < kNV; ++v) acc[v] = 0.f;
  // image group slowest: the blocks one XCD receives share their rows of GYN
  const int per_group = a.d_tm * a.d_nz;
  const int tni = L / per_group, rem = L - tni * per_group;
  const int z = rem / a.d_tm, tmi = rem - z * a.d_tm;
  const int t = tni * a.d_tm + tmi;
  const int m0 = tmi * kTile;                 // first c_i
  const int img0 = tni * a.ipt;               // first image
  const int kc0 = z * a.d_cpz, kc1 = min(kc0 + a.d_cpz, a.d_chunks);
  mainloop<T>(static_cast<const T*>(a.wt), tmi, static_cast<const T*>(a.gyn), tni, a.d_chunks, kc0, kc1,
                         smem, smem + (sizeof(T) == 4 ? 3 * kTermBytes : kTile * kPitch), acc);
  if (a.d_nz > 1 &&
      !reduce_slabs(acc, a.partD + (long)t * a.d_nz * kTile * kTile, z, a.tickD + t, a.d_nz, s_flag))
    return;
  constexpr int SC = kTile + 1;
  float* Cs = reinterpret_cast<float*>(smem);
  int* patch_of = reinterpret_cast<int*>(smem + kTile * SC * sizeof(float));   // [H * W]: patch of a pixel
  const int tid = threadIdx.x;
  const int nimg = min(a.ipt, a.N - img0);
  const int nr = min(kTile, a.Ci - m0);
  T* out = static_cast<T*>(a.out);
  const T* mask = static_cast<const T*>(a.mask);
  constexpr int VE = El<T>::VE;
  __syncthreads();
  gather_tile(acc, Cs);
  if (!a.reduced)
    for (int p = tid; p < a.HW; p += kT) {
      const int h = (int)a.d_w.div((uint32_t)p), w = p - h * a.W;
      patch_of[p] = (int)a.d_rx.div((uint32_t)h) * a.Wp + (int)a.d_rx.div((uint32_t)w);
    }
  __syncthreads();
  if (a.reduced) {   // one value per patch: the rows of an image are one contiguous run of nr * P
    for (int il = 0; il < nimg; ++il) {
      const long o0 = ((long)(img0 + il) * a.Ci + m0) * a.P;
      for (int e = tid; e < nr * a.P; e += kT) {
        const int row = (int)a.d_p.div((uint32_t)e);
        T v = from_f32<T>(Cs[row * SC + il * a.P + e - row * a.P] * a.dscale);
        if (mask) v = from_f32<T>(to_f32(v) * to_f32(mask[o0 + e]));
        out[o0 + e] = v;
      }
    }
    return;
  }
  // Full resolution: the nr planes (n, m0 ...) of an image are one contiguous run that starts on a 16-byte
  // boundary; a lane forms 16 bytes of it at a time -- every pixel takes the value of its patch, rounded
  // once -- and stores them (a pass through an LDS image of the planes, written patch by patch, took
  // 3.6 us per 32 rows here against 0.8 us for the tile's gather).
  const int nel = nr * a.HW, nvec = nel / VE;
  if (nvec > 0) {   // the runs of all images of the tile in one loop, a few vectors of a lane in flight
    const int dq = kT / nvec, dm = kT - dq * nvec;
    int il = tid / nvec, v = tid - il * nvec;
#pragma unroll 4
    for (int idx = tid; idx < nimg * nvec; idx += kT) {
      int row = (int)a.d_hw.div((uint32_t)(v * VE));
      int pix = v * VE - row * a.HW;
      const float* Ci_ = Cs + il * a.P;
      __attribute__((aligned(16))) T vals[VE];
#pragma unroll
      for (int k = 0; k < VE; ++k) {
        vals[k] = from_f32<T>(Ci_[row * SC + patch_of[pix]] * a.dscale);
        if (++pix == a.HW) { pix = 0; ++row; }
      }
      store_stream16(reinterpret_cast<uint4*>(out + ((long)(img0 + il) * a.Ci + m0) * a.HW) + v,
                     *reinterpret_cast<const uint4*>(vals));
      v += dm; il += dq;
      if (v >= nvec) { v -= nvec; ++il; }
    }
  }
  for (int il = 0; il < nimg; ++il) {   // fewer than 16 trailing bytes of a run (storage types of 2 bytes only)
    T* d = out + ((long)(img0 + il) * a.Ci + m0) * a.HW;
    const float* Ci_ = Cs + il * a.P;
    for (int e = nvec * VE + tid; e < nel; e += kT) {
      const int row = (int)a.d_hw.div((uint32_t)e);
      d[e] = from_f32<T>(Ci_[row * SC + patch_of[e - row * a.HW]] * a.dscale);
    }
  }
}

constexpr int kEpilogueBytes = kTile * (kTile + 1) * 4 + 256 * 4;   // the tile as floats, the patch of every pixel of a plane
constexpr int gemm_smem_bytes(int elem_bytes) {
  const int operands = elem_bytes == 4 ? 2 * 3 * kTermBytes : 2 * kTile * kPitch;
  return operands > kEpilogueBytes ? operands : kEpilogueBytes;
}

template <class T>
__global__ __launch_bounds__(kT) void dense_gemm_k(GemmArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[gemm_smem_bytes(sizeof(T))];
  __shared__ int s_flag;
  // blocks b, b + 8, b + 16 ... run on one XCD: give them consecutive work items of one product
  int b = blockIdx.x;
  if (b < a.nW8) {
    const int L = (b & 7) * (a.nW8 >> 3) + (b >> 3);
    if (L < a.nW) wgrad_block<T>(a, L, smem, &s_flag);
    return;
  }
  b -= a.nW8;
  const int L = (b & 7) * (a.nD8 >> 3) + (b >> 3);
  if (L < a.nD) dgrad_block<T>(a, L, smem, &s_flag);
}

long round_up(long v, long m) { return (v + m - 1) / m * m; }

struct Plan {
  long kpj, kpc;
  int w_tm, w_tn, w_nz, w_cpz, w_chunks;
  int d_tm, d_tn, d_nz, d_cpz, d_chunks, ipt;
  size_t off_tick, off_gyt, off_xut, off_gyn, off_wt, off_pw, off_pd, total;
};

int slabs_for(int tiles, int chunks, int want_blocks) {
  int nz = cdiv(want_blocks, tiles);
  const int most = chunks / 4 > 1 ? chunks / 4 : 1;   // at least four chunks per block
  if (nz > most) nz = most;
  if (nz < 1) nz = 1;
  return nz;
}

Plan make_plan(const Geom& g, bool want_w, bool want_d) {
  Plan p;
  const int KB = g.b == 2 ? 64 : 32;
  const long J = (long)g.N * g.P;
  p.kpj = round_up(J, KB);      // K extents padded to whole chunks
  p.kpc = round_up(g.Co, KB);
  p.w_tm = cdiv(g.Co, kTile);
  p.w_tn = cdiv(g.Ci, kTile);
  p.w_chunks = (int)(p.kpj / KB);
  // K slabs: enough (tile, slab) blocks for about three per CU over both products; the run time
  // was measured flat between 256 and 1024 blocks per product
  constexpr int want_w_blocks = 384, want_d_blocks = 384;
  p.w_nz = slabs_for(p.w_tm * p.w_tn, p.w_chunks, want_w_blocks);
  p.w_cpz = cdiv(p.w_chunks, p.w_nz);
  p.w_nz = cdiv(p.w_chunks, p.w_cpz);
  p.ipt = kTile / g.P;
  p.d_tm = cdiv(g.Ci, kTile);
  p.d_tn = cdiv(g.N, p.ipt);
  p.d_chunks = (int)(p.kpc / KB);
  p.d_nz = slabs_for(p.d_tm * p.d_tn, p.d_chunks, want_d_blocks);
  p.d_cpz = cdiv(p.d_chunks, p.d_nz);
  p.d_nz = cdiv(p.d_chunks, p.d_cpz);
  auto al = [](size_t v) { return (v + 255) & ~(size_t)255; };
  size_t o = 0;
  p.off_tick = o; o += al(((size_t)p.w_tm * p.w_tn + (size_t)p.d_tm * p.d_tn) * sizeof(int));
  // blocked matrices hold whole 64-row tiles (rows past the last channel are never written and only
  // feed outputs that are never stored)
  p.off_gyt = o; if (want_w) o += al((size_t)p.w_tm * kTile * p.kpj * g.b);
  p.off_xut = o; if (want_w) o += al((size_t)p.w_tn * kTile * p.kpj * g.b);
  p.off_gyn = o; if (want_d) o += al((size_t)p.d_tn * kTile * p.kpc * g.b);
  p.off_wt = o; if (want_d) o += al((size_t)p.d_tm * kTile * p.kpc * g.b);
  p.off_pw = o; if (want_w && p.w_nz > 1) o += al((size_t)p.w_tm * p.w_tn * p.w_nz * kTile * kTile * sizeof(float));
  p.off_pd = o; if (want_d && p.d_nz > 1) o += al((size_t)p.d_tm * p.d_tn * p.d_nz * kTile * kTile * sizeof(float));
  p.total = o;
  return p;
}

int prep_planes_per_block(const Geom& g, int H, int W) {
  int R = kPrepInBytes / (H * W * g.b) / 8 * 8;
  const int most = 128 / g.b;   // runs of about 6 KB on 7 x 7 maps: 32 fp32 planes, 64 bf16 planes
  if (R > most) R = most;
  if (R < 8) R = 8;
  return R;
}

template <class T>
hipError_t launch_t(const Geom& g, const void* src, bool src_is_gy, const void* x_u, const void* w, void* gy_u_out,
                    float* g_w, void* g_x, bool reduced, const void* mask_u, void* ws, hipStream_t st) {
  const bool want_w = g_w != nullptr, want_d = g_x != nullptr;
  const Plan p = make_plan(g, want_w, want_d);
  char* wsb = static_cast<char*>(ws);
  const int J = g.N * g.P;
  PrepArgs a;
  a.in = src;
  a.planes = g.N * g.Co;
  a.C = g.Co;
  if (src_is_gy) { a.H = g.Hy; a.W = g.Wy; a.q = g.r; a.mean = 1; }
  else { a.H = g.Hp; a.W = g.Wp; a.q = 1; a.mean = 0; }
  a.Hp = g.Hp; a.Wp = g.Wp; a.P = g.P;
  a.vfirst = src_is_gy && patch_reduce_uses_rows(g.dtype, a.planes, a.H, a.W, a.q) ? 1 : 0;
  a.R = prep_planes_per_block(g, a.H, a.W);
  a.pw_log = 0;
  while ((1 << a.pw_log) < g.P) ++a.pw_log;
  a.total_in = (long)a.planes * a.H * a.W;
  a.d_p = FastDiv((uint32_t)g.P);
  a.d_wp = FastDiv((uint32_t)g.Wp);
  a.d_c = FastDiv((uint32_t)g.Co);
  a.gyu = gy_u_out;
  a.gyt = want_w ? wsb + p.off_gyt : nullptr;
  a.gyn = want_d ? wsb + p.off_gyn : nullptr;
  a.J = J; a.kpj = (int)p.kpj; a.kpc = (int)p.kpc;
  a.chj = p.w_chunks; a.chc = p.d_chunks;
  a.ipt = p.ipt; a.gyn_rows = p.d_tn * kTile; a.d_ipt = FastDiv((uint32_t)p.ipt);
  a.xu = want_w ? x_u : nullptr;
  a.xut = want_w ? wsb + p.off_xut : nullptr;
  a.Ci = g.Ci;
  a.nxu = g.N * g.Ci * g.P;
  a.d_cip = FastDiv((uint32_t)(g.Ci * g.P));
  a.w = want_d ? w : nullptr;
  a.wt = want_d ? wsb + p.off_wt : nullptr;
  a.Co = g.Co; a.KK = g.KK;
  a.tickets = reinterpret_cast<int*>(wsb + p.off_tick);
  a.ntickets = p.w_tm * p.w_tn + p.d_tm * p.d_tn;
  a.N = g.N;
  a.relay_t = (g.P % El<T>::VE != 0 && g.N % 8 == 0) ? 1 : 0;
  a.d_nvi = FastDiv((uint32_t)(8 * g.P / El<T>::VE));
  a.blk_w0 = !want_w ? 0 : a.relay_t ? imin_host((g.N / 8) * (g.Ci / 8), 512)
                                     : imin_host(cdiv(g.P % El<T>::VE == 0 ? a.nxu / El<T>::VE : a.nxu, kT), 512);
  a.blk_pad0 = a.blk_w0 + (want_d ? cdiv(g.Ci, 32) * cdiv(g.Co, 32) : 0);
  a.blk_red0 = a.blk_pad0 + 8;
  // filter blocks: at most eight per CU, each walks its share of the runs
  const int nruns = cdiv(a.planes, a.R);
  const int nred = nruns < 2048 ? nruns : 2048;
  const int VE = El<T>::VE;
  size_t lds = (size_t)((a.R * a.H * a.W + VE - 1) / VE * VE + a.R * (g.P + 1)) * sizeof(T) + 16;
  if (a.relay_t && want_w) lds = std::max(lds, (size_t)8 * (8 * g.P + VE) * sizeof(T));
  GF_LAUNCH(dense_prep_k<T>, dim3(a.blk_red0 + nred), dim3(kT), lds, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;

  GemmArgs q;
  q.Ci = g.Ci; q.Co = g.Co; q.N = g.N; q.P = g.P; q.J = J; q.KK = g.KK;
  q.gyt = a.gyt; q.xut = a.xut;
  q.g_w = g_w;
  q.wscale = 1.f / ((float)g.s * (float)g.s);
  q.partW = reinterpret_cast<float*>(wsb + p.off_pw);
  q.tickW = a.tickets;
  q.w_tm = p.w_tm; q.w_tn = p.w_tn; q.w_nz = p.w_nz; q.w_cpz = p.w_cpz; q.w_chunks = p.w_chunks;
  q.nW = want_w ? p.w_tm * p.w_tn * p.w_nz : 0;
  q.nW8 = (q.nW + 7) & ~7;
  q.wt = a.wt; q.gyn = a.gyn;
  q.out = g_x; q.mask = reduced ? mask_u : nullptr; q.reduced = reduced ? 1 : 0;
  q.dscale = q.wscale;
  q.partD = reinterpret_cast<float*>(wsb + p.off_pd);
  q.tickD = a.tickets + p.w_tm * p.w_tn;
  q.d_tm = p.d_tm; q.d_tn = p.d_tn; q.d_nz = p.d_nz; q.d_cpz = p.d_cpz; q.d_chunks = p.d_chunks;
  q.nD = want_d ? p.d_tm * p.d_tn * p.d_nz : 0;
  q.nD8 = (q.nD + 7) & ~7;
  q.ipt = p.ipt; q.H = g.H; q.W = g.W; q.Wp = g.Wp; q.rx = g.rx; q.HW = g.H * g.W;
  q.d_p = a.d_p; q.d_kk = FastDiv((uint32_t)g.KK);
  q.d_w = FastDiv((uint32_t)g.W); q.d_rx = FastDiv((uint32_t)g.rx); q.d_hw = FastDiv((uint32_t)(g.H * g.W));
  GF_LAUNCH(dense_gemm_k<T>, dim3(q.nW8 + q.nD8), dim3(kT), 0, st, q);
  return hipGetLastError();
}

}  // namespace

// Layers this path takes: dense, filtered, at most 64 patches per plane (a column tile of the
// input gradient is whole images) and at least 4 (at most sixteen images per tile), planes of at most 256
// pixels, C_x a multiple of 8 (every run of planes the epilogue stores then starts on a 16-byte
// boundary) -- the shapes on which it measured faster than filter -> merged launch -> finalize
// (gf_mfma.hip).  Measured on MI355X, whole backward of a layer, this path against the general one:
//   one image per column tile (P > 32: 14 x 14 and 16 x 16 maps at r = 2), 1 x 1 and 3 x 3 kernels,
//     N = 32 ... 128: 47 / 76, 34 / 46 us (512 and 256 channels 3 x 3), 55 / 85, 46 / 80 us (96 <-> 576);
//   four images per tile (P = 16: 7 x 7 maps at r = 2, 14 x 14 at r = 4): 1 x 1 kernels 54 / 72, 38 / 63,
//     36 / 47, 30 / 41, 27 / 29 us; 3 x 3 kernels at r_x = 4 33 / 35, 28 / 29 us;
//   16 images per tile (P = 4: 7 x 7 maps at r = 4): 512 channels 3 x 3, bf16, 23 / 31 us -- taken while a
//     tile's share of g_x stays below 256 KB (256 -> 512 channels, stride 2, 14 x 14 planes: 16 tiles of 401 KB,
//     44 / 27 us); 64 images per tile (P = 1), measured with an earlier epilogue: 280 - 295 / 32 - 106 us: not taken;
//   with bf16 storage the contractions cost a sixteenth and a layer is a chain of fixed costs either way:
//     1 x 1 kernels (MobileNetV2 tail, seven layers) 218 / 234 us; 3 x 3 kernels (ResNet-18 tail) 24 / 25,
//     23 / 21 (stride 2), 23 / 27 us at r = 2 and 22 / 21 us at r = 4: taken as well.
bool dense_ok(const Geom& g) {
  if (g.g != 1 || g.r == 1) return false;
  if (g.P > kTile || (long)g.H * g.W > 256 || (long)g.Hy * g.Wy > 256) return false;
  const int ipt = kTile / g.P;   // images per column tile of the input gradient
  // a finishing block of the input gradient stores the planes of all images of its tile: 64 rows x ipt planes
  if (ipt > 16 || (long)kTile * ipt * g.H * g.W * g.b > 256 * 1024) return false;
  if (g.Ci % 8 != 0) return false;
  // 32-bit indices into the blocked matrices
  const long KB = g.b == 2 ? 64 : 32;
  const long J = (long)g.N * g.P;
  const long lim = (1L << 31) - (1L << 20);
  const long rows = round_up(g.Co > g.Ci ? g.Co : g.Ci, kTile);
  if (rows * round_up(J, KB) > lim || ((long)g.N + 1) * kTile * round_up(g.Co, KB) > lim) return false;
  return true;
}

size_t ws_dense(const Geom& g, bool want_w, bool want_d) { return make_plan(g, want_w, want_d).total; }

hipError_t launch_dense(const Geom& g, const void* src, bool src_is_gy, const void* x_u, const void* w,
                        void* gy_u_out, float* g_w, void* g_x, bool reduced, const void* mask_u, void* ws,
                        hipStream_t st) {
  if (g.dtype != GF_F32) return launch_t<bf16_t>(g, src, src_is_gy, x_u, w, gy_u_out, g_w, g_x, reduced, mask_u, ws, st);
  return launch_t<float>(g, src, src_is_gy, x_u, w, gy_u_out, g_w, g_x, reduced, mask_u, ws, st);
}

}  // namespace gf
