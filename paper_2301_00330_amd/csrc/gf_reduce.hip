// Patch reduction: the gradient filter (Eq. 2, patch mean of g_y) and the
// activation pooling (text after Eq. 5, patch sum of x).  Both are one streaming
// read of an NCHW tensor, so everything here is about coalesced 16-byte loads.
//
//  * patch_reduce_rows  -- maps whose rows are 16-byte multiples and whose width
//    is a multiple of the patch: every lane loads one 16-byte vector from each of
//    the q rows of a patch-row strip, adds them vertically in registers and then
//    horizontally inside the vector; no LDS, no barrier, U independent strips per
//    lane in flight.
//  * patch_reduce_lds   -- every other shape (7x7, 14x14, ragged widths, odd q):
//    NCHW planes are treated as one flat stream; a block loads a contiguous run of
//    whole strips into LDS with 16-byte loads and each lane then sums one patch.
//  * patch_reduce_direct -- strips too large for LDS.
#include "gf_internal.h"

namespace gf {

namespace {

constexpr int kThreads = 256;
// what a reduction launch produces beside the patch sums / means
constexpr int kPlain = 0, kStats = 1, kMask = 2, kQ8 = 3;
constexpr int kLdsBudget = 32 * 1024;  // per block: 5 blocks fit a CU's 160 KB
constexpr int kLdsMax = 64 * 1024;

struct ReduceArgs {
  const void* in;
  void* out;
  int H, W, q, Hp, Wp;
  int total_in;      // planes * H * W
  int total_strips;  // planes * Hp
  int spb;           // strips per block (LDS kernel)
  int mean;
  int ipr;           // items per row (rows kernel)
  int total_items;   // total_strips * ipr
  FastDiv d_hp, d_wp, d_ipr;
  // side job (text after Eq. 3): blocks from ks_block0 on form kernel sums instead
  const void* ks_w;
  void* ks_out;
  int ks_pairs, ks_KK, ks_block0;
  float ks_qinv;   // > 0: the kernel sums are written as signed 8-bit codes
  // noise figures of the filter (kStats kernels): per-block partial sums {sum v^2, sum (v - patch mean)^2}
  float2* stats_part;
  // kMask kernels: out2[patch] = fraction of the patch's in-bounds elements with 0 < v < mask_hi
  void* out2;
  float mask_hi;
  // kQ8 kernels: `out` holds signed 8-bit codes of the patch sum / mean (see q8_code), q_inv = 1 / step size
  float q_inv;
};

// Fixed-order sum over the block of two floats per lane; block 0's lane 0 ... every block's
// lane 0 writes its pair.  `red` is 2 * (kThreads / 64) floats of LDS.
__device__ __forceinline__ void block_stats(float e, float n, float* red, float2* dst) {
  for (int m = 32; m > 0; m >>= 1) {
    e += __shfl_xor(e, m, 64);
    n += __shfl_xor(n, m, 64);
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { red[2 * wave] = e; red[2 * wave + 1] = n; }
  __syncthreads();
  if (threadIdx.x == 0) {
    float se = 0.f, sn = 0.f;
    for (int k = 0; k < kThreads / 64; ++k) { se += red[2 * k]; sn += red[2 * k + 1]; }
    dst[blockIdx.x] = make_float2(se, sn);
  }
}

// the kernel-sum side job; true if this block belongs to it (uniform for the block)
template <class T>
__device__ __forceinline__ bool ksum_side_job(const ReduceArgs& a) {
  if (a.ks_pairs == 0 || (int)blockIdx.x < a.ks_block0) return false;
  const int e = ((int)blockIdx.x - a.ks_block0) * kThreads + threadIdx.x;
  if (e < a.ks_pairs) {
    const float v = kernel_sum_of(static_cast<const T*>(a.ks_w), e, a.ks_KK);
    if (a.ks_qinv > 0.f) static_cast<int8_t*>(a.ks_out)[e] = q8_code(v, a.ks_qinv);
    else static_cast<T*>(a.ks_out)[e] = from_f32<T>(v);
  }
  return true;
}

// ---------------------------------------------------------------------------
// rows kernel: requires W % max(VE, Q) == 0 and (W * sizeof(T)) % 16 == 0
// ---------------------------------------------------------------------------
template <class T, int Q, int U, int MODE = kPlain>
__device__ __forceinline__ void rows_body(const ReduceArgs& a, const int blk) {
  constexpr bool STATS = MODE == kStats;
  __shared__ float red[STATS ? 2 * (kThreads / 64) : 1];
  float energy = 0.f, noise = 0.f;
  constexpr int VE = Vec16<T>::N;            // elements per 16-byte vector
  constexpr int IW = VE > Q ? VE : Q;        // elements of one row an item covers
  constexpr int VW = IW / VE;                // vectors per row per item
  constexpr int NOUT = IW / Q;               // patches per item
  const T* in = static_cast<const T*>(a.in);
  T* out = static_cast<T*>(a.out);
  uint4 v[U][Q][VW];
  int strip[U], col[U], rows[U];
  const int t0 = blk * (kThreads * U) + threadIdx.x;
  // all loads are issued unconditionally (indices clamped into the tensor) so that the
  // U * Q * VW vectors of a lane are in flight together; invalid ones are dropped below
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int t = t0 + u * kThreads;
    const int tc = min(t, a.total_items - 1);
    const int s = (int)a.d_ipr.div((uint32_t)tc);
    const int c = tc - s * a.ipr;
    const int pl = (int)a.d_hp.div((uint32_t)s);
    const int hp = s - pl * a.Hp;
    strip[u] = t < a.total_items ? s : -1;
    col[u] = c;
    rows[u] = min(Q, a.H - hp * Q);
    const T* p = in + ((long)pl * a.H + (long)hp * Q) * a.W + c * IW;
#pragma unroll
    for (int i = 0; i < Q; ++i) {
      const int ri = min(i, rows[u] - 1);
#pragma unroll
      for (int k = 0; k < VW; ++k)
        v[u][i][k] = load_stream16(p + (long)ri * a.W + k * VE);
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (strip[u] < 0) continue;
    float colsum[IW];
#pragma unroll
    for (int e = 0; e < IW; ++e) colsum[e] = 0.f;
#pragma unroll
    for (int i = 0; i < Q; ++i)
#pragma unroll
      for (int k = 0; k < VW; ++k) {
        float f[VE];
        Vec16<T>::unpack(v[u][i][k], f);
        const bool keep = i < rows[u];  // rows past the ragged edge were clamped
#pragma unroll
        for (int e = 0; e < VE; ++e) colsum[k * VE + e] += keep ? f[e] : 0.f;
      }
    const float den = a.mean ? (float)(rows[u] * Q) : 1.f;
    T res[NOUT];
    float mean[NOUT];
#pragma unroll
    for (int o = 0; o < NOUT; ++o) {
      float acc = 0.f;
#pragma unroll
      for (int j = 0; j < Q; ++j) acc += colsum[o * Q + j];
      mean[o] = acc / den;
      res[o] = from_f32<T>(mean[o]);
    }
    if constexpr (STATS) {  // second pass over the registers: energy and distance to the patch mean
#pragma unroll
      for (int i = 0; i < Q; ++i)
#pragma unroll
        for (int k = 0; k < VW; ++k) {
          float f[VE];
          Vec16<T>::unpack(v[u][i][k], f);
          const bool keep = i < rows[u];
#pragma unroll
          for (int e = 0; e < VE; ++e) {
            const float val = keep ? f[e] : 0.f;
            const float dv = keep ? f[e] - mean[(k * VE + e) / Q] : 0.f;
            energy += val * val;
            noise += dv * dv;
          }
        }
    }
    if constexpr (MODE == kMask) {  // second pass over the registers: how many elements pass a gradient
      T frac[NOUT];
#pragma unroll
      for (int o = 0; o < NOUT; ++o) {
        float cnt = 0.f;
#pragma unroll
        for (int i = 0; i < Q; ++i)
#pragma unroll
          for (int j = 0; j < Q; ++j) {
            const int e = o * Q + j;
            float f[VE];
            Vec16<T>::unpack(v[u][i][e / VE], f);
            const float val = f[e % VE];
            cnt += (i < rows[u] && val > 0.f && val < a.mask_hi) ? 1.f : 0.f;
          }
        frac[o] = from_f32<T>(cnt / (float)(rows[u] * Q));
      }
      T* d2 = static_cast<T*>(a.out2) + (long)strip[u] * a.Wp + col[u] * NOUT;
#pragma unroll
      for (int o = 0; o < NOUT; ++o) d2[o] = frac[o];
    }
    if constexpr (MODE == kQ8) {
      int8_t* d8 = static_cast<int8_t*>(a.out) + (long)strip[u] * a.Wp + col[u] * NOUT;
#pragma unroll
      for (int o = 0; o < NOUT; ++o) d8[o] = q8_code(mean[o], a.q_inv);
      continue;
    }
    T* dst = out + (long)strip[u] * a.Wp + col[u] * NOUT;
    if constexpr (NOUT * sizeof(T) == 8) {
      store_stream8(dst, *reinterpret_cast<const uint2*>(res));
    } else if constexpr (NOUT * sizeof(T) == 4) {
      store_stream4(dst, *reinterpret_cast<const uint32_t*>(res));
    } else {
#pragma unroll
      for (int o = 0; o < NOUT; ++o) dst[o] = res[o];
    }
  }
  if constexpr (STATS) block_stats(energy, noise, red, a.stats_part);
}

template <class T, int Q, int U, int MODE = kPlain>
__global__ __launch_bounds__(kThreads) void patch_reduce_rows(ReduceArgs a) {
  if (ksum_side_job<T>(a)) return;
  rows_body<T, Q, U, MODE>(a, blockIdx.x);
}

// ---------------------------------------------------------------------------
// LDS kernel: any shape whose strip fits the staging buffer
// ---------------------------------------------------------------------------
template <class T, int QT, int MODE = kPlain>  // QT: compile-time patch size, 0 = run-time
__device__ __forceinline__ void lds_body(const ReduceArgs& a, const int blk) {
  constexpr bool STATS = MODE == kStats;
  __shared__ float red[STATS ? 2 * (kThreads / 64) : 1];
  float energy = 0.f, noise = 0.f;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x;
  const int s0 = blk * a.spb;
  const int s1 = min(s0 + a.spb, a.total_strips);
  const int pl0 = (int)a.d_hp.div((uint32_t)s0);
  const int hp0 = s0 - pl0 * a.Hp;
  const int e0 = pl0 * a.H * a.W + hp0 * a.q * a.W;
  int e1 = a.total_in;
  if (s1 != a.total_strips) {
    const int pl1 = (int)a.d_hp.div((uint32_t)s1);
    e1 = pl1 * a.H * a.W + (s1 - pl1 * a.Hp) * a.q * a.W;
  }
  const long byte0 = (long)e0 * (long)sizeof(T);
  const long byte1 = (long)e1 * (long)sizeof(T);
  const long a0 = byte0 & ~15L;  // the tensor base is 16-byte aligned
  const int span = (int)(byte1 - a0);
  const int nvec = span >> 4;
  const uint4* src = reinterpret_cast<const uint4*>(static_cast<const unsigned char*>(a.in) + a0);
  uint4* dst = reinterpret_cast<uint4*>(smem);
  for (int v = tid; v < nvec; v += 4 * kThreads) {
    // four loads in flight per lane, no branches: past-the-end indices are clamped to the
    // last vector, which is then simply written again with the same bytes
    uint4 rg[4];
    int idx[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) idx[k] = min(v + k * kThreads, nvec - 1);
#pragma unroll
    for (int k = 0; k < 4; ++k) rg[k] = load_stream16(src + idx[k]);
#pragma unroll
    for (int k = 0; k < 4; ++k) dst[idx[k]] = rg[k];
  }
  {  // fewer than 16 trailing bytes: the range ends where the tensor ends
    const int tail0 = nvec << 4;
    const int ntail = (span - tail0) / (int)sizeof(T);
    if (tid < ntail)
      reinterpret_cast<T*>(smem + tail0)[tid] =
          reinterpret_cast<const T*>(reinterpret_cast<const unsigned char*>(src) + tail0)[tid];
  }
  __syncthreads();
  const T* lds = reinterpret_cast<const T*>(smem + (int)(byte0 - a0));  // lds[e - e0]
  T* out = static_cast<T*>(a.out);
  const int nout = (s1 - s0) * a.Wp;
  const int HW = a.H * a.W;
  for (int lo = tid; lo < nout; lo += kThreads) {
    const int ls = (int)a.d_wp.div((uint32_t)lo);
    const int wp = lo - ls * a.Wp;
    const int hq = hp0 + ls;                        // patch row counted from plane pl0
    const int dpl = (int)a.d_hp.div((uint32_t)hq);  // planes past pl0
    const int hp = hq - dpl * a.Hp;
    const int ch = min(a.q, a.H - hp * a.q);
    const int cw = min(a.q, a.W - wp * a.q);
    const int base = (pl0 + dpl) * HW + hp * a.q * a.W + wp * a.q - e0;
    const int q = QT ? QT : a.q;
    constexpr int UQ = QT ? QT : 1;  // unroll count of the q x q loops (1: run-time q, no unrolling)
    float acc = 0.f;
    // uniform q x q loop (no divergent branches): out-of-patch positions read the patch's
    // first element and are not added
#pragma unroll UQ
    for (int i = 0; i < q; ++i)
#pragma unroll UQ
      for (int j = 0; j < q; ++j) {
        const bool ok = i < ch && j < cw;
        const float val = to_f32(lds[base + (ok ? i * a.W + j : 0)]);
        acc += ok ? val : 0.f;
      }
    if (a.mean) acc = acc / (float)(ch * cw);
    if constexpr (MODE == kQ8)
      static_cast<int8_t*>(a.out)[s0 * a.Wp + lo] = q8_code(acc, a.q_inv);
    else
      out[s0 * a.Wp + lo] = from_f32<T>(acc);
    if constexpr (MODE == kMask) {
      float cnt = 0.f;
#pragma unroll UQ
      for (int i = 0; i < q; ++i)
#pragma unroll UQ
        for (int j = 0; j < q; ++j) {
          const bool ok = i < ch && j < cw;
          const float val = to_f32(lds[base + (ok ? i * a.W + j : 0)]);
          cnt += (ok && val > 0.f && val < a.mask_hi) ? 1.f : 0.f;
        }
      static_cast<T*>(a.out2)[s0 * a.Wp + lo] = from_f32<T>(cnt / (float)(ch * cw));
    }
    if constexpr (STATS) {
#pragma unroll UQ
      for (int i = 0; i < q; ++i)
#pragma unroll UQ
        for (int j = 0; j < q; ++j) {
          const bool ok = i < ch && j < cw;
          const float val = to_f32(lds[base + (ok ? i * a.W + j : 0)]);
          const float dv = val - acc;
          energy += ok ? val * val : 0.f;
          noise += ok ? dv * dv : 0.f;
        }
    }
  }
  if constexpr (STATS) block_stats(energy, noise, red, a.stats_part);
}

template <class T, int QT, int MODE = kPlain>
__global__ __launch_bounds__(kThreads) void patch_reduce_lds(ReduceArgs a) {
  if (ksum_side_job<T>(a)) return;
  lds_body<T, QT, MODE>(a, blockIdx.x);
}

// ---------------------------------------------------------------------------
// Several tensors in ONE launch (the activation pooling of all layers of a step): every block looks up
// the job its index falls into and runs that job's variant of the two kernels above.
// ---------------------------------------------------------------------------
constexpr int kMaxBatch = 16;
constexpr int kRowsBlocksCap = 2048;   // launched blocks of one register-variant job
enum { kVarRows2, kVarRows4, kVarRows8, kVarLds2, kVarLds4, kVarLds8, kVarLds0 };
struct BatchArgs {
  int njobs;
  int first_block[kMaxBatch + 1];   // of the launched blocks
  int variant[kMaxBatch];
  int nblocks[kMaxBatch];           // blocks of work of the job (register variant: walked by fewer launched blocks)
  ReduceArgs job[kMaxBatch];
};
static_assert(sizeof(BatchArgs) <= 3584, "the job table travels as a kernel argument");

template <class T, int MODE = kPlain>
__global__ __launch_bounds__(kThreads) void patch_reduce_batch_k(BatchArgs b) {
  int j = 0;
  while (j + 1 < b.njobs && (int)blockIdx.x >= b.first_block[j + 1]) ++j;
  const int blk = (int)blockIdx.x - b.first_block[j];
  const ReduceArgs& a = b.job[j];
  switch (b.variant[j]) {
    // the register variant has no barrier and no LDS: a launched block walks several blocks of work
    case kVarRows2: for (int w = blk; w < b.nblocks[j]; w += b.first_block[j + 1] - b.first_block[j]) rows_body<T, 2, 1, MODE>(a, w); break;
    case kVarRows4: for (int w = blk; w < b.nblocks[j]; w += b.first_block[j + 1] - b.first_block[j]) rows_body<T, 4, 1, MODE>(a, w); break;
    case kVarRows8: for (int w = blk; w < b.nblocks[j]; w += b.first_block[j + 1] - b.first_block[j]) rows_body<T, 8, 1, MODE>(a, w); break;
    case kVarLds2: lds_body<T, 2, MODE>(a, blk); break;
    case kVarLds4: lds_body<T, 4, MODE>(a, blk); break;
    case kVarLds8: lds_body<T, MODE == kPlain ? 8 : 0, MODE>(a, blk); break;   // as the single-tensor launch picks
    default: lds_body<T, 0, MODE>(a, blk); break;
  }
}

// Fallback without LDS for strips too large to stage: one lane per patch.
template <class T, int MODE = kPlain>
__global__ __launch_bounds__(kThreads) void patch_reduce_direct(ReduceArgs a) {
  constexpr bool STATS = MODE == kStats;
  if (ksum_side_job<T>(a)) return;
  __shared__ float red[STATS ? 2 * (kThreads / 64) : 1];
  float energy = 0.f, noise = 0.f;
  const T* in = static_cast<const T*>(a.in);
  T* out = static_cast<T*>(a.out);
  const long nout = (long)a.total_strips * a.Wp;
  for (long o = (long)blockIdx.x * kThreads + threadIdx.x; o < nout;
       o += (long)(a.ks_pairs ? a.ks_block0 : (int)gridDim.x) * kThreads) {
    const int strip = (int)(o / a.Wp);
    const int wp = (int)(o - (long)strip * a.Wp);
    const int pl = strip / a.Hp;
    const int hp = strip - pl * a.Hp;
    const int ch = min(a.q, a.H - hp * a.q);
    const int cw = min(a.q, a.W - wp * a.q);
    const T* p = in + (long)pl * a.H * a.W + (long)hp * a.q * a.W + wp * a.q;
    float acc = 0.f;
    for (int i = 0; i < ch; ++i)
      for (int j = 0; j < cw; ++j) acc += to_f32(p[(long)i * a.W + j]);
    if (a.mean) acc = acc / (float)(ch * cw);
    if constexpr (MODE == kQ8)
      static_cast<int8_t*>(a.out)[o] = q8_code(acc, a.q_inv);
    else
      out[o] = from_f32<T>(acc);
    if constexpr (MODE == kMask) {
      float cnt = 0.f;
      for (int i = 0; i < ch; ++i)
        for (int j = 0; j < cw; ++j) {
          const float val = to_f32(p[(long)i * a.W + j]);
          cnt += (val > 0.f && val < a.mask_hi) ? 1.f : 0.f;
        }
      static_cast<T*>(a.out2)[o] = from_f32<T>(cnt / (float)(ch * cw));
    }
    if constexpr (STATS) {
      for (int i = 0; i < ch; ++i)
        for (int j = 0; j < cw; ++j) {
          const float val = to_f32(p[(long)i * a.W + j]);
          energy += val * val;
          noise += (val - acc) * (val - acc);
        }
    }
  }
  if constexpr (STATS) block_stats(energy, noise, red, a.stats_part);
}

// stats[0] = sum of the blocks' energies, stats[1] = sum of their noise terms, in double: one
// block, every lane a strided share of the partials, then a fixed tree (same result every run)
constexpr int kFinalThreads = 1024;
__global__ __launch_bounds__(kFinalThreads) void stats_final_k(const float2* part, int n, double* stats) {
  __shared__ double red[2 * (kFinalThreads / 64)];
  double e = 0.0, v = 0.0;
  for (int i = threadIdx.x; i < n; i += kFinalThreads) {
    const float2 p = part[i];
    e += (double)p.x;
    v += (double)p.y;
  }
  for (int m = 32; m > 0; m >>= 1) {
    e += __shfl_xor(e, m, 64);
    v += __shfl_xor(v, m, 64);
  }
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (lane == 0) { red[2 * wave] = e; red[2 * wave + 1] = v; }
  __syncthreads();
  if (wave == 0) {
    e = lane < kFinalThreads / 64 ? red[2 * lane] : 0.0;
    v = lane < kFinalThreads / 64 ? red[2 * lane + 1] : 0.0;
    for (int m = 8; m > 0; m >>= 1) {
      e += __shfl_xor(e, m, 64);
      v += __shfl_xor(v, m, 64);
    }
    if (lane == 0) { stats[0] = e; stats[1] = v; }
  }
}

template <class T, int Q, int MODE>
hipError_t launch_rows(ReduceArgs& a, hipStream_t st, int* nblocks) {
  constexpr int VE = Vec16<T>::N;
  constexpr int IW = VE > Q ? VE : Q;
  constexpr int U = 1;
  a.ipr = a.W / IW;
  a.total_items = a.total_strips * a.ipr;
  a.d_ipr = FastDiv((uint32_t)a.ipr);
  const int blocks = cdiv(a.total_items, kThreads * U);
  a.ks_block0 = blocks;
  // the kernel-sum side job (plain mode only) runs in extra blocks at the end of the grid
  GF_LAUNCH((patch_reduce_rows<T, Q, U, MODE>), dim3(blocks + cdiv(a.ks_pairs, kThreads)), dim3(kThreads), 0, st, a);
  *nblocks = blocks;
  return hipGetLastError();
}

template <class T>
bool rows_ok(int W, int q) {
  constexpr int VE = Vec16<T>::N;
  if (q != 2 && q != 4 && q != 8) return false;
  const int IW = VE > q ? VE : q;
  return W % IW == 0 && (W * (int)sizeof(T)) % 16 == 0;
}

// One reduction launch in mode MODE.  *nblocks: the number of reduction blocks launched
// (side-job blocks not counted)
template <class T, int MODE>
hipError_t launch_mode(ReduceArgs& a, hipStream_t st, int* nblocks) {
  if (rows_ok<T>(a.W, a.q) && (long)a.total_strips * (a.W / 4) < 2147483647L) {
    if (a.q == 2) return launch_rows<T, 2, MODE>(a, st, nblocks);
    if (a.q == 4) return launch_rows<T, 4, MODE>(a, st, nblocks);
    return launch_rows<T, 8, MODE>(a, st, nblocks);
  }
  const long strip_bytes = (long)imin_host(a.q, a.H) * a.W * (long)sizeof(T);
  if (strip_bytes + 32 > kLdsMax) {
    a.spb = 1;
    const long nout = (long)a.total_strips * a.Wp;
    int blocks = (int)((nout + kThreads - 1) / kThreads);
    if (blocks > 65536) blocks = 65536;
    a.ks_block0 = blocks;
    GF_LAUNCH((patch_reduce_direct<T, MODE>), dim3(blocks + cdiv(a.ks_pairs, kThreads)), dim3(kThreads), 0, st, a);
    *nblocks = blocks;
    return hipGetLastError();
  }
  int spb = (int)((kLdsBudget - 32) / strip_bytes);
  if (spb < 1) spb = 1;
  // about four blocks per CU when the tensor is large enough (a block costs about the same few
  // microseconds whatever it stages: 1024 blocks measured 1.5 us per launch faster than 2048 on the
  // 3 - 6 MB maps of the ResNet-18 tail and equal on larger ones; 512 and 256 slower again)
  const int want_blocks = 1024;
  if (a.total_strips / spb < want_blocks) spb = a.total_strips / want_blocks;
  if (spb < 1) spb = 1;
  a.spb = spb;
  const size_t lds = (size_t)spb * strip_bytes + 32;
  const int blocks = (a.total_strips + spb - 1) / spb;
  a.ks_block0 = blocks;
  *nblocks = blocks;
  const dim3 grid(blocks + cdiv(a.ks_pairs, kThreads));
  if (a.q == 2)
    GF_LAUNCH((patch_reduce_lds<T, 2, MODE>), grid, dim3(kThreads), lds, st, a);
  else if (a.q == 4)
    GF_LAUNCH((patch_reduce_lds<T, 4, MODE>), grid, dim3(kThreads), lds, st, a);
  else if (MODE == kPlain && a.q == 8)   // the plain mode also has an unrolled variant for q = 8
    GF_LAUNCH((patch_reduce_lds<T, MODE == kPlain ? 8 : 0, MODE>), grid, dim3(kThreads), lds, st, a);
  else
    GF_LAUNCH((patch_reduce_lds<T, 0, MODE>), grid, dim3(kThreads), lds, st, a);
  return hipGetLastError();
}

// the mode follows from what the arguments ask for
template <class T>
hipError_t launch_t(ReduceArgs& a, hipStream_t st, int* nblocks) {
  if (a.q_inv > 0.f) return launch_mode<T, kQ8>(a, st, nblocks);
  if (a.stats_part) return launch_mode<T, kStats>(a, st, nblocks);
  if (a.out2) return launch_mode<T, kMask>(a, st, nblocks);
  return launch_mode<T, kPlain>(a, st, nblocks);
}

}  // namespace

// upper bound of the blocks any variant uses for this shape (size of the partial buffer)
long patch_reduce_max_blocks(long planes, int H, int W, int q) {
  const long strips = planes * cdiv(H, q);
  const long a = cdiv(strips * cdiv(W, 4), kThreads) + 1;   // rows variant: at least 4 elements per item
  const long b = strips + 1;                                // LDS variant: at least one strip per block
  const long c = 65536;                                     // direct variant
  return (a > b ? a : b) > c ? (a > b ? a : b) : c;
}

hipError_t launch_filter_stats(const void* g_y, void* gy_u, long planes, int H, int W, int q, int dtype,
                               float* part, double* stats, hipStream_t st) {
  ReduceArgs a = {};
  int blocks = 0;
  a.stats_part = reinterpret_cast<float2*>(part);
  a.in = g_y; a.out = gy_u; a.H = H; a.W = W; a.q = q;
  a.Hp = cdiv(H, q); a.Wp = cdiv(W, q);
  a.total_in = (int)(planes * H * W);
  a.total_strips = (int)(planes * a.Hp);
  a.mean = 1;
  a.d_hp = FastDiv((uint32_t)a.Hp);
  a.d_wp = FastDiv((uint32_t)a.Wp);
  hipError_t e = dtype == GF_BF16 ? launch_t<bf16_t>(a, st, &blocks) : launch_t<float>(a, st, &blocks);
  if (e != hipSuccess) return e;
  GF_LAUNCH(stats_final_k, dim3(1), dim3(kFinalThreads), 0, st, a.stats_part, blocks, stats);
  return hipGetLastError();
}

template <class T>
__global__ __launch_bounds__(kThreads) void mask_mul_k(T* dst, const T* m, long n) {
  const long e = (long)blockIdx.x * kThreads + threadIdx.x;
  if (e < n) dst[e] = from_f32<T>(to_f32(dst[e]) * to_f32(m[e]));
}

hipError_t launch_mask_mul(void* dst, const void* m, long n, int dtype, hipStream_t st) {
  const dim3 grid((unsigned)((n + kThreads - 1) / kThreads)), block(kThreads);
  if (dtype == GF_BF16)
    GF_LAUNCH(mask_mul_k<bf16_t>, grid, block, 0, st, static_cast<bf16_t*>(dst), static_cast<const bf16_t*>(m), n);
  else
    GF_LAUNCH(mask_mul_k<float>, grid, block, 0, st, static_cast<float*>(dst), static_cast<const float*>(m), n);
  return hipGetLastError();
}

hipError_t launch_pool_mask(const void* x, void* x_u, void* m_u, long planes, int H, int W, int q, float hi,
                            int dtype, hipStream_t st) {
  ReduceArgs a = {};
  int blocks = 0;
  a.in = x; a.out = x_u; a.out2 = m_u; a.mask_hi = hi; a.H = H; a.W = W; a.q = q;
  a.Hp = cdiv(H, q); a.Wp = cdiv(W, q);
  a.total_in = (int)(planes * H * W);
  a.total_strips = (int)(planes * a.Hp);
  a.mean = 0;
  a.d_hp = FastDiv((uint32_t)a.Hp);
  a.d_wp = FastDiv((uint32_t)a.Wp);
  return dtype == GF_BF16 ? launch_t<bf16_t>(a, st, &blocks) : launch_t<float>(a, st, &blocks);
}

hipError_t launch_patch_reduce_q8(const void* in, int8_t* out_q, long planes, int H, int W, int q, bool mean,
                                  float inv_delta, int dtype, hipStream_t st, const KsumJob* ksum) {
  ReduceArgs a = {};
  int blocks = 0;
  if (ksum) {
    a.ks_w = ksum->w; a.ks_out = ksum->out; a.ks_pairs = ksum->pairs; a.ks_KK = ksum->KK; a.ks_qinv = ksum->q_inv;
  }
  a.in = in; a.out = out_q; a.q_inv = inv_delta; a.H = H; a.W = W; a.q = q;
  a.Hp = cdiv(H, q); a.Wp = cdiv(W, q);
  a.total_in = (int)(planes * H * W);
  a.total_strips = (int)(planes * a.Hp);
  a.mean = mean ? 1 : 0;
  a.d_hp = FastDiv((uint32_t)a.Hp);
  a.d_wp = FastDiv((uint32_t)a.Wp);
  return dtype == GF_BF16 ? launch_t<bf16_t>(a, st, &blocks) : launch_t<float>(a, st, &blocks);
}

hipError_t launch_patch_reduce(const void* in, void* out, long planes, int H, int W, int q,
                               bool mean, int dtype, hipStream_t st, const KsumJob* ksum) {
  ReduceArgs a = {};
  int blocks = 0;
  if (ksum) {
    a.ks_w = ksum->w; a.ks_out = ksum->out; a.ks_pairs = ksum->pairs; a.ks_KK = ksum->KK; a.ks_qinv = ksum->q_inv;
  }
  a.in = in;
  a.out = out;
  a.H = H;
  a.W = W;
  a.q = q;
  a.Hp = cdiv(H, q);
  a.Wp = cdiv(W, q);
  a.total_in = (int)(planes * H * W);
  a.total_strips = (int)(planes * a.Hp);
  a.mean = mean ? 1 : 0;
  a.d_hp = FastDiv((uint32_t)a.Hp);
  a.d_wp = FastDiv((uint32_t)a.Wp);
  if (dtype == GF_BF16) return launch_t<bf16_t>(a, st, &blocks);
  return launch_t<float>(a, st, &blocks);
}

// How launch_mode would run this plain reduction: the variant and its block count (and a.spb / a.ipr ...
// filled in), or false when it needs the kernel without LDS.
// block_bytes: how much of its tensor a block of the LDS variant should stage (capped by the LDS budget)
template <class T>
static bool plan_plain(ReduceArgs& a, long block_bytes, int* variant, int* blocks, size_t* lds) {
  *lds = 0;
  if (rows_ok<T>(a.W, a.q) && (long)a.total_strips * (a.W / 4) < 2147483647L) {
    constexpr int VE = Vec16<T>::N;
    const int IW = VE > a.q ? VE : a.q;
    a.ipr = a.W / IW;
    a.total_items = a.total_strips * a.ipr;
    a.d_ipr = FastDiv((uint32_t)a.ipr);
    *blocks = cdiv(a.total_items, kThreads);
    *variant = a.q == 2 ? kVarRows2 : a.q == 4 ? kVarRows4 : kVarRows8;
    return true;
  }
  const long strip_bytes = (long)imin_host(a.q, a.H) * a.W * (long)sizeof(T);
  if (strip_bytes + 32 > kLdsMax) return false;
  int spb = (int)((kLdsBudget - 32) / strip_bytes);
  if (spb < 1) spb = 1;
  if ((long)spb * strip_bytes > block_bytes) spb = (int)(block_bytes / strip_bytes);
  if (spb < 1) spb = 1;
  a.spb = spb;
  *lds = (size_t)spb * strip_bytes + 32;
  *blocks = (a.total_strips + spb - 1) / spb;
  *variant = a.q == 2 ? kVarLds2 : a.q == 4 ? kVarLds4 : a.q == 8 ? kVarLds8 : kVarLds0;
  return true;
}

template <class T>
static hipError_t batch_t(const PoolJob* jobs, int count, hipStream_t st) {
  const bool codes = count > 0 && jobs[0].q_inv > 0.f;   // all jobs of a call write codes, or none does
  // Blocks of the LDS variant: as large as the LDS budget allows, as long as the whole call still has
  // about eight blocks per CU.  A block costs about the same few microseconds whatever it stages
  // (kernel arguments, job table, one round of loads, a barrier), and the tensors of a call fill
  // the chip together: measured on the ten tensors of the MobileNetV2 tail, 2048 blocks per tensor
  // 79 us (fp32) / 53 us (bf16), 28 KB blocks 66 / 44 us, 64 KB blocks (two per CU) 80 / 62 us.
  long bytes_total = 0;
  for (int k = 0; k < count; ++k) bytes_total += jobs[k].planes * jobs[k].H * jobs[k].W * (long)sizeof(T);
  long block_bytes = bytes_total / 2048;
  if (block_bytes < 4096) block_bytes = 4096;
  int i = 0;
  while (i < count) {
    BatchArgs b = {};
    size_t lds_max = 0;
    int blocks_total = 0;
    while (i < count && b.njobs < kMaxBatch) {
      const PoolJob& pj = jobs[i];
      ReduceArgs a = {};
      a.in = pj.in; a.out = pj.out; a.H = pj.H; a.W = pj.W; a.q = pj.q;
      a.Hp = cdiv(pj.H, pj.q); a.Wp = cdiv(pj.W, pj.q);
      a.total_in = (int)(pj.planes * pj.H * pj.W);
      a.total_strips = (int)(pj.planes * a.Hp);
      a.mean = 0;
      a.q_inv = pj.q_inv;
      a.d_hp = FastDiv((uint32_t)a.Hp);
      a.d_wp = FastDiv((uint32_t)a.Wp);
      int variant = 0, blocks = 0;
      size_t lds = 0;
      if (!plan_plain<T>(a, block_bytes, &variant, &blocks, &lds)) {   // a strip larger than LDS: a launch of its own
        if (b.njobs > 0) break;
        const int dt = sizeof(T) == 2 ? GF_BF16 : GF_F32;
        hipError_t e = codes ? launch_patch_reduce_q8(pj.in, static_cast<int8_t*>(pj.out), pj.planes, pj.H, pj.W, pj.q,
                                                      false, pj.q_inv, dt, st, nullptr)
                             : launch_patch_reduce(pj.in, pj.out, pj.planes, pj.H, pj.W, pj.q, false, dt, st, nullptr);
        if (e != hipSuccess) return e;
        ++i;
        continue;
      }
      b.first_block[b.njobs] = blocks_total;
      b.variant[b.njobs] = variant;
      b.nblocks[b.njobs] = blocks;
      b.job[b.njobs] = a;
      ++b.njobs;
      // Thin blocks are dispatch-bound: a register-variant job launches at most kRowsBlocksCap blocks
      // (eight per CU), each walking its share of the job (measured on the MobileNetV2 and DeepLab
      // tails: 32 -> 29 us and 45 -> 40 us for the whole call).
      blocks_total += (variant <= kVarRows8 && blocks > kRowsBlocksCap) ? kRowsBlocksCap : blocks;
      if (lds > lds_max) lds_max = lds;
      ++i;
    }
    if (b.njobs == 0) continue;
    b.first_block[b.njobs] = blocks_total;
    if (codes) GF_LAUNCH((patch_reduce_batch_k<T, kQ8>), dim3(blocks_total), dim3(kThreads), lds_max, st, b);
    else GF_LAUNCH((patch_reduce_batch_k<T, kPlain>), dim3(blocks_total), dim3(kThreads), lds_max, st, b);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_pool_batch(const PoolJob* jobs, int count, int dtype, hipStream_t st) {
  return dtype == GF_BF16 ? batch_t<bf16_t>(jobs, count, st) : batch_t<float>(jobs, count, st);
}

// true when launch_patch_reduce sums a patch in the order of the register kernel (columns first)
bool patch_reduce_uses_rows(int dtype, long planes, int H, int W, int q) {
  const bool ok = dtype == GF_BF16 ? rows_ok<bf16_t>(W, q) : rows_ok<float>(W, q);
  return ok && planes * cdiv(H, q) * (W / 4) < 2147483647L;
}

}  // namespace gf
