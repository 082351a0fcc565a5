// Patch reduction: the gradient filter (Eq. 2, patch mean of g_y) and the
// activation pooling (text after Eq. 5, patch sum of x).  Both are one streaming
// read of an NCHW tensor, so the kernel is built around coalesced 16-byte loads
// of a flat run of whole patch-row strips into LDS, from which each lane sums
// one patch.  NCHW planes are treated as one flat stream: a block's input range
// is contiguous in memory whatever H, W and q are (7x7 planes included).
#include "gf_internal.h"

namespace gf {

namespace {

constexpr int kThreads = 256;
constexpr int kLdsBudget = 32 * 1024;  // per block: 5 blocks fit a CU's 160 KB
constexpr int kLdsMax = 64 * 1024;

struct ReduceArgs {
  const void* in;
  void* out;
  int H, W, q, Hp, Wp;
  int total_in;      // planes * H * W
  int total_strips;  // planes * Hp
  int spb;           // strips per block
  int mean;
};

// element offset of strip s = (plane, hp): rows hp*q .. of that plane
__device__ __forceinline__ int strip_offset(const ReduceArgs& a, int s) {
  int pl = s / a.Hp;
  int hp = s - pl * a.Hp;
  return pl * a.H * a.W + hp * a.q * a.W;
}

template <class T>
__global__ __launch_bounds__(kThreads) void patch_reduce_lds(ReduceArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x;
  const int s0 = blockIdx.x * a.spb;
  const int s1 = min(s0 + a.spb, a.total_strips);
  const int e0 = strip_offset(a, s0);
  const int e1 = (s1 == a.total_strips) ? a.total_in : strip_offset(a, s1);
  const long byte0 = (long)e0 * (long)sizeof(T);
  const long byte1 = (long)e1 * (long)sizeof(T);
  const long a0 = byte0 & ~15L;  // the tensor base is 16-byte aligned
  const int span = (int)(byte1 - a0);
  const int nvec = span >> 4;
  const uint4* src = reinterpret_cast<const uint4*>(static_cast<const unsigned char*>(a.in) + a0);
  uint4* dst = reinterpret_cast<uint4*>(smem);
  for (int v = tid; v < nvec; v += 4 * kThreads) {
    uint4 rg[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (v + k * kThreads < nvec) rg[k] = src[v + k * kThreads];
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (v + k * kThreads < nvec) dst[v + k * kThreads] = rg[k];
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
  for (int lo = tid; lo < nout; lo += kThreads) {
    const int ls = lo / a.Wp;
    const int wp = lo - ls * a.Wp;
    const int strip = s0 + ls;
    const int pl = strip / a.Hp;
    const int hp = strip - pl * a.Hp;
    const int ch = min(a.q, a.H - hp * a.q);
    const int cw = min(a.q, a.W - wp * a.q);
    const int base = pl * a.H * a.W + hp * a.q * a.W + wp * a.q - e0;
    float acc = 0.f;
    for (int i = 0; i < ch; ++i)
      for (int j = 0; j < cw; ++j) acc += to_f32(lds[base + i * a.W + j]);
    if (a.mean) acc = acc / (float)(ch * cw);
    out[s0 * a.Wp + lo] = from_f32<T>(acc);
  }
}

// Fallback without LDS for strips too large to stage: one lane per patch.
template <class T>
__global__ __launch_bounds__(kThreads) void patch_reduce_direct(ReduceArgs a) {
  const T* in = static_cast<const T*>(a.in);
  T* out = static_cast<T*>(a.out);
  const long nout = (long)a.total_strips * a.Wp;
  for (long o = (long)blockIdx.x * kThreads + threadIdx.x; o < nout; o += (long)gridDim.x * kThreads) {
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
    out[o] = from_f32<T>(acc);
  }
}

}  // namespace

hipError_t launch_patch_reduce(const void* in, void* out, long planes, int H, int W, int q,
                               bool mean, int dtype, hipStream_t st) {
  ReduceArgs a;
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
  const int b = dtype == GF_BF16 ? 2 : 4;
  const long strip_bytes = (long)imin_host(q, H) * W * b;
  if (strip_bytes + 32 > kLdsMax) {
    a.spb = 1;
    const long nout = (long)a.total_strips * a.Wp;
    int blocks = (int)((nout + kThreads - 1) / kThreads);
    if (blocks > 65536) blocks = 65536;
    if (dtype == GF_BF16)
      hipLaunchKernelGGL(patch_reduce_direct<bf16_t>, dim3(blocks), dim3(kThreads), 0, st, a);
    else
      hipLaunchKernelGGL(patch_reduce_direct<float>, dim3(blocks), dim3(kThreads), 0, st, a);
    return hipGetLastError();
  }
  int spb = (int)((kLdsBudget - 32) / strip_bytes);
  if (spb < 1) spb = 1;
  // keep at least ~8 blocks per CU in flight when the tensor is large enough
  const int want_blocks = 2048;
  if (a.total_strips / spb < want_blocks) spb = a.total_strips / want_blocks;
  if (spb < 1) spb = 1;
  a.spb = spb;
  const size_t lds = (size_t)spb * strip_bytes + 32;
  const int blocks = (a.total_strips + spb - 1) / spb;
  if (dtype == GF_BF16)
    hipLaunchKernelGGL(patch_reduce_lds<bf16_t>, dim3(blocks), dim3(kThreads), lds, st, a);
  else
    hipLaunchKernelGGL(patch_reduce_lds<float>, dim3(blocks), dim3(kThreads), lds, st, a);
  return hipGetLastError();
}

}  // namespace gf
