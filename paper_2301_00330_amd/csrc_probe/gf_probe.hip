// Measurement probes for bench.py --ceilings (not part of libgf): what this chip sustains for the
// two resources the kernels of libgf are bound by.
//  * streaming reads, writes and copies of a buffer with 16-byte vectors (HBM ceilings),
//  * register-only loops of independent matrix instructions, no memory traffic (MFMA ceilings).
// Every kernel runs a bounded loop; the host checks sizes before a launch.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr int kThreads = 256;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

// each lane loads U vectors; the grid covers the buffer once
template <int U>
__global__ __launch_bounds__(kThreads) void read_k(const uint4* in, uint32_t* out, long nvec) {
  const long base = (long)blockIdx.x * kThreads * U + threadIdx.x;
  uint4 r[U];
#pragma unroll
  for (int k = 0; k < U; ++k) {
    const long i = base + (long)k * kThreads;
    r[k] = i < nvec ? in[i] : make_uint4(0, 0, 0, 0);
  }
  uint32_t acc = 0;
#pragma unroll
  for (int k = 0; k < U; ++k) acc ^= r[k].x ^ r[k].y ^ r[k].z ^ r[k].w;
  if (acc == 0x12345678u) out[0] = acc;   // keeps the loads alive; practically never true
}

__global__ __launch_bounds__(kThreads) void write_k(uint4* out, long nvec) {
  const long i = (long)blockIdx.x * kThreads + threadIdx.x;
  if (i < nvec) out[i] = make_uint4(1, 2, 3, 4);
}

__global__ __launch_bounds__(kThreads) void copy_k(const uint4* in, uint4* out, long nvec) {
  const long i = (long)blockIdx.x * kThreads + threadIdx.x;
  if (i < nvec) out[i] = in[i];
}

constexpr int NACC = 8;   // independent accumulators per wave

template <int KIND>
__global__ __launch_bounds__(kThreads) void mfma_k(float* out, int iters) {
  float s = 0.f;
  if constexpr (KIND == 0 || KIND == 1) {   // bf16: 32x32x16 (0) or 16x16x32 (1)
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(float)((threadIdx.x + i) & 7); b[i] = (__bf16)(float)(i + 1); }
    if constexpr (KIND == 0) {
      f32x16 acc[NACC / 2];
      for (int j = 0; j < NACC / 2; ++j) for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
      for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int j = 0; j < NACC / 2; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
      for (int j = 0; j < NACC / 2; ++j) for (int e = 0; e < 16; ++e) s += acc[j][e];
    } else {
      f32x4 acc[NACC];
      for (int j = 0; j < NACC; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
      for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int j = 0; j < NACC; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[j], 0, 0, 0);
      for (int j = 0; j < NACC; ++j) s += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
    }
  } else if constexpr (KIND == 2) {         // fp32 16x16x4
    const float a = (float)(threadIdx.x & 7), b = 1.5f;
    f32x4 acc[NACC];
    for (int j = 0; j < NACC; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it)
#pragma unroll
      for (int j = 0; j < NACC; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[j], 0, 0, 0);
    for (int j = 0; j < NACC; ++j) s += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
  } else {                                  // int8 16x16x64
    const i32x4 a = {(int)(threadIdx.x & 3), 1, 2, 3}, b = {4, 5, 6, (int)(threadIdx.x & 1)};
    i32x4 acc[NACC];
    for (int j = 0; j < NACC; ++j) acc[j] = i32x4{0, 0, 0, 0};
    for (int it = 0; it < iters; ++it)
#pragma unroll
      for (int j = 0; j < NACC; ++j) acc[j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, acc[j], 0, 0, 0);
    int t = 0;
    for (int j = 0; j < NACC; ++j) t += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
    s = (float)t;
  }
  out[(long)blockIdx.x * kThreads + threadIdx.x] = s;
}

constexpr int kMfmaBlocks = 256 * 8;   // 8 waves per SIMD on 256 compute units

}  // namespace

extern "C" {

// 0 on success, 1 on a rejected argument, 2 if the launch failed
int gfp_read(const void* in, void* flag, long bytes, void* stream) {
  if (!in || !flag || bytes < 16 || bytes > (1L << 36)) return 1;
  const long nvec = bytes / 16;
  hipLaunchKernelGGL(read_k<4>, dim3((unsigned)((nvec + 4 * kThreads - 1) / (4 * kThreads))), dim3(kThreads), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint4*>(in), static_cast<uint32_t*>(flag), nvec);
  return hipGetLastError() == hipSuccess ? 0 : 2;
}

int gfp_write(void* out, long bytes, void* stream) {
  if (!out || bytes < 16 || bytes > (1L << 36)) return 1;
  const long nvec = bytes / 16;
  hipLaunchKernelGGL(write_k, dim3((unsigned)((nvec + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                     static_cast<hipStream_t>(stream), static_cast<uint4*>(out), nvec);
  return hipGetLastError() == hipSuccess ? 0 : 2;
}

int gfp_copy(const void* in, void* out, long bytes, void* stream) {
  if (!in || !out || bytes < 16 || bytes > (1L << 36)) return 1;
  const long nvec = bytes / 16;
  hipLaunchKernelGGL(copy_k, dim3((unsigned)((nvec + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint4*>(in), static_cast<uint4*>(out), nvec);
  return hipGetLastError() == hipSuccess ? 0 : 2;
}

// floats the MFMA probes write: one per lane
long gfp_mfma_out_floats(void) { return (long)kMfmaBlocks * kThreads; }

// kind: 0 = bf16 32x32x16, 1 = bf16 16x16x32, 2 = fp32 16x16x4, 3 = int8 16x16x64.
// *ops = multiply-adds x 2 of the whole launch.  iters in 1 .. 100000.
int gfp_mfma(int kind, int iters, float* out, double* ops, void* stream) {
  if (!out || !ops || iters < 1 || iters > 100000 || kind < 0 || kind > 3) return 1;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const dim3 grid(kMfmaBlocks), block(kThreads);
  double per = 0;   // operations of one instruction
  int n = NACC;     // instructions per iteration and wave
  if (kind == 0) { hipLaunchKernelGGL(mfma_k<0>, grid, block, 0, st, out, iters); per = 2.0 * 32 * 32 * 16; n = NACC / 2; }
  else if (kind == 1) { hipLaunchKernelGGL(mfma_k<1>, grid, block, 0, st, out, iters); per = 2.0 * 16 * 16 * 32; }
  else if (kind == 2) { hipLaunchKernelGGL(mfma_k<2>, grid, block, 0, st, out, iters); per = 2.0 * 16 * 16 * 4; }
  else { hipLaunchKernelGGL(mfma_k<3>, grid, block, 0, st, out, iters); per = 2.0 * 16 * 16 * 64; }
  *ops = (double)kMfmaBlocks * (kThreads / 64) * iters * n * per;
  return hipGetLastError() == hipSuccess ? 0 : 2;
}

}  // extern "C"
