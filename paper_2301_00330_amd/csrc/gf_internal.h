// Internal declarations shared by the translation units of libgf (HIP path only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gf.h"

namespace gf {

// Validated layer geometry in the paper's symbols, plus derived sizes.
struct Geom {
  int N, Ci, Co, H, W, Kh, Kw, s, p, dl, g, r;
  int Hy, Wy;   // output map
  int Hp, Wp;   // patch grid (Sec. 3.3)
  int rx;       // input-side patch r*s (1 when r == 1)
  int Cg, Og;   // channels per group on the input / output side
  int KK, P;    // taps, patches per plane
  int dtype, b; // gf_dtype, bytes per element
};

gf_status make_geom(const gf_conv_desc* d, Geom* g);

typedef __bf16 bf16_t;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
template <class T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }

static inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }
static inline int imin_host(int a, int b) { return a < b ? a : b; }

// ---- launchers; each returns the hipError_t of its launches ----------------

// S0 / S1: out[plane, hp, wp] = sum or mean of in[plane] over q x q patches.
hipError_t launch_patch_reduce(const void* in, void* out, long planes, int H, int W, int q,
                               bool mean, int dtype, hipStream_t st);

// S2: wsum[co, cl] = sum over taps of w[co, cl, :, :], fp32.
hipError_t launch_kernel_sum(const void* w, float* wsum, long pairs, int KK, int dtype,
                             hipStream_t st);

// S3 (filtered): g_w from reduced maps; ws as sized by ws_bwd_weight().
size_t ws_bwd_weight(const Geom& g);
hipError_t launch_gf_bwd_weight(const Geom& g, const void* x_u, const void* gy_u, float* g_w,
                                void* ws, hipStream_t st);

// S2 + S4 (filtered): g_x from gy_u and w; ws as sized by ws_bwd_input().
size_t ws_bwd_input(const Geom& g, bool reduced_out);
hipError_t launch_gf_bwd_input(const Geom& g, const void* gy_u, const void* w, void* g_x,
                               bool reduced_out, void* ws, hipStream_t st);

// S5: exact K x K backward.
size_t ws_exact(const Geom& g, bool want_gw, bool want_gx);
hipError_t launch_exact_wgrad(const Geom& g, const void* x, const void* g_y, float* g_w, void* ws,
                              hipStream_t st);
hipError_t launch_exact_dgrad(const Geom& g, const void* w, const void* g_y, void* g_x, void* ws,
                              hipStream_t st);

}  // namespace gf
