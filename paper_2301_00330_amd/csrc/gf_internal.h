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

// Launch observer (gf_set_launch_observer): told, on the host, right before (phase 0) and right
// after (phase 1) every kernel the library enqueues.  No observer set: one relaxed load per launch.
void observe_launch(const char* kernel_expr, int phase, hipStream_t st);
#define GF_LAUNCH(kern, grid, block, shmem, st, ...)                   \
  do {                                                                 \
    ::gf::observe_launch(#kern, 0, st);                                \
    hipLaunchKernelGGL(kern, grid, block, shmem, st, __VA_ARGS__);     \
    ::gf::observe_launch(#kern, 1, st);                                \
  } while (0)

typedef __bf16 bf16_t;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
template <class T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }

// 16-byte vectors of the storage type, unpacked to / packed from fp32
__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ uint32_t bf_pack(float lo, float hi) {
  const bf16_t a = (bf16_t)lo, b = (bf16_t)hi;
  return (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
}

// Loads and stores of data that is touched once per launch (the full-resolution maps): the
// non-temporal hint keeps them from displacing what the caches could reuse and lets written
// lines leave the L2 while the kernel still runs instead of at its end.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  const u32x4_t r = __builtin_nontemporal_load(static_cast<const u32x4_t*>(p));
  return make_uint4(r.x, r.y, r.z, r.w);
}
__device__ __forceinline__ void store_stream16(void* p, const uint4& v) {
  const u32x4_t r = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(r, static_cast<u32x4_t*>(p));
}
__device__ __forceinline__ void store_stream8(void* p, const uint2& v) {
  const u32x2_t r = {v.x, v.y};
  __builtin_nontemporal_store(r, static_cast<u32x2_t*>(p));
}
__device__ __forceinline__ void store_stream4(void* p, uint32_t v) {
  __builtin_nontemporal_store(v, static_cast<uint32_t*>(p));
}

template <class T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void unpack(const uint4& v, float* f) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
  static __device__ __forceinline__ uint4 pack(const float* f) {
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]),
                      __float_as_uint(f[3]));
  }
};
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void unpack(const uint4& v, float* f) {
    f[0] = bf_lo(v.x); f[1] = bf_hi(v.x); f[2] = bf_lo(v.y); f[3] = bf_hi(v.y);
    f[4] = bf_lo(v.z); f[5] = bf_hi(v.z); f[6] = bf_lo(v.w); f[7] = bf_hi(v.w);
  }
  static __device__ __forceinline__ uint4 pack(const float* f) {
    return make_uint4(bf_pack(f[0], f[1]), bf_pack(f[2], f[3]), bf_pack(f[4], f[5]),
                      bf_pack(f[6], f[7]));
  }
};

// Spatial sum of one kernel (text after Eq. 3), taps added in index order.  Taps are
// fetched eight at a time with clamped indices so the loads are in flight together.
template <class T>
__device__ __forceinline__ float kernel_sum_of(const T* w, long pair, int KK) {
  const T* p = w + pair * KK;
  float s = 0.f;
  for (int t0 = 0; t0 < KK; t0 += 8) {
    T v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = p[min(t0 + k, KK - 1)];
#pragma unroll
    for (int k = 0; k < 8; ++k) s += (t0 + k < KK) ? to_f32(v[k]) : 0.f;
  }
  return s;
}

// Signed 8-bit code of a value on a grid of step 1 / inv: the product and the rounding (half to
// even) are taken in fp32, the code is clipped to +-127 (never -128)
__device__ __forceinline__ int8_t q8_code(float v, float inv) {
  const float r = fminf(fmaxf(__builtin_rintf(v * inv), -127.f), 127.f);
  return (int8_t)(int)r;
}

static inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }
static inline int imin_host(int a, int b) { return a < b ? a : b; }

// Division of a 31-bit unsigned number by a run-time constant as multiply-high,
// add and shift (round-up method: m = floor(2^32 (2^s - d) / d) + 1, s = ceil(log2 d)).
struct FastDiv {
  uint32_t m, s, d;
  FastDiv() : m(1), s(0), d(1) {}
  explicit FastDiv(uint32_t dd) : d(dd) {
    s = 0;
    while ((1ull << s) < dd) ++s;
    m = (uint32_t)((((1ull << 32) * ((1ull << s) - dd)) / dd) + 1);
  }
  __device__ __forceinline__ uint32_t div(uint32_t n) const { return (__umulhi(n, m) + n) >> s; }
};

// ---- launchers; each returns the hipError_t of its launches ----------------

// S2 as a side job of another launch: out[e] = spatial sum of kernel e (pairs of them, KK taps
// each), rounded to the storage type -- or, with q_inv > 0, its signed 8-bit code (one byte per kernel).
struct KsumJob {
  const void* w;
  void* out;
  int pairs, KK;
  float q_inv;
};

// S0 / S1: out[plane, hp, wp] = sum or mean of in[plane] over q x q patches.  With `ksum` the
// same launch also forms the kernel sums (extra blocks at the end of the grid).
hipError_t launch_patch_reduce(const void* in, void* out, long planes, int H, int W, int q,
                               bool mean, int dtype, hipStream_t st, const KsumJob* ksum = nullptr);

// S0 of several tensors in one launch: out[plane, hp, wp] = sum of in[plane] over q x q patches
struct PoolJob {
  const void* in;
  void* out;
  long planes;
  int H, W, q;
  float q_inv;   // > 0 (in every job of a call, or in none): out holds signed 8-bit codes, step size 1 / q_inv
};
hipError_t launch_pool_batch(const PoolJob* jobs, int count, int dtype, hipStream_t st);

// ---- 8-bit codes (gf_q8.hip; the reductions with code output live in gf_reduce.hip) ----
// S0 / S1 with the result as signed 8-bit codes: round_half_even(value * inv_delta), clipped to +-127
// (with `ksum`: the kernel sums ride along, as in launch_patch_reduce)
hipError_t launch_patch_reduce_q8(const void* in, int8_t* out_q, long planes, int H, int W, int q, bool mean,
                                  float inv_delta, int dtype, hipStream_t st, const KsumJob* ksum = nullptr);
bool q8_shape_ok(const Geom& g);
hipError_t launch_kernel_sum_q8(const Geom& g, const void* w, float inv_delta, int8_t* w_q, hipStream_t st);
size_t ws_bwd_weight_q8(const Geom& g);
size_t ws_bwd_input_q8(const Geom& g, bool reduced_out);
hipError_t launch_bwd_weight_q8(const Geom& g, const int8_t* x_q, const int8_t* gy_q, float scale, float* g_w,
                                void* ws, hipStream_t st);
hipError_t launch_bwd_input_q8(const Geom& g, const int8_t* gy_q, const int8_t* w_q, float scale, void* g_x,
                               bool reduced_out, void* ws, hipStream_t st);
// full-resolution g_x from an fp32 reduced map [N, C_in, H_p, W_p] (rounded once to the storage type)
hipError_t launch_expand_f32(const Geom& g, const float* red, void* g_x, hipStream_t st);
// the same from a reduced map in the storage type
hipError_t launch_replicate(const Geom& g, const void* red, void* g_x, hipStream_t st);

// S1 with the noise figures of the filter: gy_u as launch_patch_reduce(mean), plus
// stats[0] = sum g_y^2 and stats[1] = sum (g_y - patch mean)^2 (doubles, device memory);
// `part` holds patch_reduce_max_blocks() float pairs.
long patch_reduce_max_blocks(long planes, int H, int W, int q);
hipError_t launch_filter_stats(const void* g_y, void* gy_u, long planes, int H, int W, int q, int dtype,
                               float* part, double* stats, hipStream_t st);

// S0 with the mask fraction: x_u as launch_patch_reduce(sum), m_u[patch] = share of the patch's
// in-bounds elements with 0 < x < hi (storage type)
hipError_t launch_pool_mask(const void* x, void* x_u, void* m_u, long planes, int H, int W, int q, float hi,
                            int dtype, hipStream_t st);
// dst[e] = dst[e] * m[e] (storage type, fp32 product rounded once)
hipError_t launch_mask_mul(void* dst, const void* m, long n, int dtype, hipStream_t st);

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

// MFMA kernels for groups == 1 (gf_mfma.hip).  The weight gradient writes nz K-slab
// partials [nz, Co, Ci] to `part`; the input gradient writes the reduced map
// [N, Ci, P] in the storage type to `dst`, using wsum_t ([Co, Ci], storage type)
// for the rounded kernel sum when the kernel is larger than 1x1.
int mfma_wgrad_splits(const Geom& g, int* chunks_per_z);
hipError_t launch_mfma_wgrad(const Geom& g, const void* x_u, const void* gy_u, float* part,
                             int* nz_out, hipStream_t st);
hipError_t launch_mfma_dgrad(const Geom& g, const void* gy_u, const void* w, void* wsum_t, void* dst,
                             void* full, hipStream_t st);
// vanilla BP of depthwise layers whose planes fit LDS (ws: ws_dw_exact_wgrad bytes for the weight gradient)
bool dw_exact_dgrad_ok(const Geom& g);
bool dw_exact_wgrad_ok(const Geom& g);
size_t ws_dw_exact_wgrad(const Geom& g);
hipError_t launch_dw_exact_dgrad(const Geom& g, const void* w, const void* g_y, void* g_x, hipStream_t st);
hipError_t launch_dw_exact_wgrad(const Geom& g, const void* x, const void* g_y, float* g_w, void* ws,
                                 hipStream_t st);

// whole filtered backward of a pointwise stride-1 layer with at most 32 input channels in one
// launch (then launch_finalize on `part`, *nz slabs of Co * Ci); gy_u may be null
bool onepass_ok(const Geom& g, int* nz);
hipError_t launch_onepass(const Geom& g, const void* g_y, const void* x_u, const void* w, void* gy_u,
                          void* g_x, float* part, hipStream_t st);

// both gradients of a dense layer in one launch (then launch_finalize on `part`, nz slabs);
// mask_u: with `reduced`, the reduced input gradient is multiplied by this map of the same shape
// With `reduced` the input gradient is written as the reduced map [N, Ci, P] instead of g_x.
bool mfma_s3s4_ok(const Geom& g, bool reduced = false);
hipError_t launch_mfma_s3s4(const Geom& g, const void* x_u, const void* gy_u, const void* w,
                            void* wsum_t, float* part, int* nz_out, void* g_x, hipStream_t st,
                            bool wsum_ready = false, bool reduced = false, const void* mask_u = nullptr);
// depthwise layer of a chain of filtered layers (gf_filtered.hip): partials [N, C] + reduced g_x
bool is_depthwise_layer(const Geom& g);
hipError_t launch_dw_chain(const Geom& g, const void* x_u, const void* gy_u, const void* w, float* part,
                           void* g_xu, const void* mask_u, hipStream_t st);
// true when the input-gradient GEMM can replicate its tile to [N, Ci, H, W] itself (pass `full`)
bool mfma_dgrad_writes_full(const Geom& g);

// Dense layers on small maps (gf_dense.hip): filter / relayout launch + one launch for both products with
// the slab sums folded in.  src: g_y (src_is_gy) or the filtered gradient gy_u; g_w or g_x may be null
// to skip that gradient; gy_u_out (nullable) receives the filtered gradient in the caller's layout.
bool dense_ok(const Geom& g);
size_t ws_dense(const Geom& g, bool want_w, bool want_d);
hipError_t launch_dense(const Geom& g, const void* src, bool src_is_gy, const void* x_u, const void* w,
                        void* gy_u_out, float* g_w, void* g_x, bool reduced, const void* mask_u, void* ws,
                        hipStream_t st);

// One-pass filtered backward of a depthwise stride-1 layer (gf_fused.hip): filter, weight
// gradient partials ([nz, C] in `part`, to be finalized) and input gradient.
bool dw_fused_ok(const Geom& g, int* nz);
hipError_t launch_dw_fused(const Geom& g, const void* g_y, const void* x_u, const void* w, void* gy_u,
                           void* g_x, float* part, hipStream_t st);
hipError_t launch_finalize(const float* part, float* g_w, int pairs, int nz, int KK, float scale,
                           hipStream_t st);


// S5: exact K x K backward.
size_t ws_exact(const Geom& g, bool want_gw, bool want_gx);
hipError_t launch_exact_wgrad(const Geom& g, const void* x, const void* g_y, float* g_w, void* ws,
                              hipStream_t st);
hipError_t launch_exact_dgrad(const Geom& g, const void* w, const void* g_y, void* g_x, void* ws,
                              hipStream_t st);


// S5 for dense stride-1 "same"-size layers: implicit GEMMs without a column tensor
// (gf_implicit.hip).  ws as sized by ws_implicit().
bool implicit_ok(const Geom& g);
size_t ws_implicit(const Geom& g, bool want_gw, bool want_gx);
// plain contraction part[z][co][ci] = sum_{n, p} gy_u * x_u on the same 128 x 128 tiles (large dense S3)
bool plain_wgrad_ok(const Geom& g);
int plain_wgrad_splits(const Geom& g);
hipError_t launch_plain_wgrad(const Geom& g, const void* x_u, const void* gy_u, float* part, int* nz_out,
                              hipStream_t st);
hipError_t launch_implicit(const Geom& g, const void* x, const void* w, const void* g_y, float* g_w, void* g_x,
                           void* ws, hipStream_t st);

}  // namespace gf
