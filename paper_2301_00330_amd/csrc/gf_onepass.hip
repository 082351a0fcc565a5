// One launch for the whole filtered backward of a pointwise (1x1), stride-1, ungrouped layer with
// at most 32 input channels (the MobileNetV2 expand shape): gradient filter (Eq. 2),
// weight gradient (Eq. 5) and input gradient (Eq. 3).  g_y is read once and the patch means
// never travel through HBM.
//
// A block owns a column tile of `prt` whole patch rows (at most 64 patches).  It walks the C_y
// channels in chunks of 32: every lane reduces its share of the chunk's r x r patches in
// registers exactly as the stand-alone filter does (vertical adds, horizontal adds, one divide,
// one rounding to the storage type) and puts the means into LDS; the loads of the next chunk
// are already in flight.  From LDS the chunk feeds two MFMA contractions:
//   input gradient   X[c_i, col]   += theta[k, c_i] * mean[k, col]          (kept in registers)
//   weight gradient  Gw[k, c_i]     = sum_col mean[k, col] * x_u[c_i, col]  (the tile's partial)
// The weight-gradient partial of every tile goes to a workspace slab (summed in fixed order by
// the finalize kernel, so results do not depend on scheduling), and X is replicated to the
// r rows x W pixels of every patch row with contiguous streaming stores.
#include "gf_mma.h"

namespace gf {

namespace {

constexpr int kThreads = 256;
// channels of g_y per chunk: 32 (one bf16 MFMA k-step), 16 for fp32 at r = 4, where a chunk of 32
// would need 32 vectors per lane and buffer
template <class T, int Q> constexpr int chunk_of() { return sizeof(T) == 4 && Q == 4 ? 16 : 32; }
constexpr int BN = 64;   // padded patch columns per tile (N of the input gradient, K of the weight gradient)

struct OnePassArgs {
  const void* gy;
  const void* xu;
  const void* w;
  void* gyu;    // nullable
  void* gx;
  float* part;  // [tiles, Co, Ci]
  int N, Ci, Co, H, W, Hp, Wp, P;
  int prt;      // patch rows per tile
  int cols;     // prt * Wp
  int units;    // N * Hp patch rows in the batch
  int ipr;      // 16-byte items per g_y pixel row
  int ppi;      // prt * ipr: items per channel of a tile
  int items;    // KC * ppi
  int nchunks;  // ceil(Co / KC)
  int xvr;      // x_u vectors per patch row of one channel
  float scale;
  FastDiv d_ppi, d_ipr, d_hp, d_xvr, d_xvc;
};

template <int XB> struct XWord;
template <> struct XWord<4> { typedef uint32_t type; };
template <> struct XWord<8> { typedef u32x2_t type; };
template <> struct XWord<16> { typedef u32x4_t type; };

// LDS strides (elements): rows stay 16-byte aligned and consecutive rows fall into different banks
template <class T> constexpr int pad_of() { return 16 / (int)sizeof(T); }

template <class T, int CIT, int KC>
struct Layout {
  static constexpr bool BF = sizeof(T) == 2;
  static constexpr int SB = BN + pad_of<T>();       // Bs / Xs / Cs rows: [row][col]
  static constexpr int ST = KC + 8;                 // bf16 BsT rows: [col][k]
  __host__ __device__ static int wt_elems(int nchunks) {
    // fp32: Wt[k][CIT*16 + 4]; bf16: WtT[c_i][nchunks*KC + 8]
    return BF ? CIT * 16 * (nchunks * KC + 8) : nchunks * KC * (CIT * 16 + 4);
  }
  __host__ __device__ static int bytes(int nchunks) {
    int e = wt_elems(nchunks) + KC * SB + CIT * 16 * SB + (BF ? BN * ST : 0);
    return (e * (int)sizeof(T) + 15) & ~15;
  }
};

// XB: bytes per x_u load (4, 8 or 16; the host picks what the row alignment allows)
template <class T, int Q, int CIT, int XB>
__global__ __launch_bounds__(kThreads) void onepass_k(OnePassArgs a) {
  constexpr int KC = chunk_of<T, Q>();
  using L = Layout<T, CIT, KC>;
  constexpr bool BF = L::BF;
  constexpr int VE = Mma<T>::VE;
  constexpr int NOUT = VE / Q;                       // patches per 16-byte item
  constexpr int MAXI = (KC * BN * Q / VE) / kThreads;  // items per lane and chunk: 4 (fp32), 2 (bf16) at Q = 2; 4 at Q = 4
  constexpr int SB = L::SB, ST = L::ST;
  constexpr int SW = CIT * 16 + 4;                   // fp32 Wt row
  constexpr int XV = XB / (int)sizeof(T);            // x_u elements per load
  static_assert(MAXI >= 1 && Q <= VE, "shape");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  T* Wt = reinterpret_cast<T*>(smem);
  T* Bs = Wt + L::wt_elems(a.nchunks);
  T* Xs = Bs + KC * SB;
  T* BsT = Xs + CIT * 16 * SB;   // bf16 only
  T* Cs = Xs;                    // the finished tile reuses the x_u tile
  const int SWT = a.nchunks * KC + 8;  // bf16 WtT row

  const T* gy = static_cast<const T*>(a.gy);
  const T* xu = static_cast<const T*>(a.xu);
  const T* w = static_cast<const T*>(a.w);
  T* gyu = static_cast<T*>(a.gyu);
  T* gx = static_cast<T*>(a.gx);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, kg = lane >> 4;
  const int tile = blockIdx.x;
  const int gr0 = tile * a.prt;  // first patch row of the tile, counted over the whole batch

  // ---- this lane's g_y items: the same (channel in chunk, patch row, vector) in every chunk ----
  long goff[MAXI];   // element offset of the item's first vector in channel 0 of the chunk's image
  int lds_off[MAXI], gyu_off[MAXI], chl[MAXI], rows[MAXI];
  bool live[MAXI];
#pragma unroll
  for (int g = 0; g < MAXI; ++g) {
    const int it = tid + g * kThreads;
    const int itc = min(it, a.items - 1);
    chl[g] = (int)a.d_ppi.div((uint32_t)itc);
    const int rem = itc - chl[g] * a.ppi;
    const int pr = (int)a.d_ipr.div((uint32_t)rem);
    const int col = rem - pr * a.ipr;
    const int gr = min(gr0 + pr, a.units - 1);
    const int n = (int)a.d_hp.div((uint32_t)gr);
    const int hp = gr - n * a.Hp;
    live[g] = it < a.items && gr0 + pr < a.units;
    rows[g] = min(Q, a.H - hp * Q);
    goff[g] = (((long)n * a.Co) * a.H + (long)hp * Q) * a.W + col * VE;
    lds_off[g] = pr * a.Wp + col * NOUT;
    gyu_off[g] = n * a.Co * a.P + hp * a.Wp + col * NOUT;   // + channel * P (host: fits 31 bits)
  }
  const long chan = (long)a.H * a.W;

  uint4 buf[2][MAXI][Q];   // the next chunk is in flight while this one is consumed
  auto fetch = [&](uint4 (*dst)[Q], int c) {
#pragma unroll
    for (int g = 0; g < MAXI; ++g) {
      const int ch = min(c * KC + chl[g], a.Co - 1);
      const T* p = gy + goff[g] + ch * chan;
#pragma unroll
      for (int i = 0; i < Q; ++i) dst[g][i] = load_stream16(p + (long)min(i, rows[g] - 1) * a.W);
    }
  };
  fetch(buf[0], 0);

  // ---- LDS: zero (pad rows and columns must read as zero), kernel matrix, x_u tile ----
  for (int i = tid; i < (L::bytes(a.nchunks) >> 4); i += kThreads)
    reinterpret_cast<uint4*>(smem)[i] = make_uint4(0, 0, 0, 0);
  __syncthreads();
  {  // theta[k][c_i], 16-byte vectors along c_i (host: Ci % VE == 0)
    const int vpr = a.Ci / VE;
    for (int s = tid; s < a.Co * vpr; s += kThreads) {
      const int k = s / vpr, v = s - k * vpr;
      const uint4 q = *reinterpret_cast<const uint4*>(w + (long)k * a.Ci + v * VE);
      if constexpr (BF) {
        const uint32_t wd[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int e = 0; e < VE; ++e)
          reinterpret_cast<uint16_t*>(Wt)[(v * VE + e) * SWT + k] = (uint16_t)(wd[e >> 1] >> ((e & 1) * 16));
      } else {
        *reinterpret_cast<uint4*>(Wt + k * SW + v * VE) = q;
      }
    }
  }
  {  // x_u[c_i][col]: XB-byte pieces of the tile's patch rows, four loads in flight per lane
    typedef typename XWord<XB>::type xw_t;
    const int per_c = a.prt * a.xvr;
    const int total = a.Ci * per_c;
    for (int s0 = tid; s0 < total; s0 += 4 * kThreads) {
      xw_t v[4];
      int dst[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int s = min(s0 + u * kThreads, total - 1);
        const int ci = (int)a.d_xvc.div((uint32_t)s);
        const int rem = s - ci * per_c;
        const int pr = (int)a.d_xvr.div((uint32_t)rem);
        const int xv = rem - pr * a.xvr;
        const int gr = min(gr0 + pr, a.units - 1);
        const int n = (int)a.d_hp.div((uint32_t)gr);
        const int hp = gr - n * a.Hp;
        v[u] = *reinterpret_cast<const xw_t*>(xu + ((long)n * a.Ci + ci) * a.P + hp * a.Wp + xv * XV);
        dst[u] = (s0 + u * kThreads < total && gr0 + pr < a.units) ? ci * SB + pr * a.Wp + xv * XV : -1;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (dst[u] >= 0) *reinterpret_cast<xw_t*>(Xs + dst[u]) = v[u];
    }
  }

  f32x4 accd[CIT];
#pragma unroll
  for (int m = 0; m < CIT; ++m) accd[m] = f32x4{0.f, 0.f, 0.f, 0.f};
  float* part = a.part + (long)tile * a.Co * a.Ci;

  auto chunk = [&](const uint4 (*src)[Q], uint4 (*nxt)[Q], int c) {
    // 1. patch means of the chunk -> LDS (and gy_u when the caller wants it)
#pragma unroll
    for (int g = 0; g < MAXI; ++g) {
      float colsum[VE];
#pragma unroll
      for (int e = 0; e < VE; ++e) colsum[e] = 0.f;
#pragma unroll
      for (int i = 0; i < Q; ++i) {
        float f[VE];
        Vec16<T>::unpack(src[g][i], f);
        const bool keep = i < rows[g];
#pragma unroll
        for (int e = 0; e < VE; ++e) colsum[e] += keep ? f[e] : 0.f;
      }
      const float den = (float)(rows[g] * Q);
      const int ch = c * KC + chl[g];
      if (live[g] && ch < a.Co) {
#pragma unroll
        for (int o = 0; o < NOUT; ++o) {
          float s = 0.f;
#pragma unroll
          for (int j = 0; j < Q; ++j) s += colsum[o * Q + j];
          const T m = from_f32<T>(s / den);
          Bs[chl[g] * SB + lds_off[g] + o] = m;
          if constexpr (BF) BsT[(lds_off[g] + o) * ST + chl[g]] = m;
          if (gyu) gyu[gyu_off[g] + ch * a.P + o] = m;
        }
      } else if (live[g]) {  // channel past C_y in the last chunk: the previous chunk's value must go
#pragma unroll
        for (int o = 0; o < NOUT; ++o) {
          Bs[chl[g] * SB + lds_off[g] + o] = from_f32<T>(0.f);
          if constexpr (BF) BsT[(lds_off[g] + o) * ST + chl[g]] = from_f32<T>(0.f);
        }
      }
    }
    __syncthreads();
    if (c + 1 < a.nchunks) fetch(nxt, c + 1);
    // 2. input gradient: this wave's 16 columns, all c_i tiles
    if constexpr (BF) {
      const uint4 fb = *reinterpret_cast<const uint4*>(BsT + (wave * 16 + r) * ST + kg * 8);
#pragma unroll
      for (int m = 0; m < CIT; ++m) {
        const uint4 fa = *reinterpret_cast<const uint4*>(Wt + (m * 16 + r) * SWT + c * KC + kg * 8);
        accd[m] = mma16(fa, fb, accd[m]);
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < KC / 4; ++ks) {
        const float fb = Bs[(ks * 4 + kg) * SB + wave * 16 + r];
#pragma unroll
        for (int m = 0; m < CIT; ++m) {
          const float fa = Wt[(c * KC + ks * 4 + kg) * SW + m * 16 + r];
          accd[m] = mma16(fa, fb, accd[m]);
        }
      }
    }
    // 3. weight gradient of the chunk's channels: (KC / 16) x CIT tiles over the four waves
    for (int t = wave; t < (KC / 16) * CIT; t += 4) {
      const int mt = t / CIT, nt = t - mt * CIT;
      f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
      if constexpr (BF) {
#pragma unroll
        for (int ks = 0; ks < BN / 32; ++ks) {
          const uint4 fa = *reinterpret_cast<const uint4*>(Bs + (mt * 16 + r) * SB + ks * 32 + kg * 8);
          const uint4 fb = *reinterpret_cast<const uint4*>(Xs + (nt * 16 + r) * SB + ks * 32 + kg * 8);
          acc = mma16(fa, fb, acc);
        }
      } else {
#pragma unroll
        for (int ks = 0; ks < BN / 4; ++ks) {
          const float fa = Bs[(mt * 16 + r) * SB + ks * 4 + kg];
          const float fb = Xs[(nt * 16 + r) * SB + ks * 4 + kg];
          acc = mma16(fa, fb, acc);
        }
      }
      const int ci = nt * 16 + r;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int co = c * KC + mt * 16 + 4 * kg + v;
        if (co < a.Co && ci < a.Ci) part[(long)co * a.Ci + ci] = acc[v];
      }
    }
    __syncthreads();
  };

  __syncthreads();  // kernel matrix and x_u tile are in place
  for (int c = 0; c < a.nchunks; c += 2) {
    chunk(buf[0], buf[1], c);
    if (c + 1 < a.nchunks) chunk(buf[1], buf[0], c + 1);
  }

  // ---- finished tile -> LDS (scaled, rounded once), then the full-resolution store ----
#pragma unroll
  for (int m = 0; m < CIT; ++m)
#pragma unroll
    for (int v = 0; v < 4; ++v)
      Cs[(m * 16 + 4 * kg + v) * SB + wave * 16 + r] = from_f32<T>(accd[m][v] * a.scale);
  __syncthreads();
  {
    // lane = one 16-byte vector of the contiguous run (prt patch rows x Q pixel rows x W pixels)
    // that one c_i owns; consecutive lanes store consecutive vectors, `rpp` rows of c_i per pass
    constexpr int sh = Q == 2 ? 1 : Q == 4 ? 2 : 3;
    const int vpr = a.W / VE;
    const int ipr = a.prt * Q * vpr;
    const int rpp = kThreads / ipr;
    const int rl = tid / ipr, slot = tid - rl * ipr;
    const int pr = slot / (Q * vpr), rem = slot - pr * Q * vpr;
    const int i = rem / vpr, vv = rem - i * vpr;
    const int gr = gr0 + pr;
    if (rl < rpp && gr < a.units) {
      const int n = (int)a.d_hp.div((uint32_t)gr);
      const int hp = gr - n * a.Hp;
      const int h = hp * Q + i;
      if (h < a.H) {
        const T* src = Cs + pr * a.Wp;
        T* d = gx + (((long)n * a.Ci) * a.H + h) * a.W + vv * VE;
        for (int row = rl; row < a.Ci; row += rpp) {
          T vals[VE];
#pragma unroll
          for (int e = 0; e < VE; ++e) vals[e] = src[row * SB + ((vv * VE + e) >> sh)];
          store_stream16(d + (long)row * chan, *reinterpret_cast<const uint4*>(vals));
        }
      }
    }
  }
}

template <class T>
bool plan(const Geom& g, OnePassArgs* out, int* cit, int* xb) {
  constexpr int VE = 16 / (int)sizeof(T);
  if (g.g != 1 || g.s != 1 || g.KK != 1 || g.Hy != g.H || g.Wy != g.W) return false;
  if (g.r != 2 && g.r != 4) return false;
  // fp32 at r = 4 (chunks of 16 channels, twice the barriers) measured slower than filter + merged launch
  if (g.r == 4 && sizeof(T) == 4) return false;
  const int KC = g.r == 4 ? chunk_of<T, 4>() : chunk_of<T, 2>();
  if (g.W % VE != 0 || g.W != g.Wp * g.r || g.Wp > BN) return false;
  if (g.Ci % VE != 0) return false;
  // few c_i tiles (the expand shape).  With many c_i tiles and one chunk (the project shape) the
  // same kernel was measured no faster than filter + merged GEMM launch, so it is not built.
  const int tiles_ci = cdiv(g.Ci, 16), nchunks = cdiv(g.Co, KC);
  if (tiles_ci > 2 || nchunks * KC > 256) return false;
  const int CIT = 2;
  OnePassArgs a = {};
  a.N = g.N; a.Ci = g.Ci; a.Co = g.Co; a.H = g.H; a.W = g.W; a.Hp = g.Hp; a.Wp = g.Wp; a.P = g.P;
  a.units = g.N * g.Hp;
  a.ipr = g.W / VE;
  int prt = BN / g.Wp;
  const int per_patch_row = g.r * a.ipr;   // output vectors of one patch row of one c_i
  if (per_patch_row > kThreads) return false;
  if (prt > kThreads / per_patch_row) prt = kThreads / per_patch_row;
  // fewer patch rows per tile when the tiles would not fill the chip (the kernel is bound by the
  // bytes in flight, not by the MFMA columns a narrow tile leaves idle)
  while (prt > 1 && cdiv(a.units, prt) < 384) --prt;
  a.prt = prt;
  a.cols = prt * g.Wp;
  a.ppi = prt * a.ipr;
  a.items = KC * a.ppi;
  a.nchunks = nchunks;
  a.scale = 1.f;
  if ((long)g.N * g.Co * g.P >= (1L << 31)) return false;
  // x_u pieces: the widest load that every patch row start is aligned to
  int XB = 16;
  while (XB > 4 && ((g.Wp * (int)sizeof(T)) % XB != 0 || ((long)g.P * sizeof(T)) % XB != 0)) XB >>= 1;
  if ((g.Wp * (int)sizeof(T)) % XB != 0 || ((long)g.P * sizeof(T)) % XB != 0) return false;
  a.xvr = g.Wp * (int)sizeof(T) / XB;
  a.d_ppi = FastDiv((uint32_t)a.ppi);
  a.d_ipr = FastDiv((uint32_t)a.ipr);
  a.d_hp = FastDiv((uint32_t)g.Hp);
  a.d_xvr = FastDiv((uint32_t)a.xvr);
  a.d_xvc = FastDiv((uint32_t)(prt * a.xvr));
  const int lds = g.r == 4 ? Layout<T, 2, chunk_of<T, 4>()>::bytes(nchunks) : Layout<T, 2, chunk_of<T, 2>()>::bytes(nchunks);
  if (lds > 80 * 1024) return false;
  if (out) *out = a;
  if (cit) *cit = CIT;
  if (xb) *xb = XB;
  return true;
}

template <class T, int Q, int CIT>
hipError_t launch_x(OnePassArgs& a, int xb, hipStream_t st) {
  const int tiles = cdiv(a.units, a.prt);
  const size_t lds = (size_t)Layout<T, CIT, chunk_of<T, Q>()>::bytes(a.nchunks);
  const dim3 grid(tiles), block(kThreads);
  if (xb == 16) GF_LAUNCH((onepass_k<T, Q, CIT, 16>), grid, block, lds, st, a);
  else if (xb == 8) GF_LAUNCH((onepass_k<T, Q, CIT, 8>), grid, block, lds, st, a);
  else GF_LAUNCH((onepass_k<T, Q, CIT, 4>), grid, block, lds, st, a);
  return hipGetLastError();
}

template <class T>
hipError_t onepass_t(const Geom& g, const void* g_y, const void* x_u, const void* w, void* gy_u,
                     void* g_x, float* part, hipStream_t st) {
  OnePassArgs a;
  int cit = 0, xb = 0;
  if (!plan<T>(g, &a, &cit, &xb)) return hipErrorInvalidValue;
  a.gy = g_y; a.xu = x_u; a.w = w; a.gyu = gy_u; a.gx = g_x; a.part = part;
  if constexpr (sizeof(T) == 2) {   // r = 4 is built for bf16 only (see plan)
    if (g.r == 4) return launch_x<T, 4, 2>(a, xb, st);
  }
  return launch_x<T, 2, 2>(a, xb, st);
}

}  // namespace

bool onepass_ok(const Geom& g, int* nz) {
  OnePassArgs a;
  const bool ok = g.dtype == GF_BF16 ? plan<bf16_t>(g, &a, nullptr, nullptr) : plan<float>(g, &a, nullptr, nullptr);
  if (ok && nz) *nz = cdiv(a.units, a.prt);
  return ok;
}

hipError_t launch_onepass(const Geom& g, const void* g_y, const void* x_u, const void* w, void* gy_u,
                          void* g_x, float* part, hipStream_t st) {
  if (g.dtype == GF_BF16) return onepass_t<bf16_t>(g, g_y, x_u, w, gy_u, g_x, part, st);
  return onepass_t<float>(g, g_y, x_u, w, gy_u, g_x, part, st);
}

}  // namespace gf
