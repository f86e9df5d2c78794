// Convolution forward, backward-data and backward-weight as implicit GEMMs on
// the fp32 MFMA core (gemm.h), and the dense layers on the same core.
#include <algorithm>

#include "gemm_bf16.h"
#include "kernels.h"

namespace ax {

constexpr int kBK = 16;  // depth of a k-tile
typedef Tile<128, 128, kBK, 2, 2> T128;  // wave tile 64 x 64
typedef Tile<128, 96, kBK, 4, 1> T96;    // wave tile 32 x 96
typedef Tile<128, 64, kBK, 4, 1> T64;    // wave tile 32 x 64
// 48 columns out of 16x16x4 blocks (wave tile 32 x 48), k-tile 32; only with the whole-tile loaders
constexpr int kBK48 = 32;
typedef Tile<128, 48, kBK48, 4, 1, 16> T48;
// (256 x 128 and 256 x 96 tiles were measured too: their 128 accumulator
// registers leave one wave per SIMD, and with nobody to cover barrier and LDS
// latency they ran 8-12 % slower than 128 x 128 on every AlexNet layer.)

// ------------------------------------------------------------ tile + split-k ---
// A launch is as slow as its busiest compute unit.  With few output tiles (338
// for a 21632 x 256 output at 128 x 128) a third of the chip idles while the
// rest runs a second tile, so the reduction can be cut into `ns` slices whose
// partial tiles go to slabs and are added by a finishing kernel in a fixed
// order.  Larger tiles spend fewer non-MFMA instructions per MFMA but make
// that quantisation worse.  plan_gemm() prices every (tile, ns) pair with a
// small model -- rounds of tiles over 256 compute units at the tile's measured
// MFMA efficiency, padded columns, slab traffic -- and takes the cheapest.
struct GemmPlan {
  int bm, bn, ns, kchunk;
};
struct TileOption {
  int bm, bn, bk;
  double eff;  // fraction of the per-CU fp32 MFMA rate this tile reaches on a long reduction
};
static const TileOption kTileOptions[] = {{128, 128, kBK, 0.80}, {128, 96, kBK, 0.68}, {128, 64, kBK, 0.62},
                                          {128, 48, kBK48, 0.60}};
// bf16 MFMA tiles: k-tile of 32; no longer MFMA-bound, priced at ~4x the fp32 rate
constexpr int kBKbf = 32;
typedef Tile<128, 128, kBKbf, 2, 2> B128;
typedef Tile<128, 64, kBKbf, 4, 1> B64;
// 256 x 128 (wave tile 128 x 64): three fragment reads for every four MFMAs instead of four for four -- these
// kernels are paced by LDS, not by the matrix cores; only with operands stored as bf16 (half the staging registers)
typedef Tile<256, 128, kBKbf, 2, 2> B256;
// 256 x 96 (wave tile 64 x 96) for the first layer's 96 output channels, which the 128-wide tiles pad by a third
typedef Tile<256, 96, kBKbf, 4, 1> B256n96;
static const TileOption kTileOptionsBf[] = {{128, 128, kBKbf, 3.2}, {128, 64, kBKbf, 2.2}, {256, 128, kBKbf, 4.2}};

// precision of the GEMMs launched by the calling thread: 0 fp32 MFMA, 1 bf16 MFMA with fp32 accumulation
static thread_local int g_bf16 = 0;
void set_gemm_precision(int bf16) { g_bf16 = bf16 ? 1 : 0; }

static GemmPlan plan_gemm(int M, int N, int K, int groups, double out_bytes, int max_s, bool bf = false,
                          bool allow48 = false, int max_chunk = 0, bool allow256 = false) {
  const TileOption* opts = bf ? kTileOptionsBf : kTileOptions;
  const int nopts = bf ? (allow256 ? 3 : 2) : (allow48 ? 4 : 3);
  GemmPlan best{128, 128, 1, ceil_div(K, opts[0].bk) * opts[0].bk};
  double best_t = 1e30;
  for (int o = 0; o < nopts; ++o) {
    const TileOption& to = opts[o];
    const int bk = to.bk, ktiles = ceil_div(K, bk);
    const long tiles = (long)ceil_div(M, to.bm) * ceil_div(N, to.bn) * groups;
    const double t_tile = 2.0 * to.bm * to.bn * (double)ktiles * bk / (0.614e12 * to.eff);
    for (int s = 1; s <= max_s && s <= ktiles; ++s) {
      const int per = ceil_div(ktiles, s);
      if (ceil_div(ktiles, per) != s) continue;
      if (s > 1 && per * bk < 96) break;
      if (max_chunk && per * bk > max_chunk) continue;  // the workgroup's k range must fit its pixel table
      const double rounds = (double)ceil_div(tiles * s, 256);
      double t = rounds * t_tile * per / ktiles + 4e-6;
      if (s > 1) t += (s + 1) * out_bytes / 2.5e12 + 6e-6;
      if (t < best_t * 0.98) {  // prefer earlier (larger, unsplit) candidates unless clearly better
        best_t = t;
        best = GemmPlan{to.bm, to.bn, s, per * bk};
      }
    }
  }
  return best;
}


// Algorithmic flops of the launch being prepared (2 x multiply-adds of the
// operation, not of the padded GEMM); 0 means "use 2*M*N*K".
static thread_local double g_algo_flops = 0;
// Algorithmic bytes of the same launch: every operand tensor read once and the result written once (for a
// convolution the activation tensor itself, not its im2col expansion); 0 means "(M*K + K*N + M*N) floats".
static thread_local double g_algo_bytes = 0;
struct AlgoFlops {
  explicit AlgoFlops(double f, double b = 0) { g_algo_flops = f; g_algo_bytes = b; }
  ~AlgoFlops() { g_algo_flops = 0; g_algo_bytes = 0; }
};
static inline double conv_flops(const ConvGeom& c) { return 2.0 * c.P() * c.Cout * c.cg() * c.k * c.k; }
static inline double conv_bytes(const ConvGeom& c) {
  return 4.0 * ((double)c.in_elems() + (double)c.w_elems() + (double)c.out_elems());
}
static inline double gemm_bytes(int M, int N, int K, int groups) {
  return g_algo_bytes > 0 ? g_algo_bytes : 4.0 * groups * ((double)M * K + (double)K * N + (double)M * N);
}

template <class T, class AL, class BL, class Epi>
static int launch_tile(const typename AL::Params& ap, const typename BL::Params& bp, const Epi& ep, int M, int N, int K,
                       int kchunk, int nsplit, int groups, hipStream_t st, size_t dyn_lds = 0) {
  if (M <= 0 || N <= 0) return ALEXNET_OK;
  dim3 grid(ceil_div(M, T::BM), ceil_div(N, T::BN), groups * nsplit);
  if (grid.y > 65535 || grid.z > 65535) {
    set_error("GEMM grid too large (%u,%u,%u)", grid.x, grid.y, grid.z);
    return ALEXNET_ESHAPE;
  }
  KernelScope ks("gemm", g_algo_flops > 0 ? g_algo_flops : 2.0 * M * N * (double)K * groups,
                 gemm_bytes(M, N, K, groups), st);
  hipLaunchKernelGGL((gemm_kernel<T, AL, BL, Epi>), grid, dim3(kThreads), dyn_lds, st, ap, bp, ep, M, N, K, kchunk,
                     nsplit);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

template <class T, class AL, class BL, class Epi>
static int launch_tile_bf(const typename AL::Params& ap, const typename BL::Params& bp, const Epi& ep, int M, int N,
                          int K, int kchunk, int nsplit, int groups, hipStream_t st, size_t dyn_lds = 0) {
  if (M <= 0 || N <= 0) return ALEXNET_OK;
  // one-dimensional launch: the kernel deals the tiles to the XCDs itself (xcd_tile)
  const int gx = ceil_div(M, T::BM), gy = ceil_div(N, T::BN), gz = groups * nsplit;
  const long total = (long)gx * gy * gz;
  if (total > 0x7fffffffL) {
    set_error("GEMM grid too large (%d,%d,%d)", gx, gy, gz);
    return ALEXNET_ESHAPE;
  }
  KernelScope ks("gemm_bf16", g_algo_flops > 0 ? g_algo_flops : 2.0 * M * N * (double)K * groups,
                 gemm_bytes(M, N, K, groups), st);
  hipLaunchKernelGGL((gemm_bf16_kernel<T, AL, BL, Epi>), dim3((unsigned)total), dim3(kThreads), dyn_lds, st, ap, bp, ep,
                     M, N, K, kchunk, nsplit, gx, gy);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

static inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

// One struct per GEMM flavour: names the loaders for a tile and a pair of
// vector/scalar choices, so that the dispatch below stays a table.
template <int MODE>
struct ConvGather {  // rows = pixels (forward, backward-data)
  template <class T, bool AV, bool BV, class Epi>
  static int go(const Im2colParams& a, const DenseParams& b, const Epi& e, const GemmDims& d, int kchunk, int ns,
                hipStream_t st) {
    return launch_tile<T, Im2colKInner<T::BM, T::BK, AV, MODE>, DenseRowInner<T::BN, T::BK, BV>, Epi>(
        a, b, e, d.M, d.N, d.K, kchunk, ns, d.groups, st);
  }
};
struct ConvWeightGrad {  // rows = taps (backward-weight)
  template <class T, bool AV, bool BV, class Epi>
  static int go(const Im2colParams& a, const DenseParams& b, const Epi& e, const GemmDims& d, int kchunk, int ns,
                hipStream_t st) {
    return launch_tile<T, Im2colRowInner<T::BM, T::BK, AV>, DenseRowInner<T::BN, T::BK, BV>, Epi>(
        a, b, e, d.M, d.N, d.K, kchunk, ns, d.groups, st);
  }
};

// backward-weight with the pixel table in LDS (see Im2colRowTable): 16-byte loads, whole k-tiles
struct ConvWeightGradTable {
  template <class T, class Epi>
  static int go(const Im2colParams& a, const DenseParams& b, const Epi& e, const GemmDims& d, int kchunk, int ns,
                hipStream_t st) {
    return launch_tile<T, Im2colRowTable<T::BM, T::BK>, DenseRowWhole<T::BN, T::BK>, Epi>(
        a, b, e, d.M, d.N, d.K, kchunk, ns, d.groups, st, (size_t)std::min(kchunk, d.K) * sizeof(PixelEntry));
  }
};
static inline bool table_ok(const Im2colParams& a, const GemmDims& d) {
  return a.kh * a.kw <= 31 && d.K % kBK == 0;
}

// a k-tile inside one tap (see Im2colKTap): 16-byte loads, whole k-tiles
template <int MODE>
struct ConvGatherTap {
  template <class T, class Epi>
  static int go(const Im2colParams& a, const DenseParams& b, const Epi& e, const GemmDims& d, int kchunk, int ns,
                hipStream_t st) {
    return launch_tile<T, Im2colKTap<T::BM, T::BK, MODE>, DenseRowWhole<T::BN, T::BK>, Epi>(
        a, b, e, d.M, d.N, d.K, kchunk, ns, d.groups, st);
  }
};
static inline bool tap_ok(const Im2colParams& a, const GemmDims& d, int bk = kBK) {
  return a.Cg % bk == 0 && a.kh * a.kw <= 32 && d.K % bk == 0;
}

// bf16 flavours (vector loads only)
template <int MODE>
struct ConvGatherBf {
  template <class T, class Epi>
  static int go(const Im2colParams& a, const DenseParams& b, const Epi& e, const GemmDims& d, int kchunk, int ns,
                hipStream_t st) {
    return launch_tile_bf<T, BfRowMajor<Im2colKInner<T::BM, T::BK, true, MODE>, T::BM, T::BK>,
                          BfDenseRowInner<T::BN, T::BK>, Epi>(a, b, e, d.M, d.N, d.K, kchunk, ns, d.groups, st);
  }
};
struct ConvWeightGradBf {
  template <class T, class Epi>
  static int go(const Im2colParams& a, const DenseParams& b, const Epi& e, const GemmDims& d, int kchunk, int ns,
                hipStream_t st) {
    return launch_tile_bf<T, BfIm2colRowInner<T::BM, T::BK>, BfDenseRowInner<T::BN, T::BK>, Epi>(
        a, b, e, d.M, d.N, d.K, kchunk, ns, d.groups, st);
  }
};
// bf16 with the uniform-tap / whole-tile / pixel-table loaders
template <int MODE>
struct ConvGatherTapBf {
  template <class T, class Epi>
  static int go(const Im2colParams& a, const DenseParams& b, const Epi& e, const GemmDims& d, int kchunk, int ns,
                hipStream_t st) {
    return launch_tile_bf<T, BfRowMajor<Im2colKTap<T::BM, T::BK, MODE>, T::BM, T::BK>, BfDenseRowWhole<T::BN, T::BK>,
                          Epi>(a, b, e, d.M, d.N, d.K, kchunk, ns, d.groups, st);
  }
};
struct ConvWeightGradTableBf {
  template <class T, class Epi>
  static int go(const Im2colParams& a, const DenseParams& b, const Epi& e, const GemmDims& d, int kchunk, int ns,
                hipStream_t st) {
    return launch_tile_bf<T, BfIm2colRowTable<T::BM, T::BK>, BfDenseRowWhole<T::BN, T::BK>, Epi>(
        a, b, e, d.M, d.N, d.K, kchunk, ns, d.groups, st, (size_t)std::min(kchunk, d.K) * sizeof(PixelEntry));
  }
};
// bf16 MFMA over operands that are stored as bf16 (gemm_bf16.h, "16" loaders)
template <int MODE>
struct ConvGather16 {
  template <class T, class Epi>
  static int go(const Im2colParams& a, const DenseParams& b, const Epi& e, const GemmDims& d, int kchunk, int ns,
                hipStream_t st) {
    return launch_tile_bf<T, Im2colKInner16<T::BM, T::BK, MODE>, DenseKInner16<T::BN, T::BK>, Epi>(
        a, b, e, d.M, d.N, d.K, kchunk, ns, d.groups, st);
  }
};
template <int MODE>
struct ConvGatherTap16 {
  template <class T, class Epi>
  static int go(const Im2colParams& a, const DenseParams& b, const Epi& e, const GemmDims& d, int kchunk, int ns,
                hipStream_t st) {
    return launch_tile_bf<T, Im2colKTap16<T::BM, T::BK, MODE>, DenseKInner16<T::BN, T::BK>, Epi>(
        a, b, e, d.M, d.N, d.K, kchunk, ns, d.groups, st);
  }
};
struct ConvWeightGradTable16 {
  template <class T, class Epi>
  static int go(const Im2colParams& a, const DenseParams& b, const Epi& e, const GemmDims& d, int kchunk, int ns,
                hipStream_t st) {
    return launch_tile_bf<T, Im2colRowTable16<T::BM, T::BK>, DenseRowInner16<T::BN, T::BK>, Epi>(
        a, b, e, d.M, d.N, d.K, kchunk, ns, d.groups, st, (size_t)std::min(kchunk, d.K) * sizeof(PixelEntry));
  }
};
template <class F, class Epi>
static int by_tile_16(const GemmPlan& p, const Im2colParams& a, const DenseParams& b, const Epi& e, const GemmDims& d,
                      hipStream_t st) {
  if (p.bm == 256) return F::template go<B256, Epi>(a, b, e, d, p.kchunk, p.ns, st);
  if (p.bn == 128) return F::template go<B128, Epi>(a, b, e, d, p.kchunk, p.ns, st);
  return F::template go<B64, Epi>(a, b, e, d, p.kchunk, p.ns, st);
}
template <class F, class Epi>
static int by_tile_bf(const GemmPlan& p, const Im2colParams& a, const DenseParams& b, const Epi& e, const GemmDims& d,
                      hipStream_t st) {
  if (p.bn == 128) return F::template go<B128, Epi>(a, b, e, d, p.kchunk, p.ns, st);
  return F::template go<B64, Epi>(a, b, e, d, p.kchunk, p.ns, st);
}

// vector loads on both operands, on B only, or on neither
template <class F, class T, class Epi>
static int by_vec(bool av, bool bv, const Im2colParams& a, const DenseParams& b, const Epi& e, const GemmDims& d,
                  int kchunk, int ns, hipStream_t st) {
  if (av && bv) return F::template go<T, true, true, Epi>(a, b, e, d, kchunk, ns, st);
  if (bv) return F::template go<T, false, true, Epi>(a, b, e, d, kchunk, ns, st);
  return F::template go<T, false, false, Epi>(a, b, e, d, kchunk, ns, st);
}
template <class F, class Epi>
static int by_tile(const GemmPlan& p, bool av, bool bv, const Im2colParams& a, const DenseParams& b, const Epi& e,
                   const GemmDims& d, hipStream_t st) {
  if (p.bn == 128) return by_vec<F, T128, Epi>(av, bv, a, b, e, d, p.kchunk, p.ns, st);
  if (p.bn == 96) return by_vec<F, T96, Epi>(av, bv, a, b, e, d, p.kchunk, p.ns, st);
  return by_vec<F, T64, Epi>(av, bv, a, b, e, d, p.kchunk, p.ns, st);
}

// out[m][g*N + n] = post(sum_s ws[(g*ns + s)][m][n]); post = +bias, ReLU, or gate by a forward activation
__global__ void slab_finish_kernel(const float* __restrict__ ws, int ns, int groups, long M, int N,
                                   const float* __restrict__ bias, int relu, const float* __restrict__ gate,
                                   float* __restrict__ out) {
  const size_t total = (size_t)M * groups * N;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // index into out
  if (i >= total) return;
  const int col = (int)(i % ((size_t)groups * N));
  const size_t m = i / ((size_t)groups * N);
  const int g = col / N, n = col - g * N;
  const size_t slab = (size_t)M * N;
  const float* p = ws + (size_t)g * ns * slab + m * N + n;
  float v = 0.f;
#pragma unroll 8
  for (int k = 0; k < ns; ++k) v += p[(size_t)k * slab];  // loads in flight together, added in order
  if (bias) v += bias[col];
  if (relu) v = v > 0.f ? v : 0.f;
  if (gate && !(gate[i] > 0.f)) v = 0.f;
  out[i] = v;
}
static int launch_slab_finish(const float* ws, int ns, int groups, long M, int N, const float* bias, int relu,
                              const float* gate, float* out, hipStream_t st) {
  const size_t total = (size_t)M * groups * N;
  KernelScope ks("slab_finish", 0, (double)total * 4.0 * (ns + 1 + (gate ? 1 : 0)), st);
  hipLaunchKernelGGL(slab_finish_kernel, dim3(ceil_div(total, 256)), dim3(256), 0, st, ws, ns, groups, M, N, bias,
                     relu, gate, out);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// ------------------------------------------------------------- convolution ---
template <class F, class Epi>
static int by_tile_tap(const GemmPlan& p, const Im2colParams& a, const DenseParams& b, const Epi& e,
                       const GemmDims& d, hipStream_t st) {
  if (p.bn == 128) return F::template go<T128, Epi>(a, b, e, d, p.kchunk, p.ns, st);
  if (p.bn == 96) return F::template go<T96, Epi>(a, b, e, d, p.kchunk, p.ns, st);
  if (p.bn == 48) return F::template go<T48, Epi>(a, b, e, d, p.kchunk, p.ns, st);
  return F::template go<T64, Epi>(a, b, e, d, p.kchunk, p.ns, st);
}

// t48: the 48-column tile may be used (its loaders need a k-tile of 32 inside one tap)
static GemmPlan run16_fwd_plan(const ConvGeom& c);
// t256: the 256-row tile may be used (bf16-stored operands)
static GemmPlan fwd_plan(const ConvGeom& c, bool run, bool bf, bool t48 = false, bool t256 = false) {
  const GemmDims d = fwd_dims(c);
  return plan_gemm(d.M, d.N, run ? run_k(c) : d.K, d.groups, (double)c.out_elems() * 4, 8, bf, t48, 0, t256);
}
static GemmPlan bwdd_plan(const ConvGeom& c, bool bf, bool t48 = false, bool t256 = false) {
  const GemmDims d = bwdd_dims(c);
  return plan_gemm(d.M, d.N, d.K, d.groups, (double)c.in_elems() * 4, 8, bf, t48, 0, t256);
}
static GemmPlan bwdw_plan(const ConvGeom& c, bool run, bool bf, bool table = false) {
  const GemmDims d = bwdw_dims(c);
  return plan_gemm(run ? run_k(c) : d.M, d.N, d.K, d.groups, (double)(run ? run_w_elems(c) : c.w_elems()) * 4, 256,
                   bf, false, table ? kMaxTableK : 0);
}
// scratch sizes cover every variant (generic / run mode, fp32 / bf16) of the op
size_t conv_fwd_ws_floats(const ConvGeom& c) {
  int ns = 0;
  for (int run = 0; run < 2; ++run)
    for (int bf = 0; bf < 2; ++bf) ns = std::max(ns, fwd_plan(c, run && run_mode(c), bf).ns);
  ns = std::max(ns, fwd_plan(c, false, false, true).ns);
  ns = std::max(ns, fwd_plan(c, false, true, false, true).ns);
  if (run16_mode(c)) ns = std::max(ns, run16_fwd_plan(c).ns);
  return ns > 1 ? (size_t)ns * c.out_elems() : 0;
}
size_t conv_bwd_data_ws_floats(const ConvGeom& c) {
  const int ns = std::max(std::max(bwdd_plan(c, false).ns, bwdd_plan(c, true).ns),
                          std::max(bwdd_plan(c, false, true).ns, bwdd_plan(c, true, false, true).ns));
  return ns > 1 ? (size_t)ns * c.in_elems() : 0;
}
size_t conv_bwd_weight_ws_floats(const ConvGeom& c) {
  size_t n = 0;
  for (int bf = 0; bf < 2; ++bf)
    for (int table = 0; table < 2; ++table) {
      const GemmPlan p = bwdw_plan(c, false, bf, table);
      if (p.ns > 1) n = std::max(n, (size_t)p.ns * c.w_elems());
      if (run_mode(c)) n = std::max(n, (size_t)bwdw_plan(c, true, bf, table).ns * run_w_elems(c));
    }
  return n;
}

// ---- run mode helpers: padded copies of the forward weights / of their gradient ----
bool conv_run_mode(const ConvGeom& c) { return run_mode(c); }
size_t conv_run_w_floats(const ConvGeom& c) { return run_mode(c) ? (size_t)run_w_elems(c) : 0; }
// dir 0: wrun[(r,j)][o] = j < k*Cin ? wf[(r, j)][o] : 0;  dir 1: wf[(r,j)][o] = wrun[(r,j)][o] for j < k*Cin
__global__ void run_repack_kernel(const float* __restrict__ src, float* __restrict__ dst, int k, int kc, int run,
                                  int cout, int dir) {
  const size_t total = (size_t)k * run * cout;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // index into the padded layout
  if (i >= total) return;
  const int o = (int)(i % cout);
  const size_t q = i / cout;
  const int j = (int)(q % run), r = (int)(q / run);
  const size_t packed = ((size_t)r * kc + j) * cout + o;
  if (dir == 0)
    dst[i] = j < kc ? src[packed] : 0.f;
  else if (j < kc)
    dst[packed] = src[i];
}
int launch_conv_run_pack(const ConvGeom& c, const float* wf, float* wrun, hipStream_t st) {
  const size_t total = (size_t)run_w_elems(c);
  KernelScope ks("run_repack", 0, (double)total * 8.0, st);
  hipLaunchKernelGGL(run_repack_kernel, dim3(ceil_div(total, 256)), dim3(256), 0, st, wf, wrun, c.k, c.k * c.Cin,
                     run_len(c), c.Cout, 0);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}
static int launch_conv_run_unpack(const ConvGeom& c, const float* dwrun, float* dwf, hipStream_t st) {
  const size_t total = (size_t)run_w_elems(c);
  KernelScope ks("run_repack", 0, (double)total * 8.0, st);
  hipLaunchKernelGGL(run_repack_kernel, dim3(ceil_div(total, 256)), dim3(256), 0, st, dwrun, dwf, c.k, c.k * c.Cin,
                     run_len(c), c.Cout, 1);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

bool conv_bf16_stored_ok(const ConvGeom& c) { return conv16_ok(c) && c.Cin % 8 == 0 && c.Cout % 8 == 0; }

int launch_conv_fwd(const ConvGeom& c, const float* x, const float* wf, const float* wrun, const float* bias,
                    int relu, float* y, float* ws, hipStream_t st, const uint16_t* x16, const uint16_t* wf16,
                    uint16_t* y16) {
  // y16: also leave a bf16 copy of y there -- written by the epilogue of a single-pass product, else converted
  struct Copy16 {
    const float* y; uint16_t* y16; size_t n; hipStream_t st; bool pending;
  } copy{y, y16, (size_t)c.out_elems(), st, false};
  auto finish = [&copy](int rc) { return rc == ALEXNET_OK && copy.pending ? launch_to_bf16(copy.y, copy.y16, copy.n, copy.st) : rc; };
  const bool run = wrun && run_mode(c) && c.Cout % 4 == 0;
  AlgoFlops af(conv_flops(c), conv_bytes(c));
  GemmDims d = fwd_dims(c);
  if (g_bf16 && x16 && wf16 && !run && conv_bf16_stored_ok(c) && aligned16(x16) && aligned16(wf16)) {
    const Im2colParams a = im2col16(fwd_A(c, nullptr), x16);
    const DenseParams b = fwd_B16k(c, wf16);
    const GemmPlan p = fwd_plan(c, false, true, false, d.N % 128 == 0);  // 256-row tiles only without padded columns
    const bool tap = tap_ok(a, d, kBKbf);
    if (p.ns == 1) {
      EpiBiasAct ep{y, c.Cout, bias, relu, c.og(), 0, 0, y16};
      if (tap) return by_tile_16<ConvGatherTap16<IM2COL_FWD>>(p, a, b, ep, d, st);
      return by_tile_16<ConvGather16<IM2COL_FWD>>(p, a, b, ep, d, st);
    }
    copy.pending = y16 != nullptr;
    EpiSlab ep{ws, (long)d.M * d.N, d.N, nullptr};
    if (tap)
      AX_TRY((by_tile_16<ConvGatherTap16<IM2COL_FWD>>(p, a, b, ep, d, st)));
    else
      AX_TRY((by_tile_16<ConvGather16<IM2COL_FWD>>(p, a, b, ep, d, st)));
    return finish(launch_slab_finish(ws, p.ns, d.groups, d.M, d.N, bias, relu, nullptr, y, st));
  }
  if (run) d.K = run_k(c);
  const bool av = run || fwd_A_vec(c, x), bv = run || fwd_B_vec(c, wf);
  const bool bf = g_bf16 && av && bv;
  const Im2colParams a = run ? run_A(c, x) : fwd_A(c, x);
  const DenseParams b = run ? run_B(c, wrun) : fwd_B(c, wf);
  const bool t48 = !run && !bf && av && bv && tap_ok(a, d, kBK48);
  const GemmPlan p = fwd_plan(c, run, bf, t48);
  const bool tap = !run && !bf && av && bv && tap_ok(a, d);
  const bool tapbf = bf && !run && tap_ok(a, d, kBKbf);
  if (p.ns == 1) {
    EpiBiasAct ep{y, c.Cout, bias, relu, c.og(), 0, 0, y16};
    if (tapbf) return by_tile_bf<ConvGatherTapBf<IM2COL_FWD>>(p, a, b, ep, d, st);
    if (bf) return by_tile_bf<ConvGatherBf<IM2COL_FWD>>(p, a, b, ep, d, st);
    if (tap) return by_tile_tap<ConvGatherTap<IM2COL_FWD>>(p, a, b, ep, d, st);
    return by_tile<ConvGather<IM2COL_FWD>>(p, av, bv, a, b, ep, d, st);
  }
  EpiSlab ep{ws, (long)d.M * d.N, d.N, nullptr};
  if (tapbf)
    AX_TRY((by_tile_bf<ConvGatherTapBf<IM2COL_FWD>>(p, a, b, ep, d, st)));
  else if (bf)
    AX_TRY((by_tile_bf<ConvGatherBf<IM2COL_FWD>>(p, a, b, ep, d, st)));
  else if (tap)
    AX_TRY((by_tile_tap<ConvGatherTap<IM2COL_FWD>>(p, a, b, ep, d, st)));
  else
    AX_TRY((by_tile<ConvGather<IM2COL_FWD>>(p, av, bv, a, b, ep, d, st)));
  copy.pending = y16 != nullptr;
  return finish(launch_slab_finish(ws, p.ns, d.groups, d.M, d.N, bias, relu, nullptr, y, st));
}

// ---- the first layer over bf16 pictures with four channels per pixel (conv_plan.h, run16) ----
bool conv_run16_ok(const ConvGeom& c) { return run16_mode(c); }
size_t conv_run16_x_elems(const ConvGeom& c) { return run16_mode(c) ? (size_t)run16_x_elems(c) : 0; }
size_t conv_run16_w_elems(const ConvGeom& c) { return run16_mode(c) ? (size_t)run16_w_elems(c) : 0; }
static GemmPlan run16_fwd_plan(const ConvGeom& c) {
  const GemmDims d = fwd_dims(c);
  return plan_gemm(d.M, d.N, run16_k(c), 1, (double)c.out_elems() * 4, 8, true, false, 0, true);
}
struct ConvRun16 {
  template <class T, class Epi>
  static int go(const Im2colParams& a, const DenseParams& b, const Epi& e, const GemmDims& d, int kchunk, int ns,
                hipStream_t st) {
    return launch_tile_bf<T, Im2colKInner16<T::BM, T::BK, IM2COL_FWD>, DenseKInner16<T::BN, T::BK>, Epi>(
        a, b, e, d.M, d.N, d.K, kchunk, ns, d.groups, st);
  }
};
int launch_conv_fwd_run16(const ConvGeom& c, const uint16_t* x4, const uint16_t* wk, const float* bias, int relu,
                          float* y, float* ws, hipStream_t st, uint16_t* y16) {
  if (!run16_mode(c) || !aligned16(x4) || !aligned16(wk)) {
    set_error("conv run16: geometry or alignment does not allow it");
    return ALEXNET_EINVAL;
  }
  AlgoFlops af(conv_flops(c), conv_bytes(c));
  GemmDims d = fwd_dims(c);
  d.K = run16_k(c);
  const Im2colParams a = run16_A(c, x4);
  const DenseParams b = run16_Bk(c, wk);
  const GemmPlan p = run16_fwd_plan(c);
  if (p.ns == 1) {
    EpiBiasAct ep{y, c.Cout, bias, relu, c.og(), 0, 0, y16};
    if (p.bm == 256 && d.N % 96 == 0 && d.N % 128 != 0)  // whole 96-column tiles instead of padded 128-column ones
      return ConvRun16::go<B256n96, EpiBiasAct>(a, b, ep, d, round_up(d.K, kBKbf), 1, st);
    return by_tile_16<ConvRun16>(p, a, b, ep, d, st);
  }
  EpiSlab ep{ws, (long)d.M * d.N, d.N, nullptr};
  AX_TRY((by_tile_16<ConvRun16>(p, a, b, ep, d, st)));
  AX_TRY(launch_slab_finish(ws, p.ns, 1, d.M, d.N, bias, relu, nullptr, y, st));
  return y16 ? launch_to_bf16(y, y16, (size_t)c.out_elems(), st) : ALEXNET_OK;
}
// ---- strided backward data by phases (conv_plan.h) ----
bool conv_phase_mode(const ConvGeom& c) { return phase_mode(c) && c.Cout % 4 == 0 && phase_n(c) % 4 == 0; }
size_t conv_phase_w_floats(const ConvGeom& c) { return conv_phase_mode(c) ? (size_t)phase_w_elems(c) : 0; }
__global__ void phase_pack_kernel(const float* __restrict__ wf, float* __restrict__ wp, int k, int st, int ka, int cin,
                                  int cout) {
  const int pn = st * st * cin;
  const size_t total = (size_t)ka * ka * cout * pn;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // index into wp[(a,b,o)][(py,px,c)]
  if (i >= total) return;
  const int col = (int)(i % pn);
  size_t q = i / pn;
  const int o = (int)(q % cout);
  q /= cout;
  const int b = (int)(q % ka), a = (int)(q / ka);
  const int c = col % cin, pp = col / cin, px = pp % st, py = pp / st;
  const int r = py + st * a, s = px + st * b;
  wp[i] = (r < k && s < k) ? wf[((size_t)(r * k + s) * cin + c) * cout + o] : 0.f;
}
static int launch_conv_bwd_data_phases(const ConvGeom& c, const float* dy, const float* wf, float* wphase, float* dx,
                                       hipStream_t st) {
  const size_t total = (size_t)phase_w_elems(c);
  {
    KernelScope ks("phase_pack", 0, (double)total * 8.0, st);
    hipLaunchKernelGGL(phase_pack_kernel, dim3(ceil_div(total, 256)), dim3(256), 0, st, wf, wphase, c.k, c.stride,
                       phase_taps(c), c.Cin, c.Cout);
    AX_LAUNCH_CHECK();
  }
  const GemmDims d = phase_dims(c);
  AlgoFlops af(conv_flops(c), conv_bytes(c));
  GemmPlan p = plan_gemm(d.M, d.N, d.K, 1, 0, 1, false);  // never split: the epilogue scatters; fp32 only
  return by_tile<ConvGather<IM2COL_T1>>(p, true, true, phase_A(c, dy), phase_B(c, wphase), phase_epilogue(c, dx), d,
                                        st);
}

int launch_conv_bwd_data(const ConvGeom& c, const float* dy, const float* wf, const float* wb, float* wphase,
                         const float* gate, float* dx, float* ws, hipStream_t st, const uint16_t* dy16,
                         const uint16_t* wb16, uint16_t* dx16) {
  // dx16: also leave a bf16 copy of dx there (see launch_conv_fwd)
  struct Copy16 {
    const float* y; uint16_t* y16; size_t n; hipStream_t st; bool pending;
  } copy{dx, dx16, (size_t)c.in_elems(), st, false};
  auto finish = [&copy](int rc) { return rc == ALEXNET_OK && copy.pending ? launch_to_bf16(copy.y, copy.y16, copy.n, copy.st) : rc; };
  if (wphase && !gate && conv_phase_mode(c) && aligned16(dy)) {
    copy.pending = dx16 != nullptr;
    return finish(launch_conv_bwd_data_phases(c, dy, wf, wphase, dx, st));
  }
  const GemmDims d = bwdd_dims(c);
  AlgoFlops af(conv_flops(c), conv_bytes(c));
  if (g_bf16 && dy16 && wb16 && conv_bf16_stored_ok(c) && aligned16(dy16) && aligned16(wb16)) {
    const Im2colParams a = im2col16(bwdd_A(c, nullptr), dy16);
    const DenseParams b = bwdd_B16k(c, wb16);
    const GemmPlan p = bwdd_plan(c, true, false, d.N % 128 == 0);
    const bool tap = tap_ok(a, d, kBKbf);
    if (p.ns == 1) {
      EpiGate ep{dx, c.Cin, gate, c.cg(), 0, 0, dx16};
      if (tap) return by_tile_16<ConvGatherTap16<IM2COL_T1>>(p, a, b, ep, d, st);
      return by_tile_16<ConvGather16<IM2COL_T1>>(p, a, b, ep, d, st);
    }
    copy.pending = dx16 != nullptr;
    EpiSlab ep{ws, (long)d.M * d.N, d.N, nullptr};
    if (tap)
      AX_TRY((by_tile_16<ConvGatherTap16<IM2COL_T1>>(p, a, b, ep, d, st)));
    else
      AX_TRY((by_tile_16<ConvGather16<IM2COL_T1>>(p, a, b, ep, d, st)));
    return finish(launch_slab_finish(ws, p.ns, d.groups, d.M, d.N, nullptr, 0, gate, dx, st));
  }
  const bool av = bwdd_A_vec(c, dy) && bwdd_B_vec(c, wb), bv = bwdd_B_vec(c, wb);
  const bool bf = g_bf16 && av && bv && c.stride == 1;
  const Im2colParams a = bwdd_A(c, dy);
  const DenseParams b = bwdd_B(c, wb);
  const bool t48 = !bf && c.stride == 1 && av && bv && tap_ok(a, d, kBK48);
  const GemmPlan p = bwdd_plan(c, bf, t48);
  const bool tap = !bf && c.stride == 1 && av && bv && tap_ok(a, d);
  const bool tapbf = bf && tap_ok(a, d, kBKbf);
  if (p.ns == 1) {
    EpiGate ep{dx, c.Cin, gate, c.cg(), 0, 0, dx16};
    if (tapbf) return by_tile_bf<ConvGatherTapBf<IM2COL_T1>>(p, a, b, ep, d, st);
    if (bf) return by_tile_bf<ConvGatherBf<IM2COL_T1>>(p, a, b, ep, d, st);
    if (tap) return by_tile_tap<ConvGatherTap<IM2COL_T1>>(p, a, b, ep, d, st);
    if (c.stride == 1) return by_tile<ConvGather<IM2COL_T1>>(p, av, bv, a, b, ep, d, st);
    return by_tile<ConvGather<IM2COL_TS>>(p, av, bv, a, b, ep, d, st);
  }
  EpiSlab ep{ws, (long)d.M * d.N, d.N, nullptr};
  if (tapbf)
    AX_TRY((by_tile_bf<ConvGatherTapBf<IM2COL_T1>>(p, a, b, ep, d, st)));
  else if (bf)
    AX_TRY((by_tile_bf<ConvGatherBf<IM2COL_T1>>(p, a, b, ep, d, st)));
  else if (tap)
    AX_TRY((by_tile_tap<ConvGatherTap<IM2COL_T1>>(p, a, b, ep, d, st)));
  else if (c.stride == 1)
    AX_TRY((by_tile<ConvGather<IM2COL_T1>>(p, av, bv, a, b, ep, d, st)));
  else
    AX_TRY((by_tile<ConvGather<IM2COL_TS>>(p, av, bv, a, b, ep, d, st)));
  copy.pending = dx16 != nullptr;
  return finish(launch_slab_finish(ws, p.ns, d.groups, d.M, d.N, nullptr, 0, gate, dx, st));
}

// defer_ns (generic layout only): the split-k slices are left in ws, [group][slice][slab], and their number is
// returned there for the caller to add them up later (1: the result is in dwf already)
int launch_conv_bwd_weight(const ConvGeom& c, const float* x, const float* dy, float* dwf, float* dwrun, float* ws,
                           hipStream_t st, int* defer_ns, const uint16_t* x16, const uint16_t* dy16) {
  const bool run = dwrun && run_mode(c) && bwdw_B_vec(c, dy);
  AlgoFlops af(conv_flops(c), conv_bytes(c));
  GemmDims d = bwdw_dims(c);
  if (run) d.M = run_k(c);
  const bool av = run || bwdw_A_vec(c, x), bv = bwdw_B_vec(c, dy);
  const bool bf = g_bf16 && av && bv;
  const Im2colParams a = run ? run_A(c, x) : bwdw_A(c, x);
  bool table = av && bv && table_ok(a, d) && (!bf || d.K % kBKbf == 0);
  GemmPlan p = bwdw_plan(c, run, bf, table);
  if (table && p.kchunk > kMaxTableK) {  // no split count within reach keeps the k range inside the table
    table = false;
    p = bwdw_plan(c, run, bf, false);
  }
  const long slab = (long)d.M * d.N;
  float* out = run ? dwrun : dwf;
  EpiSlab ep{p.ns > 1 ? ws : out, slab, d.N, nullptr};
  const bool s16 = bf && table && !run && x16 && dy16 && conv_bf16_stored_ok(c) && aligned16(x16) && aligned16(dy16);
  if (s16)
    AX_TRY((by_tile_bf<ConvWeightGradTable16>(p, im2col16(a, x16), dense16(bwdw_B(c, dy), dy16), ep, d, st)));
  else if (bf && table)
    AX_TRY((by_tile_bf<ConvWeightGradTableBf>(p, a, bwdw_B(c, dy), ep, d, st)));
  else if (bf)
    AX_TRY((by_tile_bf<ConvWeightGradBf>(p, a, bwdw_B(c, dy), ep, d, st)));
  else if (table)
    AX_TRY((by_tile_tap<ConvWeightGradTable>(p, a, bwdw_B(c, dy), ep, d, st)));
  else
    AX_TRY((by_tile<ConvWeightGrad>(p, av, bv, a, bwdw_B(c, dy), ep, d, st)));
  if (defer_ns && !run) {
    *defer_ns = p.ns;
    return ALEXNET_OK;
  }
  if (defer_ns) *defer_ns = 1;
  if (run && p.ns > 1)  // slices of the padded layout straight to the packed one
    return launch_reduce_slabs_unpack(ws, p.ns, slab, run_len(c), c.k * c.Cin, c.Cout, dwf, st);
  if (p.ns > 1) AX_TRY(launch_reduce_slabs(ws, p.ns, slab, d.groups, out, st));
  if (run) AX_TRY(launch_conv_run_unpack(c, dwrun, dwf, st));
  return ALEXNET_OK;
}

// ------------------------------------------------------------ dense layers ---
// y = act(x w^T + b),  dx = gate(dy w),  dw = dy^T x.  The batch is the small
// dimension, so forward and backward-data split the reduction over several
// workgroups and finish in a second kernel that also applies the activation.
// The dense layers always use the 128 x 128 tile.

static int fc_split(int B, int N, int K, int* kchunk, bool bf) {
  const int bk = bf ? kBKbf : kBK;
  const int ktiles = ceil_div(K, bk);
  const long tiles = (long)ceil_div(B, 128) * ceil_div(N, 128);
  const double t_tile = 2.0 * 128 * 128 * (double)ktiles * bk / (0.614e12 * (bf ? 3.2 : 0.8));
  int best = 1, best_per = ktiles;
  double best_t = 1e30;
  for (int s = 1; s <= 64 && s <= ktiles; ++s) {
    const int per = ceil_div(ktiles, s);
    if (ceil_div(ktiles, per) != s) continue;
    if (s > 1 && per < 6) break;
    double t = (double)ceil_div(tiles * s, 256) * t_tile * per / ktiles;
    if (s > 1) t += (s + 1) * (double)B * N * 4 / 2.5e12;
    if (t < best_t * 0.98) {
      best_t = t;
      best = s;
      best_per = per;
    }
  }
  *kchunk = best_per * bk;
  return best;
}
size_t fc_ws_floats(int B, int in, int out) {
  int kc;
  size_t n = 0;
  for (int bf = 0; bf < 2; ++bf) {
    n = std::max(n, (size_t)fc_split(B, out, in, &kc, bf) * B * out);
    n = std::max(n, (size_t)fc_split(B, in, out, &kc, bf) * B * in);
  }
  return n;
}

__global__ void fc_fwd_finish_kernel(const float* __restrict__ ws, int nsplit, int B, int out, FcAct act,
                                     float* __restrict__ y, uint16_t* __restrict__ y16) {
  const size_t total = (size_t)B * out;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  float s = 0.f;
#pragma unroll 8
  for (int k = 0; k < nsplit; ++k) s += ws[(size_t)k * total + i];  // loads in flight together, added in order
  const int o = (int)(i % out);
  if (act.bias) s += act.bias[o];
  if (act.relu) s = s > 0.f ? s : 0.f;
  if (act.dropout && !dropout_keep(act.key, act.tag, i, act.thresh24)) s = 0.f;
  y[i] = s * act.scale;
  if (y16) store_bf16(y16 + i, s * act.scale);
}
__global__ void fc_bwd_finish_kernel(const float* __restrict__ ws, int nsplit, size_t total,
                                     const float* __restrict__ gate, float* __restrict__ dx,
                                     uint16_t* __restrict__ dx16) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  float s = 0.f;
#pragma unroll 8
  for (int k = 0; k < nsplit; ++k) s += ws[(size_t)k * total + i];  // loads in flight together, added in order
  if (gate && !(gate[i] > 0.f)) s = 0.f;
  dx[i] = s;
  if (dx16) store_bf16(dx16 + i, s);
}

static inline bool vec_ok(const float* p, long ld) { return aligned16(p) && ld % 4 == 0; }

template <template <int, int, bool> class ALT, template <int, int, bool> class BLT>
static int launch_dense(bool vec, const DenseParams& a, const DenseParams& b, const EpiSlab& ep, int M, int N, int K,
                        int kchunk, int ns, hipStream_t st) {
  if (vec)
    return launch_tile<T128, ALT<128, kBK, true>, BLT<128, kBK, true>, EpiSlab>(a, b, ep, M, N, K, kchunk, ns, 1, st);
  return launch_tile<T128, ALT<128, kBK, false>, BLT<128, kBK, false>, EpiSlab>(a, b, ep, M, N, K, kchunk, ns, 1, st);
}

typedef BfRowMajor<DenseKInner<128, kBKbf, true>, 128, kBKbf> BfDenseK;
typedef BfDenseRowInner<128, kBKbf> BfDenseR;

typedef DenseKInner16<128, kBKbf> Dense16K;
typedef DenseRowInner16<128, kBKbf> Dense16R;
bool fc_bf16_stored_ok(int in, int out) { return in % 8 == 0 && out % 8 == 0; }
static inline DenseParams dense16_of(const uint16_t* p, long ld, int rows, size_t elems) {
  return DenseParams{reinterpret_cast<const float*>(p), ld, 0, rows, (uint32_t)(elems * 2)};
}

int launch_fc_fwd(int B, int in, int out, const float* x, const float* w, const FcAct& act, float* y, float* ws,
                  hipStream_t st, const uint16_t* x16, const uint16_t* w16, uint16_t* y16) {
  const bool vec = vec_ok(x, in) && vec_ok(w, in), bf = g_bf16 && vec;
  const bool s16 = bf && x16 && w16 && fc_bf16_stored_ok(in, out) && aligned16(x16) && aligned16(w16);
  int kchunk;
  const int ns = fc_split(B, out, in, &kchunk, bf);
  DenseParams a{x, in, 0, B, (uint32_t)((size_t)B * in * 4)};
  DenseParams b{w, in, 0, out, (uint32_t)((size_t)out * in * 4)};
  EpiSlab ep{ws, (long)B * out, out, nullptr};
  // both operands run along k = in
  if (s16)
    AX_TRY((launch_tile_bf<B128, Dense16K, Dense16K, EpiSlab>(dense16_of(x16, in, B, (size_t)B * in),
                                                                dense16_of(w16, in, out, (size_t)out * in), ep, B, out,
                                                                in, kchunk, ns, 1, st)));
  else if (bf)
    AX_TRY((launch_tile_bf<B128, BfDenseK, BfDenseK, EpiSlab>(a, b, ep, B, out, in, kchunk, ns, 1, st)));
  else
    AX_TRY((launch_dense<DenseKInner, DenseKInner>(vec, a, b, ep, B, out, in, kchunk, ns, st)));
  const size_t total = (size_t)B * out;
  KernelScope ks("fc_finish", 0, (double)total * 4.0 * (ns + 1), st);
  hipLaunchKernelGGL(fc_fwd_finish_kernel, dim3(ceil_div(total, 256)), dim3(256), 0, st, ws, ns, B, out, act, y, y16);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

int launch_fc_bwd_data(int B, int in, int out, const float* dy, const float* w, const float* gate, float* dx,
                       float* ws, hipStream_t st, const uint16_t* dy16, const uint16_t* w16, uint16_t* dx16) {
  const bool vec = vec_ok(dy, out) && vec_ok(w, in), bf = g_bf16 && vec;
  const bool s16 = bf && dy16 && w16 && fc_bf16_stored_ok(in, out) && aligned16(dy16) && aligned16(w16);
  int kchunk;
  const int ns = fc_split(B, in, out, &kchunk, bf);
  DenseParams a{dy, out, 0, B, (uint32_t)((size_t)B * out * 4)};
  DenseParams b{w, in, 0, in, (uint32_t)((size_t)out * in * 4)};
  EpiSlab ep{ws, (long)B * in, in, nullptr};
  // A runs along k = out, B along its rows = in
  if (s16)
    AX_TRY((launch_tile_bf<B128, Dense16K, Dense16R, EpiSlab>(dense16_of(dy16, out, B, (size_t)B * out),
                                                                dense16_of(w16, in, in, (size_t)out * in), ep, B, in,
                                                                out, kchunk, ns, 1, st)));
  else if (bf)
    AX_TRY((launch_tile_bf<B128, BfDenseK, BfDenseR, EpiSlab>(a, b, ep, B, in, out, kchunk, ns, 1, st)));
  else
    AX_TRY((launch_dense<DenseKInner, DenseRowInner>(vec, a, b, ep, B, in, out, kchunk, ns, st)));
  const size_t total = (size_t)B * in;
  KernelScope ks("fc_finish", 0, (double)total * 4.0 * (ns + 1 + (gate ? 1 : 0)), st);
  hipLaunchKernelGGL(fc_bwd_finish_kernel, dim3(ceil_div(total, 256)), dim3(256), 0, st, ws, ns, total, gate, dx,
                     dx16);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

int launch_fc_bwd_weight(int B, int in, int out, const float* x, const float* dy, float* dw, hipStream_t st,
                         const uint16_t* x16, const uint16_t* dy16) {
  DenseParams a{dy, out, 0, out, (uint32_t)((size_t)B * out * 4)};
  DenseParams b{x, in, 0, in, (uint32_t)((size_t)B * in * 4)};
  EpiSlab ep{dw, (long)out * in, in, nullptr};
  const bool vec = vec_ok(dy, out) && vec_ok(x, in);
  if (g_bf16 && vec && x16 && dy16 && fc_bf16_stored_ok(in, out) && aligned16(x16) && aligned16(dy16))
    return launch_tile_bf<B128, Dense16R, Dense16R, EpiSlab>(dense16_of(dy16, out, out, (size_t)B * out),
                                                             dense16_of(x16, in, in, (size_t)B * in), ep, out, in, B,
                                                             round_up(B, kBKbf), 1, 1, st);
  if (g_bf16 && vec)
    return launch_tile_bf<B128, BfDenseR, BfDenseR, EpiSlab>(a, b, ep, out, in, B, round_up(B, kBKbf), 1, 1, st);
  return launch_dense<DenseRowInner, DenseRowInner>(vec, a, b, ep, out, in, B, round_up(B, kBK), 1, st);
}

}  // namespace ax
