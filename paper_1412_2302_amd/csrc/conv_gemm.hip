// Convolution forward, backward-data and backward-weight as implicit GEMMs on
// the fp32 MFMA core (gemm.h), and the dense layers on the same core.
#include "kernels.h"

namespace ax {

typedef Tile<128, 128, 16, 2, 2> T128;
typedef Tile<128, 96, 16, 4, 1> T96;
typedef Tile<128, 64, 16, 4, 1> T64;

// Width of the N tile that wastes the fewest padded columns (ties: wider).
static int pick_bn(int N) {
  const int opts[3] = {128, 96, 64};
  int best = 128;
  long best_cost = -1;
  for (int i = 0; i < 3; ++i) {
    const long cost = (long)ceil_div(N, opts[i]) * opts[i];
    if (best_cost < 0 || cost < best_cost) {
      best_cost = cost;
      best = opts[i];
    }
  }
  return best;
}

static const int kTargetBlocks = 512;  // two workgroups per compute unit

template <class T, template <int, int> class ALT, template <int, int> class BLT, class Epi>
static int launch_tile(const typename ALT<T::BM, T::BK>::Params& ap, const typename BLT<T::BN, T::BK>::Params& bp,
                       const Epi& ep, int M, int N, int K, int kchunk, int nsplit, int groups, hipStream_t st) {
  if (M <= 0 || N <= 0) return ALEXNET_OK;
  dim3 grid(ceil_div(M, T::BM), ceil_div(N, T::BN), groups * nsplit);
  if (grid.y > 65535 || grid.z > 65535) {
    set_error("GEMM grid too large (%u,%u,%u)", grid.x, grid.y, grid.z);
    return ALEXNET_ESHAPE;
  }
  KernelScope ks("gemm", 2.0 * M * N * (double)K * groups, 0, st);
  hipLaunchKernelGGL((gemm_kernel<T, ALT<T::BM, T::BK>, BLT<T::BN, T::BK>, Epi>), grid, dim3(kThreads), 0, st, ap, bp,
                     ep, M, N, K, kchunk, nsplit);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

template <template <int, int> class ALT, template <int, int> class BLT, class AP, class BP, class Epi>
static int launch_any(int bn, const AP& ap, const BP& bp, const Epi& ep, int M, int N, int K, int kchunk, int nsplit,
                      int groups, hipStream_t st) {
  switch (bn) {
    case 128: return launch_tile<T128, ALT, BLT, Epi>(ap, bp, ep, M, N, K, kchunk, nsplit, groups, st);
    case 96: return launch_tile<T96, ALT, BLT, Epi>(ap, bp, ep, M, N, K, kchunk, nsplit, groups, st);
    default: return launch_tile<T64, ALT, BLT, Epi>(ap, bp, ep, M, N, K, kchunk, nsplit, groups, st);
  }
}

static inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

// ------------------------------------------------------------- convolution ---
int launch_conv_fwd(const ConvGeom& c, const float* x, const float* wf, const float* bias, int relu, float* y,
                    hipStream_t st) {
  const GemmDims d = fwd_dims(c);
  EpiBiasAct ep{y, c.Cout, bias, relu, c.og(), 0};
  return launch_any<Im2colKInner, DenseRowInner>(pick_bn(d.N), fwd_A(c, x), fwd_B(c, wf), ep, d.M, d.N, d.K,
                                                 round_up(d.K, 16), 1, d.groups, st);
}

int launch_conv_bwd_data(const ConvGeom& c, const float* dy, const float* wb, const float* gate, float* dx,
                         hipStream_t st) {
  const GemmDims d = bwdd_dims(c);
  EpiGate ep{dx, c.Cin, gate, c.cg(), 0};
  return launch_any<Im2colKInner, DenseRowInner>(pick_bn(d.N), bwdd_A(c, dy), bwdd_B(c, wb), ep, d.M, d.N, d.K,
                                                 round_up(d.K, 16), 1, d.groups, st);
}

static int bwdw_split(const ConvGeom& c, int* kchunk, int* bn) {
  const GemmDims d = bwdw_dims(c);
  *bn = pick_bn(d.N);
  const long tiles = (long)ceil_div(d.M, 128) * ceil_div(d.N, *bn) * d.groups;
  return plan_split(tiles, d.K, 16, kTargetBlocks, 256, kchunk);
}
size_t conv_bwd_weight_ws_floats(const ConvGeom& c) {
  int kchunk, bn;
  const int ns = bwdw_split(c, &kchunk, &bn);
  return ns > 1 ? (size_t)ns * c.w_elems() : 0;
}
int launch_conv_bwd_weight(const ConvGeom& c, const float* x, const float* dy, float* dwf, float* ws,
                           hipStream_t st) {
  const GemmDims d = bwdw_dims(c);
  int kchunk, bn;
  const int ns = bwdw_split(c, &kchunk, &bn);
  const long slab = (long)d.M * d.N;
  EpiSlab ep{ns > 1 ? ws : dwf, slab, d.N, nullptr};
  AX_TRY((launch_any<Im2colRowInner, DenseRowInner>(bn, bwdw_A(c, x), bwdw_B(c, dy), ep, d.M, d.N, d.K, kchunk, ns,
                                                    d.groups, st)));
  if (ns > 1) AX_TRY(launch_reduce_slabs(ws, ns, slab, d.groups, dwf, st));
  return ALEXNET_OK;
}

// ------------------------------------------------------------ dense layers ---
// y = act(x w^T + b),  dx = gate(dy w),  dw = dy^T x.  The batch is the small
// dimension, so forward and backward-data split the reduction over several
// workgroups and finish in a second kernel that also applies the activation.

static int fc_split(int B, int N, int K, int* kchunk) {
  const long tiles = (long)ceil_div(B, 128) * ceil_div(N, 128);
  return plan_split(tiles, K, 16, kTargetBlocks / 2, 64, kchunk);
}
size_t fc_ws_floats(int B, int in, int out) {
  int kc;
  const size_t f = (size_t)fc_split(B, out, in, &kc) * B * out;
  const size_t b = (size_t)fc_split(B, in, out, &kc) * B * in;
  return f > b ? f : b;
}

__global__ void fc_fwd_finish_kernel(const float* __restrict__ ws, int nsplit, int B, int out, FcAct act,
                                     float* __restrict__ y) {
  const size_t total = (size_t)B * out;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  float s = 0.f;
  for (int k = 0; k < nsplit; ++k) s += ws[(size_t)k * total + i];
  const int o = (int)(i % out);
  if (act.bias) s += act.bias[o];
  if (act.relu) s = s > 0.f ? s : 0.f;
  if (act.dropout && !dropout_keep(act.key, act.tag, i, act.thresh24)) s = 0.f;
  y[i] = s * act.scale;
}
__global__ void fc_bwd_finish_kernel(const float* __restrict__ ws, int nsplit, size_t total,
                                     const float* __restrict__ gate, float* __restrict__ dx) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  float s = 0.f;
  for (int k = 0; k < nsplit; ++k) s += ws[(size_t)k * total + i];
  if (gate && !(gate[i] > 0.f)) s = 0.f;
  dx[i] = s;
}

static inline bool vec_ok(const float* p, long ld) { return aligned16(p) && ld % 4 == 0; }

int launch_fc_fwd(int B, int in, int out, const float* x, const float* w, const FcAct& act, float* y, float* ws,
                  hipStream_t st) {
  int kchunk;
  const int ns = fc_split(B, out, in, &kchunk);
  DenseParams a{x, in, 0, B, vec_ok(x, in) ? 1 : 0};
  DenseParams b{w, in, 0, out, vec_ok(w, in) ? 1 : 0};
  EpiSlab ep{ws, (long)B * out, out, nullptr};
  AX_TRY((launch_tile<T128, DenseKInner, DenseKInner, EpiSlab>(a, b, ep, B, out, in, kchunk, ns, 1, st)));
  const size_t total = (size_t)B * out;
  KernelScope ks("fc_finish", 0, (double)total * 4.0 * (ns + 1), st);
  hipLaunchKernelGGL(fc_fwd_finish_kernel, dim3(ceil_div(total, 256)), dim3(256), 0, st, ws, ns, B, out, act, y);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

int launch_fc_bwd_data(int B, int in, int out, const float* dy, const float* w, const float* gate, float* dx,
                       float* ws, hipStream_t st) {
  int kchunk;
  const int ns = fc_split(B, in, out, &kchunk);
  DenseParams a{dy, out, 0, B, vec_ok(dy, out) ? 1 : 0};
  DenseParams b{w, in, 0, in, vec_ok(w, in) ? 1 : 0};
  EpiSlab ep{ws, (long)B * in, in, nullptr};
  AX_TRY((launch_tile<T128, DenseKInner, DenseRowInner, EpiSlab>(a, b, ep, B, in, out, kchunk, ns, 1, st)));
  const size_t total = (size_t)B * in;
  KernelScope ks("fc_finish", 0, (double)total * 4.0 * (ns + 1 + (gate ? 1 : 0)), st);
  hipLaunchKernelGGL(fc_bwd_finish_kernel, dim3(ceil_div(total, 256)), dim3(256), 0, st, ws, ns, total, gate, dx);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

int launch_fc_bwd_weight(int B, int in, int out, const float* x, const float* dy, float* dw, hipStream_t st) {
  DenseParams a{dy, out, 0, out, vec_ok(dy, out) ? 1 : 0};
  DenseParams b{x, in, 0, in, vec_ok(x, in) ? 1 : 0};
  EpiSlab ep{dw, (long)out * in, in, nullptr};
  return launch_tile<T128, DenseRowInner, DenseRowInner, EpiSlab>(a, b, ep, out, in, B, round_up(B, 16), 1, 1, st);
}

}  // namespace ax
