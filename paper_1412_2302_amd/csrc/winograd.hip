// Kernels and launchers of the F(4x4, 3x3) convolution path (see winograd.h): five bandwidth-bound
// transforms; the 36 channel products between them are launched through the grouped implicit-GEMM
// kernels as a 1x1 convolution with 36*groups groups.
#include "winograd.h"

#include <algorithm>

#include "kernels.h"

namespace ax {

__global__ void __launch_bounds__(256) wino_in_kernel(WinoGeom g, int Cg, const float* __restrict__ x,
                                                       float* __restrict__ V, long total) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < total) wino_in_thread(g, Cg, x, V, idx);
}
__global__ void __launch_bounds__(256) wino_dy_kernel(WinoGeom g, int Og, const float* __restrict__ dy,
                                                       float* __restrict__ Y, long total) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < total) wino_dy_thread(g, Og, dy, Y, idx);
}
__global__ void __launch_bounds__(256) wino_out_kernel(WinoGeom g, int Ng, const float* __restrict__ M,
                                                        const float* __restrict__ bias, int relu,
                                                        const float* __restrict__ gate, float* __restrict__ y,
                                                        long total) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < total) wino_out_thread(g, Ng, M, bias, relu, gate, y, idx);
}
__global__ void __launch_bounds__(256) wino_filter_kernel(int groups, int Na, int Nb, int k, int nsub, int q_in_cols,
                                                           const float* __restrict__ w, float* __restrict__ U,
                                                           long total) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < total) wino_filter_thread(groups, Na, Nb, k, nsub, q_in_cols, w, U, idx);
}
// one workgroup per (picture, block of CQ channel quads); dynamic LDS: H*W*CQ float4
__global__ void __launch_bounds__(256) wino_dx_kernel(WinoDx d, int rounds, const float* __restrict__ M,
                                                       const float* __restrict__ gate, float* __restrict__ dx) {
  extern __shared__ __attribute__((aligned(16))) float4 wino_dx_lds[];
  Vec4* lds = reinterpret_cast<Vec4*>(wino_dx_lds);
  const int tid = threadIdx.x;
  const WinoDxPlan plan = wino_dx_plan(d, blockIdx.x);
  wino_dx_zero(d, lds, tid);
  __syncthreads();
  for (int r = 0; r < rounds; ++r) {
    Vec2 z[36];
    const WinoDxTask task = wino_dx_load(d, plan, M, tid, r, z);
    int lo, hi;  // the same for every thread of the block
    wino_dx_round_phases(d, plan, r, &lo, &hi);
    for (int ph = lo; ph <= hi; ++ph) {
      wino_dx_add(d, plan, lds, tid, task, z, ph);
      __syncthreads();
    }
  }
  wino_dx_flush(d, plan, lds, gate, dx, tid);
}
__global__ void __launch_bounds__(256) wino_dw_kernel(int groups, int Na, int Nb, int k, int nsub,
                                                       const float* __restrict__ dU, float* __restrict__ dw,
                                                       long total) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < total) wino_dw_thread(groups, Na, Nb, k, nsub, dU, dw, idx);
}
// the same for several stages in one launch (see WgradTail): the jobs' grids laid end to end
__global__ void __launch_bounds__(256) wino_dw_batch_kernel(WgradTail t) {
  int ji = 0;
#pragma unroll
  for (int k = 1; k < kMaxWgradJobs; ++k)
    if (k < t.n && (int)blockIdx.x >= t.first_t[k]) ji = k;
  const WgradJob& j = t.job[ji];
  const long idx = (long)(blockIdx.x - t.first_t[ji]) * blockDim.x + threadIdx.x;
  if (idx < j.total) wino_dw_thread(j.groups, j.Na, j.Nb, j.k, j.nsub, j.dU, j.dwf, idx);
}

// ---- geometry ----------------------------------------------------------------------------------
static inline int nsub_of(const ConvGeom& c) { return (c.k + 2) / 3; }
static inline int nq_of(const ConvGeom& c) { return nsub_of(c) * nsub_of(c); }
static WinoGeom fwd_geom(const ConvGeom& c) {
  return WinoGeom{c.B, c.H, c.W, c.pad, c.Ho, c.Wo, (c.Ho + 3) / 4, (c.Wo + 3) / 4, c.groups, c.k, nsub_of(c)};
}
bool wino_ok(const ConvGeom& c) {
  if ((c.k != 3 && c.k != 5) || c.stride != 1 || c.pad > c.k - 1 || c.cg() % 4 || c.og() % 4) return false;
  // the transformed tensors are 36/16 (tiles cut exactly) to ~4x larger than the activations, times the
  // number of sub-kernels on the gathered side
  return (long)fwd_geom(c).tiles() * 36 * std::max(nq_of(c) * c.Cin, c.Cout) <= 0x1ffffff0L;
}
// The data gradient is the adjoint of the forward form: the products of the transformed output gradient (the
// one the weight gradient uses) with the transformed taps go back through B . Bt, overlapping patches added up
// in LDS (wino_dx_kernel), which needs one picture row of one channel quad to fit the budget at the very least.
// (The other way, the forward form applied to dy with reversed taps, needs a second transform of dy -- four of
// them, with Cout channels each, for a 5x5 layer -- and measured 15-20 us slower per 3x3 layer.)
constexpr size_t kDxLdsBytes = 48 * 1024;
bool wino_bwd_data_ok(const ConvGeom& c) { return wino_ok(c) && (size_t)c.W * 16 <= kDxLdsBytes; }
// multiplies of the direct form per multiply of the products, at this map size
double wino_gain(const ConvGeom& c) {
  const double covered = (double)c.Ho * c.Wo / (16.0 * ((c.Ho + 3) / 4) * ((c.Wo + 3) / 4));
  return covered * 16.0 * c.k * c.k / (36.0 * nq_of(c));
}
// the 36*groups channel products as a 1x1 grouped convolution over one row of `tiles` pixels
static ConvGeom product_geom(int tiles, int groups, int kin, int nout) {
  ConvGeom p;
  p.B = 1; p.H = 1; p.W = tiles; p.Cin = 36 * groups * kin; p.Cout = 36 * groups * nout;
  p.k = 1; p.stride = 1; p.pad = 0; p.groups = 36 * groups; p.Ho = 1; p.Wo = tiles;
  return p;
}
size_t wino_v_floats(const ConvGeom& c) { return (size_t)fwd_geom(c).tiles() * 36 * nq_of(c) * c.Cin; }
size_t wino_u_floats(const ConvGeom& c) { return (size_t)36 * nq_of(c) * c.cg() * c.og() * c.groups; }
size_t wino_scratch_floats(const ConvGeom& c) {
  const size_t tf = (size_t)fwd_geom(c).tiles();
  size_t n = 36 * tf * c.Cout;  // forward products, transformed output gradient
  if (wino_bwd_data_ok(c)) n = std::max(n, 36 * tf * nq_of(c) * c.Cin);  // data-gradient products
  return n;
}
// split-k slices of the weight-gradient products alone (the part of wino_gemm_ws_floats() that a deferred tail
// keeps to itself)
size_t wino_wgrad_ws_floats(const ConvGeom& c) {
  return conv_bwd_weight_ws_floats(product_geom(fwd_geom(c).tiles(), c.groups, nq_of(c) * c.cg(), c.og()));
}
size_t wino_gemm_ws_floats(const ConvGeom& c) {
  const ConvGeom pf = product_geom(fwd_geom(c).tiles(), c.groups, nq_of(c) * c.cg(), c.og());
  size_t n = std::max(conv_fwd_ws_floats(pf), conv_bwd_weight_ws_floats(pf));
  if (wino_bwd_data_ok(c))
    n = std::max(n, conv_fwd_ws_floats(product_geom(fwd_geom(c).tiles(), c.groups, c.og(), nq_of(c) * c.cg())));
  return n;
}

// ---- launchers -----------------------------------------------------------------------------------
static inline dim3 blocks_for(long total) { return dim3((unsigned)((total + 255) / 256)); }

int launch_wino_filter(const ConvGeom& c, const float* wf, float* U, hipStream_t st) {
  const long total = (long)c.groups * nq_of(c) * c.cg() * (c.og() / 4);
  KernelScope ks("wino_filter", 0, ((double)c.w_elems() + (double)wino_u_floats(c)) * 4.0, st);
  hipLaunchKernelGGL(wino_filter_kernel, blocks_for(total), dim3(256), 0, st, c.groups, c.cg(), c.og(), c.k, nsub_of(c),
                     0, wf, U, total);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}
int launch_wino_filter_bwd(const ConvGeom& c, const float* wb, float* Ub, hipStream_t st) {
  const long total = (long)c.groups * nq_of(c) * c.og() * (c.cg() / 4);
  KernelScope ks("wino_filter", 0, ((double)c.w_elems() + (double)wino_u_floats(c)) * 4.0, st);
  // the operand of the data-gradient products: [z][o][(q, c)]
  hipLaunchKernelGGL(wino_filter_kernel, blocks_for(total), dim3(256), 0, st, c.groups, c.og(), c.cg(), c.k, nsub_of(c),
                     1, wb, Ub, total);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

int launch_wino_input(const ConvGeom& c, const float* x, float* V, hipStream_t st) {
  const WinoGeom g = fwd_geom(c);
  const int T = g.tiles();
  const long total = (long)T * nq_of(c) * (c.Cin / 4);
  KernelScope ks("wino_in", 0, ((double)c.in_elems() + (double)T * 36 * nq_of(c) * c.Cin) * 4.0, st);
  hipLaunchKernelGGL(wino_in_kernel, blocks_for(total), dim3(256), 0, st, g, c.cg(), x, V, total);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// x -> V (kept by the caller for the weight gradient), V x U -> m, m -> y = act(. + bias)
int launch_wino_fwd(const ConvGeom& c, const float* x, const float* U, const float* bias, int relu, float* y, float* V,
                    float* m, float* ws, hipStream_t st) {
  const WinoGeom g = fwd_geom(c);
  const int T = g.tiles();
  AX_TRY(launch_wino_input(c, x, V, st));
  const ConvGeom p = product_geom(T, c.groups, nq_of(c) * c.cg(), c.og());
  AX_TRY(launch_conv_fwd(p, V, U, nullptr, nullptr, 0, m, ws, st));
  const long total = (long)T * (c.Cout / 4);
  KernelScope ks("wino_out", 0, ((double)c.out_elems() + (double)T * 36 * c.Cout) * 4.0, st);
  hipLaunchKernelGGL(wino_out_kernel, blocks_for(total), dim3(256), 0, st, g, c.og(), m, bias, relu,
                     (const float*)nullptr, y, total);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

int launch_wino_output_grad(const ConvGeom& c, const float* dy, float* yt, hipStream_t st) {
  const WinoGeom g = fwd_geom(c);
  const int T = g.tiles();
  const long total = (long)T * (c.Cout / 4);
  KernelScope ks("wino_dy", 0, ((double)c.out_elems() + (double)T * 36 * c.Cout) * 4.0, st);
  hipLaunchKernelGGL(wino_dy_kernel, blocks_for(total), dim3(256), 0, st, g, c.og(), dy, yt, total);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// yt x Ut -> m (36 products, columns (sub-kernel, input channel)), m -> dx gated by gate > 0 (gate may be null).
// yt is the transformed output gradient (launch_wino_output_grad, or what launch_wino_bwd_weight left there).
int launch_wino_bwd_data(const ConvGeom& c, const float* yt, const float* Ut, const float* gate, float* dx,
                                 float* m, float* ws, hipStream_t st) {
  const WinoGeom g = fwd_geom(c);
  const int T = g.tiles();
  const ConvGeom p = product_geom(T, c.groups, c.og(), nq_of(c) * c.cg());
  AX_TRY(launch_conv_fwd(p, yt, Ut, nullptr, nullptr, 0, m, ws, st));
  // eight channel quads (one 128-byte line of m) per workgroup where the channels allow, and as few row bands
  // as make that fit; at most 16 quads when whole pictures fit
  WinoDx d{g, c.cg(), 1, 1};
  const int want = c.Cin / 4 >= 8 ? 8 : (c.Cin / 4 >= 4 ? 4 : (c.Cin / 4 >= 2 ? 2 : 1));
  d.CQ = want;
  while ((size_t)d.lds_vec4() * 16 > kDxLdsBytes && d.bands < c.H) ++d.bands;
  while (d.bands == 1 && d.CQ < 16 && d.CQ * 2 <= c.Cin / 4 && (size_t)d.lds_vec4() * 32 <= kDxLdsBytes) d.CQ *= 2;
  KernelScope ks("wino_dx", 0, ((double)c.in_elems() * (gate ? 2 : 1) + (double)T * 36 * nq_of(c) * c.Cin) * 4.0, st);
  hipLaunchKernelGGL(wino_dx_kernel, dim3((unsigned)d.blocks()), dim3(256), (size_t)d.lds_vec4() * 16, st, d,
                     wino_dx_rounds(d), m, gate, dx);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// dy -> yt, V^T x yt -> dU (36 products over the tiles), dU -> dwf.  V is the forward pass's.
// With `tail`, the slices of the products stay in ws and their sum and the transform back are left to
// launch_wgrad_tail(): ws and dU must then be this stage's own until that has run.
int launch_wino_bwd_weight(const ConvGeom& c, const float* V, const float* dy, float* dwf, float* yt, float* dU,
                           float* ws, hipStream_t st, WgradTail* tail) {
  const WinoGeom g = fwd_geom(c);
  const int T = g.tiles();
  AX_TRY(launch_wino_output_grad(c, dy, yt, st));
  const ConvGeom p = product_geom(T, c.groups, nq_of(c) * c.cg(), c.og());
  const long total = (long)c.groups * nq_of(c) * c.cg() * (c.og() / 4);
  if (tail) {
    if (tail->n >= kMaxWgradJobs) {
      set_error("weight-gradient tail: more than %d stages", kMaxWgradJobs);
      return ALEXNET_EINVAL;
    }
    int ns = 1;
    AX_TRY(launch_conv_bwd_weight(p, V, yt, dU, nullptr, ws, st, &ns));
    WgradJob j;
    j.slices = ws; j.dU = dU; j.dwf = dwf;
    j.slab = (long)p.kf() * p.og(); j.total = total;
    j.nsplit = ns; j.groups36 = p.groups; j.groups = c.groups; j.Na = c.cg(); j.Nb = c.og(); j.k = c.k;
    j.nsub = nsub_of(c); j.vec = 0;
    wgrad_tail_add(*tail, j);
    return ALEXNET_OK;
  }
  // (split over the tiles where that fills the chip; the slices are added by the wide reduction kernel: letting
  // the transform below add them, with its 12 to 25 thousand threads, measured 15-50 us slower)
  AX_TRY(launch_conv_bwd_weight(p, V, yt, dU, nullptr, ws, st));
  KernelScope ks("wino_dw", 0, ((double)wino_u_floats(c) + (double)c.w_elems()) * 4.0, st);
  hipLaunchKernelGGL(wino_dw_kernel, blocks_for(total), dim3(256), 0, st, c.groups, c.cg(), c.og(), c.k, nsub_of(c), dU,
                     dwf, total);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}
int launch_wino_dw_batch(const WgradTail& t, hipStream_t st) {
  if (t.blocks_t == 0) return ALEXNET_OK;
  double bytes = 0;
  for (int i = 0; i < t.n; ++i)
    bytes += ((double)t.job[i].slab * t.job[i].groups36 + (double)t.job[i].groups * t.job[i].k * t.job[i].k * t.job[i].Na * t.job[i].Nb) * 4.0;
  KernelScope ks("wino_dw", 0, bytes, st);
  hipLaunchKernelGGL(wino_dw_batch_kernel, dim3(t.blocks_t), dim3(256), 0, st, t);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}
int launch_wgrad_tail(const WgradTail& t, hipStream_t st) {
  AX_TRY(launch_reduce_slabs_batch(t, st));
  return launch_wino_dw_batch(t, st);
}

}  // namespace ax
