// Maps one convolution stage onto the three implicit GEMMs that compute it.
// Plain host code shared by the launchers and by the CPU emulation test.
//
// Internal layouts (channel-last):
//   activations  x[B][H][W][Cin],  y / dy[B][Ho][Wo][Cout]
//   forward weights   wf[g][(r,s,c)][o]   r,s taps, c < Cin/G, o < Cout/G
//   backward weights  wb[g][(r,s,o)][c]   same numbers, last two axes swapped
//
//   forward   y [p][g*og + o]  = sum_{(r,s,c)} im2col(x)[p][(r,s,c)] * wf[g][(r,s,c)][o]
//   bwd-data  dx[q][g*cg + c]  = sum_{(r,s,o)} im2colT(dy)[q][(r,s,o)] * wb[g][(r,s,o)][c]
//   bwd-wgt   dwf[g][(r,s,c)][o] = sum_p im2col(x)[p][(r,s,c)] * dy[p][g*og + o]
#pragma once
#include <stdint.h>

#include "gemm.h"

namespace ax {

struct ConvGeom {
  int B, H, W, Cin, Cout, k, stride, pad, groups, Ho, Wo;
  int cg() const { return Cin / groups; }
  int og() const { return Cout / groups; }
  long in_elems() const { return (long)B * H * W * Cin; }
  long out_elems() const { return (long)B * Ho * Wo * Cout; }
  long w_elems() const { return (long)Cout * cg() * k * k; }
  int kf() const { return k * k * cg(); }  // reduction length of the forward GEMM
  int kb() const { return k * k * og(); }  // reduction length of the backward-data GEMM
  long P() const { return (long)B * Ho * Wo; }
  long Q() const { return (long)B * H * W; }
};

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

struct GemmDims {
  int M, N, K, groups;
};

inline void fill_divs(Im2colParams& a) {
  a.d_cg = make_fastdiv((uint32_t)a.Cg);
  a.d_kw = make_fastdiv((uint32_t)a.kw);
  a.d_ohw = make_fastdiv((uint32_t)(a.OH * a.OW));
  a.d_ow = make_fastdiv((uint32_t)a.OW);
  a.d_stride = make_fastdiv((uint32_t)a.stride);
}

// ---- forward ----
inline GemmDims fwd_dims(const ConvGeom& c) { return {(int)c.P(), c.og(), c.kf(), c.groups}; }
inline Im2colParams fwd_A(const ConvGeom& c, const float* x) {
  Im2colParams a;
  a.x = x; a.bytes = (uint32_t)(c.in_elems() * 4);
  a.H = c.H; a.W = c.W; a.Ctot = c.Cin; a.Cg = c.cg(); a.c_stride_g = c.cg();
  a.kh = a.kw = c.k; a.stride = c.stride; a.pad = c.pad; a.stride_x = c.stride; a.pad_x = c.pad;
  a.OH = c.Ho; a.OW = c.Wo; a.P = (int)c.P();
  fill_divs(a);
  return a;
}
inline bool fwd_A_vec(const ConvGeom& c, const float* x) { return c.cg() % 4 == 0 && c.Cin % 4 == 0 && aligned16(x); }
inline DenseParams fwd_B(const ConvGeom& c, const float* wf) {
  DenseParams b;
  b.p = wf; b.ld = c.og(); b.gstride = (long)c.kf() * c.og(); b.R = c.og(); b.bytes = (uint32_t)(c.w_elems() * 4);
  return b;
}
inline bool fwd_B_vec(const ConvGeom& c, const float* wf) { return c.og() % 4 == 0 && aligned16(wf); }

// ---- run mode (see gemm.h): forward and backward-weight of an unpadded conv with Cin % 4 != 0 ----
inline bool run_mode(const ConvGeom& c) { return c.pad == 0 && c.groups == 1 && c.Cin % 4 != 0; }
inline int run_len(const ConvGeom& c) { return (c.k * c.Cin + 3) / 4 * 4; }  // padded run of one kernel row
inline int run_k(const ConvGeom& c) { return c.k * run_len(c); }             // reduction length in run mode
inline long run_w_elems(const ConvGeom& c) { return (long)run_k(c) * c.Cout; }
inline Im2colParams run_A(const ConvGeom& c, const float* x) {
  Im2colParams a;
  a.x = x; a.bytes = (uint32_t)(c.in_elems() * 4);
  a.H = c.H; a.W = c.W * c.Cin; a.Ctot = 1; a.Cg = run_len(c); a.c_stride_g = 0;
  a.kh = c.k; a.kw = 1; a.stride = c.stride; a.pad = 0; a.stride_x = c.stride * c.Cin; a.pad_x = 0;
  a.OH = c.Ho; a.OW = c.Wo; a.P = (int)c.P();
  fill_divs(a);
  return a;
}
inline DenseParams run_B(const ConvGeom& c, const float* wrun) {  // wrun[(r, j)][o], zero for j >= k*Cin
  DenseParams b;
  b.p = wrun; b.ld = c.Cout; b.gstride = 0; b.R = c.Cout; b.bytes = (uint32_t)(run_w_elems(c) * 4);
  return b;
}

// ---- backward data ----
inline GemmDims bwdd_dims(const ConvGeom& c) { return {(int)c.Q(), c.cg(), c.kb(), c.groups}; }
inline Im2colParams bwdd_A(const ConvGeom& c, const float* dy) {
  Im2colParams a;
  a.x = dy; a.bytes = (uint32_t)(c.out_elems() * 4);
  a.H = c.Ho; a.W = c.Wo; a.Ctot = c.Cout; a.Cg = c.og(); a.c_stride_g = c.og();
  a.kh = a.kw = c.k; a.stride = c.stride; a.pad = c.pad; a.stride_x = c.stride; a.pad_x = c.pad;
  a.OH = c.H; a.OW = c.W; a.P = (int)c.Q();
  fill_divs(a);
  return a;
}
inline bool bwdd_A_vec(const ConvGeom& c, const float* dy) { return c.og() % 4 == 0 && c.Cout % 4 == 0 && aligned16(dy); }
inline DenseParams bwdd_B(const ConvGeom& c, const float* wb) {
  DenseParams b;
  b.p = wb; b.ld = c.cg(); b.gstride = (long)c.kb() * c.cg(); b.R = c.cg(); b.bytes = (uint32_t)(c.w_elems() * 4);
  return b;
}
inline bool bwdd_B_vec(const ConvGeom& c, const float* wb) { return c.cg() % 4 == 0 && aligned16(wb); }

// ---- backward data of a strided convolution, by phases ----
// Input pixel iy = st*qy + py - pad only receives taps r = py + st*a, so all st*st phases (py, px) together
// are one unit-stride transposed gather over dy with ceil(k/st)^2 taps and st*st*Cin output columns:
//   dxall[(n,qy,qx)][(py,px,c)] = sum_{(a,b,o)} dy[n][qy-a][qx-b][o] * wp[(a,b,o)][(py,px,c)],
//   wp[(a,b,o)][(py,px,c)] = w[o][c][py+st*a][px+st*b]  (0 where that tap does not exist).
inline bool phase_mode(const ConvGeom& c) { return c.stride > 1 && c.groups == 1; }
inline int phase_taps(const ConvGeom& c) { return (c.k + c.stride - 1) / c.stride; }
inline int phase_qh(const ConvGeom& c) { return (c.H - 1 + c.pad) / c.stride + 1; }
inline int phase_qw(const ConvGeom& c) { return (c.W - 1 + c.pad) / c.stride + 1; }
inline int phase_n(const ConvGeom& c) { return c.stride * c.stride * c.Cin; }
inline int phase_k(const ConvGeom& c) { return phase_taps(c) * phase_taps(c) * c.Cout; }
inline long phase_w_elems(const ConvGeom& c) { return (long)phase_k(c) * phase_n(c); }
inline GemmDims phase_dims(const ConvGeom& c) { return {c.B * phase_qh(c) * phase_qw(c), phase_n(c), phase_k(c), 1}; }
inline Im2colParams phase_A(const ConvGeom& c, const float* dy) {
  Im2colParams a;
  a.x = dy; a.bytes = (uint32_t)(c.out_elems() * 4);
  a.H = c.Ho; a.W = c.Wo; a.Ctot = c.Cout; a.Cg = c.Cout; a.c_stride_g = 0;
  a.kh = a.kw = phase_taps(c); a.stride = 1; a.pad = 0; a.stride_x = 1; a.pad_x = 0;
  a.OH = phase_qh(c); a.OW = phase_qw(c); a.P = c.B * phase_qh(c) * phase_qw(c);
  fill_divs(a);
  return a;
}
inline DenseParams phase_B(const ConvGeom& c, const float* wp) {
  DenseParams b;
  b.p = wp; b.ld = phase_n(c); b.gstride = 0; b.R = phase_n(c); b.bytes = (uint32_t)(phase_w_elems(c) * 4);
  return b;
}
inline EpiPhases phase_epilogue(const ConvGeom& c, float* dx) {
  EpiPhases e;
  e.dx = dx; e.H = c.H; e.W = c.W; e.C = c.Cin; e.st = c.stride; e.pad = c.pad; e.QW = phase_qw(c);
  e.d_qhw = make_fastdiv((uint32_t)(phase_qh(c) * phase_qw(c)));
  e.d_qw = make_fastdiv((uint32_t)phase_qw(c));
  e.d_stc = make_fastdiv((uint32_t)(c.stride * c.Cin));
  e.d_c = make_fastdiv((uint32_t)c.Cin);
  return e;
}

// ---- backward weight ----
inline GemmDims bwdw_dims(const ConvGeom& c) { return {c.kf(), c.og(), (int)c.P(), c.groups}; }
inline Im2colParams bwdw_A(const ConvGeom& c, const float* x) { return fwd_A(c, x); }
inline bool bwdw_A_vec(const ConvGeom& c, const float* x) { return fwd_A_vec(c, x); }
inline DenseParams bwdw_B(const ConvGeom& c, const float* dy) {
  DenseParams b;
  b.p = dy; b.ld = c.Cout; b.gstride = c.og(); b.R = c.og(); b.bytes = (uint32_t)(c.out_elems() * 4);
  return b;
}
inline bool bwdw_B_vec(const ConvGeom& c, const float* dy) { return c.og() % 4 == 0 && c.Cout % 4 == 0 && aligned16(dy); }

// The same operands over tensors that hold bf16: the pointer is carried in the same field, the extent counts
// 2-byte elements (only the "16" loaders of gemm_bf16.h may be given these)
inline Im2colParams im2col16(Im2colParams a, const uint16_t* p) {
  a.x = reinterpret_cast<const float*>(p);
  a.bytes /= 2;
  return a;
}
inline DenseParams dense16(DenseParams b, const uint16_t* p) {
  b.p = reinterpret_cast<const float*>(p);
  b.bytes /= 2;
  return b;
}
// Weights of the forward and backward-data products as bf16 with the reduction contiguous, wfk[g][o][(r,s,c)]
// and wbk[g][c][(r,s,o)] (the transposes of wf and wb): both operands of those products are then read along k,
// which is the cheap direction for the matrix cores' fragments (one 16-byte LDS read per fragment)
inline DenseParams fwd_B16k(const ConvGeom& c, const uint16_t* wfk) {
  DenseParams b;
  b.p = reinterpret_cast<const float*>(wfk); b.ld = c.kf(); b.gstride = (long)c.og() * c.kf(); b.R = c.og();
  b.bytes = (uint32_t)(c.w_elems() * 2);
  return b;
}
inline DenseParams bwdd_B16k(const ConvGeom& c, const uint16_t* wbk) {
  DenseParams b;
  b.p = reinterpret_cast<const float*>(wbk); b.ld = c.kb(); b.gstride = (long)c.cg() * c.kb(); b.R = c.cg();
  b.bytes = (uint32_t)(c.w_elems() * 2);
  return b;
}
// ---- run mode over pictures stored as bf16 with their channels padded to four ----
// The first layer's pictures have three channels.  Stored as bf16 x4[N][H][W][4] (fourth channel zero), viewed as
// a one-channel tensor x'[N][H][W*4], all taps (s, c) of kernel row r are one contiguous run of k*4 values
// starting at column x*stride*4, which is a multiple of 8 bytes: it is read in 16-byte pieces of eight values
// and padded to a multiple of eight with weights that are zero.  The padding reads values of the next pixels (of
// the next row at the right edge; nothing past the end of the tensor, where the loads return zero), which meet
// zero weights.  Reduction length k * run16_len(); the weights are wk[o][(r, s*4 + c)], k-contiguous.
inline bool run16_mode(const ConvGeom& c) { return run_mode(c) && c.Cin < 4 && c.Cout % 8 == 0; }
inline int run16_len(const ConvGeom& c) { return (c.k * 4 + 7) / 8 * 8; }
inline int run16_k(const ConvGeom& c) { return c.k * run16_len(c); }
inline long run16_x_elems(const ConvGeom& c) { return (long)c.B * c.H * c.W * 4; }
inline long run16_w_elems(const ConvGeom& c) { return (long)run16_k(c) * c.Cout; }
inline Im2colParams run16_A(const ConvGeom& c, const uint16_t* x4) {
  Im2colParams a;
  a.x = reinterpret_cast<const float*>(x4); a.bytes = (uint32_t)(run16_x_elems(c) * 2);
  a.H = c.H; a.W = c.W * 4; a.Ctot = 1; a.Cg = run16_len(c); a.c_stride_g = 0;
  a.kh = c.k; a.kw = 1; a.stride = c.stride; a.pad = 0; a.stride_x = c.stride * 4; a.pad_x = 0;
  a.OH = c.Ho; a.OW = c.Wo; a.P = (int)c.P();
  fill_divs(a);
  return a;
}
inline DenseParams run16_Bk(const ConvGeom& c, const uint16_t* wk) {
  DenseParams b;
  b.p = reinterpret_cast<const float*>(wk); b.ld = run16_k(c); b.gstride = 0; b.R = c.Cout;
  b.bytes = (uint32_t)(run16_w_elems(c) * 2);
  return b;
}
// every extent a 16-byte load of bf16 must not straddle is a multiple of 8
inline bool conv16_ok(const ConvGeom& c) { return c.cg() % 8 == 0 && c.og() % 8 == 0 && c.stride == 1; }

// Split of the reduction so that a launch has enough workgroups: returns the
// number of splits and sets kchunk (a multiple of bk).
inline int plan_split(long tiles, int K, int bk, int target_blocks, int max_split, int* kchunk) {
  int ktiles = (K + bk - 1) / bk;
  int want = (int)((target_blocks + tiles - 1) / tiles);
  if (want < 1) want = 1;
  if (want > max_split) want = max_split;
  if (want > ktiles) want = ktiles;
  int per = (ktiles + want - 1) / want;
  *kchunk = per * bk;
  return (ktiles + per - 1) / per;
}

}  // namespace ax
