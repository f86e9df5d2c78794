// 3x3 unit-stride convolutions through the minimal-filtering identity F(4x4, 3x3).
//
// A 1-D correlation y_i = sum_j g_j d_{i+j} (4 outputs, 3 taps, 6 inputs) is the bilinear form
//     y = At [ (G g) .* (Bt d) ]
// with the Cook-Toom matrices for the points 0, +-1, +-2 and infinity: 6 products instead of 12.
// Nesting it in both image directions turns a 3x3 convolution over 4x4 output tiles into 36
// independent matrix products over the channels (one per position of the transformed 6x6 tile),
// 36 multiplies per tile and channel pair instead of 144.  Writing the same trilinear form
// T[i][j][k] = sum_p At[i][p] G[p][j] Bt[p][k] for the other two arguments gives the adjoints:
//     dg = Gt [ (A dy) .* (Bt d) ]         (gradient of the taps: A = At^T applied to the 4 output gradients)
//     dd = B  [ (A dy) .* (G g)  ]         (gradient of the input patch: B = Bt^T; overlapping patches add up)
//
// Data layout of the transformed tensors: one row per tile t = (picture, tile row, tile column) and
// 36 * groups * Cg columns, column (p*groups + g)*Cg + c for tile position p = 6*row + column.  That is
// exactly a channel-last activation tensor of a 1x1 convolution with 36*groups groups, so the 36 products
// run as one launch of the grouped implicit-GEMM kernels (conv_gemm.hip) and need no kernel of their own.
//
// 5x5 kernels (the second layer) use the same transforms: a 5x5 correlation is the sum of four 3x3
// correlations of the input shifted by 0 or 3 pixels in each direction, with the sub-kernels
// w[3qy + i][3qx + j] (zero where that tap does not exist).  The four sub-kernels q are concatenated
// along the reduction of the products, column (p*groups + g)*(4*Cg) + q*Cg + c, so the sum over them
// happens inside the matrix product: 36 * 4 multiplies per tile and channel pair instead of 400.
//
// Everything here is per-thread code shared by the kernels (winograd.hip) and by the CPU emulation test,
// which runs it thread by thread under an address sanitizer.
#pragma once

#include <stdint.h>

#include "gemm.h"

namespace ax {

struct Vec4 {
  float x, y, z, w;
};
AX_HD Vec4 operator+(Vec4 a, Vec4 b) { return {a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w}; }
AX_HD Vec4 operator-(Vec4 a, Vec4 b) { return {a.x - b.x, a.y - b.y, a.z - b.z, a.w - b.w}; }
AX_HD Vec4 operator*(float s, Vec4 a) { return {s * a.x, s * a.y, s * a.z, s * a.w}; }
AX_HD Vec4 vzero() { return {0.f, 0.f, 0.f, 0.f}; }
AX_HD Vec4 vload(const float* p) {
  const float4 v = *reinterpret_cast<const float4*>(p);
  return {v.x, v.y, v.z, v.w};
}
AX_HD void vstore(float* p, Vec4 v) {
  float4 o;
  o.x = v.x; o.y = v.y; o.z = v.z; o.w = v.w;
  *reinterpret_cast<float4*>(p) = o;
}

// two channels of a pixel (the overlap-add of the data gradient works on half quads, see WinoDx)
struct Vec2 {
  float x, y;
};
AX_HD Vec2 operator+(Vec2 a, Vec2 b) { return {a.x + b.x, a.y + b.y}; }
AX_HD Vec2 operator-(Vec2 a, Vec2 b) { return {a.x - b.x, a.y - b.y}; }
AX_HD Vec2 operator*(float s, Vec2 a) { return {s * a.x, s * a.y}; }
AX_HD Vec2 vload2(const float* p) {
  const float2 v = *reinterpret_cast<const float2*>(p);
  return {v.x, v.y};
}

// ---- the five 1-D maps (strided in / out so that they serve rows and columns of a register tile) ----
// Bt (6x6): data transform
template <int SI, int SO>
AX_HD void wino_bt(const Vec4* d, Vec4* o) {
  const Vec4 d0 = d[0], d1 = d[SI], d2 = d[2 * SI], d3 = d[3 * SI], d4 = d[4 * SI], d5 = d[5 * SI];
  o[0] = 4.f * d0 - 5.f * d2 + d4;
  o[SO] = d3 + d4 - 4.f * (d1 + d2);
  o[2 * SO] = 4.f * (d1 - d2) - d3 + d4;
  o[3 * SO] = 2.f * (d3 - d1) - d2 + d4;
  o[4 * SO] = 2.f * (d1 - d3) - d2 + d4;
  o[5 * SO] = 4.f * d1 - 5.f * d3 + d5;
}
// B (6x6) = (Bt)^T: adjoint of the data transform
template <int SI, int SO, class V>
AX_HD void wino_b(const V* m, V* o) {
  const V m0 = m[0], m1 = m[SI], m2 = m[2 * SI], m3 = m[3 * SI], m4 = m[4 * SI], m5 = m[5 * SI];
  o[0] = 4.f * m0;
  o[SO] = 4.f * (m2 - m1 + m5) + 2.f * (m4 - m3);
  o[2 * SO] = (-5.f) * m0 - 4.f * (m1 + m2) - m3 - m4;
  o[3 * SO] = m1 - m2 + 2.f * (m3 - m4) - 5.f * m5;
  o[4 * SO] = m0 + m1 + m2 + m3 + m4;
  o[5 * SO] = m5;
}
// At (4x6): output transform
template <int SI, int SO>
AX_HD void wino_at(const Vec4* m, Vec4* o) {
  const Vec4 m0 = m[0], m1 = m[SI], m2 = m[2 * SI], m3 = m[3 * SI], m4 = m[4 * SI], m5 = m[5 * SI];
  const Vec4 s12 = m1 + m2, d12 = m1 - m2, s34 = m3 + m4, d34 = m3 - m4;
  o[0] = m0 + s12 + s34;
  o[SO] = d12 + 2.f * d34;
  o[2 * SO] = s12 + 4.f * s34;
  o[3 * SO] = d12 + 8.f * d34 + m5;
}
// A (6x4): transform of the four output gradients
template <int SI, int SO>
AX_HD void wino_a(const Vec4* e, Vec4* o) {
  const Vec4 e0 = e[0], e1 = e[SI], e2 = e[2 * SI], e3 = e[3 * SI];
  const Vec4 ev = e0 + e2, od = e1 + e3, ev4 = e0 + 4.f * e2, od4 = e1 + 4.f * e3;
  o[0] = e0;
  o[SO] = ev + od;
  o[2 * SO] = ev - od;
  o[3 * SO] = ev4 + 2.f * od4;
  o[4 * SO] = ev4 - 2.f * od4;
  o[5 * SO] = e3;
}
// G (6x3): tap transform
template <int SI, int SO>
AX_HD void wino_g(const Vec4* g, Vec4* o) {
  const Vec4 g0 = g[0], g1 = g[SI], g2 = g[2 * SI];
  const Vec4 a = (1.f / 6.f) * (g0 + g2), b = (1.f / 6.f) * g1;
  const Vec4 c = (1.f / 24.f) * g0 + (1.f / 6.f) * g2, d = (1.f / 12.f) * g1;
  o[0] = 0.25f * g0;
  o[SO] = vzero() - a - b;
  o[2 * SO] = b - a;
  o[3 * SO] = c + d;
  o[4 * SO] = c - d;
  o[5 * SO] = g2;
}
// Gt (3x6): back from the 6 transformed positions to the gradient of the 3 taps
template <int SI, int SO>
AX_HD void wino_gt(const Vec4* m, Vec4* o) {
  const Vec4 m0 = m[0], m1 = m[SI], m2 = m[2 * SI], m3 = m[3 * SI], m4 = m[4 * SI], m5 = m[5 * SI];
  const Vec4 s12 = m1 + m2, d12 = m2 - m1, s34 = m3 + m4, d34 = m3 - m4;
  o[0] = 0.25f * m0 - (1.f / 6.f) * s12 + (1.f / 24.f) * s34;
  o[SO] = (1.f / 6.f) * d12 + (1.f / 12.f) * d34;
  o[2 * SO] = (1.f / 6.f) * (s34 - s12) + m5;
}

// ---- geometry of one transformed convolution -----------------------------------------------------
// `H x W` is the tensor the 6x6 tiles are cut from (pad `pad` on every side), `OH x OW` the tensor
// of 4x4 tiles (OH = H + 2*pad - 2).  Ctot = groups * Cg channels on the gathered side.
// k x k taps are handled as nsub x nsub sub-kernels of 3x3 (k = 3: one, k = 5: four).
struct WinoGeom {
  int B, H, W, pad, OH, OW, th, tw, groups, k, nsub;
  AX_HD int tiles() const { return B * th * tw; }
  AX_HD int nq() const { return nsub * nsub; }
};
struct WinoTile {
  int n, ty, tx;
};
AX_HD WinoTile wino_tile(const WinoGeom& g, int t) {
  WinoTile r;
  const int per = g.th * g.tw;
  r.n = t / per;
  const int rem = t - r.n * per;
  r.ty = rem / g.tw;
  r.tx = rem - r.ty * g.tw;
  return r;
}

// V[t][(p*groups + g)*(nq*Cg) + q*Cg + c] = (Bt d B)[p] of the 6x6 patch of x that sub-kernel q of tile t
// reads (zero outside x).  idx enumerates (tile, sub-kernel, channel quad); x is [B][H][W][groups*Cg].
AX_HD void wino_in_thread(const WinoGeom& g, int Cg, const float* x, float* V, long idx) {
  const int Ctot = g.groups * Cg, quads = Ctot / 4, nq = g.nq();
  const int t = (int)(idx / ((long)nq * quads));
  const int rem = (int)(idx - (long)t * nq * quads);
  const int q = rem / quads, c = 4 * (rem - q * quads);
  const int qy = q / g.nsub, qx = q - qy * g.nsub;
  const WinoTile tl = wino_tile(g, t);
  const int y0 = 4 * tl.ty - g.pad + 3 * qy, x0 = 4 * tl.tx - g.pad + 3 * qx;
  Vec4 d[36], u[36];
#pragma unroll
  for (int i = 0; i < 6; ++i)
#pragma unroll
    for (int j = 0; j < 6; ++j) {
      const int iy = y0 + i, ix = x0 + j;
      const bool in = (uint32_t)iy < (uint32_t)g.H && (uint32_t)ix < (uint32_t)g.W;
      d[6 * i + j] = vzero();
      if (in) d[6 * i + j] = vload(x + (((long)tl.n * g.H + iy) * g.W + ix) * Ctot + c);
    }
#pragma unroll
  for (int j = 0; j < 6; ++j) wino_bt<6, 6>(d + j, u + j);  // columns
  const int grp = c / Cg, cl = c - grp * Cg;
  const long pstride = (long)nq * Ctot;
  float* out = V + (long)t * 36 * pstride + (long)grp * nq * Cg + (long)q * Cg + cl;
#pragma unroll
  for (int i = 0; i < 6; ++i) {
    Vec4 r[6];
    wino_bt<1, 1>(u + 6 * i, r);  // row i
#pragma unroll
    for (int j = 0; j < 6; ++j) vstore(out + (long)(6 * i + j) * pstride, r[j]);
  }
}

// Y[t][(p*groups + g)*Og + o] = (A e At)[p] of the 4x4 block of dy that tile t owns (zero outside dy).
// idx enumerates (tile, channel quad); dy is [B][OH][OW][groups*Og].
AX_HD void wino_dy_thread(const WinoGeom& g, int Og, const float* dy, float* Y, long idx) {
  const int Ctot = g.groups * Og, quads = Ctot / 4;
  const int t = (int)(idx / quads), c = 4 * (int)(idx - (long)t * quads);
  const WinoTile tl = wino_tile(g, t);
  Vec4 e[16], u[24];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int oy = 4 * tl.ty + i, ox = 4 * tl.tx + j;
      e[4 * i + j] = vzero();
      if (oy < g.OH && ox < g.OW) e[4 * i + j] = vload(dy + (((long)tl.n * g.OH + oy) * g.OW + ox) * Ctot + c);
    }
#pragma unroll
  for (int j = 0; j < 4; ++j) wino_a<4, 4>(e + j, u + j);  // columns: 4 -> 6 rows of 4
  const int grp = c / Og, cl = c - grp * Og;
  float* out = Y + (long)t * 36 * Ctot + (long)grp * Og + cl;
#pragma unroll
  for (int i = 0; i < 6; ++i) {
    Vec4 r[6];
    wino_a<1, 1>(u + 4 * i, r);
#pragma unroll
    for (int j = 0; j < 6; ++j) vstore(out + (long)(6 * i + j) * Ctot, r[j]);
  }
}

// y[n][4ty+i][4tx+j][c] = post((At m A)[i][j]) from M[t][(p*groups + g)*Ng + c'], inside OH x OW only.
// post: + bias[c] and ReLU (relu != 0), or zero where gate[same index] <= 0; bias and gate may be null.
AX_HD void wino_out_thread(const WinoGeom& g, int Ng, const float* M, const float* bias, int relu, const float* gate,
                           float* y, long idx) {
  const int Ctot = g.groups * Ng, quads = Ctot / 4;
  const int t = (int)(idx / quads), c = 4 * (int)(idx - (long)t * quads);
  const WinoTile tl = wino_tile(g, t);
  const int grp = c / Ng, cl = c - grp * Ng;
  const float* in = M + (long)t * 36 * Ctot + (long)grp * Ng + cl;
  Vec4 u[24];
#pragma unroll
  for (int j = 0; j < 6; ++j) {
    Vec4 col[6];
#pragma unroll
    for (int i = 0; i < 6; ++i) col[i] = vload(in + (long)(6 * i + j) * Ctot);
    wino_at<1, 6>(col, u + j);  // u[i][j], 4 rows of 6
  }
  Vec4 b = vzero();
  if (bias) b = vload(bias + c);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    Vec4 r[4];
    wino_at<1, 1>(u + 6 * i, r);
    const int oy = 4 * tl.ty + i;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int ox = 4 * tl.tx + j;
      if (oy < g.OH && ox < g.OW) {
        const long o = (((long)tl.n * g.OH + oy) * g.OW + ox) * Ctot + c;
        Vec4 v = r[j] + b;
        if (relu) {
          v.x = v.x > 0.f ? v.x : 0.f; v.y = v.y > 0.f ? v.y : 0.f;
          v.z = v.z > 0.f ? v.z : 0.f; v.w = v.w > 0.f ? v.w : 0.f;
        }
        if (gate) {
          const Vec4 q = vload(gate + o);
          if (!(q.x > 0.f)) v.x = 0.f;
          if (!(q.y > 0.f)) v.y = 0.f;
          if (!(q.z > 0.f)) v.z = 0.f;
          if (!(q.w > 0.f)) v.w = 0.f;
        }
        vstore(y + o, v);
      }
    }
  }
}

// Data gradient as the adjoint of the input transform: dx += B m Bt of every 6x6 patch, where
// m[p] = M[t][(p*groups + g)*(nq*Cg) + q*Cg + c] is the product of the transformed output gradient with the
// transformed taps.  Patches overlap, so a workgroup owns one picture and CQ channel quads, keeps the picture
// in LDS ([pixel][CQ] float4) and adds the patches in 4*nq phases -- tiles of one parity (ty % 2, tx % 2) and
// one sub-kernel are 8 pixels apart and never touch the same pixel, so within a phase every LDS word has one
// writer and the sum has a fixed order.  256 threads: a thread owns two channels (half a quad: 36 x float2 of
// patch, so that four workgroups fit a CU and one's loads run under another's adds -- with whole quads, 227
// registers, the two halves of a round took turns), tid % (2 CQ) is the channel pair, tid / (2 CQ) the worker.
// Work goes in rounds: in a round every worker loads and transforms one patch (all of them at once, so that the
// memory system sees 256 threads' loads, not one phase's), then the phases add them to the picture.  Eight quads are
// one 128-byte line of M; where a whole picture of eight quads does not fit the LDS budget the picture is cut
// into `bands` of rows, one workgroup each, and a patch that straddles two bands is transformed by both (each
// keeps its own rows).  Call order: wino_dx_zero, barrier, per round: wino_dx_load, then wino_dx_add and a
// barrier for each phase the round touches (wino_dx_round_phases); wino_dx_flush.
struct WinoDx {
  WinoGeom g;  // of the forward pass: H x W is the picture dx, th x tw the tiles of the output
  int Cg, CQ;  // channels per group of dx; quads per workgroup (a power of two dividing 256)
  int bands;   // row bands per picture
  AX_HD int Ctot() const { return g.groups * Cg; }
  AX_HD int cblocks() const { return (Ctot() / 4 + CQ - 1) / CQ; }
  AX_HD int phases() const { return 4 * g.nq(); }
  AX_HD int band_rows() const { return (g.H + bands - 1) / bands; }
  AX_HD int lds_vec4() const { return band_rows() * g.W * CQ; }
  AX_HD int lanes() const { return 2 * CQ; }               // channel pairs, one thread each
  AX_HD int workers() const { return kThreads / lanes(); }  // patches per round
  AX_HD int blocks() const { return g.B * bands * cblocks(); }
};
struct WinoDxBlock {
  int n, cblk, h0, h1;  // picture, channel block, rows [h0, h1)
};
AX_HD WinoDxBlock wino_dx_block(const WinoDx& d, int block) {
  WinoDxBlock b;
  b.cblk = block % d.cblocks();
  const int r = block / d.cblocks();
  b.n = r / d.bands;
  const int band = r - b.n * d.bands;
  b.h0 = band * d.band_rows();
  b.h1 = b.h0 + d.band_rows() < d.g.H ? b.h0 + d.band_rows() : d.g.H;
  return b;
}
AX_HD void wino_dx_zero(const WinoDx& d, Vec4* lds, int tid) {
  for (int i = tid; i < d.lds_vec4(); i += kThreads) lds[i] = vzero();
}
// The tiles whose patches can reach the rows of a block, listed phase by phase (phase = parity*nq + q with
// parity = 2*(ty & 1) + (tx & 1)): all tasks of phase 0, then of phase 1, ...  Workers take consecutive tasks,
// so the lanes of a wave mostly share a phase and a round spans few phases.
struct WinoDxTasks {
  int ty_lo, ty_hi;  // tile rows that can reach the block's rows (inclusive; hi < lo: none)
  int count;         // tasks of the block
};
AX_HD int wino_dx_rows_of_parity(const WinoDxTasks& t, int py) {  // tile rows in [ty_lo, ty_hi] with ty % 2 == py
  if (t.ty_hi < t.ty_lo) return 0;
  const int first = t.ty_lo + ((t.ty_lo & 1) != py);
  return first > t.ty_hi ? 0 : (t.ty_hi - first) / 2 + 1;
}
AX_HD int wino_dx_phase_count(const WinoDx& d, const WinoDxTasks& t, int phase) {
  const int par = phase / d.g.nq(), py = par >> 1, px = par & 1;
  return wino_dx_rows_of_parity(t, py) * ((d.g.tw - px + 1) / 2);
}
AX_HD WinoDxTasks wino_dx_tasks(const WinoDx& d, const WinoDxBlock& bk) {
  const WinoGeom& g = d.g;
  // patch rows of (ty, qy): 4ty - pad + 3qy + [0, 6)
  int lo = bk.h0 - 5 + g.pad - 3 * (g.nsub - 1);
  lo = lo <= 0 ? 0 : (lo + 3) / 4;
  int hi = bk.h1 - 1 + g.pad;
  hi = hi < 0 ? -1 : hi / 4;
  if (hi > g.th - 1) hi = g.th - 1;
  WinoDxTasks t;
  t.ty_lo = lo;
  t.ty_hi = hi;
  t.count = 0;
  for (int ph = 0; ph < d.phases(); ++ph) t.count += wino_dx_phase_count(d, t, ph);
  return t;
}
// Everything about a block that does not change from round to round, worked out once per thread
struct WinoDxPlan {
  WinoDxBlock bk;
  WinoDxTasks tk;
  int prefix[17];  // tasks before phase ph; prefix[phases()] = count
};
AX_HD WinoDxPlan wino_dx_plan(const WinoDx& d, int block) {
  WinoDxPlan p;
  p.bk = wino_dx_block(d, block);
  p.tk = wino_dx_tasks(d, p.bk);
  p.prefix[0] = 0;
#pragma unroll
  for (int ph = 0; ph < 16; ++ph)
    p.prefix[ph + 1] = p.prefix[ph] + (ph < d.phases() ? wino_dx_phase_count(d, p.tk, ph) : 0);
  return p;
}
// phase of task j (j < count) and the number of tasks before that phase; only constant indices into prefix[],
// so that it stays in registers
AX_HD int wino_dx_phase_of(const WinoDxPlan& p, int j, int* before) {
  int ph = 0, b = 0;
#pragma unroll
  for (int k = 1; k < 16; ++k)
    if (j >= p.prefix[k]) {
      ph = k;
      b = p.prefix[k];
    }
  *before = b;
  return ph;
}
AX_HD int wino_dx_rounds(const WinoDx& d) {  // the same for every block: the largest need of any band
  int most = 0;
  for (int b = 0; b < d.bands; ++b) {
    WinoDxBlock bk;
    bk.n = 0; bk.cblk = 0;
    bk.h0 = b * d.band_rows();
    bk.h1 = bk.h0 + d.band_rows() < d.g.H ? bk.h0 + d.band_rows() : d.g.H;
    const int c = wino_dx_tasks(d, bk).count;
    most = c > most ? c : most;
  }
  const int workers = d.workers();
  return (most + workers - 1) / workers;
}
// phases that round `round` of a block touches: [*lo, *hi] (lo > hi: the round has no task)
AX_HD void wino_dx_round_phases(const WinoDx& d, const WinoDxPlan& p, int round, int* lo, int* hi) {
  const int workers = d.workers(), first = round * workers;
  int last = first + workers - 1;
  if (last > p.tk.count - 1) last = p.tk.count - 1;
  if (first > last) {
    *lo = 1; *hi = 0;
    return;
  }
  int before;
  *lo = wino_dx_phase_of(p, first, &before);
  *hi = wino_dx_phase_of(p, last, &before);
}
// One task of a thread: phase < 0 means none.  z = B m Bt of the patch, to be added at (y0 + i, x0 + j).
struct WinoDxTask {
  int phase, y0, x0;
};
// Round r of a block: every worker loads and transforms one patch (all threads at once: this is where the
// memory traffic is), ...
AX_HD WinoDxTask wino_dx_load(const WinoDx& d, const WinoDxPlan& p, const float* M, int tid, int round, Vec2* z) {
  const WinoGeom& g = d.g;
  const int nq = g.nq(), Ctot = d.Ctot();
  const WinoDxBlock& bk = p.bk;
  const int cp = tid % d.lanes(), worker = tid / d.lanes(), workers = d.workers();
  const int c = 4 * bk.cblk * d.CQ + 2 * cp;  // Ctot and Cg are multiples of four: the pair lies in one group
  WinoDxTask task;
  task.phase = -1; task.y0 = 0; task.x0 = 0;
  const int j = round * workers + worker;
  if (c >= Ctot || j >= p.tk.count) return task;
  int before;
  const int ph = wino_dx_phase_of(p, j, &before), within = j - before;
  const int q = ph % nq, par = ph / nq, py = par >> 1, px = par & 1;
  const int nx = (g.tw - px + 1) / 2;
  const int ty = p.tk.ty_lo + ((p.tk.ty_lo & 1) != py) + 2 * (within / nx), tx = px + 2 * (within % nx);
  const int qy = q / g.nsub, qx = q - qy * g.nsub;
  const int y0 = 4 * ty - g.pad + 3 * qy, x0 = 4 * tx - g.pad + 3 * qx;
  if (y0 + 6 <= bk.h0 || y0 >= bk.h1) return task;  // the patch lies in another band
  task.phase = ph;
  task.y0 = y0; task.x0 = x0;
  const int grp = c / d.Cg, cl = c - grp * d.Cg;
  const long pstride = (long)nq * Ctot;
  const long t = ((long)bk.n * g.th + ty) * g.tw + tx;
  const float* in = M + t * 36 * pstride + (long)grp * nq * d.Cg + (long)q * d.Cg + cl;
  Vec2 u[36];
#pragma unroll
  for (int jj = 0; jj < 6; ++jj) {
    Vec2 col[6];
#pragma unroll
    for (int i = 0; i < 6; ++i) col[i] = vload2(in + (long)(6 * i + jj) * pstride);
    wino_b<1, 6>(col, u + jj);  // u[i][jj]
  }
#pragma unroll
  for (int i = 0; i < 6; ++i) wino_b<1, 1>(u + 6 * i, z + 6 * i);
  return task;
}
// ... then the patches are added to the picture phase by phase (a barrier after each call).
AX_HD void wino_dx_add(const WinoDx& d, const WinoDxPlan& p, Vec4* lds, int tid, const WinoDxTask& task, const Vec2* z,
                       int phase) {
  if (task.phase != phase) return;
  const WinoDxBlock& bk = p.bk;
  const int cp = tid % d.lanes();
  Vec2* half = reinterpret_cast<Vec2*>(lds);  // [pixel][2 CQ] channel pairs over the same memory
#pragma unroll
  for (int i = 0; i < 6; ++i) {
    const int iy = task.y0 + i;
#pragma unroll
    for (int jj = 0; jj < 6; ++jj) {
      const int ix = task.x0 + jj;
      if (iy >= bk.h0 && iy < bk.h1 && (uint32_t)ix < (uint32_t)d.g.W) {
        Vec2* acc = half + ((long)(iy - bk.h0) * d.g.W + ix) * d.lanes() + cp;
        *acc = *acc + z[6 * i + jj];
      }
    }
  }
}
// dx[n][pixel][c] = the picture in LDS, zero where gate <= 0 (gate may be null)
AX_HD void wino_dx_flush(const WinoDx& d, const WinoDxPlan& p, const Vec4* lds, const float* gate, float* dx, int tid) {
  const int Ctot = d.Ctot();
  const WinoDxBlock& bk = p.bk;
  const int count = (bk.h1 - bk.h0) * d.g.W * d.CQ;  // the last band may be shorter
  for (int i = tid; i < count; i += kThreads) {
    const int cq = i % d.CQ, pix = i / d.CQ;
    const int c = 4 * (bk.cblk * d.CQ + cq);
    if (c >= Ctot) continue;
    const long o = ((long)bk.n * d.g.H * d.g.W + (long)bk.h0 * d.g.W + pix) * Ctot + c;
    Vec4 v = lds[i];
    if (gate) {
      const Vec4 q = vload(gate + o);
      if (!(q.x > 0.f)) v.x = 0.f;
      if (!(q.y > 0.f)) v.y = 0.f;
      if (!(q.z > 0.f)) v.z = 0.f;
      if (!(q.w > 0.f)) v.w = 0.f;
    }
    vstore(dx + o, v);
  }
}

// Taps to transformed taps and back.  `w` is [groups][(r, s, a)][b] (k x k taps; a < Na rows, b < Nb
// columns: the forward weights with a = input channel, b = output channel, or the backward-data
// weights with the roles swapped), `U` is [(p*groups + g)][q*Na + a][b] for sub-kernel q = (qy, qx) with the
// taps (3qy + i, 3qx + j), zero where they do not exist.  q_in_cols stores U as [(p*groups + g)][a][q*Nb + b]
// instead (the operand of the data-gradient products, whose columns are (sub-kernel, input channel)).
// idx enumerates (group, sub-kernel, a, column quad).
AX_HD void wino_filter_thread(int groups, int Na, int Nb, int k, int nsub, int q_in_cols, const float* w, float* U,
                              long idx) {
  const int quads = Nb / 4, nq = nsub * nsub;
  const long row = idx / quads;  // (g*nq + q)*Na + a
  const int b = 4 * (int)(idx - row * quads);
  const int grp = (int)(row / ((long)nq * Na)), r2 = (int)(row - (long)grp * nq * Na);
  const int q = r2 / Na, a = r2 - q * Na, qy = q / nsub, qx = q - qy * nsub;
  Vec4 t[9], u[18];
#pragma unroll
  for (int i = 0; i < 3; ++i)
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      const int r = 3 * qy + i, s2 = 3 * qx + j;
      t[3 * i + j] = vzero();
      if (r < k && s2 < k) t[3 * i + j] = vload(w + (((long)grp * k * k + r * k + s2) * Na + a) * Nb + b);
    }
#pragma unroll
  for (int j = 0; j < 3; ++j) wino_g<3, 3>(t + j, u + j);  // columns: 3 -> 6 rows of 3
#pragma unroll
  for (int i = 0; i < 6; ++i) {
    Vec4 r[6];
    wino_g<1, 1>(u + 3 * i, r);
#pragma unroll
    for (int j = 0; j < 6; ++j) {
      const long z = (long)(6 * i + j) * groups + grp;
      vstore(U + (q_in_cols ? ((z * Na + a) * nq + q) * Nb + b : ((z * nq + q) * Na + a) * Nb + b), r[j]);
    }
  }
}
// dw[groups][(r, s, a)][b] = (Gt m G)[i][j] at r = 3qy + i, s = 3qx + j (taps that exist only),
// m[p] = dU[(p*groups + g)][q*Na + a][b].  idx as in wino_filter_thread.
AX_HD void wino_dw_thread(int groups, int Na, int Nb, int k, int nsub, const float* dU, float* dw, long idx) {
  const int quads = Nb / 4, nq = nsub * nsub;
  const long row = idx / quads;
  const int b = 4 * (int)(idx - row * quads);
  const int grp = (int)(row / ((long)nq * Na)), r2 = (int)(row - (long)grp * nq * Na);
  const int q = r2 / Na, a = r2 - q * Na, qy = q / nsub, qx = q - qy * nsub;
  const long slab = (long)nq * Na * Nb;
  Vec4 u[18];
#pragma unroll
  for (int j = 0; j < 6; ++j) {
    Vec4 col[6];
#pragma unroll
    for (int i = 0; i < 6; ++i) {
      col[i] = vload(dU + ((long)(6 * i + j) * groups + grp) * slab + ((long)q * Na + a) * Nb + b);
    }
    wino_gt<1, 6>(col, u + j);  // u[i][j], 3 rows of 6
  }
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    Vec4 o[3];
    wino_gt<1, 1>(u + 6 * i, o);
    const int r = 3 * qy + i;
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      const int s2 = 3 * qx + j;
      if (r < k && s2 < k) vstore(dw + (((long)grp * k * k + r * k + s2) * Na + a) * Nb + b, o[j]);
    }
  }
}

}  // namespace ax
