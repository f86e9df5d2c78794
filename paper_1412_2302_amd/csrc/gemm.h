// fp32 MFMA GEMM core for gfx950 with pluggable operand loaders and epilogues.
//
//   C[m][n] = sum_k A(m,k) * B(k,n)          (per group, per split of k)
//
// A workgroup of four 64-lane waves owns a BM x BN tile of C.  Both operands
// are staged through LDS k-major (tile[k][row]) so that one ds_read_b32 per
// lane feeds v_mfma_f32_32x32x2_f32 directly: lane l supplies A[l%32][l/32]
// and B[l/32][l%32].  Global loads of tile t+1 are issued before the MFMA
// loop of tile t and written to the other LDS buffer afterwards, so a single
// barrier per k-tile is enough.
//
// Loaders know how an operand lives in memory:
//   DenseKInner     elem(row,k) = p[row*ld + k]      (contiguous along k)
//   DenseRowInner   elem(row,k) = p[k*ld + row]      (contiguous along rows)
//   Im2colKInner    rows = output pixels, k = (r,s,c): the implicit im2col
//                   matrix of a channel-last activation tensor (convolution
//                   forward, and backward-data in its transposed modes)
//   Im2colRowInner  rows = (r,s,c), k = output pixels: its transpose
//                   (convolution backward-weight)
// Every loader zero-fills outside the operand, so ragged tiles need no care
// in the MFMA loop.  Loads are predicated, never branched around: an element
// outside the operand reads the operand's first element and is then replaced
// by zero, which keeps the k-loop one straight-line block that the compiler
// can software-pipeline.  Index decoding uses multiply-shift division by
// launch constants.  A loader works in steps that the kernel places one by one:
// addr_step<S>() computes offsets and predicates of a later k-tile (pure VALU
// work), fetch<SET>() issues its global loads into one of two register sets,
// store_step<SET>(s) zeroes what was outside the operand and writes one load
// to LDS.  VEC selects 16-byte loads (legal only when the launcher
// has checked alignment and divisibility) or four 4-byte loads.
//
// Everything here is also compiled for the host by the CPU emulation test
// (AX_HOST_EMU), which is why loaders and epilogues are plain structs with
// host+device members.
#pragma once

#include <stdint.h>

#ifndef AX_HOST_EMU
#include <hip/hip_runtime.h>
#define AX_HD __host__ __device__ __forceinline__
#else
#define AX_HD inline
#endif

namespace ax {

constexpr int kThreads = 256;

template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_>
struct Tile {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int TM = BM / (32 * WAVES_M), TN = BN / (32 * WAVES_N);
  static constexpr int PAD = 4;
  static constexpr int LDA = BM + PAD, LDB = BN + PAD;
  static_assert(WAVES_M * WAVES_N * 64 == kThreads, "four waves per workgroup");
  static_assert(TM * 32 * WAVES_M == BM && TN * 32 * WAVES_N == BN, "tile must be whole 32x32 MFMA blocks");
  static_assert(BK % 4 == 0, "k tile is loaded in quads");
};

AX_HD float4 zero4() {
  float4 v;
  v.x = v.y = v.z = v.w = 0.f;
  return v;
}
AX_HD float4 ld4(const float* q) { return *reinterpret_cast<const float4*>(q); }
// ---- division by a launch constant -------------------------------------------
// q = n / d for 0 <= n < 2^31:  umulhi(n, mul) >> shift, mul = ceil(2^(31+l)/d),
// l = ceil(log2 d), shift = l - 1; d == 1 is handled by mul == 0.
struct FastDiv {
  uint32_t mul, shift, d;
};
inline FastDiv make_fastdiv(uint32_t d) {
  FastDiv f;
  f.d = d;
  if (d <= 1) {
    f.mul = 0;
    f.shift = 0;
    return f;
  }
  uint32_t l = 0;
  while ((1u << l) < d) ++l;
  const uint64_t num = 1ull << (31 + l);
  f.mul = (uint32_t)((num + d - 1) / d);
  f.shift = l - 1;
  return f;
}
AX_HD uint32_t umulhi32(uint32_t a, uint32_t b) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __umulhi(a, b);
#else
  return (uint32_t)(((uint64_t)a * b) >> 32);
#endif
}
AX_HD uint32_t fdiv(uint32_t n, const FastDiv& f) {
  const uint32_t q = umulhi32(n, f.mul) >> f.shift;
  return f.mul ? q : n;
}

// ---- fragment and accumulator index maps of v_mfma_f32_32x32x2_f32 ---------
// A/B fragment for k-pair kk: lane reads tile[(2*kk + lane/32)][base + lane%32].
AX_HD int frag_k(int lane, int kk) { return 2 * kk + (lane >> 5); }
// accumulator register r of a lane holds C[acc_row(lane,r)][lane%32] of the 32x32 block
AX_HD int acc_row(int lane, int r) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// =========================== operand loaders ================================

struct DenseParams {
  const float* p;
  long ld;       // leading dimension in floats
  long gstride;  // added per group
  int R;         // number of valid rows
};

// Per-thread bookkeeping shared by all loaders.  A thread makes NL loads per
// k-tile (16 bytes each when VEC, else four 4-byte loads).  `off`/`okn` describe
// the tile that will be fetched next; two register sets can be in flight, and
// ok[set] remembers which of their elements were inside the operand.
template <int NL_, bool VEC>
struct PlanRegs {
  static constexpr int NL = NL_, NE = VEC ? NL : 4 * NL;
  uint32_t off[NE];
  uint32_t okn;
  uint32_t ok[2];
  AX_HD void put(int e, uint32_t o, bool good) {
    off[e] = good ? o : 0u;  // an element outside reads element 0 and is zeroed when stored
    okn |= (uint32_t)good << e;
  }
  template <int SET>
  AX_HD void fetch(const float* p, float4* r) {
    ok[SET] = okn;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      if (VEC) {
        r[i] = *reinterpret_cast<const float4*>(p + off[i]);
      } else {
        r[i].x = p[off[4 * i]];
        r[i].y = p[off[4 * i + 1]];
        r[i].z = p[off[4 * i + 2]];
        r[i].w = p[off[4 * i + 3]];
      }
    }
  }
  template <int SET>
  AX_HD float4 masked(const float4& v, int i) const {
    const uint32_t m = ok[SET] >> (VEC ? i : 4 * i);
    float4 o;
    o.x = (m & 1u) ? v.x : 0.f;
    o.y = (VEC ? (m & 1u) : (m & 2u)) ? v.y : 0.f;
    o.z = (VEC ? (m & 1u) : (m & 4u)) ? v.z : 0.f;
    o.w = (VEC ? (m & 1u) : (m & 8u)) ? v.w : 0.f;
    return o;
  }
};
// four floats that are consecutive in k go to four LDS rows
AX_HD void lds_put_k4(float* d, int ldt, const float4& v) {
  d[0] = v.x;
  d[ldt] = v.y;
  d[2 * ldt] = v.z;
  d[3 * ldt] = v.w;
}

template <int ROWS, int BK, bool VEC>
struct DenseKInner {
  static constexpr int QK = BK / 4, NQ = ROWS * QK, NL = NQ / kThreads, NA = NL;
  static_assert(NQ % kThreads == 0, "tile must be a whole number of loads per thread");
  typedef DenseParams Params;
  const float* p;
  uint32_t ld;
  int R, tid, row0;
  PlanRegs<NL, VEC> pl;
  AX_HD DenseKInner(const Params& a, int g, int tid_, int row0_)
      : p(a.p + (long)g * a.gstride), ld((uint32_t)a.ld), R(a.R), tid(tid_), row0(row0_) {}
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    if (S == 0) pl.okn = 0;
    const int idx = tid + S * kThreads;
    const int row = row0 + idx / QK, k = k0 + 4 * (idx % QK);
    const bool rok = row < R;
    const uint32_t off = (uint32_t)row * ld + (uint32_t)k;
    if (VEC) {
      pl.put(S, off, rok && k < kend);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) pl.put(4 * S + j, off + j, rok && k + j < kend);
    }
  }
  template <int SET>
  AX_HD void fetch(float4* r) { pl.template fetch<SET>(p, r); }
  template <int SET>
  AX_HD void store_step(int s, float* lds, int ldt, const float4* r) const {
    const int idx = tid + s * kThreads;
    lds_put_k4(lds + (4 * (idx % QK)) * ldt + idx / QK, ldt, pl.template masked<SET>(r[s], s));
  }
};

template <int ROWS, int BK, bool VEC>
struct DenseRowInner {
  static constexpr int QR = ROWS / 4, NQ = QR * BK, NL = (NQ + kThreads - 1) / kThreads, NA = NL;
  static constexpr bool kWhole = NQ % kThreads == 0;  // else the last load of some threads is outside the tile
  typedef DenseParams Params;
  const float* p;
  uint32_t ld;
  int R, tid, row0;
  PlanRegs<NL, VEC> pl;
  AX_HD DenseRowInner(const Params& a, int g, int tid_, int row0_)
      : p(a.p + (long)g * a.gstride), ld((uint32_t)a.ld), R(a.R), tid(tid_), row0(row0_) {}
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    if (S == 0) pl.okn = 0;
    const int idx = tid + S * kThreads;
    const int row = row0 + 4 * (idx % QR), k = k0 + idx / QR;
    const bool kok = k < kend && (kWhole || idx < NQ);
    const uint32_t off = (uint32_t)k * ld + (uint32_t)row;
    if (VEC) {
      pl.put(S, off, kok && row < R);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) pl.put(4 * S + j, off + j, kok && row + j < R);
    }
  }
  template <int SET>
  AX_HD void fetch(float4* r) { pl.template fetch<SET>(p, r); }
  template <int SET>
  AX_HD void store_step(int s, float* lds, int ldt, const float4* r) const {
    const int idx = tid + s * kThreads;
    if (kWhole || idx < NQ)
      *reinterpret_cast<float4*>(lds + (idx / QR) * ldt + 4 * (idx % QR)) = pl.template masked<SET>(r[s], s);
  }
};

// Geometry of an implicit im2col operand over a channel-last tensor
// x[N][H][W][Ctot].  Pixels (n, y, x) run over an OH x OW grid; tap (r, s)
// of pixel (y, x) reads x[n][iy][ix][c_off + c] with
//   mode 0 (forward):            iy = y*stride - pad + r
//   mode 1 (transposed, unit):   iy = y + pad - r                    (stride 1)
//   mode 2 (transposed, strided) iy = (y + pad - r)/stride, only where exact
// (modes 1 and 2 are the gather form of the adjoint of a convolution).
struct Im2colParams {
  const float* x;
  int H, W, Ctot;   // tensor being gathered from
  int Cg;           // channels per group (extent of c)
  int c_stride_g;   // channel offset added per group
  int kh, kw, stride, pad;
  int OH, OW;       // pixel grid
  int P;            // number of pixels = N*OH*OW
  FastDiv d_cg, d_kw, d_ohw, d_ow, d_stride;
};
enum { IM2COL_FWD = 0, IM2COL_T1 = 1, IM2COL_TS = 2 };

struct TapCoord {
  int r, s, c;
};
AX_HD TapCoord decode_tap(int k, const Im2colParams& g) {
  TapCoord t;
  const int rs = (int)fdiv((uint32_t)k, g.d_cg);
  t.c = k - rs * g.Cg;
  t.r = (int)fdiv((uint32_t)rs, g.d_kw);
  t.s = rs - t.r * g.kw;
  return t;
}
struct PixCoord {
  int n, y, x;
};
AX_HD PixCoord decode_pixel(int p, const Im2colParams& g) {
  PixCoord c;
  c.n = (int)fdiv((uint32_t)p, g.d_ohw);
  const int rem = p - c.n * (g.OH * g.OW);
  c.y = (int)fdiv((uint32_t)rem, g.d_ow);
  c.x = rem - c.y * g.OW;
  return c;
}
// pixel offset iy*W + ix of tap (r,s) seen from origin (y0,x0); ok = inside the tensor
template <int MODE>
AX_HD uint32_t tap_offset(const Im2colParams& g, int y0, int x0, int r, int s, bool& ok) {
  int iy, ix;
  if (MODE == IM2COL_FWD) {
    iy = y0 + r;
    ix = x0 + s;
    ok = (uint32_t)iy < (uint32_t)g.H && (uint32_t)ix < (uint32_t)g.W;
  } else if (MODE == IM2COL_T1) {
    iy = y0 - r;
    ix = x0 - s;
    ok = (uint32_t)iy < (uint32_t)g.H && (uint32_t)ix < (uint32_t)g.W;
  } else {
    const int ty = y0 - r, tx = x0 - s;
    const bool pos = ty >= 0 && tx >= 0;
    iy = (int)fdiv((uint32_t)(pos ? ty : 0), g.d_stride);
    ix = (int)fdiv((uint32_t)(pos ? tx : 0), g.d_stride);
    ok = pos && iy * g.stride == ty && ix * g.stride == tx && iy < g.H && ix < g.W;
  }
  return (uint32_t)iy * (uint32_t)g.W + (uint32_t)ix;  // unsigned: wraps harmlessly when the tap is outside
}
constexpr int kInvalidCoord = -(1 << 28);

template <int ROWS, int BK, bool VEC, int MODE>
struct Im2colKInner {
  static constexpr int QK = BK / 4, NQ = ROWS * QK, NL = NQ / kThreads, NA = NL + 1;
  static_assert(kThreads % QK == 0 && NQ % kThreads == 0, "every load of a thread shares its k quad");
  typedef Im2colParams Params;
  Im2colParams g;
  int c_off, tid, kq;
  uint32_t nb[NL];  // pixel index of (n, 0, 0)
  int y0[NL], x0[NL];
  TapCoord tap[VEC ? 1 : 4];
  uint32_t kok;
  PlanRegs<NL, VEC> pl;
  AX_HD Im2colKInner(const Params& a, int grp, int tid_, int row0) : g(a), c_off(grp * a.c_stride_g), tid(tid_) {
    kq = tid % QK;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int p = row0 + (tid + i * kThreads) / QK;
      const bool in = p < g.P;
      const PixCoord c = decode_pixel(in ? p : 0, g);
      nb[i] = (uint32_t)c.n * (uint32_t)(g.H * g.W);
      if (MODE == IM2COL_FWD) {
        y0[i] = in ? c.y * g.stride - g.pad : kInvalidCoord;
        x0[i] = c.x * g.stride - g.pad;
      } else {
        // rows past the end get an origin whose every tap is above the tensor
        y0[i] = in ? c.y + g.pad : -1;
        x0[i] = c.x + g.pad;
      }
    }
  }
  // step 0 decodes the taps of the thread's k quad, step 1+i places load i
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    const int k = k0 + 4 * kq;
    if (S == 0) {
      pl.okn = 0;
      kok = 0;
#pragma unroll
      for (int j = 0; j < (VEC ? 1 : 4); ++j) {
        tap[j] = decode_tap(k + j, g);
        kok |= (uint32_t)(k + j < kend) << j;
      }
    } else {
      constexpr int i = S - 1;
#pragma unroll
      for (int j = 0; j < (VEC ? 1 : 4); ++j) {
        bool ok;
        const uint32_t po = tap_offset<MODE>(g, y0[i], x0[i], tap[j].r, tap[j].s, ok);
        const uint32_t off = (nb[i] + po) * (uint32_t)g.Ctot + (uint32_t)(c_off + tap[j].c);
        pl.put(VEC ? i : 4 * i + j, off, ok && ((kok >> j) & 1u));
      }
    }
  }
  template <int SET>
  AX_HD void fetch(float4* r) { pl.template fetch<SET>(g.x, r); }
  template <int SET>
  AX_HD void store_step(int s, float* lds, int ldt, const float4* r) const {
    lds_put_k4(lds + (4 * kq) * ldt + (tid + s * kThreads) / QK, ldt, pl.template masked<SET>(r[s], s));
  }
};

template <int ROWS, int BK, bool VEC>
struct Im2colRowInner {
  static constexpr int QR = ROWS / 4, NQ = QR * BK, NL = NQ / kThreads, NA = NL;
  static_assert(kThreads % QR == 0 && NQ % kThreads == 0, "every load of a thread shares its row quad");
  typedef Im2colParams Params;
  Im2colParams g;
  int c_off, tid, rq;
  int rr[VEC ? 1 : 4], ss[VEC ? 1 : 4], cc[VEC ? 1 : 4];  // taps of the thread's rows; rr = kInvalidCoord past the end
  PlanRegs<NL, VEC> pl;
  AX_HD Im2colRowInner(const Params& a, int grp, int tid_, int row0) : g(a), c_off(grp * a.c_stride_g), tid(tid_) {
    rq = tid % QR;
    const int rtot = g.kh * g.kw * g.Cg;
#pragma unroll
    for (int j = 0; j < (VEC ? 1 : 4); ++j) {
      const int m = row0 + 4 * rq + j;
      const bool in = m < rtot;
      const TapCoord t = decode_tap(in ? m : 0, g);
      rr[j] = in ? t.r : kInvalidCoord;  // pushes every tap above the tensor
      ss[j] = t.s;
      cc[j] = t.c;
    }
  }
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    if (S == 0) pl.okn = 0;
    const int p = k0 + (tid + S * kThreads) / QR;
    const bool pok = p < kend;
    const PixCoord c = decode_pixel(pok ? p : 0, g);
    const uint32_t nbase = (uint32_t)c.n * (uint32_t)(g.H * g.W);
    const int y0 = c.y * g.stride - g.pad, x0 = c.x * g.stride - g.pad;
#pragma unroll
    for (int j = 0; j < (VEC ? 1 : 4); ++j) {
      bool ok;
      const uint32_t po = tap_offset<IM2COL_FWD>(g, y0, x0, rr[j], ss[j], ok);
      const uint32_t off = (nbase + po) * (uint32_t)g.Ctot + (uint32_t)(c_off + cc[j]);
      pl.put(VEC ? S : 4 * S + j, off, ok && pok);
    }
  }
  template <int SET>
  AX_HD void fetch(float4* r) { pl.template fetch<SET>(g.x, r); }
  template <int SET>
  AX_HD void store_step(int s, float* lds, int ldt, const float4* r) const {
    *reinterpret_cast<float4*>(lds + ((tid + s * kThreads) / QR) * ldt + 4 * rq) = pl.template masked<SET>(r[s], s);
  }
};

// Whole-tile helpers (prologue of the kernel, CPU emulation).
template <class L, int S = 0>
AX_HD void plan_all(L& l, int k0, int kend) {
  if constexpr (S < L::NA) {
    l.template addr_step<S>(k0, kend);
    plan_all<L, S + 1>(l, k0, kend);
  }
}
template <int SET, class L>
AX_HD void store_all(const L& l, float* lds, int ldt, const float4* r) {
#pragma unroll
  for (int s = 0; s < L::NL; ++s) l.template store_step<SET>(s, lds, ldt, r);
}

// ================================ epilogues ==================================
// apply(m, n, v) is called once per valid element of the tile.

// y[m][col_off + n] = act(v + bias[col_off + n]); col_off = group * cols_per_group
struct EpiBiasAct {
  float* y;
  long ldc;
  const float* bias;  // may be null
  int relu, cols_per_group, col_off;
  AX_HD void set_group(int g, int /*z*/) { col_off = g * cols_per_group; }
  AX_HD void apply(int m, int n, float v) const {
    if (bias) v += bias[col_off + n];
    if (relu) v = v > 0.f ? v : 0.f;
    y[(long)m * ldc + col_off + n] = v;
  }
};

// dx[m][col_off + n] = gate ? (gate[m][col_off+n] > 0 ? v : 0) : v
struct EpiGate {
  float* dx;
  long ldc;
  const float* gate;  // forward activation with the layout of dx, or null
  int cols_per_group, col_off;
  AX_HD void set_group(int g, int /*z*/) { col_off = g * cols_per_group; }
  AX_HD void apply(int m, int n, float v) const {
    const long o = (long)m * ldc + col_off + n;
    if (gate && !(gate[o] > 0.f)) v = 0.f;
    dx[o] = v;
  }
};

// ws[z][m][n] = v   (z = group*nsplit + split); one M x N slab per launch slice
struct EpiSlab {
  float* ws;
  long slab;  // M*N
  long ldc;   // N
  float* base;
  AX_HD void set_group(int /*g*/, int z) { base = ws + (long)z * slab; }
  AX_HD void apply(int m, int n, float v) const { base[(long)m * ldc + n] = v; }
};

// ================================= kernel ====================================
#ifndef AX_HOST_EMU
typedef float v16f __attribute__((ext_vector_type(16)));

// ---- the k-tile: MFMAs with the rest of the pipeline in their shadow ----------
// While the MFMAs of tile t run, the same wave (a) writes tile t+1, which was
// fetched one iteration ago, to the other LDS buffer and (b) computes the
// addresses of tile t+3.  That side work is cut into steps and dealt out over
// the k-pairs of the tile; a scheduling fence after every k-pair keeps each
// portion in the shadow of that pair's MFMAs instead of in one lump after them.
template <class T, class AL, class BL, int SET, int IDX>
__device__ __forceinline__ void side_step(AL& al, BL& bl, float* as_next, float* bs_next, const float4* ra,
                                          const float4* rb, int k_plan, int kend) {
  constexpr int S0 = AL::NL, S1 = S0 + BL::NL, S2 = S1 + AL::NA, S3 = S2 + BL::NA;
  if constexpr (IDX < S0) {
    al.template store_step<SET>(IDX, as_next, T::LDA, ra);
  } else if constexpr (IDX < S1) {
    bl.template store_step<SET>(IDX - S0, bs_next, T::LDB, rb);
  } else if constexpr (IDX < S2) {
    al.template addr_step<IDX - S1>(k_plan, kend);
  } else if constexpr (IDX < S3) {
    bl.template addr_step<IDX - S2>(k_plan, kend);
  }
}
template <class T, class AL, class BL, int SET, int Q, int U = 0>
__device__ __forceinline__ void side_slot(AL& al, BL& bl, float* as_next, float* bs_next, const float4* ra,
                                          const float4* rb, int k_plan, int kend) {
  constexpr int TOTAL = AL::NL + BL::NL + AL::NA + BL::NA, KP = T::BK / 2, PER = (TOTAL + KP - 1) / KP;
  if constexpr (U < PER) {
    side_step<T, AL, BL, SET, Q * PER + U>(al, bl, as_next, bs_next, ra, rb, k_plan, kend);
    side_slot<T, AL, BL, SET, Q, U + 1>(al, bl, as_next, bs_next, ra, rb, k_plan, kend);
  }
}

template <class T, class AL, class BL, int SET, bool SIDE, int Q = 0>
__device__ __forceinline__ void tile_stream(const float* __restrict__ as, const float* __restrict__ bs, int kh,
                                            v16f (&acc)[T::TM][T::TN], float (&a)[2][T::TM], float (&b)[2][T::TN],
                                            AL& al, BL& bl, float* as_next, float* bs_next, const float4* ra,
                                            const float4* rb, int k_plan, int kend) {
  constexpr int KP = T::BK / 2;
  if constexpr (Q < KP) {
    constexpr int c = Q & 1, n = c ^ 1;
    if constexpr (Q + 1 < KP) {  // fragments of the next k-pair, one pair ahead of their MFMAs
      const int kr = 2 * (Q + 1) + kh;
#pragma unroll
      for (int i = 0; i < T::TM; ++i) a[n][i] = as[kr * T::LDA + i * 32];
#pragma unroll
      for (int j = 0; j < T::TN; ++j) b[n][j] = bs[kr * T::LDB + j * 32];
    }
#pragma unroll
    for (int i = 0; i < T::TM; ++i)
#pragma unroll
      for (int j = 0; j < T::TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[c][i], b[c][j], acc[i][j], 0, 0, 0);
    if constexpr (SIDE) side_slot<T, AL, BL, SET, Q>(al, bl, as_next, bs_next, ra, rb, k_plan, kend);
    __builtin_amdgcn_sched_barrier(0);
    tile_stream<T, AL, BL, SET, SIDE, Q + 1>(as, bs, kh, acc, a, b, al, bl, as_next, bs_next, ra, rb, k_plan, kend);
  }
}

// One iteration of the main loop for tile t, PAR = t & 1.  Register set PAR
// receives tile t+2, register set PAR^1 (tile t+1) is written to LDS buffer PAR^1.
template <class T, class AL, class BL, int PAR>
__device__ __forceinline__ void main_iter(float (&As)[2][T::BK * T::LDA], float (&Bs)[2][T::BK * T::LDB], int a_off,
                                          int b_off, int kh, v16f (&acc)[T::TM][T::TN], AL& al, BL& bl,
                                          float4 (&ra)[2][AL::NL], float4 (&rb)[2][BL::NL], int k_plan, int kend) {
  al.template fetch<PAR>(ra[PAR]);
  bl.template fetch<PAR>(rb[PAR]);
  float a[2][T::TM], b[2][T::TN];
  const float* as = As[PAR] + a_off;
  const float* bs = Bs[PAR] + b_off;
#pragma unroll
  for (int i = 0; i < T::TM; ++i) a[0][i] = as[kh * T::LDA + i * 32];
#pragma unroll
  for (int j = 0; j < T::TN; ++j) b[0][j] = bs[kh * T::LDB + j * 32];
  __builtin_amdgcn_sched_barrier(0);
  tile_stream<T, AL, BL, PAR ^ 1, true>(as, bs, kh, acc, a, b, al, bl, As[PAR ^ 1], Bs[PAR ^ 1], ra[PAR ^ 1],
                                        rb[PAR ^ 1], k_plan, kend);
  __syncthreads();
}

template <class T, class AL, class BL, class Epi>
__global__ void __launch_bounds__(kThreads)
gemm_kernel(typename AL::Params ap, typename BL::Params bp, Epi ep, int M, int N, int K, int kchunk, int nsplit) {
  __shared__ __attribute__((aligned(16))) float As[2][T::BK * T::LDA];
  __shared__ __attribute__((aligned(16))) float Bs[2][T::BK * T::LDB];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % T::WAVES_M, wn = wave / T::WAVES_M;
  const int z = blockIdx.z, g = z / nsplit, split = z - g * nsplit;
  const int m0 = blockIdx.x * T::BM, n0 = blockIdx.y * T::BN;
  const int kbeg = split * kchunk;
  const int kend = min(K, kbeg + kchunk);
  const int nt = kend > kbeg ? (kend - kbeg + T::BK - 1) / T::BK : 0;

  AL al(ap, g, tid, m0);
  BL bl(bp, g, tid, n0);
  ep.set_group(g, z);

  v16f acc[T::TM][T::TN];
#pragma unroll
  for (int i = 0; i < T::TM; ++i)
#pragma unroll
    for (int j = 0; j < T::TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int a_off = wm * (T::TM * 32) + (lane & 31), b_off = wn * (T::TN * 32) + (lane & 31), kh = lane >> 5;
  if (nt > 0) {
    // prologue: tile 0 -> LDS buffer 0, tile 1 in flight in register set 1, addresses of tile 2 ready.
    // Tiles past the end have every predicate off: they fetch element 0 and store zeros, harmlessly.
    float4 ra[2][AL::NL], rb[2][BL::NL];
    plan_all(al, kbeg, kend);
    plan_all(bl, kbeg, kend);
    al.template fetch<0>(ra[0]);
    bl.template fetch<0>(rb[0]);
    plan_all(al, kbeg + T::BK, kend);
    plan_all(bl, kbeg + T::BK, kend);
    al.template fetch<1>(ra[1]);
    bl.template fetch<1>(rb[1]);
    store_all<0>(al, As[0], T::LDA, ra[0]);
    store_all<0>(bl, Bs[0], T::LDB, rb[0]);
    plan_all(al, kbeg + 2 * T::BK, kend);
    plan_all(bl, kbeg + 2 * T::BK, kend);
    __syncthreads();
    for (int t = 0; t < nt; t += 2) {
      main_iter<T, AL, BL, 0>(As, Bs, a_off, b_off, kh, acc, al, bl, ra, rb, kbeg + (t + 3) * T::BK, kend);
      if (t + 1 < nt)
        main_iter<T, AL, BL, 1>(As, Bs, a_off, b_off, kh, acc, al, bl, ra, rb, kbeg + (t + 4) * T::BK, kend);
    }
  }

#pragma unroll
  for (int i = 0; i < T::TM; ++i)
#pragma unroll
    for (int j = 0; j < T::TN; ++j) {
      const int n = n0 + wn * (T::TN * 32) + j * 32 + (lane & 31);
      if (n >= N) continue;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * (T::TM * 32) + i * 32 + acc_row(lane, r);
        if (m < M) ep.apply(m, n, acc[i][j][r]);
      }
    }
}
#endif  // AX_HOST_EMU

}  // namespace ax
