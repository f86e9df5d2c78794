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
//                   forward, and backward-data when `transposed` is set)
//   Im2colRowInner  rows = (r,s,c), k = output pixels: its transpose
//                   (convolution backward-weight)
// Every loader zero-fills outside the operand, so ragged tiles need no care
// in the MFMA loop.  Everything here is also compiled for the host by the
// CPU emulation test (AX_HOST_EMU), which is why loaders and epilogues are
// plain structs with host+device members.
#pragma once

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
AX_HD float& at4(float4& v, int j) { return j == 0 ? v.x : j == 1 ? v.y : j == 2 ? v.z : v.w; }

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
  int vec;       // 1: 16-byte loads are legal (alignment and divisibility checked by the launcher)
};

template <int ROWS, int BK>
struct DenseKInner {
  static constexpr int QK = BK / 4, NQ = ROWS * QK, NL = (NQ + kThreads - 1) / kThreads;
  typedef DenseParams Params;
  const float* p;
  long ld;
  int R, vec, tid, row0;
  AX_HD DenseKInner(const Params& a, int g, int tid_, int row0_)
      : p(a.p + (long)g * a.gstride), ld(a.ld), R(a.R), vec(a.vec), tid(tid_), row0(row0_) {}
  AX_HD void load(int k0, int kend, float4* r) const {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int idx = tid + i * kThreads;
      float4 v = zero4();
      if (idx < NQ) {
        const int row = row0 + idx / QK, k = k0 + 4 * (idx % QK);
        if (row < R && k < kend) {
          const float* q = p + (long)row * ld + k;
          if (vec && k + 3 < kend) {
            v = ld4(q);
          } else {
            v.x = q[0];
            if (k + 1 < kend) v.y = q[1];
            if (k + 2 < kend) v.z = q[2];
            if (k + 3 < kend) v.w = q[3];
          }
        }
      }
      r[i] = v;
    }
  }
  AX_HD void store(float* lds, int ldt, const float4* r) const {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int idx = tid + i * kThreads;
      if (idx < NQ) {
        float* d = lds + (4 * (idx % QK)) * ldt + idx / QK;
        d[0] = r[i].x;
        d[ldt] = r[i].y;
        d[2 * ldt] = r[i].z;
        d[3 * ldt] = r[i].w;
      }
    }
  }
};

template <int ROWS, int BK>
struct DenseRowInner {
  static constexpr int QR = ROWS / 4, NQ = QR * BK, NL = (NQ + kThreads - 1) / kThreads;
  typedef DenseParams Params;
  const float* p;
  long ld;
  int R, vec, tid, row0;
  AX_HD DenseRowInner(const Params& a, int g, int tid_, int row0_)
      : p(a.p + (long)g * a.gstride), ld(a.ld), R(a.R), vec(a.vec), tid(tid_), row0(row0_) {}
  AX_HD void load(int k0, int kend, float4* r) const {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int idx = tid + i * kThreads;
      float4 v = zero4();
      if (idx < NQ) {
        const int row = row0 + 4 * (idx % QR), k = k0 + idx / QR;
        if (k < kend && row < R) {
          const float* q = p + (long)k * ld + row;
          if (vec && row + 3 < R) {
            v = ld4(q);
          } else {
            v.x = q[0];
            if (row + 1 < R) v.y = q[1];
            if (row + 2 < R) v.z = q[2];
            if (row + 3 < R) v.w = q[3];
          }
        }
      }
      r[i] = v;
    }
  }
  AX_HD void store(float* lds, int ldt, const float4* r) const {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int idx = tid + i * kThreads;
      if (idx < NQ) *reinterpret_cast<float4*>(lds + (idx / QR) * ldt + 4 * (idx % QR)) = r[i];
    }
  }
};

// Geometry of an implicit im2col operand over a channel-last tensor
// x[N][H][W][Ctot].  Pixels (n, y, x) run over an OH x OW grid; tap (r, s)
// of pixel (y, x) reads x[n][iy][ix][c_off + c] with
//   forward:     iy = y*stride - pad + r
//   transposed:  iy = (y + pad - r)/stride, only where that division is exact
// (the gather form of the adjoint of a strided convolution).
struct Im2colParams {
  const float* x;
  int H, W, Ctot;   // tensor being gathered from
  int Cg;           // channels per group (extent of c)
  int c_stride_g;   // channel offset added per group
  int kh, kw, stride, pad, transposed;
  int OH, OW;       // pixel grid
  int P;            // number of pixels = N*OH*OW
  int vec;          // 1: Cg % 4 == 0, Ctot % 4 == 0, aligned base
};

struct TapCoord {
  int r, s, c;
};
AX_HD TapCoord decode_tap(int k, int Cg, int kw) {
  TapCoord t;
  const int rs = k / Cg;
  t.c = k - rs * Cg;
  t.r = rs / kw;
  t.s = rs - t.r * kw;
  return t;
}
// returns the pixel offset iy*W + ix or -1 when the tap falls outside
AX_HD int tap_offset(const Im2colParams& g, int y0, int x0, int r, int s) {
  int iy, ix;
  if (!g.transposed) {
    iy = y0 + r;
    ix = x0 + s;
  } else {
    const int ty = y0 - r, tx = x0 - s;
    if (ty < 0 || tx < 0) return -1;
    if (g.stride == 1) {
      iy = ty;
      ix = tx;
    } else {
      iy = ty / g.stride;
      ix = tx / g.stride;
      if (iy * g.stride != ty || ix * g.stride != tx) return -1;
    }
  }
  if (iy < 0 || iy >= g.H || ix < 0 || ix >= g.W) return -1;
  return iy * g.W + ix;
}
constexpr int kInvalidCoord = -(1 << 28);

template <int ROWS, int BK>
struct Im2colKInner {
  static constexpr int QK = BK / 4, NQ = ROWS * QK, NL = (NQ + kThreads - 1) / kThreads;
  static_assert(kThreads % QK == 0, "every load of a thread must share its k quad");
  typedef Im2colParams Params;
  Im2colParams g;
  int c_off, tid, kq;
  long nb[NL];
  int y0[NL], x0[NL];
  AX_HD Im2colKInner(const Params& a, int grp, int tid_, int row0) : g(a), c_off(grp * a.c_stride_g), tid(tid_) {
    kq = tid % QK;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int idx = tid + i * kThreads;
      const int p = row0 + idx / QK;
      nb[i] = 0;
      y0[i] = x0[i] = kInvalidCoord;
      if (idx < NQ && p < g.P) {
        const int n = p / (g.OH * g.OW), rem = p - n * (g.OH * g.OW);
        const int y = rem / g.OW, x = rem - y * g.OW;
        nb[i] = (long)n * g.H * g.W;
        y0[i] = g.transposed ? y + g.pad : y * g.stride - g.pad;
        x0[i] = g.transposed ? x + g.pad : x * g.stride - g.pad;
      }
    }
  }
  AX_HD void load(int k0, int kend, float4* r) const {
    const int k = k0 + 4 * kq;
    if (g.vec) {
      const TapCoord t = decode_tap(k, g.Cg, g.kw);
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        float4 v = zero4();
        if (k < kend && y0[i] != kInvalidCoord) {
          const int off = tap_offset(g, y0[i], x0[i], t.r, t.s);
          if (off >= 0) v = ld4(g.x + (nb[i] + off) * g.Ctot + c_off + t.c);
        }
        r[i] = v;
      }
    } else {
#pragma unroll
      for (int i = 0; i < NL; ++i) r[i] = zero4();
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (k + j >= kend) continue;
        const TapCoord t = decode_tap(k + j, g.Cg, g.kw);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
          if (y0[i] == kInvalidCoord) continue;
          const int off = tap_offset(g, y0[i], x0[i], t.r, t.s);
          if (off >= 0) at4(r[i], j) = g.x[(nb[i] + off) * g.Ctot + c_off + t.c];
        }
      }
    }
  }
  AX_HD void store(float* lds, int ldt, const float4* r) const {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int idx = tid + i * kThreads;
      if (idx < NQ) {
        float* d = lds + (4 * kq) * ldt + idx / QK;
        d[0] = r[i].x;
        d[ldt] = r[i].y;
        d[2 * ldt] = r[i].z;
        d[3 * ldt] = r[i].w;
      }
    }
  }
};

template <int ROWS, int BK>
struct Im2colRowInner {
  static constexpr int QR = ROWS / 4, NQ = QR * BK, NL = (NQ + kThreads - 1) / kThreads;
  static_assert(kThreads % QR == 0, "every load of a thread must share its row quad");
  typedef Im2colParams Params;
  Im2colParams g;
  int c_off, tid, rq;
  int rr[4], ss[4], cc[4];  // taps of the thread's four rows; cc < 0 marks a row past the end
  AX_HD Im2colRowInner(const Params& a, int grp, int tid_, int row0) : g(a), c_off(grp * a.c_stride_g), tid(tid_) {
    rq = tid % QR;
    const int rtot = g.kh * g.kw * g.Cg;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = row0 + 4 * rq + j;
      rr[j] = ss[j] = 0;
      cc[j] = -1;
      if (m < rtot) {
        const TapCoord t = decode_tap(m, g.Cg, g.kw);
        rr[j] = t.r;
        ss[j] = t.s;
        cc[j] = t.c;
      }
    }
  }
  AX_HD void load(int k0, int kend, float4* r) const {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int idx = tid + i * kThreads;
      float4 v = zero4();
      const int p = k0 + idx / QR;
      if (idx < NQ && p < kend) {
        const int n = p / (g.OH * g.OW), rem = p - n * (g.OH * g.OW);
        const int y = rem / g.OW, x = rem - y * g.OW;
        const long nbase = (long)n * g.H * g.W;
        const int y0 = y * g.stride - g.pad, x0 = x * g.stride - g.pad;
        if (g.vec) {
          if (cc[0] >= 0) {
            const int off = tap_offset(g, y0, x0, rr[0], ss[0]);
            if (off >= 0) v = ld4(g.x + (nbase + off) * g.Ctot + c_off + cc[0]);
          }
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (cc[j] < 0) continue;
            const int off = tap_offset(g, y0, x0, rr[j], ss[j]);
            if (off >= 0) at4(v, j) = g.x[(nbase + off) * g.Ctot + c_off + cc[j]];
          }
        }
      }
      r[i] = v;
    }
  }
  AX_HD void store(float* lds, int ldt, const float4* r) const {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int idx = tid + i * kThreads;
      if (idx < NQ) *reinterpret_cast<float4*>(lds + (idx / QR) * ldt + 4 * rq) = r[i];
    }
  }
};

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

  float4 ra[AL::NL], rb[BL::NL];
  if (nt > 0) {
    al.load(kbeg, kend, ra);
    bl.load(kbeg, kend, rb);
    al.store(As[0], T::LDA, ra);
    bl.store(Bs[0], T::LDB, rb);
  }
  __syncthreads();

  for (int t = 0; t < nt; ++t) {
    const int cur = t & 1;
    const bool more = t + 1 < nt;
    if (more) {
      al.load(kbeg + (t + 1) * T::BK, kend, ra);
      bl.load(kbeg + (t + 1) * T::BK, kend, rb);
    }
    const float* as = As[cur] + wm * (T::TM * 32) + (lane & 31);
    const float* bs = Bs[cur] + wn * (T::TN * 32) + (lane & 31);
#pragma unroll
    for (int kk = 0; kk < T::BK / 2; ++kk) {
      float a[T::TM], b[T::TN];
      const int kr = frag_k(lane, kk);
#pragma unroll
      for (int i = 0; i < T::TM; ++i) a[i] = as[kr * T::LDA + i * 32];
#pragma unroll
      for (int j = 0; j < T::TN; ++j) b[j] = bs[kr * T::LDB + j * 32];
#pragma unroll
      for (int i = 0; i < T::TM; ++i)
#pragma unroll
        for (int j = 0; j < T::TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (more) {
      al.store(As[cur ^ 1], T::LDA, ra);
      bl.store(Bs[cur ^ 1], T::LDB, rb);
    }
    __syncthreads();
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
