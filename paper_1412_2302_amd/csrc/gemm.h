// fp32 MFMA GEMM core for gfx950 with pluggable operand loaders and epilogues.
//
//   C[m][n] = sum_k A(m,k) * B(k,n)          (per group, per split of k)
//
// A workgroup of four 64-lane waves owns a BM x BN tile of C and walks the
// reduction in k-tiles of BK.  On this hardware every VALU or LDS instruction
// a wave issues takes issue time away from its MFMAs (measured: ~5 cycles
// each against 64 per v_mfma_f32_32x32x2_f32), so the design goal is few
// instructions per MFMA:
//  * operands are fetched with raw buffer loads: an element outside the operand
//    gets a byte offset past the buffer and the hardware returns zero, so there
//    are no predicated selects and no 64-bit address arithmetic;
//  * an operand that is contiguous along k in memory is kept [row][k] in LDS:
//    one 16-byte store per load, and one 16-byte read gives a lane its values
//    for four MFMAs (the MFMAs then take k in the order 8q+j, 8q+4+j, which is
//    as good as any since both operands agree on it);
//  * an operand that is contiguous along rows is kept [k][row]: one 16-byte
//    store per load, 4-byte reads one k-pair ahead of their MFMAs;
//  * index decoding uses multiply-shift division by launch constants, and
//    everything that does not depend on the k-tile is computed once per thread.
// Global loads run two k-tiles ahead (two register sets), LDS is double
// buffered with one barrier per k-tile, and the LDS stores and address
// arithmetic of later tiles are dealt out between the MFMAs of the current one.
//
// Loaders know how an operand lives in memory:
//   DenseKInner     elem(row,k) = p[row*ld + k]      (contiguous along k)
//   DenseRowInner   elem(row,k) = p[k*ld + row]      (contiguous along rows)
//   Im2colKInner    rows = output pixels, k = (r,s,c): the implicit im2col
//                   matrix of a channel-last activation tensor (convolution
//                   forward, and backward-data in its transposed modes)
//   Im2colRowInner  rows = (r,s,c), k = output pixels: its transpose
//                   (convolution backward-weight)
// VEC selects 16-byte loads (legal only when the launcher has checked alignment
// and divisibility) or four 4-byte loads.  Every operand must be smaller than
// 2 GiB (byte offsets are 32-bit and 0x80000000 marks "outside").
//
// Everything here is also compiled for the host by the CPU emulation test
// (AX_HOST_EMU), which is why loaders and epilogues are plain structs with
// host+device members.
#pragma once

#include <stdint.h>
#include <string.h>

#include <type_traits>

#ifndef AX_HOST_EMU
#include <hip/hip_runtime.h>
#define AX_HD __host__ __device__ __forceinline__
#else
#define AX_HD inline
#endif

namespace ax {

constexpr int kThreads = 256;
constexpr uint32_t kOob = 0x80000000u;  // byte offset no operand reaches

// Workgroup tile BM x BN x BK computed by WAVES_M x WAVES_N waves out of RB x RB MFMA blocks:
// RB = 32 is v_mfma_f32_32x32x2_f32 (lane l supplies A[l%32][l/32] and B[l/32][l%32]; accumulator register
// r of lane l is C[8*(r/4) + 4*(l/32) + r%4][l%32]), RB = 16 is v_mfma_f32_16x16x4_f32 (A[l%16][l/16],
// B[l/16][l%16], C[4*(l/16) + r][l%16]).  Both run at the same rate; the small block exists for operands
// whose extent is a multiple of 16 but not of 32.
template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, int RB_ = 32>
struct Tile {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, RB = RB_;
  static constexpr int G = 64 / RB;          // k depth of one MFMA = lane groups along k
  static constexpr int KP = BK / G;          // MFMA steps per k-tile
  static constexpr int NACC = RB * RB / 64;  // accumulator registers per block
  static constexpr int TM = BM / (RB * WAVES_M), TN = BN / (RB * WAVES_N);
  static_assert(RB == 32 || RB == 16, "MFMA block is 32x32x2 or 16x16x4");
  static_assert(WAVES_M * WAVES_N * 64 == kThreads, "four waves per workgroup");
  static_assert(TM * RB * WAVES_M == BM && TN * RB * WAVES_N == BN, "tile must be whole MFMA blocks");
  static_assert(BK % (4 * G) == 0, "a lane's four consecutive k feed four MFMA steps");
  // k consumed by MFMA step u from lane group g (the same on both operands, so any order is a valid contraction)
  AX_HD static int step_k(int u, int g) { return 4 * G * (u >> 2) + 4 * g + (u & 3); }
  // Register r of a lane holds element [acc_row(lane, r)][lane % RB] of the MFMA's result block.  With an
  // epilogue that asks for it (kTransposed) the kernel feeds the B fragment as the MFMA's first operand, so the
  // block comes out transposed: C[lane % RB][acc_row(lane, r)], four consecutive columns per register quad
  // and one 16-byte store per quad.
  AX_HD static int acc_row(int lane, int r) {
    return RB == 32 ? 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3) : 4 * (lane >> 4) + r;
  }
};

// ---- buffer views --------------------------------------------------------------
#ifdef AX_HOST_EMU
struct BufView {
  const float* p;
  uint32_t bytes;
};
inline BufView make_view(const float* p, uint32_t bytes) { return BufView{p, bytes}; }
// Range checking is per dword, as measured on gfx950: the dwords of a 16-byte
// load that lie past num_records come back as zero, the others are loaded.
inline void emu_fail(const char* what);
inline float4 buf_ld4(const BufView& v, uint32_t off) {
  if (off & 3) emu_fail("unaligned buffer load");
  float r[4];
  for (int j = 0; j < 4; ++j) {
    const uint32_t o = off + 4u * j;
    r[j] = (o >= off && (uint64_t)o + 4 <= v.bytes) ? *reinterpret_cast<const float*>(reinterpret_cast<const char*>(v.p) + o) : 0.f;
  }
  float4 z;
  z.x = r[0]; z.y = r[1]; z.z = r[2]; z.w = r[3];
  return z;
}
inline float buf_ld1(const BufView& v, uint32_t off) {
  if (off >= v.bytes) return 0.f;
  if (off & 3) emu_fail("unaligned 4-byte load");
  return *reinterpret_cast<const float*>(reinterpret_cast<const char*>(v.p) + off);
}
#else
typedef __amdgpu_buffer_rsrc_t BufView;
__device__ __forceinline__ BufView make_view(const float* p, uint32_t bytes) {
  // raw buffer (stride 0): the range check is offset >= num_records -> 0
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ float4 buf_ld4(const BufView& v, uint32_t off) {
  typedef unsigned v4u __attribute__((ext_vector_type(4)));
  const v4u r = __builtin_amdgcn_raw_buffer_load_b128(v, (int)off, 0, 0);
  return __builtin_bit_cast(float4, r);
}
__device__ __forceinline__ float buf_ld1(const BufView& v, uint32_t off) {
  return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(v, (int)off, 0, 0));
}
#endif

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

// ---- index maps of v_mfma_f32_32x32x2_f32 ---------------------------------------
// MFMA step u = 4q + j of a k-tile consumes k = 8q + j (lanes 0..31) and
// k = 8q + 4 + j (lanes 32..63).
AX_HD int step_k(int u, int kh) { return 8 * (u >> 2) + 4 * kh + (u & 3); }
// accumulator register r of a lane holds D[acc_row(lane,r)][lane%32] of a 32x32 MFMA result D
AX_HD int acc_row(int lane, int r) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// =========================== operand loaders ================================
// Common interface (NL loads per thread and k-tile, NA address steps):
//   addr_step<S>(k0, kend)   byte offsets of the tile starting at k0 (S = 0..NA-1)
//   fetch(r)                 issue the NL loads of the last addressed tile
//   store_step(s, lds, r)    write load s to the LDS tile
//   kRowMajor, LD, LDS_FLOATS  layout of the LDS tile ([row][k] or [k][row])

struct DenseParams {
  const float* p;
  long ld;         // leading dimension in floats
  long gstride;    // floats added per group
  int R;           // number of valid rows
  uint32_t bytes;  // extent of the operand from p, all groups
};

template <int NL, bool VEC>
struct Offsets {
  static constexpr int NE = VEC ? NL : 4 * NL;
  uint32_t off[NE];
  AX_HD void fetch(const BufView& v, float4* r) const {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      if (VEC) {
        r[i] = buf_ld4(v, off[i]);
      } else {
        r[i].x = buf_ld1(v, off[4 * i]);
        r[i].y = buf_ld1(v, off[4 * i + 1]);
        r[i].z = buf_ld1(v, off[4 * i + 2]);
        r[i].w = buf_ld1(v, off[4 * i + 3]);
      }
    }
  }
};

template <int ROWS, int BK, bool VEC>
struct DenseKInner {
  static constexpr int QK = BK / 4, NQ = ROWS * QK, NL = NQ / kThreads, NA = NL;
  static constexpr bool kRowMajor = true;
  static constexpr int LD = BK + 4, LDS_FLOATS = ROWS * LD;
  static_assert(NQ % kThreads == 0, "tile must be a whole number of loads per thread");
  typedef DenseParams Params;
  BufView v;
  int tid, kq;
  uint32_t base[NL];  // byte offset of (row, 4*kq), or kOob for a row past the end
  Offsets<NL, VEC> pl;
  AX_HD DenseKInner(const Params& a, int g, int tid_, int row0)
      : v(make_view(a.p + (long)g * a.gstride, a.bytes - (uint32_t)(g * a.gstride * 4))), tid(tid_) {
    kq = tid % QK;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int row = row0 + (tid + i * kThreads) / QK;
      base[i] = row < a.R ? ((uint32_t)row * (uint32_t)a.ld + 4u * kq) * 4u : kOob;
    }
  }
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    const int k = k0 + 4 * kq;
    if (VEC) {
      pl.off[S] = k < kend ? base[S] + (uint32_t)k0 * 4u : kOob;
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) pl.off[4 * S + j] = k + j < kend ? base[S] + (uint32_t)(k0 + j) * 4u : kOob;
    }
  }
  AX_HD void fetch(float4* r) const { pl.fetch(v, r); }
  AX_HD void store_step(int s, float* lds, const float4* r) const {
    *reinterpret_cast<float4*>(lds + ((tid + s * kThreads) / QK) * LD + 4 * kq) = r[s];
  }
};

template <int ROWS, int BK, bool VEC>
struct DenseRowInner {
  static constexpr int QR = ROWS / 4, NQ = QR * BK, NL = (NQ + kThreads - 1) / kThreads, NA = NL;
  static constexpr bool kWhole = NQ % kThreads == 0;  // else the last load of some threads is outside the tile
  static constexpr bool kRowMajor = false;
  static constexpr int LD = ROWS + 4, LDS_FLOATS = BK * LD;
  typedef DenseParams Params;
  BufView v;
  int tid;
  uint32_t ld4;                          // leading dimension in bytes
  uint32_t base[VEC ? NL : 4 * NL];      // byte offset of (kl, row), or kOob
  Offsets<NL, VEC> pl;
  AX_HD DenseRowInner(const Params& a, int g, int tid_, int row0)
      : v(make_view(a.p + (long)g * a.gstride, a.bytes - (uint32_t)(g * a.gstride * 4))), tid(tid_) {
    ld4 = (uint32_t)a.ld * 4u;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int idx = tid + i * kThreads;
      const int row = row0 + 4 * (idx % QR), kl = idx / QR;
      const bool in = kWhole || idx < NQ;
#pragma unroll
      for (int j = 0; j < (VEC ? 1 : 4); ++j)
        base[VEC ? i : 4 * i + j] = in && row + j < a.R ? (uint32_t)kl * ld4 + (uint32_t)(row + j) * 4u : kOob;
    }
  }
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    const int k = k0 + (tid + S * kThreads) / QR;
    const uint32_t adv = (uint32_t)k0 * ld4;
#pragma unroll
    for (int j = 0; j < (VEC ? 1 : 4); ++j) {
      const int e = VEC ? S : 4 * S + j;
      pl.off[e] = k < kend ? base[e] + adv : kOob;
    }
  }
  AX_HD void fetch(float4* r) const { pl.fetch(v, r); }
  AX_HD void store_step(int s, float* lds, const float4* r) const {
    const int idx = tid + s * kThreads;
    if (kWhole || idx < NQ) *reinterpret_cast<float4*>(lds + (idx / QR) * LD + 4 * (idx % QR)) = r[s];
  }
};

// DenseRowInner for GEMMs whose K and split chunk are multiples of BK: every k-tile is whole, the k test
// is the same for all threads, and an address is one add.  A k-tile past the end is only ever prefetched,
// never multiplied, so it may read real data: k0 is clamped to the last tile instead of being zero-filled.
template <int ROWS, int BK>
struct DenseRowWhole : DenseRowInner<ROWS, BK, true> {
  typedef DenseRowInner<ROWS, BK, true> Base;
  using Base::Base;
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    const int kc = k0 < kend ? k0 : kend - BK;  // uniform
    this->pl.off[S] = this->base[S] + (uint32_t)kc * this->ld4;
  }
};

// Geometry of an implicit im2col operand over a channel-last tensor
// x[N][H][W][Ctot].  Pixels (n, y, x) run over an OH x OW grid; tap (r, s)
// of pixel (y, x) reads x[n][iy][ix][c_off + c] with
//   mode 0 (forward):            iy = y*stride - pad + r
//   mode 1 (transposed, unit):   iy = y + pad - r                    (stride 1)
//   mode 2 (transposed, strided) iy = (y + pad - r)/stride, only where exact
// (modes 1 and 2 are the gather form of the adjoint of a convolution).
//
// Run mode (forward geometry only): an unpadded convolution whose channel count
// is not a multiple of four (3-channel pictures) is viewed as a tensor
// x'[N][H][W*C] with one channel: all taps (s, c) of one kernel row r are then
// one contiguous run of kw*C floats starting at column x*stride*C, which is
// read in 16-byte pieces (4-byte aligned) and padded to a multiple of four with
// weights that are zero.  In the struct this is kw = 1, Cg = run length,
// Ctot = 1, W = W*C, stride_x = stride*C.
struct Im2colParams {
  const float* x;
  uint32_t bytes;   // extent of the tensor
  int H, W, Ctot;   // tensor being gathered from
  int Cg;           // channels per group (extent of c)
  int c_stride_g;   // channel offset added per group
  int kh, kw, stride, pad;
  int stride_x, pad_x;  // forward mode only: step and padding along x (differ from stride/pad in run mode)
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
constexpr int kFar = 1 << 28;  // coordinate that puts every tap outside the tensor

// Byte offset of tap (r,s,c) seen from a pixel whose origin is (y0, x0) and
// whose origin offset is rowbase = ((n*H*W + y0*W + x0)*Ctot + c_off)*ES (mod 2^32); ES = bytes per element.
template <int MODE, int ES = 4>
AX_HD uint32_t tap_address(const Im2colParams& g, uint32_t rowbase, int y0, int x0, const TapCoord& t) {
  if (MODE == IM2COL_TS) {
    const int ty = y0 - t.r, tx = x0 - t.s;
    const bool pos = ty >= 0 && tx >= 0;
    const int iy = (int)fdiv((uint32_t)(pos ? ty : 0), g.d_stride);
    const int ix = (int)fdiv((uint32_t)(pos ? tx : 0), g.d_stride);
    const bool ok = pos && iy * g.stride == ty && ix * g.stride == tx && iy < g.H && ix < g.W;
    // rowbase is the offset of (n, 0, 0, c_off) in this mode
    return ok ? rowbase + ((uint32_t)(iy * g.W + ix) * (uint32_t)g.Ctot + (uint32_t)t.c) * (uint32_t)ES : kOob;
  }
  const int iy = MODE == IM2COL_FWD ? y0 + t.r : y0 - t.r;
  const int ix = MODE == IM2COL_FWD ? x0 + t.s : x0 - t.s;
  const bool ok = (uint32_t)iy < (uint32_t)g.H && (uint32_t)ix < (uint32_t)g.W;
  const uint32_t tap = (((uint32_t)t.r * (uint32_t)g.W + (uint32_t)t.s) * (uint32_t)g.Ctot) * (uint32_t)ES;
  const uint32_t o = (MODE == IM2COL_FWD ? rowbase + tap : rowbase - tap) + (uint32_t)t.c * (uint32_t)ES;
  return ok ? o : kOob;
}
template <int MODE, int ES = 4>
AX_HD uint32_t row_base(const Im2colParams& g, int n, int y0, int x0, int c_off) {
  const uint32_t img = (uint32_t)n * (uint32_t)(g.H * g.W);
  if (MODE == IM2COL_TS) return (img * (uint32_t)g.Ctot + (uint32_t)c_off) * (uint32_t)ES;
  return ((img + (uint32_t)y0 * (uint32_t)g.W + (uint32_t)x0) * (uint32_t)g.Ctot + (uint32_t)c_off) * (uint32_t)ES;
}

template <int ROWS, int BK, bool VEC, int MODE>
struct Im2colKInner {
  static constexpr int QK = BK / 4, NQ = ROWS * QK, NL = NQ / kThreads, NA = NL + 1;
  static constexpr bool kRowMajor = true;
  static constexpr int LD = BK + 4, LDS_FLOATS = ROWS * LD;
  static_assert(kThreads % QK == 0 && NQ % kThreads == 0, "every load of a thread shares its k quad");
  typedef Im2colParams Params;
  Im2colParams g;
  BufView v;
  int tid, kq;
  uint32_t rowbase[NL];
  int y0[NL], x0[NL];
  TapCoord tap[VEC ? 1 : 4];
  Offsets<NL, VEC> pl;
  AX_HD Im2colKInner(const Params& a, int grp, int tid_, int row0) : g(a), v(make_view(a.x, a.bytes)), tid(tid_) {
    kq = tid % QK;
    const int c_off = grp * a.c_stride_g;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int p = row0 + (tid + i * kThreads) / QK;
      const bool in = p < g.P;
      const PixCoord c = decode_pixel(in ? p : 0, g);
      if (MODE == IM2COL_FWD) {
        y0[i] = in ? c.y * g.stride - g.pad : -kFar;
        x0[i] = c.x * g.stride_x - g.pad_x;
      } else {
        y0[i] = in ? c.y + g.pad : -kFar;
        x0[i] = c.x + g.pad;
      }
      rowbase[i] = row_base<MODE>(g, c.n, in ? y0[i] : 0, x0[i], c_off);
    }
  }
  // step 0 decodes the taps of the thread's k quad, step 1+i places load i
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    const int k = k0 + 4 * kq;
    if (S == 0) {
#pragma unroll
      for (int j = 0; j < (VEC ? 1 : 4); ++j) {
        tap[j] = decode_tap(k + j, g);
        // a k past the end turns into a tap far outside the picture
        if (k + j >= kend) tap[j].r = MODE == IM2COL_FWD ? 2 * kFar : -2 * kFar;
      }
    } else {
      constexpr int i = S - 1;
#pragma unroll
      for (int j = 0; j < (VEC ? 1 : 4); ++j)
        pl.off[VEC ? i : 4 * i + j] = tap_address<MODE>(g, rowbase[i], y0[i], x0[i], tap[j]);
    }
  }
  AX_HD void fetch(float4* r) const { pl.fetch(v, r); }
  AX_HD void store_step(int s, float* lds, const float4* r) const {
    *reinterpret_cast<float4*>(lds + ((tid + s * kThreads) / QK) * LD + 4 * kq) = r[s];
  }
};

// Im2colKInner for the common case that a k-tile lies inside one tap: channels per group a multiple of
// BK (so K is too), at most 32 taps, 16-byte loads, modes 0 and 1.  The tap (r, s) and first channel of a
// k-tile are then the same for the whole workgroup (scalar registers), and whether tap (r, s) of a pixel
// lies inside the tensor is looked up in a per-pixel bit mask built once per tile: an address costs an
// add, a bit-field extract and a bit-field insert.  K-tiles past the end are clamped as in DenseRowWhole.
template <int ROWS, int BK, int MODE>
struct Im2colKTap {
  static constexpr int QK = BK / 4, NQ = ROWS * QK, NL = NQ / kThreads, NA = NL + 1;
  static constexpr bool kRowMajor = true;
  static constexpr int LD = BK + 4, LDS_FLOATS = ROWS * LD;
  static_assert(kThreads % QK == 0 && NQ % kThreads == 0, "every load of a thread shares its k quad");
  static_assert(MODE == IM2COL_FWD || MODE == IM2COL_T1, "unit-step gathers only");
  typedef Im2colParams Params;
  Im2colParams g;
  BufView v;
  int tid, kq;
  uint32_t rowbase[NL];  // byte offset of the pixel's origin, its group's first channel and the thread's k quad
  uint32_t outside[NL];  // bit r*kw + s set: that tap of the pixel lies outside the tensor
  uint32_t tapoff;       // byte offset of the k-tile's tap and first channel from a pixel's origin (mod 2^32)
  int tapbit;
  Offsets<NL, true> pl;
  AX_HD Im2colKTap(const Params& a, int grp, int tid_, int row0) : g(a), v(make_view(a.x, a.bytes)), tid(tid_) {
    kq = tid % QK;
    const int c_off = grp * a.c_stride_g + 4 * kq;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int p = row0 + (tid + i * kThreads) / QK;
      const bool in = p < g.P;
      const PixCoord c = decode_pixel(in ? p : 0, g);
      const int y0 = MODE == IM2COL_FWD ? c.y * g.stride - g.pad : c.y + g.pad;
      const int x0 = MODE == IM2COL_FWD ? c.x * g.stride_x - g.pad_x : c.x + g.pad;
      rowbase[i] = row_base<MODE>(g, c.n, y0, x0, c_off);
      uint32_t inside = 0;
      int bit = 0;
      for (int r = 0; r < g.kh; ++r)
        for (int s2 = 0; s2 < g.kw; ++s2, ++bit) {
          const int iy = MODE == IM2COL_FWD ? y0 + r : y0 - r, ix = MODE == IM2COL_FWD ? x0 + s2 : x0 - s2;
          const bool ok = in && (uint32_t)iy < (uint32_t)g.H && (uint32_t)ix < (uint32_t)g.W;
          inside |= (ok ? 1u : 0u) << bit;
        }
      outside[i] = ~inside;
    }
  }
  // step 0 decodes the k-tile's tap (uniform), step 1+i places load i
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    if (S == 0) {
      const TapCoord t = decode_tap(k0 < kend ? k0 : kend - BK, g);
      const uint32_t tap = (((uint32_t)t.r * (uint32_t)g.W + (uint32_t)t.s) * (uint32_t)g.Ctot) * 4u;
      tapoff = (MODE == IM2COL_FWD ? tap : 0u - tap) + (uint32_t)t.c * 4u;
      tapbit = t.r * g.kw + t.s;
    } else {
      constexpr int i = S - 1;
      // all ones where the tap is outside: the offset then becomes exactly kOob (the sum itself may be
      // anything there, also close to 2^32, where a range check could wrap)
      const uint32_t out = 0u - ((outside[i] >> tapbit) & 1u);
      pl.off[i] = (out & kOob) | (~out & (rowbase[i] + tapoff));
    }
  }
  AX_HD void fetch(float4* r) const { pl.fetch(v, r); }
  AX_HD void store_step(int s, float* lds, const float4* r) const {
    *reinterpret_cast<float4*>(lds + ((tid + s * kThreads) / QK) * LD + 4 * kq) = r[s];
  }
};

template <int ROWS, int BK, bool VEC>
struct Im2colRowInner {
  static constexpr int QR = ROWS / 4, NQ = QR * BK, NL = NQ / kThreads, NA = NL;
  static constexpr bool kRowMajor = false;
  static constexpr int LD = ROWS + 4, LDS_FLOATS = BK * LD;
  static_assert(kThreads % QR == 0 && NQ % kThreads == 0, "every load of a thread shares its row quad");
  typedef Im2colParams Params;
  Im2colParams g;
  BufView v;
  int tid, rq, c_off;
  TapCoord tap[VEC ? 1 : 4];  // taps of the thread's rows; r = 2*kFar for a row past the end
  Offsets<NL, VEC> pl;
  AX_HD Im2colRowInner(const Params& a, int grp, int tid_, int row0)
      : g(a), v(make_view(a.x, a.bytes)), tid(tid_), c_off(grp * a.c_stride_g) {
    rq = tid % QR;
    const int rtot = g.kh * g.kw * g.Cg;
#pragma unroll
    for (int j = 0; j < (VEC ? 1 : 4); ++j) {
      const int m = row0 + 4 * rq + j;
      const bool in = m < rtot;
      tap[j] = decode_tap(in ? m : 0, g);
      if (!in) tap[j].r = 2 * kFar;
    }
  }
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    const int p = k0 + (tid + S * kThreads) / QR;
    const bool pok = p < kend;
    const PixCoord c = decode_pixel(pok ? p : 0, g);
    const int y0 = pok ? c.y * g.stride - g.pad : -kFar, x0 = c.x * g.stride_x - g.pad_x;
    const uint32_t rb = row_base<IM2COL_FWD>(g, c.n, pok ? y0 : 0, x0, c_off);
#pragma unroll
    for (int j = 0; j < (VEC ? 1 : 4); ++j)
      pl.off[VEC ? S : 4 * S + j] = tap_address<IM2COL_FWD>(g, rb, y0, x0, tap[j]);
  }
  AX_HD void fetch(float4* r) const { pl.fetch(v, r); }
  AX_HD void store_step(int s, float* lds, const float4* r) const {
    *reinterpret_cast<float4*>(lds + ((tid + s * kThreads) / QR) * LD + 4 * rq) = r[s];
  }
};

// Im2colRowInner for the common case of whole k-tiles, at most 31 taps and 16-byte loads.  The pixels of
// the workgroup's k range are decoded once, by all threads together, into a table in LDS: the byte offset
// of the pixel's origin and a bit mask of the taps that fall outside the tensor there.  A thread's tap never
// changes, so an address is a table read, an add, a mask test and a select.  K-tiles past the end are
// clamped as in DenseRowWhole.
struct PixelEntry {
  uint32_t base;     // byte offset of (n, y*stride - pad, x*stride_x - pad_x, channel 0), mod 2^32
  uint32_t outside;  // bit r*kw + s: that tap is outside the tensor; bit 31 always set
};
constexpr int kMaxTableK = 3072;  // longest k range of one workgroup with a table (24 KiB of LDS)
template <int ROWS, int BK>
struct Im2colRowTable {
  static constexpr int QR = ROWS / 4, NQ = QR * BK, NL = NQ / kThreads, NA = NL;
  static constexpr bool kRowMajor = false;
  static constexpr bool kUsesTable = true;
  static constexpr int LD = ROWS + 4, LDS_FLOATS = BK * LD;
  static_assert(kThreads % QR == 0 && NQ % kThreads == 0, "every load of a thread shares its row quad");
  typedef Im2colParams Params;
  BufView v;
  int tid, rq;
  uint32_t tapoff;   // byte offset of the thread's tap, first channel and group from a pixel's origin
  uint32_t tapmask;  // that tap's bit in PixelEntry::outside; bit 31 for a row past the end
  const PixelEntry* tbl;
  int kbase, klast;
  Offsets<NL, true> pl;
  AX_HD Im2colRowTable(const Params& a, int grp, int tid_, int row0)
      : v(make_view(a.x, a.bytes)), tid(tid_), tbl(nullptr), kbase(0), klast(0) {
    rq = tid % QR;
    const int m = row0 + 4 * rq;
    const bool in = m < a.kh * a.kw * a.Cg;
    const TapCoord t = decode_tap(in ? m : 0, a);
    tapoff = (((uint32_t)t.r * (uint32_t)a.W + (uint32_t)t.s) * (uint32_t)a.Ctot + (uint32_t)t.c +
              (uint32_t)(grp * a.c_stride_g)) * 4u;
    tapmask = in ? 1u << (t.r * a.kw + t.s) : 0x80000000u;
  }
  // all threads of the workgroup: entries of pixels kbeg .. kend-1; a barrier must follow
  static AX_HD void build_table(const Params& g, PixelEntry* table, int kbeg, int kend, int tid) {
    for (int e = tid; e < kend - kbeg; e += kThreads) {
      const PixCoord c = decode_pixel(kbeg + e, g);
      const int y0 = c.y * g.stride - g.pad, x0 = c.x * g.stride_x - g.pad_x;
      uint32_t inside = 0;
      int bit = 0;
      for (int r = 0; r < g.kh; ++r)
        for (int s2 = 0; s2 < g.kw; ++s2, ++bit)
          inside |= ((uint32_t)(y0 + r) < (uint32_t)g.H && (uint32_t)(x0 + s2) < (uint32_t)g.W ? 1u : 0u) << bit;
      PixelEntry pe;
      pe.base = row_base<IM2COL_FWD>(g, c.n, y0, x0, 0);
      pe.outside = ~inside | 0x80000000u;
      table[e] = pe;
    }
  }
  AX_HD void set_table(const PixelEntry* table, int kbeg, int kend) {
    tbl = table;
    kbase = kbeg;
    klast = kend - BK;
  }
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    const int kc = k0 < kend ? k0 : klast;  // uniform
    const PixelEntry pe = tbl[kc - kbase + (tid + S * kThreads) / QR];
    pl.off[S] = (pe.outside & tapmask) ? kOob : pe.base + tapoff;
  }
  AX_HD void fetch(float4* r) const { pl.fetch(v, r); }
  AX_HD void store_step(int s, float* lds, const float4* r) const {
    *reinterpret_cast<float4*>(lds + ((tid + s * kThreads) / QR) * LD + 4 * rq) = r[s];
  }
};
template <class L, class = void>
struct uses_table : std::false_type {};
template <class L>
struct uses_table<L, std::void_t<decltype(L::kUsesTable)>> : std::true_type {};

// Whole-tile helpers (prologue of the kernel, CPU emulation).
template <class L, int S = 0>
AX_HD void plan_all(L& l, int k0, int kend) {
  if constexpr (S < L::NA) {
    l.template addr_step<S>(k0, kend);
    plan_all<L, S + 1>(l, k0, kend);
  }
}
template <class L>
AX_HD void store_all(const L& l, float* lds, const float4* r) {
#pragma unroll
  for (int s = 0; s < L::NL; ++s) l.store_step(s, lds, r);
}
// element (row, k) of an LDS tile written by loader L
template <class L>
AX_HD int lds_index(int row, int k) {
  return L::kRowMajor ? row * L::LD + k : k * L::LD + row;
}

// ---- bf16 packing (round to nearest even) -----------------------------------------
#if defined(__HIP_DEVICE_COMPILE__)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
  bf2 v;
  v[0] = (__bf16)lo;
  v[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}
#else
inline uint32_t bf16_bits(float f) {  // finite inputs
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
inline uint32_t pack_bf16(float lo, float hi) { return bf16_bits(lo) | (bf16_bits(hi) << 16); }
#endif
// one bf16 / four consecutive bf16 (8-byte aligned) of a copy that shadows an fp32 tensor
AX_HD void store_bf16(uint16_t* p, float v) { *p = (uint16_t)(pack_bf16(v, 0.f) & 0xffffu); }
AX_HD void store_bf16x4(uint16_t* p, const float4& v) {
  uint32_t* q = reinterpret_cast<uint32_t*>(p);
#if defined(__HIP_DEVICE_COMPILE__)
  typedef uint32_t v2u __attribute__((ext_vector_type(2)));
  v2u w;
  w[0] = pack_bf16(v.x, v.y);
  w[1] = pack_bf16(v.z, v.w);
  *reinterpret_cast<v2u*>(q) = w;
#else
  q[0] = pack_bf16(v.x, v.y);
  q[1] = pack_bf16(v.z, v.w);
#endif
}

// ================================ epilogues ==================================
// kTransposed selects how a lane's accumulators map to the tile (see Tile::acc_row):
//  * true: apply4(m, n, v) is called for four consecutive valid columns n .. n+3 (n a multiple of 4) of row m
//    (apply(m, n, v) for the elements of a ragged last quad): a quarter of the store instructions, each
//    touching 32 rows.  Measured 3-4 % faster per launch where the tile is written once to its final place.
//  * false: apply(m, n, v) per element, 32 consecutive columns of one row per store instruction (whole
//    128-byte lines).  Measured 7-13 % faster for the split-k slabs and weight gradients, which are
//    short reductions with large outputs.
// set_group() runs once per workgroup and also decides whether quads may be stored 16 bytes at a time.
AX_HD bool epi_aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// y[m][col_off + n] = act(v + bias[col_off + n]); col_off = group * cols_per_group
struct EpiBiasAct {
  static constexpr bool kTransposed = true;
  float* y;
  long ldc;
  const float* bias;  // may be null
  int relu, cols_per_group, col_off;
  int vec;
  uint16_t* y16;  // may be null: a bf16 copy of y (same layout), for the product that reads y next
  AX_HD void set_group(int g, int /*z*/) {
    col_off = g * cols_per_group;
    vec = (ldc & 3) == 0 && (col_off & 3) == 0 && epi_aligned16(y) && epi_aligned16(bias) &&
          (((uintptr_t)y16 & 7) == 0);
  }
  AX_HD void apply(int m, int n, float v) const {
    if (bias) v += bias[col_off + n];
    if (relu) v = v > 0.f ? v : 0.f;
    y[(long)m * ldc + col_off + n] = v;
    if (y16) store_bf16(y16 + (long)m * ldc + col_off + n, v);
  }
  AX_HD void apply4(int m, int n, float4 v) const {
    if (!vec) {
      apply(m, n, v.x); apply(m, n + 1, v.y); apply(m, n + 2, v.z); apply(m, n + 3, v.w);
      return;
    }
    if (bias) {
      const float4 b = *reinterpret_cast<const float4*>(bias + col_off + n);
      v.x += b.x; v.y += b.y; v.z += b.z; v.w += b.w;
    }
    if (relu) {
      v.x = v.x > 0.f ? v.x : 0.f; v.y = v.y > 0.f ? v.y : 0.f;
      v.z = v.z > 0.f ? v.z : 0.f; v.w = v.w > 0.f ? v.w : 0.f;
    }
    *reinterpret_cast<float4*>(y + (long)m * ldc + col_off + n) = v;
    if (y16) store_bf16x4(y16 + (long)m * ldc + col_off + n, v);
  }
};

// dx[m][col_off + n] = gate ? (gate[m][col_off+n] > 0 ? v : 0) : v
struct EpiGate {
  static constexpr bool kTransposed = true;
  float* dx;
  long ldc;
  const float* gate;  // forward activation with the layout of dx, or null
  int cols_per_group, col_off;
  int vec;
  uint16_t* dx16;  // may be null: a bf16 copy of dx (same layout), for the products that read dx next
  AX_HD void set_group(int g, int /*z*/) {
    col_off = g * cols_per_group;
    vec = (ldc & 3) == 0 && (col_off & 3) == 0 && epi_aligned16(dx) && epi_aligned16(gate) &&
          (((uintptr_t)dx16 & 7) == 0);
  }
  AX_HD void apply(int m, int n, float v) const {
    const long o = (long)m * ldc + col_off + n;
    if (gate && !(gate[o] > 0.f)) v = 0.f;
    dx[o] = v;
    if (dx16) store_bf16(dx16 + o, v);
  }
  AX_HD void apply4(int m, int n, float4 v) const {
    if (!vec) {
      apply(m, n, v.x); apply(m, n + 1, v.y); apply(m, n + 2, v.z); apply(m, n + 3, v.w);
      return;
    }
    const long o = (long)m * ldc + col_off + n;
    if (gate) {
      const float4 q = *reinterpret_cast<const float4*>(gate + o);
      if (!(q.x > 0.f)) v.x = 0.f;
      if (!(q.y > 0.f)) v.y = 0.f;
      if (!(q.z > 0.f)) v.z = 0.f;
      if (!(q.w > 0.f)) v.w = 0.f;
    }
    *reinterpret_cast<float4*>(dx + o) = v;
    if (dx16) store_bf16x4(dx16 + o, v);
  }
};

// Depth-to-space store of a strided backward-data pass computed per phase:
// row m = (n, qy, qx) on the coarse grid, column = (py, px, c);
// dx[n][st*qy + py - pad][st*qx + px - pad][c] = v where that lies inside the picture.
struct EpiPhases {
  static constexpr bool kTransposed = false;
  float* dx;
  int H, W, C, st, pad, QW;
  FastDiv d_qhw, d_qw, d_stc, d_c;  // divisors QH*QW, QW, st*C, C
  AX_HD void set_group(int /*g*/, int /*z*/) {}
  AX_HD void apply4(int m, int n, float4 v) const {  // neighbouring columns may land in different pixels
    apply(m, n, v.x); apply(m, n + 1, v.y); apply(m, n + 2, v.z); apply(m, n + 3, v.w);
  }
  AX_HD void apply(int m, int n, float v) const {
    const int img = (int)fdiv((uint32_t)m, d_qhw);
    const int rem = m - img * (int)d_qhw.d;
    const int qy = (int)fdiv((uint32_t)rem, d_qw), qx = rem - qy * QW;
    const int py = (int)fdiv((uint32_t)n, d_stc), r2 = n - py * (int)d_stc.d;
    const int px = (int)fdiv((uint32_t)r2, d_c), c = r2 - px * C;
    const int iy = st * qy + py - pad, ix = st * qx + px - pad;
    if ((uint32_t)iy < (uint32_t)H && (uint32_t)ix < (uint32_t)W) dx[(((long)img * H + iy) * W + ix) * C + c] = v;
  }
};

// ws[z][m][n] = v   (z = group*nsplit + split); one M x N slab per launch slice
struct EpiSlab {
  static constexpr bool kTransposed = false;
  float* ws;
  long slab;  // M*N
  long ldc;   // N
  float* base;
  int vec;
  AX_HD void set_group(int /*g*/, int z) {
    base = ws + (long)z * slab;
    vec = (ldc & 3) == 0 && epi_aligned16(base);
  }
  AX_HD void apply(int m, int n, float v) const { base[(long)m * ldc + n] = v; }
  AX_HD void apply4(int m, int n, float4 v) const {
    if (vec) {
      *reinterpret_cast<float4*>(base + (long)m * ldc + n) = v;
    } else {
      apply(m, n, v.x); apply(m, n + 1, v.y); apply(m, n + 2, v.z); apply(m, n + 3, v.w);
    }
  }
};

// Hands one accumulator block of a lane to the epilogue: row m, register quads at columns nb + acc_row(lane, 4q).
template <class T, class Epi, class Acc>
AX_HD void store_block(const Epi& ep, const Acc& acc, int m, int nb, int lane, int M, int N) {
  if (m >= M) return;
#pragma unroll
  for (int q = 0; q < T::NACC / 4; ++q) {
    const int n = nb + T::acc_row(lane, 4 * q);
    if (n + 3 < N) {
      float4 v;
      v.x = acc[4 * q]; v.y = acc[4 * q + 1]; v.z = acc[4 * q + 2]; v.w = acc[4 * q + 3];
      ep.apply4(m, n, v);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (n + e < N) ep.apply(m, n + e, acc[4 * q + e]);
    }
  }
}

// ================================= kernel ====================================
#ifndef AX_HOST_EMU
typedef float v16f __attribute__((ext_vector_type(16)));

// Fragments of one operand for a wave: TT blocks of T::RB rows starting at LDS row `row`.
// [row][k] tiles give a lane its values of four MFMA steps in one 16-byte read;
// [k][row] tiles are read 4 bytes at a time.  Everything is fetched one MFMA step ahead of its use,
// and the first values of a tile (start) during the last step of the tile before.
template <class L, int TT, class T>
struct Frags {
  static constexpr int NQ = T::BK / (4 * T::G);
  static_assert(((T::KP - 1) >> 2) >= 1, "the last step of a tile must not use the registers that start() refills");
  float4 rk[L::kRowMajor ? TT : 1][L::kRowMajor ? NQ : 1];
  float kr[2][TT];
  const float* base;
  int g;
  __device__ __forceinline__ void start(const float* lds, int row, int g_) {
    g = g_;
    if (L::kRowMajor) {
      base = lds + row * L::LD + 4 * g;
      quad<0>();
    } else {
      base = lds + row;
      column<0>();
    }
  }
  template <int Q>
  __device__ __forceinline__ void quad() {
#pragma unroll
    for (int t = 0; t < TT; ++t)
      rk[t][Q] = *reinterpret_cast<const float4*>(base + t * T::RB * L::LD + 4 * T::G * Q);
  }
  template <int U>
  __device__ __forceinline__ void column() {
    const int k = T::step_k(U, g);
#pragma unroll
    for (int t = 0; t < TT; ++t) kr[U & 1][t] = base[k * L::LD + t * T::RB];
  }
  template <int U>
  __device__ __forceinline__ void read() {  // values of MFMA step U >= 1
    if (!L::kRowMajor) {
      column<U>();
    } else if (U % 4 == 0) {
      quad<U / 4>();
    }
  }
  template <int U>
  __device__ __forceinline__ float get(int t) const {
    if (L::kRowMajor) {
      const float4& v = rk[t][U >> 2];
      return (U & 3) == 0 ? v.x : (U & 3) == 1 ? v.y : (U & 3) == 2 ? v.z : v.w;
    }
    return kr[U & 1][t];
  }
};

typedef float v4f __attribute__((ext_vector_type(4)));
template <int RB>
struct MfmaBlock;
template <>
struct MfmaBlock<32> {
  typedef v16f Acc;
  static __device__ __forceinline__ Acc mma(float a, float b, Acc c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
  }
};
template <>
struct MfmaBlock<16> {
  typedef v4f Acc;
  static __device__ __forceinline__ Acc mma(float a, float b, Acc c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
  }
};

// Side work of one main-loop iteration, in this order: addresses of tile t+3, then the LDS stores of
// tile t+1 (as late as possible: its loads were issued almost two iterations earlier).
template <class T, class AL, class BL, int IDX>
__device__ __forceinline__ void side_step(AL& al, BL& bl, float* as_next, float* bs_next, const float4* ra,
                                          const float4* rb, int k_plan, int kend) {
  constexpr int S0 = AL::NA, S1 = S0 + BL::NA, S2 = S1 + AL::NL, S3 = S2 + BL::NL;
  if constexpr (IDX < 0) {
  } else if constexpr (IDX < S0) {
    al.template addr_step<IDX>(k_plan, kend);
  } else if constexpr (IDX < S1) {
    bl.template addr_step<IDX - S0>(k_plan, kend);
  } else if constexpr (IDX < S2) {
    al.store_step(IDX - S1, as_next, ra);
  } else if constexpr (IDX < S3) {
    bl.store_step(IDX - S2, bs_next, rb);
  }
}
// The side steps are dealt over the MFMA steps 0 .. KP-2, ending in step KP-2 (step KP-1 follows the barrier).
template <class T, class AL, class BL, int U, int W = 0>
__device__ __forceinline__ void side_slot(AL& al, BL& bl, float* as_next, float* bs_next, const float4* ra,
                                          const float4* rb, int k_plan, int kend) {
  constexpr int TOTAL = AL::NL + BL::NL + AL::NA + BL::NA, SLOTS = T::KP - 1, PER = (TOTAL + SLOTS - 1) / SLOTS,
                PAD = SLOTS * PER - TOTAL;
  if constexpr (W < PER) {
    side_step<T, AL, BL, U * PER + W - PAD>(al, bl, as_next, bs_next, ra, rb, k_plan, kend);
    side_slot<T, AL, BL, U, W + 1>(al, bl, as_next, bs_next, ra, rb, k_plan, kend);
  }
}

// The MFMA steps of one k-tile.  Before the last step all waves meet: by then every wave has read the
// last values of this tile and stored its share of the next one, so the barrier also frees this tile's
// buffer; the first reads of the next tile run under the last step's MFMAs.
// TR: feed the B fragment first, so that the result blocks come out transposed (see Tile::acc_row).
template <class T, class AL, class BL, bool TR, int U = 0>
__device__ __forceinline__ void tile_stream(Frags<AL, T::TM, T>& fa, Frags<BL, T::TN, T>& fb,
                                            typename MfmaBlock<T::RB>::Acc (&acc)[T::TM][T::TN], AL& al, BL& bl,
                                            float* as_next, float* bs_next, const float4* ra, const float4* rb,
                                            int k_plan, int kend, int a_row, int b_row, int kh) {
  constexpr int KP = T::KP;
  if constexpr (U < KP) {
    if constexpr (U + 1 < KP) {
      fa.template read<U + 1>();
      fb.template read<U + 1>();
    } else {
      __syncthreads();
      fa.start(as_next, a_row, kh);
      fb.start(bs_next, b_row, kh);
    }
#pragma unroll
    for (int i = 0; i < T::TM; ++i)
#pragma unroll
      for (int j = 0; j < T::TN; ++j)
        acc[i][j] = TR ? MfmaBlock<T::RB>::mma(fb.template get<U>(j), fa.template get<U>(i), acc[i][j])
                       : MfmaBlock<T::RB>::mma(fa.template get<U>(i), fb.template get<U>(j), acc[i][j]);
    if constexpr (U + 1 < KP) side_slot<T, AL, BL, U>(al, bl, as_next, bs_next, ra, rb, k_plan, kend);
    __builtin_amdgcn_sched_barrier(0);
    tile_stream<T, AL, BL, TR, U + 1>(fa, fb, acc, al, bl, as_next, bs_next, ra, rb, k_plan, kend, a_row, b_row, kh);
  }
}

// Workgroups the compiler must fit on a CU.  Two co-resident workgroups that started together stay in
// step, and a pass over a short reduction (the first layer's 25 k-tiles, the 12 to 16 of the transformed
// 3x3 layers) spends a good part of a tile's life in its prologue and epilogue; a third workgroup per CU
// fills those gaps (measured: 1-4 % per launch).  Three need at most 168 registers per lane, which every
// variant reaches without spilling (the accumulators then live in ordinary registers) except the 128 x 128
// tile with 4-byte loads, which keeps two.
template <class L>
struct loads_scalars : std::false_type {};
template <int ROWS, int BK>
struct loads_scalars<DenseKInner<ROWS, BK, false>> : std::true_type {};
template <int ROWS, int BK>
struct loads_scalars<DenseRowInner<ROWS, BK, false>> : std::true_type {};
template <int ROWS, int BK, int MODE>
struct loads_scalars<Im2colKInner<ROWS, BK, false, MODE>> : std::true_type {};
template <int ROWS, int BK>
struct loads_scalars<Im2colRowInner<ROWS, BK, false>> : std::true_type {};
template <class T, class AL, class BL>
struct MinBlocks {
  static constexpr int value =
      (T::BM * T::BN >= 128 * 128 && (loads_scalars<AL>::value || loads_scalars<BL>::value)) ? 2 : 3;
};

template <class T, class AL, class BL, class Epi>
__global__ void __launch_bounds__(kThreads, (MinBlocks<T, AL, BL>::value))
gemm_kernel(typename AL::Params ap, typename BL::Params bp, Epi ep, int M, int N, int K, int kchunk, int nsplit) {
  __shared__ __attribute__((aligned(16))) float As[2][AL::LDS_FLOATS];
  __shared__ __attribute__((aligned(16))) float Bs[2][BL::LDS_FLOATS];
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
  if constexpr (uses_table<AL>::value) {  // launched with (kend - kbeg) * sizeof(PixelEntry) bytes of dynamic LDS
    extern __shared__ __attribute__((aligned(16))) PixelEntry pixel_table[];
    AL::build_table(ap, pixel_table, kbeg, kend, tid);
    al.set_table(pixel_table, kbeg, kend);
    __syncthreads();
  }

  typename MfmaBlock<T::RB>::Acc acc[T::TM][T::TN];
#pragma unroll
  for (int i = 0; i < T::TM; ++i)
#pragma unroll
    for (int j = 0; j < T::TN; ++j)
#pragma unroll
      for (int r = 0; r < T::NACC; ++r) acc[i][j][r] = 0.f;

  constexpr int RB = T::RB;
  const int a_row = wm * (T::TM * RB) + lane % RB, b_row = wn * (T::TN * RB) + lane % RB, kh = lane / RB;
  if (nt > 0) {
    // prologue: tile 0 -> LDS buffer 0, tile 1 in flight in register set 1, addresses of tile 2 ready.
    // Tiles past the end are fetched and stored like any other but never multiplied: their loads return
    // zeros (every offset outside) or, with the whole-tile loaders, repeat the last tile.
    float4 ra[2][AL::NL], rb[2][BL::NL];
    plan_all(al, kbeg, kend);
    plan_all(bl, kbeg, kend);
    al.fetch(ra[0]);
    bl.fetch(rb[0]);
    plan_all(al, kbeg + T::BK, kend);
    plan_all(bl, kbeg + T::BK, kend);
    al.fetch(ra[1]);
    bl.fetch(rb[1]);
    store_all(al, As[0], ra[0]);
    store_all(bl, Bs[0], rb[0]);
    plan_all(al, kbeg + 2 * T::BK, kend);
    plan_all(bl, kbeg + 2 * T::BK, kend);
    __syncthreads();
    Frags<AL, T::TM, T> fa;
    Frags<BL, T::TN, T> fb;
    fa.start(As[0], a_row, kh);
    fb.start(Bs[0], b_row, kh);
    // iteration t (parity p): fetch tile t+2 into register set p, MFMAs of tile t from LDS buffer p,
    // meanwhile address tile t+3 and store register set p^1 (tile t+1) to LDS buffer p^1.
    for (int t = 0; t < nt; t += 2) {
      al.fetch(ra[0]);
      bl.fetch(rb[0]);
      __builtin_amdgcn_sched_barrier(0);
      tile_stream<T, AL, BL, Epi::kTransposed>(fa, fb, acc, al, bl, As[1], Bs[1], ra[1], rb[1], kbeg + (t + 3) * T::BK, kend, a_row,
                             b_row, kh);
      if (t + 1 < nt) {
        al.fetch(ra[1]);
        bl.fetch(rb[1]);
        __builtin_amdgcn_sched_barrier(0);
        tile_stream<T, AL, BL, Epi::kTransposed>(fa, fb, acc, al, bl, As[0], Bs[0], ra[0], rb[0], kbeg + (t + 4) * T::BK, kend, a_row,
                               b_row, kh);
      }
    }
  }

#pragma unroll
  for (int i = 0; i < T::TM; ++i)
#pragma unroll
    for (int j = 0; j < T::TN; ++j) {
      if constexpr (Epi::kTransposed) {
        store_block<T>(ep, acc[i][j], m0 + wm * (T::TM * RB) + i * RB + lane % RB, n0 + wn * (T::TN * RB) + j * RB,
                       lane, M, N);
      } else {
        const int n = n0 + wn * (T::TN * RB) + j * RB + lane % RB;
        if (n >= N) continue;
#pragma unroll
        for (int r = 0; r < T::NACC; ++r) {
          const int m = m0 + wm * (T::TM * RB) + i * RB + T::acc_row(lane, r);
          if (m < M) ep.apply(m, n, acc[i][j][r]);
        }
      }
    }
}
#endif  // AX_HOST_EMU

}  // namespace ax
