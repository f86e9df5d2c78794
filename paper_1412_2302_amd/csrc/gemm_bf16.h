// bf16 MFMA variant of the GEMM core (gemm.h): operands are fetched as fp32 and
// rounded to bf16 (round to nearest even, v_cvt_pk_bf16_f32) on their way into
// LDS, or fetched from tensors that already hold bf16 (the "16" loaders at the
// end), multiplied with v_mfma_f32_32x32x16_bf16 and accumulated in fp32.
// Addressing, zero fill, split-k and epilogues are those of the fp32 core.
//
// LDS layouts (32-bit words holding two bf16, even k in the low half):
//   k-contiguous operands   [row][k/2]   one 8-byte store per load; a lane reads
//                                        its 8 values of a 16-deep MFMA step as 16 bytes
//   row-contiguous operands [k/2][row]   a thread fetches k and k+1 of its four rows
//                                        and stores one 16-byte row of (k,k+1) pairs;
//                                        a lane reads its 8 values as four words
// One MFMA step covers k = 16*ks + 8*kh + e (kh = lane/32, e = 0..7) on both operands.
#pragma once

#include <string.h>

#include "gemm.h"

namespace ax {

// LDS word that holds elements (k, k+1), k even, of `row` in a tile written by loader L
template <class L>
AX_HD int bf_word(int row, int k) {
  return L::kRowMajor ? row * L::LDW + (k >> 1) : (k >> 1) * L::LDW + row;
}

// LDS word that holds values 2w and 2w+1 of the 8 that the lane of (row, kh) feeds to MFMA step ks
template <class L>
AX_HD int bf_frag_word(int row, int ks, int kh, int w) {
  return L::kRowMajor ? row * L::LDW + 8 * ks + 4 * kh + w : (8 * ks + 4 * kh + w) * L::LDW + row;
}

// ---- k-contiguous operands: reuse the fp32 loader's addressing -------------------
template <class L, int ROWS, int BK>
struct BfRowMajor : L {
  using L::L;
  static constexpr bool kRowMajor = true;
  static constexpr int LDW = BK / 2 + 4, LDS_WORDS = ROWS * LDW, NS = L::NL;
  AX_HD void store_step(int s, uint32_t* lds, const float4* r) const {
    uint32_t* d = lds + ((this->tid + s * kThreads) / L::QK) * LDW + 2 * this->kq;
    d[0] = pack_bf16(r[s].x, r[s].y);
    d[1] = pack_bf16(r[s].z, r[s].w);
  }
};

// ---- row-contiguous operands: a unit = rows 4*rq..4*rq+3 at k = 2*kp and 2*kp+1 ----
template <int ROWS, int BK>
struct BfDenseRowInner {
  static constexpr int QR = ROWS / 4, NU = QR * (BK / 2), NUT = NU / kThreads, NL = 2 * NUT, NA = NL, NS = NUT;
  static_assert(NU % kThreads == 0, "tile must be a whole number of units per thread");
  static constexpr bool kRowMajor = false;
  static constexpr int LDW = ROWS + 4, LDS_WORDS = (BK / 2) * LDW;
  typedef DenseParams Params;
  BufView v;
  int tid;
  uint32_t ld4;
  uint32_t base[NL];  // byte offset of (k local, row), or kOob
  Offsets<NL, true> pl;
  AX_HD BfDenseRowInner(const Params& a, int g, int tid_, int row0)
      : v(make_view(a.p + (long)g * a.gstride, a.bytes - (uint32_t)(g * a.gstride * 4))), tid(tid_) {
    ld4 = (uint32_t)a.ld * 4u;
#pragma unroll
    for (int u = 0; u < NUT; ++u) {
      const int idx = tid + u * kThreads;
      const int row = row0 + 4 * (idx % QR), kp = idx / QR;
#pragma unroll
      for (int h = 0; h < 2; ++h)
        base[2 * u + h] = row < a.R ? (uint32_t)(2 * kp + h) * ld4 + (uint32_t)row * 4u : kOob;
    }
  }
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    const int k = k0 + 2 * ((tid + (S / 2) * kThreads) / QR) + (S & 1);
    pl.off[S] = k < kend ? base[S] + (uint32_t)k0 * ld4 : kOob;
  }
  AX_HD void fetch(float4* r) const { pl.fetch(v, r); }
  AX_HD void store_step(int u, uint32_t* lds, const float4* r) const {
    const int idx = tid + u * kThreads;
    uint32_t* d = lds + (idx / QR) * LDW + 4 * (idx % QR);
    const float4 a = r[2 * u], b = r[2 * u + 1];
    d[0] = pack_bf16(a.x, b.x);
    d[1] = pack_bf16(a.y, b.y);
    d[2] = pack_bf16(a.z, b.z);
    d[3] = pack_bf16(a.w, b.w);
  }
};

template <int ROWS, int BK>
struct BfIm2colRowInner {
  static constexpr int QR = ROWS / 4, NU = QR * (BK / 2), NUT = NU / kThreads, NL = 2 * NUT, NA = NL, NS = NUT;
  static_assert(NU % kThreads == 0 && kThreads % QR == 0, "every unit of a thread shares its row quad");
  static constexpr bool kRowMajor = false;
  static constexpr int LDW = ROWS + 4, LDS_WORDS = (BK / 2) * LDW;
  typedef Im2colParams Params;
  Im2colParams g;
  BufView v;
  int tid, rq, c_off;
  TapCoord tap;  // tap of the thread's four rows; r = 2*kFar for rows past the end
  Offsets<NL, true> pl;
  AX_HD BfIm2colRowInner(const Params& a, int grp, int tid_, int row0)
      : g(a), v(make_view(a.x, a.bytes)), tid(tid_), c_off(grp * a.c_stride_g) {
    rq = tid % QR;
    const int m = row0 + 4 * rq;
    const bool in = m < g.kh * g.kw * g.Cg;
    tap = decode_tap(in ? m : 0, g);
    if (!in) tap.r = 2 * kFar;
  }
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    const int p = k0 + 2 * ((tid + (S / 2) * kThreads) / QR) + (S & 1);
    const bool pok = p < kend;
    const PixCoord c = decode_pixel(pok ? p : 0, g);
    const int y0 = pok ? c.y * g.stride - g.pad : -kFar, x0 = c.x * g.stride_x - g.pad_x;
    const uint32_t rb = row_base<IM2COL_FWD>(g, c.n, pok ? y0 : 0, x0, c_off);
    pl.off[S] = tap_address<IM2COL_FWD>(g, rb, y0, x0, tap);
  }
  AX_HD void fetch(float4* r) const { pl.fetch(v, r); }
  AX_HD void store_step(int u, uint32_t* lds, const float4* r) const {
    uint32_t* d = lds + ((tid + u * kThreads) / QR) * LDW + 4 * rq;
    const float4 a = r[2 * u], b = r[2 * u + 1];
    d[0] = pack_bf16(a.x, b.x);
    d[1] = pack_bf16(a.y, b.y);
    d[2] = pack_bf16(a.z, b.z);
    d[3] = pack_bf16(a.w, b.w);
  }
};

// BfDenseRowInner for whole k-tiles (see DenseRowWhole): one add per address, k-tiles past the end clamped.
template <int ROWS, int BK>
struct BfDenseRowWhole : BfDenseRowInner<ROWS, BK> {
  typedef BfDenseRowInner<ROWS, BK> Base;
  using Base::Base;
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    const int kc = k0 < kend ? k0 : kend - BK;  // uniform
    this->pl.off[S] = this->base[S] + (uint32_t)kc * this->ld4;
  }
};

// BfIm2colRowInner through the workgroup's pixel table (see Im2colRowTable): whole k-tiles, at most 31 taps.
template <int ROWS, int BK>
struct BfIm2colRowTable {
  static constexpr int QR = ROWS / 4, NU = QR * (BK / 2), NUT = NU / kThreads, NL = 2 * NUT, NA = NL, NS = NUT;
  static_assert(NU % kThreads == 0 && kThreads % QR == 0, "every unit of a thread shares its row quad");
  static constexpr bool kRowMajor = false;
  static constexpr bool kUsesTable = true;
  static constexpr int LDW = ROWS + 4, LDS_WORDS = (BK / 2) * LDW;
  typedef Im2colParams Params;
  BufView v;
  int tid, rq;
  uint32_t tapoff, tapmask;
  const PixelEntry* tbl;
  int kbase, klast;
  Offsets<NL, true> pl;
  AX_HD BfIm2colRowTable(const Params& a, int grp, int tid_, int row0)
      : v(make_view(a.x, a.bytes)), tid(tid_), tbl(nullptr), kbase(0), klast(0) {
    rq = tid % QR;
    const int m = row0 + 4 * rq;
    const bool in = m < a.kh * a.kw * a.Cg;
    const TapCoord t = decode_tap(in ? m : 0, a);
    tapoff = (((uint32_t)t.r * (uint32_t)a.W + (uint32_t)t.s) * (uint32_t)a.Ctot + (uint32_t)t.c +
              (uint32_t)(grp * a.c_stride_g)) * 4u;
    tapmask = in ? 1u << (t.r * a.kw + t.s) : 0x80000000u;
  }
  static AX_HD void build_table(const Params& g, PixelEntry* table, int kbeg, int kend, int tid) {
    Im2colRowTable<ROWS, 16>::build_table(g, table, kbeg, kend, tid);
  }
  AX_HD void set_table(const PixelEntry* table, int kbeg, int kend) {
    tbl = table;
    kbase = kbeg;
    klast = kend - BK;
  }
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    const int kc = k0 < kend ? k0 : klast;  // uniform
    const PixelEntry pe = tbl[kc - kbase + 2 * ((tid + (S / 2) * kThreads) / QR) + (S & 1)];
    pl.off[S] = (pe.outside & tapmask) ? kOob : pe.base + tapoff;
  }
  AX_HD void fetch(float4* r) const { pl.fetch(v, r); }
  AX_HD void store_step(int u, uint32_t* lds, const float4* r) const {
    uint32_t* d = lds + ((tid + u * kThreads) / QR) * LDW + 4 * rq;
    const float4 a = r[2 * u], b = r[2 * u + 1];
    d[0] = pack_bf16(a.x, b.x);
    d[1] = pack_bf16(a.y, b.y);
    d[2] = pack_bf16(a.z, b.z);
    d[3] = pack_bf16(a.w, b.w);
  }
};

// ======================= operands stored as bf16 in memory ==========================
// The loaders above fetch fp32 and round on the way into LDS: twice the bytes through L1 and a conversion per
// pair of values.  The ones below read tensors that already hold bf16 (nearest-even copies made by
// to_bf16 or by the producing kernel): a 16-byte load brings eight consecutive elements, byte offsets count
// 2-byte elements, and no arithmetic touches the values on their way to LDS.  Same LDS layouts as above, so the
// kernel and its fragment reads do not change.  All of them need extents that are multiples of 8 elements
// (channels per group, total channels, rows) and 16-byte aligned tensors; the launcher checks that.

// word j of the (k, k+1) pairs of eight rows: a = rows r..r+7 at k, b = the same rows at k+1
AX_HD uint32_t bf_pair_lo(uint32_t a, uint32_t b) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_perm(b, a, 0x05040100u);
#else
  return (a & 0xffffu) | (b << 16);
#endif
}
AX_HD uint32_t bf_pair_hi(uint32_t a, uint32_t b) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_perm(b, a, 0x07060302u);
#else
  return (a >> 16) | (b & 0xffff0000u);
#endif
}
AX_HD uint32_t f_bits(float f) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __float_as_uint(f);
#else
  uint32_t u;
  memcpy(&u, &f, 4);
  return u;
#endif
}
// rows r..r+7 at k (a) and k+1 (b), eight bf16 each -> eight words of (k, k+1) pairs at d[0..7]
AX_HD void bf_store_pairs(uint32_t* d, const float4& a, const float4& b) {
  const uint32_t a0 = f_bits(a.x), a1 = f_bits(a.y), a2 = f_bits(a.z), a3 = f_bits(a.w);
  const uint32_t b0 = f_bits(b.x), b1 = f_bits(b.y), b2 = f_bits(b.z), b3 = f_bits(b.w);
#if defined(__HIP_DEVICE_COMPILE__)
  typedef uint32_t v4u __attribute__((ext_vector_type(4)));
  v4u lo, hi;
  lo[0] = bf_pair_lo(a0, b0); lo[1] = bf_pair_hi(a0, b0); lo[2] = bf_pair_lo(a1, b1); lo[3] = bf_pair_hi(a1, b1);
  hi[0] = bf_pair_lo(a2, b2); hi[1] = bf_pair_hi(a2, b2); hi[2] = bf_pair_lo(a3, b3); hi[3] = bf_pair_hi(a3, b3);
  *reinterpret_cast<v4u*>(d) = lo;  // two 16-byte LDS stores
  *reinterpret_cast<v4u*>(d + 4) = hi;
#else
  d[0] = bf_pair_lo(a0, b0); d[1] = bf_pair_hi(a0, b0); d[2] = bf_pair_lo(a1, b1); d[3] = bf_pair_hi(a1, b1);
  d[4] = bf_pair_lo(a2, b2); d[5] = bf_pair_hi(a2, b2); d[6] = bf_pair_lo(a3, b3); d[7] = bf_pair_hi(a3, b3);
#endif
}

// k-contiguous implicit im2col (rows = pixels, k = (r,s,c)) over a bf16 tensor: a load is eight consecutive
// channels of one tap.  General taps, k tails zero-filled (K and the split chunk are multiples of 8).
template <int ROWS, int BK, int MODE>
struct Im2colKInner16 {
  static constexpr int QK = BK / 8, NQ = ROWS * QK, NL = NQ / kThreads, NA = NL + 1, NS = NL;
  static constexpr bool kRowMajor = true;
  static constexpr int LDW = BK / 2 + 4, LDS_WORDS = ROWS * LDW;
  static_assert(kThreads % QK == 0 && NQ % kThreads == 0 && NL >= 1, "every load of a thread shares its k octet");
  typedef Im2colParams Params;
  Im2colParams g;
  BufView v;
  int tid, kq;
  uint32_t rowbase[NL];
  int y0[NL], x0[NL];
  TapCoord tap;
  Offsets<NL, true> pl;
  AX_HD Im2colKInner16(const Params& a, int grp, int tid_, int row0) : g(a), v(make_view(a.x, a.bytes)), tid(tid_) {
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
      rowbase[i] = row_base<MODE, 2>(g, c.n, in ? y0[i] : 0, x0[i], c_off);
    }
  }
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    if (S == 0) {
      const int k = k0 + 8 * kq;
      tap = decode_tap(k, g);
      if (k >= kend) tap.r = MODE == IM2COL_FWD ? 2 * kFar : -2 * kFar;
    } else {
      constexpr int i = S - 1;
      pl.off[i] = tap_address<MODE, 2>(g, rowbase[i], y0[i], x0[i], tap);
    }
  }
  AX_HD void fetch(float4* r) const { pl.fetch(v, r); }
  AX_HD void store_step(int s, uint32_t* lds, const float4* r) const {
    *reinterpret_cast<float4*>(lds + ((tid + s * kThreads) / QK) * LDW + 4 * kq) = r[s];
  }
};

// Im2colKInner16 for k-tiles that lie inside one tap (see Im2colKTap): channels per group a multiple of BK, at
// most 32 taps, modes 0 and 1; k-tiles past the end are clamped to the last one.
template <int ROWS, int BK, int MODE>
struct Im2colKTap16 {
  static constexpr int QK = BK / 8, NQ = ROWS * QK, NL = NQ / kThreads, NA = NL + 1, NS = NL;
  static constexpr bool kRowMajor = true;
  static constexpr int LDW = BK / 2 + 4, LDS_WORDS = ROWS * LDW;
  static_assert(kThreads % QK == 0 && NQ % kThreads == 0 && NL >= 1, "every load of a thread shares its k octet");
  static_assert(MODE == IM2COL_FWD || MODE == IM2COL_T1, "unit-step gathers only");
  typedef Im2colParams Params;
  Im2colParams g;
  BufView v;
  int tid, kq;
  uint32_t rowbase[NL];
  uint32_t outside[NL];
  uint32_t tapoff;
  int tapbit;
  Offsets<NL, true> pl;
  AX_HD Im2colKTap16(const Params& a, int grp, int tid_, int row0) : g(a), v(make_view(a.x, a.bytes)), tid(tid_) {
    kq = tid % QK;
    const int c_off = grp * a.c_stride_g + 8 * kq;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int p = row0 + (tid + i * kThreads) / QK;
      const bool in = p < g.P;
      const PixCoord c = decode_pixel(in ? p : 0, g);
      const int y0 = MODE == IM2COL_FWD ? c.y * g.stride - g.pad : c.y + g.pad;
      const int x0 = MODE == IM2COL_FWD ? c.x * g.stride_x - g.pad_x : c.x + g.pad;
      rowbase[i] = row_base<MODE, 2>(g, c.n, y0, x0, c_off);
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
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    if (S == 0) {
      const TapCoord t = decode_tap(k0 < kend ? k0 : kend - BK, g);
      const uint32_t tap = (((uint32_t)t.r * (uint32_t)g.W + (uint32_t)t.s) * (uint32_t)g.Ctot) * 2u;
      tapoff = (MODE == IM2COL_FWD ? tap : 0u - tap) + (uint32_t)t.c * 2u;
      tapbit = t.r * g.kw + t.s;
    } else {
      constexpr int i = S - 1;
      const uint32_t out = 0u - ((outside[i] >> tapbit) & 1u);
      pl.off[i] = (out & kOob) | (~out & (rowbase[i] + tapoff));
    }
  }
  AX_HD void fetch(float4* r) const { pl.fetch(v, r); }
  AX_HD void store_step(int s, uint32_t* lds, const float4* r) const {
    *reinterpret_cast<float4*>(lds + ((tid + s * kThreads) / QK) * LDW + 4 * kq) = r[s];
  }
};

// k-contiguous dense operand elem(row, k) = p[row*ld + k] stored as bf16 (dense-layer activations and weights)
template <int ROWS, int BK>
struct DenseKInner16 {
  static constexpr int QK = BK / 8, NQ = ROWS * QK, NL = (NQ + kThreads - 1) / kThreads, NA = NL, NS = NL;
  static constexpr bool kWhole = NQ % kThreads == 0;  // else some threads own no load in the last round (96 rows)
  static constexpr bool kRowMajor = true;
  static constexpr int LDW = BK / 2 + 4, LDS_WORDS = ROWS * LDW;
  static_assert(kThreads % QK == 0 && NL >= 1, "every load of a thread shares its k octet");
  typedef DenseParams Params;
  BufView v;
  int tid, kq;
  uint32_t base[NL];
  Offsets<NL, true> pl;
  AX_HD DenseKInner16(const Params& a, int g, int tid_, int row0)
      : v(make_view(reinterpret_cast<const float*>(reinterpret_cast<const uint16_t*>(a.p) + (long)g * a.gstride),
                    a.bytes - (uint32_t)(g * a.gstride * 2))),
        tid(tid_) {
    kq = tid % QK;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int idx = tid + i * kThreads, row = row0 + idx / QK;
      base[i] = (kWhole || idx < NQ) && row < a.R ? ((uint32_t)row * (uint32_t)a.ld + 8u * kq) * 2u : kOob;
    }
  }
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    pl.off[S] = k0 + 8 * kq < kend ? base[S] + (uint32_t)k0 * 2u : kOob;
  }
  AX_HD void fetch(float4* r) const { pl.fetch(v, r); }
  AX_HD void store_step(int s, uint32_t* lds, const float4* r) const {
    const int idx = tid + s * kThreads;
    if (kWhole || idx < NQ) *reinterpret_cast<float4*>(lds + (idx / QK) * LDW + 4 * kq) = r[s];
  }
};

// row-contiguous dense operand elem(row, k) = p[k*ld + row] stored as bf16 (packed weights, output gradients):
// a unit = rows 8*rq .. 8*rq+7 at k = 2*kp and 2*kp+1, two loads, interleaved into eight words of pairs
template <int ROWS, int BK>
struct DenseRowInner16 {
  static constexpr int QR = ROWS / 8, NU = QR * (BK / 2), NUT = (NU + kThreads - 1) / kThreads, NL = 2 * NUT, NA = NL,
                       NS = NUT;
  static constexpr bool kWhole = NU % kThreads == 0;  // else some threads own no unit in the last round
  static constexpr bool kRowMajor = false;
  static constexpr int LDW = ROWS + 4, LDS_WORDS = (BK / 2) * LDW;
  typedef DenseParams Params;
  BufView v;
  int tid;
  uint32_t ld2;       // leading dimension in bytes
  uint32_t base[NL];  // byte offset of (k local, row), or kOob
  Offsets<NL, true> pl;
  AX_HD DenseRowInner16(const Params& a, int g, int tid_, int row0)
      : v(make_view(reinterpret_cast<const float*>(reinterpret_cast<const uint16_t*>(a.p) + (long)g * a.gstride),
                    a.bytes - (uint32_t)(g * a.gstride * 2))),
        tid(tid_) {
    ld2 = (uint32_t)a.ld * 2u;
#pragma unroll
    for (int u = 0; u < NUT; ++u) {
      const int idx = tid + u * kThreads;
      const int row = row0 + 8 * (idx % QR), kp = idx / QR;
      const bool in = (kWhole || idx < NU) && row < a.R;
#pragma unroll
      for (int h = 0; h < 2; ++h) base[2 * u + h] = in ? (uint32_t)(2 * kp + h) * ld2 + (uint32_t)row * 2u : kOob;
    }
  }
  template <int S>
  AX_HD void addr_step(int k0, int kend) {
    const int k = k0 + 2 * ((tid + (S / 2) * kThreads) / QR) + (S & 1);
    // base may be kOob: adding less than 2^31 to it stays outside every operand
    pl.off[S] = k < kend ? base[S] + (uint32_t)k0 * ld2 : kOob;
  }
  AX_HD void fetch(float4* r) const { pl.fetch(v, r); }
  AX_HD void store_step(int u, uint32_t* lds, const float4* r) const {
    const int idx = tid + u * kThreads;
    if (kWhole || idx < NU) bf_store_pairs(lds + (idx / QR) * LDW + 8 * (idx % QR), r[2 * u], r[2 * u + 1]);
  }
};

// transpose of the implicit im2col (rows = (r,s,c), k = pixels: backward-weight) over a bf16 tensor, through the
// workgroup's pixel table (see Im2colRowTable): whole k-tiles, at most 31 taps; a unit = eight channels of one tap
// at two consecutive pixels
template <int ROWS, int BK>
struct Im2colRowTable16 {
  static constexpr int QR = ROWS / 8, NU = QR * (BK / 2), NUT = NU / kThreads, NL = 2 * NUT, NA = NL, NS = NUT;
  static_assert(NU % kThreads == 0 && kThreads % QR == 0 && NUT >= 1, "every unit of a thread shares its row octet");
  static constexpr bool kRowMajor = false;
  static constexpr bool kUsesTable = true;
  static constexpr int LDW = ROWS + 4, LDS_WORDS = (BK / 2) * LDW;
  typedef Im2colParams Params;
  BufView v;
  int tid, rq;
  uint32_t tapoff, tapmask;
  const PixelEntry* tbl;
  int kbase, klast;
  Offsets<NL, true> pl;
  AX_HD Im2colRowTable16(const Params& a, int grp, int tid_, int row0)
      : v(make_view(a.x, a.bytes)), tid(tid_), tbl(nullptr), kbase(0), klast(0) {
    rq = tid % QR;
    const int m = row0 + 8 * rq;
    const bool in = m < a.kh * a.kw * a.Cg;
    const TapCoord t = decode_tap(in ? m : 0, a);
    tapoff = (((uint32_t)t.r * (uint32_t)a.W + (uint32_t)t.s) * (uint32_t)a.Ctot + (uint32_t)t.c +
              (uint32_t)(grp * a.c_stride_g)) * 2u;
    tapmask = in ? 1u << (t.r * a.kw + t.s) : 0x80000000u;
  }
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
      pe.base = row_base<IM2COL_FWD, 2>(g, c.n, y0, x0, 0);
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
    const PixelEntry pe = tbl[kc - kbase + 2 * ((tid + (S / 2) * kThreads) / QR) + (S & 1)];
    pl.off[S] = (pe.outside & tapmask) ? kOob : pe.base + tapoff;
  }
  AX_HD void fetch(float4* r) const { pl.fetch(v, r); }
  AX_HD void store_step(int u, uint32_t* lds, const float4* r) const {
    bf_store_pairs(lds + ((tid + u * kThreads) / QR) * LDW + 8 * rq, r[2 * u], r[2 * u + 1]);
  }
};

template <class L>
AX_HD void bf_store_all(const L& l, uint32_t* lds, const float4* r) {
#pragma unroll
  for (int s = 0; s < L::NS; ++s) l.store_step(s, lds, r);
}

// ================================= kernel ====================================
#ifndef AX_HOST_EMU
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

template <class L, int TT>
struct BfFrags {
  v8bf f[TT];
  // the 8 values of MFMA step KS for each of the wave's TT row blocks
  template <int KS>
  __device__ __forceinline__ void read(const uint32_t* lds, int row, int kh) {
#pragma unroll
    for (int t = 0; t < TT; ++t) {
      typedef uint32_t v4u __attribute__((ext_vector_type(4)));
      v4u w;
      if (L::kRowMajor) {
        w = *reinterpret_cast<const v4u*>(lds + bf_frag_word<L>(row + 32 * t, KS, kh, 0));
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) w[q] = lds[bf_frag_word<L>(row + 32 * t, KS, kh, q)];
      }
      f[t] = __builtin_bit_cast(v8bf, w);
    }
  }
};

template <class T, class AL, class BL, int IDX>
__device__ __forceinline__ void bf_side_step(AL& al, BL& bl, uint32_t* as_next, uint32_t* bs_next, const float4* ra,
                                             const float4* rb, int k_plan, int kend) {
  constexpr int S0 = AL::NS, S1 = S0 + BL::NS, S2 = S1 + AL::NA, S3 = S2 + BL::NA;
  if constexpr (IDX < S0) {
    al.store_step(IDX, as_next, ra);
  } else if constexpr (IDX < S1) {
    bl.store_step(IDX - S0, bs_next, rb);
  } else if constexpr (IDX < S2) {
    al.template addr_step<IDX - S1>(k_plan, kend);
  } else if constexpr (IDX < S3) {
    bl.template addr_step<IDX - S2>(k_plan, kend);
  }
}
template <class T, class AL, class BL, int SLOT, int W = 0>
__device__ __forceinline__ void bf_side_slot(AL& al, BL& bl, uint32_t* as_next, uint32_t* bs_next, const float4* ra,
                                             const float4* rb, int k_plan, int kend) {
  constexpr int TOTAL = AL::NS + BL::NS + AL::NA + BL::NA, SLOTS = T::BK / 16, PER = (TOTAL + SLOTS - 1) / SLOTS;
  if constexpr (W < PER) {
    bf_side_step<T, AL, BL, SLOT * PER + W>(al, bl, as_next, bs_next, ra, rb, k_plan, kend);
    bf_side_slot<T, AL, BL, SLOT, W + 1>(al, bl, as_next, bs_next, ra, rb, k_plan, kend);
  }
}

template <class T, class AL, class BL, int KS = 0>
__device__ __forceinline__ void bf_tile_stream(const uint32_t* as, const uint32_t* bs, int a_row, int b_row, int kh,
                                               v16f (&acc)[T::TM][T::TN], AL& al, BL& bl, uint32_t* as_next,
                                               uint32_t* bs_next, const float4* ra, const float4* rb, int k_plan,
                                               int kend) {
  if constexpr (KS < T::BK / 16) {
    BfFrags<AL, T::TM> fa;
    BfFrags<BL, T::TN> fb;
    fa.template read<KS>(as, a_row, kh);
    fb.template read<KS>(bs, b_row, kh);
#pragma unroll
    for (int i = 0; i < T::TM; ++i)
#pragma unroll
      for (int j = 0; j < T::TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.f[i], fb.f[j], acc[i][j], 0, 0, 0);
    bf_side_slot<T, AL, BL, KS>(al, bl, as_next, bs_next, ra, rb, k_plan, kend);
    bf_tile_stream<T, AL, BL, KS + 1>(as, bs, a_row, b_row, kh, acc, al, bl, as_next, bs_next, ra, rb, k_plan, kend);
  }
}

// Output tile of a workgroup in a one-dimensional launch of gx * gy * gz workgroups.  The hardware hands
// workgroups to the eight XCDs round-robin (workgroup L runs on XCD L % 8, as the (L / 8)-th of that XCD), and
// each XCD has an L2 of its own.  These kernels are paced by memory, so the tiles are dealt such that the
// workgroups that follow each other on one XCD walk the column tiles of one row tile, then the next row tile,
// then the next group or k-slice: what they share (the rows' operand, read once per column tile) is then
// found in that XCD's L2 instead of being fetched again from memory by every column tile.
struct TileCoord {
  int x, y, z;
};
__device__ __forceinline__ TileCoord xcd_tile(int gx, int gy) {
  const int total = (int)gridDim.x, L = (int)blockIdx.x;
  const int q = total >> 3, r = total & 7, c = L & 7;
  const int t = c * q + min(c, r) + (L >> 3);  // XCD c owns tiles [c*q + min(c,r), +q + (c < r))
  const int rest = t / gy;
  TileCoord o;
  o.y = t - rest * gy;
  o.z = rest / gx;
  o.x = rest - o.z * gx;
  return o;
}

// two workgroups per CU at least (256 registers per lane, accumulators included): a lone workgroup has nobody to
// hide its barriers and its waits for memory behind
template <class T, class AL, class BL, class Epi>
__global__ void __launch_bounds__(kThreads, 2)
gemm_bf16_kernel(typename AL::Params ap, typename BL::Params bp, Epi ep, int M, int N, int K, int kchunk,
                 int nsplit, int gx, int gy) {
  __shared__ __attribute__((aligned(16))) uint32_t As[2][AL::LDS_WORDS];
  __shared__ __attribute__((aligned(16))) uint32_t Bs[2][BL::LDS_WORDS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % T::WAVES_M, wn = wave / T::WAVES_M;
  const TileCoord tc = xcd_tile(gx, gy);
  const int z = tc.z, g = z / nsplit, split = z - g * nsplit;
  const int m0 = tc.x * T::BM, n0 = tc.y * T::BN;
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

  v16f acc[T::TM][T::TN];
#pragma unroll
  for (int i = 0; i < T::TM; ++i)
#pragma unroll
    for (int j = 0; j < T::TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int a_row = wm * (T::TM * 32) + (lane & 31), b_row = wn * (T::TN * 32) + (lane & 31), kh = lane >> 5;
  if (nt > 0) {
    // same schedule as the fp32 kernel: tile t from LDS buffer t&1, tile t+1 on its way
    // from registers to the other buffer, tile t+2 being fetched, tile t+3 being addressed
    float4 ra[2][AL::NL], rb[2][BL::NL];
    plan_all(al, kbeg, kend);
    plan_all(bl, kbeg, kend);
    al.fetch(ra[0]);
    bl.fetch(rb[0]);
    plan_all(al, kbeg + T::BK, kend);
    plan_all(bl, kbeg + T::BK, kend);
    al.fetch(ra[1]);
    bl.fetch(rb[1]);
    bf_store_all(al, As[0], ra[0]);
    bf_store_all(bl, Bs[0], rb[0]);
    plan_all(al, kbeg + 2 * T::BK, kend);
    plan_all(bl, kbeg + 2 * T::BK, kend);
    __syncthreads();
    for (int t = 0; t < nt; t += 2) {
      al.fetch(ra[0]);
      bl.fetch(rb[0]);
      bf_tile_stream<T, AL, BL>(As[0], Bs[0], a_row, b_row, kh, acc, al, bl, As[1], Bs[1], ra[1], rb[1],
                                kbeg + (t + 3) * T::BK, kend);
      __syncthreads();
      if (t + 1 < nt) {
        al.fetch(ra[1]);
        bl.fetch(rb[1]);
        bf_tile_stream<T, AL, BL>(As[1], Bs[1], a_row, b_row, kh, acc, al, bl, As[0], Bs[0], ra[0], rb[0],
                                  kbeg + (t + 4) * T::BK, kend);
        __syncthreads();
      }
    }
  }

#pragma unroll
  for (int i = 0; i < T::TM; ++i)
#pragma unroll
    for (int j = 0; j < T::TN; ++j) {
      // Blocks are not transposed here (A fragment first): register r of a lane is C[acc_row(lane, r)][lane % 32].
      // These kernels wait on memory rather than on instruction issue, and 4-byte stores that fill whole
      // 128-byte lines measured faster than the fp32 kernel's 16-byte stores, which touch 32 lines each.
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
