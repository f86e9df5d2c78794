// CPU emulation of the workgroup programs in csrc/gemm.h and csrc/gemm_bf16.h.
//
// Runs the real operand loaders, LDS stores, fragment index maps and epilogues
// thread by thread on the host, with the MFMA replaced by its definition, and
// checks the three convolution GEMMs against direct loops.  Built with
// -fsanitize=address so that any out-of-range global or LDS access of a loader
// aborts here, on the CPU, before the kernel ever runs on a GPU.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <vector>

struct float4 {
  float x, y, z, w;
};
#define AX_HOST_EMU 1
#include "../../paper_1412_2302_amd/csrc/conv_plan.h"
namespace ax {
inline void emu_fail(const char* what) {
  fprintf(stderr, "EMULATION FAULT: %s\n", what);
  abort();
}
}  // namespace ax

#include "../../paper_1412_2302_amd/csrc/gemm_bf16.h"

using namespace ax;

template <class T, class AL, class BL, class Epi>
static void emu_gemm(typename AL::Params ap, typename BL::Params bp, Epi ep, int M, int N, int K, int kchunk,
                     int nsplit, int groups) {
  const int gx = (M + T::BM - 1) / T::BM, gy = (N + T::BN - 1) / T::BN, gz = groups * nsplit;
  std::vector<float> As(AL::LDS_FLOATS), Bs(BL::LDS_FLOATS);
  std::vector<float> acc((size_t)4 * T::TM * T::TN * 64 * 16);
  auto ACC = [&](int wave, int i, int j, int lane, int r) -> float& {
    return acc[((((size_t)wave * T::TM + i) * T::TN + j) * 64 + lane) * 16 + r];
  };
  for (int bz = 0; bz < gz; ++bz)
    for (int by = 0; by < gy; ++by)
      for (int bx = 0; bx < gx; ++bx) {
        const int g = bz / nsplit, split = bz - g * nsplit;
        const int m0 = bx * T::BM, n0 = by * T::BN;
        const int kbeg = split * kchunk, kend = std::min(K, kbeg + kchunk);
        const int nt = kend > kbeg ? (kend - kbeg + T::BK - 1) / T::BK : 0;
        std::fill(acc.begin(), acc.end(), 0.f);
        Epi e = ep;
        e.set_group(g, bz);
        for (int t = 0; t < nt; ++t) {
          // poison LDS so that a slot nobody wrote shows up
          std::fill(As.begin(), As.end(), NAN);
          std::fill(Bs.begin(), Bs.end(), NAN);
          // the workgroup's pixel table (loaders that use one): exactly as many entries as the kernel gets
          std::vector<PixelEntry> table;
          if constexpr (uses_table<AL>::value) {
            table.assign(kend - kbeg, PixelEntry{0xdeadbeefu, 0u});
            for (int tid = 0; tid < kThreads; ++tid) AL::build_table(ap, table.data(), kbeg, kend, tid);
          }
          for (int tid = 0; tid < kThreads; ++tid) {
            AL al(ap, g, tid, m0);
            BL bl(bp, g, tid, n0);
            if constexpr (uses_table<AL>::value) al.set_table(table.data(), kbeg, kend);
            float4 ra[AL::NL], rb[BL::NL];
            plan_all(al, kbeg + t * T::BK, kend);
            plan_all(bl, kbeg + t * T::BK, kend);
            al.fetch(ra);
            bl.fetch(rb);
            store_all(al, As.data(), ra);
            store_all(bl, Bs.data(), rb);
          }
          for (int wave = 0; wave < 4; ++wave) {
            const int wm = wave % T::WAVES_M, wn = wave / T::WAVES_M;
            constexpr int RB = T::RB, G = T::G;
            for (int kk = 0; kk < T::KP; ++kk) {
              float a[64][T::TM], b[64][T::TN];
              for (int lane = 0; lane < 64; ++lane) {
                const int kr = T::step_k(kk, lane / RB);
                for (int i = 0; i < T::TM; ++i) a[lane][i] = As[lds_index<AL>(wm * (T::TM * RB) + lane % RB + i * RB, kr)];
                for (int j = 0; j < T::TN; ++j) b[lane][j] = Bs[lds_index<BL>(wn * (T::TN * RB) + lane % RB + j * RB, kr)];
              }
              // one MFMA: D[ii][jj] += sum over g < G of X[ii][g] * Y[g][jj]; lane g*RB+ii holds X[ii][g],
              // lane g*RB+jj holds Y[g][jj]; register r of lane l is D[acc_row(l, r)][l % RB].  For an epilogue
              // with kTransposed the kernel passes the B fragment as X and the A fragment as Y, so D is the
              // block of C transposed; otherwise X = A, Y = B.
              for (int i = 0; i < T::TM; ++i)
                for (int j = 0; j < T::TN; ++j)
                  for (int lane = 0; lane < 64; ++lane)
                    for (int r = 0; r < T::NACC; ++r) {
                      const int ii = T::acc_row(lane, r), jj = lane % RB;
                      float s = 0.f;
                      for (int k2 = 0; k2 < G; ++k2)
                        s += Epi::kTransposed ? b[k2 * RB + ii][j] * a[k2 * RB + jj][i]
                                              : a[k2 * RB + ii][i] * b[k2 * RB + jj][j];
                      ACC(wave, i, j, lane, r) += s;
                    }
            }
          }
        }
        for (int wave = 0; wave < 4; ++wave) {
          const int wm = wave % T::WAVES_M, wn = wave / T::WAVES_M;
          constexpr int RB = T::RB;
          for (int lane = 0; lane < 64; ++lane)
            for (int i = 0; i < T::TM; ++i)
              for (int j = 0; j < T::TN; ++j) {
                if (Epi::kTransposed) {
                  store_block<T>(e, &ACC(wave, i, j, lane, 0), m0 + wm * (T::TM * RB) + i * RB + lane % RB,
                                 n0 + wn * (T::TN * RB) + j * RB, lane, M, N);
                  continue;
                }
                const int n = n0 + wn * (T::TN * RB) + j * RB + lane % RB;
                if (n >= N) continue;
                for (int r = 0; r < T::NACC; ++r) {
                  const int m = m0 + wm * (T::TM * RB) + i * RB + T::acc_row(lane, r);
                  if (m < M) e.apply(m, n, ACC(wave, i, j, lane, r));
                }
              }
        }
      }
}

static float bf_value(uint32_t word, int half) {
  const uint32_t u = (half ? word >> 16 : word & 0xffffu) << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

// The bf16 workgroup program: same loaders' addressing, packed LDS words, and the
// 32x32x16 MFMA by its definition: the lane of (row, kh) supplies 8 values of k-block kh,
// D[i][j] += sum over kh < 2, e < 8 of A[i][kh][e] * B[j][kh][e].
template <class T, class AL, class BL, class Epi>
static void emu_gemm_bf(typename AL::Params ap, typename BL::Params bp, Epi ep, int M, int N, int K, int kchunk,
                        int nsplit, int groups) {
  const int gx = (M + T::BM - 1) / T::BM, gy = (N + T::BN - 1) / T::BN, gz = groups * nsplit;
  std::vector<uint32_t> As(AL::LDS_WORDS), Bs(BL::LDS_WORDS);
  std::vector<float> acc((size_t)T::BM * T::BN);
  for (int bz = 0; bz < gz; ++bz)
    for (int by = 0; by < gy; ++by)
      for (int bx = 0; bx < gx; ++bx) {
        const int g = bz / nsplit, split = bz - g * nsplit;
        const int m0 = bx * T::BM, n0 = by * T::BN;
        const int kbeg = split * kchunk, kend = std::min(K, kbeg + kchunk);
        const int nt = kend > kbeg ? (kend - kbeg + T::BK - 1) / T::BK : 0;
        std::fill(acc.begin(), acc.end(), 0.f);
        Epi e = ep;
        e.set_group(g, bz);
        for (int t = 0; t < nt; ++t) {
          std::fill(As.begin(), As.end(), 0x7fc07fc0u);  // two bf16 NaNs: an unwritten slot shows up
          std::fill(Bs.begin(), Bs.end(), 0x7fc07fc0u);
          std::vector<PixelEntry> table;
          if constexpr (uses_table<AL>::value) {
            table.assign(kend - kbeg, PixelEntry{0xdeadbeefu, 0u});
            for (int tid = 0; tid < kThreads; ++tid) AL::build_table(ap, table.data(), kbeg, kend, tid);
          }
          for (int tid = 0; tid < kThreads; ++tid) {
            AL al(ap, g, tid, m0);
            BL bl(bp, g, tid, n0);
            if constexpr (uses_table<AL>::value) al.set_table(table.data(), kbeg, kend);
            float4 ra[AL::NL], rb[BL::NL];
            plan_all(al, kbeg + t * T::BK, kend);
            plan_all(bl, kbeg + t * T::BK, kend);
            al.fetch(ra);
            bl.fetch(rb);
            bf_store_all(al, As.data(), ra);
            bf_store_all(bl, Bs.data(), rb);
          }
          for (int ks = 0; ks < T::BK / 16; ++ks)
            for (int i = 0; i < T::BM; ++i)
              for (int j = 0; j < T::BN; ++j) {
                float s = 0.f;
                for (int kh = 0; kh < 2; ++kh)
                  for (int w = 0; w < 4; ++w) {
                    const int ia = bf_frag_word<AL>(i, ks, kh, w), ib = bf_frag_word<BL>(j, ks, kh, w);
                    if (ia < 0 || ia >= AL::LDS_WORDS || ib < 0 || ib >= BL::LDS_WORDS) emu_fail("LDS read out of range");
                    for (int h = 0; h < 2; ++h) s += bf_value(As[ia], h) * bf_value(Bs[ib], h);
                  }
                acc[(size_t)i * T::BN + j] += s;
              }
        }
        // every accumulator element belongs to exactly one (wave, block, lane, register)
        for (int wave = 0; wave < 4; ++wave) {
          const int wm = wave % T::WAVES_M, wn = wave / T::WAVES_M;
          for (int lane = 0; lane < 64; ++lane)
            for (int i = 0; i < T::TM; ++i)
              for (int j = 0; j < T::TN; ++j) {
                const int nl = wn * (T::TN * 32) + j * 32 + (lane & 31);
                if (n0 + nl >= N) continue;
                for (int r = 0; r < 16; ++r) {
                  const int ml = wm * (T::TM * 32) + i * 32 + acc_row(lane, r);
                  if (m0 + ml < M) e.apply(m0 + ml, n0 + nl, acc[(size_t)ml * T::BN + nl]);
                }
              }
        }
      }
}

static bool g_round_bf = false;  // draw values that bf16 holds exactly, so both arithmetic kinds share the references
static float frand() {
  float f = (float)rand() / RAND_MAX * 2.f - 1.f;
  if (g_round_bf) {
    const uint32_t u = bf16_bits(f) << 16;
    memcpy(&f, &u, 4);
  }
  return f;
}

struct Case {
  ConvGeom c;
  const char* name;
};

static int failures = 0;
static void check(const char* what, const char* name, const std::vector<float>& got, const std::vector<double>& want) {
  double num = 0, den = 0;
  bool nan = false;
  for (size_t i = 0; i < want.size(); ++i) {
    if (!(got[i] == got[i])) nan = true;
    num += (got[i] - want[i]) * (got[i] - want[i]);
    den += want[i] * want[i];
  }
  double rel = sqrt(num / (den > 0 ? den : 1));
  bool ok = !nan && rel < 1e-5;
  printf("%-10s %-28s rel_l2=%.3e %s\n", what, name, rel, ok ? "ok" : "FAIL");
  if (!ok) ++failures;
}

template <class T, bool BF = false>
static void run_case(const Case& cs) {
  g_round_bf = BF;
  const ConvGeom& c = cs.c;
  const int cg = c.cg(), og = c.og(), k = c.k;
  // exact-size heap buffers: the sanitizer flags any access past either end
  float* x = new float[c.in_elems()];
  float* dy = new float[c.out_elems()];
  float* w = new float[c.w_elems()];  // canonical OIHW
  float* wf = new float[c.w_elems()];
  float* wb = new float[c.w_elems()];
  float* bias = new float[c.Cout];
  for (long i = 0; i < c.in_elems(); ++i) x[i] = frand();
  for (long i = 0; i < c.out_elems(); ++i) dy[i] = frand();
  for (long i = 0; i < c.w_elems(); ++i) w[i] = frand();
  for (int i = 0; i < c.Cout; ++i) bias[i] = frand();
  for (int o = 0; o < c.Cout; ++o)
    for (int ci = 0; ci < cg; ++ci)
      for (int r = 0; r < k; ++r)
        for (int s = 0; s < k; ++s) {
          const int g = o / og, ol = o % og;
          const float v = w[((o * cg + ci) * k + r) * k + s];
          wf[((long)g * c.kf() + (r * k + s) * cg + ci) * og + ol] = v;
          wb[((long)g * c.kb() + (r * k + s) * og + ol) * cg + ci] = v;
        }
  auto X = [&](int n, int iy, int ix, int ch) -> double {
    if (iy < 0 || iy >= c.H || ix < 0 || ix >= c.W) return 0.0;
    return x[(((long)n * c.H + iy) * c.W + ix) * c.Cin + ch];
  };
  // ---- direct references (channel-last) ----
  std::vector<double> y_ref(c.out_elems()), dx_ref(c.in_elems(), 0.0), dwf_ref(c.w_elems(), 0.0);
  for (int n = 0; n < c.B; ++n)
    for (int yy = 0; yy < c.Ho; ++yy)
      for (int xx = 0; xx < c.Wo; ++xx)
        for (int o = 0; o < c.Cout; ++o) {
          const int g = o / og, ol = o % og;
          double a = bias[o];
          const double d = dy[(((long)n * c.Ho + yy) * c.Wo + xx) * c.Cout + o];
          for (int ci = 0; ci < cg; ++ci)
            for (int r = 0; r < k; ++r)
              for (int s = 0; s < k; ++s) {
                const int iy = yy * c.stride - c.pad + r, ix = xx * c.stride - c.pad + s;
                const double wv = w[((o * cg + ci) * k + r) * k + s];
                const double xv = X(n, iy, ix, g * cg + ci);
                a += wv * xv;
                dwf_ref[((long)g * c.kf() + (r * k + s) * cg + ci) * og + ol] += d * xv;
                if (iy >= 0 && iy < c.H && ix >= 0 && ix < c.W)
                  dx_ref[(((long)n * c.H + iy) * c.W + ix) * c.Cin + g * cg + ci] += d * wv;
              }
          y_ref[(((long)n * c.Ho + yy) * c.Wo + xx) * c.Cout + o] = a > 0 ? a : 0;
        }
  char nm[128];
  snprintf(nm, sizeof nm, "%s/%dx%d%s", cs.name, T::BM, T::BN, BF ? "/bf16" : "");
  typedef BfRowMajor<Im2colKInner<T::BM, T::BK, true, IM2COL_FWD>, T::BM, T::BK> BfGatherF;
  typedef BfRowMajor<Im2colKInner<T::BM, T::BK, true, IM2COL_T1>, T::BM, T::BK> BfGatherT;
  typedef BfDenseRowInner<T::BN, T::BK> BfRows;
  if constexpr (BF) {
    if constexpr (T::BM == 128) {  // the loaders that round fp32 on the fly exist for 128-row tiles only
    // the bf16 kernels exist for 16-byte loads only; other shapes keep the fp32 kernels
    const int kcf = ((fwd_dims(c).K + T::BK - 1) / T::BK) * T::BK;
    if (fwd_A_vec(c, x) && fwd_B_vec(c, wf)) {
      std::vector<float> y(c.out_elems(), NAN);
      const GemmDims d = fwd_dims(c);
      EpiBiasAct e{y.data(), c.Cout, bias, 1, og, 0};
      emu_gemm_bf<T, BfGatherF, BfRows, EpiBiasAct>(fwd_A(c, x), fwd_B(c, wf), e, d.M, d.N, d.K, kcf, 1, d.groups);
      check("fwd", nm, y, y_ref);
      const Im2colParams fa = fwd_A(c, x);
      if (fa.Cg % T::BK == 0 && c.k * c.k <= 32) {
        std::fill(y.begin(), y.end(), NAN);
        emu_gemm_bf<T, BfRowMajor<Im2colKTap<T::BM, T::BK, IM2COL_FWD>, T::BM, T::BK>, BfDenseRowWhole<T::BN, T::BK>,
                    EpiBiasAct>(fa, fwd_B(c, wf), e, d.M, d.N, d.K, kcf, 1, d.groups);
        check("fwd_tap", nm, y, y_ref);
      }
    }
    if (run_mode(c) && c.Cout % 4 == 0) {
      const int run = run_len(c), kc = c.k * c.Cin;
      float* wrun = new float[run_w_elems(c)];
      for (int r = 0; r < c.k; ++r)
        for (int j = 0; j < run; ++j)
          for (int o = 0; o < c.Cout; ++o) wrun[((long)r * run + j) * c.Cout + o] = j < kc ? wf[((long)r * kc + j) * c.Cout + o] : 0.f;
      {
        std::vector<float> y(c.out_elems(), NAN);
        GemmDims d = fwd_dims(c);
        d.K = run_k(c);
        EpiBiasAct e{y.data(), c.Cout, bias, 1, og, 0};
        emu_gemm_bf<T, BfGatherF, BfRows, EpiBiasAct>(run_A(c, x), run_B(c, wrun), e, d.M, d.N, d.K,
                                                       ((d.K + T::BK - 1) / T::BK) * T::BK, 1, 1);
        check("fwd_run", nm, y, y_ref);
      }
      {
        GemmDims d = bwdw_dims(c);
        d.M = run_k(c);
        std::vector<float> dwr((size_t)d.M * d.N, NAN);
        EpiSlab e{dwr.data(), (long)d.M * d.N, d.N, nullptr};
        emu_gemm_bf<T, BfIm2colRowInner<T::BM, T::BK>, BfRows, EpiSlab>(run_A(c, x), bwdw_B(c, dy), e, d.M, d.N, d.K,
                                                                         ((d.K + T::BK - 1) / T::BK) * T::BK, 1, 1);
        std::vector<float> dwf(c.w_elems(), 0.f);
        for (int r = 0; r < c.k; ++r)
          for (int j = 0; j < kc; ++j)
            for (int o = 0; o < c.Cout; ++o) dwf[((long)r * kc + j) * c.Cout + o] = dwr[((long)r * run + j) * c.Cout + o];
        check("bwdw_run", nm, dwf, dwf_ref);
      }
      delete[] wrun;
    }
    if (c.stride == 1 && bwdd_A_vec(c, dy) && bwdd_B_vec(c, wb)) {
      std::vector<float> dx(c.in_elems(), NAN);
      const GemmDims d = bwdd_dims(c);
      EpiGate e{dx.data(), c.Cin, nullptr, cg, 0};
      emu_gemm_bf<T, BfGatherT, BfRows, EpiGate>(bwdd_A(c, dy), bwdd_B(c, wb), e, d.M, d.N, d.K,
                                                 ((d.K + T::BK - 1) / T::BK) * T::BK, 1, d.groups);
      check("bwd_data", nm, dx, dx_ref);
      const Im2colParams ba = bwdd_A(c, dy);
      if (ba.Cg % T::BK == 0 && c.k * c.k <= 32) {
        std::fill(dx.begin(), dx.end(), NAN);
        emu_gemm_bf<T, BfRowMajor<Im2colKTap<T::BM, T::BK, IM2COL_T1>, T::BM, T::BK>, BfDenseRowWhole<T::BN, T::BK>,
                    EpiGate>(ba, bwdd_B(c, wb), e, d.M, d.N, d.K, d.K, 1, d.groups);
        check("bwdd_tap", nm, dx, dx_ref);
      }
    }
    if (bwdw_A_vec(c, x) && bwdw_B_vec(c, dy)) {
      const GemmDims d = bwdw_dims(c);
      int kchunk;
      long tiles = (long)((d.M + T::BM - 1) / T::BM) * ((d.N + T::BN - 1) / T::BN) * d.groups;
      int nsplit = plan_split(tiles, d.K, T::BK, 7, 5, &kchunk);
      std::vector<float> ws((size_t)d.groups * nsplit * d.M * d.N, NAN);
      EpiSlab e{ws.data(), (long)d.M * d.N, d.N, nullptr};
      emu_gemm_bf<T, BfIm2colRowInner<T::BM, T::BK>, BfRows, EpiSlab>(bwdw_A(c, x), bwdw_B(c, dy), e, d.M, d.N, d.K,
                                                                       kchunk, nsplit, d.groups);
      std::vector<float> dwf(c.w_elems(), 0.f);
      for (int g = 0; g < d.groups; ++g)
        for (int sp = 0; sp < nsplit; ++sp)
          for (long i = 0; i < (long)d.M * d.N; ++i) dwf[(long)g * d.M * d.N + i] += ws[((long)g * nsplit + sp) * d.M * d.N + i];
      snprintf(nm, sizeof nm, "%s/%dx%d/s%d/bf16", cs.name, T::BM, T::BN, nsplit);
      check("bwd_wgt", nm, dwf, dwf_ref);
      if (d.K % T::BK == 0 && c.k * c.k <= 31 && kchunk % T::BK == 0) {
        std::fill(ws.begin(), ws.end(), NAN);
        emu_gemm_bf<T, BfIm2colRowTable<T::BM, T::BK>, BfDenseRowWhole<T::BN, T::BK>, EpiSlab>(
            bwdw_A(c, x), bwdw_B(c, dy), e, d.M, d.N, d.K, kchunk, nsplit, d.groups);
        std::fill(dwf.begin(), dwf.end(), 0.f);
        for (int g = 0; g < d.groups; ++g)
          for (int sp = 0; sp < nsplit; ++sp)
            for (long i = 0; i < (long)d.M * d.N; ++i) {
              const float v = ws[((long)g * nsplit + sp) * d.M * d.N + i];
              if (v == v) dwf[(long)g * d.M * d.N + i] += v;
            }
        check("bwd_wgt_tbl", nm, dwf, dwf_ref);
      }
    }
    }
    // ---- run mode over bf16 pictures with four channels per pixel ----
    if (run16_mode(c)) {
      const int run = run16_len(c), K16 = run16_k(c);
      uint16_t* x4 = new uint16_t[run16_x_elems(c)];
      for (long p = 0; p < (long)c.B * c.H * c.W; ++p)
        for (int ch = 0; ch < 4; ++ch) x4[p * 4 + ch] = ch < c.Cin ? (uint16_t)bf16_bits(x[p * c.Cin + ch]) : 0;
      uint16_t* wk = new uint16_t[run16_w_elems(c)];
      for (int o = 0; o < c.Cout; ++o)
        for (int r = 0; r < c.k; ++r)
          for (int j = 0; j < run; ++j) {
            const int s2 = j / 4, ch = j % 4;
            wk[(long)o * K16 + r * run + j] =
                (s2 < c.k && ch < c.Cin) ? (uint16_t)bf16_bits(wf[((long)(r * c.k + s2) * c.Cin + ch) * c.Cout + o]) : 0;
          }
      {
        std::vector<float> y(c.out_elems(), NAN);
        GemmDims d = fwd_dims(c);
        d.K = K16;
        EpiBiasAct e{y.data(), c.Cout, bias, 1, og, 0};
        emu_gemm_bf<T, Im2colKInner16<T::BM, T::BK, IM2COL_FWD>, DenseKInner16<T::BN, T::BK>, EpiBiasAct>(
            run16_A(c, x4), run16_Bk(c, wk), e, d.M, d.N, d.K, ((d.K + T::BK - 1) / T::BK) * T::BK, 1, 1);
        check("fwd_run16", nm, y, y_ref);
      }
      delete[] x4; delete[] wk;
    }
    // ---- operands stored as bf16 (values are exact in bf16 here, so the same references hold) ----
    if constexpr (T::BN != 96)  // the 96-column tile serves the padded-run forward product above only
    if (conv16_ok(c)) {
      auto to16 = [](const float* src, long n) {
        uint16_t* d = new uint16_t[n];  // exact size: the sanitizer sees any access past the end
        for (long i = 0; i < n; ++i) d[i] = (uint16_t)bf16_bits(src[i]);
        return d;
      };
      uint16_t* x16 = to16(x, c.in_elems());
      uint16_t* dy16 = to16(dy, c.out_elems());
      uint16_t* wf16 = to16(wf, c.w_elems());
      uint16_t* wb16 = to16(wb, c.w_elems());
      // the same weights with the reduction contiguous: wfk[g][o][(r,s,c)], wbk[g][c][(r,s,o)]
      uint16_t* wfk = new uint16_t[c.w_elems()];
      uint16_t* wbk = new uint16_t[c.w_elems()];
      for (int g = 0; g < c.groups; ++g) {
        for (int kk = 0; kk < c.kf(); ++kk)
          for (int o = 0; o < og; ++o) wfk[((long)g * og + o) * c.kf() + kk] = wf16[((long)g * c.kf() + kk) * og + o];
        for (int kk = 0; kk < c.kb(); ++kk)
          for (int ci = 0; ci < cg; ++ci) wbk[((long)g * cg + ci) * c.kb() + kk] = wb16[((long)g * c.kb() + kk) * cg + ci];
      }
      {
        std::vector<float> y(c.out_elems(), NAN);
        const GemmDims d = fwd_dims(c);
        const int kcf = ((d.K + T::BK - 1) / T::BK) * T::BK;
        EpiBiasAct e{y.data(), c.Cout, bias, 1, og, 0};
        const Im2colParams fa = im2col16(fwd_A(c, x), x16);
        const DenseParams fb = dense16(fwd_B(c, wf), wf16);
        emu_gemm_bf<T, Im2colKInner16<T::BM, T::BK, IM2COL_FWD>, DenseRowInner16<T::BN, T::BK>, EpiBiasAct>(
            fa, fb, e, d.M, d.N, d.K, kcf, 1, d.groups);
        check("fwd16", nm, y, y_ref);
        if (fa.Cg % T::BK == 0 && c.k * c.k <= 32) {
          std::fill(y.begin(), y.end(), NAN);
          emu_gemm_bf<T, Im2colKTap16<T::BM, T::BK, IM2COL_FWD>, DenseRowInner16<T::BN, T::BK>, EpiBiasAct>(
              fa, fb, e, d.M, d.N, d.K, kcf, 1, d.groups);
          check("fwd_tap16", nm, y, y_ref);
        }
        {  // weights with the reduction contiguous
          const DenseParams fk = fwd_B16k(c, wfk);
          std::fill(y.begin(), y.end(), NAN);
          emu_gemm_bf<T, Im2colKInner16<T::BM, T::BK, IM2COL_FWD>, DenseKInner16<T::BN, T::BK>, EpiBiasAct>(
              fa, fk, e, d.M, d.N, d.K, kcf, 1, d.groups);
          check("fwd16k", nm, y, y_ref);
          if (fa.Cg % T::BK == 0 && c.k * c.k <= 32) {
            std::fill(y.begin(), y.end(), NAN);
            emu_gemm_bf<T, Im2colKTap16<T::BM, T::BK, IM2COL_FWD>, DenseKInner16<T::BN, T::BK>, EpiBiasAct>(
                fa, fk, e, d.M, d.N, d.K, kcf, 1, d.groups);
            check("fwd_tap16k", nm, y, y_ref);
          }
        }
        if (d.K / T::BK >= 3) {  // split-k, chunks of whole k-tiles, the last one ragged
          const int ns = 3, chunk = (((d.K + T::BK - 1) / T::BK + ns - 1) / ns) * T::BK;
          std::vector<float> ws((size_t)d.groups * ns * d.M * d.N, NAN), ysum(c.out_elems(), 0.f);
          EpiSlab es{ws.data(), (long)d.M * d.N, d.N, nullptr};
          emu_gemm_bf<T, Im2colKInner16<T::BM, T::BK, IM2COL_FWD>, DenseRowInner16<T::BN, T::BK>, EpiSlab>(
              fa, fb, es, d.M, d.N, d.K, chunk, ns, d.groups);
          for (int g = 0; g < d.groups; ++g)
            for (int sp = 0; sp < ns; ++sp)
              for (int m = 0; m < d.M; ++m)
                for (int n = 0; n < d.N; ++n) {
                  const float v = ws[(((size_t)g * ns + sp) * d.M + m) * d.N + n];
                  if (v == v) ysum[(size_t)m * c.Cout + g * og + n] += v;
                }
          for (long i = 0; i < c.out_elems(); ++i) {
            const float v = ysum[i] + bias[i % c.Cout];
            ysum[i] = v > 0 ? v : 0;
          }
          check("fwd16_s3", nm, ysum, y_ref);
        }
      }
      {
        std::vector<float> dx(c.in_elems(), NAN);
        const GemmDims d = bwdd_dims(c);
        EpiGate e{dx.data(), c.Cin, nullptr, cg, 0};
        const Im2colParams ba = im2col16(bwdd_A(c, dy), dy16);
        const DenseParams bb = dense16(bwdd_B(c, wb), wb16);
        emu_gemm_bf<T, Im2colKInner16<T::BM, T::BK, IM2COL_T1>, DenseRowInner16<T::BN, T::BK>, EpiGate>(
            ba, bb, e, d.M, d.N, d.K, ((d.K + T::BK - 1) / T::BK) * T::BK, 1, d.groups);
        check("bwd_data16", nm, dx, dx_ref);
        if (ba.Cg % T::BK == 0 && c.k * c.k <= 32) {
          std::fill(dx.begin(), dx.end(), NAN);
          emu_gemm_bf<T, Im2colKTap16<T::BM, T::BK, IM2COL_T1>, DenseRowInner16<T::BN, T::BK>, EpiGate>(
              ba, bb, e, d.M, d.N, d.K, d.K, 1, d.groups);
          check("bwdd_tap16", nm, dx, dx_ref);
        }
        const DenseParams bk = bwdd_B16k(c, wbk);
        std::fill(dx.begin(), dx.end(), NAN);
        emu_gemm_bf<T, Im2colKInner16<T::BM, T::BK, IM2COL_T1>, DenseKInner16<T::BN, T::BK>, EpiGate>(
            ba, bk, e, d.M, d.N, d.K, ((d.K + T::BK - 1) / T::BK) * T::BK, 1, d.groups);
        check("bwd_data16k", nm, dx, dx_ref);
        if (ba.Cg % T::BK == 0 && c.k * c.k <= 32) {
          std::fill(dx.begin(), dx.end(), NAN);
          emu_gemm_bf<T, Im2colKTap16<T::BM, T::BK, IM2COL_T1>, DenseKInner16<T::BN, T::BK>, EpiGate>(
              ba, bk, e, d.M, d.N, d.K, d.K, 1, d.groups);
          check("bwdd_tap16k", nm, dx, dx_ref);
        }
      }
      {
        const GemmDims d = bwdw_dims(c);
        int kchunk;
        long tiles = (long)((d.M + T::BM - 1) / T::BM) * ((d.N + T::BN - 1) / T::BN) * d.groups;
        int nsplit = plan_split(tiles, d.K, T::BK, 7, 5, &kchunk);
        if (d.K % T::BK == 0 && c.k * c.k <= 31 && kchunk % T::BK == 0) {
          std::vector<float> ws((size_t)d.groups * nsplit * d.M * d.N, NAN);
          EpiSlab e{ws.data(), (long)d.M * d.N, d.N, nullptr};
          emu_gemm_bf<T, Im2colRowTable16<T::BM, T::BK>, DenseRowInner16<T::BN, T::BK>, EpiSlab>(
              im2col16(bwdw_A(c, x), x16), dense16(bwdw_B(c, dy), dy16), e, d.M, d.N, d.K, kchunk, nsplit, d.groups);
          std::vector<float> dwf(c.w_elems(), 0.f);
          for (int g = 0; g < d.groups; ++g)
            for (int sp = 0; sp < nsplit; ++sp)
              for (long i = 0; i < (long)d.M * d.N; ++i) {
                const float v = ws[((long)g * nsplit + sp) * d.M * d.N + i];
                if (v == v) dwf[(long)g * d.M * d.N + i] += v;
              }
          snprintf(nm, sizeof nm, "%s/%dx%d/s%d/bf16", cs.name, T::BM, T::BN, nsplit);
          check("bwd_wgt_tbl16", nm, dwf, dwf_ref);
        }
      }
      delete[] x16; delete[] dy16; delete[] wf16; delete[] wb16; delete[] wfk; delete[] wbk;
    }
    delete[] x; delete[] dy; delete[] w; delete[] wf; delete[] wb; delete[] bias;
    g_round_bf = false;
    return;
  }
  // ---- forward ----
  {
    std::vector<float> y(c.out_elems(), NAN);
    GemmDims d = fwd_dims(c);
    EpiBiasAct e{y.data(), c.Cout, bias, 1, og, 0};
    const int kc = ((d.K + T::BK - 1) / T::BK) * T::BK;
    if (fwd_A_vec(c, x) && fwd_B_vec(c, wf))
      emu_gemm<T, Im2colKInner<T::BM, T::BK, true, IM2COL_FWD>, DenseRowInner<T::BN, T::BK, true>, EpiBiasAct>(
          fwd_A(c, x), fwd_B(c, wf), e, d.M, d.N, d.K, kc, 1, d.groups);
    else if (fwd_B_vec(c, wf))
      emu_gemm<T, Im2colKInner<T::BM, T::BK, false, IM2COL_FWD>, DenseRowInner<T::BN, T::BK, true>, EpiBiasAct>(
          fwd_A(c, x), fwd_B(c, wf), e, d.M, d.N, d.K, kc, 1, d.groups);
    else
      emu_gemm<T, Im2colKInner<T::BM, T::BK, false, IM2COL_FWD>, DenseRowInner<T::BN, T::BK, false>, EpiBiasAct>(
          fwd_A(c, x), fwd_B(c, wf), e, d.M, d.N, d.K, kc, 1, d.groups);
    check("fwd", nm, y, y_ref);
    // a k-tile inside one tap: uniform tap decode, per-pixel tap masks, whole k-tiles
    const Im2colParams fa = fwd_A(c, x);
    if (fwd_A_vec(c, x) && fwd_B_vec(c, wf) && fa.Cg % T::BK == 0 && c.k * c.k <= 32) {
      std::fill(y.begin(), y.end(), NAN);
      emu_gemm<T, Im2colKTap<T::BM, T::BK, IM2COL_FWD>, DenseRowWhole<T::BN, T::BK>, EpiBiasAct>(
          fa, fwd_B(c, wf), e, d.M, d.N, d.K, kc, 1, d.groups);
      check("fwd_tap", nm, y, y_ref);
      // split-k with whole-tile chunks
      if (d.K / T::BK >= 3) {
        const int ns = 3, chunk = ((d.K / T::BK + ns - 1) / ns) * T::BK;
        std::vector<float> ws((size_t)d.groups * ns * d.M * d.N, NAN), ysum(c.out_elems(), 0.f);
        EpiSlab es{ws.data(), (long)d.M * d.N, d.N, nullptr};
        emu_gemm<T, Im2colKTap<T::BM, T::BK, IM2COL_FWD>, DenseRowWhole<T::BN, T::BK>, EpiSlab>(
            fa, fwd_B(c, wf), es, d.M, d.N, d.K, chunk, ns, d.groups);
        for (int g = 0; g < d.groups; ++g)
          for (int sp = 0; sp < ns; ++sp)
            for (int m = 0; m < d.M; ++m)
              for (int n = 0; n < d.N; ++n) {
                const float v = ws[(((size_t)g * ns + sp) * d.M + m) * d.N + n];
                if (v == v) ysum[(size_t)m * c.Cout + g * og + n] += v;  // a chunk past K leaves its slab unwritten
              }
        for (long i = 0; i < c.out_elems(); ++i) {
          const float v = ysum[i] + bias[i % c.Cout];
          ysum[i] = v > 0 ? v : 0;
        }
        check("fwd_tap_s3", nm, ysum, y_ref);
      }
    }
  }
  // ---- run mode: forward and backward weight through the padded-row view ----
  if (run_mode(c) && c.Cout % 4 == 0) {
    const int run = run_len(c), kc = c.k * c.Cin;
    float* wrun = new float[run_w_elems(c)];
    for (int r = 0; r < c.k; ++r)
      for (int j = 0; j < run; ++j)
        for (int o = 0; o < c.Cout; ++o) wrun[((long)r * run + j) * c.Cout + o] = j < kc ? wf[((long)r * kc + j) * c.Cout + o] : 0.f;
    {
      std::vector<float> y(c.out_elems(), NAN);
      GemmDims d = fwd_dims(c);
      d.K = run_k(c);
      EpiBiasAct e{y.data(), c.Cout, bias, 1, og, 0};
      emu_gemm<T, Im2colKInner<T::BM, T::BK, true, IM2COL_FWD>, DenseRowInner<T::BN, T::BK, true>, EpiBiasAct>(
          run_A(c, x), run_B(c, wrun), e, d.M, d.N, d.K, ((d.K + T::BK - 1) / T::BK) * T::BK, 1, 1);
      check("fwd_run", nm, y, y_ref);
    }
    {
      GemmDims d = bwdw_dims(c);
      d.M = run_k(c);
      std::vector<float> dwr((size_t)d.M * d.N, NAN);
      EpiSlab e{dwr.data(), (long)d.M * d.N, d.N, nullptr};
      emu_gemm<T, Im2colRowInner<T::BM, T::BK, true>, DenseRowInner<T::BN, T::BK, true>, EpiSlab>(
          run_A(c, x), bwdw_B(c, dy), e, d.M, d.N, d.K, ((d.K + T::BK - 1) / T::BK) * T::BK, 1, 1);
      std::vector<float> dwf(c.w_elems(), 0.f);
      for (int r = 0; r < c.k; ++r)
        for (int j = 0; j < kc; ++j)
          for (int o = 0; o < c.Cout; ++o) dwf[((long)r * kc + j) * c.Cout + o] = dwr[((long)r * run + j) * c.Cout + o];
      check("bwdw_run", nm, dwf, dwf_ref);
      if (d.K % T::BK == 0) {  // pixel table in LDS, whole k-tiles, two splits
        const int ns = 2, chunk = ((d.K / T::BK + ns - 1) / ns) * T::BK;
        std::vector<float> ws((size_t)ns * d.M * d.N, NAN);
        EpiSlab es{ws.data(), (long)d.M * d.N, d.N, nullptr};
        emu_gemm<T, Im2colRowTable<T::BM, T::BK>, DenseRowWhole<T::BN, T::BK>, EpiSlab>(run_A(c, x), bwdw_B(c, dy), es,
                                                                                       d.M, d.N, d.K, chunk, ns, 1);
        std::fill(dwf.begin(), dwf.end(), 0.f);
        for (int sp = 0; sp < ns; ++sp)
          for (int r = 0; r < c.k; ++r)
            for (int j = 0; j < kc; ++j)
              for (int o = 0; o < c.Cout; ++o) {
                const float v = ws[((size_t)sp * d.M + (size_t)r * run + j) * d.N + o];
                if (v == v) dwf[((long)r * kc + j) * c.Cout + o] += v;
              }
        check("bwdw_run_tbl", nm, dwf, dwf_ref);
      }
    }
    delete[] wrun;
  }
  // ---- backward data ----
  {
    std::vector<float> dx(c.in_elems(), NAN);
    GemmDims d = bwdd_dims(c);
    EpiGate e{dx.data(), c.Cin, nullptr, cg, 0};
    const int kc = ((d.K + T::BK - 1) / T::BK) * T::BK;
    const bool vv = bwdd_A_vec(c, dy) && bwdd_B_vec(c, wb);
    if (c.stride == 1 && vv)
      emu_gemm<T, Im2colKInner<T::BM, T::BK, true, IM2COL_T1>, DenseRowInner<T::BN, T::BK, true>, EpiGate>(
          bwdd_A(c, dy), bwdd_B(c, wb), e, d.M, d.N, d.K, kc, 1, d.groups);
    else if (c.stride == 1)
      emu_gemm<T, Im2colKInner<T::BM, T::BK, false, IM2COL_T1>, DenseRowInner<T::BN, T::BK, false>, EpiGate>(
          bwdd_A(c, dy), bwdd_B(c, wb), e, d.M, d.N, d.K, kc, 1, d.groups);
    else if (vv)
      emu_gemm<T, Im2colKInner<T::BM, T::BK, true, IM2COL_TS>, DenseRowInner<T::BN, T::BK, true>, EpiGate>(
          bwdd_A(c, dy), bwdd_B(c, wb), e, d.M, d.N, d.K, kc, 1, d.groups);
    else
      emu_gemm<T, Im2colKInner<T::BM, T::BK, false, IM2COL_TS>, DenseRowInner<T::BN, T::BK, false>, EpiGate>(
          bwdd_A(c, dy), bwdd_B(c, wb), e, d.M, d.N, d.K, kc, 1, d.groups);
    check("bwd_data", nm, dx, dx_ref);
    const Im2colParams ba = bwdd_A(c, dy);
    if (c.stride == 1 && vv && ba.Cg % T::BK == 0 && c.k * c.k <= 32) {
      std::fill(dx.begin(), dx.end(), NAN);
      emu_gemm<T, Im2colKTap<T::BM, T::BK, IM2COL_T1>, DenseRowWhole<T::BN, T::BK>, EpiGate>(
          ba, bwdd_B(c, wb), e, d.M, d.N, d.K, kc, 1, d.groups);
      check("bwdd_tap", nm, dx, dx_ref);
    }
  }
  // ---- backward data by phases (strided, ungrouped) ----
  if (phase_mode(c) && c.Cout % 4 == 0 && phase_n(c) % 4 == 0) {
    const int ka = phase_taps(c), st = c.stride, pn = phase_n(c);
    float* wp = new float[phase_w_elems(c)];
    for (int a = 0; a < ka; ++a)
      for (int b2 = 0; b2 < ka; ++b2)
        for (int o = 0; o < c.Cout; ++o)
          for (int py = 0; py < st; ++py)
            for (int px = 0; px < st; ++px)
              for (int ci = 0; ci < c.Cin; ++ci) {
                const int r = py + st * a, s2 = px + st * b2;
                wp[(((long)a * ka + b2) * c.Cout + o) * pn + (py * st + px) * c.Cin + ci] =
                    (r < k && s2 < k) ? w[((o * cg + ci) * k + r) * k + s2] : 0.f;
              }
    std::vector<float> dx(c.in_elems(), NAN);
    const GemmDims d = phase_dims(c);
    emu_gemm<T, Im2colKInner<T::BM, T::BK, true, IM2COL_T1>, DenseRowInner<T::BN, T::BK, true>, EpiPhases>(
        phase_A(c, dy), phase_B(c, wp), phase_epilogue(c, dx.data()), d.M, d.N, d.K,
        ((d.K + T::BK - 1) / T::BK) * T::BK, 1, 1);
    check("bwdd_phase", nm, dx, dx_ref);
    delete[] wp;
  }
  // ---- backward weight with split-k ----
  {
    GemmDims d = bwdw_dims(c);
    int kchunk;
    long tiles = (long)((d.M + T::BM - 1) / T::BM) * ((d.N + T::BN - 1) / T::BN) * d.groups;
    int nsplit = plan_split(tiles, d.K, T::BK, 7, 5, &kchunk);
    std::vector<float> ws((size_t)d.groups * nsplit * d.M * d.N, NAN);
    EpiSlab e{ws.data(), (long)d.M * d.N, d.N, nullptr};
    if (bwdw_A_vec(c, x) && bwdw_B_vec(c, dy))
      emu_gemm<T, Im2colRowInner<T::BM, T::BK, true>, DenseRowInner<T::BN, T::BK, true>, EpiSlab>(
          bwdw_A(c, x), bwdw_B(c, dy), e, d.M, d.N, d.K, kchunk, nsplit, d.groups);
    else if (bwdw_B_vec(c, dy))
      emu_gemm<T, Im2colRowInner<T::BM, T::BK, false>, DenseRowInner<T::BN, T::BK, true>, EpiSlab>(
          bwdw_A(c, x), bwdw_B(c, dy), e, d.M, d.N, d.K, kchunk, nsplit, d.groups);
    else
      emu_gemm<T, Im2colRowInner<T::BM, T::BK, false>, DenseRowInner<T::BN, T::BK, false>, EpiSlab>(
          bwdw_A(c, x), bwdw_B(c, dy), e, d.M, d.N, d.K, kchunk, nsplit, d.groups);
    std::vector<float> dwf(c.w_elems(), 0.f);
    for (int g = 0; g < d.groups; ++g)
      for (int sp = 0; sp < nsplit; ++sp)
        for (long i = 0; i < (long)d.M * d.N; ++i) dwf[(long)g * d.M * d.N + i] += ws[((long)g * nsplit + sp) * d.M * d.N + i];
    snprintf(nm, sizeof nm, "%s/%dx%d/s%d", cs.name, T::BM, T::BN, nsplit);
    check("bwd_wgt", nm, dwf, dwf_ref);
    if (bwdw_A_vec(c, x) && bwdw_B_vec(c, dy) && d.K % T::BK == 0 && c.k * c.k <= 31 && kchunk % T::BK == 0) {
      std::fill(ws.begin(), ws.end(), NAN);
      emu_gemm<T, Im2colRowTable<T::BM, T::BK>, DenseRowWhole<T::BN, T::BK>, EpiSlab>(
          bwdw_A(c, x), bwdw_B(c, dy), e, d.M, d.N, d.K, kchunk, nsplit, d.groups);
      std::fill(dwf.begin(), dwf.end(), 0.f);
      for (int g = 0; g < d.groups; ++g)
        for (int sp = 0; sp < nsplit; ++sp)
          for (long i = 0; i < (long)d.M * d.N; ++i) {
            const float v = ws[((long)g * nsplit + sp) * d.M * d.N + i];
            if (v == v) dwf[(long)g * d.M * d.N + i] += v;  // a chunk past K leaves its slab unwritten
          }
      check("bwd_wgt_tbl", nm, dwf, dwf_ref);
    }
  }
  delete[] x; delete[] dy; delete[] w; delete[] wf; delete[] wb; delete[] bias;
}

static ConvGeom geom(int B, int H, int Cin, int Cout, int k, int st, int pad, int groups) {
  ConvGeom c;
  c.B = B; c.H = H; c.W = H + 1; c.Cin = Cin; c.Cout = Cout; c.k = k; c.stride = st; c.pad = pad; c.groups = groups;
  c.Ho = (c.H + 2 * pad - k) / st + 1;
  c.Wo = (c.W + 2 * pad - k) / st + 1;
  return c;
}

static ConvGeom product_geom(int tiles, int groups, int kin, int nout) {
  // the channel products of a transformed 3x3 convolution: a 1x1 convolution with many groups over one row of pixels
  ConvGeom c;
  c.B = 1; c.H = 1; c.W = tiles; c.Cin = groups * kin; c.Cout = groups * nout; c.k = 1; c.stride = 1; c.pad = 0;
  c.groups = groups; c.Ho = 1; c.Wo = tiles;
  return c;
}

template <int ROWS, int BK>
static void dense_case() {
  // fully connected layer shapes with ragged and non-multiple-of-4 extents
  const int Bn = 6, In = 20, Out = 10;
  float* x = new float[Bn * In];
  float* w = new float[Out * In];
  float* dy = new float[Bn * Out];
  for (int i = 0; i < Bn * In; ++i) x[i] = frand();
  for (int i = 0; i < Out * In; ++i) w[i] = frand();
  for (int i = 0; i < Bn * Out; ++i) dy[i] = frand();
  typedef Tile<128, 128, 16, 2, 2> T;
  {  // y = x w^T : both operands contiguous along k
    std::vector<float> y(Bn * Out, NAN);
    std::vector<double> ref(Bn * Out, 0.0);
    for (int n = 0; n < Bn; ++n) for (int o = 0; o < Out; ++o) for (int i = 0; i < In; ++i) ref[n * Out + o] += (double)x[n * In + i] * w[o * In + i];
    DenseParams a{x, In, 0, Bn, Bn * In * 4}, b{w, In, 0, Out, Out * In * 4};
    EpiSlab e{y.data(), (long)Bn * Out, Out, nullptr};
    emu_gemm<T, DenseKInner<128, 16, true>, DenseKInner<128, 16, true>, EpiSlab>(a, b, e, Bn, Out, In, 32, 1, 1);
    check("fc_fwd", "6x20->10 vec", y, ref);
    std::fill(y.begin(), y.end(), NAN);
    emu_gemm<T, DenseKInner<128, 16, false>, DenseKInner<128, 16, false>, EpiSlab>(a, b, e, Bn, Out, In, 32, 1, 1);
    check("fc_fwd", "6x20->10", y, ref);
  }
  {  // dx = dy w : A contiguous along k (=Out, not a multiple of 4 -> scalar), B along rows
    std::vector<float> dx(Bn * In, NAN);
    std::vector<double> ref(Bn * In, 0.0);
    for (int n = 0; n < Bn; ++n) for (int o = 0; o < Out; ++o) for (int i = 0; i < In; ++i) ref[n * In + i] += (double)dy[n * Out + o] * w[o * In + i];
    DenseParams a{dy, Out, 0, Bn, Bn * Out * 4}, b{w, In, 0, In, Out * In * 4};
    EpiSlab e{dx.data(), (long)Bn * In, In, nullptr};
    emu_gemm<T, DenseKInner<128, 16, false>, DenseRowInner<128, 16, false>, EpiSlab>(a, b, e, Bn, In, Out, 16, 1, 1);
    check("fc_bwd_x", "6x20->10", dx, ref);
  }
  {  // dw = dy^T x : both contiguous along rows; A scalar path
    std::vector<float> dw(Out * In, NAN);
    std::vector<double> ref(Out * In, 0.0);
    for (int n = 0; n < Bn; ++n) for (int o = 0; o < Out; ++o) for (int i = 0; i < In; ++i) ref[o * In + i] += (double)dy[n * Out + o] * x[n * In + i];
    DenseParams a{dy, Out, 0, Out, Bn * Out * 4}, b{x, In, 0, In, Bn * In * 4};
    EpiSlab e{dw.data(), (long)Out * In, In, nullptr};
    emu_gemm<T, DenseRowInner<128, 16, false>, DenseRowInner<128, 16, false>, EpiSlab>(a, b, e, Out, In, Bn, 16, 1, 1);
    check("fc_bwd_w", "6x20->10", dw, ref);
  }
  delete[] x; delete[] w; delete[] dy;
}

static void dense_case_bf() {
  // vector-aligned dense shapes: ragged rows, k that ends inside a k-tile, split-k
  g_round_bf = true;
  const int Bn = 6, In = 72, Out = 36;
  float* x = new float[Bn * In];
  float* w = new float[Out * In];
  float* dy = new float[Bn * Out];
  for (int i = 0; i < Bn * In; ++i) x[i] = frand();
  for (int i = 0; i < Out * In; ++i) w[i] = frand();
  for (int i = 0; i < Bn * Out; ++i) dy[i] = frand();
  typedef Tile<128, 128, 32, 2, 2> T;
  typedef BfRowMajor<DenseKInner<128, 32, true>, 128, 32> KIn;
  typedef BfDenseRowInner<128, 32> RIn;
  {
    const int ns = 2, kc = 64;
    std::vector<float> ws(ns * Bn * Out, NAN), y(Bn * Out, 0.f);
    std::vector<double> ref(Bn * Out, 0.0);
    for (int n = 0; n < Bn; ++n) for (int o = 0; o < Out; ++o) for (int i = 0; i < In; ++i) ref[n * Out + o] += (double)x[n * In + i] * w[o * In + i];
    DenseParams a{x, In, 0, Bn, Bn * In * 4}, b{w, In, 0, Out, Out * In * 4};
    EpiSlab e{ws.data(), (long)Bn * Out, Out, nullptr};
    emu_gemm_bf<T, KIn, KIn, EpiSlab>(a, b, e, Bn, Out, In, kc, ns, 1);
    for (int sp = 0; sp < ns; ++sp) for (int i = 0; i < Bn * Out; ++i) y[i] += ws[sp * Bn * Out + i];
    check("fc_fwd", "6x72->36 bf16 s2", y, ref);
  }
  {
    std::vector<float> dx(Bn * In, NAN);
    std::vector<double> ref(Bn * In, 0.0);
    for (int n = 0; n < Bn; ++n) for (int o = 0; o < Out; ++o) for (int i = 0; i < In; ++i) ref[n * In + i] += (double)dy[n * Out + o] * w[o * In + i];
    DenseParams a{dy, Out, 0, Bn, Bn * Out * 4}, b{w, In, 0, In, Out * In * 4};
    EpiSlab e{dx.data(), (long)Bn * In, In, nullptr};
    emu_gemm_bf<T, KIn, RIn, EpiSlab>(a, b, e, Bn, In, Out, 64, 1, 1);
    check("fc_bwd_x", "6x72->36 bf16", dx, ref);
  }
  {
    std::vector<float> dw(Out * In, NAN);
    std::vector<double> ref(Out * In, 0.0);
    for (int n = 0; n < Bn; ++n) for (int o = 0; o < Out; ++o) for (int i = 0; i < In; ++i) ref[o * In + i] += (double)dy[n * Out + o] * x[n * In + i];
    DenseParams a{dy, Out, 0, Out, Bn * Out * 4}, b{x, In, 0, In, Bn * In * 4};
    EpiSlab e{dw.data(), (long)Out * In, In, nullptr};
    emu_gemm_bf<T, RIn, RIn, EpiSlab>(a, b, e, Out, In, Bn, 32, 1, 1);
    check("fc_bwd_w", "6x72->36 bf16", dw, ref);
  }
  {  // the same three products over operands stored as bf16 (extents are multiples of 8: 72, 40)
    const int Out8 = 40;
    auto to16 = [](const float* src, long n) {
      uint16_t* d = new uint16_t[n];
      for (long i = 0; i < n; ++i) d[i] = (uint16_t)bf16_bits(src[i]);
      return d;
    };
    float* w8 = new float[Out8 * In];
    float* dy8 = new float[Bn * Out8];
    for (int i = 0; i < Out8 * In; ++i) w8[i] = frand();
    for (int i = 0; i < Bn * Out8; ++i) dy8[i] = frand();
    uint16_t *x16 = to16(x, Bn * In), *w16 = to16(w8, Out8 * In), *dy16 = to16(dy8, Bn * Out8);
    typedef DenseKInner16<128, 32> K16;
    typedef DenseRowInner16<128, 32> R16;
    {
      const int ns = 2, kc = 64;
      std::vector<float> ws(ns * Bn * Out8, NAN), y(Bn * Out8, 0.f);
      std::vector<double> ref(Bn * Out8, 0.0);
      for (int n = 0; n < Bn; ++n) for (int o = 0; o < Out8; ++o) for (int i = 0; i < In; ++i) ref[n * Out8 + o] += (double)x[n * In + i] * w8[o * In + i];
      DenseParams a{(const float*)x16, In, 0, Bn, Bn * In * 2}, b{(const float*)w16, In, 0, Out8, Out8 * In * 2};
      EpiSlab e{ws.data(), (long)Bn * Out8, Out8, nullptr};
      emu_gemm_bf<T, K16, K16, EpiSlab>(a, b, e, Bn, Out8, In, kc, ns, 1);
      for (int sp = 0; sp < ns; ++sp) for (int i = 0; i < Bn * Out8; ++i) y[i] += ws[sp * Bn * Out8 + i];
      check("fc_fwd16", "6x72->40 s2", y, ref);
    }
    {
      std::vector<float> dx(Bn * In, NAN);
      std::vector<double> ref(Bn * In, 0.0);
      for (int n = 0; n < Bn; ++n) for (int o = 0; o < Out8; ++o) for (int i = 0; i < In; ++i) ref[n * In + i] += (double)dy8[n * Out8 + o] * w8[o * In + i];
      DenseParams a{(const float*)dy16, Out8, 0, Bn, Bn * Out8 * 2}, b{(const float*)w16, In, 0, In, Out8 * In * 2};
      EpiSlab e{dx.data(), (long)Bn * In, In, nullptr};
      emu_gemm_bf<T, K16, R16, EpiSlab>(a, b, e, Bn, In, Out8, 64, 1, 1);
      check("fc_bwd_x16", "6x72->40", dx, ref);
    }
    {
      std::vector<float> dw(Out8 * In, NAN);
      std::vector<double> ref(Out8 * In, 0.0);
      for (int n = 0; n < Bn; ++n) for (int o = 0; o < Out8; ++o) for (int i = 0; i < In; ++i) ref[o * In + i] += (double)dy8[n * Out8 + o] * x[n * In + i];
      DenseParams a{(const float*)dy16, Out8, 0, Out8, Bn * Out8 * 2}, b{(const float*)x16, In, 0, In, Bn * In * 2};
      EpiSlab e{dw.data(), (long)Out8 * In, In, nullptr};
      emu_gemm_bf<T, R16, R16, EpiSlab>(a, b, e, Out8, In, Bn, 32, 1, 1);
      check("fc_bwd_w16", "6x72->40", dw, ref);
    }
    delete[] w8; delete[] dy8; delete[] x16; delete[] w16; delete[] dy16;
  }
  delete[] x; delete[] w; delete[] dy;
  g_round_bf = false;
}

static void check_fastdiv() {
  const uint32_t ds[] = {1, 2, 3, 4, 5, 7, 8, 11, 12, 13, 16, 24, 27, 36, 48, 55, 96, 169, 192, 256, 729, 3025, 51529, 1000003};
  long bad = 0;
  for (uint32_t d : ds) {
    FastDiv f = make_fastdiv(d);
    for (uint32_t n = 0; n < 3000000u; ++n) bad += fdiv(n, f) != n / d;
    for (uint64_t n = 0x7fffffffull - 100000; n <= 0x7fffffffull; ++n) bad += fdiv((uint32_t)n, f) != (uint32_t)n / d;
    for (int i = 0; i < 2000000; ++i) {
      uint32_t n = ((uint32_t)rand() << 16 ^ (uint32_t)rand()) & 0x7fffffffu;
      bad += fdiv(n, f) != n / d;
    }
  }
  printf("fastdiv %s\n", bad ? "FAIL" : "ok");
  if (bad) ++failures;
}

template <class T>
static void check_acc_map() {
  // registers x lanes of one MFMA block cover its RB x RB outputs exactly once
  std::vector<int> seen(T::RB * T::RB, 0);
  for (int lane = 0; lane < 64; ++lane)
    for (int r = 0; r < T::NACC; ++r) ++seen[T::acc_row(lane, r) * T::RB + lane % T::RB];
  bool ok = true;
  for (int v : seen) ok = ok && v == 1;
  // the k of the steps and lane groups of one k-tile cover 0..BK-1 exactly once
  std::vector<int> ks(T::BK, 0);
  for (int u = 0; u < T::KP; ++u)
    for (int g = 0; g < T::G; ++g) ++ks[T::step_k(u, g)];
  for (int v : ks) ok = ok && v == 1;
  printf("acc/k map RB=%d BK=%d %s\n", T::RB, T::BK, ok ? "ok" : "FAIL");
  if (!ok) ++failures;
}

int main() {
  srand(1234);
  check_fastdiv();
  check_acc_map<Tile<128, 128, 16, 2, 2>>();
  check_acc_map<Tile<128, 48, 32, 4, 1, 16>>();
  std::vector<Case> cases = {
      {geom(2, 23, 3, 8, 11, 4, 0, 1), "k11s4c3"},      // scalar gather, stride 4
      {geom(3, 13, 3, 16, 7, 2, 0, 1), "k7s2c3"},       // mini conv1
      {geom(2, 7, 8, 40, 5, 1, 2, 2), "k5p2g2"},        // grouped, padded
      {geom(3, 6, 24, 36, 3, 1, 1, 1), "k3p1"},
      {geom(2, 6, 72, 72, 3, 1, 1, 2), "k3p1g2c36"},
      {geom(1, 9, 12, 20, 3, 2, 1, 2), "k3s2p1g2"},      // strided transposed gather with groups
      {geom(5, 5, 132, 136, 3, 1, 1, 1), "k3wide"},      // more than one tile along N and K rows
      {geom(2, 7, 64, 64, 3, 1, 1, 2), "k3p1g2c32"},     // a k-tile inside one tap (32 channels per group)
      {geom(3, 6, 32, 96, 5, 1, 2, 1), "k5p2c32"},       // 25 taps, ragged rows and columns
      {geom(4, 7, 8, 24, 3, 1, 1, 2), "k3p1g2px224"},    // 4*7*8 = 224 pixels: whole k-tiles for backward-weight
      {geom(4, 15, 3, 8, 5, 2, 0, 1), "k5s2c3px192"},    // run mode with 4*6*8 = 192 output pixels
      {geom(4, 10, 2, 8, 3, 1, 0, 1), "k3c2px256"},      // run mode with a run of 6 floats (padded to 8)
      {geom(2, 9, 3, 6, 5, 2, 1, 1), "k5s2p1c3o6"},      // channel counts that are no multiples of four:
      {geom(2, 7, 6, 10, 3, 1, 1, 2), "k3g2c3o5"},       // every operand falls back to 4-byte loads
      {geom(2, 3, 10, 9, 3, 1, 1, 1), "k3c10o9"},
      {geom(2, 3, 9, 15, 3, 1, 1, 3), "k3g3c3o5"},
      {geom(2, 3, 15, 7, 1, 1, 0, 1), "k1c15o7"},
      {product_geom(48, 12, 16, 8), "1x1g12c16t48"},    // whole k-tiles in every product
      {product_geom(40, 9, 20, 12), "1x1g9c20t40"},     // ragged k and pixel counts
      {product_geom(160, 4, 32, 32), "1x1g4c32t160"},   // two row tiles
      {geom(4, 7, 48, 80, 3, 1, 1, 2), "k3p1g2c24o40"}, // multiples of 8 but not of 32: bf16-stored operands, general taps
      {geom(4, 7, 16, 24, 5, 1, 2, 1), "k5p2c16o24"},   // 25 taps over bf16-stored operands, 24 columns in a 64-wide tile
      {geom(1, 7, 64, 136, 3, 1, 1, 1), "k3c64o136"},   // bf16-stored operands: two column tiles, the second ragged
      {geom(3, 31, 3, 96, 11, 4, 0, 1), "k11s4c3o96"},  // the first layer's shape: 96 columns, 3*6*6 = 108 pixels
      {geom(2, 19, 3, 104, 7, 2, 0, 1), "k7s2c3o104"},  // two 96-column tiles, the second ragged; 98 pixels
  };
  for (const Case& cs : cases) {
    if (strstr(cs.name, "o96") || strstr(cs.name, "o104")) {  // pictures as bf16 with four channels per pixel
      run_case<Tile<256, 96, 32, 4, 1>, true>(cs);
      run_case<Tile<256, 128, 32, 2, 2>, true>(cs);
      continue;
    }
    if (strstr(cs.name, "o40") || strstr(cs.name, "o24") || strstr(cs.name, "o136")) {  // the bf16-stored cases
      run_case<Tile<128, 128, 32, 2, 2>, true>(cs);
      run_case<Tile<128, 64, 32, 4, 1>, true>(cs);
      run_case<Tile<256, 128, 32, 2, 2>, true>(cs);
      continue;
    }
    run_case<Tile<128, 128, 32, 2, 2>>(cs);
    run_case<Tile<128, 96, 32, 4, 1>>(cs);
    run_case<Tile<128, 64, 32, 4, 1>>(cs);
    run_case<Tile<128, 128, 16, 2, 2>>(cs);
    run_case<Tile<128, 48, 32, 4, 1, 16>>(cs);
    run_case<Tile<128, 128, 32, 2, 2>, true>(cs);
    run_case<Tile<128, 64, 32, 4, 1>, true>(cs);
    run_case<Tile<256, 128, 32, 2, 2>, true>(cs);
  }
  dense_case<128, 16>();
  dense_case_bf();
  printf(failures ? "FAILED %d\n" : "ALL OK\n", failures);
  return failures ? 1 : 0;
}
