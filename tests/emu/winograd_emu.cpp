// CPU run of the per-thread programs in csrc/winograd.h (the F(4x4, 3x3) transforms), thread by thread,
// with the channel products between them written as plain loops, checked against direct convolution
// loops in double precision.  Buffers have exactly the sizes the library allocates and the test is built
// with -fsanitize=address, so an out-of-range access of a transform aborts here, on the CPU.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include <algorithm>
#include <vector>

struct float4 {
  float x, y, z, w;
};
struct float2 {
  float x, y;
};
#define AX_HOST_EMU 1
namespace ax {
inline void emu_fail(const char* what) {
  fprintf(stderr, "EMULATION FAULT: %s\n", what);
  abort();
}
}  // namespace ax
#include "../../paper_1412_2302_amd/csrc/winograd.h"

using namespace ax;

static int g_fail = 0;
static unsigned g_seed = 12345;
static float rnd() {
  g_seed = g_seed * 1664525u + 1013904223u;
  return ((g_seed >> 8) & 0xffff) / 32768.0f - 1.0f;
}
static void check(const char* what, const char* nm, const std::vector<float>& got, const std::vector<double>& ref,
                  double tol = 2e-5) {
  double num = 0, den = 0;
  for (size_t i = 0; i < ref.size(); ++i) {
    const double d = (double)got[i] - ref[i];
    num += d * d;
    den += ref[i] * ref[i];
  }
  const double rel = sqrt(num / (den > 0 ? den : 1));
  const bool ok = rel <= tol && got.size() == ref.size();
  printf("%-10s %-28s rel_l2=%.3e %s\n", what, nm, rel, ok ? "ok" : "FAIL");
  if (!ok) ++g_fail;
}

// the 1-D identities behind everything else: y = At[(G g) .* (Bt d)] is the correlation, and the two adjoint forms
static void check_1d() {
  Vec4 d[6], g[3], e[4];
  for (auto& v : d) v = {rnd(), rnd(), rnd(), rnd()};
  for (auto& v : g) v = {rnd(), rnd(), rnd(), rnd()};
  for (auto& v : e) v = {rnd(), rnd(), rnd(), rnd()};
  Vec4 bd[6], gg[6], ae[6], prod[6], y[4], dg[3];
  wino_bt<1, 1>(d, bd);
  wino_g<1, 1>(g, gg);
  wino_a<1, 1>(e, ae);
  for (int p = 0; p < 6; ++p) prod[p] = {gg[p].x * bd[p].x, gg[p].y * bd[p].y, gg[p].z * bd[p].z, gg[p].w * bd[p].w};
  wino_at<1, 1>(prod, y);
  std::vector<float> got;
  std::vector<double> ref;
  for (int i = 0; i < 4; ++i) {
    double r = 0;
    for (int j = 0; j < 3; ++j) r += (double)g[j].x * d[i + j].x;
    got.push_back(y[i].x);
    ref.push_back(r);
  }
  check("1d", "y = sum_j g_j d_{i+j}", got, ref, 1e-5);
  for (int p = 0; p < 6; ++p) prod[p] = {ae[p].x * bd[p].x, ae[p].y * bd[p].y, ae[p].z * bd[p].z, ae[p].w * bd[p].w};
  wino_gt<1, 1>(prod, dg);
  got.clear();
  ref.clear();
  for (int j = 0; j < 3; ++j) {
    double r = 0;
    for (int i = 0; i < 4; ++i) r += (double)e[i].y * d[i + j].y;
    got.push_back(dg[j].y);
    ref.push_back(r);
  }
  check("1d", "dg_j = sum_i e_i d_{i+j}", got, ref, 1e-5);
  Vec4 dd[6];
  for (int p = 0; p < 6; ++p) prod[p] = {ae[p].x * gg[p].x, ae[p].y * gg[p].y, ae[p].z * gg[p].z, ae[p].w * gg[p].w};
  wino_b<1, 1>(prod, dd);
  got.clear();
  ref.clear();
  for (int k = 0; k < 6; ++k) {
    double r = 0;
    for (int i = 0; i < 4; ++i)
      if (k - i >= 0 && k - i < 3) r += (double)e[i].z * g[k - i].z;
    got.push_back(dd[k].z);
    ref.push_back(r);
  }
  check("1d", "dd_k = sum_i e_i g_{k-i}", got, ref, 1e-5);
}

struct Case {
  const char* name;
  int B, H, W, pad, groups, cg, og, k;  // k x k taps: 3, or 5 as four 3x3 sub-kernels
};

// m[t][z*N + o] = sum_c a[t][z*K + c] * u[z][c][o]
static void products(int T, int Z, int K, int N, const std::vector<float>& a, const std::vector<float>& u,
                     std::vector<float>& m) {
  for (int t = 0; t < T; ++t)
    for (int z = 0; z < Z; ++z)
      for (int o = 0; o < N; ++o) {
        float s = 0.f;
        for (int c = 0; c < K; ++c) s += a[((size_t)t * Z + z) * K + c] * u[((size_t)z * K + c) * N + o];
        m[((size_t)t * Z + z) * N + o] = s;
      }
}

static void run(const Case& k) {
  const int K = k.k, KK = K * K, nsub = (K + 2) / 3, nq = nsub * nsub;
  const int Ho = k.H + 2 * k.pad - (K - 1), Wo = k.W + 2 * k.pad - (K - 1), G = k.groups, Cin = G * k.cg, Cout = G * k.og;
  const WinoGeom gf{k.B, k.H, k.W, k.pad, Ho, Wo, (Ho + 3) / 4, (Wo + 3) / 4, G, K, nsub};
  const int Tf = gf.tiles();
  std::vector<float> x((size_t)k.B * k.H * k.W * Cin), dy((size_t)k.B * Ho * Wo * Cout), bias(Cout);
  std::vector<float> wf((size_t)G * KK * k.cg * k.og), wb(wf.size());
  for (auto& v : x) v = rnd();
  for (auto& v : dy) v = rnd();
  for (auto& v : bias) v = 0.3f * rnd();
  for (auto& v : wf) v = 0.2f * rnd();
  for (int g = 0; g < G; ++g)
    for (int t = 0; t < KK; ++t)
      for (int c = 0; c < k.cg; ++c)
        for (int o = 0; o < k.og; ++o)
          wb[(((size_t)g * KK + t) * k.og + o) * k.cg + c] = wf[(((size_t)g * KK + t) * k.cg + c) * k.og + o];
  auto X = [&](int n, int y, int xx, int c) -> double {
    return (y < 0 || y >= k.H || xx < 0 || xx >= k.W) ? 0.0 : x[(((size_t)n * k.H + y) * k.W + xx) * Cin + c];
  };
  auto WF = [&](int g, int r, int s, int c, int o) -> double {
    return wf[(((size_t)g * KK + r * K + s) * k.cg + c) * k.og + o];
  };
  // ---- forward ----
  std::vector<float> U((size_t)36 * nq * G * k.cg * k.og, NAN), V((size_t)Tf * 36 * nq * Cin, NAN);
  std::vector<float> m((size_t)Tf * 36 * Cout), y(dy.size(), NAN);
  for (long i = 0; i < (long)G * nq * k.cg * (k.og / 4); ++i)
    wino_filter_thread(G, k.cg, k.og, K, nsub, 0, wf.data(), U.data(), i);
  for (long i = 0; i < (long)Tf * nq * (Cin / 4); ++i) wino_in_thread(gf, k.cg, x.data(), V.data(), i);
  products(Tf, 36 * G, nq * k.cg, k.og, V, U, m);
  for (long i = 0; i < (long)Tf * (Cout / 4); ++i) wino_out_thread(gf, k.og, m.data(), bias.data(), 1, nullptr, y.data(), i);
  std::vector<double> y_ref(y.size());
  for (int n = 0; n < k.B; ++n)
    for (int oy = 0; oy < Ho; ++oy)
      for (int ox = 0; ox < Wo; ++ox)
        for (int g = 0; g < G; ++g)
          for (int o = 0; o < k.og; ++o) {
            double s = bias[g * k.og + o];
            for (int r = 0; r < K; ++r)
              for (int q = 0; q < K; ++q)
                for (int c = 0; c < k.cg; ++c) s += X(n, oy - k.pad + r, ox - k.pad + q, g * k.cg + c) * WF(g, r, q, c, o);
            y_ref[(((size_t)n * Ho + oy) * Wo + ox) * Cout + g * k.og + o] = s > 0 ? s : 0;
          }
  check("fwd", k.name, y, y_ref);
  // ---- reference of the data gradient (gated by x > 0) ----
  std::vector<double> dx_ref(x.size(), 0.0);
  for (int n = 0; n < k.B; ++n)
    for (int oy = 0; oy < Ho; ++oy)
      for (int ox = 0; ox < Wo; ++ox)
        for (int g = 0; g < G; ++g)
          for (int o = 0; o < k.og; ++o) {
            const double e = dy[(((size_t)n * Ho + oy) * Wo + ox) * Cout + g * k.og + o];
            for (int r = 0; r < K; ++r)
              for (int q = 0; q < K; ++q) {
                const int iy = oy - k.pad + r, ix = ox - k.pad + q;
                if (iy < 0 || iy >= k.H || ix < 0 || ix >= k.W) continue;
                for (int c = 0; c < k.cg; ++c)
                  dx_ref[(((size_t)n * k.H + iy) * k.W + ix) * Cin + g * k.cg + c] += e * WF(g, r, q, c, o);
              }
          }
  for (size_t i = 0; i < dx_ref.size(); ++i)
    if (!(x[i] > 0.f)) dx_ref[i] = 0;
  // ---- backward weight ----
  const int kc = nq * k.cg;  // rows of one product's result: (sub-kernel, channel)
  std::vector<float> yt((size_t)Tf * 36 * Cout), dU(U.size()), dw(wf.size(), NAN);
  for (long i = 0; i < (long)Tf * (Cout / 4); ++i) wino_dy_thread(gf, k.og, dy.data(), yt.data(), i);
  for (int z = 0; z < 36 * G; ++z)
    for (int c = 0; c < kc; ++c)
      for (int o = 0; o < k.og; ++o) {
        float s = 0.f;
        for (int t = 0; t < Tf; ++t) s += V[((size_t)t * 36 * G + z) * kc + c] * yt[((size_t)t * 36 * G + z) * k.og + o];
        dU[((size_t)z * kc + c) * k.og + o] = s;
      }
  for (long i = 0; i < (long)G * nq * k.cg * (k.og / 4); ++i)
    wino_dw_thread(G, k.cg, k.og, K, nsub, dU.data(), dw.data(), i);
  std::vector<double> dw_ref(wf.size(), 0.0);
  for (int n = 0; n < k.B; ++n)
    for (int oy = 0; oy < Ho; ++oy)
      for (int ox = 0; ox < Wo; ++ox)
        for (int g = 0; g < G; ++g)
          for (int o = 0; o < k.og; ++o) {
            const double e = dy[(((size_t)n * Ho + oy) * Wo + ox) * Cout + g * k.og + o];
            for (int r = 0; r < K; ++r)
              for (int q = 0; q < K; ++q)
                for (int c = 0; c < k.cg; ++c)
                  dw_ref[(((size_t)g * KK + r * K + q) * k.cg + c) * k.og + o] +=
                      e * X(n, oy - k.pad + r, ox - k.pad + q, g * k.cg + c);
          }
  check("bwd_weight", k.name, dw, dw_ref);
  // ---- backward data: dx = sum over patches of B [(A dy At) .* (G w Gt)] Bt, gated ----
  for (int variant = 0; variant < 4; ++variant) {
    const int CQ = variant == 0 ? 1 : 4, bands = variant < 2 ? 1 : (variant == 2 ? 2 : 3);
    if (bands > k.H) continue;
    WinoDx d{gf, k.cg, CQ, bands};
    std::vector<float> Ut(U.size(), NAN), ma((size_t)Tf * 36 * nq * Cin), dxa(x.size(), NAN);
    for (long i = 0; i < (long)G * nq * k.og * (k.cg / 4); ++i)
      wino_filter_thread(G, k.og, k.cg, K, nsub, 1, wb.data(), Ut.data(), i);
    products(Tf, 36 * G, k.og, nq * k.cg, yt, Ut, ma);
    std::vector<Vec4> lds(d.lds_vec4());  // exactly what the kernel is given
    for (int block = 0; block < d.blocks(); ++block) {
      for (auto& v : lds) v = {NAN, NAN, NAN, NAN};
      for (int tid = 0; tid < kThreads; ++tid) wino_dx_zero(d, lds.data(), tid);
      const WinoDxPlan plan = wino_dx_plan(d, block);
      std::vector<Vec2> z((size_t)kThreads * 36);
      std::vector<WinoDxTask> task(kThreads);
      for (int r = 0; r < wino_dx_rounds(d); ++r) {
        for (auto& v : z) v = {NAN, NAN};
        for (int tid = 0; tid < kThreads; ++tid) task[tid] = wino_dx_load(d, plan, ma.data(), tid, r, &z[tid * 36]);
        int ph_lo, ph_hi;
        wino_dx_round_phases(d, plan, r, &ph_lo, &ph_hi);
        for (int tid = 0; tid < kThreads; ++tid)
          if (task[tid].phase >= 0 && (task[tid].phase < ph_lo || task[tid].phase > ph_hi))
            emu_fail("a task's phase lies outside the phases its round runs");
        for (int ph = ph_lo; ph <= ph_hi; ++ph) {
          // within a phase no two threads may touch the same LDS word (on the GPU they run at once)
          std::vector<int> writer((size_t)d.lds_vec4() * 2, -1);  // one per channel pair
          const WinoDxBlock bk = plan.bk;
          for (int tid = 0; tid < kThreads; ++tid) {
            if (task[tid].phase != ph) continue;
            for (int i = 0; i < 6; ++i)
              for (int jj = 0; jj < 6; ++jj) {
                const int iy = task[tid].y0 + i, ix = task[tid].x0 + jj;
                if (iy < bk.h0 || iy >= bk.h1 || ix < 0 || ix >= d.g.W) continue;
                int& wtr = writer[((size_t)(iy - bk.h0) * d.g.W + ix) * d.lanes() + tid % d.lanes()];
                if (wtr >= 0) emu_fail("two threads add to the same LDS word in one phase");
                wtr = tid;
              }
          }
          for (int tid = 0; tid < kThreads; ++tid) wino_dx_add(d, plan, lds.data(), tid, task[tid], &z[tid * 36], ph);
        }
      }
      for (int tid = 0; tid < kThreads; ++tid) wino_dx_flush(d, plan, lds.data(), x.data(), dxa.data(), tid);
    }
    char nm[64];
    snprintf(nm, sizeof nm, "%s CQ%d b%d", k.name, CQ, bands);
    check("bwd_data", nm, dxa, dx_ref);
  }
}

int main() {
  check_1d();
  const Case cases[] = {
      {"13x13 pad1 g1", 2, 13, 13, 1, 1, 8, 12, 3},  {"13x13 pad1 g2", 2, 13, 13, 1, 2, 4, 8, 3},
      {"6x6 pad1 g2", 3, 6, 6, 1, 2, 8, 4, 3},        {"5x7 pad0 g1", 2, 5, 7, 0, 1, 4, 4, 3},
      {"4x9 pad2 g1", 1, 4, 9, 2, 1, 4, 8, 3},        {"3x3 pad1 g1", 2, 3, 3, 1, 1, 4, 4, 3},
      {"5x5: 27x27 pad2 g2", 2, 27, 27, 2, 2, 4, 8, 5}, {"5x5: 14x14 pad2 g1", 2, 14, 14, 2, 1, 8, 4, 5},
      {"5x5: 7x9 pad0 g1", 1, 7, 9, 0, 1, 4, 4, 5},     {"5x5: 6x5 pad4 g2", 2, 6, 5, 4, 2, 4, 4, 5},
  };
  for (const Case& c : cases) run(c);
  if (g_fail) {
    printf("%d FAILED\n", g_fail);
    return 1;
  }
  printf("ALL OK\n");
  return 0;
}
