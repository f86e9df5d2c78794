// The C ABI of include/alexnet.h: handle, workspace plan and the sequencing of
// one training / inference pass over the kernels of this library.
#include <stdarg.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <string>
#include <utility>
#include <vector>

#include "kernels.h"

namespace ax {

static thread_local char g_err[512] = "";
void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
}
const char* get_error() { return g_err; }

thread_local ProfSink* g_prof = nullptr;
thread_local const char* g_prof_ctx = "";

// Accumulates (event pair, work) per kernel name; elapsed times are read in finish().
struct Profiler : ProfSink {
  struct Entry {
    std::string name;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> ev;
    double flops = 0, bytes = 0;
  };
  std::vector<Entry> entries;
  Entry* cur = nullptr;
  bool failed = false;
  void begin(const char* kernel, double flops, double bytes, hipStream_t st) override {
    std::string nm = std::string(g_prof_ctx) + (g_prof_ctx[0] ? ":" : "") + kernel;
    cur = nullptr;
    for (auto& e : entries)
      if (e.name == nm) cur = &e;
    if (!cur) {
      entries.emplace_back();
      cur = &entries.back();
      cur->name = nm;
    }
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess || hipEventRecord(a, st) != hipSuccess) {
      failed = true;
      cur = nullptr;
      return;
    }
    cur->ev.emplace_back(a, b);
    cur->flops += flops;
    cur->bytes += bytes;
  }
  void end(hipStream_t st) override {
    if (cur && hipEventRecord(cur->ev.back().second, st) != hipSuccess) failed = true;
    cur = nullptr;
  }
  ~Profiler() override {
    for (auto& e : entries)
      for (auto& p : e.ev) {
        (void)hipEventDestroy(p.first);
        (void)hipEventDestroy(p.second);
      }
  }
};
static thread_local Profiler* g_profiler = nullptr;

static const int kStages = 5, kFc = 3, kSlots = 3;  // slot 2 is the inference input
static_assert(kMaxColsumJobs >= kStages + kFc, "one bias-gradient job per layer");
static_assert(kMaxWgradJobs >= kStages, "one weight-gradient tail per stage");

struct Stage {
  ConvGeom g;
  bool lrn, pool;
  bool fused_ok;        // normalisation and pool run as one kernel, forward and backward
  int Hp, Wp;           // stage output size (after the pool when present)
  size_t w_off, b_off;  // offsets into the flat parameter vector
  float *act, *lrn_out, *pool_out, *dact, *d_lrn, *d_out, *wb;
  float *wino_du, *wino_slices;  // weight-gradient products and their split-k slices (transformed stages)
  float* wphase;        // weights regrouped by phase for a strided backward-data pass (null when not used)
  // 3x3 unit-stride stages run through the F(4x4, 3x3) transforms: the transformed input of the forward pass
  // (kept for the weight gradient) and the transformed taps of the forward and backward-data passes
  bool wino;     // forward and weight gradient
  bool wino_bx;  // data gradient too
  float *wino_v, *wino_u, *wino_ub;
  float *wrun, *dwrun;  // run-mode copies of the weights and their gradient (null when not used)
  // bf16 handles: copies in bf16 (nearest even) of the stage's GEMM operands -- input, output gradient, and the
  // forward and backward-data weights with the reduction contiguous, wf16[g][o][(r,s,c)], wb16[g][c][(r,s,o)] --
  // which the products then read instead of rounding fp32 values on the fly
  bool b16;
  uint16_t *x16, *dy16, *wf16, *wb16;
  // bf16 handles, first layer (three-channel pictures): the pictures as bf16 with four channels per pixel and the
  // weights for that view (conv_plan.h, run16); x16 then holds the padded pictures, wf16 those weights
  bool r16;
  uint16_t* x16_own;  // the stage's own x16; in a training or inference pass the first layer's x16 points at the
                      // padded copy that preprocessing left beside the input slot instead
  uint8_t* slot;
  char lab[4][16];  // profiling labels: stage, .fwd, .bwd_w, .bwd_x
  long act_elems() const { return g.out_elems(); }
  long out_elems() const { return (long)g.B * Hp * Wp * g.Cout; }
  const float* out() const { return pool ? pool_out : lrn ? lrn_out : act; }
  bool plain() const { return !lrn && !pool; }
  bool fused() const { return fused_ok; }
};
struct Dense {
  int in, out;
  size_t w_off, b_off;
  float *act, *dz;
  uint16_t *act16, *dz16;  // bf16 copies for the products of a bf16 handle (null otherwise)
  char lab[4][16];
};

// Bump allocator over the caller's workspace; with base == null it only sizes.
struct Arena {
  char* base;
  size_t off;
  template <class T>
  T* take(size_t n) {
    off = (off + 255) & ~(size_t)255;
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += n * sizeof(T);
    return p;
  }
};

}  // namespace ax

using namespace ax;

struct alexnet {
  alexnet_config_t cfg;
  Stage st[kStages];
  Dense fc[kFc];
  size_t n_params, n_weights, ws_bytes;
  float *params, *mom, *grads;
  float* input[kSlots];
  uint16_t* input16[kSlots];  // bf16 handles whose first layer takes them: the inputs with four channels per pixel
  // bf16 handles whose dense shapes allow it: the dense layers' products read bf16 copies of their operands --
  // all dense weights (same order and layout as in the parameter vector, made anew from it in every pass) and
  // the flattened output of the last stage; Dense holds the copies of the activations and their gradients
  bool fc16;
  uint16_t *fcw16, *flat16;
  int32_t *crop_x[kSlots], *crop_y[kSlots], *flip[kSlots];
  float *gemm_ws, *colsum_ws, *row_loss, *scratch_x, *scratch_y, *scratch_w[3];
  float *wino_a, *wino_m, *wino_du;  // transformed operand / product / tap-gradient scratch shared by the stages
  int32_t* err_flag;
  size_t gemm_ws_floats, colsum_ws_floats_;
  int flat;  // flatten size feeding fc6
  // the dense-layer update starts on the side stream in this stage of the backward pass, just before its
  // weight gradient (behind its pooling adjoint) or just before its data gradient
  int upd_fork_stage;
  bool upd_fork_before_bx;
  // The dense layers hold 96 % of the parameters and finish their backward pass first: their update, which is
  // bound by memory bandwidth, runs on this stream under the convolution backward pass, which is not.
  hipStream_t upd_stream;
  hipEvent_t ev_fc_done, ev_upd_done, ev_step_begin, ev_wb_done, ev_u_done, ev_fcw_done;
};

// F(4x4, 3x3) pays when the 4x4 tiles cover the output without much waste (2.6x fewer multiplies for the 3x3
// layers at 13 x 13 and for the 5x5 layer, as four 3x3 sub-kernels, at 27 x 27);
// ALEXNET_FLAG_DIRECT_CONV in the configuration keeps every stage on the direct implicit GEMM.
static bool use_winograd(const alexnet_config_t& c, const ConvGeom& g) {
  if (c.precision != ALEXNET_PRECISION_FP32 || !wino_ok(g)) return false;
  if (c.flags & ALEXNET_FLAG_DIRECT_CONV) return false;
  return wino_gain(g) >= 1.5;
}

static int plan(alexnet* n, const alexnet_config_t* cfg, char* base) {
  const alexnet_config_t& c = *cfg;
  if (c.batch <= 0 || c.in_c <= 0 || c.crop_h <= 0 || c.crop_w <= 0 || c.raw_h < c.crop_h || c.raw_w < c.crop_w) {
    set_error("bad batch/input size");
    return ALEXNET_ESHAPE;
  }
  if (c.precision != ALEXNET_PRECISION_FP32 && c.precision != ALEXNET_PRECISION_BF16) {
    set_error("precision %d is not available (0: fp32, 1: bf16 products with fp32 accumulation)", c.precision);
    return ALEXNET_ENOTIMPL;
  }
  if (c.flags & ~ALEXNET_FLAG_DIRECT_CONV) {
    set_error("unknown bits in flags: 0x%x", (unsigned)c.flags);
    return ALEXNET_EINVAL;
  }
  if (c.lrn_n < 1 || c.lrn_n % 2 == 0 || !(c.dropout_p >= 0.f && c.dropout_p < 1.f)) {
    set_error("bad lrn_n (must be odd) or dropout_p");
    return ALEXNET_EINVAL;
  }
  n->cfg = c;
  int C = c.in_c, H = c.crop_h, W = c.crop_w;
  size_t off = 0;
  for (int i = 0; i < kStages; ++i) {
    const alexnet_conv_t& cv = c.conv[i];
    if (cv.cout <= 0 || cv.k <= 0 || cv.stride <= 0 || cv.pad < 0 || cv.groups <= 0 || C % cv.groups ||
        cv.cout % cv.groups) {
      set_error("conv%d: bad hyper-parameters", i + 1);
      return ALEXNET_ESHAPE;
    }
    Stage& s = n->st[i];
    s.g.B = c.batch; s.g.H = H; s.g.W = W; s.g.Cin = C; s.g.Cout = cv.cout; s.g.k = cv.k;
    s.g.stride = cv.stride; s.g.pad = cv.pad; s.g.groups = cv.groups;
    s.g.Ho = (H + 2 * cv.pad - cv.k) / cv.stride + 1;
    s.g.Wo = (W + 2 * cv.pad - cv.k) / cv.stride + 1;
    if (H + 2 * cv.pad < cv.k || W + 2 * cv.pad < cv.k || s.g.Ho <= 0 || s.g.Wo <= 0) {
      set_error("conv%d: kernel larger than its input", i + 1);
      return ALEXNET_ESHAPE;
    }
    s.lrn = cv.lrn != 0;
    s.pool = cv.pool != 0;
    s.Hp = s.g.Ho; s.Wp = s.g.Wo;
    if (s.pool) {
      if (s.g.Ho < 3 || s.g.Wo < 3) {
        set_error("conv%d: output too small to pool", i + 1);
        return ALEXNET_ESHAPE;
      }
      s.Hp = (s.g.Ho - 3) / 2 + 1;
      s.Wp = (s.g.Wo - 3) / 2 + 1;
    }
    if (s.g.in_elems() > 0x1ffffff0L || s.g.out_elems() > 0x1ffffff0L || s.g.w_elems() > 0x1ffffff0L) {
      set_error("conv%d: a tensor reaches 2 GiB; byte offsets in the kernels are 32-bit", i + 1);
      return ALEXNET_ESHAPE;
    }
    snprintf(s.lab[0], 16, "conv%d", i + 1);
    snprintf(s.lab[1], 16, "conv%d.fwd", i + 1);
    snprintf(s.lab[2], 16, "conv%d.bwd_w", i + 1);
    snprintf(s.lab[3], 16, "conv%d.bwd_x", i + 1);
    s.w_off = off;
    off += (size_t)s.g.w_elems();
    C = cv.cout; H = s.Hp; W = s.Wp;
  }
  n->flat = C * H * W;
  int in = n->flat;
  n->upd_fork_stage = kStages - 1;
  for (int j = 0; j < kFc; ++j) {
    if (c.fc[j] <= 0) {
      set_error("fc width must be positive");
      return ALEXNET_ESHAPE;
    }
    if ((long)in * c.fc[j] > 0x1ffffff0L || (long)c.batch * in > 0x1ffffff0L || (long)c.batch * c.fc[j] > 0x1ffffff0L) {
      set_error("fc%d: a tensor reaches 2 GiB; byte offsets in the kernels are 32-bit", kStages + 1 + j);
      return ALEXNET_ESHAPE;
    }
    n->fc[j].in = in; n->fc[j].out = c.fc[j];
    snprintf(n->fc[j].lab[0], 16, "fc%d", kStages + 1 + j);
    snprintf(n->fc[j].lab[1], 16, "fc%d.fwd", kStages + 1 + j);
    snprintf(n->fc[j].lab[2], 16, "fc%d.bwd_w", kStages + 1 + j);
    snprintf(n->fc[j].lab[3], 16, "fc%d.bwd_x", kStages + 1 + j);
    n->fc[j].w_off = off;
    off += (size_t)in * c.fc[j];
    in = c.fc[j];
  }
  n->n_weights = off;
  for (int i = 0; i < kStages; ++i) { n->st[i].b_off = off; off += n->st[i].g.Cout; }
  for (int j = 0; j < kFc; ++j) { n->fc[j].b_off = off; off += n->fc[j].out; }
  n->n_params = off;

  // ---- workspace ----
  Arena a{base, 0};
  const size_t in_elems = (size_t)c.batch * c.crop_h * c.crop_w * c.in_c;
  for (int s = 0; s < kSlots; ++s) {
    n->input[s] = a.take<float>(in_elems);
    n->crop_x[s] = a.take<int32_t>(c.batch);
    n->crop_y[s] = a.take<int32_t>(c.batch);
    n->flip[s] = a.take<int32_t>(c.batch);
  }
  size_t max_in = in_elems, max_out = 0, max_w = 0, gws = 0, cws = 0, cws_batch = 0, wscr = 0, wdu = 0;
  for (int i = 0; i < kStages; ++i) {
    Stage& s = n->st[i];
    const size_t ae = s.act_elems(), oe = s.out_elems();
    s.act = a.take<float>(ae);
    s.dact = a.take<float>(ae);
    s.lrn_out = s.lrn ? a.take<float>(ae) : nullptr;
    s.pool_out = s.pool ? a.take<float>(oe) : nullptr;
    s.slot = s.pool ? a.take<uint8_t>(oe) : nullptr;
    s.d_lrn = (s.lrn && s.pool) ? a.take<float>(ae) : nullptr;
    s.d_out = s.plain() ? s.dact : a.take<float>(oe);
    s.fused_ok = s.lrn && s.pool && base &&
                 lrn_pool_fused_ok(s.act, s.pool_out, s.d_out, s.dact, s.slot, s.g.Cout, c.lrn_n);
    s.wb = a.take<float>(s.g.w_elems());
    s.wphase = conv_phase_mode(s.g) ? a.take<float>(conv_phase_w_floats(s.g)) : nullptr;
    s.wrun = conv_run_mode(s.g) ? a.take<float>(conv_run_w_floats(s.g)) : nullptr;
    s.dwrun = conv_run_mode(s.g) ? a.take<float>(conv_run_w_floats(s.g)) : nullptr;
    s.b16 = c.precision == ALEXNET_PRECISION_BF16 && conv_bf16_stored_ok(s.g) && s.w_off % 4 == 0;
    s.r16 = c.precision == ALEXNET_PRECISION_BF16 && !s.b16 && conv_run16_ok(s.g) && s.w_off % 4 == 0;
    s.x16 = s.b16 ? a.take<uint16_t>(s.g.in_elems()) : s.r16 ? a.take<uint16_t>(conv_run16_x_elems(s.g)) : nullptr;
    s.x16_own = s.x16;
    s.dy16 = s.b16 ? a.take<uint16_t>(ae) : nullptr;
    s.wf16 = s.b16 ? a.take<uint16_t>(s.g.w_elems()) : s.r16 ? a.take<uint16_t>(conv_run16_w_elems(s.g)) : nullptr;
    s.wb16 = s.b16 ? a.take<uint16_t>(s.g.w_elems()) : nullptr;
    s.wino = use_winograd(c, s.g) && s.w_off % 4 == 0 && s.b_off % 4 == 0;
    s.wino_bx = s.wino && wino_bwd_data_ok(s.g);
    s.wino_v = s.wino ? a.take<float>(wino_v_floats(s.g)) : nullptr;
    s.wino_u = s.wino ? a.take<float>(wino_u_floats(s.g)) : nullptr;
    s.wino_ub = s.wino_bx ? a.take<float>(wino_u_floats(s.g)) : nullptr;
    // the products of the weight gradient and their split-k slices, kept until the end of the backward pass
    s.wino_du = s.wino ? a.take<float>(wino_u_floats(s.g)) : nullptr;
    s.wino_slices = s.wino && wino_wgrad_ws_floats(s.g) ? a.take<float>(wino_wgrad_ws_floats(s.g)) : nullptr;
    if (s.wino) {
      wscr = std::max(wscr, wino_scratch_floats(s.g));
      wdu = std::max(wdu, wino_u_floats(s.g));
      gws = std::max(gws, wino_gemm_ws_floats(s.g));
    }
    max_in = std::max(max_in, (size_t)s.g.in_elems());
    max_out = std::max(max_out, ae);
    max_w = std::max(max_w, (size_t)s.g.w_elems());
    gws = std::max(gws, conv_bwd_weight_ws_floats(s.g));
    gws = std::max(gws, conv_fwd_ws_floats(s.g));
    gws = std::max(gws, conv_bwd_data_ws_floats(s.g));
    cws = std::max(cws, colsum_ws_floats(s.g.P(), s.g.Cout));
    cws_batch += colsum_batch_ws_floats(s.g.P(), s.g.Cout);
    if (s.lrn && s.pool) {
      cws = std::max(cws, lrn_part_floats(s.g.Cout));
      cws_batch += lrn_part_floats(s.g.Cout);
    }
  }
  {
    // The dense-layer update shares the chip best with a direct fp32 convolution GEMM of the backward pass, the
    // largest one: the transformed layers move several times their activations and compete with it for
    // bandwidth, and so do the bf16 products (those keep the fork behind the last stage, the earliest possible).
    double best = -1;
    n->upd_fork_before_bx = false;
    for (int i = 0; i < kStages && c.precision == ALEXNET_PRECISION_FP32; ++i) {
      const Stage& s = n->st[i];
      const double fl = (double)s.g.P() * s.g.Cout * s.g.cg() * s.g.k * s.g.k;
      if (!s.wino && fl > best) {
        best = fl;
        n->upd_fork_stage = i;
        n->upd_fork_before_bx = false;
      }
      if (i > 0 && !s.wino_bx && fl > best) {
        best = fl;
        n->upd_fork_stage = i;
        n->upd_fork_before_bx = s.wino;  // behind a transformed weight gradient, else before both GEMMs
      }
    }
  }
  n->fc16 = c.precision == ALEXNET_PRECISION_BF16 && n->fc[0].w_off % 4 == 0;
  for (int j = 0; j < kFc; ++j) n->fc16 = n->fc16 && fc_bf16_stored_ok(n->fc[j].in, n->fc[j].out);
  n->fcw16 = n->fc16 ? a.take<uint16_t>(n->n_weights - n->fc[0].w_off) : nullptr;
  n->flat16 = n->fc16 ? a.take<uint16_t>((size_t)c.batch * n->flat) : nullptr;
  for (int j = 0; j < kFc; ++j) {
    Dense& f = n->fc[j];
    f.act = a.take<float>((size_t)c.batch * f.out);
    f.dz = a.take<float>((size_t)c.batch * f.out);
    f.act16 = n->fc16 ? a.take<uint16_t>((size_t)c.batch * f.out) : nullptr;
    f.dz16 = n->fc16 ? a.take<uint16_t>((size_t)c.batch * f.out) : nullptr;
    gws = std::max(gws, fc_ws_floats(c.batch, f.in, f.out));
    cws = std::max(cws, colsum_ws_floats(c.batch, f.out));
    cws_batch += colsum_batch_ws_floats(c.batch, f.out);
  }
  for (int sl = 0; sl < kSlots; ++sl)
    n->input16[sl] = n->st[0].r16 ? a.take<uint16_t>(conv_run16_x_elems(n->st[0].g)) : nullptr;
  n->grads = a.take<float>(n->n_params);
  n->wino_a = wscr ? a.take<float>(wscr) : nullptr;
  n->wino_m = wscr ? a.take<float>(wscr) : nullptr;
  n->wino_du = wdu ? a.take<float>(wdu) : nullptr;
  n->gemm_ws = a.take<float>(gws);
  n->gemm_ws_floats = gws;
  cws = std::max(cws, cws_batch);  // the backward pass sums all its bias gradients in one batch
  n->colsum_ws = a.take<float>(cws);
  n->colsum_ws_floats_ = cws;
  n->row_loss = a.take<float>(c.batch);
  n->err_flag = a.take<int32_t>(64);
  n->scratch_x = a.take<float>(max_in);
  n->scratch_y = a.take<float>(max_out);
  for (int k = 0; k < 3; ++k) n->scratch_w[k] = a.take<float>(max_w);
  n->ws_bytes = (a.off + 255) & ~(size_t)255;
  return ALEXNET_OK;
}

static inline hipStream_t S(void* s) { return reinterpret_cast<hipStream_t>(s); }
static inline bool aligned256(const void* p) { return ((uintptr_t)p & 255) == 0; }

#define REQUIRE(cond, code, msg)   \
  do {                             \
    if (!(cond)) {                 \
      ax::set_error("%s", msg);    \
      return code;                 \
    }                              \
  } while (0)

static uint32_t drop_thresh(float p) { return (uint32_t)floor((double)p * (double)(1 << 24)); }

// ---- one convolution stage, by the F(4x4, 3x3) path when the stage has one and the tensors allow 16-byte access ----
static bool wino_usable(const Stage& s, const void* a, const void* b, const void* c, const void* d = nullptr) {
  return s.wino && aligned16(a) && aligned16(b) && aligned16(c) && aligned16(d);
}
// bf16 handles, stages whose operands have bf16 copies: true when this call can use them
static bool b16_usable(const Stage& s, const void* a, const void* b) { return s.b16 && aligned16(a) && aligned16(b); }

// taps_ready: the forms of wf that the stage multiplies with are in place already (s.wino_u, the transform of wf;
// s.wf16, its bf16 copy)
// x16_ready: s.x16 already holds the bf16 copy of x (the kernel that made x wrote it);
// y16 (may be null): where to leave a bf16 copy of y for the stage that reads y next
static int stage_fwd(alexnet* n, Stage& s, const float* x, const float* wf, const float* bias, int relu, float* y,
                     bool taps_ready, hipStream_t st, bool x16_ready = false, uint16_t* y16 = nullptr) {
  if (wino_usable(s, x, wf, y, bias)) {
    if (!taps_ready) AX_TRY(launch_wino_filter(s.g, wf, s.wino_u, st));
    AX_TRY(launch_wino_fwd(s.g, x, s.wino_u, bias, relu, y, s.wino_v, n->wino_m, n->gemm_ws, st));
    return y16 ? launch_to_bf16(y, y16, (size_t)s.g.out_elems(), st) : ALEXNET_OK;
  }
  if (b16_usable(s, x, wf)) {
    if (!x16_ready) AX_TRY(launch_to_bf16(x, s.x16, (size_t)s.g.in_elems(), st));
    if (!taps_ready) AX_TRY(launch_to_bf16_transposed(wf, s.wf16, s.g.groups, s.g.kf(), s.g.og(), st));
    return launch_conv_fwd(s.g, x, wf, nullptr, bias, relu, y, n->gemm_ws, st, s.x16, s.wf16, y16);
  }
  if (s.r16) {  // x16_ready: s.x16 holds the pictures padded to four channels
    if (!x16_ready) AX_TRY(launch_pad4_bf16(x, s.x16, (size_t)s.g.Q(), s.g.Cin, st));
    if (!taps_ready) AX_TRY(launch_run16_pack(wf, s.wf16, s.g.k, s.g.Cin, (int)(conv_run16_w_elems(s.g) / ((size_t)s.g.k * s.g.Cout)), s.g.Cout, st));
    return launch_conv_fwd_run16(s.g, s.x16, s.wf16, bias, relu, y, n->gemm_ws, st, y16);
  }
  if (s.wrun) AX_TRY(launch_conv_run_pack(s.g, wf, s.wrun, st));
  return launch_conv_fwd(s.g, x, wf, s.wrun, bias, relu, y, n->gemm_ws, st, nullptr, nullptr, y16);
}
// have_v: the forward pass of the same minibatch left its form of x in place (s.wino_v, the transform of x; s.x16,
// its bf16 copy)
// tail: put the end of a transformed stage's weight gradient off to launch_wgrad_tail() (see WgradTail)
// dy16_ready: s.dy16 already holds the bf16 copy of dy (the kernel that made dy wrote it)
static int stage_bwd_weight(alexnet* n, Stage& s, const float* x, const float* dy, float* dwf, bool have_v,
                            hipStream_t st, WgradTail* tail = nullptr, bool dy16_ready = false) {
  if (wino_usable(s, x, dy, dwf)) {
    if (!have_v) AX_TRY(launch_wino_input(s.g, x, s.wino_v, st));
    if (tail) return launch_wino_bwd_weight(s.g, s.wino_v, dy, dwf, n->wino_a, s.wino_du, s.wino_slices, st, tail);
    return launch_wino_bwd_weight(s.g, s.wino_v, dy, dwf, n->wino_a, n->wino_du, n->gemm_ws, st);
  }
  if (b16_usable(s, x, dy)) {
    if (!have_v) AX_TRY(launch_to_bf16(x, s.x16, (size_t)s.g.in_elems(), st));
    if (!dy16_ready) AX_TRY(launch_to_bf16(dy, s.dy16, (size_t)s.g.out_elems(), st));
    return launch_conv_bwd_weight(s.g, x, dy, dwf, nullptr, n->gemm_ws, st, nullptr, s.x16, s.dy16);
  }
  return launch_conv_bwd_weight(s.g, x, dy, dwf, s.dwrun, n->gemm_ws, st);
}
// taps_ready: the forms of wb are in place (s.wino_ub; s.wb16); yt_ready: so is that of dy (n->wino_a, the
// transformed output gradient; s.dy16): stage_bwd_weight of the same minibatch ran just before
// dx16 (may be null): where to leave a bf16 copy of dx for the stage below
static int stage_bwd_data(alexnet* n, Stage& s, const float* dy, const float* wf, const float* wb, float* wphase,
                          const float* gate, float* dx, bool taps_ready, bool yt_ready, hipStream_t st,
                          uint16_t* dx16 = nullptr) {
  if (s.wino_bx && wino_usable(s, dy, wb, dx, gate)) {
    if (!taps_ready) AX_TRY(launch_wino_filter_bwd(s.g, wb, s.wino_ub, st));
    if (!yt_ready) AX_TRY(launch_wino_output_grad(s.g, dy, n->wino_a, st));
    AX_TRY(launch_wino_bwd_data(s.g, n->wino_a, s.wino_ub, gate, dx, n->wino_m, n->gemm_ws, st));
    return dx16 ? launch_to_bf16(dx, dx16, (size_t)s.g.in_elems(), st) : ALEXNET_OK;
  }
  if (b16_usable(s, dy, wb)) {
    if (!yt_ready) AX_TRY(launch_to_bf16(dy, s.dy16, (size_t)s.g.out_elems(), st));
    if (!taps_ready) AX_TRY(launch_to_bf16_transposed(wb, s.wb16, s.g.groups, s.g.kb(), s.g.cg(), st));
    return launch_conv_bwd_data(s.g, dy, wf, wb, nullptr, gate, dx, n->gemm_ws, st, s.dy16, s.wb16, dx16);
  }
  return launch_conv_bwd_data(s.g, dy, wf, wb, wphase, gate, dx, n->gemm_ws, st, nullptr, nullptr, dx16);
}

// --------------------------------------------------------------- passes ------
// taps_ready: recorded on another stream once every stage's transformed forward taps are in place (null: they
// are made here)
// in16: the padded bf16 copy of `in` that preprocessing left (bf16 handles; null: the first layer makes its own)
// fcw_ready: recorded on another stream once the bf16 copy of the dense weights is in place (null: made here)
static int fcw16_refresh(alexnet* n, hipStream_t st) {
  return launch_to_bf16(n->params + n->fc[0].w_off, n->fcw16, n->n_weights - n->fc[0].w_off, st);
}
static int run_forward(alexnet* n, const float* in, bool train, uint64_t step, hipStream_t st,
                       hipEvent_t taps_ready = nullptr, uint16_t* in16 = nullptr, hipEvent_t fcw_ready = nullptr) {
  const alexnet_config_t& c = n->cfg;
  set_gemm_precision(c.precision);
  if (n->fc16 && !fcw_ready) AX_TRY(fcw16_refresh(n, st));
  const float* h = in;
  bool waited = false;
  bool x16_ready = false;  // the kernel that made h also left its bf16 copy in the next stage's x16
  n->st[0].x16 = n->st[0].x16_own;
  if (in16 && n->st[0].r16) {
    n->st[0].x16 = in16;
    x16_ready = true;
  }
  for (int i = 0; i < kStages; ++i) {
    Stage& s = n->st[i];
    // bf16 handles: whoever writes this stage's output also writes the bf16 copy the next stage multiplies with
    uint16_t* next16 = i + 1 == kStages ? n->flat16 : n->st[i + 1].b16 ? n->st[i + 1].x16 : nullptr;
    {
      ProfContext pc(s.lab[1]);
      if ((s.wino || s.b16 || s.r16) && taps_ready && !waited) {
        AX_HIP(hipStreamWaitEvent(st, taps_ready, 0));
        waited = true;
      }
      AX_TRY(stage_fwd(n, s, h, n->params + s.w_off, n->params + s.b_off, 1, s.act, taps_ready != nullptr, st,
                       x16_ready, s.plain() ? next16 : nullptr));
    }
    x16_ready = s.plain() && next16 != nullptr;
    ProfContext pc(s.lab[0]);
    h = s.act;
    if (s.fused()) {  // normalise and pool in one pass; the normalised tensor is only made on request
      AX_TRY(launch_lrn_pool_fwd(s.act, s.pool_out, s.slot, s.g.B, s.g.Ho, s.g.Wo, s.g.Cout, s.Hp, s.Wp, c.lrn_n,
                                 c.lrn_k, c.lrn_alpha, c.lrn_beta, st, next16));
      x16_ready = next16 != nullptr;
      h = s.pool_out;
      continue;
    }
    if (s.lrn) {
      AX_TRY(launch_lrn_fwd(s.act, s.lrn_out, s.g.P(), s.g.Cout, c.lrn_n, c.lrn_k, c.lrn_alpha, c.lrn_beta, st));
      h = s.lrn_out;
      x16_ready = false;
    }
    if (s.pool) {
      AX_TRY(launch_pool_fwd(h, s.pool_out, s.slot, s.g.B, s.g.Ho, s.g.Wo, s.g.Cout, s.Hp, s.Wp, st, next16));
      x16_ready = next16 != nullptr;
      h = s.pool_out;
    }
  }
  if (n->fc16) {
    if (!x16_ready) AX_TRY(launch_to_bf16(h, n->flat16, (size_t)c.batch * n->flat, st));
    if (fcw_ready) AX_HIP(hipStreamWaitEvent(st, fcw_ready, 0));
  }
  const uint16_t* h16 = n->flat16;
  const uint64_t key = step_key(c.seed, step);
  for (int j = 0; j < kFc; ++j) {
    Dense& f = n->fc[j];
    FcAct act;
    act.bias = n->params + f.b_off;
    const bool hidden = j < kFc - 1;
    act.relu = hidden ? 1 : 0;
    act.dropout = (hidden && train && c.dropout_p > 0.f) ? 1 : 0;
    act.key = key;
    act.tag = j == 0 ? TAG_DROP6 : TAG_DROP7;
    act.thresh24 = drop_thresh(c.dropout_p);
    act.scale = (hidden && !train) ? 1.0f - c.dropout_p : 1.0f;
    ProfContext pc(f.lab[1]);
    AX_TRY(launch_fc_fwd(c.batch, f.in, f.out, h, n->params + f.w_off, act, f.act, n->gemm_ws, st, h16,
                         n->fc16 ? n->fcw16 + (f.w_off - n->fc[0].w_off) : nullptr, f.act16));
    h = f.act;
    h16 = f.act16;
  }
  return ALEXNET_OK;
}

static int update_range(alexnet* n, size_t begin, size_t end, hipStream_t st) {
  const alexnet_config_t& c = n->cfg;
  if (end <= begin) return ALEXNET_OK;
  const size_t decayed = n->n_weights > begin ? std::min(n->n_weights, end) - begin : 0;
  // Beside the bf16 products, which lean on the memory system themselves, the update is held to one workgroup
  // per CU: it still ends well inside the convolution backward pass, and the step is about 1.5 % shorter.
  return launch_sgd_update(n->params + begin, n->mom + begin, n->grads + begin, end - begin, decayed, c.lr, c.momentum,
                           c.weight_decay, st, c.precision == ALEXNET_PRECISION_BF16 ? 256u : 0u);
}

// early_update: also start the update of the dense-layer weights on the side stream as soon as the dense
// layers' backward pass is done (the caller updates the rest and joins, see alexnet_train_step)
static int run_backward(alexnet* n, const float* in, hipStream_t st, bool early_update = false) {
  const alexnet_config_t& c = n->cfg;
  set_gemm_precision(c.precision);
  // Bias gradients (column sums of every layer's output gradient) not made by a fused kernel on the way are
  // collected and summed in two launches at the end: those tensors all outlive the pass, and eight small
  // reductions of their own cost more in launches than in work.
  ColsumBatch bias_sums;
  size_t bias_ws_used = 0;
  // Likewise the end of every transformed stage's weight gradient (slices added up, products back to taps).
  WgradTail wgrad_tail;
  // dense layers, last to first
  for (int j = kFc - 1; j >= 0; --j) {
    Dense& f = n->fc[j];
    const float* x = j == 0 ? n->st[kStages - 1].out() : n->fc[j - 1].act;
    const uint16_t* x16 = j == 0 ? n->flat16 : n->fc[j - 1].act16;
    const uint16_t* w16 = n->fc16 ? n->fcw16 + (f.w_off - n->fc[0].w_off) : nullptr;
    {
      ProfContext pc(f.lab[2]);
      AX_TRY(launch_fc_bwd_weight(c.batch, f.in, f.out, x, f.dz, n->grads + f.w_off, st, x16, f.dz16));
      AX_TRY(colsum_batch_add(bias_sums, f.dz, c.batch, f.out, n->grads + f.b_off, n->colsum_ws, &bias_ws_used));
    }
    ProfContext pc(f.lab[3]);
    if (j > 0) {
      // fc(j-1) output is ReLU+dropout: it is positive exactly where the gradient passes
      AX_TRY(launch_fc_bwd_data(c.batch, f.in, f.out, f.dz, n->params + f.w_off, n->fc[j - 1].act, n->fc[j - 1].dz,
                                n->gemm_ws, st, f.dz16, w16, n->fc[j - 1].dz16));
    } else {
      Stage& last = n->st[kStages - 1];
      AX_TRY(launch_fc_bwd_data(c.batch, f.in, f.out, f.dz, n->params + f.w_off, last.plain() ? last.act : nullptr,
                                last.d_out, n->gemm_ws, st, f.dz16, w16, nullptr));
    }
  }
  bool dy16_ready = false;  // the kernel that made this stage's output gradient also left its bf16 copy in s.dy16
  for (int i = kStages - 1; i >= 0; --i) {
    Stage& s = n->st[i];
    ProfContext pc0(s.lab[0]);
    bool bias_done = false;
    uint16_t* own16 = s.b16 ? s.dy16 : nullptr;
    if (s.fused()) {  // pool adjoint, normalisation adjoint, ReLU gate and the bias gradient's partial sums in one pass
      // the kernel leaves one row of sums per workgroup; those rows are one more matrix for the batch at the end
      float* part = n->colsum_ws + bias_ws_used;
      const size_t part_rows = lrn_part_rows(s.g.P(), s.g.Cout);
      bias_ws_used += (part_rows * s.g.Cout + 3) / 4 * 4;
      if (bias_ws_used > n->colsum_ws_floats_) {
        set_error("bias gradients: partial sums do not fit their workspace");
        return ALEXNET_EINVAL;
      }
      AX_TRY(launch_pool_lrn_bwd(s.act, s.d_out, s.slot, s.dact, s.g.B, s.g.Ho, s.g.Wo, s.g.Cout, s.Hp, s.Wp, c.lrn_n,
                                 c.lrn_k, c.lrn_alpha, c.lrn_beta, 1, nullptr, part, st, true, own16));
      dy16_ready = own16 != nullptr;
      AX_TRY(colsum_batch_add(bias_sums, part, (long)part_rows, s.g.Cout, n->grads + s.b_off, n->colsum_ws,
                              &bias_ws_used));
      bias_done = true;
    } else if (s.pool) {
      if (s.lrn)
        AX_TRY(launch_pool_bwd(s.d_out, s.slot, nullptr, s.d_lrn, s.g.B, s.g.Ho, s.g.Wo, s.g.Cout, s.Hp, s.Wp, st));
      else
      {
        AX_TRY(launch_pool_bwd(s.d_out, s.slot, s.act, s.dact, s.g.B, s.g.Ho, s.g.Wo, s.g.Cout, s.Hp, s.Wp, st, own16));
        dy16_ready = own16 != nullptr;
      }
    }
    if (s.lrn && !s.fused()) {
      AX_TRY(launch_lrn_bwd(s.act, s.pool ? s.d_lrn : s.d_out, s.dact, s.g.P(), s.g.Cout, c.lrn_n, c.lrn_k,
                            c.lrn_alpha, c.lrn_beta, 1, st));
      dy16_ready = false;
    }
    // Fork of the dense-layer update (see upd_fork_stage), never in front of this stage's pooling adjoint: that
    // kernel is bound by bandwidth like the update and would be starved by it.
    auto fork_update = [&]() -> int {
      AX_HIP(hipEventRecord(n->ev_fc_done, st));
      AX_HIP(hipStreamWaitEvent(n->upd_stream, n->ev_fc_done, 0));
      AX_TRY(update_range(n, n->fc[0].w_off, n->n_weights, n->upd_stream));
      AX_HIP(hipEventRecord(n->ev_upd_done, n->upd_stream));
      return ALEXNET_OK;
    };
    const bool fork_here = early_update && i == n->upd_fork_stage;
    if (fork_here && !n->upd_fork_before_bx) AX_TRY(fork_update());
    const float* x = i == 0 ? in : n->st[i - 1].out();
    {
      ProfContext pc(s.lab[2]);
      AX_TRY(stage_bwd_weight(n, s, x, s.dact, n->grads + s.w_off, true, st, &wgrad_tail, dy16_ready));
      if (!bias_done)
        AX_TRY(colsum_batch_add(bias_sums, s.dact, s.g.P(), s.g.Cout, n->grads + s.b_off, n->colsum_ws, &bias_ws_used));
    }
    if (fork_here && n->upd_fork_before_bx) AX_TRY(fork_update());
    if (i > 0) {
      ProfContext pc(s.lab[3]);
      Stage& prev = n->st[i - 1];
      if (early_update) {  // the side stream re-packed the weights during the forward pass
        if (i == kStages - 1) AX_HIP(hipStreamWaitEvent(st, n->ev_wb_done, 0));
      } else {
        AX_TRY(launch_conv_weight_wb(n->params + s.w_off, s.wb, s.g.Cout, s.g.cg(), s.g.k, s.g.groups, st));
      }
      // a stage below without LRN or pool takes this data gradient as its output gradient as it is
      uint16_t* below16 = (prev.plain() && prev.b16) ? prev.dy16 : nullptr;
      AX_TRY(stage_bwd_data(n, s, s.dact, n->params + s.w_off, s.wb, s.wphase, prev.plain() ? prev.act : nullptr,
                            prev.d_out, early_update, true, st, below16));
      dy16_ready = below16 != nullptr;
    } else {
      dy16_ready = false;
    }
  }
  if (bias_ws_used > n->colsum_ws_floats_) {
    set_error("bias gradients: %zu floats of partial sums in a workspace of %zu", bias_ws_used, n->colsum_ws_floats_);
    return ALEXNET_EINVAL;
  }
  {
    ProfContext pct("wgrad_tail");
    AX_TRY(launch_wgrad_tail(wgrad_tail, st));
  }
  ProfContext pcb("bias_grads");
  return launch_colsum_batch(bias_sums, st);
}

static int fwd_bwd(alexnet* n, int32_t slot, const int32_t* d_labels, uint64_t step, float* d_loss, hipStream_t st,
                   bool early_update = false) {
  const alexnet_config_t& c = n->cfg;
  AX_TRY(run_forward(n, n->input[slot], true, step, st, early_update ? n->ev_u_done : nullptr, n->input16[slot],
                     early_update && n->fc16 ? n->ev_fcw_done : nullptr));
  Dense& last = n->fc[kFc - 1];
  AX_TRY(launch_softmax_xent(last.act, d_labels, c.batch, last.out, 0, last.dz, n->row_loss, n->err_flag, st));
  if (n->fc16) AX_TRY(launch_to_bf16(last.dz, last.dz16, (size_t)c.batch * last.out, st));
  AX_TRY(launch_mean_loss(n->row_loss, c.batch, d_loss, st));
  return run_backward(n, n->input[slot], st, early_update);
}

static int apply_update(alexnet* n, hipStream_t st) {
  const alexnet_config_t& c = n->cfg;
  return launch_sgd_update(n->params, n->mom, n->grads, n->n_params, n->n_weights, c.lr, c.momentum, c.weight_decay,
                           st);
}

// canonical <-> internal for one flat vector
static int convert_flat(alexnet* n, const float* src, float* dst, int dir, hipStream_t st) {
  for (int i = 0; i < kStages; ++i) {
    Stage& s = n->st[i];
    AX_TRY(launch_conv_weight_pack(src + s.w_off, dst + s.w_off, s.g.Cout, s.g.cg(), s.g.k, s.g.groups, dir, st));
    AX_TRY(launch_copy(src + s.b_off, dst + s.b_off, s.g.Cout, st));
  }
  for (int j = 0; j < kFc; ++j) {
    Dense& f = n->fc[j];
    if (j == 0) {
      Stage& l = n->st[kStages - 1];
      AX_TRY(launch_fc_weight_permute(src + f.w_off, dst + f.w_off, f.out, l.g.Cout, l.Hp * l.Wp, dir, st));
    } else {
      AX_TRY(launch_copy(src + f.w_off, dst + f.w_off, (size_t)f.in * f.out, st));
    }
    AX_TRY(launch_copy(src + f.b_off, dst + f.b_off, f.out, st));
  }
  return ALEXNET_OK;
}

static int stage_of(alexnet* n, int32_t layer, Stage** s) {
  if (!n || layer < 1 || layer > kStages) {
    set_error("layer must be 1..5");
    return ALEXNET_EINVAL;
  }
  *s = &n->st[layer - 1];
  (*s)->x16 = (*s)->x16_own;
  set_gemm_precision(n->cfg.precision);
  return ALEXNET_OK;
}

// ================================ C ABI =======================================
extern "C" {

const char* alexnet_last_error(void) { return ax::get_error(); }
const char* alexnet_version(void) { return "alexnet-hip gfx950 fp32-mfma 0.1"; }

int alexnet_profile_begin(void) {
  if (g_profiler) {
    set_error("alexnet_profile_begin: already profiling on this thread");
    return ALEXNET_EINVAL;
  }
  g_profiler = new (std::nothrow) Profiler;
  if (!g_profiler) {
    set_error("out of host memory");
    return ALEXNET_EINVAL;
  }
  g_prof = g_profiler;
  return ALEXNET_OK;
}

int alexnet_profile_end(alexnet_prof_entry_t* out, int32_t cap, int32_t* n_out) {
  if (!g_profiler) {
    set_error("alexnet_profile_end: not profiling");
    return ALEXNET_EINVAL;
  }
  Profiler* p = g_profiler;
  g_profiler = nullptr;
  g_prof = nullptr;
  int rc = ALEXNET_OK;
  int32_t k = 0;
  if (p->failed) {
    set_error("alexnet_profile_end: an event call failed while profiling");
    rc = ALEXNET_EHIP;
  }
  for (auto& e : p->entries) {
    if (rc != ALEXNET_OK) break;
    float total = 0.f;
    for (auto& pr : e.ev) {
      float ms = 0.f;
      if (hipEventSynchronize(pr.second) != hipSuccess || hipEventElapsedTime(&ms, pr.first, pr.second) != hipSuccess) {
        set_error("alexnet_profile_end: reading an event failed");
        rc = ALEXNET_EHIP;
        break;
      }
      total += ms;
    }
    if (rc == ALEXNET_OK && out && k < cap) {
      alexnet_prof_entry_t& o = out[k];
      snprintf(o.name, sizeof o.name, "%s", e.name.c_str());
      o.calls = (int32_t)e.ev.size();
      o.total_ms = total;
      o.flops = e.flops;
      o.bytes = e.bytes;
    }
    ++k;
  }
  if (n_out) *n_out = k;
  delete p;
  return rc;
}

int alexnet_query(const alexnet_config_t* cfg, size_t* n_params, size_t* workspace_bytes) {
  REQUIRE(cfg && n_params && workspace_bytes, ALEXNET_EINVAL, "alexnet_query: null argument");
  alexnet tmp;
  memset(&tmp, 0, sizeof tmp);
  AX_TRY(plan(&tmp, cfg, nullptr));
  *n_params = tmp.n_params;
  *workspace_bytes = tmp.ws_bytes;
  return ALEXNET_OK;
}

int alexnet_create(const alexnet_config_t* cfg, void* d_params, void* d_momentum, void* d_workspace,
                   size_t workspace_bytes, void* stream, alexnet_t** out) {
  REQUIRE(cfg && d_params && d_momentum && d_workspace && out, ALEXNET_EINVAL, "alexnet_create: null argument");
  REQUIRE(aligned256(d_params) && aligned256(d_momentum) && aligned256(d_workspace), ALEXNET_EALIGN,
          "alexnet_create: device pointers must be 256-byte aligned");
  alexnet* n = new (std::nothrow) alexnet;
  REQUIRE(n, ALEXNET_EINVAL, "out of host memory");
  memset(n, 0, sizeof *n);
  int r = plan(n, cfg, (char*)d_workspace);
  if (r == ALEXNET_OK && workspace_bytes < n->ws_bytes) {
    set_error("workspace too small: %zu < %zu bytes", workspace_bytes, n->ws_bytes);
    r = ALEXNET_ENOMEM;
  }
  if (r == ALEXNET_OK) {
    n->params = (float*)d_params;
    n->mom = (float*)d_momentum;
    r = launch_fill_bytes(d_workspace, n->ws_bytes, S(stream));
  }
  if (r == ALEXNET_OK) {
    hipError_t e = hipStreamCreateWithFlags(&n->upd_stream, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&n->ev_fc_done, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&n->ev_upd_done, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&n->ev_step_begin, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&n->ev_wb_done, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&n->ev_u_done, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&n->ev_fcw_done, hipEventDisableTiming);
    if (e != hipSuccess) {
      set_error("alexnet_create: %s", hipGetErrorString(e));
      r = ALEXNET_EHIP;
    }
  }
  if (r != ALEXNET_OK) {
    alexnet_destroy(n);
    return r;
  }
  *out = n;
  return ALEXNET_OK;
}

void alexnet_destroy(alexnet_t* net) {
  if (!net) return;
  if (net->upd_stream) {
    (void)hipStreamSynchronize(net->upd_stream);
    (void)hipStreamDestroy(net->upd_stream);
  }
  if (net->ev_fc_done) (void)hipEventDestroy(net->ev_fc_done);
  if (net->ev_upd_done) (void)hipEventDestroy(net->ev_upd_done);
  if (net->ev_step_begin) (void)hipEventDestroy(net->ev_step_begin);
  if (net->ev_wb_done) (void)hipEventDestroy(net->ev_wb_done);
  if (net->ev_u_done) (void)hipEventDestroy(net->ev_u_done);
  if (net->ev_fcw_done) (void)hipEventDestroy(net->ev_fcw_done);
  delete net;
}

int alexnet_preprocess(alexnet_t* n, const uint8_t* d_raw, const float* d_mean, uint64_t step, int32_t slot,
                       void* stream) {
  REQUIRE(n && d_raw && d_mean, ALEXNET_EINVAL, "alexnet_preprocess: null argument");
  REQUIRE(slot == 0 || slot == 1, ALEXNET_EINVAL, "alexnet_preprocess: slot must be 0 or 1");
  const alexnet_config_t& c = n->cfg;
  const uint64_t key = step_key(c.seed, step);
  AX_TRY(launch_crop_params(key, c.batch, c.raw_w - c.crop_w + 1, c.raw_h - c.crop_h + 1, n->crop_x[slot],
                            n->crop_y[slot], n->flip[slot], S(stream)));
  return launch_preprocess(d_raw, d_mean, n->crop_x[slot], n->crop_y[slot], n->flip[slot], c.batch, c.in_c, c.raw_h,
                           c.raw_w, c.crop_h, c.crop_w, n->input[slot], S(stream), n->input16[slot]);
}

int alexnet_preprocess_center(alexnet_t* n, const uint8_t* d_raw, const float* d_mean, int32_t slot, void* stream) {
  REQUIRE(n && d_raw && d_mean, ALEXNET_EINVAL, "alexnet_preprocess_center: null argument");
  REQUIRE(slot == 0 || slot == 1, ALEXNET_EINVAL, "alexnet_preprocess_center: slot must be 0 or 1");
  const alexnet_config_t& c = n->cfg;
  AX_TRY(launch_crop_center(c.batch, (c.raw_w - c.crop_w) / 2, (c.raw_h - c.crop_h) / 2, n->crop_x[slot],
                            n->crop_y[slot], n->flip[slot], S(stream)));
  return launch_preprocess(d_raw, d_mean, n->crop_x[slot], n->crop_y[slot], n->flip[slot], c.batch, c.in_c, c.raw_h,
                           c.raw_w, c.crop_h, c.crop_w, n->input[slot], S(stream), n->input16[slot]);
}

int alexnet_set_input(alexnet_t* n, const float* d_input_nchw, int32_t slot, void* stream) {
  REQUIRE(n && d_input_nchw, ALEXNET_EINVAL, "alexnet_set_input: null argument");
  REQUIRE(slot == 0 || slot == 1, ALEXNET_EINVAL, "alexnet_set_input: slot must be 0 or 1");
  const alexnet_config_t& c = n->cfg;
  AX_TRY(launch_nchw_to_nhwc(d_input_nchw, n->input[slot], c.batch, c.in_c, c.crop_h, c.crop_w, S(stream)));
  if (n->input16[slot])
    AX_TRY(launch_pad4_bf16(n->input[slot], n->input16[slot], (size_t)c.batch * c.crop_h * c.crop_w, c.in_c, S(stream)));
  return ALEXNET_OK;
}

int alexnet_forward_backward(alexnet_t* n, int32_t slot, const int32_t* d_labels, uint64_t step, float* d_loss,
                             void* stream) {
  REQUIRE(n && d_labels && d_loss, ALEXNET_EINVAL, "alexnet_forward_backward: null argument");
  REQUIRE(slot == 0 || slot == 1, ALEXNET_EINVAL, "alexnet_forward_backward: slot must be 0 or 1");
  return fwd_bwd(n, slot, d_labels, step, d_loss, S(stream));
}

int alexnet_apply_update(alexnet_t* n, void* stream) {
  REQUIRE(n, ALEXNET_EINVAL, "alexnet_apply_update: null handle");
  return apply_update(n, S(stream));
}

int alexnet_train_step(alexnet_t* n, int32_t slot, const int32_t* d_labels, uint64_t step, float* d_loss,
                       void* stream) {
  REQUIRE(n && d_labels && d_loss, ALEXNET_EINVAL, "alexnet_train_step: null argument");
  REQUIRE(slot == 0 || slot == 1, ALEXNET_EINVAL, "alexnet_train_step: slot must be 0 or 1");
  // the dense-layer weights start at a 16-byte boundary of the flat vector in every AlexNet-like shape; if not,
  // one update at the end
  const size_t fc_begin = n->fc[0].w_off;
  const bool early = fc_begin % 4 == 0 && n->n_weights % 4 == 0;
  if (early) {
    // the backward-data packing of the convolution weights depends on the weights only: it runs on the side
    // stream under the forward pass
    AX_HIP(hipEventRecord(n->ev_step_begin, S(stream)));
    AX_HIP(hipStreamWaitEvent(n->upd_stream, n->ev_step_begin, 0));
    for (int i = 0; i < kStages; ++i) {  // transformed taps of the forward pass first: it needs them soonest
      Stage& s = n->st[i];
      ProfContext pc(s.lab[1]);
      if (s.wino) AX_TRY(launch_wino_filter(s.g, n->params + s.w_off, s.wino_u, n->upd_stream));
      if (s.b16)
        AX_TRY(launch_to_bf16_transposed(n->params + s.w_off, s.wf16, s.g.groups, s.g.kf(), s.g.og(), n->upd_stream));
      if (s.r16)
        AX_TRY(launch_run16_pack(n->params + s.w_off, s.wf16, s.g.k, s.g.Cin,
                                 (int)(conv_run16_w_elems(s.g) / ((size_t)s.g.k * s.g.Cout)), s.g.Cout, n->upd_stream));
    }
    AX_HIP(hipEventRecord(n->ev_u_done, n->upd_stream));
    if (n->fc16) {  // needed next, by the dense layers' forward products
      ProfContext pc("fc.weights16");
      AX_TRY(fcw16_refresh(n, n->upd_stream));
      AX_HIP(hipEventRecord(n->ev_fcw_done, n->upd_stream));
    }
    for (int i = 1; i < kStages; ++i) {
      Stage& s = n->st[i];
      ProfContext pc(s.lab[3]);
      AX_TRY(launch_conv_weight_wb(n->params + s.w_off, s.wb, s.g.Cout, s.g.cg(), s.g.k, s.g.groups, n->upd_stream));
      if (s.wino_bx) AX_TRY(launch_wino_filter_bwd(s.g, s.wb, s.wino_ub, n->upd_stream));
      if (s.b16) AX_TRY(launch_to_bf16_transposed(s.wb, s.wb16, s.g.groups, s.g.kb(), s.g.cg(), n->upd_stream));
    }
    AX_HIP(hipEventRecord(n->ev_wb_done, n->upd_stream));
  }
  AX_TRY(fwd_bwd(n, slot, d_labels, step, d_loss, S(stream), early));
  if (!early) return apply_update(n, S(stream));
  // convolution weights and all biases, the two ends of the flat vector, in one launch
  AX_TRY(launch_sgd_update_two(n->params, n->mom, n->grads, fc_begin, n->n_weights, n->n_params, n->n_weights,
                               n->cfg.lr, n->cfg.momentum, n->cfg.weight_decay, S(stream)));
  AX_HIP(hipStreamWaitEvent(S(stream), n->ev_upd_done, 0));      // join the dense-layer update
  return ALEXNET_OK;
}

int alexnet_forward(alexnet_t* n, const float* d_input_nchw, float* d_probs, void* stream) {
  REQUIRE(n && d_input_nchw && d_probs, ALEXNET_EINVAL, "alexnet_forward: null argument");
  const alexnet_config_t& c = n->cfg;
  AX_TRY(launch_nchw_to_nhwc(d_input_nchw, n->input[2], c.batch, c.in_c, c.crop_h, c.crop_w, S(stream)));
  AX_TRY(run_forward(n, n->input[2], false, 0, S(stream)));  // the first layer pads its own bf16 copy
  Dense& last = n->fc[kFc - 1];
  return launch_softmax_xent(last.act, nullptr, c.batch, last.out, 1, d_probs, n->row_loss, n->err_flag, S(stream));
}

int alexnet_validate(alexnet_t* n, int32_t slot, const int32_t* d_labels, const int32_t* ks, int32_t nk,
                     int32_t* d_counts, void* stream) {
  REQUIRE(n && d_labels && ks && d_counts, ALEXNET_EINVAL, "alexnet_validate: null argument");
  REQUIRE(slot == 0 || slot == 1, ALEXNET_EINVAL, "alexnet_validate: slot must be 0 or 1");
  REQUIRE(nk >= 1 && nk <= 8, ALEXNET_EINVAL, "alexnet_validate: between 1 and 8 values of k");
  for (int j = 0; j < nk; ++j) REQUIRE(ks[j] >= 1, ALEXNET_EINVAL, "alexnet_validate: k must be positive");
  AX_TRY(run_forward(n, n->input[slot], false, 0, S(stream), nullptr, n->input16[slot]));
  Dense& last = n->fc[kFc - 1];
  // the order of the scores is the order of the probabilities, so the logits are counted directly
  return launch_topk_count(last.act, d_labels, n->cfg.batch, last.out, ks, nk, d_counts, n->err_flag, S(stream));
}

int alexnet_average_gradients_update(alexnet_t* a, alexnet_t* b, void* stream) {
  REQUIRE(a && b, ALEXNET_EINVAL, "alexnet_average_gradients_update: null handle");
  REQUIRE(a != b, ALEXNET_EINVAL, "alexnet_average_gradients_update: the two replicas must be distinct");
  REQUIRE(a->n_params == b->n_params && a->n_weights == b->n_weights, ALEXNET_ESHAPE,
          "alexnet_average_gradients_update: configurations differ");
  const alexnet_config_t& c = a->cfg;
  REQUIRE(c.lr == b->cfg.lr && c.momentum == b->cfg.momentum && c.weight_decay == b->cfg.weight_decay, ALEXNET_ESHAPE,
          "alexnet_average_gradients_update: optimiser constants differ");
  return launch_avg_grad_update(a->params, a->mom, a->grads, b->params, b->mom, b->grads, a->n_params, a->n_weights,
                                c.lr, c.momentum, c.weight_decay, S(stream));
}

int alexnet_average_replicas(alexnet_t* a, alexnet_t* b, void* stream) {
  REQUIRE(a && b, ALEXNET_EINVAL, "alexnet_average_replicas: null handle");
  REQUIRE(a != b, ALEXNET_EINVAL, "alexnet_average_replicas: the two replicas must be distinct");
  REQUIRE(a->n_params == b->n_params && a->n_weights == b->n_weights, ALEXNET_ESHAPE,
          "alexnet_average_replicas: configurations differ");
  AX_TRY(launch_average(a->params, b->params, a->n_params, S(stream)));
  return launch_average(a->mom, b->mom, a->n_params, S(stream));
}

int alexnet_set_params(alexnet_t* n, const float* d, void* stream) {
  REQUIRE(n && d, ALEXNET_EINVAL, "alexnet_set_params: null argument");
  return convert_flat(n, d, n->params, 0, S(stream));
}
int alexnet_get_params(alexnet_t* n, float* d, void* stream) {
  REQUIRE(n && d, ALEXNET_EINVAL, "alexnet_get_params: null argument");
  return convert_flat(n, n->params, d, 1, S(stream));
}
int alexnet_set_momentum(alexnet_t* n, const float* d, void* stream) {
  REQUIRE(n && d, ALEXNET_EINVAL, "alexnet_set_momentum: null argument");
  return convert_flat(n, d, n->mom, 0, S(stream));
}
int alexnet_get_momentum(alexnet_t* n, float* d, void* stream) {
  REQUIRE(n && d, ALEXNET_EINVAL, "alexnet_get_momentum: null argument");
  return convert_flat(n, n->mom, d, 1, S(stream));
}
int alexnet_get_grads(alexnet_t* n, float* d, void* stream) {
  REQUIRE(n && d, ALEXNET_EINVAL, "alexnet_get_grads: null argument");
  return convert_flat(n, n->grads, d, 1, S(stream));
}

int alexnet_tensor_elems(alexnet_t* n, int32_t kind, int32_t layer, size_t* elems) {
  REQUIRE(n && elems, ALEXNET_EINVAL, "alexnet_tensor_elems: null argument");
  const alexnet_config_t& c = n->cfg;
  switch (kind) {
    case ALEXNET_T_INPUT:
      REQUIRE(layer >= 0 && layer < kSlots, ALEXNET_EINVAL, "bad slot");
      *elems = (size_t)c.batch * c.in_c * c.crop_h * c.crop_w;
      return ALEXNET_OK;
    case ALEXNET_T_CROP_X:
    case ALEXNET_T_CROP_Y:
    case ALEXNET_T_FLIP:
      REQUIRE(layer >= 0 && layer < 2, ALEXNET_EINVAL, "bad slot");
      *elems = c.batch;
      return ALEXNET_OK;
    case ALEXNET_T_DLOGITS:
      *elems = (size_t)c.batch * n->fc[kFc - 1].out;
      return ALEXNET_OK;
    case ALEXNET_T_FC_ACT:
      REQUIRE(layer > kStages && layer <= kStages + kFc, ALEXNET_EINVAL, "dense layer must be 6..8");
      *elems = (size_t)c.batch * n->fc[layer - kStages - 1].out;
      return ALEXNET_OK;
    default: break;
  }
  Stage* s;
  AX_TRY(stage_of(n, layer, &s));
  switch (kind) {
    case ALEXNET_T_CONV_ACT:
    case ALEXNET_T_CONV_DACT: *elems = s->act_elems(); return ALEXNET_OK;
    case ALEXNET_T_LRN:
      REQUIRE(s->lrn, ALEXNET_EINVAL, "stage has no LRN");
      *elems = s->act_elems();
      return ALEXNET_OK;
    case ALEXNET_T_POOL:
    case ALEXNET_T_ARGMAX:
      REQUIRE(s->pool, ALEXNET_EINVAL, "stage has no pool");
      *elems = s->out_elems();
      return ALEXNET_OK;
    default: break;
  }
  set_error("unknown tensor kind %d", kind);
  return ALEXNET_EINVAL;
}

int alexnet_get_tensor(alexnet_t* n, int32_t kind, int32_t layer, void* d_out, void* stream) {
  REQUIRE(n && d_out, ALEXNET_EINVAL, "alexnet_get_tensor: null argument");
  size_t elems;
  AX_TRY(alexnet_tensor_elems(n, kind, layer, &elems));
  const alexnet_config_t& c = n->cfg;
  hipStream_t st = S(stream);
  switch (kind) {
    case ALEXNET_T_INPUT: return launch_nhwc_to_nchw(n->input[layer], (float*)d_out, c.batch, c.in_c, c.crop_h, c.crop_w, st);
    case ALEXNET_T_CROP_X: return launch_copy((const float*)n->crop_x[layer], (float*)d_out, elems, st);
    case ALEXNET_T_CROP_Y: return launch_copy((const float*)n->crop_y[layer], (float*)d_out, elems, st);
    case ALEXNET_T_FLIP: return launch_copy((const float*)n->flip[layer], (float*)d_out, elems, st);
    case ALEXNET_T_DLOGITS: return launch_copy(n->fc[kFc - 1].dz, (float*)d_out, elems, st);
    case ALEXNET_T_FC_ACT: return launch_copy(n->fc[layer - kStages - 1].act, (float*)d_out, elems, st);
    default: break;
  }
  Stage& s = n->st[layer - 1];
  switch (kind) {
    case ALEXNET_T_CONV_ACT: return launch_nhwc_to_nchw(s.act, (float*)d_out, s.g.B, s.g.Cout, s.g.Ho, s.g.Wo, st);
    case ALEXNET_T_CONV_DACT: return launch_nhwc_to_nchw(s.dact, (float*)d_out, s.g.B, s.g.Cout, s.g.Ho, s.g.Wo, st);
    case ALEXNET_T_LRN:
      if (s.fused())  // the training path does not store it: normalise the stored activations now
        AX_TRY(launch_lrn_fwd(s.act, s.lrn_out, s.g.P(), s.g.Cout, n->cfg.lrn_n, n->cfg.lrn_k, n->cfg.lrn_alpha,
                              n->cfg.lrn_beta, st));
      return launch_nhwc_to_nchw(s.lrn_out, (float*)d_out, s.g.B, s.g.Cout, s.g.Ho, s.g.Wo, st);
    case ALEXNET_T_POOL: return launch_nhwc_to_nchw(s.pool_out, (float*)d_out, s.g.B, s.g.Cout, s.Hp, s.Wp, st);
    case ALEXNET_T_ARGMAX:
      return launch_pool_argmax_canonical(s.slot, (int32_t*)d_out, s.g.B, s.g.Cout, s.Hp, s.Wp, s.g.Wo, st);
    default: break;
  }
  return ALEXNET_EINVAL;
}

int alexnet_check(alexnet_t* n, void* stream) {
  REQUIRE(n, ALEXNET_EINVAL, "alexnet_check: null handle");
  int32_t flag = 0;
  AX_HIP(hipMemcpyAsync(&flag, n->err_flag, sizeof flag, hipMemcpyDeviceToHost, S(stream)));
  AX_HIP(hipStreamSynchronize(S(stream)));
  if (flag) {
    AX_TRY(launch_fill_bytes(n->err_flag, 4, S(stream)));
    set_error("a label outside [0, classes) was passed to a training step");
    return ALEXNET_ELABEL;
  }
  return ALEXNET_OK;
}

// ---- single operators ---------------------------------------------------------
int alexnet_nchw_to_nhwc(const float* s, float* d, int32_t n, int32_t c, int32_t h, int32_t w, void* stream) {
  REQUIRE(s && d && n >= 0 && c > 0 && h > 0 && w > 0, ALEXNET_EINVAL, "alexnet_nchw_to_nhwc: bad argument");
  return launch_nchw_to_nhwc(s, d, n, c, h, w, S(stream));
}
int alexnet_nhwc_to_nchw(const float* s, float* d, int32_t n, int32_t c, int32_t h, int32_t w, void* stream) {
  REQUIRE(s && d && n >= 0 && c > 0 && h > 0 && w > 0, ALEXNET_EINVAL, "alexnet_nhwc_to_nchw: bad argument");
  return launch_nhwc_to_nchw(s, d, n, c, h, w, S(stream));
}
int alexnet_pack_conv_weight(alexnet_t* n, int32_t layer, const float* w, float* wf, float* wb, void* stream) {
  Stage* s;
  AX_TRY(stage_of(n, layer, &s));
  REQUIRE(w && wf, ALEXNET_EINVAL, "alexnet_pack_conv_weight: null argument");
  AX_TRY(launch_conv_weight_pack(w, wf, s->g.Cout, s->g.cg(), s->g.k, s->g.groups, 0, S(stream)));
  if (wb) AX_TRY(launch_conv_weight_wb(wf, wb, s->g.Cout, s->g.cg(), s->g.k, s->g.groups, S(stream)));
  return ALEXNET_OK;
}
int alexnet_unpack_conv_weight(alexnet_t* n, int32_t layer, const float* wf, float* w, void* stream) {
  Stage* s;
  AX_TRY(stage_of(n, layer, &s));
  REQUIRE(w && wf, ALEXNET_EINVAL, "alexnet_unpack_conv_weight: null argument");
  return launch_conv_weight_pack(wf, w, s->g.Cout, s->g.cg(), s->g.k, s->g.groups, 1, S(stream));
}
int alexnet_conv_forward_nhwc(alexnet_t* n, int32_t layer, const float* x, const float* wf, const float* b,
                              int32_t relu, float* y, void* stream) {
  Stage* s;
  AX_TRY(stage_of(n, layer, &s));
  REQUIRE(x && wf && y, ALEXNET_EINVAL, "alexnet_conv_forward_nhwc: null argument");
  return stage_fwd(n, *s, x, wf, b, relu, y, false, S(stream));
}
int alexnet_conv_backward_data_nhwc(alexnet_t* n, int32_t layer, const float* dy, const float* wf, const float* wb,
                                    float* dx, void* stream) {
  Stage* s;
  AX_TRY(stage_of(n, layer, &s));
  REQUIRE(dy && wb && dx, ALEXNET_EINVAL, "alexnet_conv_backward_data_nhwc: null argument");
  return stage_bwd_data(n, *s, dy, wf, wb, wf ? s->wphase : nullptr, nullptr, dx, false, false, S(stream));
}
int alexnet_conv_backward_weight_nhwc(alexnet_t* n, int32_t layer, const float* x, const float* dy, float* dwf,
                                      float* db, void* stream) {
  Stage* s;
  AX_TRY(stage_of(n, layer, &s));
  REQUIRE(x && dy && dwf, ALEXNET_EINVAL, "alexnet_conv_backward_weight_nhwc: null argument");
  AX_TRY(stage_bwd_weight(n, *s, x, dy, dwf, false, S(stream)));
  if (db) AX_TRY(launch_colsum(dy, s->g.P(), s->g.Cout, db, n->colsum_ws, S(stream)));
  return ALEXNET_OK;
}
int alexnet_conv_forward(alexnet_t* n, int32_t layer, const float* x, const float* w, const float* b, int32_t relu,
                         float* y, void* stream) {
  Stage* s;
  AX_TRY(stage_of(n, layer, &s));
  REQUIRE(x && w && y, ALEXNET_EINVAL, "alexnet_conv_forward: null argument");
  const ConvGeom& g = s->g;
  AX_TRY(launch_nchw_to_nhwc(x, n->scratch_x, g.B, g.Cin, g.H, g.W, S(stream)));
  AX_TRY(launch_conv_weight_pack(w, n->scratch_w[0], g.Cout, g.cg(), g.k, g.groups, 0, S(stream)));
  AX_TRY(stage_fwd(n, *s, n->scratch_x, n->scratch_w[0], b, relu, n->scratch_y, false, S(stream)));
  return launch_nhwc_to_nchw(n->scratch_y, y, g.B, g.Cout, g.Ho, g.Wo, S(stream));
}
int alexnet_conv_backward_data(alexnet_t* n, int32_t layer, const float* dy, const float* w, float* dx,
                               void* stream) {
  Stage* s;
  AX_TRY(stage_of(n, layer, &s));
  REQUIRE(dy && w && dx, ALEXNET_EINVAL, "alexnet_conv_backward_data: null argument");
  const ConvGeom& g = s->g;
  AX_TRY(launch_nchw_to_nhwc(dy, n->scratch_y, g.B, g.Cout, g.Ho, g.Wo, S(stream)));
  AX_TRY(launch_conv_weight_pack(w, n->scratch_w[0], g.Cout, g.cg(), g.k, g.groups, 0, S(stream)));
  AX_TRY(launch_conv_weight_wb(n->scratch_w[0], n->scratch_w[1], g.Cout, g.cg(), g.k, g.groups, S(stream)));
  AX_TRY(stage_bwd_data(n, *s, n->scratch_y, n->scratch_w[0], n->scratch_w[1], s->wphase, nullptr, n->scratch_x, false,
                        false, S(stream)));
  return launch_nhwc_to_nchw(n->scratch_x, dx, g.B, g.Cin, g.H, g.W, S(stream));
}
int alexnet_conv_backward_weight(alexnet_t* n, int32_t layer, const float* x, const float* dy, float* dw, float* db,
                                 void* stream) {
  Stage* s;
  AX_TRY(stage_of(n, layer, &s));
  REQUIRE(x && dy && dw, ALEXNET_EINVAL, "alexnet_conv_backward_weight: null argument");
  const ConvGeom& g = s->g;
  AX_TRY(launch_nchw_to_nhwc(x, n->scratch_x, g.B, g.Cin, g.H, g.W, S(stream)));
  AX_TRY(launch_nchw_to_nhwc(dy, n->scratch_y, g.B, g.Cout, g.Ho, g.Wo, S(stream)));
  AX_TRY(stage_bwd_weight(n, *s, n->scratch_x, n->scratch_y, n->scratch_w[2], false, S(stream)));
  AX_TRY(launch_conv_weight_pack(n->scratch_w[2], dw, g.Cout, g.cg(), g.k, g.groups, 1, S(stream)));
  if (db) AX_TRY(launch_colsum(n->scratch_y, g.P(), g.Cout, db, n->colsum_ws, S(stream)));
  return ALEXNET_OK;
}

// ---- single bandwidth-bound operators on canonical tensors --------------------
// These reuse the stage's own training buffers as staging space.
int alexnet_lrn_forward(alexnet_t* n, int32_t layer, const float* d_a, float* d_b, void* stream) {
  Stage* s;
  AX_TRY(stage_of(n, layer, &s));
  REQUIRE(d_a && d_b, ALEXNET_EINVAL, "alexnet_lrn_forward: null argument");
  REQUIRE(s->lrn, ALEXNET_EINVAL, "alexnet_lrn_forward: stage has no LRN");
  const ConvGeom& g = s->g;
  const alexnet_config_t& c = n->cfg;
  AX_TRY(launch_nchw_to_nhwc(d_a, s->act, g.B, g.Cout, g.Ho, g.Wo, S(stream)));
  AX_TRY(launch_lrn_fwd(s->act, s->lrn_out, g.P(), g.Cout, c.lrn_n, c.lrn_k, c.lrn_alpha, c.lrn_beta, S(stream)));
  return launch_nhwc_to_nchw(s->lrn_out, d_b, g.B, g.Cout, g.Ho, g.Wo, S(stream));
}
int alexnet_lrn_backward(alexnet_t* n, int32_t layer, const float* d_a, const float* d_db, int32_t relu_gate,
                         float* d_da, void* stream) {
  Stage* s;
  AX_TRY(stage_of(n, layer, &s));
  REQUIRE(d_a && d_db && d_da, ALEXNET_EINVAL, "alexnet_lrn_backward: null argument");
  REQUIRE(s->lrn, ALEXNET_EINVAL, "alexnet_lrn_backward: stage has no LRN");
  const ConvGeom& g = s->g;
  const alexnet_config_t& c = n->cfg;
  AX_TRY(launch_nchw_to_nhwc(d_a, s->act, g.B, g.Cout, g.Ho, g.Wo, S(stream)));
  AX_TRY(launch_nchw_to_nhwc(d_db, s->lrn_out, g.B, g.Cout, g.Ho, g.Wo, S(stream)));
  AX_TRY(launch_lrn_bwd(s->act, s->lrn_out, s->dact, g.P(), g.Cout, c.lrn_n, c.lrn_k, c.lrn_alpha, c.lrn_beta,
                        relu_gate, S(stream)));
  return launch_nhwc_to_nchw(s->dact, d_da, g.B, g.Cout, g.Ho, g.Wo, S(stream));
}
int alexnet_pool_forward(alexnet_t* n, int32_t layer, const float* d_x, float* d_y, int32_t* d_argmax,
                         void* stream) {
  Stage* s;
  AX_TRY(stage_of(n, layer, &s));
  REQUIRE(d_x && d_y, ALEXNET_EINVAL, "alexnet_pool_forward: null argument");
  REQUIRE(s->pool, ALEXNET_EINVAL, "alexnet_pool_forward: stage has no pool");
  const ConvGeom& g = s->g;
  AX_TRY(launch_nchw_to_nhwc(d_x, s->act, g.B, g.Cout, g.Ho, g.Wo, S(stream)));
  AX_TRY(launch_pool_fwd(s->act, s->pool_out, s->slot, g.B, g.Ho, g.Wo, g.Cout, s->Hp, s->Wp, S(stream)));
  AX_TRY(launch_nhwc_to_nchw(s->pool_out, d_y, g.B, g.Cout, s->Hp, s->Wp, S(stream)));
  if (d_argmax) AX_TRY(launch_pool_argmax_canonical(s->slot, d_argmax, g.B, g.Cout, s->Hp, s->Wp, g.Wo, S(stream)));
  return ALEXNET_OK;
}
int alexnet_pool_backward(alexnet_t* n, int32_t layer, const float* d_x, const float* d_dy, int32_t relu_gate,
                          float* d_dx, void* stream) {
  Stage* s;
  AX_TRY(stage_of(n, layer, &s));
  REQUIRE(d_x && d_dy && d_dx, ALEXNET_EINVAL, "alexnet_pool_backward: null argument");
  REQUIRE(s->pool, ALEXNET_EINVAL, "alexnet_pool_backward: stage has no pool");
  const ConvGeom& g = s->g;
  AX_TRY(launch_nchw_to_nhwc(d_x, s->act, g.B, g.Cout, g.Ho, g.Wo, S(stream)));
  AX_TRY(launch_pool_fwd(s->act, s->pool_out, s->slot, g.B, g.Ho, g.Wo, g.Cout, s->Hp, s->Wp, S(stream)));
  AX_TRY(launch_nchw_to_nhwc(d_dy, s->d_out, g.B, g.Cout, s->Hp, s->Wp, S(stream)));
  AX_TRY(launch_pool_bwd(s->d_out, s->slot, relu_gate ? s->act : nullptr, s->dact, g.B, g.Ho, g.Wo, g.Cout, s->Hp,
                         s->Wp, S(stream)));
  return launch_nhwc_to_nchw(s->dact, d_dx, g.B, g.Cout, g.Ho, g.Wo, S(stream));
}

// The two kernels a training step runs for a stage that normalises and pools (conv1 and conv2 of the paper's
// network), alone: normalisation + pool in one pass, and pool adjoint + normalisation adjoint + ReLU gate +
// bias-gradient sums in one pass.
int alexnet_lrn_pool_forward(alexnet_t* n, int32_t layer, const float* d_a, float* d_y, int32_t* d_argmax,
                             void* stream) {
  Stage* s;
  AX_TRY(stage_of(n, layer, &s));
  REQUIRE(d_a && d_y, ALEXNET_EINVAL, "alexnet_lrn_pool_forward: null argument");
  REQUIRE(s->fused(), ALEXNET_ENOTIMPL, "alexnet_lrn_pool_forward: this stage does not run the fused kernels");
  const ConvGeom& g = s->g;
  const alexnet_config_t& c = n->cfg;
  AX_TRY(launch_nchw_to_nhwc(d_a, s->act, g.B, g.Cout, g.Ho, g.Wo, S(stream)));
  AX_TRY(launch_lrn_pool_fwd(s->act, s->pool_out, s->slot, g.B, g.Ho, g.Wo, g.Cout, s->Hp, s->Wp, c.lrn_n, c.lrn_k,
                             c.lrn_alpha, c.lrn_beta, S(stream)));
  AX_TRY(launch_nhwc_to_nchw(s->pool_out, d_y, g.B, g.Cout, s->Hp, s->Wp, S(stream)));
  if (d_argmax) AX_TRY(launch_pool_argmax_canonical(s->slot, d_argmax, g.B, g.Cout, s->Hp, s->Wp, g.Wo, S(stream)));
  return ALEXNET_OK;
}
int alexnet_pool_lrn_backward(alexnet_t* n, int32_t layer, const float* d_a, const float* d_dy, int32_t relu_gate,
                              float* d_da, float* d_db, void* stream) {
  Stage* s;
  AX_TRY(stage_of(n, layer, &s));
  REQUIRE(d_a && d_dy && d_da, ALEXNET_EINVAL, "alexnet_pool_lrn_backward: null argument");
  REQUIRE(s->fused(), ALEXNET_ENOTIMPL, "alexnet_pool_lrn_backward: this stage does not run the fused kernels");
  REQUIRE(!d_db || aligned16(d_db), ALEXNET_EALIGN, "alexnet_pool_lrn_backward: d_db must be 16-byte aligned");
  const ConvGeom& g = s->g;
  const alexnet_config_t& c = n->cfg;
  AX_TRY(launch_nchw_to_nhwc(d_a, s->act, g.B, g.Cout, g.Ho, g.Wo, S(stream)));
  // the winning taps come from the fused forward kernel, as in a training step
  AX_TRY(launch_lrn_pool_fwd(s->act, s->pool_out, s->slot, g.B, g.Ho, g.Wo, g.Cout, s->Hp, s->Wp, c.lrn_n, c.lrn_k,
                             c.lrn_alpha, c.lrn_beta, S(stream)));
  AX_TRY(launch_nchw_to_nhwc(d_dy, s->d_out, g.B, g.Cout, s->Hp, s->Wp, S(stream)));
  AX_TRY(launch_pool_lrn_bwd(s->act, s->d_out, s->slot, s->dact, g.B, g.Ho, g.Wo, g.Cout, s->Hp, s->Wp, c.lrn_n,
                             c.lrn_k, c.lrn_alpha, c.lrn_beta, relu_gate, d_db, n->colsum_ws, S(stream)));
  return launch_nhwc_to_nchw(s->dact, d_da, g.B, g.Cout, g.Ho, g.Wo, S(stream));
}

static int dense_of(alexnet* n, int32_t layer, Dense** f) {
  if (!n || layer <= kStages || layer > kStages + kFc) {
    set_error("dense layer must be 6..8");
    return ALEXNET_EINVAL;
  }
  *f = &n->fc[layer - kStages - 1];
  set_gemm_precision(n->cfg.precision);
  return ALEXNET_OK;
}
int alexnet_fc_forward(alexnet_t* n, int32_t layer, const float* d_x, const float* d_w, const float* d_b,
                       int32_t relu, float* d_y, void* stream) {
  Dense* f;
  AX_TRY(dense_of(n, layer, &f));
  REQUIRE(d_x && d_w && d_y, ALEXNET_EINVAL, "alexnet_fc_forward: null argument");
  FcAct act;
  act.bias = d_b; act.relu = relu; act.dropout = 0; act.key = 0; act.tag = 0; act.thresh24 = 0; act.scale = 1.0f;
  return launch_fc_fwd(n->cfg.batch, f->in, f->out, d_x, d_w, act, d_y, n->gemm_ws, S(stream));
}
int alexnet_fc_backward(alexnet_t* n, int32_t layer, const float* d_x, const float* d_w, const float* d_dy,
                        float* d_dx, float* d_dw, float* d_db, void* stream) {
  Dense* f;
  AX_TRY(dense_of(n, layer, &f));
  REQUIRE(d_x && d_w && d_dy && d_dx && d_dw && d_db, ALEXNET_EINVAL, "alexnet_fc_backward: null argument");
  const int B = n->cfg.batch;
  AX_TRY(launch_fc_bwd_weight(B, f->in, f->out, d_x, d_dy, d_dw, S(stream)));
  AX_TRY(launch_colsum(d_dy, B, f->out, d_db, n->colsum_ws, S(stream)));
  return launch_fc_bwd_data(B, f->in, f->out, d_dy, d_w, nullptr, d_dx, n->gemm_ws, S(stream));
}
int alexnet_softmax_xent(alexnet_t* n, const float* d_logits, const int32_t* d_labels, float* d_dz, float* d_loss,
                         void* stream) {
  REQUIRE(n && d_logits && d_labels && d_dz && d_loss, ALEXNET_EINVAL, "alexnet_softmax_xent: null argument");
  const int B = n->cfg.batch, classes = n->fc[kFc - 1].out;
  AX_TRY(launch_softmax_xent(d_logits, d_labels, B, classes, 0, d_dz, n->row_loss, n->err_flag, S(stream)));
  return launch_mean_loss(n->row_loss, B, d_loss, S(stream));
}

// ---- softmax cross-entropy for callers that cannot allocate ------------------
// Scratch of alexnet_softmax_xent_static: the per-row losses of one call, then the label flag.  One copy per
// GPU, held until the process ends; every call on a GPU shares it.
constexpr int kStaticMaxRows = 4096;
static __device__ __align__(256) float scratch[kStaticMaxRows + 64];
constexpr int kMaxDevices = 64;
static float* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, looked up once
static std::mutex g_scratch_mu;

static int static_scratch(float** out) {
  int dev = -1;
  AX_HIP(hipGetDevice(&dev));
  REQUIRE(dev >= 0 && dev < kMaxDevices, ALEXNET_EINVAL, "alexnet_softmax_xent_static: device index out of range");
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    // in host code `scratch` is only a handle of the symbol: its address on the current device comes from the
    // runtime, and each GPU has its own
    float* p = nullptr;
    AX_HIP(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
    REQUIRE(p, ALEXNET_EHIP, "alexnet_softmax_xent_static: no device address for the scratch array");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return ALEXNET_OK;
}

int alexnet_softmax_xent_static(const float* d_logits, const int32_t* d_labels, int32_t batch, int32_t classes,
                                float* d_dz, float* d_loss, int32_t* d_bad_label, void* stream) {
  REQUIRE(d_logits && d_labels && d_dz && d_loss, ALEXNET_EINVAL, "alexnet_softmax_xent_static: null argument");
  REQUIRE(batch >= 1 && classes >= 1, ALEXNET_ESHAPE, "alexnet_softmax_xent_static: batch and classes must be positive");
  if (batch > kStaticMaxRows) {
    set_error("alexnet_softmax_xent_static: batch %d exceeds the %d rows of the built-in scratch; use "
              "alexnet_softmax_xent with a handle's workspace", batch, kStaticMaxRows);
    return ALEXNET_ENOMEM;
  }
  REQUIRE((long)batch * classes <= 0x1ffffff0L, ALEXNET_ESHAPE, "alexnet_softmax_xent_static: logits reach 2 GiB");
  float* ws = nullptr;
  AX_TRY(static_scratch(&ws));
  float* row_loss = ws;
  int32_t* flag = reinterpret_cast<int32_t*>(ws + kStaticMaxRows);
  // the flag must start at zero; a fill kernel rather than a memset node, so that the call can be captured
  AX_TRY(launch_fill_bytes(flag, 4, S(stream)));
  AX_TRY(launch_softmax_xent(d_logits, d_labels, batch, classes, 0, d_dz, row_loss, flag, S(stream)));
  AX_TRY(launch_mean_loss(row_loss, batch, d_loss, S(stream)));
  if (d_bad_label) AX_TRY(launch_copy(reinterpret_cast<const float*>(flag), reinterpret_cast<float*>(d_bad_label), 1, S(stream)));
  return ALEXNET_OK;
}

}  // extern "C"
