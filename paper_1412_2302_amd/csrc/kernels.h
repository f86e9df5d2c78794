// Host-side launch functions of every kernel in the library.  All tensors are
// device pointers in the internal channel-last layout unless a name says
// otherwise; every function only enqueues work on `st` and returns a status.
#pragma once
#include "common.h"
#include "conv_plan.h"

namespace ax {

// The tail of the weight gradient of a transformed stage -- adding up the split-k slices of the products, then
// the transform back to taps -- can be put off to the end of a backward pass and run for all such stages in two
// launches: each of those kernels is too short to fill the chip on its own.  The slices and the products then
// need memory of their own until the tail runs.
constexpr int kMaxWgradJobs = 5;
struct WgradJob {
  const float* slices;  // [groups36][nsplit][slab]; unused when nsplit == 1 (the products are in dU already)
  float* dU;            // [groups36][slab]
  float* dwf;
  long slab, total;     // floats per product group; threads of the transform back
  int nsplit, groups36, groups, Na, Nb, k, nsub;
  int vec;              // set by wgrad_tail_add: the slices are added 16 bytes at a time
};
struct WgradTail {
  WgradJob job[kMaxWgradJobs];
  int first_r[kMaxWgradJobs], first_t[kMaxWgradJobs];  // first workgroup of each job in the two launches
  int n = 0, blocks_r = 0, blocks_t = 0;
};
void wgrad_tail_add(WgradTail& t, const WgradJob& job);  // t.n < kMaxWgradJobs
int launch_reduce_slabs_batch(const WgradTail& t, hipStream_t st);
int launch_wino_dw_batch(const WgradTail& t, hipStream_t st);
int launch_wgrad_tail(const WgradTail& t, hipStream_t st);

// ---- convolution as implicit GEMM (conv_gemm.hip) ---------------------------
// Arithmetic of the GEMMs the calling thread launches from now on: 0 = fp32 MFMA, 1 = operands rounded to
// bf16 (nearest even) on their way into LDS, products accumulated in fp32.  Operands that cannot be read
// 16 bytes at a time keep the fp32 kernels.
void set_gemm_precision(int bf16);
// `ws` is split-k scratch of at least the matching *_ws_floats() floats (may be null when that is 0)
size_t conv_fwd_ws_floats(const ConvGeom& c);
size_t conv_bwd_data_ws_floats(const ConvGeom& c);
size_t conv_bwd_weight_ws_floats(const ConvGeom& c);
// Run mode (unpadded conv over 3-channel pictures, see gemm.h): `wrun` / `dwrun` are padded copies of the
// forward weights and of their gradient, conv_run_w_floats() floats each; null selects the generic gather.
bool conv_run_mode(const ConvGeom& c);
size_t conv_run_w_floats(const ConvGeom& c);
int launch_conv_run_pack(const ConvGeom& c, const float* wf, float* wrun, hipStream_t st);
// x16 / dy16: copies of the activations in bf16, same layout; wf16 / wb16: bf16 copies of the packed weights with
// the reduction contiguous, wf16[g][o][(r,s,c)] and wb16[g][c][(r,s,o)] (launch_to_bf16_transposed of wf / wb).
// When both operands of a product are given, the handle's GEMMs are bf16 and conv_bf16_stored_ok(), the product
// reads those instead of rounding fp32 on the fly.  y16 / dx16: where to leave a bf16 copy of the result for the
// products that read it next (written by the epilogue, or converted after a split-k pass).
bool conv_bf16_stored_ok(const ConvGeom& c);
int launch_conv_fwd(const ConvGeom& c, const float* x, const float* wf, const float* wrun, const float* bias,
                    int relu, float* y, float* ws, hipStream_t st, const uint16_t* x16 = nullptr,
                    const uint16_t* wf16 = nullptr, uint16_t* y16 = nullptr);
// The first layer with bf16 products over pictures stored as bf16, four channels per pixel (conv_plan.h, run16):
// x4 from launch_pad4_bf16 (or the preprocessing kernel), wk from launch_run16_pack.  conv_run16_ok(): the
// geometry allows it.  (The weight gradient keeps the fp32 pictures: over this view its reduction has 528 rows,
// five 128-row tiles where the run mode of gemm.h has four, and measured slower.)
bool conv_run16_ok(const ConvGeom& c);
size_t conv_run16_x_elems(const ConvGeom& c);
size_t conv_run16_w_elems(const ConvGeom& c);
int launch_conv_fwd_run16(const ConvGeom& c, const uint16_t* x4, const uint16_t* wk, const float* bias, int relu,
                          float* y, float* ws, hipStream_t st, uint16_t* y16 = nullptr);
// Strided, ungrouped, ungated backward-data runs by phases when `wphase` (conv_phase_w_floats() floats of
// scratch) is given; it then reads the forward weights wf instead of wb.
bool conv_phase_mode(const ConvGeom& c);
size_t conv_phase_w_floats(const ConvGeom& c);
int launch_conv_bwd_data(const ConvGeom& c, const float* dy, const float* wf, const float* wb, float* wphase,
                         const float* gate, float* dx, float* ws, hipStream_t st, const uint16_t* dy16 = nullptr,
                         const uint16_t* wb16 = nullptr, uint16_t* dx16 = nullptr);
int launch_conv_bwd_weight(const ConvGeom& c, const float* x, const float* dy, float* dwf, float* dwrun, float* ws,
                           hipStream_t st, int* defer_ns = nullptr, const uint16_t* x16 = nullptr,
                           const uint16_t* dy16 = nullptr);

// ---- 3x3 and 5x5 unit-stride convolutions through F(4x4, 3x3) (winograd.hip) ----
// All tensors 16-byte aligned, channels per group multiples of 4.  V: wino_v_floats(), U / Ub / dU:
// wino_u_floats(), every other transformed tensor (v, m, yt): wino_scratch_floats(); ws: wino_gemm_ws_floats().
// wino_ok: forward and weight gradient can take this path; wino_bwd_data_ok: the data gradient too;
// wino_gain: multiplies of the direct form per multiply of the transformed one at this layer's map size.
bool wino_ok(const ConvGeom& c);
bool wino_bwd_data_ok(const ConvGeom& c);
double wino_gain(const ConvGeom& c);
size_t wino_v_floats(const ConvGeom& c);
size_t wino_u_floats(const ConvGeom& c);
size_t wino_scratch_floats(const ConvGeom& c);
size_t wino_gemm_ws_floats(const ConvGeom& c);
size_t wino_wgrad_ws_floats(const ConvGeom& c);
int launch_wino_filter(const ConvGeom& c, const float* wf, float* U, hipStream_t st);
int launch_wino_filter_bwd(const ConvGeom& c, const float* wb, float* Ub, hipStream_t st);
int launch_wino_input(const ConvGeom& c, const float* x, float* V, hipStream_t st);
int launch_wino_fwd(const ConvGeom& c, const float* x, const float* U, const float* bias, int relu, float* y, float* V,
                    float* m, float* ws, hipStream_t st);
int launch_wino_bwd_weight(const ConvGeom& c, const float* V, const float* dy, float* dwf, float* yt, float* dU,
                           float* ws, hipStream_t st, WgradTail* tail = nullptr);
int launch_wino_output_grad(const ConvGeom& c, const float* dy, float* yt, hipStream_t st);
// the data gradient starts from the transformed output gradient yt (launch_wino_output_grad, or what
// launch_wino_bwd_weight left in its `yt`), not from dy
int launch_wino_bwd_data(const ConvGeom& c, const float* yt, const float* Ut, const float* gate, float* dx, float* m,
                         float* ws, hipStream_t st);

// ---- dense layers (conv_gemm.hip) -------------------------------------------
struct FcAct {
  const float* bias;  // [out]
  int relu;
  int dropout;        // 1: multiply by the keep mask of (key, tag)
  uint64_t key;
  uint32_t tag, thresh24;
  float scale;        // applied after the ReLU (1 - p at inference, else 1)
};
size_t fc_ws_floats(int B, int in, int out);
// x16 / w16 / dy16: bf16 copies of the operands (same layouts); when those of a product are given, the handle's
// GEMMs are bf16 and fc_bf16_stored_ok(), the product reads them.  y16 / dx16: where to leave a bf16 copy of the result.
bool fc_bf16_stored_ok(int in, int out);
int launch_fc_fwd(int B, int in, int out, const float* x, const float* w, const FcAct& act, float* y, float* ws,
                  hipStream_t st, const uint16_t* x16 = nullptr, const uint16_t* w16 = nullptr, uint16_t* y16 = nullptr);
int launch_fc_bwd_data(int B, int in, int out, const float* dy, const float* w, const float* gate, float* dx,
                       float* ws, hipStream_t st, const uint16_t* dy16 = nullptr, const uint16_t* w16 = nullptr,
                       uint16_t* dx16 = nullptr);
int launch_fc_bwd_weight(int B, int in, int out, const float* x, const float* dy, float* dw, hipStream_t st,
                         const uint16_t* x16 = nullptr, const uint16_t* dy16 = nullptr);

// ---- bandwidth-bound kernels (ops.hip) --------------------------------------
int launch_fill(float* p, size_t n, float v, hipStream_t st);
// dst[i] = bf16(src[i]), round to nearest even
int launch_to_bf16(const float* src, uint16_t* dst, size_t n, hipStream_t st);
// dst[g][n][k] = bf16(src[g][k][n]) for G matrices of K x N
int launch_to_bf16_transposed(const float* src, uint16_t* dst, int G, int K, int N, hipStream_t st);
// pictures with C < 4 channels as bf16 with four channels per pixel (the rest zero); the first layer's packed
// weights as bf16 wk[o][(r, s*4 + c)] for that view
int launch_pad4_bf16(const float* x, uint16_t* x4, size_t pixels, int C, hipStream_t st);
int launch_run16_pack(const float* wf, uint16_t* wk, int k, int C, int run, int cout, hipStream_t st);
int launch_fill_bytes(void* p, size_t nbytes, hipStream_t st);  // zero fill, nbytes % 4 == 0
int launch_crop_params(uint64_t key, int B, int range_x, int range_y, int32_t* ox, int32_t* oy, int32_t* flip,
                       hipStream_t st);
int launch_preprocess(const uint8_t* raw, const float* mean, const int32_t* ox, const int32_t* oy,
                      const int32_t* flip, int B, int C, int RH, int RW, int CH, int CW, float* out, hipStream_t st,
                      uint16_t* out4 = nullptr);  // out4: also the pictures as bf16, four channels per pixel (C <= 4)
int launch_nchw_to_nhwc(const float* src, float* dst, int N, int C, int H, int W, hipStream_t st);
int launch_nhwc_to_nchw(const float* src, float* dst, int N, int C, int H, int W, hipStream_t st);
int launch_lrn_fwd(const float* a, float* b, long pixels, int C, int n, float k, float alpha, float beta,
                   hipStream_t st);
// da = (dL/db through the normalisation) gated by a > 0 when relu_gate is set
int launch_lrn_bwd(const float* a, const float* db, float* da, long pixels, int C, int n, float k, float alpha,
                   float beta, int relu_gate, hipStream_t st);
// Normalisation fused with the 3x3 stride-2 max-pool after it (forward: the normalised tensor is never
// stored) and with that pool's adjoint before it (backward: dy is the pooled gradient).  Usable when
// lrn_pool_fused_ok(); colsum_out (may be null) receives the per-channel sums of da, `part` is scratch of
// lrn_part_floats(C) floats.
bool lrn_pool_fused_ok(const float* a, const float* y, const float* dy, const float* da, const uint8_t* slot, int C,
                       int n);
size_t lrn_part_floats(int C);
// y16 / da16 / dx16 (may be null): where to leave a bf16 copy of the result
int launch_lrn_pool_fwd(const float* a, float* y, uint8_t* slot, int N, int H, int W, int C, int Ho, int Wo, int n,
                        float k, float alpha, float beta, hipStream_t st, uint16_t* y16 = nullptr);
int launch_pool_lrn_bwd(const float* a, const float* dy, const uint8_t* slot, float* da, int N, int H, int W, int C,
                        int Ho, int Wo, int n, float k, float alpha, float beta, int relu_gate, float* colsum_out,
                        float* part, hipStream_t st, bool partials_only = false, uint16_t* da16 = nullptr);
// partials_only: leave the lrn_part_rows(pixels, C) rows of per-workgroup sums in `part` for the caller to add up
size_t lrn_part_rows(long pixels, int C);
int launch_pool_fwd(const float* x, float* y, uint8_t* slot, int N, int H, int W, int C, int Ho, int Wo,
                    hipStream_t st, uint16_t* y16 = nullptr);
// dx[n][y][x][c] = sum of dy over the windows whose winning tap is (y,x); gated by gate > 0 when gate != null
int launch_pool_bwd(const float* dy, const uint8_t* slot, const float* gate, float* dx, int N, int H, int W, int C,
                    int Ho, int Wo, hipStream_t st, uint16_t* dx16 = nullptr);
int launch_pool_argmax_canonical(const uint8_t* slot, int32_t* out_nchw, int N, int C, int Ho, int Wo, int W,
                                 hipStream_t st);
// mode 0: dz = (p - onehot)/B and per-row loss; mode 1: p only
int launch_softmax_xent(const float* z, const int32_t* labels, int B, int classes, int mode, float* out,
                        float* row_loss, int32_t* err_flag, hipStream_t st);
int launch_mean_loss(const float* row_loss, int B, float* loss, hipStream_t st);
int launch_colsum(const float* m, long rows, int cols, float* out, float* ws, hipStream_t st);
size_t colsum_ws_floats(long rows, int cols);
// Several column sums in two launches: add the jobs (each takes its partial sums from ws at *ws_used and moves
// that on by colsum_batch_ws_floats(rows, cols)), then launch; every input must still hold its values then.
constexpr int kMaxColsumJobs = 8;
struct ColsumJob {
  const float* m;
  float *part, *out;
  long rows;
  int cols, rpb, nparts;
};
struct ColsumBatch {
  ColsumJob job[kMaxColsumJobs];
  int first1[kMaxColsumJobs], first2[kMaxColsumJobs];  // first workgroup of each job in the two launches
  int n = 0, blocks1 = 0, blocks2 = 0;
};
int colsum_batch_add(ColsumBatch& b, const float* m, long rows, int cols, float* out, float* ws, size_t* ws_used);
size_t colsum_batch_ws_floats(long rows, int cols);
int launch_colsum_batch(const ColsumBatch& b, hipStream_t st);
int launch_reduce_slabs(const float* ws, int nsplit, long slab, int groups, float* out, hipStream_t st);
// one result of k*run rows by cout columns, rows (r, j >= kc) dropped and the rest packed to r*kc + j
int launch_reduce_slabs_unpack(const float* ws, int nsplit, long slab, int run, int kc, int cout, float* out,
                               hipStream_t st);
// max_blocks: upper limit of the grid (0: the default, four workgroups per CU)
int launch_sgd_update(float* w, float* v, const float* g, size_t n, size_t n_decay, float lr, float mu, float wd,
                      hipStream_t st, unsigned max_blocks = 0);
// the same for elements [0, n1) and [begin2, end2) of the vectors in one launch (n1 and begin2 multiples of four);
// positions below n_decay are decayed
int launch_sgd_update_two(float* w, float* v, const float* g, size_t n1, size_t begin2, size_t end2, size_t n_decay,
                          float lr, float mu, float wd, hipStream_t st);
int launch_average(float* a, float* b, size_t n, hipStream_t st);
int launch_avg_grad_update(float* wa, float* va, const float* ga, float* wb, float* vb, const float* gb, size_t n,
                           size_t n_decay, float lr, float mu, float wd, hipStream_t st);
// counts[j] += rows whose label is among the ks[j] highest scores (ties go to the label); nk <= 8, ks on the host
int launch_topk_count(const float* z, const int32_t* labels, int B, int classes, const int32_t* ks, int nk,
                      int32_t* counts, int32_t* err_flag, hipStream_t st);
int launch_crop_center(int B, int off_x, int off_y, int32_t* ox, int32_t* oy, int32_t* flip, hipStream_t st);
// layout conversions of parameters; dir 0: canonical -> internal, 1: internal -> canonical
int launch_conv_weight_pack(const float* src, float* dst, int Cout, int Cg, int k, int groups, int dir,
                            hipStream_t st);
int launch_conv_weight_wb(const float* wf, float* wb, int Cout, int Cg, int k, int groups, hipStream_t st);
int launch_fc_weight_permute(const float* src, float* dst, int out, int C, int HW, int dir, hipStream_t st);
int launch_copy(const float* src, float* dst, size_t n, hipStream_t st);

}  // namespace ax
