// Bandwidth-bound kernels of the AlexNet step: preprocessing, response
// normalisation, max pooling, softmax cross-entropy, reductions, the momentum
// update, replica averaging and layout conversions.  Activations are
// channel-last ([N][H][W][C]); a lane owns four consecutive channels wherever
// C % 4 == 0 so that every global access is a coalesced 16-byte load/store.
#include <math.h>

#include <algorithm>

#include "kernels.h"

namespace ax {

static inline unsigned grid_for(size_t n, unsigned block) { return (unsigned)((n + block - 1) / block); }

// ------------------------------------------------------------------ fill ---
__global__ void fill_kernel(float* p, size_t n, float v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}
int launch_fill(float* p, size_t n, float v, hipStream_t st) {
  if (n == 0) return ALEXNET_OK;
  unsigned g = grid_for(n, 256);
  if (g > 4096) g = 4096;
  hipLaunchKernelGGL(fill_kernel, dim3(g), dim3(256), 0, st, p, n, v);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}
int launch_fill_bytes(void* p, size_t nbytes, hipStream_t st) { return launch_fill((float*)p, nbytes / 4, 0.f, st); }

// fp32 -> bf16 (nearest even) copies of GEMM operands: eight values per lane and trip
__global__ void __launch_bounds__(256) to_bf16_kernel(const float* __restrict__ s, uint16_t* __restrict__ d, size_t n8,
                                                      size_t n) {
  typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
  typedef uint32_t v4u __attribute__((ext_vector_type(4)));
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += stride) {
    const float4 a = *reinterpret_cast<const float4*>(s + 8 * i);
    const float4 b = *reinterpret_cast<const float4*>(s + 8 * i + 4);
    v4u o;
    bf2 t;
    t[0] = (__bf16)a.x; t[1] = (__bf16)a.y; o[0] = __builtin_bit_cast(uint32_t, t);
    t[0] = (__bf16)a.z; t[1] = (__bf16)a.w; o[1] = __builtin_bit_cast(uint32_t, t);
    t[0] = (__bf16)b.x; t[1] = (__bf16)b.y; o[2] = __builtin_bit_cast(uint32_t, t);
    t[0] = (__bf16)b.z; t[1] = (__bf16)b.w; o[3] = __builtin_bit_cast(uint32_t, t);
    *reinterpret_cast<v4u*>(d + 8 * i) = o;
  }
  // tail (n % 8 values), by the first lanes of the grid
  const size_t i = 8 * n8 + (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    const __bf16 v = (__bf16)s[i];
    d[i] = __builtin_bit_cast(uint16_t, v);
  }
}
int launch_to_bf16(const float* src, uint16_t* dst, size_t n, hipStream_t st) {
  if (n == 0) return ALEXNET_OK;
  if ((((uintptr_t)src | (uintptr_t)dst) & 15) != 0) {
    set_error("to_bf16: tensors must be 16-byte aligned");
    return ALEXNET_EALIGN;
  }
  KernelScope ks("to_bf16", 0, (double)n * 6.0, st);
  const size_t n8 = n / 8;
  unsigned g = grid_for(std::max<size_t>(n8, 1), 256);
  if (g > 4096) g = 4096;
  hipLaunchKernelGGL(to_bf16_kernel, dim3(g), dim3(256), 0, st, src, dst, n8, n);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// dst[g][n][k] = bf16(src[g][k][n]): 32 x 32 tiles through LDS, reads and writes both along their rows
__global__ void __launch_bounds__(256) to_bf16_transposed_kernel(const float* __restrict__ s, uint16_t* __restrict__ d,
                                                                 int K, int N) {
  __shared__ float tile[32][33];
  const size_t g = blockIdx.z;
  const int k0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  for (int r = ty; r < 32; r += 8) {
    const int k = k0 + r, n = n0 + tx;
    tile[r][tx] = (k < K && n < N) ? s[(g * K + k) * N + n] : 0.f;
  }
  __syncthreads();
  for (int r = ty; r < 32; r += 8) {
    const int n = n0 + r, k = k0 + tx;
    if (n < N && k < K) {
      const __bf16 v = (__bf16)tile[tx][r];
      d[(g * N + n) * K + k] = __builtin_bit_cast(uint16_t, v);
    }
  }
}
int launch_to_bf16_transposed(const float* src, uint16_t* dst, int G, int K, int N, hipStream_t st) {
  if (G <= 0 || K <= 0 || N <= 0) return ALEXNET_OK;
  KernelScope ks("to_bf16", 0, (double)G * K * N * 6.0, st);
  hipLaunchKernelGGL(to_bf16_transposed_kernel, dim3(ceil_div(N, 32), ceil_div(K, 32), G), dim3(256), 0, st, src, dst, K,
                     N);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// x4[p][0..3] = bf16(x[p][0..C-1]), 0 for the channels past C (C < 4): pictures for the first layer's bf16 products
__global__ void __launch_bounds__(256) pad4_bf16_kernel(const float* __restrict__ x, uint16_t* __restrict__ x4,
                                                        size_t pixels, int C) {
  const size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= pixels) return;
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  const float* s = x + p * C;
  v.x = s[0];
  if (C > 1) v.y = s[1];
  if (C > 2) v.z = s[2];
  store_bf16x4(x4 + p * 4, v);
}
int launch_pad4_bf16(const float* x, uint16_t* x4, size_t pixels, int C, hipStream_t st) {
  if (!pixels) return ALEXNET_OK;
  KernelScope ks("to_bf16", 0, (double)pixels * (C * 4.0 + 8.0), st);
  hipLaunchKernelGGL(pad4_bf16_kernel, dim3(grid_for(pixels, 256)), dim3(256), 0, st, x, x4, pixels, C);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}
// wk[o][r*run + s*4 + c] = bf16(wf[(r, s, c)][o]) for s < k, c < C, else 0
__global__ void __launch_bounds__(256) run16_pack_kernel(const float* __restrict__ wf, uint16_t* __restrict__ wk, int k,
                                                         int C, int run, int cout) {
  const size_t total = (size_t)cout * k * run;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // index into wk
  if (i >= total) return;
  const int j = (int)(i % run);
  const size_t q = i / run;
  const int r = (int)(q % k), o = (int)(q / k);
  const int s2 = j >> 2, c = j & 3;
  const float v = (s2 < k && c < C) ? wf[((size_t)(r * k + s2) * C + c) * cout + o] : 0.f;
  store_bf16(wk + i, v);
}
int launch_run16_pack(const float* wf, uint16_t* wk, int k, int C, int run, int cout, hipStream_t st) {
  const size_t total = (size_t)cout * k * run;
  KernelScope ks("to_bf16", 0, (double)total * 6.0, st);
  hipLaunchKernelGGL(run16_pack_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, wf, wk, k, C, run, cout);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

__global__ void copy_kernel(const float* __restrict__ s, float* __restrict__ d, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) d[i] = s[i];
}
int launch_copy(const float* src, float* dst, size_t n, hipStream_t st) {
  if (n == 0) return ALEXNET_OK;
  unsigned g = grid_for(n, 256);
  if (g > 8192) g = 8192;
  hipLaunchKernelGGL(copy_kernel, dim3(g), dim3(256), 0, st, src, dst, n);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// ------------------------------------------------------------ preprocess ---
// Paper Section 2.1 (footnote): mean subtraction, random crop, random flip.
__global__ void crop_params_kernel(uint64_t key, int B, int range_x, int range_y, int32_t* ox, int32_t* oy,
                                   int32_t* flip) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= B) return;
  ox[n] = (int32_t)((rand_u64(key, TAG_CROP_X, n) >> 32) % (uint64_t)range_x);
  oy[n] = (int32_t)((rand_u64(key, TAG_CROP_Y, n) >> 32) % (uint64_t)range_y);
  flip[n] = (int32_t)(rand_u64(key, TAG_FLIP, n) >> 63);
}
// the central crop, not mirrored (validation)
__global__ void crop_center_kernel(int B, int off_x, int off_y, int32_t* ox, int32_t* oy, int32_t* flip) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= B) return;
  ox[n] = off_x;
  oy[n] = off_y;
  flip[n] = 0;
}
int launch_crop_center(int B, int off_x, int off_y, int32_t* ox, int32_t* oy, int32_t* flip, hipStream_t st) {
  KernelScope ks("crop_params", 0, (double)B * 12.0, st);
  hipLaunchKernelGGL(crop_center_kernel, dim3(grid_for(B, 64)), dim3(64), 0, st, B, off_x, off_y, ox, oy, flip);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}
int launch_crop_params(uint64_t key, int B, int range_x, int range_y, int32_t* ox, int32_t* oy, int32_t* flip,
                       hipStream_t st) {
  KernelScope ks("crop_params", 0, (double)B * 12.0, st);
  hipLaunchKernelGGL(crop_params_kernel, dim3(grid_for(B, 64)), dim3(64), 0, st, key, B, range_x, range_y, ox, oy,
                     flip);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// out[n][y][x][c] = raw[n][c][oy+y][ox + (flip ? CW-1-x : x)] - mean[c][same place].  A wave owns one output
// row (n, y): picture, source row, crop offset and mirror flag are the same for all its lanes, a lane's work per
// element is one division by C, and the wave's stores are consecutive floats of the flat output.
constexpr int kPreRows = 4;  // rows (waves) per workgroup
__global__ void __launch_bounds__(64 * kPreRows)
preprocess_kernel(const uint8_t* __restrict__ raw, const float* __restrict__ mean, const int32_t* __restrict__ ox,
                  const int32_t* __restrict__ oy, const int32_t* __restrict__ flip, uint32_t rows, int C, int RH,
                  int RW, int CH, int CW, FastDiv div_c, FastDiv div_ch, float* __restrict__ out,
                  uint16_t* __restrict__ out4) {
  const uint32_t row = blockIdx.x * kPreRows + (threadIdx.x >> 6);  // n*CH + y, the same for the whole wave
  if (row >= rows) return;
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t n = fdiv(row, div_ch), y = row - n * (uint32_t)CH;
  const uint32_t plane = (uint32_t)(RH * RW);
  const int32_t x0 = ox[n], mirror = flip[n];
  const uint32_t src_row = ((uint32_t)oy[n] + y) * (uint32_t)RW;
  const uint8_t* rp = raw + (size_t)n * C * plane + src_row;
  const float* mp = mean + src_row;
  const uint32_t len = (uint32_t)(CW * C);
  float* op = out + (size_t)row * len;
#pragma unroll 4
  for (uint32_t e = lane; e < len; e += 64) {
    const uint32_t x = fdiv(e, div_c), c = e - x * (uint32_t)C;
    const uint32_t src = c * plane + (uint32_t)x0 + (mirror ? (uint32_t)CW - 1u - x : x);
    op[e] = (float)rp[src] - mp[src];
  }
  if (out4) {  // the same row as bf16 with four channels per pixel (the rest zero), for bf16 first-layer products:
               // a lane owns whole pixels, so that a wave stores 512 consecutive bytes
    uint16_t* o4 = out4 + (size_t)row * CW * 4;
    for (uint32_t x = lane; x < (uint32_t)CW; x += 64) {
      const uint32_t sx = (uint32_t)x0 + (mirror ? (uint32_t)CW - 1u - x : x);
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      v.x = (float)rp[sx] - mp[sx];
      if (C > 1) v.y = (float)rp[plane + sx] - mp[plane + sx];
      if (C > 2) v.z = (float)rp[2 * plane + sx] - mp[2 * plane + sx];
      if (C > 3) v.w = (float)rp[3 * plane + sx] - mp[3 * plane + sx];
      store_bf16x4(o4 + (size_t)x * 4, v);
    }
  }
}
int launch_preprocess(const uint8_t* raw, const float* mean, const int32_t* ox, const int32_t* oy,
                      const int32_t* flip, int B, int C, int RH, int RW, int CH, int CW, float* out, hipStream_t st,
                      uint16_t* out4) {
  if (out4 && C > 4) {
    set_error("preprocess: the four-channel bf16 copy needs at most four channels");
    return ALEXNET_EINVAL;
  }
  const size_t total = (size_t)B * CH * CW * C;
  if (!total) return ALEXNET_OK;
  if (total >= 0x7fffffffu || (size_t)C * RH * RW >= 0x7fffffffu) {
    set_error("preprocess: more than 2^31 elements");
    return ALEXNET_ESHAPE;
  }
  KernelScope ks("preprocess", 0, (double)total * 5.0, st);
  const uint32_t rows = (uint32_t)B * (uint32_t)CH;
  hipLaunchKernelGGL(preprocess_kernel, dim3(ceil_div(rows, kPreRows)), dim3(64 * kPreRows), 0, st, raw, mean, ox, oy,
                     flip, rows, C, RH, RW, CH, CW, make_fastdiv((uint32_t)C), make_fastdiv((uint32_t)CH), out, out4);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// ------------------------------------------------------ layout transposes ---
__global__ void nchw_to_nhwc_kernel(const float* __restrict__ s, float* __restrict__ d, int N, int C, int HW) {
  const size_t total = (size_t)N * C * HW;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // index into nhwc
  if (i >= total) return;
  const int c = (int)(i % C);
  const size_t p = i / C;
  const int hw = (int)(p % HW);
  const size_t n = p / HW;
  d[i] = s[(n * C + c) * HW + hw];
}
__global__ void nhwc_to_nchw_kernel(const float* __restrict__ s, float* __restrict__ d, int N, int C, int HW) {
  const size_t total = (size_t)N * C * HW;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // index into nchw
  if (i >= total) return;
  const int hw = (int)(i % HW);
  const size_t q = i / HW;
  const int c = (int)(q % C);
  const size_t n = q / C;
  d[i] = s[(n * HW + hw) * C + c];
}
int launch_nchw_to_nhwc(const float* src, float* dst, int N, int C, int H, int W, hipStream_t st) {
  const size_t total = (size_t)N * C * H * W;
  if (!total) return ALEXNET_OK;
  hipLaunchKernelGGL(nchw_to_nhwc_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, src, dst, N, C, H * W);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}
int launch_nhwc_to_nchw(const float* src, float* dst, int N, int C, int H, int W, hipStream_t st) {
  const size_t total = (size_t)N * C * H * W;
  if (!total) return ALEXNET_OK;
  hipLaunchKernelGGL(nhwc_to_nchw_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, src, dst, N, C, H * W);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// ------------------------------------------------------------------- LRN ---
// b_i = a_i * s_i^-beta, s_i = k + alpha * sum_{j in [i-n/2, i+n/2] clipped} a_j^2
// s^-beta.  The AlexNet exponent 3/4 is two square roots, taken with the hardware's one-instruction
// v_rsq_f32 / v_sqrt_f32 (about 1 ulp each; s >= k is a normal number): the correctly rounded library
// routines cost some forty instructions per call, which made these kernels ALU-bound.
__device__ __forceinline__ float neg_pow(float s, float beta) {
  if (beta == 0.75f) {
    const float r = __builtin_amdgcn_rsqf(s);
    return r * __builtin_amdgcn_sqrtf(r);
  }
  return powf(s, -beta);
}
// s^-beta / s
__device__ __forceinline__ float neg_pow_over_s(float s, float p, float beta) {
  if (beta == 0.75f) {
    const float r = __builtin_amdgcn_rsqf(s);
    return p * (r * r);
  }
  return p / s;
}

__global__ void lrn_fwd_kernel(const float* __restrict__ a, float* __restrict__ b, size_t total, int C, int half,
                               float k, float alpha, float beta) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % C);
  const int lo = max(c - half, 0), hi = min(c + half, C - 1);
  const float* row = a + (i - c);
  float s = 0.f;
  for (int j = lo; j <= hi; ++j) s += row[j] * row[j];
  s = k + alpha * s;
  b[i] = row[c] * neg_pow(s, beta);
}

__global__ void lrn_bwd_kernel(const float* __restrict__ a, const float* __restrict__ db, float* __restrict__ da,
                               size_t total, int C, int half, float k, float alpha, float beta, int relu_gate) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % C);
  const float* row = a + (i - c);
  const float* drow = db + (i - c);
  const float ai = row[c];
  float out = 0.f;
  if (!relu_gate || ai > 0.f) {
    float acc = 0.f, si = 0.f;
    const int lo = max(c - half, 0), hi = min(c + half, C - 1);
    for (int j = lo; j <= hi; ++j) {
      const int l2 = max(j - half, 0), h2 = min(j + half, C - 1);
      float s = 0.f;
      for (int q = l2; q <= h2; ++q) s += row[q] * row[q];
      s = k + alpha * s;
      if (j == c) si = s;
      acc += drow[j] * row[j] * neg_pow(s, beta) / s;
    }
    out = drow[c] * neg_pow(si, beta) - 2.f * alpha * beta * ai * acc;
  }
  da[i] = out;
}

// Vector versions (C % 4 == 0, C <= 1024): a workgroup owns PB whole pixels, a
// lane owns four consecutive channels of one pixel.  Squares (and, backward,
// the per-channel terms dy*a*s^(-beta-1)) are staged in LDS rows that carry
// `half` zeros on both sides, so the clipped window needs no branches and every
// tensor is read from and written to HBM exactly once with 16-byte accesses.
// x*x as a rounded product of its own: the pragma keeps the compiler from contracting it into a later sum
__device__ __forceinline__ float sq_rounded(float x) {
#pragma clang fp contract(off)
  return x * x;
}
constexpr int kLrnMaxHalf = 4;
constexpr int kLrnPad = 4;  // zeros on both sides of an LDS row; keeps 16-byte alignment
// sums of v[4+j-half .. 4+j+half] for j = 0..3, each added up directly (v = values of channels c-4 .. c+7)
__device__ __forceinline__ float4 lrn_window_sum_regs(const float* v, int half) {
  float s[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float w = v[4 + j];
#pragma unroll
    for (int d = 1; d <= kLrnMaxHalf; ++d)
      if (d <= half) w += v[4 + j - d] + v[4 + j + d];
    s[j] = w;
  }
  return make_float4(s[0], s[1], s[2], s[3]);
}
__device__ __forceinline__ float4 lrn_window_sum(const float* row, int c, int half) {
  float v[12];
  *reinterpret_cast<float4*>(v) = *reinterpret_cast<const float4*>(row + c - 4);
  *reinterpret_cast<float4*>(v + 4) = *reinterpret_cast<const float4*>(row + c);
  *reinterpret_cast<float4*>(v + 8) = *reinterpret_cast<const float4*>(row + c + 4);
  return lrn_window_sum_regs(v, half);
}

// Where the gradient of the normalised activations comes from: a tensor, or (dy != null) the adjoint of the
// 3x3 stride-2 max-pool that follows, gathered on the fly from the pooled gradient and the winning taps.
struct PoolGather {
  const float* dy;       // [N][Ho][Wo][C]
  const uint8_t* slot;   // winning tap 0..8 of each pooled element
  int H, W, Ho, Wo;
  FastDiv d_w, d_h;
};
// The (at most four) pooled windows over an input pixel, as loaded: the reduction is a separate step so
// that the loads can be issued a trip ahead of their use.
struct PoolTaps {
  uint32_t s4[4];    // winning taps of four channels
  float4 d[4];       // pooled gradient of four channels
  uint32_t want[4];  // this pixel's tap number in that window; 9 (never a winner) for a window that does not exist
};
__device__ __forceinline__ void pool_taps_fetch(const PoolGather& pg, long pix, int c, int C, PoolTaps& t) {
  const uint32_t q = fdiv((uint32_t)pix, pg.d_w);  // pix < 2^31: a tensor is smaller than 2 GiB
  const int x = (int)((uint32_t)pix - q * (uint32_t)pg.W);
  const uint32_t n = fdiv(q, pg.d_h);
  const int y = (int)(q - n * (uint32_t)pg.H);
  const int yo_lo = y >= 2 ? (y - 1) / 2 : 0, yo_hi = min(y / 2, pg.Ho - 1);
  const int xo_lo = x >= 2 ? (x - 1) / 2 : 0, xo_hi = min(x / 2, pg.Wo - 1);
#pragma unroll
  for (int wy = 0; wy < 2; ++wy)
#pragma unroll
    for (int wx = 0; wx < 2; ++wx) {
      const int yo = min(yo_lo + wy, yo_hi), xo = min(xo_lo + wx, xo_hi);
      // a pixel in a last row or column that no window covers has lo > hi: the clamped address is still inside
      const bool valid = yo_lo + wy <= yo_hi && xo_lo + wx <= xo_hi;
      const uint32_t o = ((n * (uint32_t)pg.Ho + (uint32_t)yo) * (uint32_t)pg.Wo + (uint32_t)xo) * (uint32_t)C + c;
      t.want[wy * 2 + wx] = valid ? (uint32_t)((y - 2 * yo) * 3 + (x - 2 * xo)) : 9u;
      t.s4[wy * 2 + wx] = *reinterpret_cast<const uint32_t*>(pg.slot + o);
      t.d[wy * 2 + wx] = *reinterpret_cast<const float4*>(pg.dy + o);
    }
}
__device__ __forceinline__ float4 pool_taps_reduce(const PoolTaps& t) {
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const uint32_t s4 = t.s4[w], want = t.want[w];
    acc.x += (s4 & 0xffu) == want ? t.d[w].x : 0.f;
    acc.y += ((s4 >> 8) & 0xffu) == want ? t.d[w].y : 0.f;
    acc.z += ((s4 >> 16) & 0xffu) == want ? t.d[w].z : 0.f;
    acc.w += (s4 >> 24) == want ? t.d[w].w : 0.f;
  }
  return acc;
}

template <bool BWD, bool GATHER>
__global__ void __launch_bounds__(256)
lrn_vec_kernel(const float* __restrict__ a, const float* __restrict__ db, float* __restrict__ out, long pixels, int C,
               int half, int PB, float k, float alpha, float beta, int relu_gate, PoolGather pg,
               float* __restrict__ part, uint16_t* __restrict__ out16) {
  extern __shared__ __attribute__((aligned(16))) float sh[];  // [2][PB][kLrnPad + C + kLrnPad]
  const int q = C >> 2;                                        // lanes per pixel
  const int ld = C + 2 * kLrnPad;
  const int pl = threadIdx.x / q, cq = threadIdx.x - pl * q;
  float* sq = sh + (size_t)pl * ld + kLrnPad;
  float* tt = sh + (size_t)PB * ld + (size_t)pl * ld + kLrnPad;
  if (pl < PB && cq < 2) {  // zero the pads of this pixel's two rows
    const int o = cq == 0 ? -kLrnPad : C;
    *reinterpret_cast<float4*>(sq + o) = make_float4(0.f, 0.f, 0.f, 0.f);
    *reinterpret_cast<float4*>(tt + o) = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  const int c = cq * 4;
  float4 colsum = make_float4(0.f, 0.f, 0.f, 0.f);  // of this lane's outputs over all its pixels
  // every workgroup makes the same number of trips, so the barriers inside are uniform; the loads of a
  // trip are issued during the trip before
  const long stride = (long)gridDim.x * PB;
  float4 nav = make_float4(0.f, 0.f, 0.f, 0.f), ndv = nav;
  PoolTaps taps;
  {
    const long pix = (long)blockIdx.x * PB + pl;
    if (pl < PB && pix < pixels) {
      nav = *reinterpret_cast<const float4*>(a + pix * C + c);
      if (BWD && GATHER) pool_taps_fetch(pg, pix, c, C, taps);
      if (BWD && !GATHER) ndv = *reinterpret_cast<const float4*>(db + pix * C + c);
    }
  }
  for (long first = (long)blockIdx.x * PB; first < pixels; first += stride) {
    const long pix = first + pl;
    const bool on = pl < PB && pix < pixels;
    const float4 av = nav;
    float4 dv = ndv;
    if (BWD && GATHER && on) dv = pool_taps_reduce(taps);
    if (on) *reinterpret_cast<float4*>(sq + c) = make_float4(av.x * av.x, av.y * av.y, av.z * av.z, av.w * av.w);
    {
      const long npix = pix + stride;
      if (pl < PB && npix < pixels) {
        nav = *reinterpret_cast<const float4*>(a + npix * C + c);
        if (BWD && GATHER) pool_taps_fetch(pg, npix, c, C, taps);
        if (BWD && !GATHER) ndv = *reinterpret_cast<const float4*>(db + npix * C + c);
      }
    }
    __syncthreads();
    float4 p = av;  // s^-beta per channel
    float4 sv = av;
    if (on) {
      const float4 w = lrn_window_sum(sq, c, half);
      sv = make_float4(k + alpha * w.x, k + alpha * w.y, k + alpha * w.z, k + alpha * w.w);
      p = make_float4(neg_pow(sv.x, beta), neg_pow(sv.y, beta), neg_pow(sv.z, beta), neg_pow(sv.w, beta));
    }
    if (!BWD) {
      if (on)
        *reinterpret_cast<float4*>(out + pix * C + c) = make_float4(av.x * p.x, av.y * p.y, av.z * p.z, av.w * p.w);
      __syncthreads();  // the next trip overwrites the squares
      continue;
    }
    if (on)
      *reinterpret_cast<float4*>(tt + c) =
          make_float4(dv.x * av.x * neg_pow_over_s(sv.x, p.x, beta), dv.y * av.y * neg_pow_over_s(sv.y, p.y, beta),
                      dv.z * av.z * neg_pow_over_s(sv.z, p.z, beta), dv.w * av.w * neg_pow_over_s(sv.w, p.w, beta));
    __syncthreads();
    if (on) {
      const float4 acc = lrn_window_sum(tt, c, half);
      const float f = 2.f * alpha * beta;
      float4 r = make_float4(dv.x * p.x - f * av.x * acc.x, dv.y * p.y - f * av.y * acc.y,
                             dv.z * p.z - f * av.z * acc.z, dv.w * p.w - f * av.w * acc.w);
      if (relu_gate) {
        r.x = av.x > 0.f ? r.x : 0.f;
        r.y = av.y > 0.f ? r.y : 0.f;
        r.z = av.z > 0.f ? r.z : 0.f;
        r.w = av.w > 0.f ? r.w : 0.f;
      }
      *reinterpret_cast<float4*>(out + pix * C + c) = r;
      if (out16) store_bf16x4(out16 + pix * C + c, r);  // bf16 copy for the products that read the gradient next
      colsum.x += r.x;
      colsum.y += r.y;
      colsum.z += r.z;
      colsum.w += r.w;
    }
    // the next trip writes the squares, which were last read before the barrier above, and writes the
    // products only after its own first barrier, when every lane is done with this trip's
  }
  if (BWD && part) {  // part[workgroup][channel] = sum of this workgroup's outputs, in a fixed order
    __syncthreads();
    if (pl < PB) *reinterpret_cast<float4*>(sh + (size_t)pl * C + c) = colsum;
    __syncthreads();
    if (pl == 0) {
      float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
      for (int r = 0; r < PB; ++r) {
        const float4 v = *reinterpret_cast<const float4*>(sh + (size_t)r * C + c);
        t.x += v.x;
        t.y += v.y;
        t.z += v.z;
        t.w += v.w;
      }
      *reinterpret_cast<float4*>(part + (size_t)blockIdx.x * C + c) = t;
    }
  }
}

// Normalisation and the max-pool that follows it in one pass (C % 4 == 0).  A workgroup owns PH x PW pooled
// pixels of one picture: it normalises the (2PH+1) x (2PW+1) input pixels under them into LDS (a lane takes
// four channels of a pixel and reads that pixel's channels c-4 .. c+7 itself), then pools out of LDS.  The
// normalised tensor never goes to memory.  Same arithmetic and tie-break (first maximum in row-major tap
// order) as the separate kernels.
__global__ void __launch_bounds__(256)
lrn_pool_fwd_kernel(const float* __restrict__ a, float* __restrict__ y, uint8_t* __restrict__ slot, int H, int W,
                    int C, int Ho, int Wo, int PH, int PW, int tiles_y, int tiles_x, int half, float k, float alpha,
                    float beta, uint16_t* __restrict__ y16) {
  extern __shared__ __attribute__((aligned(16))) float bbuf[];  // [(2PH+1)*(2PW+1)][C]
  const int q = C >> 2;
  int t = blockIdx.x;
  const int tx = t % tiles_x;
  t /= tiles_x;
  const int ty = t % tiles_y;
  const int n = t / tiles_y;
  const int py0 = ty * PH, px0 = tx * PW;
  const int ph = min(PH, Ho - py0), pw = min(PW, Wo - px0);
  const int ih = 2 * ph + 1, iw = 2 * pw + 1;  // always inside the picture: 2*Ho <= H-1
  const float* src = a + (((size_t)n * H + 2 * py0) * W + 2 * px0) * C;
  // a lane keeps its four channels and walks over every PB-th pixel; coordinates advance without divisions
  const int PB = 256 / q, pl = threadIdx.x / q, c = (threadIdx.x - pl * q) * 4;
  const bool lane_on = pl < PB;
  {
    // four pixels per trip with all twelve loads issued before the first use: one memory latency per
    // four pixels instead of one per pixel (a pixel past the end re-reads the tile's first pixel)
    constexpr int U = 2;
    const int dq = PB / iw, dr = PB - dq * iw, np = ih * iw;
    int ly = pl / iw, lx = pl - ly * iw;
    for (int pxl0 = pl; lane_on && pxl0 < np; pxl0 += U * PB) {
      float4 m[U], l[U], h[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const bool valid = pxl0 + u * PB < np;
        const float* px = src + (valid ? ((size_t)ly * W + lx) * C : 0) + c;
        m[u] = *reinterpret_cast<const float4*>(px);
        l[u] = h[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (c >= 4) l[u] = *reinterpret_cast<const float4*>(px - 4);
        if (c + 4 < C) h[u] = *reinterpret_cast<const float4*>(px + 4);
        ly += dq;
        lx += dr;
        if (lx >= iw) {
          lx -= iw;
          ++ly;
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int pxl = pxl0 + u * PB;
        // rounded squares (no contraction into the window sums): the separate normalisation kernel adds
        // squares that went through LDS, and the two must give the same bits for the same input
        const float v[12] = {sq_rounded(l[u].x), sq_rounded(l[u].y), sq_rounded(l[u].z),
                             sq_rounded(l[u].w), sq_rounded(m[u].x), sq_rounded(m[u].y),
                             sq_rounded(m[u].z), sq_rounded(m[u].w), sq_rounded(h[u].x),
                             sq_rounded(h[u].y), sq_rounded(h[u].z), sq_rounded(h[u].w)};
        const float4 w = lrn_window_sum_regs(v, half);
        if (pxl < np)
          *reinterpret_cast<float4*>(bbuf + (size_t)pxl * C + c) = make_float4(
              m[u].x * neg_pow(k + alpha * w.x, beta), m[u].y * neg_pow(k + alpha * w.y, beta),
              m[u].z * neg_pow(k + alpha * w.z, beta), m[u].w * neg_pow(k + alpha * w.w, beta));
      }
    }
  }
  __syncthreads();
  const int dq = PB / pw, dr = PB - dq * pw;
  int oy = pl / pw, ox = pl - oy * pw;
  for (int o = pl; lane_on && o < ph * pw; o += PB, oy += dq, ox += dr) {
    if (ox >= pw) {
      ox -= pw;
      ++oy;
    }
    const float* win = bbuf + ((size_t)(2 * oy) * iw + 2 * ox) * C + c;
    float4 best = *reinterpret_cast<const float4*>(win);
    uint32_t bs = 0;
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
      for (int s2 = 0; s2 < 3; ++s2) {
        if (r == 0 && s2 == 0) continue;
        const float4 b = *reinterpret_cast<const float4*>(win + ((size_t)r * iw + s2) * C);
        const uint32_t tap = (uint32_t)(r * 3 + s2);
        if (b.x > best.x) { best.x = b.x; bs = (bs & 0xffffff00u) | tap; }
        if (b.y > best.y) { best.y = b.y; bs = (bs & 0xffff00ffu) | (tap << 8); }
        if (b.z > best.z) { best.z = b.z; bs = (bs & 0xff00ffffu) | (tap << 16); }
        if (b.w > best.w) { best.w = b.w; bs = (bs & 0x00ffffffu) | (tap << 24); }
      }
    const size_t e = (((size_t)n * Ho + py0 + oy) * Wo + px0 + ox) * C + c;
    *reinterpret_cast<float4*>(y + e) = best;
    if (y16) store_bf16x4(y16 + e, best);  // bf16 copy for the product that reads the pooled tensor next
    *reinterpret_cast<uint32_t*>(slot + e) = bs;
  }
}

constexpr int kLrnMaxBlocks = 2048;  // workgroups of the vector kernels (= rows of their column-sum partials)
static int lrn_grid(long pixels, int PB) { return (int)std::min<long>(ceil_div(pixels, PB), kLrnMaxBlocks); }
static bool lrn_vec_ok(const void* p0, const void* p1, const void* p2, int C, int half) {
  return C % 4 == 0 && C <= 1024 && half <= kLrnMaxHalf && aligned16(p0) && aligned16(p1) && aligned16(p2);
}

int launch_lrn_fwd(const float* a, float* b, long pixels, int C, int n, float k, float alpha, float beta,
                   hipStream_t st) {
  const size_t total = (size_t)pixels * C;
  if (!total) return ALEXNET_OK;
  KernelScope ks("lrn_fwd", 0, (double)total * 8.0, st);
  const int half = n / 2;
  if (lrn_vec_ok(a, b, b, C, half)) {
    const int PB = 256 / (C / 4);
    const size_t lds = (size_t)2 * PB * (C + 2 * kLrnPad) * sizeof(float);
    hipLaunchKernelGGL((lrn_vec_kernel<false, false>), dim3(lrn_grid(pixels, PB)), dim3(256), lds, st, a, nullptr, b,
                       pixels, C, half, PB, k, alpha, beta, 0, PoolGather{}, nullptr, nullptr);
  } else {
    hipLaunchKernelGGL(lrn_fwd_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, a, b, total, C, half, k, alpha,
                       beta);
  }
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}
int launch_lrn_bwd(const float* a, const float* db, float* da, long pixels, int C, int n, float k, float alpha,
                   float beta, int relu_gate, hipStream_t st) {
  const size_t total = (size_t)pixels * C;
  if (!total) return ALEXNET_OK;
  KernelScope ks("lrn_bwd", 0, (double)total * 12.0, st);
  const int half = n / 2;
  if (lrn_vec_ok(a, db, da, C, half)) {
    const int PB = 256 / (C / 4);
    const size_t lds = (size_t)2 * PB * (C + 2 * kLrnPad) * sizeof(float);
    hipLaunchKernelGGL((lrn_vec_kernel<true, false>), dim3(lrn_grid(pixels, PB)), dim3(256), lds, st, a, db, da,
                       pixels, C, half, PB, k, alpha, beta, relu_gate, PoolGather{}, nullptr, nullptr);
  } else {
    hipLaunchKernelGGL(lrn_bwd_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, a, db, da, total, C, half, k,
                       alpha, beta, relu_gate);
  }
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// out[c..c+3] = sum over the rows of part[nparts][cols] (cols % 4 == 0): one workgroup per four columns,
// 256 interleaved row sets added up by a fixed tree
__global__ void __launch_bounds__(256)
colsum_finish_kernel(const float* __restrict__ part, int nparts, int cols, float* __restrict__ out) {
  __shared__ float4 sh[256];
  const int c = blockIdx.x * 4;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int p = threadIdx.x; p < nparts; p += 256) {
    const float4 v = *reinterpret_cast<const float4*>(part + (size_t)p * cols + c);
    s.x += v.x;
    s.y += v.y;
    s.z += v.z;
    s.w += v.w;
  }
  sh[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) {
      const float4 o = sh[threadIdx.x + w];
      float4& m = sh[threadIdx.x];
      m.x += o.x;
      m.y += o.y;
      m.z += o.z;
      m.w += o.w;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) *reinterpret_cast<float4*>(out + c) = sh[0];
}

bool lrn_pool_fused_ok(const float* a, const float* y, const float* dy, const float* da, const uint8_t* slot, int C,
                       int n) {
  // the smallest pooled tile (2 x 2) needs 25 normalised pixels in LDS
  return lrn_vec_ok(a, y, dy ? dy : a, C, n / 2) && C <= 512 && aligned16(da ? da : a) && ((uintptr_t)slot & 3) == 0;
}
size_t lrn_part_floats(int C) { return (size_t)kLrnMaxBlocks * C; }
// 20 KiB measured best (conv1: 103 us per step against 150 with 64 KiB tiles, which leave too few workgroups per CU)
constexpr size_t kLrnPoolLds = 20 * 1024;

int launch_lrn_pool_fwd(const float* a, float* y, uint8_t* slot, int N, int H, int W, int C, int Ho, int Wo, int n,
                        float k, float alpha, float beta, hipStream_t st, uint16_t* y16) {
  const size_t total = (size_t)N * Ho * Wo * C;
  if (!total) return ALEXNET_OK;
  // pooled tile edge: the normalised input pixels under a tile fill at most kLrnPoolLds bytes of LDS (25 pixels
  // at least); a tile of p x p pooled pixels reads (2p+1)^2 input pixels for the 4p^2 it owns
  int pt = 2;
  while ((size_t)(2 * pt + 3) * (2 * pt + 3) * C * 4 <= kLrnPoolLds && pt < 8) ++pt;
  const int PH = std::min(pt, Ho), PW = std::min(pt, Wo);
  const int tiles_y = ceil_div(Ho, PH), tiles_x = ceil_div(Wo, PW);
  const size_t lds = (size_t)(2 * PH + 1) * (2 * PW + 1) * C * sizeof(float);
  KernelScope ks("lrn_pool_fwd", 0, (double)N * H * W * C * 4.0 + (double)total * 5.0, st);
  hipLaunchKernelGGL(lrn_pool_fwd_kernel, dim3((unsigned)(N * tiles_y * tiles_x)), dim3(256), lds, st, a, y, slot, H, W,
                     C, Ho, Wo, PH, PW, tiles_y, tiles_x, n / 2, k, alpha, beta, y16);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

size_t lrn_part_rows(long pixels, int C) { return (size_t)lrn_grid(pixels, 256 / (C / 4)); }
int launch_pool_lrn_bwd(const float* a, const float* dy, const uint8_t* slot, float* da, int N, int H, int W, int C,
                        int Ho, int Wo, int n, float k, float alpha, float beta, int relu_gate, float* colsum_out,
                        float* part, hipStream_t st, bool partials_only, uint16_t* da16) {
  const long pixels = (long)N * H * W;
  if (!pixels) return ALEXNET_OK;
  const int PB = 256 / (C / 4);
  const int blocks = lrn_grid(pixels, PB);
  const bool sums = colsum_out || partials_only;
  {
    KernelScope ks("pool_lrn_bwd", 0, (double)pixels * C * 8.0 + (double)N * Ho * Wo * C * 5.0, st);
    const size_t lds = (size_t)2 * PB * (C + 2 * kLrnPad) * sizeof(float);
    const PoolGather pg{dy, slot, H, W, Ho, Wo, make_fastdiv((uint32_t)W), make_fastdiv((uint32_t)H)};
    hipLaunchKernelGGL((lrn_vec_kernel<true, true>), dim3(blocks), dim3(256), lds, st, a, nullptr, da, pixels, C, n / 2,
                       PB, k, alpha, beta, relu_gate, pg, sums ? part : nullptr, da16);
    AX_LAUNCH_CHECK();
  }
  if (colsum_out && !partials_only) {
    KernelScope ks("colsum_finish", 0, (double)blocks * C * 4.0, st);
    hipLaunchKernelGGL(colsum_finish_kernel, dim3(C / 4), dim3(256), 0, st, part, blocks, C, colsum_out);
    AX_LAUNCH_CHECK();
  }
  return ALEXNET_OK;
}

// -------------------------------------------------------------- max pool ---
// 3x3 stride-2 windows scanned row-major; a tap replaces the running maximum
// only when strictly greater (first maximum wins).  slot = r*3 + s of the
// winner, one byte per output element.
__global__ void pool_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, uint8_t* __restrict__ slot,
                                int N, int H, int W, int C, int Ho, int Wo, uint16_t* __restrict__ y16) {
  const size_t total = (size_t)N * Ho * Wo * C;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % C);
  size_t p = i / C;
  const int xo = (int)(p % Wo);
  p /= Wo;
  const int yo = (int)(p % Ho);
  const size_t n = p / Ho;
  const float* base = x + ((n * H + 2 * yo) * W + 2 * xo) * C + c;
  float best = base[0];
  int bs = 0;
#pragma unroll
  for (int r = 0; r < 3; ++r)
#pragma unroll
    for (int s = 0; s < 3; ++s) {
      if (r == 0 && s == 0) continue;
      const float v = base[((size_t)r * W + s) * C];
      if (v > best) {
        best = v;
        bs = r * 3 + s;
      }
    }
  y[i] = best;
  if (y16) store_bf16(y16 + i, best);
  slot[i] = (uint8_t)bs;
}
int launch_pool_fwd(const float* x, float* y, uint8_t* slot, int N, int H, int W, int C, int Ho, int Wo,
                    hipStream_t st, uint16_t* y16) {
  const size_t total = (size_t)N * Ho * Wo * C;
  if (!total) return ALEXNET_OK;
  KernelScope ks("pool_fwd", 0, (double)N * H * W * C * 4.0 + (double)total * 5.0, st);
  hipLaunchKernelGGL(pool_fwd_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, x, y, slot, N, H, W, C, Ho, Wo,
                     y16);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// Gather form of the pooling adjoint: each input element looks at the (at
// most four) windows covering it and adds dy of those that chose it.
__global__ void pool_bwd_kernel(const float* __restrict__ dy, const uint8_t* __restrict__ slot,
                                const float* __restrict__ gate, float* __restrict__ dx, int N, int H, int W, int C,
                                int Ho, int Wo) {
  const size_t total = (size_t)N * H * W * C;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % C);
  size_t p = i / C;
  const int x = (int)(p % W);
  p /= W;
  const int y = (int)(p % H);
  const size_t n = p / H;
  float acc = 0.f;
  if (!gate || gate[i] > 0.f) {
    const int yo_lo = y >= 2 ? (y - 1) / 2 : 0, yo_hi = min(y / 2, Ho - 1);
    const int xo_lo = x >= 2 ? (x - 1) / 2 : 0, xo_hi = min(x / 2, Wo - 1);
    for (int yo = yo_lo; yo <= yo_hi; ++yo)
      for (int xo = xo_lo; xo <= xo_hi; ++xo) {
        const size_t o = ((n * Ho + yo) * Wo + xo) * C + c;
        const int want = (y - 2 * yo) * 3 + (x - 2 * xo);
        if ((int)slot[o] == want) acc += dy[o];
      }
  }
  dx[i] = acc;
}
// Same gather with a lane owning four consecutive channels (C % 4 == 0).
__global__ void pool_bwd_vec_kernel(const float* __restrict__ dy, const uint8_t* __restrict__ slot,
                                    const float* __restrict__ gate, float* __restrict__ dx, int N, int H, int W, int C,
                                    int Ho, int Wo, uint16_t* __restrict__ dx16) {
  const int cq = C >> 2;
  const size_t total = (size_t)N * H * W * cq;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % cq) * 4;
  size_t p = i / cq;
  const int x = (int)(p % W);
  p /= W;
  const int y = (int)(p % H);
  const size_t n = p / H;
  const size_t e = i * 4;  // element index of (n, y, x, c)
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  const int yo_lo = y >= 2 ? (y - 1) / 2 : 0, yo_hi = min(y / 2, Ho - 1);
  const int xo_lo = x >= 2 ? (x - 1) / 2 : 0, xo_hi = min(x / 2, Wo - 1);
  for (int yo = yo_lo; yo <= yo_hi; ++yo)
    for (int xo = xo_lo; xo <= xo_hi; ++xo) {
      const size_t o = ((n * Ho + yo) * Wo + xo) * C + c;
      const uint32_t want = (uint32_t)((y - 2 * yo) * 3 + (x - 2 * xo));
      const uint32_t s4 = *reinterpret_cast<const uint32_t*>(slot + o);
      const float4 d = *reinterpret_cast<const float4*>(dy + o);
      acc.x += (s4 & 0xffu) == want ? d.x : 0.f;
      acc.y += ((s4 >> 8) & 0xffu) == want ? d.y : 0.f;
      acc.z += ((s4 >> 16) & 0xffu) == want ? d.z : 0.f;
      acc.w += (s4 >> 24) == want ? d.w : 0.f;
    }
  if (gate) {
    const float4 g = *reinterpret_cast<const float4*>(gate + e);
    acc.x = g.x > 0.f ? acc.x : 0.f;
    acc.y = g.y > 0.f ? acc.y : 0.f;
    acc.z = g.z > 0.f ? acc.z : 0.f;
    acc.w = g.w > 0.f ? acc.w : 0.f;
  }
  *reinterpret_cast<float4*>(dx + e) = acc;
  if (dx16) store_bf16x4(dx16 + e, acc);
}
// dx16 (may be null): where to leave a bf16 copy of dx
int launch_pool_bwd(const float* dy, const uint8_t* slot, const float* gate, float* dx, int N, int H, int W, int C,
                    int Ho, int Wo, hipStream_t st, uint16_t* dx16) {
  const size_t total = (size_t)N * H * W * C;
  if (!total) return ALEXNET_OK;
  {
    KernelScope ks("pool_bwd", 0, (double)total * (gate ? 8.0 : 4.0) + (double)N * Ho * Wo * C * 5.0, st);
    if (C % 4 == 0 && aligned16(dy) && aligned16(dx) && (!gate || aligned16(gate)) && ((uintptr_t)slot & 3) == 0 &&
        ((uintptr_t)dx16 & 7) == 0) {
      hipLaunchKernelGGL(pool_bwd_vec_kernel, dim3(grid_for(total / 4, 256)), dim3(256), 0, st, dy, slot, gate, dx, N,
                         H, W, C, Ho, Wo, dx16);
      AX_LAUNCH_CHECK();
      return ALEXNET_OK;
    }
    hipLaunchKernelGGL(pool_bwd_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, dy, slot, gate, dx, N, H, W, C, Ho,
                       Wo);
    AX_LAUNCH_CHECK();
  }
  return dx16 ? launch_to_bf16(dx, dx16, total, st) : ALEXNET_OK;
}

// slot bytes (channel-last) -> canonical int32 NCHW index y_in*W + x_in
__global__ void pool_argmax_canonical_kernel(const uint8_t* __restrict__ slot, int32_t* __restrict__ out, int N,
                                             int C, int Ho, int Wo, int W) {
  const size_t total = (size_t)N * C * Ho * Wo;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // nchw index
  if (i >= total) return;
  const int xo = (int)(i % Wo);
  size_t q = i / Wo;
  const int yo = (int)(q % Ho);
  q /= Ho;
  const int c = (int)(q % C);
  const size_t n = q / C;
  const int s = slot[((n * Ho + yo) * Wo + xo) * C + c];
  out[i] = (2 * yo + s / 3) * W + 2 * xo + s % 3;
}
int launch_pool_argmax_canonical(const uint8_t* slot, int32_t* out_nchw, int N, int C, int Ho, int Wo, int W,
                                 hipStream_t st) {
  const size_t total = (size_t)N * C * Ho * Wo;
  if (!total) return ALEXNET_OK;
  hipLaunchKernelGGL(pool_argmax_canonical_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, slot, out_nchw, N,
                     C, Ho, Wo, W);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// --------------------------------------------------- softmax cross-entropy ---
__device__ __forceinline__ float wave_max(float v) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
// all 256 threads receive the block-wide result; order of combination is fixed
__device__ __forceinline__ float block_reduce(float v, float* sh, bool is_max) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  v = is_max ? wave_max(v) : wave_sum(v);
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  float r = sh[0];
  for (int w = 1; w < (int)(blockDim.x >> 6); ++w) r = is_max ? fmaxf(r, sh[w]) : r + sh[w];
  return r;
}

// one workgroup per row; p = exp(z - max - log(sum exp))
__global__ void __launch_bounds__(256)
softmax_xent_kernel(const float* __restrict__ z, const int32_t* __restrict__ labels, int B, int classes, int mode,
                    float* __restrict__ out, float* __restrict__ row_loss, int32_t* __restrict__ err_flag) {
  __shared__ float sh[4];
  const int n = blockIdx.x;
  const float* zr = z + (size_t)n * classes;
  float m = -INFINITY;
  for (int j = threadIdx.x; j < classes; j += blockDim.x) m = fmaxf(m, zr[j]);
  m = block_reduce(m, sh, true);
  float s = 0.f;
  for (int j = threadIdx.x; j < classes; j += blockDim.x) s += expf(zr[j] - m);
  s = block_reduce(s, sh, false);
  const float lse = logf(s);
  int lab = 0;
  if (mode == 0) {
    lab = labels[n];
    if (lab < 0 || lab >= classes) {
      if (threadIdx.x == 0) atomicOr(err_flag, 1);
      lab = lab < 0 ? 0 : classes - 1;
    }
    if (threadIdx.x == 0) row_loss[n] = -(zr[lab] - m - lse);
  }
  const float inv_b = 1.0f / (float)B;
  for (int j = threadIdx.x; j < classes; j += blockDim.x) {
    const float p = expf(zr[j] - m - lse);
    out[(size_t)n * classes + j] = mode == 0 ? (p - (j == lab ? 1.f : 0.f)) * inv_b : p;
  }
}
int launch_softmax_xent(const float* z, const int32_t* labels, int B, int classes, int mode, float* out,
                        float* row_loss, int32_t* err_flag, hipStream_t st) {
  KernelScope ks("softmax_xent", 0, (double)B * classes * 8.0, st);
  hipLaunchKernelGGL(softmax_xent_kernel, dim3(B), dim3(256), 0, st, z, labels, B, classes, mode, out, row_loss,
                     err_flag);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

__global__ void __launch_bounds__(256) mean_loss_kernel(const float* __restrict__ row_loss, int B, float* loss) {
  __shared__ float sh[4];
  float s = 0.f;
  for (int j = threadIdx.x; j < B; j += blockDim.x) s += row_loss[j];
  s = block_reduce(s, sh, false);
  if (threadIdx.x == 0) *loss = s / (float)B;
}
int launch_mean_loss(const float* row_loss, int B, float* loss, hipStream_t st) {
  KernelScope ks("mean_loss", 0, (double)B * 4.0, st);
  hipLaunchKernelGGL(mean_loss_kernel, dim3(1), dim3(256), 0, st, row_loss, B, loss);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// ------------------------------------------------------------ reductions ---
// Column sums of a row-major [rows][cols] matrix (bias gradients), in two
// passes with a fixed combination order so results do not depend on timing.
// Stage 1: a workgroup sums `rpb` rows of a 64-column stripe; 16 row lanes x
// 16 column quads (16-byte loads when VEC), then a fixed-order LDS reduction.
// rpb is chosen by the launcher so that the grid has about a thousand workgroups.
template <bool VEC>
__device__ __forceinline__ void colsum_stage1_block(const float* __restrict__ m, long rows, int cols, int rpb,
                                                    float* __restrict__ part, int stripe, int chunk) {
  __shared__ float sh[16][65];
  const int cq = threadIdx.x & 15, rl = threadIdx.x >> 4;
  const int col = stripe * 64 + cq * 4;
  const long r0 = (long)chunk * rpb;
  const long r1 = min(rows, r0 + rpb);
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (VEC) {
    if (col < cols)
#pragma unroll 8
      for (long r = r0 + rl; r < r1; r += 16) {
        const float4 v = *reinterpret_cast<const float4*>(m + r * cols + col);
        s.x += v.x;
        s.y += v.y;
        s.z += v.z;
        s.w += v.w;
      }
  } else {
    for (long r = r0 + rl; r < r1; r += 16) {
      const float* p = m + r * cols + col;
      if (col < cols) s.x += p[0];
      if (col + 1 < cols) s.y += p[1];
      if (col + 2 < cols) s.z += p[2];
      if (col + 3 < cols) s.w += p[3];
    }
  }
  sh[rl][cq * 4] = s.x;
  sh[rl][cq * 4 + 1] = s.y;
  sh[rl][cq * 4 + 2] = s.z;
  sh[rl][cq * 4 + 3] = s.w;
  __syncthreads();
  if (threadIdx.x < 64) {
    const int c = stripe * 64 + threadIdx.x;
    float t = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) t += sh[r][threadIdx.x];
    if (c < cols) part[(size_t)chunk * cols + c] = t;
  }
}
template <bool VEC>
__global__ void __launch_bounds__(256)
colsum_stage1(const float* __restrict__ m, long rows, int cols, int rpb, float* __restrict__ part) {
  colsum_stage1_block<VEC>(m, rows, cols, rpb, part, blockIdx.x, blockIdx.y);
}
__device__ __forceinline__ void colsum_stage2_block(const float* __restrict__ part, int nparts, int cols,
                                                    float* __restrict__ out, int stripe) {
  __shared__ float sh[4][64];
  const int cl = threadIdx.x & 63, pl = threadIdx.x >> 6;
  const int col = stripe * 64 + cl;
  float s = 0.f;
  if (col < cols) {
#pragma unroll 8
    for (int p = pl; p < nparts; p += 4) s += part[(size_t)p * cols + col];  // eight loads in flight, added in order
  }
  sh[pl][cl] = s;
  __syncthreads();
  if (pl == 0 && col < cols) out[col] = (sh[0][cl] + sh[1][cl]) + (sh[2][cl] + sh[3][cl]);
}
__global__ void __launch_bounds__(256)
colsum_stage2(const float* __restrict__ part, int nparts, int cols, float* __restrict__ out) {
  colsum_stage2_block(part, nparts, cols, out, blockIdx.x);
}
// Several column sums in two launches (the bias gradients of a backward pass, whose inputs all still exist at
// its end).  The jobs' grids are laid end to end: a workgroup finds its job from the running totals (first1,
// first2) and its place in that job's own grid.  Same arithmetic and order per job as colsum_stage1 +
// colsum_stage2.
__device__ __forceinline__ int colsum_job_of(const int* first, int n, int block) {
  int j = 0;
#pragma unroll
  for (int k = 1; k < kMaxColsumJobs; ++k)
    if (k < n && block >= first[k]) j = k;
  return j;
}
template <bool VEC>
__global__ void __launch_bounds__(256) colsum_batch_stage1(ColsumBatch b) {
  const int ji = colsum_job_of(b.first1, b.n, blockIdx.x);
  const ColsumJob& j = b.job[ji];
  const int local = blockIdx.x - b.first1[ji], stripes = (j.cols + 63) / 64;
  colsum_stage1_block<VEC>(j.m, j.rows, j.cols, j.rpb, j.part, local % stripes, local / stripes);
}
__global__ void __launch_bounds__(256) colsum_batch_stage2(ColsumBatch b) {
  const int ji = colsum_job_of(b.first2, b.n, blockIdx.x);
  const ColsumJob& j = b.job[ji];
  colsum_stage2_block(j.part, j.nparts, j.cols, j.out, blockIdx.x - b.first2[ji]);
}
// rows per workgroup: enough row chunks for ~1024 workgroups, at least 64 rows each
static int colsum_rows_per_block(long rows, int cols) {
  const int stripes = ceil_div(cols, 64);
  const int want_chunks = std::max(1, 1024 / stripes);
  long rpb = (rows + want_chunks - 1) / want_chunks;
  rpb = (rpb + 15) / 16 * 16;
  return (int)std::max(64L, rpb);
}
size_t colsum_ws_floats(long rows, int cols) {
  return (size_t)ceil_div(rows, colsum_rows_per_block(rows, cols)) * cols;
}
int launch_colsum(const float* m, long rows, int cols, float* out, float* ws, hipStream_t st) {
  const int rpb = colsum_rows_per_block(rows, cols);
  const int nparts = ceil_div(rows, rpb);
  KernelScope ks("colsum", 0, (double)rows * cols * 4.0, st);
  if (cols % 4 == 0 && aligned16(m))
    hipLaunchKernelGGL((colsum_stage1<true>), dim3(ceil_div(cols, 64), nparts), dim3(256), 0, st, m, rows, cols, rpb,
                       ws);
  else
    hipLaunchKernelGGL((colsum_stage1<false>), dim3(ceil_div(cols, 64), nparts), dim3(256), 0, st, m, rows, cols, rpb,
                       ws);
  AX_LAUNCH_CHECK();
  if (cols % 4 == 0)
    hipLaunchKernelGGL(colsum_finish_kernel, dim3(cols / 4), dim3(256), 0, st, ws, nparts, cols, out);
  else
    hipLaunchKernelGGL(colsum_stage2, dim3(ceil_div(cols, 64)), dim3(256), 0, st, ws, nparts, cols, out);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

int colsum_batch_add(ColsumBatch& b, const float* m, long rows, int cols, float* out, float* ws, size_t* ws_used) {
  if (b.n >= kMaxColsumJobs) {
    set_error("colsum batch: more than %d jobs", kMaxColsumJobs);
    return ALEXNET_EINVAL;
  }
  ColsumJob& j = b.job[b.n++];
  j.m = m; j.rows = rows; j.cols = cols; j.out = out;
  j.rpb = colsum_rows_per_block(rows, cols);
  j.nparts = ceil_div(rows, j.rpb);
  j.part = ws + *ws_used;
  *ws_used += ((size_t)j.nparts * cols + 3) / 4 * 4;  // every job's partials start on a 16-byte boundary
  const int stripes = ceil_div(cols, 64), k = b.n - 1;
  b.first1[k] = b.blocks1;
  b.first2[k] = b.blocks2;
  b.blocks1 += stripes * j.nparts;
  b.blocks2 += stripes;
  return ALEXNET_OK;
}
size_t colsum_batch_ws_floats(long rows, int cols) { return (colsum_ws_floats(rows, cols) + 3) / 4 * 4; }
int launch_colsum_batch(const ColsumBatch& b, hipStream_t st) {
  if (b.n == 0) return ALEXNET_OK;
  bool vec = true;
  double bytes = 0;
  for (int i = 0; i < b.n; ++i) {
    const ColsumJob& j = b.job[i];
    vec = vec && j.cols % 4 == 0 && aligned16(j.m);
    bytes += (double)j.rows * j.cols * 4.0;
  }
  KernelScope ks("colsum", 0, bytes, st);
  if (vec)
    hipLaunchKernelGGL((colsum_batch_stage1<true>), dim3(b.blocks1), dim3(256), 0, st, b);
  else
    hipLaunchKernelGGL((colsum_batch_stage1<false>), dim3(b.blocks1), dim3(256), 0, st, b);
  AX_LAUNCH_CHECK();
  hipLaunchKernelGGL(colsum_batch_stage2, dim3(b.blocks2), dim3(256), 0, st, b);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// out[g][i] = sum_s ws[g*nsplit + s][i]  (split-k partial slabs)
__device__ __forceinline__ void reduce_slabs_block(const float* __restrict__ ws, int nsplit, size_t slab, int groups,
                                                   float* __restrict__ out, unsigned block) {
  // 64 consecutive elements per workgroup; four lanes per element take every fourth slab, then add up in a
  // fixed order
  __shared__ float sh[4][64];
  const size_t total = slab * groups;
  const int el = threadIdx.x & 63, part = threadIdx.x >> 6;
  const size_t i = (size_t)block * 64 + el;
  float s = 0.f;
  if (i < total) {
    const size_t g = i / slab, e = i - g * slab;
    const float* p = ws + g * nsplit * slab + e;
#pragma unroll 8
    for (int k = part; k < nsplit; k += 4) s += p[(size_t)k * slab];
  }
  sh[part][el] = s;
  __syncthreads();
  if (part == 0 && i < total) out[i] = (sh[0][el] + sh[1][el]) + (sh[2][el] + sh[3][el]);
}
__global__ void __launch_bounds__(256)
reduce_slabs_kernel(const float* __restrict__ ws, int nsplit, size_t slab, int groups, float* __restrict__ out) {
  reduce_slabs_block(ws, nsplit, slab, groups, out, blockIdx.x);
}
// The same for one result whose rows are runs padded to `run` entries (run mode of the first layer's weight
// gradient): row (r, j) goes to row r*kc + j of the packed layout, the padding rows j >= kc nowhere.
__global__ void __launch_bounds__(256)
reduce_slabs_unpack_kernel(const float* __restrict__ ws, int nsplit, size_t slab, int run, int kc, int cout,
                           float* __restrict__ out) {
  __shared__ float sh[4][64];
  const int el = threadIdx.x & 63, part = threadIdx.x >> 6;
  const size_t i = (size_t)blockIdx.x * 64 + el;
  float s = 0.f;
  if (i < slab) {
    const float* p = ws + i;
#pragma unroll 8
    for (int k = part; k < nsplit; k += 4) s += p[(size_t)k * slab];
  }
  sh[part][el] = s;
  __syncthreads();
  if (part == 0 && i < slab) {
    const size_t row = i / cout;
    const int o = (int)(i - row * cout), r = (int)(row / run), j = (int)(row - (size_t)r * run);
    if (j < kc) out[((size_t)r * kc + j) * cout + o] = (sh[0][el] + sh[1][el]) + (sh[2][el] + sh[3][el]);
  }
}
int launch_reduce_slabs_unpack(const float* ws, int nsplit, long slab, int run, int kc, int cout, float* out,
                               hipStream_t st) {
  if (!slab) return ALEXNET_OK;
  KernelScope ks("reduce_slabs", 0, (double)slab * 4.0 * (nsplit + 1), st);
  hipLaunchKernelGGL(reduce_slabs_unpack_kernel, dim3(grid_for((size_t)slab, 64)), dim3(256), 0, st, ws, nsplit,
                     (size_t)slab, run, kc, cout, out);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}
// Few slices of a large result (slab a multiple of four floats, 16-byte aligned): a lane owns four consecutive
// elements and adds its slices in order, 16 bytes per load.
constexpr int kReduceVecMaxSlices = 32;
__device__ __forceinline__ void reduce_slabs_vec_block(const float* __restrict__ ws, int nsplit, size_t slab,
                                                       int groups, float* __restrict__ out, unsigned block) {
  const size_t i = ((size_t)block * 256 + threadIdx.x) * 4;
  if (i >= slab * groups) return;
  const size_t g = i / slab, e = i - g * slab;
  const float* p = ws + g * nsplit * slab + e;
  float4 acc = *reinterpret_cast<const float4*>(p);
#pragma unroll 4
  for (int k = 1; k < nsplit; ++k) {
    const float4 v = *reinterpret_cast<const float4*>(p + (size_t)k * slab);
    acc.x += v.x;
    acc.y += v.y;
    acc.z += v.z;
    acc.w += v.w;
  }
  *reinterpret_cast<float4*>(out + i) = acc;
}
static bool reduce_vec_ok(const float* ws, const float* out, int nsplit, long slab) {
  return nsplit <= kReduceVecMaxSlices && slab % 4 == 0 && aligned16(ws) && aligned16(out);
}
static int reduce_blocks(bool vec, long slab, int groups) {
  return vec ? ceil_div(slab * groups / 4, 256) : ceil_div(slab * groups, 64);
}
__global__ void __launch_bounds__(256)
reduce_slabs_vec_kernel(const float* __restrict__ ws, int nsplit, size_t slab, int groups, float* __restrict__ out) {
  reduce_slabs_vec_block(ws, nsplit, slab, groups, out, blockIdx.x);
}
// the same for several results in one launch (see WgradTail): the jobs' grids laid end to end
__global__ void __launch_bounds__(256) reduce_slabs_batch_kernel(WgradTail t) {
  int ji = 0;
#pragma unroll
  for (int k = 1; k < kMaxWgradJobs; ++k)
    if (k < t.n && (int)blockIdx.x >= t.first_r[k]) ji = k;
  const WgradJob& j = t.job[ji];
  if (j.vec)  // uniform over the workgroup
    reduce_slabs_vec_block(j.slices, j.nsplit, (size_t)j.slab, j.groups36, j.dU, blockIdx.x - t.first_r[ji]);
  else
    reduce_slabs_block(j.slices, j.nsplit, (size_t)j.slab, j.groups36, j.dU, blockIdx.x - t.first_r[ji]);
}
void wgrad_tail_add(WgradTail& t, const WgradJob& job) {
  const int k = t.n++;
  WgradJob& j = t.job[k];
  j = job;
  j.vec = reduce_vec_ok(j.slices, j.dU, j.nsplit, j.slab) ? 1 : 0;
  t.first_r[k] = t.blocks_r;
  t.first_t[k] = t.blocks_t;
  if (j.nsplit > 1) t.blocks_r += reduce_blocks(j.vec != 0, j.slab, j.groups36);
  t.blocks_t += ceil_div(j.total, 256);
}
int launch_reduce_slabs_batch(const WgradTail& t, hipStream_t st) {
  if (t.blocks_r == 0) return ALEXNET_OK;
  double bytes = 0;
  for (int i = 0; i < t.n; ++i)
    if (t.job[i].nsplit > 1) bytes += (double)t.job[i].slab * t.job[i].groups36 * 4.0 * (t.job[i].nsplit + 1);
  KernelScope ks("reduce_slabs", 0, bytes, st);
  hipLaunchKernelGGL(reduce_slabs_batch_kernel, dim3(t.blocks_r), dim3(256), 0, st, t);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}
int launch_reduce_slabs(const float* ws, int nsplit, long slab, int groups, float* out, hipStream_t st) {
  const size_t total = (size_t)slab * groups;
  if (!total) return ALEXNET_OK;
  KernelScope ks("reduce_slabs", 0, (double)total * 4.0 * (nsplit + 1), st);
  if (reduce_vec_ok(ws, out, nsplit, slab))
    hipLaunchKernelGGL(reduce_slabs_vec_kernel, dim3(reduce_blocks(true, slab, groups)), dim3(256), 0, st, ws, nsplit,
                       (size_t)slab, groups, out);
  else
    hipLaunchKernelGGL(reduce_slabs_kernel, dim3(grid_for(total, 64)), dim3(256), 0, st, ws, nsplit, (size_t)slab,
                       groups, out);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// ---------------------------------------------------------------- update ---
// v <- mu v - lr (g + wd w);  w <- w + v.  Elements below n_decay are weights
// (decayed), the rest are biases (not decayed).
// Two pieces of the vectors in one launch: elements [0, n1) and [n1 + gap, n + gap) (n1 a multiple of four, or
// gap = 0); n_decay counts positions in the vectors, not elements of the launch.
__global__ void __launch_bounds__(256)
sgd_update_kernel(float* __restrict__ w, float* __restrict__ v, const float* __restrict__ g, size_t n, size_t n1,
                  size_t gap, size_t n_decay, float lr, float mu, float wd) {
  // grid-stride over groups of four: a bounded number of workgroups, so that a GEMM running beside this
  // kernel on another stream still finds room on every CU
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x; q * 4 < n; q += stride) {
    const size_t e = q * 4, i = e < n1 ? e : e + gap;
    if (e + 3 < n) {
      float4 w4 = *reinterpret_cast<float4*>(w + i);
      float4 v4 = *reinterpret_cast<float4*>(v + i);
      const float4 g4 = *reinterpret_cast<const float4*>(g + i);
      const float d0 = i + 0 < n_decay ? wd : 0.f, d1 = i + 1 < n_decay ? wd : 0.f;
      const float d2 = i + 2 < n_decay ? wd : 0.f, d3 = i + 3 < n_decay ? wd : 0.f;
      v4.x = mu * v4.x - lr * (g4.x + d0 * w4.x);
      v4.y = mu * v4.y - lr * (g4.y + d1 * w4.y);
      v4.z = mu * v4.z - lr * (g4.z + d2 * w4.z);
      v4.w = mu * v4.w - lr * (g4.w + d3 * w4.w);
      w4.x += v4.x;
      w4.y += v4.y;
      w4.z += v4.z;
      w4.w += v4.w;
      *reinterpret_cast<float4*>(v + i) = v4;
      *reinterpret_cast<float4*>(w + i) = w4;
    } else {
      for (size_t j = i; j < n + (e < n1 ? 0 : gap); ++j) {
        const float d = j < n_decay ? wd : 0.f;
        v[j] = mu * v[j] - lr * (g[j] + d * w[j]);
        w[j] += v[j];
      }
    }
  }
}
constexpr unsigned kUpdateMaxBlocks = 1024;  // 4 per CU
int launch_sgd_update(float* w, float* v, const float* g, size_t n, size_t n_decay, float lr, float mu, float wd,
                      hipStream_t st, unsigned max_blocks) {
  if (!n) return ALEXNET_OK;
  KernelScope ks("sgd_update", 0, (double)n * 20.0, st);
  const unsigned blocks = std::min<unsigned>(grid_for((n + 3) / 4, 256), max_blocks ? max_blocks : kUpdateMaxBlocks);
  hipLaunchKernelGGL(sgd_update_kernel, dim3(blocks), dim3(256), 0, st, w, v, g, n, n, (size_t)0, n_decay, lr, mu, wd);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}
// elements [0, n1) and [begin2, end2) of the vectors in one launch; n1 a multiple of four, begin2 >= n1
int launch_sgd_update_two(float* w, float* v, const float* g, size_t n1, size_t begin2, size_t end2, size_t n_decay,
                          float lr, float mu, float wd, hipStream_t st) {
  const size_t n = n1 + (end2 - begin2);
  if (!n) return ALEXNET_OK;
  KernelScope ks("sgd_update", 0, (double)n * 20.0, st);
  const unsigned blocks = std::min<unsigned>(grid_for((n + 3) / 4, 256), kUpdateMaxBlocks);
  hipLaunchKernelGGL(sgd_update_kernel, dim3(blocks), dim3(256), 0, st, w, v, g, n, n1, begin2 - n1, n_decay, lr, mu,
                     wd);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// --------------------------------------------------- replica averaging ------
// Paper Section 2.2, steps 2+3 on one GPU: the peer replica is the staging
// copy, so exchange and average collapse into one pass that writes the mean
// to both sides.
__global__ void average_kernel(float* __restrict__ a, float* __restrict__ b, size_t n) {
  const size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t i = q * 4;
  if (i + 3 < n) {
    const float4 x = *reinterpret_cast<const float4*>(a + i);
    const float4 y = *reinterpret_cast<const float4*>(b + i);
    float4 m;
    m.x = 0.5f * (x.x + y.x);
    m.y = 0.5f * (x.y + y.y);
    m.z = 0.5f * (x.z + y.z);
    m.w = 0.5f * (x.w + y.w);
    *reinterpret_cast<float4*>(a + i) = m;
    *reinterpret_cast<float4*>(b + i) = m;
  } else {
    for (size_t j = i; j < n; ++j) {
      const float m = 0.5f * (a[j] + b[j]);
      a[j] = m;
      b[j] = m;
    }
  }
}
int launch_average(float* a, float* b, size_t n, hipStream_t st) {
  if (!n) return ALEXNET_OK;
  KernelScope ks("average", 0, (double)n * 16.0, st);
  hipLaunchKernelGGL(average_kernel, dim3(grid_for((n + 3) / 4, 256)), dim3(256), 0, st, a, b, n);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// Gradient exchange: g = 0.5 (ga + gb), then each replica's own  v <- mu v - lr (g + wd w);  w <- w + v.
// Replicas that hold the same w and v end up bit-identical (same arithmetic on the same values).
__device__ __forceinline__ void sgd_one(float& w, float& v, float g, float d, float lr, float mu) {
  v = mu * v - lr * (g + d * w);
  w += v;
}
__global__ void avg_grad_update_kernel(float* __restrict__ wa, float* __restrict__ va, const float* __restrict__ ga,
                                       float* __restrict__ wb, float* __restrict__ vb, const float* __restrict__ gb,
                                       size_t n, size_t n_decay, float lr, float mu, float wd) {
  const size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t i = q * 4;
  if (i + 3 < n) {
    float4 w1 = *reinterpret_cast<float4*>(wa + i), v1 = *reinterpret_cast<float4*>(va + i);
    float4 w2 = *reinterpret_cast<float4*>(wb + i), v2 = *reinterpret_cast<float4*>(vb + i);
    const float4 g1 = *reinterpret_cast<const float4*>(ga + i), g2 = *reinterpret_cast<const float4*>(gb + i);
    const float4 g = make_float4(0.5f * (g1.x + g2.x), 0.5f * (g1.y + g2.y), 0.5f * (g1.z + g2.z), 0.5f * (g1.w + g2.w));
    const float d0 = i + 0 < n_decay ? wd : 0.f, d1 = i + 1 < n_decay ? wd : 0.f;
    const float d2 = i + 2 < n_decay ? wd : 0.f, d3 = i + 3 < n_decay ? wd : 0.f;
    sgd_one(w1.x, v1.x, g.x, d0, lr, mu);
    sgd_one(w1.y, v1.y, g.y, d1, lr, mu);
    sgd_one(w1.z, v1.z, g.z, d2, lr, mu);
    sgd_one(w1.w, v1.w, g.w, d3, lr, mu);
    sgd_one(w2.x, v2.x, g.x, d0, lr, mu);
    sgd_one(w2.y, v2.y, g.y, d1, lr, mu);
    sgd_one(w2.z, v2.z, g.z, d2, lr, mu);
    sgd_one(w2.w, v2.w, g.w, d3, lr, mu);
    *reinterpret_cast<float4*>(va + i) = v1;
    *reinterpret_cast<float4*>(wa + i) = w1;
    *reinterpret_cast<float4*>(vb + i) = v2;
    *reinterpret_cast<float4*>(wb + i) = w2;
  } else {
    for (size_t j = i; j < n; ++j) {
      const float d = j < n_decay ? wd : 0.f, g = 0.5f * (ga[j] + gb[j]);
      sgd_one(wa[j], va[j], g, d, lr, mu);
      sgd_one(wb[j], vb[j], g, d, lr, mu);
    }
  }
}
int launch_avg_grad_update(float* wa, float* va, const float* ga, float* wb, float* vb, const float* gb, size_t n,
                           size_t n_decay, float lr, float mu, float wd, hipStream_t st) {
  if (!n) return ALEXNET_OK;
  KernelScope ks("avg_grad_update", 0, (double)n * 40.0, st);
  hipLaunchKernelGGL(avg_grad_update_kernel, dim3(grid_for((n + 3) / 4, 256)), dim3(256), 0, st, wa, va, ga, wb, vb, gb,
                     n, n_decay, lr, mu, wd);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// counts[j] += number of rows whose label has fewer than ks[j] classes scoring strictly higher (one
// workgroup per row; integer atomics, so the result does not depend on the order)
struct TopK {
  int n;
  int k[8];
};
__global__ void __launch_bounds__(256)
topk_count_kernel(const float* __restrict__ z, const int32_t* __restrict__ labels, int classes, TopK tk,
                  int32_t* __restrict__ counts, int32_t* __restrict__ err_flag) {
  __shared__ int sh[4];
  const int row = blockIdx.x;
  int lab = labels[row];
  if (lab < 0 || lab >= classes) {
    if (threadIdx.x == 0) *err_flag = 1;
    lab = min(max(lab, 0), classes - 1);
  }
  const float* zr = z + (size_t)row * classes;
  const float own = zr[lab];
  int higher = 0;
  for (int c = threadIdx.x; c < classes; c += 256) higher += zr[c] > own ? 1 : 0;
  for (int o = 32; o > 0; o >>= 1) higher += __shfl_down(higher, o, 64);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = higher;
  __syncthreads();
  if (threadIdx.x == 0) {
    const int total = sh[0] + sh[1] + sh[2] + sh[3];
    for (int j = 0; j < tk.n; ++j)
      if (total < tk.k[j]) atomicAdd(counts + j, 1);
  }
}
int launch_topk_count(const float* z, const int32_t* labels, int B, int classes, const int32_t* ks, int nk,
                      int32_t* counts, int32_t* err_flag, hipStream_t st) {
  if (nk < 1 || nk > 8) {
    set_error("top-k count: between 1 and 8 values of k");
    return ALEXNET_EINVAL;
  }
  TopK tk;
  tk.n = nk;
  for (int j = 0; j < 8; ++j) tk.k[j] = j < nk ? ks[j] : 0;
  KernelScope ks_("topk_count", 0, (double)B * classes * 4.0, st);
  hipLaunchKernelGGL(topk_count_kernel, dim3(B), dim3(256), 0, st, z, labels, classes, tk, counts, err_flag);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

// ------------------------------------------------- parameter layouts --------
// canonical w[o][c][r][s]  <->  internal wf[g][(r,s,c)][o%og]
__global__ void conv_weight_pack_kernel(const float* __restrict__ src, float* __restrict__ dst, int Cout, int Cg,
                                        int k, int groups, int dir) {
  const int og = Cout / groups;
  const size_t total = (size_t)Cout * Cg * k * k;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // internal index
  if (i >= total) return;
  const int ol = (int)(i % og);
  size_t q = i / og;
  const int c = (int)(q % Cg);
  q /= Cg;
  const int s = (int)(q % k);
  q /= k;
  const int r = (int)(q % k);
  const int g = (int)(q / k);
  const size_t canon = ((((size_t)(g * og + ol)) * Cg + c) * k + r) * k + s;
  if (dir == 0)
    dst[i] = src[canon];
  else
    dst[canon] = src[i];
}
int launch_conv_weight_pack(const float* src, float* dst, int Cout, int Cg, int k, int groups, int dir,
                            hipStream_t st) {
  const size_t total = (size_t)Cout * Cg * k * k;
  hipLaunchKernelGGL(conv_weight_pack_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, src, dst, Cout, Cg, k,
                     groups, dir);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}
// wb[g][(r,s,o)][c] = wf[g][(r,s,c)][o]
__global__ void conv_weight_wb_kernel(const float* __restrict__ wf, float* __restrict__ wb, int Cout, int Cg, int k,
                                      int groups) {
  const int og = Cout / groups;
  const size_t total = (size_t)Cout * Cg * k * k;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // index into wb
  if (i >= total) return;
  const int c = (int)(i % Cg);
  size_t q = i / Cg;
  const int ol = (int)(q % og);
  q /= og;
  const size_t grs = q;  // (g*k + r)*k + s
  wb[i] = wf[(grs * Cg + c) * og + ol];
}
int launch_conv_weight_wb(const float* wf, float* wb, int Cout, int Cg, int k, int groups, hipStream_t st) {
  const size_t total = (size_t)Cout * Cg * k * k;
  KernelScope ks("weight_transpose", 0, (double)total * 8.0, st);
  hipLaunchKernelGGL(conv_weight_wb_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, wf, wb, Cout, Cg, k,
                     groups);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}
// canonical w[o][(c,hw)]  <->  internal w[o][(hw,c)]
__global__ void fc_weight_permute_kernel(const float* __restrict__ src, float* __restrict__ dst, int out, int C,
                                         int HW, int dir) {
  const size_t total = (size_t)out * C * HW;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // internal index
  if (i >= total) return;
  const int c = (int)(i % C);
  size_t q = i / C;
  const int hw = (int)(q % HW);
  const size_t o = q / HW;
  const size_t canon = (o * C + c) * HW + hw;
  if (dir == 0)
    dst[i] = src[canon];
  else
    dst[canon] = src[i];
}
int launch_fc_weight_permute(const float* src, float* dst, int out, int C, int HW, int dir, hipStream_t st) {
  const size_t total = (size_t)out * C * HW;
  hipLaunchKernelGGL(fc_weight_permute_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, src, dst, out, C, HW,
                     dir);
  AX_LAUNCH_CHECK();
  return ALEXNET_OK;
}

}  // namespace ax
