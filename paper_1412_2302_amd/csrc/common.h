// Shared declarations of the AlexNet HIP library: error plumbing, the
// counter-based generator behind crop / flip / dropout, small device helpers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/alexnet.h"

namespace ax {

// ---- error plumbing ------------------------------------------------------
void set_error(const char* fmt, ...);
const char* get_error();

#define AX_HIP(expr)                                                                 \
  do {                                                                               \
    hipError_t _e = (expr);                                                          \
    if (_e != hipSuccess) {                                                          \
      ax::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e), __FILE__, __LINE__); \
      return ALEXNET_EHIP;                                                           \
    }                                                                                \
  } while (0)

#define AX_LAUNCH_CHECK() AX_HIP(hipGetLastError())

#define AX_TRY(expr)              \
  do {                            \
    int _r = (expr);              \
    if (_r != ALEXNET_OK) return _r; \
  } while (0)

// ---- counter-based random numbers -----------------------------------------
// r(tag, idx) = mix64(k1 ^ (tag << 56) ^ idx), k1 = mix64(mix64(seed + G) ^ step)
// where mix64 is the output function of the public-domain splitmix64 generator.
// Purposes: 1 crop-x, 2 crop-y, 3 flip (idx = picture), 6 / 7 dropout after
// fc6 / fc7 (idx = n*width + f).
enum { TAG_CROP_X = 1, TAG_CROP_Y = 2, TAG_FLIP = 3, TAG_DROP6 = 6, TAG_DROP7 = 7 };

__host__ __device__ inline uint64_t mix64(uint64_t z) {
  z ^= z >> 30;
  z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27;
  z *= 0x94D049BB133111EBull;
  z ^= z >> 31;
  return z;
}
__host__ __device__ inline uint64_t step_key(uint64_t seed, uint64_t step) {
  return mix64(mix64(seed + 0x9E3779B97F4A7C15ull) ^ step);
}
__host__ __device__ inline uint64_t rand_u64(uint64_t key, uint32_t tag, uint64_t idx) {
  return mix64(key ^ ((uint64_t)tag << 56) ^ idx);
}
// keep decision of dropout: top 24 bits against floor(p * 2^24)
__host__ __device__ inline bool dropout_keep(uint64_t key, uint32_t tag, uint64_t idx, uint32_t thresh24) {
  return (uint32_t)(rand_u64(key, tag, idx) >> 40) >= thresh24;
}

inline int ceil_div(long a, long b) { return (int)((a + b - 1) / b); }

// ---- optional per-kernel timing ---------------------------------------------
// When a sink is installed for the calling thread, every kernel launch of the
// library is bracketed by two HIP events on its own stream.  `flops` / `bytes`
// are the algorithmic work of the launch (what the operation must do, not what
// the kernel happens to move).
struct ProfSink {
  virtual void begin(const char* kernel, double flops, double bytes, hipStream_t st) = 0;
  virtual void end(hipStream_t st) = 0;
  virtual ~ProfSink() {}
};
extern thread_local ProfSink* g_prof;
extern thread_local const char* g_prof_ctx;  // e.g. "conv2.bwd_w"; prefixed to kernel names
struct KernelScope {
  hipStream_t st;
  bool on;
  KernelScope(const char* kernel, double flops, double bytes, hipStream_t s) : st(s), on(g_prof != nullptr) {
    if (on) g_prof->begin(kernel, flops, bytes, s);
  }
  ~KernelScope() {
    if (on) g_prof->end(st);
  }
};
struct ProfContext {
  const char* prev;
  explicit ProfContext(const char* c) : prev(g_prof_ctx) { g_prof_ctx = c; }
  ~ProfContext() { g_prof_ctx = prev; }
};

}  // namespace ax
