// Loading thread of Section 2.1 (Figure 1): while the GPU trains on minibatch k, a host thread copies
// minibatch k+1 from the stored pictures ("disk", here an array in ordinary host memory) into pinned
// staging memory and on to the GPU over the caller's side stream (or a stream of its own); mean subtraction,
// crop and mirror then run on the device (alexnet_preprocess) on the caller's side stream.  Uses only the public C ABI and the
// HIP runtime; all buffers are the caller's.
#include <hip/hip_runtime.h>
#include <string.h>

#include <condition_variable>
#include <mutex>
#include <thread>
#include <vector>

#include "common.h"  // brings in the public header

using ax::set_error;

struct alexnet_loader {
  alexnet_t* net;
  int device;
  int batch, depth;
  size_t image_bytes;  // one stored picture
  const uint8_t* host_images;
  const int32_t* host_labels;
  int64_t count;
  uint8_t *pinned_raw, *d_raw;
  int32_t *pinned_labels, *d_labels;
  hipStream_t copy_stream;
  bool own_stream;  // copy_stream was created here (the caller gave none)
  std::vector<hipEvent_t> copy_done, pre_done, step_done;  // one of each per staging set
  std::thread worker;
  std::mutex mu;
  std::condition_variable cv;
  uint64_t produced;  // minibatches whose copies have been issued
  uint64_t staged;    // minibatches handed to alexnet_loader_stage
  uint64_t released;  // minibatches whose training step has been enqueued (alexnet_loader_done)
  bool stop;
  int worker_error;  // hipError_t of the first failure in the thread, 0 if none
};

namespace {

constexpr int kCopyThreads = 4;  // threads that copy one minibatch from the stored pictures into pinned staging

void loader_thread(alexnet_loader* L) {
  if (hipSetDevice(L->device) != hipSuccess) {
    std::lock_guard<std::mutex> g(L->mu);
    L->worker_error = 1;
    L->cv.notify_all();
    return;
  }
  const size_t raw_bytes = (size_t)L->batch * L->image_bytes;
  for (uint64_t k = 0;; ++k) {
    {
      // staging set k % depth is free once the step that used minibatch k - depth has been enqueued
      std::unique_lock<std::mutex> g(L->mu);
      L->cv.wait(g, [&] { return L->stop || k < L->released + (uint64_t)L->depth; });
      if (L->stop) return;
    }
    const int set = (int)(k % (uint64_t)L->depth);
    hipError_t e = hipSuccess;
    if (k >= (uint64_t)L->depth) e = hipEventSynchronize(L->copy_done[set]);  // pinned set no longer being read
    uint8_t* stage = L->pinned_raw + (size_t)set * raw_bytes;
    int32_t* lab = L->pinned_labels + (size_t)set * L->batch;
    // "disk" -> host memory; the data set wraps around.  One core copies ~5 GB/s, a minibatch of 25 MB in about
    // a training step's time, so the pictures are dealt to a few helper threads.
    auto copy_slice = [&](int lo, int hi) {
      for (int i = lo; i < hi; ++i) {
        const int64_t src = (int64_t)((k * (uint64_t)L->batch + (uint64_t)i) % (uint64_t)L->count);
        memcpy(stage + (size_t)i * L->image_bytes, L->host_images + (size_t)src * L->image_bytes, L->image_bytes);
        lab[i] = L->host_labels[src];
      }
    };
    {
      const int nh = L->batch >= 4 * kCopyThreads ? kCopyThreads : 1;
      std::vector<std::thread> helpers;
      for (int h = 1; h < nh; ++h)
        helpers.emplace_back(copy_slice, (int)((long)L->batch * h / nh), (int)((long)L->batch * (h + 1) / nh));
      copy_slice(0, (int)((long)L->batch / nh));
      for (std::thread& t : helpers) t.join();
    }
    // the device buffers of this set were last read by minibatch k - depth (preprocess and training step)
    if (e == hipSuccess && k >= (uint64_t)L->depth) e = hipStreamWaitEvent(L->copy_stream, L->step_done[set], 0);
    if (e == hipSuccess)
      e = hipMemcpyAsync(L->d_raw + (size_t)set * raw_bytes, stage, raw_bytes, hipMemcpyHostToDevice, L->copy_stream);
    if (e == hipSuccess)
      e = hipMemcpyAsync(L->d_labels + (size_t)set * L->batch, lab, (size_t)L->batch * sizeof(int32_t),
                         hipMemcpyHostToDevice, L->copy_stream);
    if (e == hipSuccess) e = hipEventRecord(L->copy_done[set], L->copy_stream);
    {
      std::lock_guard<std::mutex> g(L->mu);
      if (e != hipSuccess) {
        L->worker_error = (int)e;
        L->cv.notify_all();
        return;
      }
      L->produced = k + 1;
    }
    L->cv.notify_all();
  }
}

void destroy_events(std::vector<hipEvent_t>& v) {
  for (hipEvent_t e : v)
    if (e) (void)hipEventDestroy(e);
  v.clear();
}

}  // namespace

extern "C" {

int alexnet_loader_create(alexnet_t* net, const alexnet_config_t* cfg, const uint8_t* host_images,
                          const int32_t* host_labels, int64_t count, int32_t depth, void* pinned_raw,
                          void* pinned_labels, void* d_raw, void* d_labels, void* copy_stream,
                          alexnet_loader_t** out) {
  if (!net || !cfg || !host_images || !host_labels || !pinned_raw || !pinned_labels || !d_raw || !d_labels || !out) {
    set_error("alexnet_loader_create: null argument");
    return ALEXNET_EINVAL;
  }
  if (count < 1 || depth < 2 || depth > 16) {
    set_error("alexnet_loader_create: need at least one picture and 2..16 staging sets");
    return ALEXNET_EINVAL;
  }
  alexnet_loader* L = new alexnet_loader();
  L->net = net;
  L->batch = cfg->batch;
  L->depth = depth;
  L->image_bytes = (size_t)cfg->in_c * cfg->raw_h * cfg->raw_w;
  L->host_images = host_images;
  L->host_labels = host_labels;
  L->count = count;
  L->pinned_raw = (uint8_t*)pinned_raw;
  L->pinned_labels = (int32_t*)pinned_labels;
  L->d_raw = (uint8_t*)d_raw;
  L->d_labels = (int32_t*)d_labels;
  L->produced = L->staged = L->released = 0;
  L->stop = false;
  L->worker_error = 0;
  L->copy_stream = (hipStream_t)copy_stream;
  L->own_stream = copy_stream == nullptr;
  hipError_t e = hipGetDevice(&L->device);
  if (e == hipSuccess && L->own_stream) e = hipStreamCreateWithFlags(&L->copy_stream, hipStreamNonBlocking);
  for (int i = 0; e == hipSuccess && i < depth; ++i) {
    hipEvent_t a = nullptr, b = nullptr, c = nullptr;
    e = hipEventCreateWithFlags(&a, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&b, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c, hipEventDisableTiming);
    L->copy_done.push_back(a);
    L->pre_done.push_back(b);
    L->step_done.push_back(c);
  }
  if (e != hipSuccess) {
    set_error("alexnet_loader_create: %s", hipGetErrorString(e));
    destroy_events(L->copy_done);
    destroy_events(L->pre_done);
    destroy_events(L->step_done);
    if (L->own_stream && L->copy_stream) (void)hipStreamDestroy(L->copy_stream);
    delete L;
    return ALEXNET_EHIP;
  }
  L->worker = std::thread(loader_thread, L);
  *out = L;
  return ALEXNET_OK;
}

int alexnet_loader_stage(alexnet_loader_t* L, uint64_t k, const float* d_mean, void* side_stream,
                         void* compute_stream, const int32_t** d_labels_k) {
  if (!L || !d_mean || !d_labels_k) {
    set_error("alexnet_loader_stage: null argument");
    return ALEXNET_EINVAL;
  }
  {
    std::unique_lock<std::mutex> g(L->mu);
    if (k != L->staged || k >= L->released + 2) {
      // out of order, or the step that read input slot k % 2 last (minibatch k - 2) has not been enqueued yet
      set_error("alexnet_loader_stage: minibatch %llu is not the next one, or more than two ahead of "
                "alexnet_loader_done", (unsigned long long)k);
      return ALEXNET_EINVAL;
    }
    L->cv.wait(g, [&] { return L->worker_error != 0 || L->produced > k; });
    if (L->worker_error) {
      set_error("alexnet_loader: the loading thread failed (HIP error %d)", L->worker_error);
      return ALEXNET_EHIP;
    }
    L->staged = k + 1;
  }
  const int set = (int)(k % (uint64_t)L->depth);
  hipStream_t side = (hipStream_t)side_stream, comp = (hipStream_t)compute_stream;
  AX_HIP(hipStreamWaitEvent(side, L->copy_done[set], 0));
  // input slot k % 2 was last read by the step of minibatch k - 2 (with two staging sets the copy waited
  // for it already; with more it did not)
  if (k >= 2) AX_HIP(hipStreamWaitEvent(side, L->step_done[(int)((k - 2) % (uint64_t)L->depth)], 0));
  const size_t raw_bytes = (size_t)L->batch * L->image_bytes;
  AX_TRY(alexnet_preprocess(L->net, L->d_raw + (size_t)set * raw_bytes, d_mean, k, (int32_t)(k & 1), side_stream));
  AX_HIP(hipEventRecord(L->pre_done[set], side));
  AX_HIP(hipStreamWaitEvent(comp, L->pre_done[set], 0));
  *d_labels_k = L->d_labels + (size_t)set * L->batch;
  return ALEXNET_OK;
}

int alexnet_loader_done(alexnet_loader_t* L, uint64_t k, void* compute_stream) {
  if (!L) {
    set_error("alexnet_loader_done: null handle");
    return ALEXNET_EINVAL;
  }
  {
    std::lock_guard<std::mutex> g(L->mu);
    if (k != L->released || k >= L->staged) {
      set_error("alexnet_loader_done: minibatch %llu has not been staged, or an earlier one is still open",
                (unsigned long long)k);
      return ALEXNET_EINVAL;
    }
  }
  const int set = (int)(k % (uint64_t)L->depth);
  AX_HIP(hipEventRecord(L->step_done[set], (hipStream_t)compute_stream));
  {
    std::lock_guard<std::mutex> g(L->mu);
    L->released = k + 1;
  }
  L->cv.notify_all();
  return ALEXNET_OK;
}

int alexnet_loader_destroy(alexnet_loader_t* L) {
  if (!L) return ALEXNET_OK;
  {
    std::lock_guard<std::mutex> g(L->mu);
    L->stop = true;
  }
  L->cv.notify_all();
  if (L->worker.joinable()) L->worker.join();
  (void)hipStreamSynchronize(L->copy_stream);  // copies still in flight read the caller's pinned memory
  destroy_events(L->copy_done);
  destroy_events(L->pre_done);
  destroy_events(L->step_done);
  if (L->own_stream) (void)hipStreamDestroy(L->copy_stream);
  delete L;
  return ALEXNET_OK;
}

}  // extern "C"
