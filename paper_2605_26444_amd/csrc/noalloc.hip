// nanospec_dense_topk_static: the full-vocabulary selection for callers that cannot allocate device memory
// (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same kernels as
// nanospec_dense_topk; the per-chunk candidates go to a fixed device array of this library instead of a
// caller-supplied workspace.
#include <mutex>

#include "common.h"

using namespace nanospec;

namespace {

constexpr int64_t kScratchBytes = 4ll << 20;              // 4 MiB per GPU, held until the process ends
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices] = {};                    // device address of `scratch` on each GPU, looked up once

// The array's name is only a host-side handle; the address the kernels need comes from the runtime, per device.
void* scratch_on_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

}  // namespace

extern "C" {

int64_t nanospec_dense_topk_static_limit(void) { return kScratchBytes; }

nanospec_status nanospec_dense_topk_static(const float* d_logits, int32_t V, int32_t M_total, int32_t k,
                                           int32_t* d_out_ids, float* d_out_vals, void* hip_stream) {
  if (!d_logits || !d_out_ids || V < 1 || M_total < 1 || k < 1 || k > kMaxK) return NANOSPEC_EINVAL;
  if ((int64_t)V > (int64_t)kTopkChunk * 16) return NANOSPEC_EINVAL;
  const int64_t need = topk_workspace_bytes(V, M_total, k);
  if (need > kScratchBytes) return NANOSPEC_ECAPACITY;
  void* ws = scratch_on_current_device();
  if (!ws) return NANOSPEC_EHIP;
  // every candidate slot the merge kernel reads is written by the selection kernel of the same call, so
  // nothing in the array has to be cleared between calls
  hipError_t e = launch_topk(d_logits, V, nullptr, 0, nullptr, V, V, 1, M_total, k, d_out_ids, d_out_vals, false,
                             static_cast<char*>(ws), kScratchBytes, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? NANOSPEC_OK : NANOSPEC_EHIP;
}

}  // extern "C"
