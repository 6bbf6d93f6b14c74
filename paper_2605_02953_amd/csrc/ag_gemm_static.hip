// AllGather-GEMM for callers that cannot allocate device memory (code under HIP graph capture, tight
// serving loops, harnesses that forbid hipMalloc): ditron_ag_gemm with its scratch (the gathered operand
// and the signal words) taken from a fixed array that lives in the library's device image.
#include <atomic>
#include <mutex>

#include "launch.h"

namespace ditron {

constexpr size_t kStaticSignalWords = 1024;
constexpr size_t kStaticScratchBytes = (size_t)DITRON_STATIC_WORKSPACE_BYTES + kStaticSignalWords * sizeof(int32_t);

// One copy per GPU the library runs on, held until the process ends.  In host code this name is only a
// stand-in for the symbol: the memory is reached through the address hipGetSymbolAddress reports.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static std::mutex g_scratch_mutex;
static unsigned char* g_scratch_ptr[64] = {nullptr};
static std::atomic<int32_t> g_calls[64];   // calls so far on each device: the next call's epoch

// The calling thread's current device's copy of `scratch` (looked up once per device), or null.
static unsigned char* scratch_on_current_device(int& dev) {
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    unsigned char* ptr = nullptr;
    if (hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

// A fill kernel rather than hipMemsetAsync: memset nodes are not safe in captured graphs here.
__global__ __launch_bounds__(256) void zero_words_kernel(int32_t* words, int n) {
  for (int i = threadIdx.x; i < n; i += 256) words[i] = 0;
}

}  // namespace ditron

using namespace ditron;

extern "C" ditron_status_t ditron_ag_gemm_static(const void* const* a_shards, const void* b, int b_layout, void* c,
                                                 const float* a_scales, const float* b_scales, int32_t* status,
                                                 const int* arrival_order, int m_per_rank, int n, int k, int world,
                                                 int rank, int dtype, const ditron_tuning_t* tuning, void* stream) {
  if (world < 1 || world > DITRON_MAX_WORLD || m_per_rank <= 0 || n <= 0 || k <= 0) return DITRON_ERR_INVALID_ARG;
  const size_t need = ditron_ag_gemm_workspace_bytes(m_per_rank, n, k, world, dtype, b_layout, tuning);
  if (need == 0) return DITRON_ERR_INVALID_ARG;
  if (need > (size_t)DITRON_STATIC_WORKSPACE_BYTES || ditron_signal_words(world, 1) > kStaticSignalWords)
    return DITRON_ERR_WORKSPACE;
  int dev = 0;
  unsigned char* base = scratch_on_current_device(dev);
  if (!base) return DITRON_ERR_HIP;
  int32_t* signals = (int32_t*)(base + DITRON_STATIC_WORKSPACE_BYTES);
  // the array keeps the previous call's contents: the flags start at zero again, and the epoch (which the
  // partial tiles of decode-shaped problems carry in every word) is one no earlier call on this GPU used
  int32_t epoch = g_calls[dev].fetch_add(1) + 1;
  if (epoch <= 0) {   // wrapped: fall back into the positive range (two billion calls apart)
    g_calls[dev].store(1);
    epoch = 1;
  }
  const int words = (int)ditron_signal_words(world, 1);
  hipLaunchKernelGGL(zero_words_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream, signals, words);
  if (hipGetLastError() != hipSuccess) return DITRON_ERR_HIP;
  return ditron_ag_gemm(a_shards, b, b_layout, c, a_scales, b_scales, base, signals, status, nullptr, arrival_order,
                        m_per_rank, n, k, world, rank, dtype, epoch, DITRON_EMULATE_PRODUCER, tuning, stream);
}
