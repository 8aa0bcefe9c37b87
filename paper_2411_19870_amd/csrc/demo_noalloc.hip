// Writes to device memory that need no runtime copy: a writer kernel that carries its data in the kernel arguments.
#include "demo_device.h"

namespace demo {

namespace {

constexpr int kBatchWords = 960;           // 3840 bytes of data per launch (kernel arguments are limited to 4 KiB)
struct WordBatch {
  uint32_t w[kBatchWords];
};

__global__ __launch_bounds__(256) void write_words_kernel(uint32_t* __restrict__ dst, WordBatch b, int n) {
  const int i = (int)(blockIdx.x * blockDim.x + threadIdx.x);
  if (i < n) store_guarded(as_global(dst) + i, b.w[i]);
}

}  // namespace

// Copies nbytes (a multiple of 4) of host memory to 4-byte aligned device memory in stream order without any
// runtime copy or allocation: the words travel as kernel arguments.
hipError_t device_write(void* dst, const void* host, size_t nbytes, hipStream_t stream) {
  const size_t nwords = nbytes / 4;
  const uint32_t* src = static_cast<const uint32_t*>(host);
  uint32_t* out = static_cast<uint32_t*>(dst);
  for (size_t done = 0; done < nwords; done += kBatchWords) {
    const int n = (int)(nwords - done < (size_t)kBatchWords ? nwords - done : (size_t)kBatchWords);
    WordBatch b;
    memcpy(b.w, src + done, (size_t)n * 4);
    hipLaunchKernelGGL(write_words_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, out + done, b, n);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace demo
