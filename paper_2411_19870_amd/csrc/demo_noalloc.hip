// Device memory that needs no allocation: a writer kernel that carries its data in the kernel arguments, and the
// static scratch array behind demo_encode_noalloc (basis tables, descriptor tables and the fallback queue of one
// call at a time, per GPU).
#include "demo_device.h"

namespace demo {

namespace {

// Each GPU the library runs on holds its own copy of this array, at its own address, until the process ends.
static __device__ __align__(256) unsigned char scratch[kNoallocScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};     // device address of `scratch` on each GPU (hipGetSymbolAddress)
int g_basis_resident[kMaxDevices] = {};    // chunk size whose basis tables lie in the scratch of each GPU, 0 = none

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

// Address of the static scratch array on the current device (looked up once per device).
hipError_t noalloc_scratch(int device, void** ptr) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  if (g_scratch_ptr[device] == nullptr) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[device] = p;
  }
  *ptr = g_scratch_ptr[device];
  return hipSuccess;
}

int noalloc_basis_resident(int device) { return device >= 0 && device < kMaxDevices ? g_basis_resident[device] : 0; }
void noalloc_set_basis_resident(int device, int s) {
  if (device >= 0 && device < kMaxDevices) g_basis_resident[device] = s;
}

}  // namespace demo
