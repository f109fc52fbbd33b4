// The library's own workspace for callers that cannot allocate device memory (code under HIP graph capture,
// tight serving loops, harnesses that forbid allocation): one file-scope device array per GPU, which holds
// everything oz2_dgemm_static keeps between its kernels (shift vectors, flag words, residue planes, product
// planes) in the same layout as a caller-owned workspace.
//
// In host code the array's name is only a handle of the symbol, not a device address: the address on a device
// comes from hipGetSymbolAddress, looked up once per device with that device current, and that pointer is
// what every kernel argument is built from.  Each GPU holds its own copy of the array until the process ends.
// Calls that use it share it: calls that overlap in time on one GPU race.
#include <mutex>

#include "oz2_internal.h"

namespace {

static __device__ __align__(256) unsigned char scratch[OZ2_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
char* g_ptr[kMaxDevices] = {};

}  // namespace

hipError_t oz2_static_scratch(char** ptr, size_t* bytes) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mu);
  if (g_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr || (reinterpret_cast<uintptr_t>(p) & 255u)) return hipErrorInvalidSymbol;
    g_ptr[dev] = static_cast<char*>(p);
  }
  *ptr = g_ptr[dev];
  *bytes = OZ2_STATIC_SCRATCH_BYTES;
  return hipSuccess;
}
