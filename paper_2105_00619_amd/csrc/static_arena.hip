// The activation arena of optorch_seq_step_static: a file-scope device array that exists once per GPU for the life of
// the process, so that the call never has to allocate.  The array's name is only a host-side handle of the symbol;
// its device address differs per GPU and is looked up once per device (with that device current) and kept.
#include <hip/hip_runtime.h>

#include <mutex>

#include "kernels.h"
#include "optorch_seq.h"

static __device__ __align__(256) unsigned char scratch[OPTORCH_STATIC_ARENA_BYTES];

namespace oseq {

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_ptr[kMaxDevices] = {nullptr};
}  // namespace

// Device address of the static arena on the current device, or an error.  Allocates nothing.
hipError_t static_arena(void** ptr, uint64_t* bytes) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p || (reinterpret_cast<uintptr_t>(p) & 255)) return hipErrorInvalidSymbol;
    g_ptr[dev] = p;
  }
  *ptr = g_ptr[dev];
  *bytes = OPTORCH_STATIC_ARENA_BYTES;
  return hipSuccess;
}

}  // namespace oseq
