// Host-side helpers shared by the kernel launchers.
#include <hip/hip_runtime.h>

#include <mutex>
#include <set>
#include <utility>

#include "kernels.h"

namespace otas {

// Kernels that use more than 64 KB of dynamic LDS need hipFuncAttributeMaxDynamicSharedMemorySize set
// before their first launch, on every device they run on.  Done once per (kernel, device); safe to
// call from several host threads.
hipError_t set_max_dynamic_lds(const void* kernel, int bytes) {
  static std::mutex mu;
  static std::set<std::pair<const void*, int>> done;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> lock(mu);
  const std::pair<const void*, int> key(kernel, dev);
  if (done.count(key)) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done.insert(key);
  return e;
}

}  // namespace otas
