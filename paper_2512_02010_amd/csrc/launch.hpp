// Host side: one kernel launch whose status is this launch's own.
#pragma once

#include <hip/hip_runtime.h>

#include <tuple>

#include "nvfp4_46.h"

namespace nvfp4_46 {

// Launches through hipLaunchKernel, whose return value belongs to this launch (the
// runtime's "last error" also holds whatever another library left there, and reading it
// clears it).  The arguments are converted to the kernel's parameter types first.
template <typename... Params, typename... Args>
static int launch(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds_bytes,
                  hipStream_t stream, Args... args) {
  static_assert(sizeof...(Params) == sizeof...(Args), "one argument per kernel parameter");
  std::tuple<Params...> vals{static_cast<Params>(args)...};
  void *ptrs[sizeof...(Params)];
  std::apply([&](auto &...v) { int i = 0; ((ptrs[i++] = static_cast<void *>(&v)), ...); }, vals);
  return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, lds_bytes,
                         stream) == hipSuccess
             ? NVFP4_OK
             : NVFP4_ERR_HIP;
}

}  // namespace nvfp4_46
