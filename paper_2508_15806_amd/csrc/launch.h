// Kernel launch that carries a pair of timing events while the profile recorder is on.
#ifndef SLKV_LAUNCH_H
#define SLKV_LAUNCH_H

#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include "slkv_internal.h"

namespace slkv {

template <class K, class... A>
inline void launch_k(K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st, A... args) {
  void *e0 = nullptr, *e1 = nullptr;
  if (profile_events(&e0, &e1))
    hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, st, (hipEvent_t)e0, (hipEvent_t)e1, 0u, args...);
  else
    hipLaunchKernelGGL(kernel, grid, block, lds, st, args...);
}

}  // namespace slkv

#define SLKV_LAUNCH(kernel, grid, block, lds, st, ...) ::slkv::launch_k(kernel, grid, block, lds, st, __VA_ARGS__)

#endif
