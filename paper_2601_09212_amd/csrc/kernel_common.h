// What every translation unit of the kernel library shares: resampling-law modes, the workgroup
// shapes of the per-sequence kernels, LDS layouts, and the checked launch helper.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include <tuple>
#include <utility>

#include "device_utils.h"
#include "kernels.h"

namespace csd {

enum { kModeOpt = 0, kModeVanilla = 1, kModeP = 2 };
constexpr int kThreadsW = 1024;    // workgroup size of the per-row / per-sequence kernels
constexpr int kWavesW = kThreadsW / 64;

struct Smem {
  float tile_part[kWaves][16];
  float tile_tot[16];
  float scan_tot[kWaves];
  int pick_first[kWaves];
  int pick_last[kWaves];
  int bcast_i;
  int trust;            // chunk_select: the fp32 draw stands
  float4 rowstat;
};

__device__ __forceinline__ const char* row_ptr(const void* base, int64_t elem_off, int es) {
  return base ? reinterpret_cast<const char*>(base) + elem_off * es : nullptr;
}

// Launch through hipLaunchKernel, which returns the launch status itself: the per-thread "last
// error" of the HIP runtime is neither read nor cleared, so an error the host program has pending
// from its own earlier calls stays where it is.  Arguments are converted to the kernel's exact
// parameter types first.
template <typename... KA, typename... A>
inline hipError_t launch(const char* what, void (*kernel)(KA...), dim3 grid, dim3 block, hipStream_t stream,
                         const A&... args) {
  static_assert(sizeof...(KA) == sizeof...(A), "argument count");
  std::tuple<std::decay_t<KA>...> copy(args...);
  hipError_t e = std::apply(
      [&](auto&... c) {
        void* argv[] = {static_cast<void*>(&c)...};
        return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, argv, 0, stream);
      },
      copy);
  if (e != hipSuccess) fprintf(stderr, "cool_sd: launch of %s failed: %s\n", what, hipGetErrorString(e));
  return e;
}

}  // namespace csd
