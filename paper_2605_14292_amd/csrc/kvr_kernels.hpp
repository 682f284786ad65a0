// Launch interface between the host entry points and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvr {

struct Layout {
  int heads, n, d, dtype;
  long long stride_head, stride_tok;
};

hipError_t launch_score(const void* K, const void* Q, int G, const Layout& lay,
                        float* s_out, hipStream_t st);
hipError_t launch_select_generic(const void* V, const float* s, const Layout& lay, int b,
                                 float lambda, float eps, int32_t* idx_sorted,
                                 int32_t* pick_order, float* pick_gain, hipStream_t st);
hipError_t launch_compact(const void* K, const void* V, const Layout& lay, const int32_t* idx,
                          int b, void* K_out, void* V_out, hipStream_t st);

}  // namespace kvr
