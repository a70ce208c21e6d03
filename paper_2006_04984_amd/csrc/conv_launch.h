// Dispatch from a run-time tile plan to the compiled instantiations of the
// convolution kernel.  Each filter-block count is compiled in its own
// translation unit (conv_inst.hip with -DINST_WK=<n>) so the build runs in parallel.
#pragma once
#include <hip/hip_runtime.h>
#include "conv_kernel.h"

namespace abed {

// Returns false if (wm, wk, aug) is not a compiled configuration.
bool launch_conv_i8(int wm, int wk, bool aug, const ConvParams &p, int grid, hipStream_t st);

bool launch_conv_i8_wk1(int wm, bool aug, const ConvParams &p, int grid, hipStream_t st);
bool launch_conv_i8_wk4(int wm, bool aug, const ConvParams &p, int grid, hipStream_t st);
bool launch_conv_i8_wk8(int wm, bool aug, const ConvParams &p, int grid, hipStream_t st);
bool launch_conv_i8_wk16(int wm, bool aug, const ConvParams &p, int grid, hipStream_t st);

}  // namespace abed
