// Dispatch from a run-time tile plan to the compiled instantiations of the
// convolution kernel.  Each filter-block count WK is compiled in its own
// translation unit (conv_inst.hip with -DINST_WK=<n>) so the build runs in parallel.
#pragma once
#include <hip/hip_runtime.h>
#include "conv_kernel.h"

namespace abed {

// compiled tile shapes: WM (batch entries per wave), WK (filter blocks per tile)
static const int kWmList[] = {1, 2, 3, 5, 9};
static const int kWkList[] = {1, 4, 5, 8, 9};
#ifndef ABED_STAGES
#define ABED_STAGES 3
#endif
#ifndef ABED_LDS_BUDGET
#define ABED_LDS_BUDGET (128 * 1024)
#endif
// LDS stages of the load pipeline for a tile shape: as many as asked for, within a per-workgroup LDS
// budget and within the 6-bit vector-memory counter the hand-counted waits rely on.
constexpr int stages_for(int wm, int wk)
{
    const int nb = wk + 4 * wm, l = (nb + 3) / 4;
    int n = ABED_STAGES;
    while (n > 2 && (n * nb * 1024 > ABED_LDS_BUDGET || (n - 1) * l > 63)) --n;
    return n;
}

// Returns false if (wm, wk) is not a compiled configuration.
bool launch_conv(bool f16, int wm, int wk, const ConvParams &p, int grid, hipStream_t st);

bool launch_conv_wk1(bool f16, int wm, const ConvParams &p, int grid, hipStream_t st);
bool launch_conv_wk4(bool f16, int wm, const ConvParams &p, int grid, hipStream_t st);
bool launch_conv_wk5(bool f16, int wm, const ConvParams &p, int grid, hipStream_t st);
bool launch_conv_wk8(bool f16, int wm, const ConvParams &p, int grid, hipStream_t st);
bool launch_conv_wk9(bool f16, int wm, const ConvParams &p, int grid, hipStream_t st);

}  // namespace abed
