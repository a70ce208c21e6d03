// Dispatch from a run-time tile plan to the compiled instantiations of the
// convolution kernel.  Each filter-block count WK is compiled in its own
// translation unit (conv_inst.hip with -DINST_WK=<n>) so the build runs in parallel.
#pragma once
#include <hip/hip_runtime.h>
#include "conv_kernel.h"

namespace abed {

// compiled tile shapes: WM (batch entries per wave), WK (filter blocks per tile), KG (groups of
// 4 waves along the reduction axis)
static const int kWmList[] = {1, 2, 3, 5, 9};
static const int kWkList[] = {1, 4, 5, 8, 9};
static const int kKgList[] = {1, 2, 4};
#ifndef ABED_STAGES
#define ABED_STAGES 3
#endif
#ifndef ABED_LDS_BUDGET
#define ABED_LDS_BUDGET (128 * 1024)
#endif
// LDS stages of the load pipeline for a tile shape: as many as asked for, within a per-workgroup LDS
// budget and within the 6-bit vector-memory counter the hand-counted waits rely on.
constexpr int stages_for(int wm, int wk, int kg)
{
    const int nb = wk + 4 * wm, l = (nb + 3) / 4;
    int n = ABED_STAGES;
    while (n > 2 && (n * kg * nb * 1024 > ABED_LDS_BUDGET || (n - 1) * l > 63)) --n;
    return n;
}
// Whether (wm, wk, kg) is compiled: the accumulators, the operand fragments and the loader state must
// fit the registers a wave gets when 4*kg waves share a CU's SIMDs (512 / kg), and two pipeline stages
// and the group-sum buffer must fit LDS.
constexpr bool tile_ok(int wm, int wk, int kg)
{
    const int regs = 4 * wm * wk + 4 * wm + 4 + 72;
    const int nb = wk + 4 * wm;
    if (kg == 4 && wm * wk > 8) return false;   // 128 registers per wave
    return regs <= 512 / kg && 2 * kg * nb * 1024 <= 160 * 1024 - 1024 && (kg - 1) * 4 * wm * wk * 1024 <= 160 * 1024 - 1024;
}

// Whether launch_conv has an instantiation for (wm, wk, kg)
inline bool tile_compiled(int wm, int wk, int kg)
{
    bool a = false, b = false, c = false;
    for (int v : kWmList) a |= v == wm;
    for (int v : kWkList) b |= v == wk;
    for (int v : kKgList) c |= v == kg;
    return a && b && c && tile_ok(wm, wk, kg);
}

// Returns false if (wm, wk, kg) is not a compiled configuration.  dyn_lds: bytes of dynamic LDS behind the
// kernel's own (the digits of the FIC scheme's in-loop input side), else 0.
bool launch_conv(bool f16, int wm, int wk, int kg, const ConvParams &p, int grid, hipStream_t st, unsigned dyn_lds = 0);

#define ABED_DECL_LAUNCH(WK, KG) bool launch_conv_wk##WK##_kg##KG(bool f16, int wm, const ConvParams &p, int grid, hipStream_t st, unsigned dyn_lds);
#define ABED_FOR_ALL_WK_KG(X) \
    X(1, 1) X(4, 1) X(5, 1) X(8, 1) X(9, 1) X(1, 2) X(4, 2) X(5, 2) X(8, 2) X(9, 2) X(1, 4) X(4, 4) X(5, 4) X(8, 4) X(9, 4)
ABED_FOR_ALL_WK_KG(ABED_DECL_LAUNCH)

}  // namespace abed
