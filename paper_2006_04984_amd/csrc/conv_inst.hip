// One translation unit per filter-block count WK (set with -DINST_WK=<n>).
#include "conv_launch.h"

#ifndef INST_WK
#error "compile with -DINST_WK=<filter blocks per tile>"
#endif

#define CAT_(a, b) a##b
#define CAT(a, b) CAT_(a, b)

namespace abed {

template <int WM>
static void go(bool f16, const ConvParams &p, int grid, hipStream_t st)
{
    if (f16) conv_kernel<true, WM, INST_WK, stages_for(WM, INST_WK)><<<dim3(grid), dim3(256), 0, st>>>(p);
    else conv_kernel<false, WM, INST_WK, stages_for(WM, INST_WK)><<<dim3(grid), dim3(256), 0, st>>>(p);
}

bool CAT(launch_conv_wk, INST_WK)(bool f16, int wm, const ConvParams &p, int grid, hipStream_t st)
{
    switch (wm) {
    case 1: go<1>(f16, p, grid, st); return true;
    case 2: go<2>(f16, p, grid, st); return true;
    case 3: go<3>(f16, p, grid, st); return true;
    case 5: go<5>(f16, p, grid, st); return true;
    case 9: go<9>(f16, p, grid, st); return true;
    }
    return false;
}

}  // namespace abed
