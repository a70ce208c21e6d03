// One translation unit per filter-block count WK (set with -DINST_WK=1|4|8|16).
#include "conv_launch.h"

#ifndef INST_WK
#error "compile with -DINST_WK=<filter blocks per tile>"
#endif

#define CAT_(a, b) a##b
#define CAT(a, b) CAT_(a, b)

namespace abed {

template <int WM, bool AUG>
static void go(const ConvParams &p, int grid, hipStream_t st)
{
    conv_i8_kernel<WM, INST_WK, AUG><<<dim3(grid), dim3(256), 0, st>>>(p);
}

bool CAT(launch_conv_i8_wk, INST_WK)(int wm, bool aug, const ConvParams &p, int grid, hipStream_t st)
{
#if INST_WK >= 4
    if (aug) {
        switch (wm) {
        case 1: go<1, true>(p, grid, st); return true;
        case 2: go<2, true>(p, grid, st); return true;
        case 4: go<4, true>(p, grid, st); return true;
        }
        return false;
    }
#else
    if (aug) return false;
#endif
    switch (wm) {
    case 1: go<1, false>(p, grid, st); return true;
    case 2: go<2, false>(p, grid, st); return true;
    case 4: go<4, false>(p, grid, st); return true;
    }
    return false;
}

}  // namespace abed
