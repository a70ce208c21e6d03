#include "conv_launch.h"

namespace abed {

bool launch_conv_i8(int wm, int wk, const ConvParams &p, int grid, hipStream_t st)
{
    switch (wk) {
    case 1: return launch_conv_i8_wk1(wm, p, grid, st);
    case 4: return launch_conv_i8_wk4(wm, p, grid, st);
    case 5: return launch_conv_i8_wk5(wm, p, grid, st);
    case 8: return launch_conv_i8_wk8(wm, p, grid, st);
    case 9: return launch_conv_i8_wk9(wm, p, grid, st);
    }
    return false;
}

}  // namespace abed
