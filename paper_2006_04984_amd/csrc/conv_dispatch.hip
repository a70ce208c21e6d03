#include "conv_launch.h"

namespace abed {

bool launch_conv(bool f16, int wm, int wk, const ConvParams &p, int grid, hipStream_t st)
{
    switch (wk) {
    case 1: return launch_conv_wk1(f16, wm, p, grid, st);
    case 4: return launch_conv_wk4(f16, wm, p, grid, st);
    case 5: return launch_conv_wk5(f16, wm, p, grid, st);
    case 8: return launch_conv_wk8(f16, wm, p, grid, st);
    case 9: return launch_conv_wk9(f16, wm, p, grid, st);
    }
    return false;
}

}  // namespace abed
