#include "conv_launch.h"

namespace abed {

bool launch_conv_i8(int wm, int wk, bool aug, const ConvParams &p, int grid, hipStream_t st)
{
    switch (wk) {
    case 1: return launch_conv_i8_wk1(wm, aug, p, grid, st);
    case 4: return launch_conv_i8_wk4(wm, aug, p, grid, st);
    case 8: return launch_conv_i8_wk8(wm, aug, p, grid, st);
    case 16: return launch_conv_i8_wk16(wm, aug, p, grid, st);
    }
    return false;
}

}  // namespace abed
