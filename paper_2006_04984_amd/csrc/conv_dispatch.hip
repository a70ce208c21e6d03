#include "conv_launch.h"

namespace abed {

bool launch_conv(bool f16, int wm, int wk, int kg, const ConvParams &p, int grid, hipStream_t st, unsigned dyn_lds)
{
#define ABED_CASE(WK, KG) if (wk == WK && kg == KG) return launch_conv_wk##WK##_kg##KG(f16, wm, p, grid, st, dyn_lds);
    ABED_FOR_ALL_WK_KG(ABED_CASE)
    return false;
}

}  // namespace abed
