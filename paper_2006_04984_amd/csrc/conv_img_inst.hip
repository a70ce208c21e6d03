// The instantiations of the one-wave-per-SIMD convolution kernel, in a translation unit of their own (parallel build).
#include "conv_img_kernel.h"
#include "conv_img_launch.h"

namespace abed {

bool launch_img(int iw, const ImgParams &p, int grid, hipStream_t st)
{
    const bool out8 = p.scale != nullptr;
    if (iw == 1 && !out8) { img_conv_kernel<1, false><<<dim3(grid), dim3(256), 0, st>>>(p); return true; }
    if (iw == 2 && !out8) { img_conv_kernel<2, false><<<dim3(grid), dim3(256), 0, st>>>(p); return true; }
    if (iw == 1 && out8) { img_conv_kernel<1, true><<<dim3(grid), dim3(256), 0, st>>>(p); return true; }
    if (iw == 2 && out8) { img_conv_kernel<2, true><<<dim3(grid), dim3(256), 0, st>>>(p); return true; }
    return false;
}

}  // namespace abed
