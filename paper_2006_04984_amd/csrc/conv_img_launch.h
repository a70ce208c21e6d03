// Dispatch to the compiled instantiations of the one-wave-per-SIMD convolution kernel (conv_img_kernel.h).
#pragma once
#include <hip/hip_runtime.h>

namespace abed {

struct ImgParams;
// iw: images a wave holds at once (1: regions of up to 128 positions, 2: of up to 64).  Returns false if not compiled.
bool launch_img(int iw, const ImgParams &p, int grid, hipStream_t st);
inline bool img_compiled(int iw) { return iw == 1 || iw == 2; }

}  // namespace abed
