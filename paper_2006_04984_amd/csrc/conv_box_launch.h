// Dispatch from a run-time plan to the compiled instantiations of the box convolution kernel
// (conv_box_kernel.h).  One translation unit per chunk count of the batch checksum
// (conv_box_inst.hip with -DBOX_XCH=<n>), so the build runs in parallel.
#pragma once
#include <hip/hip_runtime.h>
#include "conv_box_kernel.h"

namespace abed {

// fb: filter blocks per tile incl. the digit block (4, 5, 8, 9); fc: digit block present; xch: 0 or C/64
// (1, 2, 4, 8) when the batch checksum runs; eh: 2 = workgroups of 8 waves and batches of 8 entries, 1 = of 4 waves
// and 4 entries (two per CU).  Returns false if the combination is not compiled.
bool launch_box(int fb, bool fc, int xch, int eh, const BoxParams &p, int grid, hipStream_t st);
inline bool box_compiled(int fb, bool fc, int xch, int eh)
{
    if (!(xch == 0 || xch == 1 || xch == 2 || xch == 4 || xch == 8)) return false;
    if (eh == 1) return xch <= 2 && (fc ? fb == 5 : fb == 4);
    if (eh != 2) return false;
    if (fc) return fb == 5 || (fb == 9 && xch == 0);
    return fb == 4 || (fb == 8 && xch == 0);
}

#define ABED_DECL_BOX(X) bool launch_box_x##X(int fb, bool fc, int eh, const BoxParams &p, int grid, hipStream_t st);
ABED_DECL_BOX(0) ABED_DECL_BOX(1) ABED_DECL_BOX(2) ABED_DECL_BOX(4) ABED_DECL_BOX(8)

}  // namespace abed
