// One translation unit per chunk count of the batch checksum, set with -DBOX_XCH=<0|1|2|4|8>.
#include "conv_box_launch.h"

#ifndef BOX_XCH
#error "compile with -DBOX_XCH=<chunks of the batch checksum, 0 = none>"
#endif
#define CAT2_(a, b) a##b
#define CAT2(a, b) CAT2_(a, b)

namespace abed {

bool CAT2(launch_box_x, BOX_XCH)(int fb, bool fc, int eh, const BoxParams &p, int grid, hipStream_t st)
{
    if (eh == 2) {
        if (fc && fb == 5) { box_conv_kernel<5, true, BOX_XCH, 3><<<dim3(grid), dim3(512), 0, st>>>(p); return true; }
        if (!fc && fb == 4) { box_conv_kernel<4, false, BOX_XCH, 3><<<dim3(grid), dim3(512), 0, st>>>(p); return true; }
#if BOX_XCH == 0
        if (!fc && fb == 8) { box_conv_kernel<8, false, 0, 2><<<dim3(grid), dim3(512), 0, st>>>(p); return true; }
        if (fc && fb == 9) { box_conv_kernel<9, true, 0, 2><<<dim3(grid), dim3(512), 0, st>>>(p); return true; }
#endif
    }
#if BOX_XCH <= 2
    if (eh == 1) {
        // four waves and at most 80 KB of LDS: two workgroups per CU
        if (fc && fb == 5) { box_conv_kernel<5, true, BOX_XCH, 2, 1><<<dim3(grid), dim3(256), 0, st>>>(p); return true; }
        if (!fc && fb == 4) { box_conv_kernel<4, false, BOX_XCH, 2, 1><<<dim3(grid), dim3(256), 0, st>>>(p); return true; }
    }
#endif
    return false;
}

#if BOX_XCH == 0
bool launch_box(int fb, bool fc, int xch, int eh, const BoxParams &p, int grid, hipStream_t st)
{
    switch (xch) {
    case 0: return launch_box_x0(fb, fc, eh, p, grid, st);
    case 1: return launch_box_x1(fb, fc, eh, p, grid, st);
    case 2: return launch_box_x2(fb, fc, eh, p, grid, st);
    case 4: return launch_box_x4(fb, fc, eh, p, grid, st);
    case 8: return launch_box_x8(fb, fc, eh, p, grid, st);
    }
    return false;
}
#endif

}  // namespace abed
