// One translation unit per (filter-block count WK, reduction-axis group count KG), set with
// -DINST_WK=<n> -DINST_KG=<n>, so the build runs in parallel.
#include "conv_launch.h"

#if !defined(INST_WK) || !defined(INST_KG)
#error "compile with -DINST_WK=<filter blocks per tile> -DINST_KG=<wave groups>"
#endif

#define CAT4_(a, b, c, d) a##b##c##d
#define CAT4(a, b, c, d) CAT4_(a, b, c, d)

namespace abed {

template <int WM>
static bool go(bool f16, const ConvParams &p, int grid, hipStream_t st, unsigned dyn_lds)
{
    if constexpr (tile_ok(WM, INST_WK, INST_KG)) {
        constexpr int NST = stages_for(WM, INST_WK, INST_KG);
        if (f16) conv_kernel<true, WM, INST_WK, NST, INST_KG><<<dim3(grid), dim3(256 * INST_KG), dyn_lds, st>>>(p);
        else if (p.fic_wdig) conv_kernel<false, WM, INST_WK, NST, INST_KG, true><<<dim3(grid), dim3(256 * INST_KG), dyn_lds, st>>>(p);
        else conv_kernel<false, WM, INST_WK, NST, INST_KG><<<dim3(grid), dim3(256 * INST_KG), dyn_lds, st>>>(p);
        return true;
    } else {
        return false;
    }
}

bool CAT4(launch_conv_wk, INST_WK, _kg, INST_KG)(bool f16, int wm, const ConvParams &p, int grid, hipStream_t st, unsigned dyn_lds)
{
    switch (wm) {
    case 1: return go<1>(f16, p, grid, st, dyn_lds);
    case 2: return go<2>(f16, p, grid, st, dyn_lds);
    case 3: return go<3>(f16, p, grid, st, dyn_lds);
    case 5: return go<5>(f16, p, grid, st, dyn_lds);
    case 9: return go<9>(f16, p, grid, st, dyn_lds);
    }
    return false;
}

}  // namespace abed
