// Instances of the register/LDS recurrence kernel for 65-128 layers (5-8 waves per workgroup
// along the first-layer axis), in a translation unit of their own so that the two halves
// compile side by side.
#include "fast_kernel.hpp"

namespace alpa {

hipError_t launch_recurrence_fast_deep(hipStream_t st, const FastArgs &a, int mode, int nc, int grid)
{
    switch ((a.p.K + 15) / 16) {
    case 5: return launch_nwk<5>(st, a, mode, nc, grid);
    case 6: return launch_nwk<6>(st, a, mode, nc, grid);
    case 7: return launch_nwk<7>(st, a, mode, nc, grid);
    case 8: return launch_nwk<8>(st, a, mode, nc, grid);
    default: return hipErrorInvalidValue;
    }
}

int fast_kernel_blocks_per_cu_deep(int K, int nc)
{
#define ALPA_BPC(NWK_) (nc == 2 ? blocks_per_cu<NWK_, 2>() : blocks_per_cu<NWK_, 1>())
    switch ((K + 15) / 16) {
    case 5: return ALPA_BPC(5);
    case 6: return ALPA_BPC(6);
    case 7: return ALPA_BPC(7);
    case 8: return ALPA_BPC(8);
    default: return 0;
    }
#undef ALPA_BPC
}

}  // namespace alpa
