// Matrix-core kernel instantiations for coefficients stored pixel-major, [N][H][W][L] (see PSM = 8 in
// sr_mfma_kernel.h; a storage order beyond the paper): 5x5 atoms, three channels, all of 72 fp16 atoms.
#include "sr_mfma_kernel.h"

namespace srd {

// The 18 KB of staging scratch leave room for 128 x 16 tiles at scale 4 (half the LR footprint) and 128 x 8 below.
hipError_t launch_mfma_k5_pm(const AssembleArgs& a, hipStream_t st) {
    if (a.C != 3 || a.L != 72) return hipErrorInvalidValue;
    if (a.s == 4) return launch_one<5, 3, 9, 4, 1, 4, 4, 2, CT_F16, 4, false, 8>(a, st);
    return launch_one<5, 3, 9, 4, 1, 4, 2, 2, CT_F16, 2, false, 8>(a, st);
}

}  // namespace srd
