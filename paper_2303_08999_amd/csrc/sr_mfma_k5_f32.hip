// Matrix-core kernel instantiations for 5x5 atoms and fp32 coefficients (see
// sr_mfma_kernel.h): 2 pixels per lane (8-byte loads), tile 64 x 16.
#include "sr_mfma_kernel.h"

namespace srd {

// np8: capacity in groups of 8 folded atoms (kept lists read only their own planes)
hipError_t launch_mfma_k5_f32(const AssembleArgs& a, int np8, hipStream_t st) {
    if (a.C == 3) {
        switch (np8) {
        case 1:  return launch_one<5, 3, 1, 2, 1, 4, 4, 2, CT_F32>(a, st);
        case 2:  return launch_one<5, 3, 2, 2, 1, 4, 4, 2, CT_F32>(a, st);
        case 4:  return launch_one<5, 3, 4, 2, 1, 4, 4, 2, CT_F32>(a, st);
        case 6:  return launch_one<5, 3, 6, 2, 1, 4, 4, 2, CT_F32>(a, st);
        case 9:  return launch_one<5, 3, 9, 2, 1, 4, 4, 2, CT_F32>(a, st);
        default: return hipErrorInvalidValue;
        }
    }
    if (np8 != 9) return hipErrorInvalidValue;
    return launch_one<5, 1, 9, 2, 1, 4, 4, 2, CT_F32>(a, st);
}

}  // namespace srd
