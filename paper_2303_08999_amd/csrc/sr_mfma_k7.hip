// Matrix-core kernel instantiations for 7x7 atoms (see sr_mfma_kernel.h).
// 49 taps need two 32-row MFMA blocks per pixel slot, so a lane carries two
// pixels (4-byte loads) to keep the accumulators within the register budget.
// Tile 64 x 16: 4 wavefronts x 4 one-row units (measured 5 % faster than 2 units;
// 6 units and more no longer leave room for two workgroups per CU in LDS).
#include "sr_mfma_kernel.h"

namespace srd {

hipError_t launch_mfma_k7(const AssembleArgs& a, int np8, int shape, hipStream_t st) {
    (void)shape;
    if (a.C == 3) {
        switch (np8) {
        case 2:  return launch_one<7, 3, 2, 2, 1, 4, 4, 2>(a, st);
        case 9:  return launch_one<7, 3, 9, 2, 1, 4, 4, 2>(a, st);
        case 16: return launch_one<7, 3, 16, 2, 1, 4, 4, 2>(a, st);
        default: return hipErrorInvalidValue;
        }
    }
    switch (np8) {
    case 16: return launch_one<7, 1, 16, 2, 1, 4, 4, 2>(a, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace srd
