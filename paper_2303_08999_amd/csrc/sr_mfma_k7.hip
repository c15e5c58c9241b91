// Matrix-core kernel instantiations for 7x7 atoms (see sr_mfma_kernel.h).
// 49 taps need two 32-row MFMA blocks per pixel slot, so a lane carries two
// pixels (4-byte loads) to keep the accumulators within the register budget.
// Tile 64 x 16: 4 wavefronts x 4 one-row units (measured 5 % faster than 2 units;
// 6 units and more no longer leave room for two workgroups per CU in LDS), except
// at scale 4, where the smaller LR footprint makes room for 64 x 24 (2.5 % faster).
#include "sr_mfma_kernel.h"

namespace srd {

template <int C, int NP8>
static hipError_t launch_k7(const AssembleArgs& a, hipStream_t st) {
    if (a.s == 4) return launch_one<7, C, NP8, 2, 1, 4, 6, 2, CT_F16, 4>(a, st);
    return launch_one<7, C, NP8, 2, 1, 4, 4, 2>(a, st);
}

hipError_t launch_mfma_k7(const AssembleArgs& a, int np8, int shape, hipStream_t st) {
    (void)shape;
    if (a.C == 3) {
        switch (np8) {
        case 2:  return launch_k7<3, 2>(a, st);
        case 9:  return launch_k7<3, 9>(a, st);
        case 16: return launch_k7<3, 16>(a, st);
        default: return hipErrorInvalidValue;
        }
    }
    switch (np8) {
    case 2:  return launch_k7<1, 2>(a, st);
    case 9:  return launch_k7<1, 9>(a, st);
    case 16: return launch_k7<1, 16>(a, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace srd
