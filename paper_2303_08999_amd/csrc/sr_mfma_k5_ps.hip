// Matrix-core kernel instantiations that read the coefficients in the layout they have before
// the coefficient network's pixel-shuffle layer (see PS in sr_mfma_kernel.h): 5x5 atoms, three
// channels, fp16 coefficients, up to 8 or 65 to 72 folded atoms.
#include "sr_mfma_kernel.h"

namespace srd {

hipError_t launch_mfma_k5_ps(const AssembleArgs& a, int np8, hipStream_t st) {
    if (a.C != 3) return hipErrorInvalidValue;
    // Every 16-bit load occupies a register until its pair is packed, so a unit in flight takes twice
    // the registers of the HR-planar form.  72 atoms: one wavefront per SIMD (371 registers), as two
    // workgroups of two wavefronts per CU, so that one streams while the other up-samples.
    switch (np8) {
    case 1:
        if (a.s == 4) return launch_one<5, 3, 1, 4, 2, 4, 4, 2, CT_F16, 4, false, true>(a, st);     //  64 x 32
        return launch_one<5, 3, 1, 4, 2, 4, 2, 2, CT_F16, 2, false, true>(a, st);                   //  64 x 16
    case 9:
        if (a.s == 4) return launch_one<5, 3, 9, 4, 1, 2, 6, 1, CT_F16, 4, false, true>(a, st);     // 128 x 12
        return launch_one<5, 3, 9, 4, 1, 2, 4, 1, CT_F16, 2, false, true>(a, st);                   // 128 x 8
    default: return hipErrorInvalidValue;
    }
}

}  // namespace srd
