// Matrix-core kernel instantiations for 7x7 atoms with fp8 (e4m3) coefficients (see
// sr_mfma_kernel.h).  The 4-byte loads of the 8-bit planes carry four pixels per
// lane, and four pixel slots of two 32-row MFMA blocks each take the whole register
// file of a SIMD: one wavefront per SIMD, tile 128 x 16.
#include "sr_mfma_kernel.h"

namespace srd {

hipError_t launch_mfma_k7_f8(const AssembleArgs& a, int np8, hipStream_t st) {
    if (a.C == 3) {
        switch (np8) {
        case 9:  return launch_one<7, 3, 9, 4, 1, 4, 4, 1, CT_F8>(a, st);
        case 16: return launch_one<7, 3, 16, 4, 1, 4, 4, 1, CT_F8>(a, st);
        default: return hipErrorInvalidValue;
        }
    }
    switch (np8) {
    case 9:  return launch_one<7, 1, 9, 4, 1, 4, 4, 1, CT_F8>(a, st);
    case 16: return launch_one<7, 1, 16, 4, 1, 4, 4, 1, CT_F8>(a, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace srd
