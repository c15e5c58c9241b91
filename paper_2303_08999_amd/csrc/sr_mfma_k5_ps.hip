// Matrix-core kernel instantiations that read the coefficients in the layout they have before
// the coefficient network's pixel-shuffle layer (see PSM in sr_mfma_kernel.h): 5x5 atoms, three
// channels, fp16 coefficients with up to 8 or 65 to 72 folded atoms, bfloat16 coefficients with 65 to 72.
#include "sr_mfma_kernel.h"

namespace srd {

hipError_t launch_mfma_k5_ps(const AssembleArgs& a, int np8, hipStream_t st) {
    if (a.C != 3) return hipErrorInvalidValue;
    if (a.coeff_dtype == SR_BF16) {          // bfloat16 coefficients: the permuted-slot forms, 65 to 72 atoms
        if (np8 != 9 || a.w % 4 != 0) return hipErrorInvalidValue;
        if (a.s == 4) return launch_one<5, 3, 9, 4, 1, 4, 4, 2, CT_BF16, 4, false, 4>(a, st);
        if (a.s == 3) return launch_one<5, 3, 9, 4, 1, 8, 3, 2, CT_BF16, 3, false, 3>(a, st);
        return launch_one<5, 3, 9, 4, 1, 4, 4, 2, CT_BF16, 2, false, 2>(a, st);
    }
    // LR width a multiple of 4: the fast forms (permuted pixel slots, the planar form's loads).  Scale 3 needs
    // 384-pixel rows for whole cache lines; its tile takes most of a CU's LDS: one workgroup of eight wavefronts.
    const bool perm = a.w % 4 == 0;
    switch (np8) {
    case 1:
        if (perm && a.s == 4) return launch_one<5, 3, 1, 4, 1, 4, 4, 2, CT_F16, 4, false, 4>(a, st);   // 256 x 8
        if (perm && a.s == 3) return launch_one<5, 3, 1, 4, 1, 8, 3, 2, CT_F16, 3, false, 3>(a, st);   // 384 x 8
        if (perm) return launch_one<5, 3, 1, 4, 1, 4, 2, 2, CT_F16, 2, false, 2>(a, st);               // 128 x 8
        if (a.s == 4) return launch_one<5, 3, 1, 4, 2, 4, 4, 2, CT_F16, 4, false, 1>(a, st);           //  64 x 32
        return launch_one<5, 3, 1, 4, 2, 4, 2, 2, CT_F16, 2, false, 1>(a, st);                         //  64 x 16
    case 9:
        if (perm && a.s == 4) return launch_one<5, 3, 9, 4, 1, 4, 4, 2, CT_F16, 4, false, 4>(a, st);   // 256 x 8
        if (perm && a.s == 3) return launch_one<5, 3, 9, 4, 1, 8, 3, 2, CT_F16, 3, false, 3>(a, st);   // 384 x 8
        if (perm) return launch_one<5, 3, 9, 4, 1, 4, 4, 2, CT_F16, 2, false, 2>(a, st);               // 128 x 16
        // LR widths that are not a multiple of 4: one 16-bit load per pixel and plane.  Every load occupies a
        // register until its pair is packed, twice the registers of the planar form for a unit in flight: one
        // wavefront per SIMD, as two workgroups of two wavefronts per CU, so that one streams while the other
        // up-samples.
        if (a.s == 4) return launch_one<5, 3, 9, 4, 1, 2, 6, 1, CT_F16, 4, false, 1>(a, st);           // 128 x 12
        return launch_one<5, 3, 9, 4, 1, 2, 4, 1, CT_F16, 2, false, 1>(a, st);                         // 128 x 8
    default: return hipErrorInvalidValue;
    }
}

}  // namespace srd
