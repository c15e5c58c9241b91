// Matrix-core kernel instantiations for 5x5 atoms, three channels, fp16 or bfloat16
// coefficients on images whose coefficient tensor exceeds 4 GB (see sr_mfma_kernel.h, BIG):
// offsets in elements instead of bytes.  Same tiles as the ordinary instantiations for
// large frames.
#include "sr_mfma_kernel.h"

namespace srd {

template <int CT>
static hipError_t launch_big(const AssembleArgs& a, int np8, hipStream_t st) {
    switch (np8) {
    case 1:
        if (a.s == 4) return launch_one<5, 3, 1, 4, 2, 4, 4, 3, CT, 4, true>(a, st);     //  64 x 32
        return launch_one<5, 3, 1, 4, 2, 4, 2, 3, CT, 2, true>(a, st);                   //  64 x 16
    case 4:
        if (a.s == 4) return launch_one<5, 3, 4, 4, 1, 4, 6, 2, CT, 4, true>(a, st);     // 128 x 24
        return launch_one<5, 3, 4, 4, 1, 4, 4, 2, CT, 2, true>(a, st);                   // 128 x 16
    case 9:
        if (a.s == 4) return launch_one<5, 3, 9, 4, 1, 4, 6, 2, CT, 4, true>(a, st);
        return launch_one<5, 3, 9, 4, 1, 4, 4, 2, CT, 2, true>(a, st);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_mfma_k5_big(const AssembleArgs& a, int np8, hipStream_t st) {
    if (a.C != 3) return hipErrorInvalidValue;
    if (a.coeff_dtype == SR_F16) return launch_big<CT_F16>(a, np8, st);
    if (a.coeff_dtype == SR_BF16) return launch_big<CT_BF16>(a, np8, st);
    return hipErrorInvalidValue;
}

}  // namespace srd
