// Matrix-core kernel instantiations for coefficients stored blocked (see PSM = 9 in sr_mfma_kernel.h and
// SR_COEFF_BLOCKED; a storage order beyond the paper): 5x5 atoms, three channels, all of 72 fp16, bfloat16 or 8-bit atoms.
#include "sr_mfma_kernel.h"

namespace srd {

// The tiles of the planar form: 128 x 24 at scale 4 (half the LR footprint), 128 x 16 below.
hipError_t launch_mfma_k5_blk(const AssembleArgs& a, hipStream_t st) {
    if (a.C != 3 || a.L != 72) return hipErrorInvalidValue;
    if (a.coeff_dtype == SR_F8E4M3) {
        if (a.s == 4) return launch_one<5, 3, 9, 4, 1, 4, 6, 2, CT_F8, 4, false, 9>(a, st);
        return launch_one<5, 3, 9, 4, 1, 4, 4, 2, CT_F8, 2, false, 9>(a, st);
    }
    if (a.coeff_dtype == SR_BF16 && !a.logits) {
        if (a.s == 4) return launch_one<5, 3, 9, 4, 1, 4, 6, 2, CT_BF16, 4, false, 9>(a, st);
        return launch_one<5, 3, 9, 4, 1, 4, 4, 2, CT_BF16, 2, false, 9>(a, st);
    }
    if (a.coeff_dtype != SR_F16) return hipErrorInvalidValue;
    if (a.logits) {                     // logits in the blocked order: the softmax in the operand path (see CT_LOGIT)
        if (a.s == 4) return launch_one<5, 3, 9, 4, 1, 4, 6, 2, CT_LOGIT, 4, false, 9>(a, st);
        return launch_one<5, 3, 9, 4, 1, 4, 4, 2, CT_LOGIT, 2, false, 9>(a, st);
    }
    if (a.s == 4) return launch_one<5, 3, 9, 4, 1, 4, 6, 2, CT_F16, 4, false, 9>(a, st);
    return launch_one<5, 3, 9, 4, 1, 4, 4, 2, CT_F16, 2, false, 9>(a, st);
}

}  // namespace srd
