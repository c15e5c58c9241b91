// Matrix-core kernel instantiations for coefficients handed over as LOGITS (see CT_LOGIT in sr_mfma_kernel.h; an
// extension beyond the paper): 5x5 atoms, three channels, 49 to 72 fp16 or bfloat16 planes (the capacity of nine
// groups of eight atoms), all of them folded.
#include "sr_mfma_kernel.h"

namespace srd {

// The tiles of the fp16 form: 128 x 24 at scale 4 (half the LR footprint), 128 x 16 below.  Logits in the layout
// before the network's pixel-shuffle (what its last convolution writes): the permuted-slot forms of that layout,
// LR widths that are multiples of 4.
template <int CT>
static hipError_t launch_lg(const AssembleArgs& a, hipStream_t st) {
    if (a.pre_shuffle) {
        if (a.w % 4 != 0) return hipErrorInvalidValue;
        if (a.s == 4) return launch_one<5, 3, 9, 4, 1, 4, 4, 2, CT, 4, false, 4>(a, st);   // 256 x 8
        if (a.s == 3) return launch_one<5, 3, 9, 4, 1, 8, 3, 2, CT, 3, false, 3>(a, st);   // 384 x 8
        return launch_one<5, 3, 9, 4, 1, 4, 4, 2, CT, 2, false, 2>(a, st);                 // 128 x 16
    }
    if (a.s == 4) return launch_one<5, 3, 9, 4, 1, 4, 6, 2, CT, 4>(a, st);
    return launch_one<5, 3, 9, 4, 1, 4, 4, 2, CT, 2>(a, st);
}

hipError_t launch_mfma_k5_lg(const AssembleArgs& a, hipStream_t st) {
    if (a.C != 3 || a.L < 1 || a.L > 72) return hipErrorInvalidValue;
    if (a.coeff_dtype == SR_BF16) return launch_lg<CT_LOGIT_BF16>(a, st);
    if (a.coeff_dtype == SR_F16) return launch_lg<CT_LOGIT>(a, st);
    return hipErrorInvalidValue;
}

}  // namespace srd
