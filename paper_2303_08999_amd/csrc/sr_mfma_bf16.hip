// Matrix-core kernel instantiations for bfloat16 coefficients (see sr_mfma_kernel.h, CT_BF16):
// the same flow and tiles as fp16 coefficients, with the fold on the bfloat16 matrix
// instructions and the dictionary split into two bfloat16 operands.
// 5x5 atoms, one or three channels, capacities of 8, 32 and 72 atoms; 7x7 atoms, three
// channels, 72 and 128 atoms.
#include "sr_mfma_kernel.h"

namespace srd {

template <int C>
static hipError_t launch_k5(const AssembleArgs& a, int np8, hipStream_t st) {
    switch (np8) {
    case 1:
        if (a.s == 4) return launch_one<5, C, 1, 4, 2, 4, 4, 3, CT_BF16, 4>(a, st);      //  64 x 32
        return launch_one<5, C, 1, 4, 2, 4, 2, 3, CT_BF16>(a, st);                       //  64 x 16
    case 4:
        if (a.s == 4) return launch_one<5, C, 4, 4, 1, 4, 6, 2, CT_BF16, 4>(a, st);      // 128 x 24
        return launch_one<5, C, 4, 4, 1, 4, 4, 2, CT_BF16>(a, st);                       // 128 x 16
    case 9:
        // small frames: 128 x 4 tiles put more CUs to work (as with fp16 coefficients)
        if ((long long)a.N * a.H * a.W <= 400000) return launch_one<5, C, 9, 4, 1, 4, 1, 2, CT_BF16>(a, st);
        if (a.s == 4) return launch_one<5, C, 9, 4, 1, 4, 6, 2, CT_BF16, 4>(a, st);
        return launch_one<5, C, 9, 4, 1, 4, 4, 2, CT_BF16>(a, st);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_mfma_bf16(const AssembleArgs& a, int k, int np8, hipStream_t st) {
    if (k == 5) {
        if (a.C == 3) return launch_k5<3>(a, np8, st);
        if (a.C == 1) return launch_k5<1>(a, np8, st);
        return hipErrorInvalidValue;
    }
    if (k == 7 && a.C == 3) {
        switch (np8) {
        case 9:
            if (a.s == 4) return launch_one<7, 3, 9, 2, 1, 4, 6, 2, CT_BF16, 4>(a, st);
            return launch_one<7, 3, 9, 2, 1, 4, 4, 2, CT_BF16>(a, st);
        case 16:
            if (a.s == 4) return launch_one<7, 3, 16, 2, 1, 4, 6, 2, CT_BF16, 4>(a, st);
            return launch_one<7, 3, 16, 2, 1, 4, 4, 2, CT_BF16>(a, st);
        default: return hipErrorInvalidValue;
        }
    }
    return hipErrorInvalidValue;
}

}  // namespace srd
