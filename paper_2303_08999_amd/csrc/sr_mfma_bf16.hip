// Matrix-core kernel instantiations for bfloat16 coefficients (see sr_mfma_kernel.h, CT_BF16):
// the same flow and tiles as fp16 coefficients, with the fold on the bfloat16 matrix
// instructions and the dictionary split into two bfloat16 operands.
// The capacities built for fp16: 5x5 atoms with 8, 16 (three channels), 32, 48 and 72 atoms
// (two or four channels: 32 and 72); 7x7 atoms with 16, 72 and 128.  (3x3 atoms:
// sr_mfma_k3.hip.)
#include "sr_mfma_kernel.h"

namespace srd {

template <int C>
static hipError_t launch_k5(const AssembleArgs& a, int np8, hipStream_t st) {
    switch (np8) {
    case 1:
        if (a.s == 4) return launch_one<5, C, 1, 4, 2, 4, 4, 3, CT_BF16, 4>(a, st);      //  64 x 32
        return launch_one<5, C, 1, 4, 2, 4, 2, 3, CT_BF16>(a, st);                       //  64 x 16
    case 2:
        if (C != 3) return hipErrorInvalidValue;
        if (a.s == 4) return launch_one<5, 3, 2, 4, 2, 4, 4, 3, CT_BF16, 4>(a, st);
        return launch_one<5, 3, 2, 4, 2, 4, 2, 3, CT_BF16>(a, st);
    case 4:
        if (a.s == 4) return launch_one<5, C, 4, 4, 1, 4, 6, 2, CT_BF16, 4>(a, st);      // 128 x 24
        return launch_one<5, C, 4, 4, 1, 4, 4, 2, CT_BF16>(a, st);                       // 128 x 16
    case 6:
        if (a.s == 4) return launch_one<5, C, 6, 4, 1, 4, 6, 2, CT_BF16, 4>(a, st);
        return launch_one<5, C, 6, 4, 1, 4, 4, 2, CT_BF16>(a, st);
    case 9:
        // small frames: 128 x 4 tiles put more CUs to work (as with fp16 coefficients)
        if ((long long)a.N * a.H * a.W <= 400000) return launch_one<5, C, 9, 4, 1, 4, 1, 2, CT_BF16>(a, st);
        if (a.s == 4) return launch_one<5, C, 9, 4, 1, 4, 6, 2, CT_BF16, 4>(a, st);
        return launch_one<5, C, 9, 4, 1, 4, 4, 2, CT_BF16>(a, st);
    case 16:                                                             // 73 to 128 atoms: two pixels per lane, as 7x7
        if (a.s == 4) return launch_one<5, C, 16, 2, 1, 4, 6, 2, CT_BF16, 4>(a, st);
        return launch_one<5, C, 16, 2, 1, 4, 4, 2, CT_BF16>(a, st);
    default: return hipErrorInvalidValue;
    }
}

template <int C>
static hipError_t launch_k7(const AssembleArgs& a, int np8, hipStream_t st) {
    switch (np8) {
    case 2:
        if (a.s == 4) return launch_one<7, C, 2, 2, 1, 4, 6, 2, CT_BF16, 4>(a, st);
        return launch_one<7, C, 2, 2, 1, 4, 4, 2, CT_BF16>(a, st);
    case 9:
        if (a.s == 4) return launch_one<7, C, 9, 2, 1, 4, 6, 2, CT_BF16, 4>(a, st);
        return launch_one<7, C, 9, 2, 1, 4, 4, 2, CT_BF16>(a, st);
    case 16:
        if (a.s == 4) return launch_one<7, C, 16, 2, 1, 4, 6, 2, CT_BF16, 4>(a, st);
        return launch_one<7, C, 16, 2, 1, 4, 4, 2, CT_BF16>(a, st);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_mfma_bf16(const AssembleArgs& a, int k, int np8, hipStream_t st) {
    if (k == 5) {
        if (a.C == 3) return launch_k5<3>(a, np8, st);
        if (a.C == 1) return launch_k5<1>(a, np8, st);
        // two and four channels: tiles as with fp16 coefficients
        if (a.C == 2) return np8 == 4 ? launch_one<5, 2, 4, 4, 1, 4, 4, 2, CT_BF16>(a, st)
                           : np8 == 9 ? launch_one<5, 2, 9, 4, 1, 4, 4, 2, CT_BF16>(a, st) : hipErrorInvalidValue;
        if (a.C == 4) return np8 == 4 ? launch_one<5, 4, 4, 4, 1, 4, 2, 2, CT_BF16>(a, st)
                           : np8 == 9 ? launch_one<5, 4, 9, 4, 1, 4, 2, 2, CT_BF16>(a, st) : hipErrorInvalidValue;
        return hipErrorInvalidValue;
    }
    if (k == 7 && a.C == 3) return launch_k7<3>(a, np8, st);
    if (k == 7 && a.C == 1) return launch_k7<1>(a, np8, st);
    return hipErrorInvalidValue;
}

}  // namespace srd
