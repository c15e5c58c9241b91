// Matrix-core kernel instantiations for 3x3 atoms (see sr_mfma_kernel.h): the nine
// taps use nine of the 32 MFMA rows, which costs matrix-core time but no memory
// traffic, so the kernel stays on the coefficient stream like the 5x5 one.
// Tiles as for 5x5.
#include "sr_mfma_kernel.h"

namespace srd {

template <int C, int NP8, int CT>
static hipError_t launch_k3(const AssembleArgs& a, hipStream_t st) {
    constexpr int PX = CT == CT_F32 ? 2 : 4;
    if (a.s == 4 && CT != CT_F32) return launch_one<3, C, NP8, PX, 1, 4, 6, 2, CT, 4>(a, st);
    return launch_one<3, C, NP8, PX, 1, 4, 4, 2, CT>(a, st);
}

template <int C, int CT>
static hipError_t launch_k3_np8(const AssembleArgs& a, int np8, hipStream_t st) {
    switch (np8) {
    case 1:  return launch_k3<C, 1, CT>(a, st);
    case 4:  return launch_k3<C, 4, CT>(a, st);
    case 9:  return launch_k3<C, 9, CT>(a, st);
    case 16:                                         // 73 to 128 atoms, as the 5x5 and 7x7 instantiations of that size:
        // 16-bit coefficients with two pixels per lane, the others with one wavefront per SIMD
        if constexpr (CT == CT_F16 || CT == CT_BF16) return launch_one<3, C, 16, 2, 1, 4, 4, 2, CT>(a, st);
        else return launch_one<3, C, 16, CT == CT_F32 ? 2 : 4, 1, 4, 4, 1, CT>(a, st);
    default: return hipErrorInvalidValue;
    }
}

// np8: capacity in groups of 8 folded atoms (8, 32, 72 or 128 atoms)
hipError_t launch_mfma_k3(const AssembleArgs& a, int np8, hipStream_t st) {
    if (a.coeff_dtype == SR_F32)
        return a.C == 3 ? launch_k3_np8<3, CT_F32>(a, np8, st) : launch_k3_np8<1, CT_F32>(a, np8, st);
    if (a.coeff_dtype == SR_F8E4M3)
        return a.C == 3 ? launch_k3_np8<3, CT_F8>(a, np8, st) : launch_k3_np8<1, CT_F8>(a, np8, st);
    if (a.coeff_dtype == SR_BF16)
        return a.C == 3 ? launch_k3_np8<3, CT_BF16>(a, np8, st) : launch_k3_np8<1, CT_BF16>(a, np8, st);
    return a.C == 3 ? launch_k3_np8<3, CT_F16>(a, np8, st) : launch_k3_np8<1, CT_F16>(a, np8, st);
}

}  // namespace srd
