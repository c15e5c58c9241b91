// Matrix-core kernel instantiations for 5x5 atoms with fp8 (e4m3) coefficients
// (see sr_mfma_kernel.h): 4 pixels per lane (4-byte loads, one 128-byte line per
// plane and lane half), widened to fp16 in registers, then the fp16 matrix-core
// fold with the hi + lo dictionary.  Tile 128 x 16 (128 x 24 at scale 4, measured
// 8 % faster there), or 64 x 16 for few atoms.
// (Smaller tiles at three wavefronts per SIMD fit the registers with fp8, but were
// measured 30 % slower: the up-sampling share grows faster than latency hiding pays.)
#include "sr_mfma_kernel.h"

namespace srd {

hipError_t launch_mfma_k5_f8(const AssembleArgs& a, int np8, hipStream_t st) {
    if (a.C == 3) {
        switch (np8) {
        case 1:
            if (a.s == 4) return launch_one<5, 3, 1, 4, 2, 4, 4, 3, CT_F8, 4>(a, st);        //  64 x 32
            return launch_one<5, 3, 1, 4, 2, 4, 2, 3, CT_F8>(a, st);
        case 4:
            if (a.s == 4) return launch_one<5, 3, 4, 4, 1, 4, 6, 2, CT_F8, 4>(a, st);
            return launch_one<5, 3, 4, 4, 1, 4, 4, 2, CT_F8>(a, st);
        case 6:
            if (a.s == 4) return launch_one<5, 3, 6, 4, 1, 4, 6, 2, CT_F8, 4>(a, st);
            return launch_one<5, 3, 6, 4, 1, 4, 4, 2, CT_F8>(a, st);
        case 9: {
            // small frames: 128 x 4 tiles put more CUs to work (512 x 512: 24.6 -> 13.4 us); 64 x 16
            // for medium frames, which pays with fp16 coefficients, measured 3-7 % slower here
            if ((long long)a.N * a.H * a.W <= 400000) return launch_one<5, 3, 9, 4, 1, 4, 1, 2, CT_F8>(a, st);
            if (a.s == 4) return launch_one<5, 3, 9, 4, 1, 4, 6, 2, CT_F8, 4>(a, st);    // 128 x 24
            return launch_one<5, 3, 9, 4, 1, 4, 4, 2, CT_F8>(a, st);
        }
        case 16: return launch_one<5, 3, 16, 4, 1, 4, 4, 1, CT_F8>(a, st);       // 73 to 128 atoms: one wavefront per SIMD, as 7x7
        default: return hipErrorInvalidValue;
        }
    }
    switch (np8) {
    case 16: return launch_one<5, 1, 16, 4, 1, 4, 4, 1, CT_F8>(a, st);
    case 1:  return launch_one<5, 1, 1, 4, 1, 4, 4, 2, CT_F8>(a, st);
    case 4:  return launch_one<5, 1, 4, 4, 1, 4, 4, 2, CT_F8>(a, st);
    case 9:
        if (a.s == 4) return launch_one<5, 1, 9, 4, 1, 4, 6, 2, CT_F8, 4>(a, st);
        return launch_one<5, 1, 9, 4, 1, 4, 4, 2, CT_F8>(a, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace srd
