// Matrix-core kernel instantiations for 5x5 atoms (see sr_mfma_kernel.h).
#include "sr_mfma_kernel.h"

namespace srd {

// np8: capacity in groups of 8 folded atoms; shape: tile shape index (C = 3, np8 = 9 only)
hipError_t launch_mfma_k5(const AssembleArgs& a, int np8, int shape, hipStream_t st) {
    // Few atoms: the kernel is bound by up-sampling, filtering and the output
    // write rather than by the coefficient stream; the register budget then
    // allows three wavefronts per SIMD, which measured 25 % faster.
    if (a.C == 3) {
        switch (np8) {
        case 1:
            // x4: 64 x 32 still fits three workgroups per CU (measured 11 % faster)
            if (a.s == 4) return launch_one<5, 3, 1, 4, 2, 4, 4, 3, CT_F16, 4>(a, st);
            return launch_one<5, 3, 1, 4, 2, 4, 2, 3>(a, st);        //  64 x 16
        case 2:
            if (a.s == 4) return launch_one<5, 3, 2, 4, 2, 4, 4, 3, CT_F16, 4>(a, st);
            return launch_one<5, 3, 2, 4, 2, 4, 2, 3>(a, st);
        case 4:
            if (a.s == 4) return launch_one<5, 3, 4, 4, 1, 4, 6, 2, CT_F16, 4>(a, st);   // 128 x 24 (6-10 % faster)
            return launch_one<5, 3, 4, 4, 1, 4, 4, 2>(a, st);
        case 6:
            if (a.s == 4) return launch_one<5, 3, 6, 4, 1, 4, 6, 2, CT_F16, 4>(a, st);
            return launch_one<5, 3, 6, 4, 1, 4, 4, 2>(a, st);
        case 9:
            switch (shape) {
            case 1:  return launch_one<5, 3, 9, 4, 2, 4, 1, 2>(a, st);    //  64 x 8
            case 2:  return launch_one<5, 3, 9, 4, 1, 4, 1, 2>(a, st);    // 128 x 4
            case 3:  return launch_one<5, 3, 9, 4, 2, 4, 2, 2>(a, st);    //  64 x 16, 2 units per wavefront
            case 4:  return launch_one<5, 3, 9, 4, 1, 4, 2, 2>(a, st);    // 128 x 8,  2 units
            case 5:  return launch_one<5, 3, 9, 4, 2, 4, 4, 2>(a, st);    //  64 x 32, 4 units
            default: {
                // Tile by frame size (measured, 0.26 to 8.3 Mpixel frames at every scale).
                // Small frames: 128 x 4 tiles put more CUs to work (512 x 512: 37 -> 26 us).
                const long long px = (long long)a.N * a.H * a.W;
                if (px <= 400000) return launch_one<5, 3, 9, 4, 1, 4, 1, 2>(a, st);
                // x4: half the footprint in LDS leaves room for a 128 x 24 tile (6 units); up to
                // about 1080p its few hundred tiles fill the second round of the grid badly
                // and 64 x 16 is 7-13 % faster
                if (a.s == 4) {
                    if (px <= 2600000) return launch_one<5, 3, 9, 4, 2, 4, 2, 2>(a, st);
                    return launch_one<5, 3, 9, 4, 1, 4, 6, 2, CT_F16, 4>(a, st);
                }
                return launch_one<5, 3, 9, 4, 1, 4, 4, 2>(a, st);    // 128 x 16, 4 units
            }
            }
        case 16:                                                         // 73 to 128 atoms: two pixels per lane, as 7x7
            if (a.s == 4) return launch_one<5, 3, 16, 2, 1, 4, 6, 2, CT_F16, 4>(a, st);
            return launch_one<5, 3, 16, 2, 1, 4, 4, 2>(a, st);
        default: return hipErrorInvalidValue;
        }
    }
    // Two and four channels (fp16 coefficients only): 32 and 72 atoms.  Four channels
    // fill the LDS tile and the registers faster: tile 128 x 8.
    if (a.C == 2) {
        switch (np8) {
        case 4:  return launch_one<5, 2, 4, 4, 1, 4, 4, 2>(a, st);
        case 9:  return launch_one<5, 2, 9, 4, 1, 4, 4, 2>(a, st);
        default: return hipErrorInvalidValue;
        }
    }
    if (a.C == 4) {
        switch (np8) {
        case 4:  return launch_one<5, 4, 4, 4, 1, 4, 2, 2>(a, st);
        case 9:  return launch_one<5, 4, 9, 4, 1, 4, 2, 2>(a, st);
        default: return hipErrorInvalidValue;
        }
    }
    switch (np8) {
    case 1:  return launch_one<5, 1, 1, 4, 1, 4, 4, 2>(a, st);
    case 4:  return launch_one<5, 1, 4, 4, 1, 4, 4, 2>(a, st);
    case 6:  return launch_one<5, 1, 6, 4, 1, 4, 4, 2>(a, st);
    case 9:
        if (a.s == 4) return launch_one<5, 1, 9, 4, 1, 4, 6, 2, CT_F16, 4>(a, st);
        return launch_one<5, 1, 9, 4, 1, 4, 4, 2>(a, st);
    case 16:
        if (a.s == 4) return launch_one<5, 1, 16, 2, 1, 4, 6, 2, CT_F16, 4>(a, st);
        return launch_one<5, 1, 16, 2, 1, 4, 4, 2>(a, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace srd
