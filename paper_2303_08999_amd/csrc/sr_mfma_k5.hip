// Matrix-core kernel instantiations for 5x5 atoms (see sr_mfma_kernel.h).
#include "sr_mfma_kernel.h"

namespace srd {

// Launch shapes of the family with alternatives (three channels, 65 to 72 fp16 atoms), by index
// 1 .. 9: tile width x height in HR pixels, wavefronts per workgroup, workgroups resident per CU.
// Index 7 holds half the LR footprint in LDS and runs at scale 4 only.  Indices 8 and 9 are the
// 128 x 16 tile of index 6 in other arrangements: one workgroup of eight wavefronts per CU (two
// units per wavefront), and two workgroups of two wavefronts (eight units each, one wavefront
// per SIMD with the whole register file).
static const int kShapes = 9;
static const int kShapeW[kShapes + 1] = {0, 64, 128, 64, 128, 64, 128, 128, 128, 128};
static const int kShapeH[kShapes + 1] = {0, 8, 4, 16, 8, 32, 16, 24, 16, 16};
static const int kShapeWaves[kShapes + 1] = {0, 4, 4, 4, 4, 4, 4, 4, 8, 2};
static const int kShapeGroups[kShapes + 1] = {0, 2, 2, 2, 2, 2, 2, 2, 1, 2};

// Index 0 = the default for the frame (measured, 0.26 to 8.3 Mpixel frames at every scale):
// small frames take 128 x 4 tiles, which put more CUs to work (512 x 512: 37 -> 26 us); at x4
// half the footprint in LDS leaves room for 128 x 24, but up to about 1080p its few hundred tiles
// fill the second round of the grid badly and 64 x 16 is 7-13 % faster; else 128 x 16.
int resolve_shape_k5(const AssembleArgs& a, int shape) {
    if (shape != 0) return (shape >= 1 && shape <= kShapes && (shape != 7 || a.s == 4)) ? shape : -1;
    const long long px = (long long)a.N * a.H * a.W;
    if (px <= 400000) return 2;
    if (a.s == 4) return px <= 2600000 ? 3 : 7;
    return 6;
}
bool tile_shape_k5(const AssembleArgs& a, int shape, int* tw, int* th, int* waves, int* groups) {
    const int r = resolve_shape_k5(a, shape);
    if (r < 1) return false;
    *tw = kShapeW[r];
    *th = kShapeH[r];
    if (waves) *waves = kShapeWaves[r];
    if (groups) *groups = kShapeGroups[r];
    return true;
}

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
            switch (resolve_shape_k5(a, shape)) {
            case 1:  return launch_one<5, 3, 9, 4, 2, 4, 1, 2>(a, st);    //  64 x 8
            case 2:  return launch_one<5, 3, 9, 4, 1, 4, 1, 2>(a, st);    // 128 x 4
            case 3:  return launch_one<5, 3, 9, 4, 2, 4, 2, 2>(a, st);    //  64 x 16, 2 units per wavefront
            case 4:  return launch_one<5, 3, 9, 4, 1, 4, 2, 2>(a, st);    // 128 x 8,  2 units
            case 5:  return launch_one<5, 3, 9, 4, 2, 4, 4, 2>(a, st);    //  64 x 32, 4 units
            case 6:  return launch_one<5, 3, 9, 4, 1, 4, 4, 2>(a, st);    // 128 x 16, 4 units
            case 7:  return launch_one<5, 3, 9, 4, 1, 4, 6, 2, CT_F16, 4>(a, st);   // 128 x 24, 6 units (x4 only)
            case 8:  return launch_one<5, 3, 9, 4, 1, 8, 2, 2>(a, st);    // 128 x 16, eight wavefronts, 2 units
            case 9:  return launch_one<5, 3, 9, 4, 1, 2, 8, 1>(a, st);    // 128 x 16, two wavefronts, 8 units, one per SIMD
            default: return hipErrorInvalidValue;
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
