// Matrix-core kernel instantiations for fp32 coefficients (see sr_mfma_kernel.h):
// 2 pixels per lane (8-byte loads), tile 64 x 16 unless noted.
#include "sr_mfma_kernel.h"

namespace srd {

// A frame of a few tiles leaves most CUs idle and takes as long as one workgroup
// needs for its tile: such frames go in 64 x 4 tiles (one unit per wavefront).
static bool few_tiles(const AssembleArgs& a) { return (long long)a.N * a.H * a.W <= 64LL * 64 * 16; }

// np8: capacity in groups of 8 folded atoms (kept lists read only their own planes)
hipError_t launch_mfma_k5_f32(const AssembleArgs& a, int np8, hipStream_t st) {
    if (np8 == 9 && few_tiles(a))
        return a.C == 3 ? launch_one<5, 3, 9, 2, 1, 4, 1, 2, CT_F32>(a, st) : launch_one<5, 1, 9, 2, 1, 4, 1, 2, CT_F32>(a, st);
    if (a.C == 3) {
        switch (np8) {
        case 1:  return launch_one<5, 3, 1, 2, 1, 4, 4, 2, CT_F32>(a, st);
        case 2:  return launch_one<5, 3, 2, 2, 1, 4, 4, 2, CT_F32>(a, st);
        case 4:  return launch_one<5, 3, 4, 2, 1, 4, 4, 2, CT_F32>(a, st);
        case 6:  return launch_one<5, 3, 6, 2, 1, 4, 4, 2, CT_F32>(a, st);
        case 9:
            // x4 from about 720p on: the smaller footprint leaves room for 64 x 32 (2-5 % faster;
            // 720p fits the grid in one round of 460 tiles)
            if (a.s == 4 && (long long)a.N * a.H * a.W > 600000) return launch_one<5, 3, 9, 2, 1, 4, 8, 2, CT_F32, 4>(a, st);
            return launch_one<5, 3, 9, 2, 1, 4, 4, 2, CT_F32>(a, st);
        case 16: return launch_one<5, 3, 16, 2, 1, 4, 4, 1, CT_F32>(a, st);      // 73 to 128 atoms: one wavefront per SIMD, as 7x7
        default: return hipErrorInvalidValue;
        }
    }
    switch (np8) {
    case 1:  return launch_one<5, 1, 1, 2, 1, 4, 4, 2, CT_F32>(a, st);
    case 4:  return launch_one<5, 1, 4, 2, 1, 4, 4, 2, CT_F32>(a, st);
    case 6:  return launch_one<5, 1, 6, 2, 1, 4, 4, 2, CT_F32>(a, st);
    case 9:  return launch_one<5, 1, 9, 2, 1, 4, 4, 2, CT_F32>(a, st);
    case 16: return launch_one<5, 1, 16, 2, 1, 4, 4, 1, CT_F32>(a, st);
    default: return hipErrorInvalidValue;
    }
}

// 7x7 atoms: two 32-row MFMA blocks per pixel slot; 128 atoms need the whole
// register file of a SIMD (one wavefront per SIMD).  Lists of up to 16 atoms are
// left to the generic kernel, which measured faster there (62 against 80 us at 1080p).
hipError_t launch_mfma_k7_f32(const AssembleArgs& a, int np8, hipStream_t st) {
    if (a.C == 3) {
        switch (np8) {
        case 9:  return launch_one<7, 3, 9, 2, 1, 4, 4, 2, CT_F32>(a, st);
        case 16: return launch_one<7, 3, 16, 2, 1, 4, 4, 1, CT_F32>(a, st);
        default: return hipErrorInvalidValue;
        }
    }
    switch (np8) {
    case 9:  return launch_one<7, 1, 9, 2, 1, 4, 4, 2, CT_F32>(a, st);
    case 16: return launch_one<7, 1, 16, 2, 1, 4, 4, 1, CT_F32>(a, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace srd
