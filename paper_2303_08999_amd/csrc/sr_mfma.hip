// Matrix-core path, host side: which kernel instantiation serves a call.
// The kernel itself is in sr_mfma_kernel.h; its instantiations are compiled in
// sr_mfma_k3.hip, sr_mfma_k5*.hip and sr_mfma_k7*.hip.
#include "sr_launch.h"

namespace srd {

hipError_t launch_mfma_k3(const AssembleArgs& a, int np8, hipStream_t st);
hipError_t launch_mfma_k5(const AssembleArgs& a, int np8, int shape, hipStream_t st);
bool tile_shape_k5(const AssembleArgs& a, int shape, int* tw, int* th, int* waves, int* groups);
hipError_t launch_mfma_k7(const AssembleArgs& a, int np8, int shape, hipStream_t st);
hipError_t launch_mfma_k5_f32(const AssembleArgs& a, int np8, hipStream_t st);
hipError_t launch_mfma_k7_f32(const AssembleArgs& a, int np8, hipStream_t st);
hipError_t launch_mfma_k5_f8(const AssembleArgs& a, int np8, hipStream_t st);
hipError_t launch_mfma_k7_f8(const AssembleArgs& a, int np8, hipStream_t st);
hipError_t launch_mfma_k5_big(const AssembleArgs& a, int np8, hipStream_t st);
hipError_t launch_mfma_bf16(const AssembleArgs& a, int k, int np8, hipStream_t st);
hipError_t launch_mfma_k5_ps(const AssembleArgs& a, int np8, hipStream_t st);
hipError_t launch_mfma_k5_pm(const AssembleArgs& a, hipStream_t st);
hipError_t launch_mfma_k5_lg(const AssembleArgs& a, hipStream_t st);
hipError_t launch_mfma_k5_blk(const AssembleArgs& a, hipStream_t st);

namespace {


// Capacity (in groups of 8 folded atoms) of the smallest built instantiation
// that holds n_fold atoms; 0 = none.  Unused capacity costs MFMA issue slots
// only: padding atoms meet zero dictionary rows and re-read a cached plane.
int np8_for(int k, int channels, int n_fold, int coeff_dtype) {
    const int need = (n_fold + 7) / 8;
    if (channels == 2 || channels == 4)                                 // 5x5, 16-bit coefficients: 32 and 72 atoms
        return (k == 5 && (coeff_dtype == SR_F16 || coeff_dtype == SR_BF16) && need <= 9) ? (need <= 4 ? 4 : 9) : 0;
    if (k == 3) {                                                       // 3x3: up to 128 atoms
        if (need > 16) return 0;
        return need <= 1 ? 1 : (need <= 4 ? 4 : (need <= 9 ? 9 : 16));
    }
    if (coeff_dtype == SR_F32) {                                        // fp32 coefficients
        static const int k5c3[] = {1, 2, 4, 6, 9, 16, 0}, k5c1[] = {1, 4, 6, 9, 16, 0}, k7[] = {9, 16, 0};
        if (k == 7 && need <= 2) return 0;                                // short 7x7 lists: the generic kernel is faster
        const int* built = k == 5 ? (channels == 3 ? k5c3 : k5c1) : k7;
        for (; *built; ++built)
            if (*built >= need) return *built;
        return 0;
    }
    if (coeff_dtype == SR_F8E4M3) {                                     // 8-bit coefficients
        static const int c3[] = {1, 4, 6, 9, 16, 0}, c1[] = {1, 4, 9, 16, 0};
        if (k == 7) return need <= 2 ? 0 : (need <= 9 ? 9 : (need <= 16 ? 16 : 0));   // short lists: generic kernel
        for (const int* built = channels == 3 ? c3 : c1; *built; ++built)
            if (*built >= need) return *built;
        return 0;
    }
    // fp16 and bfloat16 coefficients
    static const int k5c3[] = {1, 2, 4, 6, 9, 16, 0}, k5c1[] = {1, 4, 6, 9, 16, 0};
    static const int k7c3[] = {2, 9, 16, 0}, k7c1[] = {2, 9, 16, 0};
    const int* built = k == 5 ? (channels == 3 ? k5c3 : k5c1) : (channels == 3 ? k7c3 : k7c1);
    for (; *built; ++built)
        if (*built >= need) return *built;
    return 0;
}

// An image's coefficients beyond 4 GB: byte offsets no longer fit 32 bits.  Instantiations
// with element offsets exist for 5x5 atoms, three channels, fp16 or bfloat16 coefficients (an 8K frame
// with 72 planes), in capacities 1, 4 and 9.
unsigned long long coeff_bytes(int coeff_dtype) {
    return coeff_dtype == SR_F32 ? 4ull : (coeff_dtype == SR_F8E4M3 ? 1ull : 2ull);
}
bool beyond_4gb(const AssembleArgs& a, int coeff_dtype) {
    return (unsigned long long)a.L * a.H * a.W * coeff_bytes(coeff_dtype) >= (1ull << 32);
}
int np8_big(int np8) { return np8 <= 1 ? 1 : (np8 <= 4 ? 4 : (np8 <= 9 ? 9 : 0)); }   // 0: none built

}  // namespace

static bool has_tile_shapes(const AssembleArgs& a, int k, int np8, int coeff_dtype) {
    return k == 5 && a.C == 3 && np8 == 9 && coeff_dtype == SR_F16 && !beyond_4gb(a, coeff_dtype);
}

// Tile of the instantiation that serves the call, where the library can say (the family with
// alternative shapes); false elsewhere.
bool mfma_tile_shape(const AssembleArgs& a, int k, int coeff_dtype, int tile, int* tw, int* th, int* waves, int* groups) {
    const int np8 = np8_for(k, a.C, a.n_fold, coeff_dtype);
    return !a.logits && !a.blocked && has_tile_shapes(a, k, np8, coeff_dtype) && tile_shape_k5(a, tile, tw, th, waves, groups);
}

// pixels a lane loads with one vector load (its pixel group)
static int pixel_group(int k, int coeff_dtype) {
    return coeff_dtype == SR_F8E4M3 ? 4 : ((k != 7 && coeff_dtype != SR_F32) ? 4 : 2);
}

bool mfma_supported(const AssembleArgs& a, int k, int coeff_dtype, int tile) {
    if ((k != 3 && k != 5 && k != 7) || a.C < 1 || a.C > 4) return false;
    // A lane loads one pixel group of a row and stores half a group per channel.  Rows
    // need not keep the groups' alignment (gfx950 global loads and stores take any
    // element-aligned address); a width that is not a whole number of groups needs
    // at least one full tile (128 columns), see tile_x0 in the kernel.
    const int px = pixel_group(k, coeff_dtype);
    if (a.W < px || a.H < 1 || (a.W % px != 0 && a.W < 128)) return false;
    // the fp8 instantiations read the LR image as aligned 32-bit words: the image must start on one and,
    // when it is fp16, end on one
    if (coeff_dtype == SR_F8E4M3 &&
        (((uintptr_t)a.lr % 4) != 0 || (a.io_f16 && (((unsigned long long)a.N * a.C * a.h * a.w) & 1ull)))) return false;
    if (beyond_4gb(a, coeff_dtype) &&                                                      // 32-bit plane offsets
        !(k == 5 && a.C == 3 && (coeff_dtype == SR_F16 || coeff_dtype == SR_BF16) &&
          (unsigned long long)a.L * a.H * a.W < (1ull << 32)))
        return false;
    if ((unsigned long long)a.C * a.H * a.W * 4ull >= (1ull << 32)) return false;          // 32-bit offsets within an image
    const int np8 = np8_for(k, a.C, a.n_fold, coeff_dtype);
    if (np8 == 0) return false;
    // coefficients in the layout before the network's pixel-shuffle: one family built
    // coefficients stored pixel-major: one family built (all of 72 fp16 atoms in their own order, whole 128-pixel units)
    if (a.pixel_major) {
        if (a.pre_shuffle || !(k == 5 && a.C == 3 && coeff_dtype == SR_F16 && a.L == 72 && a.n_fold == 72 &&
                               !beyond_4gb(a, coeff_dtype) && a.W % 128 == 0 && tile == 0)) return false;
        for (int i = 0; i < 72; ++i)
            if (a.kept[i] != i) return false;
    }
    // coefficients stored blocked: one family built (all of 72 fp16, bfloat16 or 8-bit atoms; fp16 logits)
    if (a.blocked) {
        if (a.pre_shuffle || a.pixel_major || (a.logits && coeff_dtype != SR_F16) ||
            !(k == 5 && a.C == 3 && (coeff_dtype == SR_F16 || coeff_dtype == SR_BF16 || coeff_dtype == SR_F8E4M3) && a.L == 72 && a.n_fold == 72 &&
              !beyond_4gb(a, coeff_dtype) && a.W % 128 == 0 && tile == 0)) return false;
        for (int i = 0; i < 72; ++i)
            if (a.kept[i] != i) return false;
    }
    // logits instead of coefficients: one family built (5x5, three channels, 49 to 72 fp16 or bfloat16 planes)
    // (in the layout before the pixel-shuffle: its permuted-slot forms, LR widths that are multiples of 4)
    if (a.logits && !a.blocked && !(k == 5 && a.C == 3 && (coeff_dtype == SR_F16 || coeff_dtype == SR_BF16) && np8 == 9 && a.n_fold == a.L && !a.pixel_major &&
                      (!a.pre_shuffle || a.w % 4 == 0) && !beyond_4gb(a, coeff_dtype) && tile == 0))
        return false;
    // (bfloat16: the forms with permuted pixel slots only, i.e. LR widths that are multiples of 4, all atoms)
    if (a.pre_shuffle && !(k == 5 && a.C == 3 && (np8 == 1 || np8 == 9) && !beyond_4gb(a, coeff_dtype) && a.W % px == 0 &&
                           tile == 0 && (coeff_dtype == SR_F16 || (coeff_dtype == SR_BF16 && np8 == 9 && a.w % 4 == 0))))
        return false;
    if (beyond_4gb(a, coeff_dtype) && np8_big(np8) == 0) return false;                     // element offsets: up to 72 atoms
    // Alternative tile shapes exist for one family only (5x5 atoms, three channels, 65 to 72 fp16
    // atoms, byte offsets); everywhere else only the default (index 0) is accepted, so that a
    // sweep over the indices never times one kernel under several names.
    if (tile < 0) return false;
    if (tile != 0) {
        int tw, th;
        if (!has_tile_shapes(a, k, np8, coeff_dtype) || !tile_shape_k5(a, tile, &tw, &th, nullptr, nullptr)) return false;
    }
    return true;
}

hipError_t launch_mfma(const AssembleArgs& a, int k, bool io_f16, int tile, hipStream_t st) {
    (void)io_f16;
    const int np8 = np8_for(k, a.C, a.n_fold, a.coeff_dtype);
    if (a.blocked) return launch_mfma_k5_blk(a, st);
    if (a.logits) return launch_mfma_k5_lg(a, st);
    if (a.pixel_major) return launch_mfma_k5_pm(a, st);
    if (a.pre_shuffle) return launch_mfma_k5_ps(a, np8, st);
    if (beyond_4gb(a, a.coeff_dtype))
        return np8_big(np8) ? launch_mfma_k5_big(a, np8_big(np8), st) : hipErrorInvalidValue;
    if (a.coeff_dtype == SR_BF16 && k != 3) return launch_mfma_bf16(a, k, np8, st);
    if (k == 3) return launch_mfma_k3(a, np8, st);
    if (a.coeff_dtype == SR_F32) return k == 5 ? launch_mfma_k5_f32(a, np8, st) : launch_mfma_k7_f32(a, np8, st);
    if (a.coeff_dtype == SR_F8E4M3) return k == 5 ? launch_mfma_k5_f8(a, np8, st) : launch_mfma_k7_f8(a, np8, st);
    if (k == 5) return launch_mfma_k5(a, np8, tile, st);
    if (k == 7) return launch_mfma_k7(a, np8, tile, st);
    return hipErrorInvalidValue;
}

}  // namespace srd
