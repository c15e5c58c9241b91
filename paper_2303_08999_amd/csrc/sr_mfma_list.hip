// Matrix-core kernel instantiations for coefficients given as per-pixel lists (CT_LIST8 / CT_LIST16 in
// sr_mfma_kernel.h; an extension beyond the paper, see sr_dict_assemble_list): 5x5 atoms, three
// channels, fp16 values, up to 72 or up to 128 atoms in the dictionary, up to 8 or up to 16 entries per pixel.
#include "sr_mfma_kernel.h"

namespace srd {

bool mfma_list_supported(const AssembleArgs& a, int k, bool value_f16) {
    if (k != 5 || a.C != 3 || !value_f16 || a.L > 128 || a.T < 1 || a.T > LIST_MAX_ENTRIES) return false;
    if (a.W < 4 || a.W % 4 != 0 || a.H < 1) return false;
    if ((unsigned long long)a.T * a.H * a.W >= (1ull << 32)) return false;             // 32-bit element offsets within an image
    if ((unsigned long long)a.C * a.H * a.W * 4ull >= (1ull << 32)) return false;
    return true;
}

// Up to 72 atoms: the dense form's operand steps (four of 16 atoms and one of 8) and its tiles; up to 128: eight
// steps, 128 x 8 tiles at every scale (35 KB of scatter scratch).  Lists of up to 8 entries keep half the registers.
template <int CT>
static hipError_t launch_ct(const AssembleArgs& a, hipStream_t st) {
    if (a.L <= 72) {
        if (a.s == 4) return launch_one<5, 3, 9, 4, 1, 4, 4, 2, CT, 4>(a, st);
        return launch_one<5, 3, 9, 4, 1, 4, 2, 2, CT, 2>(a, st);
    }
    return launch_one<5, 3, 16, 4, 1, 4, 2, 2, CT, 2>(a, st);
}

hipError_t launch_mfma_list(const AssembleArgs& a, hipStream_t st) {
    return a.T <= 8 ? launch_ct<CT_LIST8>(a, st) : launch_ct<CT_LIST16>(a, st);
}

}  // namespace srd
