// Host-side launch entry points of the individual kernel families.
#pragma once
#include <hip/hip_runtime.h>
#include "sr_device.h"

namespace srd {

hipError_t launch_generic(const AssembleArgs& a, int k, bool io_f16, hipStream_t st);   // coefficient dtype: a.coeff_dtype
hipError_t launch_bicubic(const BicubicArgs& a, bool in_f16, bool out_f16, hipStream_t st);

// Matrix-core kernel.  mfma_supported() is a pure host-side predicate.
bool mfma_supported(const AssembleArgs& a, int k, int coeff_dtype, int tile);
hipError_t launch_mfma(const AssembleArgs& a, int k, bool io_f16, int tile, hipStream_t st);
// Per-pixel list form (sr_dict_assemble_list) on the matrix cores: a.coeff = values, a.index, a.T set; kept = identity.
bool mfma_list_supported(const AssembleArgs& a, int k, bool value_f16);
hipError_t launch_mfma_list(const AssembleArgs& a, hipStream_t st);
bool mfma_tile_shape(const AssembleArgs& a, int k, int coeff_dtype, int tile, int* tw, int* th, int* waves = nullptr,
                     int* groups = nullptr);

}  // namespace srd
