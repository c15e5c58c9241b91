// placeholder until the matrix-core kernel lands
#include "sr_launch.h"
namespace srd {
bool mfma_supported(const AssembleArgs&, int, bool, int) { return false; }
hipError_t launch_mfma(const AssembleArgs&, int, bool, int, hipStream_t) { return hipErrorNotSupported; }
}
