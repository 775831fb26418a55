// Instantiations of the matrix-core unit kernel for head dimension 128, up to four waves per workgroup.
#include "zp_mfma.h"

namespace zp {
hipError_t launch_mfma_d128(const Args &a, int units, int NW, int RB, hipStream_t s) { return launch_d<128, 0>(a, units, NW, RB, s); }
}  // namespace zp
