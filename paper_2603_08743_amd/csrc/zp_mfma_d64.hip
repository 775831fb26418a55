// Instantiations of the matrix-core unit kernel for head dimension 64, up to four waves per workgroup.
#include "zp_mfma.h"

namespace zp {
hipError_t launch_mfma_d64(const Args &a, int units, int NW, int RB, hipStream_t s) { return launch_d<64, 0>(a, units, NW, RB, s); }
}  // namespace zp
