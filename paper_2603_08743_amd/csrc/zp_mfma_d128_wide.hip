// Instantiations of the matrix-core unit kernel for head dimension 128, eight waves per workgroup.
#include "zp_mfma.h"

namespace zp {
hipError_t launch_mfma_d128_wide(const Args &a, int units, int NW, int RB, hipStream_t s) { return launch_d<128, 1>(a, units, NW, RB, s); }
}  // namespace zp
