// Instantiations of the split-unit kernel for head dimension 64.
#include "zp_split.h"

namespace zp {
hipError_t launch_split_d64(const Args &a, int units, int NW, int RB, hipStream_t s) { return launch_d<64>(a, units, NW, RB, s); }
}  // namespace zp
