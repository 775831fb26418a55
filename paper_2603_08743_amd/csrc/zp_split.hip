// Split-unit path of libzp: dispatch, the word-clearing kernel and the instantiations for head dimension 128
// (those for 64 live in zp_split_d64.hip so that the two compile in parallel).
#include "zp_split.h"

namespace zp {

__global__ void zero_words(int *p, int n) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0;
}

hipError_t launch_zero_words(int *p, int n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    int blocks = (n + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(zero_words, dim3(blocks), dim3(256), 0, s, p, n);
    return hipGetLastError();
}

hipError_t launch_split_d128(const Args &a, int units, int NW, int RB, hipStream_t s) { return launch_d<128>(a, units, NW, RB, s); }

hipError_t launch_unit_split(const Args &a, int units, int NW, int RB, hipStream_t s) {
    if (units <= 0) return hipSuccess;
    if (a.d == 128) return launch_split_d128(a, units, NW, RB, s);
    if (a.d == 64) return launch_split_d64(a, units, NW, RB, s);
    return hipErrorInvalidConfiguration;
}

}  // namespace zp
