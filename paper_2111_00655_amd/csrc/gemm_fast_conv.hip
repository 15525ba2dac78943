// Instantiations of the tuned implicit-GEMM convolution kernel: the im2col
// index (channel, tap) is decomposed with compile-time kernel sizes for the
// shapes of the workloads (3x3, strided 1x1, the 7x7 stem), with a run-time
// fallback for any other kernel of at most 64 taps.
#include "gemm_fast.h"

namespace clg {

int launch_fast_conv(const GemmArgs &a, bool vec, hipStream_t s) {
    if (a.KH == 3 && a.KW == 3)
        return vec ? launch_fast<F_CONV, 3, 3, true>(a, s) : launch_fast<F_CONV, 3, 3, false>(a, s);
    if (a.KH == 1 && a.KW == 1)
        return vec ? launch_fast<F_CONV, 1, 1, true>(a, s) : launch_fast<F_CONV, 1, 1, false>(a, s);
    if (a.KH == 7 && a.KW == 7) return launch_fast<F_CONV, 7, 7, false>(a, s);
    return launch_fast<F_CONV, 0, 0, false>(a, s);
}

}  // namespace clg
