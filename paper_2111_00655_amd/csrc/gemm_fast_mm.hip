// Instantiations of the tuned GEMM kernel for plain matrix products: dense
// (x W^T), batched matmul in both operand orientations, 1x1 stride-1
// convolution (a GEMM per image).
#include "gemm_fast.h"

namespace clg {

int launch_fast_mm(const GemmArgs &a, bool vec, hipStream_t s) {
    if (a.mode == GM_NT)
        return vec ? launch_fast<F_NT, 0, 0, true>(a, s) : launch_fast<F_NT, 0, 0, false>(a, s);
    return vec ? launch_fast<F_NN, 0, 0, true>(a, s) : launch_fast<F_NN, 0, 0, false>(a, s);
}

}  // namespace clg
