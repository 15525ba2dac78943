// Instantiations and dispatch of the lean 3x3 convolution kernel.
#include <algorithm>

#include "gemm_lean.h"

namespace clg {

namespace {

template <int S, int WGK, int NP>
int launch_c3(GemmArgs a, hipStream_t s) {
    using T = Conv3Cfg<S, WGK, NP>;
    const int npix = a.HO * a.WO;
    const int tiles = ((a.Cout + 31) / 32) * ((npix + 31) / 32);
    const size_t lds = (size_t)(T::SMEM_A + T::CS * a.patch_sz) * sizeof(float);
    hipLaunchKernelGGL((conv3x3_lean_kernel<S, WGK, NP>), dim3(tiles, a.Nimg, a.splitk), dim3(T::NT), lds, s, a);
    return (int)hipGetLastError();
}

template <int S>
int launch_c3_stride(GemmArgs a, hipStream_t s) {
    const bool want8 = (a.tile == TILE_S8 || a.tile == TILE_S16) && a.Cin % 32 == 0;
    if (want8 && a.patch_sz <= 512) return launch_c3<S, 8, 1>(a, s);
    if (a.Cin % 16) return -1;
    if (a.patch_sz <= 256) return launch_c3<S, 4, 1>(a, s);
    if (a.patch_sz <= 512) return launch_c3<S, 4, 2>(a, s);
    return -1;
}

}  // namespace

int launch_lean_conv3x3(const GemmArgs &a_in, hipStream_t s) {
    GemmArgs a = a_in;
    if (a.mode != GM_CONV || a.KH != 3 || a.KW != 3 || a.sh != a.sw || (a.sh != 1 && a.sh != 2)) return -1;
    if (a.tile == TILE_M || a.tile == TILE_L) return -1;
    if (((uintptr_t)a.A & 15) || a.Cin % 16) return -1;
    // 32 consecutive output pixels span at most this many output rows
    const int rows = std::min(a.HO, (30 + a.WO) / a.WO + 1);
    a.patch_sz = ((rows - 1) * a.sh + 3) * (a.W + 2 * a.pw);
    return a.sh == 1 ? launch_c3_stride<1>(a, s) : launch_c3_stride<2>(a, s);
}

}  // namespace clg
