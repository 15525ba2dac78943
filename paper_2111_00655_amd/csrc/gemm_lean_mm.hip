// Instantiations and dispatch of the lean matrix-product kernel.
#include "gemm_lean.h"

namespace clg {

namespace {

bool al16(const void *p) { return ((uintptr_t)p & 15) == 0; }

template <int MODE, class T>
int launch_mm_tile(const GemmArgs &a, hipStream_t s) {
    const int tiles = ((a.M + T::BM - 1) / T::BM) * ((a.N + T::BN - 1) / T::BN);
    hipLaunchKernelGGL((mm_lean_kernel<MODE, T>), dim3(tiles, a.batch, a.splitk), dim3(T::NT),
                       T::SMEM * sizeof(float), s, a);
    return (int)hipGetLastError();
}

template <int MODE>
int launch_mm_mode(const GemmArgs &a, hipStream_t s) {
    switch (a.tile) {
    case TILE_S16:
        if (a.K % 128 == 0) return launch_mm_tile<MODE, LTileS16>(a, s);
        [[fallthrough]];
    case TILE_S8:
        if (a.K % 128 == 0) return launch_mm_tile<MODE, LTileS8>(a, s);
        [[fallthrough]];
    case TILE_S:
        return a.K % 64 == 0 ? launch_mm_tile<MODE, LTileS>(a, s) : -1;
    case TILE_L:
        return a.K % 32 == 0 ? launch_mm_tile<MODE, LTileL>(a, s) : -1;
    default:
        return a.K % 64 == 0 ? launch_mm_tile<MODE, LTileM>(a, s) : -1;
    }
}

}  // namespace

bool lean_mm_shape_ok(const GemmArgs &a, int epi_flags) {
    if (epi_flags & EF_GENERIC) return false;
    if (a.lda % 4 || a.ldb % 4 || a.strideA % 4 || a.strideB % 4) return false;
    if (a.mode == GM_NN && (a.N % 4 != 0 || a.N < 4)) return false;
    if (a.mode != GM_NT && a.mode != GM_NN) return false;
    switch (a.tile) {
    case TILE_S16: case TILE_S8: case TILE_S: return a.K % 64 == 0;
    case TILE_L: return a.K % 32 == 0;
    default: return a.K % 64 == 0;
    }
}

int launch_lean_mm(const GemmArgs &a, hipStream_t s) {
    if (a.ef.flags & EF_GENERIC) return -1;
    if (a.lda % 4 || a.ldb % 4 || a.strideA % 4 || a.strideB % 4 || !al16(a.A) || !al16(a.B)) return -1;
    if (a.mode == GM_NT) return launch_mm_mode<F_NT>(a, s);
    if (a.mode == GM_NN && a.N % 4 == 0 && a.N >= 4) return launch_mm_mode<F_NN>(a, s);
    return -1;
}

}  // namespace clg
