// Instantiations, planning and dispatch of the register-fed convolution kernels.
#include <algorithm>

#include "gemm_rf.h"

namespace clg {

namespace {

int dense_tiles(const GemmArgs &a);

template <int TS, int TAPK, int WGK, int GEO>
int launch_rf_one_t(const GemmArgs &a, hipStream_t s) {
    const int npix = a.rf_d2s ? a.H * a.W : (a.rf_convt ? (a.HO / a.sh) * (a.WO / a.sw) : a.HO * a.WO);
    const int tiles = (((a.rf_d2s ? 4 * a.Cout : a.Cout) + TS - 1) / TS) * ((npix + TS - 1) / TS);
    const size_t lds = WGK > 1 ? (size_t)WGK * RfMfma<TS>::NACC * kWave * sizeof(float) : 0;
    const int gz = a.rf_convt ? a.sh * a.sw : a.splitk;      // sub-pixel phases, or K splits
    const int gy = a.Nimg * (a.DO > 1 ? a.DO : 1);           // images, or (image, output depth) pairs
    if (gy > 65535) return (int)hipErrorInvalidValue;
    constexpr int DEEP = rf_depth<TAPK, WGK>();
    if (DEEP > 1 && a.rf_nch > 1)
        hipLaunchKernelGGL((conv_rf_kernel<TS, TAPK, WGK, GEO, DEEP>), dim3(tiles, gy, gz), dim3(WGK * kWave), lds, s, a);
    else
        hipLaunchKernelGGL((conv_rf_kernel<TS, TAPK, WGK, GEO, 1>), dim3(tiles, gy, gz), dim3(WGK * kWave), lds, s, a);
    return (int)hipGetLastError();
}

// transposed convolutions run the 2x2 and the any-filter paths only, folded depth taps the 3x3 and the
// any-filter paths
template <int TS, int TAPK, int WGK>
int launch_rf_one(const GemmArgs &a, hipStream_t s) {
    if constexpr (TAPK == 4 || TAPK == 0) {
        if (a.rf_convt) return launch_rf_one_t<TS, TAPK, WGK, 1>(a, s);
    }
    if constexpr (TAPK == 9 || TAPK == 0) {
        if (a.rf_fold && !a.rf_convt) return launch_rf_one_t<TS, TAPK, WGK, 2>(a, s);
    }
    if constexpr (TAPK == 9 && TS == 16) {
        if (a.rf_d2s) return launch_rf_one_t<TS, TAPK, WGK, 5>(a, s);
    }
    if (a.rf_d2s) return (int)hipErrorInvalidValue;
    if (a.rf_convt || a.rf_fold) return (int)hipErrorInvalidValue;
    if constexpr (TAPK == 1) {
        if (a.rf_prelu && a.D <= 1) return launch_rf_one_t<TS, TAPK, WGK, 4>(a, s);
    }
    if (a.rf_prelu) return (int)hipErrorInvalidValue;        // only the 2-D 1x1 path clamps its input
    if constexpr (TAPK != 4) {
        if (a.D > 1) return launch_rf_one_t<TS, TAPK, WGK, 3>(a, s);
    }
    if (a.D > 1 || a.DO > 1) return (int)hipErrorInvalidValue;
    return launch_rf_one_t<TS, TAPK, WGK, 0>(a, s);
}

template <int TS, int TAPK>
int launch_rf_wgk(const GemmArgs &a, hipStream_t s) {
    switch (a.rf_wgk) {
    case 1: return launch_rf_one<TS, TAPK, 1>(a, s);
    case 2: return launch_rf_one<TS, TAPK, 2>(a, s);
    case 4: return launch_rf_one<TS, TAPK, 4>(a, s);
    case 8: return launch_rf_one<TS, TAPK, 8>(a, s);
    case 16: return launch_rf_one<TS, TAPK, 16>(a, s);
    default: return (int)hipErrorInvalidValue;
    }
}

template <int TS>
int launch_rf_tap(const GemmArgs &a, hipStream_t s) {
    switch (a.rf_tapk) {
    case 1: return launch_rf_wgk<TS, 1>(a, s);
    case 9: return launch_rf_wgk<TS, 9>(a, s);
    case 4: return launch_rf_wgk<TS, 4>(a, s);
    default: return launch_rf_wgk<TS, 0>(a, s);
    }
}

template <int WGK>
int launch_rfd2_one(const GemmArgs &a, hipStream_t s) {
    const size_t lds = (size_t)WGK * 2 * RfPark<16>::PERW * sizeof(float);      // at most 40 KB
    hipLaunchKernelGGL((dense_rf2_kernel<WGK>), dim3(dense_tiles(a), 1, 1), dim3(WGK * kWave), lds, s, a);
    return (int)hipGetLastError();
}

int launch_rfd2_wgk(const GemmArgs &a, hipStream_t s) {
    switch (a.rf_wgk) {
    case 1: return launch_rfd2_one<1>(a, s);
    case 2: return launch_rfd2_one<2>(a, s);
    case 4: return launch_rfd2_one<4>(a, s);
    case 8: return launch_rfd2_one<8>(a, s);
    case 16: return launch_rfd2_one<16>(a, s);
    default: return (int)hipErrorInvalidValue;
    }
}

template <int WGK>
int launch_rfd2_multi_t(const RfMultiArgs &m, hipStream_t s) {
    const size_t lds = (size_t)WGK * 2 * RfPark<16>::PERW * sizeof(float);
    hipLaunchKernelGGL((dense_rf2_multi_kernel<WGK>), dim3(m.tile_end[m.n - 1], 1, 1), dim3(WGK * kWave), lds, s, m);
    return (int)hipGetLastError();
}

int launch_rfd2_multi_wgk(const RfMultiArgs &m, int wgk, hipStream_t s) {
    switch (wgk) {
    case 1: return launch_rfd2_multi_t<1>(m, s);
    case 2: return launch_rfd2_multi_t<2>(m, s);
    case 4: return launch_rfd2_multi_t<4>(m, s);
    case 8: return launch_rfd2_multi_t<8>(m, s);
    case 16: return launch_rfd2_multi_t<16>(m, s);
    default: return (int)hipErrorInvalidValue;
    }
}

template <int TS, int WGK>
int launch_rfd_one(const GemmArgs &a, hipStream_t s) {
    const int tiles = ((a.N + TS - 1) / TS) * ((a.M + TS - 1) / TS);
    const size_t lds = (size_t)WGK * RfPark<TS>::PERW * sizeof(float);
    if (lds > 64 * 1024) {
        static bool raised = false;              // more than 64 KB of dynamic LDS has to be allowed per kernel, once
        if (!raised) {
            const hipError_t e = hipFuncSetAttribute((const void *)dense_rf_kernel<TS, WGK>,
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return (int)e;
            raised = true;
        }
    }
    hipLaunchKernelGGL((dense_rf_kernel<TS, WGK>), dim3(tiles, 1, a.splitk), dim3(WGK * kWave), lds, s, a);
    return (int)hipGetLastError();
}

template <int TS>
int launch_rfd_wgk(const GemmArgs &a, hipStream_t s) {
    switch (a.rf_wgk) {
    case 1: return launch_rfd_one<TS, 1>(a, s);
    case 2: return launch_rfd_one<TS, 2>(a, s);
    case 4: return launch_rfd_one<TS, 4>(a, s);
    case 8: return launch_rfd_one<TS, 8>(a, s);
    case 16: return launch_rfd_one<TS, 16>(a, s);
    default: return (int)hipErrorInvalidValue;
    }
}

// geometry variant of the convolution kernel that runs `a` (its fourth template argument)
int rf_geo(const GemmArgs &a) {
    if (a.rf_convt) return 1;
    if (a.rf_d2s) return 5;
    if (a.rf_fold) return 2;
    if (a.rf_prelu) return 4;
    return a.D > 1 ? 3 : 0;
}

int conv_tiles(const GemmArgs &a) {
    const int npix = a.rf_convt ? (a.HO / a.sh) * (a.WO / a.sw) : a.HO * a.WO;
    return ((a.Cout + a.rf_ts - 1) / a.rf_ts) * ((npix + a.rf_ts - 1) / a.rf_ts);
}

int dense_tiles(const GemmArgs &a) {
    const int wt = (a.N + a.rf_ts - 1) / a.rf_ts;            // weight-row tiles; a wave may own two of them
    return (a.rf_nb == 2 ? (wt + 1) / 2 : wt) * ((a.M + a.rf_ts - 1) / a.rf_ts);
}

template <int TS, int WGK, int GEO>
int launch_rf_multi_t(const RfMultiArgs &m, int gy, hipStream_t s) {
    const size_t lds = WGK > 1 ? (size_t)WGK * RfMfma<TS>::NACC * kWave * sizeof(float) : 0;
    hipLaunchKernelGGL((conv_rf_multi_kernel<TS, WGK, GEO>), dim3(m.tile_end[m.n - 1], gy, 1), dim3(WGK * kWave), lds, s, m);
    return (int)hipGetLastError();
}

template <int TS, int WGK>
int launch_rf_multi_geo(const RfMultiArgs &m, int geo, int gy, hipStream_t s) {
    switch (geo) {
    case 0: return launch_rf_multi_t<TS, WGK, 0>(m, gy, s);
    case 3: return launch_rf_multi_t<TS, WGK, 3>(m, gy, s);
    case 4: return launch_rf_multi_t<TS, WGK, 4>(m, gy, s);
    default: return (int)hipErrorInvalidValue;
    }
}

template <int TS>
int launch_rf_multi_wgk(const RfMultiArgs &m, int wgk, int geo, int gy, hipStream_t s) {
    switch (wgk) {
    case 1: return launch_rf_multi_geo<TS, 1>(m, geo, gy, s);
    case 2: return launch_rf_multi_geo<TS, 2>(m, geo, gy, s);
    case 4: return launch_rf_multi_geo<TS, 4>(m, geo, gy, s);
    case 8: return launch_rf_multi_geo<TS, 8>(m, geo, gy, s);
    case 16: return launch_rf_multi_geo<TS, 16>(m, geo, gy, s);
    default: return (int)hipErrorInvalidValue;
    }
}

template <int TS, int WGK>
int launch_rfd_multi_t(const RfMultiArgs &m, hipStream_t s) {
    const size_t lds = (size_t)WGK * RfPark<TS>::PERW * sizeof(float);
    if (lds > 64 * 1024) {
        static bool raised = false;
        if (!raised) {
            const hipError_t e = hipFuncSetAttribute((const void *)dense_rf_multi_kernel<TS, WGK>,
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return (int)e;
            raised = true;
        }
    }
    hipLaunchKernelGGL((dense_rf_multi_kernel<TS, WGK>), dim3(m.tile_end[m.n - 1], 1, 1), dim3(WGK * kWave), lds, s, m);
    return (int)hipGetLastError();
}

template <int TS>
int launch_rfd_multi_wgk(const RfMultiArgs &m, int wgk, hipStream_t s) {
    switch (wgk) {
    case 1: return launch_rfd_multi_t<TS, 1>(m, s);
    case 2: return launch_rfd_multi_t<TS, 2>(m, s);
    case 4: return launch_rfd_multi_t<TS, 4>(m, s);
    case 8: return launch_rfd_multi_t<TS, 8>(m, s);
    case 16: return launch_rfd_multi_t<TS, 16>(m, s);
    default: return (int)hipErrorInvalidValue;
    }
}

// K-waves per workgroup: enough to give every wave one chunk.  With `cap_grid`
// (dense, and the per-MFMA tap path, whose chunks are short) no more than keeps
// the whole grid at about four waves per SIMD (1024 SIMDs): a tile whose K is
// cut into many short pieces pays the fixed cost of a wave once per piece.  The
// 1x1 / 3x3 convolution paths measured best with one chunk per wave throughout.
int pick_waves(int chunks, int64_t tiles, int forced, bool cap_grid) {
    if (forced == 1 || forced == 2 || forced == 4 || forced == 8 || forced == 16) return forced;
    int wgk = 1;
    while (wgk < 16 && wgk < chunks) wgk *= 2;
    // a negative count is an upper bound: waves with several chunks each keep all their loads in flight
    // (a kernel variant of its own for the placement search to price)
    if (forced == -1 || forced == -2 || forced == -4 || forced == -8 || forced == -16) return wgk < -forced ? wgk : -forced;
    if (!cap_grid) return wgk;
    int cap = 1;
    while (cap < 16 && (int64_t)cap * 2 * tiles <= 4096) cap *= 2;
    return wgk < cap ? wgk : cap;
}

// Tile order: tile = hi * div + lo with lo running over the m-tiles (j-major) or the n-tiles.
bool set_tile_order(GemmArgs *a, int tiles_m, int tiles_n) {
    a->rf_tile_div = a->rf_jmajor ? tiles_m : tiles_n;
    a->rf_tile_magic = (((uint64_t)1 << 32) / (uint64_t)a->rf_tile_div) + 1;
    return (int64_t)tiles_m * tiles_n * a->rf_tile_div < ((int64_t)1 << 32);      // range in which the multiply-high is exact
}

int chunk_mfmas(int tapk) { return tapk == 1 || tapk == 4 ? 16 : (tapk == 9 ? 36 : 4); }
int chunk_groups(int tapk) { return tapk == 1 || tapk == 4 ? 4 : (tapk == 9 ? 9 : 1); }

}  // namespace

#ifdef CLG_RF_STAMPS
void rf_set_stamps(long long *dev) { (void)hipMemcpyToSymbol(HIP_SYMBOL(g_rf_stamps), &dev, sizeof(dev)); }
#endif

int launch_rf_conv(const GemmArgs &a, hipStream_t s) {
    if (a.rf_tapk == -1) {
        if (((uintptr_t)a.A & 15) != 0) return (int)hipErrorInvalidValue;      // activations are read 16 bytes at a time
        if (a.rf_nb == 2) return a.rf_ts == 16 && a.splitk == 1 ? launch_rfd2_wgk(a, s) : (int)hipErrorInvalidValue;
        return a.rf_ts == 32 ? launch_rfd_wgk<32>(a, s) : launch_rfd_wgk<16>(a, s);
    }
    return a.rf_ts == 32 ? launch_rf_tap<32>(a, s) : launch_rf_tap<16>(a, s);
}

bool rf_same_launch_shape(const GemmArgs &a, const GemmArgs &b) {
    if (!a.rf_ts || a.rf_ts != b.rf_ts || a.rf_tapk != b.rf_tapk || a.rf_wgk != b.rf_wgk) return false;
    if (a.splitk != 1 || b.splitk != 1) return false;
    if (a.rf_tapk == -1) return a.rf_nb == b.rf_nb;           // dense: grid.y = grid.z = 1
    if (a.rf_tapk != 1) return false;                         // of the convolutions the 1x1 path is built as a region kernel
    const int ga = rf_geo(a), gb = rf_geo(b);
    if (ga != gb || (ga != 0 && ga != 3 && ga != 4)) return false;
    return a.Nimg * (a.DO > 1 ? a.DO : 1) == b.Nimg * (b.DO > 1 ? b.DO : 1);
}

int launch_rf_multi(const GemmArgs *members, int n, hipStream_t s) {
    if (n < 2 || n > kMaxRegion) return (int)hipErrorInvalidValue;
    RfMultiArgs m{};
    m.n = n;
    const GemmArgs &a = members[0];
    const bool dense = a.rf_tapk == -1;
    int end = 0;
    for (int k = 0; k < n; ++k) {
        if (k && !rf_same_launch_shape(a, members[k])) return (int)hipErrorInvalidValue;
        if (dense && ((uintptr_t)members[k].A & 15) != 0) return (int)hipErrorInvalidValue;
        end += dense ? dense_tiles(members[k]) : conv_tiles(members[k]);
        m.tile_end[k] = end;
        m.p[k] = members[k];
    }
    for (int k = n; k < kMaxRegion; ++k) m.tile_end[k] = end;
    if (dense && a.rf_nb == 2) return launch_rfd2_multi_wgk(m, a.rf_wgk, s);
    if (dense) return a.rf_ts == 32 ? launch_rfd_multi_wgk<32>(m, a.rf_wgk, s) : launch_rfd_multi_wgk<16>(m, a.rf_wgk, s);
    const int gy = a.Nimg * (a.DO > 1 ? a.DO : 1);
    if (gy > 65535) return (int)hipErrorInvalidValue;
    return a.rf_ts == 32 ? launch_rf_multi_wgk<32>(m, a.rf_wgk, rf_geo(a), gy, s)
                         : launch_rf_multi_wgk<16>(m, a.rf_wgk, rf_geo(a), gy, s);
}

bool rf_resolve_dense(GemmArgs *a, int ts, int epi_flags, int n_cus, int waves, int nb) {
    (void)n_cus;
    if (a->mode != GM_NT || a->batch != 1 || (epi_flags & EF_GENERIC)) return false;
    if (nb != 1 && !(nb == 2 && ts == 16)) return false;
    const int nslot = ts == 32 ? 2 : 4;
    if (a->K % (4 * nslot) || a->lda % 4) return false;
    if ((int64_t)a->M * a->lda >= ((int64_t)1 << 31)) return false;     // 32-bit lane offsets
    if (a->cs_len && a->cs_len % ts) return false;           // a tile's columns must stay within one block of the split
    const int ng = a->K / (4 * nslot);                       // weight groups (4 MFMAs each)
    const int nc = (ng + 3) / 4;                             // chunks per tile
    const int wtiles = nb == 2 ? ((a->N + ts - 1) / ts + 1) / 2 : (a->N + ts - 1) / ts;      // tiles (or pairs of tiles) of weight rows
    const int wgk = pick_waves(nc, (int64_t)((a->M + ts - 1) / ts) * wtiles, waves, true);
    a->rf_ts = ts;
    a->rf_nb = nb;
    a->rf_tapk = -1;
    a->rf_wgk = wgk;
    a->rf_nch = (nc + wgk - 1) / wgk;
    a->splitk = 1;
    a->rf_ngtot = wgk * a->splitk * a->rf_nch * 4;
    a->rf_nm = ng * 4;
    a->rf_jmajor = a->M > a->N ? 1 : 0;
    if (set_tile_order(a, wtiles, (a->M + ts - 1) / ts)) return true;
    a->rf_ts = 0;
    a->rf_nb = 0;
    return false;
}

bool rf_resolve(GemmArgs *a, int ts, int epi_flags, int n_cus, int waves, bool split) {
    (void)n_cus;
    if (a->mode != GM_CONV || (epi_flags & EF_GENERIC)) return false;
    const int nslot = ts == 32 ? 2 : 4;
    const int64_t npix = (int64_t)a->HO * a->WO;
    if (npix * a->WO >= ((int64_t)1 << 32)) return false;             // multiply-high division range
    // depth geometry: a 2-D convolution has depth 1 everywhere; with KD > 1 the depth taps are folded into
    // the channel index, and Cin counts folded channels (the weights [Cout][Cin][KD][KH*KW] are then
    // [Cout][Cin * KD][KH*KW] as they lie)
    if (a->D < 1) { a->D = 1; a->KD = 1; a->sd = 1; a->pd = 0; a->DO = 1; }
    const int cin_real = a->Cin;
    a->rf_fold = a->KD > 1 ? 1 : 0;
    a->rf_cs = a->D * a->H * a->W;
    a->rf_img_stride = (int64_t)cin_real * a->rf_cs;
    a->rf_kd_magic = (((uint64_t)1 << 32) / (uint64_t)a->KD) + 1;
    if (a->rf_img_stride >= ((int64_t)1 << 30)) return false;         // 32-bit lane offsets
    if (!a->rf_fold && a->pd != 0) return false;                      // a single depth tap must lie inside
    const int groups = a->rf_groups > 1 ? a->rf_groups : 1;
    if ((a->rf_fold || a->D > 1) && groups > 1) return false;      // the depth variants take ungrouped convolutions
    a->Cin = cin_real * a->KD;
    const int taps = a->KH * a->KW;
    // grouped: an m-tile contracts the channels of the groups its rows belong to
    int cin_tile = a->Cin;
    if (groups > 1) {
        if (a->Cin % groups || a->Cout % groups) return false;
        const int cpg_in = a->Cin / groups, cpg_out = a->Cout / groups;
        if (ts % cpg_out != 0 && cpg_out % ts != 0) return false;
        cin_tile = (ts > cpg_out ? ts / cpg_out : 1) * cpg_in;
        a->rf_cpg_in = cpg_in;
        a->rf_cpg_out = cpg_out;
    }
    a->rf_groups = groups;
    a->rf_cin_tile = cin_tile;
    const int ncq = (cin_tile + nslot - 1) / nslot;
    int tapk = 0;
    if (cin_tile % nslot == 0 && (groups == 1 || a->rf_cpg_in % nslot == 0)) {
        if (taps == 1 && a->ph == 0 && a->pw == 0 && !a->rf_fold) tapk = 1;
        else if (a->KH == 3 && a->KW == 3) tapk = 9;
    }
    const int nm = ncq * taps;
    const int nc = (nm + chunk_mfmas(tapk) - 1) / chunk_mfmas(tapk);   // chunks per tile
    const int wgk = pick_waves(nc, (int64_t)((a->Cout + ts - 1) / ts) * ((npix + ts - 1) / ts) * a->Nimg * a->DO, waves, tapk == 0);
    a->rf_ts = ts;
    a->rf_tapk = tapk;
    a->rf_wgk = wgk;
    // K split across workgroups (grid.z) for a long reduction over few output tiles: partial tiles go to scratch
    // memory in slice order and a second kernel adds them and applies the tail.  As long as the grid stays within
    // two workgroups per compute unit and every wave keeps a whole chunk.
    int splitk = 1;
    if (split && groups == 1) {
        const int64_t wgs = (int64_t)((a->Cout + ts - 1) / ts) * ((npix + ts - 1) / ts) * a->Nimg * a->DO;
        while (splitk < 16 && wgs * splitk * 2 <= 512 && wgk * splitk * 2 <= nc) splitk *= 2;
    }
    a->rf_nch = (nc + wgk * splitk - 1) / (wgk * splitk);
    a->splitk = splitk;
    a->rf_ngtot = wgk * a->splitk * a->rf_nch * chunk_groups(tapk);
    a->rf_nm = nm;
    a->rf_jmajor = (int64_t)a->Cin * a->H * a->W > (int64_t)a->Cout * a->K ? 1 : 0;
    a->rf_wo_magic = (((uint64_t)1 << 32) / (uint64_t)a->WO) + 1;
    if (set_tile_order(a, (a->Cout + ts - 1) / ts, (int)((npix + ts - 1) / ts))) return true;
    a->rf_ts = 0;
    a->rf_convt = 0;
    a->rf_fold = 0;
    a->splitk = 1;
    a->Cin = cin_real;
    return false;
}

bool rf_resolve_convt(GemmArgs *a, int ts, int epi_flags, int n_cus, int waves) {
    (void)n_cus;
    if (a->mode != GM_CONVT || (epi_flags & EF_GENERIC)) return false;
    if (a->sh < 1 || a->sw < 1 || a->KH % a->sh || a->KW % a->sw || a->HO % a->sh || a->WO % a->sw) return false;
    const int khe = a->KH / a->sh, kwe = a->KW / a->sw, hoe = a->HO / a->sh, woe = a->WO / a->sw;
    // every phase's padding must be non-negative (it is for pad <= kernel / stride - 1 ... checked directly)
    for (int ph = 0; ph < a->sh; ++ph)
        if (khe - 1 - (ph + a->ph) / a->sh < 0) return false;
    for (int pw = 0; pw < a->sw; ++pw)
        if (kwe - 1 - (pw + a->pw) / a->sw < 0) return false;
    const int nslot = ts == 32 ? 2 : 4;
    if ((int64_t)a->Cin * a->H * a->W >= ((int64_t)1 << 30)) return false;
    // few output channels, 4x4 filter, stride 2, pad 1: the layer as one 3x3 convolution over the input whose rows are
    // (channel, phase)
    if (ts == 16 && a->KH == 4 && a->KW == 4 && a->sh == 2 && a->sw == 2 && a->ph == 1 && a->pw == 1 && 4 * a->Cout <= 16 &&
        a->Cin % nslot == 0 && a->HO == 2 * a->H && a->WO == 2 * a->W && (int64_t)a->H * a->W * a->W < ((int64_t)1 << 32)) {
        const int nm = (a->Cin / nslot) * 9;
        const int nc = (nm + 35) / 36;
        const int64_t tiles2 = (int64_t)(((int64_t)a->H * a->W + ts - 1) / ts) * a->Nimg;
        const int wgk = pick_waves(nc, tiles2, waves, false);
        a->rf_ts = ts;
        a->rf_tapk = 9;
        a->rf_wgk = wgk;
        a->rf_nch = (nc + wgk - 1) / wgk;
        a->splitk = 1;
        a->rf_ngtot = wgk * a->rf_nch * 9;
        a->rf_nm = nm;
        a->rf_groups = 1;
        a->rf_cin_tile = a->Cin;
        a->rf_convt = 0;
        a->rf_d2s = 1;
        a->D = a->KD = a->sd = a->DO = 1;
        a->pd = 0;
        a->rf_fold = 0;
        a->rf_cs = a->H * a->W;
        a->rf_img_stride = (int64_t)a->Cin * a->rf_cs;
        a->rf_kd_magic = 0;
        a->rf_jmajor = 1;
        a->rf_wo_magic = (((uint64_t)1 << 32) / (uint64_t)a->W) + 1;
        if (set_tile_order(a, 1, (int)(((int64_t)a->H * a->W + ts - 1) / ts))) return true;
        a->rf_ts = 0;
        a->rf_d2s = 0;
        return false;
    }
    const int64_t npix = (int64_t)hoe * woe;
    if (npix * woe >= ((int64_t)1 << 32)) return false;
    const int taps = khe * kwe;
    const int ncq = (a->Cin + nslot - 1) / nslot;
    const int tapk = (khe == 2 && kwe == 2 && a->Cin % nslot == 0) ? 4 : 0;
    const int nm = ncq * taps;
    const int nc = (nm + chunk_mfmas(tapk) - 1) / chunk_mfmas(tapk);
    const int64_t tiles = (int64_t)((a->Cout + ts - 1) / ts) * ((npix + ts - 1) / ts) * a->Nimg * a->sh * a->sw;
    const int wgk = pick_waves(nc, tiles, waves, true);
    a->rf_ts = ts;
    a->rf_tapk = tapk;
    a->rf_wgk = wgk;
    a->rf_nch = (nc + wgk - 1) / wgk;
    a->splitk = 1;
    a->rf_ngtot = wgk * a->rf_nch * chunk_groups(tapk);
    a->rf_nm = nm;
    a->rf_groups = 1;
    a->rf_cin_tile = a->Cin;
    a->rf_convt = 1;
    a->D = a->KD = a->sd = a->DO = 1;
    a->pd = 0;
    a->rf_fold = 0;
    a->rf_cs = a->H * a->W;
    a->rf_img_stride = (int64_t)a->Cin * a->rf_cs;
    a->rf_kd_magic = 0;
    a->rf_jmajor = (int64_t)a->Cin * a->H * a->W > (int64_t)a->Cout * a->Cin * taps ? 1 : 0;
    a->rf_wo_magic = (((uint64_t)1 << 32) / (uint64_t)woe) + 1;
    if (set_tile_order(a, (a->Cout + ts - 1) / ts, (int)((npix + ts - 1) / ts))) return true;
    a->rf_ts = 0;
    a->rf_convt = 0;
    return false;
}

size_t rf_pack_bytes(const GemmArgs &a) {
    if (!a.rf_ts) return 0;
    const size_t tiles_m = (size_t)((a.rf_tapk == -1 ? a.N : (a.rf_d2s ? 4 * a.Cout : a.Cout)) + a.rf_ts - 1) / a.rf_ts;
    return (a.rf_convt ? (size_t)a.sh * a.sw : 1) * tiles_m * (size_t)a.rf_ngtot * 256 * sizeof(float);
}

int launch_rf_pack(const GemmArgs &a, const float *w, float *dst, void *stream) {
    const int64_t total = (int64_t)(rf_pack_bytes(a) / sizeof(float));
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (a.rf_tapk == -1) {
        if (a.rf_ts == 32)
            hipLaunchKernelGGL((rf_pack_dense_kernel<32>), dim3(blocks), dim3(256), 0, (hipStream_t)stream, w, dst, a, total);
        else
            hipLaunchKernelGGL((rf_pack_dense_kernel<16>), dim3(blocks), dim3(256), 0, (hipStream_t)stream, w, dst, a, total);
        return (int)hipGetLastError();
    }
    if (a.rf_ts == 32)
        hipLaunchKernelGGL((rf_pack_kernel<32>), dim3(blocks), dim3(256), 0, (hipStream_t)stream, w, dst, a, total);
    else
        hipLaunchKernelGGL((rf_pack_kernel<16>), dim3(blocks), dim3(256), 0, (hipStream_t)stream, w, dst, a, total);
    return (int)hipGetLastError();
}

}  // namespace clg
