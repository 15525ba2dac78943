// Register-fed fp32 MFMA convolution kernels for gfx950 (no LDS staging).
//
// At batch 1 the deep layers of the CNN workloads (paper Sec. 5.1) have few
// output pixels (14x14, 7x7) and long reductions (K up to 4608).  With one
// 32x32 output tile per workgroup such a layer has a few dozen tiles: most of
// the 256 compute units idle unless K is split across workgroups, which costs a
// second kernel to add the partial sums.  Splitting K across the WAVES of one
// workgroup has no operand reuse between waves, so staging operands through LDS
// buys nothing there.  These kernels therefore
//  * feed the MFMAs straight from global memory: the weights are re-packed once
//    (when a plan is compiled) into the order in which lanes consume them, so a
//    wave's A operand for four MFMAs is one 16-byte load per lane, 1 KB
//    contiguous per wave; the B operand (input pixels) is one 4-byte load per
//    lane and MFMA, lanes running along consecutive pixels;
//  * have no barrier and no LDS access inside the K loop; the K-waves meet once,
//    in LDS, to add their accumulators;
//  * come with 32x32 tiles (v_mfma_f32_32x32x2_f32) and 16x16 tiles
//    (v_mfma_f32_16x16x4_f32): the small tile gives a 14x14 layer 200+
//    workgroups without any split across workgroups.
//
// K order.  MFMA number n of a tile contracts NSLOT input channels (NSLOT = 2
// or 4 k-slots of the instruction: lane / TS) at one filter tap:
//   n = cq * TAPS + t,  channel = cq * NSLOT + slot,  tap t = kh * KW + kw.
// Packed weights: [m-tile][group g][lane][4], element q of group g = MFMA 4g+q,
// lane = slot * TS + row; zero beyond Cout, Cin and the last MFMA, so padded
// work adds exact zeros.
//
// Grouped convolution (ResNeXt, paper Sec. 5.1): the TS output channels of an
// m-tile belong to one or a few consecutive channel groups; the tile contracts
// the input channels of exactly those groups (rf_cin_tile of them, starting at
// the first group's first channel), and the packed weights hold zeros where a
// row's group and a channel's group differ.  With 4 channels per group a 16-row
// tile spans 4 groups and a quarter of its MFMA work is useful; from 16
// channels per group on none is wasted.
#pragma once

#include <hip/hip_runtime.h>

#include "device_common.h"
#include "gemm_lean.h"

namespace clg {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// Phase time stamps, compiled in only for the phase probe (rf_phase_probe.hip, built with
// -DCLG_RF_STAMPS): thread 0 of every workgroup writes the device's 100 MHz wall clock at five points
// of the convolution kernel into g_rf_stamps[workgroup * 8 + point].  The library itself is built
// without the macro and carries none of this.
#ifdef CLG_RF_STAMPS
static __device__ long long *g_rf_stamps;
#define CLG_STAMP(i)                                                                                          \
    do {                                                                                                      \
        if (threadIdx.x == 0)                                                                                 \
            g_rf_stamps[((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 8 + (i)] = wall_clock64(); \
    } while (0)
#else
#define CLG_STAMP(i) do { } while (0)
#endif

template <int TS>
struct RfMfma;

template <>
struct RfMfma<32> {
    typedef floatx16 acc_t;
    static constexpr int NSLOT = 2, NACC = 16;
    static __device__ __forceinline__ acc_t mma(float a, float b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    // accumulator register g of a lane in slot s holds this row of the tile (column = lane % 32)
    static __device__ __forceinline__ int row(int g, int s) { return 8 * (g / 4) + 4 * s + (g % 4); }
};

template <>
struct RfMfma<16> {
    typedef floatx4 acc_t;
    static constexpr int NSLOT = 4, NACC = 4;
    static __device__ __forceinline__ acc_t mma(float a, float b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row(int g, int s) { return 4 * s + g; }
};

// TAPK: 1 = 1x1 filter without padding, 9 = 3x3 filter, 4 = 2x2 filter, 0 = any
// filter (tap geometry computed per MFMA).  TAPK 1, 9 and 4 need Cin % NSLOT == 0.
// Work units per wave ("chunks"): 16 MFMAs (TAPK 1), 36 MFMAs = all taps of
// four channel groups (TAPK 9), 16 MFMAs likewise (TAPK 4), 4 MFMAs (TAPK 0).
//
// Transposed convolution (DCGAN, paper Sec. 5.1) with stride s: the output pixels
// with (oh % s, ow % s) = (a, b) form a "phase" that only meets the taps
// kh = (a + pad) % s + s*u.  Written with u' = KH/s - 1 - u, a phase is an
// ordinary stride-1 convolution over the (HO/s x WO/s) grid of its pixels, with
// KH/s x KW/s taps and padding KH/s - 1 - (a + pad) / s; one grid.z slice per
// phase, each with its own packed (tap-flipped) weights.  k4 s2 p1 gives four
// 2x2 phases.

// Transposed convolution with few output channels (DCGAN's last layer, 64 -> 3): one phase is a GEMM
// with 3 rows, and a 16-row tile wastes 13 of them.  For k4 s2 p1 the four phases of output pixel block
// (2i + a, 2j + b) read the same 3x3 neighbourhood of input pixel (i, j) - tap kh = a + 1 - 2 dh of the
// filter sits at neighbour dh in {-1, 0, 1}, two of the three per axis - so the whole layer is ONE 3x3
// stride-1 pad-1 convolution over the input with 4 * Cout rows (row = 4 * channel + 2 a + b), zero
// weights where a phase does not meet a neighbour, and a store that puts row (channel, a, b) of input
// pixel (i, j) at output pixel (2i + a, 2j + b): 12 of 16 rows useful instead of 3, 9 operand loads per
// channel group for all four phases instead of 16.  GEO = 5.
//
// GEO: 0 = 2-D convolution, 1 = transposed convolution, 2 = 3-D convolution with the depth taps
// folded into the channel index, 3 = 3-D convolution with a single depth tap, 4 = 2-D 1x1 convolution
// with a relu on its input (the operand values are clamped on their way into the MFMA).  The depth code is
// compiled into GEO 2 and 3 only: a few more kernel arguments and one division are a measurable
// part of a four-microsecond kernel.
// The body takes its tile number as (bx of gx) instead of reading blockIdx.x, so that one launch can
// run the tiles of several convolutions (conv_rf_multi_kernel below); grid.y and grid.z are read as usual.
// Loads in flight per wave, in chunks: a wave that owns several chunks issues the loads of up to
// rf_depth<TAPK, WGK>() of them before its first MFMA.  A kernel whose waves own one chunk each is
// instantiated with PF = 1 instead: the deeper variant holds its extra operand registers whether it
// uses them or not, and fewer registers mean more resident waves.
template <int TAPK, int WGK>
constexpr int rf_depth() {
    return TAPK == 1 ? (WGK >= 16 ? 2 : 4) : (TAPK == 9 ? (WGK >= 16 ? 1 : 2) : 1);
}

template <int TS, int TAPK, int WGK, int GEO, int PF>
__device__ __forceinline__ void conv_rf_body(const GemmCore &p, const int bx, const int gx) {
    using MF = RfMfma<TS>;
    typedef typename MF::acc_t acc_t;
    constexpr int NSLOT = MF::NSLOT, NACC = MF::NACC;
    constexpr int NT = WGK * kWave;
    constexpr int PER_WAVE = NACC * kWave;                  // outputs of a tile
    constexpr int EPT = (PER_WAVE + NT - 1) / NT;           // outputs finished per thread
    extern __shared__ float red[];
    constexpr bool CONVT = GEO == 1;
    constexpr bool FOLD = GEO == 2;
    constexpr bool DEPTH = GEO == 2 || GEO == 3;
    constexpr bool PRELU = GEO == 4;
    constexpr bool D2S = GEO == 5;

    CLG_STAMP(0);                                            // entry
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int r = lane % TS, s = lane / TS;

    // effective geometry: the convolution itself, or one phase of a transposed convolution
    int KHe = p.KH, KWe = p.KW, she = p.sh, swe = p.sw, phe = p.ph, pwe = p.pw, HOe = p.HO, WOe = p.WO;
    int a_h = 0, a_w = 0, phase = 0, ks = blockIdx.z;
    if constexpr (CONVT) {
        phase = blockIdx.z;
        ks = 0;
        a_h = phase / p.sw;
        a_w = phase - a_h * p.sw;
        KHe = p.KH / p.sh;
        KWe = p.KW / p.sw;
        phe = KHe - 1 - (a_h + p.ph) / p.sh;
        pwe = KWe - 1 - (a_w + p.pw) / p.sw;
        she = swe = 1;
        HOe = p.HO / p.sh;
        WOe = p.WO / p.sw;
    }
    if constexpr (D2S) {                                     // the 3x3 convolution over the input that stands for the layer
        KHe = KWe = 3;
        she = swe = 1;
        phe = pwe = 1;
        HOe = p.H;
        WOe = p.W;
    }
    const int CoutE = D2S ? 4 * p.Cout : p.Cout;              // rows of the GEMM
    const int npix = HOe * WOe;
    const int tiles_m = (CoutE + TS - 1) / TS;
    const int tile = xcd_remap(bx, gx);
    // neighbouring workgroups share the larger operand: weights rows (i-major) or pixels (j-major);
    // tile / rf_tile_div by multiply-high (an integer division costs some thirty instructions)
    const int t_hi = (int)(((uint64_t)(uint32_t)tile * p.rf_tile_magic) >> 32), t_lo = tile - t_hi * p.rf_tile_div;
    const int mt = p.rf_jmajor ? t_lo : t_hi;
    const int nt = p.rf_jmajor ? t_hi : t_lo;
    const int i0 = mt * TS, j0 = nt * TS;
    // grid.y: the image, or (image, output depth) of a 3-D convolution
    int img = blockIdx.y, od = 0, DOe = 1;
    if constexpr (DEPTH) {
        DOe = p.DO;
        img = blockIdx.y / p.DO;
        od = blockIdx.y - img * p.DO;
    }
    const int id0 = DEPTH ? od * p.sd - p.pd : 0;            // input depth of depth tap 0

    const int jp = min(j0 + r, npix - 1);
    const int oh = (int)(((uint64_t)(uint32_t)jp * p.rf_wo_magic) >> 32);
    const int ow = jp - oh * WOe;
    const int ih0 = oh * she - phe, iw0 = ow * swe - pwe;
    const int HW = p.H * p.W;
    const int CS = DEPTH ? p.rf_cs : HW;                     // elements between channels: HW, or D * HW
    const int cbase = p.rf_groups > 1 ? (i0 / p.rf_cpg_out) * p.rf_cpg_in : 0;
    const int cin = min(p.rf_cin_tile, p.Cin - cbase);       // input channels this m-tile contracts
    // without folded depth taps the single depth tap's plane is part of the base address
    const float *const x_img = DEPTH ? p.B + (int64_t)img * p.rf_img_stride + (FOLD ? 0 : (int64_t)id0 * HW)
                                     : p.B + ((int64_t)img * p.Cin + cbase) * HW;
    // packed weights of this m-tile; a wave's load is base + uniform group offset + lane
    const f32x4 *const Ab = reinterpret_cast<const f32x4 *>(p.A) + ((int64_t)phase * tiles_m + mt) * p.rf_ngtot * kWave;
    const uint32_t lane_u = (uint32_t)lane;
    const int nch = p.rf_nch;                                // chunks per wave
    const int c0 = (ks * WGK + w) * nch;                     // this wave's first chunk
    const int cq_last = (cin + NSLOT - 1) / NSLOT - 1;

    // outputs this thread finishes, and the operands of their fused tail.  In the 1x1 path with 16x16 tiles
    // this runs behind the first round of operand loads: those are what the kernel waits for, and they
    // should leave before anything that is only needed at the end (measured: 0.35 - 1.0 us off the deep
    // layers; with 32x32 tiles, sixteen outputs per thread, and in the 3x3 path it cost 0.2 - 0.4 us instead).
    // (transposed convolution: the phase's pixel (oh', ow') is output pixel (a_h + s oh', a_w + s ow'))
    constexpr bool LATE_TAIL = TAPK == 1 && TS == 16;
    int64_t e_off[EPT];
    float e_bias[EPT], e_add[EPT];
#define CLG_RF_TAIL_SETUP()                                                                   \
    do {                                                                                      \
    _Pragma("unroll")                                                                         \
        for (int t = 0; t < EPT; ++t) {                                                       \
            const int e = tid + t * NT;                                                       \
            const int l = e % kWave, g = e / kWave;                                           \
            const int i = i0 + MF::row(g, l / TS), j = j0 + l % TS;                           \
            e_off[t] = (e < PER_WAVE && i < CoutE && j < npix) ? (((int64_t)img * p.Cout + i) * DOe + od) * npix + j : -1;\
            if (D2S && e_off[t] >= 0) {                                                       \
                const int ohh = (int)(((uint64_t)(uint32_t)j * p.rf_wo_magic) >> 32), oww = j - ohh * WOe;\
                e_off[t] = (((int64_t)img * p.Cout + (i >> 2)) * p.HO + 2 * ohh + ((i >> 1) & 1)) * p.WO + 2 * oww + (i & 1);\
            }                                                                                 \
            if (CONVT && e_off[t] >= 0) {                                                     \
                const int ohh = (int)(((uint64_t)(uint32_t)j * p.rf_wo_magic) >> 32), oww = j - ohh * WOe;\
                e_off[t] = (((int64_t)img * p.Cout + i) * p.HO + a_h + p.sh * ohh) * p.WO + a_w + p.sw * oww;\
            }                                                                                 \
            e_bias[t] = 0.f;                                                                  \
            e_add[t] = 0.f;                                                                   \
            if (p.splitk == 1 && e_off[t] >= 0) {                                             \
                if (p.ef.flags & EF_BIAS) e_bias[t] = p.ef.bias[D2S ? i >> 2 : i];            \
                if (p.ef.flags & EF_ADD) e_add[t] = p.ef.add[e_off[t]];                       \
            }                                                                                 \
        }                                                                                     \
    } while (0)
    if constexpr (!LATE_TAIL) CLG_RF_TAIL_SETUP();

    acc_t acc;
#pragma unroll
    for (int g = 0; g < NACC; ++g) acc[g] = 0.f;
    CLG_STAMP(1);                                            // arguments read, indices set up

    if constexpr (TAPK == 1) {
        // ---- 1x1: MFMA n contracts channels n*NSLOT .. n*NSLOT+NSLOT-1 at this lane's pixel
        // addresses are "uniform base + 32-bit lane offset": one scalar multiply and no 64-bit
        // vector arithmetic per load (offsets within an image fit 32 bits: checked on the host)
        const uint32_t lane_off = (uint32_t)(s * CS + ih0 * p.W + iw0);
        const uint32_t cq_step = (uint32_t)(NSLOT * CS);
        // Up to PF chunks of loads are in flight before the first MFMA: a wave that owns one to four
        // chunks pays one memory round trip for all of them (the K loop of these kernels is a few
        // hundred MFMA cycles against a microsecond of memory latency).  Sixteen waves per workgroup
        // leave a wave 128 registers: two chunks then.
        f32x4 a[PF][4];
        float b[PF][16];
#define CLG_RF_LOAD(set, c)                                                                   \
    do {                                                                                      \
        const int ch_ = (c) + c0;                                                             \
        _Pragma("unroll") for (int u = 0; u < 4; ++u) a[set][u] = (Ab + (uint32_t)(ch_ * 4 + u) * kWave)[lane_u]; \
        _Pragma("unroll") for (int u = 0; u < 16; ++u) {                                      \
            const int cq_ = min(ch_ * 16 + u, cq_last);                                       \
            b[set][u] = (x_img + (uint32_t)cq_ * cq_step)[lane_off];                          \
        }                                                                                     \
    } while (0)
#define CLG_RF_MMA(set)                                                                       \
    do {                                                                                      \
        _Pragma("unroll") for (int u = 0; u < 16; ++u)                                        \
            acc = MF::mma(a[set][u / 4][u % 4], PRELU ? fmaxf(b[set][u], 0.f) : b[set][u], acc); \
    } while (0)
        for (int c = 0; c < nch; c += PF) {
            const int left = nch - c;                        // wave-uniform
            CLG_RF_LOAD(0, c);
            if constexpr (PF > 1) {
                if (left > 1) CLG_RF_LOAD(1, c + 1);
            }
            if constexpr (PF > 2) {
                if (left > 2) CLG_RF_LOAD(2, c + 2);
                if (left > 3) CLG_RF_LOAD(3, c + 3);
            }
            if constexpr (LATE_TAIL) {
                if (c == 0) CLG_RF_TAIL_SETUP();
            }
            __builtin_amdgcn_sched_barrier(0);               // every load of the round goes out before its first MFMA
            CLG_RF_MMA(0);
            if constexpr (PF > 1) {
                if (left > 1) CLG_RF_MMA(1);
            }
            if constexpr (PF > 2) {
                if (left > 2) CLG_RF_MMA(2);
                if (left > 3) CLG_RF_MMA(3);
            }
        }
#undef CLG_RF_LOAD
#undef CLG_RF_MMA
    } else if constexpr (TAPK == 9) {
        // ---- 3x3: the nine tap offsets of this lane's pixel are fixed; a chunk is
        // four channel groups x nine taps
        uint32_t voff[9];
        bool ok[9];
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const int ih = ih0 + t / 3, iw = iw0 + t % 3;
            ok[t] = ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
            voff[t] = (uint32_t)((FOLD ? 0 : s * CS) + (ok[t] ? ih * p.W + iw : 0));
        }
        const uint32_t cq_step = (uint32_t)(NSLOT * CS);
        // two chunks of loads in flight (2 x 45 loads) before the first MFMA of a round; one with
        // sixteen waves per workgroup (128 registers per wave)
        f32x4 a[PF][9];
        float b[PF][36];
        bool okd[PF][4];
#define CLG_RF_LOAD(set, c)                                                                   \
    do {                                                                                      \
        const int ch = c0 + (c);                                                              \
        _Pragma("unroll") for (int u = 0; u < 9; ++u) a[set][u] = (Ab + (uint32_t)(ch * 9 + u) * kWave)[lane_u]; \
        _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                       \
            const float *xc;                                                                  \
            okd[set][q] = true;                                                               \
            if constexpr (FOLD) {                                                             \
                /* this lane's folded channel c * KD + kd: plane (c, id0 + kd) of the volume */ \
                const uint32_t chq = (uint32_t)(min(ch * 4 + q, cq_last) * NSLOT + s);        \
                const uint32_t cc = (uint32_t)(((uint64_t)chq * p.rf_kd_magic) >> 32);        \
                const int idd = id0 + (int)(chq - cc * (uint32_t)p.KD);                       \
                okd[set][q] = idd >= 0 && idd < p.D;                                          \
                xc = x_img + (cc * (uint32_t)p.D + (uint32_t)(okd[set][q] ? idd : 0)) * (uint32_t)HW; \
            } else {                                                                          \
                xc = x_img + (uint32_t)min(ch * 4 + q, cq_last) * cq_step;                    \
            }                                                                                 \
            _Pragma("unroll") for (int t = 0; t < 9; ++t) b[set][q * 9 + t] = xc[voff[t]];    \
        }                                                                                     \
    } while (0)
#define CLG_RF_MMA(set)                                                                       \
    do {                                                                                      \
        _Pragma("unroll") for (int u = 0; u < 36; ++u) b[set][u] = (ok[u % 9] && okd[set][u / 9]) ? b[set][u] : 0.f; \
        _Pragma("unroll") for (int u = 0; u < 36; ++u) acc = MF::mma(a[set][u / 4][u % 4], b[set][u], acc); \
    } while (0)
        for (int c = 0; c < nch; c += PF) {
            const int left = nch - c;                        // wave-uniform
            CLG_RF_LOAD(0, c);
            if constexpr (PF > 1) {
                if (left > 1) CLG_RF_LOAD(1, c + 1);
            }
            __builtin_amdgcn_sched_barrier(0);               // all loads of the round go out before the first MFMA waits
            CLG_RF_MMA(0);
            if constexpr (PF > 1) {
                if (left > 1) CLG_RF_MMA(1);
            }
        }
#undef CLG_RF_LOAD
#undef CLG_RF_MMA
    } else if constexpr (TAPK == 4) {
        // ---- 2x2 (a phase of a k4 s2 transposed convolution): like 3x3, a chunk is four
        // channel groups x four taps
        uint32_t voff[4];
        bool ok[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int ih = ih0 + t / 2, iw = iw0 + t % 2;
            ok[t] = ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
            voff[t] = (uint32_t)(s * CS + (ok[t] ? ih * p.W + iw : 0));
        }
        const uint32_t cq_step = (uint32_t)(NSLOT * CS);
        f32x4 a[2][4];
        float b[2][16];
#define CLG_RF_LOAD(set, c)                                                                   \
    do {                                                                                      \
        const int ch_ = min((c), nch - 1) + c0;                                               \
        _Pragma("unroll") for (int u = 0; u < 4; ++u) a[set][u] = (Ab + (uint32_t)(ch_ * 4 + u) * kWave)[lane_u]; \
        _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                       \
            const float *xc_ = x_img + (uint32_t)min(ch_ * 4 + q, cq_last) * cq_step;         \
            _Pragma("unroll") for (int t = 0; t < 4; ++t) b[set][q * 4 + t] = xc_[voff[t]];   \
        }                                                                                     \
        __builtin_amdgcn_sched_barrier(0);                                                    \
    } while (0)
#define CLG_RF_MMA(set)                                                                       \
    do {                                                                                      \
        _Pragma("unroll") for (int u = 0; u < 16; ++u)                                        \
            acc = MF::mma(a[set][u / 4][u % 4], ok[u % 4] ? b[set][u] : 0.f, acc);            \
    } while (0)
        CLG_RF_LOAD(0, 0);
        int c = 0;
        for (; c + 1 < nch; c += 2) {
            CLG_RF_LOAD(1, c + 1);
            CLG_RF_MMA(0);
            CLG_RF_LOAD(0, c + 2);
            CLG_RF_MMA(1);
        }
        if (c < nch) CLG_RF_MMA(0);
#undef CLG_RF_LOAD
#undef CLG_RF_MMA
    } else {
        // ---- any filter: tap geometry per MFMA; (cq, kh, kw) advance with n
        const int taps = KHe * KWe;
        const int nm = p.rf_nm;
        int n = c0 * 4;
        int cq = n / taps, t = n - cq * taps;
        int kh = t / KWe, kw = t - kh * KWe;
        for (int c = 0; c < nch; ++c) {
            const f32x4 a = (Ab + (uint32_t)(c0 + c) * kWave)[lane_u];
            float b[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int ch = cq * NSLOT + s;
                const int ih = ih0 + kh, iw = iw0 + kw;
                bool ok = n < nm && ch < cin && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
                int64_t plane = (int64_t)ch * CS;
                if constexpr (FOLD) {
                    const uint32_t cc = (uint32_t)(((uint64_t)(uint32_t)ch * p.rf_kd_magic) >> 32);
                    const int idd = id0 + (ch - (int)cc * p.KD);
                    ok = ok && idd >= 0 && idd < p.D;
                    plane = ((int64_t)cc * p.D + idd) * HW;
                }
                const float v = x_img[ok ? plane + ih * p.W + iw : 0];
                b[q] = ok ? v : 0.f;
                ++n;
                if (++kw == KWe) {
                    kw = 0;
                    if (++kh == KHe) {
                        kh = 0;
                        ++cq;
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) acc = MF::mma(a[q], b[q], acc);
        }
    }

    // ---- the K-waves add their accumulators in LDS, in wave order
#ifdef CLG_RF_STAMPS
    if (threadIdx.x == 0) {                                  // the first wave's accumulator is final: its K loop is over
        float sink = 0.f;
        for (int g = 0; g < NACC; ++g) sink += acc[g];
        asm volatile("" ::"v"(sink));
    }
#endif
    CLG_STAMP(2);                                            // K loop of the first wave done
    if constexpr (WGK > 1) {
#pragma unroll
        for (int g = 0; g < NACC; ++g) red[w * PER_WAVE + g * kWave + lane] = acc[g];
        __syncthreads();
    }
    CLG_STAMP(3);                                            // all K-waves have arrived
#pragma unroll
    for (int t = 0; t < EPT; ++t) {
        float v;
        if constexpr (WGK > 1) {
            const int e = min(tid + t * NT, PER_WAVE - 1);
            v = 0.f;
#pragma unroll
            for (int ww = 0; ww < WGK; ++ww) v += red[ww * PER_WAVE + e];
        } else {
            v = acc[t];
        }
        if (e_off[t] >= 0) {
            if (p.splitk > 1) p.partial[(int64_t)ks * p.c_numel + e_off[t]] = v;
            else p.C[e_off[t]] = finish_value(p, v, e_bias[t], e_add[t]);
        }
    }
#ifdef CLG_RF_STAMPS
    __builtin_amdgcn_s_waitcnt(0);                           // the stores have left the wave
#endif
    CLG_STAMP(4);                                            // sums taken, tail applied, stores issued
#undef CLG_RF_TAIL_SETUP
}

template <int TS, int TAPK, int WGK, int GEO, int PF>
__global__ __launch_bounds__(WGK *kWave) void conv_rf_kernel(GemmArgs p) {
    conv_rf_body<TS, TAPK, WGK, GEO, PF>(p, blockIdx.x, gridDim.x);
}

// Several independent problems of one kernel shape in ONE launch (a region of sibling kernels,
// paper Sec. 4.3: what a graph-level backend gains over kernels placed one by one is work across
// kernel boundaries; here, two or more kernels that do not depend on each other share a dispatch
// and fill the chip together).  Workgroup bx belongs to problem k with tile_end[k-1] <= bx <
// tile_end[k]; the choice is wave-uniform and the problem's arguments are read from the
// kernel-argument segment at a uniform offset, so each problem runs exactly the code it runs alone.
template <int TS, int WGK, int GEO>
__global__ __launch_bounds__(WGK *kWave) void conv_rf_multi_kernel(RfMultiArgs m) {
    const int bx = blockIdx.x;
    int k = 0;
#pragma unroll
    for (int i = 0; i + 1 < kMaxRegion; ++i) k += (i + 1 < m.n && bx >= m.tile_end[i]) ? 1 : 0;
    const int start = k ? m.tile_end[k - 1] : 0;
    conv_rf_body<TS, 1, WGK, GEO, rf_depth<1, WGK>()>(m.p[k], bx - start, m.tile_end[k] - start);
}

// ---- dense: y[m][n] = sum_k x[m][k] * w[n][k] -------------------------------------------------
// The weights are the A operand (rows i = n, packed), the activations the B
// operand (columns j = m): lane (slot s, column r) reads 16 bytes of row j0 + r,
// k = (g * NSLOT + s) * 4 .. + 3, and element q feeds MFMA q of group g; the
// packed weights follow that k order.  A chunk is four groups (16 MFMAs).
// Needs K % (4 * NSLOT) == 0, lda % 4 == 0 and 16-byte aligned x.
// The tile is finished through LDS with rows and columns swapped, so that
// consecutive threads store consecutive n (the contiguous index of y).
template <int TS>
struct RfPark;          // where accumulator register g of lane (s, r) is parked: rows spread over LDS banks
template <>
struct RfPark<32> {
    static constexpr int PERW = 1056;
    static __device__ __forceinline__ int at(int g, int s, int r) { return g * 66 + s * 33 + r; }
    static __device__ __forceinline__ int of(int row, int col) { return at(4 * (row / 8) + row % 4, (row / 4) % 2, col); }
};
template <>
struct RfPark<16> {
    static constexpr int PERW = 320;
    static __device__ __forceinline__ int at(int g, int s, int r) { return g * 81 + s * 20 + r; }
    static __device__ __forceinline__ int of(int row, int col) { return at(row % 4, row / 4, col); }
};

template <int TS, int WGK>
__device__ __forceinline__ void dense_rf_body(const GemmCore &p, const int bx, const int gx) {
    using MF = RfMfma<TS>;
    using PK = RfPark<TS>;
    typedef typename MF::acc_t acc_t;
    constexpr int NSLOT = MF::NSLOT, NACC = MF::NACC;
    constexpr int NT = WGK * kWave;
    constexpr int OUTS = TS * TS;
    constexpr int EPT = (OUTS + NT - 1) / NT;
    extern __shared__ float red[];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int r = lane % TS, s = lane / TS;

    const int tile = xcd_remap(bx, gx);
    const int t_hi = (int)(((uint64_t)(uint32_t)tile * p.rf_tile_magic) >> 32), t_lo = tile - t_hi * p.rf_tile_div;
    const int mt = p.rf_jmajor ? t_lo : t_hi;     // weight-row tile
    const int nt = p.rf_jmajor ? t_hi : t_lo;     // activation-row tile
    const int i0 = mt * TS, j0 = nt * TS;
    const int ks = blockIdx.z;

    // addresses are "uniform base + 32-bit lane offset" (no 64-bit vector arithmetic per load)
    const f32x4 *const Ab = reinterpret_cast<const f32x4 *>(p.B) + (int64_t)mt * p.rf_ngtot * kWave;
    const f32x4 *const Xb = reinterpret_cast<const f32x4 *>(p.A);
    const uint32_t lane_u = (uint32_t)lane;
    // The 16 bytes lane (slot s, column r) needs lie at row r, k-part s.  Loaded by that lane itself, neighbouring
    // lanes would touch different rows; instead lane l loads row l / NSLOT, part l % NSLOT (neighbouring lanes
    // read neighbouring addresses) and the values change lanes afterwards (ds_bpermute: no memory access).
    const int lrow = lane / NSLOT, lpart = lane % NSLOT;
    const uint32_t x_lane = (uint32_t)(min(j0 + lrow, p.M - 1) * (p.lda / 4) + lpart);      // in 16-byte units
    const int src_lane4 = (r * NSLOT + s) * 4;                                            // byte address for ds_bpermute
    const int nch = p.rf_nch;
    const int c0 = (ks * WGK + w) * nch;
    const int g_last = p.K / (4 * NSLOT) - 1;

    // outputs this thread finishes: row (n) runs fastest over the threads
    const int tile_base = p.cs_len ? (i0 / p.cs_len) * (int)p.cs_stride + i0 % p.cs_len : i0;
    int64_t e_off[EPT];
    float e_bias[EPT], e_add[EPT];
    int e_idx[EPT];
    // (filled behind the first operand loads, which are what the kernel waits for: 0.1 - 0.25 us; in the
    // two-tile kernel below the same move cost 0.1 - 0.3 us and was not made)
    acc_t acc;
#pragma unroll
    for (int g = 0; g < NACC; ++g) acc[g] = 0.f;

    f32x4 a[2][4], b[2][4];
#define CLG_RFD_LOAD(set, c)                                                                  \
    do {                                                                                      \
        const int ch_ = min((c), nch - 1) + c0;                                               \
        _Pragma("unroll") for (int u = 0; u < 4; ++u) a[set][u] = (Ab + (uint32_t)(ch_ * 4 + u) * kWave)[lane_u]; \
        _Pragma("unroll") for (int u = 0; u < 4; ++u) b[set][u] = (Xb + (uint32_t)min(ch_ * 4 + u, g_last) * NSLOT)[x_lane]; \
        __builtin_amdgcn_sched_barrier(0);                                                    \
    } while (0)
#define CLG_RFD_MMA(set)                                                                      \
    do {                                                                                      \
        _Pragma("unroll") for (int u = 0; u < 16; ++u) {                                      \
            const float own_ = b[set][u / 4][u % 4];      /* (a copy: not the vector element itself) */ \
            const float bv_ = __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane4, __float_as_int(own_))); \
            acc = MF::mma(a[set][u / 4][u % 4], bv_, acc);                                    \
        }                                                                                     \
    } while (0)
    CLG_RFD_LOAD(0, 0);
#pragma unroll
    for (int t = 0; t < EPT; ++t) {
        const int e = min(tid + t * NT, OUTS - 1);
        const int row = e % TS, col = e / TS;
        e_idx[t] = PK::of(row, col);
        const bool ok = tid + t * NT < OUTS && i0 + row < p.N && j0 + col < p.M;
        e_off[t] = ok ? (int64_t)(j0 + col) * p.ldc + tile_base + row : -1;
        e_bias[t] = 0.f;
        e_add[t] = 0.f;
        if (p.splitk == 1 && ok) {
            if (p.ef.flags & EF_BIAS) e_bias[t] = p.ef.bias[i0 + row];
            if (p.ef.flags & EF_ADD) e_add[t] = p.ef.add[e_off[t]];
        }
    }
    int c = 0;
    for (; c + 1 < nch; c += 2) {
        CLG_RFD_LOAD(1, c + 1);
        CLG_RFD_MMA(0);
        CLG_RFD_LOAD(0, c + 2);
        CLG_RFD_MMA(1);
    }
    if (c < nch) CLG_RFD_MMA(0);
#undef CLG_RFD_LOAD
#undef CLG_RFD_MMA

#pragma unroll
    for (int g = 0; g < NACC; ++g) red[w * PK::PERW + PK::at(g, s, r)] = acc[g];
    __syncthreads();
#pragma unroll
    for (int t = 0; t < EPT; ++t) {
        float v = 0.f;
#pragma unroll
        for (int ww = 0; ww < WGK; ++ww) v += red[ww * PK::PERW + e_idx[t]];
        if (e_off[t] >= 0) {
            if (p.splitk > 1) p.partial[(int64_t)ks * p.c_numel + e_off[t]] = v;
            else p.C[e_off[t]] = finish_value(p, v, e_bias[t], e_add[t]);
        }
    }
}

template <int TS, int WGK>
__global__ __launch_bounds__(WGK *kWave) void dense_rf_kernel(GemmArgs p) {
    dense_rf_body<TS, WGK>(p, blockIdx.x, gridDim.x);
}

// Several dense problems in one launch (see conv_rf_multi_kernel): e.g. the query, key and value
// projections of an attention layer, which read the same activations.
template <int TS, int WGK>
__global__ __launch_bounds__(WGK *kWave) void dense_rf_multi_kernel(RfMultiArgs m) {
    const int bx = blockIdx.x;
    int k = 0;
#pragma unroll
    for (int i = 0; i + 1 < kMaxRegion; ++i) k += (i + 1 < m.n && bx >= m.tile_end[i]) ? 1 : 0;
    const int start = k ? m.tile_end[k - 1] : 0;
    dense_rf_body<TS, WGK>(m.p[k], bx - start, m.tile_end[k] - start);
}

// Two weight tiles per wave.  Every MFMA of the kernel above needs 16 bytes per lane of weights and
// 16 bytes per lane of activations for four MFMAs, and a lane shuffle per MFMA: at the matrix cores'
// full rate that is the whole bandwidth of the vector memory path.  Here a wave owns 32 output
// columns (two 16-row tiles of packed weights) and 16 activation rows: the activation operand and its
// shuffle are shared by two MFMAs with independent accumulators (a quarter less load traffic, half the
// shuffles, two MFMA chains in flight).  Same packed weights, same k order, TS = 16.
template <int WGK>
__device__ __forceinline__ void dense_rf2_body(const GemmCore &p, const int bx, const int gx) {
    using MF = RfMfma<16>;
    using PK = RfPark<16>;
    typedef MF::acc_t acc_t;
    constexpr int TS = 16, NSLOT = 4, NACC = 4;
    constexpr int NT = WGK * kWave;
    constexpr int OUTS = 2 * TS * TS;
    constexpr int EPT = (OUTS + NT - 1) / NT;
    extern __shared__ float red[];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int r = lane % TS, s = lane / TS;

    const int tile = xcd_remap(bx, gx);
    const int t_hi = (int)(((uint64_t)(uint32_t)tile * p.rf_tile_magic) >> 32), t_lo = tile - t_hi * p.rf_tile_div;
    const int mp = p.rf_jmajor ? t_lo : t_hi;     // pair of weight-row tiles
    const int nt = p.rf_jmajor ? t_hi : t_lo;     // activation-row tile
    const int i0 = mp * 2 * TS, j0 = nt * TS;
    const int tiles_m = (p.N + TS - 1) / TS;
    const int m1 = min(mp * 2 + 1, tiles_m - 1);  // an odd tile count: the last pair's second tile repeats the first (its outputs are masked)

    const f32x4 *const Ab0 = reinterpret_cast<const f32x4 *>(p.B) + (int64_t)(mp * 2) * p.rf_ngtot * kWave;
    const f32x4 *const Ab1 = reinterpret_cast<const f32x4 *>(p.B) + (int64_t)m1 * p.rf_ngtot * kWave;
    const f32x4 *const Xb = reinterpret_cast<const f32x4 *>(p.A);
    const uint32_t lane_u = (uint32_t)lane;
    const int lrow = lane / NSLOT, lpart = lane % NSLOT;
    const uint32_t x_lane = (uint32_t)(min(j0 + lrow, p.M - 1) * (p.lda / 4) + lpart);      // in 16-byte units
    const int src_lane4 = (r * NSLOT + s) * 4;
    const int nch = p.rf_nch;
    const int c0 = w * nch;
    const int g_last = p.K / (4 * NSLOT) - 1;

    int64_t e_off[EPT];
    float e_bias[EPT], e_add[EPT];
    int e_idx[EPT];
#pragma unroll
    for (int t = 0; t < EPT; ++t) {
        const int e = min(tid + t * NT, OUTS - 1);
        const int sub = e / (TS * TS), in = e % (TS * TS);
        const int row = in % TS, col = in / TS;
        const int it = i0 + sub * TS;                 // first output column of this tile
        const int tile_base = p.cs_len ? (it / p.cs_len) * (int)p.cs_stride + it % p.cs_len : it;
        e_idx[t] = sub * PK::PERW + PK::of(row, col);
        const bool ok = tid + t * NT < OUTS && it + row < p.N && j0 + col < p.M;
        e_off[t] = ok ? (int64_t)(j0 + col) * p.ldc + tile_base + row : -1;
        e_bias[t] = 0.f;
        e_add[t] = 0.f;
        if (ok) {
            if (p.ef.flags & EF_BIAS) e_bias[t] = p.ef.bias[it + row];
            if (p.ef.flags & EF_ADD) e_add[t] = p.ef.add[e_off[t]];
        }
    }

    acc_t acc0, acc1;
#pragma unroll
    for (int g = 0; g < NACC; ++g) acc0[g] = acc1[g] = 0.f;

    f32x4 a0[2][4], a1[2][4], b[2][4];
#define CLG_RFD_LOAD(set, c)                                                                  \
    do {                                                                                      \
        const int ch_ = min((c), nch - 1) + c0;                                               \
        _Pragma("unroll") for (int u = 0; u < 4; ++u) a0[set][u] = (Ab0 + (uint32_t)(ch_ * 4 + u) * kWave)[lane_u]; \
        _Pragma("unroll") for (int u = 0; u < 4; ++u) a1[set][u] = (Ab1 + (uint32_t)(ch_ * 4 + u) * kWave)[lane_u]; \
        _Pragma("unroll") for (int u = 0; u < 4; ++u) b[set][u] = (Xb + (uint32_t)min(ch_ * 4 + u, g_last) * NSLOT)[x_lane]; \
        __builtin_amdgcn_sched_barrier(0);                                                    \
    } while (0)
#define CLG_RFD_MMA(set)                                                                      \
    do {                                                                                      \
        _Pragma("unroll") for (int u = 0; u < 16; ++u) {                                      \
            const float own_ = b[set][u / 4][u % 4];                                          \
            const float bv_ = __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane4, __float_as_int(own_))); \
            acc0 = MF::mma(a0[set][u / 4][u % 4], bv_, acc0);                                 \
            acc1 = MF::mma(a1[set][u / 4][u % 4], bv_, acc1);                                 \
        }                                                                                     \
    } while (0)
    CLG_RFD_LOAD(0, 0);
    int c = 0;
    for (; c + 1 < nch; c += 2) {
        CLG_RFD_LOAD(1, c + 1);
        CLG_RFD_MMA(0);
        CLG_RFD_LOAD(0, c + 2);
        CLG_RFD_MMA(1);
    }
    if (c < nch) CLG_RFD_MMA(0);
#undef CLG_RFD_LOAD
#undef CLG_RFD_MMA

#pragma unroll
    for (int g = 0; g < NACC; ++g) {
        red[w * 2 * PK::PERW + PK::at(g, s, r)] = acc0[g];
        red[w * 2 * PK::PERW + PK::PERW + PK::at(g, s, r)] = acc1[g];
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < EPT; ++t) {
        float v = 0.f;
#pragma unroll
        for (int ww = 0; ww < WGK; ++ww) v += red[ww * 2 * PK::PERW + e_idx[t]];
        if (e_off[t] >= 0) p.C[e_off[t]] = finish_value(p, v, e_bias[t], e_add[t]);
    }
}

template <int WGK>
__global__ __launch_bounds__(WGK *kWave) void dense_rf2_kernel(GemmArgs p) {
    dense_rf2_body<WGK>(p, blockIdx.x, gridDim.x);
}

template <int WGK>
__global__ __launch_bounds__(WGK *kWave) void dense_rf2_multi_kernel(RfMultiArgs m) {
    const int bx = blockIdx.x;
    int k = 0;
#pragma unroll
    for (int i = 0; i + 1 < kMaxRegion; ++i) k += (i + 1 < m.n && bx >= m.tile_end[i]) ? 1 : 0;
    const int start = k ? m.tile_end[k - 1] : 0;
    dense_rf2_body<WGK>(m.p[k], bx - start, m.tile_end[k] - start);
}

// Dense weights w [N][K] -> [n-tile][group][lane][4] in the k order above.
template <int TS>
__global__ void rf_pack_dense_kernel(const float *w, float *dst, GemmArgs p, int64_t total) {
    constexpr int NSLOT = RfMfma<TS>::NSLOT;
    const int64_t d = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (d >= total) return;
    const int q = (int)(d & 3), lane = (int)((d >> 2) & 63);
    const int64_t gg = d >> 8;
    const int g = (int)(gg % p.rf_ngtot), mt = (int)(gg / p.rf_ngtot);
    const int i = mt * TS + lane % TS;
    const int k = (g * NSLOT + lane / TS) * 4 + q;
    dst[d] = (i < p.N && k < p.K) ? w[(int64_t)i * p.ldb + k] : 0.f;
}

// Weight re-packing (once per compiled kernel): w is [Cout][Cin / groups][KH*KW].
template <int TS>
__global__ void rf_pack_kernel(const float *w, float *dst, GemmArgs p, int64_t total) {
    constexpr int NSLOT = RfMfma<TS>::NSLOT;
    const int64_t d = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (d >= total) return;
    const int KHe = p.rf_d2s ? 3 : (p.rf_convt ? p.KH / p.sh : p.KH), KWe = p.rf_d2s ? 3 : (p.rf_convt ? p.KW / p.sw : p.KW);
    const int taps = KHe * KWe;
    const int tiles_m = ((p.rf_d2s ? 4 * p.Cout : p.Cout) + TS - 1) / TS;
    const int q = (int)(d & 3), lane = (int)((d >> 2) & 63);
    const int64_t gg = d >> 8;
    const int g = (int)(gg % p.rf_ngtot);
    const int mt = (int)((gg / p.rf_ngtot) % tiles_m), phase = (int)(gg / p.rf_ngtot / tiles_m);
    const int n = 4 * g + q;
    const int cq = n / taps, t = n - cq * taps;
    const int i = mt * TS + lane % TS, cl = cq * NSLOT + lane / TS;      // output channel, channel within the tile's span
    float v = 0.f;
    if (p.rf_d2s) {
        // row i = (channel i / 4, phase a = (i / 2) % 2, b = i % 2); tap t = (dh + 1) * 3 + (dw + 1) of the 3x3
        // neighbourhood meets filter tap kh = a + 1 - 2 dh, kw = b + 1 - 2 dw of w [Cin][Cout][4][4] if that exists
        const int co = i >> 2, a_h = (i >> 1) & 1, a_w = i & 1;
        const int kh = a_h + 1 - 2 * (t / 3 - 1), kw = a_w + 1 - 2 * (t % 3 - 1);
        if (n < p.rf_nm && co < p.Cout && cl < p.Cin && kh >= 0 && kh < 4 && kw >= 0 && kw < 4)
            v = w[(((int64_t)cl * p.Cout + co) * 4 + kh) * 4 + kw];
    } else if (n < p.rf_nm && i < p.Cout && cl < p.rf_cin_tile) {
        if (p.rf_convt) {
            // w is [Cin][Cout][KH][KW]; tap u' of the phase is kernel tap r + s * (KH/s - 1 - u')
            const int a_h = phase / p.sw, a_w = phase - a_h * p.sw;
            const int uh = t / KWe, uw = t - uh * KWe;
            const int kh = (a_h + p.ph) % p.sh + p.sh * (KHe - 1 - uh), kw = (a_w + p.pw) % p.sw + p.sw * (KWe - 1 - uw);
            v = w[(((int64_t)cl * p.Cout + i) * p.KH + kh) * p.KW + kw];
        } else if (p.rf_groups > 1) {
            const int ch = (mt * TS / p.rf_cpg_out) * p.rf_cpg_in + cl;  // input channel
            const int grp = i / p.rf_cpg_out;
            if (ch / p.rf_cpg_in == grp) v = w[((int64_t)i * p.rf_cpg_in + (ch - grp * p.rf_cpg_in)) * taps + t];
        } else {
            v = w[((int64_t)i * p.Cin + cl) * taps + t];
        }
    }
    dst[d] = v;
}

// gemm_rf.hip
#ifdef CLG_RF_STAMPS
void rf_set_stamps(long long *dev);      // where the stamps go (device memory, 8 values per workgroup)
#endif
int launch_rf_conv(const GemmArgs &a, hipStream_t s);
int launch_rf_multi(const GemmArgs *members, int n, hipStream_t s);

}  // namespace clg
