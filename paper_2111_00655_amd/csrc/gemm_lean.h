// Instruction-lean fp32 MFMA kernels for gfx950: matrix products with aligned
// operands (dense, batched matmul, 1x1 convolution) and 3x3 convolution.
//
// At batch 1 the contractions of the workloads (paper Sec. 5.1) are a few
// hundred MFLOP each: one to two thousand MFMA instructions per SIMD.  A wave64
// vector instruction occupies its SIMD for 4 cycles and a 32x32x2 fp32 MFMA for
// 64, so a kernel that spends twenty address-arithmetic instructions per loaded
// element is bound by those, not by the matrix cores or by memory.  These
// kernels therefore keep everything but loads, LDS traffic and MFMAs out of the
// K loop:
//  * every thread's global and LDS addresses are fixed before the loop; per
//    slice a uniform base pointer advances (scalar unit), the per-lane offsets
//    stay; out-of-range rows / columns are clamped to the last valid one, so
//    loads need no predicate and the surplus results are simply not stored;
//  * K must be a multiple of the slice, operands 16-byte aligned: other shapes
//    go to the general kernel (gemm_fast.h);
//  * MM: operands keep their global orientation in LDS ([row][k] read as
//    ds_read_b128 fragments, [k][col] as ds_read_b32), slot mapping "lane half
//    h, MFMA q of four -> k = 8g + 4h + q";
//  * 3x3 convolution: instead of gathering im2col columns from global memory
//    (nine loads and an index decomposition per input value), the workgroup
//    copies the raw input patch its 32 output pixels touch, channel by channel,
//    into LDS once, and MFMA B-fragments are read from the patch at
//    "pixel base + tap offset": the two k-slots of an MFMA are the same tap of
//    two channels, so the offset between lane halves is a constant folded into
//    the per-lane base, and the tap offset is wave-uniform;
//  * the fused elementwise tail in its common form (scale, bias, residual,
//    activation) is a few flag tests; bias and residual values of the outputs a
//    thread will finish are fetched before the K loop.
#pragma once

#include <hip/hip_runtime.h>

#include "device_common.h"
#include "gemm_fast.h"

namespace clg {

// 16-byte values as a native vector (a first-class register value: the HIP
// f32x4 struct is copied with memcpy, which keeps staging arrays in scratch)
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---- common-form epilogue -------------------------------------------------------------
// (a tail that is not in the common form is not run by these kernels: the
// launcher sends it to the general kernel, which interprets any step list)
__device__ __forceinline__ float finish_value(const GemmCore &p, float v, float bias_v, float add_v) {
    const int f = p.ef.flags;
    if (f & EF_SCALE) v *= p.ef.scale;
    v += bias_v;
    v += add_v;
    if (f & EF_RELU) v = v > 0.f ? v : 0.f;
    else if (f & EF_GELU) v = gelu_erf(v);
    else if (f & EF_TANH) v = tanhf(v);
    return v;
}

template <int BM_, int BN_, int BK_, int WGM_, int WGN_, int WGK_>
struct LeanTile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_, WGK = WGK_;
    static constexpr int NT = WGM * WGN * WGK * kWave;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;
    static constexpr int TM = WTM / 32, TN = WTN / 32;
    static constexpr int G = BK / 8, GW = G / WGK;
    static constexpr int LDR = BK + 4, LDK = BN + 4;
    static constexpr int A_V = BM * BK / 4 / NT, B_V = BN * BK / 4 / NT;
    static constexpr int SMEM_A = BM * LDR;
    static constexpr int SMEM_B = (BN * LDR > BK * LDK) ? BN * LDR : BK * LDK;
    static constexpr int RED_WAVES = WGK > 8 ? 8 : WGK;
    static constexpr int PER_WAVE = TM * TN * 16 * kWave;
    static constexpr int RED = (WGK > 1) ? RED_WAVES * PER_WAVE : 0;
    static constexpr int STAGE = SMEM_A + SMEM_B;            // one operand buffer; the kernel keeps two
    static constexpr int SMEM = (2 * STAGE > RED) ? 2 * STAGE : RED;
    static constexpr int EPT = (WGK > 1) ? PER_WAVE / NT : 0;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && BK % 8 == 0 && G % WGK == 0, "tile shape");
    static_assert(BM * BK / 4 % NT == 0 && BN * BK / 4 % NT == 0, "tile must divide among the threads");
    static_assert(WGK == 1 || (WGM == 1 && WGN == 1 && PER_WAVE % NT == 0), "K-split tiles are one wave tile");
    static_assert(WGK <= 16, "at most two reduction rounds");
};

using LTileS = LeanTile<32, 32, 64, 1, 1, 4>;
using LTileS8 = LeanTile<32, 32, 128, 1, 1, 8>;
using LTileS16 = LeanTile<32, 32, 128, 1, 1, 16>;
using LTileM = LeanTile<64, 64, 64, 2, 2, 1>;
using LTileL = LeanTile<128, 128, 32, 2, 2, 1>;

// K-waves of a 32x32 tile: park the accumulators in LDS (16-wave tiles fold the
// upper eight waves into the lower eight first), so that afterwards output e of
// the tile is the sum over w < RED_WAVES of red[w * PER_WAVE + e], added in wave
// order.  `red` may alias the operand buffers: the caller guarantees they are
// no longer read.  Ends on a barrier.
template <class T>
__device__ __forceinline__ void park_k_waves(float *red, floatx16 acc, int wk, int lane) {
    if (T::WGK > 8) {
        if (wk >= 8) {
#pragma unroll
            for (int r = 0; r < 16; ++r) red[(wk - 8) * T::PER_WAVE + r * kWave + lane] = acc[r];
        }
        __syncthreads();
        if (wk < 8 && wk + 8 < T::WGK) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] += red[wk * T::PER_WAVE + r * kWave + lane];
        }
        __syncthreads();
    }
    if (wk < T::RED_WAVES) {
#pragma unroll
        for (int r = 0; r < 16; ++r) red[wk * T::PER_WAVE + r * kWave + lane] = acc[r];
    }
    __syncthreads();
}

template <class T>
__device__ __forceinline__ float sum_k_waves(const float *red, int e) {
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < T::RED_WAVES; ++w) v += red[w * T::PER_WAVE + e];
    return v;
}

// ---- matrix product -----------------------------------------------------------------------
// MODE F_NT: A[M,K], B[N,K]; F_NN: A[M,K], B[K,N].  Requires K % BK == 0, lda,
// ldb, batch strides multiples of 4, 16-byte aligned A and B, and for F_NN
// N % 4 == 0 (so that clamped 16-byte column chunks stay inside a row).
template <int MODE, class T>
__global__ __launch_bounds__(T::NT) void mm_lean_kernel(GemmArgs p) {
    extern __shared__ float smem[];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int wk = wave % T::WGK;
    const int wj = (wave / T::WGK) % T::WGN;
    const int wi = wave / (T::WGK * T::WGN);
    const int half = lane >> 5, l32 = lane & 31;

    const int tiles_n = (p.N + T::BN - 1) / T::BN;
    const int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int i0 = (tile / tiles_n) * T::BM, j0 = (tile % tiles_n) * T::BN;
    const int batch = blockIdx.y;
    const int ks = blockIdx.z;
    const int slices = p.K / T::BK;
    const int per = (slices + p.splitk - 1) / p.splitk;
    const int s_begin = ks * per, s_end = min(slices, s_begin + per);

    const float *const A = p.A + (int64_t)batch * p.strideA + (int64_t)s_begin * T::BK;
    const float *const B = p.B + (int64_t)batch * p.strideB +
                     (MODE == F_NN ? (int64_t)s_begin * T::BK * p.ldb : (int64_t)s_begin * T::BK);
    const int64_t b_step = (MODE == F_NN) ? (int64_t)T::BK * p.ldb : (int64_t)T::BK;

    // per-thread load descriptors: global offset (floats) and LDS slot (floats)
    int offA[T::A_V], offB[T::B_V];
#pragma unroll
    for (int r = 0; r < T::A_V; ++r) {
        const int e = tid + r * T::NT;
        offA[r] = min(i0 + e / (T::BK / 4), p.M - 1) * p.lda + (e % (T::BK / 4)) * 4;
    }
#pragma unroll
    for (int r = 0; r < T::B_V; ++r) {
        const int e = tid + r * T::NT;
        if (MODE == F_NT)
            offB[r] = min(j0 + e / (T::BK / 4), p.N - 1) * p.ldb + (e % (T::BK / 4)) * 4;
        else
            offB[r] = (e / (T::BN / 4)) * p.ldb + min(j0 + (e % (T::BN / 4)) * 4, p.N - 4);
    }

    // outputs this thread finishes (K-split tiles) and the operands of their tail
    constexpr int EPT = T::EPT > 0 ? T::EPT : 1;
    int64_t e_off[EPT];
    float e_bias[EPT], e_add[EPT];
    int e_chan[EPT];
    if constexpr (T::WGK > 1) {
#pragma unroll
        for (int t = 0; t < EPT; ++t) {
            const int e = tid + t * T::NT;
            const int l = e % kWave, r = e / kWave;
            const int i = i0 + 8 * (r / 4) + 4 * (l / 32) + (r % 4), j = j0 + (l & 31);
            // cs_len: column j lives in block j / cs_len of the output (a result stored split into heads)
            const int64_t jo = p.cs_len ? (int64_t)(j / p.cs_len) * p.cs_stride + j % p.cs_len : j;
            e_off[t] = (i < p.M && j < p.N) ? (int64_t)batch * p.strideC + (int64_t)i * p.ldc + jo : -1;
            e_chan[t] = p.bias_on_row ? i : j;
            e_bias[t] = 0.f;
            e_add[t] = 0.f;
            if (p.splitk == 1 && e_off[t] >= 0) {
                if (p.ef.flags & EF_BIAS) e_bias[t] = p.ef.bias[e_chan[t]];
                if (p.ef.flags & EF_ADD) e_add[t] = p.ef.add[e_off[t]];
            }
        }
    }

    // Software pipeline over the K slices of this workgroup: two LDS operand
    // buffers and two register sets.  While slice n is multiplied out of LDS
    // buffer n%2, slice n+1 moves from registers to the other buffer and the
    // loads of slice n+3 are issued, so a load has two slices of MFMA work to
    // arrive and there is one barrier per slice.  Loads past the last slice are
    // clamped to it (in bounds, unused), which keeps the loop free of branches.
    const int nsl = s_end - s_begin;
    f32x4 ra[2][T::A_V], rb[2][T::B_V];
#define CLG_MM_LOAD(set, n)                                                                     \
    do {                                                                                        \
        const int sl_ = min((n), nsl - 1);                                                      \
        const float *a_ = A + (int64_t)sl_ * T::BK;                                             \
        const float *b_ = B + (int64_t)sl_ * b_step;                                            \
        _Pragma("unroll") for (int r = 0; r < T::A_V; ++r)                                      \
            ra[set][r] = *reinterpret_cast<const f32x4 *>(a_ + offA[r]);                        \
        _Pragma("unroll") for (int r = 0; r < T::B_V; ++r)                                      \
            rb[set][r] = *reinterpret_cast<const f32x4 *>(b_ + offB[r]);                        \
        __builtin_amdgcn_sched_barrier(0);   /* keep the loads ahead of the MFMAs */            \
    } while (0)
#define CLG_MM_STORE(set, buf)                                                                  \
    do {                                                                                        \
        float *as_ = smem + (buf) * T::STAGE, *bs_ = as_ + T::SMEM_A;                            \
        _Pragma("unroll") for (int r = 0; r < T::A_V; ++r) {                                    \
            const int e = tid + r * T::NT;                                                      \
            *reinterpret_cast<f32x4 *>(&as_[(e / (T::BK / 4)) * T::LDR + (e % (T::BK / 4)) * 4]) = ra[set][r]; \
        }                                                                                       \
        _Pragma("unroll") for (int r = 0; r < T::B_V; ++r) {                                    \
            const int e = tid + r * T::NT;                                                      \
            if (MODE == F_NT)                                                                   \
                *reinterpret_cast<f32x4 *>(&bs_[(e / (T::BK / 4)) * T::LDR + (e % (T::BK / 4)) * 4]) = rb[set][r]; \
            else                                                                                \
                *reinterpret_cast<f32x4 *>(&bs_[(e / (T::BN / 4)) * T::LDK + (e % (T::BN / 4)) * 4]) = rb[set][r]; \
        }                                                                                       \
    } while (0)

    floatx16 acc[T::TM][T::TN];
#pragma unroll
    for (int tm = 0; tm < T::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < T::TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tm][tn][r] = 0.f;

    auto multiply = [&](int buf) {
        const float *As = smem + buf * T::STAGE;
        const float *Bs = As + T::SMEM_A;
#pragma unroll
        for (int gg = 0; gg < T::GW; ++gg) {
            const int kb = (wk * T::GW + gg) * 8 + 4 * half;
            float fa[T::TM][4], fb[T::TN][4];
#pragma unroll
            for (int tm = 0; tm < T::TM; ++tm) {
                const f32x4 v = *reinterpret_cast<const f32x4 *>(&As[(wi * T::WTM + tm * 32 + l32) * T::LDR + kb]);
                fa[tm][0] = v[0]; fa[tm][1] = v[1]; fa[tm][2] = v[2]; fa[tm][3] = v[3];
            }
#pragma unroll
            for (int tn = 0; tn < T::TN; ++tn) {
                if (MODE == F_NT) {
                    const f32x4 v = *reinterpret_cast<const f32x4 *>(&Bs[(wj * T::WTN + tn * 32 + l32) * T::LDR + kb]);
                    fb[tn][0] = v[0]; fb[tn][1] = v[1]; fb[tn][2] = v[2]; fb[tn][3] = v[3];
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q) fb[tn][q] = Bs[(kb + q) * T::LDK + wj * T::WTN + tn * 32 + l32];
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int tm = 0; tm < T::TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < T::TN; ++tn)
                        acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[tm][q], fb[tn][q], acc[tm][tn], 0, 0, 0);
        }
    };

    if (nsl > 0) {
        CLG_MM_LOAD(0, 0);
        CLG_MM_LOAD(1, 1);
        CLG_MM_STORE(0, 0);
        CLG_MM_LOAD(0, 2);
        __syncthreads();
        int n = 0;
        for (; n + 1 < nsl; n += 2) {    // two slices per trip, no branch inside
            CLG_MM_STORE(1, 1);          // slice n+1
            CLG_MM_LOAD(1, n + 3);
            multiply(0);                 // slice n
            __syncthreads();
            CLG_MM_STORE(0, 0);          // slice n+2 (a clamped repeat after the last one: unused)
            CLG_MM_LOAD(0, n + 4);
            multiply(1);                 // slice n+1
            __syncthreads();
        }
        if (n < nsl) multiply(0);        // odd count: the last slice sits in buffer 0
        __syncthreads();
    }
#undef CLG_MM_LOAD
#undef CLG_MM_STORE

    if constexpr (T::WGK > 1) {
        park_k_waves<T>(smem, acc[0][0], wk, lane);
#pragma unroll
        for (int t = 0; t < T::EPT; ++t) {
            const float v = sum_k_waves<T>(smem, tid + t * T::NT);
            if (e_off[t] >= 0) {
                if (p.splitk > 1) p.partial[(int64_t)ks * p.c_numel + e_off[t]] = v;
                else p.C[e_off[t]] = finish_value(p, v, e_bias[t], e_add[t]);
            }
        }
    } else {
        const int64_t c_batch = (int64_t)batch * p.strideC;
        const int f = p.ef.flags;
#pragma unroll
        for (int tm = 0; tm < T::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < T::TN; ++tn) {
                const int j = j0 + wj * T::WTN + tn * 32 + l32;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int i = i0 + wi * T::WTM + tm * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                    if (i >= p.M || j >= p.N) continue;
                    const int64_t off = c_batch + (int64_t)i * p.ldc + j;
                    if (p.splitk > 1) {
                        p.partial[(int64_t)ks * p.c_numel + off] = acc[tm][tn][r];
                    } else {
                        const int chan = p.bias_on_row ? i : j;
                        const float bv = (f & EF_BIAS) ? p.ef.bias[chan] : 0.f;
                        const float av = (f & EF_ADD) ? p.ef.add[off] : 0.f;
                        p.C[off] = finish_value(p, acc[tm][tn][r], bv, av);
                    }
                }
            }
    }
}

// ---- 3x3 convolution -------------------------------------------------------------------------
// One workgroup: 32 output channels x 32 consecutive output pixels of one image,
// WGK waves.  A K-slice is 4*WGK input channels (36*WGK values of k): the
// weights [32][36*WGK] go to LDS as they lie in memory, the input patch of those
// channels ([4*WGK][PSZ], PSZ = patch rows x (W + 2*pad), zero where the
// padding is) next to them.  Wave w multiplies channels 4w..4w+3 of the slice:
// for c in {0,1} and each tap, one MFMA whose k-slot h is channel c + 2h.
// Requires Cin % (4*WGK) == 0, 16-byte aligned weights, PSZ <= NP * NT.
template <int S_, int WGK_, int NP_>
struct Conv3Cfg {
    static constexpr int WGK = WGK_;
    static constexpr int NT = WGK * kWave;
    static constexpr int CS = 4 * WGK;            // channels per slice
    static constexpr int KS = CS * 9;             // k per slice
    static constexpr int LDA = KS + 4;
    static constexpr int A_CHUNKS = 32 * KS / 4;  // f32x4 per slice
    static constexpr int A_V = (A_CHUNKS + NT - 1) / NT;
    static constexpr int RED_WAVES = WGK > 8 ? 8 : WGK;
    static constexpr int PER_WAVE = 16 * kWave;
    static constexpr int EPT = PER_WAVE / NT;
    static constexpr int SMEM_A = 32 * LDA;
};

template <int S, int WGK, int NP>
__global__ __launch_bounds__(WGK *kWave) void conv3x3_lean_kernel(GemmArgs p) {
    using T = Conv3Cfg<S, WGK, NP>;
    extern __shared__ float smem[];
    float *As = smem;
    float *Ps = smem + T::SMEM_A;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wk = tid / kWave;
    const int half = lane >> 5, l32 = lane & 31;

    const int npix = p.HO * p.WO;
    const int tiles_n = (npix + 31) / 32;
    const int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int i0 = (tile / tiles_n) * 32, j0 = (tile % tiles_n) * 32;
    const int img = blockIdx.y;
    const int ks = blockIdx.z;
    const int slices = p.Cin / T::CS;
    const int per = (slices + p.splitk - 1) / p.splitk;
    const int s_begin = ks * per, s_end = min(slices, s_begin + per);

    const int PW = p.W + 2 * p.pw;
    const int PSZ = p.patch_sz;                      // floats per channel in the LDS patch
    const int oh_lo = j0 / p.WO;
    const int ih_lo = oh_lo * S - p.ph;
    const int hw_in = p.H * p.W;

    const float *Wt = p.A + (int64_t)s_begin * T::KS;                                        // weights [Cout][Cin*9]
    const float *X = p.B + ((int64_t)img * p.Cin + (int64_t)s_begin * T::CS) * hw_in;        // input image
    // weights: f32x4 chunk e -> row e / (KS/4), k-chunk e % (KS/4)
    int offA[T::A_V];
#pragma unroll
    for (int r = 0; r < T::A_V; ++r) {
        const int e = min(tid + r * T::NT, T::A_CHUNKS - 1);
        offA[r] = min(i0 + e / (T::KS / 4), p.Cout - 1) * p.K + (e % (T::KS / 4)) * 4;
    }
    // patch: position -> (row, x) of the padded window, fixed for the whole kernel
    int goff[NP];
    bool gok[NP];
#pragma unroll
    for (int n = 0; n < NP; ++n) {
        const int pos = tid + n * T::NT;
        const int r = pos / PW, x = pos - r * PW;
        const int ih = ih_lo + r, iw = x - p.pw;
        gok[n] = pos < PSZ && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
        goff[n] = gok[n] ? ih * p.W + iw : 0;
    }
    // this lane's pixel and fragment bases
    const int jp = min(j0 + l32, npix - 1);
    const int oh = jp / p.WO, ow = jp - oh * p.WO;
    const int b_base = (oh - oh_lo) * S * PW + ow * S + (wk * 4 + 2 * half) * PSZ;
    const int a_base = l32 * T::LDA + (wk * 4 + 2 * half) * 9;

    // outputs this thread finishes and the operands of their tail
    int64_t e_off[T::EPT];
    float e_bias[T::EPT], e_add[T::EPT];
    int e_chan[T::EPT];
#pragma unroll
    for (int t = 0; t < T::EPT; ++t) {
        const int e = tid + t * T::NT;
        const int l = e % kWave, r = e / kWave;
        const int i = i0 + 8 * (r / 4) + 4 * (l / 32) + (r % 4), j = j0 + (l & 31);
        e_off[t] = (i < p.Cout && j < npix) ? ((int64_t)img * p.Cout + i) * npix + j : -1;
        e_chan[t] = i;
        e_bias[t] = 0.f;
        e_add[t] = 0.f;
        if (p.splitk == 1 && e_off[t] >= 0) {
            if (p.ef.flags & EF_BIAS) e_bias[t] = p.ef.bias[i];
            if (p.ef.flags & EF_ADD) e_add[t] = p.ef.add[e_off[t]];
        }
    }

    f32x4 ra[T::A_V];
    float rp[NP][T::CS];
    auto load_slice = [&]() {
#pragma unroll
        for (int r = 0; r < T::A_V; ++r) ra[r] = *reinterpret_cast<const f32x4 *>(Wt + offA[r]);
#pragma unroll
        for (int n = 0; n < NP; ++n)
#pragma unroll
            for (int c = 0; c < T::CS; ++c) {
                const float v = X[c * hw_in + goff[n]];      // goff = 0 (in bounds) where the padding is
                rp[n][c] = gok[n] ? v : 0.f;
            }
    };
    auto store_slice = [&]() {
#pragma unroll
        for (int r = 0; r < T::A_V; ++r) {
            const int e = tid + r * T::NT;
            if (e < T::A_CHUNKS)
                *reinterpret_cast<f32x4 *>(&As[(e / (T::KS / 4)) * T::LDA + (e % (T::KS / 4)) * 4]) = ra[r];
        }
#pragma unroll
        for (int n = 0; n < NP; ++n) {
            const int pos = tid + n * T::NT;
            if (pos < PSZ) {
#pragma unroll
                for (int c = 0; c < T::CS; ++c) Ps[c * PSZ + pos] = rp[n][c];
            }
        }
    };

    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;

    if (s_begin < s_end) load_slice();
    for (int s = s_begin; s < s_end; ++s) {
        store_slice();
        __syncthreads();
        if (s + 1 < s_end) {
            Wt += T::KS;
            X += (int64_t)T::CS * hw_in;
            load_slice();
        }
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) {
                const float *brow = Ps + b_base + c * PSZ + kh * PW;
                const float *arow = As + a_base + c * 9 + kh * 3;
#pragma unroll
                for (int kw = 0; kw < 3; ++kw)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(arow[kw], brow[kw], acc, 0, 0, 0);
            }
        __syncthreads();
    }

    park_k_waves<T>(smem, acc, wk, lane);
#pragma unroll
    for (int t = 0; t < T::EPT; ++t) {
        const float v = sum_k_waves<T>(smem, tid + t * T::NT);
        if (e_off[t] >= 0) {
            if (p.splitk > 1) p.partial[(int64_t)ks * p.c_numel + e_off[t]] = v;
            else p.C[e_off[t]] = finish_value(p, v, e_bias[t], e_add[t]);
        }
    }
}

// Launchers (gemm_lean_mm.hip / gemm_lean_conv.hip).  Return -1 when the shape
// is not eligible for a lean kernel (the caller then uses the general one).
int launch_lean_mm(const GemmArgs &a, hipStream_t s);
int launch_lean_conv3x3(const GemmArgs &a, hipStream_t s);

}  // namespace clg
