// Tuned fp32 MFMA GEMM / implicit-GEMM convolution kernel for gfx950.
//
// The contractions of the workloads (paper Sec. 5.1) at batch 1 are small:
// what bounds them is memory latency and the number of workgroups, not MFMA
// throughput.  The kernel is built around that:
//  * K is consumed in big slices (BK = 64, or 32 for the 128x128 tile): each
//    thread has 8-32 floats of loads in flight before the first wait, and a
//    workgroup needs few dependent round trips to memory;
//  * the slice s+1 is fetched into registers while slice s is multiplied out of
//    LDS (one LDS buffer, register prefetch);
//  * operands are loaded with 16-byte accesses along their contiguous
//    dimension and keep that orientation in LDS, so no transposing stores:
//    a K-contiguous operand (weights, dense inputs) is stored [row][k] and its
//    MFMA fragments are read as one ds_read_b128 per four MFMAs; a row-contiguous
//    operand (activations of a convolution, B of a NN matmul) is stored [k][col]
//    and read as conflict-free ds_read_b32.  Both agree on the slot mapping
//    "lane half h, MFMA q of a group of four -> k = 8*g + 4*h + q";
//  * the im2col gather of a convolution is done on the fly: each thread owns
//    one output pixel for the whole kernel (its padding mask is a bit field
//    computed once) and walks the (channel, tap) index with constant divisors;
//  * workgroup ids are remapped so that consecutive tiles, which share weights
//    and overlapping input windows, run on the same XCD and meet in its L2.
#pragma once

#include <hip/hip_runtime.h>

#include "device_common.h"

namespace clg {

typedef float floatx16 __attribute__((ext_vector_type(16)));

enum FastMode : int { F_NT = 0, F_NN = 1, F_CONV = 2 };

template <int BM_, int BN_, int BK_, int WGM_, int WGN_, int WGK_, int PD_>
struct FastTile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_, WGK = WGK_;
    static constexpr int PD = PD_;                          // K slices whose loads are in flight at once
    static constexpr int NT = WGM * WGN * WGK * kWave;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;
    static constexpr int TM = WTM / 32, TN = WTN / 32;
    static constexpr int G = BK / 8, GW = G / WGK;          // k-groups of 8 per slice / per wave
    static constexpr int LDR = BK + 4;                      // [row][k] operands
    static constexpr int LDK = BN + 4;                      // [k][col] operand
    static constexpr int A_V = BM * BK / 4 / NT;            // float4 per thread
    static constexpr int B_V = BN * BK / 4 / NT;
    static constexpr int B_S = BK * BN / NT;                // scalars per thread (conv gather)
    static constexpr int SMEM_A = BM * LDR;
    static constexpr int SMEM_B = (BN * LDR > BK * LDK) ? BN * LDR : BK * LDK;
    static constexpr int RED_WAVES = WGK > 8 ? 8 : WGK;     // waves whose accumulators sit in LDS at once
    static constexpr int RED = (WGK > 1) ? RED_WAVES * TM * TN * 16 * kWave : 0;
    static constexpr int SMEM = (SMEM_A + SMEM_B > RED) ? SMEM_A + SMEM_B : RED;
    static constexpr int EPT = (WGK > 1) ? TM * TN * 16 * kWave / NT : 0;   // outputs per thread after the K-wave sum
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");
    static_assert(BM * BK / 4 % NT == 0 && BN * BK / 4 % NT == 0, "tile must divide among the threads");
    static_assert(NT % BN == 0 && G % WGK == 0 && BK % 8 == 0, "tile shape");
    static_assert(WGK == 1 || (WGM == 1 && WGN == 1 && TM * TN * 16 * kWave % NT == 0), "K-split tiles are one wave tile");
    static_assert(WGK <= 16, "at most two reduction rounds");
};

using FTileS = FastTile<32, 32, 64, 1, 1, 4, 1>;       // 4 waves share K inside the workgroup
using FTileM = FastTile<64, 64, 64, 2, 2, 1, 1>;
using FTileL = FastTile<128, 128, 32, 2, 2, 1, 1>;

// blockIdx.x -> tile index such that the ids an XCD receives (id % 8 under
// round-robin dispatch) form one contiguous range of tiles.
__device__ __forceinline__ int xcd_remap(int id, int n) {
    const int q = n / 8, r = n % 8;
    const int xcd = id % 8, idx = id / 8;
    return xcd * q + (xcd < r ? xcd : r) + idx;
}

template <int MODE, int KH, int KW, bool VEC, class T>
__global__ __launch_bounds__(T::NT) void gemm_fast_kernel(GemmArgs p) {
    extern __shared__ float smem[];
    float *As = smem;
    float *Bs = smem + T::SMEM_A;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int wk = wave % T::WGK;
    const int wj = (wave / T::WGK) % T::WGN;
    const int wi = wave / (T::WGK * T::WGN);
    const int half = lane >> 5, l32 = lane & 31;

    const int tiles_n = (p.N + T::BN - 1) / T::BN;
    const int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int tile_i = tile / tiles_n, tile_j = tile % tiles_n;
    const int i0 = tile_i * T::BM, j0 = tile_j * T::BN;
    const int batch = blockIdx.y;
    const int ks = blockIdx.z;
    const int slices = (p.K + T::BK - 1) / T::BK;
    const int per = (slices + p.splitk - 1) / p.splitk;
    const int s_begin = ks * per, s_end = min(slices, s_begin + per);

    const float *A = p.A + (int64_t)batch * p.strideA;
    const float *B = p.B + (int64_t)batch * p.strideB;

    // ---- convolution: this thread's output pixel, fixed for the whole kernel
    constexpr int KHc = KH, KWc = KW;
    const int kh_n = KHc > 0 ? KHc : p.KH, kw_n = KWc > 0 ? KWc : p.KW;
    const int taps = kh_n * kw_n;
    int64_t xoff = 0;
    uint64_t mask = 0;
    const int jl = tid % T::BN;
    if (MODE == F_CONV) {
        const int j = j0 + jl;
        const int hw = p.HO * p.WO;
        const int n = j / hw, q = j - n * hw;
        const int oh = q / p.WO, ow = q - oh * p.WO;
        const int ih0 = oh * p.sh - p.ph, iw0 = ow * p.sw - p.pw;
        xoff = ((int64_t)n * p.Cin * p.H + ih0) * p.W + iw0;
        if (j < p.N)
            for (int kh = 0; kh < kh_n; ++kh)
                for (int kw = 0; kw < kw_n; ++kw)
                    if (ih0 + kh >= 0 && ih0 + kh < p.H && iw0 + kw >= 0 && iw0 + kw < p.W)
                        mask |= (uint64_t)1 << (kh * kw_n + kw);
    }

    // ---- K-split tiles: the outputs this thread will finish are known now, so the
    // operands of their fused steps (bias, residual) are fetched before the main
    // loop instead of at its end, where their latency would be exposed
    constexpr int EPT = T::EPT > 0 ? T::EPT : 1;
    int64_t e_off[EPT];
    int e_chan[EPT];
    float e_pre[EPT][kMaxEpi];
    if (T::WGK > 1) {
#pragma unroll
        for (int t = 0; t < EPT; ++t) {
            const int e = tid + t * T::NT;
            const int l = e % kWave, r = (e / kWave) % 16, blk = e / (16 * kWave);
            const int i = i0 + (blk / T::TN) * 32 + 8 * (r / 4) + 4 * (l / 32) + (r % 4);
            const int j = j0 + (blk % T::TN) * 32 + (l & 31);
            e_off[t] = -1;
            e_chan[t] = p.bias_on_row ? i : j;
            if (i < p.M && j < p.N) {
                if (MODE == F_CONV) {
                    const int hw = p.HO * p.WO;
                    const int n = j / hw, q = j - n * hw;
                    e_off[t] = ((int64_t)n * p.Cout + i) * hw + q;
                } else {
                    e_off[t] = (int64_t)batch * p.strideC + (int64_t)i * p.ldc + j;
                }
            }
#pragma unroll
            for (int st = 0; st < kMaxEpi; ++st) {
                float v = 0.f;
                if (p.splitk == 1 && st < p.epi.n && e_off[t] >= 0) {
                    if (p.epi.s[st].op == EPI_BIAS) v = p.epi.s[st].ptr[e_chan[t]];
                    else if (p.epi.s[st].op == EPI_ADD) v = p.epi.s[st].ptr[e_off[t]];
                }
                e_pre[t][st] = v;
            }
        }
    }

    // register staging: PD slices deep
    float4 ra[T::PD][T::A_V];
    float4 rb[T::PD][(MODE == F_CONV) ? 1 : T::B_V];
    float rs[T::PD][(MODE == F_CONV) ? T::B_S : 1];

    auto load_rows = [&](const float *base, int ld, int row0, int rows, int k0, float4 *dst, int count) {
        // [row][k] operand: float4 e covers row e / (BK/4), k-chunk e % (BK/4)
#pragma unroll
        for (int r = 0; r < count; ++r) {
            const int e = tid + r * T::NT;
            const int row = row0 + e / (T::BK / 4), k = k0 + (e % (T::BK / 4)) * 4;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < rows) {
                const float *src = base + (int64_t)row * ld + k;
                if (VEC) {
                    if (k < p.K) v = *reinterpret_cast<const float4 *>(src);
                } else {
                    if (k < p.K) v.x = src[0];
                    if (k + 1 < p.K) v.y = src[1];
                    if (k + 2 < p.K) v.z = src[2];
                    if (k + 3 < p.K) v.w = src[3];
                }
            }
            dst[r] = v;
        }
    };
    auto load_slice = [&](int s, float4 *ra, float4 *rb, float *rs) {
        const int k0 = s * T::BK;
        load_rows(A, p.lda, i0, p.M, k0, ra, T::A_V);
        if (MODE == F_NT) {
            load_rows(B, p.ldb, j0, p.N, k0, rb, T::B_V);
        } else if (MODE == F_NN) {
#pragma unroll
            for (int r = 0; r < T::B_V; ++r) {
                const int e = tid + r * T::NT;
                const int k = k0 + e / (T::BN / 4), j = j0 + (e % (T::BN / 4)) * 4;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (k < p.K) {
                    const float *src = B + (int64_t)k * p.ldb + j;
                    if (VEC) {
                        if (j < p.N) v = *reinterpret_cast<const float4 *>(src);
                    } else {
                        if (j < p.N) v.x = src[0];
                        if (j + 1 < p.N) v.y = src[1];
                        if (j + 2 < p.N) v.z = src[2];
                        if (j + 3 < p.N) v.w = src[3];
                    }
                }
                rb[r] = v;
            }
        } else {
            const int64_t chw = (int64_t)p.H * p.W;
#pragma unroll
            for (int r = 0; r < T::B_S; ++r) {
                const int k = k0 + tid / T::BN + r * (T::NT / T::BN);
                const int ci = k / taps, t = k - ci * taps;
                const int kh = t / kw_n, kw = t - kh * kw_n;
                float v = 0.f;
                if (k < p.K && ((mask >> t) & 1)) v = B[xoff + ci * chw + kh * p.W + kw];
                rs[r] = v;
            }
        }
    };
    auto store_slice = [&](const float4 *ra, const float4 *rb, const float *rs) {
#pragma unroll
        for (int r = 0; r < T::A_V; ++r) {
            const int e = tid + r * T::NT;
            *reinterpret_cast<float4 *>(&As[(e / (T::BK / 4)) * T::LDR + (e % (T::BK / 4)) * 4]) = ra[r];
        }
        if (MODE == F_NT) {
#pragma unroll
            for (int r = 0; r < T::B_V; ++r) {
                const int e = tid + r * T::NT;
                *reinterpret_cast<float4 *>(&Bs[(e / (T::BK / 4)) * T::LDR + (e % (T::BK / 4)) * 4]) = rb[r];
            }
        } else if (MODE == F_NN) {
#pragma unroll
            for (int r = 0; r < T::B_V; ++r) {
                const int e = tid + r * T::NT;
                *reinterpret_cast<float4 *>(&Bs[(e / (T::BN / 4)) * T::LDK + (e % (T::BN / 4)) * 4]) = rb[r];
            }
        } else {
#pragma unroll
            for (int r = 0; r < T::B_S; ++r)
                Bs[(tid / T::BN + r * (T::NT / T::BN)) * T::LDK + jl] = rs[r];
        }
    };

    floatx16 acc[T::TM][T::TN];
#pragma unroll
    for (int tm = 0; tm < T::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < T::TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tm][tn][r] = 0.f;

    auto multiply_slice = [&]() {
#pragma unroll
        for (int gg = 0; gg < T::GW; ++gg) {
            const int kb = (wk * T::GW + gg) * 8 + 4 * half;
            float fa[T::TM][4], fb[T::TN][4];
#pragma unroll
            for (int tm = 0; tm < T::TM; ++tm) {
                const float4 v = *reinterpret_cast<const float4 *>(&As[(wi * T::WTM + tm * 32 + l32) * T::LDR + kb]);
                fa[tm][0] = v.x; fa[tm][1] = v.y; fa[tm][2] = v.z; fa[tm][3] = v.w;
            }
#pragma unroll
            for (int tn = 0; tn < T::TN; ++tn) {
                if (MODE == F_NT) {
                    const float4 v = *reinterpret_cast<const float4 *>(&Bs[(wj * T::WTN + tn * 32 + l32) * T::LDR + kb]);
                    fb[tn][0] = v.x; fb[tn][1] = v.y; fb[tn][2] = v.z; fb[tn][3] = v.w;
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

    // software pipeline over K: the loads of the next PD slices are always in
    // flight, so a workgroup pays the memory latency about once, not per slice
#pragma unroll
    for (int d = 0; d < T::PD; ++d)
        if (s_begin + d < s_end) load_slice(s_begin + d, ra[d], rb[d], rs[d]);
    for (int s = s_begin; s < s_end; s += T::PD) {
#pragma unroll
        for (int d = 0; d < T::PD; ++d) {
            if (s + d < s_end) {
                store_slice(ra[d], rb[d], rs[d]);
                __syncthreads();
                if (s + d + T::PD < s_end) load_slice(s + d + T::PD, ra[d], rb[d], rs[d]);
                multiply_slice();
                __syncthreads();
            }
        }
    }

    // ---- write-back: accumulator register r of lane l is row 8*(r/4) + 4*(l/32) + r%4,
    // column l%32 of its 32x32 block
    const int64_t c_batch = (int64_t)batch * p.strideC;
    auto emit = [&](int i, int j, float v) {
        if (i >= p.M || j >= p.N) return;
        int64_t off;
        if (MODE == F_CONV) {
            const int hw = p.HO * p.WO;
            const int n = j / hw, q = j - n * hw;
            off = ((int64_t)n * p.Cout + i) * hw + q;
        } else {
            off = c_batch + (int64_t)i * p.ldc + j;
        }
        if (p.splitk > 1)
            p.partial[(int64_t)ks * p.c_numel + off] = v;
        else
            p.C[off] = apply_steps(p.epi, v, off, p.bias_on_row ? i : j);
    };
    if (T::WGK == 1) {
#pragma unroll
        for (int tm = 0; tm < T::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < T::TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    emit(i0 + wi * T::WTM + tm * 32 + 8 * (r / 4) + 4 * half + (r % 4),
                         j0 + wj * T::WTN + tn * 32 + l32, acc[tm][tn][r]);
    } else {
        float *red = smem;      // operand buffers are dead: the loop ended on a barrier
        constexpr int PER_WAVE = T::TM * T::TN * 16 * kWave;
        if (T::WGK > 8) {
            // first round: waves 8.. park their accumulators, waves 0..7 add their partner's
            if (wk >= 8) {
#pragma unroll
                for (int tm = 0; tm < T::TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < T::TN; ++tn)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            red[(wk - 8) * PER_WAVE + ((tm * T::TN + tn) * 16 + r) * kWave + lane] = acc[tm][tn][r];
            }
            __syncthreads();
            if (wk < 8 && wk + 8 < T::WGK) {
#pragma unroll
                for (int tm = 0; tm < T::TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < T::TN; ++tn)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            acc[tm][tn][r] += red[wk * PER_WAVE + ((tm * T::TN + tn) * 16 + r) * kWave + lane];
            }
            __syncthreads();
        }
        if (wk < T::RED_WAVES) {
#pragma unroll
            for (int tm = 0; tm < T::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < T::TN; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        red[wk * PER_WAVE + ((tm * T::TN + tn) * 16 + r) * kWave + lane] = acc[tm][tn][r];
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < EPT; ++t) {
            const int e = tid + t * T::NT;
            float v = 0.f;
#pragma unroll
            for (int w = 0; w < T::RED_WAVES; ++w) v += red[w * PER_WAVE + e];
            if (e_off[t] < 0) continue;
            if (p.splitk > 1) {
                p.partial[(int64_t)ks * p.c_numel + e_off[t]] = v;
            } else {
#pragma unroll
                for (int st = 0; st < kMaxEpi; ++st) {
                    if (st >= p.epi.n) break;
                    switch (p.epi.s[st].op) {
                    case EPI_BIAS: case EPI_ADD: v += e_pre[t][st]; break;
                    case EPI_RELU: v = v > 0.f ? v : 0.f; break;
                    case EPI_GELU: v = gelu_erf(v); break;
                    case EPI_TANH: v = tanhf(v); break;
                    case EPI_SCALE: v *= p.epi.s[st].scalar; break;
                    default: break;
                    }
                }
                p.C[e_off[t]] = v;
            }
        }
    }
}

template <int MODE, int KH, int KW, bool VEC, class T>
int launch_fast_tile(const GemmArgs &a, hipStream_t s) {
    const int tiles = ((a.M + T::BM - 1) / T::BM) * ((a.N + T::BN - 1) / T::BN);
    const dim3 grid(tiles, a.batch, a.splitk);
    hipLaunchKernelGGL((gemm_fast_kernel<MODE, KH, KW, VEC, T>), grid, dim3(T::NT), T::SMEM * sizeof(float), s, a);
    return (int)hipGetLastError();
}

template <int MODE, int KH, int KW, bool VEC>
int launch_fast(const GemmArgs &a, hipStream_t s) {
    switch (a.tile) {
    case TILE_S: case TILE_S8: case TILE_S16: return launch_fast_tile<MODE, KH, KW, VEC, FTileS>(a, s);
    case TILE_L: return launch_fast_tile<MODE, KH, KW, VEC, FTileL>(a, s);
    default: return launch_fast_tile<MODE, KH, KW, VEC, FTileM>(a, s);
    }
}

// defined in gemm_fast_mm.hip / gemm_fast_conv.hip
int launch_fast_mm(const GemmArgs &a, bool vec, hipStream_t s);
int launch_fast_conv(const GemmArgs &a, bool vec, hipStream_t s);

}  // namespace clg
