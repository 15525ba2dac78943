// fp32 MFMA implicit GEMM for gfx950: dense, batched matmul, convolution as
// implicit GEMM (M = Cout, N = output pixels, K = Cin*kh*kw) and transposed
// convolution as stride*stride sub-pixel phase GEMMs, with the fused
// elementwise epilogue applied to the accumulators in registers.
//
// These are the dense contractions of the workloads (paper Sec. 5.1:
// convolutions for vision models, matrix multiplications for transformers) and
// the fusions the placement search selects around them (Sec. 5.5: Conv+ReLU,
// Conv+Add+ReLU).  gfx950 has no reduced-precision-input fp32 MFMA, and the
// parity tolerance (1e-4) rules one out anyway: v_mfma_f32_32x32x2_f32.
//
// Structure of one workgroup: a BM x BN output tile; per BK-slice of K the A
// (BM x BK) and B (BK x BN) operands are gathered from global memory into
// registers, stored k-major into LDS (so that the 32 lanes of a half-wave read
// 32 consecutive floats for an MFMA operand: no bank conflicts), and consumed
// by WGM x WGN x WGK waves.  LDS is double-buffered: the global loads of slice
// t+1 are in flight while slice t is multiplied, one barrier per slice.  WGK > 1
// splits the K-slice between waves of the same tile (for tiles too small to
// give every SIMD work) and adds the partial accumulators in LDS in fixed
// order.  grid.z can split K across workgroups; partial tiles then go to a
// scratch buffer and a second kernel adds them in fixed order and applies the
// epilogue, so results do not depend on scheduling.
#include <algorithm>

#include <hip/hip_runtime.h>

#include "device_common.h"
#include "gemm_fast.h"
#include "gemm_lean.h"
#include "gemm_rf.h"

namespace clg {

namespace {

constexpr int kPad = 4;

template <int BM_, int BN_, int BK_, int WGM_, int WGN_, int WGK_>
struct TileCfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_, WGK = WGK_;
    static constexpr int NT = WGM * WGN * WGK * kWave;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;     // wave tile
    static constexpr int TM = WTM / 32, TN = WTN / 32;       // 32x32 MFMA blocks per wave
    static constexpr int KK = BK / 2 / WGK;                  // MFMA k-steps per wave per slice
    static constexpr int LDA = BM + kPad, LDB = BN + kPad;
    static constexpr int A_ELEMS = BM * BK, B_ELEMS = BK * BN;
    static constexpr int A_PER = A_ELEMS / NT, B_PER = B_ELEMS / NT;
    static constexpr int STAGE = BK * LDA + BK * LDB;        // floats per LDS buffer
    static constexpr int RED = (WGK > 1) ? WGK * TM * TN * 16 * kWave : 0;
    static constexpr int SMEM = (2 * STAGE > RED) ? 2 * STAGE : RED;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");
    static_assert(A_ELEMS % NT == 0 && B_ELEMS % NT == 0, "tile must divide among the threads");
    static_assert((BK / 2) % WGK == 0, "K-slice must divide among the K-waves");
};

using TileS = TileCfg<32, 32, 32, 1, 1, 4>;     // small tile, 4 waves share K
using TileM = TileCfg<64, 64, 16, 2, 2, 1>;
using TileL = TileCfg<128, 128, 16, 2, 2, 1>;

struct ConvGeom {            // per-thread decomposition of an output pixel index j
    int n, oh, ow;
};

// ---- operand element fetch (bounds-checked; out of range = 0) -----------------------
template <int MODE>
__device__ __forceinline__ float fetch_a(const GemmArgs &p, const float *A, int i, int k, int rh, int rw) {
    if (i >= p.M || k >= p.K) return 0.f;
    if (MODE == GM_CONVT) {
        const int tw = p.KW / p.sw, th = p.KH / p.sh;
        const int b = k % tw, a = (k / tw) % th, ci = k / (tw * th);
        const int kh = rh + p.sh * a, kw = rw + p.sw * b;
        return A[(((int64_t)ci * p.Cout + i) * p.KH + kh) * p.KW + kw];
    }
    return A[(int64_t)i * p.lda + k];
}

template <int MODE>
__device__ __forceinline__ float fetch_b(const GemmArgs &p, const float *B, int k, int j, const ConvGeom &g,
                                         int base_h, int base_w) {
    if (j >= p.N || k >= p.K) return 0.f;
    if (MODE == GM_NT) return B[(int64_t)j * p.ldb + k];
    if (MODE == GM_NN) return B[(int64_t)k * p.ldb + j];
    if (MODE == GM_CONV) {
        const int khw = p.KH * p.KW;
        const int ci = k / khw, r = k - ci * khw;
        const int kh = r / p.KW, kw = r - kh * p.KW;
        const int ih = g.oh * p.sh - p.ph + kh, iw = g.ow * p.sw - p.pw + kw;
        if (ih < 0 || ih >= p.H || iw < 0 || iw >= p.W) return 0.f;
        return B[(((int64_t)g.n * p.Cin + ci) * p.H + ih) * p.W + iw];
    }
    // GM_CONVT: g.oh / g.ow hold the phase-local pixel (th, tw)
    const int tw = p.KW / p.sw, th = p.KH / p.sh;
    const int b = k % tw, a = (k / tw) % th, ci = k / (tw * th);
    const int ih = g.oh + base_h - a, iw = g.ow + base_w - b;
    if (ih < 0 || ih >= p.H || iw < 0 || iw >= p.W) return 0.f;
    return B[(((int64_t)g.n * p.Cin + ci) * p.H + ih) * p.W + iw];
}

template <int MODE, class T>
__global__ __launch_bounds__(T::NT) void igemm_kernel(GemmArgs p) {
    extern __shared__ float smem[];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int wk = wave % T::WGK;
    const int wj = (wave / T::WGK) % T::WGN;
    const int wi = wave / (T::WGK * T::WGN);

    const int tiles_n = (p.N + T::BN - 1) / T::BN;
    const int tile_i = blockIdx.x / tiles_n, tile_j = blockIdx.x % tiles_n;
    const int i0 = tile_i * T::BM, j0 = tile_j * T::BN;
    const int batch = blockIdx.y;
    const int ks = blockIdx.z;

    // K range of this workgroup (split-K across grid.z in whole BK slices)
    const int slices = (p.K + T::BK - 1) / T::BK;
    const int per = (slices + p.splitk - 1) / p.splitk;
    const int s_begin = ks * per, s_end = min(slices, s_begin + per);

    const float *A = p.A, *B = p.B;
    int rh = 0, rw = 0, base_h = 0, base_w = 0, oh0 = 0, ow0 = 0;
    if (MODE == GM_CONVT) {
        // phase (rh, rw): output rows oh with (oh + ph) % sh == rh, taps kh = rh + sh*a
        rh = batch / p.sw;
        rw = batch % p.sw;
        oh0 = ((rh - p.ph) % p.sh + p.sh) % p.sh;
        ow0 = ((rw - p.pw) % p.sw + p.sw) % p.sw;
        base_h = (oh0 + p.ph - rh) / p.sh;
        base_w = (ow0 + p.pw - rw) / p.sw;
    } else {
        A += (int64_t)batch * p.strideA;
        B += (int64_t)batch * p.strideB;
    }

    // staging registers and the fixed part of each thread's addresses
    float ra[T::A_PER], rb[T::B_PER];
    // B: NT mode is K-contiguous like A; the others are j-contiguous
    constexpr bool B_KMAJOR = (MODE == GM_NT);
    ConvGeom geo[B_KMAJOR ? 1 : T::B_PER];
    if (MODE == GM_CONV || MODE == GM_CONVT) {
        const int wo = (MODE == GM_CONV) ? p.WO : p.WO / p.sw;
        const int ho = (MODE == GM_CONV) ? p.HO : p.HO / p.sh;
#pragma unroll
        for (int r = 0; r < T::B_PER; ++r) {
            const int e = tid + r * T::NT;
            const int j = j0 + e % T::BN;
            const int q = j % (ho * wo);
            geo[r].n = j / (ho * wo);
            geo[r].oh = q / wo;
            geo[r].ow = q % wo;
        }
    }

    auto load_slice = [&](int s) {
        const int k0 = s * T::BK;
#pragma unroll
        for (int r = 0; r < T::A_PER; ++r) {
            const int e = tid + r * T::NT;
            ra[r] = fetch_a<MODE>(p, A, i0 + e / T::BK, k0 + e % T::BK, rh, rw);
        }
#pragma unroll
        for (int r = 0; r < T::B_PER; ++r) {
            const int e = tid + r * T::NT;
            if (B_KMAJOR)
                rb[r] = fetch_b<MODE>(p, B, k0 + e % T::BK, j0 + e / T::BK, geo[0], 0, 0);
            else
                rb[r] = fetch_b<MODE>(p, B, k0 + e / T::BN, j0 + e % T::BN, geo[B_KMAJOR ? 0 : r], base_h, base_w);
        }
    };
    auto store_slice = [&](int buf) {
        float *As = smem + buf * T::STAGE;
        float *Bs = As + T::BK * T::LDA;
#pragma unroll
        for (int r = 0; r < T::A_PER; ++r) {
            const int e = tid + r * T::NT;
            As[(e % T::BK) * T::LDA + e / T::BK] = ra[r];
        }
#pragma unroll
        for (int r = 0; r < T::B_PER; ++r) {
            const int e = tid + r * T::NT;
            if (B_KMAJOR)
                Bs[(e % T::BK) * T::LDB + e / T::BK] = rb[r];
            else
                Bs[(e / T::BN) * T::LDB + e % T::BN] = rb[r];
        }
    };

    floatx16 acc[T::TM][T::TN];
#pragma unroll
    for (int tm = 0; tm < T::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < T::TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tm][tn][r] = 0.f;

    if (s_begin < s_end) {
        load_slice(s_begin);
        store_slice(0);
    }
    __syncthreads();
    for (int s = s_begin; s < s_end; ++s) {
        const int buf = (s - s_begin) & 1;
        if (s + 1 < s_end) load_slice(s + 1);
        const float *As = smem + buf * T::STAGE;
        const float *Bs = As + T::BK * T::LDA;
#pragma unroll
        for (int kk = 0; kk < T::KK; ++kk) {
            const int krow = (wk * T::KK + kk) * 2 + lane / 32;
            float fa[T::TM], fb[T::TN];
#pragma unroll
            for (int tm = 0; tm < T::TM; ++tm) fa[tm] = As[krow * T::LDA + wi * T::WTM + tm * 32 + (lane & 31)];
#pragma unroll
            for (int tn = 0; tn < T::TN; ++tn) fb[tn] = Bs[krow * T::LDB + wj * T::WTN + tn * 32 + (lane & 31)];
#pragma unroll
            for (int tm = 0; tm < T::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < T::TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[tm], fb[tn], acc[tm][tn], 0, 0, 0);
        }
        if (s + 1 < s_end) store_slice(buf ^ 1);
        __syncthreads();
    }

    // ---- write-back: accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4,
    // column l%32 of its 32x32 block
    const int64_t c_batch = (MODE == GM_CONVT) ? 0 : (int64_t)batch * p.strideC;
    auto emit = [&](int i, int j, float v) {
        if (i >= p.M || j >= p.N) return;
        int64_t off;
        if (MODE == GM_CONV) {
            const int hw = p.HO * p.WO;
            const int n = j / hw, q = j - n * hw;
            off = ((int64_t)n * p.Cout + i) * hw + q;
        } else if (MODE == GM_CONVT) {
            const int wo = p.WO / p.sw, ho = p.HO / p.sh;
            const int n = j / (ho * wo), q = j % (ho * wo);
            const int oh = oh0 + p.sh * (q / wo), ow = ow0 + p.sw * (q % wo);
            off = (((int64_t)n * p.Cout + i) * p.HO + oh) * p.WO + ow;
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
                for (int r = 0; r < 16; ++r) {
                    const int i = i0 + wi * T::WTM + tm * 32 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
                    const int j = j0 + wj * T::WTN + tn * 32 + (lane & 31);
                    emit(i, j, acc[tm][tn][r]);
                }
    } else {
        // K-waves of one tile: add their accumulators in LDS in wave order
        float *red = smem;          // the operand buffers are no longer read (barrier above)
        constexpr int PER_WAVE = T::TM * T::TN * 16 * kWave;
#pragma unroll
        for (int tm = 0; tm < T::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < T::TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    red[wk * PER_WAVE + ((tm * T::TN + tn) * 16 + r) * kWave + lane] = acc[tm][tn][r];
        __syncthreads();
        // WGM = WGN = 1 for the K-split tile: every thread sums a share of the tile
        for (int e = tid; e < PER_WAVE; e += T::NT) {
            float v = 0.f;
#pragma unroll
            for (int w = 0; w < T::WGK; ++w) v += red[w * PER_WAVE + e];
            const int l = e % kWave, r = (e / kWave) % 16, blk = e / (16 * kWave);
            const int tm = blk / T::TN, tn = blk % T::TN;
            const int i = i0 + tm * 32 + 8 * (r / 4) + 4 * (l / 32) + (r % 4);
            const int j = j0 + tn * 32 + (l & 31);
            emit(i, j, v);
        }
    }
}

// Adds the split-K partial tiles in slice order and applies the epilogue.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *partial, float *out, int64_t numel,
                                                            int splitk, Epilogue epi) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= numel) return;
    float v = 0.f;
    for (int s = 0; s < splitk; ++s) v += partial[(int64_t)s * numel + i];
    out[i] = apply_steps(epi, v, i, chan_of(epi, i));
}

template <int MODE, class T>
int launch_tile(const GemmArgs &a, hipStream_t s) {
    const int tiles = ((a.M + T::BM - 1) / T::BM) * ((a.N + T::BN - 1) / T::BN);
    const dim3 grid(tiles, a.batch, a.splitk);
    hipLaunchKernelGGL((igemm_kernel<MODE, T>), grid, dim3(T::NT), T::SMEM * sizeof(float), s, a);
    return (int)hipGetLastError();
}

template <int MODE>
int launch_mode(const GemmArgs &a, hipStream_t s) {
    switch (a.tile) {
    case TILE_S: case TILE_S8: case TILE_S16: return launch_tile<MODE, TileS>(a, s);
    case TILE_L: return launch_tile<MODE, TileL>(a, s);
    default: return launch_tile<MODE, TileM>(a, s);
    }
}

void tile_dims(int tile, int *bm, int *bn, int *bk) {
    switch (tile) {
    case TILE_S: case TILE_S8: case TILE_S16: *bm = TileS::BM; *bn = TileS::BN; *bk = TileS::BK; break;
    case TILE_L: *bm = TileL::BM; *bn = TileL::BN; *bk = TileL::BK; break;
    default: *bm = TileM::BM; *bn = TileM::BN; *bk = TileM::BK; break;
    }
}

int64_t count_tiles(const GemmArgs &a, int tile) {
    int bm, bn, bk;
    tile_dims(tile, &bm, &bn, &bk);
    return (int64_t)((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn) * a.batch;
}

}  // namespace

// Tile: the largest whose grid still gives every CU a workgroup, else the
// smallest.  Split-K: only when even the chosen tile leaves most CUs idle and K
// is long enough to leave every split at least 128 values of k.
void gemm_resolve(GemmArgs *a, int n_cus) {
    const bool fixed = a->tile != TILE_AUTO;
    if (!fixed) {
        if (count_tiles(*a, TILE_L) >= 2 * (int64_t)n_cus) a->tile = TILE_L;
        else if (count_tiles(*a, TILE_M) >= (int64_t)n_cus) a->tile = TILE_M;
        else a->tile = TILE_S;
    }
    const int64_t tiles = count_tiles(*a, a->tile);
    int split = 1;
    if (tiles * 2 <= n_cus) {
        split = (int)std::min<int64_t>((n_cus + tiles - 1) / tiles, 16);
        split = std::min(split, std::max(1, a->K / 128));
    }
    a->splitk = split;
}

size_t gemm_scratch_bytes(const GemmArgs &a) {
    return a.splitk > 1 ? (size_t)a.splitk * (size_t)a.c_numel * sizeof(float) : 0;
}

static bool al16(const void *p) { return ((uintptr_t)p & 15) == 0; }

// Recognises the common form [scale] [bias] [add] [activation] of a fused tail.
EpiFast make_epi_fast(const Epilogue &e) {
    EpiFast f{0, 1.f, nullptr, nullptr};
    int stage = 0;      // 0 scale, 1 bias, 2 add, 3 activation, 4 done
    for (int i = 0; i < e.n; ++i) {
        const EpiStep &st = e.s[i];
        if (st.op == EPI_SCALE && stage <= 0) { f.flags |= EF_SCALE; f.scale = st.scalar; stage = 1; }
        else if (st.op == EPI_BIAS && stage <= 1) { f.flags |= EF_BIAS; f.bias = st.ptr; stage = 2; }
        else if (st.op == EPI_ADD && stage <= 2) { f.flags |= EF_ADD; f.add = st.ptr; stage = 3; }
        else if (st.op == EPI_RELU && stage <= 3) { f.flags |= EF_RELU; stage = 4; }
        else if (st.op == EPI_GELU && stage <= 3) { f.flags |= EF_GELU; stage = 4; }
        else if (st.op == EPI_TANH && stage <= 3) { f.flags |= EF_TANH; stage = 4; }
        else return EpiFast{EF_GENERIC, 1.f, nullptr, nullptr};
    }
    return f;
}

int epi_fast_flags(const Epilogue &e) { return make_epi_fast(e).flags; }

// ---- matrix-vector product: dense with a handful of rows (a classifier at batch 1) --------------
// y[m][n] = sum_k x[m][k] * w[n][k], M <= 8.  The weights are read exactly once and
// bound the kernel (HBM), so one wave owns one column n: it streams the 4K-byte
// class row of w with 16-byte loads, all issued before the first use, multiplies it
// with every row of x, and reduces across its lanes.
constexpr int kGemvRows = 8;

__global__ __launch_bounds__(256) void gemv_nt_kernel(GemmArgs p) {
    const int lane = threadIdx.x & (kWave - 1);
    const int n = blockIdx.x * (256 / kWave) + threadIdx.x / kWave;
    if (n >= p.N) return;
    const f32x4 *wrow = reinterpret_cast<const f32x4 *>(p.B + (int64_t)n * p.ldb);
    const int k4 = p.K / 4;
    float acc[kGemvRows];
#pragma unroll
    for (int m = 0; m < kGemvRows; ++m) acc[m] = 0.f;
    for (int c0 = 0; c0 < k4; c0 += 8 * kWave) {
        f32x4 w[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) w[u] = wrow[min(c0 + u * kWave + lane, k4 - 1)];
#pragma unroll
        for (int m = 0; m < kGemvRows; ++m) {
            if (m >= p.M) break;
            const f32x4 *xrow = reinterpret_cast<const f32x4 *>(p.A + (int64_t)m * p.lda);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int c = c0 + u * kWave + lane;
                const f32x4 x = xrow[min(c, k4 - 1)];
                const float d = w[u][0] * x[0] + w[u][1] * x[1] + w[u][2] * x[2] + w[u][3] * x[3];
                acc[m] += c < k4 ? d : 0.f;
            }
        }
    }
#pragma unroll
    for (int m = 0; m < kGemvRows; ++m) acc[m] = wave_sum(acc[m]);
    float mine = 0.f;
#pragma unroll
    for (int m = 0; m < kGemvRows; ++m) mine = lane == m ? acc[m] : mine;      // lane m finishes row m
    if (lane < p.M) {
        const int64_t off = (int64_t)lane * p.ldc + n;
        const float bv = (p.ef.flags & EF_BIAS) ? p.ef.bias[n] : 0.f;
        const float av = (p.ef.flags & EF_ADD) ? p.ef.add[off] : 0.f;
        p.C[off] = finish_value(p, mine, bv, av);
    }
}

bool gemv_shape_ok(const GemmArgs &a, int epi_flags) {
    // rows shorter than two 16-byte loads per lane leave most of a wave idle: those stay with the tiled kernels
    return a.mode == GM_NT && a.batch == 1 && a.M >= 1 && a.M <= kGemvRows && a.K % 4 == 0 && a.K >= 512 && a.lda % 4 == 0 &&
           a.ldb % 4 == 0 && a.cs_len == 0 && !(epi_flags & EF_GENERIC);
}

int launch_gemm_region(const GemmArgs *members, int n, void *stream) {
    if (n < 2 || n > kMaxRegion) return (int)hipErrorInvalidValue;
    GemmArgs local[kMaxRegion];
    for (int k = 0; k < n; ++k) {
        local[k] = members[k];
        local[k].ef = make_epi_fast(local[k].epi);
    }
    return launch_rf_multi(local, n, (hipStream_t)stream);
}

int launch_gemm(const GemmArgs &a_in, void *stream) {
    hipStream_t s = (hipStream_t)stream;
    GemmArgs a = a_in;
    a.ef = make_epi_fast(a.epi);
    if (a.rf_ts) {
        const int e = launch_rf_conv(a, s);
        if (e || a.splitk <= 1 || a.rf_convt) return e;      // (a transposed convolution's grid.z counts phases)
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((a.c_numel + 255) / 256)), dim3(256), 0, s,
                           a.partial, a.C, a.c_numel, a.splitk, a.epi);
        return (int)hipGetLastError();
    }
    if (a.gemv) {
        if (!al16(a.A) || !al16(a.B)) return (int)hipErrorInvalidValue;       // rows are read 16 bytes at a time
        hipLaunchKernelGGL(gemv_nt_kernel, dim3((unsigned)((a.N + 3) / 4)), dim3(256), 0, s, a);
        return (int)hipGetLastError();
    }
    int err;
    const bool a_vec = a.K % 4 == 0 && a.lda % 4 == 0 && a.strideA % 4 == 0 && al16(a.A);
    switch (a.mode) {
    case GM_NT:
        err = launch_lean_mm(a, s);
        if (err == -1 && a.cs_len) return (int)hipErrorInvalidValue;     // only the lean kernel stores column blocks
        if (err == -1) err = launch_fast_mm(a, a_vec && a.ldb % 4 == 0 && a.strideB % 4 == 0 && al16(a.B), s);
        break;
    case GM_NN:
        err = launch_lean_mm(a, s);
        if (err == -1)
            err = launch_fast_mm(a, a_vec && a.N % 4 == 0 && a.ldb % 4 == 0 && a.strideB % 4 == 0 && al16(a.B), s);
        break;
    case GM_CONV:
        err = launch_lean_conv3x3(a, s);
        if (err == -1) {
            if (a.KH * a.KW <= 64) err = launch_fast_conv(a, a_vec, s);
            else err = launch_mode<GM_CONV>(a, s);
        }
        break;
    default: err = launch_mode<GM_CONVT>(a, s); break;
    }
    if (err) return err;
    if (a.splitk > 1) {
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((a.c_numel + 255) / 256)), dim3(256), 0, s,
                           a.partial, a.C, a.c_numel, a.splitk, a.epi);
        err = (int)hipGetLastError();
    }
    return err;
}

}  // namespace clg
