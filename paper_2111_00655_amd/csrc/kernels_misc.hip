// Memory-bound kernels of the fused-operator set for gfx950: elementwise
// chains and embedding gather, softmax / layer norm with a fused prologue
// (wavefront shuffle reductions, one 64-lane wave per row), direct convolution
// for grouped and small-channel layers, pooling, layout copies.
//
// These operators move O(1) flops per byte (paper Sec. 5.1 lists them as the
// non-contraction part of the workloads), so the design rule is: every tensor
// is read once and written once, with consecutive lanes on consecutive
// addresses; anything elementwise rides along in registers.
#include <algorithm>

#include <hip/hip_runtime.h>

#include "device_common.h"

namespace clg {

// ------------------------------------------------------------------ elementwise
// y = steps(x) (or steps(table[ids])).  VEC = 4: numel % 4 == 0, and the four
// elements of a float4 share a bias channel layout the kernel can index:
// inner % 4 == 0 (same channel) or inner == 1 with C % 4 == 0 (four channels).
template <int VEC>
__global__ __launch_bounds__(256) void eltwise_kernel(EltwiseArgs a) {
    const int64_t n = a.numel / VEC;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const int64_t off = i * VEC;
        float v[VEC];
        const float *src = a.x + off;
        if (a.ids) {
            const int64_t row = off / a.row_len, col = off % a.row_len;
            int id = a.ids[row];
            id = id < 0 ? 0 : (id >= a.table_rows ? a.table_rows - 1 : id);
            src = a.x + (int64_t)id * a.row_len + col;
        }
        if constexpr (VEC == 4) {
            const float4 t = *reinterpret_cast<const float4 *>(src);
            v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
        } else {
            v[0] = src[0];
        }
#pragma unroll
        for (int q = 0; q < VEC; ++q) v[q] = apply_steps(a.epi, v[q], off + q, chan_of(a.epi, off + q));
        if constexpr (VEC == 4) {
            *reinterpret_cast<float4 *>(a.y + off) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
            a.y[off] = v[0];
        }
    }
}

static bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

int launch_eltwise(const EltwiseArgs &a, void *stream) {
    bool vec = a.numel % 4 == 0 && aligned16(a.x) && aligned16(a.y) && (!a.ids || a.row_len % 4 == 0);
    for (int s = 0; s < a.epi.n; ++s)
        if (a.epi.s[s].op == EPI_ADD && !aligned16(a.epi.s[s].ptr)) vec = false;
    const int64_t items = vec ? a.numel / 4 : a.numel;
    const int block = 256;
    const int grid = (int)std::min<int64_t>((items + block - 1) / block, 256 * 16);
    if (vec)
        hipLaunchKernelGGL(eltwise_kernel<4>, dim3(grid), dim3(block), 0, (hipStream_t)stream, a);
    else
        hipLaunchKernelGGL(eltwise_kernel<1>, dim3(grid), dim3(block), 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

// --------------------------------------------------------------- softmax / LN
// One wave per row; the row (after the fused prologue) is held in registers:
// ITEMS values per lane, element c = lane + 64 * t.  Reads x once, writes y
// once.  Softmax: max, sum of exp, normalise.  Layer norm: mean, then the
// biased variance of the centred values, then scale and shift.
template <int ITEMS>
__global__ __launch_bounds__(256) void rowwise_kernel(RowwiseArgs a) {
    const int lane = threadIdx.x & (kWave - 1);
    const int row = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (row >= a.rows) return;
    const float *xr = a.x + (int64_t)row * a.len;
    float *yr = a.y + (int64_t)row * a.len;
    float v[ITEMS];
#pragma unroll
    for (int t = 0; t < ITEMS; ++t) {
        const int c = lane + kWave * t;
        v[t] = 0.f;
        if (c < a.len) v[t] = apply_steps(a.pro, xr[c], (int64_t)row * a.len + c, c);
    }
    if (a.mode == 0) {
        float mx = -INFINITY;
#pragma unroll
        for (int t = 0; t < ITEMS; ++t)
            if (lane + kWave * t < a.len) mx = fmaxf(mx, v[t]);
        mx = wave_max(mx);
        float sum = 0.f;
#pragma unroll
        for (int t = 0; t < ITEMS; ++t) {
            v[t] = (lane + kWave * t < a.len) ? expf(v[t] - mx) : 0.f;
            sum += v[t];
        }
        sum = wave_sum(sum);
        const float inv = 1.0f / sum;
#pragma unroll
        for (int t = 0; t < ITEMS; ++t)
            if (lane + kWave * t < a.len) yr[lane + kWave * t] = v[t] * inv;
    } else {
        float sum = 0.f;
#pragma unroll
        for (int t = 0; t < ITEMS; ++t) sum += v[t];          // padding lanes hold 0
        const float mean = wave_sum(sum) / (float)a.len;
        float sq = 0.f;
#pragma unroll
        for (int t = 0; t < ITEMS; ++t) {
            const float d = (lane + kWave * t < a.len) ? v[t] - mean : 0.f;
            v[t] = d;
            sq += d * d;
        }
        const float var = wave_sum(sq) / (float)a.len;
        const float inv = 1.0f / sqrtf(var + a.eps);
#pragma unroll
        for (int t = 0; t < ITEMS; ++t) {
            const int c = lane + kWave * t;
            if (c < a.len) yr[c] = v[t] * inv * a.gamma[c] + a.beta[c];
        }
    }
}

// One workgroup (four waves) per row: for few, long rows (layer norm over 128 x 768,
// the 1 x 1000 softmax of a classifier) a wave per row leaves most of the chip
// idle and strings ITEMS dependent loads and exponentials behind each other.
// Each reduction is a wave reduction plus four partial values through LDS, added
// in wave order.  gamma / beta are fetched before the reductions.
template <int ITEMS>
__global__ __launch_bounds__(256) void rowwise_block_kernel(RowwiseArgs a) {
    __shared__ float part[2][4];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int row = blockIdx.x;
    const float *xr = a.x + (int64_t)row * a.len;
    float *yr = a.y + (int64_t)row * a.len;
    float v[ITEMS], ga[ITEMS], be[ITEMS];
#pragma unroll
    for (int t = 0; t < ITEMS; ++t) {
        const int c = tid + 256 * t;
        v[t] = 0.f;
        ga[t] = 0.f;
        be[t] = 0.f;
        if (c < a.len) {
            v[t] = apply_steps(a.pro, xr[c], (int64_t)row * a.len + c, c);
            if (a.mode == 1) {
                ga[t] = a.gamma[c];
                be[t] = a.beta[c];
            }
        }
    }
    auto block_sum = [&](float x, int slot) {
        x = wave_sum(x);
        if (lane == 0) part[slot][wave] = x;
        __syncthreads();
        return (part[slot][0] + part[slot][1]) + (part[slot][2] + part[slot][3]);
    };
    if (a.mode == 0) {
        float mx = -INFINITY;
#pragma unroll
        for (int t = 0; t < ITEMS; ++t)
            if (tid + 256 * t < a.len) mx = fmaxf(mx, v[t]);
        mx = wave_max(mx);
        if (lane == 0) part[0][wave] = mx;
        __syncthreads();
        mx = fmaxf(fmaxf(part[0][0], part[0][1]), fmaxf(part[0][2], part[0][3]));
        float sum = 0.f;
#pragma unroll
        for (int t = 0; t < ITEMS; ++t) {
            v[t] = (tid + 256 * t < a.len) ? expf(v[t] - mx) : 0.f;
            sum += v[t];
        }
        const float inv = 1.0f / block_sum(sum, 1);
#pragma unroll
        for (int t = 0; t < ITEMS; ++t)
            if (tid + 256 * t < a.len) yr[tid + 256 * t] = v[t] * inv;
    } else {
        float sum = 0.f;
#pragma unroll
        for (int t = 0; t < ITEMS; ++t) sum += v[t];          // padding lanes hold 0
        const float mean = block_sum(sum, 0) / (float)a.len;
        float sq = 0.f;
#pragma unroll
        for (int t = 0; t < ITEMS; ++t) {
            const float d = (tid + 256 * t < a.len) ? v[t] - mean : 0.f;
            v[t] = d;
            sq += d * d;
        }
        const float var = block_sum(sq, 1) / (float)a.len;
        const float inv = 1.0f / sqrtf(var + a.eps);
#pragma unroll
        for (int t = 0; t < ITEMS; ++t) {
            const int c = tid + 256 * t;
            if (c < a.len) yr[c] = v[t] * inv * ga[t] + be[t];
        }
    }
}

// Layer norm, a wave per row and a row per workgroup, for the transformer's shapes (128 rows of 768):
// every load of the row - the value, the fused bias and residual, gamma and beta, 16 bytes per lane
// each - is issued before anything is computed, so the kernel pays one memory round trip; the two
// reductions stay inside the wave (no LDS, no barrier).  The row comes from x with an optional
// [bias] [residual add] in front (the common form of a fused prologue), or is the sum of two or three
// gathered table rows (an embedding).  Same arithmetic as above: mean, biased variance of the centred
// values, scale and shift.  len % 4 == 0, len <= 256 * V4, all pointers 16-byte aligned.
template <int V4>
__global__ __launch_bounds__(64) void ln_wave_kernel(RowwiseArgs a, EpiFast ef) {
    const int lane = threadIdx.x;
    const int row = blockIdx.x;
    const int len4 = a.len >> 2;
    const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
    float4 v[V4], t1[V4], t2[V4], ga[V4], be[V4];
    const float4 *p0, *p1 = nullptr, *p2 = nullptr;
    if (a.n_gather) {
        auto row_of = [&](int k) {
            int id = a.gid[k][row];
            id = id < 0 ? 0 : (id >= a.tab_rows[k] ? a.tab_rows[k] - 1 : id);
            return reinterpret_cast<const float4 *>(a.tab[k] + (int64_t)id * a.len);
        };
        p0 = row_of(0);
        p1 = row_of(1);
        if (a.n_gather > 2) p2 = row_of(2);
    } else {
        p0 = reinterpret_cast<const float4 *>(a.x + (int64_t)row * a.len);
        if (ef.flags & EF_BIAS) p1 = reinterpret_cast<const float4 *>(ef.bias);
        if (ef.flags & EF_ADD) p2 = reinterpret_cast<const float4 *>(ef.add + (int64_t)row * a.len);
    }
    const float4 *g4 = reinterpret_cast<const float4 *>(a.gamma), *b4 = reinterpret_cast<const float4 *>(a.beta);
#pragma unroll
    for (int q = 0; q < V4; ++q) {
        const int c = lane + kWave * q;
        const bool in = c < len4;
        const int cc = in ? c : 0;
        v[q] = p0[cc];
        t1[q] = p1 ? p1[cc] : zero;
        t2[q] = p2 ? p2[cc] : zero;
        ga[q] = g4[cc];
        be[q] = b4[cc];
        if (!in) v[q] = t1[q] = t2[q] = zero;
    }
    float sum = 0.f;
#pragma unroll
    for (int q = 0; q < V4; ++q) {
        // the operators' own order, one rounding each: (x + bias) + residual, or (row0 + row1) + row2
        if (p1) { v[q].x += t1[q].x; v[q].y += t1[q].y; v[q].z += t1[q].z; v[q].w += t1[q].w; }
        if (p2) { v[q].x += t2[q].x; v[q].y += t2[q].y; v[q].z += t2[q].z; v[q].w += t2[q].w; }
        sum += (v[q].x + v[q].y) + (v[q].z + v[q].w);
    }
    const float mean = wave_sum_dpp(sum) / (float)a.len;
    float sq = 0.f;
#pragma unroll
    for (int q = 0; q < V4; ++q) {
        if (lane + kWave * q < len4) {
            v[q].x -= mean; v[q].y -= mean; v[q].z -= mean; v[q].w -= mean;
        }
        sq += (v[q].x * v[q].x + v[q].y * v[q].y) + (v[q].z * v[q].z + v[q].w * v[q].w);
    }
    const float inv = 1.0f / sqrtf(wave_sum_dpp(sq) / (float)a.len + a.eps);
    float4 *y4 = reinterpret_cast<float4 *>(a.y + (int64_t)row * a.len);
#pragma unroll
    for (int q = 0; q < V4; ++q) {
        const int c = lane + kWave * q;
        if (c < len4)
            y4[c] = make_float4(v[q].x * inv * ga[q].x + be[q].x, v[q].y * inv * ga[q].y + be[q].y,
                                v[q].z * inv * ga[q].z + be[q].z, v[q].w * inv * ga[q].w + be[q].w);
    }
}

// Whether the one-round-trip layer norm takes these arguments; fills *ef with the prologue's common form.
static bool ln_wave_ok(const RowwiseArgs &a, EpiFast *ef) {
    if (a.mode != 1 || a.len % 4 || a.len > 256 * 8 || a.len < 64 || a.rows > 65535 * 16) return false;
    auto al = [](const void *p) { return ((uintptr_t)p & 15) == 0; };
    if (!al(a.y) || !al(a.gamma) || !al(a.beta)) return false;
    ef->flags = 0;
    if (a.n_gather) {
        for (int k = 0; k < a.n_gather; ++k)
            if (!al(a.tab[k]) || a.tab_rows[k] < 1) return false;
        return a.n_gather == 2 || a.n_gather == 3;
    }
    *ef = make_epi_fast(a.pro);
    if (ef->flags & ~(EF_BIAS | EF_ADD)) return false;
    if (ef->flags & EF_BIAS) {
        if (a.pro.bias_inner != 1 || a.pro.bias_c != a.len || !al(ef->bias)) return false;
    }
    if ((ef->flags & EF_ADD) && !al(ef->add)) return false;
    return al(a.x);
}

// Rows longer than 64 * 32: same arithmetic, the row is re-read per pass.
__global__ __launch_bounds__(256) void rowwise_long_kernel(RowwiseArgs a) {
    const int lane = threadIdx.x & (kWave - 1);
    const int row = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (row >= a.rows) return;
    const float *xr = a.x + (int64_t)row * a.len;
    float *yr = a.y + (int64_t)row * a.len;
    auto val = [&](int c) { return apply_steps(a.pro, xr[c], (int64_t)row * a.len + c, c); };
    if (a.mode == 0) {
        float mx = -INFINITY;
        for (int c = lane; c < a.len; c += kWave) mx = fmaxf(mx, val(c));
        mx = wave_max(mx);
        float sum = 0.f;
        for (int c = lane; c < a.len; c += kWave) sum += expf(val(c) - mx);
        sum = wave_sum(sum);
        const float inv = 1.0f / sum;
        for (int c = lane; c < a.len; c += kWave) yr[c] = expf(val(c) - mx) * inv;
    } else {
        float sum = 0.f;
        for (int c = lane; c < a.len; c += kWave) sum += val(c);
        const float mean = wave_sum(sum) / (float)a.len;
        float sq = 0.f;
        for (int c = lane; c < a.len; c += kWave) {
            const float d = val(c) - mean;
            sq += d * d;
        }
        const float inv = 1.0f / sqrtf(wave_sum(sq) / (float)a.len + a.eps);
        for (int c = lane; c < a.len; c += kWave) yr[c] = (val(c) - mean) * inv * a.gamma[c] + a.beta[c];
    }
}

int launch_rowwise(const RowwiseArgs &a, void *stream) {
    const int block = 256, rows_per_block = block / kWave;
    const dim3 grid((a.rows + rows_per_block - 1) / rows_per_block);
    const int items = (a.len + kWave - 1) / kWave;
    hipStream_t s = (hipStream_t)stream;
    EpiFast ef{};
    if (a.rows <= 4096 && ln_wave_ok(a, &ef)) {                    // layer norm in one memory round trip
        const int v4 = (a.len / 4 + kWave - 1) / kWave;
        if (v4 <= 1) hipLaunchKernelGGL(ln_wave_kernel<1>, dim3(a.rows), dim3(kWave), 0, s, a, ef);
        else if (v4 <= 2) hipLaunchKernelGGL(ln_wave_kernel<2>, dim3(a.rows), dim3(kWave), 0, s, a, ef);
        else if (v4 <= 4) hipLaunchKernelGGL(ln_wave_kernel<4>, dim3(a.rows), dim3(kWave), 0, s, a, ef);
        else hipLaunchKernelGGL(ln_wave_kernel<8>, dim3(a.rows), dim3(kWave), 0, s, a, ef);
        return (int)hipGetLastError();
    }
    if (a.n_gather) return (int)hipErrorInvalidValue;              // only the kernel above gathers
    if (a.len > 256 && a.len <= 2048 && a.rows <= 1024) {          // few long rows: a workgroup per row
        const int bi = (a.len + 255) / 256;
        if (bi <= 2) hipLaunchKernelGGL(rowwise_block_kernel<2>, dim3(a.rows), dim3(256), 0, s, a);
        else if (bi <= 4) hipLaunchKernelGGL(rowwise_block_kernel<4>, dim3(a.rows), dim3(256), 0, s, a);
        else hipLaunchKernelGGL(rowwise_block_kernel<8>, dim3(a.rows), dim3(256), 0, s, a);
        return (int)hipGetLastError();
    }
    if (items <= 1) hipLaunchKernelGGL(rowwise_kernel<1>, grid, dim3(block), 0, s, a);
    else if (items <= 2) hipLaunchKernelGGL(rowwise_kernel<2>, grid, dim3(block), 0, s, a);
    else if (items <= 4) hipLaunchKernelGGL(rowwise_kernel<4>, grid, dim3(block), 0, s, a);
    else if (items <= 8) hipLaunchKernelGGL(rowwise_kernel<8>, grid, dim3(block), 0, s, a);
    else if (items <= 16) hipLaunchKernelGGL(rowwise_kernel<16>, grid, dim3(block), 0, s, a);
    else if (items <= 32) hipLaunchKernelGGL(rowwise_kernel<32>, grid, dim3(block), 0, s, a);
    else hipLaunchKernelGGL(rowwise_long_kernel, grid, dim3(block), 0, s, a);
    return (int)hipGetLastError();
}

// ------------------------------------------------------------ direct convolution
// One thread per output pixel and COB consecutive output channels of one group:
// every input value loaded is used COB times; the weights of those channels are
// wave-uniform (scalar loads).  blockIdx.y = channel block, blockIdx.z = image.
template <int COB>
__global__ __launch_bounds__(256) void direct_conv_kernel(DirectConvArgs a) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    const int npix = a.HO * a.WO;
    const int Cg = a.C / a.G, Og = a.O / a.G;
    const int co0 = blockIdx.y * COB;
    const int g = co0 / Og;
    const int n = blockIdx.z;
    if (p >= npix) return;
    const int oh = p / a.WO, ow = p % a.WO;
    float acc[COB];
#pragma unroll
    for (int j = 0; j < COB; ++j) acc[j] = 0.f;
    const float *xg = a.x + ((int64_t)n * a.C + (int64_t)g * Cg) * a.H * a.W;
    const float *wg = a.w + (int64_t)co0 * Cg * a.KH * a.KW;
    const int wstride = Cg * a.KH * a.KW;
    for (int ci = 0; ci < Cg; ++ci) {
        for (int kh = 0; kh < a.KH; ++kh) {
            const int ih = oh * a.sh - a.ph + kh;
            if (ih < 0 || ih >= a.H) continue;
            for (int kw = 0; kw < a.KW; ++kw) {
                const int iw = ow * a.sw - a.pw + kw;
                if (iw < 0 || iw >= a.W) continue;
                const float xv = xg[((int64_t)ci * a.H + ih) * a.W + iw];
                const float *wp = wg + (ci * a.KH + kh) * a.KW + kw;
#pragma unroll
                for (int j = 0; j < COB; ++j) acc[j] = fmaf(xv, wp[j * wstride], acc[j]);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < COB; ++j) {
        const int co = co0 + j;
        const int64_t off = ((int64_t)n * a.O + co) * npix + p;
        a.y[off] = apply_steps(a.epi, acc[j], off, co);
    }
}

// Transposed convolution of any filter size, stride and pad (w is [C][O][KH][KW]), gather form: one
// thread per output pixel, blockIdx.y = output channel, blockIdx.z = image.  Output row oh takes
// filter row kh from input row (oh + ph - kh) / sh where that division is exact and the row exists;
// the same along the width.  The kernel that runs what the phase-decomposed MFMA kernels refuse
// (a filter size that the stride does not divide).
__global__ __launch_bounds__(256) void direct_convt_kernel(DirectConvArgs a) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    const int npix = a.HO * a.WO;
    const int co = blockIdx.y, n = blockIdx.z;
    if (p >= npix) return;
    const int oh = p / a.WO, ow = p % a.WO;
    const float *xn = a.x + (int64_t)n * a.C * a.H * a.W;
    const float *wo = a.w + (int64_t)co * a.KH * a.KW;
    const int64_t xstride = (int64_t)a.H * a.W, wstride = (int64_t)a.O * a.KH * a.KW;
    float acc = 0.f;
    for (int kh = 0; kh < a.KH; ++kh) {
        const int th = oh + a.ph - kh;
        if (th < 0 || th % a.sh != 0 || th / a.sh >= a.H) continue;
        const int ih = th / a.sh;
        for (int kw = 0; kw < a.KW; ++kw) {
            const int tw = ow + a.pw - kw;
            if (tw < 0 || tw % a.sw != 0 || tw / a.sw >= a.W) continue;
            const float *xp = xn + (int64_t)ih * a.W + tw / a.sw;
            const float *wp = wo + kh * a.KW + kw;
            for (int ci = 0; ci < a.C; ++ci) acc = fmaf(xp[ci * xstride], wp[ci * wstride], acc);
        }
    }
    const int64_t off = ((int64_t)n * a.O + co) * npix + p;
    a.y[off] = apply_steps(a.epi, acc, off, co);
}

// Depthwise convolution (one input channel per output channel), square filter KS: one output per
// thread, taps unrolled, loads without branches (clamped addresses, masked values) so that they all
// go out together; optional relu on the input, fused tail.
template <int KS>
__device__ __forceinline__ void depthwise_body(const DirectConvArgs &a, const uint32_t block) {
    const uint32_t npix = (uint32_t)(a.HO * a.WO);
    const uint32_t total = (uint32_t)(a.N * a.C) * npix;
    const uint32_t i = block * 256u + threadIdx.x;
    if (i >= total) return;
    const uint32_t nc = i / npix, p = i - nc * npix;
    const uint32_t c = nc % (uint32_t)a.C;
    const int oh = (int)(p / (uint32_t)a.WO), ow = (int)(p - (uint32_t)oh * a.WO);
    const int ih0 = oh * a.sh - a.ph, iw0 = ow * a.sw - a.pw;
    const float *xc = a.x + (int64_t)nc * a.H * a.W;
    const float *wc = a.w + c * (KS * KS);
    const float lo = a.pro_relu ? 0.f : -INFINITY;
    int ro[KS], co[KS];
    bool vr[KS], vc[KS];
#pragma unroll
    for (int t = 0; t < KS; ++t) {
        const int ih = ih0 + t, iw = iw0 + t;
        vr[t] = ih >= 0 && ih < a.H;
        vc[t] = iw >= 0 && iw < a.W;
        ro[t] = (ih < 0 ? 0 : (ih >= a.H ? a.H - 1 : ih)) * a.W;
        co[t] = iw < 0 ? 0 : (iw >= a.W ? a.W - 1 : iw);
    }
    float xv[KS * KS], wv[KS * KS];
#pragma unroll
    for (int kh = 0; kh < KS; ++kh)
#pragma unroll
        for (int kw = 0; kw < KS; ++kw) {
            xv[kh * KS + kw] = xc[ro[kh] + co[kw]];
            wv[kh * KS + kw] = wc[kh * KS + kw];
        }
    // bias and residual of this output, fetched with the taps
    const int f = a.ef.flags;
    const bool fast = !(f & EF_GENERIC);
    float bias_v = 0.f, add_v = 0.f;
    if (fast && (f & EF_BIAS)) bias_v = a.ef.bias[c];
    if (fast && (f & EF_ADD)) add_v = a.ef.add[i];
    float v = 0.f;
#pragma unroll
    for (int kh = 0; kh < KS; ++kh)
#pragma unroll
        for (int kw = 0; kw < KS; ++kw) {
            const float t = (vr[kh] && vc[kw]) ? fmaxf(xv[kh * KS + kw], lo) : 0.f;
            v = fmaf(wv[kh * KS + kw], t, v);
        }
    if (fast) {
        if (f & EF_SCALE) v *= a.ef.scale;
        v += bias_v;
        v += add_v;
        if (f & EF_RELU) v = v > 0.f ? v : 0.f;
        else if (f & EF_GELU) v = gelu_erf(v);
        else if (f & EF_TANH) v = tanhf(v);
    } else {
        v = apply_steps(a.epi, v, i, (int)c);
    }
    a.y[i] = v;
}

template <int KS>
__global__ __launch_bounds__(256) void depthwise_kernel(DirectConvArgs a) {
    depthwise_body<KS>(a, blockIdx.x);
}

bool depthwise_fast_ok(const DirectConvArgs &a) {
    return !a.transposed && a.G == a.C && a.O == a.C && a.KH == a.KW && (a.KH == 3 || a.KH == 5 || a.KH == 7) &&
           (int64_t)a.N * a.C * a.HO * a.WO < ((int64_t)1 << 31) && (int64_t)a.H * a.W < ((int64_t)1 << 31);
}

int launch_direct_conv(const DirectConvArgs &a_in, void *stream) {
    DirectConvArgs a = a_in;
    a.ef = make_epi_fast(a.epi);
    if (depthwise_fast_ok(a)) {
        const int64_t total = (int64_t)a.N * a.C * a.HO * a.WO;
        const dim3 grid((unsigned)((total + 255) / 256));
        if (a.KH == 3) hipLaunchKernelGGL(depthwise_kernel<3>, grid, dim3(256), 0, (hipStream_t)stream, a);
        else if (a.KH == 5) hipLaunchKernelGGL(depthwise_kernel<5>, grid, dim3(256), 0, (hipStream_t)stream, a);
        else hipLaunchKernelGGL(depthwise_kernel<7>, grid, dim3(256), 0, (hipStream_t)stream, a);
        return (int)hipGetLastError();
    }
    if (a.pro_relu) return (int)hipErrorInvalidValue;      // only the depthwise kernel applies the relu
    const int npix = a.HO * a.WO;
    const int Og = a.O / a.G;
    const int block = npix >= 256 ? 256 : (npix > 64 ? 128 : 64);
    hipStream_t s = (hipStream_t)stream;
    if (a.transposed) {
        if (a.G != 1 || a.O > 65535 || a.N > 65535) return (int)hipErrorInvalidValue;
        hipLaunchKernelGGL(direct_convt_kernel, dim3((npix + block - 1) / block, a.O, a.N), dim3(block), 0, s, a);
        return (int)hipGetLastError();
    }
    if (Og % 4 == 0) {
        const dim3 grid((npix + block - 1) / block, a.O / 4, a.N);
        hipLaunchKernelGGL(direct_conv_kernel<4>, grid, dim3(block), 0, s, a);
    } else {
        const dim3 grid((npix + block - 1) / block, a.O, a.N);
        hipLaunchKernelGGL(direct_conv_kernel<1>, grid, dim3(block), 0, s, a);
    }
    return (int)hipGetLastError();
}

// ------------------------------------------------------------------------ pooling
// One output pixel per thread.  AVG: mean over the window's pixels inside the image.
template <bool AVG>
__device__ __forceinline__ void window_pool_body(const PoolArgs &a, const uint32_t block) {
    // 32-bit index arithmetic (the launcher checks the sizes): a 64-bit division is a long routine
    const uint32_t total = (uint32_t)(a.NC * a.DO * a.HO * a.WO);
    const uint32_t i = block * 256u + threadIdx.x;
    if (i >= total) return;
    const uint32_t q1 = i / (uint32_t)a.WO, q2 = q1 / (uint32_t)a.HO;
    const int ow = (int)(i - q1 * a.WO), oh = (int)(q1 - q2 * a.HO);
    int od = 0;
    uint32_t nc = q2;
    if (a.DO > 1) {
        nc = q2 / (uint32_t)a.DO;
        od = (int)(q2 - nc * a.DO);
    }
    const float *xp = a.x + (int64_t)nc * a.D * a.H * a.W;
    float acc = AVG ? 0.f : -INFINITY;
    int cnt = 0;
    for (int kd = 0; kd < a.KD; ++kd) {
        const int id = od * a.sd - a.pd + kd;
        if (id < 0 || id >= a.D) continue;
        for (int kh = 0; kh < a.KH; ++kh) {
            const int ih = oh * a.sh - a.ph + kh;
            if (ih < 0 || ih >= a.H) continue;
            for (int kw = 0; kw < a.KW; ++kw) {
                const int iw = ow * a.sw - a.pw + kw;
                if (iw < 0 || iw >= a.W) continue;
                const float v = xp[(id * a.H + ih) * a.W + iw];
                acc = AVG ? acc + v : fmaxf(acc, v);
                ++cnt;
            }
        }
    }
    if (AVG) acc = cnt ? acc / (float)cnt : 0.f;
    if (a.epi.n) acc = apply_steps(a.epi, acc, i, a.epi.bias_c ? (int)((i / (uint32_t)a.epi.bias_inner) % (uint32_t)a.epi.bias_c) : 0);
    a.y[i] = acc;
}

template <bool AVG>
__global__ __launch_bounds__(256) void window_pool_kernel(PoolArgs a) {
    window_pool_body<AVG>(a, blockIdx.x);
}

// Several independent thread-per-output problems in one launch: the depthwise convolutions and window
// pools that the branches of a cell apply to the same few tensors.  Workgroup -> problem by a
// wave-uniform look-up, then exactly the code the problem runs alone (same results bit for bit).
__global__ __launch_bounds__(256) void plane_multi_kernel(PlaneMultiArgs m) {
    const int bx = blockIdx.x;
    int k = 0;
#pragma unroll
    for (int i = 0; i + 1 < kMaxPlaneRegion; ++i) k += (i + 1 < m.n && bx >= m.block_end[i]) ? 1 : 0;
    const uint32_t block = (uint32_t)(bx - (k ? m.block_end[k - 1] : 0));
    switch (m.kind[k]) {
    case 3: depthwise_body<3>(m.p[k].dw, block); break;
    case 5: depthwise_body<5>(m.p[k].dw, block); break;
    case 7: depthwise_body<7>(m.p[k].dw, block); break;
    case 10: window_pool_body<false>(m.p[k].pool, block); break;
    default: window_pool_body<true>(m.p[k].pool, block); break;
    }
}

bool plane_region_pool_ok(const PoolArgs &a) {
    return (a.mode == 0 || a.mode == 2) && a.D >= 1 && a.KD >= 1 && a.sd >= 1 && a.DO >= 1 &&
           (int64_t)a.NC * a.DO * a.HO * a.WO < ((int64_t)1 << 31) && (int64_t)a.D * a.H * a.W < ((int64_t)1 << 31);
}

int launch_plane_region(const PlaneMultiArgs &m_in, void *stream) {
    PlaneMultiArgs m = m_in;
    if (m.n < 2 || m.n > kMaxPlaneRegion) return (int)hipErrorInvalidValue;
    int64_t end = 0;
    for (int k = 0; k < m.n; ++k) {
        int64_t total;
        if (m.kind[k] == 3 || m.kind[k] == 5 || m.kind[k] == 7) {
            DirectConvArgs &a = m.p[k].dw;
            if (!depthwise_fast_ok(a) || a.KH != m.kind[k]) return (int)hipErrorInvalidValue;
            a.ef = make_epi_fast(a.epi);
            total = (int64_t)a.N * a.C * a.HO * a.WO;
        } else if (m.kind[k] == 10 || m.kind[k] == 11) {
            const PoolArgs &a = m.p[k].pool;
            if (!plane_region_pool_ok(a) || a.mode != (m.kind[k] == 10 ? 0 : 2)) return (int)hipErrorInvalidValue;
            total = (int64_t)a.NC * a.DO * a.HO * a.WO;
        } else {
            return (int)hipErrorInvalidValue;
        }
        end += (total + 255) / 256;
        if (end >= ((int64_t)1 << 31)) return (int)hipErrorInvalidValue;
        m.block_end[k] = (int32_t)end;
    }
    for (int k = m.n; k < kMaxPlaneRegion; ++k) m.block_end[k] = (int32_t)end;
    hipLaunchKernelGGL(plane_multi_kernel, dim3((unsigned)end), dim3(256), 0, (hipStream_t)stream, m);
    return (int)hipGetLastError();
}

// one wave per (n, c) plane
__global__ __launch_bounds__(256) void global_avg_pool_kernel(PoolArgs a) {
    const int lane = threadIdx.x & (kWave - 1);
    const int nc = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (nc >= a.NC) return;
    const int hw = a.H * a.W;
    const float *xp = a.x + (int64_t)nc * hw;
    float sum = 0.f;
    for (int i = lane; i < hw; i += kWave) sum += xp[i];
    sum = wave_sum(sum);
    if (lane == 0) a.y[nc] = sum / (float)hw;
}

int launch_pool(const PoolArgs &a, void *stream) {
    hipStream_t s = (hipStream_t)stream;
    if (a.D < 1 || a.KD < 1 || a.sd < 1 || a.DO < 1) return (int)hipErrorInvalidValue;
    if ((int64_t)a.NC * a.DO * a.HO * a.WO >= ((int64_t)1 << 31) || (int64_t)a.D * a.H * a.W >= ((int64_t)1 << 31))
        return (int)hipErrorInvalidValue;                      // the window kernels index with 32 bits
    if (a.mode == 0 || a.mode == 2) {
        const int64_t total = (int64_t)a.NC * a.DO * a.HO * a.WO;
        const dim3 grid((unsigned)((total + 255) / 256));
        if (a.mode == 0) hipLaunchKernelGGL(window_pool_kernel<false>, grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL(window_pool_kernel<true>, grid, dim3(256), 0, s, a);
    } else {
        hipLaunchKernelGGL(global_avg_pool_kernel, dim3((a.NC + 3) / 4), dim3(256), 0, s, a);
    }
    return (int)hipGetLastError();
}

// --------------------------------------------------------------------- layout copy
__global__ __launch_bounds__(256) void layout_kernel(LayoutArgs a) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < a.numel; o += stride) {
        int64_t rem = o, src = 0;
        for (int d = a.ndim - 1; d >= 0; --d) {
            const int64_t q = rem / a.out_dims[d];
            src += (rem - q * a.out_dims[d]) * a.in_strides[d];
            rem = q;
        }
        a.y[o] = a.x[src];
    }
}

int launch_layout(const LayoutArgs &a, void *stream) {
    const int grid = (int)std::min<int64_t>((a.numel + 255) / 256, 256 * 16);
    hipLaunchKernelGGL(layout_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

// ------------------------------------------------------------------------- concat
// Output element o = (r, col): the operand whose column range holds col supplies it.
template <int VEC>
__global__ __launch_bounds__(256) void concat_kernel(ConcatArgs a) {
    const int64_t n = a.outer * a.row / VEC;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const int64_t o = i * VEC;
        const int64_t r = o / a.row;
        int64_t col = o - r * a.row;
        int s = 0;
        while (s < a.n - 1 && col >= a.chunk[s]) col -= a.chunk[s++];
        const float *src = a.src[s] + r * a.chunk[s] + col;
        if constexpr (VEC == 4) *reinterpret_cast<float4 *>(a.y + o) = *reinterpret_cast<const float4 *>(src);
        else a.y[o] = *src;
    }
}

int launch_concat(const ConcatArgs &a, void *stream) {
    bool vec = aligned16(a.y);
    for (int s = 0; s < a.n; ++s) vec = vec && a.chunk[s] % 4 == 0 && aligned16(a.src[s]);
    const int64_t items = a.outer * a.row / (vec ? 4 : 1);
    const int grid = (int)std::min<int64_t>((items + 255) / 256, 256 * 16);
    if (vec) hipLaunchKernelGGL(concat_kernel<4>, dim3(grid), dim3(256), 0, (hipStream_t)stream, a);
    else hipLaunchKernelGGL(concat_kernel<1>, dim3(grid), dim3(256), 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

// ------------------------------------------------------- measurer scratch operands
__global__ __launch_bounds__(256) void fill_kernel(float *p, int64_t n, uint64_t seed) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        uint64_t z = seed + 0x9E3779B97F4A7C15ull * (uint64_t)(i + 1);    // splitmix64 finaliser
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        z ^= z >> 31;
        p[i] = (float)((z >> 40) & 0xFFFFFF) * (2.0f / 16777216.0f) - 1.0f;
    }
}

int launch_fill(float *p, int64_t n, uint64_t seed, void *stream) {
    const int grid = (int)std::min<int64_t>((n + 255) / 256, 256 * 16);
    hipLaunchKernelGGL(fill_kernel, dim3(grid > 0 ? grid : 1), dim3(256), 0, (hipStream_t)stream, p, n, seed);
    return (int)hipGetLastError();
}

// Row ids for a gather: uniform over [0, rows) from the same counter hash, so that a measured
// gather touches rows spread over the whole table, as a real one does.
__global__ __launch_bounds__(256) void fill_ids_kernel(int32_t *p, int64_t n, int32_t rows, uint64_t seed) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        uint64_t z = seed + 0x9E3779B97F4A7C15ull * (uint64_t)(i + 1);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        z ^= z >> 31;
        p[i] = (int32_t)(((z >> 32) * (uint64_t)(rows > 0 ? rows : 1)) >> 32);
    }
}

int launch_fill_ids(int32_t *p, int64_t n, int32_t rows, uint64_t seed, void *stream) {
    const int grid = (int)std::min<int64_t>((n + 255) / 256, 256 * 16);
    hipLaunchKernelGGL(fill_ids_kernel, dim3(grid > 0 ? grid : 1), dim3(256), 0, (hipStream_t)stream, p, n, rows, seed);
    return (int)hipGetLastError();
}

__global__ void empty_kernel() {}

int launch_empty(void *stream) {
    hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream);
    return (int)hipGetLastError();
}

}  // namespace clg
