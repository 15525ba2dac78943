// Separable convolution as ONE kernel (gfx950): [relu] -> depthwise k x k ->
// 1x1 convolution -> fused elementwise tail, or [relu] -> 1x1 convolution ->
// tail without the depthwise stage.  NasNet-A (paper Sec. 5.1) is built from
// these; run operator by operator a separable convolution is five launches of
// a few microseconds each, and at batch 1 the launch is what costs.
//
// A workgroup (4 waves) owns 16 consecutive output pixels.  Phase 1: its 256
// threads compute the depthwise result (or relu(x)) for those pixels and every
// input channel into LDS, B[c][pixel]; the depthwise values never go to memory.
// Phase 2: the 1x1 convolution is C[cout][pixel] = sum_c Wp[cout][c] B[c][pixel]
// on v_mfma_f32_16x16x4_f32: a wave takes a 16-row tile of output channels (or,
// when a workgroup holds fewer than four such tiles, a part of the channel
// range of one; the parts meet in LDS and are added in a fixed order).  The 1x1
// weights are re-packed once per plan so that a lane's A operands for four
// MFMAs are one 16-byte load.
#include <algorithm>

#include <hip/hip_runtime.h>

#include "device_common.h"
#include "kernels.h"

namespace clg {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kPix = 16;          // output pixels per workgroup = MFMA tile width
constexpr int kRows = 16;         // output channels per MFMA tile
constexpr int kGroup = 16;        // input channels per packed group (4 MFMAs x 4 k-slots)

// Packed 1x1 weights: [m-tile][group][lane][4]; value j of lane l in group g of
// m-tile mt is Wp[mt*16 + l%16][(4g + j)*4 + l/16], zero outside the matrix.
__global__ void sepconv_pack_kernel(const float *w, float *dst, int Cout, int C, int ngroups, int64_t total) {
    const int64_t d = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (d >= total) return;
    const int j = (int)(d & 3), lane = (int)((d >> 2) & 63);
    const int64_t gg = d >> 8;
    const int g = (int)(gg % ngroups), mt = (int)(gg / ngroups);
    const int row = mt * kRows + lane % 16, c = (4 * g + j) * 4 + lane / 16;
    dst[d] = (row < Cout && c < C) ? w[(int64_t)row * C + c] : 0.f;
}

// How many channels a thread handles per round of phase 1 (their loads are in flight together); a
// 16-wave workgroup has 128 registers per lane, the smaller ones more.
constexpr int sep_round_channels(int ks, int nw) {
    return ks == 0 ? 8 : (ks == 3 ? (nw == 16 ? 3 : 4) : (ks == 5 ? (nw == 16 ? 1 : 2) : 1));
}

// KS: 0 = no depthwise stage, 3 / 5 / 7 = square depthwise filter of that size (taps unrolled, loads
// without branches: clamped addresses, masked values), -1 = any other filter.
// NW = 4, 8 or 16 waves per workgroup: enough threads that phase 1 is one or two rounds of loads.
template <int KS, int NW>
__device__ __forceinline__ void sepconv_body(const SepConvArgs &a, const int block_x, const int block_y) {
    constexpr int kPre = KS == 0 ? 8 : 4;   // channel groups whose A operands a wave holds in registers per round
    extern __shared__ float lds[];       // B tile [cpad][16] | meeting area [waves][256] | depthwise weights [C][KS*KS]
    constexpr int nt = NW * 64, nw = NW;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cpad = a.ngroups * kGroup;
    float *red = lds + cpad * kPix;
    float *wl = red + nw * 256;
    const int hwo = a.HO * a.WO;
    const int total_pix = a.N * hwo;

    // depthwise weights -> LDS (coalesced; every thread of a 16-lane group reads the same ones later).
    // The first four per thread are only loaded here and written to LDS after every other load of
    // the prologue has been issued: a store to LDS waits for its data, and nothing behind it would
    // go out meanwhile.
    constexpr int kWdEarly = 4;
    float wd_reg[kWdEarly];
    const int nwd = KS > 0 ? a.C * KS * KS : 0;
    if constexpr (KS > 0) {
#pragma unroll
        for (int u = 0; u < kWdEarly; ++u) wd_reg[u] = a.wd[min(tid + u * nt, nwd - 1)];
    }

    // this wave's part of phase 2, and its first A operands (in flight during phase 1)
    const int mi = wave % a.mt_per_wg, kw = wave / a.mt_per_wg;
    const int kparts = nw / a.mt_per_wg;
    const int mt = block_y * a.mt_per_wg + mi;
    const bool have_tile = mt < a.m_tiles;
    const int g0 = kw * a.ngroups / kparts, g1 = (kw + 1) * a.ngroups / kparts;
    const float4 *ap = reinterpret_cast<const float4 *>(a.wp) + ((int64_t)(have_tile ? mt : 0) * a.ngroups) * 64 + lane;
    float4 a_pre[kPre];
#pragma unroll
    for (int u = 0; u < kPre; ++u) {
        a_pre[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (have_tile && g0 + u < g1) a_pre[u] = ap[(int64_t)(g0 + u) * 64];
    }

    // operands of the bias and the residual-add step for the outputs this lane will finish
    // (accumulator r: channel mt*16 + 4*(lane/16) + r, pixel lane%16), fetched now.  A tail outside
    // the common form (EF_GENERIC) is interpreted step by step at the end instead.
    const int ef = a.ef.flags;
    const bool fast = !(ef & EF_GENERIC);
    float e_bias[4] = {0.f, 0.f, 0.f, 0.f}, e_add[4] = {0.f, 0.f, 0.f, 0.f};
    int64_t e_off[4] = {-1, -1, -1, -1};
    if (have_tile && kw == 0) {
        const int p = block_x * kPix + (lane & 15);
        if (p < total_pix) {
            const int n_img = p / hwo, rem = p - n_img * hwo;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int co = mt * kRows + 4 * (lane >> 4) + r;
                if (co >= a.Cout) continue;
                e_off[r] = ((int64_t)n_img * a.Cout + co) * hwo + rem;
                if (fast && (ef & EF_BIAS)) e_bias[r] = a.ef.bias[co];
                if (fast && (ef & EF_ADD)) e_add[r] = a.ef.add[e_off[r]];
            }
        }
    }

    // ---- phase 1: B[c][pixel]
    {
        const int px = tid & 15;
        const int p = block_x * kPix + px;
        const bool valid = p < total_pix;
        const int pc = valid ? p : total_pix - 1;
        const int n_img = pc / hwo, rem = pc - n_img * hwo;
        const int oh = rem / a.WO, ow = rem - oh * a.WO;
        const int ih0 = oh * a.sh - a.ph, iw0 = ow * a.sw - a.pw;
        const int hw = a.H * a.W;
        const float *xb = a.x + (int64_t)n_img * a.C * hw;
        const float lo = a.pro_relu ? 0.f : -INFINITY;
        constexpr int cstep = nt >> 4;                    // channels covered by the workgroup at once
        if constexpr (KS > 0) {
            constexpr int CU = sep_round_channels(KS, NW);
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
            // every thread runs the same number of rounds (the barrier below is inside the loop);
            // channels past the end are clamped for the loads and not stored
            const int rounds = (cpad + cstep * CU - 1) / (cstep * CU);
            for (int it = 0; it < rounds; ++it) {
                const int c0 = (tid >> 4) + it * cstep * CU;
                float xv[CU][KS * KS];
#pragma unroll
                for (int u = 0; u < CU; ++u) {
                    const int c = c0 + u * cstep;
                    const float *xc = xb + (int64_t)(c < a.C ? c : a.C - 1) * hw;
#pragma unroll
                    for (int kh = 0; kh < KS; ++kh)
#pragma unroll
                        for (int kx = 0; kx < KS; ++kx) xv[u][kh * KS + kx] = xc[ro[kh] + co[kx]];
                }
                if (it == 0) {                             // the first round's loads are on their way: now the weights
#pragma unroll
                    for (int u = 0; u < kWdEarly; ++u)
                        if (tid + u * nt < nwd) wl[tid + u * nt] = wd_reg[u];
                    for (int i = tid + kWdEarly * nt; i < nwd; i += nt) wl[i] = a.wd[i];
                    __syncthreads();
                }
#pragma unroll
                for (int u = 0; u < CU; ++u) {
                    const int c = c0 + u * cstep;
                    const float *wc = wl + (c < a.C ? c : a.C - 1) * (KS * KS);
                    float v = 0.f;
#pragma unroll
                    for (int kh = 0; kh < KS; ++kh)
#pragma unroll
                        for (int kx = 0; kx < KS; ++kx) {
                            const float t = (vr[kh] && vc[kx]) ? fmaxf(xv[u][kh * KS + kx], lo) : 0.f;
                            v = fmaf(wc[kh * KS + kx], t, v);
                        }
                    if (c < cpad) lds[c * kPix + px] = (c < a.C && valid) ? v : 0.f;
                }
            }
        } else if constexpr (KS == 0) {
            constexpr int CU = sep_round_channels(0, NW);
            const int64_t at = (int64_t)ih0 * a.W + iw0;        // 1x1, no padding: always inside
            for (int c0 = tid >> 4; c0 < cpad; c0 += cstep * CU) {
                float xv[CU];
#pragma unroll
                for (int u = 0; u < CU; ++u) {
                    const int c = c0 + u * cstep;
                    xv[u] = xb[(int64_t)(c < a.C ? c : a.C - 1) * hw + at];
                }
#pragma unroll
                for (int u = 0; u < CU; ++u) {
                    const int c = c0 + u * cstep;
                    if (c < cpad) lds[c * kPix + px] = (c < a.C && valid) ? fmaxf(xv[u], lo) : 0.f;
                }
            }
        } else {
            for (int c = tid >> 4; c < cpad; c += cstep) {
                float v = 0.f;
                if (c < a.C && valid) {
                    const float *xc = xb + (int64_t)c * hw;
                    const float *wc = a.wd + c * a.KH * a.KW;
                    for (int kh = 0; kh < a.KH; ++kh) {
                        const int ih = ih0 + kh;
                        if (ih < 0 || ih >= a.H) continue;
                        for (int kx = 0; kx < a.KW; ++kx) {
                            const int iw = iw0 + kx;
                            if (iw < 0 || iw >= a.W) continue;
                            v = fmaf(wc[kh * a.KW + kx], fmaxf(xc[ih * a.W + iw], lo), v);
                        }
                    }
                }
                lds[c * kPix + px] = v;
            }
        }
    }
    __syncthreads();

    // ---- phase 2: 16 x 16 output tile, contraction over this wave's channel groups
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    if (have_tile) {
        const float *bp = lds + (lane >> 4) * kPix + (lane & 15);
        for (int gb = g0; gb < g1; gb += kPre) {           // kPre groups per round: their A operands are in registers
#pragma unroll
            for (int u = 0; u < kPre; ++u) {
                if (gb + u < g1) {
                    const float *bg = bp + (gb + u) * (kGroup * kPix);
                    const float4 av = a_pre[u];
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av.x, bg[0 * 4 * kPix], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av.y, bg[1 * 4 * kPix], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av.z, bg[2 * 4 * kPix], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av.w, bg[3 * 4 * kPix], acc, 0, 0, 0);
                }
            }
            if (gb + kPre < g1) {
#pragma unroll
                for (int u = 0; u < kPre; ++u)
                    if (gb + kPre + u < g1) a_pre[u] = ap[(int64_t)(gb + kPre + u) * 64];
            }
        }
    }
    if (kparts > 1) {                                      // uniform over the workgroup
        if (kw > 0)
            for (int r = 0; r < 4; ++r) red[wave * 256 + r * 64 + lane] = acc[r];
        __syncthreads();
        if (kw == 0)
            for (int k2 = 1; k2 < kparts; ++k2)
                for (int r = 0; r < 4; ++r) acc[r] += red[(k2 * a.mt_per_wg + mi) * 256 + r * 64 + lane];
    }
    if (!have_tile || kw != 0) return;

#pragma unroll
    for (int r = 0; r < 4; ++r) {
        if (e_off[r] < 0) continue;
        float v = acc[r];
        if (fast) {
            if (ef & EF_SCALE) v *= a.ef.scale;
            v += e_bias[r];
            v += e_add[r];
            if (ef & EF_RELU) v = v > 0.f ? v : 0.f;
            else if (ef & EF_GELU) v = gelu_erf(v);
            else if (ef & EF_TANH) v = tanhf(v);
        } else {
            v = apply_steps(a.epi, v, e_off[r], mt * kRows + 4 * (lane >> 4) + r);
        }
        a.y[e_off[r]] = v;
    }
}

template <int KS, int NW>
__global__ __launch_bounds__(NW * 64) void sepconv_kernel(SepConvArgs a) {
    sepconv_body<KS, NW>(a, blockIdx.x, blockIdx.y);
}

// Several separable convolutions of one kernel shape (filter size, waves per workgroup) in one launch:
// sibling branches of a cell.  Workgroup -> problem by a wave-uniform look-up, then the problem's own
// (pixel tile, channel-tile block) and exactly the code it runs alone.
template <int KS, int NW>
__global__ __launch_bounds__(NW * 64) void sepconv_multi_kernel(SepMultiArgs m) {
    const int bx = blockIdx.x;
    int k = 0;
#pragma unroll
    for (int i = 0; i + 1 < kMaxSepRegion; ++i) k += (i + 1 < m.n && bx >= m.block_end[i]) ? 1 : 0;
    const int local = bx - (k ? m.block_end[k - 1] : 0);
    const int nt = m.p[k].n_tiles;
    const int by = local / nt;
    sepconv_body<KS, NW>(m.p[k], local - by * nt, by);
}

}  // namespace

// Launch shape for these sizes.  Waves per workgroup: as many as it takes for phase 1 to be about one
// round of loads per thread.  The waves then share phase 2: each takes one 16-row tile of output
// channels, and when there are more waves than tiles (or long channel ranges) several waves split a
// tile's channel range.
static int pow2_ceil(int v) {
    int p = 1;
    while (p < v) p *= 2;
    return p;
}

void sepconv_resolve(SepConvArgs *a) {
    a->ngroups = (a->C + kGroup - 1) / kGroup;
    a->m_tiles = (a->Cout + kRows - 1) / kRows;
    a->n_tiles = (int32_t)(((int64_t)a->N * a->HO * a->WO + kPix - 1) / kPix);
    const int ks = !a->has_dw ? 0 : ((a->KH == a->KW && (a->KH == 3 || a->KH == 5 || a->KH == 7)) ? a->KH : -1);
    a->nwaves = (ks == 5 || ks == 7) ? 8 : 16;                 // those two would not fit 16 waves' register budget
    for (int nw : {8, 4})                                      // the fewest waves that finish phase 1 in one round
        if (a->ngroups * kGroup <= nw * 4 * sep_round_channels(ks, nw)) a->nwaves = nw;
    // waves per tile: so many that a wave's channel groups are all in registers before phase 1
    const int pre = ks == 0 ? 8 : 4;
    const int kparts = std::min(a->nwaves, pow2_ceil((a->ngroups + pre - 1) / pre));
    a->mt_per_wg = std::min(a->nwaves / kparts, pow2_ceil(a->m_tiles));
}

size_t sepconv_pack_bytes(const SepConvArgs &a) {
    return (size_t)a.m_tiles * a.ngroups * 64 * 4 * sizeof(float);
}

size_t sepconv_lds_bytes(const SepConvArgs &a) {
    return ((size_t)a.ngroups * kGroup * kPix + (size_t)a.nwaves * 256 + (a.has_dw ? (size_t)a.C * a.KH * a.KW : 0)) * sizeof(float);
}

int launch_sepconv_pack(const SepConvArgs &a, const float *w, float *dst, void *stream) {
    const int64_t total = (int64_t)a.m_tiles * a.ngroups * 256;
    hipLaunchKernelGGL(sepconv_pack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       w, dst, a.Cout, a.C, a.ngroups, total);
    return (int)hipGetLastError();
}

static int sep_ks(const SepConvArgs &a) {
    return !a.has_dw ? 0 : ((a.KH == a.KW && (a.KH == 3 || a.KH == 5 || a.KH == 7)) ? a.KH : -1);
}

int sepconv_region_key(const SepConvArgs &a) { return (sep_ks(a) + 1) * 100 + a.nwaves; }

int launch_sepconv_region(const SepConvArgs *members, int n, void *stream) {
    if (n < 2 || n > kMaxSepRegion) return (int)hipErrorInvalidValue;
    SepMultiArgs m{};
    m.n = n;
    size_t lds = 0;
    int64_t end = 0;
    const int ks = sep_ks(members[0]), nw = members[0].nwaves;
    for (int k = 0; k < n; ++k) {
        SepConvArgs &a = m.p[k];
        a = members[k];
        a.ef = make_epi_fast(a.epi);
        if (sep_ks(a) != ks || a.nwaves != nw || (a.has_dw != 0) != (a.wd != nullptr)) return (int)hipErrorInvalidValue;
        lds = std::max(lds, sepconv_lds_bytes(a));
        end += (int64_t)a.n_tiles * ((a.m_tiles + a.mt_per_wg - 1) / a.mt_per_wg);
        if (end >= ((int64_t)1 << 31)) return (int)hipErrorInvalidValue;
        m.block_end[k] = (int32_t)end;
    }
    for (int k = n; k < kMaxSepRegion; ++k) m.block_end[k] = (int32_t)end;
    if (lds > 160 * 1024) return (int)hipErrorInvalidValue;
    void (*kern)(SepMultiArgs) = nullptr;
#define CLG_SEP_PICK(KS_, NW_) if (ks == KS_ && nw == NW_) kern = sepconv_multi_kernel<KS_, NW_>;
    CLG_SEP_PICK(-1, 4) CLG_SEP_PICK(-1, 8) CLG_SEP_PICK(-1, 16)
    CLG_SEP_PICK(0, 4) CLG_SEP_PICK(0, 8) CLG_SEP_PICK(0, 16)
    CLG_SEP_PICK(3, 4) CLG_SEP_PICK(3, 8) CLG_SEP_PICK(3, 16)
    CLG_SEP_PICK(5, 4) CLG_SEP_PICK(5, 8) CLG_SEP_PICK(7, 4) CLG_SEP_PICK(7, 8)
#undef CLG_SEP_PICK
    if (!kern) return (int)hipErrorInvalidValue;
    if (lds > 64 * 1024) {
        const hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return (int)e;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)end), dim3(nw * 64), lds, (hipStream_t)stream, m);
    return (int)hipGetLastError();
}

int launch_sepconv(const SepConvArgs &a_in, void *stream) {
    SepConvArgs a = a_in;
    a.ef = make_epi_fast(a.epi);
    const dim3 grid((unsigned)a.n_tiles, (unsigned)((a.m_tiles + a.mt_per_wg - 1) / a.mt_per_wg));
    const size_t lds = sepconv_lds_bytes(a);
    if (lds > 160 * 1024) return (int)hipErrorInvalidValue;
    const int ks = !a.wd ? 0 : ((a.KH == a.KW && (a.KH == 3 || a.KH == 5 || a.KH == 7)) ? a.KH : -1);
    void (*kern)(SepConvArgs) = nullptr;
#define CLG_SEP_PICK(KS_, NW_) if (ks == KS_ && a.nwaves == NW_) kern = sepconv_kernel<KS_, NW_>;
    CLG_SEP_PICK(-1, 4) CLG_SEP_PICK(-1, 8) CLG_SEP_PICK(-1, 16)
    CLG_SEP_PICK(0, 4) CLG_SEP_PICK(0, 8) CLG_SEP_PICK(0, 16)
    CLG_SEP_PICK(3, 4) CLG_SEP_PICK(3, 8) CLG_SEP_PICK(3, 16)
    CLG_SEP_PICK(5, 4) CLG_SEP_PICK(5, 8) CLG_SEP_PICK(7, 4) CLG_SEP_PICK(7, 8)
#undef CLG_SEP_PICK
    if (!kern || (a.has_dw != 0) != (a.wd != nullptr))
        return (int)hipErrorInvalidValue;
    if (lds > 64 * 1024) {
        const hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return (int)e;
    }
    hipLaunchKernelGGL(kern, grid, dim3(a.nwaves * 64), lds, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

}  // namespace clg
