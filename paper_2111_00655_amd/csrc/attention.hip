// Scaled-dot-product attention as ONE kernel (gfx950):
//   batch_matmul(q, k^T) -> [mul_scalar] -> softmax -> batch_matmul(p, v) [-> transpose -> reshape]
// i.e. out[h] = softmax(scale * q[h] k[h]^T) v[h] per head h, the heads optionally merged on store
// ([H, S, d] -> [S, H*d]).  Run operator by operator this is three launches plus the score tensor's
// round trip through memory; at batch 1 and sequence 128 (BERT-base, paper Sec. 5.1) each of them
// is a few microseconds of mostly launch.
//
// A workgroup (4 waves) owns 16 query rows of one head.  Scores: the 16 x Sk block is cut into
// 16 x 16 tiles (v_mfma_f32_16x16x4_f32, contraction over d), a tile per wave and round; q and k are
// both read 16 bytes per lane along d: lane (slot s, row r) takes elements 16g + 4s .. + 3 of its row
// for the four MFMAs of group g - the order of the contraction index does not matter as long as both
// operands use the same one.  The scaled scores go to LDS; each wave then normalises four rows
// (sixteen lanes per row: max, exp, sum); the probabilities stay in LDS and are the A operand of the
// second product (read 16 bytes per lane, the same index order), v is the B operand, 4 bytes per lane
// along d.  Nothing but q, k, v and the result touches memory.
#include <algorithm>

#include <hip/hip_runtime.h>

#include "device_common.h"
#include "kernels.h"

namespace clg {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// Value of another lane of the same row of 16 lanes through the data-parallel-primitive path of the
// vector ALU (no LDS round trip as a general shuffle has): CTRL 0xB1 = lane ^ 1, 0x4E = lane ^ 2
// (quad permutations), 0x141 = mirror within 8 lanes, 0x140 = mirror within 16 lanes.  Applied in
// this order with max or + they leave the reduction over the 16 lanes in every one of them.
template <int CTRL>
__device__ __forceinline__ float dpp_peer(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float row16_max(float v) {
    v = fmaxf(v, dpp_peer<0xB1>(v));
    v = fmaxf(v, dpp_peer<0x4E>(v));
    v = fmaxf(v, dpp_peer<0x141>(v));
    return fmaxf(v, dpp_peer<0x140>(v));
}
__device__ __forceinline__ float row16_sum(float v) {
    v += dpp_peer<0xB1>(v);
    v += dpp_peer<0x4E>(v);
    v += dpp_peer<0x141>(v);
    return v + dpp_peer<0x140>(v);
}

constexpr int kRows = 16;          // query rows per workgroup
constexpr int kMaxKeys = 512;
constexpr int kVPre = 8;           // key groups whose v operands a wave loads ahead

// D16 = head size / 16.  MAXT = score tiles per wave the code is unrolled for: 2 (up to 128 keys) or
// 8 (up to 512); the short form is a third of the code, and a kernel of a few microseconds that starts
// with a cold instruction cache feels its length.
template <int D16, int MAXT>
__global__ __launch_bounds__(256) void attention_kernel(AttentionArgs a) {
    constexpr int kMaxTiles = MAXT;
    extern __shared__ float lds[];                           // [16][ldp]: scores, then probabilities
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, s = lane >> 4;
    const int h = blockIdx.y, q0 = blockIdx.x * kRows;
    constexpr int d = D16 * 16;
    const int nct = (a.Sk + 15) / 16;                        // key tiles = key groups of the second product
    const int ldp = nct * 16 + 4;
    const float *Q = a.q + (int64_t)h * a.Sq * d;
    const float *K = a.k + (int64_t)h * a.Sk * d;
    const float *V = a.v + (int64_t)h * a.Sk * d;

    // ---- scores: tile t = wave + 4u of this wave
    const float4 *qp = reinterpret_cast<const float4 *>(Q + (int64_t)min(q0 + r, a.Sq - 1) * d) + s;
    float4 qa[D16];
#pragma unroll
    for (int g = 0; g < D16; ++g) qa[g] = qp[4 * g];
    // two tiles per round: their k rows are loaded together (one memory latency per round, tiles past
    // the end re-read the last key row and are not stored), and their MFMA chains are interleaved
    floatx4 acc[kMaxTiles];
#pragma unroll
    for (int u = 0; u < kMaxTiles; u += 2) {
        acc[u] = floatx4{0.f, 0.f, 0.f, 0.f};
        acc[u + 1] = floatx4{0.f, 0.f, 0.f, 0.f};
        const int t0 = wave + 4 * u, t1 = t0 + 4;
        if (t0 < nct) {                                      // uniform over the wave
            const float4 *kp0 = reinterpret_cast<const float4 *>(K + (int64_t)min(t0 * 16 + r, a.Sk - 1) * d) + s;
            const float4 *kp1 = reinterpret_cast<const float4 *>(K + (int64_t)min(t1 * 16 + r, a.Sk - 1) * d) + s;
            float4 kb0[D16], kb1[D16];
#pragma unroll
            for (int g = 0; g < D16; ++g) {
                kb0[g] = kp0[4 * g];
                kb1[g] = kp1[4 * g];
            }
#pragma unroll
            for (int g = 0; g < D16; ++g) {
                acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[g].x, kb0[g].x, acc[u], 0, 0, 0);
                acc[u + 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[g].x, kb1[g].x, acc[u + 1], 0, 0, 0);
                acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[g].y, kb0[g].y, acc[u], 0, 0, 0);
                acc[u + 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[g].y, kb1[g].y, acc[u + 1], 0, 0, 0);
                acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[g].z, kb0[g].z, acc[u], 0, 0, 0);
                acc[u + 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[g].z, kb1[g].z, acc[u + 1], 0, 0, 0);
                acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[g].w, kb0[g].w, acc[u], 0, 0, 0);
                acc[u + 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[g].w, kb1[g].w, acc[u + 1], 0, 0, 0);
            }
        }
    }
    // v operands of the first key groups of this wave's first output tile: in flight during the softmax
    const int vt = wave;                                     // output tile (16 columns of d) of this wave, first round
    float vb[kVPre][4];
    if (vt < D16) {
#pragma unroll
        for (int g = 0; g < kVPre; ++g)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                vb[g][q] = g < nct ? V[(int64_t)min(16 * g + 4 * s + q, a.Sk - 1) * d + vt * 16 + r] : 0.f;
    }
    // accumulator g of a lane: row 4s + g, column r of the tile
#pragma unroll
    for (int u = 0; u < kMaxTiles; ++u) {
        const int t = wave + 4 * u;
        if (t < nct) {
            const int col = t * 16 + r;
#pragma unroll
            for (int g = 0; g < 4; ++g) lds[(4 * s + g) * ldp + col] = col < a.Sk ? acc[u][g] * a.scale : -INFINITY;
        }
    }
    __syncthreads();

    // ---- softmax: this wave's four rows at once, sixteen lanes (one slot s) per row, a lane takes the
    // columns r, r + 16, ...; the reductions stay within 16 lanes (four exchange steps instead of six,
    // and one pass instead of four)
    {
        float *row = lds + (4 * wave + s) * ldp;
        float v[4 * kMaxTiles];                                            // 4 * MAXT >= nct
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4 * kMaxTiles; ++i) {
            v[i] = i < nct ? row[r + 16 * i] : -INFINITY;
            mx = fmaxf(mx, v[i]);
        }
        mx = row16_max(mx);
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < 4 * kMaxTiles; ++i) {
            v[i] = i < nct ? __expf(v[i] - mx) : 0.f;                     // exp(-inf) = 0 for the padded columns
            sum += v[i];
        }
        sum = row16_sum(sum);
        const float inv = 1.0f / sum;
#pragma unroll
        for (int i = 0; i < 4 * kMaxTiles; ++i)
            if (i < nct) row[r + 16 * i] = v[i] * inv;
    }
    __syncthreads();

    // ---- out tile = P[16 x Sk] V[Sk x 16]; A operand from LDS (row r), 16 bytes per lane
    for (int t = wave; t < D16; t += 4) {
        // two accumulators, even and odd key groups: half as long a chain of dependent MFMAs
        floatx4 o = {0.f, 0.f, 0.f, 0.f}, o2 = {0.f, 0.f, 0.f, 0.f};
        const float *prow = lds + r * ldp + 4 * s;
        int g = 0;
        if (t == vt) {                                       // the key groups whose v operands are already in registers
#pragma unroll
            for (int gg = 0; gg < kVPre; gg += 2) {
                if (gg < nct) {
                    const float4 pa = *reinterpret_cast<const float4 *>(prow + 16 * gg);
                    float4 pb = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (gg + 1 < nct) pb = *reinterpret_cast<const float4 *>(prow + 16 * (gg + 1));
                    o = __builtin_amdgcn_mfma_f32_16x16x4f32(pa.x, vb[gg][0], o, 0, 0, 0);
                    o2 = __builtin_amdgcn_mfma_f32_16x16x4f32(pb.x, vb[gg + 1][0], o2, 0, 0, 0);
                    o = __builtin_amdgcn_mfma_f32_16x16x4f32(pa.y, vb[gg][1], o, 0, 0, 0);
                    o2 = __builtin_amdgcn_mfma_f32_16x16x4f32(pb.y, vb[gg + 1][1], o2, 0, 0, 0);
                    o = __builtin_amdgcn_mfma_f32_16x16x4f32(pa.z, vb[gg][2], o, 0, 0, 0);
                    o2 = __builtin_amdgcn_mfma_f32_16x16x4f32(pb.z, vb[gg + 1][2], o2, 0, 0, 0);
                    o = __builtin_amdgcn_mfma_f32_16x16x4f32(pa.w, vb[gg][3], o, 0, 0, 0);
                    o2 = __builtin_amdgcn_mfma_f32_16x16x4f32(pb.w, vb[gg + 1][3], o2, 0, 0, 0);
                }
            }
            g = min(nct, kVPre);
        }
        for (; g < nct; ++g) {
            const float4 pa = *reinterpret_cast<const float4 *>(prow + 16 * g);
            float b[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) b[q] = V[(int64_t)min(16 * g + 4 * s + q, a.Sk - 1) * d + t * 16 + r];
            o = __builtin_amdgcn_mfma_f32_16x16x4f32(pa.x, b[0], o, 0, 0, 0);
            o = __builtin_amdgcn_mfma_f32_16x16x4f32(pa.y, b[1], o, 0, 0, 0);
            o = __builtin_amdgcn_mfma_f32_16x16x4f32(pa.z, b[2], o, 0, 0, 0);
            o = __builtin_amdgcn_mfma_f32_16x16x4f32(pa.w, b[3], o, 0, 0, 0);
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) o[g] += o2[g];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int qi = q0 + 4 * s + g;
            if (qi >= a.Sq) continue;
            const int64_t off = a.merge ? ((int64_t)qi * a.B + h) * d + t * 16 + r : ((int64_t)h * a.Sq + qi) * d + t * 16 + r;
            a.y[off] = o[g];
        }
    }
}

}  // namespace

bool attention_shape_ok(const AttentionArgs &a) {
    return a.B >= 1 && a.B <= 65535 && a.Sq >= 1 && a.Sk >= 1 && a.Sk <= kMaxKeys &&
           (a.d == 32 || a.d == 64 || a.d == 128) && (int64_t)a.Sq * a.d < ((int64_t)1 << 31);
}

int launch_attention(const AttentionArgs &a, void *stream) {
    if (!attention_shape_ok(a)) return (int)hipErrorInvalidValue;
    for (const void *p : {(const void *)a.q, (const void *)a.k})
        if (((uintptr_t)p & 15) != 0) return (int)hipErrorInvalidValue;        // rows are read 16 bytes at a time
    const dim3 grid((unsigned)((a.Sq + kRows - 1) / kRows), (unsigned)a.B);
    const int nct = (a.Sk + 15) / 16;
    const size_t lds = (size_t)kRows * (nct * 16 + 4) * sizeof(float);
    void (*kern)(AttentionArgs);
    if (a.Sk <= 128) kern = a.d == 32 ? attention_kernel<2, 2> : (a.d == 64 ? attention_kernel<4, 2> : attention_kernel<8, 2>);
    else kern = a.d == 32 ? attention_kernel<2, 8> : (a.d == 64 ? attention_kernel<4, 8> : attention_kernel<8, 8>);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

}  // namespace clg
