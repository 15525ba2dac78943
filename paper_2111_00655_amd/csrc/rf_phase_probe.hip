// Phase probe of the register-fed convolution kernel: where the microseconds of one launch go.
//
// A developer tool, not part of the library: it is compiled together with gemm_rf.hip under
// -DCLG_RF_STAMPS (see paper_2111_00655_amd/phase_probe.py), which makes thread 0 of every workgroup
// write the device's 100 MHz wall clock at five points of the kernel.  One invocation runs one
// convolution layer with one kernel shape, checks the result against a direct convolution on the GPU,
// times the launch with and without the L2 scrubbed in front of it, and prints per phase the earliest,
// median and latest workgroup (microseconds after the first workgroup's entry) and the median and
// longest duration of the phase.
//
//   rf_phase_probe TS N Cin Cout H K stride pad waves add
//     TS 16|32 tile edge, N images, H = W input size, K filter size, waves: K-waves per workgroup
//     (0: one chunk of MFMAs per wave), add 1: residual operand in the tail
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "gemm_rf.h"

using namespace clg;

#define CK(x)                                                                      \
    do {                                                                           \
        hipError_t e_ = (x);                                                       \
        if (e_ != hipSuccess) {                                                    \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            exit(1);                                                               \
        }                                                                          \
    } while (0)

__global__ void direct_reference(const float *x, const float *w, const float *bias, const float *add, float *y, int N, int C,
                                 int H, int O, int K, int S, int P, int HO) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long total = (long)N * O * HO * HO;
    if (idx >= total) return;
    const int ow = idx % HO, oh = (idx / HO) % HO, o = (idx / ((long)HO * HO)) % O, n = idx / ((long)HO * HO * O);
    double acc = 0;
    for (int c = 0; c < C; ++c)
        for (int kh = 0; kh < K; ++kh)
            for (int kw = 0; kw < K; ++kw) {
                const int ih = oh * S - P + kh, iw = ow * S - P + kw;
                if (ih < 0 || ih >= H || iw < 0 || iw >= H) continue;
                acc += (double)x[((long)(n * C + c) * H + ih) * H + iw] * w[((long)(o * C + c) * K + kh) * K + kw];
            }
    float v = (float)acc + bias[o];
    if (add) v += add[idx];
    y[idx] = v > 0 ? v : 0;
}

__global__ void hash_fill(float *p, long n, unsigned seed) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    unsigned h = (unsigned)i * 2654435761u + seed;
    h ^= h >> 15;
    h *= 2246822519u;
    h ^= h >> 13;
    p[i] = (h & 0xffff) / 32768.0f - 1.0f;
}

__global__ void scrub(float *p, long n, float v) {
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) p[i] = v;
}

int main(int argc, char **argv) {
    if (argc < 11) {
        printf("usage: rf_phase_probe TS N Cin Cout H K stride pad waves add\n");
        return 1;
    }
    const int ts = atoi(argv[1]), N = atoi(argv[2]), Cin = atoi(argv[3]), Cout = atoi(argv[4]), H = atoi(argv[5]);
    const int K = atoi(argv[6]), S = atoi(argv[7]), P = atoi(argv[8]), waves = atoi(argv[9]), with_add = atoi(argv[10]);
    const int HO = (H + 2 * P - K) / S + 1;
    if ((ts != 16 && ts != 32) || N < 1 || Cin < 1 || Cout < 1 || HO < 1) {
        printf("bad arguments\n");
        return 1;
    }
    GemmArgs a;
    memset(&a, 0, sizeof a);
    a.mode = GM_CONV; a.batch = 1; a.M = Cout; a.N = N * HO * HO; a.K = Cin * K * K;
    a.Nimg = N; a.Cin = Cin; a.H = H; a.W = H; a.Cout = Cout; a.KH = K; a.KW = K; a.sh = S; a.sw = S; a.ph = P; a.pw = P;
    a.HO = HO; a.WO = HO; a.bias_on_row = 1; a.c_numel = (int64_t)N * Cout * HO * HO;
    a.ef.flags = EF_BIAS | EF_RELU | (with_add ? EF_ADD : 0);
    if (!rf_resolve(&a, ts, a.ef.flags, 256, waves)) {
        printf("the register-fed kernel does not take this layer\n");
        return 1;
    }
    const int tiles = ((Cout + ts - 1) / ts) * ((HO * HO + ts - 1) / ts);
    const int nwg = tiles * N;
    if (nwg > 65536) {
        printf("too many workgroups for the stamp buffer\n");
        return 1;
    }
    const size_t xn = (size_t)N * Cin * H * H, wn = (size_t)Cout * Cin * K * K, yn = (size_t)a.c_numel;
    float *x, *w, *bias, *add, *y, *yref, *packed, *junk;
    long long *stamps;
    const long junk_n = 32l << 20;                 // 128 MB: more than the eight L2s hold
    CK(hipMalloc(&x, xn * 4)); CK(hipMalloc(&w, wn * 4)); CK(hipMalloc(&bias, Cout * 4)); CK(hipMalloc(&add, yn * 4));
    CK(hipMalloc(&y, yn * 4)); CK(hipMalloc(&yref, yn * 4)); CK(hipMalloc(&packed, rf_pack_bytes(a)));
    CK(hipMalloc(&junk, junk_n * 4)); CK(hipMalloc(&stamps, (size_t)65536 * 8 * 8));
    CK(hipMemset(stamps, 0, (size_t)65536 * 8 * 8));
    rf_set_stamps(stamps);
    hash_fill<<<(xn + 255) / 256, 256>>>(x, xn, 1);
    hash_fill<<<(wn + 255) / 256, 256>>>(w, wn, 2);
    hash_fill<<<(Cout + 255) / 256, 256>>>(bias, Cout, 3);
    hash_fill<<<(yn + 255) / 256, 256>>>(add, yn, 4);
    CK(hipMemset(y, 0xff, yn * 4));
    direct_reference<<<(yn + 255) / 256, 256>>>(x, w, bias, with_add ? add : nullptr, yref, N, Cin, H, Cout, K, S, P, HO);
    CK(hipDeviceSynchronize());
    if (launch_rf_pack(a, w, packed, nullptr)) { printf("pack launch failed\n"); return 1; }
    a.A = packed; a.B = x; a.C = y; a.ef.bias = bias; a.ef.add = with_add ? add : nullptr;
    if (launch_rf_conv(a, nullptr)) { printf("launch failed\n"); return 1; }
    CK(hipDeviceSynchronize());
    std::vector<float> hy(yn), hr(yn);
    CK(hipMemcpy(hy.data(), y, yn * 4, hipMemcpyDeviceToHost));
    CK(hipMemcpy(hr.data(), yref, yn * 4, hipMemcpyDeviceToHost));
    double maxerr = 0, maxref = 0;
    for (size_t i = 0; i < yn; ++i) {
        maxerr = std::max(maxerr, (double)std::fabs(hy[i] - hr[i]));
        maxref = std::max(maxref, (double)std::fabs(hr[i]));
        if (std::isnan(hy[i])) maxerr = 1e30;
    }
    const bool ok = maxerr <= 1e-4 * std::max(1.0, maxref);

    // launch-inclusive time of back-to-back launches (everything cached)
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    for (int i = 0; i < 30; ++i) launch_rf_conv(a, nullptr);
    float hot_us = 1e9f;
    for (int b = 0; b < 5; ++b) {
        CK(hipEventRecord(e0));
        for (int i = 0; i < 100; ++i) launch_rf_conv(a, nullptr);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        float ms;
        CK(hipEventElapsedTime(&ms, e0, e1));
        hot_us = std::min(hot_us, ms * 10.f);
    }
    printf("tile %d  %d -> %d channels  %dx%d  filter %d stride %d pad %d  residual %d | tap mode %d  K-waves %d  chunks per wave %d  "
           "workgroups %d | %.2f us per launch back to back | max error %.1e of %.1f %s\n",
           ts, Cin, Cout, H, H, K, S, P, with_add, a.rf_tapk, a.rf_wgk, a.rf_nch, nwg, hot_us, maxerr, maxref, ok ? "OK" : "MISMATCH");

    const char *phase[5] = {"entry", "set-up done", "K loop done", "K-waves met", "stores out"};
    for (int cold = 0; cold < 2; ++cold) {
        std::vector<std::vector<double>> at(5), len(5);
        for (int rep = 0; rep < 9; ++rep) {
            if (cold) scrub<<<2048, 256>>>(junk, junk_n, (float)rep);      // the L2s now hold none of the layer's operands
            CK(hipDeviceSynchronize());
            launch_rf_conv(a, nullptr);
            CK(hipDeviceSynchronize());
            std::vector<long long> h((size_t)nwg * 8);
            CK(hipMemcpy(h.data(), stamps, h.size() * 8, hipMemcpyDeviceToHost));
            long long t0 = h[0];
            for (int g = 0; g < nwg; ++g) t0 = std::min(t0, h[(size_t)g * 8]);
            for (int i = 0; i < 5; ++i)
                for (int g = 0; g < nwg; ++g) {
                    at[i].push_back((h[(size_t)g * 8 + i] - t0) * 0.01);
                    if (i) len[i].push_back((h[(size_t)g * 8 + i] - h[(size_t)g * 8 + i - 1]) * 0.01);
                }
        }
        printf("  %s (us after the first workgroup's entry; over %d workgroups x 9 launches)\n",
               cold ? "L2 scrubbed before the launch (operands come from the memory-side cache / HBM, as inside a network)"
                    : "operands in the L2 (the same launch repeated)", nwg);
        for (int i = 0; i < 5; ++i) {
            std::sort(at[i].begin(), at[i].end());
            printf("    %-12s first %5.2f  median %5.2f  last %5.2f", phase[i], at[i].front(), at[i][at[i].size() / 2], at[i].back());
            if (i) {
                std::sort(len[i].begin(), len[i].end());
                printf("   | phase takes: median %4.2f  longest %4.2f", len[i][len[i].size() / 2], len[i].back());
            }
            printf("\n");
        }
    }
    return ok ? 0 : 2;
}
