// Grid-barrier probe: what would a persistent kernel that runs several layers pay per layer boundary?
//
// A developer tool, not part of the library (built and run by python -m paper_2111_00655_amd.barrier_probe).
// G workgroups of 256 threads exchange data for `rounds` rounds: in every round each workgroup checks
// 256 values another workgroup wrote in the round before, writes 256 values of its own, and all
// workgroups meet.  That is the traffic pattern of consecutive layers whose tiles live on different
// compute units (and, on this chip, on different dies with separate L2s).  Four ways to order the rounds:
//   launches    one kernel launch per round on one stream (what the library does between layers)
//   fence       one persistent kernel; plain stores and loads, device-scope release / acquire fences
//               around a single arrival counter
//   through     one persistent kernel; the data is written and read with device-scope atomic accesses
//               (they bypass the non-coherent L2s), the counter is relaxed, no fences
//   through8    as `through`, with eight arrival counters (one per workgroup index modulo 8, the way
//               workgroups are dealt to the dies) and a ninth that the last arrival of each adds to
// Every wait is bounded: a wave that has spun 2^18 times sets a flag and every workgroup leaves at its
// next check, so the kernel ends whatever happens.  Mismatches count values that were not the ones
// written in the previous round.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#define CK(x)                                                                      \
    do {                                                                           \
        hipError_t e_ = (x);                                                       \
        if (e_ != hipSuccess) {                                                    \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            exit(1);                                                               \
        }                                                                          \
    } while (0)

constexpr int kSpinMax = 1 << 18;

__device__ __forceinline__ unsigned value_of(int r, int b, int t) { return (unsigned)r * 1048576u + (unsigned)b * 256u + (unsigned)t; }

// ctl[0] arrival counter, ctl[1] time-out flag, ctl[2] mismatches, ctl[16 + 16 k] counter of group k, ctl[160] top counter
template <int MODE>
__global__ __launch_bounds__(256) void persistent(unsigned *buf, unsigned *ctl, int rounds, int G) {
    const int b = blockIdx.x, t = threadIdx.x;
    unsigned bad = 0;
    bool dead = false;
    for (int r = 0; r < rounds && !dead; ++r) {
        unsigned *cur = buf + (size_t)(r & 1) * G * 256;
        const unsigned *prev = buf + (size_t)((r + 1) & 1) * G * 256;
        if (r > 0) {
            const int ob = (b + 37) % G;
            unsigned got;
            if (MODE == 0) got = prev[ob * 256 + t];
            else got = __hip_atomic_load(prev + ob * 256 + t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (got != value_of(r - 1, ob, t)) ++bad;
        }
        if (MODE == 0) cur[b * 256 + t] = value_of(r, b, t);
        else __hip_atomic_store(cur + b * 256 + t, value_of(r, b, t), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (MODE == 0) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        else __builtin_amdgcn_s_waitcnt(0);          // the stores have been acknowledged
        __syncthreads();
        if (t == 0) {
            unsigned *top = ctl;
            unsigned target = (unsigned)(r + 1) * (unsigned)G;
            if (MODE == 2) {
                // the last arrival of a group of workgroups reports for the group
                const int grp = b & 7;
                const unsigned members = (unsigned)((G - grp + 7) / 8);
                const unsigned old = __hip_atomic_fetch_add(ctl + 16 + 16 * grp, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                top = ctl + 160;
                target = (unsigned)(r + 1) * (unsigned)(G < 8 ? G : 8);
                if ((old + 1) % members == 0) __hip_atomic_fetch_add(top, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                __hip_atomic_fetch_add(top, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            int spins = 0;
            while (__hip_atomic_load(top, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
                __builtin_amdgcn_s_sleep(1);
                if (++spins > kSpinMax) {
                    atomicOr(ctl + 1, 1u);
                    break;
                }
            }
        }
        __syncthreads();
        if (MODE == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        if (__hip_atomic_load(ctl + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) dead = true;
    }
    if (bad) atomicAdd(ctl + 2, bad);
}

__global__ __launch_bounds__(256) void one_round(unsigned *buf, unsigned *ctl, int r, int G) {
    const int b = blockIdx.x, t = threadIdx.x;
    unsigned *cur = buf + (size_t)(r & 1) * G * 256;
    const unsigned *prev = buf + (size_t)((r + 1) & 1) * G * 256;
    if (r > 0) {
        const int ob = (b + 37) % G;
        if (prev[ob * 256 + t] != value_of(r - 1, ob, t)) atomicAdd(ctl + 2, 1u);
    }
    cur[b * 256 + t] = value_of(r, b, t);
}

int main() {
    const int rounds = 200;
    const char *names[4] = {"launches", "fence", "through", "through8"};
    printf("%d rounds; microseconds per round (best of 3), time-out flag, mismatches\n", rounds);
    for (int G : {64, 128, 256, 512}) {          // 256 threads each: every workgroup is resident at once (256 compute units)
        unsigned *buf, *ctl;
        CK(hipMalloc(&buf, sizeof(unsigned) * 2 * G * 256));
        CK(hipMalloc(&ctl, 4096));
        hipEvent_t e0, e1;
        CK(hipEventCreate(&e0));
        CK(hipEventCreate(&e1));
        for (int mode = 0; mode < 4; ++mode) {
            float best = 1e9f;
            unsigned flags = 0, bad = 0;
            for (int rep = 0; rep < 3; ++rep) {
                CK(hipMemset(ctl, 0, 4096));
                CK(hipMemset(buf, 0, sizeof(unsigned) * 2 * G * 256));
                CK(hipDeviceSynchronize());
                CK(hipEventRecord(e0));
                if (mode == 0) for (int r = 0; r < rounds; ++r) hipLaunchKernelGGL(one_round, dim3(G), dim3(256), 0, 0, buf, ctl, r, G);
                else if (mode == 1) hipLaunchKernelGGL(persistent<0>, dim3(G), dim3(256), 0, 0, buf, ctl, rounds, G);
                else if (mode == 2) hipLaunchKernelGGL(persistent<1>, dim3(G), dim3(256), 0, 0, buf, ctl, rounds, G);
                else hipLaunchKernelGGL(persistent<2>, dim3(G), dim3(256), 0, 0, buf, ctl, rounds, G);
                CK(hipGetLastError());
                CK(hipEventRecord(e1));
                CK(hipEventSynchronize(e1));
                float ms = 0;
                CK(hipEventElapsedTime(&ms, e0, e1));
                unsigned h[3];
                CK(hipMemcpy(h, ctl, 12, hipMemcpyDeviceToHost));
                best = ms < best ? ms : best;
                flags |= h[1];
                bad += h[2];
            }
            printf("  %3d workgroups  %-9s %7.2f us   timed out %u   mismatches %u\n", G, names[mode], best * 1000.0 / rounds, flags, bad);
            fflush(stdout);
            if (flags) {                               // a wait that did not end: nothing more is started
                printf("stopping: a bounded wait ran out\n");
                return 3;
            }
        }
        CK(hipFree(buf));
        CK(hipFree(ctl));
    }
    return 0;
}
