/*
 * CPU oracle: plain definitions of the primitive tensor operators.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the parity anchor for the GPU
 * library: only the tests, the smoke check and the benchmark's cpu_baseline
 * leg may build, load or call it.  It shares no code with the GPU path.
 *
 * Every operator is its textbook definition written as direct loops, with all
 * sums carried in double and the result rounded to float once, at the
 * operator's output.  A fused group of operators therefore equals the same
 * operators run one after the other, bit for bit (paper Sec. 4.2: a matched
 * subgraph is one or several operators lowered to one kernel; fusing must not
 * change what is computed).  Layouts: activations NCHW, conv weights OIHW,
 * transposed-conv weights IOHW, dense weights [units, in] (paper Sec. 3
 * listing: the conv patterns constrain data_layout to NCHW).
 *
 * Nothing here is blocked, tiled or reordered beyond the definition.  The
 * only concession to run time is an OpenMP "parallel for" over the outermost
 * output dimension, which does not change any result.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

void orc_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* y[n,co,oh,ow] = sum_{ci,kh,kw} x[n, g*Cg+ci, oh*s-p+kh, ow*s-p+kw] * w[co,ci,kh,kw]
 * with g = co / (O/G), Cg = C/G, out-of-range x = 0 (cross-correlation). */
void orc_conv2d(const float *x, const float *w, float *y,
                int N, int C, int H, int W, int O, int KH, int KW,
                int sh, int sw, int ph, int pw, int G)
{
    const int Cg = C / G, Og = O / G;
    const int HO = (H + 2 * ph - KH) / sh + 1;
    const int WO = (W + 2 * pw - KW) / sw + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < O; ++co) {
            const int g = co / Og;
            for (int oh = 0; oh < HO; ++oh)
                for (int ow = 0; ow < WO; ++ow) {
                    double acc = 0.0;
                    for (int ci = 0; ci < Cg; ++ci)
                        for (int kh = 0; kh < KH; ++kh) {
                            const int ih = oh * sh - ph + kh;
                            if (ih < 0 || ih >= H) continue;
                            for (int kw = 0; kw < KW; ++kw) {
                                const int iw = ow * sw - pw + kw;
                                if (iw < 0 || iw >= W) continue;
                                const double xv = x[(((size_t)n * C + g * Cg + ci) * H + ih) * W + iw];
                                const double wv = w[(((size_t)co * Cg + ci) * KH + kh) * KW + kw];
                                acc += xv * wv;
                            }
                        }
                    y[(((size_t)n * O + co) * HO + oh) * WO + ow] = (float)acc;
                }
        }
}

/* 3-D convolution (3D-ResNet50, paper Sec. 5.1): x[N,C,D,H,W], w[O,C,KD,KH,KW];
 * y[n,co,od,oh,ow] = sum_{ci,kd,kh,kw} x[n,ci,od*sd-pd+kd,oh*sh-ph+kh,ow*sw-pw+kw] * w[co,ci,kd,kh,kw],
 * zero padding. */
void orc_conv3d(const float *x, const float *w, float *y,
                int N, int C, int D, int H, int W, int O, int KD, int KH, int KW,
                int sd, int sh, int sw, int pd, int ph, int pw)
{
    const int DO = (D + 2 * pd - KD) / sd + 1;
    const int HO = (H + 2 * ph - KH) / sh + 1;
    const int WO = (W + 2 * pw - KW) / sw + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < O; ++co)
            for (int od = 0; od < DO; ++od)
                for (int oh = 0; oh < HO; ++oh)
                    for (int ow = 0; ow < WO; ++ow) {
                        double acc = 0.0;
                        for (int ci = 0; ci < C; ++ci)
                            for (int kd = 0; kd < KD; ++kd) {
                                const int id = od * sd - pd + kd;
                                if (id < 0 || id >= D) continue;
                                for (int kh = 0; kh < KH; ++kh) {
                                    const int ih = oh * sh - ph + kh;
                                    if (ih < 0 || ih >= H) continue;
                                    for (int kw = 0; kw < KW; ++kw) {
                                        const int iw = ow * sw - pw + kw;
                                        if (iw < 0 || iw >= W) continue;
                                        const double xv = x[((((size_t)n * C + ci) * D + id) * H + ih) * W + iw];
                                        const double wv = w[((((size_t)co * C + ci) * KD + kd) * KH + kh) * KW + kw];
                                        acc += xv * wv;
                                    }
                                }
                            }
                        y[((((size_t)n * O + co) * DO + od) * HO + oh) * WO + ow] = (float)acc;
                    }
}

/* max over the 3-D window; padding counts as -infinity */
void orc_max_pool3d(const float *x, float *y, int NC, int D, int H, int W,
                    int KD, int KH, int KW, int sd, int sh, int sw, int pd, int ph, int pw)
{
    const int DO = (D + 2 * pd - KD) / sd + 1;
    const int HO = (H + 2 * ph - KH) / sh + 1;
    const int WO = (W + 2 * pw - KW) / sw + 1;
    for (int nc = 0; nc < NC; ++nc)
        for (int od = 0; od < DO; ++od)
            for (int oh = 0; oh < HO; ++oh)
                for (int ow = 0; ow < WO; ++ow) {
                    float best = -INFINITY;
                    for (int kd = 0; kd < KD; ++kd) {
                        const int id = od * sd - pd + kd;
                        if (id < 0 || id >= D) continue;
                        for (int kh = 0; kh < KH; ++kh) {
                            const int ih = oh * sh - ph + kh;
                            if (ih < 0 || ih >= H) continue;
                            for (int kw = 0; kw < KW; ++kw) {
                                const int iw = ow * sw - pw + kw;
                                if (iw < 0 || iw >= W) continue;
                                const float v = x[(((size_t)nc * D + id) * H + ih) * W + iw];
                                if (v > best) best = v;
                            }
                        }
                    }
                    y[(((size_t)nc * DO + od) * HO + oh) * WO + ow] = best;
                }
}

/* y[n,co,oh,ow] = sum over (ci,ih,iw,kh,kw) with oh = ih*s-p+kh, ow = iw*s-p+kw
 * of x[n,ci,ih,iw] * w[ci,co,kh,kw];  HO = (H-1)*s - 2p + KH. */
void orc_conv2d_transpose(const float *x, const float *w, float *y,
                          int N, int C, int H, int W, int O, int KH, int KW,
                          int sh, int sw, int ph, int pw)
{
    const int HO = (H - 1) * sh - 2 * ph + KH;
    const int WO = (W - 1) * sw - 2 * pw + KW;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < O; ++co)
            for (int oh = 0; oh < HO; ++oh)
                for (int ow = 0; ow < WO; ++ow) {
                    double acc = 0.0;
                    for (int ci = 0; ci < C; ++ci)
                        for (int kh = 0; kh < KH; ++kh) {
                            const int th = oh + ph - kh;
                            if (th < 0 || th % sh != 0) continue;
                            const int ih = th / sh;
                            if (ih >= H) continue;
                            for (int kw = 0; kw < KW; ++kw) {
                                const int tw = ow + pw - kw;
                                if (tw < 0 || tw % sw != 0) continue;
                                const int iw = tw / sw;
                                if (iw >= W) continue;
                                const double xv = x[(((size_t)n * C + ci) * H + ih) * W + iw];
                                const double wv = w[(((size_t)ci * O + co) * KH + kh) * KW + kw];
                                acc += xv * wv;
                            }
                        }
                    y[(((size_t)n * O + co) * HO + oh) * WO + ow] = (float)acc;
                }
}

/* y[m,u] = sum_k x[m,k] * w[u,k] */
void orc_dense(const float *x, const float *w, float *y, int M, int K, int U)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int m = 0; m < M; ++m)
        for (int u = 0; u < U; ++u) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += (double)x[(size_t)m * K + k] * (double)w[(size_t)u * K + k];
            y[(size_t)m * U + u] = (float)acc;
        }
}

/* y[b,m,n] = sum_k a[b,m,k] * (tb ? bm[b,n,k] : bm[b,k,n]) */
void orc_batch_matmul(const float *a, const float *bm, float *y,
                      int B, int M, int N, int K, int tb)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int m = 0; m < M; ++m)
            for (int n = 0; n < N; ++n) {
                double acc = 0.0;
                for (int k = 0; k < K; ++k) {
                    const double av = a[((size_t)b * M + m) * K + k];
                    const double bv = tb ? bm[((size_t)b * N + n) * K + k]
                                         : bm[((size_t)b * K + k) * N + n];
                    acc += av * bv;
                }
                y[((size_t)b * M + m) * N + n] = (float)acc;
            }
}

/* x viewed as [outer, C, inner]; y = x + b[c] */
void orc_bias_add(const float *x, const float *b, float *y,
                  int64_t outer, int64_t C, int64_t inner)
{
    for (int64_t o = 0; o < outer; ++o)
        for (int64_t c = 0; c < C; ++c)
            for (int64_t i = 0; i < inner; ++i) {
                const size_t k = ((size_t)o * C + c) * inner + i;
                y[k] = (float)((double)x[k] + (double)b[c]);
            }
}

void orc_add(const float *x, const float *z, float *y, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) y[i] = (float)((double)x[i] + (double)z[i]);
}

void orc_mul_scalar(const float *x, double s, float *y, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) y[i] = (float)((double)x[i] * s);
}

void orc_relu(const float *x, float *y, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) y[i] = x[i] > 0.0f ? x[i] : 0.0f;
}

/* gelu(x) = x/2 * (1 + erf(x / sqrt 2)) */
void orc_gelu(const float *x, float *y, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        const double v = x[i];
        y[i] = (float)(0.5 * v * (1.0 + erf(v / sqrt(2.0))));
    }
}

void orc_tanh(const float *x, float *y, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) y[i] = (float)tanh((double)x[i]);
}

/* softmax over the last axis: exp(x - max) / sum exp(x - max) */
void orc_softmax(const float *x, float *y, int64_t rows, int64_t len)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const float *xr = x + (size_t)r * len;
        float *yr = y + (size_t)r * len;
        double mx = xr[0];
        for (int64_t i = 1; i < len; ++i) if (xr[i] > mx) mx = xr[i];
        double sum = 0.0;
        for (int64_t i = 0; i < len; ++i) sum += exp((double)xr[i] - mx);
        for (int64_t i = 0; i < len; ++i) yr[i] = (float)(exp((double)xr[i] - mx) / sum);
    }
}

/* layer norm over the last axis with the biased variance */
void orc_layer_norm(const float *x, const float *gamma, const float *beta,
                    float *y, int64_t rows, int64_t len, double eps)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const float *xr = x + (size_t)r * len;
        float *yr = y + (size_t)r * len;
        double mean = 0.0;
        for (int64_t i = 0; i < len; ++i) mean += xr[i];
        mean /= (double)len;
        double var = 0.0;
        for (int64_t i = 0; i < len; ++i) {
            const double d = (double)xr[i] - mean;
            var += d * d;
        }
        var /= (double)len;
        const double inv = 1.0 / sqrt(var + eps);
        for (int64_t i = 0; i < len; ++i)
            yr[i] = (float)(((double)xr[i] - mean) * inv * (double)gamma[i] + (double)beta[i]);
    }
}

/* max over the window; padding counts as -infinity */
void orc_max_pool2d(const float *x, float *y, int N, int C, int H, int W,
                    int KH, int KW, int sh, int sw, int ph, int pw)
{
    const int HO = (H + 2 * ph - KH) / sh + 1;
    const int WO = (W + 2 * pw - KW) / sw + 1;
    for (int nc = 0; nc < N * C; ++nc)
        for (int oh = 0; oh < HO; ++oh)
            for (int ow = 0; ow < WO; ++ow) {
                float best = -INFINITY;
                for (int kh = 0; kh < KH; ++kh) {
                    const int ih = oh * sh - ph + kh;
                    if (ih < 0 || ih >= H) continue;
                    for (int kw = 0; kw < KW; ++kw) {
                        const int iw = ow * sw - pw + kw;
                        if (iw < 0 || iw >= W) continue;
                        const float v = x[((size_t)nc * H + ih) * W + iw];
                        if (v > best) best = v;
                    }
                }
                y[((size_t)nc * HO + oh) * WO + ow] = best;
            }
}

/* mean over the part of the window that lies inside the image (padding is
 * not counted, neither in the sum nor in the divisor) */
void orc_avg_pool2d(const float *x, float *y, int N, int C, int H, int W,
                    int KH, int KW, int sh, int sw, int ph, int pw)
{
    const int HO = (H + 2 * ph - KH) / sh + 1;
    const int WO = (W + 2 * pw - KW) / sw + 1;
    for (int nc = 0; nc < N * C; ++nc)
        for (int oh = 0; oh < HO; ++oh)
            for (int ow = 0; ow < WO; ++ow) {
                double acc = 0.0;
                int cnt = 0;
                for (int kh = 0; kh < KH; ++kh) {
                    const int ih = oh * sh - ph + kh;
                    if (ih < 0 || ih >= H) continue;
                    for (int kw = 0; kw < KW; ++kw) {
                        const int iw = ow * sw - pw + kw;
                        if (iw < 0 || iw >= W) continue;
                        acc += x[((size_t)nc * H + ih) * W + iw];
                        ++cnt;
                    }
                }
                y[((size_t)nc * HO + oh) * WO + ow] = cnt ? (float)(acc / (double)cnt) : 0.0f;
            }
}

/* mean over H*W; output [N, C] */
void orc_global_avg_pool2d(const float *x, float *y, int NC, int HW)
{
    for (int nc = 0; nc < NC; ++nc) {
        double acc = 0.0;
        for (int i = 0; i < HW; ++i) acc += x[(size_t)nc * HW + i];
        y[nc] = (float)(acc / (double)HW);
    }
}

/* y[l,:] = table[ids[l],:]; returns -1 on an id outside [0,V) */
int orc_take(const float *table, const int32_t *ids, float *y,
             int64_t L, int64_t Hd, int64_t V)
{
    for (int64_t l = 0; l < L; ++l) {
        if (ids[l] < 0 || ids[l] >= V) return -1;
        for (int64_t h = 0; h < Hd; ++h)
            y[(size_t)l * Hd + h] = table[(size_t)ids[l] * Hd + h];
    }
    return 0;
}
