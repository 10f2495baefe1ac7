/*
 * CPU oracle for layer-by-layer (unfused) CNN inference.  TEST INFRASTRUCTURE ONLY: it is called
 * by the tests, by the smoke check and by the benchmark's CPU-baseline leg, never by the GPU
 * library, and it shares no code with it.
 *
 * Layer fusion is an execution schedule that is mathematically equivalent to running the layers
 * one after another (paper, Sec. I and Sec. III-B), so the oracle is the plain definition of each
 * layer, written as direct nested loops over NHWC tensors, with no tiling, blocking or fusion.
 *
 *   convolution (cross-correlation, zero padding, optional channel groups):
 *     out[n,y,x,co] = bias[co] + sum_{kh,kw,ci} in[n, y*s-p+kh, x*s-p+kw, g*cig+ci] * w[co,kh,kw,ci]
 *     with Hout = floor((H + 2p - Kh)/s) + 1, the Hout/Wout that Eq. 1 counts operations over;
 *     terms whose input coordinate falls outside the image contribute nothing.
 *   fully connected (Eq. 2, M = batch): out[n,co] = bias[co] + sum_k in[n,k] * w[co,k]
 *   max pooling pads with -infinity; global average pooling is the mean over H*W.
 *
 * Precision: every function has two builds, `_f32` (float accumulator; summation order kh, kw,
 * ci ascending) and `_f64` (double accumulator, rounded to float once at the end).  Tensors are
 * float in both; callers pass values that are already rounded to fp16 where the workload says so.
 * OpenMP splits work over (n, y) only, so the result for each output element does not depend on
 * the thread count.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Threads the loops below will use (reported next to oracle timings). */
int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

#define ORC_DEFINE_CONV(NAME, ACC)                                                              \
void NAME(const float* in, int N, int H, int W, int Cin, const float* w, const float* bias,     \
          int Cout, int Kh, int Kw, int stride, int pad, int groups, float* out)                \
{                                                                                               \
    const int Ho = (H + 2 * pad - Kh) / stride + 1;                                             \
    const int Wo = (W + 2 * pad - Kw) / stride + 1;                                             \
    const int cig = Cin / groups;  /* input channels per group  */                              \
    const int cog = Cout / groups; /* output channels per group */                              \
    _Pragma("omp parallel for collapse(2) schedule(static)")                                    \
    for (int n = 0; n < N; ++n)                                                                 \
        for (int y = 0; y < Ho; ++y)                                                            \
            for (int x = 0; x < Wo; ++x)                                                        \
                for (int co = 0; co < Cout; ++co) {                                             \
                    const int g = co / cog;                                                     \
                    ACC acc = bias ? (ACC)bias[co] : (ACC)0;                                    \
                    for (int kh = 0; kh < Kh; ++kh) {                                           \
                        const int iy = y * stride - pad + kh;                                   \
                        if (iy < 0 || iy >= H) continue;                                        \
                        for (int kw = 0; kw < Kw; ++kw) {                                       \
                            const int ix = x * stride - pad + kw;                               \
                            if (ix < 0 || ix >= W) continue;                                    \
                            const float* ip = in + (((size_t)n * H + iy) * W + ix) * Cin        \
                                              + (size_t)g * cig;                                \
                            const float* wp = w + (((size_t)co * Kh + kh) * Kw + kw) * cig;     \
                            for (int ci = 0; ci < cig; ++ci)                                    \
                                acc += (ACC)ip[ci] * (ACC)wp[ci];                               \
                        }                                                                       \
                    }                                                                           \
                    out[(((size_t)n * Ho + y) * Wo + x) * Cout + co] = (float)acc;              \
                }                                                                               \
}

ORC_DEFINE_CONV(orc_conv2d_f32, float)
ORC_DEFINE_CONV(orc_conv2d_f64, double)

#define ORC_DEFINE_FC(NAME, ACC)                                                                \
void NAME(const float* in, int N, int K, const float* w, const float* bias, int Cout,           \
          float* out)                                                                           \
{                                                                                               \
    _Pragma("omp parallel for collapse(2) schedule(static)")                                    \
    for (int n = 0; n < N; ++n)                                                                 \
        for (int co = 0; co < Cout; ++co) {                                                     \
            ACC acc = bias ? (ACC)bias[co] : (ACC)0;                                            \
            const float* ip = in + (size_t)n * K;                                               \
            const float* wp = w + (size_t)co * K;                                               \
            for (int k = 0; k < K; ++k) acc += (ACC)ip[k] * (ACC)wp[k];                         \
            out[(size_t)n * Cout + co] = (float)acc;                                            \
        }                                                                                       \
}

ORC_DEFINE_FC(orc_fc_f32, float)
ORC_DEFINE_FC(orc_fc_f64, double)

/* Max pooling, window Kh x Kw, padding value -infinity. */
void orc_maxpool(const float* in, int N, int H, int W, int C, int Kh, int Kw, int stride, int pad,
                 float* out)
{
    const int Ho = (H + 2 * pad - Kh) / stride + 1;
    const int Wo = (W + 2 * pad - Kw) / stride + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int y = 0; y < Ho; ++y)
            for (int x = 0; x < Wo; ++x)
                for (int c = 0; c < C; ++c) {
                    float m = -INFINITY;
                    for (int kh = 0; kh < Kh; ++kh) {
                        const int iy = y * stride - pad + kh;
                        if (iy < 0 || iy >= H) continue;
                        for (int kw = 0; kw < Kw; ++kw) {
                            const int ix = x * stride - pad + kw;
                            if (ix < 0 || ix >= W) continue;
                            const float v = in[(((size_t)n * H + iy) * W + ix) * C + c];
                            if (v > m) m = v;
                        }
                    }
                    out[(((size_t)n * Ho + y) * Wo + x) * C + c] = m;
                }
}

#define ORC_DEFINE_GAP(NAME, ACC)                                                               \
void NAME(const float* in, int N, int H, int W, int C, float* out)                              \
{                                                                                               \
    for (int n = 0; n < N; ++n)                                                                 \
        for (int c = 0; c < C; ++c) {                                                           \
            ACC acc = 0;                                                                        \
            for (int y = 0; y < H; ++y)                                                         \
                for (int x = 0; x < W; ++x)                                                     \
                    acc += (ACC)in[(((size_t)n * H + y) * W + x) * C + c];                      \
            out[(size_t)n * C + c] = (float)(acc / (ACC)(H * W));                               \
        }                                                                                       \
}

ORC_DEFINE_GAP(orc_global_avgpool_f32, float)
ORC_DEFINE_GAP(orc_global_avgpool_f64, double)

/* Residual add: out = a + b (element-wise, fp32). */
void orc_add(const float* a, const float* b, size_t n, float* out)
{
    for (size_t i = 0; i < n; ++i) out[i] = a[i] + b[i];
}

/* Activation in place: 0 = identity, 1 = ReLU max(x,0), 2 = ReLU6 min(max(x,0),6). */
void orc_act(float* x, size_t n, int act)
{
    if (act == 1) {
        for (size_t i = 0; i < n; ++i) x[i] = x[i] > 0.0f ? x[i] : 0.0f;
    } else if (act == 2) {
        for (size_t i = 0; i < n; ++i) {
            float v = x[i] > 0.0f ? x[i] : 0.0f;
            x[i] = v < 6.0f ? v : 6.0f;
        }
    }
}
