/*
 * CPU oracle for a quantised (int8) convolution layer.  TEST INFRASTRUCTURE ONLY: called by the
 * tests, the smoke check and the benchmark's CPU-baseline leg, never by the GPU library, and it
 * shares no code with it.
 *
 * The paper's chip lists an INT8 mode beside FP16 (table of the MLU100's specification) but the
 * paper fixes no quantisation scheme; the reading taken here is the common integer-arithmetic
 * one, stated so that every step has exactly one result:
 *
 *   acc[n,y,x,co] = sum_{kh,kw,ci} in[n, y*s-p+kh, x*s-p+kw, ci] * w[co,kh,kw,ci]
 *       over int8 operands, exact in integers (terms outside the image contribute nothing;
 *       Hout = floor((H + 2p - Kh)/s) + 1 as in Eq. 1); the sum must fit 32 bits;
 *   t   = fma((float)acc, scale[co], bias[co])     one fp32 fused multiply-add, (float) rounds
 *                                                  to nearest even when |acc| > 2^24;
 *   r   = t rounded to the nearest integer, ties to even;
 *   out = min(max(r, lo), 127) as int8, lo = 0 with ReLU, else -128.
 *
 * Returns 0, or 1 if some accumulator left the 32-bit range (outputs are then meaningless).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

int orc_conv2d_i8(const int8_t* in, int N, int H, int W, int Cin, const int8_t* w,
                  const float* scale, const float* bias, int Cout, int Kh, int Kw, int stride,
                  int pad, int relu, int8_t* out, int32_t* acc_out)
{
    const int Ho = (H + 2 * pad - Kh) / stride + 1;
    const int Wo = (W + 2 * pad - Kw) / stride + 1;
    int overflow = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : overflow)
    for (int n = 0; n < N; ++n)
        for (int y = 0; y < Ho; ++y)
            for (int x = 0; x < Wo; ++x)
                for (int co = 0; co < Cout; ++co) {
                    int64_t acc = 0;
                    for (int kh = 0; kh < Kh; ++kh) {
                        const int iy = y * stride - pad + kh;
                        if (iy < 0 || iy >= H) continue;
                        for (int kw = 0; kw < Kw; ++kw) {
                            const int ix = x * stride - pad + kw;
                            if (ix < 0 || ix >= W) continue;
                            const int8_t* ip = in + (((size_t)n * H + iy) * W + ix) * Cin;
                            const int8_t* wp = w + (((size_t)co * Kh + kh) * Kw + kw) * Cin;
                            for (int ci = 0; ci < Cin; ++ci) acc += (int64_t)ip[ci] * (int64_t)wp[ci];
                        }
                    }
                    if (acc > INT32_MAX || acc < INT32_MIN) overflow |= 1;
                    const size_t o = (((size_t)n * Ho + y) * Wo + x) * Cout + co;
                    if (acc_out) acc_out[o] = (int32_t)acc;
                    const float t = fmaf((float)(int32_t)acc, scale[co], bias[co]);
                    float r = rintf(t);   /* default rounding mode: to nearest, ties to even */
                    const float lo = relu ? 0.0f : -128.0f;
                    r = r < lo ? lo : r;
                    r = r > 127.0f ? 127.0f : r;
                    out[o] = (int8_t)r;
                }
    return overflow;
}
