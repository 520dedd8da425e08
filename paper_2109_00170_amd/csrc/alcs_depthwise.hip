// alcs_depthwise_conv: the depthwise 3x3 layer (one filter per channel, zero padding 1,
// stride 1 or 2, bias, ReLU / ReLU6) that sits in front of every pointwise convolution of
// the MobileNet pruned in Section 4 of arXiv 2109.00170.  Stand-alone form: the unfused
// reference for alcs_dw_sparse_conv_fused and its fallback for layouts the fused kernels do
// not cover.  The layer moves each element once (one read, one write) and does 9 multiply-adds
// per output: a streaming kernel, one thread per output element of the flattened
// [N*C, Ho*Wo] tensor, the nine taps served by the vector cache.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "alcs_internal.h"

namespace alcs {

struct DwArgs {
    const float *D;     // [C, 3, 3]
    const float *X;     // [N, C, H, W]
    const float *bias;  // [C] or null
    float *Z;           // [N, C, Ho, Wo]
    long long total;    // N * C * Ho * Wo
    int C, H, W, Ho, Wo, P, Pin, stride, act;
};

__global__ void __launch_bounds__(256) k_depthwise(const DwArgs a) {
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= a.total) return;
    const long long plane = idx / a.P;           // n * C + c
    const int po = (int)(idx - plane * a.P);
    const int c = (int)(plane % a.C);
    const int ho = po / a.Wo, wo = po - ho * a.Wo;
    const int hi0 = ho * a.stride - 1, wi0 = wo * a.stride - 1;
    const float *xc = a.X + (size_t)plane * a.Pin;
    const float *d = a.D + (size_t)c * 9;
    float x[9];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int t = 0; t < 3; ++t) {
            const int hi = hi0 + r, wi = wi0 + t;
            const bool ok = hi >= 0 && hi < a.H && wi >= 0 && wi < a.W;
            x[r * 3 + t] = ok ? xc[hi * a.W + wi] : 0.f;
        }
    float acc = a.bias ? a.bias[c] : 0.f;
#pragma unroll
    for (int t = 0; t < 9; ++t) acc = fmaf(d[t], x[t], acc);
    if (a.act >= 1) acc = fmaxf(acc, 0.f);
    if (a.act == 2) acc = fminf(acc, 6.f);
    __builtin_nontemporal_store(acc, a.Z + idx);
}

}  // namespace alcs

using namespace alcs;

extern "C" int alcs_depthwise_conv(const float *dw_weights_dev, const float *X_dev, const float *bias_dev,
                                   float *Y_dev, int N, int C, int H, int W, int stride, int activation,
                                   void *stream) {
    if (N < 0 || C <= 0 || H <= 0 || W <= 0) return ALCS_E_INVALID_ARG;
    if (stride != 1 && stride != 2) return ALCS_E_UNSUPPORTED;
    if (activation < 0 || activation > 2) return ALCS_E_INVALID_ARG;
    if (N == 0) return ALCS_OK;
    if (!dw_weights_dev || !X_dev || !Y_dev) return ALCS_E_INVALID_ARG;
    const int Ho = (H - 1) / stride + 1, Wo = (W - 1) / stride + 1;  // (H + 2 - 3) / stride + 1
    const long long P = (long long)Ho * Wo, Pin = (long long)H * W;
    if (P > INT32_MAX || Pin > INT32_MAX) return ALCS_E_UNSUPPORTED;
    if ((long double)N * C * Pin >= 9e18L) return ALCS_E_UNSUPPORTED;
    DwArgs a{};
    a.D = dw_weights_dev; a.X = X_dev; a.bias = bias_dev; a.Z = Y_dev;
    a.total = (long long)N * C * P;
    a.C = C; a.H = H; a.W = W; a.Ho = Ho; a.Wo = Wo; a.P = (int)P; a.Pin = (int)Pin;
    a.stride = stride; a.act = activation;
    const long long blocks = (a.total + 255) / 256;
    if (blocks > INT32_MAX) return ALCS_E_UNSUPPORTED;
    hipLaunchKernelGGL(k_depthwise, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error((int)e); return ALCS_E_HIP; }
    return ALCS_OK;
}
