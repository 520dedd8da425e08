// alcs_depthwise_conv: the depthwise 3x3 layer (one filter per channel, zero padding 1,
// stride 1 or 2, bias, ReLU / ReLU6) that sits in front of every pointwise convolution of
// the MobileNet pruned in Section 4 of arXiv 2109.00170.  Stand-alone form: the unfused
// reference for alcs_dw_sparse_conv_fused and its fallback for layouts the fused kernels do
// not cover.  The layer moves each element once (one read, one write) and does 9 multiply-adds
// per output: a streaming kernel; a wavefront takes 64 consecutive pixels of a few planes and
// neighbouring lanes share taps (alcs_dw_taps.h).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "alcs_internal.h"
#include "alcs_dw_taps.h"

namespace alcs {

struct DwArgs {
    const float *D;     // [C, 3, 3]
    const float *X;     // [N, C, H, W]
    const float *bias;  // [C] or null
    float *Z;           // [N, C, Ho, Wo]
    long long planes;   // N * C
    int nchunks;        // 64-pixel chunks per plane
    unsigned wg_per_xcd, total_wgs, xcds;
    int C, H, W, Ho, Wo, P, Pin, stride, act;
};

constexpr int kPlanesPerWave = 8;

// A wavefront owns 64 consecutive output pixels of kPlanesPerWave (n, c) planes: the pixel
// geometry (row / column, border flags, tap offsets) is worked out once and reused for every
// plane, the filter and the bias are wave-uniform.  All lanes stay in the loop (neighbours take
// taps from them); lanes beyond the plane's last pixel re-read its first element and store nothing.
template <int MODE>
__global__ void __launch_bounds__(256) k_depthwise(const DwArgs a) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Workgroups are dealt round-robin to the XCDs, each with its own L2.  Renumber them so that
    // neighbouring 64-pixel chunks of the same planes - which share two of their three input rows -
    // run on one XCD and find those rows in its L2 (without this every row came from HBM about
    // three times: 42 us instead of 25 us for 32 channels at 112x112, batch 32).
    const unsigned logical = (blockIdx.x % a.xcds) * a.wg_per_xcd + blockIdx.x / a.xcds;
    if (logical >= a.total_wgs) return;
    const unsigned chunk = logical % (unsigned)a.nchunks;
    const long long pg = (long long)(logical / (unsigned)a.nchunks) * 4 + wave;  // plane group
    const int po = (int)chunk * 64 + lane;
    const bool valid = po < a.P;
    const int ho = valid ? po / a.Wo : 0, wo = valid ? po - ho * a.Wo : 0;
    DwTaps<MODE, 64> taps;
    taps.init(valid, 0, ho, wo, a.H, a.W, a.stride, lane);
    const long long p0 = pg * kPlanesPerWave;
    if (p0 >= a.planes) return;  // the whole wavefront
    const auto wts = reinterpret_cast<const float __attribute__((address_space(4))) *>((uintptr_t)a.D);
    const auto bs = reinterpret_cast<const float __attribute__((address_space(4))) *>((uintptr_t)a.bias);
    int c0 = __builtin_amdgcn_readfirstlane((int)(p0 % a.C));  // channel of plane p0; the next planes count up
    auto finish = [&](long long plane, int c, const typename DwTaps<MODE, 64>::Raw &x) {
        float acc = taps.apply(x, wts + c * 9, a.bias ? bs[c] : 0.f);   // wave-uniform: scalar loads
        if (a.act >= 1) acc = fmaxf(acc, 0.f);
        if (a.act == 2) acc = fminf(acc, 6.f);
        if (valid) __builtin_nontemporal_store(acc, a.Z + (size_t)plane * a.P + po);
    };
    // Software pipeline over pairs of planes: the loads of the next pair are issued before the
    // current pair is finished, so up to four planes' taps are in flight per wavefront (the
    // kernel is bound by the latency of these round trips, not by bytes or arithmetic).
    typedef typename DwTaps<MODE, 64>::Raw Raw;
    const float *xb = a.X + (size_t)p0 * a.Pin;
    const long long left = a.planes - p0;            // planes this wavefront owns (>= 1)
    const int np = left < kPlanesPerWave ? (int)left : kPlanesPerWave;
    auto chan = [&](int i) { return __builtin_amdgcn_readfirstlane((c0 + i) % a.C); };  // wave-uniform
    Raw x0 = {}, x1 = {}, y0 = {}, y1 = {};
    taps.load(xb, x0);
    if (np > 1) taps.load(xb + (size_t)a.Pin, x1);
#pragma unroll
    for (int i = 0; i < kPlanesPerWave; i += 2) {
        if (i >= np) break;  // wave-uniform
        if (i + 2 < np) taps.load(xb + (size_t)(i + 2) * a.Pin, y0);
        if (i + 3 < np) taps.load(xb + (size_t)(i + 3) * a.Pin, y1);
        finish(p0 + i, chan(i), x0);
        if (i + 1 < np) finish(p0 + i + 1, chan(i + 1), x1);
        x0 = y0;
        x1 = y1;
    }
}

// Stride 1 and a width that is a multiple of 4: a lane owns four consecutive pixels of a row, so
// every tap row is one aligned 16-byte load plus its left and right neighbour, and the outputs
// leave as one 16-byte store - a quarter of the memory instructions of the kernel above.  The
// neighbours beyond the image are read from the row's own end (in bounds) and zeroed.
typedef float dw_f4 __attribute__((ext_vector_type(4)));

constexpr int kPlanesPerWaveQuad = 2;  // few planes per wavefront: four pixels per lane leave few wavefronts

__global__ void __launch_bounds__(256) k_depthwise_quad(const DwArgs a) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned logical = (blockIdx.x % a.xcds) * a.wg_per_xcd + blockIdx.x / a.xcds;
    if (logical >= a.total_wgs) return;
    const unsigned chunk = logical % (unsigned)a.nchunks;
    const long long pg = (long long)(logical / (unsigned)a.nchunks) * 4 + wave;
    const long long p0 = pg * kPlanesPerWaveQuad;
    if (p0 >= a.planes) return;  // the whole wavefront
    const int po = ((int)chunk * 64 + lane) * 4;
    const bool valid = po < a.P;
    const int ho = valid ? po / a.W : 0, wo = valid ? po - ho * a.W : 0;   // stride 1: Wo == W
    bool rok[3];
    uint32_t roff[3], loff[3], qoff[3];
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int hi = ho - 1 + r;
        rok[r] = valid && hi >= 0 && hi < a.H;
        const uint32_t at = (uint32_t)(min(max(hi, 0), a.H - 1) * a.W + wo);
        roff[r] = at * 4u;
        loff[r] = (wo > 0 ? at - 1u : at) * 4u;
        qoff[r] = (wo + 4 < a.W ? at + 4u : at + 3u) * 4u;
    }
    const bool hasl = wo > 0, hasr = wo + 4 < a.W;
    const auto wts = reinterpret_cast<const float __attribute__((address_space(4))) *>((uintptr_t)a.D);
    const auto bs = reinterpret_cast<const float __attribute__((address_space(4))) *>((uintptr_t)a.bias);
    const int c0 = __builtin_amdgcn_readfirstlane((int)(p0 % a.C));
    const long long left = a.planes - p0;
    const int np = left < kPlanesPerWaveQuad ? (int)left : kPlanesPerWaveQuad;
#pragma unroll
    for (int i = 0; i < kPlanesPerWaveQuad; ++i) {
        if (i >= np) break;  // wave-uniform
        const int c = __builtin_amdgcn_readfirstlane((c0 + i) % a.C);
        const char *b = reinterpret_cast<const char *>(a.X + (size_t)(p0 + i) * a.Pin);
        float x[3][6];
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const dw_f4 m = *reinterpret_cast<const dw_f4 *>(b + roff[r]);
            const float l = *reinterpret_cast<const float *>(b + loff[r]);
            const float q = *reinterpret_cast<const float *>(b + qoff[r]);
            x[r][0] = (rok[r] && hasl) ? l : 0.f;
            x[r][1] = rok[r] ? m[0] : 0.f;
            x[r][2] = rok[r] ? m[1] : 0.f;
            x[r][3] = rok[r] ? m[2] : 0.f;
            x[r][4] = rok[r] ? m[3] : 0.f;
            x[r][5] = (rok[r] && hasr) ? q : 0.f;
        }
        const float bias = a.bias ? bs[c] : 0.f;
        dw_f4 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float acc = bias;   // taps in the order (r, t) ascending, as in the other forms
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int t = 0; t < 3; ++t) acc = fmaf(wts[c * 9 + r * 3 + t], x[r][j + t], acc);
            if (a.act >= 1) acc = fmaxf(acc, 0.f);
            if (a.act == 2) acc = fminf(acc, 6.f);
            o[j] = acc;
        }
        if (valid) __builtin_nontemporal_store(o, reinterpret_cast<dw_f4 *>(a.Z + (size_t)(p0 + i) * a.P + po));
    }
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
    if (P > INT32_MAX || Pin >= (1LL << 30)) return ALCS_E_UNSUPPORTED;  // 32-bit byte offsets inside a plane
    if ((long double)N * C * Pin >= 9e18L) return ALCS_E_UNSUPPORTED;
    DwArgs a{};
    a.D = dw_weights_dev; a.X = X_dev; a.bias = bias_dev; a.Z = Y_dev;
    a.planes = (long long)N * C;
    const bool quad = stride == 1 && (W % 4) == 0 && ((((uintptr_t)X_dev) | ((uintptr_t)Y_dev)) & 15) == 0;
    a.nchunks = (int)((P + (quad ? 255 : 63)) / (quad ? 256 : 64));
    a.C = C; a.H = H; a.W = W; a.Ho = Ho; a.Wo = Wo; a.P = (int)P; a.Pin = (int)Pin;
    a.stride = stride; a.act = activation;
    const int ppw = quad ? kPlanesPerWaveQuad : kPlanesPerWave;
    const long long groups = (a.planes + 4 * ppw - 1) / (4 * ppw);
    const long long blocks = groups * a.nchunks;
    if (blocks > INT32_MAX - 256) return ALCS_E_UNSUPPORTED;
    int cus = 0, xcds = 0;
    if (current_device_shape(&cus, &xcds) != ALCS_OK) return ALCS_E_HIP;
    a.total_wgs = (unsigned)blocks;
    a.xcds = (unsigned)xcds;
    a.wg_per_xcd = (unsigned)((blocks + xcds - 1) / xcds);
    const int mode = dw_mode_for(stride, W, X_dev);
    void (*kern)(const DwArgs) = quad ? k_depthwise_quad : mode == kDwPair ? k_depthwise<kDwPair> : k_depthwise<kDwNine>;
    hipLaunchKernelGGL(kern, dim3(a.wg_per_xcd * a.xcds), dim3(256), 0, (hipStream_t)stream, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error((int)e); return ALCS_E_HIP; }
    return ALCS_OK;
}
