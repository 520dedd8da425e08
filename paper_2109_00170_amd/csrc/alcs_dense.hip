// alcs_dense_conv: the sparsity-0 reference on the same GPU (the role dense models
// play in the timing protocol of Section 4.1 of arXiv 2109.00170), written as an
// implicit GEMM  Y[o, q] = sum_k W[o, k] * I*[k, q]  on fp32 matrix cores
// (v_mfma_f32_32x32x2_f32), with I* the virtual patch matrix of Section 3.2.2
// ("Overview"): row k = (c*kernel + r)*kernel + s, column q = flattened (n, ho, wo).
//
// A workgroup of four wavefronts (2 x 2) owns a BM x 128 tile of Y and walks K in
// steps of 16: the weight tile is transposed into LDS as As[k][m], the patch tile is
// gathered as Bs[k][q]; each wavefront owns (BM/64) x 2 MFMA tiles of 32 x 32.  The
// global loads of step k+1 are issued before the multiplies of step k and written to the
// other half of a two-deep LDS buffer afterwards, so a step costs one barrier and the
// load latency is covered by the matrix instructions.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "alcs_internal.h"

namespace alcs {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));

struct DenseArgs {
    const float *Wt;
    const float *X;
    const float *bias;
    float *Y;
    long long NP;
    int N, Cin, Cout, H, W, Ho, Wo, stride, k;
    int P, Pin, K;
    int mt, nt;  // tiles along Cout and along pixels
    int wg_per_xcd, total_wgs, xcds;
};

constexpr int BK = 16;
constexpr int BN = 128;

template <int BM, bool PW_VEC>
__global__ void __launch_bounds__(256) k_dense(const DenseArgs a) {
    constexpr int LDA = BM + 4;
    constexpr int TM = BM / 64;  // 32x32 tiles per wavefront along M
    constexpr int A_ROWS_PER_PASS = 128;  // 256 threads / 2
    constexpr int NA = (BM + A_ROWS_PER_PASS - 1) / A_ROWS_PER_PASS;  // weight-tile passes per thread
    __shared__ float As[2][BK * LDA];
    __shared__ float Bs[2][BK * BN];
    const int id = blockIdx.x;
    const int logical = (id % a.xcds) * a.wg_per_xcd + id / a.xcds;
    if (logical >= a.total_wgs) return;
    // consecutive logical ids share the pixel tile (the large operand) and differ in the channel tile
    const int ntile = logical / a.mt, mtile = logical - ntile * a.mt;
    const int m0 = mtile * BM;
    const long long q0 = (long long)ntile * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    f16v acc[TM][2];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // weight tile: thread -> (row of W, half of the 16 k's)
    const int a_row = tid >> 1, a_k = (tid & 1) * 8;
    // patch tile, vector form (1x1, stride 1, P % 4 == 0): thread -> (k row, pixel quad)
    const int bq = tid & 31, bk0 = tid >> 5;  // 32 quads x 8 rows per pass
    long long vq = q0 + bq * 4;
    const bool vvalid = vq < a.NP;
    const int vn = vvalid ? (int)(vq / a.P) : 0;
    const int vp = vvalid ? (int)(vq - (long long)vn * a.P) : 0;
    // patch tile, gather form: thread -> (pixel column, k rows tid/128 + 2*i)
    const int gcol = tid & 127, gk0 = tid >> 7;
    const long long gq = q0 + gcol;
    const bool gvalid = gq < a.NP;
    const int gn = gvalid ? (int)(gq / a.P) : 0;
    const int gpo = gvalid ? (int)(gq - (long long)gn * a.P) : 0;
    const int gho = gpo / a.Wo, gwo = gpo - gho * a.Wo;
    const int pad = (a.k - 1) / 2;
    const int giy = gho * a.stride - pad, gix = gwo * a.stride - pad;
    const int kk = a.k * a.k;
    const float *gx = a.X + (size_t)gn * a.Cin * a.Pin;
    // channel and tap of the thread's first gather row; advanced by 2 per row and kept
    // across steps (8 rows * 2 = one step of 16), so no division in the loop
    int gc = gk0 / kk, gtap = gk0 - gc * kk;

    float ra[NA][8];   // the step's weights: 8 consecutive k of one row of W per pass
    f4 rbv[2];         // vector form: two rows of the patch tile
    float rbg[8];      // gather form: 8 rows of one pixel column

    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int pass = 0; pass < NA; ++pass) {
            const int row = pass * A_ROWS_PER_PASS + a_row;
            const int o = m0 + row;
            const bool full = o < a.Cout && k0 + a_k + 8 <= a.K && (a.K % 4 == 0);
            if (full) {
                const f4 *src = reinterpret_cast<const f4 *>(a.Wt + (size_t)o * a.K + k0 + a_k);
                const f4 t0 = src[0], t1 = src[1];
                ra[pass][0] = t0[0]; ra[pass][1] = t0[1]; ra[pass][2] = t0[2]; ra[pass][3] = t0[3];
                ra[pass][4] = t1[0]; ra[pass][5] = t1[1]; ra[pass][6] = t1[2]; ra[pass][7] = t1[3];
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int kx = k0 + a_k + i;
                    ra[pass][i] = (o < a.Cout && kx < a.K) ? a.Wt[(size_t)o * a.K + kx] : 0.f;
                }
            }
        }
        if constexpr (PW_VEC) {
#pragma unroll
            for (int pass = 0; pass < 2; ++pass) {
                const int c = k0 + bk0 + pass * 8;
                rbv[pass] = f4{0, 0, 0, 0};
                if (vvalid && c < a.K)
                    rbv[pass] = *reinterpret_cast<const f4 *>(a.X + ((size_t)vn * a.Cin + c) * a.P + vp);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float v = 0.f;
                if (gvalid && gc < a.Cin) {
                    const int r = a.k == 1 ? 0 : gtap / 3, s = a.k == 1 ? 0 : gtap - r * 3;
                    const int iy = giy + r, ix = gix + s;
                    if (iy >= 0 && iy < a.H && ix >= 0 && ix < a.W)
                        v = gx[(size_t)gc * a.Pin + (size_t)iy * a.W + ix];
                }
                rbg[i] = v;
                gtap += 2;   // next row of this thread: k + 2
                if (gtap >= kk) { gtap -= kk; ++gc; }
                if (gtap >= kk) { gtap -= kk; ++gc; }   // kk = 1: two channels per row step
            }
        }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int pass = 0; pass < NA; ++pass) {
            const int row = pass * A_ROWS_PER_PASS + a_row;
            if (BM >= A_ROWS_PER_PASS || row < BM) {
#pragma unroll
                for (int i = 0; i < 8; ++i) As[buf][(a_k + i) * LDA + row] = ra[pass][i];
            }
        }
        if constexpr (PW_VEC) {
#pragma unroll
            for (int pass = 0; pass < 2; ++pass)
                *reinterpret_cast<f4 *>(&Bs[buf][(bk0 + pass * 8) * BN + bq * 4]) = rbv[pass];
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) Bs[buf][(gk0 + 2 * i) * BN + gcol] = rbg[i];
        }
    };

    load_tiles(0);
    store_tiles(0);
    __syncthreads();
    int buf = 0;
    for (int k0 = 0; k0 < a.K; k0 += BK) {
        const bool more = k0 + BK < a.K;
        if (more) load_tiles(k0 + BK);   // in flight during the multiplies below
        // ---- multiply ----
#pragma unroll
        for (int ks = 0; ks < BK; ks += 2) {
            const int kl = ks + (lane >> 5);
            float av[TM], bv[2];
#pragma unroll
            for (int i = 0; i < TM; ++i) av[i] = As[buf][kl * LDA + (wm * TM + i) * 32 + (lane & 31)];
#pragma unroll
            for (int j = 0; j < 2; ++j) bv[j] = Bs[buf][kl * BN + (wn * 2 + j) * 32 + (lane & 31)];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
        // the other buffer was last read in the previous step, before that step's barrier
        if (more) store_tiles(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
    // ---- epilogue: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32 ----
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const long long q = q0 + (wn * 2 + j) * 32 + (lane & 31);
        if (q >= a.NP) continue;
        const int n = (int)(q / a.P);
        const int p = (int)(q - (long long)n * a.P);
        float *ybase = a.Y + (size_t)n * a.Cout * a.P + p;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int o = m0 + (wm * TM + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (o < a.Cout) ybase[(size_t)o * a.P] = acc[i][j][r] + (a.bias ? a.bias[o] : 0.f);
            }
    }
}

}  // namespace alcs

using namespace alcs;

extern "C" int alcs_dense_conv(const float *W_dev, const float *X_dev, const float *bias_dev,
                               float *Y_dev, int N, int Cin, int Cout, int H, int W, int kernel,
                               int stride, void *stream) {
    if (N < 0 || Cin <= 0 || Cout <= 0 || H <= 0 || W <= 0) return ALCS_E_INVALID_ARG;
    if (kernel != 1 && kernel != 3) return ALCS_E_UNSUPPORTED;
    if (stride != 1 && stride != 2) return ALCS_E_UNSUPPORTED;
    if (N == 0) return ALCS_OK;
    if (!W_dev || !X_dev || !Y_dev) return ALCS_E_INVALID_ARG;
    if (((uintptr_t)W_dev | (uintptr_t)X_dev | (uintptr_t)Y_dev) & 15) return ALCS_E_INVALID_ARG;
    const int pad = (kernel - 1) / 2;
    const int Ho = (H + 2 * pad - kernel) / stride + 1, Wo = (W + 2 * pad - kernel) / stride + 1;
    if (Ho <= 0 || Wo <= 0) return ALCS_E_INVALID_ARG;
    const long long P = (long long)Ho * Wo, Pin = (long long)H * W, K = (long long)Cin * kernel * kernel;
    if (P > INT32_MAX || Pin > INT32_MAX || K > (1 << 24)) return ALCS_E_UNSUPPORTED;
    if ((long double)N * Cin * Pin >= 9e18L || (long double)N * Cout * P >= 9e18L) return ALCS_E_UNSUPPORTED;
    DenseArgs a{};
    a.Wt = W_dev; a.X = X_dev; a.bias = bias_dev; a.Y = Y_dev;
    a.N = N; a.Cin = Cin; a.Cout = Cout; a.H = H; a.W = W; a.Ho = Ho; a.Wo = Wo;
    a.stride = stride; a.k = kernel; a.P = (int)P; a.Pin = (int)Pin; a.K = (int)K;
    a.NP = (long long)N * P;
    const bool vec = kernel == 1 && stride == 1 && (P % 4 == 0);
    const long long ntile = (a.NP + BN - 1) / BN;
    // 128 output channels per workgroup, or 64 when that leaves fewer workgroups than compute units
    int cus = 0, xcds = 0;
    if (current_device_shape(&cus, &xcds) != ALCS_OK) return ALCS_E_HIP;
    const int BM = (Cout > 64 && ntile * ((Cout + 127) / 128) >= cus) ? 128 : 64;
    a.mt = (Cout + BM - 1) / BM;
    const long long total = ntile * a.mt;
    if (total > (1LL << 30)) return ALCS_E_UNSUPPORTED;
    a.nt = (int)ntile;
    a.total_wgs = (int)total;
    a.xcds = xcds;
    a.wg_per_xcd = (int)((total + xcds - 1) / xcds);
    void (*kern)(const DenseArgs) = nullptr;
    if (BM == 128) kern = vec ? k_dense<128, true> : k_dense<128, false>;
    else kern = vec ? k_dense<64, true> : k_dense<64, false>;
    hipLaunchKernelGGL(kern, dim3(a.wg_per_xcd * xcds), dim3(256), 0, (hipStream_t)stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error((int)e); return ALCS_E_HIP; }
    return ALCS_OK;
}
