// The storage format of Section 3.2.2 of arXiv 2109.00170 ("Storage format": per filter group
// the number of kept columns, their ascending column offsets and one V-vector of values per
// kept column) built on the GPU from device-resident weights and keep / drop flags - e.g. the
// flags that alcs_project_latency leaves on the device - so that a re-pruning loop neither
// downloads the dense weights nor scans them on the host.  Three small kernels: kept columns
// per group, an exclusive scan over the groups (row_ptr), and an order-preserving compaction
// of every group (ballot + population count per wavefront).  Values are moved, never
// computed: the result is the canonical form bit for bit.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "alcs_internal.h"

namespace alcs {

// counts[g + 1] = kept columns of group g (counts[0] = 0); mask == null keeps everything
__global__ void __launch_bounds__(256) k_pack_count(const uint8_t *mask, int K, int32_t *counts) {
    __shared__ int total;
    if (threadIdx.x == 0) total = 0;
    __syncthreads();
    const int g = blockIdx.x;
    int mine = 0;
    if (mask) {
        const uint8_t *m = mask + (size_t)g * K;
        for (int col = threadIdx.x; col < K; col += 256) mine += m[col] != 0;
    } else {
        for (int col = threadIdx.x; col < K; col += 256) mine += 1;
    }
    if (mine) atomicAdd(&total, mine);
    __syncthreads();
    if (threadIdx.x == 0) {
        counts[g + 1] = total;
        if (g == 0) counts[0] = 0;
    }
}

// In-place inclusive scan of counts[1 .. G] by one workgroup, 1024 entries per round.
__global__ void __launch_bounds__(1024) k_pack_scan(int32_t *row_ptr, int G) {
    __shared__ int buf[1024];
    __shared__ int carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < G; base += 1024) {
        const int i = base + threadIdx.x;
        int v = i < G ? row_ptr[i + 1] : 0;
        buf[threadIdx.x] = v;
        __syncthreads();
        for (int d = 1; d < 1024; d <<= 1) {
            const int add = threadIdx.x >= d ? buf[threadIdx.x - d] : 0;
            __syncthreads();
            buf[threadIdx.x] += add;
            __syncthreads();
        }
        if (i < G) row_ptr[i + 1] = buf[threadIdx.x] + carry;
        __syncthreads();
        if (threadIdx.x == 0) carry += buf[1023];
        __syncthreads();
    }
}

// One workgroup per group: its kept columns in ascending order, V values per column.
template <int V>
__global__ void __launch_bounds__(256) k_pack_fill(const float *W, const uint8_t *mask, int Cout, int K,
                                                   const int32_t *row_ptr, int32_t *col_idx, float *vals) {
    __shared__ int wave_cnt[4];
    __shared__ int base;
    const int g = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) base = row_ptr[g];
    __syncthreads();
    for (int c0 = 0; c0 < K; c0 += 256) {
        const int col = c0 + threadIdx.x;
        const bool keep = col < K && (!mask || mask[(size_t)g * K + col] != 0);
        const unsigned long long ballot = __ballot(keep);
        if (lane == 0) wave_cnt[wave] = __popcll(ballot);
        __syncthreads();
        int off = base + __popcll(ballot & ((1ull << lane) - 1ull));
        for (int w = 0; w < wave; ++w) off += wave_cnt[w];
        if (keep) {
            col_idx[off] = col;
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const int o = g * V + v;
                vals[(size_t)off * V + v] = o < Cout ? W[(size_t)o * K + col] : 0.0f;
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) base += wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
        __syncthreads();
    }
}

static int check(hipError_t e) {
    if (e == hipSuccess) return ALCS_OK;
    set_hip_error((int)e);
    return ALCS_E_HIP;
}

int enqueue_csr_count(const uint8_t *mask_dev, int G, int K, int32_t *row_ptr_dev, hipStream_t st) {
    hipLaunchKernelGGL(k_pack_count, dim3(G), dim3(256), 0, st, mask_dev, K, row_ptr_dev);
    hipLaunchKernelGGL(k_pack_scan, dim3(1), dim3(1024), 0, st, row_ptr_dev, G);
    return check(hipGetLastError());
}

int enqueue_csr_fill(const float *W_dev, const uint8_t *mask_dev, int Cout, int K, int V, int G,
                     const int32_t *row_ptr_dev, int32_t *col_idx_dev, float *vals_dev, hipStream_t st) {
    void (*kern)(const float *, const uint8_t *, int, int, const int32_t *, int32_t *, float *) = nullptr;
    switch (V) {
        case 1: kern = k_pack_fill<1>; break;
        case 2: kern = k_pack_fill<2>; break;
        case 4: kern = k_pack_fill<4>; break;
        case 8: kern = k_pack_fill<8>; break;
        default: kern = k_pack_fill<16>; break;
    }
    hipLaunchKernelGGL(kern, dim3(G), dim3(256), 0, st, W_dev, mask_dev, Cout, K, row_ptr_dev, col_idx_dev, vals_dev);
    return check(hipGetLastError());
}

}  // namespace alcs

using namespace alcs;

extern "C" int alcs_pack_csr_device(const float *W_dev, const uint8_t *mask_dev, int Cout, int Cin, int kernel,
                                    int V, int32_t *row_ptr_dev, int32_t *col_idx_dev, float *vals_dev,
                                    long long capacity_blocks, long long *nnzb_out, void *stream) {
    if (!W_dev || !row_ptr_dev || Cout <= 0 || Cin <= 0 || capacity_blocks < 0) return ALCS_E_INVALID_ARG;
    if (kernel != 1 && kernel != 3) return ALCS_E_UNSUPPORTED;
    if (V != 1 && V != 2 && V != 4 && V != 8 && V != 16) return ALCS_E_UNSUPPORTED;
    const long long K64 = (long long)Cin * kernel * kernel;
    if (K64 > (1 << 24) || Cout > (1 << 24)) return ALCS_E_UNSUPPORTED;
    const int K = (int)K64, G = (Cout + V - 1) / V;
    if ((long long)G * K > (long long)INT32_MAX - 1024) return ALCS_E_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    int rc = enqueue_csr_count(mask_dev, G, K, row_ptr_dev, st);
    if (rc != ALCS_OK) return rc;
    int32_t nnzb = 0;
    rc = check(hipMemcpyAsync(&nnzb, row_ptr_dev + G, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    if (rc != ALCS_OK) return rc;
    rc = check(hipStreamSynchronize(st));
    if (rc != ALCS_OK) return rc;
    if (nnzb_out) *nnzb_out = nnzb;
    if (!col_idx_dev && !vals_dev) return ALCS_OK;  // counting pass only
    if (!col_idx_dev || !vals_dev || nnzb > capacity_blocks) return ALCS_E_INVALID_ARG;
    if (nnzb == 0) return ALCS_OK;
    return enqueue_csr_fill(W_dev, mask_dev, Cout, K, V, G, row_ptr_dev, col_idx_dev, vals_dev, st);
}
