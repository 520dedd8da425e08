// Projection onto the latency constraint, Section 3.4, Algorithm 1 of arXiv 2109.00170, on the
// GPU: the squared L2 norm of every block of V weights (steps 1-2), the selection of the N
// blocks with the largest norm over all layers (step 7) and the bisection on N against the
// latency model of Section 3.3 (steps 3-15).
//
// Nothing is sorted.  A block's key is 64 bits wide - the score's bit pattern above the
// complement of the block's index - so that keys are distinct and "larger score first, lower
// index first among equal scores" is plain integer order.  The N-th largest key is found by a
// radix select: eight passes, most significant byte first, each a histogram of the byte over
// the keys that match the bytes chosen so far (per-workgroup histograms in LDS, merged with
// atomics); the next launch starts by walking the 256 bins from the top and fixing that byte
// (every workgroup for itself: a kernel boundary is the only synchronisation).  A last pass
// writes the keep / drop flags and counts the kept blocks per layer; the host loop of the
// bisection reads only those counts.  All state lives in a caller-provided workspace; a
// selection is ten launches (one to set up, eight passes, one to emit) that stream the 4-byte
// scores nine times.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <mutex>
#include <vector>

#include "alcs_internal.h"

namespace alcs {

constexpr int kPasses = 8;  // bytes of a key

// hist[p] = histogram of pass p; prefix[p], remaining[p] = the bytes of the N-th largest key fixed
// before pass p and its rank (1 = largest) among the keys that share them.
struct SelectState {
    unsigned long long hist[kPasses][256];
    unsigned long long prefix[kPasses + 1];
    unsigned long long remaining[kPasses + 1];
};

__device__ __forceinline__ unsigned long long key_of(const float *scores, unsigned long long i) {
    const unsigned int bits = __float_as_uint(scores[i]);
    return ((unsigned long long)bits << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned int)i);
}

// Steps 1-2: one thread per block (group g, column col of the stretched filter); the V rows of
// the group are K floats apart, so a wavefront reads V contiguous runs.  The sum is the one the
// definition fixes: float32, rows in ascending order, product and sum rounded separately.
template <int V>
__global__ void __launch_bounds__(256) k_block_scores(const float *W, float *scores, int Cout, long long K,
                                                      long long total) {
#pragma clang fp contract(off)  // no fused multiply-add: product and sum round separately
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const long long g = idx / K, col = idx - g * K;
    float s = 0.f;
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const long long row = g * V + v;
        const float w = row < Cout ? W[row * K + col] : 0.f;
        const float p = w * w;
        s = s + p;
    }
    scores[idx] = s;
}

__global__ void k_select_init(SelectState *st, unsigned long long N, unsigned long long *counts, int n_seg) {
    const int t = threadIdx.x;
    for (int p = 0; p < kPasses; ++p)
        if (t < 256) st->hist[p][t] = 0;
    if (t == 0) { st->prefix[0] = 0; st->remaining[0] = N; }
    for (int s = t; s < n_seg; s += blockDim.x) counts[s] = 0;
}

// What pass p - 1 decided, worked out by every workgroup of the next launch for itself from the
// finished histogram (a kernel boundary is the only synchronisation): walk the 256 bins from
// the largest byte down until `remaining` keys are covered and fix that byte.  Workgroup 0
// also records the result for the launch after this one.  Called by all threads; p >= 1.
__device__ __forceinline__ void decide(SelectState *st, int p, unsigned long long &prefix, unsigned long long &remaining) {
    __shared__ unsigned long long bins[256];
    __shared__ unsigned long long out[2];
    bins[threadIdx.x] = st->hist[p - 1][threadIdx.x];
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned long long rem = st->remaining[p - 1];
        unsigned long long above = 0;
        int b = 255;
        for (; b > 0; --b) {
            if (above + bins[b] >= rem) break;
            above += bins[b];
        }
        out[0] = st->prefix[p - 1] | ((unsigned long long)b << (56 - 8 * (p - 1)));
        out[1] = rem - above;
        if (blockIdx.x == 0 && blockIdx.y == 0) { st->prefix[p] = out[0]; st->remaining[p] = out[1]; }
    }
    __syncthreads();
    prefix = out[0];
    remaining = out[1];
}

// Pass p: byte 7 - p of the keys whose higher bytes equal the prefix.
__global__ void __launch_bounds__(256) k_select_hist(const float *scores, unsigned long long n, SelectState *st,
                                                     int p) {
    __shared__ unsigned int h[256];
    h[threadIdx.x] = 0;
    unsigned long long prefix = 0, remaining = 0;
    if (p > 0) decide(st, p, prefix, remaining);
    else __syncthreads();
    const int shift = 56 - 8 * p;
    const unsigned long long stride = (unsigned long long)gridDim.x * 256;
    for (unsigned long long i = (unsigned long long)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        const unsigned long long key = key_of(scores, i);
        const bool match = p == 0 || ((key ^ prefix) >> (shift + 8)) == 0;
        if (match) atomicAdd(&h[(key >> shift) & 255], 1u);
    }
    __syncthreads();
    const unsigned int c = h[threadIdx.x];
    if (c) atomicAdd(&st->hist[p][threadIdx.x], (unsigned long long)c);
}

// Keep flags and kept blocks per segment (layer).  mode 0: keep keys >= the selected key,
// 1: keep nothing, 2: keep everything.  blockIdx.y = segment.
__global__ void __launch_bounds__(256) k_select_emit(const float *scores, const long long *seg_starts,
                                                     SelectState *st, int mode, uint8_t *mask,
                                                     unsigned long long *counts) {
    __shared__ unsigned int total;
    if (threadIdx.x == 0) total = 0;
    unsigned long long kth = 0, rank = 0;
    if (mode == 0) decide(st, kPasses, kth, rank);  // the last byte
    else __syncthreads();
    const unsigned long long lo = (unsigned long long)seg_starts[blockIdx.y], hi = (unsigned long long)seg_starts[blockIdx.y + 1];
    const unsigned long long stride = (unsigned long long)gridDim.x * 256;
    unsigned int mine = 0;
    for (unsigned long long i = lo + (unsigned long long)blockIdx.x * 256 + threadIdx.x; i < hi; i += stride) {
        const bool keep = mode == 2 || (mode == 0 && key_of(scores, i) >= kth);
        if (mask) mask[i] = keep ? 1 : 0;
        mine += keep ? 1u : 0u;
    }
    if (mine) atomicAdd(&total, mine);
    __syncthreads();
    if (threadIdx.x == 0 && total && counts) atomicAdd(&counts[blockIdx.y], (unsigned long long)total);
}

// Workspace layout: SelectState | seg_starts[n_seg + 1] | counts[n_seg].
struct Workspace {
    SelectState *st;
    long long *seg_starts;
    unsigned long long *counts;
};
static size_t workspace_bytes(int n_seg) {
    return sizeof(SelectState) + sizeof(long long) * (size_t)(n_seg + 1) + sizeof(unsigned long long) * (size_t)n_seg;
}
static Workspace carve(void *ws, int n_seg) {
    Workspace w;
    char *p = (char *)ws;
    w.st = (SelectState *)p;
    p += sizeof(SelectState);
    w.seg_starts = (long long *)p;
    p += sizeof(long long) * (size_t)(n_seg + 1);
    w.counts = (unsigned long long *)p;
    return w;
}

static int check(hipError_t e) {
    if (e == hipSuccess) return ALCS_OK;
    set_hip_error((int)e);
    return ALCS_E_HIP;
}

constexpr int kSelectBlocks = 2048;  // 8 workgroups of 256 threads per compute unit

// The selection of the N largest keys and the per-segment counts, all asynchronous on `stream`.
static int select_async(const float *scores, long long n, long long N, const Workspace &w, int n_seg,
                        uint8_t *mask, hipStream_t stream) {
    hipLaunchKernelGGL(k_select_init, dim3(1), dim3(256), 0, stream, w.st, (unsigned long long)N, w.counts, n_seg);
    const int blocks = (int)std::min<long long>(kSelectBlocks, (n + 255) / 256);
    int mode = N <= 0 ? 1 : N >= n ? 2 : 0;
    if (mode == 0) {
        for (int p = 0; p < kPasses; ++p)
            hipLaunchKernelGGL(k_select_hist, dim3(blocks), dim3(256), 0, stream, scores, (unsigned long long)n, w.st, p);
    }
    hipLaunchKernelGGL(k_select_emit, dim3(std::max(1, std::min(blocks, 256)), n_seg), dim3(256), 0, stream, scores,
                       w.seg_starts, w.st, mode, mask, w.counts);
    return check(hipGetLastError());
}

}  // namespace alcs

using namespace alcs;

extern "C" int alcs_block_scores(const float *W_dev, int Cout, int Cin, int kernel, int V, float *scores_dev,
                                 void *stream) {
    if (!W_dev || !scores_dev || Cout <= 0 || Cin <= 0) return ALCS_E_INVALID_ARG;
    if (kernel != 1 && kernel != 3) return ALCS_E_UNSUPPORTED;
    const long long K = (long long)Cin * kernel * kernel, G = (Cout + V - 1) / V, total = G * K;
    if ((total + 255) / 256 > INT32_MAX) return ALCS_E_UNSUPPORTED;
    void (*kern)(const float *, float *, int, long long, long long) = nullptr;
    switch (V) {
        case 1: kern = k_block_scores<1>; break;
        case 2: kern = k_block_scores<2>; break;
        case 4: kern = k_block_scores<4>; break;
        case 8: kern = k_block_scores<8>; break;
        case 16: kern = k_block_scores<16>; break;
        default: return ALCS_E_UNSUPPORTED;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream, W_dev,
                       scores_dev, Cout, K, total);
    return check(hipGetLastError());
}

extern "C" size_t alcs_select_workspace_bytes(int n_segments) {
    return n_segments < 0 ? 0 : workspace_bytes(n_segments);
}

// alcs_topn_mask with its selection state at `workspace_dev` (device memory of at least
// workspace_bytes(n_segments) bytes, 8-byte aligned).  Allocates nothing, on the host or the device.
static int topn_mask_in(const float *scores_dev, long long n_blocks, long long N, const long long *seg_starts_host,
                        int n_segments, uint8_t *mask_dev, long long *seg_counts_host, void *workspace_dev,
                        void *stream) {
    if (!scores_dev || !workspace_dev || n_blocks <= 0 || N < 0 || N > n_blocks) return ALCS_E_INVALID_ARG;
    if (n_blocks > 0xFFFFFFFFLL) return ALCS_E_UNSUPPORTED;  // the index half of a key is 32 bits
    if ((uintptr_t)workspace_dev & 7) return ALCS_E_INVALID_ARG;
    const long long whole[2] = {0, n_blocks};
    if (!seg_starts_host) { seg_starts_host = whole; n_segments = 1; }
    if (n_segments <= 0 || n_segments > 65535) return ALCS_E_INVALID_ARG;
    if (seg_starts_host[0] != 0 || seg_starts_host[n_segments] != n_blocks) return ALCS_E_INVALID_ARG;
    for (int s = 0; s < n_segments; ++s)
        if (seg_starts_host[s] > seg_starts_host[s + 1]) return ALCS_E_INVALID_ARG;
    const Workspace w = carve(workspace_dev, n_segments);
    hipStream_t st = (hipStream_t)stream;
    int rc = check(hipMemcpyAsync(w.seg_starts, seg_starts_host, sizeof(long long) * (size_t)(n_segments + 1),
                                  hipMemcpyHostToDevice, st));
    if (rc != ALCS_OK) return rc;
    rc = check(hipStreamSynchronize(st));  // the host array may be a temporary
    if (rc != ALCS_OK) return rc;
    rc = select_async(scores_dev, n_blocks, N, w, n_segments, mask_dev, st);
    if (rc != ALCS_OK) return rc;
    if (seg_counts_host) {
        rc = check(hipMemcpyAsync(seg_counts_host, w.counts, sizeof(long long) * (size_t)n_segments,
                                  hipMemcpyDeviceToHost, st));
        if (rc != ALCS_OK) return rc;
        rc = check(hipStreamSynchronize(st));
    }
    return rc;
}

extern "C" int alcs_topn_mask(const float *scores_dev, long long n_blocks, long long N,
                              const long long *seg_starts_host, int n_segments, uint8_t *mask_dev,
                              long long *seg_counts_host, void *workspace_dev, void *stream) {
    return topn_mask_in(scores_dev, n_blocks, N, seg_starts_host, n_segments, mask_dev, seg_counts_host,
                        workspace_dev, stream);
}

// ---------------------------------------------------------------- selection without any allocation
//
// The selection state of alcs_topn_mask_static lives in a file-scope device array instead of a
// caller-provided workspace: every GPU the library runs on holds one copy of it (kStaticBytes,
// about 33 KB) until the process ends.  In host code the array's name is only a stand-in for the
// symbol, not a device address; the address on the current device comes from
// hipGetSymbolAddress, once per device, and is what the kernels and copies are given.
namespace {
constexpr int kStaticMaxSegments = ALCS_TOPN_STATIC_MAX_SEGMENTS;
constexpr size_t kStaticBytes =
    (sizeof(SelectState) + sizeof(long long) * (kStaticMaxSegments + 1) + sizeof(unsigned long long) * kStaticMaxSegments + 255) &
    ~(size_t)255;
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call there).
int static_scratch(void **out) {
    int dev = -1;
    int rc = check(hipGetDevice(&dev));
    if (rc != ALCS_OK) return rc;
    if (dev < 0 || dev >= kMaxDevices) return ALCS_E_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        rc = check(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (rc != ALCS_OK) return rc;
        if (!ptr) return ALCS_E_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return ALCS_OK;
}
}  // namespace

extern "C" int alcs_topn_mask_static(const float *scores_dev, long long n_blocks, long long N,
                                     const long long *seg_starts_host, int n_segments, uint8_t *mask_dev,
                                     long long *seg_counts_host, void *stream) {
    // the size limit first: it does not depend on a device
    if (seg_starts_host && n_segments > kStaticMaxSegments) return ALCS_E_UNSUPPORTED;
    static_assert(kStaticBytes >= sizeof(SelectState) + 8 * (size_t)(2 * kStaticMaxSegments + 1), "scratch size");
    void *ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != ALCS_OK) return rc;
    return topn_mask_in(scores_dev, n_blocks, N, seg_starts_host, n_segments, mask_dev, seg_counts_host, ws, stream);
}

extern "C" int alcs_project_latency(const float *scores_dev, const long long *seg_starts_host, const int *V_host,
                                    int n_layers, double tau, const double *k_host, const double *t_host,
                                    const int *n_host, double budget, double eps, uint8_t *mask_dev,
                                    long long *N_out, double *t0_out, double *t1_out, void *workspace_dev,
                                    void *stream) {
    if (!scores_dev || !seg_starts_host || !V_host || !k_host || !t_host || !n_host || !workspace_dev)
        return ALCS_E_INVALID_ARG;
    if (n_layers <= 0 || n_layers > 65535 || !(eps >= 0.0) || budget != budget) return ALCS_E_INVALID_ARG;
    if ((uintptr_t)workspace_dev & 7) return ALCS_E_INVALID_ARG;
    const long long n = seg_starts_host[n_layers];
    if (seg_starts_host[0] != 0 || n <= 0) return ALCS_E_INVALID_ARG;
    if (n > 0xFFFFFFFFLL) return ALCS_E_UNSUPPORTED;
    for (int l = 0; l < n_layers; ++l)
        if (seg_starts_host[l] > seg_starts_host[l + 1] || V_host[l] <= 0) return ALCS_E_INVALID_ARG;
    const Workspace w = carve(workspace_dev, n_layers);
    hipStream_t st = (hipStream_t)stream;
    int rc = check(hipMemcpyAsync(w.seg_starts, seg_starts_host, sizeof(long long) * (size_t)(n_layers + 1),
                                  hipMemcpyHostToDevice, st));
    if (rc != ALCS_OK) return rc;
    std::vector<long long> counts(n_layers);
    std::vector<double> nnz(n_layers);
    // the latency of the network that keeps the N largest blocks (Section 3.3, Eq. (2))
    auto latency = [&](long long N, uint8_t *mask, double *t) -> int {
        int r = select_async(scores_dev, n, N, w, n_layers, mask, st);
        if (r != ALCS_OK) return r;
        r = check(hipMemcpyAsync(counts.data(), w.counts, sizeof(long long) * (size_t)n_layers, hipMemcpyDeviceToHost, st));
        if (r != ALCS_OK) return r;
        r = check(hipStreamSynchronize(st));
        if (r != ALCS_OK) return r;
        for (int l = 0; l < n_layers; ++l) nnz[l] = (double)counts[l] * V_host[l];
        return alcs_network_latency(tau, k_host, t_host, n_host, n_layers, nnz.data(), t);
    };
    long long N0 = 0, N1 = n;
    double t0 = 0, t1 = 0, t = 0;
    if ((rc = latency(N0, nullptr, &t0)) != ALCS_OK) return rc;
    if ((rc = latency(N1, nullptr, &t1)) != ALCS_OK) return rc;
    while (t1 - t0 > eps && N1 - N0 > 1) {
        const long long N = (N0 + N1) / 2;
        if ((rc = latency(N, nullptr, &t)) != ALCS_OK) return rc;
        if (t < budget) { t0 = t; N0 = N; }
        else { t1 = t; N1 = N; }
    }
    const long long N = (N0 + N1) / 2;
    if (mask_dev && (rc = latency(N, mask_dev, &t)) != ALCS_OK) return rc;
    if (N_out) *N_out = N;
    if (t0_out) *t0_out = t0;
    if (t1_out) *t1_out = t1;
    return ALCS_OK;
}
