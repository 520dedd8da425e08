// Channel records for 3x3 handles whose pattern is shared by the nine taps (every kept input
// channel of a group keeps all of its taps): Section 3.2.2 of arXiv 2109.00170 stores one column
// offset per kept column; when the nine columns of a channel are kept or dropped together one
// record per CHANNEL says the same - the channel's index and its 9 x V weights - and the kernel
// can fetch a pixel's three input rows once and take the left and right neighbours from the lanes
// beside it, instead of one on-chip read per tap.  The records are derived on the device from the
// layout every handle has (host- or device-built), so both kinds of handle get them the same way:
//   k_chan_scan  per (bundle, chunk): records = padded columns / 9 (the padding is < 8), and
//                their first index by an exclusive scan;
//   k_chan_fill  per record: the channel from the first tap's row selector, the weights of
//                taps 0..8 copied to [tap][row] with taps 9..15 zero (one 256-byte line a record
//                and plane, in the lane order of the matrix instruction's block broadcast).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "alcs_internal.h"

namespace alcs {
namespace {

__global__ void __launch_bounds__(1024) k_chan_scan(const Work *work, int nseg, int32_t *cwork) {
    __shared__ int buf[1024];
    __shared__ int carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < nseg; base += 1024) {
        const int i = base + threadIdx.x;
        const int n = i < nseg ? work[i].cnt / 9 : 0;
        buf[threadIdx.x] = n;
        __syncthreads();
        for (int d = 1; d < 1024; d <<= 1) {
            const int add = threadIdx.x >= d ? buf[threadIdx.x - d] : 0;
            __syncthreads();
            buf[threadIdx.x] += add;
            __syncthreads();
        }
        if (i < nseg) {
            cwork[2 * i] = carry + buf[threadIdx.x] - n;
            cwork[2 * i + 1] = n;
        }
        __syncthreads();
        if (threadIdx.x == 0) carry += buf[1023];
        __syncthreads();
    }
}

// one workgroup of 64 lanes per (bundle, chunk)
__global__ void __launch_bounds__(64) k_chan_fill(const Work *work, const int32_t *cwork, const float *w, long long wplane,
                                                  const int32_t *off0, int planes, int nchunks, int KC, float *cw,
                                                  long long cwplane, int32_t *csel) {
    const int seg = blockIdx.x, lane = threadIdx.x;
    const int start = work[seg].start;
    const int first = cwork[2 * seg], n = cwork[2 * seg + 1];
    const int c0 = (seg % nchunks) * KC;
    const int t = lane >> 2, i = lane & 3;
    constexpr int kPlane0 = halo_area3(1, 0, false) * 4;  // bytes per channel plane in selector table 0
    for (int j = 0; j < n; ++j) {
        const long long col = (long long)start + 9 * j;
        for (int q = 0; q < planes; ++q)
            cw[(size_t)q * cwplane + (size_t)(first + j) * 64 + lane] = t < 9 ? w[(size_t)q * wplane + (col + t) * 4 + i] : 0.f;
        if (lane == 0) csel[first + j] = off0[col] / kPlane0 - c0;
    }
}

}  // namespace

int add_channel_records(alcs_packed *p, void *stream) {
    const Layout &L = p->lay;
    if (!L.tap_shared || p->k != 3 || p->V < 4 || L.GS != 1 || !p->dev.blob || p->dev.chan_blob) return ALCS_OK;
    const long long nseg = (long long)L.nbundles * L.nchunks;
    const long long cap = L.ncol / 9 + 1;  // records: at most padded columns / 9
    const long long cwplane = cap * 64;
    auto align256 = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t o_cw = 0;
    const size_t o_sel = align256(4 * (size_t)cwplane * L.planes);
    const size_t o_work = align256(o_sel + 4 * (size_t)cap);
    const size_t total = align256(o_work + 8 * (size_t)nseg) + 256;
    void *blob = nullptr;
    hipError_t e = hipMalloc(&blob, total);
    if (e != hipSuccess) {
        set_hip_error((int)e);
        (void)hipGetLastError();
        return e == hipErrorOutOfMemory ? ALCS_E_ALLOC : ALCS_E_HIP;
    }
    char *bb = (char *)blob;
    hipStream_t st = (hipStream_t)stream;
    e = hipMemsetAsync(bb + o_sel, 0, 4 * (size_t)cap, st);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(k_chan_scan, dim3(1), dim3(1024), 0, st, p->dev.work, (int)nseg, (int32_t *)(bb + o_work));
        hipLaunchKernelGGL(k_chan_fill, dim3((unsigned)nseg), dim3(64), 0, st, p->dev.work, (const int32_t *)(bb + o_work),
                           p->dev.w, (long long)L.wplane, p->dev.off[0], L.planes, L.nchunks, L.KC, (float *)(bb + o_cw),
                           cwplane, (int32_t *)(bb + o_sel));
        e = hipGetLastError();
    }
    if (e != hipSuccess) {
        set_hip_error((int)e);
        (void)hipFree(blob);
        return ALCS_E_HIP;
    }
    p->dev.chan_blob = blob;
    p->dev.cw = (const float *)(bb + o_cw);
    p->dev.csel = (const int32_t *)(bb + o_sel);
    p->dev.cwork = (const int32_t *)(bb + o_work);
    p->dev.cwplane = cwplane;
    return ALCS_OK;
}

}  // namespace alcs
