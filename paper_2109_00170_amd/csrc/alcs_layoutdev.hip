// The device layout of a packed tensor built on the GPU: alcs_pack_from_csr_device makes a handle
// from the canonical arrays of Section 3.2.2 of arXiv 2109.00170 ("Storage format": kept columns
// per group, ascending column offsets, one V-vector per kept column) that are already on the
// device - what alcs_pack_csr_device leaves there - without a round trip of the arrays through
// the host.  In a re-pruning loop (Section 3.4, Algorithm 1: scores -> projection -> flags ->
// arrays -> handle) the host then sees a handful of scalars per layer.
//
// The layout is the one alcs_pack.cpp builds on the host (alcs_internal.h: bundles of groups in
// order of descending length, segments per channel chunk padded to runs, weight planes in the
// lane order of the matrix instruction, selector tables; with several groups per wavefront the
// parity-aware column order) and is built to the same bytes:
//   1. per group: length and validity (columns ascend, lie below K)            k_ld_stats
//   2. the groups' ranks by descending length, ties by index                   k_ld_rank
//   3. per group: running count of even-channel columns (parity-aware order)   k_ld_parity
//   4. per (bundle, chunk): the slots' column ranges, the segment's length     k_ld_segments
//   5. segment starts = exclusive scan of the padded lengths                   k_ld_scan
//   6. every kept block to its place: weights, selectors, parity note          k_ld_scatter
//   7. padded places: selector of the zero row that avoids the partner's banks k_ld_pads
// The host reads back two sets of scalars (longest group / block count, then padded columns /
// longest segment) to size the allocation; values are moved, never computed.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <new>
#include <vector>

#include "alcs_internal.h"

namespace alcs {
namespace {

constexpr int kRankLimit = 16384;  // groups the quadratic rank kernel takes; beyond, the host builds the layout

struct LdShape {
    int G, K, kk, V, VV, planes, Cin, k, KC, nchunks, GS, nbundles, noff;
    long long nnzb;
};

// scal[0] = longest group, scal[1] = 1 if the arrays are not canonical, scal[2] = padded columns in
// use, scal[3] = longest segment
__global__ void __launch_bounds__(256) k_ld_stats(const int32_t *row_ptr, const int32_t *col_idx, int G, int K,
                                                  long long nnzb, int *scal) {
    const int g = blockIdx.x * 256 + threadIdx.x;
    if (g >= G) return;
    const long long lo = row_ptr[g], hi = row_ptr[g + 1];
    bool bad = lo < 0 || hi < lo || hi > nnzb || hi - lo > K || (g == 0 && lo != 0);
    if (!bad) {
        for (long long t = lo; t < hi; ++t) {
            const int col = col_idx[t];
            if (col < 0 || col >= K || (t > lo && col <= col_idx[t - 1])) { bad = true; break; }
        }
        atomicMax(&scal[0], (int)(hi - lo));
    }
    if (bad) atomicMax(&scal[1], 1);
}

// order[rank] = g with rank = groups that are longer, or as long with a lower index (the stable
// descending sort of the host)
__global__ void __launch_bounds__(256) k_ld_rank(const int32_t *row_ptr, int G, int32_t *order, int32_t *pos) {
    const int g = blockIdx.x * 256 + threadIdx.x;
    if (g >= G) return;
    const int mine = row_ptr[g + 1] - row_ptr[g];
    int rank = 0;
    for (int h = 0; h < G; ++h) {
        const int c = row_ptr[h + 1] - row_ptr[h];
        rank += (c > mine) || (c == mine && h < g);
    }
    order[rank] = g;
    pos[g] = rank;
}

// evens[t + g] = columns of even channel among the group's blocks before t, for t in
// [row_ptr[g], row_ptr[g+1]] (one slot more per group for the total); one wavefront per group
__global__ void __launch_bounds__(64) k_ld_parity(const int32_t *row_ptr, const int32_t *col_idx, int kk,
                                                  int32_t *evens) {
    const int g = blockIdx.x, lane = threadIdx.x;
    const int lo = row_ptr[g], hi = row_ptr[g + 1];
    int base = 0;
    for (int t0 = lo; t0 <= hi; t0 += 64) {
        const int t = t0 + lane;
        const bool even = t < hi && (((col_idx[t] / kk) & 1) == 0);
        const unsigned long long ballot = __ballot(even);
        if (t <= hi) evens[t + g] = base + __popcll(ballot & ((1ull << lane) - 1ull));
        base += __popcll(ballot);
    }
}

__device__ __forceinline__ int lower_bound_dev(const int32_t *a, int lo, int hi, int key) {
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid] < key) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

// per (bundle, chunk): the work record (start filled by the scan), every slot's column range in
// the canonical arrays, the padded length
__global__ void __launch_bounds__(256) k_ld_segments(LdShape sh, const int32_t *row_ptr, const int32_t *col_idx,
                                                     const int32_t *order, Work *work, int32_t *seg_lo,
                                                     int32_t *seg_n, int32_t *span, int *scal) {
    const int si = blockIdx.x * 256 + threadIdx.x;
    if (si >= sh.nbundles * sh.nchunks) return;
    const int b = si / sh.nchunks, ch = si - b * sh.nchunks;
    const int c_lo = ch * sh.KC, c_hi = min(sh.Cin, c_lo + sh.KC);
    Work wk;
    wk.start = 0;
    wk.reserved[0] = wk.reserved[1] = 0;
    int longest = 0;
    for (int s = 0; s < kMaxSlots; ++s) {
        wk.group[s] = -1;
        const int p = b * sh.GS + s;
        if (s >= sh.GS || p >= sh.G) {
            if (s < sh.GS) { seg_lo[si * kMaxSlots + s] = 0; seg_n[si * kMaxSlots + s] = 0; }
            continue;
        }
        const int g = order[p];
        wk.group[s] = g;
        const int lo = lower_bound_dev(col_idx, row_ptr[g], row_ptr[g + 1], c_lo * sh.kk);
        const int hi = lower_bound_dev(col_idx, lo, row_ptr[g + 1], c_hi * sh.kk);
        seg_lo[si * kMaxSlots + s] = lo;
        seg_n[si * kMaxSlots + s] = hi - lo;
        longest = max(longest, hi - lo);
    }
    wk.cnt = (longest + kCntAlign - 1) / kCntAlign * kCntAlign;
    work[si] = wk;
    span[si] = (wk.cnt + kSegAlign - 1) / kSegAlign * kSegAlign;
    atomicMax(&scal[3], wk.cnt);
}

// exclusive scan of the padded lengths by one workgroup: the segments' first columns
__global__ void __launch_bounds__(1024) k_ld_scan(const int32_t *span, Work *work, int n, int *scal) {
    __shared__ long long buf[1024];
    __shared__ long long carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < n; base += 1024) {
        const int i = base + threadIdx.x;
        const long long v = i < n ? span[i] : 0;
        buf[threadIdx.x] = v;
        __syncthreads();
        for (int d = 1; d < 1024; d <<= 1) {
            const long long add = threadIdx.x >= d ? buf[threadIdx.x - d] : 0;
            __syncthreads();
            buf[threadIdx.x] += add;
            __syncthreads();
        }
        const long long start = carry + buf[threadIdx.x] - v;
        if (i < n) work[i].start = (int32_t)min(start, (long long)INT32_MAX);
        __syncthreads();
        if (threadIdx.x == 0) carry += buf[1023];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        scal[2] = (int)min(carry, (long long)INT32_MAX);
        scal[4] = carry > (long long)INT32_MAX ? 1 : 0;
    }
}

// every kept block to its place
__global__ void __launch_bounds__(256) k_ld_scatter(LdShape sh, const int32_t *row_ptr, const int32_t *col_idx,
                                                    const float *vals, const int32_t *pos, const int32_t *evens,
                                                    const Work *work, const int32_t *seg_lo, const int32_t *seg_n,
                                                    float *w, long long wplane, int32_t *off, long long offlen,
                                                    uint8_t *par) {
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= sh.nnzb) return;
    // the block's group: the last g with row_ptr[g] <= t
    int lo = 0, hi = sh.G;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (row_ptr[mid] <= t) lo = mid;
        else hi = mid;
    }
    const int g = lo;
    const int col = col_idx[t];
    const int c = col / sh.kk, ch = c / sh.KC;
    const int p = pos[g], b = p / sh.GS, s = p - b * sh.GS;
    const int si = b * sh.nchunks + ch;
    const Work wk = work[si];
    const int first = seg_lo[si * kMaxSlots + s], n = seg_n[si * kMaxSlots + s];
    int j = (int)(t - first);
    const int parity = c & 1;
    if (sh.GS > 1) {
        // even slots: even channels from the front, odd ones right-aligned at the back; odd slots
        // the other way round
        const int e_first = evens[first + g], e_here = evens[t + g], e_all = evens[first + n + g] - e_first;
        const int front_parity = (s & 1) ? 1 : 0;
        const int rank_even = e_here - e_first, rank_odd = j - rank_even;
        const int n_back = front_parity == 0 ? n - e_all : e_all;
        if (parity == front_parity) j = parity == 0 ? rank_even : rank_odd;
        else j = wk.cnt - n_back + (parity == 0 ? rank_even : rank_odd);
    }
    const long long at = (long long)wk.start + j;
    for (int v = 0; v < sh.V; ++v) {
        const int q = sh.V < 4 ? 0 : v / 4, i = sh.V < 4 ? v : v % 4;
        w[(size_t)q * wplane + layout_w_index(sh.GS, sh.VV, at, s, i)] = vals[t * sh.V + v];
    }
    const size_t oi = layout_off_index(sh.GS, at, s);
    for (int tb = 0; tb < sh.noff; ++tb) off[(size_t)tb * offlen + oi] = layout_off_of(col, sh.k, tb, sh.GS);
    par[oi] = (uint8_t)parity;
}

// the padded places of a segment (one workgroup per segment), and the spare run behind the last one
__global__ void __launch_bounds__(256) k_ld_pads(LdShape sh, const Work *work, int32_t *off, long long offlen,
                                                 const uint8_t *par, long long used, long long ncol) {
    const int nseg = sh.nbundles * sh.nchunks;
    if ((int)blockIdx.x == nseg) {
        for (long long i = used * sh.GS + threadIdx.x; i < ncol * sh.GS; i += 256) {
            const long long col = used + (i - used * sh.GS) / sh.GS;
            const int s = (int)((i - used * sh.GS) % sh.GS);
            const size_t oi = layout_off_index(sh.GS, col, s);
            for (int tb = 0; tb < sh.noff; ++tb) off[(size_t)tb * offlen + oi] = layout_pad_off(0, sh.KC, sh.k, tb, sh.GS, 0);
        }
        return;
    }
    const int si = blockIdx.x;
    const int ch = si % sh.nchunks;
    const Work wk = work[si];
    const int c0 = ch * sh.KC;
    const int span = (wk.cnt + kSegAlign - 1) / kSegAlign * kSegAlign;
    for (int i = threadIdx.x; i < span * sh.GS; i += 256) {
        const int j = i / sh.GS, s = i - j * sh.GS;
        const size_t oi = layout_off_index(sh.GS, (long long)wk.start + j, s);
        if (par[oi] != 0xFF) continue;  // a kept block sits here
        int which = 0;
        if (sh.GS > 1 && j < wk.cnt) {
            const int m = s ^ 1;
            const uint8_t mate = (m < sh.GS && wk.group[m] >= 0) ? par[layout_off_index(sh.GS, (long long)wk.start + j, m)] : 0xFF;
            if (mate != 0xFF) which = ((c0 + sh.KC) & 1) == mate ? 1 : 0;
            else which = s & 1;
        }
        for (int tb = 0; tb < sh.noff; ++tb) off[(size_t)tb * offlen + oi] = layout_pad_off(c0, sh.KC, sh.k, tb, sh.GS, which);
    }
}

int check(hipError_t e) {
    if (e == hipSuccess) return ALCS_OK;
    set_hip_error((int)e);
    return e == hipErrorOutOfMemory ? ALCS_E_ALLOC : ALCS_E_HIP;
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace
}  // namespace alcs

using namespace alcs;

extern "C" int alcs_pack_from_csr_device(const int32_t *row_ptr_dev, const int32_t *col_idx_dev, const float *vals_dev,
                                         int Cout, int Cin, int kernel, int V, const alcs_options *options,
                                         void *stream, alcs_packed_t **out) {
    if (out) *out = nullptr;
    if (!row_ptr_dev || !out || Cout <= 0 || Cin <= 0) return ALCS_E_INVALID_ARG;
    if (kernel != 1 && kernel != 3) return ALCS_E_UNSUPPORTED;
    if (V != 1 && V != 2 && V != 4 && V != 8 && V != 16) return ALCS_E_UNSUPPORTED;
    const int64_t K64 = (int64_t)Cin * kernel * kernel;
    if (K64 > (1 << 24) || Cout > (1 << 24)) return ALCS_E_UNSUPPORTED;
    const int K = (int)K64, G = (Cout + V - 1) / V;
    if ((int64_t)G * K > (int64_t)INT32_MAX - 1024) return ALCS_E_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    int dev = 0;
    int rc = check(hipGetDevice(&dev));
    if (rc != ALCS_OK) return rc;

    // block count and, if the arrays are not the canonical form, nothing else
    int32_t nnzb32 = 0;
    rc = check(hipMemcpyAsync(&nnzb32, row_ptr_dev + G, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    if (rc != ALCS_OK) return rc;
    int *scal = nullptr;
    rc = check(hipMalloc((void **)&scal, 8 * sizeof(int)));
    if (rc != ALCS_OK) return rc;
    void *tmp = nullptr, *blob = nullptr;
    alcs_packed *p = nullptr;
    auto fail = [&](int code) {
        if (scal) (void)hipFree(scal);
        if (tmp) (void)hipFree(tmp);
        if (blob) (void)hipFree(blob);
        delete p;
        return code;
    };
    if ((rc = check(hipMemsetAsync(scal, 0, 8 * sizeof(int), st))) != ALCS_OK) return fail(rc);
    if ((rc = check(hipStreamSynchronize(st))) != ALCS_OK) return fail(rc);
    const long long nnzb = nnzb32;
    if (nnzb < 0 || nnzb > (long long)G * K) return fail(ALCS_E_INVALID_ARG);
    if (nnzb > 0 && (!col_idx_dev || !vals_dev)) return fail(ALCS_E_INVALID_ARG);
    hipLaunchKernelGGL(k_ld_stats, dim3((G + 255) / 256), dim3(256), 0, st, row_ptr_dev, col_idx_dev, G, K, nnzb, scal);
    int h_scal[8] = {0};
    if ((rc = check(hipMemcpyAsync(h_scal, scal, sizeof(h_scal), hipMemcpyDeviceToHost, st))) != ALCS_OK) return fail(rc);
    if ((rc = check(hipStreamSynchronize(st))) != ALCS_OK) return fail(rc);
    if (h_scal[1]) return fail(ALCS_E_INVALID_ARG);

    p = new (std::nothrow) alcs_packed();
    if (!p) return fail(ALCS_E_ALLOC);
    p->Cout = Cout; p->Cin = Cin; p->k = kernel; p->V = V; p->G = G; p->K = K;
    p->nnzb = nnzb;
    p->max_count = h_scal[0];
    if (options) {
        if ((rc = check_options(options)) != ALCS_OK) return fail(rc);
        p->opt = *options;
    }
    int KC = 0, GS = 1;
    choose_tiles(p, &KC, &GS);
    Layout &L = p->lay;
    L.KC = KC;
    L.nchunks = (Cin + KC - 1) / KC;
    L.GS = GS;
    L.nbundles = (G + GS - 1) / GS;
    L.planes = V >= 4 ? V / 4 : 1;
    L.VV = V >= 4 ? 4 : V;
    L.noff = kernel == 1 ? 1 : kMaxOff;
    if (GS > 1 && (V < 4 || kernel != 1 || L.nchunks != 1)) return fail(ALCS_E_INVALID_ARG);
    if (G > kRankLimit) return fail(ALCS_E_UNSUPPORTED);  // the caller goes through the host (alcs_pack_from_csr)

    const LdShape sh{G, K, kernel * kernel, V, L.VV, L.planes, Cin, kernel, KC, L.nchunks, GS, L.nbundles, L.noff, nnzb};
    const long long nseg = (long long)L.nbundles * L.nchunks;
    if (nseg > (1LL << 26)) return fail(ALCS_E_UNSUPPORTED);
    // temporaries: pos[G] | evens[nnzb + G + 1] | seg_lo[nseg * 4] | seg_n[nseg * 4] | span[nseg] | work[nseg] | order[G]
    size_t o = 0;
    const size_t o_pos = o; o = align256(o + 4 * (size_t)G);
    const size_t o_ev = o; o = align256(o + 4 * (size_t)(nnzb + G + 1));
    const size_t o_lo = o; o = align256(o + 4 * (size_t)nseg * kMaxSlots);
    const size_t o_n = o; o = align256(o + 4 * (size_t)nseg * kMaxSlots);
    const size_t o_span = o; o = align256(o + 4 * (size_t)nseg);
    const size_t o_work = o; o = align256(o + sizeof(Work) * (size_t)nseg);
    const size_t o_order = o; o = align256(o + 4 * (size_t)G);
    if ((rc = check(hipMalloc(&tmp, o))) != ALCS_OK) return fail(rc);
    char *tb = (char *)tmp;
    int32_t *d_pos = (int32_t *)(tb + o_pos), *d_ev = (int32_t *)(tb + o_ev), *d_lo = (int32_t *)(tb + o_lo);
    int32_t *d_n = (int32_t *)(tb + o_n), *d_span = (int32_t *)(tb + o_span), *d_order = (int32_t *)(tb + o_order);
    Work *d_work = (Work *)(tb + o_work);
    hipLaunchKernelGGL(k_ld_rank, dim3((G + 255) / 256), dim3(256), 0, st, row_ptr_dev, G, d_order, d_pos);
    if (GS > 1) hipLaunchKernelGGL(k_ld_parity, dim3(G), dim3(64), 0, st, row_ptr_dev, col_idx_dev, kernel * kernel, d_ev);
    hipLaunchKernelGGL(k_ld_segments, dim3((unsigned)((nseg + 255) / 256)), dim3(256), 0, st, sh, row_ptr_dev, col_idx_dev,
                       d_order, d_work, d_lo, d_n, d_span, scal);
    hipLaunchKernelGGL(k_ld_scan, dim3(1), dim3(1024), 0, st, d_span, d_work, (int)nseg, scal);
    if ((rc = check(hipGetLastError())) != ALCS_OK) return fail(rc);
    if ((rc = check(hipMemcpyAsync(h_scal, scal, sizeof(h_scal), hipMemcpyDeviceToHost, st))) != ALCS_OK) return fail(rc);
    if ((rc = check(hipStreamSynchronize(st))) != ALCS_OK) return fail(rc);
    const long long used = h_scal[2];
    if (h_scal[4] || used > INT32_MAX / (4 * GS) - 64) return fail(ALCS_E_UNSUPPORTED);
    L.max_cnt = h_scal[3];
    L.ncol = used + kSegAlign;
    L.wplane = L.ncol * L.VV * GS;

    // the handle's allocation: work | weight planes | selector tables | order | canonical arrays | (parity notes)
    const size_t b_work = sizeof(Work) * (size_t)nseg, b_w = 4 * (size_t)L.planes * (size_t)L.wplane;
    const size_t b_off = 4 * (size_t)L.ncol * GS;
    size_t q = 0;
    const size_t q_work = q; q = align256(q + b_work);
    const size_t q_w = q; q = align256(q + b_w);
    const size_t q_off = q; q = align256(q + b_off * L.noff);
    const size_t q_order = q; q = align256(q + 4 * (size_t)G);
    const size_t q_rp = q; q = align256(q + 4 * (size_t)(G + 1));
    const size_t q_ci = q; q = align256(q + 4 * (size_t)nnzb);
    const size_t q_va = q; q = align256(q + 4 * (size_t)nnzb * V);
    const size_t total = q + 256;
    const size_t b_par = (size_t)L.ncol * GS;
    if ((rc = check(hipMalloc(&blob, total + align256(b_par)))) != ALCS_OK) return fail(rc);
    char *bb = (char *)blob;
    uint8_t *d_par = (uint8_t *)(bb + total);
    float *d_w = (float *)(bb + q_w);
    int32_t *d_off = (int32_t *)(bb + q_off);
    hipError_t e = hipMemsetAsync(d_w, 0, b_w, st);
    if (e == hipSuccess) e = hipMemsetAsync(d_par, 0xFF, b_par, st);
    if (e == hipSuccess) e = hipMemcpyAsync(bb + q_work, d_work, b_work, hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess) e = hipMemcpyAsync(bb + q_order, d_order, 4 * (size_t)G, hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess) e = hipMemcpyAsync(bb + q_rp, row_ptr_dev, 4 * (size_t)(G + 1), hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess && nnzb) e = hipMemcpyAsync(bb + q_ci, col_idx_dev, 4 * (size_t)nnzb, hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess && nnzb) e = hipMemcpyAsync(bb + q_va, vals_dev, 4 * (size_t)nnzb * V, hipMemcpyDeviceToDevice, st);
    if ((rc = check(e)) != ALCS_OK) return fail(rc);
    if (nnzb)
        hipLaunchKernelGGL(k_ld_scatter, dim3((unsigned)((nnzb + 255) / 256)), dim3(256), 0, st, sh, row_ptr_dev, col_idx_dev,
                           vals_dev, d_pos, d_ev, (const Work *)(bb + q_work), d_lo, d_n, d_w, (long long)L.wplane, d_off,
                           (long long)(b_off / 4), d_par);
    hipLaunchKernelGGL(k_ld_pads, dim3((unsigned)nseg + 1), dim3(256), 0, st, sh, (const Work *)(bb + q_work), d_off,
                       (long long)(b_off / 4), d_par, used, (long long)L.ncol);
    if ((rc = check(hipGetLastError())) != ALCS_OK) return fail(rc);
    if ((rc = check(hipStreamSynchronize(st))) != ALCS_OK) return fail(rc);  // the temporaries go away below

    p->host_arrays = false;
    p->dev.device = dev;
    device_shape(dev, &p->dev.cus, &p->dev.xcds);
    p->dev.blob = blob;
    p->dev.bytes = total;
    p->dev.work = (const Work *)(bb + q_work);
    p->dev.w = d_w;
    for (int t = 0; t < kMaxOff; ++t) p->dev.off[t] = t < L.noff ? d_off + (size_t)t * (b_off / 4) : nullptr;
    p->dev.order = (const int32_t *)(bb + q_order);
    p->dev.row_ptr = (const int32_t *)(bb + q_rp);
    p->dev.col_idx = (const int32_t *)(bb + q_ci);
    p->dev.vals = (const float *)(bb + q_va);
    (void)hipFree(tmp);
    (void)hipFree(scal);
    *out = p;
    return ALCS_OK;
}

extern "C" int alcs_pack_weights_device(const float *W_dev, const uint8_t *mask_dev, int Cout, int Cin, int kernel, int V,
                                        const alcs_options *options, void *stream, alcs_packed_t **out) {
    if (out) *out = nullptr;
    if (!W_dev || !out || Cout <= 0 || Cin <= 0) return ALCS_E_INVALID_ARG;
    if (kernel != 1 && kernel != 3) return ALCS_E_UNSUPPORTED;
    if (V != 1 && V != 2 && V != 4 && V != 8 && V != 16) return ALCS_E_UNSUPPORTED;
    const int64_t K64 = (int64_t)Cin * kernel * kernel;
    if (K64 > (1 << 24) || Cout > (1 << 24)) return ALCS_E_UNSUPPORTED;
    const int G = (Cout + V - 1) / V;
    const long long cap = (long long)G * K64;
    if (cap > (long long)INT32_MAX - 1024) return ALCS_E_UNSUPPORTED;
    // canonical arrays sized for every block kept: one allocation, no counting pass of its own
    const size_t o_rp = 0, o_ci = align256(4 * (size_t)(G + 1)), o_va = align256(o_ci + 4 * (size_t)cap);
    void *tmp = nullptr;
    int rc = check(hipMalloc(&tmp, o_va + 4 * (size_t)cap * V));
    if (rc != ALCS_OK) return rc;
    char *tb = (char *)tmp;
    rc = alcs_pack_csr_device(W_dev, mask_dev, Cout, Cin, kernel, V, (int32_t *)(tb + o_rp), (int32_t *)(tb + o_ci),
                              (float *)(tb + o_va), cap, nullptr, stream);
    if (rc == ALCS_OK)
        rc = alcs_pack_from_csr_device((const int32_t *)(tb + o_rp), (const int32_t *)(tb + o_ci), (const float *)(tb + o_va),
                                       Cout, Cin, kernel, V, options, stream, out);
    (void)hipFree(tmp);
    return rc;
}
