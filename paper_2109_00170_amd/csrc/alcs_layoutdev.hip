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
// longest segment) to choose the tiles and to size the allocation; values are moved, never
// computed.  Several layers are built in one call (alcs_pack_network_device): every step is
// enqueued for all of them before the host waits, so a network costs three waits, not three a layer.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <new>
#include <vector>

#include "alcs_internal.h"

namespace alcs {

// alcs_packdev.hip: the canonical arrays from weights and flags (counts + scan; compaction)
int enqueue_csr_count(const uint8_t *mask_dev, int G, int K, int32_t *row_ptr_dev, hipStream_t st);
int enqueue_csr_fill(const float *W_dev, const uint8_t *mask_dev, int Cout, int K, int V, int G,
                     const int32_t *row_ptr_dev, int32_t *col_idx_dev, float *vals_dev, hipStream_t st);

namespace {

constexpr int kRankLimit = 16384;  // groups the quadratic rank kernel takes; beyond, the host builds the layout

struct LdShape {
    int G, K, kk, V, VV, planes, Cin, k, KC, nchunks, GS, nbundles, noff;
    long long nnzb;
};

// scal[0] = longest group, scal[1] = 1 if the arrays are not canonical, scal[2] = padded columns in
// use, scal[3] = longest segment, scal[4] = 1 if the padded columns overflow
// scal[5] = blocks in all (row_ptr[G]).  `walk` = 0 skips the columns (arrays the library's own
// kernels have written).
__global__ void __launch_bounds__(256) k_ld_stats(const int32_t *row_ptr, const int32_t *col_idx, int G, int K,
                                                  long long room, int walk, int *scal) {
    const int g = blockIdx.x * 256 + threadIdx.x;
    if (g >= G) return;
    const long long nnzb = row_ptr[G];
    const long long lo = row_ptr[g], hi = row_ptr[g + 1];
    if (g == G - 1) scal[5] = (int)nnzb;
    bool bad = lo < 0 || hi < lo || hi > nnzb || nnzb > room || hi - lo > K || (g == 0 && lo != 0);
    if (!bad) {
        if (walk)
            for (long long t = lo; t < hi; ++t) {
                const int col = col_idx[t];
                if (col < 0 || col >= K || (t > lo && col <= col_idx[t - 1])) { bad = true; break; }
            }
        atomicMax(&scal[0], (int)(hi - lo));
    }
    if (bad) atomicMax(&scal[1], 1);
}

// scal[6] = 1 unless every group's kept columns are whole channels of nine taps (3x3 handles)
__global__ void __launch_bounds__(256) k_ld_tapshared(const int32_t *row_ptr, const int32_t *col_idx, int G, long long nnzb,
                                                      int *scal) {
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= nnzb) return;
    int lo = 0, hi = G;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (row_ptr[mid] <= t) lo = mid;
        else hi = mid;
    }
    const int rel = (int)(t - row_ptr[lo]);
    bool ok = rel % 9 == 0 ? col_idx[t] % 9 == 0 : col_idx[t] == col_idx[t - 1] + 1;
    if (rel == 0) ok = ok && (row_ptr[lo + 1] - row_ptr[lo]) % 9 == 0;
    if (!ok) atomicMax(&scal[6], 1);
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

int check_shape(int Cout, int Cin, int kernel, int V) {  // the limits of alcs_pack_weights
    if (Cout <= 0 || Cin <= 0) return ALCS_E_INVALID_ARG;
    if (kernel != 1 && kernel != 3) return ALCS_E_UNSUPPORTED;
    if (V != 1 && V != 2 && V != 4 && V != 8 && V != 16) return ALCS_E_UNSUPPORTED;
    const int64_t K64 = (int64_t)Cin * kernel * kernel;
    if (K64 > (1 << 24) || Cout > (1 << 24)) return ALCS_E_UNSUPPORTED;
    const int G = (Cout + V - 1) / V;
    if ((int64_t)G * K64 > (int64_t)INT32_MAX - 1024) return ALCS_E_UNSUPPORTED;
    return ALCS_OK;
}

// More groups than the quadratic rank kernel takes (an FC layer with more than 16384 * V outputs):
// the canonical arrays go to the host once and alcs_pack.cpp builds the layout there.
bool too_many_groups(int Cout, int V) { return (Cout + V - 1) / V > kRankLimit; }

int through_the_host(const int32_t *rp_dev, const int32_t *ci_dev, const float *va_dev, int Cout, int Cin, int kernel, int V,
                     const alcs_options *options, hipStream_t st, alcs_packed_t **out) {
    const int G = (Cout + V - 1) / V;
    std::vector<int32_t> rp, ci;
    std::vector<float> va;
    try {
        rp.resize((size_t)G + 1);
        int rc = check(hipMemcpyAsync(rp.data(), rp_dev, 4 * ((size_t)G + 1), hipMemcpyDeviceToHost, st));
        if (rc == ALCS_OK) rc = check(hipStreamSynchronize(st));
        if (rc != ALCS_OK) return rc;
        const long long nnzb = rp[(size_t)G];
        if (nnzb < 0 || nnzb > (long long)G * Cin * kernel * kernel) return ALCS_E_INVALID_ARG;
        if (nnzb > 0 && (!ci_dev || !va_dev)) return ALCS_E_INVALID_ARG;
        ci.resize((size_t)nnzb);
        va.resize((size_t)nnzb * V);
        if (nnzb) {
            rc = check(hipMemcpyAsync(ci.data(), ci_dev, 4 * (size_t)nnzb, hipMemcpyDeviceToHost, st));
            if (rc == ALCS_OK) rc = check(hipMemcpyAsync(va.data(), va_dev, 4 * (size_t)nnzb * V, hipMemcpyDeviceToHost, st));
            if (rc == ALCS_OK) rc = check(hipStreamSynchronize(st));
            if (rc != ALCS_OK) return rc;
        }
    } catch (const std::bad_alloc &) {
        return ALCS_E_ALLOC;
    }
    return pack_from_csr_host(rp.data(), ci.data(), va.data(), Cout, Cin, kernel, V, options, out);
}

// One layer on its way to a handle.
struct Job {
    // what the caller gave: weights + flags, or the canonical arrays
    const float *W = nullptr;
    const uint8_t *mask = nullptr;
    const int32_t *rp = nullptr, *ci = nullptr;
    const float *va = nullptr;
    bool own_arrays = false;  // rp / ci / va lie in the temporary and are filled here
    alcs_packed *p = nullptr;
    long long cap = 0;        // blocks the temporaries have room for
    long long max_seg = 0;    // (bundle, chunk) pairs they have room for
    // temporaries
    int *scal = nullptr;
    int32_t *t_rp = nullptr, *t_ci = nullptr, *pos = nullptr, *ev = nullptr, *lo = nullptr, *n = nullptr, *span = nullptr,
            *order = nullptr;
    float *t_va = nullptr;
    Work *work = nullptr;
    LdShape sh{};
    long long used = 0;
    void *blob = nullptr;
};

// Upper bound of the (bundle, chunk) pairs of a layer: one group per bundle, the chunk size of the
// tile policy (which does not depend on the flags).
long long seg_bound(int Cout, int Cin, int kernel, int V, const alcs_options *opt) {
    alcs_packed probe;
    probe.Cout = Cout; probe.Cin = Cin; probe.k = kernel; probe.V = V;
    probe.G = (Cout + V - 1) / V;
    probe.K = Cin * kernel * kernel;
    if (opt) probe.opt = *opt;
    int KC = 0, GS = 1;
    choose_tiles(&probe, &KC, &GS);
    return (long long)probe.G * ((Cin + KC - 1) / KC);
}

// Bytes of temporary a layer needs, and (carve != null) the pointers into one.
size_t carve(Job *j, char *base, int Cout, int Cin, int kernel, int V, const alcs_options *opt, bool own_arrays) {
    const int G = (Cout + V - 1) / V;
    const long long cap = (long long)G * Cin * kernel * kernel;
    const long long nseg = seg_bound(Cout, Cin, kernel, V, opt);
    size_t o = 0;
    auto take = [&](size_t bytes) { const size_t at = o; o = align256(o + bytes); return at; };
    const size_t o_rp = take(own_arrays ? 4 * (size_t)(G + 1) : 0);
    const size_t o_ci = take(own_arrays ? 4 * (size_t)cap : 0);
    const size_t o_va = take(own_arrays ? 4 * (size_t)cap * V : 0);
    const size_t o_pos = take(4 * (size_t)G);
    const size_t o_ev = take(4 * (size_t)(cap + G + 1));
    const size_t o_lo = take(4 * (size_t)nseg * kMaxSlots);
    const size_t o_n = take(4 * (size_t)nseg * kMaxSlots);
    const size_t o_span = take(4 * (size_t)nseg);
    const size_t o_work = take(sizeof(Work) * (size_t)nseg);
    const size_t o_order = take(4 * (size_t)G);
    if (j) {
        j->cap = cap;
        j->max_seg = nseg;
        j->t_rp = (int32_t *)(base + o_rp);
        j->t_ci = (int32_t *)(base + o_ci);
        j->t_va = (float *)(base + o_va);
        j->pos = (int32_t *)(base + o_pos);
        j->ev = (int32_t *)(base + o_ev);
        j->lo = (int32_t *)(base + o_lo);
        j->n = (int32_t *)(base + o_n);
        j->span = (int32_t *)(base + o_span);
        j->work = (Work *)(base + o_work);
        j->order = (int32_t *)(base + o_order);
    }
    return o;
}

struct LayerIn {
    const float *W;
    const uint8_t *mask;
    const int32_t *rp, *ci;
    const float *va;
    int Cout, Cin, kernel, V;
    const alcs_options *opt;
};

// All layers through the three steps; out[i] receive the handles (all or none).
int build_all(const LayerIn *in, int n, void *workspace, size_t workspace_bytes, hipStream_t st, alcs_packed_t **out) {
    for (int i = 0; i < n; ++i) out[i] = nullptr;
    for (int i = 0; i < n; ++i) {
        int rc = check_shape(in[i].Cout, in[i].Cin, in[i].kernel, in[i].V);
        if (rc == ALCS_OK && too_many_groups(in[i].Cout, in[i].V)) rc = ALCS_E_UNSUPPORTED;
        if (rc == ALCS_OK && in[i].opt) rc = check_options(in[i].opt);
        if (rc != ALCS_OK) return rc;
        if (!in[i].W && !in[i].rp) return ALCS_E_INVALID_ARG;
    }
    int dev = 0;
    int rc = check(hipGetDevice(&dev));
    if (rc != ALCS_OK) return rc;
    int cus = 0, xcds = 0;
    device_shape(dev, &cus, &xcds);
    std::vector<Job> jobs;
    std::vector<int> h_scal;
    try {
        jobs.resize((size_t)n);
        h_scal.resize((size_t)n * 8);
    } catch (const std::bad_alloc &) {
        return ALCS_E_ALLOC;
    }
    // the jobs' scalars (8 ints each) lie together at the start, so that one copy reads them all
    const size_t scal_bytes = align256(8 * sizeof(int) * (size_t)n);
    size_t need = scal_bytes;
    for (int i = 0; i < n; ++i) need += carve(nullptr, nullptr, in[i].Cout, in[i].Cin, in[i].kernel, in[i].V, in[i].opt, in[i].W != nullptr);
    void *own_ws = nullptr;
    if (!workspace) {
        if ((rc = check(hipMalloc(&own_ws, need))) != ALCS_OK) return rc;
        workspace = own_ws;
    } else if (workspace_bytes < need || ((uintptr_t)workspace & 255) != 0) {
        return ALCS_E_INVALID_ARG;
    }
    auto fail = [&](int code) {
        (void)hipStreamSynchronize(st);  // nothing may still write what is freed here
        for (Job &j : jobs) {
            if (j.blob) (void)hipFree(j.blob);
            if (j.p && j.p->dev.chan_blob) (void)hipFree(j.p->dev.chan_blob);
            delete j.p;
        }
        if (own_ws) (void)hipFree(own_ws);
        return code;
    };
    {
        char *base = (char *)workspace + scal_bytes;
        for (int i = 0; i < n; ++i) {
            Job &j = jobs[(size_t)i];
            j.scal = (int *)workspace + 8 * i;
            j.own_arrays = in[i].W != nullptr;
            base += carve(&j, base, in[i].Cout, in[i].Cin, in[i].kernel, in[i].V, in[i].opt, j.own_arrays);
            j.W = in[i].W; j.mask = in[i].mask;
            j.rp = j.own_arrays ? j.t_rp : in[i].rp;
            j.ci = j.own_arrays ? j.t_ci : in[i].ci;
            j.va = j.own_arrays ? j.t_va : in[i].va;
            j.p = new (std::nothrow) alcs_packed();
            if (!j.p) return fail(ALCS_E_ALLOC);
            alcs_packed *p = j.p;
            p->Cout = in[i].Cout; p->Cin = in[i].Cin; p->k = in[i].kernel; p->V = in[i].V;
            p->G = (p->Cout + p->V - 1) / p->V;
            p->K = p->Cin * p->k * p->k;
            if (in[i].opt) p->opt = *in[i].opt;
        }
    }
    auto read_scalars = [&]() {
        const int r = check(hipMemcpyAsync(h_scal.data(), workspace, 8 * sizeof(int) * (size_t)n, hipMemcpyDeviceToHost, st));
        return r != ALCS_OK ? r : check(hipStreamSynchronize(st));
    };

    // step 1: arrays' row pointers (own arrays), lengths, validity
    if ((rc = check(hipMemsetAsync(workspace, 0, 8 * sizeof(int) * (size_t)n, st))) != ALCS_OK) return fail(rc);
    for (Job &j : jobs) {
        const alcs_packed *p = j.p;
        if (j.own_arrays && (rc = enqueue_csr_count(j.mask, p->G, p->K, j.t_rp, st)) != ALCS_OK) return fail(rc);
        hipLaunchKernelGGL(k_ld_stats, dim3((p->G + 255) / 256), dim3(256), 0, st, j.rp, j.ci, p->G, p->K, j.cap,
                           j.own_arrays ? 0 : 1, j.scal);
    }
    if ((rc = check(hipGetLastError())) != ALCS_OK) return fail(rc);
    if ((rc = read_scalars()) != ALCS_OK) return fail(rc);

    // step 2: tiles, then order, segments and their starts
    for (int i = 0; i < n; ++i) {
        Job &j = jobs[(size_t)i];
        alcs_packed *p = j.p;
        const int *hs = &h_scal[(size_t)i * 8];
        if (hs[1]) return fail(ALCS_E_INVALID_ARG);
        p->max_count = hs[0];
        p->nnzb = hs[5];
        if (p->nnzb > 0 && !j.own_arrays && (!j.ci || !j.va)) return fail(ALCS_E_INVALID_ARG);
        int KC = 0, GS = 1;
        choose_tiles(p, &KC, &GS);
        Layout &L = p->lay;
        L.KC = KC;
        L.nchunks = (p->Cin + KC - 1) / KC;
        L.GS = GS;
        L.nbundles = (p->G + GS - 1) / GS;
        L.planes = p->V >= 4 ? p->V / 4 : 1;
        L.VV = p->V >= 4 ? 4 : p->V;
        L.noff = p->k == 1 ? 1 : kMaxOff;
        if (GS > 1 && (p->V < 4 || p->k != 1 || L.nchunks != 1)) return fail(ALCS_E_INVALID_ARG);
        const long long nseg = (long long)L.nbundles * L.nchunks;
        if (nseg > j.max_seg) return fail(ALCS_E_INVALID_ARG);  // cannot happen: the bound takes one group per bundle
        j.sh = LdShape{p->G, p->K, p->k * p->k, p->V, L.VV, L.planes, p->Cin, p->k, KC, L.nchunks, GS, L.nbundles, L.noff, p->nnzb};
        if (j.own_arrays && p->nnzb &&
            (rc = enqueue_csr_fill(j.W, j.mask, p->Cout, p->K, p->V, p->G, j.t_rp, j.t_ci, j.t_va, st)) != ALCS_OK)
            return fail(rc);
        if (p->k == 3 && p->nnzb > 0 && p->nnzb % 9 == 0)
            hipLaunchKernelGGL(k_ld_tapshared, dim3((unsigned)((p->nnzb + 255) / 256)), dim3(256), 0, st, j.rp, j.ci, p->G,
                               (long long)p->nnzb, j.scal);
        hipLaunchKernelGGL(k_ld_rank, dim3((p->G + 255) / 256), dim3(256), 0, st, j.rp, p->G, j.order, j.pos);
        if (GS > 1) hipLaunchKernelGGL(k_ld_parity, dim3(p->G), dim3(64), 0, st, j.rp, j.ci, p->k * p->k, j.ev);
        hipLaunchKernelGGL(k_ld_segments, dim3((unsigned)((nseg + 255) / 256)), dim3(256), 0, st, j.sh, j.rp, j.ci, j.order,
                           j.work, j.lo, j.n, j.span, j.scal);
        hipLaunchKernelGGL(k_ld_scan, dim3(1), dim3(1024), 0, st, j.span, j.work, (int)nseg, j.scal);
    }
    if ((rc = check(hipGetLastError())) != ALCS_OK) return fail(rc);
    if ((rc = read_scalars()) != ALCS_OK) return fail(rc);

    // step 3: the handles' allocations, every block to its place
    for (int i = 0; i < n; ++i) {
        Job &j = jobs[(size_t)i];
        alcs_packed *p = j.p;
        Layout &L = p->lay;
        const int *hs = &h_scal[(size_t)i * 8];
        const int GS = L.GS, G = p->G, V = p->V;
        const long long nnzb = p->nnzb, nseg = (long long)L.nbundles * L.nchunks;
        j.used = hs[2];
        if (hs[4] || j.used > INT32_MAX / (4 * GS) - 64) return fail(ALCS_E_UNSUPPORTED);
        L.max_cnt = hs[3];
        L.tap_shared = p->k == 3 && nnzb > 0 && nnzb % 9 == 0 && hs[6] == 0;
        L.ncol = j.used + kSegAlign;
        L.wplane = L.ncol * L.VV * GS;
        // work | weight planes | selector tables | order | canonical arrays | (parity notes, build only)
        const size_t b_work = sizeof(Work) * (size_t)nseg, b_w = 4 * (size_t)L.planes * (size_t)L.wplane;
        const size_t b_off = 4 * (size_t)L.ncol * GS;
        size_t q = 0;
        auto take = [&](size_t bytes) { const size_t at = q; q = align256(q + bytes); return at; };
        const size_t q_work = take(b_work), q_w = take(b_w), q_off = take(b_off * L.noff), q_order = take(4 * (size_t)G);
        const size_t q_rp = take(4 * (size_t)(G + 1)), q_ci = take(4 * (size_t)nnzb), q_va = take(4 * (size_t)nnzb * V);
        const size_t total = q + 256;
        const size_t b_par = (size_t)L.ncol * GS;
        if ((rc = check(hipMalloc(&j.blob, total + align256(b_par)))) != ALCS_OK) return fail(rc);
        char *bb = (char *)j.blob;
        uint8_t *d_par = (uint8_t *)(bb + total);
        float *d_w = (float *)(bb + q_w);
        int32_t *d_off = (int32_t *)(bb + q_off);
        hipError_t e = hipMemsetAsync(d_w, 0, b_w, st);
        if (e == hipSuccess) e = hipMemsetAsync(d_par, 0xFF, b_par, st);
        if (e == hipSuccess) e = hipMemcpyAsync(bb + q_work, j.work, b_work, hipMemcpyDeviceToDevice, st);
        if (e == hipSuccess) e = hipMemcpyAsync(bb + q_order, j.order, 4 * (size_t)G, hipMemcpyDeviceToDevice, st);
        if (e == hipSuccess) e = hipMemcpyAsync(bb + q_rp, j.rp, 4 * (size_t)(G + 1), hipMemcpyDeviceToDevice, st);
        if (e == hipSuccess && nnzb) e = hipMemcpyAsync(bb + q_ci, j.ci, 4 * (size_t)nnzb, hipMemcpyDeviceToDevice, st);
        if (e == hipSuccess && nnzb) e = hipMemcpyAsync(bb + q_va, j.va, 4 * (size_t)nnzb * V, hipMemcpyDeviceToDevice, st);
        if ((rc = check(e)) != ALCS_OK) return fail(rc);
        if (nnzb)
            hipLaunchKernelGGL(k_ld_scatter, dim3((unsigned)((nnzb + 255) / 256)), dim3(256), 0, st, j.sh, j.rp, j.ci, j.va, j.pos,
                               j.ev, (const Work *)(bb + q_work), j.lo, j.n, d_w, (long long)L.wplane, d_off,
                               (long long)(b_off / 4), d_par);
        hipLaunchKernelGGL(k_ld_pads, dim3((unsigned)nseg + 1), dim3(256), 0, st, j.sh, (const Work *)(bb + q_work), d_off,
                           (long long)(b_off / 4), d_par, j.used, (long long)L.ncol);
        p->host_arrays = false;
        p->dev.device = dev;
        p->dev.cus = cus;
        p->dev.xcds = xcds;
        p->dev.bytes = total;
        p->dev.work = (const Work *)(bb + q_work);
        p->dev.w = d_w;
        for (int t = 0; t < kMaxOff; ++t) p->dev.off[t] = t < L.noff ? d_off + (size_t)t * (b_off / 4) : nullptr;
        p->dev.order = (const int32_t *)(bb + q_order);
        p->dev.row_ptr = (const int32_t *)(bb + q_rp);
        p->dev.col_idx = (const int32_t *)(bb + q_ci);
        p->dev.vals = (const float *)(bb + q_va);
        p->dev.blob = j.blob;  // for the channel records; taken back below if the call fails
        rc = add_channel_records(p, st);
        p->dev.blob = nullptr;
        if (rc != ALCS_OK) return fail(rc);
    }
    if ((rc = check(hipGetLastError())) != ALCS_OK) return fail(rc);
    if ((rc = check(hipStreamSynchronize(st))) != ALCS_OK) return fail(rc);  // the temporaries are free again
    for (int i = 0; i < n; ++i) {
        Job &j = jobs[(size_t)i];
        j.p->dev.blob = j.blob;
        out[i] = j.p;
    }
    if (own_ws) (void)hipFree(own_ws);
    return ALCS_OK;
}

}  // namespace
}  // namespace alcs

using namespace alcs;

extern "C" int alcs_pack_from_csr_device(const int32_t *row_ptr_dev, const int32_t *col_idx_dev, const float *vals_dev,
                                         int Cout, int Cin, int kernel, int V, const alcs_options *options,
                                         void *stream, alcs_packed_t **out) {
    if (out) *out = nullptr;
    if (!row_ptr_dev || !out) return ALCS_E_INVALID_ARG;
    if (check_shape(Cout, Cin, kernel, V) == ALCS_OK && too_many_groups(Cout, V))
        return through_the_host(row_ptr_dev, col_idx_dev, vals_dev, Cout, Cin, kernel, V, options, (hipStream_t)stream, out);
    const LayerIn in{nullptr, nullptr, row_ptr_dev, col_idx_dev, vals_dev, Cout, Cin, kernel, V, options};
    return build_all(&in, 1, nullptr, 0, (hipStream_t)stream, out);
}

extern "C" int alcs_pack_weights_device(const float *W_dev, const uint8_t *mask_dev, int Cout, int Cin, int kernel, int V,
                                        const alcs_options *options, void *stream, alcs_packed_t **out) {
    if (out) *out = nullptr;
    if (!W_dev || !out) return ALCS_E_INVALID_ARG;
    if (check_shape(Cout, Cin, kernel, V) == ALCS_OK && too_many_groups(Cout, V)) {
        // the storage format on the device, then through the host
        const int G = (Cout + V - 1) / V;
        const long long cap = (long long)G * Cin * kernel * kernel;
        const size_t o_ci = align256(4 * (size_t)(G + 1)), o_va = align256(o_ci + 4 * (size_t)cap);
        void *tmp = nullptr;
        int rc = check(hipMalloc(&tmp, o_va + 4 * (size_t)cap * V));
        if (rc != ALCS_OK) return rc;
        char *tb = (char *)tmp;
        rc = alcs_pack_csr_device(W_dev, mask_dev, Cout, Cin, kernel, V, (int32_t *)tb, (int32_t *)(tb + o_ci),
                                  (float *)(tb + o_va), cap, nullptr, stream);
        if (rc == ALCS_OK)
            rc = through_the_host((const int32_t *)tb, (const int32_t *)(tb + o_ci), (const float *)(tb + o_va), Cout, Cin,
                                  kernel, V, options, (hipStream_t)stream, out);
        (void)hipFree(tmp);
        return rc;
    }
    const LayerIn in{W_dev, mask_dev, nullptr, nullptr, nullptr, Cout, Cin, kernel, V, options};
    return build_all(&in, 1, nullptr, 0, (hipStream_t)stream, out);
}

extern "C" long long alcs_pack_workspace_bytes(const alcs_layer_desc *layers, int n_layers) {
    if (!layers || n_layers <= 0) return ALCS_E_INVALID_ARG;
    size_t need = align256(8 * sizeof(int) * (size_t)n_layers);
    for (int i = 0; i < n_layers; ++i) {
        const alcs_layer_desc &d = layers[i];
        int rc = check_shape(d.Cout, d.Cin, d.kernel, d.V);
        if (rc == ALCS_OK && too_many_groups(d.Cout, d.V)) rc = ALCS_E_UNSUPPORTED;
        if (rc == ALCS_OK && d.options) rc = check_options(d.options);
        if (rc != ALCS_OK) return rc;
        need += carve(nullptr, nullptr, d.Cout, d.Cin, d.kernel, d.V, d.options, true);
    }
    return (long long)need;
}

extern "C" int alcs_pack_network_device(const alcs_layer_desc *layers, int n_layers, void *workspace_dev,
                                        long long workspace_bytes, void *stream, alcs_packed_t **out) {
    if (!layers || n_layers <= 0 || !out || workspace_bytes < 0) return ALCS_E_INVALID_ARG;
    std::vector<LayerIn> in;
    try {
        in.reserve((size_t)n_layers);
    } catch (const std::bad_alloc &) {
        return ALCS_E_ALLOC;
    }
    for (int i = 0; i < n_layers; ++i) {
        out[i] = nullptr;
        const alcs_layer_desc &d = layers[i];
        if (!d.W_dev) return ALCS_E_INVALID_ARG;
        in.push_back(LayerIn{d.W_dev, d.mask_dev, nullptr, nullptr, nullptr, d.Cout, d.Cin, d.kernel, d.V, d.options});
    }
    return build_all(in.data(), n_layers, workspace_dev, (size_t)workspace_bytes, (hipStream_t)stream, out);
}
