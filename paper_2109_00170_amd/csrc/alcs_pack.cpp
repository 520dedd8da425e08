// Host side of the library: argument checks, the canonical grouped CSR of
// Section 3.2.2 ("Storage format") of arXiv 2109.00170, the padded and segmented
// layout the kernels read, its self-check, and the upload to the device.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <new>
#include <numeric>

#include "alcs_internal.h"

namespace alcs {

static thread_local int g_last_hip = 0;
static thread_local int g_last_launch[10] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
void set_hip_error(int e) { g_last_hip = e; }

void record_launch(int mode, int pv, int waves, int wgs, int lds, int gtiles, int kc, int path, int gs,
                   int tile_w) {
    int v[10] = {mode, pv, waves, wgs, lds, gtiles, kc, path, gs, tile_w};
    std::memcpy(g_last_launch, v, sizeof(v));
}

void device_shape(int device, int *cus, int *xcds) {
    constexpr int kMax = 64;
    static std::atomic<int> known[kMax];  // 0 = not looked up yet, else cus << 8 | xcds
    int packed = (device >= 0 && device < kMax) ? known[device].load(std::memory_order_relaxed) : 0;
    if (!packed) {
        int c = 0, x = 0;
        if (hipDeviceGetAttribute(&c, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || c <= 0) c = 256;
        if (hipDeviceGetAttribute(&x, hipDeviceAttributeNumberOfXccs, device) != hipSuccess || x <= 0 || x > 255) x = 8;
        (void)hipGetLastError();
        packed = c << 8 | x;
        if (device >= 0 && device < kMax) known[device].store(packed, std::memory_order_relaxed);
    }
    *cus = packed >> 8;
    *xcds = packed & 255;
}

int current_device_shape(int *cus, int *xcds) {
    int dev = 0;
    const hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { set_hip_error((int)e); return ALCS_E_HIP; }
    device_shape(dev, cus, xcds);
    return ALCS_OK;
}

static inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// Channel of a canonical column index.
static inline int col_channel(int col, int kk) { return col / kk; }

static inline int32_t off_of(int col, int k, int table, int GS) { return layout_off_of(col, k, table, GS); }
static inline int32_t pad_off(int c0, int KC, int k, int table, int GS, int which = 0) {
    return layout_pad_off(c0, KC, k, table, GS, which);
}
static inline size_t w_index(const Layout &L, int64_t col, int s, int i) { return layout_w_index(L.GS, L.VV, col, s, i); }
static inline size_t off_index(const Layout &L, int64_t col, int s) { return layout_off_index(L.GS, col, s); }

// Order of one slot's columns inside a bundle segment of L columns (several groups per wavefront).
// The 16- or 32-lane slots of a wavefront read different LDS rows in the same instruction; with
// rows of 128 bytes, rows of equal channel parity lie on the same half of the 64 LDS banks, so two
// slots that are served together (slots 0/1 and 2/3) conflict whenever their rows' parities agree.
// The accumulation order inside a group is free, so the even slot of a pair takes its
// even-channel columns from the front and its odd-channel ones right-aligned at the back, the odd
// slot the other way round, and padding sits in between; the pair then disagrees in parity at
// every step unless their like-parity columns together outnumber L.  place[j] is the index of the
// column (counted inside the group's chunk range) at step j, or -1 for padding.
static void arrange_slot(const int32_t *cols, int n, int kk, int L, bool evens_first, std::vector<int32_t> &place) {
    place.assign((size_t)L, -1);
    int front = 0, nback = 0;
    for (int i = 0; i < n; ++i) nback += ((col_channel(cols[i], kk) & 1) == (evens_first ? 1 : 0));
    int back = L - nback;
    for (int i = 0; i < n; ++i) {
        const bool to_back = (col_channel(cols[i], kk) & 1) == (evens_first ? 1 : 0);
        place[(size_t)(to_back ? back++ : front++)] = i;
    }
}

int build_layout(alcs_packed *p, int KC, int GS) {
    Layout &L = p->lay;
    const int k = p->k, kk = k * k, V = p->V, G = p->G;
    L = Layout();
    L.KC = KC;
    L.nchunks = (p->Cin + KC - 1) / KC;
    L.GS = GS;
    L.nbundles = (G + GS - 1) / GS;
    L.planes = V >= 4 ? V / 4 : 1;
    L.VV = V >= 4 ? 4 : V;
    L.noff = k == 1 ? 1 : kMaxOff;
    if (GS != 1 && (GS != 2 && GS != 4)) return ALCS_E_INVALID_ARG;
    if (GS > 1 && (V < 4 || k != 1 || L.nchunks != 1)) return ALCS_E_INVALID_ARG;
    try {
        L.order.resize(G);
        std::iota(L.order.begin(), L.order.end(), 0);
        std::stable_sort(L.order.begin(), L.order.end(), [&](int a, int b) {
            return p->row_ptr[a + 1] - p->row_ptr[a] > p->row_ptr[b + 1] - p->row_ptr[b];
        });
        // tap-shared pattern: the kept columns of every group come as whole channels, nine taps each
        if (k == 3 && p->nnzb > 0) {
            bool shared = p->nnzb % 9 == 0;
            for (int g = 0; g < G && shared; ++g) {
                const int32_t b = p->row_ptr[g], e = p->row_ptr[g + 1];
                shared = (e - b) % 9 == 0;
                for (int32_t t = b; t < e && shared; ++t)
                    shared = (t - b) % 9 == 0 ? p->col_idx[t] % 9 == 0 : p->col_idx[t] == p->col_idx[t - 1] + 1;
            }
            L.tap_shared = shared;
        }
        // canonical range [lo, hi) of every (group, chunk)
        std::vector<int32_t> lo((size_t)G * L.nchunks), hi((size_t)G * L.nchunks);
        for (int g = 0; g < G; ++g) {
            int32_t t = p->row_ptr[g], end = p->row_ptr[g + 1];
            for (int ch = 0; ch < L.nchunks; ++ch) {
                const int c_end = std::min(p->Cin, (ch + 1) * KC);
                lo[(size_t)g * L.nchunks + ch] = t;
                while (t < end && col_channel(p->col_idx[t], kk) < c_end) ++t;
                hi[(size_t)g * L.nchunks + ch] = t;
            }
        }
        // pass 1: segments
        L.work.assign((size_t)L.nbundles * L.nchunks, Work{0, 0, {-1, -1, -1, -1}, {0, 0}});
        int64_t cur = 0;
        for (int b = 0; b < L.nbundles; ++b)
            for (int ch = 0; ch < L.nchunks; ++ch) {
                Work &wk = L.work[(size_t)b * L.nchunks + ch];
                int32_t longest = 0;
                for (int s = 0; s < GS; ++s) {
                    const int pos = b * GS + s;
                    if (pos >= G) continue;
                    const int g = L.order[pos];
                    wk.group[s] = g;
                    const size_t gi = (size_t)g * L.nchunks + ch;
                    longest = std::max(longest, hi[gi] - lo[gi]);
                }
                if (cur > INT32_MAX / (4 * GS) - 64) return ALCS_E_UNSUPPORTED;
                wk.start = (int32_t)cur;
                wk.cnt = (int32_t)round_up(longest, kCntAlign);
                L.max_cnt = std::max(L.max_cnt, (int)wk.cnt);
                cur += round_up(wk.cnt, kSegAlign);
            }
        L.ncol = cur + kSegAlign;  // one spare run so that a read-ahead stays inside the arrays
        L.wplane = L.ncol * L.VV * GS;
        L.w.assign((size_t)L.planes * L.wplane, 0.0f);
        for (int tb = 0; tb < L.noff; ++tb) L.off[tb].assign((size_t)L.ncol * GS, 0);
        // pass 2: fill (padding: zero weights, selector of an all-zero row of the chunk)
        std::vector<int32_t> place[kMaxSlots];
        for (int b = 0; b < L.nbundles; ++b)
            for (int ch = 0; ch < L.nchunks; ++ch) {
                const Work wk = L.work[(size_t)b * L.nchunks + ch];
                const int c0 = ch * KC;
                const int64_t span = round_up(wk.cnt, kSegAlign);
                for (int s = 0; s < GS; ++s) {
                    const int g = wk.group[s];
                    const size_t gi = g >= 0 ? (size_t)g * L.nchunks + ch : 0;
                    const int32_t nreal = g >= 0 ? hi[gi] - lo[gi] : 0;
                    if (GS > 1) {
                        arrange_slot(nreal ? &p->col_idx[lo[gi]] : nullptr, nreal, kk, wk.cnt, (s & 1) == 0, place[s]);
                    } else {
                        place[s].assign((size_t)wk.cnt, -1);
                        for (int32_t j = 0; j < nreal; ++j) place[s][(size_t)j] = j;
                    }
                }
                for (int s = 0; s < GS; ++s) {
                    const int g = wk.group[s];
                    const size_t gi = g >= 0 ? (size_t)g * L.nchunks + ch : 0;
                    for (int64_t j = 0; j < span; ++j) {
                        const int64_t col = wk.start + j;
                        const int32_t at = j < wk.cnt ? place[s][(size_t)j] : -1;
                        if (at < 0) {
                            // padding: the zero row whose parity differs from the partner slot's row
                            // at this step (the partner's own padding takes the other zero row)
                            int which = 0;
                            if (GS > 1 && j < wk.cnt) {
                                const int m = s ^ 1;
                                const int32_t mate = m < GS && wk.group[m] >= 0 ? place[m][(size_t)j] : -1;
                                if (mate >= 0) {
                                    const size_t mi = (size_t)wk.group[m] * L.nchunks + ch;
                                    const int parity = col_channel(p->col_idx[lo[mi] + mate], kk) & 1;
                                    which = ((c0 + KC) & 1) == parity ? 1 : 0;
                                } else {
                                    which = s & 1;
                                }
                            }
                            for (int tb = 0; tb < L.noff; ++tb) L.off[tb][off_index(L, col, s)] = pad_off(c0, KC, k, tb, GS, which);
                            continue;
                        }
                        for (int tb = 0; tb < L.noff; ++tb)
                            L.off[tb][off_index(L, col, s)] = off_of(p->col_idx[lo[gi] + at], k, tb, GS);
                        const float *src = &p->vals[(size_t)(lo[gi] + at) * V];
                        for (int v = 0; v < V; ++v) {
                            const int q = V < 4 ? 0 : v / 4, i = V < 4 ? v : v % 4;
                            L.w[(size_t)q * L.wplane + w_index(L, col, s, i)] = src[v];
                        }
                    }
                }
            }
        for (int64_t col = cur; col < L.ncol; ++col)
            for (int s = 0; s < GS; ++s)
                for (int tb = 0; tb < L.noff; ++tb) L.off[tb][off_index(L, col, s)] = pad_off(0, KC, k, tb, GS);
    } catch (const std::bad_alloc &) {
        return ALCS_E_ALLOC;
    }
    return ALCS_OK;
}

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

void release_device(alcs_packed *p) {
    if (p->dev.blob) {
        int cur = -1;
        const bool elsewhere = hipGetDevice(&cur) == hipSuccess && cur != p->dev.device;
        if (elsewhere) (void)hipSetDevice(p->dev.device);
        (void)hipFree(p->dev.blob);
        if (p->dev.w16) (void)hipFree(const_cast<uint16_t *>(p->dev.w16));
        if (p->dev.chan_blob) (void)hipFree(p->dev.chan_blob);
        if (elsewhere) (void)hipSetDevice(cur);
    }
    p->dev = DeviceCopy();
}

int upload(alcs_packed *p) {
    const Layout &L = p->lay;
    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess || ndev <= 0) {
        (void)hipGetLastError();
        return ALCS_E_NO_DEVICE;
    }
    int dev = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) { set_hip_error((int)e); return ALCS_E_HIP; }
    const size_t b_work = L.work.size() * sizeof(Work);
    const size_t b_w = L.w.size() * sizeof(float);
    const size_t b_off = L.off[0].size() * sizeof(int32_t);
    size_t o_work = 0, o_w = align256(o_work + b_work), o_off[kMaxOff];
    size_t total = align256(o_w + b_w);
    for (int t = 0; t < L.noff; ++t) {
        o_off[t] = total;
        total = align256(total + b_off);
    }
    total += 256;
    void *blob = nullptr;
    if ((e = hipMalloc(&blob, total)) != hipSuccess) {
        set_hip_error((int)e);
        (void)hipGetLastError();
        return e == hipErrorOutOfMemory ? ALCS_E_ALLOC : ALCS_E_HIP;
    }
    char *base = (char *)blob;
    auto put = [&](size_t o, const void *src, size_t n) -> hipError_t {
        return n ? hipMemcpy(base + o, src, n, hipMemcpyHostToDevice) : hipSuccess;
    };
    e = put(o_work, L.work.data(), b_work);
    if (e == hipSuccess) e = put(o_w, L.w.data(), b_w);
    for (int t = 0; t < L.noff && e == hipSuccess; ++t) e = put(o_off[t], L.off[t].data(), b_off);
    if (e != hipSuccess) {
        set_hip_error((int)e);
        (void)hipFree(blob);
        return ALCS_E_HIP;
    }
    int cus = 0, xcds = 0;
    device_shape(dev, &cus, &xcds);
    p->dev.device = dev;
    p->dev.cus = cus;
    p->dev.xcds = xcds;
    p->dev.blob = blob;
    p->dev.bytes = total;
    p->dev.work = (const Work *)(base + o_work);
    p->dev.w = (const float *)(base + o_w);
    for (int t = 0; t < kMaxOff; ++t) p->dev.off[t] = t < L.noff ? (const int32_t *)(base + o_off[t]) : nullptr;
    if (L.tap_shared) {
        const int rc = add_channel_records(p, nullptr);
        if (rc == ALCS_OK && (e = hipStreamSynchronize(nullptr)) != hipSuccess) { set_hip_error((int)e); return ALCS_E_HIP; }
        return rc;  // on failure the caller frees the handle and with it the device memory
    }
    return ALCS_OK;
}

// Tile policy for kernel 1.  One group per wavefront and all input channels in one
// LDS tile while a 64-pixel tile of Cin+1 rows fits (Cin <= 639 in 160 KB); from 512
// input channels on (V >= 4 only) the tile shrinks to 32 or 16 pixels and a wavefront
// multiplies 2 or 4 groups: two workgroups then share a compute unit and one fills its
// tile while the other multiplies (512 channels: 512->1024 @7x7 16.9 -> 11.0 us).
// Up to 1279 channels, V = 4 or 8 and groups of similar length (the longest at most twice the
// mean) take 4 groups per wavefront, each on 16 lanes that hold two pixels of the 32-pixel
// tile, which halves the LDS row reads per kept weight (512->512 @14x14: 17.2 us with one
// group per wavefront, 17.1 with two, 15.6 with four; 512->128 @28x28, N=64: 58 -> 43 us).
// With groups of very different lengths a workgroup's time is the walk through its longest
// bundle, which two pixels per lane make 1.5x longer (576->96 @14x14, longest group 6x the
// mean: 39 us with two groups per wavefront, 45 with four).  V = 8 takes four as well (512->1024
// @7x7, N=32: 12.9 -> 10.0 us, 1024->1024 @7x7: 19.4 -> 15.4, 512->512 @14x14 unchanged); V = 16
// does not (512->512 @14x14: 15 us with two, 22 with four - 32 accumulator registers per pixel
// pair).  With 256 input channels one group per wavefront stays ahead.
// Beyond 2558 channels, or beyond 639 for V < 4, chunks of 256 channels.
// Kernel 3: 32 channels per chunk (the haloed tile plane is 240 to 476 floats per channel);
// 64 from 512 input channels on - such layers sit on 14x14 and 7x7 images, where a workgroup's
// time is the chain of its chunks' round trips (512->512 @7x7, N=64: 131 -> 100 us; stride 2
// from 14x14: 141 -> 131 us), while on large images the smaller chunk's higher occupancy wins
// (128->128 stride 2 @56x56: 104 us with 32 channels, 148 us with 64).
static void default_tiles(int Cin, int k, int V, bool even_groups, int *KC, int *GS) {
    *GS = 1;
    if (k == 3) { *KC = Cin >= 512 ? 64 : std::min(Cin, 32); return; }
    if (V >= 4 && Cin >= 512 && Cin <= 2558) {
        *KC = Cin;
        *GS = (Cin > 1279 || (V <= 8 && even_groups)) ? 4 : 2;
        return;
    }
    if (Cin <= 639) { *KC = Cin; return; }
    *KC = 256;
}

void choose_tiles(const alcs_packed *p, int *KC, int *GS) {
    const bool even_groups = (int64_t)p->max_count * p->G <= 2 * p->nnzb;
    default_tiles(p->Cin, p->k, p->V, even_groups, KC, GS);
    const int kc = p->opt.chunk_channels, gs = p->opt.group_slots;
    if (kc > 0) { *KC = std::min(kc, p->Cin); *GS = 1; }
    if ((gs == 1 || gs == 2 || gs == 4) && p->k == 1 && p->V >= 4 && *KC == p->Cin &&
        (long long)(p->Cin + (gs > 1 ? 2 : 1)) * (kRowBytes1 / gs) <= 160 * 1024)
        *GS = gs;
}

// A handle built on the device keeps its arrays there; export and self-check work on host
// copies, fetched on first use (blocking copies on the null stream).
int fetch_host_arrays(alcs_packed *p) {
    std::lock_guard<std::mutex> lock(p->host_mu);
    if (p->host_arrays) return ALCS_OK;
    if (!p->dev.blob || !p->dev.row_ptr) return ALCS_E_NO_DEVICE;
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) { set_hip_error((int)e); return ALCS_E_HIP; }
    if (cur != p->dev.device && (e = hipSetDevice(p->dev.device)) != hipSuccess) { set_hip_error((int)e); return ALCS_E_HIP; }
    Layout &L = p->lay;
    try {
        p->row_ptr.resize((size_t)p->G + 1);
        p->col_idx.resize((size_t)p->nnzb);
        p->vals.resize((size_t)p->nnzb * p->V);
        L.order.resize((size_t)p->G);
        L.work.resize((size_t)L.nbundles * L.nchunks);
        L.w.resize((size_t)L.planes * L.wplane);
        for (int t = 0; t < L.noff; ++t) L.off[t].resize((size_t)L.ncol * L.GS);
    } catch (const std::bad_alloc &) {
        if (cur != p->dev.device) (void)hipSetDevice(cur);
        return ALCS_E_ALLOC;
    }
    auto get = [&](void *dst, const void *src, size_t n) { return n ? hipMemcpy(dst, src, n, hipMemcpyDeviceToHost) : hipSuccess; };
    e = get(p->row_ptr.data(), p->dev.row_ptr, p->row_ptr.size() * 4);
    if (e == hipSuccess) e = get(p->col_idx.data(), p->dev.col_idx, p->col_idx.size() * 4);
    if (e == hipSuccess) e = get(p->vals.data(), p->dev.vals, p->vals.size() * 4);
    if (e == hipSuccess) e = get(L.order.data(), p->dev.order, L.order.size() * 4);
    if (e == hipSuccess) e = get(L.work.data(), p->dev.work, L.work.size() * sizeof(Work));
    if (e == hipSuccess) e = get(L.w.data(), p->dev.w, L.w.size() * 4);
    for (int t = 0; t < L.noff && e == hipSuccess; ++t) e = get(L.off[t].data(), p->dev.off[t], L.off[t].size() * 4);
    if (cur != p->dev.device) (void)hipSetDevice(cur);
    if (e != hipSuccess) { set_hip_error((int)e); return ALCS_E_HIP; }
    p->host_arrays = true;
    return ALCS_OK;
}

// Options are plain non-negative ints; the phase-skipping field is honoured by the measurement
// build only and refused by the product build.
int check_options(const alcs_options *o) {
    const int *f = reinterpret_cast<const int *>(o);
    for (size_t i = 0; i < sizeof(alcs_options) / sizeof(int); ++i)
        if (f[i] < 0) return ALCS_E_INVALID_ARG;
#if !defined(ALCS_MEASURE) || !ALCS_MEASURE
    if (o->measure_skip != 0) return ALCS_E_INVALID_ARG;
#endif
    for (int r : o->reserved)
        if (r != 0) return ALCS_E_INVALID_ARG;
    return ALCS_OK;
}

}  // namespace alcs

using namespace alcs;

extern "C" void alcs_packed_free(alcs_packed_t *p);

// The tuned device layout and its upload, once the canonical arrays of the handle are in place.
static int finish_pack(alcs_packed *p, int rc, const alcs_options *opt, alcs_packed_t **out) {
    if (rc == ALCS_OK && opt) rc = check_options(opt);
    if (rc == ALCS_OK) {
        if (opt) p->opt = *opt;
        int KC = 0, GS = 1;
        choose_tiles(p, &KC, &GS);
        rc = build_layout(p, KC, GS);
    }
    if (rc == ALCS_OK) {
        rc = upload(p);
        if (rc == ALCS_E_NO_DEVICE) rc = ALCS_OK;  // host-only handle
    }
    if (rc != ALCS_OK) {
        alcs_packed_free(p);
        return rc;
    }
    *out = p;
    return ALCS_OK;
}

extern "C" {

const char *alcs_strerror(int status) {
    switch (status) {
        case ALCS_OK: return "ALCS_OK";
        case ALCS_E_INVALID_ARG: return "ALCS_E_INVALID_ARG: bad pointer, size or shape";
        case ALCS_E_UNSUPPORTED: return "ALCS_E_UNSUPPORTED: kernel/V/stride/size outside the supported set";
        case ALCS_E_ALLOC: return "ALCS_E_ALLOC: allocation failed";
        case ALCS_E_HIP: return "ALCS_E_HIP: HIP runtime call failed";
        case ALCS_E_NO_DEVICE: return "ALCS_E_NO_DEVICE: handle has no device copy";
        default: return "ALCS: unknown status";
    }
}

int alcs_last_hip_error(void) { return g_last_hip; }

int alcs_version(void) { return 100; }

int alcs_pack_weights(const float *W_host, const uint8_t *mask_host, int Cout, int Cin, int kernel,
                      int V, alcs_packed_t **out) {
    return alcs_pack_weights_opt(W_host, mask_host, Cout, Cin, kernel, V, nullptr, out);
}

int alcs_pack_weights_opt(const float *W_host, const uint8_t *mask_host, int Cout, int Cin, int kernel,
                          int V, const alcs_options *options, alcs_packed_t **out) {
    if (out) *out = nullptr;
    if (!W_host || !out || Cout <= 0 || Cin <= 0) return ALCS_E_INVALID_ARG;
    if (kernel != 1 && kernel != 3) return ALCS_E_UNSUPPORTED;
    if (V != 1 && V != 2 && V != 4 && V != 8 && V != 16) return ALCS_E_UNSUPPORTED;
    const int64_t K64 = (int64_t)Cin * kernel * kernel;
    if (K64 > (1 << 24) || Cout > (1 << 24)) return ALCS_E_UNSUPPORTED;
    const int K = (int)K64, G = (Cout + V - 1) / V;
    if ((int64_t)G * K > (int64_t)INT32_MAX - 1024) return ALCS_E_UNSUPPORTED;
    alcs_packed *p = new (std::nothrow) alcs_packed();
    if (!p) return ALCS_E_ALLOC;
    p->Cout = Cout; p->Cin = Cin; p->k = kernel; p->V = V; p->G = G; p->K = K;
    int rc = ALCS_OK;
    try {
        // canonical grouped CSR: per group, ascending column, one V-vector per kept column
        p->row_ptr.assign((size_t)G + 1, 0);
        int64_t nnzb = 0;
        if (mask_host) {
            for (int g = 0; g < G; ++g) {
                const uint8_t *m = mask_host + (size_t)g * K;
                int64_t c = 0;
                for (int col = 0; col < K; ++col) c += m[col] != 0;
                nnzb += c;
                p->row_ptr[g + 1] = (int32_t)nnzb;
            }
        } else {
            for (int g = 0; g < G; ++g) p->row_ptr[g + 1] = (int32_t)((int64_t)(g + 1) * K);
            nnzb = (int64_t)G * K;
        }
        p->nnzb = nnzb;
        p->col_idx.resize((size_t)nnzb);
        p->vals.resize((size_t)nnzb * V);
        for (int g = 0; g < G; ++g) {
            const uint8_t *m = mask_host ? mask_host + (size_t)g * K : nullptr;
            int64_t t = p->row_ptr[g];
            for (int col = 0; col < K; ++col) {
                if (m && !m[col]) continue;
                p->col_idx[(size_t)t] = col;
                for (int v = 0; v < V; ++v) {
                    const int o = g * V + v;
                    float x = 0.0f;
                    if (o < Cout) std::memcpy(&x, &W_host[(size_t)o * K + col], sizeof(float));
                    std::memcpy(&p->vals[(size_t)t * V + v], &x, sizeof(float));
                }
                ++t;
            }
            p->max_count = std::max(p->max_count, p->row_ptr[g + 1] - p->row_ptr[g]);
        }
    } catch (const std::bad_alloc &) {
        rc = ALCS_E_ALLOC;
    }
    return finish_pack(p, rc, options, out);
}

int alcs_pack_from_csr(const int32_t *row_ptr_host, const int32_t *col_idx_host, const float *vals_host,
                       int Cout, int Cin, int kernel, int V, alcs_packed_t **out) {
    return alcs::pack_from_csr_host(row_ptr_host, col_idx_host, vals_host, Cout, Cin, kernel, V, nullptr, out);
}

}  // extern "C"

int alcs::pack_from_csr_host(const int32_t *row_ptr_host, const int32_t *col_idx_host, const float *vals_host,
                             int Cout, int Cin, int kernel, int V, const alcs_options *options, alcs_packed_t **out) {
    if (out) *out = nullptr;
    if (!row_ptr_host || !out || Cout <= 0 || Cin <= 0) return ALCS_E_INVALID_ARG;
    if (kernel != 1 && kernel != 3) return ALCS_E_UNSUPPORTED;
    if (V != 1 && V != 2 && V != 4 && V != 8 && V != 16) return ALCS_E_UNSUPPORTED;
    const int64_t K64 = (int64_t)Cin * kernel * kernel;
    if (K64 > (1 << 24) || Cout > (1 << 24)) return ALCS_E_UNSUPPORTED;
    const int K = (int)K64, G = (Cout + V - 1) / V;
    if ((int64_t)G * K > (int64_t)INT32_MAX - 1024) return ALCS_E_UNSUPPORTED;
    // the arrays must be the canonical form: counts add up, columns ascend inside a group
    if (row_ptr_host[0] != 0) return ALCS_E_INVALID_ARG;
    for (int g = 0; g < G; ++g) {
        const int64_t lo = row_ptr_host[g], hi = row_ptr_host[g + 1];
        if (hi < lo || hi - lo > K) return ALCS_E_INVALID_ARG;
    }
    const int64_t nnzb = row_ptr_host[G];
    if (nnzb > 0 && (!col_idx_host || !vals_host)) return ALCS_E_INVALID_ARG;
    for (int g = 0; g < G; ++g)
        for (int64_t t = row_ptr_host[g]; t < row_ptr_host[g + 1]; ++t) {
            const int32_t col = col_idx_host[t];
            if (col < 0 || col >= K || (t > row_ptr_host[g] && col <= col_idx_host[t - 1])) return ALCS_E_INVALID_ARG;
        }
    alcs_packed *p = new (std::nothrow) alcs_packed();
    if (!p) return ALCS_E_ALLOC;
    p->Cout = Cout; p->Cin = Cin; p->k = kernel; p->V = V; p->G = G; p->K = K;
    int rc = ALCS_OK;
    try {
        p->row_ptr.assign(row_ptr_host, row_ptr_host + G + 1);
        p->nnzb = nnzb;
        p->col_idx.assign(col_idx_host, col_idx_host + nnzb);
        p->vals.resize((size_t)nnzb * V);
        if (nnzb) std::memcpy(p->vals.data(), vals_host, (size_t)nnzb * V * sizeof(float));
        for (int g = 0; g < G; ++g) p->max_count = std::max(p->max_count, p->row_ptr[g + 1] - p->row_ptr[g]);
    } catch (const std::bad_alloc &) {
        rc = ALCS_E_ALLOC;
    }
    return finish_pack(p, rc, options, out);
}

extern "C" {

int alcs_packed_info(const alcs_packed_t *p, int *G, int *K, int64_t *nnzb) {
    if (!p) return ALCS_E_INVALID_ARG;
    if (G) *G = p->G;
    if (K) *K = p->K;
    if (nnzb) *nnzb = p->nnzb;
    return ALCS_OK;
}

int alcs_packed_on_device(const alcs_packed_t *p) {
    if (!p) return ALCS_E_INVALID_ARG;
    return p->dev.blob ? 1 : 0;
}

int alcs_packed_export(const alcs_packed_t *p, int32_t *row_ptr_host, int32_t *col_idx_host,
                       float *vals_host) {
    if (!p || !row_ptr_host) return ALCS_E_INVALID_ARG;
    if (p->nnzb > 0 && (!col_idx_host || !vals_host)) return ALCS_E_INVALID_ARG;
    if (!p->host_arrays) {
        const int rc = fetch_host_arrays(const_cast<alcs_packed_t *>(p));
        if (rc != ALCS_OK) return rc;
    }
    std::memcpy(row_ptr_host, p->row_ptr.data(), p->row_ptr.size() * sizeof(int32_t));
    if (p->nnzb > 0) {
        std::memcpy(col_idx_host, p->col_idx.data(), p->col_idx.size() * sizeof(int32_t));
        std::memcpy(vals_host, p->vals.data(), p->vals.size() * sizeof(float));
    }
    return ALCS_OK;
}

int alcs_packed_selfcheck(const alcs_packed_t *p) {
    if (!p) return ALCS_E_INVALID_ARG;
    if (!p->host_arrays) {
        // built on the device: what is checked is the layout the device built, fetched as it is
        const int rc = fetch_host_arrays(const_cast<alcs_packed_t *>(p));
        if (rc != ALCS_OK) return rc;
    }
    const Layout &L = p->lay;
    const int k = p->k, V = p->V, GS = L.GS;
    if (L.KC <= 0 || L.nchunks != (p->Cin + L.KC - 1) / L.KC) return ALCS_E_INVALID_ARG;
    if (GS != 1 && GS != 2 && GS != 4) return ALCS_E_INVALID_ARG;
    if (L.nbundles != (p->G + GS - 1) / GS || (int)L.order.size() != p->G) return ALCS_E_INVALID_ARG;
    if ((int64_t)L.work.size() != (int64_t)L.nbundles * L.nchunks) return ALCS_E_INVALID_ARG;
    if ((int64_t)L.w.size() != L.planes * L.wplane || L.wplane != L.ncol * L.VV * GS) return ALCS_E_INVALID_ARG;
    // `order` is a permutation of the groups by descending length
    std::vector<char> seen((size_t)p->G, 0);
    for (int i = 0; i < p->G; ++i) {
        int g = L.order[i];
        if (g < 0 || g >= p->G || seen[g]) return ALCS_E_INVALID_ARG;
        seen[g] = 1;
        if (i > 0) {
            int a = L.order[i - 1];
            if (p->row_ptr[a + 1] - p->row_ptr[a] < p->row_ptr[g + 1] - p->row_ptr[g]) return ALCS_E_INVALID_ARG;
        }
    }
    const uint32_t zero_bits = 0;
    std::vector<int64_t> next((size_t)p->G);  // next canonical block expected for every group
    std::vector<char> seen_block(GS > 1 ? (size_t)p->nnzb : 0, 0);  // several groups per wavefront: blocks found so far
    for (int g = 0; g < p->G; ++g) next[g] = p->row_ptr[g];
    for (int b = 0; b < L.nbundles; ++b)
        for (int ch = 0; ch < L.nchunks; ++ch) {
            const Work wk = L.work[(size_t)b * L.nchunks + ch];
            if (wk.start % kSegAlign || wk.cnt % kCntAlign || wk.cnt < 0) return ALCS_E_INVALID_ARG;
            const int c0 = ch * L.KC, c1 = std::min(p->Cin, c0 + L.KC);
            const int64_t span = round_up(wk.cnt, kSegAlign);
            if (wk.start + span > L.ncol) return ALCS_E_INVALID_ARG;
            int64_t longest = 0;
            for (int s = 0; s < kMaxSlots; ++s) {
                const int pos = b * GS + s;
                const int want = (s < GS && pos < p->G) ? L.order[pos] : -1;
                if (wk.group[s] != want) return ALCS_E_INVALID_ARG;
                if (s >= GS) continue;
                const int g = wk.group[s];
                bool in_pad = false;
                int64_t nreal = 0;
                for (int64_t j = 0; j < span; ++j) {
                    const int64_t col = wk.start + j;
                    const size_t oi = off_index(L, col, s);
                    if (oi >= L.off[0].size()) return ALCS_E_INVALID_ARG;
                    // padding selects an all-zero row (one of two with several groups per wavefront)
                    int which = -1;
                    if (L.off[0][oi] == pad_off(c0, L.KC, k, 0, GS, 0)) which = 0;
                    else if (GS > 1 && L.off[0][oi] == pad_off(c0, L.KC, k, 0, GS, 1)) which = 1;
                    const bool is_pad = which >= 0;
                    // one group per wavefront: real blocks come first, in canonical order; several:
                    // any order (see arrange_slot), every canonical block exactly once
                    if (GS == 1 && in_pad && !is_pad) return ALCS_E_INVALID_ARG;
                    in_pad = is_pad;
                    if (is_pad) {
                        for (int tb = 1; tb < L.noff; ++tb)
                            if (L.off[tb][oi] != pad_off(c0, L.KC, k, tb, GS, which)) return ALCS_E_INVALID_ARG;
                        for (int q = 0; q < L.planes; ++q)
                            for (int i = 0; i < L.VV; ++i)
                                if (std::memcmp(&L.w[(size_t)q * L.wplane + w_index(L, col, s, i)], &zero_bits, 4))
                                    return ALCS_E_INVALID_ARG;
                        continue;
                    }
                    if (g < 0 || j >= wk.cnt) return ALCS_E_INVALID_ARG;
                    // a real block: a canonical column of the slot's group (the next one with one group
                    // per wavefront), inside the chunk's channel range so that its LDS row exists
                    int64_t t = -1;
                    if (GS == 1) {
                        if (next[g] >= p->row_ptr[g + 1]) return ALCS_E_INVALID_ARG;
                        t = next[g];
                    } else {
                        // (1x1 only: the selector is the column times the row length)
                        const int32_t want_col = L.off[0][oi] / (kRowBytes1 / GS);
                        const int32_t *first = p->col_idx.data() + p->row_ptr[g], *last = p->col_idx.data() + p->row_ptr[g + 1];
                        const int32_t *it = std::lower_bound(first, last, want_col);
                        if (it == last || *it != want_col) return ALCS_E_INVALID_ARG;
                        t = it - p->col_idx.data();
                        if (seen_block[(size_t)t]) return ALCS_E_INVALID_ARG;
                        seen_block[(size_t)t] = 1;
                    }
                    const int cidx = p->col_idx[(size_t)t];
                    const int c = col_channel(cidx, k * k);
                    if (c < c0 || c >= c1) return ALCS_E_INVALID_ARG;
                    for (int tb = 0; tb < L.noff; ++tb)
                        if (L.off[tb][oi] != off_of(cidx, k, tb, GS)) return ALCS_E_INVALID_ARG;
                    for (int v = 0; v < V; ++v) {
                        const int q = V < 4 ? 0 : v / 4, i = V < 4 ? v : v % 4;
                        if (std::memcmp(&L.w[(size_t)q * L.wplane + w_index(L, col, s, i)],
                                        &p->vals[(size_t)t * V + v], 4))
                            return ALCS_E_INVALID_ARG;
                    }
                    ++next[g];
                    ++nreal;
                }
                longest = std::max(longest, nreal);
            }
            if (round_up(longest, kCntAlign) != wk.cnt) return ALCS_E_INVALID_ARG;
        }
    for (int g = 0; g < p->G; ++g)
        if (next[g] != p->row_ptr[g + 1]) return ALCS_E_INVALID_ARG;  // every canonical block was found
    return ALCS_OK;
}

int alcs_packed_layout_hash(const alcs_packed_t *p, unsigned long long *hash_out) {
    if (!p || !hash_out) return ALCS_E_INVALID_ARG;
    if (!p->host_arrays) {
        const int rc = fetch_host_arrays(const_cast<alcs_packed_t *>(p));
        if (rc != ALCS_OK) return rc;
    }
    // FNV-1a over the layout's scalars and arrays, in a fixed order
    unsigned long long h = 1469598103934665603ull;
    auto eat = [&](const void *data, size_t n) {
        const unsigned char *b = static_cast<const unsigned char *>(data);
        for (size_t i = 0; i < n; ++i) { h ^= b[i]; h *= 1099511628211ull; }
    };
    const Layout &L = p->lay;
    const int64_t scalars[] = {L.KC, L.nchunks, L.GS, L.nbundles, L.planes, L.VV, L.max_cnt, L.ncol, L.wplane, L.noff};
    eat(scalars, sizeof(scalars));
    eat(L.order.data(), L.order.size() * sizeof(int32_t));
    eat(L.work.data(), L.work.size() * sizeof(Work));
    eat(L.w.data(), L.w.size() * sizeof(float));
    for (int t = 0; t < L.noff; ++t) eat(L.off[t].data(), L.off[t].size() * sizeof(int32_t));
    *hash_out = h;
    return ALCS_OK;
}

void alcs_packed_free(alcs_packed_t *p) {
    if (!p) return;
    release_device(p);
    delete p;
}

int alcs_packed_set_options(alcs_packed_t *p, const alcs_options *options) {
    if (!p || !options) return ALCS_E_INVALID_ARG;
    const int rc = check_options(options);
    if (rc != ALCS_OK) return rc;
    // the layout is built: its fields keep the values it was built with
    alcs_options o = *options;
    o.chunk_channels = p->opt.chunk_channels;
    o.group_slots = p->opt.group_slots;
    p->opt = o;
    return ALCS_OK;
}

int alcs_packed_get_options(const alcs_packed_t *p, alcs_options *options) {
    if (!p || !options) return ALCS_E_INVALID_ARG;
    *options = p->opt;
    return ALCS_OK;
}

int alcs_last_launch(int *out, int cap) {
    if (!out || cap <= 0) return 0;
    int n = cap < 10 ? cap : 10;
    std::memcpy(out, g_last_launch, n * sizeof(int));
    return n;
}

}  // extern "C"
