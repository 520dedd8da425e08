// The multiplication of Section 3.2.2 of arXiv 2109.00170 ("Efficient multiplication
// computation") in 16-bit arithmetic: X, the residual and Y are bfloat16 tensors, the packed
// weights are rounded to bfloat16 once per handle (alcs_packed_add_bf16_weights), products are
// exact and sums float32 (the matrix instruction's accumulator), and Y is rounded to nearest even
// once, after bias, residual and activation.  Section 3.2.1 ties the group size V to the width
// of the machine's vector registers over the element width; on this GPU the unit that plays the
// register's part is the matrix instruction v_mfma_f32_4x4x4_16B_bf16, which multiplies, for
// each of 16 blocks of 4 lanes, a 4x4 tile of weights (4 output channels x 4 kept columns) with
// a 4x4 tile of inputs (4 kept columns x 4 pixels): one instruction covers 4 channels of a
// group, FOUR kept columns and 64 pixels - four times the float32 instruction's columns - and a
// group of V = 8 or 16 channels is 2 or 4 such instructions on the same input operand.
//
// Kernel (1x1 handles with one group per wavefront and all input channels in one tile):
//   - a workgroup stages a tile of 128 consecutive output pixels x Cin channels in LDS as
//     bfloat16, 256 bytes a row - the byte geometry of the float32 kernels' 64-pixel rows, so
//     the handle's row selectors are used as they are; the copy from HBM is straight, nothing
//     is converted;
//   - a lane owns two neighbouring pixels: one 4-byte LDS read per kept column fetches both, and
//     two byte permutes per column pair sort four columns' values into the two input operands;
//   - the weights of a run of 16 kept columns are 128 bytes per 4 channels: lane (b, i) of the
//     first 16 lanes holds channel i of columns 4b .. 4b+3, and the instruction's block
//     broadcast (cbsz = 4, abid = b) hands block b's weights to all 16 blocks;
//   - the epilogue writes two bfloat16 per lane and channel with one 4-byte non-temporal store.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <utility>

#include "alcs_internal.h"

namespace alcs {
namespace m16 {

typedef short s4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));

constexpr int kRowBytes = 256; // bytes per LDS row with two pixels per lane = kRowBytes1, the selectors' unit

struct Args {
    const uint16_t *X, *residual;
    uint16_t *Y;
    const float *bias;
    const Work *work;
    const uint16_t *w16;
    const int32_t *off;
    long long wplane16;  // 16-bit words between weight planes: padded columns * 4
    int N, Cin, Cout, H, W, Ho, Wo, stride;
    int P, Pin, NP;
    int G, ngt, gpt;
    int zero_rows;  // all-zero rows behind the Cin rows of the tile: 1, or 2 for handles with several groups per wavefront
    int tile_px;  // pixels of the flattened axis per workgroup (<= kTilePx, a multiple of 4)
    int wg_per_xcd, total_wgs, xcds;
    int act;
};

template <class T>
using cptr = const T __attribute__((address_space(4))) *;
typedef int i8v __attribute__((ext_vector_type(8)));

__device__ __forceinline__ Work load_work(const Work *table, size_t idx) {
    const i8v v = *reinterpret_cast<cptr<i8v>>((uintptr_t)(table + idx));
    Work w;
    w.start = __builtin_amdgcn_readfirstlane(v[0]);
    w.cnt = __builtin_amdgcn_readfirstlane(v[1]);
    w.group[0] = __builtin_amdgcn_readfirstlane(v[2]);
    w.group[1] = w.group[2] = w.group[3] = -1;
    w.reserved[0] = w.reserved[1] = 0;
    return w;
}

__device__ __forceinline__ unsigned int pack_bf2(float a, float b) {
    return __builtin_bit_cast(unsigned int, __builtin_convertvector(f2{a, b}, bf2));
}
__device__ __forceinline__ float widen(unsigned int bits16) { return __builtin_bit_cast(float, bits16 << 16); }

template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, Is...>) {
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// lane C of the lane's own row of 16, in every lane (DPP row_newbcast)
template <int C>
__device__ __forceinline__ int bcast_sel(int ov) {
    return __builtin_amdgcn_update_dpp(0, ov, 0x150 + C, 0xF, 0xF, false);
}

// The weights (V/4 operands of 4 bfloat16) and the 16 row selectors of one run of 16 columns.
template <int V>
struct Run {
    s4 a[V / 4];
    int o;
};
constexpr int kRunsAhead = 2;
template <int V>
struct Runs {
    Run<V> r[kRunsAhead];
};

template <int V>
__device__ __forceinline__ Run<V> load_run(const Args &a, int blk, int lane) {
    Run<V> r;
    const uint16_t *wp = a.w16 + (size_t)(blk >> 4) * 64 + (lane & 15) * 4;
#pragma unroll
    for (int q = 0; q < V / 4; ++q) r.a[q] = *reinterpret_cast<const s4 *>(wp + (size_t)q * a.wplane16);
    r.o = a.off[(size_t)blk + (lane & 15)];
    return r;
}
// The first runs of a segment; places beyond its last run re-read that run (the arrays end with a
// spare run, so run 0 of an empty segment exists).
template <int V>
__device__ __forceinline__ Runs<V> load_runs(const Args &a, int blk, int cnt, int lane) {
    Runs<V> rs;
    const int last = max(0, ((cnt + 15) & ~15) - 16);
#pragma unroll
    for (int i = 0; i < kRunsAhead; ++i) rs.r[i] = load_run<V>(a, blk + min(16 * i, last), lane);
    return rs;
}
template <int V>
__device__ __forceinline__ void touch_runs(Runs<V> &rs) {
#pragma unroll
    for (int i = 0; i < kRunsAhead; ++i) {
#pragma unroll
        for (int q = 0; q < V / 4; ++q) asm volatile("" : "+v"(rs.r[i].a[q]));
        asm volatile("" : "+v"(rs.r[i].o));
    }
}

// Partial sums: acc[k][q][pv][i] = channel 4q+i of the group, pixel pv of the lane; two partial
// sets (k) where a lane has a single chain per column quad (V = 4 with one pixel per lane).
template <int V, int PV>
struct Acc {
    static constexpr int NACC = (V / 4) * PV == 1 ? 2 : 1;
    f4 a[NACC][V / 4][PV];
    __device__ __forceinline__ void zero() {
#pragma unroll
        for (int k = 0; k < NACC; ++k)
#pragma unroll
            for (int q = 0; q < V / 4; ++q)
#pragma unroll
                for (int pv = 0; pv < PV; ++pv) a[k][q][pv] = f4{0.f, 0.f, 0.f, 0.f};
    }
    __device__ __forceinline__ float get(int q, int pv, int i) const {
        float s = a[0][q][pv][i];
        if constexpr (NACC == 2) s += a[1][q][pv][i];
        return s;
    }
};

// Columns B0 .. B0+7 of the current run: eight LDS reads, then per column quad the input operand(s)
// and V/4 * PV matrix instructions.  PV = 2: a 4-byte read fetches both pixels of the lane and two
// byte permutes per column pair sort the halves; PV = 1: 2-byte reads, one shift-or per column pair.
template <int B0, int V, int PV>
__device__ __forceinline__ void mfma_batch(const s4 (&aw)[V / 4], int ov, const char *lds, int base, Acc<V, PV> &acc) {
    unsigned int x[8];
    static_for<8>([&](auto c) {
        constexpr int C = decltype(c)::value;
        if constexpr (PV == 2) x[C] = *reinterpret_cast<const unsigned int *>(lds + base + bcast_sel<B0 + C>(ov));
        else x[C] = *reinterpret_cast<const uint16_t *>(lds + base + bcast_sel<B0 + C>(ov));
    });
    __builtin_amdgcn_sched_barrier(0);
    static_for<2>([&](auto kq) {
        constexpr int K4 = decltype(kq)::value;
        constexpr int ABID = B0 / 4 + K4;
        constexpr int K = ABID % Acc<V, PV>::NACC;
        // element k of an operand = column 4*ABID + k
        if constexpr (PV == 2) {
            // low halves are the lane's first pixel
            const unsigned int lo01 = __builtin_amdgcn_perm(x[4 * K4 + 1], x[4 * K4 + 0], 0x05040100u);
            const unsigned int lo23 = __builtin_amdgcn_perm(x[4 * K4 + 3], x[4 * K4 + 2], 0x05040100u);
            const unsigned int hi01 = __builtin_amdgcn_perm(x[4 * K4 + 1], x[4 * K4 + 0], 0x07060302u);
            const unsigned int hi23 = __builtin_amdgcn_perm(x[4 * K4 + 3], x[4 * K4 + 2], 0x07060302u);
            const s4 b0 = __builtin_bit_cast(s4, u2{lo01, lo23});
            const s4 b1 = __builtin_bit_cast(s4, u2{hi01, hi23});
#pragma unroll
            for (int q = 0; q < V / 4; ++q) {
                acc.a[K][q][0] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(aw[q], b0, acc.a[K][q][0], 4, ABID, 0);
                acc.a[K][q][1] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(aw[q], b1, acc.a[K][q][1], 4, ABID, 0);
            }
        } else {
            const s4 b0 = __builtin_bit_cast(s4, u2{x[4 * K4 + 0] | (x[4 * K4 + 1] << 16), x[4 * K4 + 2] | (x[4 * K4 + 3] << 16)});
#pragma unroll
            for (int q = 0; q < V / 4; ++q)
                acc.a[K][q][0] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(aw[q], b0, acc.a[K][q][0], 4, ABID, 0);
        }
    });
}

// One segment: the kept columns of one group (padded to a multiple of 8).  `rs` holds its first
// runs; longer segments re-fill register set i right after its use with the run two places on.
// The selectors are byte offsets for 256-byte rows; one pixel per lane has 128-byte rows.
template <int V, int PV>
__device__ __forceinline__ void mac_segment(const Args &a, int start, int cnt, const char *lds, int base, int lane,
                                            Runs<V> rs, Acc<V, PV> &acc) {
    auto pass = [&](int j0) {
        static_for<kRunsAhead>([&](auto ii) {
            constexpr int I = decltype(ii)::value;
            const int j = j0 + 16 * I;
            if (j < cnt) {
                const int ov = PV == 2 ? rs.r[I].o : rs.r[I].o >> 1;
                mfma_batch<0, V, PV>(rs.r[I].a, ov, lds, base, acc);
                if (j + 8 < cnt) mfma_batch<8, V, PV>(rs.r[I].a, ov, lds, base, acc);
                if (j + 16 * kRunsAhead < cnt) rs.r[I] = load_run<V>(a, start + j + 16 * kRunsAhead, lane);
            }
        });
    };
    pass(0);
    for (int j0 = 16 * kRunsAhead; j0 < cnt; j0 += 16 * kRunsAhead) pass(j0);
}

// The tile's rows (64 * PV pixels, 128 * PV bytes each) from HBM to LDS.  VEC: stride 1 and P a
// multiple of 4, so that four consecutive pixels of the flattened axis lie in one image and their 8
// bytes are aligned; with P a multiple of 8, eight pixels (16 bytes) per lane.
template <int PV, bool VEC>
__device__ __forceinline__ void stage(const Args &a, char *lds, int q0, int q_end) {
    constexpr int TP = 64 * PV, RB = 128 * PV;
    const int tid = threadIdx.x, nt = blockDim.x;
    if constexpr (VEC) {
        if ((a.P & 7) == 0) {
            typedef unsigned int u4 __attribute__((ext_vector_type(4)));
            constexpr int NO = TP / 8;
            const int oct = tid % NO, r0 = tid / NO, rpp = nt / NO;
            const int q = q0 + oct * 8;
            const bool valid = q < q_end;
            const int n = valid ? q / a.P : 0;
            const int p = valid ? q - n * a.P : 0;
            const uint16_t *src = a.X + ((size_t)n * a.Cin) * a.P + p;
            char *dst = lds + oct * 16;
            constexpr int U = 4;
            int r = r0;
            for (; r + (U - 1) * rpp < a.Cin; r += U * rpp) {
                u4 v[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    v[u] = u4{0u, 0u, 0u, 0u};
                    if (valid) v[u] = *reinterpret_cast<const u4 *>(src + (size_t)(r + u * rpp) * a.P);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) *reinterpret_cast<u4 *>(dst + (r + u * rpp) * RB) = v[u];
            }
            for (; r < a.Cin; r += rpp) {
                u4 v0 = u4{0u, 0u, 0u, 0u};
                if (valid) v0 = *reinterpret_cast<const u4 *>(src + (size_t)r * a.P);
                *reinterpret_cast<u4 *>(dst + r * RB) = v0;
            }
            return;
        }
        constexpr int NQ = TP / 4;
        const int quad = tid % NQ, r0 = tid / NQ, rpp = nt / NQ;
        const int q = q0 + quad * 4;
        const bool valid = q < q_end;
        const int n = valid ? q / a.P : 0;
        const int p = valid ? q - n * a.P : 0;
        const uint16_t *src = a.X + ((size_t)n * a.Cin) * a.P + p;
        char *dst = lds + quad * 8;
        constexpr int U = 8;
        int r = r0;
        for (; r + (U - 1) * rpp < a.Cin; r += U * rpp) {
            u2 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                v[u] = u2{0u, 0u};
                if (valid) v[u] = *reinterpret_cast<const u2 *>(src + (size_t)(r + u * rpp) * a.P);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) *reinterpret_cast<u2 *>(dst + (r + u * rpp) * RB) = v[u];
        }
        for (; r < a.Cin; r += rpp) {
            u2 v0 = u2{0u, 0u};
            if (valid) v0 = *reinterpret_cast<const u2 *>(src + (size_t)r * a.P);
            *reinterpret_cast<u2 *>(dst + r * RB) = v0;
        }
    } else {
        const int e = tid % TP, r0 = tid / TP, rpp = nt / TP;  // the launcher gives at least 128 threads
        const int q = q0 + e;
        const bool valid = q < q_end;
        const int n = valid ? q / a.P : 0;
        const int po = valid ? q - n * a.P : 0;
        const int ho = po / a.Wo, wo = po - ho * a.Wo;
        const uint16_t *src = a.X + ((size_t)n * a.Cin) * a.Pin + (size_t)(ho * a.stride) * a.W + wo * a.stride;
        uint16_t *dst = reinterpret_cast<uint16_t *>(lds) + e;
        constexpr int U = 8;
        int r = r0;
        for (; r + (U - 1) * rpp < a.Cin; r += U * rpp) {
            uint16_t v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = valid ? src[(size_t)(r + u * rpp) * a.Pin] : (uint16_t)0;
#pragma unroll
            for (int u = 0; u < U; ++u) dst[(r + u * rpp) * TP] = v[u];
        }
        for (; r < a.Cin; r += rpp) dst[r * TP] = valid ? src[(size_t)r * a.Pin] : (uint16_t)0;
    }
}

// Where the lane's pixel(s) go in Y (element offsets of channel 0), and whether they exist.
template <int PV>
struct PixOut {
    size_t o[PV];
    bool ok[PV];
};

template <int PV, bool VEC>
__device__ __forceinline__ PixOut<PV> pix_out(const Args &a, int q0, int lane, int q_end) {
    PixOut<PV> px;
    if constexpr (VEC && PV == 2) {
        const int q = q0 + 2 * lane;  // P is even: both pixels lie in one image
        px.ok[0] = px.ok[1] = q < q_end;
        const int n = px.ok[0] ? q / a.P : 0;
        px.o[0] = (size_t)n * a.Cout * a.P + (px.ok[0] ? q - n * a.P : 0);
        px.o[1] = px.o[0] + 1;
    } else {
#pragma unroll
        for (int pv = 0; pv < PV; ++pv) {
            const int q = q0 + PV * lane + pv;
            px.ok[pv] = q < q_end;
            const int n = px.ok[pv] ? q / a.P : 0;
            px.o[pv] = (size_t)n * a.Cout * a.P + (px.ok[pv] ? q - n * a.P : 0);
        }
    }
    return px;
}

__device__ __forceinline__ float activate(const Args &a, float v) {
    if (a.act >= 1) v = fmaxf(v, 0.f);
    if (a.act == 2) v = fminf(v, 6.f);
    return v;
}

template <int V, int PV, bool VEC>
__device__ __forceinline__ void store_group(const Args &a, const Acc<V, PV> &acc, int g, const PixOut<PV> &px) {
    const cptr<float> bias = (cptr<float>)(uintptr_t)a.bias;
#pragma unroll
    for (int q = 0; q < V / 4; ++q)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ch = g * V + 4 * q + i;  // wave-uniform
            if (ch >= a.Cout) continue;
            const float b = a.bias ? bias[ch] : 0.f;
            const size_t co = (size_t)ch * a.P;
            if constexpr (VEC && PV == 2) {
                if (!px.ok[0]) continue;
                float v0 = acc.get(q, 0, i) + b, v1 = acc.get(q, 1, i) + b;
                if (a.residual) {
                    const unsigned int r = *reinterpret_cast<const unsigned int *>(a.residual + px.o[0] + co);
                    v0 += widen(r & 0xffffu);
                    v1 += __builtin_bit_cast(float, r & 0xffff0000u);
                }
                __builtin_nontemporal_store(pack_bf2(activate(a, v0), activate(a, v1)),
                                            reinterpret_cast<unsigned int *>(a.Y + px.o[0] + co));
            } else {
#pragma unroll
                for (int pv = 0; pv < PV; ++pv) {
                    if (!px.ok[pv]) continue;
                    float v = acc.get(q, pv, i) + b;
                    if (a.residual) v += widen(a.residual[px.o[pv] + co]);
                    __builtin_nontemporal_store((uint16_t)(pack_bf2(activate(a, v), 0.f) & 0xffffu), a.Y + px.o[pv] + co);
                }
            }
        }
}

template <int V, int PV, bool VEC>
__global__ void __launch_bounds__(1024) k_pw16(const Args a) {
    extern __shared__ char lds[];
    constexpr int RB = 128 * PV;
    // consecutive logical ids share a pixel tile and land on the same XCD (L2)
    const int logical = ((int)blockIdx.x % a.xcds) * a.wg_per_xcd + (int)blockIdx.x / a.xcds;
    if (logical >= a.total_wgs) return;
    const int pt = logical / a.ngt, gt = logical - pt * a.ngt;
    // the workgroup's pixels [q0, q_end)
    const int q0 = pt * a.tile_px;
    const int q_end = min(a.NP, q0 + a.tile_px);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), nw = blockDim.x >> 6;
    const int g_begin = gt * a.gpt;
    const int ng = min(a.G, g_begin + a.gpt) - g_begin;
    // snake order over the length-sorted groups evens out the work per wavefront
    auto nth = [&](int k) { return k * nw + ((k & 1) ? nw - 1 - wave : wave); };
    const bool any = nth(0) < ng;
    Work w0 = Work{0, 0, {-1, -1, -1, -1}, {0, 0}}, w1 = w0;
    Runs<V> run0, run1;
    if (any) {
        w0 = load_work(a.work, g_begin + nth(0));
        run0 = load_runs<V>(a, w0.start, w0.cnt, lane);
        if (nth(1) < ng) w1 = load_work(a.work, g_begin + nth(1));
    }
    stage<PV, VEC>(a, lds, q0, q_end);
    if (tid < a.zero_rows * (RB / 4)) reinterpret_cast<unsigned int *>(lds + (size_t)a.Cin * RB)[tid] = 0u;  // the zero row(s)
    __syncthreads();
    if (!any) return;
    touch_runs<V>(run0);
    const PixOut<PV> px = pix_out<PV, VEC>(a, q0, lane, q_end);
    const int base = lane * 2 * PV;
    for (int k = 0;; ++k) {
        const bool more = nth(k + 1) < ng;
        Work w2 = Work{0, 0, {-1, -1, -1, -1}, {0, 0}};
        if (more) {
            run1 = load_runs<V>(a, w1.start, w1.cnt, lane);
            if (nth(k + 2) < ng) w2 = load_work(a.work, g_begin + nth(k + 2));
        }
        Acc<V, PV> acc;
        acc.zero();
        mac_segment<V, PV>(a, w0.start, w0.cnt, lds, base, lane, run0, acc);
        if (more) touch_runs<V>(run1);
        store_group<V, PV, VEC>(a, acc, w0.group[0], px);
        if (!more) break;
        w0 = w1;
        w1 = w2;
        run0 = run1;
    }
}

// The 16-bit layout of a handle, derived from the arrays every 1x1 handle has (one workgroup per
// bundle): every group gets a segment of its own again, also where the float32 layout interleaves
// the groups of a bundle - slot s of the bundle that starts at padded column `start` with `span`
// columns (its length rounded up to 16) goes to columns GS * start + s * span ... of the 16-bit
// arrays.  Per column: the weights rounded to bfloat16 (nearest even), word (col / 16) * 64 + ((col
// % 16) / 4) * 16 + 4 i + col % 4 of plane q = channel 4q + i; the row selector scaled to 256-byte
// rows; and per group a work record {first column, padded length, group}.
__global__ void __launch_bounds__(256) k_layout16(const Work *work, const float *w, long long wplane, const int32_t *off,
                                                  int GS, int planes, int Cin, Work *work16, uint16_t *w16,
                                                  long long wplane16, int32_t *off16) {
    const int b = blockIdx.x;
    const Work wk = work[b];
    const int span = (wk.cnt + 15) & ~15;
    for (int s = 0; s < GS; ++s) {
        const long long first = (long long)GS * wk.start + (long long)s * span;
        if (threadIdx.x == 0) work16[(size_t)b * GS + s] = Work{(int32_t)first, wk.cnt, {wk.group[s], -1, -1, -1}, {0, 0}};
        for (int e = threadIdx.x; e < span * 4 * planes; e += 256) {
            const int q = e / (span * 4), r = e - q * span * 4, j = r >> 2, i = r & 3;
            const long long col = first + j;
            const float v = j < wk.cnt ? w[(size_t)q * wplane + layout_w_index(GS, 4, (long long)wk.start + j, s, i)] : 0.f;
            w16[(size_t)q * wplane16 + (col / 16) * 64 + ((col % 16) / 4) * 16 + i * 4 + col % 4] =
                (uint16_t)(pack_bf2(v, 0.f) & 0xffffu);
        }
        for (int j = threadIdx.x; j < span; j += 256)
            off16[first + j] = j < wk.cnt ? off[layout_off_index(GS, (long long)wk.start + j, s)] * GS : Cin * kRowBytes;
    }
}

typedef void (*kern_t)(const Args);
template <int V>
static kern_t pick(int pv, bool vec) {
    if (pv == 2) return vec ? k_pw16<V, 2, true> : k_pw16<V, 2, false>;
    return vec ? k_pw16<V, 1, true> : k_pw16<V, 1, false>;
}

static int check(hipError_t e) {
    if (e == hipSuccess) return ALCS_OK;
    set_hip_error((int)e);
    return e == hipErrorOutOfMemory ? ALCS_E_ALLOC : ALCS_E_HIP;
}

}  // namespace m16
}  // namespace alcs

using namespace alcs;

static int zero_rows16(const alcs_packed_t *p) { return p->lay.GS > 1 ? 2 : 1; }

static bool math16_layout(const alcs_packed_t *p) {
    return p->k == 1 && p->V >= 4 && p->lay.nchunks == 1 &&
           (long long)(p->Cin + zero_rows16(p)) * (m16::kRowBytes / 2) <= 160 * 1024;  // one pixel per lane: 128-byte rows
}

extern "C" int alcs_packed_add_bf16_weights(alcs_packed_t *p, void *stream) {
    if (!p) return ALCS_E_INVALID_ARG;
    if (!p->dev.blob) return ALCS_E_NO_DEVICE;
    if (!math16_layout(p)) return ALCS_E_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(p->host_mu);
    if (p->dev.w16) return ALCS_OK;
    int cur = -1;
    int rc = m16::check(hipGetDevice(&cur));
    if (rc != ALCS_OK) return rc;
    if (cur != p->dev.device) return ALCS_E_INVALID_ARG;
    const Layout &L = p->lay;
    const long long ncol16 = L.ncol * L.GS, wplane16 = ncol16 * 4;
    auto align256 = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t o_w = 0;
    const size_t o_off = align256((size_t)wplane16 * L.planes * sizeof(uint16_t));
    const size_t o_work = align256(o_off + 4 * (size_t)ncol16);
    const size_t total = align256(o_work + sizeof(Work) * (size_t)L.nbundles * L.GS) + 256;
    void *buf = nullptr;
    if ((rc = m16::check(hipMalloc(&buf, total))) != ALCS_OK) return rc;
    char *bb = (char *)buf;
    hipStream_t st = (hipStream_t)stream;
    // what no bundle covers (the spare run at the end): zero weights, selector of the zero row
    hipError_t e = hipMemsetAsync(bb + o_w, 0, o_off, st);
    if (e == hipSuccess) e = hipMemsetAsync(bb + o_off, 0, 4 * (size_t)ncol16, st);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(m16::k_layout16, dim3((unsigned)L.nbundles), dim3(256), 0, st, p->dev.work, p->dev.w,
                           (long long)L.wplane, p->dev.off[0], L.GS, L.planes, p->Cin, (Work *)(bb + o_work),
                           (uint16_t *)(bb + o_w), wplane16, (int32_t *)(bb + o_off));
        e = hipGetLastError();
    }
    if ((rc = m16::check(e)) != ALCS_OK) {
        (void)hipFree(buf);
        return rc;
    }
    p->dev.w16 = (const uint16_t *)(bb + o_w);
    p->dev.off16 = (const int32_t *)(bb + o_off);
    p->dev.work16 = (const Work *)(bb + o_work);
    return ALCS_OK;
}

extern "C" int alcs_sparse_conv_bf16_mfma(const alcs_packed_t *Wp, const uint16_t *X_dev, const float *bias_dev,
                                          const uint16_t *residual_dev, uint16_t *Y_dev, int N, int Cin, int Cout, int H,
                                          int W, int kernel, int stride, int activation, void *stream) {
    if (!Wp || N < 0 || H <= 0 || W <= 0) return ALCS_E_INVALID_ARG;
    if (Cin != Wp->Cin || Cout != Wp->Cout || kernel != Wp->k) return ALCS_E_INVALID_ARG;
    if (N > 0 && (!X_dev || !Y_dev)) return ALCS_E_INVALID_ARG;
    if (stride != 1 && stride != 2) return ALCS_E_UNSUPPORTED;
    if (activation < 0 || activation > 2) return ALCS_E_INVALID_ARG;
    if (!Wp->dev.blob) return ALCS_E_NO_DEVICE;
    if (!math16_layout(Wp)) return ALCS_E_UNSUPPORTED;
    if (!Wp->dev.w16) return ALCS_E_INVALID_ARG;  // alcs_packed_add_bf16_weights first
    if (((uintptr_t)X_dev | (uintptr_t)Y_dev | (uintptr_t)residual_dev) & 15) return ALCS_E_INVALID_ARG;
    int cur = -1;
    int rc = m16::check(hipGetDevice(&cur));
    if (rc != ALCS_OK) return rc;
    if (cur != Wp->dev.device) return ALCS_E_INVALID_ARG;
    const int Ho = (H - 1) / stride + 1, Wo = (W - 1) / stride + 1;
    const long long P = (long long)Ho * Wo, Pin = (long long)H * W;
    const long long NP = (long long)N * P;
    if (NP > (long long)INT32_MAX - 1025 || (long long)N * Cin * Pin > (long long)INT32_MAX * 16LL ||
        Pin > INT32_MAX || (long long)N * Cout * P > (long long)INT32_MAX * 16LL)
        return ALCS_E_UNSUPPORTED;
    if (N == 0) return ALCS_OK;
    const Layout &L = Wp->lay;
    const Tuning T = tuning_of(Wp->opt);
    const int kCUs = Wp->dev.cus, kXcds = Wp->dev.xcds;
    m16::Args a{};
    a.X = X_dev; a.residual = residual_dev; a.Y = Y_dev; a.bias = bias_dev;
    a.work = Wp->dev.work16; a.w16 = Wp->dev.w16; a.off = Wp->dev.off16;
    a.wplane16 = L.ncol * L.GS * 4;
    a.zero_rows = zero_rows16(Wp);
    a.N = N; a.Cin = Cin; a.Cout = Cout; a.H = H; a.W = W; a.Ho = Ho; a.Wo = Wo; a.stride = stride;
    a.P = (int)P; a.Pin = (int)Pin; a.NP = (int)NP;
    a.G = Wp->G;
    const bool vec = stride == 1 && P % 4 == 0;
    // Two pixels per lane (128-pixel tiles, 256-byte rows) where the rows fit; one pixel per lane
    // (64-pixel tiles) beyond 638 input channels and for fewer than 4096 pixels in all, where the
    // many group tiles of a 128-pixel tile each stage twice the rows (512->1024 @7x7, N=32: 13.5 ->
    // 11.3 us; from 14x14 images on two pixels per lane win by 5-20 %); "pixels_per_lane" decides.
    const bool fits2 = (long long)(Cin + a.zero_rows) * m16::kRowBytes <= 160 * 1024;
    int pv = fits2 && NP >= 4096 ? 2 : 1;
    if (T.pv == 1) pv = 1;
    if (T.pv == 2 && fits2) pv = 2;
    const int tile = 64 * pv;
    const int lds = (Cin + a.zero_rows) * (m16::kRowBytes / 2) * pv;
    const int npt_full = (int)((NP + tile - 1) / tile);
    // group tiles only when the pixel tiles alone leave compute units idle (every group tile
    // stages the pixel tile's rows again)
    // With tiles of which at most two fit a compute unit aim at one round (<= one workgroup per
    // unit: 256->512 @14x14 7.9 us with 252 workgroups, 9.0 with 504; 512->512 @14x14 10.0 against
    // 15.0), else at about 1.5 workgroups per unit.
    int ngt = 1;
    const bool one_round = lds > 40 * 1024;
    const int want = one_round ? kCUs : 3 * kCUs / 2;
    if (npt_full < want)
        ngt = std::min(std::max(1, a.G / 4), std::max(1, one_round ? want / npt_full : (want + npt_full - 1) / npt_full));
    // A few workgroups per compute unit that do not come out even (784 tiles on 256 units: four on
    // some, three on most, and the layer lasts as long as the four): two group tiles halve the
    // grain (64->128 @56x56: 11.6 -> 10.7 us, 128->128 @56x56: 17.2 -> 15.2 us).
    else if (npt_full < 8 * kCUs && a.G >= 8) {
        const int most = (npt_full + kCUs - 1) / kCUs;
        if ((long long)npt_full * 100 < 85LL * most * kCUs) ngt = 2;
    }
    if (T.group_tiles > 0) ngt = std::min(T.group_tiles, a.G);
    a.gpt = (a.G + ngt - 1) / ngt;
    a.ngt = (a.G + a.gpt - 1) / a.gpt;
    // Full tiles only: narrower ones even out the workgroups per compute unit but end rows off the
    // 128-byte lines, which costs more than the idle units (64->128 @56x56: 11.4 us with 784 full
    // tiles, 13.7 us with 1004 tiles of 100 pixels).
    a.tile_px = tile;
    const int npt = (int)((NP + a.tile_px - 1) / a.tile_px);
    // wavefronts per workgroup, from sweeps over the MobileNet-shaped layers: 4 for tiles up to
    // 24 KB (32->64 @112x112: 17.0 us against 18.9 with 8), 16 beyond 40 KB, else 8; never more
    // than groups in the group tile or 8 KB of tile each, whichever is larger
    int nw = lds > 40 * 1024 ? 16 : lds > 24 * 1024 ? 8 : 4;
    nw = std::min(nw, std::max(std::max(2, a.gpt), lds / 8192));
    if (T.waves > 0) nw = std::min(std::max(T.waves, 2), 16);
    const long long total = (long long)npt * a.ngt;
    a.total_wgs = (int)total;
    a.xcds = kXcds;
    a.wg_per_xcd = (int)((total + kXcds - 1) / kXcds);
    a.act = activation;
    m16::kern_t kern = nullptr;
    switch (Wp->V) {
        case 4: kern = m16::pick<4>(pv, vec); break;
        case 8: kern = m16::pick<8>(pv, vec); break;
        default: kern = m16::pick<16>(pv, vec); break;
    }
    if (lds > 64 * 1024) {
        rc = m16::check(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        if (rc != ALCS_OK) return rc;
    }
    record_launch(6, pv, nw, a.total_wgs, lds, a.ngt, L.KC, 3, 1, 0);
    hipLaunchKernelGGL(kern, dim3((unsigned)(a.wg_per_xcd * kXcds)), dim3(nw * 64), lds, (hipStream_t)stream, a);
    return m16::check(hipGetLastError());
}
