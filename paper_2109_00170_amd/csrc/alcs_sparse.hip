// HIP kernels (gfx950) and launcher of alcs_sparse_conv: the sparse x dense
// multiplication of Section 3.2.2 ("Efficient multiplication computation") of
// arXiv 2109.00170, re-designed for 64-lane wavefronts.
//
// Mapping.  The paper puts the V output channels of a group into one SIMD register
// and broadcasts an input scalar.  Here the 64 lanes of a wavefront are 64 output
// pixels (contiguous in NCHW, so global and LDS accesses are coalesced), the V
// channels of the group are V accumulator registers per lane, and the weight block
// of a kept column is wave-uniform.  A workgroup stages the input rows of a pixel
// tile in LDS once; its wavefronts then walk the kept columns of their groups: one
// LDS row read per kept column, selected by the column's offset, feeds V
// multiply-accumulates per pixel - the same reuse the paper gets from its V-wide
// register.
//
// For V in {4, 8, 16} the multiply-accumulate is v_mfma_f32_4x4x1_16B_f32: each of
// its 16 blocks is a 4(channel) x 4(pixel) outer product, and with the block
// broadcast modifier (cbsz = 4, abid = j) all 16 blocks take their 4 weights from
// block j of the A register.  One coalesced 256-byte load therefore brings the
// weights of 16 consecutive kept columns, and every flop the instruction performs is
// a useful one (nothing is densified).  For V in {1, 2} (and optionally 4) plain
// v_fma_f32 with scalar-register weights is used.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <cstdint>
#include <mutex>
#include <map>
#include <set>
#include <utility>

#include "alcs_internal.h"
#if ALCS_DW_STAGE
#include "alcs_dw_taps.h"
#endif

// This file is compiled twice.  As it stands it gives alcs_sparse_conv and
// alcs_sparse_conv_timed, whose kernels have no trace of the fused epilogue (a run-time
// test for a residual or an activation in every store cost 3-4 % of the benchmark step).
// alcs_sparse_fused.hip defines ALCS_FUSED_EPILOGUE and includes this file: the same
// kernels with the epilogue compiled in, in namespace alcs::fused, behind
// alcs_sparse_conv_fused.
//
// alcs_sparse_dw.hip defines ALCS_DW_STAGE as well: the resident 1x1 kernels once more, in
// namespace alcs::dwpw, with the staging of the input tile replaced by the depthwise 3x3
// layer that precedes the pointwise convolution (its output goes straight into LDS and
// never to memory), behind alcs_dw_sparse_conv_fused.
#ifndef ALCS_FUSED_EPILOGUE
#define ALCS_FUSED_EPILOGUE 0
#endif
#ifndef ALCS_DW_STAGE
#define ALCS_DW_STAGE 0
#endif
//
// alcs_sparse_bf16.hip defines ALCS_IO_BF16: the resident 1x1 kernels with X, the residual and Y
// stored as bfloat16 (namespace alcs::bf16io), behind alcs_sparse_conv_bf16.  Weights, bias,
// LDS tile and accumulation stay float32; only the tensors that cross HBM are narrower.
#ifndef ALCS_IO_BF16
#define ALCS_IO_BF16 0
#endif
#if (ALCS_DW_STAGE || ALCS_IO_BF16) && !ALCS_FUSED_EPILOGUE
#error "the depthwise stage and the bfloat16 tensors come with the fused epilogue"
#endif
#if ALCS_DW_STAGE && ALCS_IO_BF16
#error "one variant per compilation"
#endif
// builds that hold only the resident 1x1 kernels
#define ALCS_RESIDENT_ONLY (ALCS_DW_STAGE || ALCS_IO_BF16)

namespace alcs {
#if ALCS_DW_STAGE
namespace dwpw {
#elif ALCS_IO_BF16
namespace bf16io {
#elif ALCS_FUSED_EPILOGUE
namespace fused {
#endif

constexpr bool kFused = ALCS_FUSED_EPILOGUE != 0;
constexpr bool kDw = ALCS_DW_STAGE != 0;

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef int i4 __attribute__((ext_vector_type(4)));

// Element type of X, the residual and Y in memory, and 1 / 2 / 4 consecutive elements of it
// as floats.  bfloat16 is the upper half of a float: widening is a shift, narrowing rounds to
// nearest even (v_cvt_pk_bf16_f32).  Stores are non-temporal: Y is not read again.
#if ALCS_IO_BF16
typedef unsigned short io_t;
typedef unsigned int u2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float io_load1(const io_t *p) { return __builtin_bit_cast(float, (unsigned int)*p << 16); }
__device__ __forceinline__ f2 io_load2(const io_t *p) {
    const unsigned int u = *reinterpret_cast<const unsigned int *>(p);
    return f2{__builtin_bit_cast(float, u << 16), __builtin_bit_cast(float, u & 0xffff0000u)};
}
__device__ __forceinline__ f4 io_load4(const io_t *p) {
    const u2v u = *reinterpret_cast<const u2v *>(p);
    return f4{__builtin_bit_cast(float, u.x << 16), __builtin_bit_cast(float, u.x & 0xffff0000u),
              __builtin_bit_cast(float, u.y << 16), __builtin_bit_cast(float, u.y & 0xffff0000u)};
}
__device__ __forceinline__ unsigned int pack_bf2(float a, float b) {
    return __builtin_bit_cast(unsigned int, __builtin_convertvector(f2{a, b}, bf2));
}
__device__ __forceinline__ void io_store1(io_t *p, float v) {
    __builtin_nontemporal_store((io_t)(pack_bf2(v, 0.f) & 0xffffu), p);
}
__device__ __forceinline__ void io_store2(io_t *p, f2 v) {
    __builtin_nontemporal_store(pack_bf2(v[0], v[1]), reinterpret_cast<unsigned int *>(p));
}
__device__ __forceinline__ void io_store4(io_t *p, f4 v) {
    __builtin_nontemporal_store(u2v{pack_bf2(v[0], v[1]), pack_bf2(v[2], v[3])}, reinterpret_cast<u2v *>(p));
}
#else
typedef float io_t;
__device__ __forceinline__ float io_load1(const io_t *p) { return *p; }
__device__ __forceinline__ f2 io_load2(const io_t *p) { return *reinterpret_cast<const f2 *>(p); }
__device__ __forceinline__ f4 io_load4(const io_t *p) { return *reinterpret_cast<const f4 *>(p); }
__device__ __forceinline__ void io_store1(io_t *p, float v) { __builtin_nontemporal_store(v, p); }
__device__ __forceinline__ void io_store2(io_t *p, f2 v) { __builtin_nontemporal_store(v, reinterpret_cast<f2 *>(p)); }
__device__ __forceinline__ void io_store4(io_t *p, f4 v) { __builtin_nontemporal_store(v, reinterpret_cast<f4 *>(p)); }
#endif
// An ordinary (write-back) store of two elements: for runs that cover cache lines only in part and
// whose neighbours are written soon after by the same workgroup, so that the L2 merges them into
// whole lines before they leave for memory.
__device__ __forceinline__ void io_store2_cached(io_t *p, f2 v) {
#if ALCS_IO_BF16
    *reinterpret_cast<unsigned int *>(p) = pack_bf2(v[0], v[1]);
#else
    *reinterpret_cast<f2 *>(p) = v;
#endif
}

struct ConvArgs {
    const io_t *X;
    const float *bias;
    const io_t *residual;  // fused epilogue: tensor of Y's shape added before the activation, or null
    io_t *Y;
    const Work *work;   // [G * nchunks] in hand-out order (longest group first)
    const float *w;
    const int32_t *off;
    long long wplane;   // floats between weight planes (nblk * VV)
    int N, Cin, Cout, H, W, Ho, Wo, stride;
    int P, Pin;         // Ho*Wo, H*W
    int NP;             // N * P, flattened output pixels (< 2^31)
    int tile_px;        // resident 1x1 kernels: pixels of the flattened axis per workgroup (<= tile width)
    int G, nchunks, KC;
    int npt, ngt, gpt;  // pixel tiles, group tiles, groups per group tile
    int tiles_x, tiles_y;  // 3x3: output tiles per image
    int wg_per_xcd, total_wgs, xcds;
    int ppw;            // streaming kernel: flattened pixels per workgroup (multiple of 4)
    int wfloats;        // streaming kernel: floats in the weight planes, planes * nblk * 4
    int nblk;           // padded blocks (= number of row selectors)
    // 3x3 with a tap-shared pattern: channel records (see alcs_chanrec.hip), null otherwise
    const float *cw;
    const int32_t *csel, *cwork;
    long long cwplane;
    int act;    // fused epilogue: 0 none, 1 max(., 0), 2 min(max(., 0), 6)
    int debug;  // measurement build only (ALCS_MEASURE): bit 0 skips staging, bit 1 the multiply, bit 2 the stores
#if ALCS_DW_STAGE
    // Depthwise stage: X is the depthwise layer's input [N, Cin, H, W]; its output
    // [N, Cin, Ho, Wo] is what the pointwise convolution (stride 1) multiplies.
    const float *dw_w;     // [Cin, 3, 3]
    const float *dw_bias;  // [Cin] or null
    int dw_stride, dw_act;
    int dw_mode;           // DwMode: how lanes share taps
#endif
};

// Phase skipping for measurements (alcs_options.measure_skip): compiled in only with
// -DALCS_MEASURE=1, which the product build never sets - there the tests below fold to false
// and the kernels hold no trace of them.
#ifndef ALCS_MEASURE
#define ALCS_MEASURE 0
#endif
__device__ __forceinline__ bool skip(const ConvArgs &a, int bit) {
    if constexpr (ALCS_MEASURE != 0) return (a.debug & bit) != 0;
    else return false;
}

// The element-wise tail of the fused epilogue (the plain convolution passes act = 0).
__device__ __forceinline__ float activate(const ConvArgs &a, float v) {
    if constexpr (kFused) {
        if (a.act >= 1) v = fmaxf(v, 0.f);
        if (a.act == 2) v = fminf(v, 6.f);
    }
    return v;
}
// The residual tensor, or null where the epilogue is compiled out.
__device__ __forceinline__ const io_t *residual_of(const ConvArgs &a) {
    if constexpr (kFused) return a.residual;
    else return nullptr;
}


// Index arrays, segment table, bias and (for the FMA form) the weights are read
// through the constant address space: the addresses are wave-uniform, and this lets
// the compiler fetch them with scalar loads into SGPRs even though the kernel also
// stores to global memory (Y never aliases them).
template <class T>
using cptr = const T __attribute__((address_space(4))) *;
template <class T>
__device__ __forceinline__ cptr<T> as_const(const T *p) {
    return (cptr<T>)(uintptr_t)p;
}

typedef int i8v __attribute__((ext_vector_type(8)));
static_assert(sizeof(Work) == 32, "Work is read as eight ints");
// One scalar 32-byte load; the values end up in SGPRs.
__device__ __forceinline__ Work load_work(const Work *table, size_t idx) {
    const i8v v = *reinterpret_cast<cptr<i8v>>((uintptr_t)(table + idx));
    Work w;
    w.start = __builtin_amdgcn_readfirstlane(v[0]);
    w.cnt = __builtin_amdgcn_readfirstlane(v[1]);
#pragma unroll
    for (int s = 0; s < kMaxSlots; ++s) w.group[s] = __builtin_amdgcn_readfirstlane(v[2 + s]);
    w.reserved[0] = w.reserved[1] = 0;
    return w;
}
__device__ __forceinline__ Work no_work() { return Work{0, 0, {-1, -1, -1, -1}, {0, 0}}; }

// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Renumber
// so that consecutive logical ids - which share a pixel tile and differ only in the
// group tile - land on the same XCD and find the tile's input rows in that L2.
__device__ __forceinline__ int logical_wg(const ConvArgs &a) {
    const int id = blockIdx.x;
    return (id % a.xcds) * a.wg_per_xcd + id / a.xcds;
}

// ------------------------------------------------------------------ accumulators

// Partial accumulators per (channel quad, pixel of the lane): 2 when a lane has a single
// MFMA per column, else 1.
constexpr int nacc_for(int mfmas_per_column) { return mfmas_per_column == 1 ? 2 : 1; }

template <int V, int PV, bool MF>
struct Acc;

template <int V, int PV>
struct Acc<V, PV, true> {  // MFMA: a[k][q][pv][i] = channel 4q+i, pixel pv of the lane, partial sum k
    // An MFMA that accumulates into the register of the one before it has to wait for its
    // result (two alternating accumulators already issue at full rate).  With a single
    // accumulator per lane (V/4 * PV == 1), consecutive columns therefore go round-robin to
    // NACC partial accumulators that are added at the end.
    static constexpr int NACC = nacc_for((V / 4) * PV);
    f4 a[NACC][V / 4][PV];
    __device__ __forceinline__ void zero() {
#pragma unroll
        for (int k = 0; k < NACC; ++k)
#pragma unroll
            for (int q = 0; q < V / 4; ++q)
#pragma unroll
                for (int pv = 0; pv < PV; ++pv) a[k][q][pv] = f4{0.f, 0.f, 0.f, 0.f};
    }
    __device__ __forceinline__ float get(int v, int pv) const {
        float r = a[0][v >> 2][pv][v & 3];
#pragma unroll
        for (int k = 1; k < NACC; ++k) r += a[k][v >> 2][pv][v & 3];
        return r;
    }
};

template <int V, int PV>
struct Acc<V, PV, false> {
    float a[V][PV];
    __device__ __forceinline__ void zero() {
#pragma unroll
        for (int v = 0; v < V; ++v)
#pragma unroll
            for (int pv = 0; pv < PV; ++pv) a[v][pv] = 0.f;
    }
    __device__ __forceinline__ float get(int v, int pv) const { return a[v][pv]; }
};

// The lane's PV pixels of one LDS row: neighbours (PD = 1), or two words PD apart, which the
// compiler fetches with one ds_read2_b32 (PD <= 255, no alignment beyond 4 bytes needed).
template <int PV, int PD = 1>
__device__ __forceinline__ void lds_read(const float *p, float (&x)[PV]) {
    if constexpr (PD != 1) {
        static_assert(PV == 2 && PD <= 255, "two pixels a fixed distance apart");
        x[0] = p[0];
        x[1] = p[PD];
    } else if constexpr (PV == 4) {
        f4 t = *reinterpret_cast<const f4 *>(p);
        x[0] = t[0]; x[1] = t[1]; x[2] = t[2]; x[3] = t[3];
    } else if constexpr (PV == 2) {
        f2 t = *reinterpret_cast<const f2 *>(p);
        x[0] = t[0]; x[1] = t[1];
    } else {
        x[0] = *p;
    }
}

constexpr int ilog2(int x) { return x <= 1 ? 0 : 1 + ilog2(x / 2); }

// Weights and row selectors of one run of 16 consecutive kept columns, as fetched by
// coalesced vector loads.  With GS groups per wavefront, lanes [s*64/GS, (s+1)*64/GS)
// are slot s; weight register r of plane q holds columns [r*16/GS, (r+1)*16/GS) of the
// run: lane l carries (slot, column (l % (64/GS)) / 4, weight row l % 4); and every
// 16-lane row holds the 16 selectors of its slot.
template <int V, bool MF, int GS = 1>
struct Run {
    float a[MF ? (V / 4) * GS : 1];
    int o;
};

// The first N runs of a segment, fetched together by the caller well ahead of their use
// (before the previous group's output stores: vector memory operations complete in
// order, so a load issued behind stores waits for them).  N = 4 covers segments of up
// to 64 columns without any load inside the multiply loop; with many weight registers
// per run (V/4 * GS > 2, except four groups of V = 4) N = 2.  The walk over a longer segment re-fills register set i
// right after its use with the run N places further on: no register is ever copied, so
// nothing waits for a load before the run that needs it.
template <int V, bool MF, int GS>
constexpr int runs_ahead() { return !MF ? 1 : ((V / 4) * GS <= 2 || (V == 4 && GS == 4)) ? 4 : 2; }

template <int V, bool MF, int GS = 1>
struct Runs {
    static constexpr int N = runs_ahead<V, MF, GS>();
    Run<V, MF, GS> r[N];
};

template <int V, bool MF, int GS = 1>
__device__ __forceinline__ Run<V, MF, GS> load_run(const ConvArgs &a, int blk, int lane);

// Runs at columns blk, blk + 16, ... of a segment of cnt (padded) columns.  All N loads
// are issued unconditionally; places beyond the segment's last run re-read that run (or
// run 0 of an empty segment, which exists: the arrays end with a spare run).
template <int V, bool MF, int GS = 1>
__device__ __forceinline__ Runs<V, MF, GS> load_runs(const ConvArgs &a, int blk, int cnt, int lane) {
    Runs<V, MF, GS> rs;
    const int last = max(0, ((cnt + 15) & ~15) - 16);
#pragma unroll
    for (int i = 0; i < Runs<V, MF, GS>::N; ++i) rs.r[i] = load_run<V, MF, GS>(a, blk + min(16 * i, last), lane);
    return rs;
}

template <int V, bool MF, int GS>
__device__ __forceinline__ Run<V, MF, GS> load_run(const ConvArgs &a, int blk, int lane) {
    Run<V, MF, GS> r;
    if constexpr (MF) {
        const float *wp = a.w + (size_t)blk * 4 * GS + lane;
#pragma unroll
        for (int q = 0; q < V / 4; ++q)
#pragma unroll
            for (int g = 0; g < GS; ++g) r.a[q * GS + g] = wp[(size_t)q * a.wplane + g * 64];
        const int slot = lane >> (6 - ilog2(GS));
        r.o = a.off[(size_t)blk * GS + slot * 16 + (lane & 15)];
    } else {
        r.a[0] = 0.f;
        r.o = 0;
    }
    return r;
}

// Compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(<N-1>); the MFMA
// block-select modifier has to be an immediate.
template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, Is...>) {
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Selector of column C of the current run, in every lane: the run's 16 selectors
// sit in lanes 0..15 of each 16-lane row of `ov`, and the DPP control row_newbcast:C
// hands lane C of its own row to every lane - no SGPR round trip, and the compiler
// folds the move into the address add.
template <int C>
__device__ __forceinline__ int bcast_sel(int ov) {
    return __builtin_amdgcn_update_dpp(0, ov, 0x150 + C, 0xF, 0xF, false);
}

// B consecutive kept columns of the current run, starting at column B0 of the run.
// All B LDS row reads are issued first, then the MFMAs: for column c all 16 blocks
// take their 4 weights from block c of the weight register (cbsz = 4, abid = c) and
// multiply them with the lane's pixel value(s).  Segment lengths are padded to a
// multiple of B (zero weights, selector of the all-zero row), so a batch never
// branches: the compiler keeps all B reads in flight ahead of the MFMAs.
// base is the lane's byte offset inside an LDS row (minus the chunk's first row); ov holds
// the run's selectors already scaled to the row length (the caller shifts the register once
// per run: a shift behind the broadcast would cost a move, a broadcast and a shift-add per
// column where one add with the broadcast folded in does).
template <int B0, int B, int V, int PV, int GS, int PD = 1>
__device__ __forceinline__ void mfma_batch(const float (&aw)[(V / 4) * GS], int ov, const char *lds,
                                           int base, Acc<V, PV, true> &acc) {
    constexpr int CPA = 16 / GS;           // columns per weight register
    constexpr int CBSZ = 4 - ilog2(GS);    // blocks that share one block's weights: 16 / GS
    float x[B][PV];
    static_for<B>([&](auto c) {
        constexpr int C = decltype(c)::value;
        lds_read<PV, PD>(reinterpret_cast<const float *>(lds + base + bcast_sel<B0 + C>(ov)), x[C]);
    });
    // With two pixels per lane the scheduler would trade reads in flight for registers and
    // interleave two reads at a time with the MFMAs; keep all B reads ahead of them.  (With
    // four pixels per lane the 32 registers this takes cost more occupancy than they gain.)
    if constexpr (PV == 2) __builtin_amdgcn_sched_barrier(0);
    static_for<B>([&](auto c) {
        constexpr int C = decltype(c)::value;
        constexpr int COL = B0 + C, AREG = COL / CPA, ABID = COL % CPA;
#pragma unroll
        for (int q = 0; q < V / 4; ++q)
#pragma unroll
            for (int pv = 0; pv < PV; ++pv) {
                constexpr int K = COL % Acc<V, PV, true>::NACC;
                acc.a[K][q][pv] = __builtin_amdgcn_mfma_f32_4x4x1f32(aw[q * GS + AREG], x[C][pv],
                                                                     acc.a[K][q][pv], CBSZ, ABID, 0);
            }
    });
}

// One segment (the kept columns of one bundle of GS groups inside one channel chunk),
// MFMA form.  start/cnt are wave-uniform; base is the lane's byte offset inside an LDS
// row (minus the chunk's first row); SH = log2(pixels per lane) for 1x1, 0 for 3x3.
// `rs` holds the segment's first runs, loaded by the caller (see Runs).
// Tells the compiler that the registers of `rs` are needed here: it places the wait for their
// loads at this point.  Used where that wait is free (the loads were issued a whole multiply
// earlier) and ahead of vector-memory operations a later wait would otherwise have to include:
// the counter of outstanding vector-memory operations is a single in-order one that covers
// loads and stores alike, and where paths of different length merge the compiler waits for it
// to reach zero - which, behind a group's output stores or the next group's prefetches, means
// waiting for those as well.
template <int V, int GS>
__device__ __forceinline__ void touch_runs(Runs<V, true, GS> &rs) {
#pragma unroll
    for (int i = 0; i < Runs<V, true, GS>::N; ++i) {
#pragma unroll
        for (int q = 0; q < (V / 4) * GS; ++q) asm volatile("" : "+v"(rs.r[i].a[q]));
        asm volatile("" : "+v"(rs.r[i].o));
    }
}
template <int V, int GS>
__device__ __forceinline__ void touch_runs(Runs<V, false, GS> &) {}

template <int V, int PV, int SH, int GS = 1, int PD = 1>
__device__ __forceinline__ void mac_segment(const ConvArgs &a, int start, int cnt,
                                            const char *lds, int base, int lane,
                                            Runs<V, true, GS> rs, Acc<V, PV, true> &acc) {
    constexpr int B = kCntAlign;  // columns whose LDS reads are in flight together
    constexpr int N = Runs<V, true, GS>::N;
    static_assert(B == 8, "a run of 16 columns is two batches");
    auto pass = [&](int j0) {
        static_for<N>([&](auto ii) {
            constexpr int I = decltype(ii)::value;
            const int j = j0 + 16 * I;
            if (j < cnt) {
                // selectors are byte offsets for 64-pixel rows: scale them to this tile's rows
                const int ov = rs.r[I].o << SH;
                mfma_batch<0, B, V, PV, GS, PD>(rs.r[I].a, ov, lds, base, acc);
                if (j + 8 < cnt) mfma_batch<8, B, V, PV, GS, PD>(rs.r[I].a, ov, lds, base, acc);
                if (j + 16 * N < cnt) rs.r[I] = load_run<V, true, GS>(a, start + j + 16 * N, lane);
            }
        });
    };
    // The first pass runs on the registers the caller loaded (and has waited for): straight-line
    // code in which nothing waits for vector memory.  Only longer segments enter the loop, whose
    // head waits for the re-fills issued one pass earlier.
    pass(0);
    for (int j0 = 16 * N; j0 < cnt; j0 += 16 * N) pass(j0);
}

// The same segment for a caller that keeps `rs` (the segment's first runs) in registers across
// many tiles: `rs` is only read; runs beyond it are fetched into two temporaries, each requested
// one run ahead of its use.
template <int V, int PV, int SH, int GS, bool TAIL>
__device__ __forceinline__ void mac_segment_keep(const ConvArgs &a, int start, int cnt, const char *lds, int base,
                                                 int lane, const Runs<V, true, GS> &rs, Acc<V, PV, true> &acc) {
    constexpr int N = Runs<V, true, GS>::N;
    // batches of four columns: the registers a batch of eight reads holds are needed for the
    // resident weights (the wavefronts that share a SIMD cover the LDS latency between them)
    auto eight = [&](auto b0, const float (&aw)[(V / 4) * GS], int ov) {
        constexpr int B0 = decltype(b0)::value;
        mfma_batch<B0, 4, V, PV, GS>(aw, ov, lds, base, acc);
        mfma_batch<B0 + 4, 4, V, PV, GS>(aw, ov, lds, base, acc);
    };
    const bool tail = TAIL && cnt > 16 * N;  // without TAIL the caller guarantees at most 16 * N columns
    Run<V, true, GS> t0, t1;
    if (tail) t0 = load_run<V, true, GS>(a, start + 16 * N, lane);
    static_for<N>([&](auto ii) {
        constexpr int I = decltype(ii)::value;
        const int j = 16 * I;
        if (j < cnt) {
            const int ov = rs.r[I].o << SH;
            eight(std::integral_constant<int, 0>{}, rs.r[I].a, ov);
            if (j + 8 < cnt) eight(std::integral_constant<int, 8>{}, rs.r[I].a, ov);
        }
    });
    if (tail) {
        for (int j = 16 * N; j < cnt; j += 32) {
            const bool second = j + 16 < cnt;
            if (second) t1 = load_run<V, true, GS>(a, start + j + 16, lane);
            {
                const int ov = t0.o << SH;
                eight(std::integral_constant<int, 0>{}, t0.a, ov);
                if (j + 8 < cnt) eight(std::integral_constant<int, 8>{}, t0.a, ov);
            }
            if (!second) break;
            if (j + 32 < cnt) t0 = load_run<V, true, GS>(a, start + j + 32, lane);
            {
                const int ov = t1.o << SH;
                eight(std::integral_constant<int, 0>{}, t1.a, ov);
                if (j + 24 < cnt) eight(std::integral_constant<int, 8>{}, t1.a, ov);
            }
        }
    }
}

// Same segment with plain FMAs; selectors and the V weights of a column come from
// scalar loads.
template <int V, int PV, int SH, int GS = 1, int PD = 1>
__device__ __forceinline__ void mac_segment(const ConvArgs &a, int start, int cnt,
                                            const char *lds, int base, int lane,
                                            Runs<V, false, GS> first, Acc<V, PV, false> &acc) {
    static_assert(V <= 4 && GS == 1 && PD == 1, "FMA path is built for V <= 4, one group per wavefront");
    (void)lane;
    (void)first;
    cptr<float> wp = as_const(a.w) + (size_t)start * V;
    cptr<int32_t> op = as_const(a.off) + start;
    for (int j = 0; j < cnt; j += 4) {
        const i4 o = *reinterpret_cast<cptr<i4>>(op + j);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float x[PV];
            lds_read<PV>(reinterpret_cast<const float *>(lds + base + (o[u] << SH)), x);
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const float wv = wp[(j + u) * V + v];
#pragma unroll
                for (int pv = 0; pv < PV; ++pv) acc.a[v][pv] = __builtin_fmaf(wv, x[pv], acc.a[v][pv]);
            }
        }
    }
}

// ------------------------------------------------------------------ 1x1: staging

// Rows [c0, c1) of the pixel tile [q0, q0 + TP) of the flattened (n, pixel) axis into
// LDS rows 0.. (row length TP).  VEC: stride 1 and P % 4 == 0, so four consecutive
// pixels never straddle an image and are 16-byte aligned.
// Place of the tile's e-th pixel in an LDS row.  SPLIT (two pixels per lane without the
// vector form, where a pair of neighbours may straddle two images): a lane owns pixels
// e and e + TP/2, stored side by side so that one 8-byte read fetches both, and a store
// instruction still writes a contiguous run of pixels.
template <int TP, bool SPLIT>
__device__ __forceinline__ int tile_pos(int e) {
    if constexpr (SPLIT) return (e % (TP / 2)) * 2 + e / (TP / 2);
    return e;
}

template <int TP, bool VEC, bool SPLIT = false>
__device__ __forceinline__ void stage_pw(const ConvArgs &a, float *lds, int q0, int c0, int c1, int q_end) {
    static_assert(!(VEC && SPLIT), "the vector form keeps neighbouring pixels together");
    const int tid = threadIdx.x, nt = blockDim.x;
    if constexpr (VEC) {
        constexpr int NQ = TP / 4;
        const int quad = tid % NQ, r0 = tid / NQ, rpp = nt / NQ;
        const int q = q0 + quad * 4;
        const bool valid = q < q_end;
        const int n = valid ? q / a.P : 0;
        const int p = valid ? q - n * a.P : 0;
        const io_t *src = a.X + ((size_t)n * a.Cin + c0) * a.P + p;
        float *dst = lds + quad * 4;
        const int rows = c1 - c0;
        constexpr int U = 8;  // independent 16-byte loads in flight per thread
        int r = r0;
        for (; r + (U - 1) * rpp < rows; r += U * rpp) {
            f4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                v[u] = f4{0, 0, 0, 0};
                if (valid) v[u] = io_load4(src + (size_t)(r + u * rpp) * a.P);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) *reinterpret_cast<f4 *>(dst + (r + u * rpp) * TP) = v[u];
        }
        for (; r < rows; r += rpp) {
            f4 v0 = f4{0, 0, 0, 0};
            if (valid) v0 = io_load4(src + (size_t)r * a.P);
            *reinterpret_cast<f4 *>(dst + r * TP) = v0;
        }
    } else {
        const int e = tid % TP, r0 = tid / TP, rpp = nt / TP;
        const int q = q0 + e;
        const bool valid = q < q_end;
        const int n = valid ? q / a.P : 0;
        const int po = valid ? q - n * a.P : 0;
        const int ho = po / a.Wo, wo = po - ho * a.Wo;
        const io_t *src = a.X + ((size_t)n * a.Cin + c0) * a.Pin + (size_t)(ho * a.stride) * a.W + wo * a.stride;
        const int rows = c1 - c0;
        constexpr int U = 16;  // independent 4-byte loads in flight per thread
        int r = r0;
        for (; r + (U - 1) * rpp < rows; r += U * rpp) {
            float v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = valid ? io_load1(src + (size_t)(r + u * rpp) * a.Pin) : 0.f;
#pragma unroll
            for (int u = 0; u < U; ++u) lds[(r + u * rpp) * TP + tile_pos<TP, SPLIT>(e)] = v[u];
        }
        for (; r < rows; r += rpp) lds[r * TP + tile_pos<TP, SPLIT>(e)] = valid ? io_load1(src + (size_t)r * a.Pin) : 0.f;
    }
}

#if ALCS_DW_STAGE
// The depthwise 3x3 layer (zero padding 1, stride 1 or 2, bias, activation) evaluated for
// the pixel tile [q0, q0 + TP) of its flattened (n, ho, wo) output axis, every channel c
// into LDS row c: the tile the pointwise convolution multiplies is produced in place and
// never visits memory.  Lanes hold consecutive pixels and share taps (alcs_dw_taps.h); a
// thread owns one pixel of the tile and every (blockDim / TP)-th channel.  With TP >= 64 a
// wavefront works on one channel at a time, so the filter and the bias come through scalar
// loads.
template <int TP, int MODE, bool SPLIT>
__device__ __forceinline__ void stage_dw_mode(const ConvArgs &a, float *lds, int q0, int q_end) {
    constexpr int SPAN = TP < 64 ? TP : 64;
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63;
    // A pass covers `span` pixels of the tile with nt / span channels side by side; a
    // workgroup with fewer threads than the tile has pixels takes several passes.
    const int span = nt < TP ? nt : TP;
    const int rpp = nt / span;
    int r0 = tid / span;
    if constexpr (TP >= 64) r0 = __builtin_amdgcn_readfirstlane(r0);  // span is a multiple of 64 then
    if (r0 >= rpp) return;  // threads beyond the last full set of channels (whole spans)
    const auto wts = as_const(a.dw_w);
    const auto bs = as_const(a.dw_bias);
    for (int e = tid - r0 * span; e < TP; e += span) {
        const int q = q0 + e;
        const bool valid = q < q_end;
        const int n = valid ? q / a.P : 0;
        const int po = valid ? q - n * a.P : 0;
        const int ho = po / a.Wo, wo = po - ho * a.Wo;
        // The wavefront's first lane holds its lowest pixel; taps are addressed from that
        // lane's image (wave-uniform) plus what the lane's own image and channel add.
        const int n0 = __builtin_amdgcn_readfirstlane(n);
        const int rl = TP >= 64 ? 0 : r0;  // channel offset inside the wavefront (narrow tiles)
        const long long delta = valid ? ((long long)(n - n0) * a.Cin + rl) * a.Pin : (long long)rl * a.Pin;
        DwTaps<MODE, SPAN> taps;
        taps.init(valid, delta, ho, wo, a.H, a.W, a.dw_stride, lane);
        const float *src = a.X + (size_t)n0 * a.Cin * a.Pin;
        auto finish = [&](int c, const typename DwTaps<MODE, SPAN>::Raw &x) {
            float acc = taps.apply(x, wts + c * 9, a.dw_bias ? bs[c] : 0.f);
            if (a.dw_act >= 1) acc = fmaxf(acc, 0.f);
            if (a.dw_act == 2) acc = fminf(acc, 6.f);
            lds[c * TP + tile_pos<TP, SPLIT>(e)] = valid ? acc : 0.f;
        };
        int c = r0;  // the lane's channel; c - rl is wave-uniform
        // two channels' loads in flight (one on the narrow tiles, whose kernels hold the
        // weights of several groups in registers meanwhile)
        for (; TP >= 64 && c + rpp < a.Cin; c += 2 * rpp) {
            typename DwTaps<MODE, SPAN>::Raw x0, x1;
            taps.load(src + (size_t)(c - rl) * a.Pin, x0);
            taps.load(src + (size_t)(c - rl + rpp) * a.Pin, x1);
            finish(c, x0);
            finish(c + rpp, x1);
        }
        for (; c < a.Cin; c += rpp) {
            typename DwTaps<MODE, SPAN>::Raw x0;
            taps.load(src + (size_t)(c - rl) * a.Pin, x0);
            finish(c, x0);
        }
    }
}

template <int TP, bool SPLIT>
__device__ __forceinline__ void stage_dw(const ConvArgs &a, float *lds, int q0, int q_end) {
    if (a.dw_mode == kDwPair) stage_dw_mode<TP, kDwPair, SPLIT>(a, lds, q0, q_end);
    else stage_dw_mode<TP, kDwNine, SPLIT>(a, lds, q0, q_end);
}
#endif

// Where a lane's PV pixels go in Y (offset of channel 0; add ch * P).
template <int PV>
struct PixOut {
    long long yoff[PV];
    bool valid[PV];
};

// PSTRIDE > 0: the lane's pixels are PSTRIDE apart (see tile_pos), else neighbours.
template <int PV, bool VEC, int PSTRIDE = 0>
__device__ __forceinline__ void pix_out(const ConvArgs &a, int q0, int lane, PixOut<PV> &px, int q_end) {
#pragma unroll
    for (int pv = 0; pv < PV; ++pv) {
        const int q = PSTRIDE > 0 ? q0 + lane + pv * PSTRIDE : q0 + lane * PV + pv;
        px.valid[pv] = q < q_end;
        if (VEC && pv > 0) {
            px.yoff[pv] = px.yoff[0] + pv;
        } else {
            const int n = px.valid[pv] ? q / a.P : 0;
            const int p = px.valid[pv] ? q - n * a.P : 0;
            px.yoff[pv] = (long long)n * a.Cout * a.P + p;
        }
    }
}

// The residual of one group for the lane's pixels, fetched before the group is multiplied
// (a load issued in the epilogue would be waited for at once).
template <int V, int PV>
struct Resid {
    float r[V][PV];
};
template <int V, int PV, bool VEC>
__device__ __forceinline__ void load_residual(const ConvArgs &a, int g, const PixOut<PV> &px, Resid<V, PV> &rr) {
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int ch = g * V + v;
#pragma unroll
        for (int pv = 0; pv < PV; ++pv) rr.r[v][pv] = 0.f;
        if (ch >= a.Cout) continue;
        const io_t *res = a.residual + (size_t)ch * a.P;
        if constexpr (VEC && PV == 4) {
            if (px.valid[0]) {
                const f4 t = io_load4(res + px.yoff[0]);
                rr.r[v][0] = t[0]; rr.r[v][1] = t[1]; rr.r[v][2] = t[2]; rr.r[v][3] = t[3];
            }
        } else if constexpr (VEC && PV == 2) {
            if (px.valid[0]) {
                const f2 t = io_load2(res + px.yoff[0]);
                rr.r[v][0] = t[0]; rr.r[v][1] = t[1];
            }
        } else {
#pragma unroll
            for (int pv = 0; pv < PV; ++pv)
                if (px.valid[pv]) rr.r[v][pv] = io_load1(res + px.yoff[pv]);
        }
    }
}

// Epilogue: Y = acc + bias for the V channels of group g (rows beyond Cout of a
// ragged last group are not stored).
template <int V, int PV, bool MF, bool VEC>
__device__ __forceinline__ void store_group(const ConvArgs &a, const Acc<V, PV, MF> &acc, int g,
                                            const PixOut<PV> &px, const Resid<V, PV> *pre = nullptr) {
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int ch = g * V + v;
        if (ch >= a.Cout) break;
        float b = a.bias ? as_const(a.bias)[ch] : 0.f;
        io_t *dst = a.Y + (size_t)ch * a.P;
        // the residual: already in registers (pre), or read here
        const io_t *res = (residual_of(a) && !pre) ? residual_of(a) + (size_t)ch * a.P : nullptr;  // wave-uniform
        if (kFused && pre) {
            if constexpr (VEC && PV == 4) {
                if (px.valid[0]) {
                    f4 o = f4{acc.get(v, 0) + b + pre->r[v][0], acc.get(v, 1) + b + pre->r[v][1],
                              acc.get(v, 2) + b + pre->r[v][2], acc.get(v, 3) + b + pre->r[v][3]};
                    if (kFused && a.act) o = f4{activate(a, o[0]), activate(a, o[1]), activate(a, o[2]), activate(a, o[3])};
                    io_store4(dst + px.yoff[0], o);
                }
            } else if constexpr (VEC && PV == 2) {
                if (px.valid[0]) {
                    f2 o = f2{acc.get(v, 0) + b + pre->r[v][0], acc.get(v, 1) + b + pre->r[v][1]};
                    if (kFused && a.act) o = f2{activate(a, o[0]), activate(a, o[1])};
                    io_store2(dst + px.yoff[0], o);
                }
            } else {
#pragma unroll
                for (int pv = 0; pv < PV; ++pv)
                    if (px.valid[pv])
                        io_store1(dst + px.yoff[pv], activate(a, acc.get(v, pv) + b + pre->r[v][pv]));
            }
            continue;
        }
        // Y is written once and not read again by this kernel: streaming (non-temporal) stores
        if constexpr (VEC && PV == 4) {
            if (px.valid[0]) {
                f4 o = f4{acc.get(v, 0) + b, acc.get(v, 1) + b, acc.get(v, 2) + b, acc.get(v, 3) + b};
                if (res) o += io_load4(res + px.yoff[0]);
                if (kFused && a.act) o = f4{activate(a, o[0]), activate(a, o[1]), activate(a, o[2]), activate(a, o[3])};
                io_store4(dst + px.yoff[0], o);
            }
        } else if constexpr (VEC && PV == 2) {
            if (px.valid[0]) {
                f2 o = f2{acc.get(v, 0) + b, acc.get(v, 1) + b};
                if (res) o += io_load2(res + px.yoff[0]);
                if (kFused && a.act) o = f2{activate(a, o[0]), activate(a, o[1])};
                io_store2(dst + px.yoff[0], o);
            }
        } else {
#pragma unroll
            for (int pv = 0; pv < PV; ++pv)
                if (px.valid[pv]) {
                    float o = acc.get(v, pv) + b;
                    if (res) o += io_load1(res + px.yoff[pv]);
                    io_store1(dst + px.yoff[pv], activate(a, o));
                }
        }
    }
}

// The group of the lane's slot: a select tree over the record's (scalar) fields by the bits
// of the slot number.  (A loop of "slot == s ? group[s] : g" is turned into an indexed
// array in scratch memory by the compiler for four slots.)
template <int GS>
__device__ __forceinline__ int lane_group(const Work &w, int lane) {
    const int slot = lane >> (6 - ilog2(GS));
    if constexpr (GS == 1) return w.group[0];
    const int g0 = w.group[0], g1 = w.group[1];
    const int lo = (slot & 1) ? g1 : g0;
    if constexpr (GS == 2) return lo;
    const int g2 = w.group[2], g3 = w.group[3];
    const int hi = (slot & 1) ? g3 : g2;
    return (slot & 2) ? hi : lo;
}

// The bias of the V channels of the lane's group (several groups per wavefront: the group
// differs between lanes, so these are vector loads), fetched before the group is multiplied:
// a load issued in the epilogue would be waited for at once, channel after channel, each
// behind the previous channel's store.
template <int V>
struct SlotBias {
    float b[V];
};
template <int V>
__device__ __forceinline__ void load_slot_bias(const ConvArgs &a, int g, SlotBias<V> &sb) {
#pragma unroll
    for (int v = 0; v < V; ++v) {
        sb.b[v] = 0.f;
        if (a.bias && g >= 0 && g * V + v < a.Cout) sb.b[v] = a.bias[g * V + v];
    }
}

// Epilogue with GS groups per wavefront: g is the group of the lane's slot (-1: none).
// In vector form the two pixels of a lane are an 8-byte aligned pair inside one image and
// go out as one store.  The output address is formed once per group and advanced by one
// image plane per channel.
template <int V, int PV, int GS, bool VEC, bool PLAIN = false>
__device__ __forceinline__ void store_slots(const ConvArgs &a, const Acc<V, PV, true> &acc, int g,
                                            const PixOut<PV> &px, const SlotBias<V> &sb) {
    static_assert(PV == 1 || PV == 2, "several groups per wavefront: one or two pixels per lane");
    if (g < 0) return;
    const size_t ch0 = (size_t)g * V * a.P;
#pragma unroll
    for (int v = 0; v < V; ++v) {
        if (g * V + v >= a.Cout) break;
        const size_t plane = ch0 + (size_t)v * a.P;
        const float b = sb.b[v];
        if constexpr (PV == 2 && VEC) {
            if (px.valid[0]) {
                f2 o = f2{acc.get(v, 0) + b, acc.get(v, 1) + b};
                if (residual_of(a)) o += io_load2(residual_of(a) + plane + px.yoff[0]);
                if (kFused && a.act) o = f2{activate(a, o[0]), activate(a, o[1])};
                if constexpr (PLAIN) io_store2_cached(a.Y + plane + px.yoff[0], o);
                else io_store2(a.Y + plane + px.yoff[0], o);
            }
        } else {
#pragma unroll
            for (int pv = 0; pv < PV; ++pv)
                if (px.valid[pv]) {
                    float o = acc.get(v, pv) + b;
                    if (residual_of(a)) o += io_load1(residual_of(a) + plane + px.yoff[pv]);
                    io_store1(a.Y + plane + px.yoff[pv], activate(a, o));
                }
        }
    }
}

// ------------------------------------------------------------------ 1x1 kernels

// Mode 1: all input channels of the pixel tile are resident in LDS (one chunk); each
// wavefront walks through the groups of the workgroup's group tile, longest first.
// The walk is software-pipelined two groups deep: the work record of group k+2 and the
// first run of group k+1 are fetched while group k is multiplied, and always before
// group k's output stores are issued (memory operations retire in order, so a load
// queued behind stores would wait for them).
template <int V, int PV, bool MF, bool VEC, int GS, bool RES, bool CACHED = false>
__device__ __forceinline__ void pw_resident_body(const ConvArgs &a) {
    static_assert(!RES || GS == 1, "residual prefetch: one group per wavefront");
    static_assert(GS == 1 || (MF && PV <= 2), "several groups per wavefront: MFMA form, one or two pixels per lane");
    extern __shared__ float lds[];
    constexpr int TP = 64 * PV / GS;
    constexpr int SH = PV == 4 ? 2 : PV == 2 ? 1 : 0;
    constexpr bool SPLIT = GS > 1 && PV == 2 && !VEC;  // the lane's two pixels are TP/2 apart
    const int logical = logical_wg(a);
    if (logical >= a.total_wgs || skip(a, 8)) return;
    const int pt = logical / a.ngt, gt = logical - pt * a.ngt;
    // the workgroup's pixels [q0, q_end): all TP of the tile, or fewer when the launcher
    // spreads the pixels over more workgroups than full tiles would give (the rest of the
    // tile is staged as zeros and not stored)
    const int q0 = pt * a.tile_px;
    const int q_end = min(a.NP, q0 + a.tile_px);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), nw = blockDim.x >> 6;
    const int g_begin = gt * a.gpt;
    const int ng = min(a.G, g_begin + a.gpt) - g_begin;
    // The wavefront's k-th bundle is entry k*nw + (wave, or mirrored in odd rounds) of
    // the length-sorted list: a snake order that evens out the work per wavefront.
    auto nth = [&](int k) { return k * nw + ((k & 1) ? nw - 1 - wave : wave); };
    const bool any = nth(0) < ng;
    Work w0 = no_work(), w1 = no_work();
    Runs<V, MF, GS> run0, run1;
    if (any) {
        w0 = load_work(a.work, g_begin + nth(0));
        run0 = load_runs<V, MF, GS>(a, w0.start, w0.cnt, lane);
        if (nth(1) < ng) w1 = load_work(a.work, g_begin + nth(1));
    }

#if ALCS_DW_STAGE
    if (!skip(a, 1)) stage_dw<TP, SPLIT>(a, lds, q0, q_end);
#else
    if (!skip(a, 1)) stage_pw<TP, VEC, SPLIT>(a, lds, q0, 0, a.Cin, q_end);
#endif
    // the all-zero row(s) padded columns select: two, one of each channel parity, with several
    // groups per wavefront (the packer picks the one that keeps the slots' reads on different banks)
    for (int t = tid; t < (GS > 1 ? 2 : 1) * TP; t += blockDim.x) lds[a.KC * TP + t] = 0.f;
    __syncthreads();
    if (!any) return;
    touch_runs<V, GS>(run0);  // fetched before the tile was staged: no wait left to inherit inside the walk

    const int plane = lane & (64 / GS - 1);  // the lane's place among the pixels (pairs, quads) of the tile
    PixOut<PV> px;
    pix_out<PV, VEC, SPLIT ? TP / 2 : 0>(a, q0, plane, px, q_end);
    const char *ldsb = reinterpret_cast<const char *>(lds);
    const int base = plane * PV * 4;
    for (int k = 0;; ++k) {
        const bool more = nth(k + 1) < ng;
        Work w2 = no_work();
        if (more) {
            run1 = load_runs<V, MF, GS>(a, w1.start, w1.cnt, lane);
            if (nth(k + 2) < ng) w2 = load_work(a.work, g_begin + nth(k + 2));
        }
        Acc<V, PV, MF> acc;
        acc.zero();
        Resid<V, PV> rr;
        if constexpr (RES) load_residual<V, PV, VEC>(a, w0.group[0], px, rr);
        SlotBias<GS == 1 ? 1 : V> sb;
        int g_lane = w0.group[0];
        if constexpr (GS > 1) {
            g_lane = lane_group<GS>(w0, lane);
            load_slot_bias<V>(a, g_lane, sb);
        }
        if (!skip(a, 2)) mac_segment<V, PV, SH, GS>(a, w0.start, w0.cnt, ldsb, base, lane, run0, acc);
        // the next group's first runs have arrived long ago: take note of that before this
        // group's stores join the queue (see touch_runs)
        if (more) touch_runs<V, GS>(run1);
        if (!skip(a, 4)) {
            if constexpr (GS == 1) store_group<V, PV, MF, VEC>(a, acc, w0.group[0], px, RES ? &rr : nullptr);
            else store_slots<V, PV, GS, VEC, CACHED>(a, acc, g_lane, px, sb);
        }
        if (!more) break;
        w0 = w1;
        w1 = w2;
        run0 = run1;
    }
}

template <int V, int PV, bool MF, bool VEC, int GS>
__global__ void __launch_bounds__(1024) k_pw_resident(const ConvArgs a) {
    pw_resident_body<V, PV, MF, VEC, GS, false>(a);
}
// Four groups per wavefront on pixel pairs, with ordinary instead of streaming stores: for launches
// of several rounds over images whose channel planes do not start on cache lines (14x14, 28x28).
// A tile's runs then cover lines in part, the neighbouring tiles - workgroups next in line, on the
// same L2 - write the rest at about the same time, and the L2 merges them into whole lines
// (512->512 @14x14, N=256, 90 % sparse: 89 -> 81 us; in a single round the streaming stores win).
template <int V>
__global__ void __launch_bounds__(1024) k_pw_resident_cached(const ConvArgs a) {
    pw_resident_body<V, 2, true, true, 4, false, true>(a);
}
// The same walk with every group's residual fetched ahead of its multiply (fused epilogue,
// MFMA and vector form, one group per wavefront).
template <int V, int PV>
__global__ void __launch_bounds__(1024) k_pw_resident_res(const ConvArgs a) {
    pw_resident_body<V, PV, true, true, 1, true>(a);
}

#if !ALCS_RESIDENT_ONLY
// Mode 2: input channels streamed through LDS in chunks of KC; every wavefront owns
// UG groups for the whole kernel and keeps their accumulators in registers.
template <int V, int PV, int UG, bool MF, bool VEC>
__global__ void __launch_bounds__(512) k_pw_chunked(const ConvArgs a) {
    extern __shared__ float lds[];
    constexpr int TP = 64 * PV;
    constexpr int SH = PV == 4 ? 2 : PV == 2 ? 1 : 0;
    const int logical = logical_wg(a);
    if (logical >= a.total_wgs || skip(a, 8)) return;
    const int pt = logical / a.ngt, gt = logical - pt * a.ngt;
    const int q0 = pt * TP;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g_begin = gt * a.gpt;
    const int ng = min(a.G, g_begin + a.gpt) - g_begin;
    const char *ldsb = reinterpret_cast<const char *>(lds);

    int slot[UG];  // position of the wavefront's u-th group in the hand-out order, or -1
    Acc<V, PV, MF> acc[UG];
#pragma unroll
    for (int u = 0; u < UG; ++u) {
        const int idx = wave * UG + u;
        slot[u] = idx < ng ? g_begin + idx : -1;
        acc[u].zero();
    }
    for (int t = tid; t < TP; t += blockDim.x) lds[a.KC * TP + t] = 0.f;
    for (int ch = 0; ch < a.nchunks; ++ch) {
        const int c0 = ch * a.KC, c1 = min(a.Cin, c0 + a.KC);
        // work records and first weight runs of this chunk: fetched ahead of the input rows
        Work wk[UG];
        Runs<V, MF> rn[UG];
#pragma unroll
        for (int u = 0; u < UG; ++u) {
            wk[u] = no_work();
            if (slot[u] >= 0) {
                wk[u] = load_work(a.work, (size_t)slot[u] * a.nchunks + ch);
                rn[u] = load_runs<V, MF>(a, wk[u].start, wk[u].cnt, lane);
            }
        }
        if (ch) __syncthreads();
        if (!skip(a, 1)) stage_pw<TP, VEC>(a, lds, q0, c0, c1, a.NP);
        __syncthreads();
        const int base = lane * PV * 4 - c0 * (kRowBytes1 << SH);
#pragma unroll
        for (int u = 0; u < UG; ++u)
            if (slot[u] >= 0 && !skip(a, 2))
                mac_segment<V, PV, SH>(a, wk[u].start, wk[u].cnt, ldsb, base, lane, rn[u], acc[u]);
    }
    PixOut<PV> px;
    pix_out<PV, VEC>(a, q0, lane, px, a.NP);
#pragma unroll
    for (int u = 0; u < UG; ++u)
        if (slot[u] >= 0 && !skip(a, 4))
            store_group<V, PV, MF, VEC>(a, acc[u], load_work(a.work, (size_t)slot[u] * a.nchunks).group[0], px);
}


// Mode 4 (streaming): for layers whose time is the HBM stream of X and Y.  Workgroups
// are persistent: each owns a contiguous range of the flattened pixel axis (all ranges
// move the same number of bytes) and walks it in tiles of TP pixels.  The input rows of
// tile t+1 are fetched into registers before tile t is multiplied and are written to
// the other LDS buffer afterwards, so loads, MFMAs and stores of one workgroup overlap
// instead of alternating in phases that all workgroups of the chip would share.  The
// packed weights and row selectors of all groups are staged in LDS once per
// workgroup: in the steady state the only vector-memory operations are the input
// prefetch and the output stores (weights fetched from memory would queue behind the
// prefetch, since vector-memory operations return in order).
template <int V, int PV, int NR>
__global__ void __launch_bounds__(512) k_pw_stream(const ConvArgs a) {
    extern __shared__ float lds[];
    constexpr int TP = 64 * PV;
    constexpr int SH = PV == 4 ? 2 : PV == 2 ? 1 : 0;
    constexpr int NQ = TP / 4;
    const int tid = threadIdx.x, lane = tid & 63, nt = blockDim.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), nw = nt >> 6;
    const int q_begin = blockIdx.x * a.ppw;
    const int q_end = min(a.NP, q_begin + a.ppw);
    if (q_begin >= q_end || skip(a, 8)) return;
    const int ntiles = (q_end - q_begin + TP - 1) / TP;
    const int bufstride = (a.Cin + 1) * TP;  // floats per buffer: Cin rows + the all-zero row
    float *wl = lds + 2 * bufstride;
    int32_t *sl = reinterpret_cast<int32_t *>(wl + a.wfloats);

    // stage weights and selectors, clear the two zero rows
    for (int i = tid * 4; i < a.wfloats; i += nt * 4)
        *reinterpret_cast<f4 *>(wl + i) = *reinterpret_cast<const f4 *>(a.w + i);
    for (int i = tid * 4; i < a.nblk; i += nt * 4)
        *reinterpret_cast<i4 *>(sl + i) = *reinterpret_cast<const i4 *>(a.off + i);
    for (int t = tid; t < 2 * TP; t += nt) lds[(t / TP) * bufstride + a.Cin * TP + (t % TP)] = 0.f;

    // this thread's share of a tile: pixel quad `quad`, rows r0, r0 + rpp, ...
    const int quad = tid % NQ, r0 = tid / NQ, rpp = nt / NQ;
    int fq = q_begin + quad * 4;       // first pixel of the quad in the tile being fetched
    int fn = fq / a.P, fp = fq - fn * a.P;
    f4 v[NR];
    auto fetch = [&]() {
        const bool valid = fq < q_end;
        const float *src = a.X + ((size_t)fn * a.Cin) * a.P + fp;
#pragma unroll
        for (int u = 0; u < NR; ++u) {
            const int r = r0 + u * rpp;
            v[u] = f4{0, 0, 0, 0};
            if (valid && r < a.Cin) v[u] = *reinterpret_cast<const f4 *>(src + (size_t)r * a.P);
        }
        fq += TP;
        fp += TP;
        while (fp >= a.P) { fp -= a.P; ++fn; }
    };
    auto commit = [&](int b) {
        float *dst = lds + b * bufstride + quad * 4;
#pragma unroll
        for (int u = 0; u < NR; ++u) {
            const int r = r0 + u * rpp;
            if (r < a.Cin) *reinterpret_cast<f4 *>(dst + r * TP) = v[u];
        }
    };
    if (!skip(a, 1)) { fetch(); commit(0); }
    __syncthreads();

    ConvArgs al = a;   // same arguments, weights and selectors read from LDS
    al.w = wl;
    al.off = sl;
    auto nth = [&](int k) { return k * nw + ((k & 1) ? nw - 1 - wave : wave); };
    const bool any = nth(0) < a.G;
    // where the lane's PV pixels of the current tile go
    int oq = q_begin + lane * PV;
    int on = oq / a.P, op = oq - on * a.P;
    for (int t = 0; t < ntiles; ++t) {
        if (t + 1 < ntiles && !skip(a, 1)) fetch();
        if (any) {
            PixOut<PV> px;
#pragma unroll
            for (int pv = 0; pv < PV; ++pv) {
                px.valid[pv] = oq + pv < q_end;
                px.yoff[pv] = (long long)on * a.Cout * a.P + op + pv;
            }
            const char *ldsb = reinterpret_cast<const char *>(lds + (t & 1) * bufstride);
            const int base = lane * PV * 4;
            Work w0 = load_work(a.work, nth(0)), w1 = no_work();
            if (nth(1) < a.G) w1 = load_work(a.work, nth(1));
            Runs<V, true> run0 = load_runs<V, true>(al, w0.start, w0.cnt, lane), run1;
            for (int k = 0;; ++k) {
                const bool more = nth(k + 1) < a.G;
                Work w2 = no_work();
                if (more) {
                    run1 = load_runs<V, true>(al, w1.start, w1.cnt, lane);
                    if (nth(k + 2) < a.G) w2 = load_work(a.work, nth(k + 2));
                }
                Acc<V, PV, true> acc;
                acc.zero();
                if (!skip(a, 2)) mac_segment<V, PV, SH>(al, w0.start, w0.cnt, ldsb, base, lane, run0, acc);
                if (!skip(a, 4)) store_group<V, PV, true, true>(a, acc, w0.group[0], px);
                if (!more) break;
                w0 = w1;
                w1 = w2;
                run0 = run1;
            }
        }
        oq += TP;
        op += TP;
        while (op >= a.P) { op -= a.P; ++on; }
        if (t + 1 < ntiles && !skip(a, 1)) commit((t + 1) & 1);
        __syncthreads();
    }
}

// ------------------------------------------------------------------ 3x3, tap-shared pattern

// One (group, chunk) of a handle whose kept channels keep all nine taps: one record per kept
// CHANNEL (its chunk-relative index and its 9 x V weights, see alcs_chanrec.hip) instead of one
// column per tap.  The nine LDS reads of a channel differ by compile-time offsets from one
// address, so the per-column selector broadcast and address add of the column-by-column walk
// (one vector instruction for every two matrix instructions) shrink to one v_readlane and one
// add per channel, and a channel's weights are one 256-byte line per plane in block-broadcast
// order (lane 4t + i = tap t, row i: abid = t) instead of nine sixteenths of two runs.
// Measured on this GPU the multiply is bound by the sum of vector and matrix instructions
// issued per SIMD, not by LDS bandwidth: a variant that read each input row once and took the
// left and right taps from the neighbouring lanes (two DPP shifts per row and pixel, halo words
// only in the row's end lanes: 3 + 3 narrow reads instead of 9) was 10-30 % SLOWER than the
// column walk (64->64 @56x56: 91 against 83 us, 256->256 @14x14: 103 against 79), because its
// 24 extra vector instructions per channel cost more than the 6 reads they saved.
template <int V, int STRIDE, int TI, bool TALL>
__device__ __forceinline__ void mac_channels(const ConvArgs &a, int first, int n, const char *ldsb, int lane_byte,
                                             int lane, Acc<V, TALL ? 2 : 1, true> &acc) {
    constexpr int PV = TALL ? 2 : 1;
    constexpr int PD = TALL ? tall_step3(TI) : 1;
    constexpr int PITCH = pitch3(STRIDE, TI);
    constexpr int PLANE = halo_area3(STRIDE, TI, TALL) * 4;
    constexpr int NACC = Acc<V, PV, true>::NACC;
    if (n <= 0) return;
    const float *wp = a.cw + (size_t)first * 64 + lane;
    float wa[V / 4], wb[V / 4];
#pragma unroll
    for (int q = 0; q < V / 4; ++q) wa[q] = wp[(size_t)q * a.cwplane];
    int selv = a.csel[first + min(lane, n - 1)];
    auto channel = [&](int j, const float (&w)[V / 4]) {
        const int crel = __builtin_amdgcn_readlane(selv, j & 63);
        const char *pl = ldsb + lane_byte + crel * PLANE;
        float x[9][PV];
        static_for<9>([&](auto tt) {
            constexpr int T = decltype(tt)::value;
            lds_read<PV, PD>(reinterpret_cast<const float *>(pl + ((T / 3) * PITCH + halo_col3(STRIDE, TI, T % 3)) * 4), x[T]);
        });
        static_for<9>([&](auto tt) {
            constexpr int T = decltype(tt)::value;
#pragma unroll
            for (int q = 0; q < V / 4; ++q)
#pragma unroll
                for (int pv = 0; pv < PV; ++pv)
                    acc.a[T % NACC][q][pv] = __builtin_amdgcn_mfma_f32_4x4x1f32(w[q], x[T][pv], acc.a[T % NACC][q][pv], 4, T, 0);
        });
    };
    for (int j = 0; j < n; j += 2) {
        // the next record's weights are requested before this one is multiplied; beyond the last
        // record the last one is read again
        if ((j & 63) == 0 && j) selv = a.csel[first + j + min(lane, n - j - 1)];
        const float *w1 = wp + (size_t)min(j + 1, n - 1) * 64;
#pragma unroll
        for (int q = 0; q < V / 4; ++q) wb[q] = w1[(size_t)q * a.cwplane];
        channel(j, wa);
        const float *w2 = wp + (size_t)min(j + 2, n - 1) * 64;
#pragma unroll
        for (int q = 0; q < V / 4; ++q) wa[q] = w2[(size_t)q * a.cwplane];
        if (j + 1 < n) channel(j + 1, wb);
    }
}

// ------------------------------------------------------------------ 3x3 kernel

// One workgroup = one TH x TW tile of output pixels of one image (lane = pixel, see the
// tile shapes in alcs_internal.h) and a tile of groups; input channels are streamed in
// chunks of KC, each channel as a haloed plane in the bank-conflict-free layout described
// with halo_col3.  The selector stored with every kept column is
// 4*(c*HA + r*pitch + col(s)), so the tap shift costs nothing at run time.
// TALL (stride 1, MFMA form): the tile has 2*TH rows and a lane owns the pixels (ly, lx) and
// (ly + TH, lx), whose LDS words one ds_read2_b32 fetches together: two MFMAs per LDS
// instruction instead of one, in a kernel whose multiply is bound by its LDS reads.
template <int V, int STRIDE, int TI, int UG, bool MF, bool TALL = false, bool TS = false>
__global__ void __launch_bounds__(512) k_conv3(const ConvArgs a) {
    static_assert(!TALL || (STRIDE == 1 && MF), "tall tiles: stride 1, MFMA form");
    static_assert(!TS || MF, "channel records: MFMA form");
    extern __shared__ float lds[];
    constexpr int PV = TALL ? 2 : 1;
    constexpr int PD = TALL ? tall_step3(TI) : 1;
    constexpr int TW = tile_w3(TI), TH = tile_h3(TI), TROWS = tile_rows3(TI, TALL);
    constexpr int ROWS = halo_rows3(STRIDE, TI, TALL), COLS = halo_cols3(STRIDE, TI);
    constexpr int PITCH = pitch3(STRIDE, TI);
    constexpr int HA = halo_area3(STRIDE, TI, TALL);
    constexpr int HPOS = ROWS * COLS;          // halo positions that are actually loaded
    const int logical = logical_wg(a);
    if (logical >= a.total_wgs || skip(a, 8)) return;
    const int pt = logical / a.ngt, gt = logical - pt * a.ngt;
    const int tiles_per_img = a.tiles_x * a.tiles_y;
    const int n = pt / tiles_per_img, trem = pt - n * tiles_per_img;
    const int tyi = trem / a.tiles_x, txi = trem - tyi * a.tiles_x;
    const int oy0 = tyi * TROWS, ox0 = txi * TW;
    const int iy0 = oy0 * STRIDE - 1, ix0 = ox0 * STRIDE - 1;
    const int tid = threadIdx.x, lane = tid & 63, nt = blockDim.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g_begin = gt * a.gpt;
    const int ng = min(a.G, g_begin + a.gpt) - g_begin;

    const char *ldsb = reinterpret_cast<const char *>(lds);
    int slot[UG];
    Acc<V, PV, MF> acc[UG];
#pragma unroll
    for (int u = 0; u < UG; ++u) {
        const int idx = wave * UG + u;
        slot[u] = idx < ng ? g_begin + idx : -1;
        acc[u].zero();
    }
    for (int t = tid; t < HA; t += nt) lds[a.KC * HA + t] = 0.f;  // the all-zero plane

    const int ly = lane / TW, lx = lane % TW;
    const int lane_base = (ly * STRIDE) * PITCH + lx;
    // staging map: a thread keeps one halo position and walks over the chunk's channels
    // (RPP = nt / HPOS channels are staged side by side); a workgroup with fewer threads
    // than halo positions uses the element loop below instead
    const int rpp = nt / HPOS;
    const int pos = tid % HPOS, r0 = tid / HPOS;
    const int phy = pos / COLS, phx = pos - phy * COLS;
    const bool pin = iy0 + phy >= 0 && iy0 + phy < a.H && ix0 + phx >= 0 && ix0 + phx < a.W;
    const float *psrc = a.X + (size_t)n * a.Cin * a.Pin + (pin ? (size_t)(iy0 + phy) * a.W + ix0 + phx : 0);
    const int pdst = phy * PITCH + halo_col3(STRIDE, TI, phx);
    for (int ch = 0; ch < a.nchunks; ++ch) {
        const int c0 = ch * a.KC, c1 = min(a.Cin, c0 + a.KC);
        // the chunk's work records and first weight runs: fetched before the input tile, so
        // that their latency is covered by the staging (vector memory returns in order)
        Work wk[UG];
        Runs<V, MF> rn[UG];
        int cfirst[UG], cn[UG];
#pragma unroll
        for (int u = 0; u < UG; ++u) {
            wk[u] = no_work();
            cfirst[u] = cn[u] = 0;
            if (slot[u] >= 0) {
                if constexpr (TS) {
                    const cptr<int32_t> cwk = as_const(a.cwork) + 2 * ((size_t)slot[u] * a.nchunks + ch);
                    cfirst[u] = __builtin_amdgcn_readfirstlane(cwk[0]);
                    cn[u] = __builtin_amdgcn_readfirstlane(cwk[1]);
                } else {
                    wk[u] = load_work(a.work, (size_t)slot[u] * a.nchunks + ch);
                    rn[u] = load_runs<V, MF>(a, wk[u].start, wk[u].cnt, lane);
                }
            }
        }
        if (ch) __syncthreads();
        if (skip(a, 1)) {
        } else if (rpp >= 1) {
            if (r0 < rpp) {
                constexpr int U = 8;
                const int rows = c1 - c0;
                int r = r0;
                for (; r + (U - 1) * rpp < rows; r += U * rpp) {
                    float v[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) v[u] = pin ? psrc[(size_t)(c0 + r + u * rpp) * a.Pin] : 0.f;
#pragma unroll
                    for (int u = 0; u < U; ++u) lds[(r + u * rpp) * HA + pdst] = v[u];
                }
                for (; r < rows; r += rpp) lds[r * HA + pdst] = pin ? psrc[(size_t)(c0 + r) * a.Pin] : 0.f;
            }
        } else {
            // element e = (channel row, halo position); a thread's elements are nt apart
            const int total = (c1 - c0) * HPOS;
            constexpr int U = 4;
            for (int e0 = tid; e0 < total; e0 += U * nt) {
                float v[U];
                int dst[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int e = e0 + u * nt;
                    v[u] = 0.f;
                    dst[u] = -1;
                    if (e < total) {
                        const int r = e / HPOS, ps = e - r * HPOS;
                        const int hy = ps / COLS, hx = ps - hy * COLS;
                        const int yy = iy0 + hy, xx = ix0 + hx;
                        dst[u] = r * HA + hy * PITCH + halo_col3(STRIDE, TI, hx);
                        if (yy >= 0 && yy < a.H && xx >= 0 && xx < a.W)
                            v[u] = a.X[((size_t)n * a.Cin + c0 + r) * a.Pin + (size_t)yy * a.W + xx];
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (dst[u] >= 0) lds[dst[u]] = v[u];
            }
        }
        __syncthreads();
        if constexpr (TS) {
#pragma unroll
            for (int u = 0; u < UG; ++u)
                if (slot[u] >= 0 && !skip(a, 2))
                    mac_channels<V, STRIDE, TI, TALL>(a, cfirst[u], cn[u], ldsb, lane_base * 4, lane, acc[u]);
        } else {
            const int base = (lane_base - c0 * HA) * 4;
#pragma unroll
            for (int u = 0; u < UG; ++u)
                if (slot[u] >= 0 && !skip(a, 2)) mac_segment<V, PV, 0, 1, PD>(a, wk[u].start, wk[u].cnt, ldsb, base, lane, rn[u], acc[u]);
        }
    }
    const int oy = oy0 + ly, ox = ox0 + lx;
    PixOut<PV> px;
#pragma unroll
    for (int pv = 0; pv < PV; ++pv) {
        px.valid[pv] = oy + pv * TH < a.Ho && ox < a.Wo;
        px.yoff[pv] = (long long)n * a.Cout * a.P + (long long)(oy + pv * TH) * a.Wo + ox;
    }
#pragma unroll
    for (int u = 0; u < UG; ++u)
        if (slot[u] >= 0 && !skip(a, 4))
            store_group<V, PV, MF, false>(a, acc[u], load_work(a.work, (size_t)slot[u] * a.nchunks).group[0], px);
}


// Mode 5 (pipelined): the many-tile regime of wide 1x1 layers (four groups per wavefront, all
// input channels of a 32-pixel tile in LDS).  With one tile per workgroup the phases of a tile -
// fetch, multiply, store - follow one another, and a launch of several rounds takes the sum of
// them per round: a workgroup slot is busy for the whole chain while each of its resources
// idles most of the time.  Here a workgroup is persistent, owns a run of consecutive tiles and
// keeps two tile buffers: the rows of tile t+1 are requested (into registers) before tile t is
// multiplied and written to the other buffer afterwards, so that memory and matrix pipes work at
// the same time.  Every wavefront multiplies the same (at most KMAX) bundles for every tile, so
// their first weight runs and their bias stay in registers for the whole kernel: in the steady
// state the only vector-memory traffic is the input prefetch and the output stores, and nothing
// in the multiply waits for it.  Per tile: prefetch -> multiply all bundles -> wait for the
// prefetch (requested a whole multiply earlier) -> write it to LDS -> stores -> barrier; the
// stores come last, because the wait that follows a store would include it (one in-order
// counter covers loads and stores).  CACHED: ordinary instead of streaming stores, for images whose
// channel planes do not start on line boundaries (the tile's runs then cover lines in part, and the
// workgroup writes the neighbouring runs with its next tiles: the L2 merges them).
template <int V, bool CACHED, int NT, int KMAX, int NR, bool TAIL>
__global__ void __launch_bounds__(NT) k_pw_pipe(const ConvArgs a) {
    constexpr int GS = 4, PV = 2, TP = 64 * PV / GS, SH = 1;
    extern __shared__ float lds[];
    const int logical = logical_wg(a);
    if (logical >= a.total_wgs) return;
    const int rg = logical / a.ngt, gt = logical - rg * a.ngt;
    // tiles rg, rg + nranges, ...: workgroups that run side by side work on neighbouring tiles, whose
    // rows are neighbours in memory
    const int nranges = a.total_wgs / a.ngt;
    const int t_begin = rg, t_end = a.npt;
    if (t_begin >= t_end) return;
    const int tid = threadIdx.x, lane = tid & 63, nt = blockDim.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), nw = nt >> 6;
    const int g_begin = gt * a.gpt;
    const int ng = min(a.G, g_begin + a.gpt) - g_begin;
    auto nth = [&](int k) { return k * nw + ((k & 1) ? nw - 1 - wave : wave); };
    const int bufstride = (a.KC + 2) * TP;  // floats per buffer: the rows and the two zero rows
    for (int t = tid; t < 2 * 2 * TP; t += nt) lds[(t / (2 * TP)) * bufstride + a.KC * TP + (t % (2 * TP))] = 0.f;
    // the bias behind the two buffers (read back per tile: LDS reads do not join the vector-memory queue)
    float *lbias = lds + 2 * bufstride;
    for (int c = tid; c < a.Cout; c += nt) lbias[c] = a.bias ? a.bias[c] : 0.f;

    // the wavefront's bundles: work records and first weight runs - fetched once
    Work wk[KMAX];
    Runs<V, true, GS> rn[KMAX];
    int g_lane[KMAX];
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
        wk[k] = no_work();
        g_lane[k] = -1;
        if (nth(k) < ng) {
            wk[k] = load_work(a.work, g_begin + nth(k));
            rn[k] = load_runs<V, true, GS>(a, wk[k].start, wk[k].cnt, lane);
            g_lane[k] = lane_group<GS>(wk[k], lane);
        } else {
#pragma unroll
            for (int i = 0; i < Runs<V, true, GS>::N; ++i) {
#pragma unroll
                for (int q = 0; q < (V / 4) * GS; ++q) rn[k].r[i].a[q] = 0.f;
                rn[k].r[i].o = 0;
            }
        }
    }

    // this thread's share of a tile: pixel quad `quad` of rows r0, r0 + rpp, ...
    constexpr int NQ = TP / 4;
    const int quad = tid % NQ, r0 = tid / NQ, rpp = nt / NQ;
    const bool in_tile = quad * 4 < a.tile_px;
    int fq = t_begin * a.tile_px + quad * 4;  // first pixel of the quad in the tile being fetched
    int fn = fq / a.P, fp = fq - fn * a.P;
    // The whole next tile is requested before the current one is multiplied: for its share of the
    // memory bandwidth a compute unit has to keep about 40 KB in flight (latency x bandwidth / 256).
    // Every load is issued, from a clamped address where the quad lies beyond the tile or the row
    // beyond the channels (what such a load brings is never committed or never stored): a
    // register that is loaded on some paths only would make the compiler wait for it where
    // the paths meet, at the top of the loop, behind the previous tile's stores.
    f4 v[NR];
    auto fetch = [&]() {
        const bool valid = in_tile && fq < a.NP;
        const io_t *src = a.X + (valid ? ((size_t)fn * a.Cin) * a.P + fp : (size_t)0);
#pragma unroll
        for (int u = 0; u < NR; ++u) {
            const int r = min(r0 + u * rpp, a.Cin - 1);
            v[u] = io_load4(src + (size_t)r * a.P);
        }
        fq += nranges * a.tile_px;
        fn = fq / a.P;
        fp = fq - fn * a.P;
    };
    auto commit = [&](int b) {
        float *dst = lds + b * bufstride + quad * 4;
#pragma unroll
        for (int u = 0; u < NR; ++u) {
            const int r = r0 + u * rpp;
            if (r < a.Cin) *reinterpret_cast<f4 *>(dst + r * TP) = v[u];
        }
    };
    fetch();
    commit(0);
    if (t_begin + nranges < t_end) fetch();  // the second tile, on its way during the first multiply
#pragma unroll
    for (int k = 0; k < KMAX; ++k) touch_runs<V, GS>(rn[k]);
    __syncthreads();

    // where the lane's pixel pair of the current tile goes
    const int plane = lane & (64 / GS - 1);
    const int base = plane * PV * 4;
    int oq = t_begin * a.tile_px + plane * PV;
    int on = oq / a.P, op = oq - on * a.P;
    const bool lane_in_tile = plane * PV < a.tile_px;
    for (int t = t_begin, it = 0; t < t_end; t += nranges, ++it) {
        const int cur = it & 1;
        const bool more = t + nranges < t_end;
        const char *ldsb = reinterpret_cast<const char *>(lds + cur * bufstride);
        Acc<V, PV, true> acc[KMAX];
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            acc[k].zero();
            mac_segment_keep<V, PV, SH, GS, TAIL>(a, wk[k].start, wk[k].cnt, ldsb, base, lane, rn[k], acc[k]);
        }
        // The registers hold the next tile, requested before the previous tile's stores: the
        // wait for it (taken on every path, see fetch) also covers those stores, which are a whole
        // multiply old.  It goes to the other buffer, and the tile after it is requested at once,
        // ahead of this tile's stores, so that no wait ever follows a fresh store.
#pragma unroll
        for (int u = 0; u < NR; ++u) asm volatile("" : "+v"(v[u]));
        if (more) {
            commit(cur ^ 1);
            if (t + 2 * nranges < t_end) fetch();
        }
        PixOut<PV> px;
        px.valid[0] = px.valid[1] = lane_in_tile && oq < a.NP;
        px.yoff[0] = (long long)on * a.Cout * a.P + op;
        px.yoff[1] = px.yoff[0] + 1;
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            SlotBias<V> sb;
#pragma unroll
            for (int c = 0; c < V; ++c) sb.b[c] = (g_lane[k] >= 0 && g_lane[k] * V + c < a.Cout) ? lbias[g_lane[k] * V + c] : 0.f;
            store_slots<V, PV, GS, true, CACHED>(a, acc[k], g_lane[k], px, sb);
        }
        oq += nranges * a.tile_px;
        on = oq / a.P;
        op = oq - on * a.P;
        __syncthreads();
    }
}

#endif  // !ALCS_RESIDENT_ONLY

// ------------------------------------------------------------------ launcher

constexpr int kMaxLds = 160 * 1024;

static inline int ceil_div(long long a, long long b) { return (int)((a + b - 1) / b); }

typedef void (*kern_t)(const ConvArgs);

template <int V, bool MF>
static kern_t pick_resident(int pv, bool vec, int gs, bool res = false) {
    if constexpr (kFused && !kDw && MF && V <= 8) {
        // with a residual: the variants that fetch it ahead of the multiply (vector form, one
        // group per wavefront, at most 16 values per lane)
        if (res && vec && gs == 1) {
            if constexpr (V * 4 <= 16) {
                if (pv == 4) return k_pw_resident_res<V, 4>;
            }
            if (pv == 2) return k_pw_resident_res<V, 2>;
            if (pv == 1) return k_pw_resident_res<V, 1>;
        }
    }
    if constexpr (MF) {
        if (gs == 2 && pv == 2) return vec ? k_pw_resident<V, 2, true, true, 2> : k_pw_resident<V, 2, true, false, 2>;
        if (gs == 4 && pv == 2) return vec ? k_pw_resident<V, 2, true, true, 4> : k_pw_resident<V, 2, true, false, 4>;
        if (gs == 2) return vec ? k_pw_resident<V, 1, true, true, 2> : k_pw_resident<V, 1, true, false, 2>;
        if (gs == 4) return vec ? k_pw_resident<V, 1, true, true, 4> : k_pw_resident<V, 1, true, false, 4>;
    }
    if (vec) {
        if (pv == 4) return k_pw_resident<V, 4, MF, true, 1>;
        if (pv == 2) return k_pw_resident<V, 2, MF, true, 1>;
        return k_pw_resident<V, 1, MF, true, 1>;
    }
    return k_pw_resident<V, 1, MF, false, 1>;
}

#if !ALCS_RESIDENT_ONLY
template <int V, bool MF>
static kern_t pick_chunked(int pv, bool vec, int ug) {
    if (vec) {
        if (pv == 4) {
            // 4 groups x 4 pixels x 16 channels of accumulators do not fit the register file
            if constexpr (V * 4 * 4 > 128) return k_pw_chunked<V, 4, 2, MF, true>;
            else return ug == 2 ? k_pw_chunked<V, 4, 2, MF, true> : k_pw_chunked<V, 4, 4, MF, true>;
        }
        if (pv == 2) return ug == 2 ? k_pw_chunked<V, 2, 2, MF, true> : k_pw_chunked<V, 2, 4, MF, true>;
        return ug == 2 ? k_pw_chunked<V, 1, 2, MF, true> : k_pw_chunked<V, 1, 4, MF, true>;
    }
    return ug == 2 ? k_pw_chunked<V, 1, 2, MF, false> : k_pw_chunked<V, 1, 4, MF, false>;
}

template <int V, int TI, bool MF>
static kern_t pick_conv3_shape(int stride, int ug, bool tall) {
    if constexpr (MF && V <= 8) {
        if (tall && stride == 1) return ug == 2 ? k_conv3<V, 1, TI, 2, true, true> : k_conv3<V, 1, TI, 4, true, true>;
    }
    if (tall) return nullptr;
    if (ug == 2) return stride == 1 ? k_conv3<V, 1, TI, 2, MF> : k_conv3<V, 2, TI, 2, MF>;
    return stride == 1 ? k_conv3<V, 1, TI, 4, MF> : k_conv3<V, 2, TI, 4, MF>;
}
// channel-record kernels (tap-shared pattern): MFMA form, V = 4 or 8
template <int V, int TI>
static kern_t pick_conv3_shared_shape(int stride, int ug, bool tall) {
    if (tall && stride == 1) return ug == 2 ? k_conv3<V, 1, TI, 2, true, true, true> : k_conv3<V, 1, TI, 4, true, true, true>;
    if (tall) return nullptr;
    if (ug == 2) return stride == 1 ? k_conv3<V, 1, TI, 2, true, false, true> : k_conv3<V, 2, TI, 2, true, false, true>;
    return stride == 1 ? k_conv3<V, 1, TI, 4, true, false, true> : k_conv3<V, 2, TI, 4, true, false, true>;
}
template <int V>
static kern_t pick_conv3_shared(int stride, int ti, int ug, bool tall) {
    if (ti == 2) return pick_conv3_shared_shape<V, 2>(stride, ug, tall);
    if (ti == 1) return pick_conv3_shared_shape<V, 1>(stride, ug, tall);
    return pick_conv3_shared_shape<V, 0>(stride, ug, tall);
}
template <int V, bool MF>
static kern_t pick_conv3(int stride, int ti, int ug, bool tall) {
    if (ti == 2) return pick_conv3_shape<V, 2, MF>(stride, ug, tall);
    if (ti == 1) return pick_conv3_shape<V, 1, MF>(stride, ug, tall);
    return pick_conv3_shape<V, 0, MF>(stride, ug, tall);
}

#endif  // !ALCS_RESIDENT_ONLY

// Tile shape of the 3x3 kernel: the share of lanes that fall on real output pixels decides,
// with a preference for wide tiles (longer contiguous loads and stores).
static int pick_tile3(int Ho, int Wo, int forced_w, bool tall) {
    if (forced_w == 8) return 0;
    if (forced_w == 16) return 1;
    if (forced_w == 32) return 2;
    static const double bonus[kTileShapes3] = {1.0, 1.2, 1.1};  // from sweeps over ResNet-shaped layers
    int best = 0;
    double best_score = 0;
    for (int ti = 0; ti < kTileShapes3; ++ti) {
        const int th = tile_rows3(ti, tall);
        const double covered = (double)ceil_div(Ho, th) * th * ceil_div(Wo, tile_w3(ti)) * tile_w3(ti);
        const double score = (double)Ho * Wo / covered * bonus[ti];
        if (score > best_score) { best_score = score; best = ti; }
    }
    return best;
}

// Groups per wavefront in the chunked kernels: 4, or 2 when the layer has too few groups
// to give every wavefront of a workgroup four of them.
static int pick_ug(int G, int nw, int forced) {
    if (forced == 2 || forced == 4) return forced;
    return G <= 2 * nw ? 2 : 4;
}

// Dynamic LDS above 64 KB has to be allowed per kernel once; remember which kernels
// already have the full 160 KB enabled.
static int set_lds_limit(kern_t k, int lds) {
    if (lds <= 64 * 1024) return ALCS_OK;
    static std::mutex mu;
    static std::set<const void *> done;
    std::lock_guard<std::mutex> lock(mu);
    if (done.count((const void *)k)) return ALCS_OK;
    hipError_t e = hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds);
    if (e != hipSuccess) { set_hip_error((int)e); return ALCS_E_HIP; }
    done.insert((const void *)k);
    return ALCS_OK;
}

// Vector registers per lane of a kernel (0 if the runtime cannot tell), looked up once.
static int kernel_registers(kern_t k) {
    static std::mutex mu;
    static std::map<const void *, int> known;
    std::lock_guard<std::mutex> lock(mu);
    auto it = known.find((const void *)k);
    if (it != known.end()) return it->second;
    hipFuncAttributes attr;
    int regs = 0;
    if (hipFuncGetAttributes(&attr, (const void *)k) == hipSuccess) regs = attr.numRegs;
    else (void)hipGetLastError();
    known[(const void *)k] = regs;
    return regs;
}

#if ALCS_DW_STAGE
}  // namespace dwpw
#elif ALCS_IO_BF16
}  // namespace bf16io
#elif ALCS_FUSED_EPILOGUE
}  // namespace fused
#endif
}  // namespace alcs

using namespace alcs;
#if ALCS_DW_STAGE
using namespace alcs::dwpw;
#elif ALCS_IO_BF16
using namespace alcs::bf16io;
#elif ALCS_FUSED_EPILOGUE
using namespace alcs::fused;
#endif

namespace {
// The depthwise layer in front of the pointwise convolution (depthwise build only).
struct DwStage {
    const float *w, *bias;
    int stride, act;
};
}  // namespace

// With a depthwise stage, H x W is the depthwise layer's input, `stride` its stride, and the
// 1x1 convolution runs at stride 1 over the depthwise layer's output.
static int launch_sparse(const alcs_packed_t *Wp, const io_t *X_dev, const float *bias_dev,
                         io_t *Y_dev, int N, int Cin, int Cout, int H, int W, int kernel,
                         int stride, void *stream, hipEvent_t ev_start, hipEvent_t ev_stop,
                         const io_t *residual_dev = nullptr, int activation = 0,
                         const DwStage *dw = nullptr, bool decline_restaged = false) {
    if (!Wp || N < 0 || H <= 0 || W <= 0) return ALCS_E_INVALID_ARG;
    if (Cin != Wp->Cin || Cout != Wp->Cout || kernel != Wp->k) return ALCS_E_INVALID_ARG;
    if (stride != 1 && stride != 2) return ALCS_E_UNSUPPORTED;
    if (kDw != (dw != nullptr)) return ALCS_E_INVALID_ARG;
    if (dw && (kernel != 1 || !dw->w || dw->act < 0 || dw->act > 2)) return ALCS_E_INVALID_ARG;
    if (N == 0) return ALCS_OK;
    if (!X_dev || !Y_dev) return ALCS_E_INVALID_ARG;
    // four consecutive elements are moved at once: 16-byte (bfloat16: 8-byte) alignment
    if (((uintptr_t)X_dev | (uintptr_t)Y_dev | (uintptr_t)residual_dev) & (4 * sizeof(io_t) - 1)) return ALCS_E_INVALID_ARG;
    if (activation < 0 || activation > 2) return ALCS_E_INVALID_ARG;
    const int pad = dw ? 1 : (kernel - 1) / 2, kin = dw ? 3 : kernel;
    const int Ho = (H + 2 * pad - kin) / stride + 1, Wo = (W + 2 * pad - kin) / stride + 1;
    if (Ho <= 0 || Wo <= 0) return ALCS_E_INVALID_ARG;
    if (dw) stride = 1;  // of the pointwise convolution; the depthwise stride stays in dw->stride
    const long long P = (long long)Ho * Wo, Pin = (long long)H * W;
    if (P > INT32_MAX || Pin > INT32_MAX) return ALCS_E_UNSUPPORTED;
    if ((long double)N * Cin * Pin >= 9e18L || (long double)N * Cout * P >= 9e18L) return ALCS_E_UNSUPPORTED;
    if (!Wp->dev.blob) return ALCS_E_NO_DEVICE;
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) { set_hip_error((int)e); return ALCS_E_HIP; }
    if (cur != Wp->dev.device) return ALCS_E_INVALID_ARG;

    const Layout &L = Wp->lay;
    const Tuning T = tuning_of(Wp->opt);
    const int V = Wp->V, G = Wp->G;
    // compute units and L2 domains (XCDs) of the device the handle lives on
    const int kCUs = Wp->dev.cus, kXcds = Wp->dev.xcds;
    ConvArgs a{};
    a.X = X_dev; a.bias = bias_dev; a.Y = Y_dev;
    a.residual = residual_dev; a.act = activation;
    a.work = Wp->dev.work; a.w = Wp->dev.w;
    a.off = Wp->dev.off[0];
    a.wplane = (long long)L.wplane;
    a.N = N; a.Cin = Cin; a.Cout = Cout; a.H = H; a.W = W; a.Ho = Ho; a.Wo = Wo; a.stride = stride;
    a.P = (int)P; a.Pin = (int)Pin;
    if ((long long)N * P > INT32_MAX - 1024) return ALCS_E_UNSUPPORTED;
    a.NP = (int)((long long)N * P);
    a.G = L.nbundles; a.nchunks = L.nchunks; a.KC = L.KC;  // kernels count bundles of GS groups
    a.debug = ALCS_MEASURE ? Wp->opt.measure_skip : 0;
#if ALCS_DW_STAGE
    a.dw_w = dw->w; a.dw_bias = dw->bias; a.dw_stride = dw->stride; a.dw_act = dw->act;
    a.dw_mode = dw_mode_for(dw->stride, W, X_dev, T.dw_own_taps != 0);
    if (!dw_offsets_fit(Cin, Pin, P)) return ALCS_E_UNSUPPORTED;  // tap offsets are 32-bit
#endif

    bool mfma = V >= 4;
    if (V == 4 && T.path == 1) mfma = false;
    kern_t kern = nullptr;
    int lds = 0, nw = 0, pv = 1, mode = 0, ug = 4, ti = 0;
    long long wg_count = 0;  // workgroups, where that is not pixel tiles x group tiles

    if (kernel == 1) {
        const bool vec = stride == 1 && (P % 4 == 0);
        // streaming kernel: everything (two input tiles, packed weights) fits in LDS and
        // there are enough pixels to give every compute unit several tiles
        bool stream_ok = false;
        int s_pv = 1, s_lds = 0, s_nw = 8, s_nwg = 0;
#if !ALCS_RESIDENT_ONLY
        if (L.nchunks == 1 && L.GS == 1 && vec && mfma && T.path == 4) {
            const long long wbytes = (long long)L.planes * L.ncol * 16 + (long long)L.ncol * 4;
            for (int cand = 4; cand >= 1 && !stream_ok; cand >>= 1) {
                if (T.pv && T.pv != cand) continue;
                const int TPc = 64 * cand;
                const long long need = 2LL * (Cin + 1) * TPc * 4 + wbytes + 64;
                if (need > kMaxLds) continue;
                const int wpc = (int)std::min<long long>(kMaxLds / need, 4);   // workgroups per compute unit
                const int nwg = kCUs * wpc;
                if (a.NP < (long long)nwg * TPc * 2) continue;                 // at least two tiles each
                int nwv = T.waves > 0 ? std::min(T.waves, 8) : (wpc >= 2 ? 4 : 8);
                while (nwv < 8 && (long long)Cin * (TPc / 4) > 8LL * nwv * 64) nwv *= 2;
                if ((long long)Cin * (TPc / 4) > 8LL * nwv * 64) continue;     // more than 8 loads per thread
                stream_ok = true;
                s_pv = cand; s_lds = (int)need; s_nw = nwv; s_nwg = nwg;
            }
        }
        if (stream_ok) {
            mode = 4;
            pv = s_pv; lds = s_lds; nw = s_nw;
            const int TPc = 64 * pv;
            int ppw = (int)(((long long)a.NP + s_nwg - 1) / s_nwg);
            ppw = (ppw + 3) & ~3;
            a.ppw = ppw;
            a.npt = ceil_div(a.NP, ppw);
            a.ngt = 1; a.gpt = G;
            a.wfloats = (int)((long long)L.planes * L.ncol * 4);
            a.nblk = (int)L.ncol;
            (void)TPc;
            switch (V) {
                case 4: kern = pv == 4 ? k_pw_stream<4, 4, 8> : pv == 2 ? k_pw_stream<4, 2, 8> : k_pw_stream<4, 1, 8>; break;
                case 8: kern = pv == 4 ? k_pw_stream<8, 4, 8> : pv == 2 ? k_pw_stream<8, 2, 8> : k_pw_stream<8, 1, 8>; break;
                case 16: kern = pv == 4 ? k_pw_stream<16, 4, 8> : pv == 2 ? k_pw_stream<16, 2, 8> : k_pw_stream<16, 1, 8>; break;
            }
        }
#else
        (void)s_pv; (void)s_lds; (void)s_nw; (void)s_nwg;
#endif
        // pipelined kernel: four groups per wavefront, two tile buffers fit, and every compute unit
        // gets several tiles (else there is nothing to overlap and the resident kernel's single
        // tile per workgroup is the better shape)
        bool pipe_ok = false;
#if !ALCS_RESIDENT_ONLY && !ALCS_FUSED_EPILOGUE
        // (not in the builds with the fused epilogue: its extra registers make this kernel spill)
        if (!stream_ok && L.nchunks == 1 && L.GS == 4 && V == 4 && vec && mfma && T.path != 6 && Cin <= 512 &&
            2LL * (Cin + 2) * 32 * 4 + 4LL * Cout <= kMaxLds) {
            // tiles of 28 pixels where they tile the image exactly and 32 do not (14x14, 28x28)
            const int tp = (P % 32 != 0 && P % 28 == 0) ? 28 : 32;
            const long long tiles = ((long long)a.NP + tp - 1) / tp;
            // 16 wavefronts with at most two bundles each, whose weights (segments of at most 64
            // columns, i.e. four runs) stay in registers for the whole kernel; 128 registers a lane
            // at 16 wavefronts per workgroup hold no more (a variant with 12 wavefronts of three
            // bundles and one with a single temporary both spilled 15-28 registers).
            // Segments of 65 to 96 columns: one bundle per wavefront (twice the group tiles), which
            // leaves registers for the two temporaries of the runs beyond the fourth - on request
            // only ("path" = 5): with every tile staged by two workgroups and loads inside the
            // multiply it is slower than the resident kernel (512->512 @14x14, N=256, 90 % sparse:
            // 91 against 80 us).
            const bool lng = L.max_cnt > 16 * Runs<4, true, 4>::N;
            const int pnw = 16, kmax = lng ? 1 : 2;
            const bool fits = L.max_cnt <= 16 * (Runs<4, true, 4>::N + 2);
            const int ngt_p = ceil_div(L.nbundles, kmax * pnw);
            // (by itself only from 257 input channels on: with fewer, a handle packed with four groups per
            // wavefront on request is faster through the resident kernel - 256->256 @28x28, N=32: 16.6 us
            // against 22.7, 32->64 @112x112: 25 against 54 - the 32-pixel tiles' 128-byte runs cost more
            // than the overlap gains when the multiply is short)
            if (fits && (T.path == 5 || (!lng && Cin > 256 && tiles * ngt_p >= 3LL * kCUs))) {
                pipe_ok = true;
                mode = 5;
                pv = 2; nw = pnw;
                lds = 2 * (Cin + 2) * 32 * 4 + 4 * Cout;
                a.tile_px = tp;
                a.npt = (int)tiles;
                a.gpt = ceil_div(L.nbundles, ngt_p);
                a.ngt = ceil_div(L.nbundles, a.gpt);
                const int ranges = (int)std::max<long long>(1, std::min<long long>(tiles, kCUs / a.ngt));
                wg_count = (long long)ranges * a.ngt;
                const bool cached = ((long long)P * sizeof(io_t)) % 128 != 0;
                // a pass of the workgroup stages 128 rows of 8 pixel quads: four rows per thread
                if (lng) kern = cached ? k_pw_pipe<4, true, 1024, 1, 4, true> : k_pw_pipe<4, false, 1024, 1, 4, true>;
                else kern = cached ? k_pw_pipe<4, true, 1024, 2, 4, false> : k_pw_pipe<4, false, 1024, 2, 4, false>;
            }
        }
#endif
        if (stream_ok || pipe_ok) {
        } else if (L.nchunks == 1) {
            mode = 1;
            // Launch shape, from sweeps over the MobileNet/ResNet-shaped layers on MI355X:
            // pixels per lane - the widest tile whose Cin+1 rows stay below ~68 KB (two
            // workgroups per compute unit) and that still leaves >= 1.5 workgroups per
            // compute unit: wider tiles mean longer contiguous runs for loads and stores.
            constexpr int kTwoPerCu = 68 * 1024;
            const int kMinWgs = 3 * kCUs / 2;
            const int GS = L.GS, NB = L.nbundles;
            if (GS > 1 && !mfma) return ALCS_E_UNSUPPORTED;  // the packer pairs groups only for V >= 4
            pv = 1;
            if (vec && GS == 1) {
                for (int cand = 4; cand >= 2; cand >>= 1) {
                    const long long need = (long long)(Cin + 1) * 64 * cand * 4;
                    const long long tiles = ((long long)a.NP + 64 * cand - 1) / (64 * cand);
                    if (need <= kTwoPerCu && tiles * (cand == 2 ? 2 : 1) >= kMinWgs) { pv = cand; break; }
                }
                // Or a still wider tile with one workgroup per compute unit (up to 160 KB), when
                // pixel tiles x group tiles then make a single round that keeps at least 3/4 of the
                // compute units busy: one wide workgroup beats two narrow ones that share a
                // compute unit (28x28 and 14x14 layers at batch 32: 5-11 % faster).
                for (int cand = 4; cand > pv; cand >>= 1) {
                    const long long need = (long long)(Cin + 1) * 64 * cand * 4;
                    const long long tiles = ((long long)a.NP + 64 * cand - 1) / (64 * cand);
                    if (need > kMaxLds || tiles > kCUs) continue;
                    const long long gts = std::min<long long>(std::max(1, NB / 4), std::max<long long>(1, kCUs / tiles));
                    if (tiles * gts >= 3 * kCUs / 4) { pv = cand; break; }
                }
                if (T.pv == 1 || T.pv == 2 || T.pv == 4) pv = T.pv;
            }
            // Several groups per wavefront: four groups of 16 lanes with a pixel pair each read
            // half as many LDS rows per kept weight as two groups of 32 lanes with one pixel
            // (same 32-pixel tile; 512->512 @14x14: 17.4 -> 15.7 us).
            if (GS > 1) {
                pv = (GS == 4 && (long long)(Cin + 2) * 32 * 4 <= kMaxLds) ? 2 : 1;
                if (T.pv == 1 || T.pv == 2) pv = T.pv;
            }
            const int TP = 64 * pv / GS;
            lds = (Cin + (GS > 1 ? 2 : 1)) * TP * 4;  // the rows and the zero row(s)
            if (lds > kMaxLds) return ALCS_E_UNSUPPORTED;
            a.npt = ceil_div(a.NP, TP);
            a.tile_px = TP;
            // Group tiles: split the bundles over several workgroups only when there are too
            // few pixel tiles (every extra group tile re-stages the pixel tile's rows).  With
            // one resident workgroup per compute unit aim at one round (<= 256 workgroups),
            // else at about 1.5 workgroups per compute unit.
            int ngt = 1;
            const bool one_round = lds > 80 * 1024 || GS > 1;  // narrow tiles: measured best at <= 256 workgroups too
            const int want = one_round ? kCUs : kMinWgs;
            if (a.npt < want) ngt = std::min(std::max(1, NB / 4), std::max(1, one_round ? want / a.npt : ceil_div(want, a.npt)));
            if (T.group_tiles > 0) ngt = std::min(T.group_tiles, NB);
            a.gpt = ceil_div(NB, ngt);
            a.ngt = ceil_div(NB, a.gpt);
            // A single round that would leave compute units idle (196 tiles of 32 pixels for
            // 32 images of 14x14): give every workgroup fewer pixels of its tile instead (a
            // multiple of 4, at least half the tile), so that all compute units share the work
            // (512->512 @14x14: 15.4 -> 14.9 us).  Only with several groups per wavefront, i.e.
            // from 512 input channels on, where the multiply weighs most: on the layers with
            // fewer channels the shorter, less aligned load and store runs cost as much as the
            // idle compute units (256->256 @28x28: 17.0 -> 17.5 us).
            if (GS > 1 && (long long)a.npt * a.ngt < kCUs && !T.full_tiles) {
                const int tiles_wanted = kCUs / a.ngt;
                const int tp = (ceil_div(a.NP, tiles_wanted) + 3) & ~3;
                if (tp < TP && 2 * tp >= TP) {
                    a.tile_px = tp;
                    a.npt = ceil_div(a.NP, tp);
                }
            }
            nw = lds > 40 * 1024 ? 16 : 8;
            // fewer wavefronts when the group tile has fewer bundles, but at least one per 8 KB
            // of tile (4 KB with four groups per wavefront, whose group tiles hold few
            // bundles): wavefronts without a bundle still help to stage it
            nw = std::min(nw, std::max(std::max(1, a.gpt), lds / (GS == 4 ? 4096 : 8192)));
            switch (V) {
                case 1: kern = pick_resident<1, false>(pv, vec, GS); break;
                case 2: kern = pick_resident<2, false>(pv, vec, GS); break;
                case 4: kern = mfma ? pick_resident<4, true>(pv, vec, GS, a.residual != nullptr) : pick_resident<4, false>(pv, vec, GS); break;
                case 8: kern = pick_resident<8, true>(pv, vec, GS, a.residual != nullptr); break;
                case 16: kern = pick_resident<16, true>(pv, vec, GS, a.residual != nullptr); break;
            }
            if (GS == 4 && pv == 2 && vec && mfma && (long long)a.npt * a.ngt > 2LL * kCUs &&
                ((long long)P * sizeof(io_t)) % 128 != 0) {
                switch (V) {
                    case 4: kern = k_pw_resident_cached<4>; break;
                    case 8: kern = k_pw_resident_cached<8>; break;
                    case 16: kern = k_pw_resident_cached<16>; break;
                }
            }
            // A kernel that holds more than 64 registers per lane fits fewer than 32 wavefronts
            // on a compute unit, so two of its 16-wavefront workgroups cannot share one.  With
            // more workgroups than compute units and tiles of which two fit, 8 wavefronts per
            // workgroup let two workgroups overlap their phases (four groups per wavefront, 86
            // registers: 512->128 @28x28, N=64: 55 -> 43 us; 512->512 @14x14, N=256: 97 -> 89 us;
            // 10 or 12 wavefronts measured no better than 16); a single round is faster with 16.
            if (nw > 8 && (long long)a.npt * a.ngt > kCUs && 2 * lds <= kMaxLds && kernel_registers(kern) > 64) nw = 8;
            if (T.waves > 0) nw = std::min(T.waves, 16);
        } else {
#if ALCS_RESIDENT_ONLY
            return ALCS_E_UNSUPPORTED;  // this build holds the resident kernels only
#else
            mode = 2;
            pv = 1;
            if (vec && (T.pv == 2 || T.pv == 4)) pv = T.pv;
            lds = (L.KC + 1) * 64 * pv * 4;
            a.npt = ceil_div(a.NP, 64 * pv);
            nw = 8;
            if (T.waves > 0) nw = std::min(T.waves, 8);
            if (L.GS != 1) return ALCS_E_UNSUPPORTED;
            ug = pick_ug(G, nw, T.ug);
            if (V * pv * ug > 128) ug = 2;  // accumulators of 4 groups would not fit the register file
            a.gpt = nw * ug;
            a.ngt = ceil_div(G, a.gpt);
            switch (V) {
                case 1: kern = pick_chunked<1, false>(pv, vec, ug); break;
                case 2: kern = pick_chunked<2, false>(pv, vec, ug); break;
                case 4: kern = mfma ? pick_chunked<4, true>(pv, vec, ug) : pick_chunked<4, false>(pv, vec, ug); break;
                case 8: kern = pick_chunked<8, true>(pv, vec, ug); break;
                case 16: kern = pick_chunked<16, true>(pv, vec, ug); break;
            }
#endif
        }
    } else {
#if ALCS_RESIDENT_ONLY
        return ALCS_E_UNSUPPORTED;
#else
        mode = 3;
        // Tall tiles (two pixels per lane): stride 1, MFMA form, accumulators of at most 8
        // channels.  By default on images of at least 12x12, which 16- or 8-row tiles
        // still cover well (128->128 @28x28, N=64: 85 -> 71 us; 64->64 @56x56: 85 -> 80 us;
        // 256->256 @14x14: 87 -> 81 us; a 7x7 image would leave most of a tall tile empty:
        // 90 -> 158 us); "pv" = 1 or 2 forces the choice.
        bool tall = stride == 1 && mfma && V <= 8 &&
                    (T.pv == 2 || (T.pv == 0 && Ho >= 12 && Wo >= 12));
        ti = pick_tile3(Ho, Wo, T.tile_w, tall);
        // Handles with channel records (the pattern is shared by the nine taps) and groups of 4 or 8
        // channels walk records instead of columns; "path" = 6 keeps the column-by-column kernel.
        // By default only with tall tiles, where it measures 0-7 % faster (128->128 @28x28, N=64: 71.4
        // -> 66.5 us; 256->256 @14x14: 80.6 -> 78.3; 64->64 @56x56 equal); with one pixel per lane it
        // is slower (512->512 stride 2: 129 -> 157 us), "path" = 7 asks for it anyway.
        if (tall && (L.KC + 1) * halo_area3(stride, ti, true) * 4 > kMaxLds) {
            tall = false;
            ti = pick_tile3(Ho, Wo, T.tile_w, false);
        }
        const bool shared = Wp->dev.cw && mfma && V <= 8 && T.path != 6 && (tall || T.path == 7);
        pv = tall ? 2 : 1;
        a.off = Wp->dev.off[off_table3(stride, ti, tall)];
        lds = (L.KC + 1) * halo_area3(stride, ti, tall) * 4;
        a.tiles_x = ceil_div(Wo, tile_w3(ti));
        a.tiles_y = ceil_div(Ho, tile_rows3(ti, tall));
        a.npt = a.tiles_x * a.tiles_y * N;
        nw = 8;
        if (T.waves > 0) nw = std::min(T.waves, 8);
        ug = pick_ug(G, nw, T.ug);
        // Groups of 8 or 16 channels: two per wavefront (their accumulators fill the register
        // file otherwise; V = 8, 256->256 @14x14, N=64: 103 us with four, 71 with two).
        if (T.ug == 0 && V >= 8) ug = 2;
        // At most one workgroup per compute unit and room for a second one: halve the groups
        // per wavefront, so that two workgroups share a compute unit and one stages a chunk
        // while the other multiplies (512->512 @7x7, N=64: 102 -> 89 us).
        if (T.ug == 0 && ug == 4 && (long long)a.npt * ceil_div(G, nw * 4) <= kCUs && 2 * lds <= kMaxLds) ug = 2;
        a.gpt = nw * ug;
        a.ngt = ceil_div(G, a.gpt);
        switch (V) {
            case 1: kern = pick_conv3<1, false>(stride, ti, ug, tall); break;
            case 2: kern = pick_conv3<2, false>(stride, ti, ug, tall); break;
            case 4: kern = mfma ? pick_conv3<4, true>(stride, ti, ug, tall) : pick_conv3<4, false>(stride, ti, ug, tall); break;
            case 8: kern = pick_conv3<8, true>(stride, ti, ug, tall); break;
            case 16: kern = pick_conv3<16, true>(stride, ti, ug, tall); break;
        }
        if (shared) {
            a.cw = Wp->dev.cw; a.csel = Wp->dev.csel; a.cwork = Wp->dev.cwork; a.cwplane = Wp->dev.cwplane;
            kern = V == 4 ? pick_conv3_shared<4>(stride, ti, ug, tall) : pick_conv3_shared<8>(stride, ti, ug, tall);
            mode = 7;
        }
#endif
    }
    (void)ug; (void)ti; (void)G;
    if (!kern || lds > kMaxLds) return ALCS_E_UNSUPPORTED;
    // Depthwise stage: every group tile of a pixel tile evaluates the depthwise layer again, so
    // a launch that splits the groups is slower than the two layers run one after the other;
    // the caller that can do that (it has a workspace) is told to.
    if (kDw && decline_restaged && a.ngt > 1 && !T.dw_one_kernel) return ALCS_E_UNSUPPORTED;
    const long long total = wg_count > 0 ? wg_count : (long long)a.npt * a.ngt;
    if (total > (1LL << 30)) return ALCS_E_UNSUPPORTED;
    a.total_wgs = (int)total;
    a.xcds = kXcds;
    a.wg_per_xcd = ceil_div(total, kXcds);
    int rc = set_lds_limit(kern, lds);
    if (rc != ALCS_OK) return rc;
    record_launch(mode, pv, nw, a.total_wgs, lds, a.ngt, L.KC, mfma ? 2 : 1, L.GS, (mode == 3 || mode == 7) ? tile_w3(ti) : 0);
    const int grid = mode == 4 ? a.npt : a.wg_per_xcd * kXcds;
    if (ev_start || ev_stop) {
        // the events take the kernel's own begin and end time stamps (no gap for event
        // packets on the stream): for benchmarks that time single launches
        void *kargs[] = {(void *)&a};
        e = hipExtLaunchKernel((const void *)kern, dim3(grid), dim3(nw * 64), kargs, lds, (hipStream_t)stream,
                               ev_start, ev_stop, 0);
    } else {
        hipLaunchKernelGGL(kern, dim3(grid), dim3(nw * 64), lds, (hipStream_t)stream, a);
        e = hipGetLastError();
    }
    if (e != hipSuccess) { set_hip_error((int)e); return ALCS_E_HIP; }
    return ALCS_OK;
}

#if ALCS_DW_STAGE
extern "C" int alcs_dw_sparse_conv_fused(const alcs_packed_t *Wp, const float *dw_weights_dev,
                                         const float *dw_bias_dev, int dw_stride, int dw_activation,
                                         const float *X_dev, const float *bias_dev, const float *residual_dev,
                                         float *Y_dev, float *workspace_dev, int N, int Cin, int Cout, int H,
                                         int W, int activation, void *stream) {
    if (!dw_weights_dev || (dw_stride != 1 && dw_stride != 2)) return ALCS_E_INVALID_ARG;
    if (dw_activation < 0 || dw_activation > 2 || activation < 0 || activation > 2) return ALCS_E_INVALID_ARG;
    const DwStage dw{dw_weights_dev, dw_bias_dev, dw_stride, dw_activation};
    const int rc = launch_sparse(Wp, X_dev, bias_dev, Y_dev, N, Cin, Cout, H, W, 1, dw_stride, stream, nullptr,
                                 nullptr, residual_dev, activation, &dw, workspace_dev != nullptr);
    if (rc != ALCS_E_UNSUPPORTED || !workspace_dev) return rc;
    // Layouts the resident kernels do not cover (input channels streamed in chunks) and layers
    // small enough that the groups are split over several workgroups per pixel tile: the two
    // layers one after the other, the intermediate tensor in the caller's workspace.
    const int rc1 = alcs_depthwise_conv(dw_weights_dev, X_dev, dw_bias_dev, workspace_dev, N, Cin, H, W,
                                        dw_stride, dw_activation, stream);
    if (rc1 != ALCS_OK) return rc1;
    const int Hd = (H - 1) / dw_stride + 1, Wd = (W - 1) / dw_stride + 1;
    return alcs_sparse_conv_fused(Wp, workspace_dev, bias_dev, residual_dev, Y_dev, N, Cin, Cout, Hd, Wd, 1, 1,
                                  activation, stream);
}

#elif ALCS_IO_BF16
extern "C" int alcs_sparse_conv_bf16(const alcs_packed_t *Wp, const uint16_t *X_dev, const float *bias_dev,
                                     const uint16_t *residual_dev, uint16_t *Y_dev, int N, int Cin, int Cout,
                                     int H, int W, int kernel, int stride, int activation, void *stream) {
    return launch_sparse(Wp, X_dev, bias_dev, Y_dev, N, Cin, Cout, H, W, kernel, stride, stream, nullptr, nullptr,
                         residual_dev, activation);
}

#elif !ALCS_FUSED_EPILOGUE
extern "C" int alcs_sparse_conv(const alcs_packed_t *Wp, const float *X_dev, const float *bias_dev,
                                float *Y_dev, int N, int Cin, int Cout, int H, int W, int kernel,
                                int stride, void *stream) {
    return launch_sparse(Wp, X_dev, bias_dev, Y_dev, N, Cin, Cout, H, W, kernel, stride, stream, nullptr, nullptr);
}

extern "C" int alcs_sparse_conv_timed(const alcs_packed_t *Wp, const float *X_dev, const float *bias_dev,
                                      float *Y_dev, int N, int Cin, int Cout, int H, int W, int kernel,
                                      int stride, void *stream, void *start_event, void *stop_event) {
    return launch_sparse(Wp, X_dev, bias_dev, Y_dev, N, Cin, Cout, H, W, kernel, stride, stream,
                         (hipEvent_t)start_event, (hipEvent_t)stop_event);
}

#else
extern "C" int alcs_sparse_conv_fused(const alcs_packed_t *Wp, const float *X_dev, const float *bias_dev,
                                      const float *residual_dev, float *Y_dev, int N, int Cin, int Cout,
                                      int H, int W, int kernel, int stride, int activation, void *stream) {
    return launch_sparse(Wp, X_dev, bias_dev, Y_dev, N, Cin, Cout, H, W, kernel, stride, stream, nullptr, nullptr,
                         residual_dev, activation);
}
#endif
