// The nine taps of a depthwise 3x3 filter (zero padding 1) for lanes that hold consecutive
// output pixels of one row-major (ho, wo) plane - shared by the stand-alone depthwise kernel
// and by the depthwise stage of the fused block kernels.
//
// What these loops are bound by is instruction issue, not bytes: a wavefront instruction
// occupies its SIMD for four cycles, so every per-tap select, address add or branch costs as
// much as the multiply-add itself.  Hence:
//   - a tap is addressed as wave-uniform base (scalar registers) + 32-bit byte offset of the
//     lane, worked out once per pixel and reused for every channel: no address arithmetic in
//     the channel loop (the host checks that the offsets fit 32 bits);
//   - taps outside the image are loaded anyway, from the nearest pixel inside it (so that a
//     lane still reads next to its neighbours and the load coalesces as before), and replaced
//     by zero with one select: no branch around the load;
//   - stride 2 with an even input width: taps 1 and 2 of a row are one aligned 8-byte load
//     and tap 0 is tap 2 of the lane to the left, moved with the DPP wavefront shift
//     (wave_shr:1: lane i reads lane i-1 across all 64 lanes, inside the vector ALU); the
//     first lane of a span fetches that tap itself.  The source lane has to be active, so
//     callers keep out-of-range pixels in the loop and mask them (valid).
// At stride 1 the same sharing (centre taps loaded, left / right taken from the neighbours)
// was measured slower than nine loads: the selects it adds cost more than the loads it saves.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace alcs {

typedef float dw_f2 __attribute__((ext_vector_type(2)));

enum DwMode { kDwNine = 0, kDwPair = 1 };

// Stride 2 shares taps when the input width is even and the input tensor 8-byte aligned.
inline int dw_mode_for(int stride, int W, const void *X, bool force_nine = false) {
    if (!force_nine && stride == 2 && (W % 2) == 0 && (((uintptr_t)X) & 7) == 0) return kDwPair;
    return kDwNine;
}

// The value lane - 1 holds (lane 0 gets 0).
__device__ __forceinline__ float from_prev_lane(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x138, 0xf, 0xf, false));
}

// SPAN: lanes that hold consecutive pixels of the flattened (n, ho, wo) axis (16, 32 or 64).
template <int MODE, int SPAN>
struct DwTaps {
    // kDwNine: flag and byte offset of every tap.  kDwPair: per row, flag and byte offset of
    // the 8-byte pair (taps 1, 2); tap 0 comes from the left neighbour or from `eoff`.
    bool ok[MODE == kDwNine ? 9 : 3];
    uint32_t boff[MODE == kDwNine ? 9 : 3];
    uint32_t eoff[3];
    bool hasl, el, eact;

    struct Raw {
        float x[9];   // kDwNine: the taps; kDwPair: x[3r] = own fetch of tap 0, x[3r+1], x[3r+2] = the pair
    };

    // `delta` = element offset of the lane's plane from the wave-uniform base the loads use.
    __device__ __forceinline__ void init(bool valid, long long delta, int ho, int wo, int H, int W, int stride,
                                         int lane) {
        const uint32_t d = (uint32_t)delta;
        if constexpr (MODE == kDwNine) {
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int t = 0; t < 3; ++t) {
                    const int hi = ho * stride - 1 + r, wi = wo * stride - 1 + t;
                    ok[r * 3 + t] = valid && hi >= 0 && hi < H && wi >= 0 && wi < W;
                    const int hc = min(max(hi, 0), H - 1), wc = min(max(wi, 0), W - 1);
                    boff[r * 3 + t] = (d + (uint32_t)(hc * W + wc)) * 4u;
                }
        } else {
            hasl = wo > 0;
            el = (lane & (SPAN - 1)) == 0;
            eact = el && hasl;
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                const int hi = ho * 2 - 1 + r;
                ok[r] = valid && hi >= 0 && hi < H;
                const uint32_t at = d + (uint32_t)(min(max(hi, 0), H - 1) * W + wo * 2);
                boff[r] = at * 4u;
                eoff[r] = (eact ? at - 1u : at) * 4u;
            }
        }
    }

    // `base`: wave-uniform pointer; every offset formed in init() is in bounds of the tensor.
    __device__ __forceinline__ void load(const float *base, Raw &v) const {
        const char *b = reinterpret_cast<const char *>(base);
        if constexpr (MODE == kDwNine) {
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                // The empty statement keeps the 32-bit offset a 32-bit register here (otherwise its
                // zero extension is hoisted out of the channel loop and every load needs a 64-bit
                // vector add): the load then takes the scalar base + vector offset form.
                uint32_t o = boff[t];
                asm volatile("" : "+v"(o));
                v.x[t] = *reinterpret_cast<const float *>(b + o);
            }
        } else {
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                uint32_t o = boff[r];
                asm volatile("" : "+v"(o));  // as above: scalar base + 32-bit vector offset
                const dw_f2 p = *reinterpret_cast<const dw_f2 *>(b + o);
                v.x[r * 3 + 1] = p.x;
                v.x[r * 3 + 2] = p.y;
            }
            // tap 0 of the span's first lane: the only lanes that fetch it themselves
#pragma unroll
            for (int r = 0; r < 3; ++r) v.x[r * 3] = 0.f;
            if (eact) {
#pragma unroll
                for (int r = 0; r < 3; ++r) v.x[r * 3] = *reinterpret_cast<const float *>(b + eoff[r]);
            }
        }
    }

    // bias + sum of the nine taps in the order (r, t) ascending; w is the channel's filter.
    template <class WT>
    __device__ __forceinline__ float apply(const Raw &v, WT w, float bias) const {
        float acc = bias;
        if constexpr (MODE == kDwNine) {
#pragma unroll
            for (int t = 0; t < 9; ++t) acc = fmaf(w[t], ok[t] ? v.x[t] : 0.f, acc);
        } else {
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                const float c0 = ok[r] ? v.x[r * 3 + 1] : 0.f, c1 = ok[r] ? v.x[r * 3 + 2] : 0.f;
                float l = from_prev_lane(c1);
                l = el ? v.x[r * 3 + 0] : l;
                l = (hasl && ok[r]) ? l : 0.f;
                acc = fmaf(w[r * 3 + 0], l, acc);
                acc = fmaf(w[r * 3 + 1], c0, acc);
                acc = fmaf(w[r * 3 + 2], c1, acc);
            }
        }
        return acc;
    }
};

// Whether 32-bit byte offsets reach every tap: a wavefront's lanes lie in at most
// 63 / P + 2 consecutive images and (in the fused kernels) up to 4 channels side by side.
inline bool dw_offsets_fit(long long Cin, long long Pin, long long P) {
    const long double span = ((long double)(63 / P + 1) * Cin + 4) * Pin * 4;
    return span < 4.0e9L;
}

}  // namespace alcs
