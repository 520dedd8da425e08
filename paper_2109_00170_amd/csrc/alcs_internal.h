// Internal declarations shared by the host packer and the HIP launchers.
// Nothing here is part of the public ABI (see include/alcs.h).
#pragma once

#include <cstdint>
#include <vector>

#include "alcs.h"

namespace alcs {

// Padding rules of the layout the kernels read: a wavefront fetches the weights of 16
// consecutive kept columns ("a run") with coalesced 256-byte loads, and the inner loop
// runs in branch-free batches of 8 columns.
constexpr int kSegAlign = 16;  // every segment starts at a multiple of 16 columns
constexpr int kCntAlign = 8;   // and its padded length is a multiple of 8 columns

// Geometry of the 3x3 kernels: an 8x8 tile of output pixels per wavefront (lane =
// 8*ly + lx), staged in LDS with its halo of (8-1)*stride+3 rows and columns, one
// plane per input channel.  The planes are laid out so that the 64 lanes of a read hit
// distinct LDS banks for every tap (true for 32 and for 64 banks):
//   stride 1: row pitch 24 floats, halo column hx at hx; lane offset ly*24 + lx;
//   stride 2: row pitch 28 floats, the 9 even halo columns at [0, 9) and the 8 odd ones
//             at [12, 20); lane offset 2*ly*28 + lx; tap column s reads {0, 12, 1}[s].
constexpr int kTile3 = 8;
constexpr int kOdd3 = 12;
inline constexpr int halo_rows3(int stride) { return (kTile3 - 1) * stride + 3; }
inline constexpr int pitch3(int stride) { return stride == 1 ? 24 : 28; }
inline constexpr int halo_area3(int stride) { return halo_rows3(stride) * pitch3(stride); }
inline constexpr int halo_col3(int stride, int hx) {
    return stride == 1 ? hx : ((hx & 1) ? kOdd3 + (hx >> 1) : (hx >> 1));
}

// Bytes per LDS row that the stored 1x1 row selectors assume with one group per
// wavefront (a 64-pixel fp32 tile); with GS groups per wavefront the tile has 64/GS
// pixels and the selectors are scaled down accordingly.  Kernels with 2 or 4 pixels
// per lane scale the selector up by that factor.
constexpr int kRowBytes1 = 256;

constexpr int kMaxSlots = 4;

// What a wavefront needs to process one bundle of GS groups inside one channel chunk.
// Bundles are formed from the groups sorted by descending kept-column count (slot s of
// bundle b is the (b*GS+s)-th longest group) and handed out in that order.
struct Work {
    int32_t start;             // first padded column of the segment (multiple of kSegAlign)
    int32_t cnt;               // padded number of columns to process (multiple of kCntAlign, may be 0)
    int32_t group[kMaxSlots];  // output-channel group of every slot, -1 for an unused slot
    int32_t reserved[2];
};

// The layout the kernels read ("tuned layout").  Input channels are cut into chunks
// of KC channels; the kept columns of a group are ascending in c, so each
// (group, chunk) pair owns a contiguous run of the group's columns = one segment.
// With GS > 1 the segments of the GS groups of a bundle are padded to a common length
// and interleaved, so that one wavefront multiplies GS groups at once, each on 64/GS
// pixels (lanes [s*64/GS, (s+1)*64/GS) belong to slot s).
//
// Addressing, for bundle column j (0-based inside the segment), slot s, weight row
// 4q+i, with R = (start + j) / 16 * 16 the first column of j's run, c = j % 16 and
// CPA = 16 / GS columns per weight register:
//   weight    w[q * wplane + R*4*GS + (c / CPA)*64 + s*(64/GS) + (c % CPA)*4 + i]
//   selector  off[t][R*GS + s*16 + c]
// which for GS = 1 is w[q*wplane + (start+j)*VV + i] and off[t][start + j].
struct Layout {
    int KC = 0;       // input channels per chunk (the LDS tile holds KC rows + 1 zero row)
    int nchunks = 0;  // ceil(Cin / KC)
    int GS = 1;       // groups per wavefront (1, 2 or 4); > 1 only with V >= 4, kernel 1, one chunk
    int nbundles = 0; // ceil(G / GS)
    int planes = 0;   // ceil(V / 4): weight rows 4q..4q+3 of every block live in plane q
    int VV = 0;       // min(V, 4) floats per block and plane
    int64_t ncol = 0; // padded columns in total (multiple of kSegAlign)
    int64_t wplane = 0;  // floats per weight plane: ncol * VV * GS
    int noff = 0;     // 1 for kernel 1; 2 for kernel 3 (stride 1, stride 2 geometry)
    std::vector<float> w;          // [planes][wplane]
    std::vector<int32_t> off[2];   // [ncol * GS] each; LDS row selector of every block, in bytes:
                                   //   kernel 1: c * kRowBytes1 / GS        (pad: (c0 + KC) * kRowBytes1 / GS)
                                   //   kernel 3: 4*(c*HA + r*pitch + col(s)) (pad: 4*(c0 + KC)*HA), see halo_col3
                                   // with c the input channel and c0 the first channel of the block's chunk
    std::vector<int32_t> order;    // [G] groups by descending kept-column count
    std::vector<Work> work;        // [nbundles * nchunks], index b * nchunks + chunk
};

struct DeviceCopy {
    int device = -1;
    void *blob = nullptr;
    size_t bytes = 0;
    const Work *work = nullptr;
    const float *w = nullptr;
    const int32_t *off[2] = {nullptr, nullptr};
};

}  // namespace alcs

struct alcs_packed {
    int Cout = 0, Cin = 0, k = 0, V = 0, G = 0, K = 0;
    int64_t nnzb = 0;
    int max_count = 0;
    // canonical grouped CSR (Section 3.2.2 of the paper)
    std::vector<int32_t> row_ptr, col_idx;
    std::vector<float> vals;
    alcs::Layout lay;
    alcs::DeviceCopy dev;
};

namespace alcs {

void set_hip_error(int e);
int build_layout(alcs_packed *p, int KC, int GS);
int upload(alcs_packed *p);
void release_device(alcs_packed *p);

struct Tuning {
    int pv = 0, waves = 0, group_tiles = 0, path = 0, kc = 0, ug = 0, debug = 0, gs = 0;
};
Tuning &tuning();
void record_launch(int mode, int pv, int waves, int wgs, int lds, int gtiles, int kc, int path, int gs);

}  // namespace alcs
