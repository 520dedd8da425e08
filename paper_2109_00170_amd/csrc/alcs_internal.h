// Internal declarations shared by the host packer and the HIP launchers.
// Nothing here is part of the public ABI (see include/alcs.h).
#pragma once

#include <cstdint>
#include <vector>

#include "alcs.h"

namespace alcs {

// Blocks are padded so that a wavefront can fetch the weights of 16 consecutive kept
// columns of one group with a single coalesced 256-byte load, and so that the inner
// loop can run in branch-free batches of 8 columns without a remainder.
constexpr int kSegAlign = 16;  // every (group, chunk) segment starts at a multiple of 16 blocks
constexpr int kCntAlign = 8;   // and its padded length is a multiple of 8 blocks

// Geometry of the 3x3 kernels: an 8x8 tile of output pixels per wavefront, staged in
// LDS with its halo, one plane of kHalo*kHalo floats per input channel.
constexpr int kTile3 = 8;
inline constexpr int halo3(int stride) { return (kTile3 - 1) * stride + 3; }

// Bytes per LDS row that the stored 1x1 row selectors assume (a 64-pixel fp32 tile);
// kernels with 2 or 4 pixels per lane scale the selector by that factor.
constexpr int kRowBytes1 = 256;

struct Seg {
    int32_t start;  // first padded block of the segment (multiple of kSegAlign)
    int32_t cnt;    // padded number of blocks to process (multiple of kCntAlign, may be 0)
};

// What a wavefront needs to process one (group, chunk) pair, in the order the kernels
// hand out work: groups by descending kept-column count.
struct Work {
    int32_t start, cnt, group, reserved;
};

// The layout the kernels read ("tuned layout").  Input channels are cut into chunks
// of KC channels; the kept columns of a group are ascending in c, so each
// (group, chunk) pair owns a contiguous run of the group's columns = one segment.
struct Layout {
    int KC = 0;       // input channels per chunk (the LDS tile holds KC rows + 1 zero row)
    int nchunks = 0;  // ceil(Cin / KC)
    int planes = 0;   // ceil(V / 4): weight rows 4q..4q+3 of every block live in plane q
    int VV = 0;       // min(V, 4) floats per block and plane
    int64_t nblk = 0; // padded blocks in total (multiple of kSegAlign)
    int noff = 0;     // 1 for kernel 1; 2 for kernel 3 (stride 1, stride 2 geometry)
    std::vector<Seg> seg;          // [G * nchunks], index g * nchunks + chunk
    std::vector<float> w;          // [planes][nblk * VV]
    std::vector<int32_t> off[2];   // [nblk] each; LDS row selector of every block, in bytes:
                                   //   kernel 1: c * kRowBytes1             (pad: (c0 + KC) * kRowBytes1)
                                   //   kernel 3: 4*(c*HA + r*halo + s)      (pad: 4*(c0 + KC)*HA)
                                   // with c the input channel and c0 the first channel of the block's chunk
    std::vector<int32_t> order;    // [G] groups by descending kept-column count
    std::vector<Work> work;        // [G * nchunks], index i * nchunks + chunk for the i-th group of `order`
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
int build_layout(alcs_packed *p, int KC);
int upload(alcs_packed *p);
void release_device(alcs_packed *p);

struct Tuning {
    int pv = 0, waves = 0, group_tiles = 0, path = 0, kc = 0, ug = 0, debug = 0;
};
Tuning &tuning();
void record_launch(int mode, int pv, int waves, int wgs, int lds, int gtiles, int kc, int path);

}  // namespace alcs
