// Internal declarations shared by the host packer and the HIP launchers.
// Nothing here is part of the public ABI (see include/alcs.h).
#pragma once

#include <cstdint>
#include <mutex>
#include <vector>

#include "alcs.h"

namespace alcs {

// Padding rules of the layout the kernels read: a wavefront fetches the weights of 16
// consecutive kept columns ("a run") with coalesced 256-byte loads, and the inner loop
// runs in branch-free batches of 8 columns.
constexpr int kSegAlign = 16;  // every segment starts at a multiple of 16 columns
constexpr int kCntAlign = 8;   // and its padded length is a multiple of 8 columns

// Geometry of the 3x3 kernels: a TH x TW tile of output pixels per wavefront, TW one of
// 8, 16, 32 ("tile shape" ti = 0, 1, 2) and TH = 64 / TW, lane = TW*ly + lx.  Wide tiles
// give long contiguous runs for the input loads and output stores of wide images; 8x8 has
// the smallest halo and fits small images best.  The tile is staged in LDS with its halo
// of (TH-1)*stride+3 rows and (TW-1)*stride+3 columns, one plane per input channel.  The
// planes are laid out so that the 64 lanes of a read hit distinct LDS banks for every tap
// (for 32 and for 64 banks): the row pitch is chosen so that the lane rows ly land on
// distinct multiples of TW banks,
//   stride 1: halo column hx at hx; lane offset ly*pitch + lx;
//   stride 2: even halo columns first, the odd ones from column odd3 on; lane offset
//             2*ly*pitch + lx; tap column s reads {0, odd3, 1}[s].
constexpr int kTileShapes3 = 3;
inline constexpr int tile_w3(int ti) { return 8 << ti; }
inline constexpr int tile_h3(int ti) { return 8 >> ti; }
// "Tall" tiles (stride 1, MFMA kernels): twice the rows, and a lane owns the pixels (ly, lx) and
// (ly + TH, lx); their LDS words are TH * pitch apart, which one ds_read2_b32 fetches together.
inline constexpr int tile_rows3(int ti, bool tall) { return tall ? 2 * tile_h3(ti) : tile_h3(ti); }
inline constexpr int halo_rows3(int stride, int ti, bool tall = false) { return (tile_rows3(ti, tall) - 1) * stride + 3; }
inline constexpr int halo_cols3(int stride, int ti) { return (tile_w3(ti) - 1) * stride + 3; }
inline constexpr int pitch3(int stride, int ti) {
    return stride == 1 ? (ti == 0 ? 24 : ti == 1 ? 48 : 96) : (ti == 0 ? 28 : ti == 1 ? 40 : 80);
}
inline constexpr int odd3(int ti) { return ti == 0 ? 12 : ti == 1 ? 20 : 40; }
inline constexpr int halo_area3(int stride, int ti, bool tall = false) { return halo_rows3(stride, ti, tall) * pitch3(stride, ti); }
inline constexpr int tall_step3(int ti) { return tile_h3(ti) * pitch3(1, ti); }  // words between a lane's two pixels
inline constexpr int halo_col3(int stride, int ti, int hx) {
    return stride == 1 ? hx : ((hx & 1) ? odd3(ti) + (hx >> 1) : (hx >> 1));
}
// Compile-time proof of the two properties the kernels rely on: the 64 lane offsets of a
// read are distinct modulo 64 (hence also no more than 2 lanes per bank of 32), and the
// farthest read (last lane, last tap) stays inside the plane.
inline constexpr bool layout3_ok(int stride, int ti, bool tall = false) {
    const int tw = tile_w3(ti), pitch = pitch3(stride, ti);
    if (tall && (stride != 1 || tall_step3(ti) > 255)) return false;  // offset field of ds_read2_b32
    bool used[64] = {};
    for (int lane = 0; lane < 64; ++lane) {
        const int o = (lane / tw) * stride * pitch + lane % tw;
        if (used[o % 64]) return false;
        used[o % 64] = true;
    }
    int far = 0;
    for (int s = 0; s < 3; ++s) {
        const int o = (tile_rows3(ti, tall) - 1) * stride * pitch + tw - 1 + 2 * pitch + halo_col3(stride, ti, s);
        far = o > far ? o : far;
    }
    // the staged columns of a row must fit the pitch as well
    int widest = 0;
    for (int hx = 0; hx < halo_cols3(stride, ti); ++hx) {
        const int o = halo_col3(stride, ti, hx);
        widest = o > widest ? o : widest;
    }
    return far < halo_area3(stride, ti, tall) && widest < pitch;
}
static_assert(layout3_ok(1, 0) && layout3_ok(1, 1) && layout3_ok(1, 2) && layout3_ok(2, 0) &&
                  layout3_ok(2, 1) && layout3_ok(2, 2) && layout3_ok(1, 0, true) && layout3_ok(1, 1, true) &&
                  layout3_ok(1, 2, true),
              "3x3 LDS plane layout");
// index of the selector table of a (stride, tile shape, tall) triple, and back
inline constexpr int off_table3(int stride, int ti, bool tall = false) {
    return tall ? 2 * kTileShapes3 + ti : (stride - 1) * kTileShapes3 + ti;
}
constexpr int kMaxOff = 3 * kTileShapes3;
inline constexpr int table_stride3(int table) { return table / kTileShapes3 == 1 ? 2 : 1; }
inline constexpr int table_ti3(int table) { return table % kTileShapes3; }
inline constexpr bool table_tall3(int table) { return table / kTileShapes3 == 2; }

// Bytes per LDS row that the stored 1x1 row selectors assume with one group per
// wavefront (a 64-pixel fp32 tile); with GS groups per wavefront the tile has 64/GS
// pixels and the selectors are scaled down accordingly.  Kernels with 2 or 4 pixels
// per lane scale the selector up by that factor.
constexpr int kRowBytes1 = 256;

constexpr int kMaxSlots = 4;

// Host and device code alike (the layout is built by alcs_pack.cpp on the host and by
// alcs_layoutdev.hip on the device, to the same bytes).
#if defined(__HIPCC__) || defined(__HIP__)
#define ALCS_HD __host__ __device__
#else
#define ALCS_HD
#endif

// LDS row selector (a byte offset) of the block at canonical column `col`, see Layout::off.
ALCS_HD inline int32_t layout_off_of(int col, int k, int table, int GS) {
    if (k == 1) return col * (kRowBytes1 / GS);
    const int c = col / 9, tap = col % 9, r = tap / 3, s = tap % 3;
    const int stride = table_stride3(table), ti = table_ti3(table);
    return (c * halo_area3(stride, ti, table_tall3(table)) + r * pitch3(stride, ti) + halo_col3(stride, ti, s)) * 4;
}
// Selector of a padded column: an all-zero row behind the chunk's rows.  Layouts with several
// groups per wavefront have two of them (rows KC and KC + 1, one of each channel parity);
// `which` picks one.
ALCS_HD inline int32_t layout_pad_off(int c0, int KC, int k, int table, int GS, int which) {
    if (k == 1) return (c0 + KC + which) * (kRowBytes1 / GS);
    return (c0 + KC) * halo_area3(table_stride3(table), table_ti3(table), table_tall3(table)) * 4;
}
// Index of (padded column `col` counted from the start of the arrays, slot s) in a weight plane
// (row i) and in a selector table; VV = min(V, 4).
ALCS_HD inline size_t layout_w_index(int GS, int VV, int64_t col, int s, int i) {
    const int cpa = 16 / GS;
    const int64_t R = col / 16 * 16;
    const int c = (int)(col % 16);
    if (VV < 4) return (size_t)(col * VV + i);  // V < 4: GS == 1, VV floats per column
    return (size_t)(R * 4 * GS + (c / cpa) * 64 + s * (64 / GS) + (c % cpa) * 4 + i);
}
ALCS_HD inline size_t layout_off_index(int GS, int64_t col, int s) {
    const int64_t R = col / 16 * 16;
    return (size_t)(R * GS + s * 16 + col % 16);
}

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
    int max_cnt = 0;  // longest segment, in padded columns
    int64_t ncol = 0; // padded columns in total (multiple of kSegAlign)
    int64_t wplane = 0;  // floats per weight plane: ncol * VV * GS
    int noff = 0;     // 1 for kernel 1; kMaxOff for kernel 3 (one table per stride and tile shape)
    // kernel 3: every kept input channel of every group keeps all nine taps (the per-channel
    // pattern copied to the taps); such handles also get channel records on the device
    bool tap_shared = false;
    std::vector<float> w;          // [planes][wplane]
    std::vector<int32_t> off[kMaxOff];   // [ncol * GS] each; LDS row selector of every block, in bytes:
                                   //   kernel 1: c * kRowBytes1 / GS        (pad: (c0 + KC) * kRowBytes1 / GS)
                                   //   kernel 3: 4*(c*HA + r*pitch + col(s)) (pad: 4*(c0 + KC)*HA), see halo_col3
                                   // with c the input channel and c0 the first channel of the block's chunk
    std::vector<int32_t> order;    // [G] groups by descending kept-column count
    std::vector<Work> work;        // [nbundles * nchunks], index b * nchunks + chunk
};

struct DeviceCopy {
    int device = -1;
    int cus = 0, xcds = 0;  // compute units and XCDs (L2 domains) of that device, from its properties
    void *blob = nullptr;
    size_t bytes = 0;
    const Work *work = nullptr;
    const float *w = nullptr;
    const int32_t *off[kMaxOff] = {};
    // handles built on the device (alcs_pack_from_csr_device) also keep, in the same blob, the
    // group order and the canonical arrays, which the host fetches only when it is asked for them
    const int32_t *order = nullptr, *row_ptr = nullptr, *col_idx = nullptr;
    const float *vals = nullptr;
    // the 16-bit layout made by alcs_packed_add_bf16_weights (null before; one allocation of its own
    // that starts at w16): weight planes rounded to bfloat16 in the order of the 16-bit matrix
    // instruction, row selectors for 256-byte rows, one work record per group
    const uint16_t *w16 = nullptr;
    const int32_t *off16 = nullptr;
    const Work *work16 = nullptr;
    // Channel records of a tap-shared 3x3 handle (an allocation of its own, null otherwise): per
    // (bundle, chunk) the first record and the number of records (cwork, two ints), per record the
    // chunk-relative input channel (csel) and, in each plane of cwplane floats, 64 weights
    // [tap 0..15][row 0..3] of which taps 9..15 are zero (cw).
    void *chan_blob = nullptr;
    const float *cw = nullptr;
    const int32_t *csel = nullptr, *cwork = nullptr;
    long long cwplane = 0;
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
    alcs_options opt = {};  // the options given at pack time / by alcs_packed_set_options; zero = automatic
    // Built on the device: the vectors above (canonical arrays, layout arrays) are empty until
    // alcs_packed_export / alcs_packed_selfcheck ask for them (host_arrays, under host_mu).
    bool host_arrays = true;
    std::mutex host_mu;
};

namespace alcs {

void set_hip_error(int e);
// Compute units and XCDs (L2 domains; workgroups are dealt to them round-robin) of a device,
// from its properties; looked up once per device and process (constants of the hardware).
void device_shape(int device, int *cus, int *xcds);
int current_device_shape(int *cus, int *xcds);  // of the current device; ALCS_OK or ALCS_E_HIP
int check_options(const alcs_options *o);  // ALCS_OK or ALCS_E_INVALID_ARG
// alcs_pack_from_csr with the handle's options (null = automatic)
int pack_from_csr_host(const int32_t *row_ptr_host, const int32_t *col_idx_host, const float *vals_host, int Cout,
                       int Cin, int kernel, int V, const alcs_options *options, alcs_packed_t **out);
int build_layout(alcs_packed *p, int KC, int GS);
// tile policy: channels per chunk and groups per wavefront of a handle, from its shape and options
void choose_tiles(const alcs_packed *p, int *KC, int *GS);
// canonical arrays and layout arrays of a handle built on the device, fetched to the host (once)
int fetch_host_arrays(alcs_packed *p);
int upload(alcs_packed *p);
// alcs_chanrec.hip: builds the channel records of a tap-shared 3x3 handle from its device arrays
// (kernels on `stream`, a hipStream_t; no wait); does nothing for other handles
int add_channel_records(alcs_packed *p, void *stream);
void release_device(alcs_packed *p);

// The launch options of a handle in the launchers' short names.
struct Tuning {
    int pv = 0, waves = 0, group_tiles = 0, path = 0, ug = 0, tile_w = 0;
    int dw_own_taps = 0, dw_one_kernel = 0, full_tiles = 0;
};
inline Tuning tuning_of(const alcs_options &o) {
    Tuning t;
    t.pv = o.pixels_per_lane; t.waves = o.waves; t.group_tiles = o.group_tiles; t.path = o.path;
    t.ug = o.groups_per_wave;
    t.tile_w = (o.tile_width == 8 || o.tile_width == 16 || o.tile_width == 32) ? o.tile_width : 0;
    t.dw_own_taps = o.dw_own_taps; t.dw_one_kernel = o.dw_one_kernel; t.full_tiles = o.full_tiles;
    return t;
}
void record_launch(int mode, int pv, int waves, int wgs, int lds, int gtiles, int kc, int path, int gs,
                   int tile_w);

}  // namespace alcs
