// Host-side plan: the layer-wise representation after filter kernel reorder, and the packed
// device streams built from it (paper section 2.3.1, "Filter Kernel Reorder and Compact
// Filter-Kernel-Weight (FKW) Storage").  No HIP types here.
#pragma once

#include <cstdint>
#include <vector>

#include "pp_conv.h"

namespace ppc {

// The sixteen tap masks the tiled kernel has specialised code for (slot = index).  A layer
// whose pattern table uses only these masks runs on the tiled kernel; any other table runs on
// the generic kernel.  Slots 0-7: T shapes and centre-holding 2x2 blocks; 8-15: diagonal and
// mixed shapes.  The paper prints no pattern set; this one is the library's own.
constexpr int kBuiltinPatterns = 16;
constexpr uint16_t kBuiltinMasks[kBuiltinPatterns] = {0x03A, 0x0B2, 0x0B8, 0x09A, 0x01B, 0x036, 0x0D8, 0x1B0,
                                                      0x055, 0x115, 0x151, 0x154, 0x152, 0x11C, 0x071, 0x095};

// Weight-stream entry: word 0 is the kernel's code = local filter slot * NP + pattern slot, or
// kEndCode for the end of this wavefront's work in the current channel chunk; the channel word is
// kSameChannel, or, on the first kernel of an input channel, the byte offset of that channel's
// tile inside the LDS chunk buffer (place in chunk * channel stride): reload the lane's window.
constexpr uint32_t kEndCode = 0x00FFFFFFu;
constexpr uint32_t kSameChannel = 0xFFFFFFFFu;

struct Canonical {          // tuning-independent result of the reorder
    std::vector<int32_t> perm, kcount, pat_off, kidx;
    std::vector<uint8_t> kpat;
    std::vector<float> wpacked;
    int64_t k_kept = 0;
};

struct TiledLayout {        // geometry of the tiled kernel for one plan
    int np = 0;             // pattern slots compiled in (8 or 16)
    int f = 0, r = 0, lw = 0, wf = 0, ks = 0, cc = 0;
    int mode = 0;           // input staging: 0 through registers, 1 direct loads in 16-byte slots, 2 in 4-byte slots
    int nbuf = 1;           // tile buffers in LDS: 1, or the ring size of direct staging (2..8)
    int sw = 1;             // workgroups that share one output tile, each on its own range of channel chunks
    int groups = 0;         // G = ceil(c_out / f)
    int chunks = 0;         // Q = ceil(c_in / cc)
    int entry_words = 8;    // 32-bit words per entry: 8 (code, channel, 2 spare, 4 fp32 weights) or 4 (code, 2 words of binary16 pairs, channel)
    int32_t idle_off = 0;   // first entry of the run of end-of-chunk entries walked by wavefronts without a filter group
    std::vector<uint32_t> stream;      // entries
    std::vector<int32_t> wave_off;     // [G*ks*sw] first entry of each (group, split) wavefront stream in each workgroup share
    std::vector<int32_t> slot_pos;     // [G*f] position in the reordered filter list of the filter in each slot, -1 for padding
    std::vector<int32_t> chan_map;     // [filter blocks][chunks*cc] input channel staged at each place of each chunk, -1 for padding
    std::vector<int32_t> perm_pad;     // [G*f] original filter index by slot, -1 for padding
    std::vector<float> bias_pad;       // [G*f]
};

struct HostPlan {
    int32_t c_in = 0, c_out = 0, h = 0, w = 0, n_hint = 1, num_patterns = 0, taps = 4;
    uint32_t flags = 0;
    int32_t dtype = 0;
    std::vector<uint16_t> masks;
    std::vector<float> bias;            // [c_out], zeros if absent
    Canonical canon;
    pp_conv_tuning_t chosen{};
    bool tiled = false;
    TiledLayout tl;
    // generic kernel tables
    std::vector<int32_t> filt_off;      // [c_out+1] prefix of kcount
    std::vector<int8_t> tap_dyx;        // [P*taps*2] (dy, dx) per tap
};

// Validate desc; PP_OK or the error the header documents.
pp_status_t validate(const pp_conv_desc_t& d);
// Reorder (fills hp.canon and the scalar fields).  desc must be valid.
void build_canonical(const pp_conv_desc_t& d, HostPlan& hp);
// Choose variant and parameters, build the device-format arrays.  PP_ERR_UNSUPPORTED if the
// tuning request cannot be honoured.
pp_status_t build_layouts(const pp_conv_desc_t& d, HostPlan& hp);
// Decode tl.stream back to canonical order.
pp_status_t unpack_stream(const HostPlan& hp, int32_t* kidx, uint8_t* kpat, float* w);

// binary16 conversion used when packing weights (round to nearest even).
uint16_t f32_to_f16_rne(float v);
float f16_to_f32(uint16_t b);

// Static geometry of a tiled-kernel instantiation (shared by host packing and device code).
constexpr int kPW = 4;      // output pixels per lane along the width
constexpr int kMaxDynamicLds = 156 * 1024;   // dynamic LDS bytes a tiled-kernel workgroup may use (CU has 160 KB)
struct TileGeom {
    int tw;        // tile width in pixels = lw * kPW
    int mrows;     // most micro-rows one wavefront's 64 micro-tiles can touch
    int rows;      // LDS tile rows = mrows * r + 2
    int rs;        // interior row stride in elements (= tw: rows are contiguous)
    int hoff;      // element offset, inside a channel, of the halo area
    int hrs;       // halo row stride in elements: lw pairs of two 32-bit words
    int chs;       // LDS channel stride in elements (multiple of 16 bytes)
};
constexpr TileGeom tile_geom(int lw, int r, int elem_bytes) {
    int tw = lw * kPW;
    int mrows = (64 % lw == 0) ? 64 / lw : (64 + lw - 1) / lw + 1;
    int rows = mrows * r + 2;
    int vec = 16 / elem_bytes;                       // elements per 128-bit access
    int hoff = (rows * tw + vec - 1) / vec * vec;
    int hrs = lw * 2 * (4 / elem_bytes);
    int chs = (hoff + rows * hrs + vec - 1) / vec * vec;
    return TileGeom{tw, mrows, rows, tw, hoff, hrs, chs};
}

// Dynamic LDS of a tiled-kernel launch: nbuf tile buffers of cc channels (one for register
// staging, a ring of 2..8 for direct staging) followed, for direct staging, by the slot tables;
// the split-channel exchange area reuses the start of it.
constexpr int k1_lds_table_offset(int lw, int r, int cc, int elem_bytes, int nbuf) {
    return nbuf * cc * tile_geom(lw, r, elem_bytes).chs * elem_bytes;
}
constexpr int64_t k1_lds_table_bytes(int lw, int r, int elem_bytes, int mode) {
    if (!mode) return 0;
    TileGeom tg = tile_geom(lw, r, elem_bytes);
    int slot = mode == 1 ? 16 : 4;
    int ni = (tg.rows * (tg.tw * elem_bytes / slot) + 63) / 64, nh = (tg.rows * lw * 2 + 63) / 64;
    return (int64_t)(ni + nh) * 64 * 4;
}
constexpr int64_t k1_lds_layout_bytes(int lw, int r, int f, int wf, int ks, int cc, int elem_bytes, int mode, int nbuf) {
    int64_t total = (int64_t)nbuf * cc * tile_geom(lw, r, elem_bytes).chs * elem_bytes + k1_lds_table_bytes(lw, r, elem_bytes, mode);
    int64_t red = ks > 1 ? (int64_t)wf * f * r * 4 * 64 * 4 : 0;
    return total > red ? total : red;
}

}  // namespace ppc
