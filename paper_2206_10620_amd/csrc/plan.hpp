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

// Weight-stream entry header bits (first 32-bit word of every entry).
constexpr uint32_t kCodeMask = 0xFFu;      // bits 0-7 : local filter slot * NP + pattern slot
constexpr uint32_t kFlagNewChannel = 0x100u;  // bit 8 : first kernel of an input channel: reload the lane's input window
constexpr uint32_t kFlagEnd = 0x200u;         // bit 9 : end of this wavefront's work for the current channel chunk
constexpr int kChanShift = 16;             // bits 16-31: channel index inside the chunk

struct Canonical {          // tuning-independent result of the reorder
    std::vector<int32_t> perm, kcount, pat_off, kidx;
    std::vector<uint8_t> kpat;
    std::vector<float> wpacked;
    int64_t k_kept = 0;
};

struct TiledLayout {        // geometry of the tiled kernel for one plan
    int np = 0;             // pattern slots compiled in (8 or 16)
    int f = 0, r = 0, lw = 0, wf = 0, ks = 0, cc = 0;
    int groups = 0;         // G = ceil(c_out / f)
    int chunks = 0;         // Q = ceil(c_in / cc)
    int entry_words = 8;    // 32-bit words per entry: header, 3 reserved, 4 fp32 weights
    std::vector<uint32_t> stream;      // entries
    std::vector<int32_t> wave_off;     // [G*ks] first entry of each (group, split) wavefront stream
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
    int hoff;      // element offset, inside a tile row, of micro-column 0's (left, right) halo pair
    int rs;        // LDS row stride in elements
    int chs;       // LDS channel stride in elements
};
constexpr TileGeom tile_geom(int lw, int r, int elem_bytes) {
    int tw = lw * kPW;
    int mrows = (64 % lw == 0) ? 64 / lw : (64 + lw - 1) / lw + 1;
    int rows = mrows * r + 2;
    int vec = 16 / elem_bytes;                       // elements per 128-bit access
    int hoff = tw + 2;                               // interior, one dummy pair, lw pairs, one dummy pair
    int rs = tw + 2 * (lw + 2);
    rs = (rs + vec - 1) / vec * vec;
    return TileGeom{tw, mrows, rows, hoff, rs, rows * rs};
}

}  // namespace ppc
