// Constants and static geometry shared by the host-side packing and the tiled kernel's device code.
#pragma once

#include <cstdint>

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
