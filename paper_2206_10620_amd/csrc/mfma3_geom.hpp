// Geometry of the direct-load matrix-core kernel (k3), shared by the host-side plan, the launcher and
// the device code.
#pragma once

#include <cstdint>

namespace ppc {

constexpr int kK3ColTiles = 2;         // 32-lane MFMA column tiles per wavefront
// input-staging instructions one wavefront issues per chunk, at most (each costs three words of LDS per lane)
constexpr int k3_max_x_units(int waves) { return waves == 8 ? 3 : 4; }
constexpr int k3_stages(int waves) { return waves == 8 ? 3 : 2; }   // ring of staged steps: what LDS has room for
constexpr int kK3WeightBytes = 18 * 1024;   // operand fragments of one 16-channel chunk: 9 taps x 2 filter halves x 1 KB

// A workgroup of `waves` wavefronts (4 or 8) computes waves * kK3ColTiles column tiles of 32 lanes.  A column tile holds 32 / sw
// row segments ("units") of sw computed columns, each with its own halo column on either side, so a
// unit yields sw - 2 outputs.  The workgroup's units form a tile of tr rows x nseg segments.
struct K3Geom {
    int sw = 32;          // computed columns per segment (32 or 16)
    int nseg = 1;         // segments per tile row
    int tr = 8;           // tile rows = units / nseg
    int waves = 4;        // wavefronts per workgroup: 4 (two workgroups share a compute unit) or 8 (one has it to itself)
    int units = 8;        // waves * kK3ColTiles * (32 / sw)
    int trp = 10;         // staged input rows = tr + 2
    int segb = 64;        // bytes per staged segment row (sw binary16 values)
    int ppc = 40;         // 16-byte pieces per channel in LDS
    int ppcp = 44;        // ... including padding: LDS bytes per channel / 16 (an odd multiple of 64 bytes,
                          // so that the four channels one transposing read touches fall into different banks)
    int chs = 704;        // LDS bytes per channel
    int nxi = 11;         // staging instructions per chunk: ceil(16 channels * ppcp / 64 lanes)
    int xbuf_bytes = 0;   // nxi * 1024
    int lds_bytes = 0;    // the ring of input and weight buffers + the wavefronts' corners
    bool ok = false;
};

inline K3Geom k3_geom(int sw, int nseg, int waves) {
    K3Geom g;
    g.sw = sw;
    g.nseg = nseg;
    g.waves = waves;
    if ((sw != 32 && sw != 16) || (waves != 4 && waves != 8) || nseg < 1) return g;
    g.units = waves * kK3ColTiles * (32 / sw);
    if (g.units % nseg != 0) return g;
    g.tr = g.units / nseg;
    g.trp = g.tr + 2;
    g.segb = sw * 2;
    g.ppc = g.trp * nseg * g.segb / 16;
    int blocks64 = (g.ppc * 16 + 63) / 64;
    if ((blocks64 & 1) == 0) ++blocks64;
    g.chs = blocks64 * 64;
    g.ppcp = g.chs / 16;
    g.nxi = (16 * g.ppcp + 63) / 64;
    g.xbuf_bytes = g.nxi * 1024;
    g.lds_bytes = k3_stages(waves) * (g.xbuf_bytes + kK3WeightBytes) + waves * (64 * 4 + 2048) + (3 * k3_max_x_units(waves) + 1) * 64 * waves * 4;   // + per wavefront: 64 bias values, a 32 x 32 binary16 tile for the epilogue; + per lane: the parked staging set of the next tile and the lane's staging constants
    // a wavefront has nine staging slots per step (one per tap): its share of the 18 weight instructions, then input
    g.ok = g.nxi <= k3_max_x_units(waves) * waves && (18 + waves - 1) / waves + (g.nxi + waves - 1) / waves <= 9 && g.tr + 2 < 256 &&
           g.lds_bytes <= 156 * 1024;                     // what a workgroup may take of the compute unit's 160 KB
    return g;
}

}  // namespace ppc
