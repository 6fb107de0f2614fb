// Constants shared by the host-side packing and the matrix-core kernel's device code.
#pragma once

namespace ppc {

constexpr int kMfmaChunk = 16;        // input channels per staged chunk = K extent of one MFMA step
constexpr int kMfmaFilters = 64;      // filters per workgroup (two 32-row MFMA tiles)
// staging units (16 pixel pairs x 4 channel pairs) per chunk that one wavefront's registers hold, by
// workgroup shape (wavefronts, column tiles per wavefront): each unit costs three vector registers
constexpr int mfma_max_units(int waves, int ntw) { return waves == 8 ? 10 : (ntw == 4 ? 14 : 8); }
constexpr int kMfmaPixelBytes = 48;   // LDS bytes per staged input pixel: 16 channels + 16 bytes of padding (bank spread)
constexpr int kMfmaMaxDynamicLds = 156 * 1024;   // dynamic LDS bytes a workgroup may use (the CU has 160 KB)

}  // namespace ppc
