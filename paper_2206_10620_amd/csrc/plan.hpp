// Host-side plan: the layer-wise representation after filter kernel reorder, and the packed
// device streams built from it (paper section 2.3.1, "Filter Kernel Reorder and Compact
// Filter-Kernel-Weight (FKW) Storage").  No HIP types here.
#pragma once

#include <cstdint>
#include <vector>

#include "pp_conv.h"
#include "tile_geom.hpp"
#include "mfma_geom.hpp"
#include "mfma3_geom.hpp"

namespace ppc {

struct Canonical {          // tuning-independent result of the reorder
    std::vector<int32_t> perm, kcount, pat_off, kidx;
    std::vector<uint8_t> kpat;
    std::vector<float> wpacked;
    int64_t k_kept = 0;
};

// One built-in four-tap pattern standing in for (part of) a layer pattern: its slot, and for each of its four
// taps (ascending) the index of the layer kernel's weight that goes there, or -1 for a zero.
struct CoverPart {
    int slot = 0;
    int src[4] = {-1, -1, -1, -1};
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
    bool covered = false;   // some pattern runs as several built-in patterns with zero weights (no round trip of the stream)
    std::vector<std::vector<CoverPart>> cover;   // [pattern] the built-in patterns that stand for it
    int32_t idle_off = 0;   // first entry of the run of end-of-chunk entries walked by wavefronts without a filter group
    std::vector<uint32_t> stream;      // entries
    std::vector<int32_t> wave_off;     // [G*ks*sw] first entry of each (group, split) wavefront stream in each workgroup share
    std::vector<int32_t> slot_pos;     // [G*f] position in the reordered filter list of the filter in each slot, -1 for padding
    std::vector<int32_t> chan_map;     // [filter blocks][chunks*cc] input channel staged at each place of each chunk, -1 for padding
    std::vector<int32_t> perm_pad;     // [G*f] original filter index by slot, -1 for padding
    std::vector<float> bias_pad;       // [G*f]
};

// Matrix-core kernel: the pruned weights zero-filled to a dense [c_out][K*K*c_in] binary16 matrix,
// cut into MFMA operand fragments in the order the kernel reads them.
struct MfmaLayout {
    int tr = 0, tc = 0, ntw = 0;      // workgroup tile (rows of the tall virtual image x columns) and MFMA column tiles per wavefront
    int waves = 4;                    // wavefronts per workgroup (4 or 8)
    bool direct = false;              // the direct-load kernel (3x3, stride 1, whole chunks of 16 channels) runs this plan
    K3Geom g3;                        // ... with this geometry
    int cpad = 0;                     // ... on this many input channels: c_in rounded up to whole chunks (a larger value than c_in means x is copied into a zero-padded buffer first)
    int ksplit = 1;                   // ... and this many workgroups sharing a tile's reduction (partial sums to a workspace)
    bool pairs = true;                // even image width: input staged as aligned 32-bit pixel pairs
    int po = 0;                       // rows per image in the tall virtual output image (ho + separator rows)
    int trp = 0, twpa = 0;            // staged input rows per tile: (tr-1)*stride + K; staged columns: (tc-1)*stride + K + 2, rounded down to even
    int fb = 0, q = 0;                // filter blocks of 64, channel chunks of 16
    int upq = 1;                      // weight units per chunk: 1 (all taps at once) or K (one tap row at a time)
    int gw = 1;                       // output elements per store (8, 4, 2 or 1)
    int xbuf_bytes = 0, wbuf_bytes = 0, out_pitch = 0;
    int64_t lds_bytes = 0;
    std::vector<uint16_t> wpk;        // [fb][q][K*K][2][64][8] binary16 bits
    std::vector<float> bias_pad;      // [fb*64]
};

struct HostPlan {
    int32_t c_in = 0, c_out = 0, h = 0, w = 0, n_hint = 1, num_patterns = 0, taps = 4;
    int32_t ks = 3, stride = 1;         // kernel size, stride
    bool pool = false;                  // fused 2x2 max-pool
    int32_t ho = 0, wo = 0;             // the convolution's output size
    int32_t out_h = 0, out_w = 0;       // size of y (pooled if pool)
    uint32_t flags = 0;
    int32_t dtype = 0;
    std::vector<uint64_t> masks;
    std::vector<float> bias;            // [c_out], zeros if absent
    Canonical canon;
    pp_conv_tuning_t chosen{};
    bool tiled = false;
    TiledLayout tl;
    bool mfma = false;
    MfmaLayout ml;
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
// Choose the matrix-core kernel's tile and pack its weights (hp.ml).  PP_ERR_UNSUPPORTED if the layer
// or the tuning request does not fit.
pp_status_t build_mfma_layout(const pp_conv_tuning_t& t, HostPlan& hp);
// Decode tl.stream back to canonical order.
pp_status_t unpack_stream(const HostPlan& hp, int32_t* kidx, uint8_t* kpat, float* w);

// binary16 conversion used when packing weights (round to nearest even).
uint16_t f32_to_f16_rne(float v);
float f16_to_f32(uint16_t b);

}  // namespace ppc
