// Host-side plan of the block-pruned matrix product (paper, section 2.1.2): compact column lists per
// row tile and the weights packed for the two kernels.  Pure host code.
#pragma once

#include <cstdint>
#include <vector>

#include "pp_block_gemm.h"

namespace ppc {

constexpr int kBlockRowTile = 64;     // rows per tile: two 32-row MFMA operands
constexpr int kBlockChunk = 16;       // columns of the compact list one MFMA consumes
constexpr int kBlockColTile = 512;    // columns of x and y per workgroup of the matrix-core kernel

struct BlockHostPlan {
    int m = 0, k = 0, bm = 0, bk = 0;
    uint32_t flags = 0;
    int dtype = PP_F32;
    int variant = 1;                  // kernel for n % 8 == 0
    bool forced = false;              // the description named the variant
    int row_tiles = 0;
    int64_t kept_weights = 0, executed_weights = 0;
    std::vector<int32_t> tile_off;    // [row_tiles + 1] offsets into tile_cols (multiples of kBlockChunk)
    std::vector<int32_t> tile_cols;   // padded compact lists
    std::vector<int32_t> tile_len;    // [row_tiles] before padding
    // generic kernel: wc[(tile_off[t] + i) * kBlockRowTile + r] = Wd[t * 64 + r][tile_cols[tile_off[t] + i]] (binary16-rounded for PP_F16)
    std::vector<float> wc;
    // matrix-core kernel (PP_F16): per chunk of 16 list entries two operands of 64 lanes x 8 binary16:
    // apk[((chunk * 2 + half) * 64 + lane) * 8 + e] = Wd[t * 64 + half * 32 + lane % 32][list[chunk * 16 + 8 * (lane / 32) + e]]
    std::vector<uint16_t> apk;
    std::vector<float> bias;          // [row_tiles * 64], zeros where there is no bias or no row
};

// Validates the description and builds the plan.  No device call.
pp_status_t build_block_plan(const pp_block_gemm_desc_t& d, BlockHostPlan& out);
// Decodes row tile `tile` back to a dense [64][k] matrix from the packed form the plan's kernel reads.
pp_status_t unpack_block_tile(const BlockHostPlan& p, int tile, float* w_out);

}  // namespace ppc


// Enqueues `batch` products with the plan's weights: matrix b of x ([k][n]) starts x_stride elements after matrix b - 1,
// likewise y ([m][n]).  Matrix-core kernel only (binary16, n a multiple of 8); used by the convolution library for 1x1 layers.
pp_status_t pp_block_gemm_launch_batched(const pp_block_gemm_plan_t* plan, const void* x_dev, void* y_dev, int32_t n, int32_t batch, int64_t x_stride,
                                         int64_t y_stride, void* hip_stream);
