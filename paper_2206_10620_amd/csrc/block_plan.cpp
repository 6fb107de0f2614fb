// Plan step of the block-pruned matrix product (paper, section 2.1.2 for the sparsity; the split into a
// compile-time packing and a run-time kernel follows section 2.3.1).
#include "block_plan.hpp"

#include <algorithm>
#include <cstring>

#include "plan.hpp"

namespace ppc {

pp_status_t build_block_plan(const pp_block_gemm_desc_t& d, BlockHostPlan& p) {
    if (!d.weights) return PP_ERR_NULL;
    if (d.m < 1 || d.k < 1 || d.block_m < 1 || d.block_k < 1) return PP_ERR_SHAPE;
    if ((int64_t)d.m * d.k >= ((int64_t)1 << 31)) return PP_ERR_SHAPE;
    if (d.dtype != PP_F32 && d.dtype != PP_F16) return PP_ERR_UNSUPPORTED;
    if (d.flags & ~(uint32_t)(PP_FLAG_RELU | PP_FLAG_HOST_ONLY)) return PP_ERR_UNSUPPORTED;
    if (d.variant < 0 || d.variant > 2 || (d.variant == 2 && d.dtype != PP_F16)) return PP_ERR_UNSUPPORTED;
    p.m = d.m, p.k = d.k, p.bm = d.block_m, p.bk = d.block_k;
    p.flags = d.flags, p.dtype = d.dtype;
    p.forced = d.variant != 0;
    p.variant = d.variant ? d.variant : (d.dtype == PP_F16 ? 2 : 1);
    const int RT = kBlockRowTile;
    const int blocks_k = (d.k + d.block_k - 1) / d.block_k;
    p.row_tiles = (d.m + RT - 1) / RT;
    auto row_kept = [&](int r, int bj) { return !d.row_keep || d.row_keep[((int64_t)(r / d.block_m) * blocks_k + bj) * d.block_m + r % d.block_m] != 0; };
    auto col_kept = [&](int bi, int c) { return !d.col_keep || d.col_keep[((int64_t)bi * blocks_k + c / d.block_k) * d.block_k + c % d.block_k] != 0; };

    p.tile_off.assign(1, 0);
    p.tile_cols.clear();
    p.tile_len.clear();
    p.kept_weights = 0;
    std::vector<uint8_t> used((size_t)d.k);
    for (int t = 0; t < p.row_tiles; ++t) {
        const int r0 = t * RT, r1 = std::min(d.m, r0 + RT);
        std::fill(used.begin(), used.end(), 0);
        // the block rows this tile overlaps; a block contributes its kept columns if it keeps one of the tile's rows
        for (int bi = r0 / d.block_m; bi <= (r1 - 1) / d.block_m; ++bi)
            for (int bj = 0; bj < blocks_k; ++bj) {
                int rows_here = 0;
                for (int r = std::max(r0, bi * d.block_m); r < std::min(r1, (bi + 1) * d.block_m); ++r) rows_here += row_kept(r, bj) ? 1 : 0;
                if (!rows_here) continue;
                for (int c = bj * d.block_k; c < std::min(d.k, (bj + 1) * d.block_k); ++c)
                    if (col_kept(bi, c)) {
                        used[c] = 1;
                        p.kept_weights += rows_here;
                    }
            }
        int len = 0;
        for (int c = 0; c < d.k; ++c)
            if (used[c]) {
                p.tile_cols.push_back(c);
                ++len;
            }
        p.tile_len.push_back(len);
        while (len % kBlockChunk) {          // pad with a column that exists; its weights are zeros
            p.tile_cols.push_back(p.tile_cols.back());
            ++len;
        }
        p.tile_off.push_back((int32_t)p.tile_cols.size());
    }
    p.executed_weights = (int64_t)p.tile_cols.size() * RT;

    const bool half = d.dtype == PP_F16;
    auto value = [&](int r, int c) -> float {      // Wd[r][c], as the kernels will see it
        if (r >= d.m || !row_kept(r, c / d.block_k) || !col_kept(r / d.block_m, c)) return 0.0f;
        const float v = d.weights[(int64_t)r * d.k + c];
        return half ? f16_to_f32(f32_to_f16_rne(v)) : v;
    };
    p.wc.assign(p.tile_cols.size() * (size_t)RT, 0.0f);
    for (int t = 0; t < p.row_tiles; ++t)
        for (int i = 0; i < p.tile_len[t]; ++i) {
            const size_t at = (size_t)p.tile_off[t] + i;
            for (int r = 0; r < RT; ++r) p.wc[at * RT + r] = value(t * RT + r, p.tile_cols[at]);
        }
    p.apk.clear();
    if (half) {
        p.apk.assign(p.tile_cols.size() * (size_t)RT, 0);
        for (int t = 0; t < p.row_tiles; ++t)
            for (int i = 0; i < p.tile_len[t]; ++i) {
                const size_t at = (size_t)p.tile_off[t] + i, chunk = at / kBlockChunk, kk = at % kBlockChunk;
                for (int r = 0; r < RT; ++r) {
                    const int lane = (r % 32) + 32 * (int)(kk / 8);
                    p.apk[((chunk * 2 + r / 32) * 64 + lane) * 8 + kk % 8] = f32_to_f16_rne(p.wc[at * RT + r]);
                }
            }
    }
    p.bias.assign((size_t)p.row_tiles * RT, 0.0f);
    if (d.bias) std::memcpy(p.bias.data(), d.bias, (size_t)d.m * sizeof(float));
    return PP_OK;
}

pp_status_t unpack_block_tile(const BlockHostPlan& p, int tile, float* w_out) {
    if (tile < 0 || tile >= p.row_tiles) return PP_ERR_SHAPE;
    const int RT = kBlockRowTile;
    std::fill(w_out, w_out + (size_t)RT * p.k, 0.0f);
    for (int32_t at = p.tile_off[tile]; at < p.tile_off[tile + 1]; ++at) {
        const int c = p.tile_cols[at];
        const bool pad = at - p.tile_off[tile] >= p.tile_len[tile];
        for (int r = 0; r < RT; ++r) {
            float v;
            if (p.dtype == PP_F16) {
                const size_t chunk = (size_t)at / kBlockChunk, kk = (size_t)at % kBlockChunk;
                v = f16_to_f32(p.apk[((chunk * 2 + r / 32) * 64 + (r % 32) + 32 * (kk / 8)) * 8 + kk % 8]);
            } else {
                v = p.wc[(size_t)at * RT + r];
            }
            if (pad) {
                if (v != 0.0f) return PP_ERR_PATTERN;      // padding must carry zeros
            } else {
                w_out[(size_t)r * p.k + c] = v;
            }
        }
    }
    return PP_OK;
}

}  // namespace ppc
