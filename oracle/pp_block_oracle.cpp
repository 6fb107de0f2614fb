// CPU checker for the block-pruned matrix product.  TEST INFRASTRUCTURE ONLY.
//
// Slow on purpose, shares nothing with the GPU library; only the tests, the smoke check and the
// benchmark's CPU-baseline leg may call it.
//
// What it computes.  Block-based pruning (paper, section 2.1.2 "Block-Based Pruning" and its figure
// "block_pruning") cuts a weight matrix W[M][K] into blocks of BM x BK and prunes, independently in
// every block, whole rows of the block and whole columns of the block.  Pruned weights are zeros of an
// ordinary fully-connected layer (or of a CONV layer written as a matrix product, as the section
// notes), so the result has a plain definition, written out here:
//
//   b(m,k)    = the block holding element (m,k): block row m / BM, block column k / BK
//               (the last block row / column is smaller when BM, BK do not divide M, K)
//   Wd[m][k]  = W[m][k]  if row (m mod BM) and column (k mod BK) are both kept in block b(m,k)
//             = 0        otherwise
//   pre[m][j] = bias[m] + sum_k Wd[m][k] * X[k][j]          X is K x N, Y is M x N, both row-major
//   y         = max(pre, 0) when ReLU is fused, else pre
//
// The paper prints no formula; this is the reading any framework gives a masked linear layer.  All
// arithmetic is in double.
//
// Pins (tests/test_oracle_block.py): a hand-worked fixture, numpy's float64 matrix product on masks
// built a second way, a gather-style brute force that never forms Wd, all-kept = dense product,
// nothing kept = bias, one kept element = a scaled row of X, linearity, and invariance of the result
// under moving a pruned weight.

#include <algorithm>
#include <cstdint>
#include <thread>
#include <vector>

namespace {

template <class Fn>
void rows_in_parallel(int64_t count, int threads, Fn fn) {
    if (threads <= 1 || count <= 1) {
        for (int64_t i = 0; i < count; ++i) fn(i);
        return;
    }
    std::vector<std::thread> pool;
    int nt = (int)std::min<int64_t>(threads, count);
    for (int t = 0; t < nt; ++t)
        pool.emplace_back([=]() {
            for (int64_t i = t; i < count; i += nt) fn(i);
        });
    for (auto& th : pool) th.join();
}

}  // namespace

extern "C" {

// Section 2.1.2: the masked dense matrix.  row_keep is [blocks_m][blocks_k][bm], col_keep is
// [blocks_m][blocks_k][bk] (nonzero = kept; entries past the matrix edge are ignored), w is the dense
// M x K matrix of which only kept elements are read.  Returns 0, or 1 on a bad shape.
int oracle_block_expand(int m, int k, int bm, int bk, const uint8_t* row_keep, const uint8_t* col_keep,
                        const double* w, double* wd) {
    if (m < 1 || k < 1 || bm < 1 || bk < 1) return 1;
    int blocks_k = (k + bk - 1) / bk;
    for (int r = 0; r < m; ++r)
        for (int c = 0; c < k; ++c) {
            int64_t blk = (int64_t)(r / bm) * blocks_k + c / bk;
            bool kept = row_keep[blk * bm + r % bm] != 0 && col_keep[blk * bk + c % bk] != 0;
            wd[(int64_t)r * k + c] = kept ? w[(int64_t)r * k + c] : 0.0;
        }
    return 0;
}

// The fully-connected layer over the masked dense matrix: three plain loops.  pre (optional) receives
// the value before the activation, scale (optional) receives |bias| + sum |Wd| |X| for error scaling.
void oracle_gemm(int m, int k, int n, const double* wd, const double* x, const double* bias, int relu,
                 double* y, double* pre, double* scale, int threads) {
    rows_in_parallel(m, threads, [=](int64_t r) {
        for (int j = 0; j < n; ++j) {
            double acc = bias ? bias[r] : 0.0;
            double mag = bias ? (bias[r] < 0 ? -bias[r] : bias[r]) : 0.0;
            for (int c = 0; c < k; ++c) {
                double a = wd[r * k + c], b = x[(int64_t)c * n + j];
                acc += a * b;
                mag += (a < 0 ? -a : a) * (b < 0 ? -b : b);
            }
            if (pre) pre[r * n + j] = acc;
            if (scale) scale[r * n + j] = mag;
            y[r * n + j] = (relu && acc < 0.0) ? 0.0 : acc;
        }
    });
}

// The same at chosen outputs only: pts holds `count` (row, column) pairs.
void oracle_gemm_at(int m, int k, int n, const double* wd, const double* x, const double* bias, int relu,
                    const int32_t* pts, int64_t count, double* y, double* pre, double* scale, int threads) {
    (void)m;
    rows_in_parallel(count, threads, [=](int64_t i) {
        int64_t r = pts[2 * i], j = pts[2 * i + 1];
        double acc = bias ? bias[r] : 0.0;
        double mag = bias ? (bias[r] < 0 ? -bias[r] : bias[r]) : 0.0;
        for (int c = 0; c < k; ++c) {
            double a = wd[r * k + c], b = x[(int64_t)c * n + j];
            acc += a * b;
            mag += (a < 0 ? -a : a) * (b < 0 ? -b : b);
        }
        if (pre) pre[i] = acc;
        if (scale) scale[i] = mag;
        y[i] = (relu && acc < 0.0) ? 0.0 : acc;
    });
}

// Gather-style brute force used as a pin: for each output it walks the blocks of its row, skips a block
// whose row is pruned, and adds only the block's kept columns.  It never forms Wd.
void oracle_block_brute(int m, int k, int n, int bm, int bk, const uint8_t* row_keep, const uint8_t* col_keep,
                        const double* w, const double* x, const double* bias, int relu, double* y) {
    int blocks_k = (k + bk - 1) / bk;
    for (int r = 0; r < m; ++r)
        for (int j = 0; j < n; ++j) {
            double acc = bias ? bias[r] : 0.0;
            for (int bc = 0; bc < blocks_k; ++bc) {
                int64_t blk = (int64_t)(r / bm) * blocks_k + bc;
                if (!row_keep[blk * bm + r % bm]) continue;
                int width = std::min(bk, k - bc * bk);
                for (int cc = 0; cc < width; ++cc)
                    if (col_keep[blk * bk + cc]) acc += w[(int64_t)r * k + bc * bk + cc] * x[(int64_t)(bc * bk + cc) * n + j];
            }
            y[(int64_t)r * n + j] = (relu && acc < 0.0) ? 0.0 : acc;
        }
}

}  // extern "C"
