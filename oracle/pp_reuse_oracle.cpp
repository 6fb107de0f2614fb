// CPU checker for deep reuse (LSH clustering of neuron vectors).  TEST INFRASTRUCTURE ONLY.
//
// Slow on purpose, shares nothing with the GPU library; only the tests, the smoke check and the
// benchmark's CPU-baseline leg may call it.
//
// What it computes.  Deep reuse (paper, section 2.3.2 "Deep Reuse", figure "basicReuse") approximates the
// product X W of a layer -- X holds one row per output position (the unfolded input of a CONV layer, or the
// tokens of a fully-connected one), W is K x M -- by cutting every row of X into neuron vectors of L
// consecutive values, clustering the neuron vectors of one column segment with locality-sensitive hashing,
// and reusing, for every member of a cluster, the dot products computed on ONE neuron vector of it.  The
// section names LSH as the clustering method and leaves the hash family, the choice of the vector that
// stands for a cluster and the reuse scope to the papers it cites.  This repository's reading, step by step:
//
//   segments      s = 0 .. K/L - 1 cover columns sL .. sL+L-1 of X (K must be a multiple of L)
//   hashing       sign random projections: for H hyperplanes h of segment s (given as input, so both sides
//                 use the same random numbers), bit h of the signature of row i is 1 iff
//                 p = fma(x[i][sL+L-1], hp[s][h][L-1], ... fma(x[i][sL], hp[s][h][0], 0)) > 0,
//                 the sum taken in binary32 in exactly that order (the decision is an integer, so it is
//                 taken in the precision and order the GPU kernel uses)
//   clusters      rows with equal signature in segment s form a cluster; its representative is the member
//                 with the lowest row index (the reuse scope is the batch of rows of one call)
//   reuse         P[s][g][m] = sum_l x[rep(s,g)][sL+l] * W[sL+l][m]        (computed once per cluster)
//   result        pre[i][m] = bias[m] + sum_s P[s][sig(i,s)][m],  y = max(pre, 0) with ReLU, else pre
//
// Everything after the signatures is in double.  Where every cluster holds identical vectors the result is
// the exact product; otherwise it is the approximation the method makes, and this file is its definition.
//
// Pins (tests/test_oracle_reuse.py): a hand-worked fixture; signatures against numpy on integer-valued
// inputs (where binary32 sums are exact in any order); +-1 inputs with axis-aligned hyperplanes, where every
// cluster holds identical vectors and the result must equal the exact product; all-zero hyperplanes, where
// every row receives row 0's exact result; substitution form (exact product of X with every neuron vector
// replaced by its representative, built with numpy).  The hash family and the representative rule are this
// repository's reading: parity unpinned against the paper for those two choices.

#include <cmath>
#include <cstdint>
#include <vector>

extern "C" {

// signatures [n][S] (S = k / seg_len); returns 0, or 1 on a bad shape
int oracle_reuse_signatures(int n, int k, int seg_len, int hash_bits, const float* x, const float* hp, uint16_t* sig) {
    if (n < 1 || k < 1 || seg_len < 1 || k % seg_len != 0 || hash_bits < 1 || hash_bits > 16) return 1;
    const int S = k / seg_len;
    for (int i = 0; i < n; ++i)
        for (int s = 0; s < S; ++s) {
            unsigned g = 0;
            for (int h = 0; h < hash_bits; ++h) {
                float p = 0.0f;
                for (int l = 0; l < seg_len; ++l) p = std::fmaf(x[(int64_t)i * k + s * seg_len + l], hp[((int64_t)s * hash_bits + h) * seg_len + l], p);
                if (p > 0.0f) g |= 1u << h;
            }
            sig[(int64_t)i * S + s] = (uint16_t)g;
        }
    return 0;
}

// representatives [S][2^hash_bits]: lowest row index of the cluster, or -1 for an empty cluster
void oracle_reuse_representatives(int n, int S, int hash_bits, const uint16_t* sig, int32_t* rep) {
    const int G = 1 << hash_bits;
    for (int64_t e = 0; e < (int64_t)S * G; ++e) rep[e] = -1;
    for (int i = n - 1; i >= 0; --i)
        for (int s = 0; s < S; ++s) rep[(int64_t)s * G + sig[(int64_t)i * S + s]] = i;
}

// the approximated layer from signatures and representatives; pre (optional) receives the value before the
// activation, scale (optional) |bias| + sum |x_rep| |w| for error scaling
void oracle_reuse_apply(int n, int k, int m, int seg_len, int hash_bits, const double* x, const double* w, const double* bias,
                        const uint16_t* sig, const int32_t* rep, int relu, double* y, double* pre, double* scale) {
    const int S = k / seg_len, G = 1 << hash_bits;
    std::vector<double> P((size_t)S * G * m, 0.0), A((size_t)S * G * m, 0.0);
    for (int s = 0; s < S; ++s)
        for (int g = 0; g < G; ++g) {
            const int r = rep[(int64_t)s * G + g];
            if (r < 0) continue;
            for (int c = 0; c < m; ++c) {
                double acc = 0.0, mag = 0.0;
                for (int l = 0; l < seg_len; ++l) {
                    const double a = x[(int64_t)r * k + s * seg_len + l], b = w[(int64_t)(s * seg_len + l) * m + c];
                    acc += a * b;
                    mag += std::fabs(a) * std::fabs(b);
                }
                P[((size_t)s * G + g) * m + c] = acc;
                A[((size_t)s * G + g) * m + c] = mag;
            }
        }
    for (int i = 0; i < n; ++i)
        for (int c = 0; c < m; ++c) {
            double acc = bias ? bias[c] : 0.0, mag = bias ? std::fabs(bias[c]) : 0.0;
            for (int s = 0; s < S; ++s) {
                const size_t at = ((size_t)s * G + sig[(int64_t)i * S + s]) * m + c;
                acc += P[at];
                mag += A[at];
            }
            if (pre) pre[(int64_t)i * m + c] = acc;
            if (scale) scale[(int64_t)i * m + c] = mag;
            y[(int64_t)i * m + c] = (relu && acc < 0.0) ? 0.0 : acc;
        }
}

}  // extern "C"
