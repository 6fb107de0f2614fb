// Host code under AddressSanitizer and UndefinedBehaviorSanitizer: the planner (validation, filter kernel
// reorder, every device layout, the weight-stream round trip) and the CPU checker are driven over a seeded
// sweep of layer descriptions, valid and invalid.  Built and run by tests/test_host_sanitizers.py with
//   g++ -std=c++17 -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all ...
// It prints "ok <cases>" and exits 0 when nothing was flagged and every round trip held.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "block_plan.hpp"
#include "plan.hpp"

extern "C" {
int oracle_expand_weights(int c_in, int c_out, int num_patterns, const uint16_t* masks, const int32_t* pattern_id,
                          const uint8_t* conn, const double* w, int taps_per_kernel, double* Wd);
int oracle_block_expand(int m, int k, int bm, int bk, const uint8_t* row_keep, const uint8_t* col_keep, const double* w, double* wd);
void oracle_gemm(int m, int k, int n, const double* wd, const double* x, const double* bias, int relu, double* y, double* pre, double* scale,
                 int threads);
void oracle_block_brute(int m, int k, int n, int bm, int bk, const uint8_t* row_keep, const uint8_t* col_keep, const double* w, const double* x,
                        const double* bias, int relu, double* y);
int oracle_reuse_signatures(int n, int k, int seg_len, int hash_bits, const float* x, const float* hp, uint16_t* sig);
void oracle_reuse_representatives(int n, int S, int hash_bits, const uint16_t* sig, int32_t* rep);
void oracle_reuse_apply(int n, int k, int m, int seg_len, int hash_bits, const double* x, const double* w, const double* bias, const uint16_t* sig,
                        const int32_t* rep, int relu, double* y, double* pre, double* scale);
int64_t oracle_plan_ref(int c_in, int c_out, int num_patterns, const int32_t* pattern_id, const uint8_t* conn,
                        int32_t* perm, int32_t* kcount, int32_t* pat_off, int32_t* kidx, uint8_t* kpat, int64_t* wsel);
}

namespace {
uint64_t mix(uint64_t z) {      // SplitMix64 finaliser: a counter-based generator for the sweep
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
struct Rng {
    uint64_t s;
    uint64_t next() { return s = mix(s); }
    int below(int n) { return (int)(next() % (uint64_t)n); }
    float unit() { return (float)((next() >> 40) / 16777216.0) * 2.0f - 1.0f; }
};
const uint16_t kSet[16] = {0x03A, 0x0B2, 0x0B8, 0x09A, 0x01B, 0x036, 0x0D8, 0x1B0, 0x055, 0x115, 0x151, 0x154, 0x152, 0x11C, 0x071, 0x095};

int fail(const char* what, int c) {
    std::fprintf(stderr, "case %d: %s\n", c, what);
    return 1;
}
}  // namespace

int main() {
    using namespace ppc;
    Rng rng{12345};
    int cases = 0;
    for (int c = 0; c < 160; ++c) {
        const int c_in = 1 + rng.below(c % 7 == 0 ? 70 : 20), c_out = 1 + rng.below(c % 5 == 0 ? 140 : 24);
        const int h = 1 + rng.below(40), w = 1 + rng.below(c % 3 == 0 ? 300 : 40);
        const int ksizes[4] = {3, 3, 1, 5};
        int ks = ksizes[rng.below(4)];
        if (c % 11 == 0) ks = 7;
        const int taps = ks == 1 ? 1 : (ks == 3 ? 4 : 1 + rng.below(9));
        const int P = ks == 1 ? 1 : 1 + rng.below(ks == 3 ? 16 : 6);
        std::vector<uint16_t> m16(P);
        std::vector<uint64_t> m64(P);
        for (int p = 0; p < P; ++p) {
            if (ks == 3) m16[p] = kSet[(p + c) % 16], m64[p] = m16[p];
            else {
                uint64_t m = 0;
                while (__builtin_popcountll(m) < taps) m |= 1ull << rng.below(ks * ks);
                m64[p] = m;
                m16[p] = (uint16_t)m;
            }
        }
        const int64_t K = (int64_t)c_in * c_out;
        std::vector<int32_t> pid(K);
        std::vector<uint8_t> conn(K);
        std::vector<float> wts((size_t)K * taps), bias(c_out);
        const int keep = (c % 13 == 0) ? 4 : rng.below(5);   // 0: nothing kept ... 4: everything (always, when no mask is passed)
        for (int64_t k = 0; k < K; ++k) {
            pid[k] = rng.below(P);
            conn[k] = keep == 4 ? 1 : (keep == 0 ? 0 : (rng.below(4) < keep));
            if (!conn[k] && (k & 1)) pid[k] = -77;           // ids of removed kernels are never read
        }
        for (float& v : wts) v = rng.unit();
        for (float& v : bias) v = rng.unit() * 0.1f;
        pp_conv_tuning_t tun{};
        pp_conv_desc_t d{};
        d.c_in = c_in, d.c_out = c_out, d.h = h, d.w = w, d.n_hint = 1 + rng.below(4);
        d.num_patterns = P;
        d.pattern_masks = m16.data();
        d.pattern_masks64 = ks > 3 ? m64.data() : nullptr;
        d.pattern_id = pid.data();
        d.conn_mask = (c % 13 == 0) ? nullptr : conn.data();
        d.weights = wts.data();
        d.bias = (c % 4 == 0) ? nullptr : bias.data();
        d.dtype = rng.below(2);
        d.kernel_size = ks == 3 && (c & 1) ? 0 : ks;
        d.stride = 1 + (ks != 3 || c % 9 == 0 ? rng.below(2) : 0);
        d.taps_per_kernel = (ks == 3 && taps == 4) ? 0 : taps;
        d.flags = PP_FLAG_HOST_ONLY | (rng.below(2) ? PP_FLAG_RELU : 0u);
        if (c % 17 == 0 && ((h - 1) / d.stride + 1) % 2 == 0 && ((w - 1) / d.stride + 1) % 2 == 0) d.flags |= PP_FLAG_POOL2;
        // tuning requests, some of them impossible: they must be refused, not crash
        tun.variant = rng.below(4);
        if (c % 3 == 0) tun.rows_per_lane = rng.below(3), tun.split_c = rng.below(5), tun.waves_f = rng.below(9), tun.filters_per_wave = 4 * rng.below(3);
        if (c % 4 == 1) tun.tile_cols = 14 * rng.below(5), tun.wg_waves = 4 * rng.below(3), tun.mfma_kind = rng.below(3);
        if (c % 5 == 2) tun.tile_rows = rng.below(20), tun.tile_cols = rng.below(80), tun.tiles_per_wave = 2 * rng.below(3);
        if (c % 6 == 3) tun.staging = rng.below(9), tun.split_wg = rng.below(4), tun.chunk_c = rng.below(40), tun.lanes_x = rng.below(17);
        d.tuning = (c % 2) ? &tun : nullptr;
        if (validate(d) != PP_OK) return fail("a valid description was refused", c);
        HostPlan hp;
        build_canonical(d, hp);
        const pp_status_t st = build_layouts(d, hp);
        if (st != PP_OK && st != PP_ERR_UNSUPPORTED) return fail("unexpected planner status", c);
        if (st == PP_OK && hp.tiled && hp.taps == 4) {
            std::vector<int32_t> kidx((size_t)hp.canon.k_kept + 1);
            std::vector<uint8_t> kpat((size_t)hp.canon.k_kept + 1);
            std::vector<float> w((size_t)hp.canon.k_kept * 4 + 4);
            if (unpack_stream(hp, kidx.data(), kpat.data(), w.data()) != PP_OK) return fail("stream round trip refused", c);
            for (int64_t k = 0; k < hp.canon.k_kept; ++k)
                if (kidx[k] != hp.canon.kidx[k] || kpat[k] != hp.canon.kpat[k]) return fail("stream round trip differs", c);
        }
        // the checker's reorder on the same layer (3x3, four taps, explicit mask), compared with the planner's
        if (ks == 3 && taps == 4 && d.conn_mask) {
            std::vector<int32_t> perm(c_out), kcount(c_out), pat_off((size_t)c_out * (P + 1)), kidx(K);
            std::vector<uint8_t> kpat(K);
            std::vector<int64_t> wsel(K);
            std::vector<int32_t> pid_ok(pid);
            for (int64_t k = 0; k < K; ++k)
                if (!conn[k]) pid_ok[k] = 0;
            const int64_t kk = oracle_plan_ref(c_in, c_out, P, pid_ok.data(), conn.data(), perm.data(), kcount.data(),
                                               pat_off.data(), kidx.data(), kpat.data(), wsel.data());
            if (kk != hp.canon.k_kept) return fail("kept-kernel counts differ", c);
            if (std::memcmp(perm.data(), hp.canon.perm.data(), (size_t)c_out * 4) != 0) return fail("filter orders differ", c);
            if (kk && std::memcmp(kidx.data(), hp.canon.kidx.data(), (size_t)kk * 4) != 0) return fail("kernel orders differ", c);
            std::vector<double> Wd((size_t)K * 9), w64(wts.begin(), wts.end());
            if (oracle_expand_weights(c_in, c_out, P, m16.data(), pid_ok.data(), conn.data(), w64.data(), 4, Wd.data()) != 0)
                return fail("checker refused the layer", c);
        }
        ++cases;
        // invalid descriptions: each must come back as a status
        pp_conv_desc_t bad = d;
        bad.c_in = 0;
        if (validate(bad) == PP_OK) return fail("c_in = 0 accepted", c);
        bad = d;
        bad.dtype = 7;
        if (validate(bad) == PP_OK) return fail("dtype 7 accepted", c);
        bad = d;
        bad.weights = nullptr;
        if (validate(bad) == PP_OK) return fail("null weights accepted", c);
        if (ks == 3) {
            std::vector<uint16_t> mb(m16);
            mb[0] = 0x1FF;
            bad = d;
            bad.pattern_masks = mb.data();
            if (validate(bad) == PP_OK) return fail("nine-bit mask accepted", c);
        }
    }
    // block-pruned product: the plan's packed tiles decode back to the masked matrix the checker builds, for both
    // packings, over ragged block and matrix sizes; invalid descriptions come back as a status
    for (int c = 0; c < 40; ++c) {
        Rng r{(uint64_t)c * 104729u + 17u};
        const int m = 1 + r.below(150), k = 1 + r.below(150), bm = 1 + r.below(40), bk = 1 + r.below(40), n = 1 + r.below(9);
        const int blocks_m = (m + bm - 1) / bm, blocks_k = (k + bk - 1) / bk;
        std::vector<uint8_t> rk((size_t)blocks_m * blocks_k * bm), ck((size_t)blocks_m * blocks_k * bk);
        for (auto& v : rk) v = r.below(100) < 55;
        for (auto& v : ck) v = r.below(100) < 55;
        std::vector<float> w((size_t)m * k), bias(m);
        for (auto& v : w) v = r.unit();
        for (auto& v : bias) v = r.unit();
        pp_block_gemm_desc_t d{};
        d.m = m, d.k = k, d.block_m = bm, d.block_k = bk;
        d.row_keep = (c % 5 == 4) ? nullptr : rk.data();
        d.col_keep = (c % 7 == 6) ? nullptr : ck.data();
        d.weights = w.data();
        d.bias = (c & 1) ? bias.data() : nullptr;
        d.flags = PP_FLAG_HOST_ONLY | ((c & 2) ? PP_FLAG_RELU : 0u);
        d.dtype = (c % 3 == 0) ? PP_F32 : PP_F16;
        d.variant = d.dtype == PP_F16 ? 2 - (c & 1) : 1;
        ppc::BlockHostPlan bp;
        if (ppc::build_block_plan(d, bp) != PP_OK) return fail("block plan refused", c);
        std::vector<uint8_t> ones_r(rk.size(), 1), ones_c(ck.size(), 1);
        std::vector<double> w64(w.begin(), w.end()), wd((size_t)m * k);
        if (d.dtype == PP_F16)
            for (auto& v : w64) v = (double)f16_to_f32(f32_to_f16_rne((float)v));
        if (oracle_block_expand(m, k, bm, bk, d.row_keep ? rk.data() : ones_r.data(), d.col_keep ? ck.data() : ones_c.data(), w64.data(), wd.data()) != 0)
            return fail("checker refused the block layer", c);
        std::vector<float> tile((size_t)ppc::kBlockRowTile * k);
        for (int t = 0; t < bp.row_tiles; ++t) {
            if (ppc::unpack_block_tile(bp, t, tile.data()) != PP_OK) return fail("block tile did not unpack", c);
            for (int rr = 0; rr < ppc::kBlockRowTile && t * ppc::kBlockRowTile + rr < m; ++rr)
                for (int cc = 0; cc < k; ++cc)
                    if ((double)tile[(size_t)rr * k + cc] != wd[(size_t)(t * ppc::kBlockRowTile + rr) * k + cc]) return fail("block tile differs from the masked matrix", c);
        }
        if (ppc::unpack_block_tile(bp, bp.row_tiles, tile.data()) == PP_OK) return fail("tile index past the end accepted", c);
        std::vector<double> x((size_t)k * n), y((size_t)m * n), yb((size_t)m * n), b64(bias.begin(), bias.end());
        for (auto& v : x) v = r.unit();
        oracle_gemm(m, k, n, wd.data(), x.data(), d.bias ? b64.data() : nullptr, (c & 2) != 0, y.data(), nullptr, nullptr, 2);
        oracle_block_brute(m, k, n, bm, bk, d.row_keep ? rk.data() : ones_r.data(), d.col_keep ? ck.data() : ones_c.data(), w64.data(), x.data(),
                           d.bias ? b64.data() : nullptr, (c & 2) != 0, yb.data());
        for (size_t i = 0; i < y.size(); ++i)
            if (std::abs(y[i] - yb[i]) > 1e-9) return fail("the checker's two evaluations differ", c);
        pp_block_gemm_desc_t bad = d;
        bad.block_m = 0;
        if (ppc::build_block_plan(bad, bp) == PP_OK) return fail("block_m = 0 accepted", c);
        bad = d;
        bad.weights = nullptr;
        if (ppc::build_block_plan(bad, bp) == PP_OK) return fail("null block weights accepted", c);
        bad = d;
        bad.dtype = PP_F32, bad.variant = 2;
        if (ppc::build_block_plan(bad, bp) == PP_OK) return fail("matrix-core kernel with fp32 accepted", c);
        ++cases;
    }
    // deep reuse checker: signatures, representatives and the approximated layer on ragged sizes
    for (int c = 0; c < 20; ++c) {
        Rng r{(uint64_t)c * 7919u + 5u};
        const int L = 1 + r.below(8), S = 1 + r.below(6), k = L * S, n = 1 + r.below(70), m = 1 + r.below(10), H = 1 + r.below(10);
        std::vector<float> x((size_t)n * k), hp((size_t)S * H * L);
        for (auto& v : x) v = r.unit();
        for (auto& v : hp) v = r.unit();
        std::vector<uint16_t> sig((size_t)n * S);
        if (oracle_reuse_signatures(n, k, L, H, x.data(), hp.data(), sig.data()) != 0) return fail("signatures refused", c);
        std::vector<int32_t> rep((size_t)S << H);
        oracle_reuse_representatives(n, S, H, sig.data(), rep.data());
        for (int i = 0; i < n; ++i)
            for (int sgm = 0; sgm < S; ++sgm) {
                const int32_t rp = rep[((size_t)sgm << H) + sig[(size_t)i * S + sgm]];
                if (rp < 0 || rp > i || sig[(size_t)rp * S + sgm] != sig[(size_t)i * S + sgm]) return fail("representative is not the cluster's first row", c);
            }
        std::vector<double> x64(x.begin(), x.end()), w((size_t)k * m), bias(m), y((size_t)n * m), pre((size_t)n * m), sc((size_t)n * m);
        for (auto& v : w) v = r.unit();
        for (auto& v : bias) v = r.unit();
        oracle_reuse_apply(n, k, m, L, H, x64.data(), w.data(), (c & 1) ? bias.data() : nullptr, sig.data(), rep.data(), c & 2, y.data(), pre.data(), sc.data());
        ++cases;
    }
    // binary16 conversion on every bit pattern and around every rounding boundary
    for (uint32_t b = 0; b < 65536; ++b) {
        const float f = f16_to_f32((uint16_t)b);
        if (f == f && f32_to_f16_rne(f) != (uint16_t)b) return fail("binary16 round trip", (int)b);
    }
    std::printf("ok %d\n", cases);
    return 0;
}
