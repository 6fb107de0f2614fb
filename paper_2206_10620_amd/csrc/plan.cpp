// Host-side planning: validation, filter kernel reorder, weight-stream packing.
// Paper section 2.3.1: the sparsity of a layer is fully known before deployment, so the order
// in which kernels are visited, and the code that visits them, is fixed ahead of time.
#include "plan.hpp"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>

namespace ppc {

namespace {

int builtin_slot(uint64_t mask) {
    for (int s = 0; s < kBuiltinPatterns; ++s)
        if ((uint64_t)kBuiltinMasks[s] == mask) return s;
    return -1;
}

// The fewest built-in patterns (at most three) whose union holds every tap of `mask`; src[j] is the index,
// among the mask's own taps in ascending order, of the weight that goes to the part's j-th tap, or -1.
std::vector<CoverPart> cover_pattern(uint32_t mask) {
    auto part_list = [&](const int* slots, int count) {
        std::vector<CoverPart> parts;
        uint32_t given = 0;
        for (int i = 0; i < count; ++i) {
            CoverPart c;
            c.slot = slots[i];
            int j = 0;
            for (int tap = 0; tap < 9; ++tap) {
                if (!((kBuiltinMasks[slots[i]] >> tap) & 1u)) continue;
                const uint32_t bit = 1u << tap;
                if ((mask & bit) && !(given & bit)) {
                    int idx = 0;
                    for (int t2 = 0; t2 < tap; ++t2) idx += (mask >> t2) & 1u;
                    c.src[j] = idx;
                    given |= bit;
                } else {
                    c.src[j] = -1;
                }
                ++j;
            }
            parts.push_back(c);
        }
        return parts;
    };
    if (mask == 0x1FFu) {                       // the unpruned kernel keeps the cover it has been measured with
        const int slots[3] = {4, 7, 8};
        return part_list(slots, 3);
    }
    const int own = builtin_slot(mask);
    if (own >= 0) return part_list(&own, 1);
    const int N = kBuiltinPatterns;
    for (int a = 0; a < N; ++a)
        if ((kBuiltinMasks[a] & mask) == mask) return part_list(&a, 1);
    for (int a = 0; a < N; ++a)
        for (int b = a + 1; b < N; ++b)
            if (((kBuiltinMasks[a] | kBuiltinMasks[b]) & mask) == mask) {
                const int slots[2] = {a, b};
                return part_list(slots, 2);
            }
    for (int a = 0; a < N; ++a)
        for (int b = a + 1; b < N; ++b)
            for (int c = b + 1; c < N; ++c)
                if (((kBuiltinMasks[a] | kBuiltinMasks[b] | kBuiltinMasks[c]) & mask) == mask) {
                    const int slots[3] = {a, b, c};
                    return part_list(slots, 3);
                }
    const int slots[3] = {4, 7, 8};             // these three hold all nine taps
    return part_list(slots, 3);
}

}  // namespace

uint16_t f32_to_f16_rne(float v) {
    uint32_t u;
    std::memcpy(&u, &v, 4);
    uint32_t sign = (u >> 16) & 0x8000u;
    uint32_t mag = u & 0x7FFFFFFFu;
    if (mag >= 0x7F800000u) return (uint16_t)(sign | (mag > 0x7F800000u ? 0x7E00u : 0x7C00u));   // nan / inf
    if (mag >= 0x477FF000u) return (uint16_t)(sign | 0x7C00u);       // rounds to >= 65520: overflow to inf
    if (mag < 0x33000001u) return (uint16_t)sign;                    // <= 2^-25: rounds to zero (tie to even)
    int32_t e = (int32_t)(mag >> 23) - 127;                          // unbiased exponent
    uint32_t man = (mag & 0x7FFFFFu) | 0x800000u;                    // 24-bit significand
    int shift = (e < -14) ? (13 + (-14 - e)) : 13;                   // bits dropped; more for subnormal results
    uint32_t kept = man >> shift;
    uint32_t rem = man & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (kept & 1u))) ++kept;
    uint32_t out;
    if (e < -14) out = kept;                                         // subnormal (a carry lands on the smallest normal)
    else out = ((uint32_t)(e + 15) << 10) + (kept - 0x400u);         // a mantissa carry bumps the exponent
    return (uint16_t)(sign | out);
}

float f16_to_f32(uint16_t b) {
    uint32_t sign = (uint32_t)(b & 0x8000u) << 16;
    int e = (b >> 10) & 31;
    uint32_t m = b & 1023u;
    float v;
    if (e == 0) v = std::ldexp((float)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = std::ldexp(1.0f + (float)m / 1024.0f, e - 15);
    uint32_t u;
    std::memcpy(&u, &v, 4);
    u |= sign;
    std::memcpy(&v, &u, 4);
    return v;
}

namespace {
struct Geometry { int ks, stride, taps; bool dense, pool; };
// kernel size, stride and taps per kernel of a description, with the zero defaults resolved; ks = 0 if invalid
Geometry geometry(const pp_conv_desc_t& d) {
    Geometry g{};
    g.dense = (d.flags & PP_FLAG_DENSE) != 0;
    g.pool = (d.flags & PP_FLAG_POOL2) != 0;
    g.ks = d.kernel_size == 0 ? 3 : d.kernel_size;
    g.stride = d.stride == 0 ? 1 : d.stride;
    if (g.ks != 1 && g.ks != 3 && g.ks != 5 && g.ks != 7) g.ks = 0;
    g.taps = g.dense ? g.ks * g.ks : (d.taps_per_kernel == 0 ? (g.ks == 1 ? 1 : 4) : d.taps_per_kernel);
    return g;
}
int popcount64(uint64_t v) {
    int n = 0;
    while (v) {
        v &= v - 1;
        ++n;
    }
    return n;
}
}  // namespace

pp_status_t validate(const pp_conv_desc_t& d) {
    const Geometry g = geometry(d);
    const bool dense = g.dense;
    if (!d.weights) return PP_ERR_NULL;
    if (g.ks == 0 || (g.stride != 1 && g.stride != 2)) return PP_ERR_UNSUPPORTED;
    const bool wide = g.ks > 3;
    if (!dense && (!(wide ? (const void*)d.pattern_masks64 : (const void*)d.pattern_masks) || !d.pattern_id)) return PP_ERR_NULL;
    if (d.c_in < 1 || d.c_out < 1 || d.h < 1 || d.w < 1) return PP_ERR_SHAPE;
    if ((int64_t)d.c_in * d.c_out >= (int64_t)1 << 28) return PP_ERR_SHAPE;
    if ((int64_t)std::max(d.c_in, d.c_out) * d.h * d.w >= (int64_t)1 << 31) return PP_ERR_SHAPE;
    if (d.flags & ~(uint32_t)(PP_FLAG_RELU | PP_FLAG_DENSE | PP_FLAG_HOST_ONLY | PP_FLAG_POOL2)) return PP_ERR_UNSUPPORTED;
    if (d.dtype != PP_F32 && d.dtype != PP_F16) return PP_ERR_UNSUPPORTED;
    if (g.pool) {
        const int ho = (d.h - 1) / g.stride + 1, wo = (d.w - 1) / g.stride + 1;
        if ((ho & 1) || (wo & 1)) return PP_ERR_SHAPE;
    }
    if (dense) return PP_OK;
    if (g.taps < 1 || g.taps > g.ks * g.ks) return PP_ERR_PATTERN;
    if (d.num_patterns < 1 || d.num_patterns > 255) return PP_ERR_PATTERN;
    for (int p = 0; p < d.num_patterns; ++p) {
        const uint64_t m = wide ? d.pattern_masks64[p] : (uint64_t)d.pattern_masks[p];
        if ((g.ks * g.ks < 64 && (m >> (g.ks * g.ks)) != 0) || popcount64(m) != g.taps) return PP_ERR_PATTERN;
    }
    const int64_t k_total = (int64_t)d.c_in * d.c_out;
    for (int64_t k = 0; k < k_total; ++k) {
        if (d.conn_mask && !d.conn_mask[k]) continue;
        if (d.pattern_id[k] < 0 || d.pattern_id[k] >= d.num_patterns) return PP_ERR_PATTERN;
    }
    return PP_OK;
}

void build_canonical(const pp_conv_desc_t& d, HostPlan& hp) {
    const Geometry geo = geometry(d);
    const bool dense = geo.dense;
    hp.c_in = d.c_in;
    hp.c_out = d.c_out;
    hp.h = d.h;
    hp.w = d.w;
    hp.n_hint = d.n_hint > 0 ? d.n_hint : 1;
    hp.flags = d.flags;
    hp.dtype = d.dtype;
    hp.ks = geo.ks;
    hp.stride = geo.stride;
    hp.pool = geo.pool;
    hp.ho = (d.h - 1) / geo.stride + 1;
    hp.wo = (d.w - 1) / geo.stride + 1;
    hp.out_h = geo.pool ? hp.ho / 2 : hp.ho;
    hp.out_w = geo.pool ? hp.wo / 2 : hp.wo;
    hp.taps = geo.taps;
    hp.num_patterns = dense ? 1 : d.num_patterns;
    const int kk = geo.ks * geo.ks;
    hp.masks.assign(hp.num_patterns, kk == 64 ? ~(uint64_t)0 : (((uint64_t)1 << kk) - 1));
    if (!dense)
        for (int p = 0; p < d.num_patterns; ++p) hp.masks[p] = geo.ks > 3 ? d.pattern_masks64[p] : (uint64_t)d.pattern_masks[p];
    hp.bias.assign(d.c_out, 0.0f);
    if (d.bias) hp.bias.assign(d.bias, d.bias + d.c_out);

    const int P = hp.num_patterns, ci_n = d.c_in, co_n = d.c_out;
    auto kept = [&](int co, int ci) { return !d.conn_mask || d.conn_mask[(int64_t)co * ci_n + ci] != 0; };
    auto pat = [&](int co, int ci) { return dense ? 0 : d.pattern_id[(int64_t)co * ci_n + ci]; };

    // per-filter pattern histograms
    std::vector<int32_t> hist((size_t)co_n * P, 0), count(co_n, 0);
    for (int co = 0; co < co_n; ++co)
        for (int ci = 0; ci < ci_n; ++ci)
            if (kept(co, ci)) {
                ++hist[(size_t)co * P + pat(co, ci)];
                ++count[co];
            }
    // filter order: heavier filters first (they set the critical path of a workgroup), equal
    // counts ordered by pattern signature so that neighbours run the same code mix
    Canonical& cn = hp.canon;
    cn.perm.resize(co_n);
    std::iota(cn.perm.begin(), cn.perm.end(), 0);
    std::sort(cn.perm.begin(), cn.perm.end(), [&](int a, int b) {
        if (count[a] != count[b]) return count[a] > count[b];
        for (int p = 0; p < P; ++p) {
            int ha = hist[(size_t)a * P + p], hb = hist[(size_t)b * P + p];
            if (ha != hb) return ha > hb;
        }
        return a < b;
    });
    cn.k_kept = std::accumulate(count.begin(), count.end(), (int64_t)0);
    cn.kcount.resize(co_n);
    cn.pat_off.assign((size_t)co_n * (P + 1), 0);
    cn.kidx.resize(cn.k_kept);
    cn.kpat.resize(cn.k_kept);
    cn.wpacked.resize((size_t)cn.k_kept * hp.taps);
    // kernels of a filter: counting sort by pattern, channels ascending inside a pattern
    int64_t base = 0;
    std::vector<int32_t> cursor(P + 1);
    for (int pos = 0; pos < co_n; ++pos) {
        const int co = cn.perm[pos];
        cn.kcount[pos] = count[co];
        int32_t* po = &cn.pat_off[(size_t)pos * (P + 1)];
        for (int p = 0; p < P; ++p) po[p + 1] = po[p] + hist[(size_t)co * P + p];
        std::copy(po, po + P + 1, cursor.begin());
        for (int ci = 0; ci < ci_n; ++ci) {
            if (!kept(co, ci)) continue;
            const int p = pat(co, ci);
            const int64_t slot = base + cursor[p]++;
            cn.kidx[slot] = ci;
            cn.kpat[slot] = (uint8_t)p;
            const float* src = d.weights + ((int64_t)co * ci_n + ci) * hp.taps;
            std::copy(src, src + hp.taps, &cn.wpacked[(size_t)slot * hp.taps]);
        }
        base += count[co];
    }
    hp.filt_off.resize(co_n + 1);
    hp.filt_off[0] = 0;
    for (int pos = 0; pos < co_n; ++pos) hp.filt_off[pos + 1] = hp.filt_off[pos] + cn.kcount[pos];
    hp.tap_dyx.clear();
    for (int p = 0; p < P; ++p)
        for (int t = 0; t < kk; ++t)
            if ((hp.masks[p] >> t) & 1u) {
                hp.tap_dyx.push_back((int8_t)(t / geo.ks - geo.ks / 2));
                hp.tap_dyx.push_back((int8_t)(t % geo.ks - geo.ks / 2));
            }
}

namespace {

bool valid_lw(int lw) { return lw == 2 || lw == 4 || lw == 7 || lw == 8 || lw == 14 || lw == 16; }

// Lanes across a tile.  The largest power of two that idles at most an eighth of the lanes: 64
// micro-tiles are then a whole number of tile rows (other widths stage one more row band) and the
// tile is the smallest per output pixel -- measured 3-7 % faster than the exact fits of 14 and 7 on
// the 28-, 56-, 112- and 224-wide fp16 layers.  Otherwise the width that wastes the fewest lanes.
int pick_lw(int w) {
    const int cand[] = {16, 14, 8, 7, 4, 2};
    int best = 16;
    double best_waste = 1e30;
    for (int lw : cand) {
        int tw = lw * kPW;
        int strips = (w + tw - 1) / tw;
        double waste = (double)strips * tw / w;
        if ((lw & (lw - 1)) == 0 && waste <= 1.15) return lw;
        if (waste < best_waste - 1e-9) {
            best_waste = waste;
            best = lw;
        }
    }
    return best;
}

int64_t spatial_waves(int n, int h, int w, int lw, int r) {
    int64_t vh = (int64_t)n * (h + 1) - 1;
    int64_t mrows = (vh + r - 1) / r;
    int strips = (w + lw * kPW - 1) / (lw * kPW);
    return strips * ((mrows * lw + 63) / 64);
}

}  // namespace

pp_status_t build_layouts(const pp_conv_desc_t& d, HostPlan& hp) {
    pp_conv_tuning_t t{};
    if (d.tuning) t = *d.tuning;
    if (t.variant < 0 || t.variant > 3) return PP_ERR_UNSUPPORTED;

    // can the tiled kernel express this layer?  (3x3, stride 1, no pooling, and a pattern table made of
    // the masks it has specialised code for)
    // A pattern the kernel has no specialised code for is run as up to three of its own four-tap patterns
    // on the same channel whose union covers the pattern's taps; every tap is given to the first of
    // them that holds it and the other positions carry zero weights.  An unpruned (nine-tap) kernel is
    // the extreme case: {0,1,3,4}, {4,5,7,8} with a zero centre weight, and {0,2,4,6} with zero
    // weights on taps 0 and 4 (12 multiply-accumulates for 9 weights).  This is the plan-time side of
    // "code for the patterns the layer has" (section 2.3.1) without generating code: a foreign table
    // costs extra multiply-accumulates on zeros, not the loss of tiling and reuse.
    const bool dense = hp.taps == 9 && hp.ks == 3;
    bool builtin = hp.ks == 3 && hp.stride == 1 && !hp.pool;
    int max_slot = -1;
    bool covered = false;                                     // some pattern needs more than its own slot
    std::vector<std::vector<CoverPart>>& cover = hp.tl.cover;
    cover.assign(hp.num_patterns, {});
    if (builtin) {
        std::vector<char> used(hp.num_patterns, 0);
        for (uint8_t p : hp.canon.kpat) used[p] = 1;
        for (int p = 0; p < hp.num_patterns; ++p) {
            if (!used[p]) continue;
            cover[p] = cover_pattern(dense ? 0x1FFu : (uint32_t)hp.masks[p]);
            covered = covered || cover[p].size() != 1 || hp.taps != 4;
            for (const CoverPart& c : cover[p]) max_slot = std::max(max_slot, c.slot);
        }
    }
    // The matrix-core kernel takes any layer whose storage is binary16.  Measured on MI355X it beats the
    // pattern-specialised vector kernel on every binary16 benchmark layer (the dense product costs
    // 9/(4*keep) times the multiply-accumulates at more than 30 times the rate), so it is the default there.
    const bool mfma_ok = hp.dtype == PP_F16;
    if (t.variant == 2 && !builtin) return PP_ERR_UNSUPPORTED;
    if (t.variant == 3 && !mfma_ok) return PP_ERR_UNSUPPORTED;
    int variant = t.variant;
    if (variant == 0) variant = mfma_ok ? 3 : (builtin ? 2 : 1);
    hp.tiled = variant == 2;
    hp.mfma = variant == 3;
    hp.chosen = pp_conv_tuning_t{};
    hp.chosen.variant = variant;
    if (t.split_k < 0 || (t.split_k > 1 && variant != 3)) return PP_ERR_UNSUPPORTED;
    if (variant == 3) return build_mfma_layout(t, hp);
    if (!hp.tiled) return PP_OK;

    TiledLayout& tl = hp.tl;
    tl.covered = covered;
    const int eb = hp.dtype == PP_F16 ? 2 : 4;
    tl.np = max_slot < 8 ? 8 : 16;
    tl.entry_words = hp.dtype == PP_F16 ? 4 : 8;   // header + two words of binary16 pairs, or header + 3 spare + 4 fp32

    // ---- parameters (the part of the layer-wise representation that is left to tuning) ----
    tl.lw = t.lanes_x ? t.lanes_x : pick_lw(hp.w);
    if (!valid_lw(tl.lw)) return PP_ERR_UNSUPPORTED;
    // Defaults measured on MI355X: four filters per wavefront keep the kernel under 64-80 vector
    // registers (6-8 wavefronts per SIMD hide the scalar dispatch and the LDS latency); two output
    // rows per lane when that still leaves a few thousand wavefronts, else one; 16 wavefronts per
    // workgroup so that an input tile is staged once for 64 filters, some of them splitting the
    // input channels instead when the layer is too small to fill the chip otherwise.
    tl.f = t.filters_per_wave ? t.filters_per_wave : 4;
    if (tl.f != 4 && tl.f != 8 && tl.f != 16) return PP_ERR_UNSUPPORTED;
    if (tl.f * tl.np > 256) return PP_ERR_UNSUPPORTED;
    const int groups_f = (hp.c_out + tl.f - 1) / tl.f;
    const int64_t want_waves = 3000;
    tl.r = t.rows_per_lane;
    if (tl.r == 0) {
        // two rows per lane double the multiply-accumulates per dispatch; worth it even when the
        // wavefront count then has to come from a two-way channel split (measured)
        const int64_t w2 = spatial_waves(hp.n_hint, hp.h, hp.w, tl.lw, 2) * groups_f;
        tl.r = (w2 >= want_waves || (2 * w2 >= want_waves && hp.c_in >= 64)) ? 2 : 1;
    }
    if (tl.r != 1 && tl.r != 2 && tl.r != 4) return PP_ERR_UNSUPPORTED;
    if (tl.r == 4 && tl.f != 4) return PP_ERR_UNSUPPORTED;
    const int max_waves = 16;                      // the kernel's launch bound
    const int64_t base_waves = spatial_waves(hp.n_hint, hp.h, hp.w, tl.lw, tl.r) * groups_f;
    tl.ks = t.split_c;
    if (tl.ks == 0) {
        tl.ks = 1;
        while (tl.ks < 4 && base_waves * tl.ks < want_waves && hp.c_in >= 32 * tl.ks) tl.ks *= 2;
        // one-row wavefronts are short of multiply-accumulates per dispatch and gain from a second
        // resident workgroup per CU (measured on 28x28 layers of 256-512 channels)
        if (tl.ks == 1 && tl.r == 1 && base_waves < 2 * want_waves && hp.c_in >= 64) tl.ks = 2;
    }
    if (tl.ks < 1 || tl.ks > max_waves) return PP_ERR_UNSUPPORTED;
    tl.wf = t.waves_f;
    if (tl.wf == 0) {
        tl.wf = std::max(1, std::min(groups_f, max_waves / tl.ks));
        // do not let one workgroup's filter block leave most of the chip idle
        while (tl.wf > 1 && spatial_waves(hp.n_hint, hp.h, hp.w, tl.lw, tl.r) * ((groups_f + tl.wf - 1) / tl.wf) < 200)
            tl.wf /= 2;
    }
    if (tl.wf < 1 || tl.wf * tl.ks > max_waves) return PP_ERR_UNSUPPORTED;
    // the split-channel partial sums are exchanged through LDS: wf * f * r * 4 accumulators * 64 lanes
    auto reduce_bytes = [&]() { return tl.ks > 1 ? tl.wf * tl.f * tl.r * 4 * 64 * 4 : 0; };
    while (!t.waves_f && tl.wf > 1 && reduce_bytes() > kMaxDynamicLds) tl.wf /= 2;
    if (reduce_bytes() > kMaxDynamicLds) return PP_ERR_UNSUPPORTED;
    const TileGeom tg = tile_geom(tl.lw, tl.r, eb);
    // How input tiles reach LDS: direct global-to-LDS loads in 16-byte slots when every image row
    // and every strip starts on a 16-byte boundary, in 4-byte slots when they start on a 4-byte
    // boundary, through registers otherwise (fp16 rows of odd width).  The direct path addresses a
    // channel's rows with 32-bit byte offsets from the first row of the tile.
    if (t.staging < 0 || t.staging > 8) return PP_ERR_UNSUPPORTED;
    tl.mode = 0;
    if (t.staging != 1 && ((int64_t)hp.c_in * hp.h * hp.w + (int64_t)tg.rows * hp.w) * eb < ((int64_t)1 << 31)) {
        if (hp.w % (16 / eb) == 0 && (tg.tw * eb) % 16 == 0) tl.mode = 1;
        else if (eb == 4 || hp.w % 2 == 0) tl.mode = 2;
    }
    if (t.staging >= 2 && tl.mode == 0) return PP_ERR_UNSUPPORTED;
    const int nw = tl.wf * tl.ks;
    const int64_t spatial_wgs = spatial_waves(hp.n_hint, hp.h, hp.w, tl.lw, tl.r);
    const int64_t total_wgs = spatial_wgs * ((groups_f + tl.wf - 1) / tl.wf);
    // LDS one workgroup may take: all of it when there is at most about one workgroup per CU anyway,
    // else a share that lets as many workgroups be resident as the wavefront slots allow (8 per SIMD
    // for the small-accumulator variants, else 4)
    const int wg_per_cu = total_wgs <= 320 ? 1 : std::max(1, ((tl.f * tl.r * 4 <= 32) ? 32 : 16) / nw);
    const int64_t budget = std::min<int64_t>(kMaxDynamicLds, 160 * 1024 / wg_per_cu - 1024);
    const int64_t chan_bytes = (int64_t)tg.chs * eb;
    const int cap = std::min(32, (hp.c_in + tl.ks - 1) / tl.ks * tl.ks);
    tl.cc = t.chunk_c;
    tl.nbuf = tl.mode ? (t.staging >= 2 ? t.staging : 0) : 1;
    auto lds_bytes = [&](int cc, int nbuf) { return k1_lds_layout_bytes(tl.lw, tl.r, tl.f, tl.wf, tl.ks, cc, eb, tl.mode, nbuf); };
    if (tl.mode == 0) {
        if (tl.cc == 0) {
            int cc = tl.ks;
            while (cc + tl.ks <= cap && lds_bytes(cc + tl.ks, 1) <= budget) cc += tl.ks;
            tl.cc = cc;
        }
    } else {
        // channels of LDS available to the ring
        auto fit = [&](int64_t bytes) { return (int)std::max<int64_t>(0, (bytes - k1_lds_table_bytes(tl.lw, tl.r, eb, tl.mode)) / chan_bytes); };
        if (tl.cc == 0 && tl.nbuf == 0) {
            // Measured: what a chunk costs besides its multiply-accumulates (barrier, stream
            // bookkeeping, issuing loads) outweighs what deeper prefetch gains, so two large buffers.
            int ct = fit(budget);
            if (ct < 2 * std::max(tl.ks, 4)) ct = fit(kMaxDynamicLds);       // a ring too small to be worth a second workgroup
            tl.nbuf = 2;
            tl.cc = std::max(tl.ks, std::min(cap, ct / tl.nbuf) / tl.ks * tl.ks);
        } else if (tl.cc == 0) {
            int ct = fit(budget);
            if (ct < tl.nbuf * tl.ks) ct = fit(kMaxDynamicLds);
            tl.cc = std::max(tl.ks, std::min(cap, ct / tl.nbuf) / tl.ks * tl.ks);
        } else if (tl.nbuf == 0) {
            tl.nbuf = std::max(2, std::min(4, fit(budget) / tl.cc));
        }
        const int chunks = (hp.c_in + tl.cc - 1) / tl.cc;
        if (t.staging < 2) tl.nbuf = std::max(2, std::min(tl.nbuf, chunks));   // no more buffers than chunks
    }
    if (tl.nbuf < 1 || tl.nbuf > 8) return PP_ERR_UNSUPPORTED;
    if (lds_bytes(std::max(tl.cc, 1), tl.nbuf) > kMaxDynamicLds) return PP_ERR_UNSUPPORTED;
    if (tl.cc < tl.ks || tl.cc % tl.ks != 0 || tl.cc > 512 || tl.cc * tg.rows >= 65536) return PP_ERR_UNSUPPORTED;
    tl.groups = groups_f;
    tl.chunks = (hp.c_in + tl.cc - 1) / tl.cc;
    // Channel split across workgroups: each of sw workgroups takes a contiguous share of the chunks
    // and the last one to finish adds the shares up.  Worth it when the layer has too few output
    // tiles to fill the chip.
    tl.sw = t.split_wg;
    if (tl.sw == 0) tl.sw = 1;
    if (tl.sw < 1 || tl.sw > 64 || tl.sw > tl.chunks) return PP_ERR_UNSUPPORTED;
    hp.chosen.filters_per_wave = tl.f;
    hp.chosen.rows_per_lane = tl.r;
    hp.chosen.lanes_x = tl.lw;
    hp.chosen.waves_f = tl.wf;
    hp.chosen.split_c = tl.ks;
    hp.chosen.chunk_c = tl.cc;
    hp.chosen.staging = tl.mode ? tl.nbuf : 1;
    hp.chosen.split_wg = tl.sw;

    // ---- device layout: which filter sits in which wavefront slot, which channel in which chunk ----
    // The wavefronts of a workgroup meet at a barrier once per channel chunk, so what a chunk costs
    // is what its busiest wavefront does in it.  Two static choices even that out; neither changes
    // the reordered layer-wise representation reported by pp_conv_plan_query:
    //  (1) inside a filter block (the wf*f consecutive filters of the new order that one workgroup
    //      computes) filters are dealt to the wf groups heaviest first, each to the group with the
    //      least kernels so far that still has a free slot;
    //  (2) per filter block the input channels are put into chunks (and, with split_c > 1, into the
    //      channel ranges of the splits) greedily, each time taking the channel that keeps the
    //      per-group cost of the range closest to an even share.
    const Canonical& cn = hp.canon;
    const int G = tl.groups, F = tl.f, KS = tl.ks, CC = tl.cc, Q = tl.chunks, CS = CC / KS, EW = tl.entry_words;
    const int WF = tl.wf, NFB = (G + WF - 1) / WF, C = hp.c_in;
    if (t.balance < 0 || t.balance > 2) return PP_ERR_UNSUPPORTED;
    const bool balance = t.balance != 1 && WF * KS > 1;
    hp.chosen.balance = balance ? 2 : 1;
    tl.slot_pos.assign((size_t)G * F, -1);
    tl.chan_map.assign((size_t)NFB * Q * CC, -1);
    std::vector<float> cost;
    std::vector<double> load, share, sums;
    std::vector<int> room, left;
    for (int fb = 0; fb < NFB; ++fb) {
        const int g0 = fb * WF, ng = std::min(WF, G - g0);
        const int pos0 = g0 * F, pos1 = std::min(hp.c_out, (g0 + ng) * F);
        int32_t* cmap = &tl.chan_map[(size_t)fb * Q * CC];
        if (!balance) {
            for (int pos = pos0; pos < pos1; ++pos) tl.slot_pos[pos] = pos;
            for (int ci = 0; ci < C; ++ci) cmap[ci] = ci;
            continue;
        }
        // (1) filters come in descending kernel count already
        load.assign(ng, 0.0);
        room.assign(ng, F);
        for (int pos = pos0; pos < pos1; ++pos) {
            int best = -1;
            for (int g = 0; g < ng; ++g)
                if (room[g] > 0 && (best < 0 || load[g] < load[best])) best = g;
            tl.slot_pos[(size_t)(g0 + best) * F + (F - room[best])] = pos;
            load[best] += cn.kcount[pos];
            --room[best];
        }
        // cost of channel ci to group g: its kernels there, plus half a kernel for loading the window
        cost.assign((size_t)ng * C, 0.0f);
        for (int g = 0; g < ng; ++g)
            for (int fl = 0; fl < F; ++fl) {
                const int pos = tl.slot_pos[(size_t)(g0 + g) * F + fl];
                if (pos < 0) continue;
                for (int64_t e = hp.filt_off[pos]; e < hp.filt_off[pos + 1]; ++e) cost[(size_t)g * C + cn.kidx[e]] += (float)tl.cover[cn.kpat[e]].size();
            }
        share.assign(ng, 0.0);
        for (int g = 0; g < ng; ++g)
            for (int ci = 0; ci < C; ++ci) {
                float& v = cost[(size_t)g * C + ci];
                if (v > 0.0f) v += 0.5f;
                share[g] += v / C;                   // the group's cost per channel if spread evenly
            }
        // (2) fill the ranges in order; candidates are looked for among the first kScan channels left
        const int kScan = 512;
        left.resize(C);
        for (int ci = 0; ci < C; ++ci) left[ci] = ci;
        sums.assign(ng, 0.0);
        for (int p = 0; p < C; ++p) {
            const int k = p % CS;                    // channels already in this range
            if (k == 0) std::fill(sums.begin(), sums.end(), 0.0);
            const int ncand = std::min<int>(kScan, (int)left.size());
            int best = 0;
            double best_score = 0.0;
            for (int j = 0; j < ncand; ++j) {
                const int ci = left[j];
                double score = -1e30;
                for (int g = 0; g < ng; ++g) score = std::max(score, sums[g] + cost[(size_t)g * C + ci] - share[g] * (k + 1));
                if (j == 0 || score < best_score) {
                    best = j;
                    best_score = score;
                }
            }
            const int ci = left[best];
            left.erase(left.begin() + best);
            for (int g = 0; g < ng; ++g) sums[g] += cost[(size_t)g * C + ci];
            cmap[p] = ci;
        }
    }
    tl.perm_pad.assign((size_t)G * F, -1);
    tl.bias_pad.assign((size_t)G * F, 0.0f);
    for (size_t sl = 0; sl < tl.slot_pos.size(); ++sl) {
        const int pos = tl.slot_pos[sl];
        if (pos < 0) continue;
        tl.perm_pad[sl] = cn.perm[pos];
        tl.bias_pad[sl] = hp.bias[cn.perm[pos]];
    }

    // ---- weight stream: one sequence of entries per (filter group, channel split) wavefront ----
    struct Item { int32_t ci; int32_t fl; int32_t slot; int64_t src; int32_t part; };
    tl.stream.clear();
    const int SW = tl.sw;
    tl.wave_off.assign((size_t)G * KS * SW, 0);
    std::vector<Item> items;
    std::vector<size_t> first(C + 1);
    const int chan_word = hp.dtype == PP_F16 ? 3 : 1;      // where the channel word sits in an entry
    const uint32_t chan_stride_bytes = (uint32_t)(tg.chs * eb);
    auto push_entry = [&](uint32_t code, uint32_t chan, const float* w4) {
        size_t at = tl.stream.size();
        tl.stream.resize(at + EW, 0u);
        tl.stream[at] = code;
        tl.stream[at + chan_word] = chan;
        if (!w4) return;
        if (hp.dtype == PP_F16) {    // binary16 storage: the weights are rounded here, once
            uint16_t hb[4];
            for (int j = 0; j < 4; ++j) hb[j] = f32_to_f16_rne(w4[j]);
            tl.stream[at + 1] = (uint32_t)hb[0] | ((uint32_t)hb[1] << 16);
            tl.stream[at + 2] = (uint32_t)hb[2] | ((uint32_t)hb[3] << 16);
        } else {
            std::memcpy(&tl.stream[at + 4], w4, 16);
        }
    };
    for (int g = 0; g < G; ++g) {
        const int32_t* cmap = &tl.chan_map[(size_t)(g / WF) * Q * CC];
        items.clear();
        for (int fl = 0; fl < F; ++fl) {
            const int pos = tl.slot_pos[(size_t)g * F + fl];
            if (pos < 0) continue;
            for (int64_t e = hp.filt_off[pos]; e < hp.filt_off[pos + 1]; ++e) {
                const std::vector<CoverPart>& parts = tl.cover[cn.kpat[e]];
                for (int part = 0; part < (int)parts.size(); ++part) items.push_back(Item{cn.kidx[e], fl, parts[part].slot, e, part});
            }
        }
        std::sort(items.begin(), items.end(), [](const Item& a, const Item& b) {
            if (a.ci != b.ci) return a.ci < b.ci;
            if (a.fl != b.fl) return a.fl < b.fl;
            return a.part < b.part;
        });
        // first[ci] .. first[ci+1]: the group's kernels on channel ci
        std::fill(first.begin(), first.end(), (size_t)0);
        for (const Item& k : items) ++first[k.ci + 1];
        for (int ci = 0; ci < C; ++ci) first[ci + 1] += first[ci];
        for (int s = 0; s < KS; ++s) {
            for (int q = 0; q < Q; ++q) {
                for (int sh = 0; sh < SW; ++sh)       // a share starts here
                    if (q == (int)((int64_t)sh * Q / SW)) tl.wave_off[((size_t)g * KS + s) * SW + sh] = (int32_t)(tl.stream.size() / EW);
                for (int cl = s * CS; cl < (s + 1) * CS; ++cl) {    // this wavefront's channels of chunk q, by place in the chunk
                    const int ci = cmap[q * CC + cl];
                    if (ci < 0) continue;
                    for (size_t j = first[ci]; j < first[ci + 1]; ++j) {
                        const Item& k = items[j];
                        const uint32_t code = (uint32_t)(k.fl * tl.np + k.slot);
                        const uint32_t chan = j == first[ci] ? (uint32_t)cl * chan_stride_bytes : kSameChannel;
                        const CoverPart& part = tl.cover[cn.kpat[k.src]][k.part];
                        float w4[4];
                        for (int j4 = 0; j4 < 4; ++j4) w4[j4] = part.src[j4] < 0 ? 0.0f : cn.wpacked[(size_t)k.src * hp.taps + part.src[j4]];
                        push_entry(code, chan, w4);
                    }
                }
                push_entry(kEndCode, kSameChannel, nullptr);
            }
        }
    }
    // what wavefronts without a filter group walk: one end-of-chunk entry per chunk
    tl.idle_off = (int32_t)(tl.stream.size() / EW);
    for (int q = 0; q < Q; ++q) push_entry(kEndCode, kSameChannel, nullptr);
    push_entry(kEndCode, kSameChannel, nullptr);     // the walker prefetches up to two entries ahead
    push_entry(kEndCode, kSameChannel, nullptr);
    if (tl.stream.size() / EW >= ((size_t)1 << 31)) return PP_ERR_SHAPE;
    return PP_OK;
}

// ---------------------------------------------------------------------------------------------
// Matrix-core kernel: tile choice and weight packing.
//
// The layer becomes the product  Y[c_out][pixels] = Wd[c_out][K*K*c_in] x patches[K*K*c_in][pixels]
// with the removed kernels and pruned taps written out as zeros.  The reduction index runs chunk of
// 16 channels slowest, then tap, then channel inside the chunk, so that one MFMA step
// (v_mfma_f32_32x32x16_f16) reduces over 16 consecutive channels at one tap: the lane that holds
// output pixel p then needs 8 consecutive channels of one input pixel, one 128-bit LDS read from a
// tile staged channel-innermost.  Weights are stored as the MFMA "A" operand fragments themselves:
// fragment (filter block, chunk, tap, half) is 64 lanes x 8 binary16 = 1 KB, lane l holding filter
// 32*half + l%32 and channels 8*(l/32) .. 8*(l/32)+7 of the chunk.
pp_status_t build_mfma_layout(const pp_conv_tuning_t& t, HostPlan& hp) {
    MfmaLayout& ml = hp.ml;
    const int KS = hp.ks, S = hp.stride, KK = KS * KS, pad = KS / 2;
    ml.fb = (hp.c_out + kMfmaFilters - 1) / kMfmaFilters;
    ml.q = (hp.c_in + kMfmaChunk - 1) / kMfmaChunk;
    ml.upq = KS <= 3 ? 1 : KS;
    ml.wbuf_bytes = (KK / ml.upq) * 2 * 1024;
    // The direct-load kernel takes 3x3, stride-1 layers; measured on MI355X it is the faster of the two wherever it
    // applies.
    // (a channel count that does not fill whole chunks is padded with zero channels into a plan-owned copy of x)
    // (a fused 2x2 max-pool needs even image sizes and a tile whose wavefronts each hold an even row and the row below it)
    const bool direct_ok = KS == 3 && S == 1 && hp.h + 2 + 66 < 65536 && (!hp.pool || (hp.h % 2 == 0 && hp.w % 2 == 0));
    // (mfma_kind 3, the product kernel for 1x1 layers, is decided by the caller of this function: the layout built here is then the fallback)
    if (t.mfma_kind < 0 || t.mfma_kind > 3 || (t.mfma_kind == 2 && !direct_ok)) return PP_ERR_UNSUPPORTED;
    // A request for a tile the direct kernel has no geometry for goes to the general kernel, unless the
    // direct one was asked for by name.
    auto direct_layout = [&]() -> bool {
        // Segment width: the one that computes the fewest columns per image row (a segment of sw computed
        // columns yields sw - 2 outputs).  Segments per tile row: the divisor of the workgroup's units
        // with the least matrix-core work (ragged last tiles) plus a quarter of the staged rows (halo).
        const int po = hp.h + (hp.pool ? 2 : 1);     // rows per image of the tall image: an even number when rows are pooled in pairs
        const int64_t vr = (int64_t)(hp.n_hint - 1) * po + hp.h;
        int sw = ((hp.w + 29) / 30) * 32 < ((hp.w + 13) / 14) * 16 ? 32 : 16;      // a tie goes to the narrow segments (measured: 3-7 % faster on 56-, 112- and 224-wide layers)
        // Workgroup size: eight wavefronts stage the weights once for twice the pixels (and have a compute
        // unit's LDS to themselves), but only a layer with several such tiles per compute unit keeps the
        // chip busy with them; four otherwise.
        if (t.wg_waves && t.wg_waves != 4 && t.wg_waves != 8) return false;
        if (t.tiles_per_wave && t.tiles_per_wave != kK3ColTiles) return false;
        auto pick = [&](int waves, int& nseg_o, double& tiles_o) -> bool {
            nseg_o = 0;
            if (ml.q < k3_stages(waves) - 1) return false;         // the kernel's ring is filled from one tile's chunks
            if (t.tile_cols) {
                if (t.tile_cols % 30 == 0) sw = 32, nseg_o = t.tile_cols / 30;
                else if (t.tile_cols % 14 == 0) sw = 16, nseg_o = t.tile_cols / 14;
                else return false;
            }
            const int units = waves * kK3ColTiles * (32 / sw), spr = (hp.w + sw - 3) / (sw - 2);
            double best = 1e300;
            for (int ns = 1; ns <= units; ++ns) {
                if (t.tile_cols && ns != nseg_o) continue;
                if (hp.pool && ns != 32 / sw) continue;      // pooled: a wavefront's two column tiles are two rows of the same segments
                if (!hp.pool && !t.tile_cols && !t.tile_rows && spr >= 2 && ns < 2) continue;   // measured: short staged rows (32 or 64 bytes) load poorly; at least two segments side by side (1080p layer: 8 x 60 tiles 225 us, 16 x 30 tiles 236 us)
                const K3Geom g = k3_geom(sw, ns, waves);
                if (!g.ok || (t.tile_rows && t.tile_rows != g.tr)) continue;
                const double tiles = (double)((spr + ns - 1) / ns) * (double)((vr + g.tr - 1) / g.tr);
                const double cost = tiles * (g.units + 0.25 * g.trp * ns);
                if (cost < best - 1e-9) best = cost, nseg_o = ns, tiles_o = tiles * ml.fb;
            }
            return best < 1e299;
        };
        int nseg = 0, waves = 0;
        double tiles = 0.0;
        if (t.wg_waves) {
            waves = t.wg_waves;
            if (!pick(waves, nseg, tiles)) return false;
        } else {
            int ns8 = 0;
            double tiles8 = 0.0;
            if (pick(8, ns8, tiles8) && tiles8 >= 4 * 256) waves = 8, nseg = ns8, tiles = tiles8;
            else if (pick(4, nseg, tiles)) waves = 4;
            else return false;
        }
        const K3Geom g = k3_geom(sw, nseg, waves);
        if (!g.ok) return false;
        ml.g3 = g;
        ml.po = po;
        ml.tr = g.tr;
        ml.tc = nseg * (sw - 2);
        ml.ntw = kK3ColTiles;
        ml.waves = waves;
        ml.lds_bytes = g.lds_bytes;
        hp.chosen.wg_waves = ml.waves;
        hp.chosen.tile_rows = ml.tr;
        hp.chosen.tile_cols = ml.tc;
        hp.chosen.tiles_per_wave = ml.ntw;
        hp.chosen.mfma_kind = 2;
        // Reduction split: a layer with fewer work items than the chip has places for workgroups lets several
        // of them share a tile, each on its own run of chunks.
        const int stages = k3_stages(waves);
        auto split_ok = [&](int k) { return k == 1 || (ml.q % k == 0 && ml.q / k >= std::max(2, stages - 1)); };
        if (t.split_k < 0 || (t.split_k > 1 && t.split_k != 2 && t.split_k != 4 && t.split_k != 8)) return false;
        int ks = 1;
        if (hp.pool) {
            if (t.split_k > 1) return false;           // the pooled epilogue stores final values only
        } else if (t.split_k) {
            if (!split_ok(t.split_k)) return false;
            ks = t.split_k;
        } else if (tiles <= 128.0 && (ml.q >= 32 || (ml.q >= 16 && tiles <= 64.0))) {
            // Measured on MI355X (512- and 256-channel layers with 56 to 128 work items): a four-way split takes
            // 512-channel layers from 49-51 us to 28-32 us and a 256-channel layer with 56 items from 28 to 23 us;
            // with 120 or more items of 16 chunks, or any layer that fills one round of workgroups, the partial
            // sums cost more than the split gains.
            if (split_ok(4)) ks = 4;
            else if (split_ok(2)) ks = 2;
        }
        ml.ksplit = ks;
        hp.chosen.split_k = ks;
        ml.cpad = ml.q * kMfmaChunk;
        return true;
    };
    ml.direct = direct_ok && t.mfma_kind != 1 && t.mfma_kind != 3 && direct_layout();
    if (t.mfma_kind == 2 && !ml.direct) return PP_ERR_UNSUPPORTED;
    if (t.split_k > 1 && !ml.direct) return PP_ERR_UNSUPPORTED;      // only the direct-load kernel splits the reduction
    // The batch is one tall virtual image: image n's output row oy is virtual row n*po + oy, and the
    // matching input rows start at virtual input row n*po*S, so that a tile may straddle images; the
    // rows between images read as zeros (they are the padding) and their outputs are not stored.
    if (!ml.direct) {
        ml.po = hp.ho + (pad + S - 1) / S;
        if (hp.pool && (ml.po & 1)) ++ml.po;
        const int64_t vrows = (int64_t)hp.n_hint * ml.po - (ml.po - hp.ho);
        const int step = hp.pool ? 2 : 1;
        ml.pairs = (hp.w & 1) == 0;
        auto staged_cols = [&](int tc) { return ((tc - 1) * S + KS + 2) & ~1; };
        auto pair_groups = [&](int tr, int tc) { return (((tr - 1) * S + KS) * (staged_cols(tc) / 2) + 15) / 16; };
        auto lds_need = [&](int tr, int tc) -> int64_t {
            const int64_t xbuf = (int64_t)pair_groups(tr, tc) * 32 * kMfmaPixelBytes;
            const int64_t main = 2 * xbuf + 2 * ml.wbuf_bytes;
            const int64_t out = (int64_t)kMfmaFilters * ((tr * tc + 7) / 8 * 8) * 2;
            return std::max(main, out) + kMfmaFilters * 4;      // + the workgroup's bias values
        };
        auto fits = [&](int tr, int tc, int waves, int ntw) {
            return lds_need(tr, tc) <= kMfmaMaxDynamicLds && (pair_groups(tr, tc) + waves / 2 - 1) / (waves / 2) <= mfma_max_units(waves, ntw);
        };
        auto evaluate = [&](int waves, int ntw, int& btr, int& btc, int64_t& bwgs) {
            const int slots = 32 * ntw * waves;
            double bcost = 1e300;
            btr = btc = 0;
            bwgs = 0;
            for (int tc = step; tc <= std::min(slots, (hp.wo + step - 1) / step * step); tc += step) {
                int tr = (int)std::min<int64_t>(slots / tc, (vrows + step - 1) / step * step);
                tr = tr / step * step;
                while (tr >= step && !fits(tr, tc, waves, ntw)) tr -= step;
                if (tr < step) continue;
                const int64_t tiles = (int64_t)((hp.wo + tc - 1) / tc) * ((vrows + tr - 1) / tr);
                const double halo = (double)((tr - 1) * S + KS) * staged_cols(tc) / ((double)tr * tc * S * S);
                // matrix-core work of all tiles, extra for the halo's staging traffic, and a preference for
                // wide tiles: rows are loaded and stored in pieces of tc elements, and pieces below 128 bytes
                // waste memory transactions
                double cost = (double)tiles * slots * (1.0 + 0.5 * (halo - 1.0)) * (1.0 + 8.0 / tc);
                if (cost < bcost - 1e-9) {
                    bcost = cost;
                    btr = tr;
                    btc = tc;
                    bwgs = tiles * ml.fb;
                }
            }
        };
        if (t.tiles_per_wave != 0 && t.tiles_per_wave != 2 && t.tiles_per_wave != 4) return PP_ERR_UNSUPPORTED;
        if (t.wg_waves != 0 && t.wg_waves != 4 && t.wg_waves != 8) return PP_ERR_UNSUPPORTED;
        // Larger tiles re-read less (weights once per tile, a thinner halo) and eight wavefronts hide each
        // other's LDS and barrier latency, but the layer needs enough workgroups to fill 256 compute units.
        static const int kShapes[3][2] = {{8, 4}, {4, 4}, {4, 2}};
        int btr = 0, btc = 0;
        ml.waves = 0;
        for (int k = 0; k < 3; ++k) {
            const int waves = kShapes[k][0], ntw = kShapes[k][1];
            if ((t.wg_waves && t.wg_waves != waves) || (t.tiles_per_wave && t.tiles_per_wave != ntw)) continue;
            int tr = 0, tc = 0;
            int64_t wgs = 0;
            evaluate(waves, ntw, tr, tc, wgs);
            if (tr == 0) continue;
            ml.waves = waves;
            ml.ntw = ntw;
            btr = tr;
            btc = tc;
            if (wgs >= 480) break;          // otherwise try the next smaller shape (the last one stands)
        }
        if (ml.waves == 0) return PP_ERR_UNSUPPORTED;
        ml.tr = btr;
        ml.tc = btc;
        if (t.tile_rows || t.tile_cols) {
            if (t.tile_rows < step || t.tile_cols < step || t.tile_rows % step || t.tile_cols % step) return PP_ERR_UNSUPPORTED;
            ml.tr = t.tile_rows;
            ml.tc = t.tile_cols;
        }
        if (ml.tr < 1 || ml.tc < 1 || ml.tr * ml.tc > 32 * ml.ntw * ml.waves || !fits(ml.tr, ml.tc, ml.waves, ml.ntw)) return PP_ERR_UNSUPPORTED;
        ml.trp = (ml.tr - 1) * S + KS;
        ml.twpa = staged_cols(ml.tc);
        ml.xbuf_bytes = pair_groups(ml.tr, ml.tc) * 32 * kMfmaPixelBytes;
        ml.out_pitch = (ml.tr * ml.tc + 7) / 8 * 8;
        ml.lds_bytes = lds_need(ml.tr, ml.tc);
        const int ow = hp.out_w, otc = hp.pool ? ml.tc / 2 : ml.tc;
        ml.gw = 1;
        for (int g = 8; g > 1; g /= 2)
            if (ow % g == 0 && otc % g == 0) {
                ml.gw = g;
                break;
            }
        hp.chosen.wg_waves = ml.waves;
        hp.chosen.tile_rows = ml.tr;
        hp.chosen.tile_cols = ml.tc;
        hp.chosen.tiles_per_wave = ml.ntw;
        hp.chosen.mfma_kind = 1;
    }

    // weights: scatter the kept kernels into zero-filled operand fragments
    const Canonical& cn = hp.canon;
    ml.wpk.assign((size_t)ml.fb * ml.q * KK * 2 * 64 * 8, 0);
    ml.bias_pad.assign((size_t)ml.fb * kMfmaFilters, 0.0f);
    for (int co = 0; co < hp.c_out; ++co) ml.bias_pad[co] = hp.bias[co];
    std::vector<int> taps_of((size_t)hp.num_patterns * hp.taps);
    for (int p = 0; p < hp.num_patterns; ++p) {
        int j = 0;
        for (int tp = 0; tp < KK; ++tp)
            if ((hp.masks[p] >> tp) & 1u) taps_of[(size_t)p * hp.taps + j++] = tp;
    }
    for (int pos = 0; pos < hp.c_out; ++pos) {
        const int co = cn.perm[pos];
        const int fbi = co / kMfmaFilters, half = (co % kMfmaFilters) / 32, row = co % 32;
        for (int64_t e = hp.filt_off[pos]; e < hp.filt_off[pos + 1]; ++e) {
            const int ci = cn.kidx[e], qi = ci / kMfmaChunk, cl = ci % kMfmaChunk;
            const int lane = row + 32 * (cl / 8), j8 = cl % 8;
            for (int j = 0; j < hp.taps; ++j) {
                const int tp = taps_of[(size_t)cn.kpat[e] * hp.taps + j];
                const size_t frag = (((size_t)fbi * ml.q + qi) * KK + tp) * 2 + half;
                ml.wpk[(frag * 64 + lane) * 8 + j8] = f32_to_f16_rne(cn.wpacked[(size_t)e * hp.taps + j]);
            }
        }
    }
    return PP_OK;
}

pp_status_t unpack_stream(const HostPlan& hp, int32_t* kidx, uint8_t* kpat, float* w) {
    if (!hp.tiled || hp.taps != 4 || hp.tl.covered) return PP_ERR_UNSUPPORTED;
    const TiledLayout& tl = hp.tl;
    const int EW = tl.entry_words;
    // slot -> lowest pattern id carrying that mask
    std::vector<int> pid_of(kBuiltinPatterns, -1);
    for (int p = hp.num_patterns - 1; p >= 0; --p) {
        int s = builtin_slot(hp.masks[p]);
        if (s >= 0) pid_of[s] = p;
    }
    const uint32_t chan_stride = (uint32_t)(tile_geom(tl.lw, tl.r, hp.dtype == PP_F16 ? 2 : 4).chs * (hp.dtype == PP_F16 ? 2 : 4));
    struct Rec { int pat, ci; float w[4]; };
    std::vector<std::vector<Rec>> per_filter(hp.c_out);
    for (int g = 0; g < tl.groups; ++g)
        for (int s = 0; s < tl.ks; ++s) {
            size_t e = (size_t)tl.wave_off[((size_t)g * tl.ks + s) * tl.sw];
            for (int q = 0; q < tl.chunks; ++q) {
                int ci = -1;
                for (;; ++e) {
                    const uint32_t* ent = &tl.stream[e * EW];
                    if (ent[0] == kEndCode) {
                        ++e;
                        break;
                    }
                    const uint32_t chan = ent[hp.dtype == PP_F16 ? 3 : 1];
                    if (chan != kSameChannel)
                        ci = tl.chan_map[((size_t)(g / tl.wf) * tl.chunks + q) * tl.cc + (int)(chan / chan_stride)];
                    int code = (int)ent[0];
                    int pos = tl.slot_pos[(size_t)g * tl.f + code / tl.np];
                    if (pos < 0 || ci < 0) return PP_ERR_UNSUPPORTED;
                    Rec r;
                    r.pat = pid_of[code % tl.np];
                    r.ci = ci;
                    if (hp.dtype == PP_F16) {
                        for (int j = 0; j < 4; ++j) r.w[j] = f16_to_f32((uint16_t)(ent[1 + j / 2] >> (16 * (j & 1))));
                    } else {
                        std::memcpy(r.w, &ent[4], 16);
                    }
                    per_filter[pos].push_back(r);
                }
            }
        }
    int64_t out = 0;
    for (int pos = 0; pos < hp.c_out; ++pos) {
        auto& v = per_filter[pos];
        std::sort(v.begin(), v.end(), [](const Rec& a, const Rec& b) {
            if (a.pat != b.pat) return a.pat < b.pat;
            return a.ci < b.ci;
        });
        for (const Rec& r : v) {
            if (out >= hp.canon.k_kept) return PP_ERR_UNSUPPORTED;
            kidx[out] = r.ci;
            kpat[out] = (uint8_t)r.pat;
            std::memcpy(&w[out * 4], r.w, 16);
            ++out;
        }
    }
    return out == hp.canon.k_kept ? PP_OK : PP_ERR_UNSUPPORTED;
}

}  // namespace ppc
