// Host planner of libxl: graph validation, storage map, tile / halo selection
// against the LDS budget (paper section 3.2), launch descriptors.
#include "plan.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstdio>
#include <cstring>
#include <map>
#include <set>
#include <tuple>

namespace xl {

// The table of compiled kernel variants (the kernels themselves are instantiated from the same list).
const std::vector<Variant> &variants()
{
    static const std::vector<Variant> v = {
#define X(ID, KIND, MF1, K1, NRT1, NPT1, MF2, NRT2, NPT2, K2A, K2B, SC, PX1) \
    Variant{ID, KIND, MF1, K1, NRT1, NPT1, MF2, NRT2, NPT2, K2A, K2B, SC, PX1, 0},
        XL_VARIANT_LIST(X)
#undef X
#define X(ID, KIND, MF1, K1, NRT1, NPT1, MF2, NRT2, NPT2, K2A, K2B, SC, PX1) \
    Variant{ID, KIND, MF1, K1, NRT1, NPT1, MF2, NRT2, NPT2, K2A, K2B, SC, PX1, 1},
        XL_VARIANT_LIST_B3(X)
#undef X
    };
    return v;
}

static int ceil_div(int a, int b) { return (a + b - 1) / b; }
static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Extent of the producing layer's output that `t` consecutive outputs of a
// K-wide window at stride s depend on (paper section 3.2: every output pixel
// depends on all inputs inside the filter window).
int required_extent(int t, int k, int s) { return (t - 1) * s + k; }

static bool is_prime(int v)
{
    if (v < 2) return false;
    for (int d = 2; d * d <= v; ++d)
        if (v % d == 0) return false;
    return true;
}

// Paper section 3.2, tuner: complementary non-trivial factors of the output
// size; a prime size is replaced by the next larger non-prime.
int tuner_candidates(int out_size, int *tile, int *grid, int cap)
{
    if (out_size < 1) return 0;
    int base = out_size;
    while (base > 3 && is_prime(base)) ++base;
    int n = 0;
    for (int t = 2; t < base; ++t) {
        if (base % t) continue;
        if (n < cap && tile && grid) {
            tile[n] = t;
            grid[n] = base / t;
        }
        ++n;
    }
    return n;
}

// ----------------------------------------------------------------------------
// Block description handed to the tile search
// ----------------------------------------------------------------------------
struct ConvSpec {
    int layer = -1;
    int cin = 0, cout = 0, k = 1, stride = 1, pad = 0, relu = 0;
};

struct BlockSpec {
    int kind = KIND_SINGLE;
    ConvSpec c1;
    ConvSpec c1b;                   // second producer of a two-producer merge block
    int n1 = 1;                     // stage-1 convolutions summed in the LDS tile
    int relu_mid = 0;               // activation of that sum
    int n2 = 0;
    ConvSpec c2[2];
    int coff2[2] = {0, 0};
    int pool_k = 0, pool_s = 1, pool_p = 0;
    int N = 0, Cin = 0, H = 0, W = 0;
    int H1 = 0, W1 = 0, Ho = 0, Wo = 0;
    int H2 = 0, W2 = 0;             // KIND_FUSED2P: stage-2 output extent, pooled (pool_k, pool_s) into Ho x Wo
    int relu_out = 0;
    bool shortcut = false;
    bool gap = false;               // KIND_SINGLE followed by a global average pooling: one tile per image
    long long alg_bytes = 0;        // algorithmic HBM bytes of the fused block
};

struct Choice {
    bool ok = false;
    double cost = 0;
    Variant v{};
    int threads = 0, waves_r1 = 0, waves_r2 = 1, csplit = 1;
    int th = 0, tw = 0, mh = 0, mw = 0, ih = 0, iw = 0, vw2 = 0;
    int pth = 0, ptw = 0;           // KIND_FUSED2P: tile of the pooled output (th x tw: the stage-2 tile under it)
    int tiles_y = 0, tiles_x = 0;
    int chunk_kg = 0, chunk_kg2[2] = {1, 1};
    int mid_floats = 0, buf_floats = 0, w_off1 = 0;
    int lds_bytes = 0, occ = 1;
    long long flops_exec = 0;
    bool lds_rejected = false;
};

static std::vector<int> tile_candidates(int extent)
{
    std::set<int> s;
    for (int g = 1; g <= extent; ++g) s.insert(ceil_div(extent, g));
    return std::vector<int>(s.begin(), s.end());
}

// matrix-pipe cycles of one K step of one (row tile, pixel tile) pair and tap: four fp32 operations of
// 64 / 32 cycles, or three bf16 ones of 32 / 16 cycles over twice the channels
static double kstep_clk(int mf, int pr) { return pr ? 3 * (mf == 32 ? 32.0 : 16.0) : 4 * (mf == 32 ? 64.0 : 32.0); }

// Largest number of K steps per chunk the stagers can hold, shortened so that one chunk keeps
// the matrix cores busy for about `want_clk` cycles (amortises the per-chunk barrier) and no more.
static int pick_chunk(int nkg, int x_units_per_kg, int w_items_per_kg, int threads, double clk_per_kg, double want_clk)
{
    int cap = nkg;
    if (x_units_per_kg > 0) cap = std::min(cap, STAGE_UNITS * threads / x_units_per_kg);
    cap = std::min(cap, MAX_W_CHUNK_BYTES / (16 * std::max(w_items_per_kg, 1)));
    if (cap < 1) return 0;
    int want = (int)std::ceil(want_clk / std::max(clk_per_kg, 1.0));
    int chunk = std::max(1, std::min(cap, want));
    const int nchunks = ceil_div(nkg, chunk);
    return std::min(cap, ceil_div(nkg, nchunks));       // balance the chunks
}

// Model of one candidate.  Times in seconds on a nominal MI355X (2.4 GHz, 8 TB/s).
static void evaluate(const BlockSpec &b, const xl_plan &pl, Choice &c)
{
    const Variant &v = c.v;
    const int nw = c.threads / 64;
    const int mf1 = v.mf1;
    const int nrt1 = ceil_div(b.c1.cout, mf1), nkg1 = ceil_div(b.c1.cin, kc_of(mf1, v.pr));
    const int taps1 = b.c1.k * b.c1.k;
    const int npx1 = c.mh * c.mw;
    const int wg_rt = c.waves_r1 * v.nrt1;
    const double wave1 = (double)v.nrt1 * v.npt1 * nkg1 * taps1 * kstep_clk(mf1, v.pr);
    double simd[4] = {0, 0, 0, 0};
    for (int w = 0; w < nw; ++w) {
        const int wr = w % c.waves_r1, wp = w / c.waves_r1;
        const int rt0 = wr * v.nrt1, pt0 = wp * v.npt1;
        const int rt_end = std::min(nrt1, wg_rt);
        if (rt0 < rt_end && pt0 * mf1 < npx1) simd[w % 4] += wave1;
    }
    double t1 = *std::max_element(simd, simd + 4) * b.n1;
    if (v.px1 < 0) t1 *= -v.px1 / 4.0;      // only -px1 of the 4 channel slots carry matrix operations
    if (v.px1 > 0) t1 *= 0.9;       // planar input chunks: no register staging, no vector-ALU work in the K loop
    int barriers = ceil_div(nkg1, c.chunk_kg) * b.n1;
    if (b.kind == KIND_DW) {
        // vector ALU: staging one float4 per (channel group, input pixel), then per (channel group,
        // intermediate pixel) one LDS read and 4 multiply-adds per tap; ~8 issue cycles per wave instruction
        const double ncg = ceil_div(b.Cin, 4);
        const double waves_per_simd = nw / 4.0;
        t1 = (ncg * c.ih * c.iw * 12.0 + ncg * npx1 * (taps1 * 6.0 + 16.0)) / c.threads * waves_per_simd * 8.0;
        barriers = 1;
    }
    double t2 = 0;
    long long flops2 = 0;
    if (b.kind == KIND_FUSED2 || b.kind == KIND_DW || b.kind == KIND_FUSED2P) {
        const int mf2 = v.mf2, NRT2 = v.nrt2, NPT2 = v.npt2;
        const int npt2 = ceil_div(c.th * c.vw2, mf2);
        const int wg_rt2 = c.waves_r2 * NRT2, wg_pt2 = (nw / c.waves_r2) * NPT2;
        for (int ci = 0; ci < b.n2; ++ci) {
            const ConvSpec &s = b.c2[ci];
            const int nrt = ceil_div(s.cout, mf2), nkg = ceil_div(s.cin, kc_of(mf2, v.pr));
            const int per = std::min(nrt, ceil_div(nrt, c.csplit));
            const double wave2 = (double)NRT2 * NPT2 * nkg * s.k * s.k * kstep_clk(mf2, v.pr);
            for (int rp = 0; rp < per; rp += wg_rt2)
                for (int pp = 0; pp < npt2; pp += wg_pt2) {
                    double s2[4] = {0, 0, 0, 0};
                    for (int w = 0; w < nw; ++w) {
                        const int r0 = rp + (w % c.waves_r2) * NRT2, p0 = pp + (w / c.waves_r2) * NPT2;
                        if (r0 < per && p0 < npt2) s2[w % 4] += wave2;
                    }
                    t2 += *std::max_element(s2, s2 + 4) + 2500.0;       // + epilogue / prologue of the pass
                    if (b.kind == KIND_FUSED2P)     // pooling of the pass from LDS: two barriers, one float4 window per item
                        t2 += 700.0 + (double)std::min(wg_rt2, per - rp) * mf2 / 4 * c.pth * c.ptw * b.pool_k * b.pool_k * 8.0 /
                                          c.threads * 4;
                    barriers += ceil_div(nkg, c.chunk_kg2[ci]);
                    flops2 += 2LL * std::min(wg_rt2, per - rp) * mf2 * std::min(wg_pt2, npt2 - pp) * mf2 * nkg *
                              kc_of(mf2, v.pr) * s.k * s.k;
                }
        }
    } else if (b.kind == KIND_POOL) {
        t2 = (double)ceil_div(b.c1.cout, 4) * c.th * c.tw * b.pool_k * b.pool_k * 8.0 / c.threads * 4;
    }
    const double ovh = (v.kind == KIND_POOLS ? 2500.0 : 6000.0) + 350.0 * barriers;   // a resident workgroup pays start-up once
    const double wg_clk = t1 + t2 + ovh;
    const long long nwg = (long long)c.tiles_x * c.tiles_y * c.csplit * b.N;
    const double rounds = std::ceil((double)nwg / pl.num_cus);
    const double t_mfma = rounds * wg_clk * (c.occ >= 2 ? 1.0 : 1.08) / 2.4e9;

    // memory side: algorithmic bytes at HBM speed plus per-workgroup cache-line traffic at L2 speed
    auto lines = [](int w) { return (double)((w * 4 + 64 + 127) / 128) * 128.0; };
    const double in_wg = (double)b.Cin * c.ih * lines(c.iw) * c.csplit;
    const bool two_stage = b.kind == KIND_FUSED2 || b.kind == KIND_DW || b.kind == KIND_FUSED2P;
    const double out_ch = two_stage ? (double)(b.c2[0].cout + (b.n2 > 1 ? b.c2[1].cout : 0)) : b.c1.cout;
    const double out_wg = b.kind == KIND_FUSED2P ? out_ch * c.pth * lines(c.ptw)
                                                 : out_ch * c.th * lines(c.tw) * (b.shortcut ? 2.0 : 1.0);
    const double t_mem = (double)b.alg_bytes / 8.0e12 + (in_wg + out_wg) * c.tiles_x * c.tiles_y * b.N / 24.0e12;
    c.cost = std::max(t_mfma, t_mem) + 0.15 * std::min(t_mfma, t_mem);
    // executed multiply-adds: stage 1 covers every row tile once per tile (per cout slice when fused),
    // with pixels and channels rounded up to whole matrix-core tiles
    const long long tiles = (long long)c.tiles_x * c.tiles_y * b.N;
    const long long s1 = b.kind == KIND_DW ? 2LL * b.Cin * npx1 * taps1
                                           : 2LL * nrt1 * mf1 * ceil_div(npx1, mf1) * mf1 * nkg1 * kc_of(mf1, v.pr) * taps1;
    c.flops_exec = tiles * (b.kind == KIND_SINGLE ? 1 : c.csplit) * s1 * b.n1 + tiles * c.csplit * flops2;
}

static std::vector<Choice> search(const BlockSpec &b, const xl_plan &pl, bool &lds_rejected, int pr)
{
    Choice best;
    std::map<std::tuple<int, int, int, int>, Choice> per_key;     // best per (variant, threads, tile)
    const std::vector<int> ths = tile_candidates(b.Ho), tws = tile_candidates(b.Wo);
    std::vector<std::pair<int, int>> tiles;
    if (b.gap) {
        tiles.push_back({b.Ho, b.Wo});          // the mean needs every pixel of the image in one workgroup
    } else if (pl.opts.force_tile_h > 0 && pl.opts.force_tile_w > 0) {
        tiles.push_back({std::min(pl.opts.force_tile_h, b.Ho), std::min(pl.opts.force_tile_w, b.Wo)});
    } else if (pl.opts.paper_tuner_only) {
        int t[64], g[64];
        const int n = std::min(64, tuner_candidates(std::max(b.Ho, b.Wo), t, g, 64));
        for (int i = 0; i < n; ++i) tiles.push_back({std::min(t[i], b.Ho), std::min(t[i], b.Wo)});
        if (tiles.empty()) tiles.push_back({b.Ho, b.Wo});
    } else {
        for (int th : ths)
            for (int tw : tws) tiles.push_back({th, tw});
    }
    bool any_lds_reject = false;
    for (const Variant &v : variants()) {
        if (v.kind == KIND_THIN) {
            // a first layer with a handful of input channels on the vector ALU, alone or with its max pooling
            // (columns of the variant: k1 = K, nrt1 = Cin, k2b = pooling window)
            const bool pooled = b.kind == KIND_POOL;
            if (pr != 0 || !(pooled || (b.kind == KIND_SINGLE && !b.gap))) continue;
            if (v.k1 != b.c1.k || v.nrt1 != b.c1.cin || v.k2b != (pooled ? b.pool_k : 0)) continue;
            const double taps = (double)b.c1.cin * b.c1.k * b.c1.k;
            const int rows16 = ceil_div(b.c1.cout, 16) * 16;
            // npt1 = 2: a lane owns the 2x2 block of convolution outputs under one pooled pixel (stride-2 layers only)
            const bool blocks = v.npt1 == 2;
            if (blocks && !(pooled && b.c1.stride == 2 && b.pool_s == 2 && b.pool_p == 0)) continue;
            for (int threads : {128, 192, 256, 512}) {
                if (pl.opts.force_threads > 0 && pl.opts.force_threads != threads) continue;
                if (blocks ? threads > 256 : threads < 256) continue;
                for (auto [th, tw] : tiles) {
                    Choice c;
                    c.v = v;
                    c.threads = threads;
                    c.waves_r1 = c.waves_r2 = 1;
                    c.th = th;
                    c.tw = tw;
                    c.vw2 = tw;
                    if (blocks) {
                        // (th + 1) x (tw + 1) lanes: the last row and column of blocks only supply neighbours
                        c.mh = th + 1;
                        c.mw = tw + 1;
                        const int lanes = c.mh * c.mw;
                        if (lanes > threads || (lanes + 64 <= threads && threads > 128)) continue;      // the smallest workgroup that holds the tile
                        if (lanes * 10 < threads * 7 && !(th == b.Ho && tw == b.Wo) && !(pl.opts.force_tile_h > 0)) continue;
                        c.ih = 4 * c.mh + 1;
                        c.iw = 4 * c.mw + 1;
                        c.tiles_y = ceil_div(b.Ho, th);
                        c.tiles_x = ceil_div(b.Wo, tw);
                        c.csplit = 1;
                        c.chunk_kg = 1;
                        c.lds_bytes = 2 * THIN_PCB * 3 * threads * 4;       // two tiles of 4 channels x 3 maxima per lane
                        if (c.lds_bytes > pl.lds_budget) {
                            any_lds_reject = true;
                            continue;
                        }
                        c.occ = std::max(1, std::min({pl.lds_per_cu / c.lds_bytes, 2048 / threads, 20 / (threads / 64)}));
                        const double nwg = (double)c.tiles_x * c.tiles_y * b.N;
                        // four multiply-adds per filter value, channel and lane, about 2.3 cycles each at full occupancy
                        const double wave_clk = rows16 * (4.0 * taps + 24.0) * 2.3 + 1500.0;
                        const double t_alu = nwg * (threads / 64) / (4.0 * pl.num_cus) * wave_clk / 2.4e9;
                        const double t_mem = (double)b.alg_bytes / 8.0e12;
                        c.cost = std::max(t_alu, t_mem) + 0.15 * std::min(t_alu, t_mem);
                        c.flops_exec = (long long)(nwg * threads * rows16 * taps * 8.0);
                        c.ok = true;
                        if (!best.ok || c.cost < best.cost) best = c;
                        per_key[std::make_tuple(v.id, threads, th, tw)] = c;
                        continue;
                    }
                    c.mh = pooled ? required_extent(th, b.pool_k, b.pool_s) : th;      // convolution outputs under the tile
                    c.mw = pooled ? required_extent(tw, b.pool_k, b.pool_s) : tw;
                    const int npx = c.mh * c.mw;
                    if (npx > threads) continue;                          // one lane per convolution output
                    if (th * tw * 16 >= 65536) continue;                 // index range of the kernel's divisions
                    // tiles that leave many lanes idle are not worth timing (the whole image may be smaller)
                    if (npx * 4 < threads * 3 && !(th == b.Ho && tw == b.Wo) && !(pl.opts.force_tile_h > 0)) continue;
                    c.ih = required_extent(c.mh, b.c1.k, b.c1.stride);
                    c.iw = required_extent(c.mw, b.c1.k, b.c1.stride);
                    c.tiles_y = ceil_div(b.Ho, th);
                    c.tiles_x = ceil_div(b.Wo, tw);
                    c.csplit = 1;
                    c.chunk_kg = 1;
                    c.lds_bytes = pooled ? 2 * 8 * threads * 4 : 0;      // two tiles of 8 channels x one float per lane
                    if (c.lds_bytes > pl.lds_budget) {
                        any_lds_reject = true;
                        continue;
                    }
                    c.occ = std::max(1, std::min(pl.lds_per_cu / std::max(c.lds_bytes, 1), 2048 / threads));
                    // one multiply-add instruction (4 cycles per wavefront) per filter value and output channel, every
                    // wavefront of the workgroup; 4 SIMDs per compute unit
                    const double nwg = (double)c.tiles_x * c.tiles_y * b.N;
                    const double wave_clk = rows16 * (taps + (pooled ? 4.0 : 2.0)) * 4.0 + 1500.0;
                    const double t_alu = std::ceil(nwg / pl.num_cus) * (threads / 64) / 4.0 * wave_clk / 2.4e9;
                    const double t_mem = (double)b.alg_bytes / 8.0e12;
                    c.cost = std::max(t_alu, t_mem) + 0.15 * std::min(t_alu, t_mem);
                    c.flops_exec = (long long)(nwg * threads * rows16 * taps * 2.0);
                    c.ok = true;
                    if (!best.ok || c.cost < best.cost) best = c;
                    per_key[std::make_tuple(v.id, threads, th, tw)] = c;
                }
            }
            continue;
        }
        const bool stream = v.kind == KIND_POOLS;          // conv -> pool as a stream of tiles: same block kind
        if ((v.kind != b.kind && !(stream && b.kind == KIND_POOL)) || v.k1 != b.c1.k || v.pr != pr) continue;
        const bool dw = b.kind == KIND_DW;                  // depthwise stage 1: no matrix-core tiling of layer 1
        const bool pool2 = b.kind == KIND_FUSED2P;          // stage 2 is pooled before it is stored
        const bool two = b.kind == KIND_FUSED2 || dw || pool2;       // stage 2 runs convolutions from the LDS tile
        if (two) {
            if (v.k2a != b.c2[0].k || v.k2b != (b.n2 > 1 ? b.c2[1].k : 0) || v.sc != (b.shortcut ? 1 : 0)) continue;
        }
        if (b.n1 == 2 && !(v.kind == KIND_FUSED2 && v.k1 == 1 && v.k2a == 1 && v.k2b == 0 && v.sc == 0)) continue;
        // variants whose stage 1 reads planar input chunks: a 1x1 filter, stride 1, no padding, whole
        // K steps of channels; the tile's ih rows of iws floats must fit px * 64 floats per channel
        // px1 < 0: the first layer's channels are packed two per channel slot (-px1 slots used): 32-wide
        // tile, at most -2 * px1 input channels
        if (v.px1 < 0 && !(v.mf1 == 32 && b.c1.cin <= -2 * v.px1)) continue;
        const int px = v.px1 > 0 ? v.px1 : 0;
        if (px > 0 && !(b.c1.k == 1 && b.c1.stride == 1 && b.c1.pad == 0 && b.c1.cin % kc_of(v.mf1) == 0)) continue;
        const int mf1 = v.mf1;
        const int nrt1 = ceil_div(b.c1.cout, mf1), nkg1 = ceil_div(b.c1.cin, kc_of(mf1, v.pr));
        const int frows = v.pr ? 2 : 1;         // 1 KB filter rows per (K step, tap, row tile): hi and lo when split
        const int taps1 = b.c1.k * b.c1.k;
        for (int threads : {256, 512}) {
            if (pl.opts.force_threads > 0 && pl.opts.force_threads != threads) continue;
            const int nw = threads / 64;
            for (int wr = 1; wr <= nw; wr *= 2) {
                const int wg_rt = wr * v.nrt1;
                if (dw && wr > 1) continue;
                if (!dw && b.kind != KIND_SINGLE && wg_rt < nrt1) continue;     // stage 1 must produce every channel
                if (!dw && wr > 1 && (wr / 2) * v.nrt1 >= nrt1) continue;       // more row waves than row tiles
                const int px_cap = dw ? (1 << 30) : (nw / wr) * v.npt1 * mf1;
                for (auto [th, tw] : tiles)
                for (double want_clk : {16000.0, 8000.0}) {     // longer chunks = fewer barriers, if LDS allows
                    Choice c;
                    c.v = v;
                    c.threads = threads;
                    c.waves_r1 = wr;
                    c.th = th;
                    c.tw = tw;
                    if (pool2) {        // (th, tw) walks the pooled output; the stage-2 tile is what its windows cover
                        c.pth = th;
                        c.ptw = tw;
                        c.th = required_extent(th, b.pool_k, b.pool_s);
                        c.tw = required_extent(tw, b.pool_k, b.pool_s);
                    }
                    c.vw2 = c.tw;
                    if (b.kind == KIND_SINGLE) {
                        c.mh = th;
                        c.mw = tw;
                    } else if (b.kind == KIND_POOL) {
                        c.mh = required_extent(th, b.pool_k, b.pool_s);
                        c.mw = required_extent(tw, b.pool_k, b.pool_s);
                    } else {
                        int P = 0, ext = 0;
                        for (int i = 0; i < b.n2; ++i) P = std::max(P, b.c2[i].pad);
                        for (int i = 0; i < b.n2; ++i) ext = std::max(ext, b.c2[i].k - b.c2[i].pad);
                        const int s2 = b.c2[0].stride;
                        c.mh = (c.th - 1) * s2 + ext + P;
                        c.mw = (c.tw - 1) * s2 + ext + P;
                    }
                    if (c.mh * c.mw > px_cap) continue;
                    c.ih = required_extent(c.mh, b.c1.k, b.c1.stride);
                    c.iw = required_extent(c.mw, b.c1.k, b.c1.stride);
                    if (px > 0 && c.ih * ((c.iw + 3) / 4 * 4) > px * 64) continue;
                    c.tiles_y = ceil_div(b.Ho, th);
                    c.tiles_x = ceil_div(b.Wo, tw);
                    // stage-1 chunk: input tile chunk + filter chunk per buffer
                    const int x_per_kg = gps_of(mf1, v.pr) * c.ih * ((c.iw + 3) / 4 * 4);       // LDS rows hold whole 4-pixel units
                    const int w_per_kg = taps1 * wg_rt * 64 * frows;
                    const double clk1 = (double)(nw / 4.0) * v.nrt1 * v.npt1 * taps1 * kstep_clk(mf1, v.pr);
                    const int x_units_per_kg = gps_of(mf1, v.pr) * c.ih * ceil_div(c.iw, 4);     // 4-pixel row pieces
                    c.chunk_kg = dw ? 1 : pick_chunk(nkg1, px > 0 ? 0 : x_units_per_kg, w_per_kg, threads, clk1, want_clk);
                    if (px > 0)     // planar chunk: kc x px x 16 quads per K step, at most PLANAR_SLOTS wave loads per wave
                        c.chunk_kg = std::min(c.chunk_kg, PLANAR_SLOTS * nw * 64 / (kc_of(mf1) * px * 16));
                    if (c.chunk_kg < 1) continue;
                    if (stream && c.chunk_kg < nkg1) continue;        // the stream kernel keeps the whole reduction in one chunk
                    c.w_off1 = c.chunk_kg * x_per_kg * 4 + 16;        // + slack for a left-edge unit running past the last row
                    if (px > 0) c.w_off1 = c.chunk_kg * kc_of(mf1) * px * 64;
                    int buf1 = c.w_off1 + c.chunk_kg * w_per_kg * 4;
                    c.mid_floats = b.kind == KIND_SINGLE ? 0 : nrt1 * mf1 / 4 * c.mh * c.mw * 4;
                    if (dw) {       // the whole input tile, every channel, staged once; no filter chunk
                        const int ncg = ceil_div(b.Cin, 4);
                        c.w_off1 = 0;
                        buf1 = ncg * c.ih * ((c.iw + 3) / 4 * 4) * 4;
                        c.mid_floats = ceil_div(b.Cin, 16) * 4 * c.mh * c.mw * 4;     // whole K steps of the pointwise stage
                    }

                    std::vector<int> splits, wr2s, vws;
                    if (two) {
                        if (pl.opts.force_cout_split > 0) {
                            splits.push_back(pl.opts.force_cout_split);
                        } else {
                            int min_nrt = 1 << 30;
                            for (int i = 0; i < b.n2; ++i) min_nrt = std::min(min_nrt, ceil_div(b.c2[i].cout, v.mf2));
                            for (int s = 1; s <= 8 && s <= min_nrt; s *= 2) splits.push_back(s);
                        }
                        for (int w2 = 1; w2 <= nw; w2 *= 2) wr2s.push_back(w2);
                        const int tw2 = c.tw;
                        vws.push_back(tw2);
                        if (!pool2) {       // (the pooled form writes its tile to LDS pixel by pixel: no padded rows)
                            if (tw2 % 16 && (tw2 + 15) / 16 * 16 - tw2 <= 4) vws.push_back((tw2 + 15) / 16 * 16);
                            // rows of a multiple of 4 pixels let the epilogue move 4 pixels per access
                            if (tw2 % 4 && (tw2 + 3) / 4 * 4 != vws.back()) vws.push_back((tw2 + 3) / 4 * 4);
                        }
                    } else {
                        splits.push_back(b.kind == KIND_SINGLE ? ceil_div(nrt1, wg_rt) : 1);
                        wr2s.push_back(1);
                        vws.push_back(c.tw);
                    }
                    for (int cs : splits)
                        for (int w2 : wr2s)
                            for (int vw : vws) {
                                c.csplit = cs;
                                c.waves_r2 = w2;
                                c.vw2 = vw;
                                // staging buffers: passes with several chunks ping-pong between two buffers
                                // `multi` floats apart, a single-chunk pass only ever touches the first one
                                int multi = 0, single = 0;
                                ((!dw && ceil_div(nkg1, c.chunk_kg) > 1) ? multi : single) = buf1;
                                bool fits = true;
                                if (two) {
                                    const int NRT2 = v.nrt2, NPT2 = v.npt2;
                                    int max_per = 0;
                                    for (int i = 0; i < b.n2; ++i)
                                        max_per = std::max(max_per, ceil_div(ceil_div(b.c2[i].cout, v.mf2), cs));
                                    if (w2 > 1 && (w2 / 2) * NRT2 >= max_per) continue;     // idle row waves
                                    if (pool2) {
                                        // one pass must cover every pixel of the stage-2 tile, and its result
                                        // (row tiles of the pass x tile pixels) is pooled from the staging area
                                        if (ceil_div(c.th * vw, v.mf2) > (nw / w2) * NPT2) continue;
                                        single = std::max(single, w2 * NRT2 * v.mf2 * c.th * c.tw);
                                    }
                                    for (int i = 0; i < b.n2; ++i) {
                                        const int nkg2 = ceil_div(b.c2[i].cin, kc_of(v.mf2, v.pr));
                                        const int w2_per_kg = b.c2[i].k * b.c2[i].k * w2 * NRT2 * 64 * frows;
                                        const double clk2 = (double)(nw / 4.0) * NRT2 * NPT2 * b.c2[i].k * b.c2[i].k *
                                                            kstep_clk(v.mf2, v.pr);
                                        c.chunk_kg2[i] = pick_chunk(nkg2, 0, w2_per_kg, threads, clk2, want_clk);
                                        if (c.chunk_kg2[i] < 1) {
                                            fits = false;
                                            break;
                                        }
                                        const int bytes2 = c.chunk_kg2[i] * w2_per_kg * 4;
                                        int &slot = ceil_div(nkg2, c.chunk_kg2[i]) > 1 ? multi : single;
                                        slot = std::max(slot, bytes2);
                                    }
                                }
                                if (!fits) continue;
                                c.buf_floats = multi;
                                c.lds_bytes = (c.mid_floats + std::max(single, 2 * multi)) * 4;
                                if (c.lds_bytes > pl.lds_budget) {
                                    any_lds_reject = true;
                                    continue;
                                }
                                // waves per SIMD the registers allow: the conv -> pool kernels are built for 4
                                // (at most 128 registers), the others for 2
                                const int reg_waves = b.kind == KIND_POOL ? 16 : 8;
                                c.occ = std::max(1, std::min({pl.lds_per_cu / std::max(c.lds_bytes, 1), 2048 / threads,
                                                              reg_waves / nw}));
                                evaluate(b, pl, c);
                                c.ok = true;
                                if (!best.ok || c.cost < best.cost) best = c;
                                auto key = std::make_tuple(v.id, threads, th, tw);
                                auto it = per_key.find(key);
                                if (it == per_key.end() || c.cost < it->second.cost) per_key[key] = c;
                            }
                }
            }
        }
    }
    lds_rejected = !best.ok && any_lds_reject;
    // ranked list: the model's best first, then the best of other (variant, threads, tile) combinations
    std::vector<Choice> ranked;
    for (auto &kv : per_key) ranked.push_back(kv.second);
    std::sort(ranked.begin(), ranked.end(), [](const Choice &a, const Choice &b) { return a.cost < b.cost; });
    if (ranked.size() > (size_t)MAX_ALTERNATIVES) {
        // The model assumes at most two waves per SIMD; kernels that need fewer registers run three
        // 256-thread workgroups per CU when their LDS share allows it, which the model cannot rank.  Keep
        // the best of those among the candidates, for xl_tune to time.
        const size_t reserve = MAX_ALTERNATIVES / 5;
        std::vector<Choice> small;
        for (size_t i = MAX_ALTERNATIVES - reserve; i < ranked.size() && small.size() < reserve; ++i)
            if (ranked[i].threads == 256 && ranked[i].lds_bytes * 3 <= pl.lds_per_cu) small.push_back(ranked[i]);
        ranked.resize(MAX_ALTERNATIVES - small.size());
        ranked.insert(ranked.end(), small.begin(), small.end());
    }
    return ranked;
}

// ----------------------------------------------------------------------------
// Plan construction
// ----------------------------------------------------------------------------
struct Builder {
    xl_plan &pl;
    std::vector<int> producer;                    // tensor -> layer
    std::vector<std::vector<int>> consumers;      // tensor -> layers
    explicit Builder(xl_plan &p) : pl(p) {}

    xl_status fail(xl_status st, const std::string &msg)
    {
        pl.error = msg;
        return st;
    }

    xl_status validate()
    {
        const int nt = (int)pl.shapes.size(), nl = (int)pl.layers.size();
        producer.assign(nt, -1);
        consumers.assign(nt, {});
        for (int t = 0; t < nt; ++t) {
            const xl_shape &s = pl.shapes[t];
            if (s.n < 0 || s.c <= 0 || s.h <= 0 || s.w <= 0) return fail(XL_E_SHAPE, "tensor " + std::to_string(t) + ": non-positive extent");
            // kernels address inside one image with 32-bit byte offsets and count workgroups in an int
            if ((long long)s.c * s.h * s.w >= (1LL << 30) || (long long)s.n * s.c * s.h * s.w >= (1LL << 40))
                return fail(XL_E_UNSUPPORTED, "tensor " + std::to_string(t) + ": 2^30 or more elements per image");
        }
        for (int li = 0; li < nl; ++li) {
            const xl_layer &L = pl.layers[li];
            const std::string at = "layer " + std::to_string(li) + ": ";
            const int nin = (L.op == XL_ADD || L.op == XL_CONCAT) ? 2 : 1;
            for (int i = 0; i < nin; ++i) {
                if (L.in[i] < 0 || L.in[i] >= nt) return fail(XL_E_GRAPH, at + "input tensor id out of range");
            }
            if (L.out < 0 || L.out >= nt) return fail(XL_E_GRAPH, at + "output tensor id out of range");
            if (producer[L.out] >= 0) return fail(XL_E_GRAPH, at + "tensor written twice");
            for (int i = 0; i < nin; ++i)
                if (L.in[i] == L.out) return fail(XL_E_GRAPH, at + "in-place layers are not supported");
            const xl_shape &x = pl.shapes[L.in[0]], &y = pl.shapes[L.out];
            if (x.n != y.n) return fail(XL_E_SHAPE, at + "batch differs between input and output");
            switch (L.op) {
            case XL_CONV: {
                if (L.groups != 1 && !(L.groups == L.cin && L.cin == L.cout))
                    return fail(XL_E_UNSUPPORTED, at + "grouped convolution other than depthwise (groups == Cin == Cout)");
                if (L.groups != 1 && L.k != 3) return fail(XL_E_UNSUPPORTED, at + "depthwise filter size must be 3");
                if (L.k != 1 && L.k != 3 && L.k != 5) return fail(XL_E_UNSUPPORTED, at + "filter size must be 1, 3 or 5");
                if (L.stride < 1 || L.pad < 0 || L.pad > L.k) return fail(XL_E_SHAPE, at + "bad stride/pad");
                if (L.k == 1 && L.pad != 0) return fail(XL_E_UNSUPPORTED, at + "1x1 convolution with padding");
                if (L.cin != x.c || L.cout != y.c) return fail(XL_E_SHAPE, at + "channel counts do not match tensors");
                if (x.h + 2 * L.pad < L.k || x.w + 2 * L.pad < L.k) return fail(XL_E_SHAPE, at + "window larger than padded input");
                if (y.h != (x.h + 2 * L.pad - L.k) / L.stride + 1 || y.w != (x.w + 2 * L.pad - L.k) / L.stride + 1)
                    return fail(XL_E_SHAPE, at + "output extent does not follow floor((H+2p-k)/s)+1");
                if (L.w_slot < 0) return fail(XL_E_GRAPH, at + "convolution without a filter slot");
                break;
            }
            case XL_MAXPOOL:
                if (L.k < 1 || L.stride < 1 || L.pad < 0 || L.pad >= L.k) return fail(XL_E_SHAPE, at + "bad pooling window");
                if (x.c != y.c) return fail(XL_E_SHAPE, at + "pooling changes channels");
                if (x.h + 2 * L.pad < L.k || x.w + 2 * L.pad < L.k) return fail(XL_E_SHAPE, at + "window larger than padded input");
                if (y.h != (x.h + 2 * L.pad - L.k) / L.stride + 1 || y.w != (x.w + 2 * L.pad - L.k) / L.stride + 1)
                    return fail(XL_E_SHAPE, at + "output extent does not follow floor((H+2p-k)/s)+1");
                break;
            case XL_GLOBAL_AVGPOOL:
                if (x.c != y.c || y.h != 1 || y.w != 1) return fail(XL_E_SHAPE, at + "global pooling output must be [N,C,1,1]");
                break;
            case XL_ADD: {
                const xl_shape &b = pl.shapes[L.in[1]];
                if (memcmp(&x, &b, sizeof x) || memcmp(&x, &y, sizeof x)) return fail(XL_E_SHAPE, at + "add operands differ in shape");
                break;
            }
            case XL_CONCAT: {
                const xl_shape &b = pl.shapes[L.in[1]];
                if (x.n != b.n || x.h != b.h || x.w != b.w || y.h != x.h || y.w != x.w || y.c != x.c + b.c)
                    return fail(XL_E_SHAPE, at + "concat shapes do not line up");
                break;
            }
            default:
                return fail(XL_E_UNSUPPORTED, at + "unknown op");
            }
            for (int i = 0; i < nin; ++i) {
                // inputs must already exist: a graph input (never produced) or produced by an earlier layer
                bool produced_later = false;
                for (int lj = li; lj < nl; ++lj)
                    if (pl.layers[lj].out == L.in[i]) produced_later = true;
                if (produced_later) return fail(XL_E_GRAPH, at + "layers are not in topological order");
                consumers[L.in[i]].push_back(li);
            }
            producer[L.out] = li;
        }
        return XL_OK;
    }

    xl_status resolve_storage()
    {
        const int nt = (int)pl.shapes.size();
        pl.storage.assign(nt, Storage{});
        for (int t = 0; t < nt; ++t) pl.storage[t] = Storage{t, 0, pl.shapes[t].c, false, 0};
        // a concat input becomes a channel slice of the concat output (walk in reverse so nesting resolves)
        for (int li = (int)pl.layers.size() - 1; li >= 0; --li) {
            const xl_layer &L = pl.layers[li];
            if (L.op != XL_CONCAT) continue;
            const Storage out = pl.storage[L.out];
            int coff = out.coff;
            for (int i = 0; i < 2; ++i) {
                const int t = L.in[i];
                if (producer[t] < 0) return fail(XL_E_UNSUPPORTED, "concat of a graph input");
                if (consumers[t].size() != 1) return fail(XL_E_UNSUPPORTED, "a concat operand has another consumer");
                if (L.in[0] == L.in[1]) return fail(XL_E_UNSUPPORTED, "concat of a tensor with itself");
                pl.storage[t] = Storage{out.root, coff, out.ctot, false, 0};
                coff += pl.shapes[t].c;
            }
        }
        // consumers that read a channel slice are not supported (inputs are dense tensors)
        for (size_t li = 0; li < pl.layers.size(); ++li) {
            const xl_layer &L = pl.layers[li];
            if (L.op == XL_CONCAT) continue;
            const int nin = L.op == XL_ADD ? 2 : 1;
            for (int i = 0; i < nin; ++i)
                if (pl.storage[L.in[i]].root != L.in[i]) return fail(XL_E_UNSUPPORTED, "layer reads a concat operand directly");
        }
        return XL_OK;
    }

    void conv_spec(int li, ConvSpec &c) const
    {
        const xl_layer &L = pl.layers[li];
        c.layer = li;
        c.cin = L.cin;
        c.cout = L.cout;
        c.k = L.k;
        c.stride = L.stride;
        c.pad = L.pad;
        c.relu = L.relu;
    }

    long long tensor_bytes(int t) const
    {
        const xl_shape &s = pl.shapes[t];
        return 4LL * s.n * s.c * s.h * s.w;
    }
    long long tensor_elems(int t) const { return tensor_bytes(t) / 4; }
    long long weight_bytes(int li) const
    {
        const xl_layer &L = pl.layers[li];
        if (L.op != XL_CONV) return 0;
        long long b = 4LL * L.cout * (L.cin / std::max(L.groups, 1)) * L.k * L.k;
        if (L.scale_slot >= 0) b += 4LL * L.cout;
        if (L.shift_slot >= 0) b += 4LL * L.cout;
        return b;
    }
    long long layer_flops(int li) const
    {
        const xl_layer &L = pl.layers[li];
        if (L.op != XL_CONV) return 0;
        const xl_shape &y = pl.shapes[L.out];
        return 2LL * y.n * y.c * y.h * y.w * (L.cin / std::max(L.groups, 1)) * L.k * L.k;
    }
    // HBM bytes / stored elements of one layer run on its own
    void layer_traffic(int li, long long &bytes, long long &stores) const
    {
        const xl_layer &L = pl.layers[li];
        bytes = stores = 0;
        if (L.op == XL_CONCAT) return;
        bytes = tensor_bytes(L.in[0]) + tensor_bytes(L.out) + weight_bytes(li);
        if (L.op == XL_ADD) bytes += tensor_bytes(L.in[1]);
        stores = tensor_elems(L.out);
    }

    int packed_index(int layer, int mf, bool pairs = false, int pr = 0)
    {
        if (mf <= 0) pr = 0;        // depthwise and thin-layer tables have one form
        for (size_t i = 0; i < pl.packed.size(); ++i)
            if (pl.packed[i].layer == layer && pl.packed[i].mf == mf && pl.packed[i].pairs == pairs && pl.packed[i].pr == pr)
                return (int)i;
        const xl_layer &L = pl.layers[layer];
        PackedFilter p;
        p.layer = layer;
        p.mf = mf;
        p.pairs = pairs;
        p.pr = pr;
        if (mf < 0) {       // thin first layer: [Cout rounded up to 16][row of Cin*K*K floats, padded] and as many shifts
            p.nkg = p.nrt = 0;
            p.bytes = (size_t)ceil_div(L.cout, 16) * 16 * thin_row_floats(L.cin * L.k * L.k) * 4;
            p.aff_bytes = (size_t)ceil_div(L.cout, 16) * 16 * 4;
        } else if (mf == 0) {      // depthwise: [channel group][tap] float4 and [channel group][scale, shift] float4
            p.nkg = p.nrt = 0;
            p.bytes = (size_t)ceil_div(L.cout, 4) * L.k * L.k * 16;
            p.aff_bytes = (size_t)ceil_div(L.cout, 4) * 2 * 16;
        } else {
            p.nkg = pairs ? 1 : ceil_div(L.cin, kc_of(mf, pr));
            p.nrt = ceil_div(L.cout, mf);
            p.bytes = (size_t)p.nkg * L.k * L.k * p.nrt * 64 * 16 * (pr ? 2 : 1);
            p.aff_bytes = (size_t)p.nrt * (mf == 32 ? 4 : 1) * 64 * 16;
        }
        p.offset = 0;
        p.aff_offset = 0;
        pl.packed.push_back(p);
        return (int)pl.packed.size() - 1;
    }

    // Turn a searched choice into a launch step.
    xl_status make_block_step(const BlockSpec &b, int x_id, int y_id, int sc_id, int coff1, Step &st, Choice &ch,
                              const std::string &what)
    {
        bool lds_rejected = false;
        // split-bf16 kernels where the plan asks for them and a variant covers the block, fp32 ones otherwise
        std::vector<Choice> ranked = search(b, pl, lds_rejected, 0);
        if (pl.opts.precision == XL_PRECISION_BF16X3) {
            // the split-bf16 candidates first (the cost model cannot rank the two kinds against each other
            // well: blocks that are not bound by the matrix cores gain nothing from the split), then the
            // best fp32 ones, for xl_tune to choose from
            bool rej1 = false;
            std::vector<Choice> split = search(b, pl, rej1, 1);
            if (!split.empty()) {
                const size_t keep32 = MAX_ALTERNATIVES / 4;
                if (split.size() > MAX_ALTERNATIVES - keep32) split.resize(MAX_ALTERNATIVES - keep32);
                if (ranked.size() > keep32) ranked.resize(keep32);
                split.insert(split.end(), ranked.begin(), ranked.end());
                ranked.swap(split);
                lds_rejected = false;
            }
        }
        if (ranked.empty())
            return fail(lds_rejected ? XL_E_LDS_BUDGET : XL_E_UNSUPPORTED,
                        what + (lds_rejected ? ": no tile fits the LDS budget" : ": no kernel variant covers this block"));
        ch = ranked[0];
        fill_step(b, ch, x_id, y_id, sc_id, coff1, st);
        // the other candidates, for xl_tune to time on the device
        for (size_t i = 0; i < ranked.size(); ++i) {
            Step alt;
            fill_step(b, ranked[i], x_id, y_id, sc_id, coff1, alt);
            xl_group_info gi;
            memset(&gi, 0, sizeof gi);
            fill_info(gi, b, ranked[i]);
            st.alts.push_back(alt);
            st.alt_info.push_back(gi);
        }
        return XL_OK;
    }

    void fill_step(const BlockSpec &b, const Choice &ch, int x_id, int y_id, int sc_id, int coff1, Step &st)
    {
        st = Step{};
        st.type = STEP_BLOCK;
        st.variant = ch.v.id;
        st.cost_us = ch.cost * 1e6;
        st.threads = ch.threads;
        st.lds_bytes = ch.lds_bytes;
        st.x_id = x_id;
        st.y_id = y_id;
        st.sc_id = sc_id;
        st.conv_layer[0] = b.c1.layer;
        st.conv_layer[1] = st.conv_layer[2] = -1;
        st.packed[0] = packed_index(b.c1.layer, b.kind == KIND_DW ? 0 : (ch.v.kind == KIND_THIN ? -1 : ch.v.mf1), ch.v.px1 < 0, ch.v.pr);
        st.packed[1] = st.packed[2] = -1;
        BlockParams &p = st.bp;
        memset(&p, 0, sizeof p);
        p.N = b.N;
        p.Cin = b.Cin;
        p.H = b.H;
        p.W = b.W;
        p.H1 = b.H1;
        p.W1 = b.W1;
        p.Ho = b.Ho;
        p.Wo = b.Wo;
        p.gap = b.gap ? 1 : 0;
        const Storage &ys = pl.storage[y_id];
        p.Cy = ys.ctot;
        p.Csc = sc_id >= 0 ? pl.shapes[sc_id].c : 0;
        auto fill = [&](ConvW &w, const ConvSpec &s, int mf) {
            w.wp = nullptr;
            w.aff = nullptr;
            w.cin = s.cin;
            w.cout = s.cout;
            w.k = s.k;
            w.stride = s.stride;
            w.pad = s.pad;
            w.relu = s.relu;
            w.nkg = ceil_div(s.cin, kc_of(mf, ch.v.pr));
            w.nrt = ceil_div(s.cout, mf);
        };
        fill(p.c1, b.c1, ch.v.mf1);
        p.n1 = b.n1;
        p.relu_mid = b.relu_mid;
        st.conv_layer[3] = -1;
        st.packed[3] = -1;
        if (b.n1 == 2) {
            fill(p.c1b, b.c1b, ch.v.mf1);
            st.conv_layer[3] = b.c1b.layer;
            st.packed[3] = packed_index(b.c1b.layer, ch.v.mf1, false, ch.v.pr);
        }
        p.coff1 = ys.coff + coff1;
        const bool two = b.kind == KIND_FUSED2 || b.kind == KIND_DW || b.kind == KIND_FUSED2P;
        p.n2 = two ? b.n2 : 0;
        int P2 = 0;
        for (int i = 0; i < p.n2; ++i) {
            fill(p.c2[i], b.c2[i], ch.v.mf2);
            p.coff2[i] = ys.coff + b.coff2[i];
            st.conv_layer[1 + i] = b.c2[i].layer;
            st.packed[1 + i] = packed_index(b.c2[i].layer, ch.v.mf2, false, ch.v.pr);
            P2 = std::max(P2, b.c2[i].pad);
        }
        p.s2 = two ? b.c2[0].stride : (b.kind == KIND_POOL ? b.pool_s : 1);
        p.P2 = two ? P2 : (b.kind == KIND_POOL ? b.pool_p : 0);
        p.pool_k = b.pool_k;
        p.ps2 = b.kind == KIND_FUSED2P ? b.pool_s : 1;
        p.pp = b.kind == KIND_FUSED2P ? b.pool_p : 0;
        p.pth = ch.pth;
        p.ptw = ch.ptw;
        p.H2 = b.H2;
        p.W2 = b.W2;
        p.relu_out = b.relu_out;
        p.th = ch.th;
        p.tw = ch.tw;
        p.mh = ch.mh;
        p.mw = ch.mw;
        p.ih = ch.ih;
        p.iw = ch.iw;
        p.iws = (ch.iw + 3) / 4 * 4;
        p.tiles_x = ch.tiles_x;
        p.tiles_y = ch.tiles_y;
        p.csplit = ch.csplit;
        p.nblocks = ch.tiles_x * ch.tiles_y * ch.csplit * b.N;
        p.chunk_kg = ch.chunk_kg;
        p.chunk_kg2[0] = ch.chunk_kg2[0];
        p.chunk_kg2[1] = ch.chunk_kg2[1];
        p.waves_r1 = ch.waves_r1;
        p.waves_r2 = ch.waves_r2;
        p.vw2 = ch.vw2;
        auto rcp = [](int d) { return d <= 1 ? 0u : (unsigned)((1ull << 32) / (unsigned)d + 1); };
        p.rcp_mw = rcp(ch.mw);
        p.rcp_vw2 = rcp(ch.vw2);
        p.rcp_qrow = rcp(p.iws / 4);
        p.rcp_tiles = rcp(ch.tiles_x * ch.tiles_y);
        p.rcp_tcs = rcp(ch.tiles_x * ch.tiles_y * ch.csplit);
        p.rcp_csplit = rcp(ch.csplit);
        p.rcp_tiles_x = rcp(ch.tiles_x);
        {
            const bool pool2 = b.kind == KIND_FUSED2P;
            const int ph = pool2 ? ch.pth : ch.th, pw = pool2 ? ch.ptw : ch.tw;
            p.rcp_npo = rcp(ph * pw);
            p.rcp_pw = rcp(pw);
            // first input column of the tx = 0 tiles, as block_kernel derives it (output -> intermediate -> input)
            const int ox0 = pool2 ? -p.pp : 0;
            const int mx0 = b.kind == KIND_SINGLE ? ox0 : ox0 * p.s2 - p.P2;
            const int ix0 = mx0 * b.c1.stride - b.c1.pad;
            p.xs_left = std::max(0, -ix0);
            for (int e = 0; e < 2; ++e) {
                const int qpr = (ch.iw - (e ? p.xs_left : 0) + 3) >> 2;
                p.rcp_qpr[e] = rcp(qpr);
                p.rcp_upg[e] = rcp(ch.ih * qpr);
            }
        }
        p.mid_gstride = ch.mh * ch.mw * 4;
        p.in_gstride = ch.ih * p.iws * 4;
        p.lds_buf_off = ch.mid_floats;
        p.buf_stride = ch.buf_floats;
        p.w_off1 = ch.w_off1;
        p.stream_wgs = ch.v.kind == KIND_POOLS ? std::min(p.nblocks, pl.num_cus * std::max(ch.occ, 1)) : 0;
        if (ch.v.kind == KIND_THIN) p.rcp_qrow = rcp(ch.th * ch.tw);
    }

    void fill_info(xl_group_info &gi, const BlockSpec &b, const Choice &ch) const
    {
        gi.tile_h = b.kind == KIND_FUSED2P ? ch.pth : ch.th;
        gi.tile_w = b.kind == KIND_FUSED2P ? ch.ptw : ch.tw;
        gi.mid_h = b.kind == KIND_SINGLE ? 0 : ch.mh;
        gi.mid_w = b.kind == KIND_SINGLE ? 0 : ch.mw;
        gi.in_h = ch.ih;
        gi.in_w = ch.iw;
        gi.tiles_y = ch.tiles_y;
        gi.tiles_x = ch.tiles_x;
        gi.cout_split = ch.csplit;
        gi.workgroups = ch.tiles_x * ch.tiles_y * ch.csplit * b.N;
        gi.threads = ch.threads;
        gi.lds_bytes = ch.lds_bytes;
        gi.workgroups_per_cu = ch.occ;
        gi.chunk_channels = ch.v.kind == KIND_THIN ? b.c1.cin : ch.chunk_kg * kc_of(ch.v.mf1, ch.v.pr);
        gi.flops_executed = ch.flops_exec;
        gi.precision = ch.v.pr ? XL_PRECISION_BF16X3 : XL_PRECISION_FP32;
        if (b.kind == KIND_SINGLE) {
            gi.redundancy = 1.0;
        } else {
            const double unique = (double)b.H1 * b.W1;
            gi.redundancy = (double)ch.mh * ch.mw * ch.tiles_x * ch.tiles_y * ch.csplit / unique;
        }
    }

    // ---- single layers (also the unfused path) ---------------------------------
    xl_status single_step(int li, Step &st, xl_group_info *gi)
    {
        const xl_layer &L = pl.layers[li];
        const xl_shape &x = pl.shapes[L.in[0]], &y = pl.shapes[L.out];
        st = Step{};
        st.x_id = L.in[0];
        st.y_id = L.out;
        st.sc_id = st.b_id = -1;
        st.N = x.n;
        st.C = x.c;
        st.H = x.h;
        st.W = x.w;
        st.Ho = y.h;
        st.Wo = y.w;
        st.k = L.k;
        st.stride = L.stride;
        st.pad = L.pad;
        st.relu = L.relu;
        if (L.op == XL_CONV && L.groups != 1) {
            st.type = STEP_DEPTHWISE;
            st.conv_layer[0] = li;
            st.packed[0] = packed_index(li, 0);
        } else if (L.op == XL_CONV) {
            BlockSpec b;
            b.kind = KIND_SINGLE;
            conv_spec(li, b.c1);
            b.N = x.n;
            b.Cin = x.c;
            b.H = x.h;
            b.W = x.w;
            b.H1 = b.Ho = y.h;
            b.W1 = b.Wo = y.w;
            if (L.k == 1 && L.stride == 1 && L.pad == 0) {
                // a pointwise convolution does not care about rows: tile the image as one row of
                // H*W pixels, so that tiles are contiguous runs and no pixel tile is half empty
                b.W = b.W1 = b.Wo = x.h * x.w;
                b.H = b.H1 = b.Ho = 1;
            }
            long long by, stv;
            layer_traffic(li, by, stv);
            b.alg_bytes = by;
            Choice ch;
            xl_status s = make_block_step(b, L.in[0], L.out, -1, 0, st, ch, "layer " + std::to_string(li));
            if (s != XL_OK) return s;
            if (gi) fill_info(*gi, b, ch);
        } else if (L.op == XL_MAXPOOL) {
            st.type = STEP_MAXPOOL;
        } else if (L.op == XL_GLOBAL_AVGPOOL) {
            st.type = STEP_GAP;
        } else if (L.op == XL_ADD) {
            st.type = STEP_ADD;
            st.b_id = L.in[1];
            st.count = tensor_elems(L.out);
        }
        return XL_OK;
    }

    bool only_consumers(int tensor, std::initializer_list<int> ls) const
    {
        for (int c : consumers[tensor])
            if (std::find(ls.begin(), ls.end(), c) == ls.end()) return false;
        return !consumers[tensor].empty();
    }

    // ---- fused blocks -------------------------------------------------------------
    xl_status fused_group(const std::vector<int> &ids, int mode, GroupPlan &gp)
    {
        const std::string at = "block starting at layer " + std::to_string(ids[0]) + ": ";
        for (size_t i = 1; i < ids.size(); ++i)
            if (ids[i] <= ids[i - 1]) return fail(XL_E_GRAPH, at + "layer ids must ascend");
        const xl_layer &L1 = pl.layers[ids[0]];
        if (L1.op != XL_CONV) return fail(XL_E_UNSUPPORTED, at + "first layer of a fused block must be a convolution");
        for (size_t i = 1; i < ids.size(); ++i)
            if (pl.layers[ids[i]].op == XL_CONV && pl.layers[ids[i]].groups != 1)
                return fail(XL_E_UNSUPPORTED, at + "a depthwise convolution can only be the first layer of a block");
        if (L1.groups != 1 && (mode != XL_STRAIGHT || ids.size() != 2 || pl.layers[ids[1]].op != XL_CONV))
            return fail(XL_E_UNSUPPORTED, at + "a depthwise convolution fuses only with one following convolution (straight mode)");
        const int t_in = L1.in[0], t_mid = L1.out;
        const xl_shape &xs = pl.shapes[t_in], &ms = pl.shapes[t_mid];
        BlockSpec b;
        conv_spec(ids[0], b.c1);
        b.N = xs.n;
        b.Cin = xs.c;
        b.H = xs.h;
        b.W = xs.w;
        b.H1 = ms.h;
        b.W1 = ms.w;
        int y_id = -1, sc_id = -1;
        if (mode == XL_STRAIGHT) {
            if (ids.size() != 2) return fail(XL_E_UNSUPPORTED, at + "straight mode fuses exactly two layers");
            const xl_layer &L2 = pl.layers[ids[1]];
            if (L2.in[0] != t_mid) return fail(XL_E_GRAPH, at + "second layer does not read the first layer's output");
            if (!only_consumers(t_mid, {ids[1]})) return fail(XL_E_UNSUPPORTED, at + "the intermediate has a consumer outside the block");
            y_id = L2.out;
            if (L2.op == XL_CONV) {
                b.kind = L1.groups != 1 ? KIND_DW : KIND_FUSED2;
                b.n2 = 1;
                conv_spec(ids[1], b.c2[0]);
            } else if (L2.op == XL_MAXPOOL) {
                b.kind = KIND_POOL;
                b.pool_k = L2.k;
                b.pool_s = L2.stride;
                b.pool_p = L2.pad;
            } else if (L2.op == XL_GLOBAL_AVGPOOL) {
                b.kind = KIND_SINGLE;
                b.gap = true;
            } else {
                return fail(XL_E_UNSUPPORTED, at + "straight mode: second layer must be a convolution, max pooling or global average pooling");
            }
        } else if (mode == XL_SPLIT) {
            if (ids.size() < 3 || ids.size() > 5)
                return fail(XL_E_UNSUPPORTED, at + "split mode is conv -> {conv, conv} [-> concat [-> max pooling]]");
            const xl_layer &A = pl.layers[ids[1]], &B = pl.layers[ids[2]];
            if (A.op != XL_CONV || B.op != XL_CONV || A.in[0] != t_mid || B.in[0] != t_mid)
                return fail(XL_E_GRAPH, at + "split mode: both siblings must be convolutions reading the first layer's output");
            if (!only_consumers(t_mid, {ids[1], ids[2]})) return fail(XL_E_UNSUPPORTED, at + "the intermediate has a consumer outside the block");
            if (A.stride != B.stride) return fail(XL_E_UNSUPPORTED, at + "split siblings must share a stride");
            if (pl.shapes[A.out].h != pl.shapes[B.out].h || pl.shapes[A.out].w != pl.shapes[B.out].w)
                return fail(XL_E_UNSUPPORTED, at + "split siblings must produce the same extent");
            const Storage &sa = pl.storage[A.out], &sb = pl.storage[B.out];
            if (sa.root != sb.root || sa.root == A.out) return fail(XL_E_UNSUPPORTED, at + "split siblings must feed one concat");
            if (ids.size() >= 4) {
                const xl_layer &C = pl.layers[ids[3]];
                if (C.op != XL_CONCAT || C.out != sa.root) return fail(XL_E_GRAPH, at + "fourth layer must be the siblings' concat");
            }
            b.kind = KIND_FUSED2;
            b.n2 = 2;
            int pooled = -1;
            if (ids.size() == 5) {
                // straight after split: the concatenated result is max-pooled before it leaves the chip
                const xl_layer &Q = pl.layers[ids[4]];
                if (Q.op != XL_MAXPOOL || Q.in[0] != sa.root) return fail(XL_E_GRAPH, at + "fifth layer must be a max pooling of the concat");
                if (!only_consumers(sa.root, {ids[4]})) return fail(XL_E_UNSUPPORTED, at + "the concat has a consumer outside the block");
                if (pl.storage[sa.root].root != sa.root) return fail(XL_E_UNSUPPORTED, at + "the concat is itself a concat operand");
                const xl_shape &cs = pl.shapes[sa.root];
                // windows may hang over the image (padding): the block writes -FLT_MAX there, which a maximum ignores
                b.kind = KIND_FUSED2P;
                b.pool_k = Q.k;
                b.pool_s = Q.stride;
                b.pool_p = Q.pad;
                b.H2 = cs.h;
                b.W2 = cs.w;
                pooled = Q.out;
            }
            // the sibling with the larger filter first (the kernel variants are compiled for that order)
            const bool a_first = A.k > B.k || (A.k == B.k && A.cout >= B.cout);
            const int first = a_first ? ids[1] : ids[2], second = a_first ? ids[2] : ids[1];
            conv_spec(first, b.c2[0]);
            conv_spec(second, b.c2[1]);
            b.coff2[0] = pl.storage[pl.layers[first].out].coff - pl.storage[sa.root].coff;
            b.coff2[1] = pl.storage[pl.layers[second].out].coff - pl.storage[sa.root].coff;
            y_id = pooled >= 0 ? pooled : sa.root;
        } else if (mode == XL_MERGE && ids.size() == 4) {
            // two producers: {conv A, conv B}(x) -> add -> conv C   (paper Fig. 4c / Table 1 c.1)
            const xl_layer &B = pl.layers[ids[1]], &S = pl.layers[ids[2]], &C = pl.layers[ids[3]];
            if (B.op != XL_CONV || S.op != XL_ADD || C.op != XL_CONV) return fail(XL_E_GRAPH, at + "merge mode wiring");
            if (B.in[0] != t_in) return fail(XL_E_UNSUPPORTED, at + "both producers of a merge block must read the block input");
            if (!((S.in[0] == t_mid && S.in[1] == B.out) || (S.in[1] == t_mid && S.in[0] == B.out)) || C.in[0] != S.out)
                return fail(XL_E_GRAPH, at + "merge mode: the add must read both producers and feed the last convolution");
            if (!only_consumers(t_mid, {ids[2]}) || !only_consumers(B.out, {ids[2]}) || !only_consumers(S.out, {ids[3]}))
                return fail(XL_E_UNSUPPORTED, at + "an intermediate has a consumer outside the block");
            if (L1.cout != B.cout || L1.k != B.k || L1.stride != B.stride || L1.pad != B.pad)
                return fail(XL_E_UNSUPPORTED, at + "the two producers must share filter size, stride, padding and channels");
            if (L1.k != 1 || C.k != 1)
                return fail(XL_E_UNSUPPORTED, at + "two-producer merge blocks are built for 1x1 convolutions");
            b.kind = KIND_FUSED2;
            conv_spec(ids[1], b.c1b);
            b.n1 = 2;
            b.relu_mid = S.relu;
            b.n2 = 1;
            conv_spec(ids[3], b.c2[0]);
            y_id = C.out;
        } else if (mode == XL_MERGE) {
            if (ids.size() != 3) return fail(XL_E_UNSUPPORTED, at + "merge mode is conv -> conv -> add(., block input) or {conv, conv} -> add -> conv");
            const xl_layer &L2 = pl.layers[ids[1]], &L3 = pl.layers[ids[2]];
            if (L2.op != XL_CONV || L3.op != XL_ADD || L2.in[0] != t_mid) return fail(XL_E_GRAPH, at + "merge mode wiring");
            const int other = L3.in[0] == L2.out ? L3.in[1] : (L3.in[1] == L2.out ? L3.in[0] : -1);
            if (other < 0) return fail(XL_E_GRAPH, at + "the add does not read the second convolution");
            if (!only_consumers(t_mid, {ids[1]}) || !only_consumers(L2.out, {ids[2]}))
                return fail(XL_E_UNSUPPORTED, at + "an intermediate has a consumer outside the block");
            if (pl.storage[other].root != other) return fail(XL_E_UNSUPPORTED, at + "shortcut is a concat operand");
            // the block runs where its first layer stands: whatever it reads from outside must exist by then
            if (producer[other] >= ids[0])
                return fail(XL_E_UNSUPPORTED, at + "the shortcut is produced after the block's first layer; list its producer before the block");
            b.kind = KIND_FUSED2;
            b.n2 = 1;
            conv_spec(ids[1], b.c2[0]);
            b.relu_out = L3.relu;
            b.shortcut = true;
            sc_id = other;
            y_id = L3.out;
        } else {
            return fail(XL_E_UNSUPPORTED, at + "unknown fusion mode");
        }
        if (b.kind == KIND_FUSED2 || b.kind == KIND_DW || b.kind == KIND_FUSED2P) {
            for (int i = 0; i < b.n2; ++i)
                if (b.c2[i].cin != b.c1.cout) return fail(XL_E_SHAPE, at + "channel mismatch inside the block");
        }
        const xl_shape &ys = pl.shapes[y_id];
        b.Ho = ys.h;
        b.Wo = ys.w;
        if (b.gap) {
            // the kernel sees the convolution's own output extent; a pointwise one as a single row
            b.Ho = ms.h;
            b.Wo = ms.w;
            if (L1.k == 1 && L1.stride == 1 && L1.pad == 0) {
                b.W = b.W1 = b.Wo = xs.h * xs.w;
                b.H = b.H1 = b.Ho = 1;
            }
        }

        // algorithmic traffic (paper Table 2 counts stored elements the same way)
        xl_group_info &gi = gp.info;
        long long wbytes = 0;
        for (int li : ids) {
            long long by, stv;
            layer_traffic(li, by, stv);
            gi.bytes_unfused += by;
            gi.stores_unfused += stv;
            gi.flops += layer_flops(li);
            wbytes += weight_bytes(li);
        }
        gi.bytes_fused = tensor_bytes(t_in) + wbytes + tensor_bytes(y_id);
        if (sc_id >= 0 && sc_id != t_in) gi.bytes_fused += tensor_bytes(sc_id);
        gi.stores_fused = tensor_elems(y_id);
        b.alg_bytes = gi.bytes_fused;

        Step st;
        Choice ch;
        xl_status s = make_block_step(b, t_in, y_id, sc_id, 0, st, ch, at.substr(0, at.size() - 2));
        if (s != XL_OK) return s;
        fill_info(gi, b, ch);
        st.group = (int)pl.groups.size();
        st.first_layer = ids[0];
        st.nlayers = (int)ids.size();
        pl.fused_steps.push_back(st);
        return XL_OK;
    }

    xl_status build(const xl_group *groups, int ngroups)
    {
        xl_status s = validate();
        if (s != XL_OK) return s;
        s = resolve_storage();
        if (s != XL_OK) return s;
        const int nl = (int)pl.layers.size();

        // unfused path: one step per layer
        for (int li = 0; li < nl; ++li) {
            if (pl.layers[li].op == XL_CONCAT) continue;
            Step st;
            s = single_step(li, st, nullptr);
            if (s != XL_OK) return s;
            st.first_layer = li;
            st.nlayers = 1;
            for (Step &a : st.alts) a.first_layer = li;
            pl.unfused_steps.push_back(st);
        }

        // fused path: blocks in graph order, uncovered layers become singles
        std::vector<int> owner(nl, -1);
        for (int g = 0; g < ngroups; ++g) {
            if (groups[g].nlayers < 1 || !groups[g].layer_ids) return fail(XL_E_GRAPH, "empty fusion block");
            for (int i = 0; i < groups[g].nlayers; ++i) {
                const int li = groups[g].layer_ids[i];
                if (li < 0 || li >= nl) return fail(XL_E_GRAPH, "fusion block names a layer that does not exist");
                if (owner[li] >= 0) return fail(XL_E_GRAPH, "layer " + std::to_string(li) + " is in two fusion blocks");
                owner[li] = g;
            }
        }
        std::vector<bool> done(std::max(ngroups, 1), false);
        for (int li = 0; li < nl; ++li) {
            const int g = owner[li];
            if (g >= 0 && done[g]) continue;
            GroupPlan gp;
            memset(&gp.info, 0, sizeof gp.info);
            if (g < 0 || groups[g].mode == XL_SINGLE) {
                if (g >= 0 && groups[g].nlayers != 1) return fail(XL_E_UNSUPPORTED, "XL_SINGLE block with more than one layer");
                if (g >= 0) done[g] = true;
                gp.layers = {li};
                gp.info.mode = XL_SINGLE;
                gp.info.first_layer = li;
                gp.info.nlayers = 1;
                layer_traffic(li, gp.info.bytes_unfused, gp.info.stores_unfused);
                gp.info.bytes_fused = gp.info.bytes_unfused;
                gp.info.stores_fused = gp.info.stores_unfused;
                gp.info.flops = gp.info.flops_executed = layer_flops(li);
                gp.info.redundancy = 1.0;
                if (pl.layers[li].op != XL_CONCAT) {
                    Step st;
                    s = single_step(li, st, &gp.info);
                    if (s != XL_OK) return s;
                    st.group = (int)pl.groups.size();
                    st.first_layer = li;
                    st.nlayers = 1;
                    pl.fused_steps.push_back(st);
                }
            } else {
                done[g] = true;
                gp.layers.assign(groups[g].layer_ids, groups[g].layer_ids + groups[g].nlayers);
                if (gp.layers[0] != li) return fail(XL_E_GRAPH, "fusion block layers must be listed in graph order");
                gp.info.mode = groups[g].mode;
                gp.info.first_layer = li;
                gp.info.nlayers = groups[g].nlayers;
                s = fused_group(gp.layers, groups[g].mode, gp);
                if (s != XL_OK) return s;
            }
            pl.groups.push_back(gp);
        }

        // workspace: packed filters, then every tensor some layer both produces and consumes
        size_t off = 0;
        for (PackedFilter &p : pl.packed) {
            p.offset = off;
            off = align_up(off + p.bytes, 256);
            p.aff_offset = off;
            off = align_up(off + p.aff_bytes, 256);
        }
        for (size_t t = 0; t < pl.shapes.size(); ++t) {
            Storage &st = pl.storage[t];
            if (st.root != (int)t) continue;
            // a root is external when nothing produces it (graph input) or nothing consumes it (graph output)
            bool consumed = !consumers[t].empty();
            bool produced = producer[t] >= 0;
            st.external = !(consumed && produced);
            if (!st.external) {
                st.offset = off;
                off = align_up(off + (size_t)tensor_bytes((int)t), 256);
            }
        }
        for (size_t t = 0; t < pl.shapes.size(); ++t) {
            Storage &st = pl.storage[t];
            if (st.root != (int)t) {
                st.external = pl.storage[st.root].external;
                st.offset = pl.storage[st.root].offset;
            }
        }
        pl.workspace_bytes = std::max<size_t>(off, 256);
        return XL_OK;
    }
};

xl_status build_plan(xl_plan &pl, const xl_group *groups, int ngroups)
{
    Builder b(pl);
    const xl_status s = b.build(groups, ngroups);
    if (s != XL_OK) return s;
    pl.layerwise.assign(pl.groups.size(), 0);
    refresh_fused_path(pl);
    return XL_OK;
}

// The launches of the fused path: one step per block, except that a block switched to layer-by-layer
// execution contributes the unfused steps of its layers, in layer order.  (Everything such a block reads
// from outside is produced before its first layer -- fused_group checks that for the shortcut of a merge
// block -- so running its layers at the block's position keeps every dependency.)
void refresh_fused_path(xl_plan &pl)
{
    pl.fused_active.clear();
    for (Step &st : pl.fused_steps) {
        const bool split = st.nlayers > 1 && st.group >= 0 && st.group < (int)pl.layerwise.size() && pl.layerwise[st.group];
        if (!split) {
            pl.fused_active.push_back(&st);
            continue;
        }
        const std::vector<int> &ls = pl.groups[st.group].layers;
        for (Step &u : pl.unfused_steps)
            if (std::find(ls.begin(), ls.end(), u.first_layer) != ls.end()) pl.fused_active.push_back(&u);
    }
}

}  // namespace xl
