// Host-only part of libwpk: descriptor validation, the configuration (chromosome) encoding and
// its constraint check, the search-result cache and the genetic search engine.  No HIP calls.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <map>
#include <mutex>
#include <numeric>
#include <string>
#include <vector>

#include "wpk_internal.h"

namespace wpk {

const int32_t kBmVals[4] = {32, 64, 128, 256};
const int32_t kBnVals[3] = {32, 64, 128};
const int32_t kBkVals[3] = {8, 16, 32};
const int32_t kWmVals[3] = {1, 2, 4};
const int32_t kWnVals[3] = {1, 2, 4};
const int32_t kSplitVals[18] = {1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16, 20, 24};
const int32_t kRemapVals[2] = {0, 1};
const int32_t kPersistVals[5] = {0, 1, 2, 3, 4};
const int32_t kStageVals[3] = {1, 2, 3};
const int32_t kReduceVals[2] = {0, 1};
const int kGeneCounts[WPK_N_GENES] = {4, 3, 3, 3, 3, 18, 2, 5, 3, 2};

const int32_t *gene_values(int g)
{
    switch (g) {
    case 0: return kBmVals;
    case 1: return kBnVals;
    case 2: return kBkVals;
    case 3: return kWmVals;
    case 4: return kWnVals;
    case 5: return kSplitVals;
    case 6: return kRemapVals;
    case 7: return kPersistVals;
    case 8: return kStageVals;
    case 9: return kReduceVals;
    }
    return nullptr;
}

#define WPK_STR2(x) #x
#define WPK_STR(x) WPK_STR2(x)
#define WPK_VARIANT(PART, BM, BN, BK, WM, WN, PD)                                                  \
    {BM, BN, BK, WM, WN, PD,                                                                       \
     "wpk_igemm_" WPK_STR(BM) "x" WPK_STR(BN) "x" WPK_STR(BK) "_" WPK_STR(WM) "x" WPK_STR(WN) "_p" WPK_STR(PD)},
const Variant kVariants[] = {
#include WPK_VARIANTS_FILE
};
#undef WPK_VARIANT
const int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));

int find_variant(int bm, int bn, int bk, int wm, int wn, int stages)
{
    for (int i = 0; i < kNumVariants; ++i) {
        const Variant &v = kVariants[i];
        if (v.bm == bm && v.bn == bn && v.bk == bk && v.wm == wm && v.wn == wn && v.stages == stages)
            return i;
    }
    return -1;
}

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(int e) { g_last_hip_error = e; }

// Written once by the first call that looks at the device, read by every cache access.
static std::mutex g_device_name_mu;
static std::string g_device_name = "unknown";
void set_device_name(const std::string &name)
{
    std::lock_guard<std::mutex> g(g_device_name_mu);
    g_device_name = name;
}
std::string device_name()
{
    std::lock_guard<std::mutex> g(g_device_name_mu);
    return g_device_name;
}

// Output extent along one axis by the floor rule; <= 0 if the dilated window does not fit.
static int64_t out_extent(int64_t in, int64_t pad, int64_t dil, int64_t win, int64_t stride)
{
    int64_t span = in + 2 * pad - dil * (win - 1) - 1;
    return span < 0 ? 0 : span / stride + 1;
}

int make_problem(const wpk_conv_desc *d, Problem *out)
{
    if (!d || !out) return WPK_E_NULL_PTR;
    if (d->n <= 0 || d->c <= 0 || d->h <= 0 || d->w <= 0 || d->k <= 0 || d->r <= 0 || d->s <= 0 ||
        d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0 || d->dil_h <= 0 ||
        d->dil_w <= 0)
        return WPK_E_BAD_DESC;
    if (d->dtype != WPK_F32 || d->layout < 0 || d->layout > WPK_NHWC) return WPK_E_UNSUPPORTED;
    int64_t P = out_extent(d->h, d->pad_h, d->dil_h, d->r, d->stride_h);
    int64_t Q = out_extent(d->w, d->pad_w, d->dil_w, d->s, d->stride_w);
    if (P <= 0 || Q <= 0) return WPK_E_BAD_DESC;
    Problem pr;
    pr.d = *d;
    pr.P = (int32_t)P;
    pr.Q = (int32_t)Q;
    pr.M = (int64_t)d->n * P * Q;
    int64_t crs = (int64_t)d->c * d->r * d->s;
    pr.x_elems = (int64_t)d->n * d->c * d->h * d->w;
    pr.w_elems = (int64_t)d->k * crs;
    pr.y_elems = pr.M * d->k;
    const int64_t lim = (int64_t)1 << 40;  // beyond this even the direct kernel is not offered
    if (pr.x_elems > lim || pr.w_elems > lim || pr.y_elems > lim || crs > (1 << 30))
        return WPK_E_UNSUPPORTED;
    pr.CRS = (int32_t)crs;
    pr.CRSpad = (int32_t)((crs + kRedAlign - 1) / kRedAlign * kRedAlign);
    pr.Kpad = (d->k + kKoutAlign - 1) / kKoutAlign * kKoutAlign;
    pr.xl = (d->layout & 1) != 0;
    pr.xquad = pr.xl && d->c % kRedAlign == 0;
    pr.tapmajor = !pr.xl && d->c % kRedAlign == 0;
    pr.yl = (d->layout & 2) != 0;
    int64_t bias = ((int64_t)d->pad_h * d->w + d->pad_w) * 4 * (pr.xl ? d->c : 1);
    pr.tiled_ok = d->r <= kMaxFilterRows && d->s <= kMaxFilterCols &&
                  pr.x_elems * 4 + bias <= kMaxTiledBytes &&
                  pr.y_elems * 4 <= kMaxTiledBytes && (int64_t)pr.CRSpad * pr.Kpad * 4 <= kMaxTiledBytes;
    *out = pr;
    return WPK_OK;
}

std::string desc_key(const wpk_conv_desc *d)
{
    char buf[256];
    snprintf(buf, sizeof buf, "%d,%d,%d,%d,%d,%d,%d,%d,%d,%d,%d,%d,%d,%d,%d", d->n, d->c, d->h,
             d->w, d->k, d->r, d->s, d->stride_h, d->stride_w, d->pad_h, d->pad_w, d->dil_h,
             d->dil_w, d->dtype, d->layout);
    return buf;
}

static int value_index(int g, int32_t v)
{
    const int32_t *vals = gene_values(g);
    for (int i = 0; i < kGeneCounts[g]; ++i)
        if (vals[i] == v) return i;
    return -1;
}

static const int32_t *cfg_fields(const wpk_conv_config *c, int32_t f[WPK_N_GENES])
{
    f[0] = c->bm; f[1] = c->bn; f[2] = c->bk; f[3] = c->wm; f[4] = c->wn; f[5] = c->split_k;
    f[6] = c->xcd_remap;
    f[7] = c->persist;
    f[8] = c->stages;
    f[9] = c->reduce;
    return f;
}

// The constraint check of Step1 for the convolution kernel family.
bool legal_for(const Problem &pr, const wpk_conv_config &cfg)
{
    int32_t f[WPK_N_GENES];
    cfg_fields(&cfg, f);
    for (int g = 0; g < WPK_N_GENES; ++g)
        if (value_index(g, f[g]) < 0) return false;
    if (!pr.tiled_ok) return false;
    if (find_variant(cfg.bm, cfg.bn, cfg.bk, cfg.wm, cfg.wn, cfg.stages) < 0) return false;
    int threads = 64 * cfg.wm * cfg.wn;
    if (threads > 1024) return false;                                             // workgroup size
    if (cfg.bm == kWaveSplitBm) {
        // the wave-split members: tap-major reduction order only, one workgroup per tile and slice
        if (!(pr.tapmajor || pr.xquad) || cfg.persist != 0) return false;
        if ((cfg.wm * cfg.wn - 1) * cfg.bn * 32 * 4 > kMaxLdsBytes) return false;  // the other waves' partial tiles
    } else {
        if (2 * (cfg.bk + 4) * (cfg.bm + cfg.bn) * 4 > kMaxLdsBytes) return false;    // two LDS stages
        if (threads > cfg.bm && (cfg.bk * cfg.bm / threads) % 4 != 0) return false;   // whole k quads per thread
    }
    int32_t nsteps = (pr.CRS + cfg.bk - 1) / cfg.bk;
    if (cfg.split_k > nsteps) return false;
    // the persistent schedule balances the reduction itself: no fixed slices; and it always maps
    // tiles and runs XCD-contiguously (the same speed as launch order within noise, a half to a
    // fifth of the L2 fill traffic: 43 -> 17 MB, 103 -> 20 MB, 94 -> 34 MB on the 64-, 128- and
    // 256-channel layers of the batched 3x3 workload), so the gene has one legal value there
    if (cfg.persist > 0 && (cfg.split_k != 1 || cfg.xcd_remap != 1)) return false;
    // how partial tiles meet is a choice only where tiles can be shared
    if (cfg.reduce != 0 && cfg.split_k == 1 && cfg.persist == 0) return false;
    int64_t tiles = ((pr.M + cfg.bm - 1) / cfg.bm) * ((pr.d.k + cfg.bn - 1) / cfg.bn);
    if (tiles * cfg.split_k > 0x7fffffff) return false;
    // the persistent schedule counts reduction steps of up to 4*CUs tiles in 32 bits
    if (cfg.persist > 0 && (int64_t)nsteps * 4096 > 0x7fffffff) return false;
    return true;
}

// Workspace of the persistent schedule's fix-up: the tiles beyond the last whole round are shared;
// a tile of nsteps consecutive units cut into runs of at least q units meets at most
// ceil((nsteps-1)/q) + 1 runs (every run holds one unit when there are fewer units than runs).
std::atomic<int64_t> g_workspace_limit{kFixupMaxBytes};

FixupNeed fixup_need(const Problem &pr, const wpk_conv_config &cfg, int compute_units)
{
    FixupNeed n = {0, 0, 0, 0};
    if (cfg.reduce != 0) return n;  // atomics asked for
    if (compute_units <= 0) compute_units = 256;
    int64_t tiles = ((pr.M + cfg.bm - 1) / cfg.bm) * ((pr.d.k + cfg.bn - 1) / cfg.bn);
    int64_t nsteps = (pr.CRS + cfg.bk - 1) / cfg.bk;
    if (cfg.persist > 0) {
        // tiles of the last partial round, their steps dealt in runs of q or q+1 to at most G
        // workgroups: a tile's nsteps steps meet at most ceil((nsteps-1)/q)+1 runs, and never
        // more than nsteps
        int64_t G = (int64_t)cfg.persist * compute_units;
        int64_t shared = tiles - tiles / G * G;
        if (shared == 0 || nsteps <= 1) return n;
        int64_t q = shared * nsteps / streamk_groups(shared * nsteps, G, cfg.bk);
        n.shared_tiles = shared;
        n.maxc = q > 0 ? std::min<int64_t>(nsteps, (nsteps - 1 + q - 1) / q + 1) : nsteps;
    } else {
        // every tile is shared by its non-empty reduction slices
        int64_t per = (nsteps + cfg.split_k - 1) / cfg.split_k;
        int64_t slices = (nsteps + per - 1) / per;
        if (slices <= 1) return n;
        n.shared_tiles = tiles;
        n.maxc = slices;
    }
    // the counters sit in a region of fixed size at the front, so that buffers reused between
    // configurations never find slot data where counters are expected
    n.slots_offset = kFixupCounterBytes;
    n.bytes = n.slots_offset + n.shared_tiles * n.maxc * cfg.bm * cfg.bn * 4;
    if (n.shared_tiles * 4 > kFixupCounterBytes || n.bytes > g_workspace_limit.load(std::memory_order_relaxed))
        n = FixupNeed{0, 0, 0, 0};  // use atomics
    return n;
}

// Untuned default, distilled from exhaustive searches over the layer shapes of the workloads:
// 32x32 wave tiles in 64-pixel workgroup tiles with the largest K-step win or come within a few
// percent nearly everywhere, provided the launch has 3-4 workgroups per compute unit; where the
// tiles alone do not give that many, the reduction is split, and many small slices add up with
// atomics rather than through the workspace.  Falls back to a crude cost model over all
// variants if that choice is illegal for the shape.
static void model_config(const Problem &pr, int compute_units, wpk_conv_config *out);
bool wave_split_candidate(const Problem &pr, int64_t max_block_octets)
{
    if (!(pr.tapmajor || pr.xquad)) return false;
    const int64_t blocks = ((pr.M + 31) / 32) * ((pr.d.k + 31) / 32), octets = pr.CRS / 8;
    return blocks * octets <= max_block_octets;
}
static bool wave_split_default(const Problem &pr, int compute_units, wpk_conv_config *out)
{
    if (!wave_split_candidate(pr, 20000)) return false;
    const int64_t blocks = ((pr.M + 31) / 32) * ((pr.d.k + 31) / 32), octets = pr.CRS / 8;
    // as many waves per tile (four at most) as keep the launch within one wave per SIMD and every wave
    // at four octets or more
    int wk = 4;
    while (wk > 1 && (blocks * wk > 4 * (int64_t)compute_units || octets / wk < 4)) wk /= 2;
    int64_t want = std::max<int64_t>(1, 4 * (int64_t)compute_units / (blocks * wk));
    while (want > 1 && octets / (wk * want) < 8) --want;
    wpk_conv_config c = {kWaveSplitBm, 32, 8, wk, 1, 1, 1, 0, 1, 0};
    for (int i = 0; i < kGeneCounts[5]; ++i)
        if (kSplitVals[i] <= want) c.split_k = kSplitVals[i];
    c.reduce = c.split_k >= 4 ? 1 : 0;
    if (!legal_for(pr, c)) return false;
    *out = c;
    return true;
}
void default_config(const Problem &pr, int compute_units, wpk_conv_config *out)
{
    if (compute_units <= 0) compute_units = 256;
    // A launch with a few microseconds of arithmetic at most (single images, late layers): the
    // wave-split members, up to four waves per 32 x 32 tile, the reduction cut further between
    // workgroups until about one wave per SIMD is busy, but not into runs of fewer than eight octets;
    // four slices or more add up with atomics.  (Measured on the single-image ResNet-50 layers: 4.3-9.8 us where
    // the tiled members' best is 4.9-10.6.)
    if (wave_split_default(pr, compute_units, out)) return;
    wpk_conv_config c = {64, pr.d.k <= 32 ? 32 : 64, pr.CRS >= 64 ? 32 : pr.CRS >= 32 ? 16 : 8, 2,
                         pr.d.k <= 32 ? 1 : 2, 1, 1, 0, 2, 0};
    int64_t tiles = ((pr.M + c.bm - 1) / c.bm) * ((pr.d.k + c.bn - 1) / c.bn);
    int64_t nsteps = (pr.CRS + c.bk - 1) / c.bk;
    // slices of at least four steps, enough of them for 3.5 workgroups per compute unit
    int64_t want = std::min<int64_t>((7 * (int64_t)compute_units / 2 + tiles / 2) / tiles, nsteps / 4);
    for (int i = 0; i < kGeneCounts[5]; ++i)
        if (kSplitVals[i] <= want) c.split_k = kSplitVals[i];
    // Just over a whole number of rounds of three workgroups per compute unit: persistent
    // workgroups run the rounds as whole tiles and deal out only the few tiles left over,
    // instead of a last round that leaves most of the device idle.
    int64_t G = 3 * (int64_t)compute_units;
    if (tiles > G && tiles % G != 0 && (tiles % G) * 8 <= G) {
        wpk_conv_config h = c;
        h.bk = pr.CRS >= 32 ? 16 : 8;
        h.split_k = 1;
        h.xcd_remap = 1;
        h.persist = 3;
        h.reduce = 0;
        if (legal_for(pr, h)) {
            *out = h;
            return;
        }
    }
    // Between one and two tiles per compute unit: one persistent workgroup per compute unit takes a
    // whole tile, the steps of the other tiles are dealt out in runs that proceed beside them (a
    // split reduction would share every tile instead of the remainder only).
    if (tiles > compute_units && tiles < 2 * (int64_t)compute_units && nsteps >= 8) {
        wpk_conv_config h = c;
        h.split_k = 1;
        h.xcd_remap = 1;
        h.persist = 1;
        h.reduce = 0;
        if (legal_for(pr, h)) {
            *out = h;
            return;
        }
    }
    // atomics where many slices meet in a small output (zeroing it is cheap and the last
    // workgroup need not read every slot); the workspace otherwise
    int64_t per = (nsteps + c.split_k - 1) / c.split_k, slices = (nsteps + per - 1) / per;
    c.reduce = (slices >= 5 && pr.y_elems * 4 <= (1 << 20)) || slices > 12 ? 1 : 0;
    if (legal_for(pr, c)) {
        *out = c;
        return;
    }
    model_config(pr, compute_units, out);
}

// Smallest estimated time under a crude model -- workgroups are dealt to the compute units in
// rounds, a workgroup costs its multiply-accumulate count plus a fixed per-step and
// per-workgroup overhead, small wave tiles pay for their operand re-reads and a split reduction
// pays for its extra passes over y.
static void model_config(const Problem &pr, int compute_units, wpk_conv_config *out)
{
    double best = 1e300;
    wpk_conv_config bc = {128, 64, 16, 2, 2, 1, 1, 0, 2, 0};
    for (int i = 0; i < kNumVariants; ++i) {
        const Variant &v = kVariants[i];
        if (v.bm == kWaveSplitBm) continue;  // (the model prices LDS-staged tiles)
        for (int si = 0; si < kGeneCounts[5]; ++si) {
            wpk_conv_config c = {v.bm, v.bn, v.bk, v.wm, v.wn, kSplitVals[si], 1, 0, v.stages, 0};
            if (!legal_for(pr, c)) continue;
            double nsteps = ceil((double)pr.CRS / v.bk);
            double steps = ceil(nsteps / c.split_k);
            double tiles = ceil((double)pr.M / v.bm) * ceil((double)pr.d.k / v.bn);
            double blocks = tiles * c.split_k;
            double waves = v.wm * v.wn;
            double tm = v.bm / v.wm, tn = v.bn / v.wn;
            // MFMA cycles per step per SIMD (waves share the 4 SIMDs of a compute unit)
            double mfma = (double)v.bm * v.bn * v.bk / 2048.0 * 64.0 / std::min(4.0, waves);
            double operand = 1.0 + 16.0 * (1.0 / tm + 1.0 / tn);  // LDS operand traffic per MFMA
            double step_cost = mfma * operand + 220.0;
            double block_cost = steps * step_cost + 2500.0;
            double rounds = ceil(blocks / compute_units);
            double cost = rounds * block_cost;
            if (c.split_k > 1) cost += (double)pr.y_elems * c.split_k / compute_units * 0.5;
            if (cost < best) { best = cost; bc = c; }
        }
    }
    int64_t nsteps = (pr.CRS + bc.bk - 1) / bc.bk, per = (nsteps + bc.split_k - 1) / bc.split_k;
    bc.reduce = (nsteps + per - 1) / per > 8 ? 1 : 0;
    *out = bc;
}

// ---- search-result cache ----------------------------------------------------------------------
struct CacheEntry {
    wpk_conv_config cfg;
    double us;
};
static std::mutex g_cache_mu;
static std::map<std::string, CacheEntry> g_cache;
static std::string cache_key(const wpk_conv_desc *d) { return desc_key(d) + "|" + device_name(); }

// ---- splitmix64 (Steele, Lea, Flood 2014): state += gamma; output = mix(state) -------------------
struct SplitMix64 {
    uint64_t s;
    explicit SplitMix64(uint64_t seed) : s(seed) {}
    uint64_t next()
    {
        s += 0x9E3779B97F4A7C15ull;
        uint64_t z = s;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    double uniform() { return (double)(next() >> 11) * (1.0 / 9007199254740992.0); }
    int32_t randint(int32_t lo, int32_t hi)
    {
        return lo + (int32_t)(next() % (uint64_t)((int64_t)hi - lo + 1));
    }
};

// ---- genetic search engine (Section 2.3 "Genetic search") -----------------------------------------
typedef std::vector<int32_t> Chrom;

struct Ga {
    int32_t n;
    const int32_t *lo, *hi;
    wpk_ga_constraint_fn constraint;
    wpk_ga_fitness_fn fitness;
    void *user;
    SplitMix64 rng;
    std::map<Chrom, double> memo;

    bool ok(const Chrom &c) { return !constraint || constraint(c.data(), n, user) != 0; }

    double eval(const Chrom &c)
    {
        auto it = memo.find(c);
        if (it != memo.end()) return it->second;
        double f = fitness(c.data(), n, user);
        if (!(f > 0.0)) f = 0.0;
        memo[c] = f;
        return f;
    }

    // Step1: uniform draws per gene, re-drawn until the constraint check passes.
    bool random_legal(Chrom &c)
    {
        c.resize(n);
        for (int t = 0; t < 100000; ++t) {
            for (int g = 0; g < n; ++g) c[g] = rng.randint(lo[g], hi[g]);
            if (ok(c)) return true;
        }
        return false;
    }
};

// Indices by decreasing fitness; equal fitness keeps population order.
static std::vector<int> sort_by_fitness(const std::vector<double> &fit)
{
    std::vector<int> idx(fit.size());
    std::iota(idx.begin(), idx.end(), 0);
    std::stable_sort(idx.begin(), idx.end(), [&](int a, int b) { return fit[a] > fit[b]; });
    return idx;
}

// Roulette wheel by inverse sampling: first i with v <= P(a_i); P(a_0) = 0, so v = 0 picks i = 1.
static int roulette_pick(const std::vector<double> &P, double v)
{
    for (size_t i = 0; i < P.size(); ++i)
        if (v <= P[i]) return (int)i;
    return (int)P.size() - 1;
}

static bool runtimes_close(const std::vector<double> &fit, double eps)
{
    double tmin = 1e300, tmax = 0;
    for (double f : fit) {
        if (f <= 0.0) return false;
        double t = 1.0 / f;
        tmin = std::min(tmin, t);
        tmax = std::max(tmax, t);
    }
    return (tmax - tmin) / tmin < eps;
}

}  // namespace wpk

using namespace wpk;

extern "C" {

int wpk_conv_out_shape(const wpk_conv_desc *d, int32_t *p, int32_t *q)
{
    Problem pr;
    int rc = make_problem(d, &pr);
    if (rc != WPK_OK) return rc;
    if (p) *p = pr.P;
    if (q) *q = pr.Q;
    return WPK_OK;
}

double wpk_conv_flops(const wpk_conv_desc *d)
{
    Problem pr;
    if (make_problem(d, &pr) != WPK_OK) return 0.0;
    return 2.0 * (double)pr.M * d->k * pr.CRS;
}

const char *wpk_status_string(int status)
{
    switch (status) {
    case WPK_OK: return "ok";
    case WPK_E_BAD_DESC: return "bad convolution descriptor";
    case WPK_E_NULL_PTR: return "null pointer argument";
    case WPK_E_UNSUPPORTED: return "unsupported dtype, layout or size";
    case WPK_E_HIP: return "HIP runtime error";
    case WPK_E_NO_CONFIG: return "configuration not legal for this descriptor";
    case WPK_E_BAD_ARG: return "bad argument";
    case WPK_E_IO: return "cache file i/o error";
    case WPK_E_VERIFY: return "no candidate passed verification";
    case WPK_E_TOO_LARGE: return "packed weights exceed the static scratch of the entry point that does not allocate";
    }
    return status > 0 ? "ok (id)" : "unknown status";
}

int wpk_last_hip_error(void) { return g_last_hip_error; }

int wpk_config_gene_ranges(int32_t lo[WPK_N_GENES], int32_t hi[WPK_N_GENES])
{
    if (!lo || !hi) return WPK_E_NULL_PTR;
    for (int g = 0; g < WPK_N_GENES; ++g) {
        lo[g] = 0;
        hi[g] = kGeneCounts[g] - 1;
    }
    return WPK_OK;
}

int wpk_config_from_genes(const int32_t genes[WPK_N_GENES], wpk_conv_config *out)
{
    if (!genes || !out) return WPK_E_NULL_PTR;
    for (int g = 0; g < WPK_N_GENES; ++g)
        if (genes[g] < 0 || genes[g] >= kGeneCounts[g]) return WPK_E_BAD_ARG;
    out->bm = kBmVals[genes[0]];
    out->bn = kBnVals[genes[1]];
    out->bk = kBkVals[genes[2]];
    out->wm = kWmVals[genes[3]];
    out->wn = kWnVals[genes[4]];
    out->split_k = kSplitVals[genes[5]];
    out->xcd_remap = kRemapVals[genes[6]];
    out->persist = kPersistVals[genes[7]];
    out->stages = kStageVals[genes[8]];
    out->reduce = kReduceVals[genes[9]];
    return WPK_OK;
}

int wpk_config_to_genes(const wpk_conv_config *cfg, int32_t genes[WPK_N_GENES])
{
    if (!cfg || !genes) return WPK_E_NULL_PTR;
    int32_t f[WPK_N_GENES];
    cfg_fields(cfg, f);
    for (int g = 0; g < WPK_N_GENES; ++g) {
        int i = value_index(g, f[g]);
        if (i < 0) return WPK_E_BAD_ARG;
        genes[g] = i;
    }
    return WPK_OK;
}

int wpk_config_legal(const wpk_conv_desc *d, const wpk_conv_config *cfg)
{
    if (!cfg) return WPK_E_NULL_PTR;
    Problem pr;
    int rc = make_problem(d, &pr);
    if (rc != WPK_OK) return rc;
    return legal_for(pr, *cfg) ? 1 : 0;
}

int wpk_config_id(const wpk_conv_config *cfg)
{
    int32_t genes[WPK_N_GENES];
    int rc = wpk_config_to_genes(cfg, genes);
    if (rc != WPK_OK) return rc;
    int id = 0;
    for (int g = WPK_N_GENES - 1; g >= 0; --g) id = id * kGeneCounts[g] + genes[g];
    return id;
}

int wpk_config_from_id(int id, wpk_conv_config *out)
{
    if (!out) return WPK_E_NULL_PTR;
    if (id < 0) return WPK_E_NO_CONFIG;
    int32_t genes[WPK_N_GENES];
    for (int g = 0; g < WPK_N_GENES; ++g) {
        genes[g] = id % kGeneCounts[g];
        id /= kGeneCounts[g];
    }
    if (id != 0) return WPK_E_NO_CONFIG;
    return wpk_config_from_genes(genes, out);
}

const char *wpk_config_kernel_name(const wpk_conv_config *cfg)
{
    if (!cfg) return "";
    int i = find_variant(cfg->bm, cfg->bn, cfg->bk, cfg->wm, cfg->wn, cfg->stages);
    return i < 0 ? "" : kVariants[i].name;
}

const char *wpk_version(void) { return "wpk-conv 0.1 (gfx950)"; }

// ---- cache -----------------------------------------------------------------------------------
int wpk_cache_lookup(const wpk_conv_desc *d, wpk_conv_config *out)
{
    Problem pr;
    int rc = make_problem(d, &pr);
    if (rc != WPK_OK) return rc;
    std::lock_guard<std::mutex> g(g_cache_mu);
    auto it = g_cache.find(cache_key(d));
    if (it == g_cache.end()) return 0;
    if (out) *out = it->second.cfg;
    return 1;
}

int wpk_cache_lookup_time(const wpk_conv_desc *d, wpk_conv_config *out, double *us)
{
    Problem pr;
    int rc = make_problem(d, &pr);
    if (rc != WPK_OK) return rc;
    std::lock_guard<std::mutex> g(g_cache_mu);
    auto it = g_cache.find(cache_key(d));
    if (it == g_cache.end()) return 0;
    if (out) *out = it->second.cfg;
    if (us) *us = it->second.us;
    return 1;
}

int wpk_cache_store(const wpk_conv_desc *d, const wpk_conv_config *cfg, double us)
{
    if (!cfg) return WPK_E_NULL_PTR;
    Problem pr;
    int rc = make_problem(d, &pr);
    if (rc != WPK_OK) return rc;
    if (!legal_for(pr, *cfg)) return WPK_E_NO_CONFIG;
    std::lock_guard<std::mutex> g(g_cache_mu);
    g_cache[cache_key(d)] = CacheEntry{*cfg, us};
    return WPK_OK;
}

int wpk_cache_clear(void)
{
    std::lock_guard<std::mutex> g(g_cache_mu);
    g_cache.clear();
    return WPK_OK;
}

int wpk_cache_size(void)
{
    std::lock_guard<std::mutex> g(g_cache_mu);
    return (int)g_cache.size();
}

int wpk_cache_save(const char *path)
{
    if (!path) return WPK_E_NULL_PTR;
    FILE *f = fopen(path, "w");
    if (!f) return WPK_E_IO;
    std::lock_guard<std::mutex> g(g_cache_mu);
    fprintf(f, "# wpk search-result cache v3: key bm bn bk wm wn split_k xcd_remap persist stages reduce microseconds\n");
    for (auto &kv : g_cache) {
        std::string key = kv.first;
        std::replace(key.begin(), key.end(), ' ', '_');
        const wpk_conv_config &c = kv.second.cfg;
        fprintf(f, "%s %d %d %d %d %d %d %d %d %d %d %.6f\n", key.c_str(), c.bm, c.bn, c.bk, c.wm, c.wn,
                c.split_k, c.xcd_remap, c.persist, c.stages, c.reduce, kv.second.us);
    }
    return fclose(f) == 0 ? WPK_OK : WPK_E_IO;
}

int wpk_cache_load(const char *path)
{
    if (!path) return WPK_E_NULL_PTR;
    FILE *f = fopen(path, "r");
    if (!f) return WPK_E_IO;
    char line[1024];
    int count = 0;
    std::lock_guard<std::mutex> g(g_cache_mu);
    while (fgets(line, sizeof line, f)) {
        if (line[0] == '#' || line[0] == '\n') continue;
        char key[512];
        wpk_conv_config c;
        double us;
        if (sscanf(line, "%511s %d %d %d %d %d %d %d %d %d %d %lf", key, &c.bm, &c.bn, &c.bk, &c.wm,
                   &c.wn, &c.split_k, &c.xcd_remap, &c.persist, &c.stages, &c.reduce, &us) != 12)
            continue;  // also skips lines of older formats: those layers are searched again
        int32_t genes[WPK_N_GENES];
        if (wpk_config_to_genes(&c, genes) != WPK_OK) continue;
        g_cache[key] = CacheEntry{c, us};
        ++count;
    }
    fclose(f);
    return count;
}

// ---- layouts of the tensors between layers (Section 2.1, data layout transformation) ----------------
// Every tensor is stored [N][C][H][W] (0) or channels-last (1); a layer's cost depends on the layouts
// of the tensor it reads and of the tensor it writes; a residual is read in the layout its layer
// writes, so the two tensors are tied into one group.  Minimise the sum of the layers' costs over
// the free groups.  Exact, by elimination along the layer order: a table over the assignments of
// the groups that layers already seen AND layers still to come refer to (a network's frontier: two
// to four groups for chains with shortcut branches); a group is minimised out after its last layer,
// with the minimising value kept per remaining assignment for the way back.
int wpk_choose_layouts(int32_t n_layers, const int32_t *x_tensor, const int32_t *y_tensor,
                       const int32_t *residual_tensor, const int32_t *tensor_layout, int32_t n_tensors,
                       const double *cost, int32_t *chosen, double *total)
{
    if (!x_tensor || !y_tensor || !tensor_layout || !cost || !chosen) return WPK_E_NULL_PTR;
    if (n_layers <= 0 || n_tensors <= 0) return WPK_E_BAD_ARG;
    for (int i = 0; i < n_layers; ++i)
        if (x_tensor[i] < 0 || x_tensor[i] >= n_tensors || y_tensor[i] < 0 || y_tensor[i] >= n_tensors ||
            (residual_tensor && residual_tensor[i] >= n_tensors))
            return WPK_E_BAD_ARG;
    for (int t = 0; t < n_tensors; ++t)
        if (tensor_layout[t] < -1 || tensor_layout[t] > 1) return WPK_E_BAD_ARG;
    // groups of tied tensors (union-find); a group is fixed if any member is
    std::vector<int> parent(n_tensors);
    std::iota(parent.begin(), parent.end(), 0);
    auto find = [&](int t) { while (parent[t] != t) t = parent[t] = parent[parent[t]]; return t; };
    if (residual_tensor)
        for (int i = 0; i < n_layers; ++i)
            if (residual_tensor[i] >= 0) parent[find(residual_tensor[i])] = find(y_tensor[i]);
    std::vector<int> fixed(n_tensors, -1), last_use(n_tensors, -1), value(n_tensors, 0);
    for (int t = 0; t < n_tensors; ++t)
        if (tensor_layout[t] >= 0) {
            int r = find(t);
            if (fixed[r] >= 0 && fixed[r] != tensor_layout[t]) return WPK_E_BAD_ARG;  // tied tensors fixed differently
            fixed[r] = tensor_layout[t];
        }
    for (int i = 0; i < n_layers; ++i) last_use[find(x_tensor[i])] = last_use[find(y_tensor[i])] = i;
    for (int t = 0; t < n_tensors; ++t)
        if (find(t) == t && fixed[t] >= 0) value[t] = fixed[t];  // also for groups no layer refers to

    const double kNever = 1e300;
    const size_t kMaxOpen = 20;
    struct Closed {
        int group;
        std::vector<int> open_after;   // the groups still open once this one is gone, in table order
        int pos;                       // where it sat among the open groups
        std::vector<char> best;        // per assignment of open_after: the value that minimised
    };
    std::vector<Closed> history;
    std::vector<int> open;
    std::vector<double> tab(1, 0.0);
    auto pos_of = [&](int g) { return (int)(std::find(open.begin(), open.end(), g) - open.begin()); };
    for (int i = 0; i < n_layers; ++i) {
        const int gs[2] = {find(x_tensor[i]), find(y_tensor[i])};
        for (int k = 0; k < 2; ++k) {
            if (pos_of(gs[k]) < (int)open.size()) continue;
            if (open.size() >= kMaxOpen) return WPK_E_UNSUPPORTED;  // a frontier no network here comes near
            const size_t n = tab.size();
            tab.resize(2 * n);
            for (size_t st = 0; st < n; ++st) {
                const double base = tab[st];
                tab[st] = fixed[gs[k]] == 1 ? kNever : base;
                tab[st + n] = fixed[gs[k]] == 0 ? kNever : base;
            }
            open.push_back(gs[k]);
        }
        const int px = pos_of(gs[0]), py = pos_of(gs[1]);
        for (size_t st = 0; st < tab.size(); ++st)
            if (tab[st] < kNever) tab[st] += cost[(size_t)i * 4 + ((st >> px) & 1) * 2 + ((st >> py) & 1)];
        for (int k = 0; k < 2; ++k) {
            const int g = gs[k];
            const int p = pos_of(g);
            if (p == (int)open.size() || last_use[g] != i) continue;  // closed already (x == y group), or used later
            Closed c;
            c.group = g;
            c.pos = p;
            const size_t n = tab.size() / 2;
            std::vector<double> next(n);
            c.best.resize(n);
            const size_t low = ((size_t)1 << p) - 1;
            for (size_t r = 0; r < n; ++r) {
                const size_t s0 = (r & low) | ((r & ~low) << 1), s1 = s0 | ((size_t)1 << p);
                c.best[r] = tab[s1] < tab[s0] ? 1 : 0;
                next[r] = std::min(tab[s0], tab[s1]);
            }
            open.erase(open.begin() + p);
            c.open_after = open;
            tab.swap(next);
            history.push_back(std::move(c));
        }
    }
    if (tab.size() != 1 || !(tab[0] < kNever)) return WPK_E_BAD_ARG;
    for (size_t h = history.size(); h-- > 0;) {
        const Closed &c = history[h];
        size_t r = 0;
        for (size_t k = 0; k < c.open_after.size(); ++k) r |= (size_t)value[c.open_after[k]] << k;
        value[c.group] = c.best[r];
    }
    for (int t = 0; t < n_tensors; ++t) chosen[t] = value[find(t)];
    if (total) *total = tab[0];
    return WPK_OK;
}

// ---- tuning options and the engine ---------------------------------------------------------------
int64_t wpk_config_workspace_bytes(const wpk_conv_desc *d, const wpk_conv_config *cfg,
                                   int32_t compute_units, int64_t *shared_tiles, int64_t *slots)
{
    if (!cfg) return WPK_E_NULL_PTR;
    Problem pr;
    int rc = make_problem(d, &pr);
    if (rc != WPK_OK) return rc;
    if (!legal_for(pr, *cfg)) return WPK_E_NO_CONFIG;
    FixupNeed n = fixup_need(pr, *cfg, compute_units);
    if (shared_tiles) *shared_tiles = n.shared_tiles;
    if (slots) *slots = n.maxc;
    return n.bytes;
}

int wpk_set_workspace_limit(int64_t bytes)
{
    if (bytes < 0) return WPK_E_BAD_ARG;
    g_workspace_limit.store(bytes, std::memory_order_relaxed);
    return WPK_OK;
}

void wpk_tune_default_options(wpk_tune_options *o)
{
    if (!o) return;
    memset(o, 0, sizeof *o);
    o->population = 64;
    o->elites = 8;
    o->next_population = 64;
    o->participants = 64;
    o->max_generations = 16;
    o->patience = 5;
    o->mutation = 0.15;
    o->eps = 0.03;
    o->seed = 2008;
    o->reps = 5;
    o->min_group_us = 200.0;
    o->mode = 0;
    o->verbose = 0;
    o->refine = 2;
    o->zero_ahead = 0;
    o->epilogue = 0;
}

int wpk_ga_search(int32_t n_genes, const int32_t *lo, const int32_t *hi,
                  wpk_ga_constraint_fn constraint, wpk_ga_fitness_fn fitness, void *user,
                  const wpk_tune_options *opt_in, int32_t *best_genes, double *best_fitness,
                  int32_t *evaluations, int32_t *history_pop, double *history_fit,
                  int32_t *history_sizes, int32_t history_capacity)
{
    if (!lo || !hi || !fitness) return WPK_E_NULL_PTR;
    wpk_tune_options opt;
    if (opt_in) opt = *opt_in; else wpk_tune_default_options(&opt);
    if (n_genes <= 0 || opt.population <= 0 || opt.max_generations <= 0) return WPK_E_BAD_ARG;
    for (int g = 0; g < n_genes; ++g)
        if (hi[g] < lo[g]) return WPK_E_BAD_ARG;
    int32_t next_pop = opt.next_population > 0 ? opt.next_population : opt.population;
    int32_t width = std::max(opt.population, next_pop);
    const int retries = 8;

    Ga ga{n_genes, lo, hi, constraint, fitness, user, SplitMix64(opt.seed), {}};
    std::vector<Chrom> pop(opt.population);
    for (auto &c : pop)                                                        // Step1
        if (!ga.random_legal(c)) return WPK_E_NO_CONFIG;

    Chrom best;
    double best_f = -1.0;
    int stall = 0, gen = 0;
    for (;; ++gen) {
        std::vector<double> fit(pop.size());
        for (size_t i = 0; i < pop.size(); ++i) fit[i] = ga.eval(pop[i]);      // Step2
        if (gen < history_capacity) {
            if (history_sizes) history_sizes[gen] = (int32_t)pop.size();
            for (int i = 0; i < width; ++i) {
                if (history_fit) history_fit[(size_t)gen * width + i] = i < (int)pop.size() ? fit[i] : -1.0;
                if (history_pop)
                    for (int g = 0; g < n_genes; ++g)
                        history_pop[((size_t)gen * width + i) * n_genes + g] =
                            i < (int)pop.size() ? pop[i][g] : -1;
            }
        }
        std::vector<int> order = sort_by_fitness(fit);
        if (fit[order[0]] > best_f) {
            best = pop[order[0]];
            best_f = fit[order[0]];
            stall = 0;
        } else {
            ++stall;
        }
        if (opt.verbose)
            fprintf(stderr, "[wpk search] generation %d: size %zu, best fitness %.6g, evaluated %zu\n",
                    gen, pop.size(), best_f, ga.memo.size());
        if (runtimes_close(fit, opt.eps) || (opt.patience > 0 && stall >= opt.patience) ||
            gen == opt.max_generations - 1)                                    // Step4
            break;

        std::vector<Chrom> nxt;
        if (opt.mode == 1) {  // random search: a fresh random generation, nothing inherited
            nxt.resize(next_pop);
            for (auto &c : nxt)
                if (!ga.random_legal(c)) return WPK_E_NO_CONFIG;
        } else {              // Step3
            int k = std::min<int>(std::max(opt.elites, 0), (int)pop.size());
            k = std::min(k, (int)next_pop);
            int m = opt.participants > 0 ? std::min<int>(opt.participants, (int)pop.size())
                                         : (int)pop.size();
            for (int i = 0; i < k; ++i) nxt.push_back(pop[order[i]]);
            // eq. (1) over the m participants, then eq. (2)
            double total = 0.0;
            for (int i = 0; i < m; ++i) total += fit[order[i]];
            std::vector<double> P(m);
            double run = 0.0;
            for (int i = 0; i < m; ++i) {
                double p = total > 0.0 ? fit[order[i]] / total : 1.0 / m;
                run += p;
                P[i] = run;
            }
            P[m - 1] = 1.0;
            while ((int)nxt.size() < next_pop) {
                Chrom child(n_genes);
                bool done = false;
                for (int t = 0; t < retries && !done; ++t) {
                    const Chrom &a = pop[order[roulette_pick(P, ga.rng.uniform())]];
                    const Chrom &b = pop[order[roulette_pick(P, ga.rng.uniform())]];
                    for (int g = 0; g < n_genes; ++g) child[g] = ga.rng.uniform() < 0.5 ? a[g] : b[g];
                    for (int g = 0; g < n_genes; ++g)
                        if (ga.rng.uniform() < opt.mutation) child[g] = ga.rng.randint(lo[g], hi[g]);
                    done = ga.ok(child);
                }
                if (!done && !ga.random_legal(child)) return WPK_E_NO_CONFIG;
                nxt.push_back(child);
            }
        }
        pop.swap(nxt);
    }
    if (best_genes)
        for (int g = 0; g < n_genes; ++g) best_genes[g] = best[g];
    if (best_fitness) *best_fitness = best_f;
    if (evaluations) *evaluations = (int32_t)ga.memo.size();
    return gen + 1;
}

}  // extern "C"
