// Internal declarations shared by the translation units of libwpk.  Not part of the ABI.
#ifndef WPK_INTERNAL_H
#define WPK_INTERNAL_H

#include <stdint.h>

#include <atomic>
#include <string>
#include <vector>

#include "wpk.h"

// The list of compiled tile combinations; a build may name a shorter list of its own (the gene
// space shrinks with it: the constraint check only admits combinations on the list).
#ifndef WPK_VARIANTS_FILE
#define WPK_VARIANTS_FILE "wpk_variants.def"
#endif

namespace wpk {

// ---- gene value lists (the search sees index ranges into them) -------------------------------
extern const int32_t kBmVals[4];     // 32 (the wave-split members), 64, 128, 256
extern const int32_t kBnVals[3];     // 32, 64, 128
extern const int32_t kBkVals[3];     // 8, 16, 32
extern const int32_t kWmVals[3];     // 1, 2, 4
extern const int32_t kWnVals[3];     // 1, 2, 4
extern const int32_t kSplitVals[18]; // 1 .. 16, 20, 24
extern const int32_t kRemapVals[2];  // 0, 1
extern const int32_t kStageVals[3];   // 1, 2, 3 tiles in flight in registers
extern const int32_t kReduceVals[2];  // 0 workspace, 1 atomics
extern const int32_t kPersistVals[5]; // 0 (off), 1, 2, 3, 4 workgroups per compute unit
extern const int kGeneCounts[WPK_N_GENES];
const int32_t *gene_values(int g);

// Reduction entries are padded up to a multiple of kRedAlign rows (the largest K-step) and
// packed output channels to a multiple of kKoutAlign (the largest channel tile), so tile loads
// of packed weights and of the tap table never need a bounds check.
static const int kRedAlign = 32;
static const int kKoutAlign = 128;
// Per pixel, filter rows and columns outside the image are tracked in one 32-bit mask: bits
// 0..15 for rows, bits 16..30 for columns, bit 31 reserved as "always outside" for the padded
// reduction rows.  So the tiled family takes filters up to 16 rows by 15 columns.
static const int kMaxFilterRows = 16;
static const int kMaxFilterCols = 15;
static const int kPadTapBit = 31;
static const int kNumXcd = 8;
// Members with this pixel tile are the wave-split form (wpk_wsplit.h): their wm x wn waves cut the
// reduction between them, bk is the octet they work in, and `stages` counts four octets in flight each.
static const int kWaveSplitBm = 32;
// LDS per workgroup: two stages of (BM + BN) columns of BK + 4 floats; two workgroups of the
// largest tile still fit the 160 KB of a compute unit.
static const int kMaxLdsBytes = 80 * 1024;
// Tensors are addressed with 32-bit byte offsets through buffer descriptors.
static const int64_t kMaxTiledBytes = 0x7fffffff;

// ---- one compiled tile combination -------------------------------------------------------------
struct Variant {
    int32_t bm, bn, bk, wm, wn, stages;
    const char *name;
};
extern const Variant kVariants[];
extern const int kNumVariants;
int find_variant(int bm, int bn, int bk, int wm, int wn, int stages);  // index or -1

// ---- everything derived from one descriptor ------------------------------------------------------
struct Problem {
    wpk_conv_desc d;
    int32_t P, Q;
    int64_t M;       // N*P*Q output pixels (GEMM columns)
    int32_t CRS;     // reduction length
    int32_t CRSpad;  // rounded up to kRedAlign
    int32_t Kpad;    // K rounded up to kKoutAlign
    int64_t x_elems, w_elems, y_elems;
    bool tiled_ok;   // the tiled family can run it (else only the direct kernel)
    bool xl, yl;     // x / y channels-last (bits 0 and 1 of the descriptor's layout)
    bool xquad;      // channels-last x gathered as 16-byte channel quads (C a multiple of every K-step)
    bool tapmajor;   // x [N][C][H][W] with C a multiple of every K-step: reduction ordered (r, s, c) as well
};
int make_problem(const wpk_conv_desc *d, Problem *out);  // WPK_OK or a WPK_E_* code
std::string desc_key(const wpk_conv_desc *d);

// Division of a 31-bit number by a launch constant as a multiply, an add and a shift (the
// divisor's multiplier is computed on the host): with L = ceil(log2 d) and
// mul = floor(2^32 * (2^L - d) / d) + 1, q = (mulhi(n, mul) + n) >> L is exact for every
// n < 2^31 and every d >= 1 (d = 1 and powers of two give mul = 1, which adds nothing), and the
// sum cannot overflow 32 bits because mulhi(n, mul) <= n.
struct FastDiv {
    uint32_t mul, sh;
};
inline FastDiv make_fastdiv(uint32_t d)
{
    uint32_t L = 0;
    while ((1ull << L) < d) ++L;
    FastDiv f = {(uint32_t)((((uint64_t)1 << 32) * ((1ull << L) - d)) / d + 1), L};
    return f;
}

// Persistent launches: the reduction steps of the tiles beyond the last whole round (`units` of
// them) are dealt to the first `streamk_groups` of the G workgroups in runs of equal length (+-1).
// A run over fewer than kMinRunRows reduction rows does not repay its prologue and its part in
// the fix-up (measured on the 56x56 layer of 64 channels: 45 us per launch with runs of 64-96
// rows against 49-59 us with runs of one or two K-steps of 16), so fewer workgroups take part
// when there is little to deal out.
static const int kMinRunRows = 64;
inline int64_t streamk_groups(int64_t units, int64_t G, int bk)
{
    if (units <= 0) return 0;
    int64_t min_steps = kMinRunRows / bk > 1 ? kMinRunRows / bk : 1;
    int64_t want = units / min_steps;
    return want < 1 ? 1 : want < G ? want : G;
}

// Kernel argument block of the tiled implicit-GEMM family (passed by value).
struct IgemmArgs {
    const float *x;
    const float *wp;      // packed weights [CRSpad/4][Kpad][4]
    float *y;
    const int32_t *ktab;  // periodic tap table [R*S phases][32 rows][2]: byte offset relative to the
                          // step's channel base (biased); mask bit of r | mask bit of s << 8
    const int32_t *ttab;  // the same for the 32 rows from the start of the last reduction step, exact
    int32_t N, C, H, W, K, P, Q, R, S;
    int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
    int32_t M, PQ, HW, CRS, Kpad;
    int32_t RS, HW4;               // R*S, H*W*4
    int32_t bk_div_rs, bk_mod_rs;  // BK / RS, BK % RS
    int32_t nsteps, steps_per_split, split_k;
    int32_t tiles_m, tiles_n, remap;
    int32_t persist;       // 0, or persistent workgroups per compute unit
    int32_t grid_persist;  // persist * compute units
    int32_t runners;       // persistent: workgroups appended to the grid that do a dealt-out run and nothing else
                           // (set by the launcher: sk_groups, or 0 when the first sk_groups workgroups do their run
                           // themselves)
    uint32_t x_bytes;   // size of x
    uint32_t x_bias;    // (pad_h*W + pad_w)*4: added to every tap offset, subtracted from the base
    uint32_t w_bytes;   // size of the packed weights
    uint32_t y_bytes;   // size of y (and of a residual)
    // fix-up workspace of shared tiles (NULL = accumulate with atomics into zeroed y instead)
    float *ws;          // [shared tiles][ws_maxc slots][BM*BN] partial tiles
    int32_t *ws_cnt;    // [shared tiles] arrival counters, zero between launches
    int32_t ws_maxc;    // slots per shared tile
    // fused epilogue, applied where y is stored plainly: y = act(acc + bias[k] + res[n][k][p][q])
    const float *bias;  // [K] or NULL
    const float *res;   // laid out like y, or NULL
    int32_t relu;       // act = max(., 0) when nonzero
    // launch constants of the work iterator and their fast divisors
    int32_t tiles;      // tiles_m * tiles_n
    int32_t tiles_dp;   // persistent: tiles done whole, floor(tiles / G) * G
    int32_t sk_groups;     // persistent: how many workgroups (the first ones) share out the other tiles' steps,
    int32_t sk_q, sk_rem;  // in runs of sk_q steps (+1 for the first sk_rem)
    FastDiv div_pq, div_q, div_tiles_n, div_tiles, div_nsteps, div_q1, div_q0;  // by PQ, Q, tiles_n,
                        // tiles, nsteps, sk_q + 1, max(sk_q, 1)
    FastDiv div_tap;    // by what a reduction row index is divided to find its first table entry: C where a
                        // K-step lies inside one filter tap, else R*S
    int32_t mfast;      // order of the tiles: 0: tile = tile_m * tiles_n + tile_n (neighbours in the order share rows
                        // of x); 1: tile = tile_n * tiles_m + tile_m (neighbours share weights) -- whichever operand is
                        // the larger, since with XCD-contiguous ranges the other one is what every XCD fetches whole
    FastDiv div_tiles_m;  // by tiles_m
    FastDiv div_s;        // by S (the wave-split members find their first filter tap with it)
    int32_t xl;         // 0: x is [N][C][H][W]; 1: channels-last, gathered row by row; 2: channels-last,
                        // gathered as 16-byte channel quads (reduction rows ordered (r, s, c)); 3: [N][C][H][W]
                        // with the reduction ordered (r, s, c), one filter tap per step
    int32_t yl;         // 1: y (and the residual) are channels-last; 2: also K % 4 == 0 and y, residual and
                        // bias 16-byte aligned, so a pixel's channel quads move as 16-byte accesses
};

// What follows the convolution inside the same launch (Section 2.1, operator fusion).
struct Epilogue {
    const float *bias = nullptr;
    const float *res = nullptr;
    int relu = 0;
    bool any() const { return bias || res || relu; }
};

static const int64_t kFixupCounterBytes = 1 << 20;   // room for 262144 shared tiles
static const int64_t kFixupMaxBytes = (int64_t)1 << 30;  // default cap; beyond it, atomics
extern std::atomic<int64_t> g_workspace_limit;  // wpk_set_workspace_limit()
// Fix-up workspace a launch of `cfg` needs (split reduction or persistent): shared tiles, slots per tile, bytes
// (a fixed-size counter region first, then the slots).  All zero when nothing is shared or the
// workspace would be too large (the launch then accumulates with atomics).
struct FixupNeed {
    int64_t shared_tiles, maxc, bytes, slots_offset;
};
FixupNeed fixup_need(const Problem &pr, const wpk_conv_config &cfg, int compute_units);

// host-side state shared between wpk_host.cpp and wpk_api.hip
void set_last_hip_error(int e);
void set_device_name(const std::string &name);
std::string device_name();
bool legal_for(const Problem &pr, const wpk_conv_config &cfg);
void default_config(const Problem &pr, int compute_units, wpk_conv_config *out);
// Whether the wave-split members can run pr at all and its 32 x 32 output blocks times its octets of
// reduction rows stay within the bound (the work is then small enough for them to be worth timing).
bool wave_split_candidate(const Problem &pr, int64_t max_block_octets);

}  // namespace wpk
#endif
