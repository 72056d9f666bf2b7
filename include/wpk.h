/*
 * wpk.h -- C ABI of the MI355X (gfx950) forward 2-D convolution library.
 *
 * The operator is the one the paper's search and code generation exist to speed up
 * (Section 2.3 "State space": problem parameters N, C_in, C_out, K_h, K_w, H, W, Stride,
 * Padding; Section 2.2: the sample algorithm is a cross-correlation, filter(r) * in(x+r-1)),
 * widened to separate h/w strides, explicit symmetric zero padding and dilation:
 *
 *   y[n,k,p,q] = sum_{c,r,s} x[n,c, p*stride_h - pad_h + r*dil_h, q*stride_w - pad_w + s*dil_w]
 *                            * w[k,c,r,s]            (taps outside the image count as zero)
 *   P = floor((H + 2*pad_h - dil_h*(R-1) - 1)/stride_h) + 1,  Q alike.
 *
 * Conventions for every entry point
 *   - x, w, y are DEVICE pointers owned by the caller: dense fp32, x = [N][C][H][W],
 *     w = [K][C][R][S], y = [N][K][P][Q] (x and/or y channels-last instead when the descriptor's
 *     layout says so), at least 4-byte aligned.  y is overwritten in full (no accumulate).  x
 *     and y must not overlap.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is enqueued
 *     on it and the call returns without synchronising, unless stated otherwise.  The one-shot
 *     entry points (wpk_conv2d_fwd, _fwd_config, _fwd_fused, _fwd_fused_config) keep library
 *     scratch that grows on demand: the first call with a new descriptor allocates its lookup
 *     table, and a call that needs more packed-weight or workspace room than any call before it
 *     frees and re-allocates that scratch, which synchronises the device.  Such a call must not be
 *     recorded by a stream capture; calls after it with the same shapes only enqueue launches.
 *     They serialise on one process-wide lock while they enqueue.  Plans allocate at build time
 *     only; wpk_conv2d_fwd_noalloc never allocates.
 *   - Descriptors and config structs are HOST memory, copied by value during the call.
 *   - Return value: 0 (WPK_OK) or a negative WPK_E_* code; functions that return an id return
 *     it as a non-negative int.  Nothing throws or aborts across this boundary.
 *   - Calls that share a stream are ordered; calls on different streams that use the one-shot
 *     entry points share library scratch (packed weights, lookup tables, the workspace in which
 *     workgroups that share an output tile meet) and must not overlap.
 *     Plans own their scratch and may run concurrently with each other; the layers of one plan
 *     share it and must run one after another (one stream, or ordered streams).
 *   - The library never falls back to the CPU: without a usable GPU every compute entry point
 *     returns WPK_E_HIP.
 */
#ifndef WPK_H
#define WPK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes --------------------------------------------------------------------- */
enum {
    WPK_OK            = 0,
    WPK_E_BAD_DESC    = -1, /* non-positive size/stride/dilation, negative pad, P<=0 or Q<=0      */
    WPK_E_NULL_PTR    = -2, /* a required pointer argument is NULL                                */
    WPK_E_UNSUPPORTED = -3, /* dtype other than fp32, layout value out of range, or a tensor beyond 2^30 elements */
    WPK_E_HIP         = -4, /* a HIP runtime call failed; wpk_last_hip_error() has the code       */
    WPK_E_NO_CONFIG   = -5, /* config id out of range, or not legal for this descriptor           */
    WPK_E_BAD_ARG     = -6, /* any other invalid argument (index out of range, bad sizes ...)     */
    WPK_E_IO          = -7, /* cache file could not be read or written                            */
    WPK_E_VERIFY      = -8, /* tuner: no candidate reproduced the reference kernel's output       */
    WPK_E_TOO_LARGE   = -9  /* wpk_conv2d_fwd_noalloc: the layer's packed weights exceed the static scratch */
};

enum { WPK_F32 = 0 };
/* Activation layouts.  Bit 0: x is channels-last [N][H][W][C]; bit 1: y (and a fused residual) is
 * channels-last [N][P][Q][K].  Weights are always [K][C][R][S].  The two mixed values make the
 * kernel that computes a layer also transform the layout (Section 2.1, data layout transformation)
 * at no extra pass over memory.  Channels-last x is gathered in 16-byte channel quads when C is a
 * multiple of 32, row by row otherwise. */
enum { WPK_NCHW = 0, WPK_X_NHWC = 1, WPK_Y_NHWC = 2, WPK_NHWC = 3 };

/* ---- the convolution problem (Section 2.3 "State space", first nine observation entries) -- */
typedef struct wpk_conv_desc {
    int32_t n, c, h, w;             /* input batch, channels C_in, height, width                  */
    int32_t k, r, s;                /* output channels C_out, filter rows K_h, filter columns K_w */
    int32_t stride_h, stride_w;     /* >= 1                                                       */
    int32_t pad_h, pad_w;           /* >= 0, zeros added on both sides (VALID = 0)                */
    int32_t dil_h, dil_w;           /* >= 1                                                       */
    int32_t dtype;                  /* WPK_F32                                                    */
    int32_t layout;                 /* WPK_NCHW, WPK_NHWC, WPK_X_NHWC or WPK_Y_NHWC              */
} wpk_conv_desc;

/* Validate `d` and return the output extent.  p, q may be NULL.  Host only. */
int wpk_conv_out_shape(const wpk_conv_desc *d, int32_t *p, int32_t *q);

/* 2*N*K*P*Q*C*R*S, the direct-convolution operation count, or 0 for an invalid descriptor. */
double wpk_conv_flops(const wpk_conv_desc *d);

/* Text of a status code (static storage). */
const char *wpk_status_string(int status);

/* hipError_t value of the most recent WPK_E_HIP on this thread (0 if none). */
int wpk_last_hip_error(void);

/* ---- the kernel family: one "configuration" = one chromosome (Section 2.3 "Search space") -- */
/*
 * Every gene is an integer with a finite range.  A chromosome is legal for a descriptor when
 * wpk_config_legal() says so (the constraint check of Step1): the tile combination must be one
 * the library was built with, its LDS and workgroup size must fit a gfx950 compute unit,
 * split_k may not exceed the number of reduction steps, and the persistent schedule excludes
 * split_k > 1 and always has xcd_remap = 1.
 *
 * Two forms of kernel share the genes.  With bm >= 64 a workgroup stages a bm x bn tile's operands
 * through LDS and its wm x wn waves each own a part of the tile (the tiled members).  With bm = 32
 * (the wave-split members, for launches of a few microseconds: single images, layers of few
 * pixels) a workgroup owns a 32 x bn tile and its wm * wn waves cut the reduction between them,
 * each fetching its operands straight into registers, and add their partial tiles up in LDS;
 * these take bk = 8 (they work in octets of reduction rows), need the reduction ordered
 * (r, s, c) (C a multiple of 32) and have no persistent schedule.
 */
#define WPK_N_GENES 10
typedef struct wpk_conv_config {
    int32_t bm;        /* output pixels per workgroup tile:      32 (wave-split), 64, 128, 256      */
    int32_t bn;        /* output channels per workgroup tile:    32, 64, 128                        */
    int32_t bk;        /* reduction (c,r,s) entries per step:    8, 16, 32                          */
    int32_t wm;        /* waves along the pixel dimension:       1, 2, 4                            */
    int32_t wn;        /* waves along the channel dimension:     1, 2, 4                            */
                       /* (bm = 32: wm * wn = 1, 2, 4 or 8 waves along the reduction)               */
    int32_t split_k;   /* slices of the reduction done by separate workgroups: 1 .. 16, 20, 24     */
    int32_t xcd_remap; /* 0: tiles in launch order; 1: contiguous tile ranges per XCD (persistent:   */
                       /* within each whole round of tiles)                                        */
    int32_t persist;   /* 0: one workgroup per tile and slice; 1..4: that many persistent          */
                       /* workgroups per compute unit taking whole tiles round by round; the      */
                       /* reduction steps of the tiles that do not fill a whole round are dealt   */
                       /* out evenly in runs, to further workgroups of the same launch when the   */
                       /* device holds them all at once, else to the first workgroups, which do   */
                       /* their run before their tiles (split_k must be 1)                        */
    int32_t stages;    /* input tiles in flight in registers between global memory and LDS: 1..3   */
                       /* (bm = 32: four octets in flight per wave for each)                        */
    int32_t reduce;    /* how workgroups that share a tile (split_k > 1 or persist > 0) add up:      */
                       /* 0: partial tiles through a device workspace, the last to arrive sums and */
                       /*    stores (no zeroing of y, fused epilogue applied in the same launch);   */
                       /* 1: fp32 atomics into y zeroed by a launch of its own (cheaper when many   */
                       /*    small slices meet).  Must be 0 when nothing is shared                  */
} wpk_conv_config;

/* Gene ranges as index ranges into the value lists above: lo[g] = 0, hi[g] = count-1.
 * wpk_config_from_genes turns gene indices into a config.  Host only. */
int wpk_config_gene_ranges(int32_t lo[WPK_N_GENES], int32_t hi[WPK_N_GENES]);
int wpk_config_from_genes(const int32_t genes[WPK_N_GENES], wpk_conv_config *out);
int wpk_config_to_genes(const wpk_conv_config *cfg, int32_t genes[WPK_N_GENES]);

/* Constraint check: 1 legal, 0 illegal, <0 error (bad descriptor).  Host only. */
int wpk_config_legal(const wpk_conv_desc *d, const wpk_conv_config *cfg);

/* Config ids: a dense non-negative encoding of the gene indices. */
int wpk_config_id(const wpk_conv_config *cfg);                 /* <0 if a value is not in its list */
int wpk_config_from_id(int id, wpk_conv_config *out);

/* The library's untuned default for a descriptor (a shape heuristic).  Always legal. */
int wpk_config_default(const wpk_conv_desc *d, wpk_conv_config *out);

/* ---- one-shot convolution ------------------------------------------------------------------ */
/*
 * y = conv(x, w) with the cached tuned config of `d` if wpk_conv_tune()/wpk_cache_load() stored
 * one, else the default.  w is in KCRS order and is re-packed into library scratch on every call
 * (weights may have changed); callers with fixed weights should use a plan.
 */
int wpk_conv2d_fwd(const wpk_conv_desc *d, const float *x, const float *w, float *y, void *stream);

/* Same with an explicit configuration (WPK_E_NO_CONFIG if illegal for d). */
int wpk_conv2d_fwd_config(const wpk_conv_desc *d, const wpk_conv_config *cfg, const float *x,
                          const float *w, float *y, void *stream);

/*
 * The fused operator (Section 2.1, operator fusion: a sub-graph computed by one kernel so that
 * the intermediate tensors never travel through memory):
 *     y[n][k][p][q] = act( conv(x, w)[n][k][p][q] + bias[k] + residual[n][k][p][q] ),
 * act = max(., 0) if relu != 0, else the identity.  bias ([K]) and residual (laid out like y)
 * are DEVICE pointers and may each be NULL (term absent); residual must not overlap y.  The
 * epilogue is applied by the workgroup that stores the output; only where a launch has to
 * accumulate with atomics (no workspace large enough) or uses the direct kernel does it follow
 * as a second launch.  Errors as wpk_conv2d_fwd.
 */
int wpk_conv2d_fwd_fused(const wpk_conv_desc *d, const float *x, const float *w, const float *bias,
                         const float *residual, int32_t relu, float *y, void *stream);

/* Same with an explicit configuration (WPK_E_NO_CONFIG if illegal for d). */
int wpk_conv2d_fwd_fused_config(const wpk_conv_desc *d, const wpk_conv_config *cfg, const float *x,
                                const float *w, const float *bias, const float *residual,
                                int32_t relu, float *y, void *stream);

/*
 * wpk_conv2d_fwd_config for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and result
 * (`cfg` may also be NULL: the cached tuned configuration of `d`, else the default); it calls no
 * hipMalloc, hipFree or other allocating routine and does not synchronise.  Its lookup table,
 * packed weights and the workspace of shared tiles live in one static device array of
 * WPK_NOALLOC_SCRATCH_BYTES (32 MiB) that every GPU the library runs on holds until the process
 * ends.  Limit: the packed weights, (C*R*S rounded up to 32) x (K rounded up to 128) floats, must
 * fit 32 MiB less 1088 KiB (e.g. 3x3 with C = K = 896, or 1x1 2048 -> 3840), else WPK_E_TOO_LARGE
 * and nothing is enqueued; where the workspace of shared tiles does not fit beside them the launch
 * sums with atomics into y instead (zeroed by a launch of its own).  Every call on a GPU uses
 * that GPU's one array: calls on the same stream are ordered and safe, calls that overlap on one
 * GPU (different streams, different threads) race.  A layer outside the tiled family runs on the
 * direct kernel, which needs no scratch.
 */
#define WPK_NOALLOC_SCRATCH_BYTES (32 << 20)
int wpk_conv2d_fwd_noalloc(const wpk_conv_desc *d, const wpk_conv_config *cfg, const float *x,
                           const float *w, float *y, void *stream);

/* Plain one-output-per-lane direct kernel (no MFMA, no LDS, 64-bit indexing).  The on-device
 * reference the tuner vets candidates against; also serves shapes the tiled family rejects. */
int wpk_conv2d_ref(const wpk_conv_desc *d, const float *x, const float *w, float *y, void *stream);

/* ---- tuning (Section 2.3 "Genetic search", Steps 1-4; cache: Section 3.3) --------------------- */
typedef struct wpk_tune_options {
    int32_t population;   /* |a|, default 64                                                     */
    int32_t elites;       /* k, default 8                                                        */
    int32_t next_population; /* |a'|, default = population                                        */
    int32_t participants; /* m, default = population                                              */
    int32_t max_generations; /* default 16                                                       */
    int32_t patience;     /* stop after this many generations without a better best, default 5   */
    double  mutation;     /* per-gene mutation probability, default 0.15                         */
    double  eps;          /* Step4: all runtimes within eps of the fastest, default 0.03         */
    uint64_t seed;        /* default 2008                                                        */
    int32_t reps;         /* timed groups per candidate (median taken), default 5                */
    double  min_group_us; /* each timed group is sized to last at least this long, default 200   */
    int32_t mode;         /* 0 genetic search, 1 random search (same budget), 2 exhaustive        */
    int32_t verbose;      /* 1: print one line per generation to stderr                          */
    int32_t refine;       /* after a search (modes 0, 1): a few dozen rule-based candidates are
                             timed beside the winner, then at most this many rounds of trying every
                             other value of one gene of the winner at a time, then the five
                             fastest candidates are timed again in groups of at least 4 ms
                             (clocks settled under load) and the fastest kept; not part of
                             the paper's search; 0 = off, default 2                               */
    int32_t zero_ahead;   /* how candidates that accumulate into y with atomics are timed: 0 (default)
                             with the launch that zeroes y, as a single call pays it; 1 without it,
                             as in a plan run as whole passes, which zeroes such outputs once per pass
                             ahead of the layers (wpk_plan_run); the candidate is charged its share of
                             that launch at 3 TB/s instead                                        */
    int32_t epilogue;     /* 1: candidates are timed with a rectifier as epilogue, for layers that will
                             run with one (wpk_plan_set_epilogue): fused into the launch where the
                             configuration allows, a pass of its own after atomics; 0 (default): none */
} wpk_tune_options;

/* Fill `o` with the defaults above. */
void wpk_tune_default_options(wpk_tune_options *o);

typedef struct wpk_tune_report {
    wpk_conv_config best;
    double best_us;        /* median runtime of the winner, microseconds                         */
    double default_us;     /* runtime of wpk_config_default() under the same protocol            */
    int32_t evaluations;   /* distinct chromosomes timed                                         */
    int32_t generations;
    int32_t rejected;      /* candidates that failed verification against wpk_conv2d_ref        */
    double seconds;        /* wall time of the search                                            */
    int32_t stage;         /* which stage found `best`: WPK_STAGE_SEARCH (the search of Section 2.3
                              itself), _RULE (a rule-based candidate), _REFINE (one gene of the winner
                              varied), _DEFAULT (nothing beat wpk_config_default); the last three are
                              the additions `refine` switches on                                  */
    double search_us;      /* runtime of the best chromosome of the search alone, as the search timed it */
} wpk_tune_report;
enum { WPK_STAGE_SEARCH = 0, WPK_STAGE_RULE = 1, WPK_STAGE_REFINE = 2, WPK_STAGE_DEFAULT = 3 };

/*
 * Search the kernel family for `d` on the current device with synthetic operands the library
 * allocates itself, verify the winner against wpk_conv2d_ref, store it in the in-memory cache and
 * return its config id (>= 0).  A cached descriptor returns at once.  Synchronises the device.
 */
int wpk_conv_tune(const wpk_conv_desc *d);

/* Same with options and a report (either may be NULL); `force` != 0 ignores a cached entry. */
int wpk_conv_tune_ex(const wpk_conv_desc *d, const wpk_tune_options *opt, int force,
                     wpk_tune_report *report);

/* Cache of search results, keyed by every descriptor field ("computationally identical"
 * operators, Section 3.1) plus the device name.  Text file, one line per entry. */
int wpk_cache_lookup(const wpk_conv_desc *d, wpk_conv_config *out); /* 1 hit, 0 miss          */
int wpk_cache_lookup_time(const wpk_conv_desc *d, wpk_conv_config *out, double *us); /* also the stored runtime */
int wpk_cache_store(const wpk_conv_desc *d, const wpk_conv_config *cfg, double us);
int wpk_cache_clear(void);
int wpk_cache_size(void);
int wpk_cache_save(const char *path);
int wpk_cache_load(const char *path);                              /* returns entries read or <0 */

/*
 * The search engine by itself, over any integer gene space, with caller-supplied constraint and
 * fitness callbacks (host function pointers; `user` is passed through).  Fitness: larger is
 * better, 0 = cannot run.  Random numbers: one splitmix64 stream seeded with opt->seed, consumed
 * in the order of Steps 1-4.  `history_pop` (generations x max(population,next_population) x
 * n_genes, int32) and `history_fit` (generations x max(...), double), if not NULL, receive every
 * generation (unused slots -1 / -1.0); `history_sizes` receives each generation's population size.
 * Returns the number of generations run (>= 1) or a negative status.  Host only, no GPU needed.
 */
typedef int (*wpk_ga_constraint_fn)(const int32_t *genes, int32_t n_genes, void *user);
typedef double (*wpk_ga_fitness_fn)(const int32_t *genes, int32_t n_genes, void *user);
int wpk_ga_search(int32_t n_genes, const int32_t *lo, const int32_t *hi,
                  wpk_ga_constraint_fn constraint, wpk_ga_fitness_fn fitness, void *user,
                  const wpk_tune_options *opt, int32_t *best_genes, double *best_fitness,
                  int32_t *evaluations, int32_t *history_pop, double *history_fit,
                  int32_t *history_sizes, int32_t history_capacity);

/* ---- plans: a list of layers with per-layer tuned configs and pre-packed weights ------------- */
typedef struct wpk_plan wpk_plan;

/* Build a plan for n_layers descriptors (host array).  Layers with identical descriptors share
 * one search.  A layer outside the tiled family runs on the direct kernel; wpk_plan_layer_config
 * reports it as an all-zero configuration.  `tune` = 0 uses cached/default configs, 1 runs wpk_conv_tune on cache misses.
 * Allocates device memory for packed weights and split-K needs; synchronises the device. */
int wpk_conv_plan(const wpk_conv_desc *layers, int32_t n_layers, int32_t tune, wpk_plan **out);

/*
 * A plan that chooses the layout of the tensors between its layers (Section 2.1, data layout
 * transformation).  The caller names tensors by small integers: layer i reads tensor x_tensor[i],
 * writes tensor y_tensor[i] and, if residual_tensor is not NULL and residual_tensor[i] >= 0, adds
 * that tensor in its epilogue (it is then stored like the layer's output).  tensor_layout[t] says
 * what the caller dictates for tensor t: 0 = [N][C][H][W], 1 = channels-last, -1 = the plan's
 * choice (typically: the network's input and output fixed, everything between free).  The
 * `layout` field of the descriptors passed in is ignored.  For every layer and every combination
 * of layouts its two tensors may take, the plan takes the runtime of the cached searched
 * configuration, searches it (tune != 0), or times the default configuration (tune == 0, a few
 * milliseconds per combination); then the layouts that minimise the sum over the layers are
 * chosen (wpk_choose_layouts) and every layer gets the layout code of its two tensors: a layer
 * whose tensors differ transforms the layout while it computes, at no extra pass over memory.
 * wpk_plan_tensor_layout tells the caller how to store, or read, tensor t.  Everything else is
 * as for wpk_conv_plan.  WPK_E_BAD_ARG for tensor numbers out of range or tied tensors fixed to
 * different layouts.
 */
int wpk_conv_plan_graph(const wpk_conv_desc *layers, int32_t n_layers, const int32_t *x_tensor,
                        const int32_t *y_tensor, const int32_t *residual_tensor,
                        const int32_t *tensor_layout, int32_t n_tensors, int32_t tune, wpk_plan **out);
int wpk_plan_tensor_layout(const wpk_plan *plan, int32_t tensor);   /* 0, 1, or a negative status */
int wpk_plan_layer_layout(const wpk_plan *plan, int32_t layer);     /* WPK_NCHW .. WPK_NHWC        */

/* The optimiser by itself (host only): cost[(i*2 + lx)*2 + ly] is layer i's cost when it reads a
 * tensor in layout lx and writes one in layout ly (any unit; combinations that cannot occur are
 * never looked at); chosen[t] receives 0 or 1 for every tensor, *total (may be NULL) the minimised sum. */
int wpk_choose_layouts(int32_t n_layers, const int32_t *x_tensor, const int32_t *y_tensor,
                       const int32_t *residual_tensor, const int32_t *tensor_layout, int32_t n_tensors,
                       const double *cost, int32_t *chosen, double *total);

/* Copy and re-pack layer `layer`'s weights (device pointer, KCRS) into the plan, on `stream`. */
int wpk_plan_set_weights(wpk_plan *plan, int32_t layer, const float *w, void *stream);

/* The run calls below only enqueue kernel launches (and, with pipelining, event records and
 * waits): they allocate nothing and may be recorded by a stream capture into a HIP graph. */
/* Run every layer in order on `stream`: y[i] = conv(x[i], weights of layer i).  x and y are HOST
 * arrays of n_layers DEVICE pointers.  Weights of every layer must have been set.  A layer with
 * an epilogue (wpk_plan_set_epilogue) applies it.  Tensors may be shared between layers in any way
 * a layer-by-layer run allows (an output feeding later layers, buffers reused in turns): outputs
 * that a layer accumulates into with atomics are zeroed by a single launch at the start of the
 * pass only where they overlap nothing that an earlier layer of the pass reads or writes, and
 * right before their layer otherwise. */
int wpk_plan_run(wpk_plan *plan, const float *const *x, float *const *y, void *stream);

/* Run one layer of the plan. */
int wpk_plan_run_layer(wpk_plan *plan, int32_t layer, const float *x, float *y, void *stream);

/* Two-way pipelining (ways = 2; 1 turns it off): every layer's batch is cut into two halves that
 * run as two independent chains, the first on the caller's stream and the second on a stream the
 * plan owns, forked from and joined to the caller's stream once per wpk_plan_run(_fused) call (once
 * per layer for the run_layer calls).  Convolution treats the images of a batch independently,
 * so the results are those of the unsplit plan whatever the layers feed each other; what it buys
 * is that the ramp, the meeting of shared tiles and the drain of one chain's launches hide
 * behind the other chain's arithmetic (about 6 % on a 53-layer stack at N = 16; it does not pay
 * for passes of a few layers).  The two chains are not ordered against each other inside a pass,
 * so a pass is split only when nothing one chain writes overlaps anything the other chain reads or
 * writes at any layer (checked from the pointers of each wpk_plan_run(_fused) call: buffers reused
 * in turns by tensors of different per-image size fail it); a pass that fails the check runs as one
 * chain, with the same results.  Each half uses the cached configuration of its own descriptor
 * (batch n/2) if there is one, else the default; wpk_plan_set_layer_config also applies to the
 * halves where the configuration is legal for them.  WPK_E_UNSUPPORTED if a layer has batch 1.
 * Synchronises the device. */
int wpk_plan_set_pipeline(wpk_plan *plan, int32_t ways);

/* Give layer `layer` a fused epilogue (see wpk_conv2d_fwd_fused): `bias` is a DEVICE pointer to K
 * floats, copied into the plan on `stream` (NULL: no bias); relu != 0 adds the rectifier.  Every
 * later run of the layer, fused or not, applies it. */
int wpk_plan_set_epilogue(wpk_plan *plan, int32_t layer, const float *bias, int32_t relu, void *stream);

/* Like wpk_plan_run_layer / wpk_plan_run with a residual tensor added before the rectifier:
 * `residual` is a DEVICE pointer laid out like y (NULL: none); for the whole plan a HOST array of
 * n_layers such pointers (the array itself, or any entry, may be NULL). */
int wpk_plan_run_layer_fused(wpk_plan *plan, int32_t layer, const float *x, const float *residual,
                             float *y, void *stream);
int wpk_plan_run_fused(wpk_plan *plan, const float *const *x, const float *const *residual,
                       float *const *y, void *stream);

int wpk_plan_num_layers(const wpk_plan *plan);
int wpk_plan_num_unique(const wpk_plan *plan);                       /* distinct descriptors     */
int wpk_plan_layer_config(const wpk_plan *plan, int32_t layer, wpk_conv_config *out);
int wpk_plan_set_layer_config(wpk_plan *plan, int32_t layer, const wpk_conv_config *cfg);
void wpk_plan_destroy(wpk_plan *plan);

/* Cap, in bytes, on the device workspace a launch may use to sum the partial tiles of split and
 * persistent schedules (default 1 GiB).  A launch that would need more accumulates with fp32
 * atomics into zeroed outputs instead (one more launch; a fused epilogue then follows as another).
 * 0 turns the workspace off.  Applies to launches prepared afterwards; WPK_E_BAD_ARG if negative. */
int wpk_set_workspace_limit(int64_t bytes);

/* Workspace a launch of `cfg` on a device with `compute_units` CUs uses to sum shared tiles: the
 * byte count (0: nothing is shared, atomics were asked for, or the cap is exceeded), and through
 * the optional pointers the number of shared tiles and of partial-tile slots per shared tile.
 * Host only; negative WPK_E_* on a bad descriptor or an illegal configuration. */
int64_t wpk_config_workspace_bytes(const wpk_conv_desc *d, const wpk_conv_config *cfg,
                                   int32_t compute_units, int64_t *shared_tiles, int64_t *slots);

/* ---- introspection used by the benchmark ----------------------------------------------------- */
/* Name of the device kernel a config launches (static storage), e.g. "wpk_igemm_128x64x16_2x2_p2". */
const char *wpk_config_kernel_name(const wpk_conv_config *cfg);
/* Device name and compute-unit count of the current device. */
int wpk_device_info(char *name, int32_t name_capacity, int32_t *compute_units);
/* Measured ceilings of the current device, for reporting beside the published ones (calibration, no
 * part of the operator; sustained clocks under matrix load lie below the peak engine clock).
 *   mfma_tflops_burst     : one 0.3 ms launch of an fp32 MFMA-only kernel (32x32x2, four independent
 *                           accumulators per wave, two waves per SIMD, varied operands) right after a
 *                           20 ms pause: clock ramp-up and launch latency included
 *   mfma_tflops_sustained : the same kernel launched back to back for sustain_ms (0 .. 10000) in all;
 *                           the rate over the second half
 *   copy_gbs              : bytes read plus bytes written per second by a 16-byte-per-lane copy of 256 MiB
 * Any of the three pointers may be NULL (that measurement is skipped; host pointers otherwise).
 * Allocates and frees its own device buffers, enqueues on `stream` and synchronises it. */
int wpk_measure_peaks(double sustain_ms, double *mfma_tflops_burst, double *mfma_tflops_sustained,
                      double *copy_gbs, void *stream);
/* Library version string. */
const char *wpk_version(void);

#ifdef __cplusplus
}
#endif
#endif /* WPK_H */
