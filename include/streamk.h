/* streamk.h - C ABI of the MI355X Stream-K++ GEMM library (libstreamk.so).
 *
 * The library computes D = A * B (fp16 / bf16 / fp8-e4m3 inputs, fp32
 * accumulation) with the work of all output tiles - tiles x K-iterations of the
 * MAC loop - divided over a persistent grid of workgroups under one of the
 * Stream-K++ scheduling policies, and holds the Bloom-filter selector that
 * prunes policies for a problem size.  Citations are to the paper
 * "Stream-K++: Adaptive GPU GEMM Kernel Selection and Scheduling for AI using
 * Bloom Filters" (arXiv 2408.11417).
 *
 * Conventions for every entry point
 *  - returns an sk_status (0 = ok, negative = error); nothing throws or aborts
 *    across this boundary; out-parameters are left untouched on error;
 *  - "host" pointers are ordinary process memory, "device" pointers are HIP
 *    device memory of the current device, at least 16-byte aligned;
 *  - the caller owns A, B, D, the workspace and the stream; the library owns
 *    the opaque sk_plan_t / sk_bloom_t objects (create / destroy pairs);
 *  - matrices are dense row-major: A is M x K (leading dimension K), B is K x N
 *    (leading dimension N), D is M x N (leading dimension N).
 */
#ifndef STREAMK_H
#define STREAMK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SK_OK = 0,
    SK_ERR_INVALID_ARG = -1,  /* null pointer, non-positive size, unknown enum value       */
    SK_ERR_UNSUPPORTED = -2,  /* no kernel for this tile / dtype, or grid cannot be resident */
    SK_ERR_WORKSPACE = -3,    /* workspace missing or too small                             */
    SK_ERR_HIP = -4,          /* a HIP runtime call failed                                  */
    SK_ERR_NOMEM = -5,        /* host allocation failed                                     */
    SK_ERR_TIMEOUT = -6       /* a tile owner gave up waiting for a partial (see sk_plan_check) */
} sk_status;

/* The seven scheduling policies (Sec. 3.2, Sec. 4.1): b Stream-K batches issued
 * first, data-parallel batches after them.  b = 0 is the conventional
 * data-parallel schedule (Sec. 1), ALL_SK is Algorithm 1 applied to every tile.
 * One Stream-K batch is one trip of Algorithm 1's outer loop per workgroup, so
 * b batches cover the remainder wave (tiles mod grid) plus b-1 full waves of
 * tiles, clamped to the tile count.  SK6_DP_EXT (b = 6) is an extension beyond
 * the seven. */
typedef enum {
    SK_POLICY_DP = 0,
    SK_POLICY_SK1_DP = 1,
    SK_POLICY_SK2_DP = 2,
    SK_POLICY_SK3_DP = 3,
    SK_POLICY_SK4_DP = 4,
    SK_POLICY_SK5_DP = 5,
    SK_POLICY_ALL_SK = 6,
    SK_POLICY_SK6_DP_EXT = 7
} sk_policy;
#define SK_NUM_POLICIES 7

typedef enum { SK_F16 = 0, SK_BF16 = 1, SK_FP8_E4M3 = 2, SK_F32 = 3 /* output only */ } sk_dtype;

/* Role of a segment in the fix-up (Sec. 5.3: partial results combined under
 * inter-workgroup synchronisation instead of Algorithm 1's atomic adds). */
typedef enum {
    SK_ROLE_FULL = 0,    /* all K-iterations of the tile: store D directly                      */
    SK_ROLE_OWNER = 1,   /* holds K-iteration 0 (under SK_SEGMENTS_K_ALIGNED: the tile's last
                            K-iteration): waits for the contributors, reduces, stores D         */
    SK_ROLE_CONTRIB = 2  /* any other part of a split tile: stores an fp32 partial tile and signals */
} sk_role;

/* How the partial results of a split tile are combined.
 * FLAGS (default): the workspace-and-flags exchange described at sk_role, the
 * alternative Sec. 5.3 names; the owner adds the partials in a fixed order
 * (see sk_segment_order; when a tile has 16 or more contributors, in two
 * levels: every 8th contributor first adds the partials of the 7 behind it to
 * its own and parks the sum), so D is bit-identical from run to run.
 * ATOMIC: the accumulation step of Algorithm 1, as printed: every workgroup that holds only
 * part of a tile's K-iterations adds its accumulators into a zero-initialised
 * fp32 image of D with atomic adds, nobody waits for anybody.  The order of the
 * additions depends on timing, so D may differ in the last bits between runs. */
typedef enum { SK_FIXUP_FLAGS = 0, SK_FIXUP_ATOMIC = 1 } sk_fixup;

/* Which phase a workgroup runs first.  STREAMK_FIRST (default): its Stream-K
 * iterations, then its data-parallel tiles, so that the exchange of partial
 * tiles overlaps with data-parallel work (Sec. 3.2, Sec. 4.1).
 * DATA_PARALLEL_FIRST: the earlier hybrid that Sec. 3.2 describes - data-parallel
 * batches followed by the Stream-K work; kept for comparison.  Which tiles are
 * split and which workgroup gets which work is the same under both. */
typedef enum { SK_STREAMK_FIRST = 0, SK_DATA_PARALLEL_FIRST = 1 } sk_batch_order;

/* In which order a workgroup runs the pieces of its Stream-K range, and who owns
 * a split tile.  ASCENDING: Algorithm 1's order - ascending iteration
 * index, i.e. the tail of the first tile, whole tiles, the head of the last tile;
 * the workgroup holding a tile's K-iteration 0 owns it.  Workgroups then sit at
 * K offsets that differ by their distance in the iteration space, and the operand
 * blocks that neighbouring tiles share are fetched at different times (the loss
 * of cache locality Sec. 5.3 remarks on).
 * K_ALIGNED (default): a range that contains a tile boundary runs its whole
 * tiles first, then the head of its last tile (K-iterations from 0), then the
 * tail of its first tile; whole tiles and head pieces then start at K-iteration
 * 0 together in all workgroups.  The workgroup holding a tile's last
 * K-iteration owns the tile - that piece is the last of its Stream-K work, so
 * it never waits while other work is pending - and adds the partials in
 * descending workgroup order.
 * Which workgroup runs which iterations is the same under both. */
typedef enum { SK_SEGMENTS_ASCENDING = 0, SK_SEGMENTS_K_ALIGNED = 1 } sk_segment_order;

/* How a tile index maps to a position in the tile grid.  The schedule (which
 * workgroup runs which tile index) does not depend on it.  GROUPED follows the
 * remark of Sec. 5.3 that work should be handed out with cache locality in
 * mind: the grid is cut into bands of 8 tile rows; inside a band the index
 * walks down the band's rows, then one column to the right, so consecutive
 * indices (which run at the same time on neighbouring workgroups) share A
 * row-blocks and B column-blocks.  When sk_config leaves the order open the
 * library takes, per plan, the order under which the tiles that one XCD's
 * workgroups hold at the same time (an eighth of the first min(tiles, grid) tile
 * indices) span fewer operand rows and columns: A row-blocks x blk_m + B
 * column-blocks x blk_n. */
typedef enum { SK_ORDER_ROW_MAJOR = 0, SK_ORDER_GROUPED = 1 } sk_tile_order;

/* Tile shape, grid and types.  A zero field means "library default": the tile
 * is then chosen from (M, N, K), grid = 256 (one workgroup per compute unit),
 * in_dtype = SK_BF16, out_dtype = in_dtype (SK_BF16 for fp8 inputs),
 * tile_order = chosen per plan (see sk_tile_order). */
typedef struct {
    int32_t blk_m, blk_n, blk_k;
    int32_t grid;
    int32_t in_dtype;    /* sk_dtype + 1, or 0 for default */
    int32_t out_dtype;   /* sk_dtype + 1, or 0 for default */
    int32_t tile_order;  /* sk_tile_order + 1, or 0 for default */
} sk_config;

/* Algorithm 1's iteration counts, and those of the Stream-K / data-parallel split. */
typedef struct {
    int64_t M, N, K;
    int32_t policy;
    int32_t blk_m, blk_n, blk_k, grid;
    int32_t in_dtype, out_dtype;          /* sk_dtype values */
    int32_t tiles_m, tiles_n, tiles;      /* ceil(M/blk_m), ceil(N/blk_n), their product    */
    int32_t iters_per_tile;               /* ceil(K/blk_k)                                  */
    int64_t total_iters;                  /* tiles * iters_per_tile                         */
    int32_t sk_tiles, dp_tiles;           /* tiles [0, sk_tiles) are split, the rest are not */
    int64_t sk_iters;                     /* sk_tiles * iters_per_tile                      */
    int32_t iters_per_wg;                 /* ceil(sk_iters / grid)                          */
    int32_t dp_waves;                     /* ceil(dp_tiles / grid)                          */
    int32_t has_kernel;                   /* 1 if sk_gemm has a kernel for this tile + dtype */
    int32_t tile_order;                   /* sk_tile_order                                   */
    int32_t fixup, batch_order, segment_order;  /* sk_fixup, sk_batch_order, sk_segment_order: the
                                             defaults, or what the sk_plan_set_* calls chose */
    int32_t xcd_remap;                    /* 1: the kernel renumbers the workgroups so that each of the 8 XCDs
                                             runs grid/8 consecutive ones (neighbours in the schedule, which share
                                             operand blocks, then share an L2); 0: hardware order, consecutive
                                             workgroups on different XCDs - chosen when the tile grid is a single
                                             row of tiles at most 64 rows high, where B is streamed once in narrow
                                             column blocks and spreading neighbouring blocks over the XCDs
                                             measured 8-10 % faster */
} sk_plan_header;

/* Work of one workgroup x: global Stream-K iterations [sk_iter_begin, sk_iter_end)
 * (Algorithm 1's per-workgroup range, clamped to sk_iters), then data-parallel tiles
 * dp_tile_first + j*grid for j in [0, dp_tile_count). */
typedef struct {
    int64_t sk_iter_begin, sk_iter_end;
    int32_t dp_tile_first, dp_tile_count;
} sk_wg_range;

/* One MAC-loop call (Algorithm 1's inner step): workgroup wg runs K-iterations
 * [k_begin, k_end) of tile `tile`.  With (tile_m, tile_n) = sk_plan_tile_coords
 * the tile covers rows tile_m * blk_m ... and columns tile_n * blk_n ... of D. */
typedef struct {
    int32_t wg, tile, k_begin, k_end, role;
} sk_segment;

typedef struct sk_plan_t sk_plan_t;

/* Build the schedule of one problem under one policy (Algorithm 1, up to the
 * per-workgroup iteration range; Sec. 3.2; Sec. 4.1).  Host only, no device contact.  cfg may be NULL (all
 * defaults).  Any positive tile shape is accepted for planning; whether sk_gemm
 * can run it is reported in sk_plan_header.has_kernel.
 * Errors: INVALID_ARG (sizes < 1, unknown policy / dtype, totals beyond int32
 * tiles or int64 iterations), NOMEM. */
int sk_plan(int64_t M, int64_t N, int64_t K, int policy, const sk_config* cfg, sk_plan_t** out);

/* Copy the plan's numbers to host memory. */
int sk_plan_info(const sk_plan_t* plan, sk_plan_header* out);

/* Per-workgroup iteration ranges: out is host memory for `grid` entries. */
int sk_plan_ranges(const sk_plan_t* plan, sk_wg_range* out);

/* Canonical expansion of the schedule: segments ordered by workgroup and, inside
 * a workgroup, in execution order (Stream-K segments in the plan's segment
 * order, then data-parallel tiles, Sec. 4.1; the other way round under
 * SK_DATA_PARALLEL_FIRST).  out is host memory for `cap` entries (may be NULL when cap = 0);
 * *n receives the number of segments; INVALID_ARG if cap is too small (then *n
 * still receives the needed count). */
int sk_plan_segments(const sk_plan_t* plan, sk_segment* out, size_t cap, size_t* n);

/* Position of a tile index in the tile grid under the plan's tile order.
 * INVALID_ARG if tile is outside [0, tiles). */
int sk_plan_tile_coords(const sk_plan_t* plan, int32_t tile, int32_t* tile_m, int32_t* tile_n);

/* Choose the fix-up of split tiles (sk_fixup; Algorithm 1's accumulation for
 * ATOMIC, Sec. 5.3 for FLAGS).  Call it before sk_workspace_bytes /
 * sk_plan_set_workspace: the workspace need depends on it.
 * Errors: INVALID_ARG (unknown mode, or a workspace is already attached). */
int sk_plan_set_fixup(sk_plan_t* plan, int fixup);

/* Choose the order of the two phases inside a workgroup (sk_batch_order;
 * Sec. 3.2).  Changes the execution order that sk_plan_segments reports.
 * Errors: INVALID_ARG (unknown value). */
int sk_plan_set_batch_order(sk_plan_t* plan, int batch_order);

/* Choose the order of the pieces of a workgroup's Stream-K range and the owner
 * of split tiles (sk_segment_order).  Changes the execution order and the roles
 * that sk_plan_segments reports.
 * Errors: INVALID_ARG (unknown value). */
int sk_plan_set_segment_order(sk_plan_t* plan, int segment_order);

/* Device bytes sk_gemm needs for this plan.  FLAGS: one flag line per workgroup,
 * a status word, and one fp32 partial tile (blk_m * blk_n) per workgroup.
 * ATOMIC: the flag and status lines, plus an fp32 image of D (M * N * 4 bytes)
 * unless the plan's output type is SK_F32 (then D itself is accumulated into).
 * Returns 0 for a NULL plan. */
size_t sk_workspace_bytes(const sk_plan_t* plan);

/* Attach caller-owned device memory (>= sk_workspace_bytes, 256-byte aligned).
 * Clears the flag and status area with a blocking memset on the null stream.
 * One workspace must not serve two launches that are in flight at once; it may
 * be shared by plans that run one after another on one stream.
 * Errors: INVALID_ARG, WORKSPACE (too small / misaligned), HIP. */
int sk_plan_set_workspace(sk_plan_t* plan, void* dev_ptr, size_t bytes);

/* Number of flag polls after which a waiting tile owner gives up, records a
 * time-out in the workspace status word and goes on (so that every wave exits
 * even if a partial never arrives).  Default 1 << 24.  0 = give up on the first
 * unsuccessful poll (for tests of the error path). */
int sk_plan_set_spin_limit(sk_plan_t* plan, uint32_t polls);

/* D = A * B under the plan (Algorithm 1 with its MAC loop on the matrix cores;
 * Sec. 4.1 persistent grid; fix-up per Sec. 5.3).  A, B, D: device pointers in
 * the plan's dtypes and the row-major layout stated above.  stream: a
 * hipStream_t (NULL = the null stream).  Asynchronous: enqueues its kernels and
 * returns; never synchronises.  D is fully overwritten.  With SK_FIXUP_FLAGS that
 * is one kernel.  With SK_FIXUP_ATOMIC and a plan that splits tiles it is a fill
 * kernel that zeroes the fp32 image, the GEMM kernel, and - for 16-bit outputs -
 * a conversion kernel from the fp32 image to D; plans without split tiles run
 * the same single kernel under both modes.  No memset or copy node is enqueued
 * and no kernel argument changes from launch to launch, so a launch captured
 * into a HIP graph may be replayed (make one ordinary launch of the plan first:
 * the first use of a kernel sets its LDS limit and asks for its occupancy, which
 * capture does not allow).
 * Co-residency: under SK_FIXUP_FLAGS a tile owner waits inside the kernel for
 * workgroups of the same launch, so all `grid` workgroups must be on the device
 * at once.  sk_gemm checks that against an otherwise idle device; the caller
 * must not let such a launch overlap with other kernels that occupy compute
 * units (e.g. a second sk_gemm on another stream): two launches that each hold
 * part of the device can wait for each other until the bounded wait gives up
 * (SK_ERR_TIMEOUT from sk_plan_check, D invalid).  Plans without split tiles and
 * SK_FIXUP_ATOMIC launches never wait and may overlap freely.
 * Cache policy: a plan with a single row of tiles at most 64 rows high reads B
 * exactly once; if B is also 128 MiB or more (too large to be found in the
 * memory-side cache by a later launch), its loads carry the non-temporal hint.
 * All other operand loads use the default policy.
 * Errors: INVALID_ARG, UNSUPPORTED (no kernel for tile + dtype + fix-up mode,
 * sizes beyond the kernels' 32-bit index range: M*K or K*N >= 2^31 elements,
 * M*N >= 2^32, or the grid cannot be co-resident while the plan has split
 * tiles), WORKSPACE (plan has split tiles but no workspace), HIP (launch failed). */
int sk_gemm(const void* A, const void* B, void* D, const sk_plan_t* plan, void* stream);

/* sk_gemm for callers that cannot allocate device memory or keep a workspace alive: code under
 * HIP-graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and same results as sk_gemm, but the flag lines and partial tiles live in an array inside
 * the library's own device image (one copy per GPU that runs the library, held until the process
 * ends) instead of caller-owned memory; whatever sk_plan_set_workspace attached to the plan is
 * ignored.  The call allocates nothing and frees nothing.  Before the GEMM kernel it enqueues a small
 * fill kernel that takes the flag and status lines down (the array keeps the previous call's
 * contents), so a launch with split tiles is two kernels; a plan without split tiles is one.
 * Limit: sk_workspace_bytes(plan) <= SK_STATIC_WORKSPACE_MAX_BYTES - enough for every tile shape on
 * the default grid of 256 workgroups; larger grids with the largest tiles are refused.
 * All calls on one GPU share that GPU's array: two calls whose kernels may run at the same time
 * (different streams, or replays of graphs that hold them) race on it; calls on one stream do not.
 * A time-out of a tile owner (see sk_plan_set_spin_limit) cannot be read back through this entry
 * point; the next call starts from cleared flags either way.  The first call on a device looks the
 * array's address up and, like sk_gemm, sets up the kernel: make it outside graph capture.
 * Errors: those of sk_gemm, plus WORKSPACE (the plan needs more than the limit) and UNSUPPORTED
 * (SK_FIXUP_ATOMIC with a 16-bit output, whose fp32 image of D has no size bound). */
#define SK_STATIC_WORKSPACE_MAX_BYTES ((size_t)257 * 128 + 384 + (size_t)256 * 256 * 256 * 4)
int sk_gemm_static(const void* A, const void* B, void* D, const sk_plan_t* plan, void* stream);

/* Blocking: waits for `stream` and reads the workspace status word.  Returns
 * SK_OK, or SK_ERR_TIMEOUT if any launch since the last check gave up waiting
 * for a partial tile; in that case the flag and status area is cleared, so the
 * workspace can be used again.  (Flags are raised by contributors and taken
 * down by the owner that waits for them inside the same launch; after a
 * time-out some may be left up, and launches made before this call returns
 * would read partial tiles too early.) */
int sk_plan_check(const sk_plan_t* plan, void* stream);

/* Ask for another compiled wave layout of the plan's tile (a tuning knob of the dispatcher,
 * Sec. 4.1: one kernel instance per tile configuration).  Variant 0 (the default) leaves the choice
 * to the library: the tile's standard kernel, except that the 256 x 256, 256 x 128 and 128 x 128 x 64
 * tiles run a four-wave kernel when the plan has no split tile (and, for the 256-row tiles, enough
 * K-iterations per tile: 48 and 16) and the eight-wave one otherwise.
 * Where a tile has further layouts compiled in they are numbered from 1 (for those three tiles: 1 = four
 * waves, 3 = eight waves, whatever the plan; 256 x 256 also 2 = eight waves with the coarser MAC loop);
 * a tile without the requested variant keeps variant 0.  The results are the same under every variant.
 * Errors: INVALID_ARG (NULL plan, negative number). */
int sk_plan_set_kernel_variant(sk_plan_t* plan, int variant);

/* The kernel that sk_gemm would launch for this plan right now (host only, no GPU
 * call): workgroup size in threads, dynamic LDS bytes per workgroup, and the
 * variant number of the tile's kernel (see sk_plan_set_kernel_variant).  Any out
 * pointer may be NULL.  Errors: INVALID_ARG (NULL plan), UNSUPPORTED (no kernel for
 * the plan's tile, input type and fix-up mode). */
int sk_plan_kernel_info(const sk_plan_t* plan, int32_t* threads, int32_t* lds_bytes, int32_t* variant);

void sk_plan_destroy(sk_plan_t* plan);

/* Measurement aid: the rate of the matrix-core instructions of the MAC loop (Sec. 2: the GEMM runs on
 * matrix cores) with nothing else in the way.  Enqueues one kernel on `stream` in which every wave of
 * `workgroups` workgroups (256 threads: one wave per SIMD) runs `iters` trips of 16 independent
 * register-resident matrix-core instructions of in_dtype (SK_BF16 / SK_F16: 32x32x16, SK_FP8_E4M3:
 * 32x32x64 with unit scales).  operands: device memory of sk_mfma_peak_operand_bytes() bytes in the
 * input type - its values are the operand values (random values and constant values reach different
 * clocks under the power limit); sink: device memory for workgroups * 256 floats (written once, keeps
 * the loop alive).  *flops (host, may be NULL) receives the floating-point operations of the launch;
 * the caller times the kernel.  Errors: INVALID_ARG, HIP. */
size_t sk_mfma_peak_operand_bytes(void);
int sk_mfma_peak_launch(int in_dtype, const void* operands, float* sink, int workgroups, int iters, void* stream, double* flops);

/* The tile shape the library picks for (M, N, K, in_dtype) when sk_config leaves
 * it zero.  out_blk: host int32[3] = blk_m, blk_n, blk_k. */
int sk_default_tile(int64_t M, int64_t N, int64_t K, int in_dtype, int32_t* out_blk);

/* The dispatcher's cost model applied to this plan: a rough time estimate in
 * microseconds (whole-tile waves, the evenly split Stream-K iterations, the
 * exchange of partial tiles: the chain of fetches of one owner plus the traffic
 * of all contributors together), from constants fitted on MI355X.  Meant for ranking
 * the policies of one problem when no tuning record knows it (the selector's
 * fall-back when the Bloom filters of Sec. 4.2 return no candidate), not for
 * predicting times.  microseconds: host double.
 * fp8 tiles are modelled as the 16-bit shape of the same byte footprint with half
 * the blk_k (same bytes and same matrix-core time per K-iteration).
 * Errors: INVALID_ARG (NULL), UNSUPPORTED (a tile shape the model has no constants
 * for: anything but the shapes sk_default_tile picks from). */
int sk_plan_estimate_us(const sk_plan_t* plan, double* microseconds);

/* ---- Bloom-filter policy selector (Sec. 4.2) --------------------------------
 * One filter per policy.  A record says which policies are winners for a
 * problem size; the size is inserted into the filter of each of them.  A query
 * returns the policies whose filter may contain the size: an inserted policy is
 * never missing from the answer (no false negatives).
 * Key: MurmurHash3 (32-bit) over M, N, K as three little-endian uint32; filter p
 * probes k bits with seeds p*k + i; bit j is bit (j % 64) of word (j / 64). */
typedef struct {
    uint32_t M, N, K;
    uint32_t policy_mask;   /* bit p set: policy p is a winner for this size */
} sk_bloom_record;

typedef struct {
    uint32_t m_bits;     /* bits per filter, multiple of 64; 0 = 95872 (10 000 sizes at ~1 %) */
    uint32_t k_probes;   /* probes per filter; 0 = 7                                          */
    uint32_t n_filters;  /* 0 = 7 (one per policy); at most 32                                */
} sk_bloom_params;

typedef struct sk_bloom_t sk_bloom_t;

/* The winner mask of one profiled problem size (Sec. 4.2: the winning configurations are inserted;
 * Sec. 5.2's tolerance thresholds widen "winning"): bit p of *mask_out is set iff policy p's time is
 * within tolerance of the fastest, times_ns[p] * 1000 <= min(times_ns) * (1000 + tol_permille), in
 * integers.  times_ns: host int64[n], 1 <= n <= 32, each in [0, 2^40].  Errors: INVALID_ARG. */
int bloom_winner_mask(const int64_t* times_ns, size_t n, uint32_t tol_permille, uint32_t* mask_out);

/* Build the filters from n records (host memory; n may be 0).  params may be NULL. */
int bloom_build(const sk_bloom_record* recs, size_t n, const sk_bloom_params* params, sk_bloom_t** out);

/* Insert one more record into existing filters. */
int bloom_insert(sk_bloom_t* bloom, const sk_bloom_record* rec);

/* Candidate policies for (M, N, K): bit p of *mask_out is set iff filter p holds all probe bits.
 * Sizes must fit uint32 (INVALID_ARG otherwise). */
int bloom_query(const sk_bloom_t* bloom, int64_t M, int64_t N, int64_t K, uint32_t* mask_out);

/* n queries at once: sizes is host uint32[3 * n] (M, N, K per query), masks_out host uint32[n]. */
int bloom_query_many(const sk_bloom_t* bloom, const uint32_t* sizes, size_t n, uint32_t* masks_out);

/* Read access to filter `filter`: *words points at library-owned 64-bit words, valid until
 * bloom_destroy; *n_words = m_bits / 64. */
int bloom_bits(const sk_bloom_t* bloom, int filter, const uint64_t** words, size_t* n_words);

/* The filters as a flat byte string and back: what a tuned library ships instead of its tuning
 * records (Sec. 4.2: the selector's table costs about one byte per profiled problem size - here
 * n_filters * m_bits / 8 bytes whatever the number of sizes, 84 KB by default).  Little-endian:
 * "SKBF", version 1, m_bits, k_probes, n_filters as uint32, then the 64-bit words of filter 0, 1, ...
 * bloom_serialize: *n_bytes receives the size of the string; buf (host memory of cap bytes) receives it;
 * (buf, cap) = (NULL, 0) asks for the size only; INVALID_ARG if cap is too small.
 * bloom_deserialize: builds new filters from such a string (bit for bit those that were serialised);
 * INVALID_ARG on a wrong magic, version, parameter or length. */
int bloom_serialize(const sk_bloom_t* bloom, void* buf, size_t cap, size_t* n_bytes);
int bloom_deserialize(const void* buf, size_t n_bytes, sk_bloom_t** out);

/* Key for problem sizes that were never profiled.  The filters of Sec. 4.2 are keyed by the exact
 * (M, N, K), so a size outside the profiled set matches nothing.  This key replaces the size by
 * what decides which schedule wins under the plan's tile shape and grid: the tile shape, the
 * number of full waves of tiles (capped at 3), how full the remainder wave is (in quarters of the
 * grid, rounded up), and floor(log2(iterations per tile)) (capped at 12).  Sizes that share a key
 * share their winners; records and queries are then made with key[0..2] in place of M, N, K.
 * key: host uint32[3]. */
int bloom_shape_key(const sk_plan_t* plan, uint32_t* key);

/* The hash itself (exported for known-answer tests). */
uint32_t bloom_murmur3_32(const void* key, size_t len, uint32_t seed);

void bloom_destroy(sk_bloom_t* bloom);

const char* sk_status_str(int status);

/* Text of the last HIP runtime error that made a call of this thread return SK_ERR_HIP. */
const char* sk_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* STREAMK_H */
