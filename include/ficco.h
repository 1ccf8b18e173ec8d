/*
 * ficco.h - C ABI of the finer-grain compute/communication overlap path on one MI355X (gfx950).
 *
 * The operation (paper Sec. II-B, Fig. 3(a)-(b)): a GPU holds a column share W [K,N] of a weight
 * and needs the row-gathered activation A = [I_0; ...; I_{G-1}] (G shards of M/G rows, [M/G,K])
 * to compute C = A * W. Serial execution gathers first and multiplies afterwards; shard-level
 * overlap (Fig. 3(c)) multiplies shard j while shard j+1 is in flight; the finer-grain scheme
 * (Sec. III, Sec. V-A/B) cuts every shard once more into `chunks` row pieces, moves piece s of
 * every shard in step s, and multiplies pieces as they land. The mirror direction streams row
 * blocks of C = A * W out to G peer buffers as they are completed (the data-movement half of
 * GEMM -> reduce-scatter; ficco_rs_reduce() is the receiving GPU's adding half). Also here: the
 * paper's 2D (k-sliced) decomposition, the fused schedule with explicit Gather/Scatter copies, and
 * an expert-parallel dispatch followed by a grouped expert GEMM (ficco_plan_grouped()).
 *
 * On one GPU the transfers are copy-engine (SDMA) copies, from pinned host memory or from a device
 * staging buffer that stands for the peers' memory: driven directly, one engine per emulated link
 * (the default), or issued with hipMemcpyAsync on the caller's copy stream. The GEMM is a
 * hand-written bf16 MFMA kernel (fp32 accumulate, one round-to-nearest-even to bf16 at the end)
 * launched per group of landed pieces, or once as a resident kernel whose tiles wait (bounded) for
 * their own piece: on the transfer's completion signal or on a ready flag in device memory
 * (Sec. VI-A uses stream write/wait between kernels for the same purpose).
 *
 * Conventions
 *   - All matrices are row-major bf16 (1-8-7). "device" = hipMalloc'ed memory of the current
 *     device; "host" = ordinary host memory; "pinned" = hipHostMalloc'ed host memory.
 *   - Streams are hipStream_t passed as void*. Every call uses the device that is current on the
 *     calling thread; a plan must be used on the device it was created on. The copy-engine
 *     backend keeps one process-wide context, set up by the first run that uses it: runs on
 *     another device of the same process return FICCO_ERR_ARG, and that first run must not race
 *     with another thread's.
 *   - Every function returns 0 (FICCO_OK) or a negative ficco_status; nothing throws or aborts.
 *     On failure output arguments are left untouched.
 *   - The caller owns every data buffer and both streams. The plan owns its flags, events,
 *     tables, packed weight and statistics. A plan is not thread safe; runs of one plan are
 *     ordered by the streams they are enqueued on, and at most one run of a plan may be in
 *     flight per pair of streams.
 *   - Result bits do not depend on schedule, chunk count, arrival order, tile shape or source
 *     kind: every output element is accumulated over k in the same order by the same
 *     instruction sequence.
 */
#ifndef FICCO_H
#define FICCO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ficco_plan_s ficco_plan_t;   /* opaque, library-owned */

typedef enum ficco_status {
    FICCO_OK          = 0,
    FICCO_ERR_ARG     = -1,   /* null pointer, unknown enum value, option set too late        */
    FICCO_ERR_SHAPE   = -2,   /* shape rule violated (see ficco_plan)                         */
    FICCO_ERR_ALLOC   = -3,   /* host or device allocation failed                             */
    FICCO_ERR_HIP     = -4,   /* a HIP call failed; ficco_last_hip_error() has the code       */
    FICCO_ERR_TIMEOUT = -5,   /* a kernel's bounded wait for a piece expired (or a transfer never completed) */
    FICCO_ERR_STATE   = -6    /* call not valid in the plan's state (e.g. stats before a run) */
} ficco_status;

/* Schedules (Sec. II-B, Sec. V-A/B). */
typedef enum ficco_schedule {
    FICCO_SERIAL          = 0,   /* all G shard transfers, then one GEMM (Fig. 3(b)); chunks must be 1 */
    FICCO_SHARD           = 1,   /* one GEMM per landed shard (Fig. 3(c)); chunks must be 1            */
    FICCO_FINE_UNFUSED    = 2,   /* G*chunks pieces, one GEMM launch per landed piece ("unfused")       */
    FICCO_FINE_FUSED      = 3,   /* one GEMM launch per step over the G pieces of that step ("fused");
                                    the kernel reads the pieces in place through a row-block table,
                                    so no Gather/Scatter copies are issued                             */
    FICCO_FINE_PERSISTENT = 4,   /* one resident kernel; every tile waits on its piece's ready flag.
                                    In the GEMM -> RS direction the kernel itself releases a piece's
                                    transfer when the piece's last tile has been stored (engine
                                    backend, FICCO_MODE_PAIR or FICCO_MODE_GEMM_ONLY, no
                                    FICCO_OPT_TIMING; N % 8 == 0 and C_dev 16-byte aligned)           */
    FICCO_FINE_2D         = 5,   /* column pieces (the 2D decomposition of Sec. V-A/B, chosen by the
                                    paper's rule when M <= K): the k range is cut into `chunks` slices,
                                    step s moves slice s of every shard, and one resident kernel adds
                                    slice s into its accumulators as it lands, so the partial products
                                    of the paper's accumulating GEMMs never leave the registers. The
                                    activation lands K-sliced in A_dev (see ficco_run); A_src is the
                                    caller's row-major matrix unless FICCO_OPT_SOURCE_LAYOUT says the
                                    sender holds it K-sliced already. AG_GEMM only, no
                                    FICCO_OPT_LOCAL_SHARD; FICCO_AUTO keeps to row pieces             */
    FICCO_AUTO            = 100, /* ficco_pick_schedule() decides schedule and chunks (Sec. V-C)        */
    FICCO_AUTO_ANY        = 101  /* ficco_pick_schedule_any() decides: the answer may be FICCO_FINE_2D,
                                    cut by ficco_pick_slice_widths() (ficco_plan_info() and
                                    ficco_plan_slices() say what was chosen). A_src stays row-major; the
                                    landing buffer A_dev is then K-sliced                            */
} ficco_schedule;

typedef enum ficco_direction {
    FICCO_DIR_AG_GEMM = 0,       /* transfers feed the GEMM                                   */
    FICCO_DIR_GEMM_RS = 1        /* the GEMM feeds transfers of C row blocks to peer buffers  */
} ficco_direction;

typedef enum ficco_order {
    FICCO_ORDER_STEP_MAJOR  = 0, /* step s moves piece s of every shard (all-to-all pattern, Sec. III-B) */
    FICCO_ORDER_SHARD_MAJOR = 1, /* all pieces of shard 0, then shard 1, ...                              */
    FICCO_ORDER_CUSTOM      = 2  /* set by ficco_plan_set_arrival()                                       */
} ficco_order;

typedef enum ficco_mode {
    FICCO_MODE_PAIR        = 0,  /* the dependent pair (default)                                        */
    FICCO_MODE_GEMM_ONLY   = 1,  /* only the plan's GEMM launches, operands resident (isolated, Sec. IV-B) */
    FICCO_MODE_COPY_ONLY   = 2,  /* only the plan's transfers (isolated)                                 */
    FICCO_MODE_INDEPENDENT = 3   /* both, concurrently, with no dependency between them (Sec. IV-C)      */
} ficco_mode;

/* Options for ficco_plan_set(). */
typedef enum ficco_option {
    FICCO_OPT_DIRECTION   = 0,   /* ficco_direction; default AG_GEMM                                    */
    FICCO_OPT_ORDER       = 1,   /* ficco_order; default STEP_MAJOR for the FINE schedules              */
    FICCO_OPT_MODE        = 2,   /* ficco_mode; default PAIR                                            */
    FICCO_OPT_TIMING      = 3,   /* 0: begin/end events only (default); 1: also per-piece and per-launch
                                    events (adds one barrier packet around every launch)                */
    FICCO_OPT_TILE        = 4,   /* 0: choose by shape (default); else a ficco_tile value               */
    FICCO_OPT_FLAG_WRITE  = 5,   /* how a waiting kernel learns that a piece has landed. 0 (default): the
                                    engine backend lets kernels read the transfers' completion signals
                                    where it can, else a 4-byte copy behind the transfer raises a flag
                                    (the stream backend always copies a flag); 1: hipStreamWriteValue32
                                    raises the flag (stream backend only); 2: always a flag copy      */
    FICCO_OPT_SPIN_LIMIT_US = 6, /* resident kernel: give up after this long without the awaited flag
                                    (default 2,000,000); the run then reports FICCO_ERR_TIMEOUT        */
    FICCO_OPT_LOCAL_SHARD = 7,   /* -1 (default): every shard arrives by transfer. j >= 0: shard j is
                                    already in A_dev and is multiplied first without waiting
                                    ("hetero" start, Sec. V-A); its transfers are skipped              */
    FICCO_OPT_HOLD_FLAGS  = 8,   /* test hook: 1 = issue the transfers but never write the ready flags,
                                    so that the kernels' bounded wait expires                          */
    FICCO_OPT_COPY_BACKEND = 9,  /* ficco_copy_backend; default AUTO                                    */
    FICCO_OPT_LINKS       = 10,  /* copy-engine backend: number of copy engines used side by side, one
                                    per emulated link (shard j travels on engine j mod links);
                                    0 (default) = min(shards, engines available)                        */
    FICCO_OPT_PACKING     = 11,  /* 1: run FICCO_FINE_FUSED the way an unmodified library GEMM forces it
                                    (Sec. V-A): every landed piece is copied by DMA into its place in a
                                    contiguous per-step input (Gather), one launch multiplies the step,
                                    and its G output blocks are copied by DMA to their rows of C
                                    (Scatter). AG_GEMM and the copy-engine backend only; applies to
                                    FICCO_MODE_PAIR runs (the other modes measure the plain parts);
                                    ficco_run() then waits on the host for each launch before it
                                    submits that launch's Scatter copies. 0 (default): the kernel
                                    reads the pieces in place through a row-block table             */
    FICCO_OPT_REPEAT      = 12,  /* measuring aid, 1..10000 (default 1): a FICCO_MODE_GEMM_ONLY run without
                                    FICCO_OPT_TIMING on the stream path enqueues its GEMM launches this many
                                    times back to back between its two events; wall_us then covers all of
                                    them and n_launches counts them. May change between runs.         */
    FICCO_OPT_TILE_GROUP  = 13,  /* tile order, row tiles per group: 0 (default) = chosen per launch from the
                                    shape, else 1, 2, 4 or 8. The order decides which tiles share an XCD's L2
                                    at a time; it never changes a result bit.                         */
    FICCO_OPT_TILE_COLUMN_LISTS = 14, /* resident kernels: column blocks their eight tile lists are split into:
                                    0 (default) = chosen from the shape, else 1, 2, 4 or 8 (at most the
                                    number of column tiles, otherwise the run fails with FICCO_ERR_ARG)   */
    FICCO_OPT_SOURCE_LAYOUT = 15 /* ficco_source_layout of A_src for FICCO_FINE_2D plans; default ROW_MAJOR       */
} ficco_option;

/*
 * How the far side holds the activation when column pieces travel (FICCO_FINE_2D; Sec. V-A/B, 2D decomposition).
 *   ROW_MAJOR - A_src is the caller's ordinary [M,K] row-major matrix, shard after shard, as for every other
 *               schedule. A column piece is then a strided rectangle ([M/G rows] x [width] at pitch K). From
 *               pinned host memory it is moved as such by a copy engine (a rectangular engine copy; measured
 *               47-53 GB/s for rows of 2-6 KB, the rate of the host link). From device memory the runtime
 *               puts every rectangular copy on one engine (56 GB/s in total, no links side by side), so the
 *               sending side re-lays its shards out instead, inside the run: a kernel on the compute stream
 *               writes each column piece as one contiguous block into a staging buffer the plan owns (M*K
 *               elements) and, piece by piece, releases that piece's transfer, which then travels on its
 *               link's engine like any other piece. On a real node every GPU would do this for the one shard
 *               it sends; here the one GPU does it for all G senders, and the step pays for all of it.
 *   K_SLICED  - the sender already holds its slices as DMA-ready blocks: A_src is K-sliced like A_dev (see
 *               ficco_run). Nothing is re-laid out.
 * A_dev is K-sliced in both cases.
 */
typedef enum ficco_source_layout {
    FICCO_LAYOUT_ROW_MAJOR = 0,
    FICCO_LAYOUT_K_SLICED  = 1,
    FICCO_LAYOUT_ROW_MAJOR_HOST = 2  /* for ficco_pick_schedule_layout only: ROW_MAJOR, and the caller says that the
                                        shards lie in pinned host memory (ficco_run itself sees where A_src lives) */
} ficco_source_layout;

/*
 * How transfers are issued.
 *   STREAM  - hipMemcpyAsync on the caller's copy stream. From pinned host memory this is one
 *             copy-engine queue over the host link. From device memory the HIP runtime would
 *             use a copy *kernel*, so AUTO never picks STREAM for device sources or peers.
 *   ENGINES - the ROCr copy-on-engine call (hsa_amd_memory_async_copy_on_engine) with the copy
 *             forced onto SDMA engines, several side by side: transfers of different shards run
 *             concurrently like the links of a fully connected node (Sec. III-B/C), and with
 *             FICCO_SHARD or FICCO_ORDER_SHARD_MAJOR they are chained one after the other like
 *             peer-to-peer exchange over one link at a time (Fig. 3(c)). GEMM launches wait for
 *             their pieces inside the kernel: they read the value word of the transfer's own
 *             completion signal, or - when the transfers cross the host link, when the signals
 *             are not readable from the GPU, or with FICCO_OPT_FLAG_WRITE = 2 - a ready flag
 *             raised by a 4-byte copy queued on the same engine behind the transfer.
 *             The copy stream argument is not used. ficco_run() first waits on the host
 *             for the plan's previous run; in the GEMM->RS direction it also waits for each GEMM
 *             launch before it submits that launch's transfers - except with
 *             FICCO_FINE_PERSISTENT, where all transfers are submitted up front, each behind a
 *             dependency signal that the resident kernel clears from the GPU.
 *             Links are mapped to every second engine id first: engines with neighbouring ids
 *             share a path and slow each other down when they copy at the same time.
 *   AUTO    - ENGINES for every run that moves data, unless FICCO_OPT_FLAG_WRITE = 1 asks for
 *             stream writes or a GEMM_RS run sends every block to pinned host memory (then
 *             STREAM); measured faster than STREAM for pinned sources too.
 *             (On STREAM the resident kernel leaves 8 CUs free: the HIP runtime writes the
 *             4-byte flags with a helper kernel.)
 */
typedef enum ficco_copy_backend {
    FICCO_COPY_AUTO    = 0,
    FICCO_COPY_STREAM  = 1,
    FICCO_COPY_ENGINES = 2
} ficco_copy_backend;

typedef enum ficco_tile {        /* workgroup tile (rows x columns of C); the k order is the same in all */
    FICCO_TILE_AUTO    = 0,
    FICCO_TILE_256x256 = 1,
    FICCO_TILE_128x128 = 2,
    FICCO_TILE_256x128 = 3,
    FICCO_TILE_128x256 = 4,
    FICCO_TILE_64x256  = 5,      /* for pieces of fewer than 128 rows */
    FICCO_TILE_32x256  = 6,      /* for pieces of fewer than 64 rows  */
    FICCO_TILE_128x128_DEEP = 7, /* 128x128 with a four-stage LDS ring, one workgroup per CU: for launches
                                    that do not fill the machine */
    FICCO_TILE_128x192 = 8,      /* for N a multiple of 192 but not of 256 (e.g. 768) */
    FICCO_TILE_256x192 = 9
} ficco_tile;

typedef struct ficco_plan_info {
    int64_t M, K, N;
    int32_t shards, chunks;          /* chunks = pieces per shard                                */
    int32_t schedule, direction, order, mode;
    int32_t n_chunks;                /* shards * chunks                                          */
    int32_t n_groups;                /* GEMM launches per run                                    */
    int64_t chunk_rows;              /* rows of one piece (M / n_chunks; M / shards for FICCO_FINE_2D; 0 for
                                        grouped plans, whose pieces differ: see ficco_plan_pieces)   */
    int32_t tile_m, tile_n, tile_k;  /* chosen workgroup tile                                    */
    int32_t resident_grid;           /* workgroups of the resident kernel (0 if not used)        */
    int32_t copy_backend, links;     /* as resolved by the last run (0 before the first run)     */
    double  otb;                     /* static op-to-byte of one launch's GEMM (Sec. IV-B)       */
    double  mt_bytes;                /* static memory traffic MK+NK+MN of it, in bytes (Sec. IV-C) */
} ficco_plan_info_t;

typedef struct ficco_stats {
    double  wall_us;          /* first transfer (or first launch) start -> last operation end           */
    double  copy_span_us;     /* first transfer start -> last transfer end (0 if no transfers)          */
    double  gemm_span_us;     /* first GEMM launch start -> last GEMM launch end                        */
    double  gemm_busy_us;     /* sum of per-launch kernel durations (TIMING=1), else = gemm_span_us     */
    double  copy_busy_us;     /* sum of per-transfer durations (TIMING=1), else = copy_span_us          */
    double  exposed_comm_us;  /* wall_us - gemm_busy_us                                                 */
    double  eff_tflops;       /* 2*M*N*K / wall_us                                                      */
    double  copy_gbps;        /* transferred bytes / copy_span_us                                       */
    int64_t flops;            /* 2*M*N*K                                                                */
    int64_t copy_bytes;       /* bytes moved by transfers in this run                                   */
    int32_t n_copies, n_launches;
    int32_t timed_out;        /* 1 if a kernel's bounded wait for a piece expired                       */
    int32_t run_index;        /* 1 for the first run of the plan                                        */
} ficco_stats_t;

typedef struct ficco_losses {       /* Sec. IV: measured on this GPU with this plan's decomposition    */
    double t_gemm_whole_us;         /* one GEMM over all M rows, isolated: span of 8 launches back to back / 8,
                                       after 40 ms of the same launches have settled the clocks           */
    double t_gemm_pieces_us;        /* the plan's GEMM launches, isolated, taken the same way (span: dispatch gaps
                                       between a decomposed schedule's launches count as decomposition cost) */
    double t_gemm_pieces_cont_us;   /* span of the same launches, one run per bracket, while the plan's transfers run
                                       independently                                                     */
    double t_copy_whole_us;         /* G shard-sized transfers, isolated                                */
    double t_copy_pieces_us;        /* the plan's transfers, isolated                                   */
    double t_copy_pieces_cont_us;   /* the plan's transfers while the GEMM launches run independently   */
    double gemm_dil, gemm_cil;      /* t_gemm_pieces_us / t_gemm_whole_us; t_gemm_pieces_cont_us / t_gemm_pieces_single_us */
    double comm_dil, comm_cil;      /* pieces / whole; contended / isolated                             */
    double ideal_us;                /* ideal-overlap time from the whole-operator times (Sec. IV-A)     */
    double t_gemm_pieces_single_us; /* span of the plan's launches, isolated, one run per bracket (CIL's denominator) */
    double t_gemm_pieces_busy_us;   /* sum of the launches' own durations (an event before and after each launch;
                                       for a resident schedule the one launch's)                       */
} ficco_losses_t;

/*
 * Build a plan for C[M,N] = A[M,K] * W[K,N] with A arriving as `shards` row shards, each cut into
 * `chunks` pieces (Sec. III-A). Validates and builds the arrival list and the launch groups for
 * the current device; the tile is chosen and flags/events/tables are allocated on first use
 * (ficco_pack_weight or ficco_run), after which most options are frozen.
 * Shape rules (FICCO_ERR_SHAPE otherwise): M, K, N >= 1; shards >= 1; chunks >= 1;
 * M % (shards*chunks) == 0; K % 64 == 0 and K <= 2^22; N % 8 == 0; chunks == 1 for SERIAL and SHARD;
 * shards*chunks <= 4096. FICCO_FINE_2D instead needs M % shards == 0 and chunks <= K/64; its
 * slices are as equal as whole k-tiles of 64 columns allow (the first (K/64) mod chunks slices
 * one k-tile wider) unless ficco_plan_set_slice_widths gives other widths.
 * With FICCO_AUTO and FICCO_AUTO_ANY, `chunks` is ignored and chosen by the heuristic.
 */
int ficco_plan(int64_t M, int64_t K, int64_t N, int shards, int chunks, int schedule,
               ficco_plan_t **out);

/*
 * Plan for an expert-parallel dispatch followed by the expert layers' GEMM (the all-to-all of
 * Sec. II-A; the amounts differ per pair of GPUs, Sec. III-C): this GPU hosts `experts` experts with
 * weights W_e [K,N]; peer j sends rows[j*experts + e] >= 0 token rows for expert e. Every (peer, expert)
 * block is cut into `chunks` pieces as equal as integers allow (the first T mod chunks one row longer).
 * Piece (e, s, j) has id (e*chunks + s)*peers + j; rows are laid out in id order, i.e. expert-major,
 * then step, then peer (ficco_plan_pieces() reports first row and row count of every piece), in
 * A_src, A_dev [M,K] and C_dev [M,N] alike, M = the sum of `rows`; W_dev is [experts][K][N].
 * C row r = A row r times the weight of the expert whose segment holds r.
 * Schedules: FICCO_SERIAL (every tile waits for every transfer), FICCO_SHARD (whole blocks, one
 * peer after the other, a tile waits for its own blocks), FICCO_FINE_PERSISTENT (step s moves
 * piece s of every peer over all links; FICCO_ORDER_SHARD_MAJOR: peer by peer). One resident
 * grouped kernel in all three; transfers on the copy engines, peer j on link j; ficco_run() as for
 * the all-gather direction (peer_out NULL). Not available: GEMM_RS, LOCAL_SHARD, PACKING, TIMING,
 * the stream backend, ficco_profile_losses, graphs.
 * Shape rules: K % 64 == 0, K <= 2^22, N % 8 == 0, peers*experts*chunks <= 4096, 1 <= M < 2^31, chunks == 1
 * for SERIAL and SHARD.
 */
int ficco_plan_grouped(int64_t K, int64_t N, int peers, int experts, const int64_t *rows, int chunks,
                       int schedule, ficco_plan_t **out);

/* First row and row count of every piece, by piece id (host arrays of at least n_chunks entries,
 * either may be NULL). For ordinary plans all pieces have chunk_rows rows. */
int ficco_plan_pieces(const ficco_plan_t *plan, int64_t *row0, int64_t *rows, int cap);

/*
 * Column pieces of unequal width for a FICCO_FINE_2D plan (Sec. V-A cuts the k range evenly; with
 * the overlap model of Sec. IV-A what stays exposed is the wait for the first piece when the GEMM
 * is the longer side and the GEMM of the last piece when the transfers are, so a narrow first or
 * last slice shortens it at no cost in transfer count). widths[s] = columns of slice s, s < n;
 * n must equal the plan's `chunks`, every width a positive multiple of 64, their sum K
 * (FICCO_ERR_SHAPE otherwise). Slice s then holds columns [k0_s, k0_s + widths[s]) of every row
 * as an [M][widths[s]] row-major block, the blocks following each other in A_src and A_dev.
 * widths == NULL (n ignored) restores equal slices. Only before the plan's first use
 * (FICCO_ERR_STATE afterwards); FICCO_ERR_ARG for other schedules. The result bits do not change.
 */
int ficco_plan_set_slice_widths(ficco_plan_t *plan, const int64_t *widths, int n);

/* First column and width of every slice of a FICCO_FINE_2D plan (host arrays of at least `chunks`
 * entries, either may be NULL; `cap` is their length). FICCO_ERR_ARG for other schedules. */
int ficco_plan_slices(const ficco_plan_t *plan, int64_t *k0, int64_t *widths, int cap);

/*
 * Chain `plan` behind `after` for callers that keep the GPU fed without waiting on the host between
 * steps (layer after layer of a model, a serving loop): from now on the transfers of every
 * ficco_run(plan) start only when the latest ficco_run(after) enqueued before it has finished on
 * the device, so the two plans may share A_dev while the host runs one step ahead. Two plans
 * chained behind each other and run in turn give back-to-back steps with no host round trip in
 * between: a run of a plan only waits (on the host) for that same plan's previous run. Runs of
 * `after` release the dependency when they end (from the resident kernel's last workgroup, or from
 * a one-thread kernel on the compute stream). Both
 * plans must run on the same compute stream and on the copy-engine backend, and `plan` in the
 * all-gather direction (ficco_run returns FICCO_ERR_ARG otherwise). `after` == NULL removes the
 * dependency. A plan cannot be chained behind itself (FICCO_ERR_ARG). Either plan may be
 * destroyed first; transfers parked behind a destroyed plan are let go. ficco_rs_reduce and
 * graph launches take no part in it.
 */
int ficco_plan_chain(ficco_plan_t *plan, ficco_plan_t *after);

/* Set an option; only before the plan's first use (FICCO_ERR_STATE afterwards), except
 * FICCO_OPT_MODE, FICCO_OPT_TIMING, FICCO_OPT_SPIN_LIMIT_US, FICCO_OPT_HOLD_FLAGS, FICCO_OPT_REPEAT,
 * FICCO_OPT_TILE_GROUP and FICCO_OPT_TILE_COLUMN_LISTS, which may change between runs. */
int ficco_plan_set(ficco_plan_t *plan, int option, int64_t value);

/* Replace the arrival order by a permutation of 0..n_chunks-1 (tests: reversed, shuffled).
 * Launch groups are rebuilt over the new order. Only before the first run. */
int ficco_plan_set_arrival(ficco_plan_t *plan, const int32_t *chunk_ids, int n);

int ficco_plan_info(const ficco_plan_t *plan, ficco_plan_info_t *out);

/* Arrival list: chunk_ids[p] = chunk issued p-th (chunk i = piece i%chunks of shard i/chunks,
 * rows [i*chunk_rows, (i+1)*chunk_rows); with FICCO_FINE_2D chunk i = k slice i/shards of shard
 * i%shards); group_ids[p] = index of the GEMM launch that consumes it. Both host arrays of at
 * least n_chunks entries; `cap` is their length. */
int ficco_plan_arrival(const ficco_plan_t *plan, int32_t *chunk_ids, int32_t *group_ids, int cap);

/*
 * Pack the static weight W_dev ([K,N] row-major, device) into the plan's kernel layout
 * ([N,K], k contiguous) on `stream`. ficco_run() does this by itself the first time it sees a
 * W_dev pointer; call it again whenever the *contents* of W change. Not part of the timed path:
 * the weight share is resident and static across calls (Sec. II-B).
 */
int ficco_pack_weight(ficco_plan_t *plan, const void *W_dev, void *stream);

/*
 * Enqueue one run of the plan. The stream backend only enqueues. On the engine backend the call
 * first waits for this plan's previous run, whose signals the host re-arms (ficco_plan_chain gives
 * back-to-back steps without that wait), and then returns without waiting for the device, with
 * two exceptions in which the host relays kernel completions to the engines and the call returns
 * when the last launch has finished: GEMM_RS with the per-launch schedules, and
 * FICCO_OPT_PACKING (GEMM_RS with FICCO_FINE_PERSISTENT keeps the host out of the loop).
 *   AG_GEMM : A_src  - the G shards, contiguous ([M,K] bf16), pinned host or device memory;
 *                      piece i is copied to the same rows of A_dev on copy_stream (may be NULL in
 *                      FICCO_MODE_GEMM_ONLY).
 *             A_dev  - [M,K] device; written by the transfers, read by the GEMM.
 *             C_dev  - [M,N] device; written by the GEMM.
 *             peer_out must be NULL.
 *             FICCO_FINE_2D: A_dev is K-sliced: slice s holds its columns of every row as an
 *             [M][width_s] row-major block, block after block ([chunks][M][K/chunks] when K/64 is a
 *             multiple of chunks; ficco_plan_slices reports the slices), so that piece s*shards + j
 *             (slice s of shard j) lands as one contiguous block. A_src is row-major like for every
 *             other schedule, or K-sliced like A_dev with FICCO_OPT_SOURCE_LAYOUT = K_SLICED (see
 *             ficco_source_layout for how the pieces leave a row-major source; on the stream
 *             backend only K_SLICED sources are accepted). In FICCO_MODE_GEMM_ONLY A_dev must
 *             already hold the K-sliced matrix. C is bitwise what FICCO_SERIAL computes from the
 *             same matrix.
 *   GEMM_RS : A_src must be NULL; A_dev is read; C_dev is written by the GEMM and its row block
 *             p (rows [p*M/G, (p+1)*M/G)) is then copied (on copy_stream, or by the engines) to
 *             peer_out[p] ([M/G, N] bf16 each, device or pinned host), piece by piece as pieces
 *             complete.
 *             peer_out is a host array of `shards` pointers.
 *   W_dev   - [K,N] device (see ficco_pack_weight).
 * compute_stream and copy_stream must differ and have the default priority. On the stream backend
 * with a resident schedule they must also not share a hardware queue (HIP maps streams round-robin
 * onto GPU_MAX_HW_QUEUES queues, so create few streams): otherwise the flag writes sit behind the
 * kernel that waits for them and the run ends with FICCO_ERR_TIMEOUT. The engine backend (the
 * default) does not use copy_stream and has no such constraint.
 */
int ficco_run(ficco_plan_t *plan, const void *A_src, void *A_dev, const void *W_dev, void *C_dev,
              void *const *peer_out, void *compute_stream, void *copy_stream);

/*
 * Receiver side of a true reduce-scatter (the paper leaves it out because a DMA engine cannot add,
 * Sec. IV-E): this GPU owns row block `block` of the output; every other GPU j sends its partial block.
 *   P_src  - [shards][M/shards][N] bf16, the peers' partial blocks where they come from (device
 *            staging or pinned host memory; slot `block` is never read)
 *   P_dev  - [shards][M/shards][N] bf16 device landing buffer, written by the transfers (slot `block`
 *            is not touched)
 *   own    - [M/shards][N] bf16 device, this GPU's own partial block (for instance rows
 *            [block*M/shards, ...) of the C_dev a GEMM_RS run produced earlier on `stream`)
 *   out    - [M/shards][N] bf16 device: out[i][j] = bf16_rne(x_0[i][j] + x_1[i][j] + ... ), the sum
 *            taken in fp32 in ascending GPU order with x_block = own and the others from P_dev
 * A block travels in `chunks` row pieces per peer, in the plan's arrival order and pattern (all
 * links side by side in step-major order; one transfer after the other for FICCO_SHARD and
 * FICCO_ORDER_SHARD_MAJOR), on the copy engines; one reduction launch is enqueued first on `stream`
 * and every tile waits (bounded, as in ficco_run) for the pieces it adds. With FICCO_SERIAL or
 * chunks = 1 a tile needs every transfer, which is the serial "receive, then add" execution.
 * ficco_query_stats() reports wall time, copy spans, and flops = the additions made. Not for
 * FICCO_FINE_2D plans; FICCO_OPT_COPY_BACKEND must not be STREAM.
 */
int ficco_rs_reduce(ficco_plan_t *plan, int block, const void *P_src, void *P_dev, const void *own,
                    void *out, void *stream);

/*
 * Capture one run of the plan into a HIP graph (the paper notes the cost of enqueueing many small
 * operations, Sec. IV-A; a graph replays the whole run with one call). For the per-launch schedules
 * (SERIAL, SHARD, FINE_UNFUSED, FINE_FUSED) in FICCO_MODE_PAIR on the stream backend, with the far
 * side (A_src, or every peer_out[j]) in pinned host memory; FICCO_OPT_TIMING must be 0 and
 * FICCO_OPT_COPY_BACKEND must not be ENGINES (FICCO_ERR_ARG otherwise). Arguments as in ficco_run();
 * the pointers are baked into the graph. The weight is packed before the capture if needed. The
 * graph holds copies, kernel launches and their dependencies only: no memset nodes.
 * ficco_graph_launch() enqueues one replay on `stream` (any stream; replays on one stream run in
 * order) and returns at once; ficco_query_stats() then reports wall time, flops and the captured
 * counts (the span fields are 0). A new capture replaces the old graph. FICCO_ERR_STATE if no
 * graph has been captured.
 * Measured on ROCm 7.2 / MI355X: the runtime executes a replay's host-to-device copy nodes with its
 * copy kernel instead of an SDMA engine, and replays of the decomposed schedules were slower than
 * the same runs enqueued call by call; prefer ficco_run() unless a capturable path is required.
 */
int ficco_graph_capture(ficco_plan_t *plan, const void *A_src, void *A_dev, const void *W_dev,
                        void *C_dev, void *const *peer_out);
int ficco_graph_launch(ficco_plan_t *plan, void *stream);

/* Block until the plan's last run has completed, then report its timings (Sec. IV-A quantities
 * are in ficco_profile_losses). FICCO_ERR_TIMEOUT (with *out filled) if the resident kernel's
 * bounded wait expired; FICCO_ERR_STATE if the plan has not run. */
int ficco_query_stats(ficco_plan_t *plan, ficco_stats_t *out);

/* Per-piece and per-launch spans of the last run, microseconds from the run's start
 * (FICCO_OPT_TIMING=1; FICCO_ERR_STATE otherwise). copy_* have n_chunks entries in arrival
 * order, gemm_* have n_groups entries; any pointer may be NULL. */
int ficco_query_spans(ficco_plan_t *plan, double *copy_begin_us, double *copy_end_us, int cap_chunks,
                      double *gemm_begin_us, double *gemm_end_us, int cap_groups);

/*
 * Measure decomposition and contention losses for this plan's decomposition (Sec. IV-A..C):
 * runs the isolated, decomposed and independent-concurrent modes `warmup`+`iters` times each
 * and averages (the paper uses 10 and 5). Synchronous. AG_GEMM plans only.
 */
int ficco_profile_losses(ficco_plan_t *plan, const void *A_src, void *A_dev, const void *W_dev,
                         void *C_dev, void *compute_stream, void *copy_stream,
                         int warmup, int iters, ficco_losses_t *out);

/*
 * Static schedule heuristic (Sec. V-C): from (M, K, N, shards) alone pick a schedule and a
 * piece count. Host-only arithmetic; thresholds are constants fitted on MI355X.
 */
int ficco_pick_schedule(int64_t M, int64_t K, int64_t N, int shards, int *schedule, int *chunks);

/* The same rule for the GEMM -> reduce-scatter direction (FICCO_OPT_DIRECTION = FICCO_DIR_GEMM_RS; data movement,
 * Sec. IV-E): a link carries (M/shards) x N output elements instead of (M/shards) x K of the activation. Answers
 * the resident schedule and the pieces per output block; the caller builds the plan with them. Meant for peer
 * buffers in device memory: towards pinned host memory every schedule is bound by the host link and the per-launch
 * schedules on the stream backend were the fastest measured. */
int ficco_pick_schedule_rs(int64_t M, int64_t K, int64_t N, int shards, int *schedule, int *chunks);

/* The same with column pieces allowed - the choice of communication shape of Sec. V-C, decided here by whether
 * the output is about one round of tiles over the machine: may also answer FICCO_FINE_2D, with the number of
 * slices in *chunks. ficco_pick_schedule_any answers for the caller's row-major A_src (what a FICCO_AUTO_ANY
 * plan uses): the step then pays for the sender-side re-layout, so column pieces are only picked where the GEMM
 * is the longer side and large enough to hide it. ficco_pick_schedule_layout takes the ficco_source_layout: for
 * a sender that holds its slices K-sliced already, column pieces are picked for every small output; for row-major
 * shards in pinned host memory (ROW_MAJOR_HOST) never: all their strided rectangles travel through one engine, and
 * row pieces were ahead at every shape tried. A FICCO_AUTO_ANY plan cannot know where the shards will lie and assumes
 * device memory (peers' memory, the paper's case): a caller with host-resident shards asks here first. */
int ficco_pick_schedule_any(int64_t M, int64_t K, int64_t N, int shards, int *schedule, int *chunks);
int ficco_pick_schedule_layout(int64_t M, int64_t K, int64_t N, int shards, int source_layout, int *schedule, int *chunks);

/* The cut of the k range that goes with a FICCO_FINE_2D answer: widths[0..slices) for
 * ficco_plan_set_slice_widths (a FICCO_AUTO_ANY plan has them applied already). Two slices of a
 * transfer-bound shape (N*shards <= 8192) are cut three quarters to one quarter, in whole k-tiles,
 * so that little GEMM is left when the last byte lands (the overlap model of Sec. IV-A); everything
 * else is cut as evenly as k-tiles allow. FICCO_ERR_ARG unless K is a multiple of 64 with at least
 * `slices` k-tiles. */
int ficco_pick_slice_widths(int64_t M, int64_t K, int64_t N, int shards, int slices, int64_t *widths);

/* Static descriptors of an (m, N, K) bf16 GEMM: op-to-byte (Sec. IV-B) and memory traffic in
 * bytes (Sec. IV-C). Host-only. */
int ficco_static_descriptors(int64_t m, int64_t N, int64_t K, double *otb, double *mt_bytes);

/* Ideal-overlap time (Sec. IV-A): n pieces, times scale exactly with the split. Host-only. */
double ficco_ideal_overlap_us(double t_comm_us, double t_gemm_us, int n);

/*
 * For callers that cannot allocate device memory - code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc: C_dev[M,N] = A_dev[M,K] * W_dev[K,N] with every operand already in
 * device memory, by the resident kernel, enqueued on `stream` (hipStream_t). It is what ficco_run()
 * does for a FICCO_FINE_PERSISTENT plan of one shard and one piece in FICCO_MODE_GEMM_ONLY, with the
 * same tile and tile order, so the result is the same bit for bit; but no plan is needed and the call
 * makes no device allocation, now or later: the kernel's ticket counters, its status word, its arrival
 * table and the packed copy of the weight ([N,K], rewritten by every call) live in one fixed array in
 * the library's device image, of FICCO_STATIC_MAX_WEIGHT_BYTES + 4096 bytes, which every GPU the
 * library runs on holds until the process ends. The call clears what must start at zero with a small
 * kernel (no memset node is recorded if the stream is being captured), packs the weight and launches
 * the GEMM, three kernels on `stream`, and returns without waiting.
 * Shape rules: M, K, N >= 1, K % 64 == 0, N % 8 == 0, M and N below 2^31, K at most 2^22, and K*N*2 bytes at most
 * FICCO_STATIC_MAX_WEIGHT_BYTES (FICCO_ERR_SHAPE otherwise; e.g. K = 4096 with N up to 1024).
 * All calls on one GPU share that GPU's array: two calls whose kernels overlap on one GPU (different
 * streams, or the same call from two threads) race; calls on one stream are ordered and safe. The
 * caller owns A_dev, W_dev and C_dev. FICCO_ERR_ARG for a null or non-device pointer.
 */
#define FICCO_STATIC_MAX_WEIGHT_BYTES (8u << 20)
int ficco_gemm_static(int64_t M, int64_t K, int64_t N, const void *A_dev, const void *W_dev, void *C_dev,
                      void *stream);

void ficco_destroy(ficco_plan_t *plan);      /* waits for the plan's runs, frees what it owns */

const char *ficco_strerror(int status);
int ficco_last_hip_error(void);              /* hipError_t of the last failed HIP call on this thread */
const char *ficco_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FICCO_H */
