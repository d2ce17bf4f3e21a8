/*
 * gbmuf.h -- C ABI of libgbmuf: the random-gossip BMUF synchronisation step on one
 * AMD MI355X (gfx950), K worker replicas resident in that GPU's HBM.
 *
 * The operation is the synchronisation branch of Algorithm 1, "gossip-MA (gossip-BMUF)
 * for node k", of "A Random Gossip BMUF Process for Neural Language Modeling"
 * (arXiv 1909.09010), applied to all K nodes at once:
 *
 *   for every component i and worker w:
 *       choose q_i of w's ring neighbours at random          (Alg. 1, sync branch; Def. 1)
 *       avg   = (theta[w] + sum_j theta[k_j]) / (q_i+1)       (Alg. 1, averaging statement)
 *       G     = avg - theta_{t-H}[w]                          (Alg. 1, gossip-BMUF statements)
 *       Delta = eta*Delta + zeta*G
 *       omega = omega + Delta
 *       theta = omega + eta*Delta
 *
 * Conventions
 *   - Every call returns a status (GBMUF_OK = 0); results come back through pointers.
 *     No exception crosses this boundary.
 *   - "host" pointers are ordinary process memory; "device" pointers are HIP device
 *     memory of the GPU that was current when the plan was made.  The caller owns every
 *     buffer it passes; the library copies what it keeps.
 *   - A plan is immutable once made: every call takes it as const and none changes it, so
 *     host threads may share one.  (Device side, syncs of one plan that use its neighbour
 *     scratch must not be in flight at the same time; see gbmuf_sync.)
 *   - Where the state lives (two layouts, see gbmuf_state_t):
 *       rows     K rows of `worker_stride` floats per array (row w = worker w); the first
 *                P = comp_offsets[m] floats of a row are parameters, the rest is never
 *                touched.  This is what the calls without "_state" in their name take.
 *       blocked  every row is cut into blocks of B floats and the blocks with the same index
 *                of all workers (and, if the caller wishes, of all three arrays) sit next to
 *                each other, so that what one workgroup streams is one short address range.
 *                This is the fast layout on MI355X (see gbmuf_recommend_layout).
 *     Component i is elements [comp_offsets[i], comp_offsets[i+1]) of every worker.  No
 *     alignment is required; 16-byte aligned bases with strides that are multiples of 4
 *     floats take the 16-byte path, and rows (blocks) that start on multiples of 4 KB let
 *     every tile of the kernel cover whole cache lines.
 *   - All parameter arithmetic is IEEE binary32, round to nearest even, every multiply and
 *     add rounded separately (no fused multiply-add).  Sampling is integer only.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Device work is
 *     only ordered by that stream; no call synchronises the host except gbmuf_plan_create /
 *     gbmuf_plan (blocking uploads of the small tables) and gbmuf_plan_destroy.
 *   - On a machine without a GPU a plan can still be made and the host-side calls work;
 *     the device calls then return GBMUF_EDEVICE.
 */
#ifndef GBMUF_H
#define GBMUF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gbmuf_plan_s gbmuf_plan_t;   /* opaque; made and destroyed by the library */

enum {
    GBMUF_OK = 0,
    GBMUF_EINVAL = 1,      /* an argument is outside what the call accepts         */
    GBMUF_ENOMEM = 2,      /* host or device allocation failed                      */
    GBMUF_EDEVICE = 3,     /* no usable GPU, or a HIP call failed                   */
    GBMUF_EUNSUPPORTED = 4 /* valid by the paper, but beyond this library's limits */
};

/* How G and the restart are formed (Alg. 1, gossip-BMUF statements).  `nesterov` below. */
enum {
    GBMUF_MODE_NO_RESTART = 0, /* classical block momentum: theta' = omega', G = avg - omega   */
    GBMUF_MODE_PAPER = 1,      /* as printed: theta' = omega' + eta*Delta'; theta_{t-H} is what
                                  the previous restart wrote, omega + eta*Delta                */
    GBMUF_MODE_LITERAL = 2,    /* G = avg - omega while keeping the restart                    */
    GBMUF_MODE_GOSSIP_MA = 3   /* Alg. 1, gossip-MA branch: theta' = avg; omega/Delta unused   */
};

#define GBMUF_MAX_K 1024       /* workers per plan */

/* Where the neighbour rows of a sync are drawn (gbmuf_plan_desc_t.sampling). */
enum {
    GBMUF_SAMPLING_AUTO = 0,      /* in the fused kernel for small, launch-bound plans, else separate */
    GBMUF_SAMPLING_IN_KERNEL = 1, /* every workgroup draws its component's rows itself (one launch)  */
    GBMUF_SAMPLING_SEPARATE = 2   /* a sampler kernel fills a table first (two launches)            */
};

/* In which direction the fused kernel walks its tile list (gbmuf_plan_desc_t.sweep). */
enum {
    GBMUF_SWEEP_AUTO = 0,         /* even rounds forwards, odd rounds backwards: what a sync wrote
                                     last is read first by the next one, while still in cache      */
    GBMUF_SWEEP_FORWARD = 1       /* always forwards */
};

/*
 * Everything a plan is made from.  Zero the struct, set struct_size = sizeof(gbmuf_plan_desc_t)
 * and fill in what is needed; every field whose value is 0 / NULL takes the library's default.
 * (Section 2.2: theta = [theta_1 .. theta_m]; Definition 1: p-symmetric ring; Alg. 1 REQUIRE
 * lines: components, sync periods H_i, q <= 2p; Section 3.3: (p, q) per deployment.)
 */
typedef struct gbmuf_plan_desc {
    uint32_t struct_size;           /* sizeof(gbmuf_plan_desc_t) of the caller's header           */
    int32_t m;                      /* components, >= 0                                           */
    int32_t K;                      /* workers, 1 .. GBMUF_MAX_K                                  */
    int32_t q;                      /* neighbours drawn per component and sync, 0 <= q <= C;
                                       used for every component unless q_per_component is set     */
    const int64_t *comp_offsets;    /* host, m+1 element offsets: [0] = 0, non-decreasing (an
                                       empty component is allowed).  Copied.                      */
    const int32_t *q_per_component; /* host, m entries 0 <= q_i <= C, or NULL.  Copied.           */
    const int32_t *periods;         /* host, m sync periods H_i >= 1 for gbmuf_sync_step, or NULL
                                       (every component syncs at every step).  Copied.            */
    int32_t p;                      /* ring degree.  0 = the paper's rule p = log2(K) - 1 (floor,
                                       at least 1; Section 3.3); -1 = every other worker is a
                                       candidate.  Values above K-1 mean K-1 (the listing of
                                       Definition 1 is complete by then).                         */
    int32_t reserved0;
    uint64_t seed;                  /* sampler key; with `round` it fixes every neighbour table   */
    /* ---- tuning; none of these changes a result bit ---- */
    int32_t tile_threads;           /* threads per workgroup of the fused kernel: 256, 512, 1024  */
    int32_t tile_slots;             /* 16-byte slots per thread: 1, 2, 4, 8, 16.  Both 0 = chosen
                                       by K and layout; a pair that is not built in -> EINVAL     */
    int32_t sampling;               /* GBMUF_SAMPLING_*                                           */
    int32_t sweep;                  /* GBMUF_SWEEP_*                                              */
    int32_t cache_hints;            /* bit 0: non-temporal stores, bit 1: non-temporal loads      */
    int32_t workgroups_per_cu;      /* upper bound on the fused kernel's resident workgroups per
                                       compute unit (enforced through its LDS request); 0 = by
                                       layout: none for rows, a small number for blocked state    */
} gbmuf_plan_desc_t;

/* What a plan was made with (after defaults were resolved) and how it will run. */
typedef struct gbmuf_info {
    int32_t m, K;
    int32_t q;              /* neighbours per component; the largest q_i if they differ      */
    int32_t p;              /* ring degree actually used                                     */
    int32_t C;              /* ring candidates per worker = min(2p, K-1)                     */
    int32_t has_device;     /* 1 if device calls are available                               */
    int64_t P;              /* parameters per worker = comp_offsets[m]                       */
    int64_t n_tiles;        /* workgroups one sync of all components launches                */
    int32_t tile_columns;   /* 16-byte columns (4 floats) of one worker row per workgroup    */
    int32_t threads;        /* threads per workgroup of the fused kernel                     */
    uint64_t seed;
    int32_t mixed_q;        /* 1 if components draw different numbers of neighbours          */
    int32_t has_periods;    /* 1 if sync periods were given                                  */
    int32_t in_kernel_sampling; /* 1 if gbmuf_sync draws the rows inside the fused kernel    */
    int32_t tile_columns_blocked, threads_blocked;   /* the same for blocked state           */
    int32_t workgroups_per_cu_blocked;               /* resident workgroups per CU, blocked  */
    int32_t tile_columns_blocked_ma;  /* tile width of the gossip-MA branch on blocked state  */
    int32_t min_block_floats;         /* smallest gbmuf_state_t.block_floats this plan takes  */
} gbmuf_info_t;

/*
 * gbmuf_plan_create -- partition, topology, sampler key, neighbour counts and sync periods
 * for a series of syncs.
 * Errors: EINVAL (NULLs, struct_size too small, K < 1, m < 0, bad offsets, q or q_i < 0 or
 * > C, p < -1, H_i < 1, unknown enum or tile shape), EUNSUPPORTED (K > GBMUF_MAX_K, or the
 * neighbour rows of all workers do not fit on chip beside a tile), ENOMEM, EDEVICE (a GPU is
 * present but a HIP call failed).
 * If a GPU is present the plan allocates its small device tables (candidates, tile lists,
 * per-component table, neighbour scratch) on the current device; sync calls allocate nothing.
 */
int gbmuf_plan_create(gbmuf_plan_t **out, const gbmuf_plan_desc_t *desc);

/* The short form: one q for all components, no periods, default tuning. */
int gbmuf_plan(gbmuf_plan_t **out, const int64_t *comp_offsets, int32_t m, int32_t K,
               int32_t q, int32_t p, uint64_t seed);

/* Frees the plan and its device tables.  Synchronises the device first.  NULL is OK. */
int gbmuf_plan_destroy(gbmuf_plan_t *plan);

/* Copies the plan's resolved settings to *info. */
int gbmuf_plan_info(const gbmuf_plan_t *plan, gbmuf_info_t *info);

/*
 * Ring candidates of worker w in the order of Definition 1: (w-1)%K .. (w-p)%K,
 * (w+1)%K .. (w+p)%K, the worker itself and repeats dropped.  out_host has room for C
 * entries (gbmuf_info_t.C).
 */
int gbmuf_candidates_host(const gbmuf_plan_t *plan, int32_t w, int32_t *out_host);

/*
 * Neighbour table of sync number `round`: int32 [m][K][q] with q = gbmuf_info_t.q (the
 * largest q_i).  Row (i, w) holds the q_i ids worker w drew for component i, ascending, drawn
 * uniformly without replacement from the worker's candidates and independently for every
 * (component, worker, round) (Alg. 1, sync branch, first statement; Section 2.2, last
 * paragraph); entries beyond q_i are -1.  The host and the device version return the same
 * bits.  gbmuf_neighbours_device enqueues on `stream` and writes device memory out_dev.
 */
int gbmuf_neighbours_host(const gbmuf_plan_t *plan, uint64_t round, int32_t *out_host);
int gbmuf_neighbours_device(const gbmuf_plan_t *plan, uint64_t round, int32_t *out_dev,
                            void *stream);

/*
 * Where the three state arrays are.  Element e (0 <= e < P) of worker w of array X is the
 * float at
 *     X + w * worker_stride + e                                         if block_floats == 0
 *     X + (e / B) * block_stride + w * worker_stride + (e % B)          if block_floats == B > 0
 * rows:     worker_stride >= P.
 * blocked:  B a power of two, at least gbmuf_info_t.min_block_floats and at most 2^30;
 *           worker_stride >= B; block_stride >= (K-1) * worker_stride + B.  The last block
 *           of a row may be partly unused; those floats are never touched.
 * theta, omega, delta: device, in/out.  omega and delta may be NULL only with
 * GBMUF_MODE_GOSSIP_MA.  The floats the three arrays cover (rows: the P parameters of every row;
 * blocked: every block in full) must not overlap (checked: EINVAL).
 */
typedef struct gbmuf_state {
    float *theta;            /* the replicas                                   */
    float *omega;            /* per-worker "global model" slot                 */
    float *delta;            /* block-momentum slot                            */
    int64_t worker_stride;
    int64_t block_floats;
    int64_t block_stride;
} gbmuf_state_t;

/*
 * gbmuf_sync -- one synchronisation of all components of all K workers, in place, state in
 * rows.  (Alg. 1, the whole sync branch.)
 *   replicas  device, in/out: theta, K rows.
 *   global    device, in/out: omega (the per-worker "global model" slot), K rows.
 *   delta     device, in/out: Delta (block momentum slot), K rows.
 *             global and delta may be NULL only with GBMUF_MODE_GOSSIP_MA.
 *   worker_stride  floats between consecutive rows, >= P; the same for the three buffers.
 *   eta, zeta      block momentum and block learning rate.  In GBMUF_MODE_PAPER the call
 *                  assumes the previous sync used the same eta.
 *   nesterov       one of GBMUF_MODE_*.
 *   round          0-based sync counter; selects the neighbour table.
 * Every average uses the workers' values from before the call (snapshot semantics), the
 * sum runs over the worker and its neighbours in ascending worker id and is multiplied by
 * the rounded constant 1/(q_i+1).  The call enqueues one or two kernels on `stream` and
 * returns; it allocates nothing.  Two syncs on the same plan must not be in flight at the
 * same time on different streams unless the plan samples in the kernel (the sampler kernel
 * writes the plan's one neighbour scratch).
 * Errors: EINVAL (NULLs, worker_stride < P, unknown mode, overlapping arrays), EDEVICE.
 * gbmuf_sync_state is the same for any gbmuf_state_t.
 */
int gbmuf_sync(const gbmuf_plan_t *plan, float *replicas, float *global, float *delta,
               int64_t worker_stride, float eta, float zeta, int32_t nesterov,
               uint64_t round, void *stream);
int gbmuf_sync_state(const gbmuf_plan_t *plan, const gbmuf_state_t *state, float eta,
                     float zeta, int32_t nesterov, uint64_t round, void *stream);

/*
 * gbmuf_sync_static -- gbmuf_sync_state for callers that must not allocate or depend on
 * memory the plan allocated for the sync: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The neighbour table of the sync is drawn (always by the
 * sampler kernel) into a table that is part of the library's device image -- one array of
 * GBMUF_STATIC_TABLE_ENTRIES int32 (2 MiB) per GPU, held until the process ends -- instead of
 * the plan's scratch.  The call makes no allocation of any kind.  Limit: m * K * q (q = the
 * largest q_i) must not exceed GBMUF_STATIC_TABLE_ENTRIES, else GBMUF_EUNSUPPORTED (nothing
 * is launched; gbmuf_last_error_detail says how large the table would be).  All plans on one
 * GPU share that one table: calls of gbmuf_sync_static that are in flight at the same time on
 * the same GPU race, whichever plans and streams they use.  Results are bit-identical to
 * gbmuf_sync_state.
 */
#define GBMUF_STATIC_TABLE_ENTRIES (1 << 19)
int gbmuf_sync_static(const gbmuf_plan_t *plan, const gbmuf_state_t *state, float eta,
                      float zeta, int32_t nesterov, uint64_t round, void *stream);

/*
 * Same update with the neighbours given by the caller: nbr_dev is device memory,
 * int32 [m][K][q] (q = gbmuf_info_t.q; component i uses the first q_i entries of a row).
 * Rows need not be sorted; an id outside [0, K) is clamped into range, the result is then
 * unspecified but memory-safe.  A row should hold distinct ids different from the worker.
 * Used to check the arithmetic against enumerated tables.
 */
int gbmuf_sync_table(const gbmuf_plan_t *plan, const int32_t *nbr_dev, float *replicas,
                     float *global, float *delta, int64_t worker_stride, float eta,
                     float zeta, int32_t nesterov, void *stream);
int gbmuf_sync_table_state(const gbmuf_plan_t *plan, const int32_t *nbr_dev,
                           const gbmuf_state_t *state, float eta, float zeta,
                           int32_t nesterov, void *stream);

/*
 * gbmuf_sync_step -- gbmuf_sync for mini-batch counter `step` under the plan's sync periods
 * (Algorithm 1: component i takes the sync branch only when t mod H_i == 0; Section 3.3 uses
 * (16,128): embedding shards every 128 mini-batches, the rest every 16).  Only the
 * components with step mod H_i == 0 are sampled and updated, the others are neither read nor
 * written; the neighbour tables are those of round = step, so every sync of every component
 * draws fresh neighbours (Section 2.2, last paragraph).  A plan without periods syncs every
 * component: the call then equals gbmuf_sync(round = step).
 * When the components that are due form one run of consecutive components (the (16,128)
 * schedule does), the kernels are launched over exactly that run; otherwise one launch covers
 * all tiles and the workgroups of components that are not due return at once.
 */
int gbmuf_sync_step(const gbmuf_plan_t *plan, float *replicas, float *global, float *delta,
                    int64_t worker_stride, float eta, float zeta, int32_t nesterov,
                    uint64_t step, void *stream);
int gbmuf_sync_step_state(const gbmuf_plan_t *plan, const gbmuf_state_t *state, float eta,
                          float zeta, int32_t nesterov, uint64_t step, void *stream);

/*
 * Final model of Algorithm 1 (RETURN statement): out_dev[e] = (1/K) * sum_k replicas[k][e]
 * for e < P, summed in ascending worker id and multiplied by the rounded constant 1/K.
 * replicas: device, read only; out_dev: device, P contiguous floats, not overlapping the
 * replicas.  gbmuf_final_average_state reads state->theta in the state's layout (omega and
 * delta are ignored).
 */
int gbmuf_final_average(const gbmuf_plan_t *plan, const float *replicas, int64_t worker_stride,
                        float *out_dev, void *stream);
int gbmuf_final_average_state(const gbmuf_plan_t *plan, const gbmuf_state_t *state,
                              float *out_dev, void *stream);

/*
 * Placement advice for the three state arrays (host only, no GPU needed).  Both layouts
 * returned are ONE arena of arena_floats floats, exactly the state's size apart from padding
 * of the last block or row:
 *     state.theta = arena, state.omega = arena + omega_offset, state.delta = arena + delta_offset
 * GBMUF_LAYOUT_BLOCKED (recommended): blocks of block_floats floats; the blocks with one index
 *   lie together as [theta: K blocks | omega: K blocks | delta: K blocks], then the next index.
 *   The fused kernel then streams ONE moving address range instead of 3K, keeps few workgroups
 *   resident per compute unit so that this range stays short, and runs at the same speed
 *   wherever the driver placed the arena.
 * GBMUF_LAYOUT_ROWS: K groups [theta_w | omega_w | delta_w] of rows padded to 4 KB.  With rows
 *   the kernel streams 3K ranges; measured bandwidth then depends on the physical placement the
 *   allocation happens to get (about 61 % or 73 % of peak for a 53 GB state).
 * EINVAL for P < 0, K < 1, an unknown kind or NULL out; EINVAL too if plan is not NULL and its
 * K or P differ.  With a plan the block size suits that plan's tile shapes; with NULL it suits
 * the shapes the library picks by itself for any K (a plan made with very wide tiles may need larger
 * blocks: gbmuf_info_t.min_block_floats).
 */
enum { GBMUF_LAYOUT_ROWS = 0, GBMUF_LAYOUT_BLOCKED = 1 };
typedef struct gbmuf_layout {
    int64_t worker_stride;   /* gbmuf_state_t.worker_stride                       */
    int64_t block_floats;    /* gbmuf_state_t.block_floats (0 for rows)           */
    int64_t block_stride;    /* gbmuf_state_t.block_stride (0 for rows)           */
    int64_t omega_offset;    /* floats from the arena start to omega              */
    int64_t delta_offset;    /* floats from the arena start to delta              */
    int64_t arena_floats;    /* floats to allocate                                */
} gbmuf_layout_t;
int gbmuf_recommend_layout(const gbmuf_plan_t *plan, int64_t P, int32_t K, int32_t kind,
                           gbmuf_layout_t *out);

/*
 * Copies the parameters (elements e < P of every worker) of the arrays selected by `which`
 * (bit 0 theta, bit 1 omega, bit 2 delta) from one placement to another, e.g. rows -> blocked
 * before a series of syncs and back afterwards.  Both states are device memory; a selected
 * array must be non-NULL in both and the two states must not overlap.  Enqueues on `stream`.
 */
int gbmuf_state_copy(const gbmuf_plan_t *plan, const gbmuf_state_t *dst, const gbmuf_state_t *src,
                     int32_t which, void *stream);

/*
 * Calibration probe, not part of the method: a plain streaming copy of n_floats floats
 * (a multiple of 4; both pointers device memory, 16-byte aligned, not overlapping) with
 * one read and one write per byte.  It gives hardware byte counters a launch of known
 * traffic (4 * n_floats bytes read, 4 * n_floats written) and shows the bandwidth a 1:1 read/write
 * stream reaches on the device.  flags: bit 0 = streaming stores, bit 1 = streaming loads.
 */
int gbmuf_probe_copy(float *dst_dev, const float *src_dev, int64_t n_floats, int32_t flags,
                     void *stream);

/* Static description of a status code. */
const char *gbmuf_strerror(int code);

/* Name and HIP error text of the most recent HIP call that failed inside the library on the
 * calling thread ("" if none); a diagnostic aid, valid until that thread's next failure. */
const char *gbmuf_last_error_detail(void);

#ifdef __cplusplus
}
#endif
#endif /* GBMUF_H */
