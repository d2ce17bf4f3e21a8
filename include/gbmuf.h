/*
 * gbmuf.h -- C ABI of libgbmuf: the random-gossip BMUF synchronisation step on one
 * AMD MI355X (gfx950), K worker replicas resident in that GPU's HBM.
 *
 * The operation is the synchronisation branch of Algorithm 1, "gossip-MA (gossip-BMUF)
 * for node k", of "A Random Gossip BMUF Process for Neural Language Modeling"
 * (arXiv 1909.09010), applied to all K nodes at once:
 *
 *   for every component i and worker w:
 *       choose q of w's ring neighbours at random            (Alg. 1, sync branch; Def. 1)
 *       avg   = (theta[w] + sum_j theta[k_j]) / (q+1)         (Alg. 1, averaging statement)
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
 *   - Parameter buffers are K rows of `worker_stride` floats (row w = worker w); the first
 *     P = comp_offsets[m] floats of a row are parameters, the rest is never touched.
 *     Component i is elements [comp_offsets[i], comp_offsets[i+1]).  No alignment is
 *     required; 16-byte aligned bases with worker_stride % 4 == 0 take the 16-byte path, and
 *     bases and strides that are multiples of 1 KB (4 KB to be safe) let every tile of the
 *     kernel cover whole cache lines, which is worth about a quarter of the bandwidth.
 *   - All parameter arithmetic is IEEE binary32, round to nearest even, every multiply and
 *     add rounded separately (no fused multiply-add).  Sampling is integer only.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Device work is
 *     only ordered by that stream; no call synchronises the host except where stated.
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

/* What a plan was made with (after defaults were resolved) and how it will run. */
typedef struct gbmuf_info {
    int32_t m, K, q;
    int32_t p;              /* ring degree actually used                                  */
    int32_t C;              /* ring candidates per worker = min(2p, K-1)                  */
    int32_t has_device;     /* 1 if device calls are available                            */
    int64_t P;              /* parameters per worker = comp_offsets[m]                    */
    int64_t n_tiles;        /* workgroups one sync launches                               */
    int32_t tile_columns;   /* 16-byte columns (4 floats) of one worker row per workgroup */
    int32_t threads;        /* threads per workgroup of the fused kernel                  */
    uint64_t seed;
} gbmuf_info_t;

/*
 * gbmuf_plan -- partition, topology and sampler key for a series of syncs.
 * (Section 2.2: theta = [theta_1 .. theta_m]; Definition 1: p-symmetric ring; Alg. 1
 * REQUIRE lines: components, q <= 2p.)
 *   out           receives the plan; destroy it with gbmuf_plan_destroy.
 *   comp_offsets  host, m+1 entries, element offsets: [0] = 0, non-decreasing (an empty
 *                 component is allowed).  Copied.
 *   m, K          components (>= 0) and workers (1 .. GBMUF_MAX_K).
 *   q             neighbours drawn per component and sync, 0 <= q <= C.
 *   p             ring degree.  0 = the paper's rule p = log2(K) - 1 (floor, at least 1;
 *                 Section 3.3); -1 = floor(K/2): every other worker is a candidate.
 *   seed          sampler key; with `round` it fixes every neighbour table.
 * Errors: EINVAL (NULLs, K < 1, m < 0, bad offsets, q < 0 or q > C, p < -1),
 * EUNSUPPORTED (K > GBMUF_MAX_K, or K*(q+1) too large for the on-chip neighbour rows),
 * ENOMEM, EDEVICE (a GPU is present but a HIP call failed).
 * If a GPU is present the plan allocates its small device tables (candidates, tile list,
 * neighbour scratch) on the current device; sync calls allocate nothing.
 */
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
 * Neighbour table of sync number `round`: int32 [m][K][q], each row ascending, drawn
 * uniformly without replacement from the worker's candidates, independently for every
 * (component, worker, round) (Alg. 1 "randomly choose q neighbors"; Section 2.2, last
 * paragraph).  The host and the device version return the same bits.
 * gbmuf_neighbours_device enqueues on `stream` and writes device memory out_dev.
 */
int gbmuf_neighbours_host(const gbmuf_plan_t *plan, uint64_t round, int32_t *out_host);
int gbmuf_neighbours_device(const gbmuf_plan_t *plan, uint64_t round, int32_t *out_dev,
                            void *stream);

/*
 * gbmuf_sync -- one synchronisation of all components of all K workers, in place.
 * (Alg. 1, the whole sync branch.)
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
 * the rounded constant 1/(q+1).  The three buffers must not overlap.  The call enqueues
 * one or two kernels on `stream` and returns; it allocates nothing.  Two syncs on the same
 * plan must not run concurrently on different streams (large plans draw the neighbour table
 * into the plan's scratch with a separate kernel; small, launch-bound plans draw it inside
 * the fused kernel and use no scratch).  Errors: EINVAL (NULLs, worker_stride < P, unknown mode), EDEVICE.
 */
int gbmuf_sync(const gbmuf_plan_t *plan, float *replicas, float *global, float *delta,
               int64_t worker_stride, float eta, float zeta, int32_t nesterov,
               uint64_t round, void *stream);

/*
 * Same update with the neighbours given by the caller: nbr_dev is device memory,
 * int32 [m][K][q], ids in [0, K) (rows need not be sorted; an id outside [0, K) is clamped
 * into range, the result is then unspecified but memory-safe).  A row should hold distinct
 * ids different from the worker.  Used to check the arithmetic against enumerated tables.
 */
int gbmuf_sync_table(const gbmuf_plan_t *plan, const int32_t *nbr_dev, float *replicas,
                     float *global, float *delta, int64_t worker_stride, float eta,
                     float zeta, int32_t nesterov, void *stream);

/*
 * Per-component synchronisation periods (Algorithm 1: component i takes the sync branch only
 * when t mod H_i == 0; Section 3.3 uses (16,128): embedding shards every 128 mini-batches,
 * the rest every 16).
 * gbmuf_plan_set_periods stores H_i >= 1 for the m components (host array, copied; NULL
 * clears them, i.e. every component syncs).  It synchronises the device and must not run
 * concurrently with syncs on the same plan.  EINVAL for NULL plan or H_i < 1.
 * gbmuf_sync_step is gbmuf_sync for mini-batch counter `step`: only the components with
 * step mod H_i == 0 are updated, the others are not read or written; the neighbour tables
 * are those of round = step, so every sync of every component draws fresh neighbours
 * (Section 2.2, last paragraph).  Without periods it equals gbmuf_sync(round = step).
 * Contiguous runs of active components are launched as ranges of the tile list (up to 8
 * runs); a more scattered schedule takes one launch that checks the period on the device.
 */
int gbmuf_plan_set_periods(gbmuf_plan_t *plan, const int32_t *periods_host);
int gbmuf_sync_step(const gbmuf_plan_t *plan, float *replicas, float *global, float *delta,
                    int64_t worker_stride, float eta, float zeta, int32_t nesterov,
                    uint64_t step, void *stream);

/*
 * Final model of Algorithm 1 (RETURN statement): out_dev[e] = (1/K) * sum_k replicas[k][e]
 * for e < P, summed in ascending worker id and multiplied by the rounded constant 1/K.
 * replicas: device, K rows of worker_stride floats (read only); out_dev: device, P floats.
 * 16-byte aligned pointers with worker_stride % 4 == 0 take 16-byte loads.
 */
int gbmuf_final_average(const gbmuf_plan_t *plan, const float *replicas, int64_t worker_stride,
                        float *out_dev, void *stream);

/*
 * Placement advice for the three state buffers (host only, no GPU needed).  The ABI takes
 * three base pointers and one row stride, so rows may be placed anywhere; on MI355X the
 * sync kernel is measurably faster (about 62 % -> 75 % of peak HBM bandwidth) when the 3K
 * rows it streams concurrently are spread over much more than ~70 GB of HBM instead of
 * sitting side by side.  The layout returned is ONE arena of arena_floats floats holding
 * [theta_w | omega_w | delta_w | gap] for w = 0..K-1:
 *     theta = arena, omega = arena + omega_offset, delta = arena + delta_offset,
 *     row w of each at + w * worker_stride.
 * span_bytes is the HBM the K rows should cover (e.g. 150e9 on a 288 GB device); the stride
 * is never smaller than three padded rows, so span_bytes = 0 gives the dense interleaving.
 * Rows are padded to a multiple of 1024 floats (4 KB) and so is the stride: with rows on
 * 4 KB boundaries the kernel's tiles cover whole cache lines.
 * EINVAL for P < 0, K < 1, span_bytes < 0 or NULL out.
 */
typedef struct gbmuf_layout {
    int64_t worker_stride;   /* floats between consecutive workers' rows          */
    int64_t omega_offset;    /* floats from the arena start to omega's first row  */
    int64_t delta_offset;    /* floats from the arena start to delta's first row  */
    int64_t arena_floats;    /* floats to allocate                                */
} gbmuf_layout_t;
int gbmuf_recommend_layout(int64_t P, int32_t K, int64_t span_bytes, gbmuf_layout_t *out);

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
