// gbmuf_plan.hip -- host half of libgbmuf: plan construction (partition, ring topology,
// tile list), the host sampler, argument checks and the C entry points of include/gbmuf.h.
#include "gbmuf_internal.h"

#include "../../include/gbmuf.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

using namespace gbmuf;

struct gbmuf_plan_s {
    int32_t m = 0, K = 0, q = 0, p = 0, C = 0;
    uint64_t seed = 0;
    int64_t P = 0;
    std::vector<int64_t> off;        // m+1 component offsets
    std::vector<int32_t> cand;       // [K][C] ring candidates, order of Definition 1
    std::vector<TileDesc> tiles;     // work list of the fused kernel, in component order
    std::vector<int64_t> tile_start; // m+1: first tile of every component
    std::vector<int32_t> periods;    // per-component sync period H_i (empty: all 1)
    Variant variant{256, 8};
    int32_t logT = 0;
    float inv = 1.0f;                // 1/(q+1), rounded once
    int32_t flags = 0;               // load/store cache hints of the fused kernel
    bool inline_sampling = false;    // workgroups draw their own neighbour rows (no sampler launch)
    bool alternate = true;           // odd rounds walk the tile list backwards (see tile_of_block)

    bool has_device = false;
    int device = -1;
    int32_t *d_cand = nullptr;
    TileDesc *d_tiles = nullptr;
    int32_t *d_nbr = nullptr;        // neighbour scratch of gbmuf_sync, [m][K][q]
    int32_t *d_periods = nullptr;    // m entries, valid when periods is not empty
};

namespace gbmuf {
static thread_local char g_detail[256] = "";
int hip_failed(const char *what, hipError_t err, int status)
{
    std::snprintf(g_detail, sizeof(g_detail), "%s: %s (%d)", what, hipGetErrorString(err), static_cast<int>(err));
    return status;
}
}  // namespace gbmuf

namespace {

// Section 3.3: p = log2(n) - 1, here floor(log2 K) - 1 and at least 1.
int32_t default_degree(int32_t K)
{
    int32_t lg = 0;
    while ((static_cast<int64_t>(2) << lg) <= K) ++lg;
    return lg - 1 > 1 ? lg - 1 : 1;
}

// Definition 1: (w-1)%K .. (w-p)%K, then (w+1)%K .. (w+p)%K; first occurrence kept, w dropped.
void ring_of(int32_t w, int32_t K, int32_t p, std::vector<int32_t> &out)
{
    out.clear();
    std::vector<char> taken(static_cast<size_t>(K), 0);
    taken[static_cast<size_t>(w)] = 1;
    for (int dir = -1; dir <= 1; dir += 2)
        for (int32_t d = 1; d <= p; ++d) {
            int64_t v = (static_cast<int64_t>(w) + static_cast<int64_t>(dir) * d) % K;
            if (v < 0) v += K;
            if (!taken[static_cast<size_t>(v)]) {
                taken[static_cast<size_t>(v)] = 1;
                out.push_back(static_cast<int32_t>(v));
            }
        }
}

struct HostPerm {
    int32_t *base;
    int32_t &operator()(int32_t x) const { return base[x]; }
};

// Tile shape.  Measured on MI355X (large states, HBM-spanning layout): short tiles of about
// 32 columns (512 B per worker row) with few 16-byte slots per thread run fastest, 75-77 % of
// peak; K > 32 needs 1024 threads to keep the columns that wide.  GBMUF_VARIANT overrides.
const Variant &choose_variant(int K)
{
    int count = 0;
    const Variant *tab = variant_table(&count);
    const int want_threads = K <= 32 ? 256 : 1024;
    const int want_slots = K <= 8 ? 1 : K <= 16 ? 2 : 4;
    int pick = 0;
    for (int i = 0; i < count; ++i)
        if (tab[i].threads == want_threads && tab[i].slots == want_slots) pick = i;
    if (const char *s = std::getenv("GBMUF_VARIANT")) {
        const int v = std::atoi(s);
        if (v >= 0 && v < count) pick = v;
    }
    return tab[pick];
}

// Split every component into runs of at most T 16-byte columns (the fused kernel's work list).
void build_tiles(gbmuf_plan_s &pl)
{
    const int64_t T = static_cast<int64_t>(1) << pl.logT;
    pl.tiles.clear();
    pl.tile_start.assign(static_cast<size_t>(pl.m) + 1, 0);
    for (int32_t i = 0; i < pl.m; ++i) {
        const int64_t a = pl.off[static_cast<size_t>(i)], b = pl.off[static_cast<size_t>(i) + 1];
        pl.tile_start[static_cast<size_t>(i)] = static_cast<int64_t>(pl.tiles.size());
        pl.tile_start[static_cast<size_t>(i) + 1] = static_cast<int64_t>(pl.tiles.size());
        if (a >= b) continue;
        // Tile boundaries sit at multiples of T columns counted from the row start, not from the
        // component start: with rows aligned to T*16 bytes every interior tile then covers whole
        // cache lines (a component that starts mid-line only gets a short first tile).  Tiles
        // that straddle lines cost a quarter of the bandwidth on MI355X.
        const int64_t ga = a >> 2, gb = (b + 3) >> 2;
        for (int64_t g = ga; g < gb;) {
            int64_t next = (g / T + 1) * T;
            if (next > gb) next = gb;
            const int64_t lo = (g << 2) > a ? (g << 2) : a;
            const int64_t end = (next << 2) < b ? (next << 2) : b;
            pl.tiles.push_back(TileDesc{lo, static_cast<int32_t>(end - lo), i});
            g = next;
        }
        pl.tile_start[static_cast<size_t>(i) + 1] = static_cast<int64_t>(pl.tiles.size());
    }
}

void free_device(gbmuf_plan_s &pl)
{
    if (pl.d_cand) (void)hipFree(pl.d_cand);
    if (pl.d_tiles) (void)hipFree(pl.d_tiles);
    if (pl.d_nbr) (void)hipFree(pl.d_nbr);
    if (pl.d_periods) (void)hipFree(pl.d_periods);
    pl.d_cand = nullptr; pl.d_tiles = nullptr; pl.d_nbr = nullptr; pl.d_periods = nullptr;
}

template <class T>
int upload(T **dst, const std::vector<T> &src)
{
    const size_t bytes = (src.empty() ? 1 : src.size()) * sizeof(T);
    hipError_t err = hipMalloc(reinterpret_cast<void **>(dst), bytes);
    if (err != hipSuccess) { *dst = nullptr; return hip_failed("hipMalloc(plan table)", err, GBMUF_ENOMEM); }
    if (!src.empty()) {
        err = hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice);
        if (err != hipSuccess) return hip_failed("hipMemcpy(plan table)", err, GBMUF_EDEVICE);
    }
    return GBMUF_OK;
}

int make_device_state(gbmuf_plan_s &pl)
{
    int ndev = 0;
    hipError_t err = hipGetDeviceCount(&ndev);
    if (err != hipSuccess || ndev < 1) {
        hip_failed("hipGetDeviceCount", err, GBMUF_OK);
        (void)hipGetLastError();
        return GBMUF_OK;                                   // host-only plan
    }
    err = hipGetDevice(&pl.device);
    if (err != hipSuccess) return hip_failed("hipGetDevice", err, GBMUF_EDEVICE);
    int rc = prepare_kernels(pl.variant, pl.K, pl.q, pl.C, &pl.inline_sampling);
    // Drawing the rows inside every workgroup saves the sampler launch (about 2 us of a 8 us
    // sync on a 200k-parameter model) but costs about 2 % once there are millions of tiles:
    // only launch-bound plans do it.  GBMUF_TWO_KERNELS / GBMUF_ONE_KERNEL force either way.
    if (pl.tiles.size() > 8192 || std::getenv("GBMUF_TWO_KERNELS")) pl.inline_sampling = false;
    if (std::getenv("GBMUF_ONE_KERNEL")) {
        bool can = false;
        rc = prepare_kernels(pl.variant, pl.K, pl.q, pl.C, &can);
        pl.inline_sampling = can;
    }
    if (rc != GBMUF_OK) return rc;
    if ((rc = upload(&pl.d_cand, pl.cand)) != GBMUF_OK) return rc;
    if ((rc = upload(&pl.d_tiles, pl.tiles)) != GBMUF_OK) return rc;
    const size_t n = static_cast<size_t>(pl.m) * pl.K * pl.q;
    err = hipMalloc(reinterpret_cast<void **>(&pl.d_nbr), (n ? n : 1) * sizeof(int32_t));
    if (err != hipSuccess) {
        pl.d_nbr = nullptr;
        return hip_failed("hipMalloc(neighbour scratch)", err, GBMUF_ENOMEM);
    }
    err = hipMalloc(reinterpret_cast<void **>(&pl.d_periods), (pl.m ? pl.m : 1) * sizeof(int32_t));
    if (err != hipSuccess) {
        pl.d_periods = nullptr;
        return hip_failed("hipMalloc(periods)", err, GBMUF_ENOMEM);
    }
    pl.has_device = true;
    return GBMUF_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int enqueue_sync(const gbmuf_plan_s *pl, const int32_t *nbr_dev, float *theta, float *omega, float *delta,
                 int64_t stride, float eta, float zeta, int32_t mode, hipStream_t stream,
                 int64_t first_tile = 0, int64_t n_tiles = -1, bool check_periods = false, uint64_t step = 0,
                 uint64_t round = 0)
{
    if (n_tiles < 0) n_tiles = static_cast<int64_t>(pl->tiles.size());
    SyncArgs a{};
    a.tiles = pl->d_tiles + first_tile;
    a.cand = pl->d_cand;                                    // used only when nbr_dev == nullptr
    a.C = pl->C;
    a.key0 = static_cast<uint32_t>(pl->seed); a.key1 = static_cast<uint32_t>(pl->seed >> 32);
    a.round0 = static_cast<uint32_t>(round); a.round1 = static_cast<uint32_t>(round >> 32);
    a.periods = check_periods ? pl->d_periods : nullptr;
    a.step = step;
    a.nbr = nbr_dev;
    a.theta = theta; a.omega = omega; a.delta = delta;
    a.stride = stride;
    a.K = pl->K; a.q = pl->q; a.logT = pl->logT; a.mode = mode;
    a.eta = eta; a.zeta = zeta; a.inv = pl->inv;
    a.flags = pl->flags | ((pl->alternate && (round & 1)) ? 8 : 0);
    bool vec4 = aligned16(theta) && (stride % 4 == 0);
    if (mode != GBMUF_MODE_GOSSIP_MA) vec4 = vec4 && aligned16(omega) && aligned16(delta);
    return launch_sync(pl->variant, vec4, a, n_tiles, stream);
}

// Device calls need the plan's GPU to be the current one: its tables live there.
int check_device(const gbmuf_plan_s *pl)
{
    if (!pl->has_device) return GBMUF_EDEVICE;
    int dev = -1;
    const hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return hip_failed("hipGetDevice", err, GBMUF_EDEVICE);
    if (dev != pl->device) return hip_failed("current device is not the plan's device", hipErrorInvalidDevice, GBMUF_EDEVICE);
    return GBMUF_OK;
}

int check_sync(const gbmuf_plan_s *pl, const float *theta, const float *omega, const float *delta,
               int64_t stride, int32_t mode)
{
    if (!pl || !theta) return GBMUF_EINVAL;
    if (mode < GBMUF_MODE_NO_RESTART || mode > GBMUF_MODE_GOSSIP_MA) return GBMUF_EINVAL;
    if (mode != GBMUF_MODE_GOSSIP_MA && (!omega || !delta)) return GBMUF_EINVAL;
    if (stride < pl->P) return GBMUF_EINVAL;
    return check_device(pl);
}

SampleArgs sample_args(const gbmuf_plan_s *pl, uint64_t round, int32_t *out)
{
    SampleArgs s{};
    s.cand = pl->d_cand;
    s.out = out;
    s.pairs = static_cast<int64_t>(pl->m) * pl->K;
    s.K = pl->K; s.C = pl->C; s.q = pl->q;
    s.key0 = static_cast<uint32_t>(pl->seed); s.key1 = static_cast<uint32_t>(pl->seed >> 32);
    s.round0 = static_cast<uint32_t>(round); s.round1 = static_cast<uint32_t>(round >> 32);
    return s;
}

}  // namespace

extern "C" {

int gbmuf_plan(gbmuf_plan_t **out, const int64_t *comp_offsets, int32_t m, int32_t K, int32_t q, int32_t p,
               uint64_t seed)
{
    if (!out) return GBMUF_EINVAL;
    *out = nullptr;
    if (!comp_offsets || m < 0 || K < 1 || q < 0 || p < -1) return GBMUF_EINVAL;
    if (comp_offsets[0] != 0) return GBMUF_EINVAL;
    for (int32_t i = 0; i < m; ++i)
        if (comp_offsets[i + 1] < comp_offsets[i]) return GBMUF_EINVAL;
    if (K > GBMUF_MAX_K) return GBMUF_EUNSUPPORTED;

    gbmuf_plan_s *pl = new (std::nothrow) gbmuf_plan_s;
    if (!pl) return GBMUF_ENOMEM;
    int rc = GBMUF_OK;
    try {
        pl->m = m; pl->K = K; pl->q = q; pl->seed = seed;
        pl->p = p == 0 ? default_degree(K) : (p < 0 ? K / 2 : p);
        pl->off.assign(comp_offsets, comp_offsets + m + 1);
        pl->P = pl->off.back();
        pl->inv = 1.0f / static_cast<float>(q + 1);

        std::vector<int32_t> ring;
        ring_of(0, K, pl->p, ring);
        pl->C = static_cast<int32_t>(ring.size());
        if (q > pl->C) rc = GBMUF_EINVAL;                  // the paper requires q <= 2p
        if (rc == GBMUF_OK) {
            pl->cand.resize(static_cast<size_t>(K) * pl->C);
            for (int32_t w = 0; w < K; ++w) {
                ring_of(w, K, pl->p, ring);
                if (pl->C > 0)
                    std::memcpy(pl->cand.data() + static_cast<size_t>(w) * pl->C, ring.data(),
                                sizeof(int32_t) * static_cast<size_t>(pl->C));
            }
            pl->variant = choose_variant(K);
            if (const char *f = std::getenv("GBMUF_FLAGS")) pl->flags = std::atoi(f) & 3;
            pl->alternate = std::getenv("GBMUF_NO_ALTERNATE") == nullptr;   // tuning switch
            const int slots = pl->variant.threads * pl->variant.slots;
            if (K > slots) rc = GBMUF_EUNSUPPORTED;
            int lg = 0;
            while (rc == GBMUF_OK && (static_cast<int64_t>(K) << (lg + 1)) <= slots) ++lg;
            pl->logT = lg;                                 // T = largest power of two with K*T <= slots
            if (rc == GBMUF_OK) build_tiles(*pl);
            if (rc == GBMUF_OK) rc = make_device_state(*pl);
        }
    } catch (const std::bad_alloc &) {
        rc = GBMUF_ENOMEM;
    }
    if (rc != GBMUF_OK) {
        free_device(*pl);
        delete pl;
        return rc;
    }
    *out = pl;
    return GBMUF_OK;
}

int gbmuf_plan_destroy(gbmuf_plan_t *plan)
{
    if (!plan) return GBMUF_OK;
    int rc = GBMUF_OK;
    if (plan->has_device) {
        if (hipDeviceSynchronize() != hipSuccess) rc = GBMUF_EDEVICE;
        free_device(*plan);
    }
    delete plan;
    return rc;
}

int gbmuf_plan_info(const gbmuf_plan_t *plan, gbmuf_info_t *info)
{
    if (!plan || !info) return GBMUF_EINVAL;
    info->m = plan->m; info->K = plan->K; info->q = plan->q; info->p = plan->p; info->C = plan->C;
    info->has_device = plan->has_device ? 1 : 0;
    info->P = plan->P;
    info->n_tiles = static_cast<int64_t>(plan->tiles.size());
    info->tile_columns = 1 << plan->logT;
    info->threads = plan->variant.threads;
    info->seed = plan->seed;
    return GBMUF_OK;
}

int gbmuf_candidates_host(const gbmuf_plan_t *plan, int32_t w, int32_t *out_host)
{
    if (!plan || w < 0 || w >= plan->K || (!out_host && plan->C > 0)) return GBMUF_EINVAL;
    if (plan->C > 0)
        std::memcpy(out_host, plan->cand.data() + static_cast<size_t>(w) * plan->C,
                    sizeof(int32_t) * static_cast<size_t>(plan->C));
    return GBMUF_OK;
}

int gbmuf_neighbours_host(const gbmuf_plan_t *plan, uint64_t round, int32_t *out_host)
{
    if (!plan) return GBMUF_EINVAL;
    const int32_t q = plan->q, C = plan->C, K = plan->K;
    if (q == 0 || plan->m == 0) return GBMUF_OK;
    if (!out_host) return GBMUF_EINVAL;
    std::vector<int32_t> work;
    try {
        work.resize(static_cast<size_t>(C));
    } catch (const std::bad_alloc &) {
        return GBMUF_ENOMEM;
    }
    const uint32_t key0 = static_cast<uint32_t>(plan->seed), key1 = static_cast<uint32_t>(plan->seed >> 32);
    const uint32_t r0 = static_cast<uint32_t>(round), r1 = static_cast<uint32_t>(round >> 32);
    for (int32_t i = 0; i < plan->m; ++i)
        for (int32_t w = 0; w < K; ++w) {
            std::memcpy(work.data(), plan->cand.data() + static_cast<size_t>(w) * C,
                        sizeof(int32_t) * static_cast<size_t>(C));
            draw_neighbours(HostPerm{work.data()}, C, q, key0, key1, r0, r1, static_cast<uint32_t>(i),
                            static_cast<uint32_t>(w));
            std::memcpy(out_host + (static_cast<size_t>(i) * K + w) * q, work.data(),
                        sizeof(int32_t) * static_cast<size_t>(q));
        }
    return GBMUF_OK;
}

int gbmuf_neighbours_device(const gbmuf_plan_t *plan, uint64_t round, int32_t *out_dev, void *stream)
{
    if (!plan) return GBMUF_EINVAL;
    const int rc = check_device(plan);
    if (rc != GBMUF_OK) return rc;
    if (plan->q == 0 || plan->m == 0) return GBMUF_OK;
    if (!out_dev) return GBMUF_EINVAL;
    return launch_sampler(sample_args(plan, round, out_dev), static_cast<hipStream_t>(stream));
}

int gbmuf_sync(const gbmuf_plan_t *plan, float *replicas, float *global, float *delta, int64_t worker_stride,
               float eta, float zeta, int32_t nesterov, uint64_t round, void *stream)
{
    int rc = check_sync(plan, replicas, global, delta, worker_stride, nesterov);
    if (rc != GBMUF_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (plan->inline_sampling)
        return enqueue_sync(plan, nullptr, replicas, global, delta, worker_stride, eta, zeta, nesterov, s, 0, -1, false,
                            0, round);
    rc = launch_sampler(sample_args(plan, round, plan->d_nbr), s);
    if (rc != GBMUF_OK) return rc;
    return enqueue_sync(plan, plan->d_nbr, replicas, global, delta, worker_stride, eta, zeta, nesterov, s, 0, -1, false,
                        0, round);
}

int gbmuf_plan_set_periods(gbmuf_plan_t *plan, const int32_t *periods_host)
{
    if (!plan) return GBMUF_EINVAL;
    if (!periods_host) {
        plan->periods.clear();
        return GBMUF_OK;
    }
    for (int32_t i = 0; i < plan->m; ++i)
        if (periods_host[i] < 1) return GBMUF_EINVAL;
    try {
        plan->periods.assign(periods_host, periods_host + plan->m);
    } catch (const std::bad_alloc &) {
        return GBMUF_ENOMEM;
    }
    if (plan->has_device && plan->m > 0) {
        // ordered after everything already enqueued on the device, and complete on return
        hipError_t err = hipDeviceSynchronize();
        if (err == hipSuccess)
            err = hipMemcpy(plan->d_periods, plan->periods.data(), sizeof(int32_t) * static_cast<size_t>(plan->m),
                            hipMemcpyHostToDevice);
        if (err != hipSuccess) return hip_failed("hipMemcpy(periods)", err, GBMUF_EDEVICE);
    }
    return GBMUF_OK;
}

int gbmuf_sync_step(const gbmuf_plan_t *plan, float *replicas, float *global, float *delta, int64_t worker_stride,
                    float eta, float zeta, int32_t nesterov, uint64_t step, void *stream)
{
    int rc = check_sync(plan, replicas, global, delta, worker_stride, nesterov);
    if (rc != GBMUF_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (plan->periods.empty())
        return gbmuf_sync(plan, replicas, global, delta, worker_stride, eta, zeta, nesterov, step, stream);
    // runs of consecutive components that sync at this step = contiguous ranges of the tile list
    struct Run { int64_t first, count; };
    Run runs[8];
    int n_runs = 0;
    bool too_many = false, any = false;
    for (int32_t i = 0; i < plan->m; ++i) {
        const bool active = step % static_cast<uint64_t>(plan->periods[static_cast<size_t>(i)]) == 0;
        const int64_t t0 = plan->tile_start[static_cast<size_t>(i)], t1 = plan->tile_start[static_cast<size_t>(i) + 1];
        if (!active || t1 == t0) continue;
        any = true;
        if (n_runs > 0 && runs[n_runs - 1].first + runs[n_runs - 1].count == t0) {
            runs[n_runs - 1].count += t1 - t0;
        } else if (n_runs < 8) {
            runs[n_runs++] = Run{t0, t1 - t0};
        } else {
            too_many = true;
            break;
        }
    }
    if (!any) return GBMUF_OK;
    const int32_t *nbr = nullptr;                           // nullptr: workgroups draw their own rows
    if (!plan->inline_sampling) {
        rc = launch_sampler(sample_args(plan, step, plan->d_nbr), s);
        if (rc != GBMUF_OK) return rc;
        nbr = plan->d_nbr;
    }
    if (too_many)                                           // scattered schedule: one launch, checked on the device
        return enqueue_sync(plan, nbr, replicas, global, delta, worker_stride, eta, zeta, nesterov, s, 0, -1, true,
                            step, step);
    for (int r = 0; r < n_runs; ++r) {
        rc = enqueue_sync(plan, nbr, replicas, global, delta, worker_stride, eta, zeta, nesterov, s, runs[r].first,
                          runs[r].count, false, 0, step);
        if (rc != GBMUF_OK) return rc;
    }
    return GBMUF_OK;
}

int gbmuf_final_average(const gbmuf_plan_t *plan, const float *replicas, int64_t worker_stride, float *out_dev,
                        void *stream)
{
    if (!plan || !replicas || !out_dev || worker_stride < plan->P) return GBMUF_EINVAL;
    const int rc = check_device(plan);
    if (rc != GBMUF_OK) return rc;
    return launch_final_average(replicas, worker_stride, plan->K, plan->P, 1.0f / static_cast<float>(plan->K), out_dev,
                                static_cast<hipStream_t>(stream));
}

int gbmuf_sync_table(const gbmuf_plan_t *plan, const int32_t *nbr_dev, float *replicas, float *global,
                     float *delta, int64_t worker_stride, float eta, float zeta, int32_t nesterov, void *stream)
{
    int rc = check_sync(plan, replicas, global, delta, worker_stride, nesterov);
    if (rc != GBMUF_OK) return rc;
    if (!nbr_dev && plan->q > 0 && plan->m > 0) return GBMUF_EINVAL;
    return enqueue_sync(plan, nbr_dev ? nbr_dev : plan->d_nbr, replicas, global, delta, worker_stride, eta,
                        zeta, nesterov, static_cast<hipStream_t>(stream));
}

int gbmuf_recommend_layout(int64_t P, int32_t K, int64_t span_bytes, gbmuf_layout_t *out)
{
    if (!out || P < 0 || K < 1 || span_bytes < 0) return GBMUF_EINVAL;
    const int64_t row = (P + 1023) / 1024 * 1024;          // rows start on 4 KB: tiles cover whole cache lines
    int64_t stride = 3 * row;
    if (K > 1) {
        const int64_t spread = (span_bytes / 4 - 3 * row) / (K - 1) / 1024 * 1024;
        if (spread > stride) stride = spread;
    }
    out->worker_stride = stride;
    out->omega_offset = row;
    out->delta_offset = 2 * row;
    out->arena_floats = static_cast<int64_t>(K - 1) * stride + 3 * row;
    return GBMUF_OK;
}

int gbmuf_probe_copy(float *dst_dev, const float *src_dev, int64_t n_floats, int32_t flags, void *stream)
{
    if (!dst_dev || !src_dev || n_floats < 0 || (n_floats & 3)) return GBMUF_EINVAL;
    if (!aligned16(dst_dev) || !aligned16(src_dev)) return GBMUF_EINVAL;
    return launch_copy_probe(dst_dev, src_dev, n_floats, flags, 256 * 16, static_cast<hipStream_t>(stream));
}

const char *gbmuf_last_error_detail(void) { return gbmuf::g_detail; }

const char *gbmuf_strerror(int code)
{
    switch (code) {
        case GBMUF_OK: return "ok";
        case GBMUF_EINVAL: return "invalid argument";
        case GBMUF_ENOMEM: return "out of host or device memory";
        case GBMUF_EDEVICE: return "no usable GPU or a HIP call failed";
        case GBMUF_EUNSUPPORTED: return "beyond the limits of this library";
        default: return "unknown status";
    }
}

}  // extern "C"
