// gbmuf_plan.hip -- host half of libgbmuf: plan construction (partition, ring topology,
// tile lists), the host sampler, argument checks and the C entry points of include/gbmuf.h.
#include "gbmuf_internal.h"

#include "../../include/gbmuf.h"

#include <algorithm>
#include <array>
#include <cstddef>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

using namespace gbmuf;

namespace {

// Work list of the fused kernel for one tile width, in component order.
struct TileSet {
    int32_t logT = 0;
    std::vector<TileDesc> tiles;
    std::vector<int64_t> tile_start;   // m+1: first tile of every component
    TileDesc *d_tiles = nullptr;
};

// How the fused kernel runs on one kind of state placement.
struct LayoutCfg {
    Variant variant{256, 8};
    int32_t logT = 0;
    int32_t set = 0;                   // which TileSet
    int32_t workgroups_per_cu = 0;     // 0 = no bound
};

enum { kRows = 0, kBlocked = 1 };
enum { kBmuf = 0, kMa = 1 };          // the three-array update, or the gossip-MA branch (theta only)
constexpr int kMaxTileSets = 4;

}  // namespace

struct gbmuf_plan_s {
    int32_t m = 0, K = 0, q = 0, p = 0, C = 0;
    uint64_t seed = 0;
    int64_t P = 0;
    bool mixed_q = false, has_periods = false;
    std::vector<int64_t> off;        // m+1 component offsets
    std::vector<int32_t> qv;         // m: neighbours per component
    std::vector<int32_t> periods;    // m: sync period H_i (all 1 without periods)
    std::vector<int32_t> cand;       // [K][C] ring candidates, order of Definition 1
    std::vector<CompDesc> comp;      // m: per-component constants of the kernels
    LayoutCfg cfg[2][2];             // [kRows, kBlocked][kBmuf, kMa]
    TileSet sets[kMaxTileSets];      // one per distinct tile width among the four configurations
    int32_t n_sets = 0;
    float inv = 1.0f;                // 1/(q+1), rounded once (plans with one q)
    int32_t flags = 0;               // load/store cache hints of the fused kernel
    bool in_kernel_sampling = false; // workgroups draw their own neighbour rows (no sampler launch)
    bool alternate = true;           // odd rounds walk the tile list backwards (see tile_of_block)

    bool has_device = false;
    int device = -1;
    int32_t lds_per_cu = 0;
    int32_t *d_cand = nullptr;
    CompDesc *d_comp = nullptr;
    int32_t *d_nbr = nullptr;        // neighbour scratch of gbmuf_sync, [m][K][q]
};

// ---------------------------------------------------------------------------------------
// Neighbour table of gbmuf_sync_static: device memory that exists without any allocation call.
// Every GPU the library runs on holds its own copy of this array (2 MiB) until the process
// ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the device
// address is looked up once per device, with that device current, when a plan is made there,
// and kernels and copies are only ever given that address.
// ---------------------------------------------------------------------------------------
static __device__ __align__(256) int32_t scratch[GBMUF_STATIC_TABLE_ENTRIES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
int32_t *g_scratch_ptr[kMaxDevices] = {};

// Looks up this device's copy of `scratch`; `device` must be the current device.
int resolve_scratch(int device)
{
    if (device < 0 || device >= kMaxDevices) return GBMUF_OK;       // gbmuf_sync_static will refuse this device
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device]) return GBMUF_OK;
    void *p = nullptr;
    const hipError_t err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (err != hipSuccess || !p) return gbmuf::hip_failed("hipGetSymbolAddress(scratch)", err, GBMUF_EDEVICE);
    g_scratch_ptr[device] = static_cast<int32_t *>(p);
    return GBMUF_OK;
}

int32_t *scratch_of(int device)
{
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    return g_scratch_ptr[device];
}
}  // namespace

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

// ---------------------------------------------------------------------------------------
// Host writing of the sampler (the device has its own in gbmuf_kernels.hip; the tests
// require the two, and the reference implementation, to agree bit for bit).
// ---------------------------------------------------------------------------------------
using Words4 = std::array<uint32_t, 4>;

// Philox-4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds, each one multiplying words
// 0 and 2 by the two round constants and mixing the high halves with the neighbouring words
// and the key, which advances by the two Weyl increments.
Words4 philox_block(Words4 ctr, uint32_t key_lo, uint32_t key_hi)
{
    for (int round = 0; round < 10; ++round) {
        const uint64_t prod0 = static_cast<uint64_t>(ctr[0]) * 0xD2511F53u;
        const uint64_t prod2 = static_cast<uint64_t>(ctr[2]) * 0xCD9E8D57u;
        ctr = Words4{static_cast<uint32_t>(prod2 >> 32) ^ ctr[1] ^ key_lo, static_cast<uint32_t>(prod2),
                     static_cast<uint32_t>(prod0 >> 32) ^ ctr[3] ^ key_hi, static_cast<uint32_t>(prod0)};
        key_lo += 0x9E3779B9u;
        key_hi += 0xBB67AE85u;
    }
    return ctr;
}

// Algorithm 1, sync branch, first statement, for worker `w` and component `comp` in sync
// `round`: q ids out of the worker's C candidates, uniformly without replacement, ascending.
// Draw j uses word j mod 4 of the block with counter (round lo, round hi, comp, w + 65536 * (j div 4))
// and exchanges pool[j] with pool[j + floor(word * (C - j) / 2^32)].
void host_pick(const int32_t *cand, int32_t C, int32_t q, uint64_t seed, uint64_t round, uint32_t comp, uint32_t w,
               std::vector<int32_t> &pool, int32_t *out)
{
    pool.assign(cand, cand + C);
    Words4 words{};
    for (int32_t j = 0; j < q; ++j) {
        if (j % 4 == 0)
            words = philox_block(Words4{static_cast<uint32_t>(round), static_cast<uint32_t>(round >> 32), comp,
                                        w + (static_cast<uint32_t>(j / 4) << 16)},
                                 static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32));
        const uint64_t remaining = static_cast<uint64_t>(C - j);
        const size_t pick = static_cast<size_t>(j) + static_cast<size_t>((words[static_cast<size_t>(j % 4)] * remaining) >> 32);
        std::swap(pool[static_cast<size_t>(j)], pool[pick]);
    }
    std::sort(pool.begin(), pool.begin() + q);
    std::copy_n(pool.begin(), q, out);
}

// ---------------------------------------------------------------------------------------
// Tile shapes
// ---------------------------------------------------------------------------------------
// Measured on MI355X.  Rows (3K address streams): short tiles of about 32 columns (512 B per
// worker row) with few 16-byte slots per thread, as many workgroups per CU as fit.  Blocked
// state (one address stream): the same 32 columns in workgroups of 512 threads, and only one
// or two workgroups per CU, so that what the whole chip has in flight is a short stretch of
// memory.
bool find_variant(int threads, int slots, Variant *out)
{
    int count = 0;
    const Variant *tab = variant_table(&count);
    for (int i = 0; i < count; ++i)
        if (tab[i].threads == threads && tab[i].slots == slots) {
            *out = tab[i];
            return true;
        }
    return false;
}

Variant default_variant(int K, int layout, int what)
{
    Variant v{1024, 4};
    if (layout == kRows) {
        const int threads = K <= 32 ? 256 : 1024;
        const int slots = K <= 8 ? 1 : K <= 16 ? 2 : 4;
        find_variant(threads, slots, &v);
    } else if (what == kBmuf) {
        // 32 columns (512 B) per worker row in workgroups of 512 threads, K/16 slots per thread
        if (K <= 4) find_variant(256, 1, &v);
        else if (K <= 16) find_variant(512, 1, &v);
        else if (K <= 32) find_variant(512, 2, &v);
        else if (K <= 64) find_variant(512, 4, &v);
        else if (K <= 128) find_variant(512, 8, &v);
    } else {
        if (K <= 16) find_variant(512, 2, &v);             // theta only: twice the columns per workgroup
        else if (K <= 64) find_variant(1024, 2, &v);
    }
    return v;
}

// Blocked state: what the chip has in flight should stay near 12-24 MB (24-48 KB per workgroup
// at two workgroups per CU, or 96 KB at one; the gossip-MA branch moves a third of that per
// workgroup and takes twice as many); more resident workgroups lose 5-15 points.
int32_t default_workgroups_per_cu(int K, int layout, int what)
{
    if (layout != kBlocked) return 0;
    if (what == kBmuf) return K <= 4 ? 4 : K <= 32 ? 2 : 1;
    return K <= 16 ? 4 : 2;
}

// Split every component into runs of at most T 16-byte columns (the fused kernel's work list).
void build_tiles(const gbmuf_plan_s &pl, TileSet &ts)
{
    const int64_t T = static_cast<int64_t>(1) << ts.logT;
    ts.tiles.clear();
    ts.tile_start.assign(static_cast<size_t>(pl.m) + 1, 0);
    for (int32_t i = 0; i < pl.m; ++i) {
        const int64_t a = pl.off[static_cast<size_t>(i)], b = pl.off[static_cast<size_t>(i) + 1];
        ts.tile_start[static_cast<size_t>(i)] = static_cast<int64_t>(ts.tiles.size());
        ts.tile_start[static_cast<size_t>(i) + 1] = static_cast<int64_t>(ts.tiles.size());
        if (a >= b) continue;
        // Tile boundaries sit at multiples of T columns counted from the row start, not from the
        // component start: with rows aligned to T*16 bytes every interior tile then covers whole
        // cache lines (a component that starts mid-line only gets a short first tile), and no tile
        // crosses a block of a blocked state.  Tiles that straddle lines cost a quarter of the
        // bandwidth on MI355X.
        const int64_t ga = a >> 2, gb = (b + 3) >> 2;
        for (int64_t g = ga; g < gb;) {
            int64_t next = (g / T + 1) * T;
            if (next > gb) next = gb;
            const int64_t lo = (g << 2) > a ? (g << 2) : a;
            const int64_t end = (next << 2) < b ? (next << 2) : b;
            ts.tiles.push_back(TileDesc{lo, static_cast<uint16_t>(end - lo),
                                        static_cast<uint16_t>(pl.qv[static_cast<size_t>(i)]), i});
            g = next;
        }
        ts.tile_start[static_cast<size_t>(i) + 1] = static_cast<int64_t>(ts.tiles.size());
    }
}

void free_device(gbmuf_plan_s &pl)
{
    if (pl.d_cand) (void)hipFree(pl.d_cand);
    if (pl.d_comp) (void)hipFree(pl.d_comp);
    if (pl.d_nbr) (void)hipFree(pl.d_nbr);
    for (TileSet &ts : pl.sets) {
        if (ts.d_tiles) (void)hipFree(ts.d_tiles);
        ts.d_tiles = nullptr;
    }
    pl.d_cand = nullptr; pl.d_comp = nullptr; pl.d_nbr = nullptr;
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

int make_device_state(gbmuf_plan_s &pl, int32_t sampling)
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
    int max_lds = 0;
    err = hipDeviceGetAttribute(&max_lds, hipDeviceAttributeMaxSharedMemoryPerBlock, pl.device);
    if (err != hipSuccess) return hip_failed("hipDeviceGetAttribute(MaxSharedMemoryPerBlock)", err, GBMUF_EDEVICE);
    pl.lds_per_cu = max_lds;                               // on this GPU one workgroup may take a CU's whole LDS
    {
        const int rc0 = resolve_scratch(pl.device);
        if (rc0 != GBMUF_OK) return rc0;
    }
    bool can = false;
    int rc = GBMUF_OK;
    for (int l = 0; l < 4 && rc == GBMUF_OK; ++l) {
        bool c = false;
        rc = prepare_kernels(pl.cfg[l / 2][l % 2].variant, pl.K, pl.q, pl.C, pl.mixed_q, &c);
        can = l == 0 ? c : (can && c);
    }
    if (rc != GBMUF_OK) return rc;
    // Drawing the rows inside every workgroup saves the sampler launch (about 2 us of a 8 us
    // sync on a 200k-parameter model) but costs about 2 % once there are millions of tiles:
    // by default only launch-bound plans do it.
    if (sampling == GBMUF_SAMPLING_IN_KERNEL) {
        if (!can) return GBMUF_EUNSUPPORTED;
        pl.in_kernel_sampling = true;
    } else if (sampling == GBMUF_SAMPLING_SEPARATE) {
        pl.in_kernel_sampling = false;
    } else {
        pl.in_kernel_sampling = can && pl.sets[pl.cfg[kRows][kBmuf].set].tiles.size() <= 8192;
    }
    if ((rc = upload(&pl.d_cand, pl.cand)) != GBMUF_OK) return rc;
    if ((rc = upload(&pl.d_comp, pl.comp)) != GBMUF_OK) return rc;
    for (int s = 0; s < pl.n_sets; ++s)
        if ((rc = upload(&pl.sets[s].d_tiles, pl.sets[s].tiles)) != GBMUF_OK) return rc;
    const size_t n = static_cast<size_t>(pl.m) * pl.K * pl.q;
    err = hipMalloc(reinterpret_cast<void **>(&pl.d_nbr), (n ? n : 1) * sizeof(int32_t));
    if (err != hipSuccess) {
        pl.d_nbr = nullptr;
        return hip_failed("hipMalloc(neighbour scratch)", err, GBMUF_ENOMEM);
    }
    pl.has_device = true;
    return GBMUF_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

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

// Do the floats two arrays of one state cover intersect?  Array X covers, for every worker w
// (and block g), `run` floats from X + g*group + w*stride.  Two such sets meet iff some
// combination d + dg*group + dw*stride lies within (-run, run); the nearest candidates decide
// because the rows of one block group do not reach into the next (validated by the caller).
bool arrays_overlap(const float *x, const float *y, int64_t K, int64_t stride, int64_t run, int64_t groups,
                    int64_t group)
{
    if (!x || !y || run <= 0) return false;
    const std::ptrdiff_t d_bytes = reinterpret_cast<const char *>(y) - reinterpret_cast<const char *>(x);
    const double d = static_cast<double>(d_bytes) / 4.0;      // in floats; a fraction still orders correctly
    auto near = [](double target, double step, int64_t limit, int64_t out[3]) {
        int64_t c = step > 0 ? static_cast<int64_t>(target / step + (target >= 0 ? 0.5 : -0.5)) : 0;
        int n = 0;
        for (int64_t k = c - 1; k <= c + 1; ++k) out[n++] = k < -limit ? -limit : (k > limit ? limit : k);
    };
    int64_t gs[3] = {0, 0, 0};
    if (groups > 1) near(-d, static_cast<double>(group), groups - 1, gs);
    for (int64_t dg : gs) {
        const double d2 = d + static_cast<double>(dg) * static_cast<double>(group);
        int64_t ws[3] = {0, 0, 0};
        if (K > 1) near(-d2, static_cast<double>(stride), K - 1, ws);
        for (int64_t dw : ws) {
            const double d3 = d2 + static_cast<double>(dw) * static_cast<double>(stride);
            if (d3 > -static_cast<double>(run) && d3 < static_cast<double>(run)) return true;
        }
    }
    return false;
}

int32_t max_blocked_logT(const gbmuf_plan_s *pl)
{
    return std::max(pl->cfg[kBlocked][kBmuf].logT, pl->cfg[kBlocked][kMa].logT);
}

// Validates a state description for this plan and turns it into the kernels' placement.
int check_state(const gbmuf_plan_s *pl, const gbmuf_state_t *st, bool need_slots, Placement *at, int *layout)
{
    if (!pl || !st || !st->theta) return GBMUF_EINVAL;
    if (need_slots && (!st->omega || !st->delta)) return GBMUF_EINVAL;
    int64_t run = pl->P, groups = 1, group = 0;
    if (st->block_floats == 0) {
        if (st->worker_stride < pl->P) return GBMUF_EINVAL;
        *at = Placement{st->worker_stride, 0, 62, 0};
        *layout = kRows;
    } else {
        const int64_t B = st->block_floats;
        if (B < 0 || (B & (B - 1)) != 0 || B > (static_cast<int64_t>(1) << 30)) return GBMUF_EINVAL;
        if (B < (static_cast<int64_t>(4) << max_blocked_logT(pl))) return GBMUF_EINVAL;      // a tile must fit a block
        if (st->worker_stride < B) return GBMUF_EINVAL;
        if (st->block_stride < static_cast<int64_t>(pl->K - 1) * st->worker_stride + B) return GBMUF_EINVAL;
        int32_t lg = 0;
        while ((static_cast<int64_t>(1) << lg) < B) ++lg;
        *at = Placement{st->worker_stride, st->block_stride - B, lg, 0};
        *layout = kBlocked;
        run = B; groups = (pl->P + B - 1) / B; group = st->block_stride;
    }
    const float *arr[3] = {st->theta, need_slots ? st->omega : nullptr, need_slots ? st->delta : nullptr};
    for (int a = 0; a < 3; ++a)
        for (int b = a + 1; b < 3; ++b)
            if (arrays_overlap(arr[a], arr[b], pl->K, st->worker_stride, run, groups, group)) return GBMUF_EINVAL;
    return GBMUF_OK;
}

gbmuf_state_t rows_state(float *theta, float *omega, float *delta, int64_t stride)
{
    gbmuf_state_t st{};
    st.theta = theta; st.omega = omega; st.delta = delta;
    st.worker_stride = stride;
    return st;
}

bool placement_vec4(const Placement &at) { return at.stride % 4 == 0 && at.block_extra % 4 == 0; }

// The dynamic LDS a workgroup asks for so that at most `workgroups_per_cu` of them fit a CU.
size_t lds_floor(const gbmuf_plan_s *pl, const LayoutCfg &cfg)
{
    const int n = cfg.workgroups_per_cu;
    if (n <= 0 || n > 8 || pl->lds_per_cu <= 0) return 0;
    const int64_t share = pl->lds_per_cu / n - 2048;         // margin for the allocation granule
    return share > 0 ? static_cast<size_t>(share) : 0;
}

struct TileRange {
    int64_t first = 0, count = -1;                            // count < 0: the whole list
};

int enqueue_sync(const gbmuf_plan_s *pl, const int32_t *nbr_dev, const gbmuf_state_t *st, const Placement &at,
                 int layout, float eta, float zeta, int32_t mode, hipStream_t stream, uint64_t round,
                 TileRange range = TileRange{}, bool check_periods = false)
{
    const LayoutCfg &cfg = pl->cfg[layout][mode == GBMUF_MODE_GOSSIP_MA ? kMa : kBmuf];
    const TileSet &ts = pl->sets[cfg.set];
    const int64_t n_tiles = range.count < 0 ? static_cast<int64_t>(ts.tiles.size()) : range.count;
    SyncArgs a{};
    a.tiles = ts.d_tiles + range.first;
    a.nbr = nbr_dev;
    a.comp = pl->d_comp;
    a.theta = st->theta; a.omega = st->omega; a.delta = st->delta;
    a.at = at;
    a.K = pl->K; a.q = pl->q; a.logT = cfg.logT; a.mode = mode;
    a.eta = eta; a.zeta = zeta; a.inv = pl->inv;
    a.flags = pl->flags | ((pl->alternate && (round & 1)) ? kFlagBackwards : 0) | (pl->mixed_q ? kFlagMixedQ : 0) |
              (check_periods ? kFlagCheckPeriods : 0);
    a.cand = pl->d_cand;                                    // used only when nbr_dev == nullptr
    a.C = pl->C;
    a.key0 = static_cast<uint32_t>(pl->seed); a.key1 = static_cast<uint32_t>(pl->seed >> 32);
    a.round0 = static_cast<uint32_t>(round); a.round1 = static_cast<uint32_t>(round >> 32);
    a.step = round;
    bool vec4 = aligned16(st->theta) && placement_vec4(at);
    if (mode != GBMUF_MODE_GOSSIP_MA) vec4 = vec4 && aligned16(st->omega) && aligned16(st->delta);
    return launch_sync(cfg.variant, vec4, a, n_tiles, lds_floor(pl, cfg), stream);
}

SampleArgs sample_args(const gbmuf_plan_s *pl, uint64_t round, int32_t *out)
{
    SampleArgs s{};
    s.cand = pl->d_cand;
    s.comp = pl->d_comp;
    s.out = out;
    s.first_pair = 0;
    s.pairs = static_cast<int64_t>(pl->m) * pl->K;
    s.K = pl->K; s.C = pl->C; s.q = pl->q; s.width = pl->q;
    s.mixed = pl->mixed_q ? 1 : 0;
    s.check_periods = 0;
    s.key0 = static_cast<uint32_t>(pl->seed); s.key1 = static_cast<uint32_t>(pl->seed >> 32);
    s.round0 = static_cast<uint32_t>(round); s.round1 = static_cast<uint32_t>(round >> 32);
    s.step = round;
    return s;
}

int check_mode(int32_t mode)
{
    return (mode < GBMUF_MODE_NO_RESTART || mode > GBMUF_MODE_GOSSIP_MA) ? GBMUF_EINVAL : GBMUF_OK;
}

// Argument checks shared by the sync entry points; argument errors come before device errors.
int check_sync(const gbmuf_plan_s *pl, const gbmuf_state_t *st, int32_t mode, Placement *at, int *layout)
{
    if (!pl || !st) return GBMUF_EINVAL;
    if (check_mode(mode) != GBMUF_OK) return GBMUF_EINVAL;
    const int rc = check_state(pl, st, mode != GBMUF_MODE_GOSSIP_MA, at, layout);
    if (rc != GBMUF_OK) return rc;
    return check_device(pl);
}

}  // namespace

extern "C" {

int gbmuf_plan_create(gbmuf_plan_t **out, const gbmuf_plan_desc_t *desc)
{
    if (!out) return GBMUF_EINVAL;
    *out = nullptr;
    if (!desc || desc->struct_size < sizeof(gbmuf_plan_desc_t)) return GBMUF_EINVAL;
    const int32_t m = desc->m, K = desc->K, p = desc->p;
    const int64_t *comp_offsets = desc->comp_offsets;
    if (!comp_offsets || m < 0 || K < 1 || desc->q < 0 || p < -1) return GBMUF_EINVAL;
    if (comp_offsets[0] != 0) return GBMUF_EINVAL;
    for (int32_t i = 0; i < m; ++i)
        if (comp_offsets[i + 1] < comp_offsets[i]) return GBMUF_EINVAL;
    if (desc->sampling < GBMUF_SAMPLING_AUTO || desc->sampling > GBMUF_SAMPLING_SEPARATE) return GBMUF_EINVAL;
    if (desc->sweep < GBMUF_SWEEP_AUTO || desc->sweep > GBMUF_SWEEP_FORWARD) return GBMUF_EINVAL;
    if (desc->cache_hints < 0 || desc->cache_hints > 3 || desc->workgroups_per_cu < 0) return GBMUF_EINVAL;
    if ((desc->tile_threads == 0) != (desc->tile_slots == 0)) return GBMUF_EINVAL;
    for (int32_t i = 0; desc->periods && i < m; ++i)
        if (desc->periods[i] < 1) return GBMUF_EINVAL;
    for (int32_t i = 0; desc->q_per_component && i < m; ++i)
        if (desc->q_per_component[i] < 0) return GBMUF_EINVAL;
    if (K > GBMUF_MAX_K) return GBMUF_EUNSUPPORTED;

    gbmuf_plan_s *pl = new (std::nothrow) gbmuf_plan_s;
    if (!pl) return GBMUF_ENOMEM;
    int rc = GBMUF_OK;
    try {
        pl->m = m; pl->K = K; pl->seed = desc->seed;
        // Beyond K-1 the listing of Definition 1 reaches nobody new (its first half alone has
        // passed every other worker), so larger degrees are the same topology.
        const int32_t want = p == 0 ? default_degree(K) : (p < 0 ? K / 2 : p);
        pl->p = want > K - 1 ? K - 1 : want;
        pl->off.assign(comp_offsets, comp_offsets + m + 1);
        pl->P = pl->off.back();
        if (desc->q_per_component) pl->qv.assign(desc->q_per_component, desc->q_per_component + m);
        else pl->qv.assign(static_cast<size_t>(m), desc->q);
        pl->q = desc->q_per_component ? 0 : desc->q;
        for (int32_t qi : pl->qv) {
            pl->q = std::max(pl->q, qi);
            if (qi != pl->qv.front()) pl->mixed_q = true;
        }
        pl->has_periods = desc->periods != nullptr;
        if (desc->periods) pl->periods.assign(desc->periods, desc->periods + m);
        else pl->periods.assign(static_cast<size_t>(m), 1);
        pl->inv = 1.0f / static_cast<float>(pl->q + 1);
        pl->comp.resize(static_cast<size_t>(m));
        for (int32_t i = 0; i < m; ++i)
            pl->comp[static_cast<size_t>(i)] = CompDesc{1.0f / static_cast<float>(pl->qv[static_cast<size_t>(i)] + 1),
                                                       pl->periods[static_cast<size_t>(i)],
                                                       pl->qv[static_cast<size_t>(i)], 0};

        std::vector<int32_t> ring;
        ring_of(0, K, pl->p, ring);
        pl->C = static_cast<int32_t>(ring.size());
        if (pl->q > pl->C) rc = GBMUF_EINVAL;              // the paper requires q <= 2p
        if (rc == GBMUF_OK) {
            pl->cand.resize(static_cast<size_t>(K) * pl->C);
            for (int32_t w = 0; w < K; ++w) {
                ring_of(w, K, pl->p, ring);
                if (pl->C > 0)
                    std::memcpy(pl->cand.data() + static_cast<size_t>(w) * pl->C, ring.data(),
                                sizeof(int32_t) * static_cast<size_t>(pl->C));
            }
            pl->flags = desc->cache_hints;
            pl->alternate = desc->sweep == GBMUF_SWEEP_AUTO;
            for (int l = 0; l < 4 && rc == GBMUF_OK; ++l) {
                LayoutCfg &cfg = pl->cfg[l / 2][l % 2];
                if (desc->tile_threads != 0) {
                    if (!find_variant(desc->tile_threads, desc->tile_slots, &cfg.variant)) rc = GBMUF_EINVAL;
                } else {
                    cfg.variant = default_variant(K, l / 2, l % 2);
                }
                if (rc != GBMUF_OK) break;
                const int slots = cfg.variant.threads * cfg.variant.slots;
                if (K > slots) { rc = desc->tile_threads != 0 ? GBMUF_EINVAL : GBMUF_EUNSUPPORTED; break; }
                int lg = 0;
                while ((static_cast<int64_t>(K) << (lg + 1)) <= slots) ++lg;
                cfg.logT = lg;                             // T = largest power of two with K*T <= slots
                cfg.workgroups_per_cu = desc->workgroups_per_cu != 0 ? desc->workgroups_per_cu
                                                                     : default_workgroups_per_cu(K, l / 2, l % 2);
            }
            if (rc == GBMUF_OK) {
                // one tile list per distinct tile width
                for (int l = 0; l < 4; ++l) {
                    LayoutCfg &cfg = pl->cfg[l / 2][l % 2];
                    int found = -1;
                    for (int s2 = 0; s2 < pl->n_sets; ++s2)
                        if (pl->sets[s2].logT == cfg.logT) found = s2;
                    if (found < 0) {
                        found = pl->n_sets++;
                        pl->sets[found].logT = cfg.logT;
                        build_tiles(*pl, pl->sets[found]);
                    }
                    cfg.set = found;
                }
                rc = make_device_state(*pl, desc->sampling);
            }
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

int gbmuf_plan(gbmuf_plan_t **out, const int64_t *comp_offsets, int32_t m, int32_t K, int32_t q, int32_t p,
               uint64_t seed)
{
    gbmuf_plan_desc_t d;
    std::memset(&d, 0, sizeof(d));
    d.struct_size = sizeof(d);
    d.m = m; d.K = K; d.q = q; d.p = p; d.seed = seed;
    d.comp_offsets = comp_offsets;
    return gbmuf_plan_create(out, &d);
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
    std::memset(info, 0, sizeof(*info));
    info->m = plan->m; info->K = plan->K; info->q = plan->q; info->p = plan->p; info->C = plan->C;
    info->has_device = plan->has_device ? 1 : 0;
    info->P = plan->P;
    info->n_tiles = static_cast<int64_t>(plan->sets[plan->cfg[kRows][kBmuf].set].tiles.size());
    info->tile_columns = 1 << plan->cfg[kRows][kBmuf].logT;
    info->threads = plan->cfg[kRows][kBmuf].variant.threads;
    info->seed = plan->seed;
    info->mixed_q = plan->mixed_q ? 1 : 0;
    info->has_periods = plan->has_periods ? 1 : 0;
    info->in_kernel_sampling = plan->in_kernel_sampling ? 1 : 0;
    info->tile_columns_blocked = 1 << plan->cfg[kBlocked][kBmuf].logT;
    info->threads_blocked = plan->cfg[kBlocked][kBmuf].variant.threads;
    info->workgroups_per_cu_blocked = plan->cfg[kBlocked][kBmuf].workgroups_per_cu;
    info->tile_columns_blocked_ma = 1 << plan->cfg[kBlocked][kMa].logT;
    info->min_block_floats = 4 << max_blocked_logT(plan);
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
    const int32_t width = plan->q, C = plan->C, K = plan->K;
    if (width == 0 || plan->m == 0) return GBMUF_OK;
    if (!out_host) return GBMUF_EINVAL;
    try {
        std::vector<int32_t> pool;
        pool.reserve(static_cast<size_t>(C));
        for (int32_t i = 0; i < plan->m; ++i) {
            const int32_t qi = plan->qv[static_cast<size_t>(i)];
            for (int32_t w = 0; w < K; ++w) {
                int32_t *row = out_host + (static_cast<size_t>(i) * K + w) * width;
                host_pick(plan->cand.data() + static_cast<size_t>(w) * C, C, qi, plan->seed, round,
                          static_cast<uint32_t>(i), static_cast<uint32_t>(w), pool, row);
                std::fill(row + qi, row + width, -1);
            }
        }
    } catch (const std::bad_alloc &) {
        return GBMUF_ENOMEM;
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

int gbmuf_sync_state(const gbmuf_plan_t *plan, const gbmuf_state_t *state, float eta, float zeta, int32_t nesterov,
                     uint64_t round, void *stream)
{
    Placement at{};
    int layout = kRows;
    int rc = check_sync(plan, state, nesterov, &at, &layout);
    if (rc != GBMUF_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (plan->in_kernel_sampling) return enqueue_sync(plan, nullptr, state, at, layout, eta, zeta, nesterov, s, round);
    rc = launch_sampler(sample_args(plan, round, plan->d_nbr), s);
    if (rc != GBMUF_OK) return rc;
    return enqueue_sync(plan, plan->d_nbr, state, at, layout, eta, zeta, nesterov, s, round);
}

int gbmuf_sync_static(const gbmuf_plan_t *plan, const gbmuf_state_t *state, float eta, float zeta, int32_t nesterov,
                      uint64_t round, void *stream)
{
    Placement at{};
    int layout = kRows;
    int rc = check_sync(plan, state, nesterov, &at, &layout);
    if (rc != GBMUF_OK) return rc;
    const int64_t entries = static_cast<int64_t>(plan->m) * plan->K * plan->q;
    if (entries > GBMUF_STATIC_TABLE_ENTRIES) {
        std::snprintf(gbmuf::g_detail, sizeof(gbmuf::g_detail),
                      "gbmuf_sync_static: the neighbour table has %lld entries, the static table holds %d",
                      static_cast<long long>(entries), GBMUF_STATIC_TABLE_ENTRIES);
        return GBMUF_EUNSUPPORTED;
    }
    int32_t *table = scratch_of(plan->device);
    if (!table) return hip_failed("no static table on this device", hipErrorInvalidDevice, GBMUF_EDEVICE);
    hipStream_t s = static_cast<hipStream_t>(stream);
    // the sampler fills every row the fused kernel reads, so nothing of an earlier call is seen
    rc = launch_sampler(sample_args(plan, round, table), s);
    if (rc != GBMUF_OK) return rc;
    return enqueue_sync(plan, table, state, at, layout, eta, zeta, nesterov, s, round);
}

int gbmuf_sync(const gbmuf_plan_t *plan, float *replicas, float *global, float *delta, int64_t worker_stride,
               float eta, float zeta, int32_t nesterov, uint64_t round, void *stream)
{
    const gbmuf_state_t st = rows_state(replicas, global, delta, worker_stride);
    return gbmuf_sync_state(plan, &st, eta, zeta, nesterov, round, stream);
}

int gbmuf_sync_step_state(const gbmuf_plan_t *plan, const gbmuf_state_t *state, float eta, float zeta,
                          int32_t nesterov, uint64_t step, void *stream)
{
    Placement at{};
    int layout = kRows;
    int rc = check_sync(plan, state, nesterov, &at, &layout);
    if (rc != GBMUF_OK) return rc;
    if (!plan->has_periods) return gbmuf_sync_state(plan, state, eta, zeta, nesterov, step, stream);
    hipStream_t s = static_cast<hipStream_t>(stream);
    // The tile list is in component order: the components that are due at this step cover one
    // or more runs of it.  One run is launched as exactly that range; several runs take one
    // launch over everything in which the workgroups of the other components return at once.
    const TileSet &ts = plan->sets[plan->cfg[layout][nesterov == GBMUF_MODE_GOSSIP_MA ? kMa : kBmuf].set];
    int64_t run_first = 0, run_end = 0;
    int32_t comp_first = -1, comp_last = -1, runs = 0;
    for (int32_t i = 0; i < plan->m; ++i) {
        if (step % static_cast<uint64_t>(plan->periods[static_cast<size_t>(i)]) != 0) continue;
        const int64_t t0 = ts.tile_start[static_cast<size_t>(i)], t1 = ts.tile_start[static_cast<size_t>(i) + 1];
        if (t1 == t0) continue;
        if (runs == 0 || t0 != run_end) {
            ++runs;
            if (runs == 1) run_first = t0;
        }
        run_end = t1;
        if (comp_first < 0) comp_first = i;
        comp_last = i;
    }
    if (runs == 0) return GBMUF_OK;
    const bool one_run = runs == 1;
    const int32_t *nbr = nullptr;                           // nullptr: workgroups draw their own rows
    if (!plan->in_kernel_sampling) {
        // only the components that are due are sampled: the launch spans first..last of them and
        // the threads of components in between that are not due leave without drawing
        SampleArgs sa = sample_args(plan, step, plan->d_nbr);
        sa.first_pair = static_cast<int64_t>(comp_first) * plan->K;
        sa.pairs = static_cast<int64_t>(comp_last - comp_first + 1) * plan->K;
        sa.check_periods = 1;
        rc = launch_sampler(sa, s);
        if (rc != GBMUF_OK) return rc;
        nbr = plan->d_nbr;
    }
    if (one_run)
        return enqueue_sync(plan, nbr, state, at, layout, eta, zeta, nesterov, s, step,
                            TileRange{run_first, run_end - run_first}, false);
    return enqueue_sync(plan, nbr, state, at, layout, eta, zeta, nesterov, s, step, TileRange{}, true);
}

int gbmuf_sync_step(const gbmuf_plan_t *plan, float *replicas, float *global, float *delta, int64_t worker_stride,
                    float eta, float zeta, int32_t nesterov, uint64_t step, void *stream)
{
    const gbmuf_state_t st = rows_state(replicas, global, delta, worker_stride);
    return gbmuf_sync_step_state(plan, &st, eta, zeta, nesterov, step, stream);
}

int gbmuf_sync_table_state(const gbmuf_plan_t *plan, const int32_t *nbr_dev, const gbmuf_state_t *state, float eta,
                           float zeta, int32_t nesterov, void *stream)
{
    Placement at{};
    int layout = kRows;
    if (plan && !nbr_dev && plan->q > 0 && plan->m > 0) return GBMUF_EINVAL;
    const int rc = check_sync(plan, state, nesterov, &at, &layout);
    if (rc != GBMUF_OK) return rc;
    return enqueue_sync(plan, nbr_dev ? nbr_dev : plan->d_nbr, state, at, layout, eta, zeta, nesterov,
                        static_cast<hipStream_t>(stream), 0);
}

int gbmuf_sync_table(const gbmuf_plan_t *plan, const int32_t *nbr_dev, float *replicas, float *global,
                     float *delta, int64_t worker_stride, float eta, float zeta, int32_t nesterov, void *stream)
{
    const gbmuf_state_t st = rows_state(replicas, global, delta, worker_stride);
    return gbmuf_sync_table_state(plan, nbr_dev, &st, eta, zeta, nesterov, stream);
}

int gbmuf_final_average_state(const gbmuf_plan_t *plan, const gbmuf_state_t *state, float *out_dev, void *stream)
{
    if (!plan || !state || !out_dev) return GBMUF_EINVAL;
    Placement at{};
    int layout = kRows;
    int rc = check_state(plan, state, false, &at, &layout);
    if (rc != GBMUF_OK) return rc;
    if ((rc = check_device(plan)) != GBMUF_OK) return rc;
    // Measured on MI355X: rows: 8 loads per thread, as many one-wave workgroups as fit.  Blocked:
    // the read stream is one address range, and 32-64 KB in flight per CU is the optimum
    // (K <= 32: 16 loads x 4 waves; larger K: 4 loads x 8 waves), worth 3-8 points.
    int rows_in_flight = 8;
    size_t floor_bytes = 0;
    if (layout == kBlocked && plan->lds_per_cu > 0) {
        const int waves = plan->K <= 32 ? 4 : 8;
        rows_in_flight = plan->K <= 32 ? 16 : 4;
        floor_bytes = static_cast<size_t>(plan->lds_per_cu / waves - 2048);
    }
    return launch_final_average(state->theta, at, plan->K, plan->P, 1.0f / static_cast<float>(plan->K), out_dev,
                                rows_in_flight, floor_bytes, static_cast<hipStream_t>(stream));
}

int gbmuf_final_average(const gbmuf_plan_t *plan, const float *replicas, int64_t worker_stride, float *out_dev,
                        void *stream)
{
    const gbmuf_state_t st = rows_state(const_cast<float *>(replicas), nullptr, nullptr, worker_stride);
    return gbmuf_final_average_state(plan, &st, out_dev, stream);
}

int gbmuf_state_copy(const gbmuf_plan_t *plan, const gbmuf_state_t *dst, const gbmuf_state_t *src, int32_t which,
                     void *stream)
{
    if (!plan || !dst || !src || which < 0 || which > 7) return GBMUF_EINVAL;
    float *const d[3] = {dst->theta, dst->omega, dst->delta};
    const float *const s[3] = {src->theta, src->omega, src->delta};
    gbmuf_state_t dsel = *dst, ssel = *src;                 // only the selected arrays take part in the checks
    float **dp[3] = {&dsel.theta, &dsel.omega, &dsel.delta};
    float **sp[3] = {&ssel.theta, &ssel.omega, &ssel.delta};
    int first = -1;
    for (int a = 0; a < 3; ++a) {
        if (which & (1 << a)) {
            if (!d[a] || !s[a]) return GBMUF_EINVAL;
            if (first < 0) first = a;
        } else {
            *dp[a] = nullptr; *sp[a] = nullptr;
        }
    }
    if (first < 0) return GBMUF_OK;
    // check_state wants theta: validate the geometry with the first selected array in its place
    gbmuf_state_t dgeo = dsel, sgeo = ssel;
    dgeo.theta = d[first]; sgeo.theta = const_cast<float *>(s[first]);
    Placement dat{}, sat{};
    int dl = kRows, sl = kRows;
    int rc = check_state(plan, &dgeo, false, &dat, &dl);
    if (rc != GBMUF_OK) return rc;
    if ((rc = check_state(plan, &sgeo, false, &sat, &sl)) != GBMUF_OK) return rc;
    if ((rc = check_device(plan)) != GBMUF_OK) return rc;
    for (int a = 0; a < 3; ++a) {
        if (!(which & (1 << a))) continue;
        rc = launch_state_copy(d[a], dat, s[a], sat, plan->K, plan->P, static_cast<hipStream_t>(stream));
        if (rc != GBMUF_OK) return rc;
    }
    return GBMUF_OK;
}

int gbmuf_recommend_layout(const gbmuf_plan_t *plan, int64_t P, int32_t K, int32_t kind, gbmuf_layout_t *out)
{
    if (!out || P < 0 || K < 1 || (kind != GBMUF_LAYOUT_ROWS && kind != GBMUF_LAYOUT_BLOCKED)) return GBMUF_EINVAL;
    if (plan && (plan->K != K || plan->P != P)) return GBMUF_EINVAL;
    std::memset(out, 0, sizeof(*out));
    if (kind == GBMUF_LAYOUT_ROWS) {
        const int64_t row = (P + 1023) / 1024 * 1024;      // rows start on 4 KB: tiles cover whole cache lines
        out->worker_stride = 3 * row;
        out->omega_offset = row;
        out->delta_offset = 2 * row;
        out->arena_floats = static_cast<int64_t>(K) * 3 * row;
        return GBMUF_OK;
    }
    // 32 KB blocks: K = 16 runs within a point of its best (8-32 KB), K = 64 at its best; 64 KB
    // blocks lose 7-10 points for both.  A plan with very wide tiles needs more.
    int64_t B = 8192;
    if (plan)
        while (B < (static_cast<int64_t>(4) << max_blocked_logT(plan))) B <<= 1;
    const int64_t blocks = (P + B - 1) / B;
    out->worker_stride = B;
    out->block_floats = B;
    out->block_stride = static_cast<int64_t>(3) * K * B;
    out->omega_offset = static_cast<int64_t>(K) * B;
    out->delta_offset = static_cast<int64_t>(2) * K * B;
    out->arena_floats = blocks * out->block_stride;
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
