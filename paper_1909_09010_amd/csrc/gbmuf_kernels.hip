// gbmuf_kernels.hip -- gfx950 kernels of libgbmuf: the neighbour sampler and the fused
// gather-average-momentum kernel (Algorithm 1, sync branch, of arXiv 1909.09010).
//
// Fused kernel, in one sentence: a workgroup owns a tile of T 16-byte columns of one
// component for ALL K workers, parks the K x T block of theta in LDS (so every worker's
// average reads its neighbours from LDS, and all reads of theta happen before any write:
// the in-place update keeps snapshot semantics), and streams omega and Delta through
// registers; every state byte is read once and written once.  Where an element lives is a
// Placement: plain rows, or blocks of 2^logB floats whose same-index blocks of all workers lie
// together (one offset per tile, since a tile never crosses a block).
#include "gbmuf_internal.h"

#include "../../include/gbmuf.h"

// Every multiply and add below is rounded on its own: the reference arithmetic has no
// fused multiply-add.  (The build also passes -ffp-contract=off.)
#pragma clang fp contract(off)

namespace gbmuf {

namespace {

// ---------------------------------------------------------------------------------------
// Device writing of the sampler.  (The host has its own, separately written one.)
// ---------------------------------------------------------------------------------------
// Philox-4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): counter (c0..c3), key (k0, k1).
__device__ inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                     uint32_t k0, uint32_t k1, uint32_t out[4])
{
    const uint64_t mul_a = 0xD2511F53ull, mul_b = 0xCD9E8D57ull;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t pa = mul_a * c0;
        const uint64_t pb = mul_b * c2;
        const uint32_t x0 = static_cast<uint32_t>(pb >> 32) ^ c1 ^ k0;
        const uint32_t x2 = static_cast<uint32_t>(pa >> 32) ^ c3 ^ k1;
        c1 = static_cast<uint32_t>(pb);
        c3 = static_cast<uint32_t>(pa);
        c0 = x0;
        c2 = x2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// The random pick of q neighbours (Algorithm 1, sync branch, first statement) for one
// (component, worker): partial Fisher-Yates shuffle of the worker's candidate list, which
// `perm(x)` exposes as a mutable sequence of C ids.  Draw j takes 32-bit word j%4 of the
// Philox block whose counter is (round low, round high, component, worker + 65536*(j/4))
// under the key (seed low, seed high) and swaps position j with j + floor(word * (C-j) / 2^32).
// Afterwards positions [0, q) are sorted ascending.  Integer arithmetic only.
template <class Perm>
__device__ inline void draw_neighbours(Perm perm, int32_t C, int32_t q, uint32_t key0,
                                       uint32_t key1, uint32_t round0, uint32_t round1,
                                       uint32_t component, uint32_t worker)
{
    uint32_t u[4] = {0u, 0u, 0u, 0u};
    for (int32_t j = 0; j < q; ++j) {
        const int lane = j & 3;
        if (lane == 0)
            philox4x32_10(round0, round1, component, worker + 65536u * static_cast<uint32_t>(j >> 2),
                          key0, key1, u);
        const uint32_t word = lane == 0 ? u[0] : lane == 1 ? u[1] : lane == 2 ? u[2] : u[3];
        const uint32_t span = static_cast<uint32_t>(C - j);
        const int32_t r = j + static_cast<int32_t>((static_cast<uint64_t>(word) * span) >> 32);
        const int32_t a = perm(j), b = perm(r);
        perm(j) = b;
        perm(r) = a;
    }
    for (int32_t a = 1; a < q; ++a) {           // insertion sort of the q chosen ids
        const int32_t v = perm(a);
        int32_t b = a - 1;
        while (b >= 0 && perm(b) > v) { perm(b + 1) = perm(b); --b; }
        perm(b + 1) = v;
    }
}

// ---------------------------------------------------------------------------------------
// Neighbour sampler: one thread per (component, worker); the thread's copy of the
// candidate list lives in LDS, interleaved so that thread t owns words t, t+TB, t+2TB...
// ---------------------------------------------------------------------------------------
struct LdsPerm {
    int32_t *base;
    int stride;
    __device__ int32_t &operator()(int32_t x) const { return base[x * stride]; }
};

__global__ void sample_kernel(SampleArgs a)
{
    extern __shared__ int32_t perm_lds[];
    const int tb = blockDim.x;
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * tb + threadIdx.x;
    if (idx >= a.pairs) return;                       // no barrier below
    const int64_t pair = a.first_pair + idx;
    const uint32_t comp = static_cast<uint32_t>(pair / a.K);
    const uint32_t w = static_cast<uint32_t>(pair % a.K);
    if (a.check_periods && a.step % static_cast<uint64_t>(a.comp[comp].period) != 0) return;   // not due
    const int32_t q = a.mixed ? a.comp[comp].q : a.q;
    LdsPerm perm{perm_lds + threadIdx.x, tb};
    const int32_t *cand = a.cand + static_cast<int64_t>(w) * a.C;
    for (int32_t x = 0; x < a.C; ++x) perm(x) = cand[x];
    draw_neighbours(perm, a.C, q, a.key0, a.key1, a.round0, a.round1, comp, w);
    int32_t *row = a.out + pair * a.width;
    for (int32_t j = 0; j < q; ++j) row[j] = perm(j);
    for (int32_t j = q; j < a.width; ++j) row[j] = -1;
}

// ---------------------------------------------------------------------------------------
// The block-momentum filter and the restart for one element (Algorithm 1, gossip-BMUF
// statements): G = avg - theta_{t-H};  Delta' = eta*Delta + zeta*G;  omega' = omega +
// Delta';  theta' = omega' + eta*Delta'.  theta_{t-H} is omega + eta*Delta in the paper's
// mode (what the previous restart wrote), omega otherwise.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void filter(float avg, float om, float de, float eta, float zeta, int mode,
                                       float &th_out, float &om_out, float &de_out)
{
    const float t = eta * de;
    const float start = (mode == GBMUF_MODE_PAPER) ? om + t : om;
    const float G = avg - start;
    const float zg = zeta * G;
    const float dn = t + zg;
    const float on = om + dn;
    float tn = on;
    if (mode != GBMUF_MODE_NO_RESTART) {
        const float r = eta * dn;
        tn = on + r;
    }
    th_out = tn; om_out = on; de_out = dn;
}

// Which tile this workgroup takes.  Normally its own index.  With the backwards flag (set on
// odd rounds unless the plan asked for forward sweeps) the list is walked backwards, so that
// what the previous sync wrote last is read first, while it may still be in the 256 MB
// memory-side cache (it is for states of up to a few GB; larger states neither gain nor lose);
// the reversal keeps the index modulo 8, i.e. the XCD (workgroups are dealt round-robin to the
// 8 XCDs) and its L2.
__device__ __forceinline__ unsigned tile_of_block(int flags)
{
    const unsigned b = blockIdx.x;
    if (!(flags & kFlagBackwards)) return b;
    const unsigned r = b & 7u;
    const unsigned in_class = (gridDim.x - r + 7u) >> 3;      // tiles with index == r (mod 8)
    return ((in_class - 1u - (b >> 3)) << 3) | r;
}

// Neighbour rows of this tile's component -> LDS, merged with the worker itself and sorted
// ascending: ids[w][0..q].  Ids are clamped into [0, K) so that a bad caller table cannot
// index outside the tile.
__device__ __forceinline__ void stage_ids(uint16_t *ids, const int32_t *nbr, int comp, int K, int q, int width,
                                          int tid, int nthreads)
{
    for (int w = tid; w < K; w += nthreads) {
        const int32_t *row = nbr + (static_cast<int64_t>(comp) * K + w) * width;
        uint16_t *dst = ids + w * (q + 1);
        dst[0] = static_cast<uint16_t>(w);
        for (int j = 0; j < q; ++j) {
            int v = row[j];
            v = v < 0 ? 0 : (v >= K ? K - 1 : v);
            int b = j;
            while (b >= 0 && dst[b] > v) { dst[b + 1] = dst[b]; --b; }
            dst[b + 1] = static_cast<uint16_t>(v);
        }
    }
}

// The same rows drawn by the workgroup itself (a.nbr == nullptr): thread w copies worker w's
// candidates into its LDS row, runs the sampler core and merges itself in.  Saves the
// separate sampler launch and the neighbour scratch; overlaps with the tile's loads in flight.
struct LdsRow {
    int32_t *base;
    __device__ int32_t &operator()(int32_t x) const { return base[x]; }
};

__device__ __forceinline__ void draw_ids(uint16_t *ids, int32_t *perm, const SyncArgs &a, int comp, int q, int tid,
                                         int nthreads)
{
    const int K = a.K, C = a.C;
    for (int w = tid; w < K; w += nthreads) {
        int32_t *mine = perm + w * C;
        const int32_t *cand = a.cand + static_cast<int64_t>(w) * C;
        for (int x = 0; x < C; ++x) mine[x] = cand[x];
        draw_neighbours(LdsRow{mine}, C, q, a.key0, a.key1, a.round0, a.round1, static_cast<uint32_t>(comp),
                        static_cast<uint32_t>(w));
        uint16_t *dst = ids + w * (q + 1);                 // mine[0..q) ascending; insert w
        int j = 0, o = 0;
        while (j < q && mine[j] < w) dst[o++] = static_cast<uint16_t>(mine[j++]);
        dst[o++] = static_cast<uint16_t>(w);
        while (j < q) dst[o++] = static_cast<uint16_t>(mine[j++]);
    }
}

__device__ __forceinline__ size_t ids_words(int K, int q)      // uint16 entries, padded to 16 bytes
{
    return (static_cast<size_t>(K) * static_cast<size_t>(q + 1) + 7) & ~static_cast<size_t>(7);
}

// ---------------------------------------------------------------------------------------
// 16-byte path: worker rows are 16-byte aligned (bases and stride), a column is 4 floats.
// Q1 = q+1 when known at compile time (the sum is then fully unrolled), 0 = run-time q.
// Slot s of the tile (s = tid + n*NT) is worker s >> logT, column s & (T-1).
// ---------------------------------------------------------------------------------------
typedef float v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ v4f load4(const float *p, bool streaming)
{
    const v4f *q = reinterpret_cast<const v4f *>(p);
    return streaming ? __builtin_nontemporal_load(q) : *q;
}

__device__ __forceinline__ void store4(float *p, v4f v, bool streaming)
{
    v4f *q = reinterpret_cast<v4f *>(p);
    if (streaming) __builtin_nontemporal_store(v, q);
    else *q = v;
}

template <int NT, int SLOTS, int Q1>
__global__ __launch_bounds__(NT) void sync_vec4_kernel(SyncArgs a)
{
    extern __shared__ float4 lds4[];
    v4f *tile = reinterpret_cast<v4f *>(lds4);
    uint16_t *ids = reinterpret_cast<uint16_t *>(lds4 + NT * SLOTS);

    const int tid = threadIdx.x;
    const TileDesc td = a.tiles[tile_of_block(a.flags)];
    if ((a.flags & kFlagCheckPeriods) && a.step % static_cast<uint64_t>(a.comp[td.comp].period) != 0)
        return;                                                   // not due: the whole workgroup leaves
    const int K = a.K, q1 = (Q1 > 0) ? Q1 : td.q + 1, q = q1 - 1;
    const float inv = (a.flags & kFlagMixedQ) ? a.comp[td.comp].inv : a.inv;
    const int logT = a.logT, T = 1 << logT;
    const int mode = a.mode;
    const bool nt_load = (a.flags & kFlagStreamLoads) != 0, nt_store = (a.flags & kFlagStreamStores) != 0;
    const int64_t lo = td.lo, hi = td.lo + td.n;
    const int64_t g0 = lo >> 2;                                  // first 4-float column
    const int ncols = static_cast<int>(((hi + 3) >> 2) - g0);     // <= T
    // a tile lies inside one block of a blocked state: one offset for all its elements
    const int64_t shift = (lo >> a.at.logB) * a.at.block_extra;

    v4f th[SLOTS], om[SLOTS], de[SLOTS];
    unsigned mask[SLOTS];                                         // which of the 4 floats are ours

#pragma unroll
    for (int n = 0; n < SLOTS; ++n) {
        const int slot = tid + n * NT;
        const int w = slot >> logT, col = slot & (T - 1);
        unsigned mk = 0;
        const int64_t e = (g0 + col) << 2;
        if (w < K && col < ncols) {
#pragma unroll
            for (int c = 0; c < 4; ++c) mk |= (e + c >= lo && e + c < hi) ? (1u << c) : 0u;
        }
        mask[n] = mk;
        th[n] = v4f{0.f, 0.f, 0.f, 0.f};
        om[n] = th[n];
        de[n] = th[n];
        const int64_t at = static_cast<int64_t>(w) * a.at.stride + e + shift;
        if (mk == 0xFu) {
            th[n] = load4(a.theta + at, nt_load);
            if (mode != GBMUF_MODE_GOSSIP_MA) {
                om[n] = load4(a.omega + at, nt_load);
                de[n] = load4(a.delta + at, nt_load);
            }
        } else if (mk != 0u) {                                    // a column cut by a component edge
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (mk & (1u << c)) {
                    th[n][c] = a.theta[at + c];
                    if (mode != GBMUF_MODE_GOSSIP_MA) { om[n][c] = a.omega[at + c]; de[n][c] = a.delta[at + c]; }
                }
            }
        }
    }

    if (a.nbr != nullptr) stage_ids(ids, a.nbr, td.comp, K, q, a.q, tid, NT);
    else draw_ids(ids, reinterpret_cast<int32_t *>(ids + ids_words(K, a.q)), a, td.comp, q, tid, NT);

#pragma unroll
    for (int n = 0; n < SLOTS; ++n) tile[tid + n * NT] = th[n];
    __syncthreads();

#pragma unroll
    for (int n = 0; n < SLOTS; ++n) {
        const unsigned mk = mask[n];
        if (mk == 0u) continue;
        const int slot = tid + n * NT;
        const int w = slot >> logT, col = slot & (T - 1);
        const uint16_t *row = ids + w * q1;

        // sum over the worker and its neighbours, ascending worker id, then * 1/(q+1)
        v4f s = tile[(static_cast<int>(row[0]) << logT) + col];
        if (Q1 > 0) {
#pragma unroll
            for (int j = 1; j < Q1; ++j) s = s + tile[(static_cast<int>(row[j]) << logT) + col];
        } else {
            for (int j = 1; j < q1; ++j) s = s + tile[(static_cast<int>(row[j]) << logT) + col];
        }
        v4f tn = s * inv, on = tn, dn = tn;
        if (mode != GBMUF_MODE_GOSSIP_MA) {
            const v4f avg = tn;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float t1, o1, d1;
                filter(avg[c], om[n][c], de[n][c], a.eta, a.zeta, mode, t1, o1, d1);
                tn[c] = t1; on[c] = o1; dn[c] = d1;
            }
        }
        const int64_t at = static_cast<int64_t>(w) * a.at.stride + ((g0 + col) << 2) + shift;
        if (mk == 0xFu) {
            store4(a.theta + at, tn, nt_store);
            if (mode != GBMUF_MODE_GOSSIP_MA) {
                store4(a.omega + at, on, nt_store);
                store4(a.delta + at, dn, nt_store);
            }
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (mk & (1u << c)) {
                    a.theta[at + c] = tn[c];
                    if (mode != GBMUF_MODE_GOSSIP_MA) { a.omega[at + c] = on[c]; a.delta[at + c] = dn[c]; }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Final model average (Algorithm 1, RETURN): out[e] = fl(1/K) * (theta[0][e] + theta[1][e] + ...),
// summed in ascending worker id.  One thread per 16-byte column; 4(K+1) bytes per parameter.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ int64_t placed(const Placement &at, int64_t e)
{
    return e + (e >> at.logB) * at.block_extra;
}

template <int B>
__global__ __launch_bounds__(256) void final_average_vec4_kernel(const float *theta, Placement at, int K,
                                                                 int64_t P, float inv, float *out)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t n4 = P >> 2;
    if (i < n4) {
        const float *col = theta + placed(at, i << 2);
        v4f s = *reinterpret_cast<const v4f *>(col);
        for (int k0 = 1; k0 < K; k0 += B) {                // B rows in flight, then added in ascending order
            v4f v[B];
#pragma unroll
            for (int j = 0; j < B; ++j)
                if (k0 + j < K) v[j] = *reinterpret_cast<const v4f *>(col + static_cast<int64_t>(k0 + j) * at.stride);
#pragma unroll
            for (int j = 0; j < B; ++j)
                if (k0 + j < K) s = s + v[j];
        }
        *reinterpret_cast<v4f *>(out + (i << 2)) = s * inv;
    } else if (i == n4) {                                  // the last P % 4 elements
        for (int64_t e = n4 << 2; e < P; ++e) {
            const float *col = theta + placed(at, e);
            float s = col[0];
            for (int k = 1; k < K; ++k) s = s + col[static_cast<int64_t>(k) * at.stride];
            out[e] = s * inv;
        }
    }
}

__global__ __launch_bounds__(256) void final_average_vec1_kernel(const float *theta, Placement at, int K,
                                                                 int64_t P, float inv, float *out)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= P) return;
    const float *col = theta + placed(at, e);
    float s = col[0];
#pragma unroll 4
    for (int k = 1; k < K; ++k) s = s + col[static_cast<int64_t>(k) * at.stride];
    out[e] = s * inv;
}

// ---------------------------------------------------------------------------------------
// Copy of one state array between two placements: blockIdx.y = worker, one thread per 16-byte
// column (V = 4) or per float (V = 1).
// ---------------------------------------------------------------------------------------
template <int V>
__global__ __launch_bounds__(256) void state_copy_kernel(float *dst, Placement da, const float *src, Placement sa,
                                                         int64_t P)
{
    const int64_t w = blockIdx.y;
    const int64_t e = (static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x) * V;
    if (e >= P) return;
    const float *s = src + w * sa.stride + placed(sa, e);
    float *d = dst + w * da.stride + placed(da, e);
    if (V == 4 && e + 4 <= P) {
        *reinterpret_cast<v4f *>(d) = *reinterpret_cast<const v4f *>(s);
    } else {
        for (int c = 0; c < V && e + c < P; ++c) d[c] = s[c];
    }
}

// Plain streaming copy of n 16-byte words (calibration of HBM counters and a reference for
// the bandwidth a 1:1 read/write stream reaches on this device).
__global__ __launch_bounds__(256) void copy_probe_kernel(v4f *dst, const v4f *src, int64_t n, int flags)
{
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride) {
        const v4f v = (flags & 2) ? __builtin_nontemporal_load(src + i) : src[i];
        if (flags & 1) __builtin_nontemporal_store(v, dst + i);
        else dst[i] = v;
    }
}

// ---------------------------------------------------------------------------------------
// 4-byte path for rows that are not 16-byte aligned: the same tile is walked in passes of
// T single-float columns.
// ---------------------------------------------------------------------------------------
template <int NT, int SLOTS>
__global__ __launch_bounds__(NT) void sync_vec1_kernel(SyncArgs a)
{
    extern __shared__ float4 lds4[];
    float *tile = reinterpret_cast<float *>(lds4);
    uint16_t *ids = reinterpret_cast<uint16_t *>(tile + NT * SLOTS);

    const int tid = threadIdx.x;
    const TileDesc td = a.tiles[tile_of_block(a.flags)];
    if ((a.flags & kFlagCheckPeriods) && a.step % static_cast<uint64_t>(a.comp[td.comp].period) != 0)
        return;                                                   // not due: the whole workgroup leaves
    const int K = a.K, q1 = td.q + 1, q = td.q;
    const float inv = (a.flags & kFlagMixedQ) ? a.comp[td.comp].inv : a.inv;
    const int logT = a.logT, T = 1 << logT;
    const int mode = a.mode;
    const int64_t hi = td.lo + td.n;
    const int64_t shift = (td.lo >> a.at.logB) * a.at.block_extra;

    if (a.nbr != nullptr) stage_ids(ids, a.nbr, td.comp, K, q, a.q, tid, NT);
    else draw_ids(ids, reinterpret_cast<int32_t *>(ids + ids_words(K, a.q)), a, td.comp, q, tid, NT);

    for (int64_t first = td.lo; first < hi; first += T) {
        const int ncols = static_cast<int>(hi - first < T ? hi - first : T);
        float th[SLOTS], om[SLOTS], de[SLOTS];
#pragma unroll
        for (int n = 0; n < SLOTS; ++n) {
            const int slot = tid + n * NT;
            const int w = slot >> logT, col = slot & (T - 1);
            th[n] = 0.f; om[n] = 0.f; de[n] = 0.f;
            if (w < K && col < ncols) {
                const int64_t at = static_cast<int64_t>(w) * a.at.stride + first + col + shift;
                th[n] = a.theta[at];
                if (mode != GBMUF_MODE_GOSSIP_MA) { om[n] = a.omega[at]; de[n] = a.delta[at]; }
            }
        }
#pragma unroll
        for (int n = 0; n < SLOTS; ++n) tile[tid + n * NT] = th[n];
        __syncthreads();
#pragma unroll
        for (int n = 0; n < SLOTS; ++n) {
            const int slot = tid + n * NT;
            const int w = slot >> logT, col = slot & (T - 1);
            if (!(w < K && col < ncols)) continue;
            const uint16_t *row = ids + w * q1;
            float s = tile[(static_cast<int>(row[0]) << logT) + col];
            for (int j = 1; j < q1; ++j) s = s + tile[(static_cast<int>(row[j]) << logT) + col];
            float tn = s * inv, on = 0.f, dn = 0.f;
            const int64_t at = static_cast<int64_t>(w) * a.at.stride + first + col + shift;
            if (mode != GBMUF_MODE_GOSSIP_MA) {
                const float avg = tn;
                filter(avg, om[n], de[n], a.eta, a.zeta, mode, tn, on, dn);
                a.omega[at] = on;
                a.delta[at] = dn;
            }
            a.theta[at] = tn;
        }
        __syncthreads();                                          // tile is reused by the next pass
    }
}

constexpr Variant kVariants[] = {
    {256, 8}, {512, 8}, {512, 4}, {256, 16}, {1024, 4}, {256, 4},
    {256, 2}, {512, 2}, {1024, 2}, {1024, 1}, {512, 1}, {256, 1},
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

using KernelFn = void (*)(SyncArgs);

template <int NT, int SLOTS>
KernelFn pick_vec4(int q1)
{
    switch (q1) {
        case 1: return sync_vec4_kernel<NT, SLOTS, 1>;
        case 2: return sync_vec4_kernel<NT, SLOTS, 2>;
        case 3: return sync_vec4_kernel<NT, SLOTS, 3>;
        case 4: return sync_vec4_kernel<NT, SLOTS, 4>;
        case 5: return sync_vec4_kernel<NT, SLOTS, 5>;
        default: return sync_vec4_kernel<NT, SLOTS, 0>;
    }
}

KernelFn pick_kernel(const Variant &v, bool vec4, int q1)
{
#define GBMUF_CASE(NT, SL) \
    if (v.threads == NT && v.slots == SL) return vec4 ? pick_vec4<NT, SL>(q1) : sync_vec1_kernel<NT, SL>;
    GBMUF_CASE(256, 8)
    GBMUF_CASE(512, 8)
    GBMUF_CASE(512, 4)
    GBMUF_CASE(256, 16)
    GBMUF_CASE(1024, 4)
    GBMUF_CASE(256, 4)
    GBMUF_CASE(256, 2)
    GBMUF_CASE(512, 2)
    GBMUF_CASE(1024, 2)
    GBMUF_CASE(1024, 1)
    GBMUF_CASE(512, 1)
    GBMUF_CASE(256, 1)
#undef GBMUF_CASE
    return nullptr;
}

size_t ids_bytes(int K, int q)
{
    return (static_cast<size_t>(K) * static_cast<size_t>(q + 1) * sizeof(uint16_t) + 15) & ~static_cast<size_t>(15);
}

size_t perm_bytes(int K, int C) { return static_cast<size_t>(K) * static_cast<size_t>(C) * sizeof(int32_t); }

// Workgroups draw their own neighbour rows when the candidates of all workers fit 8 KB of LDS.
bool can_sample_inline(int K, int C) { return perm_bytes(K, C) <= 8192; }

}  // namespace

const Variant *variant_table(int *count)
{
    *count = kNumVariants;
    return kVariants;
}

// Dynamic LDS one workgroup of the fused kernel needs: the theta tile, the merged neighbour
// rows (q = the largest q_i) and, when it draws them itself, the candidate copies.
size_t sync_lds_bytes(const Variant &v, bool vec4, int K, int q, int C, bool in_kernel_sampling)
{
    return static_cast<size_t>(v.threads) * v.slots * (vec4 ? sizeof(float4) : sizeof(float)) + ids_bytes(K, q) +
           (in_kernel_sampling ? perm_bytes(K, C) : 0);
}

// Raises the dynamic-LDS limit of the kernels this plan will launch to the device's maximum
// (so that plans with different needs can share a kernel) and says whether workgroups can
// draw their own neighbour rows.  GBMUF_EUNSUPPORTED if one workgroup's LDS exceeds the device.
int prepare_kernels(const Variant &v, int K, int q, int C, bool mixed_q, bool *can_sample_in_kernel)
{
    const bool inl = can_sample_inline(K, C);
    *can_sample_in_kernel = inl;
    const size_t lds4 = sync_lds_bytes(v, true, K, q, C, inl);
    int dev = 0, max_lds = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return hip_failed("hipGetDevice", err, GBMUF_EDEVICE);
    err = hipDeviceGetAttribute(&max_lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
    if (err != hipSuccess) return hip_failed("hipDeviceGetAttribute(MaxSharedMemoryPerBlock)", err, GBMUF_EDEVICE);
    if (lds4 > static_cast<size_t>(max_lds)) return GBMUF_EUNSUPPORTED;
    KernelFn k4 = pick_kernel(v, true, mixed_q ? 0 : q + 1), k1 = pick_kernel(v, false, q + 1);
    if (!k4 || !k1) return GBMUF_EINVAL;
    err = hipFuncSetAttribute(reinterpret_cast<const void *>(k4), hipFuncAttributeMaxDynamicSharedMemorySize, max_lds);
    if (err != hipSuccess) return hip_failed("hipFuncSetAttribute(16-byte kernel)", err, GBMUF_EDEVICE);
    err = hipFuncSetAttribute(reinterpret_cast<const void *>(k1), hipFuncAttributeMaxDynamicSharedMemorySize, max_lds);
    if (err != hipSuccess) return hip_failed("hipFuncSetAttribute(4-byte kernel)", err, GBMUF_EDEVICE);
    return GBMUF_OK;
}

// lds_floor: the workgroup asks for at least this much dynamic LDS, which bounds how many
// workgroups a compute unit holds at once (0 = only what it needs).
int launch_sync(const Variant &v, bool vec4, const SyncArgs &a, int64_t n_tiles, size_t lds_floor, hipStream_t stream)
{
    if (n_tiles <= 0) return GBMUF_OK;
    if (n_tiles > 0x7fffffffLL) return GBMUF_EUNSUPPORTED;
    const bool mixed = (a.flags & kFlagMixedQ) != 0;
    KernelFn k = pick_kernel(v, vec4, mixed ? 0 : a.q + 1);
    if (!k) return GBMUF_EINVAL;
    if (a.nbr == nullptr && (!can_sample_inline(a.K, a.C) || (a.cand == nullptr && a.C > 0))) return GBMUF_EINVAL;
    size_t lds = sync_lds_bytes(v, vec4, a.K, a.q, a.C, a.nbr == nullptr);
    if (lds < lds_floor) lds = lds_floor;
    SyncArgs args = a;
    void *argv[] = {&args};
    // the launch's own status: an earlier, unrelated error of the process is not ours to report
    const hipError_t err = hipLaunchKernel(reinterpret_cast<const void *>(k), dim3(static_cast<unsigned>(n_tiles)),
                                           dim3(v.threads), argv, lds, stream);
    return err == hipSuccess ? GBMUF_OK : hip_failed("hipLaunchKernel(sync)", err, GBMUF_EDEVICE);
}

namespace {
bool placement_vec4(const Placement &at)
{
    return at.stride % 4 == 0 && at.block_extra % 4 == 0 && at.logB >= 2;
}
}  // namespace

// rows_in_flight: 16-byte loads a thread keeps in flight (4, 8 or 16); lds_floor bounds the
// resident one-wave workgroups per compute unit like in launch_sync.
int launch_final_average(const float *theta, const Placement &at, int K, int64_t P, float inv, float *out,
                         int rows_in_flight, size_t lds_floor, hipStream_t stream)
{
    if (P <= 0) return GBMUF_OK;
    if (lds_floor > 60 * 1024) lds_floor = 60 * 1024;      // stays below what needs a raised limit
    const bool vec4 = ((reinterpret_cast<uintptr_t>(theta) | reinterpret_cast<uintptr_t>(out)) & 15u) == 0 &&
                      placement_vec4(at);
    const int64_t threads = vec4 ? (P >> 2) + 1 : P;
    const int bs = vec4 ? 64 : 256;                        // one wave per workgroup measured fastest (16-byte path)
    const int64_t blocks = (threads + bs - 1) / bs;
    if (blocks > 0x7fffffffLL) return GBMUF_EUNSUPPORTED;
    Placement pl = at;
    void *argv[] = {&theta, &pl, &K, &P, &inv, &out};
    const void *fn = !vec4 ? reinterpret_cast<const void *>(final_average_vec1_kernel)
                     : rows_in_flight <= 4 ? reinterpret_cast<const void *>(final_average_vec4_kernel<4>)
                     : rows_in_flight <= 8 ? reinterpret_cast<const void *>(final_average_vec4_kernel<8>)
                                           : reinterpret_cast<const void *>(final_average_vec4_kernel<16>);
    const hipError_t err = hipLaunchKernel(fn, dim3(static_cast<unsigned>(blocks)), dim3(bs), argv,
                                           vec4 ? lds_floor : 0, stream);
    return err == hipSuccess ? GBMUF_OK : hip_failed("hipLaunchKernel(final average)", err, GBMUF_EDEVICE);
}

int launch_state_copy(float *dst, const Placement &dst_at, const float *src, const Placement &src_at, int K,
                      int64_t P, hipStream_t stream)
{
    if (P <= 0 || K <= 0) return GBMUF_OK;
    const bool vec4 = ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15u) == 0 &&
                      placement_vec4(dst_at) && placement_vec4(src_at);
    const int64_t units = vec4 ? (P + 3) / 4 : P;
    const int64_t blocks = (units + 255) / 256;
    if (blocks > 0x7fffffffLL || K > 65535) return GBMUF_EUNSUPPORTED;
    Placement da = dst_at, sa = src_at;
    void *argv[] = {&dst, &da, &src, &sa, &P};
    const void *fn = vec4 ? reinterpret_cast<const void *>(state_copy_kernel<4>)
                          : reinterpret_cast<const void *>(state_copy_kernel<1>);
    const hipError_t err = hipLaunchKernel(fn, dim3(static_cast<unsigned>(blocks), static_cast<unsigned>(K)), dim3(256),
                                           argv, 0, stream);
    return err == hipSuccess ? GBMUF_OK : hip_failed("hipLaunchKernel(state copy)", err, GBMUF_EDEVICE);
}

int launch_copy_probe(float *dst, const float *src, int64_t n_floats, int flags, int blocks, hipStream_t stream)
{
    int64_t n = n_floats / 4;
    if (n <= 0) return GBMUF_OK;
    v4f *d = reinterpret_cast<v4f *>(dst);
    const v4f *s = reinterpret_cast<const v4f *>(src);
    void *argv[] = {&d, &s, &n, &flags};
    const hipError_t err = hipLaunchKernel(reinterpret_cast<const void *>(copy_probe_kernel), dim3(blocks), dim3(256),
                                           argv, 0, stream);
    return err == hipSuccess ? GBMUF_OK : hip_failed("hipLaunchKernel(copy probe)", err, GBMUF_EDEVICE);
}

int launch_sampler(const SampleArgs &a, hipStream_t stream)
{
    if (a.pairs <= 0 || a.width <= 0) return GBMUF_OK;
    // each thread keeps C ints in LDS: as many threads as fit 48 KB, at most 64
    int tb = 64;
    while (tb > 1 && static_cast<size_t>(tb) * a.C * sizeof(int32_t) > 48 * 1024) tb >>= 1;
    if (static_cast<size_t>(tb) * a.C * sizeof(int32_t) > 48 * 1024) return GBMUF_EUNSUPPORTED;
    const int64_t blocks = (a.pairs + tb - 1) / tb;
    if (blocks > 0x7fffffffLL) return GBMUF_EUNSUPPORTED;
    SampleArgs args = a;
    void *argv[] = {&args};
    const hipError_t err = hipLaunchKernel(reinterpret_cast<const void *>(sample_kernel),
                                           dim3(static_cast<unsigned>(blocks)), dim3(tb), argv,
                                           static_cast<size_t>(tb) * a.C * sizeof(int32_t), stream);
    return err == hipSuccess ? GBMUF_OK : hip_failed("hipLaunchKernel(sampler)", err, GBMUF_EDEVICE);
}

}  // namespace gbmuf
