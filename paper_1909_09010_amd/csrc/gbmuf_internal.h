// gbmuf_internal.h -- types and the sampler core shared by the host and device halves of
// libgbmuf.  Not part of the public interface (that is include/gbmuf.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gbmuf {

// One workgroup's share of a sync: elements [lo, lo + n) of component `comp`, for all K
// workers.  The range never crosses a component boundary and lies inside one run of
// tile_columns 16-byte columns (columns are aligned to multiples of 4 elements, so that a
// worker row with a 16-byte aligned base is read with 16-byte loads).
struct TileDesc {
    int64_t lo;
    int32_t n;
    int32_t comp;
};
static_assert(sizeof(TileDesc) == 16, "one 16-byte load per workgroup");

// Arguments of the fused gather-average-momentum kernels.
struct SyncArgs {
    const TileDesc *tiles;
    const int32_t *nbr;      // [m][K][q], device
    float *theta, *omega, *delta;
    int64_t stride;          // floats between worker rows
    int32_t K, q;
    int32_t logT;            // log2(columns per tile)
    int32_t mode;            // GBMUF_MODE_*
    float eta, zeta, inv;    // inv = 1/(q+1), rounded once on the host
    int32_t flags;           // bit 0: streaming (nontemporal) stores, bit 1: streaming loads
    // nbr == nullptr: the workgroup draws its component's neighbour rows itself (same bits as
    // the sampler kernel) from the candidates and the key below; C ints per worker go to LDS
    const int32_t *cand;     // [K][C], device
    int32_t C;
    uint32_t key0, key1, round0, round1;
    const int32_t *periods;  // per-component sync period H_i, or nullptr: every component syncs
    uint64_t step;           // with periods: component i syncs iff step % H_i == 0
};

// Arguments of the neighbour-sampling kernel.
struct SampleArgs {
    const int32_t *cand;     // [K][C] ring candidates in the order of Definition 1, device
    int32_t *out;            // [m][K][q]
    int64_t pairs;           // m*K
    int32_t K, C, q;
    uint32_t key0, key1;     // seed low / high
    uint32_t round0, round1; // round low / high
};

// Philox-4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): counter (c0..c3), key (k0, k1).
__host__ __device__ inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
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

// "Randomly choose q neighbors" (Algorithm 1, sync branch) for one (component, worker):
// partial Fisher-Yates shuffle of the worker's candidate list, which `perm(x)` exposes as
// a mutable sequence of C ids.  Draw j takes 32-bit word j%4 of the Philox block whose
// counter is (round low, round high, component, worker + 65536*(j/4)) under the key
// (seed low, seed high) and swaps position j with j + floor(word * (C-j) / 2^32).
// Afterwards positions [0, q) are sorted ascending.  Integer arithmetic only, so the host
// and the device produce the same bits.
template <class Perm>
__host__ __device__ inline void draw_neighbours(Perm perm, int32_t C, int32_t q, uint32_t key0,
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

// One tile shape of the fused kernel: threads per workgroup and 16-byte slots per thread.
// A tile holds threads*slots slots = K worker rows of tile_columns columns each.
struct Variant {
    int threads;
    int slots;
};

// Remembers the most recent failing HIP call of this thread (what gbmuf_last_error_detail
// returns) and maps it to a status.
int hip_failed(const char *what, hipError_t err, int status);

// kernels.hip
int launch_sampler(const SampleArgs &a, hipStream_t stream);
int launch_final_average(const float *theta, int64_t stride, int K, int64_t P, float inv, float *out,
                         hipStream_t stream);
int launch_copy_probe(float *dst, const float *src, int64_t n_floats, int flags, int blocks, hipStream_t stream);
int launch_sync(const Variant &v, bool vec4, const SyncArgs &a, int64_t n_tiles, hipStream_t stream);
int prepare_kernels(const Variant &v, int K, int q, int C, bool *inline_sampling_out);
const Variant *variant_table(int *count);

}  // namespace gbmuf
