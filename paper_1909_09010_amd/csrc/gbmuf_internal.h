// gbmuf_internal.h -- types shared by the host and device halves of libgbmuf.
// Not part of the public interface (that is include/gbmuf.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gbmuf {

// One workgroup's share of a sync: elements [lo, lo + n) of component `comp`, for all K
// workers.  The range never crosses a component boundary and lies inside one run of
// tile_columns 16-byte columns (columns are aligned to multiples of 4 elements, so that a
// worker row with a 16-byte aligned base is read with 16-byte loads).  q is the number of
// neighbours this component draws.
struct TileDesc {
    int64_t lo;
    uint16_t n;
    uint16_t q;
    int32_t comp;
};
static_assert(sizeof(TileDesc) == 16, "one 16-byte load per workgroup");

// Per-component constants on the device.
struct CompDesc {
    float inv;               // 1/(q_i + 1), rounded once on the host
    int32_t period;          // sync period H_i (1 if the plan has none)
    int32_t q;               // neighbours drawn for this component
    int32_t reserved;
};
static_assert(sizeof(CompDesc) == 16, "one 16-byte load");

// Placement of one state array's elements: element e of worker w is at
//   base + w * stride + e + (e >> logB) * block_extra
// Rows: logB = 62 and block_extra = 0.  Blocked: 2^logB floats per block and
// block_extra = block_stride - 2^logB.
struct Placement {
    int64_t stride;
    int64_t block_extra;
    int32_t logB;
    int32_t reserved;
};

// Arguments of the fused gather-average-momentum kernels.
struct SyncArgs {
    const TileDesc *tiles;
    const int32_t *nbr;      // [m][K][width], device; nullptr: the workgroup draws its rows itself
    const CompDesc *comp;    // [m]
    float *theta, *omega, *delta;
    Placement at;
    int32_t K, q;            // q: neighbours per component (the largest q_i when they differ)
    int32_t logT;            // log2(columns per tile)
    int32_t mode;            // GBMUF_MODE_*
    float eta, zeta, inv;    // inv = 1/(q+1), rounded once on the host (plans with one q)
    int32_t flags;           // bit 0: streaming stores, bit 1: streaming loads, bit 3: walk the
                             // tile list backwards, bit 4: components draw different q (read the
                             // tile's q and the component's inv), bit 5: skip components whose
                             // period does not divide `step`
    // in-kernel sampling (nbr == nullptr): same bits as the sampler kernel, drawn from the
    // candidates and the key below; C ints per worker go to LDS
    const int32_t *cand;     // [K][C], device
    int32_t C;
    uint32_t key0, key1, round0, round1;
    uint64_t step;           // with flag bit 5: component i syncs iff step % H_i == 0
};

enum : int32_t {
    kFlagStreamStores = 1,
    kFlagStreamLoads = 2,
    kFlagBackwards = 8,
    kFlagMixedQ = 16,
    kFlagCheckPeriods = 32,
};

// Arguments of the neighbour-sampling kernel: pairs [first_pair, first_pair + pairs) of the
// (component, worker) grid, pair = component * K + worker.
struct SampleArgs {
    const int32_t *cand;     // [K][C] ring candidates in the order of Definition 1, device
    const CompDesc *comp;    // [m]
    int32_t *out;            // [m][K][width]; entries beyond a component's q are set to -1
    int64_t first_pair, pairs;
    int32_t K, C, q, width;  // q is used unless `mixed`
    int32_t mixed;           // components draw different q: take comp[i].q
    int32_t check_periods;   // skip components whose period does not divide `step`
    uint32_t key0, key1;     // seed low / high
    uint32_t round0, round1; // round low / high
    uint64_t step;
};

// One tile shape of the fused kernel: threads per workgroup and 16-byte slots per thread.
// A tile holds threads*slots slots = K worker rows of tile_columns columns each.
struct Variant {
    int threads;
    int slots;
};

// Remembers the most recent failing HIP call of this thread (what gbmuf_last_error_detail
// returns) and maps it to a status.
int hip_failed(const char *what, hipError_t err, int status);

// gbmuf_kernels.hip
int launch_sampler(const SampleArgs &a, hipStream_t stream);
int launch_final_average(const float *theta, const Placement &at, int K, int64_t P, float inv, float *out,
                         int rows_in_flight, size_t lds_floor, hipStream_t stream);
int launch_state_copy(float *dst, const Placement &dst_at, const float *src, const Placement &src_at, int K,
                      int64_t P, hipStream_t stream);
int launch_copy_probe(float *dst, const float *src, int64_t n_floats, int flags, int blocks, hipStream_t stream);
int launch_sync(const Variant &v, bool vec4, const SyncArgs &a, int64_t n_tiles, size_t lds_floor, hipStream_t stream);
size_t sync_lds_bytes(const Variant &v, bool vec4, int K, int q, int C, bool in_kernel_sampling);
int prepare_kernels(const Variant &v, int K, int q, int C, bool mixed_q, bool *can_sample_in_kernel);
const Variant *variant_table(int *count);

}  // namespace gbmuf
