// Internal declarations shared by the host sources of libhzp (not part of the ABI).
#pragma once

#include <cstdint>
#include <mutex>
#include <vector>

#include "hzp.h"

namespace hzp {

// Set the calling thread's error text and hand the status back.
hzp_status_t fail(hzp_status_t st, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

struct TensorRec {
    uint32_t layer;
    uint32_t cls;
    uint32_t bucket;
    uint32_t index_in_bucket;
    uint64_t offset;
    uint64_t numel;
    float wd_mult;
};

// A maximal run of one tensor that lies inside one ZeRO-3 shard.  The unpack kernel walks
// pieces in fixed-size chunks; `chunk_begin` is the running chunk count before this piece.
struct Piece {
    uint64_t src_off;       // element offset inside shard `shard`
    uint64_t dst_off;       // element offset inside the tensor
    uint64_t len;           // elements
    uint32_t shard;         // ZeRO-3 index j
    uint32_t tensor;        // index in bucket
    uint32_t chunk_begin;
    uint32_t pad_;
};

struct BucketRec {
    uint32_t layer;
    uint32_t cls;
    uint32_t first_slot;    // first entry of this bucket in the per-bucket-ordered tables
    uint32_t n_tensors;
    uint64_t payload_end, P, S3, S2, S1, base;
    std::vector<uint32_t> tensor_ids;
    std::vector<Piece> pieces;
    uint32_t n_chunks;
    uint32_t piece_slot;    // first entry of this bucket in the device piece table
};

// Lookup tables of one plan on one device.
struct DeviceTables {
    int device = -1;
    uint64_t *tensor_off = nullptr;     // [n_tensors] bucket-relative offsets, bucket after bucket
    float *tensor_wd = nullptr;         // [n_tensors] weight-decay multipliers, same order
    Piece *pieces = nullptr;            // all buckets' pieces, bucket after bucket
    uint32_t *piece_chunk = nullptr;    // chunk_begin of the same pieces, densely packed
};

#ifndef HZP_UNPACK_CHUNK
#define HZP_UNPACK_CHUNK 1024
#endif
constexpr uint32_t kUnpackChunk = HZP_UNPACK_CHUNK;   // elements one wavefront moves per chunk

}  // namespace hzp

struct hzp_plan {
    uint32_t n_layers, align, z3, z2, z1;
    uint32_t K;                                 // Z1/Z3, or 0 when Z3 does not divide Z1
    uint32_t world;                             // lcm(Z1, Z2, Z3): ranks are 0 .. world-1
    uint64_t total_padded;
    bool uniform_wd;                            // every multiplier is 1: no table lookups
    std::vector<hzp::TensorRec> tensors;        // by tensor id
    std::vector<hzp::BucketRec> buckets;        // by (layer, class)
    std::vector<int32_t> bucket_of;             // [layer*2 + cls] -> bucket index or -1
    std::vector<uint64_t> slot_off;             // per-bucket-ordered copies for the device
    std::vector<float> slot_wd;
    mutable std::mutex mu;
    mutable std::vector<hzp::DeviceTables> dev; // one entry per device that has used the plan
};

namespace hzp {
const BucketRec *find_bucket(const hzp_plan_t *plan, uint32_t layer, uint32_t cls);
// Index of the shard that `rank` (< plan->world) owns at `level` (1, 2 or 3).
uint32_t level_index(const hzp_plan_t *plan, int level, uint32_t rank);

// One shard segment (one layer bucket) of a fused update call.
struct FusedSegment {
    const void *const *grads;   // R device pointers (host array)
    float *master, *m, *v;
    void *out;                  // nullable
    uint64_t n;                 // elements, a multiple of 8
    uint32_t first_slot, n_tensors;     // the bucket's rows in the weight-decay tables
    uint64_t shard_begin;       // bucket position of element 0
};

// The scalars of one step as the update kernels take them.
struct AdamScalars {
    float lr, beta1, beta2, one_minus_beta1, one_minus_beta2, eps, weight_decay, grad_scale;
    float inv_bc1, inv_bc2;     // 1/(1-beta1^t), 1/(1-beta2^t), computed in double on the host
};
static_assert(sizeof(AdamScalars) <= sizeof(hzp_adamw_scalars_t), "the public block holds the scalars");

// Launchers; their arguments have been validated by the entry points.
hzp_status_t launch_reduce(bool g32, const void *const *slices, uint32_t R, uint64_t n, float scale,
                           int accumulate, float *out, hipStream_t stream);
hzp_status_t launch_fused(const hzp_plan_t *plan, bool g32, bool o32, uint32_t R, const FusedSegment *segs,
                          size_t nseg, const AdamScalars &h, hipStream_t stream);
// The same with the step's scalars read from device memory at run time (as packed by pack_scalars).
hzp_status_t launch_fused_dev(const hzp_plan_t *plan, bool g32, bool o32, uint32_t R, const FusedSegment *segs,
                              size_t nseg, const AdamScalars *scalars_dev, hipStream_t stream);
hzp_status_t launch_concat(const void *const *srcs, uint32_t n_shards, uint64_t bytes_per_shard, void *dst,
                           hipStream_t stream);
// Concatenates `per_layer` equal pieces for each of n_layers layers; srcs[l*per_layer + k], dsts[l].
hzp_status_t launch_concat_layers(const void *const *srcs, uint32_t per_layer, const uint64_t *bytes_per_piece,
                                  void *const *dsts, uint32_t n_layers, hipStream_t stream);
// Copies n pieces of different lengths: piece s goes from srcs[s] to dst + dst_off[s] (bytes, all
// multiples of 16).
hzp_status_t launch_concat_ranges(const void *const *srcs, const uint64_t *dst_off, const uint64_t *bytes,
                                  uint32_t n, void *dst, hipStream_t stream);
// Unpacks tensors [t_begin, t_end) of the bucket (indices in the bucket); tensors[0] is t_begin's.
hzp_status_t launch_unpack(const hzp_plan_t *plan, const BucketRec &b, const void *const *shards,
                           uint32_t n_shards, void *const *tensors, uint32_t t_begin, uint32_t t_end,
                           hipStream_t stream);
// The same for all tensors of the bucket with the piece table in the library's fixed device array
// (no allocation, no copy call); refuses buckets with more than HZP_STATIC_MAX_PIECES pieces.
hzp_status_t launch_unpack_static(const BucketRec &b, const void *const *shards, uint32_t n_shards,
                                  void *const *tensors, hipStream_t stream);
// Tables for the current device (creates them on first use).  Defined with the launchers.
hzp_status_t device_tables(const hzp_plan_t *plan, const DeviceTables **out);
void free_device_tables(hzp_plan_t *plan);
}  // namespace hzp
