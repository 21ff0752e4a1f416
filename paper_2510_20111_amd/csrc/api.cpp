// Argument checking of the kernel-launching entry points of libhzp.  Everything that could make
// a kernel read or write outside a caller's buffer is rejected here with a status code: the
// kernels themselves trust their arguments.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstring>
#include <vector>

#include "hzp_internal.hpp"

namespace hzp {

static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace hzp

using namespace hzp;

extern "C" hzp_status_t hzp_reduce_shard(const hzp_plan_t *plan, uint32_t layer, uint32_t cls, int level,
                                         uint32_t rank, const void *const *grad_slices, uint32_t R,
                                         uint32_t grad_dtype, float scale, int accumulate, float *out_f32,
                                         hipStream_t stream)
{
    if (!plan || !grad_slices || !out_f32)
        return fail(HZP_ERR_INVALID_ARG, "hzp_reduce_shard: NULL plan, slice array or output");
    const BucketRec *b = find_bucket(plan, layer, cls);
    if (!b) return fail(HZP_ERR_RANGE, "hzp_reduce_shard: no bucket (layer %u, class %u)", layer, cls);
    if (rank >= plan->world) return fail(HZP_ERR_RANGE, "hzp_reduce_shard: rank %u of %u", rank, plan->world);
    if (level < 1 || level > 3)
        return fail(HZP_ERR_RANGE, "hzp_reduce_shard: level %d is not 1, 2 or 3", level);
    if (grad_dtype > HZP_GRAD_F32)
        return fail(HZP_ERR_INVALID_ARG, "hzp_reduce_shard: unknown gradient type %u", grad_dtype);
    if (R == 0) return fail(HZP_ERR_INVALID_ARG, "hzp_reduce_shard: R must be at least 1");
    if (R > HZP_MAX_REPLICAS)
        return fail(HZP_ERR_UNSUPPORTED, "hzp_reduce_shard: R=%u exceeds %u", R, HZP_MAX_REPLICAS);
    const uint64_t n = level == 1 ? b->S1 : level == 2 ? b->S2 : b->S3;
    if (n >= (1ull << 30)) return fail(HZP_ERR_UNSUPPORTED, "hzp_reduce_shard: shard of 2^30 elements or more");
    for (uint32_t r = 0; r < R; ++r) {
        if (!grad_slices[r]) return fail(HZP_ERR_INVALID_ARG, "hzp_reduce_shard: slice %u is NULL", r);
        if (!aligned16(grad_slices[r]))
            return fail(HZP_ERR_ALIGN, "hzp_reduce_shard: slice %u is not 16-byte aligned", r);
    }
    if (!aligned16(out_f32)) return fail(HZP_ERR_ALIGN, "hzp_reduce_shard: output is not 16-byte aligned");
    const bool g32 = grad_dtype == HZP_GRAD_DEFAULT ? cls == HZP_CLASS_F32 : grad_dtype == HZP_GRAD_F32;
    return launch_reduce(g32, grad_slices, R, n, scale, accumulate, out_f32, stream);
}

// The step's scalars as the kernels take them; the bias corrections are formed in double.
static AdamScalars derive_scalars(const hzp_adamw_t &hy)
{
    AdamScalars h;
    h.lr = hy.lr;
    h.beta1 = hy.beta1;
    h.beta2 = hy.beta2;
    h.one_minus_beta1 = 1.0f - hy.beta1;
    h.one_minus_beta2 = 1.0f - hy.beta2;
    h.eps = hy.eps;
    h.weight_decay = hy.weight_decay;
    h.grad_scale = hy.grad_scale;
    h.inv_bc1 = (float)(1.0 / (1.0 - std::pow((double)hy.beta1, (double)hy.step)));
    h.inv_bc2 = (float)(1.0 / (1.0 - std::pow((double)hy.beta2, (double)hy.step)));
    return h;
}

// Argument checks and segment list shared by the two forms of the update; `hy` or `scalars_dev` is given.
static hzp_status_t adamw_shard(const char *who, const hzp_plan_t *plan, uint32_t layer_begin, uint32_t layer_end,
                                uint32_t cls, uint32_t rank, const hzp_adamw_t *hy,
                                const hzp_adamw_scalars_t *scalars_dev, const void *const *grad_slices, uint32_t R,
                                float *const *master, float *const *m, float *const *v, void *const *param_out,
                                hipStream_t stream)
{
    if (!plan || (!hy && !scalars_dev) || !grad_slices || !master || !m || !v)
        return fail(HZP_ERR_INVALID_ARG, "%s: NULL plan, hyper-parameters or pointer array", who);
    if (layer_begin >= layer_end)
        return fail(HZP_ERR_INVALID_ARG, "%s: empty layer range [%u, %u)", who, layer_begin, layer_end);
    if (layer_end > plan->n_layers)
        return fail(HZP_ERR_RANGE, "%s: layer_end %u of %u", who, layer_end, plan->n_layers);
    if (cls > 1) return fail(HZP_ERR_RANGE, "%s: class %u", who, cls);
    if (rank >= plan->world) return fail(HZP_ERR_RANGE, "%s: rank %u of %u", who, rank, plan->world);
    if (hy && hy->step == 0) return fail(HZP_ERR_INVALID_ARG, "%s: step is 1-based", who);
    if (scalars_dev && !aligned16(scalars_dev))
        return fail(HZP_ERR_ALIGN, "%s: the scalars are not 16-byte aligned", who);
    if (R > HZP_MAX_REPLICAS)
        return fail(HZP_ERR_UNSUPPORTED, "%s: R=%u exceeds %u", who, R, HZP_MAX_REPLICAS);
    const bool prereduced = (R == 0);
    const uint32_t per_layer = prereduced ? 1u : R;
    const bool g32 = prereduced || cls == HZP_CLASS_F32;
    const bool o32 = cls == HZP_CLASS_F32;
    const uint64_t shard_index = level_index(plan, 1, rank);

    std::vector<FusedSegment> segs;
    try {
        segs.reserve(layer_end - layer_begin);
    } catch (const std::bad_alloc &) {
        return fail(HZP_ERR_NOMEM, "%s: out of host memory", who);
    }
    for (uint32_t layer = layer_begin; layer < layer_end; ++layer) {
        const BucketRec *b = find_bucket(plan, layer, cls);
        if (!b) continue;                       // this layer has no tensor of the class
        const size_t idx = layer - layer_begin;
        FusedSegment f{};
        f.grads = grad_slices + idx * per_layer;
        f.master = master[idx];
        f.m = m[idx];
        f.v = v[idx];
        f.out = param_out ? param_out[idx] : nullptr;
        f.n = b->S1;
        f.first_slot = b->first_slot;
        f.n_tensors = b->n_tensors;
        f.shard_begin = shard_index * b->S1;
        if (f.n >= (1ull << 30))
            return fail(HZP_ERR_UNSUPPORTED, "%s: layer %u: shard of 2^30 elements or more", who, layer);
        if (!f.master || !f.m || !f.v)
            return fail(HZP_ERR_INVALID_ARG, "%s: layer %u: NULL state pointer", who, layer);
        if (!aligned16(f.master) || !aligned16(f.m) || !aligned16(f.v) || !aligned16(f.out))
            return fail(HZP_ERR_ALIGN, "%s: layer %u: state or output not 16-byte aligned", who, layer);
        if (param_out && !f.out)
            return fail(HZP_ERR_INVALID_ARG, "%s: layer %u: NULL output pointer", who, layer);
        for (uint32_t r = 0; r < per_layer; ++r) {
            if (!f.grads[r])
                return fail(HZP_ERR_INVALID_ARG, "%s: layer %u: slice %u is NULL", who, layer, r);
            if (!aligned16(f.grads[r]))
                return fail(HZP_ERR_ALIGN, "%s: layer %u: slice %u not 16-byte aligned", who, layer, r);
        }
        segs.push_back(f);
    }
    if (segs.empty()) return HZP_OK;
    if (hy) return launch_fused(plan, g32, o32, per_layer, segs.data(), segs.size(), derive_scalars(*hy), stream);
    return launch_fused_dev(plan, g32, o32, per_layer, segs.data(), segs.size(),
                            reinterpret_cast<const AdamScalars *>(scalars_dev), stream);
}

extern "C" hzp_status_t hzp_adamw_shard(const hzp_plan_t *plan, uint32_t layer_begin, uint32_t layer_end,
                                        uint32_t cls, uint32_t rank, const hzp_adamw_t *hy,
                                        const void *const *grad_slices, uint32_t R, float *const *master,
                                        float *const *m, float *const *v, void *const *param_out,
                                        hipStream_t stream)
{
    return adamw_shard("hzp_adamw_shard", plan, layer_begin, layer_end, cls, rank, hy, nullptr, grad_slices, R, master, m,
                       v, param_out, stream);
}

extern "C" hzp_status_t hzp_adamw_scalars(const hzp_adamw_t *hy, hzp_adamw_scalars_t *out)
{
    if (!hy || !out) return fail(HZP_ERR_INVALID_ARG, "hzp_adamw_scalars: NULL argument");
    if (hy->step == 0) return fail(HZP_ERR_INVALID_ARG, "hzp_adamw_scalars: step is 1-based");
    const AdamScalars h = derive_scalars(*hy);
    std::memset(out, 0, sizeof *out);
    std::memcpy(out, &h, sizeof h);
    return HZP_OK;
}

extern "C" hzp_status_t hzp_adamw_shard_dev(const hzp_plan_t *plan, uint32_t layer_begin, uint32_t layer_end,
                                            uint32_t cls, uint32_t rank, const hzp_adamw_scalars_t *scalars,
                                            const void *const *grad_slices, uint32_t R, float *const *master,
                                            float *const *m, float *const *v, void *const *param_out,
                                            hipStream_t stream)
{
    if (!scalars) return fail(HZP_ERR_INVALID_ARG, "hzp_adamw_shard_dev: NULL scalars");
    return adamw_shard("hzp_adamw_shard_dev", plan, layer_begin, layer_end, cls, rank, nullptr, scalars, grad_slices, R,
                       master, m, v, param_out, stream);
}

extern "C" hzp_status_t hzp_gather_layer(const hzp_plan_t *plan, uint32_t layer, uint32_t cls, int level,
                                         const void *const *shard_ptrs, uint32_t n_shards, void *bucket_out,
                                         void *const *tensor_out, hipStream_t stream)
{
    if (!plan || !shard_ptrs) return fail(HZP_ERR_INVALID_ARG, "hzp_gather_layer: NULL plan or shard array");
    const BucketRec *b = find_bucket(plan, layer, cls);
    if (!b) return fail(HZP_ERR_RANGE, "hzp_gather_layer: no bucket (layer %u, class %u)", layer, cls);
    if (level != 1 && level != 3)
        return fail(HZP_ERR_RANGE, "hzp_gather_layer: level %d is neither 1 nor 3", level);
    if (level == 1 && plan->K == 0)
        return fail(HZP_ERR_UNSUPPORTED, "hzp_gather_layer: z3=%u does not divide z1=%u; use hzp_gather_shard",
                    plan->z3, plan->z1);
    const uint32_t want = level == 1 ? plan->K : plan->z3;
    if (n_shards != want)
        return fail(HZP_ERR_INVALID_ARG, "hzp_gather_layer: level %d takes %u shards, got %u", level, want,
                    n_shards);
    if (n_shards > HZP_MAX_GROUP)
        return fail(HZP_ERR_UNSUPPORTED, "hzp_gather_layer: %u shards exceed %u", n_shards, HZP_MAX_GROUP);
    if (level == 1 && tensor_out)
        return fail(HZP_ERR_INVALID_ARG, "hzp_gather_layer: tensor_out is a level-3 output");
    if (!bucket_out && !tensor_out) return fail(HZP_ERR_INVALID_ARG, "hzp_gather_layer: no output given");
    const uint32_t es = cls == HZP_CLASS_F32 ? 4u : 2u;
    for (uint32_t s = 0; s < n_shards; ++s) {
        if (!shard_ptrs[s]) return fail(HZP_ERR_INVALID_ARG, "hzp_gather_layer: shard %u is NULL", s);
        if (!aligned16(shard_ptrs[s]))
            return fail(HZP_ERR_ALIGN, "hzp_gather_layer: shard %u is not 16-byte aligned", s);
    }
    if (!aligned16(bucket_out)) return fail(HZP_ERR_ALIGN, "hzp_gather_layer: bucket_out is not 16-byte aligned");
    if (tensor_out)
        for (uint32_t t = 0; t < b->n_tensors; ++t) {
            if (!tensor_out[t]) return fail(HZP_ERR_INVALID_ARG, "hzp_gather_layer: tensor_out[%u] is NULL", t);
            if (reinterpret_cast<uintptr_t>(tensor_out[t]) % es)
                return fail(HZP_ERR_ALIGN, "hzp_gather_layer: tensor_out[%u] is not element-aligned", t);
        }
    const uint64_t len = level == 1 ? b->S1 : b->S3;
    if (bucket_out) {
        hzp_status_t st = launch_concat(shard_ptrs, n_shards, len * es, bucket_out, stream);
        if (st != HZP_OK) return st;
    }
    if (tensor_out) return launch_unpack(plan, *b, shard_ptrs, n_shards, tensor_out, 0, b->n_tensors, stream);
    return HZP_OK;
}

extern "C" hzp_status_t hzp_gather_layer_static(const hzp_plan_t *plan, uint32_t layer, uint32_t cls,
                                                const void *const *shard_ptrs, uint32_t n_shards,
                                                void *const *tensor_out, hipStream_t stream)
{
    if (!plan || !shard_ptrs || !tensor_out)
        return fail(HZP_ERR_INVALID_ARG, "hzp_gather_layer_static: NULL plan, shard array or tensor array");
    const BucketRec *b = find_bucket(plan, layer, cls);
    if (!b) return fail(HZP_ERR_RANGE, "hzp_gather_layer_static: no bucket (layer %u, class %u)", layer, cls);
    if (n_shards != plan->z3)
        return fail(HZP_ERR_INVALID_ARG, "hzp_gather_layer_static: takes %u shards, got %u", plan->z3, n_shards);
    if (n_shards > HZP_MAX_GROUP)
        return fail(HZP_ERR_UNSUPPORTED, "hzp_gather_layer_static: %u shards exceed %u", n_shards, HZP_MAX_GROUP);
    const uint32_t es = cls == HZP_CLASS_F32 ? 4u : 2u;
    for (uint32_t s = 0; s < n_shards; ++s) {
        if (!shard_ptrs[s]) return fail(HZP_ERR_INVALID_ARG, "hzp_gather_layer_static: shard %u is NULL", s);
        if (!aligned16(shard_ptrs[s]))
            return fail(HZP_ERR_ALIGN, "hzp_gather_layer_static: shard %u is not 16-byte aligned", s);
    }
    for (uint32_t t = 0; t < b->n_tensors; ++t) {
        if (!tensor_out[t]) return fail(HZP_ERR_INVALID_ARG, "hzp_gather_layer_static: tensor_out[%u] is NULL", t);
        if (reinterpret_cast<uintptr_t>(tensor_out[t]) % es)
            return fail(HZP_ERR_ALIGN, "hzp_gather_layer_static: tensor_out[%u] is not element-aligned", t);
    }
    if (b->pieces.size() > HZP_STATIC_MAX_PIECES)
        return fail(HZP_ERR_UNSUPPORTED,
                    "hzp_gather_layer_static: the bucket has %zu tensor pieces, the fixed table holds %u; "
                    "use hzp_gather_layer",
                    b->pieces.size(), (unsigned)HZP_STATIC_MAX_PIECES);
    return launch_unpack_static(*b, shard_ptrs, n_shards, tensor_out, stream);
}

extern "C" hzp_status_t hzp_gather_shard(const hzp_plan_t *plan, uint32_t layer, uint32_t cls, uint32_t j,
                                         const void *const *owner_ptrs, uint32_t n_owners, void *shard_out,
                                         hipStream_t stream)
{
    if (!plan || !owner_ptrs || !shard_out)
        return fail(HZP_ERR_INVALID_ARG, "hzp_gather_shard: NULL plan, owner array or output");
    const BucketRec *b = find_bucket(plan, layer, cls);
    if (!b) return fail(HZP_ERR_RANGE, "hzp_gather_shard: no bucket (layer %u, class %u)", layer, cls);
    if (j >= plan->z3) return fail(HZP_ERR_RANGE, "hzp_gather_shard: shard %u of %u", j, plan->z3);
    const uint64_t lo3 = j * b->S3, hi3 = lo3 + b->S3;
    const uint64_t first = lo3 / b->S1, want = (hi3 + b->S1 - 1) / b->S1 - first;
    if (n_owners != want)
        return fail(HZP_ERR_INVALID_ARG, "hzp_gather_shard: shard %u is covered by %llu ZeRO-1 shards, got %u", j,
                    (unsigned long long)want, n_owners);
    if (n_owners > HZP_MAX_GROUP)
        return fail(HZP_ERR_UNSUPPORTED, "hzp_gather_shard: %u owners exceed %u", n_owners, HZP_MAX_GROUP);
    if (!aligned16(shard_out)) return fail(HZP_ERR_ALIGN, "hzp_gather_shard: shard_out is not 16-byte aligned");
    const uint32_t es = cls == HZP_CLASS_F32 ? 4u : 2u;
    const void *src[HZP_MAX_GROUP];
    uint64_t dst_off[HZP_MAX_GROUP], bytes[HZP_MAX_GROUP];
    for (uint32_t q = 0; q < n_owners; ++q) {
        if (!owner_ptrs[q]) return fail(HZP_ERR_INVALID_ARG, "hzp_gather_shard: owner %u is NULL", q);
        if (!aligned16(owner_ptrs[q]))
            return fail(HZP_ERR_ALIGN, "hzp_gather_shard: owner %u is not 16-byte aligned", q);
        // [lo, hi) = the part of ZeRO-1 shard first+q inside shard j; S1, S3 are multiples of A >= 8
        // elements, so every offset below is a multiple of 16 bytes
        const uint64_t lo1 = (first + q) * b->S1;
        const uint64_t lo = lo1 > lo3 ? lo1 : lo3, hi = lo1 + b->S1 < hi3 ? lo1 + b->S1 : hi3;
        src[q] = static_cast<const char *>(owner_ptrs[q]) + (lo - lo1) * es;
        dst_off[q] = (lo - lo3) * es;
        bytes[q] = (hi - lo) * es;
    }
    return launch_concat_ranges(src, dst_off, bytes, n_owners, shard_out, stream);
}

extern "C" hzp_status_t hzp_gather_tensor(const hzp_plan_t *plan, uint32_t tensor_id,
                                          const void *const *shard_ptrs, uint32_t n_shards, void *tensor_out,
                                          hipStream_t stream)
{
    if (!plan || !shard_ptrs || !tensor_out)
        return fail(HZP_ERR_INVALID_ARG, "hzp_gather_tensor: NULL plan, shard array or output");
    if (tensor_id >= plan->tensors.size())
        return fail(HZP_ERR_RANGE, "hzp_gather_tensor: tensor %u of %zu", tensor_id, plan->tensors.size());
    const TensorRec &t = plan->tensors[tensor_id];
    const BucketRec &b = plan->buckets[t.bucket];
    if (n_shards != plan->z3)
        return fail(HZP_ERR_INVALID_ARG, "hzp_gather_tensor: takes %u shards, got %u", plan->z3, n_shards);
    if (n_shards > HZP_MAX_GROUP)
        return fail(HZP_ERR_UNSUPPORTED, "hzp_gather_tensor: %u shards exceed %u", n_shards, HZP_MAX_GROUP);
    const uint32_t es = t.cls == HZP_CLASS_F32 ? 4u : 2u;
    if (reinterpret_cast<uintptr_t>(tensor_out) % es)
        return fail(HZP_ERR_ALIGN, "hzp_gather_tensor: tensor_out is not element-aligned");
    // Only the shards that hold a part of the tensor are read; the other entries are not touched.
    const uint64_t j0 = t.offset / b.S3, j1 = (t.offset + t.numel - 1) / b.S3;
    const void *sh[HZP_MAX_GROUP] = {};
    for (uint64_t j = j0; j <= j1; ++j) {
        if (!shard_ptrs[j]) return fail(HZP_ERR_INVALID_ARG, "hzp_gather_tensor: shard %llu is NULL", (unsigned long long)j);
        if (!aligned16(shard_ptrs[j]))
            return fail(HZP_ERR_ALIGN, "hzp_gather_tensor: shard %llu is not 16-byte aligned", (unsigned long long)j);
        sh[j] = shard_ptrs[j];
    }
    void *out[1] = {tensor_out};
    return launch_unpack(plan, b, sh, n_shards, out, t.index_in_bucket, t.index_in_bucket + 1, stream);
}

extern "C" hzp_status_t hzp_gather_layers(const hzp_plan_t *plan, uint32_t layer_begin, uint32_t layer_end,
                                          uint32_t cls, int level, const void *const *shard_ptrs,
                                          uint32_t n_shards, void *const *bucket_out, hipStream_t stream)
{
    if (!plan || !shard_ptrs || !bucket_out)
        return fail(HZP_ERR_INVALID_ARG, "hzp_gather_layers: NULL plan, shard array or output array");
    if (layer_begin >= layer_end)
        return fail(HZP_ERR_INVALID_ARG, "hzp_gather_layers: empty layer range [%u, %u)", layer_begin, layer_end);
    if (layer_end > plan->n_layers)
        return fail(HZP_ERR_RANGE, "hzp_gather_layers: layer_end %u of %u", layer_end, plan->n_layers);
    if (cls > 1) return fail(HZP_ERR_RANGE, "hzp_gather_layers: class %u", cls);
    if (level != 1 && level != 3)
        return fail(HZP_ERR_RANGE, "hzp_gather_layers: level %d is neither 1 nor 3", level);
    if (level == 1 && plan->K == 0)
        return fail(HZP_ERR_UNSUPPORTED, "hzp_gather_layers: z3=%u does not divide z1=%u; use hzp_gather_shard",
                    plan->z3, plan->z1);
    const uint32_t want = level == 1 ? plan->K : plan->z3;
    if (n_shards != want)
        return fail(HZP_ERR_INVALID_ARG, "hzp_gather_layers: level %d takes %u shards per layer, got %u", level,
                    want, n_shards);
    if (n_shards > HZP_MAX_GROUP)
        return fail(HZP_ERR_UNSUPPORTED, "hzp_gather_layers: %u shards exceed %u", n_shards, HZP_MAX_GROUP);
    const uint32_t es = cls == HZP_CLASS_F32 ? 4u : 2u;
    std::vector<const void *> src;
    std::vector<void *> dst;
    std::vector<uint64_t> bytes;
    try {
        for (uint32_t layer = layer_begin; layer < layer_end; ++layer) {
            const BucketRec *b = find_bucket(plan, layer, cls);
            if (!b) continue;                   // this layer has no tensor of the class
            const size_t idx = layer - layer_begin;
            if (!bucket_out[idx]) return fail(HZP_ERR_INVALID_ARG, "hzp_gather_layers: layer %u: NULL output", layer);
            if (!aligned16(bucket_out[idx]))
                return fail(HZP_ERR_ALIGN, "hzp_gather_layers: layer %u: output not 16-byte aligned", layer);
            for (uint32_t s = 0; s < n_shards; ++s) {
                const void *p = shard_ptrs[idx * n_shards + s];
                if (!p) return fail(HZP_ERR_INVALID_ARG, "hzp_gather_layers: layer %u: shard %u is NULL", layer, s);
                if (!aligned16(p))
                    return fail(HZP_ERR_ALIGN, "hzp_gather_layers: layer %u: shard %u not 16-byte aligned", layer, s);
                src.push_back(p);
            }
            dst.push_back(bucket_out[idx]);
            bytes.push_back((level == 1 ? b->S1 : b->S3) * es);
        }
    } catch (const std::bad_alloc &) {
        return fail(HZP_ERR_NOMEM, "hzp_gather_layers: out of host memory");
    }
    if (dst.empty()) return HZP_OK;
    return launch_concat_layers(src.data(), n_shards, bytes.data(), dst.data(), (uint32_t)dst.size(), stream);
}

// Times the fused update of all layers under every arena layout variant that fits the caller's
// allocation and reports the fastest.  Each variant's streams are filled with ordinary non-zero
// values first (on all-zero gradients and states the update runs 1-3 % faster than on any others,
// and then shows less of the differences between the variants); the arena is all zero afterwards.
extern "C" hzp_status_t hzp_arena_tune(const hzp_plan_t *plan, uint32_t cls, uint32_t rank, uint32_t R, void *arena,
                                       uint64_t arena_bytes, hipStream_t stream, uint32_t *best_variant,
                                       double *seconds)
{
    if (!plan || !arena || !best_variant) return fail(HZP_ERR_INVALID_ARG, "hzp_arena_tune: NULL plan, arena or output");
    if (cls > 1) return fail(HZP_ERR_RANGE, "hzp_arena_tune: class %u", cls);
    if (rank >= plan->world) return fail(HZP_ERR_RANGE, "hzp_arena_tune: rank %u of %u", rank, plan->world);
    if (R == 0) return fail(HZP_ERR_INVALID_ARG, "hzp_arena_tune: R must be at least 1 (the arena holds no reduced gradient)");
    if (R > HZP_MAX_REPLICAS) return fail(HZP_ERR_UNSUPPORTED, "hzp_arena_tune: R=%u exceeds %u", R, HZP_MAX_REPLICAS);
    if (reinterpret_cast<uintptr_t>(arena) % HZP_ARENA_ALIGN)
        return fail(HZP_ERR_ALIGN, "hzp_arena_tune: the arena does not start on a multiple of %u bytes", HZP_ARENA_ALIGN);
    uint64_t total[HZP_ARENA_VARIANTS];
    for (uint32_t v = 0; v < HZP_ARENA_VARIANTS; ++v) {
        const hzp_status_t st = hzp_plan_arena(plan, cls, R, HZP_GRAD_DEFAULT, v, &total[v]);
        if (st != HZP_OK) return st;
        if (seconds) seconds[v] = 0.0;
    }
    if (arena_bytes < total[0])
        return fail(HZP_ERR_INVALID_ARG, "hzp_arena_tune: %llu bytes do not hold variant 0 (%llu bytes)",
                    (unsigned long long)arena_bytes, (unsigned long long)total[0]);

    const uint32_t L = plan->n_layers;
    const uint32_t n_streams = R + 4;           // the update's: R gradient streams, master, m, v, cast parameters
    std::vector<const void *> g;
    std::vector<float *> p, m, v;
    std::vector<void *> out;
    std::vector<uint64_t> lo, hi;               // byte range of each of the update's streams
    try {
        g.resize((size_t)L * R);
        p.resize(L);
        m.resize(L);
        v.resize(L);
        out.resize(L);
        lo.resize(n_streams);
        hi.resize(n_streams);
    } catch (const std::bad_alloc &) {
        return fail(HZP_ERR_NOMEM, "hzp_arena_tune: out of host memory");
    }
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e = hipMemsetAsync(arena, 0, arena_bytes, stream);
    if (e == hipSuccess) e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    hzp_status_t st = HZP_OK;
    const hzp_adamw_t hy = {1e-4f, 0.9f, 0.95f, 1e-8f, 0.1f, 1.0f / (float)R, 1u};
    const int warm = 1, reps = 3;
    double best = 0.0, first = 0.0;
    bool any = false;
    char *const base = static_cast<char *>(arena);
    for (uint32_t var = 0; var < HZP_ARENA_VARIANTS && e == hipSuccess && st == HZP_OK; ++var) {
        if (total[var] > arena_bytes) continue;
        for (uint32_t s = 0; s < n_streams; ++s) {
            lo[s] = ~0ull;
            hi[s] = 0;
        }
        for (uint32_t layer = 0; layer < L && st == HZP_OK; ++layer) {
            if (!find_bucket(plan, layer, cls)) continue;         // its entries are never read
            for (uint32_t s = 0; s < n_streams && st == HZP_OK; ++s) {
                uint64_t off = 0, n = 0;
                const uint32_t kind = s < R ? (uint32_t)HZP_STREAM_GRAD : HZP_STREAM_MASTER + (s - R);
                st = hzp_plan_arena_slice(plan, cls, R, HZP_GRAD_DEFAULT, var, kind, s < R ? s : 0, layer, &off, &n);
                if (st != HZP_OK) break;
                if (off < lo[s]) lo[s] = off;
                if (off + n > hi[s]) hi[s] = off + n;
                if (s < R)
                    g[(size_t)layer * R + s] = base + off;
                else if (s == R)
                    p[layer] = reinterpret_cast<float *>(base + off);
                else if (s == R + 1)
                    m[layer] = reinterpret_cast<float *>(base + off);
                else if (s == R + 2)
                    v[layer] = reinterpret_cast<float *>(base + off);
                else
                    out[layer] = base + off;
            }
        }
        // gradients 7e-4 (bf16 0x3A3A; as fp32 the same bytes are 7.1e-4), parameters 0.02, the rest zero
        for (uint32_t s = 0; s < n_streams && st == HZP_OK && e == hipSuccess; ++s) {
            if (s < R)
                e = hipMemsetAsync(base + lo[s], 0x3A, hi[s] - lo[s], stream);
            else if (s == R)
                e = hipMemsetD32Async(reinterpret_cast<hipDeviceptr_t>(base + lo[s]), 0x3CA3D70A, (hi[s] - lo[s]) / 4, stream);
            else
                e = hipMemsetAsync(base + lo[s], 0, hi[s] - lo[s], stream);
        }
        for (int i = 0; i < warm + reps && st == HZP_OK && e == hipSuccess; ++i) {
            if (i == warm) e = hipEventRecord(e0, stream);
            if (e == hipSuccess)
                st = hzp_adamw_shard(plan, 0, L, cls, rank, &hy, g.data(), R, p.data(), m.data(), v.data(), out.data(), stream);
        }
        if (st != HZP_OK || e != hipSuccess) break;
        e = hipEventRecord(e1, stream);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e != hipSuccess) break;
        const double sec = (double)ms * 1e-3 / reps;
        if (seconds) seconds[var] = sec;
        if (var == 0) first = sec;
        // another variant has to beat the default by more than the measurement's repeatability
        if (!any || (sec < best && sec < 0.995 * first)) {
            best = sec;
            *best_variant = var;
            any = true;
        }
    }
    if (e == hipSuccess) e = hipMemsetAsync(arena, 0, arena_bytes, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (st != HZP_OK) return st;
    if (e != hipSuccess) return fail(HZP_ERR_HIP, "hzp_arena_tune: %s", hipGetErrorString(e));
    return HZP_OK;
}
