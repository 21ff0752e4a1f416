/*
 * hzp.h -- C ABI of libhzp: the one-GPU share of the data-parallel hot path of
 * Asynchronous Hierarchical ZeRO Parallelism (AsyncHZP) on AMD CDNA4 (gfx950).
 *
 * Each training step a rank (1) sums the gradient contributions that land on its
 * shard, (2) applies Adam with decoupled weight decay to its ZeRO-1 shard of
 * fp32 master weights / momentum / variance and casts the result to bf16, and
 * (3) rebuilds bf16 parameter buffers out of the hierarchical ZeRO-1 / ZeRO-3
 * layout.  The contributions of other ranks are buffers that already sit in this
 * GPU's memory; no collective is issued here.
 *
 * Conventions for every entry point
 *   - returns an hzp_status_t; never throws, aborts or synchronises the device;
 *     hzp_last_error() gives a thread-local text for the last non-OK status;
 *   - "device pointer": memory the current HIP device can address; "host array":
 *     ordinary host memory read during the call and not retained;
 *   - all device buffers are owned by the caller.  The library allocates device
 *     memory only for small per-plan lookup tables, created by hzp_plan_prepare
 *     (or, without it, by the first call that needs them: that one call blocks)
 *     and freed by hzp_plan_free, and for a scheduler's pool;
 *   - kernel work is enqueued on the given stream and the call returns at once;
 *     a plan is immutable and may be used from several host threads and streams
 *     at the same time (the paper issues these operations from extra threads on
 *     dedicated streams, Section 4.2);
 *   - bf16 buffers hold 16-bit patterns (upper half of an IEEE binary32).
 */
#ifndef HZP_H
#define HZP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Same declaration as the HIP runtime's; repeated so that this header needs no HIP include. */
typedef struct ihipStream_t *hipStream_t;

typedef struct hzp_plan hzp_plan_t;     /* opaque, host-side, immutable */

typedef enum {
    HZP_OK = 0,
    HZP_ERR_INVALID_ARG = 1,    /* NULL where a pointer is required, inconsistent counts, step 0 ... */
    HZP_ERR_RANGE = 2,          /* layer / rank / tensor id / level outside the plan */
    HZP_ERR_UNSUPPORTED = 3,    /* a valid request this build does not cover (e.g. more than 32 contributions) */
    HZP_ERR_ALIGN = 4,          /* a device pointer is not aligned as the entry point requires */
    HZP_ERR_NOMEM = 5,          /* host or device allocation failed; a full scheduler pool; no group sizes fit */
    HZP_ERR_HIP = 6             /* a HIP runtime call or a kernel launch failed */
} hzp_status_t;

/* Parameter / gradient element type of a bucket.  BF16: bf16 gradient contributions and bf16
 * parameters out (Table 1 of the paper).  F32: fp32 contributions and an fp32 parameter copy
 * out (1-D norm / bias states that are kept in full precision). */
typedef enum { HZP_CLASS_BF16 = 0, HZP_CLASS_F32 = 1 } hzp_class_t;

/* Element type of gradient contributions handed to hzp_reduce_shard.  DEFAULT: the class's own
 * (bf16 for BF16 buckets, fp32 for F32 buckets).  F32 on a BF16 bucket is the paper's literal
 * setting: fp32 gradients (Table 1) next to bf16 parameters. */
typedef enum { HZP_GRAD_DEFAULT = 0, HZP_GRAD_BF16 = 1, HZP_GRAD_F32 = 2 } hzp_grad_dtype_t;

#define HZP_MAX_REPLICAS 32u    /* largest R accepted by the reduce / update entry points */
#define HZP_MAX_GROUP    64u    /* largest number of shards one gather call concatenates */

/* ------------------------------------------------------------------------------------------
 * Layout planner.
 *
 * Section 4.1.1 of the paper gives three independent sharding-group sizes; its memory model
 * M_hzp = 12N/Z1 + 4N/Z2 + 2N/Z3 fixes which is which: Z1 shards the optimizer states
 * (12 B/parameter), Z2 the gradients (4 B), Z3 the parameters (2 B).  Parameters and gradients
 * are sharded in a small group, optimizer states in a larger one (Figure 1, Section 3.1).
 *
 * The paper does not say how tensors are laid out inside a shardable buffer; this library uses
 * one flat bucket per (layer, class):
 *     off_0 = 0,  off_{t+1} = round_up(off_t + n_t, A)        every tensor starts A-aligned
 *     payload_end = off_last + n_last
 *     P  = round_up(payload_end, A*lcm(Z1,Z2,Z3))              padded length (padding holds 0)
 *     S3 = P/Z3   ZeRO-3 shard j covers [j*S3, (j+1)*S3)       parameters          (level 3)
 *     S2 = P/Z2   gradient shard s covers [s*S2, (s+1)*S2)     fp32 gradients      (level 2)
 *     S1 = P/Z1   ZeRO-1 shard i covers [i*S1, (i+1)*S1)       master, momentum, variance (level 1)
 * Every shard length is a multiple of A.  The paper's configurations all have Z2 = Z3 | Z1; then
 * lcm = Z1 and, with K = Z1/Z3,
 *     rank r in [0,Z1):  j = r mod Z3,  k = r div Z3,  i = j*K + k
 * so ZeRO-1 shard i lies inside ZeRO-3 shard j, and the K owners of one ZeRO-3 shard are the
 * ranks j, j+Z3, j+2*Z3, ...
 *
 * Section 4.1.1 leaves the three sizes free.  In general a rank r in [0, lcm(Z1,Z2,Z3)) owns the
 * shard with this index at each level (it depends on r mod Z_level only, one-to-one, and a shard
 * lies inside the rank's shard of a smaller group wherever that group's size divides its own):
 *     level 3:  j3 = r mod Z3
 *     level 2:  Z3 | Z2:       j2 = j3*(Z2/Z3) + (r div Z3) mod (Z2/Z3)     else  j2 = r mod Z2
 *     level 1:  Z3 | Z2 | Z1:  i  = j2*(Z1/Z2) + (r div Z2) mod (Z1/Z2)
 *               else Z3 | Z1:  i  = j3*(Z1/Z3) + (r div Z3) mod (Z1/Z3)
 *               else Z2 | Z1:  i  = j2*(Z1/Z2) + (r div Z2) mod (Z1/Z2)
 *               else           i  = r mod Z1
 * When Z3 does not divide Z1 a ZeRO-3 shard is covered by whole and partial ZeRO-1 shards
 * (hzp_plan_cover, hzp_gather_shard).  Buckets are ordered by (layer, class); `base` is the running
 * sum of P in that order.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
    uint32_t n_layers;                  /* >= 1 */
    const uint32_t *tensors_per_layer;  /* host array [n_layers], each >= 1 */
    const uint64_t *tensor_numel;       /* host array [sum of tensors_per_layer], each >= 1 */
    const uint8_t *tensor_class;        /* host array of hzp_class_t per tensor; NULL: all BF16 */
    const float *tensor_wd_mult;        /* host array, multiplies weight_decay per tensor; NULL: all 1 */
    uint32_t align_elems;               /* A: power of two, >= 8 */
    uint32_t z3, z2, z1;                /* each >= 1 and free; z2 == 0 means z2 = z3 */
} hzp_plan_desc_t;

typedef struct {
    uint32_t n_layers, n_buckets, n_tensors;
    uint32_t align_elems, z3, z2, z1;
    uint32_t k;                              /* z1 / z3, or 0 when z3 does not divide z1 */
    uint32_t world;                          /* lcm(z1, z2, z3): ranks are 0 .. world-1 */
    uint64_t total_padded;                   /* sum of P over all buckets */
} hzp_plan_info_t;

typedef struct {
    uint32_t layer;
    uint32_t cls;
    uint32_t n_tensors;
    uint32_t bucket_index;      /* position in (layer, class) order */
    uint64_t payload_end;       /* end of the last tensor */
    uint64_t padded;            /* P */
    uint64_t s3;                /* P / Z3 */
    uint64_t s1;                /* P / Z1 */
    uint64_t base;              /* start of the bucket in the global flat address space */
    uint64_t s2;                /* P / Z2 */
} hzp_bucket_info_t;

typedef struct {
    uint32_t layer;
    uint32_t cls;
    uint32_t bucket_index;
    uint32_t index_in_bucket;   /* position among the bucket's tensors (order of tensor_out[]) */
    uint64_t offset;            /* bucket-relative start, a multiple of A */
    uint64_t numel;
    float wd_mult;
} hzp_tensor_info_t;

/* Build a plan.  Pure 64-bit integer work on the host: makes no HIP call and needs no GPU.
 * Copies everything it needs from `desc`.  *out is owned by the library until hzp_plan_free.
 * Errors: INVALID_ARG (NULL, zero counts, bad alignment, unknown class), UNSUPPORTED
 * (lcm(z1, z2, z3) or the tensor count exceeds 32 bits), NOMEM. */
hzp_status_t hzp_plan(const hzp_plan_desc_t *desc, hzp_plan_t **out);

/* Free a plan and its device tables.  NULL is allowed.  The caller must make sure that no kernel
 * launched with this plan is still running. */
void hzp_plan_free(hzp_plan_t *plan);

/* Create the plan's lookup tables on the current device now (tensor offsets and decay multipliers
 * for updates with per-tensor decay, tensor pieces for the unpacking gathers): one allocation and
 * one blocking copy per table.  This is the one call on a plan that may allocate device memory and
 * synchronise; after it has returned, no kernel-launching call with this plan on this device
 * allocates, copies or waits (without it, the first call that needs a table creates it, and that
 * call blocks).  `stream` is waited for before returning, together with the copies, so that work
 * enqueued afterwards on any stream finds the tables in place.  May be called again (no effect) and
 * from several threads.  Call it once per device that uses the plan.
 * Errors: INVALID_ARG (NULL), NOMEM, HIP. */
hzp_status_t hzp_plan_prepare(const hzp_plan_t *plan, hipStream_t stream);

/* Read-back of the layout (what the tests compare with the oracle, bit for bit). */
hzp_status_t hzp_plan_info(const hzp_plan_t *plan, hzp_plan_info_t *out);
/* RANGE if the layer has no bucket of that class. */
hzp_status_t hzp_plan_bucket(const hzp_plan_t *plan, uint32_t layer, uint32_t cls, hzp_bucket_info_t *out);
hzp_status_t hzp_plan_tensor(const hzp_plan_t *plan, uint32_t tensor_id, hzp_tensor_info_t *out);
/* rank -> ZeRO-3 index j, outer index k = i - j*K (0 when z3 does not divide z1), ZeRO-1 shard
 * index i.  Outputs may be NULL.  RANGE if rank >= world. */
hzp_status_t hzp_plan_rank(const hzp_plan_t *plan, uint32_t rank, uint32_t *j, uint32_t *k, uint32_t *i);
/* Index of the shard the rank owns at `level` (1, 2 or 3), by the rule above. */
hzp_status_t hzp_plan_index(const hzp_plan_t *plan, int level, uint32_t rank, uint32_t *index);
/* The ZeRO-1 shards that meet ZeRO-3 shard j of a bucket: first_owner .. first_owner+n_owners-1
 * (consecutive shard indices; the first and the last may lie only partly inside shard j).  With
 * z3 | z1 these are the K whole shards j*K .. j*K+K-1. */
hzp_status_t hzp_plan_cover(const hzp_plan_t *plan, uint32_t layer, uint32_t cls, uint32_t j,
                            uint32_t *first_owner, uint32_t *n_owners);
/* Bucket-relative [begin, begin+len) of the rank's shard; level 3: parameter shard, level 2:
 * gradient shard, level 1: optimizer-state shard. */
hzp_status_t hzp_plan_shard(const hzp_plan_t *plan, uint32_t layer, uint32_t cls, int level, uint32_t rank,
                            uint64_t *begin, uint64_t *len);
/* Bytes one rank holds: 12*S1 of optimizer state, 4*P/Z2 of fp32 gradient and the parameter
 * shard (2 or 4 bytes per element), summed over buckets -- M_hzp of Section 4.1.1 with N -> P. */
hzp_status_t hzp_plan_bytes(const hzp_plan_t *plan, uint64_t *opt_bytes, uint64_t *grad_bytes,
                            uint64_t *param_bytes);

/* ------------------------------------------------------------------------------------------
 * One arena for a rank's persistent buffers of one class.
 *
 * Section 4.2 keeps communication buffers in pre-allocated contiguous memory and gives no layout.
 * This library's: the rank's buffers are streams -- R gradient contributions, master, momentum,
 * variance, cast parameters, the received ZeRO-1 pieces of the K-1 other owners of its ZeRO-3
 * shard, that shard, the Z3-1 received ZeRO-3 shards -- in that order inside ONE allocation; every
 * stream starts on a multiple of HZP_ARENA_ALIGN bytes and holds the slices (S1 or S3 elements) of
 * all buckets of the class back to back in bucket order.  The distance between the starts of
 * consecutive streams, in units of HZP_ARENA_ALIGN, is the smallest one that holds the earlier
 * stream and is congruent to r modulo M, where (M, r) is fixed by the layout variant:
 *   variant 0: (2, 1) -- an odd number of units, the default;  1: (1, 0) -- no extra spacing;
 *   2: (2, 0);  3: (16, 3);  4: (16, 13);  5: (64, 21);  6: (64, 35);  7: (64, 59).
 * The caller allocates total_bytes once, aligned to HZP_ARENA_ALIGN, and hands `base + byte_offset`
 * to the entry points; every offset is a multiple of 16.
 * Why one allocation, and why variants: the fused update reads R+3 and writes 4 of these streams
 * at the same relative position, and how their addresses lie against one another in physical
 * memory moves its bandwidth by several per cent.  Separate allocations land wherever the driver
 * puts them (measured on MI355X over 5 processes each, 7B-class share: 5.90-6.34 TB/s with one
 * allocation per stream kind, 6.46-6.52 with this arena).  Inside one allocation the spacing
 * decides: streams exactly 256 MiB apart 5.96 TB/s, an even number of units apart 1-9 % below odd
 * ones on most shapes, a 4 KiB stagger between the streams 6.1-6.2.  Which spacing is best depends
 * on the streams' sizes and on where the allocation lies (the same variant moved by 16 GiB inside
 * a larger allocation: 6.46 -> 6.16 TB/s), so hzp_arena_tune measures it on the caller's allocation.
 *   cls, R, grad_dtype : class of the buckets, number of contributions (0 .. HZP_MAX_REPLICAS) and their
 *                        element type (an hzp_grad_dtype_t) -- they fix the streams and their sizes
 *   variant            : 0 .. HZP_ARENA_VARIANTS-1
 *   stream, index      : an hzp_stream_t; index r < R for GRAD, k < K-1 for RECV1, j < Z3-1 for RECV3, else 0
 * Host-only integer work.  Errors: INVALID_ARG (NULL, unknown gradient type), RANGE (class without a
 * bucket, layer, stream, index, variant), UNSUPPORTED (R too large; RECV1 when z3 does not divide z1).
 * ------------------------------------------------------------------------------------------ */
#define HZP_ARENA_ALIGN (2u << 20)
#define HZP_ARENA_VARIANTS 8u
typedef enum {
    HZP_STREAM_GRAD = 0, HZP_STREAM_MASTER = 1, HZP_STREAM_M = 2, HZP_STREAM_V = 3, HZP_STREAM_PARAM_OUT = 4,
    HZP_STREAM_RECV1 = 5, HZP_STREAM_SHARD3 = 6, HZP_STREAM_RECV3 = 7
} hzp_stream_t;
hzp_status_t hzp_plan_arena(const hzp_plan_t *plan, uint32_t cls, uint32_t R, uint32_t grad_dtype,
                            uint32_t variant, uint64_t *total_bytes);
/* Where bucket (layer, cls)'s slice of a stream lies in the arena, and its size in bytes. */
hzp_status_t hzp_plan_arena_slice(const hzp_plan_t *plan, uint32_t cls, uint32_t R, uint32_t grad_dtype,
                                  uint32_t variant, uint32_t stream, uint32_t index, uint32_t layer,
                                  uint64_t *byte_offset, uint64_t *bytes);

/* Static model-state memory per device of Section 4.1.1 for N parameters,
 *     M_hzp = 12N/Z1 + 4N/Z2 + 2N/Z3   bytes,
 * evaluated exactly and rounded up to a whole byte.  Z1 = Z2 = Z3 = Z gives M_zp = 18N/Z, and
 * Z = DP gives vanilla ZeRO-3, M_zero3 = 18N/DP.  Host-only.
 * Errors: INVALID_ARG (NULL output, a group size of 0), UNSUPPORTED (result exceeds 64 bits). */
hzp_status_t hzp_memory_model(uint64_t n_params, uint32_t z1, uint32_t z2, uint32_t z3, uint64_t *bytes);

/* Least sharding whose M_hzp fits a per-device budget.  The paper sets the group sizes according
 * to the available device memory and keeps parameters and gradients inside a node (Section 3.1,
 * Section 4.1.1) without giving a procedure; this library's rule: candidates have Z2 = Z3 dividing
 * both `node` (devices per node) and `dp`, and Z3 | Z1 | dp; among those with
 * 12N/Z1 + 4N/Z2 + 2N/Z3 <= budget_bytes the smallest Z3 wins, then the smallest Z1.  Host-only.
 * Errors: INVALID_ARG (NULL output, dp or node 0), NOMEM (no candidate fits the budget; the
 * outputs then hold the most sharded candidate), UNSUPPORTED (dp above 2^20, or the model overflows
 * 64 bits). */
hzp_status_t hzp_choose_groups(uint64_t n_params, uint32_t dp, uint32_t node, uint64_t budget_bytes,
                               uint32_t *z1, uint32_t *z2, uint32_t *z3);

/* ------------------------------------------------------------------------------------------
 * Gradient reduction on the rank's shard: the arithmetic half of the per-layer reduce-scatter
 * ("performed using the float32 data type", Section 4.1.2, Backward Pass) together with the
 * final reduction across replicas of the model states (Section 4.1.2, Optimizer Step).
 *
 *     s      = ((G_0[x] + G_1[x]) + G_2[x]) + ...      fp32, strictly in the order r = 0..R-1
 *     out[x] = accumulate ? out[x] + scale*s : scale*s  one multiply, one add, no fused rounding
 *
 * for x in [0, n), n = S1 (level 1), S2 (level 2) or S3 (level 3) of bucket (layer, cls).  The
 * result equals the scalar definition bit for bit.
 *   grad_slices : host array [R] of device pointers; entry r points at element 0 of the rank's
 *                 slice inside contribution r, n elements of `grad_dtype`, 16-byte aligned
 *   R           : 1 .. HZP_MAX_REPLICAS
 *   grad_dtype  : an hzp_grad_dtype_t
 *   accumulate  : non-zero adds the scaled sum to what `out_f32` holds: the per-micro-batch
 *                 accumulation of Section 4.2 ("aggregate gradients of every micro batch")
 *   out_f32     : device pointer, n floats, 16-byte aligned; read first when accumulate != 0;
 *                 must not overlap any input
 * Errors: INVALID_ARG, RANGE (layer / class / level / rank), UNSUPPORTED (R too large, or a shard of 2^30 elements or more), ALIGN, HIP.
 * ------------------------------------------------------------------------------------------ */
hzp_status_t hzp_reduce_shard(const hzp_plan_t *plan, uint32_t layer, uint32_t cls, int level, uint32_t rank,
                              const void *const *grad_slices, uint32_t R, uint32_t grad_dtype, float scale,
                              int accumulate, float *out_f32, hipStream_t stream);

/* ------------------------------------------------------------------------------------------
 * Fused shard update: reduction as above (scale = grad_scale, no accumulate), then Adam with
 * decoupled weight decay on the rank's ZeRO-1 shard (mixed-precision Adam on the local
 * optimizer shard, Section 4.1.1 and Section 4.1.2 "Optimizer Step"), then the cast that
 * produces the rank's piece of the new bf16 parameters:
 *
 *     g  = grad_scale * sum_r G_r[x]
 *     m  = beta1*m + (1-beta1)*g
 *     v  = beta2*v + (1-beta2)*g*g
 *     u  = (m / (1-beta1^step)) / (sqrt(v / (1-beta2^step)) + eps)
 *     p  = p - lr*(u + weight_decay*wd_mult(tensor of x)*p)         p on the right is the old p
 *     param_out[x] = bf16_round_to_nearest_even(p)   (class F32: param_out[x] = p)
 *
 * computed in fp32 (results agree with a double-precision evaluation to about 1e-6 relative;
 * they are not promised bit for bit).  Padding positions must hold 0 in every input and then
 * stay 0.  One call covers the buckets of class `cls` of layers [layer_begin, layer_end); a layer
 * without such a bucket is skipped and its array entries are ignored.  Per-layer arrays are
 * host arrays indexed by (layer - layer_begin):
 *   grad_slices : [(layer_end-layer_begin) * max(R,1)], entry (l*R + r) as in hzp_reduce_shard
 *                 at level 1.  R == 0: a single fp32 slice per layer that is already reduced
 *                 (grad_scale is still applied)
 *   master,m,v  : device pointers to S1 floats each, 16-byte aligned, updated in place
 *   param_out   : device pointers to S1 bf16 (class BF16) or S1 floats (class F32), 16-byte
 *                 aligned; the array itself may be NULL (no cast output)
 * No buffer may overlap another.  step is 1-based.
 * Errors: INVALID_ARG (NULL, step 0, empty range), RANGE, UNSUPPORTED (R too large, or a shard of 2^30 elements or more), ALIGN, HIP.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay, grad_scale;
    uint32_t step;
} hzp_adamw_t;

hzp_status_t hzp_adamw_shard(const hzp_plan_t *plan, uint32_t layer_begin, uint32_t layer_end, uint32_t cls,
                             uint32_t rank, const hzp_adamw_t *hyper, const void *const *grad_slices,
                             uint32_t R, float *const *master, float *const *m, float *const *v,
                             void *const *param_out, hipStream_t stream);

/* The update with the step's hyper-parameters in DEVICE memory, for callers that capture their step
 * in a HIP graph once and replay it every training step: hzp_adamw_shard bakes its hyper-parameters
 * (the step number among them) into the launches it enqueues, hzp_adamw_shard_dev makes the kernels
 * read them when they run.  hzp_adamw_scalars derives, on the host, the 48-byte block the kernels read
 * (the bias corrections 1/(1-beta^step) in double precision, as hzp_adamw_shard does); the caller
 * copies it to `scalars` before each replay (any copy that is ordered before the launches).  Same
 * arithmetic, same results bit for bit, same arguments and errors otherwise.
 *   scalars : DEVICE pointer, 16-byte aligned, valid until the launches have run
 * Errors of hzp_adamw_scalars: INVALID_ARG (NULL, step 0). */
typedef struct {
    float f[12];
} hzp_adamw_scalars_t;
hzp_status_t hzp_adamw_scalars(const hzp_adamw_t *hyper, hzp_adamw_scalars_t *out);
hzp_status_t hzp_adamw_shard_dev(const hzp_plan_t *plan, uint32_t layer_begin, uint32_t layer_end, uint32_t cls,
                                 uint32_t rank, const hzp_adamw_scalars_t *scalars, const void *const *grad_slices,
                                 uint32_t R, float *const *master, float *const *m, float *const *v,
                                 void *const *param_out, hipStream_t stream);

/* Set-up time choice of the arena layout variant (see hzp_plan_arena) for the fused update of
 * Section 4.1.2's optimizer step: runs hzp_adamw_shard over all layers of the class, with the
 * streams placed by each variant whose total fits arena_bytes, four times per variant, timing the
 * last three with events on `stream`, and returns the variant with the shortest time (variant 0
 * unless another one is more than 0.5 % faster).  Call it once
 * after allocating the arena and before filling it: its contents are overwritten (each variant's
 * streams with ordinary non-zero values: on all-zero gradients and states the update runs 1-3 %
 * faster than on any others and shows less of the differences between the variants) and it is all
 * zero on return (hzp_arena_tune is not for graph capture).
 *   arena, arena_bytes : DEVICE allocation, start on a multiple of HZP_ARENA_ALIGN; it must hold
 *                        variant 0; to let every variant compete, allocate the largest of the
 *                        variants' totals (at most 63 units per stream more than variant 1)
 *   R                  : 1 .. HZP_MAX_REPLICAS contributions of the class's default gradient type
 *   best_variant       : OUT
 *   seconds            : OUT, HOST array of HZP_ARENA_VARIANTS, seconds per update of each variant
 *                        (0 for a variant that does not fit), or NULL
 * Blocks until the measurements are done; creates and destroys two events; allocates device memory
 * only if hzp_plan_prepare was not called.  The variants lie a few per cent apart at most and a
 * measurement repeats to a few tenths of a per cent, so two runs may pick different variants of
 * nearly equal speed.
 * Errors: INVALID_ARG (NULL, R == 0, arena too small for variant 0), RANGE (class, rank), ALIGN,
 * UNSUPPORTED (R too large), and those of hzp_adamw_shard. */
hzp_status_t hzp_arena_tune(const hzp_plan_t *plan, uint32_t cls, uint32_t rank, uint32_t R, void *arena,
                            uint64_t arena_bytes, hipStream_t stream, uint32_t *best_variant, double *seconds);

/* ------------------------------------------------------------------------------------------
 * Gather: the data-movement half of the two all-gathers of Section 4.1.2.
 *   level 1 : the post-step all-gather that rebuilds a ZeRO-3 parameter shard from the K
 *             ZeRO-1 owners' outputs:   bucket_out[k*S1 + x] = shard_ptrs[k][x],  n_shards == K
 *   level 3 : the all-gather that rebuilds a layer's parameters from the Z3 ZeRO-3 shards before
 *             the layer is used:        bucket_out[j*S3 + x] = shard_ptrs[j][x],  n_shards == Z3
 *             and / or, per tensor t of the bucket (padding dropped):
 *                                       tensor_out[t][y] = bucket[offset_t + y],  y < numel_t
 * Bit copies; elements are bf16 (class BF16) or fp32 (class F32).
 *   shard_ptrs : host array [n_shards] of device pointers, 16-byte aligned
 *   bucket_out : device pointer to S3 (level 1) or P (level 3) elements, 16-byte aligned; may be
 *                NULL at level 3 when tensor_out is given
 *   tensor_out : level 3 only, may be NULL; host array [n_tensors of the bucket] of device
 *                pointers, each to numel_t elements, element-aligned only
 * At least one output is required.  A shard may already lie in place: shard_ptrs[s] equal to the
 * address of piece s inside bucket_out (bucket_out + s * shard bytes) -- the case of a rank whose
 * update wrote its parameters straight into its ZeRO-3 shard -- is not copied and costs nothing; this
 * holds for hzp_gather_layers and the scheduler's gathers as well.  Any other overlap of outputs and
 * inputs is not detected and gives undefined contents.  With both outputs the shards are read twice
 * (one copy kernel per output).
 * Errors: INVALID_ARG (n_shards mismatch, no output, tensor_out at level 1), RANGE, UNSUPPORTED
 * (more than HZP_MAX_GROUP shards; level 1 on a plan whose z3 does not divide z1 -- use
 * hzp_gather_shard), ALIGN, NOMEM, HIP.
 * ------------------------------------------------------------------------------------------ */
hzp_status_t hzp_gather_layer(const hzp_plan_t *plan, uint32_t layer, uint32_t cls, int level,
                              const void *const *shard_ptrs, uint32_t n_shards, void *bucket_out,
                              void *const *tensor_out, hipStream_t stream);

/* ------------------------------------------------------------------------------------------
 * hzp_gather_layer's per-tensor output (level 3) for callers that cannot allocate device memory:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The lookup
 * table of the bucket's tensor pieces, which hzp_gather_layer keeps in per-plan device memory that it
 * allocates on first use, here goes into a fixed array inside the library's device image
 * (HZP_STATIC_MAX_PIECES entries, 176 KiB, one copy per GPU held until the process ends), written
 * on `stream` by small kernels that carry it in their arguments.  The call allocates and frees
 * nothing, makes no host-to-device copy and does not synchronise.
 *     tensor_out[t][y] = bucket[offset_t + y],   y < numel_t,   for every tensor t of the bucket
 *   shard_ptrs, n_shards, tensor_out : as hzp_gather_layer at level 3 (tensor_out is required)
 * All calls on one GPU share the one array, which keeps the last call's table: calls on different
 * streams that may run at the same time race; calls on one stream are ordered and safe.
 * Errors: INVALID_ARG, RANGE, ALIGN, HIP as hzp_gather_layer; UNSUPPORTED when the bucket has more
 * than HZP_STATIC_MAX_PIECES pieces (a piece is a run of one tensor inside one ZeRO-3 shard: at
 * most n_tensors + Z3 - 1 of them) or more than HZP_MAX_GROUP shards.
 * ------------------------------------------------------------------------------------------ */
#define HZP_STATIC_MAX_PIECES 4096u
hzp_status_t hzp_gather_layer_static(const hzp_plan_t *plan, uint32_t layer, uint32_t cls,
                                     const void *const *shard_ptrs, uint32_t n_shards,
                                     void *const *tensor_out, hipStream_t stream);

/* ------------------------------------------------------------------------------------------
 * hzp_gather_layer's bucket output for a range of layers in one call (one kernel launch for up
 * to 40 layers): the post-step gather of Section 4.1.2 runs for every layer at once, and many
 * small launches leave the memory system idle between them.
 *   shard_ptrs : host array [(layer_end-layer_begin) * n_shards]; entry (l*n_shards + s) is shard s
 *                of layer layer_begin+l, as in hzp_gather_layer; entries of layers that have no
 *                bucket of the class are not read
 *   bucket_out : host array [layer_end-layer_begin] of device pointers (S3 elements at level 1,
 *                P at level 3), 16-byte aligned
 * Errors: as hzp_gather_layer; INVALID_ARG for an empty layer range.
 * ------------------------------------------------------------------------------------------ */
hzp_status_t hzp_gather_layers(const hzp_plan_t *plan, uint32_t layer_begin, uint32_t layer_end, uint32_t cls,
                               int level, const void *const *shard_ptrs, uint32_t n_shards,
                               void *const *bucket_out, hipStream_t stream);

/* ------------------------------------------------------------------------------------------
 * Gather of one parameter: the all-gather at parameter granularity that Section 4.2 prefers to
 * whole buckets.  Rebuilds tensor `tensor_id` (numbering of hzp_plan_tensor) from the ZeRO-3 shards
 * of its bucket:
 *
 *     tensor_out[y] = shard_ptrs[j][(offset + y) - j*S3],   j = (offset + y) div S3,   y < numel
 *
 *   shard_ptrs : host array [Z3] of device pointers to the bucket's WHOLE ZeRO-3 shards, 16-byte
 *                aligned; only the shards that hold a part of the tensor are read, the other
 *                entries may be NULL
 *   tensor_out : device pointer to numel elements of the tensor's class, element-aligned only
 * Bit copy.  Errors: INVALID_ARG (NULL, n_shards != Z3, a needed shard is NULL), RANGE (tensor_id),
 * UNSUPPORTED (more than HZP_MAX_GROUP shards), ALIGN, NOMEM, HIP.
 * ------------------------------------------------------------------------------------------ */
hzp_status_t hzp_gather_tensor(const hzp_plan_t *plan, uint32_t tensor_id, const void *const *shard_ptrs,
                               uint32_t n_shards, void *tensor_out, hipStream_t stream);

/* ------------------------------------------------------------------------------------------
 * Post-step parameter gather for free group sizes (Section 4.1.1: the three sizes are independent;
 * Section 4.1.2 "Optimizer Step": updated parameters are gathered back into the parameter shards).
 * Rebuilds ZeRO-3 shard j of bucket (layer, cls) from the ZeRO-1 shards that meet it:
 *
 *     shard_out[x] = owner_ptrs[i - first_owner][(j*S3 + x) - i*S1],   i = (j*S3 + x) div S1
 *
 * for x in [0, S3).  With z3 | z1 this is the level-1 hzp_gather_layer.
 *   owner_ptrs : host array [n_owners] of device pointers; entry q points at element 0 of the WHOLE
 *                ZeRO-1 shard first_owner+q (S1 elements; only the part inside shard j is read),
 *                16-byte aligned; first_owner and n_owners are hzp_plan_cover's
 *   shard_out  : device pointer to S3 elements, 16-byte aligned, not overlapping any input
 * Bit copies; elements are bf16 (class BF16) or fp32 (class F32).
 * Errors: INVALID_ARG (NULL, n_owners differs from the cover), RANGE (layer / class / j),
 * UNSUPPORTED (more than HZP_MAX_GROUP owners), ALIGN, HIP.
 * ------------------------------------------------------------------------------------------ */
hzp_status_t hzp_gather_shard(const hzp_plan_t *plan, uint32_t layer, uint32_t cls, uint32_t j,
                              const void *const *owner_ptrs, uint32_t n_owners, void *shard_out,
                              hipStream_t stream);

/* ------------------------------------------------------------------------------------------
 * Asynchronous scheduler: the multi-stream dispatch of Section 4.2 for the local halves of the
 * collectives.  A scheduler owns one background host thread, two dedicated streams (gathers,
 * reductions; default priority) and a fixed-capacity persistent pool: one contiguous buffer,
 * allocated once, that the gathers use as a ring.  Issuing a prefetch or a reduction returns at
 * once and puts nothing on the caller's compute stream; the compute stream waits for gathered
 * parameters only where it acquires them, and their space is given back right after their use.
 *
 * Protocol per layer (or per parameter, the granularity Section 4.2 prefers):
 *     prefetch -> acquire -> (use on `consumer`) -> release.
 * A prefetch takes the next region of the ring, a release returns it; space comes back oldest
 * first, so regions should be released in the order they were prefetched (one released early keeps
 * its place until everything older is released).  When the ring has no room, or `gather_slots`
 * regions are live already, a prefetch returns HZP_ERR_NOMEM (back pressure) instead of blocking.
 * Host-side waits inside these calls are bounded (30 s) and then fail with HZP_ERR_HIP; after any
 * failure every later call on the scheduler returns that status.  All calls may come from one
 * thread at a time; the plan must outlive the scheduler.
 * ------------------------------------------------------------------------------------------ */
typedef struct hzp_sched hzp_sched_t;

typedef struct {
    uint32_t cls;               /* class of the buckets this scheduler gathers and reduces */
    uint32_t gather_slots;      /* most regions between prefetch and release at once, >= 1 */
    uint32_t queue_capacity;    /* commands that may wait for the background thread, >= 1 */
    uint32_t reserved_;         /* 0 */
    uint64_t pool_bytes;        /* 0: the ring is gather_slots equal slots of the largest bucket, so any
                                 * gather_slots regions fit.  Otherwise the ring's size (a multiple of 256):
                                 * a region then takes its own size rounded up to 256 bytes, and a prefetch
                                 * is also refused while the free space is split between the two ends */
} hzp_sched_desc_t;

typedef struct {
    uint64_t pool_bytes;            /* size of the persistent pool (allocated once) */
    uint64_t slot_bytes;            /* the largest bucket of the class, rounded to 256 bytes */
    uint64_t peak_live_bytes;       /* most gathered bytes that were between prefetch and release at once */
    uint32_t peak_live_slots;       /* most regions between prefetch and release at once */
    uint32_t reserved_;
    uint64_t gathers_issued, reduces_issued;
    uint64_t acquire_host_wait_us;  /* host time spent in acquire waiting for the gather to be issued */
    uint64_t wrap_skipped_bytes;    /* ring space passed over, in total, where a region did not fit before the end */
} hzp_sched_stats_t;

/* Allocates the pool on the current device, creates the plan's device tables (hzp_plan_prepare) and
 * starts the thread: the only scheduler call that allocates or blocks on the device.
 * Errors: INVALID_ARG, RANGE (no bucket of that class), NOMEM, HIP. */
hzp_status_t hzp_sched_create(const hzp_plan_t *plan, const hzp_sched_desc_t *desc, hzp_sched_t **out);
/* Launches what is still queued, waits for the side streams, frees everything.  NULL allowed. */
void hzp_sched_destroy(hzp_sched_t *sched);
/* Queue the level-3 gather of `layer` (hzp_gather_layer with bucket_out = the next region of the
 * ring).  shard_ptrs: host array [Z3] of device pointers, copied.  The gather runs after the work
 * enqueued on `producer` before this call (the stream that wrote the shards: the optimizer step and
 * the post-step gather of Section 4.1.2); an event is recorded there, nothing waits on it.
 * Returns at once. */
hzp_status_t hzp_sched_prefetch(hzp_sched_t *sched, uint32_t layer, const void *const *shard_ptrs, uint32_t n_shards,
                                hipStream_t producer);
/* Prefetch as far ahead as the pool allows: layers first_layer, first_layer+1, ... are queued in order
 * until n_layers are queued or the pool has no room (Section 4.1.2, "Parameter Pre-fetching": how
 * many all-gathers are issued in advance is governed by the available device memory).  *issued is
 * the number of layers dealt with (layers without a bucket of the scheduler's class count as dealt
 * with); a full pool is not an error here.
 *   shard_ptrs : host array [n_layers * n_shards], entry (l*n_shards + j) is shard j of layer first_layer+l */
hzp_status_t hzp_sched_prefetch_ahead(hzp_sched_t *sched, uint32_t first_layer, uint32_t n_layers,
                                      const void *const *shard_ptrs, uint32_t n_shards, hipStream_t producer,
                                      uint32_t *issued);
/* Make `consumer` wait for the layer's gather and return the bucket's device address.  Blocks the
 * host only until the background thread has launched that gather. */
hzp_status_t hzp_sched_acquire(hzp_sched_t *sched, uint32_t layer, hipStream_t consumer, void **bucket);
/* The work enqueued on `consumer` so far is the last use of the layer's bucket. */
hzp_status_t hzp_sched_release(hzp_sched_t *sched, uint32_t layer, hipStream_t consumer);
/* The same three calls for one parameter (hzp_gather_tensor into the next region of the ring;
 * shard_ptrs as there: entries of shards the tensor does not lie in may be NULL).  A tensor and the
 * layer it belongs to are separate regions. */
hzp_status_t hzp_sched_prefetch_tensor(hzp_sched_t *sched, uint32_t tensor_id, const void *const *shard_ptrs,
                                       uint32_t n_shards, hipStream_t producer);
hzp_status_t hzp_sched_acquire_tensor(hzp_sched_t *sched, uint32_t tensor_id, hipStream_t consumer, void **tensor);
hzp_status_t hzp_sched_release_tensor(hzp_sched_t *sched, uint32_t tensor_id, hipStream_t consumer);

/* The parameters of one layer at parameter granularity with one call each: hzp_sched_prefetch_params
 * submits one gather and takes one pool region per tensor of bucket (layer, cls), in tensor order,
 * all or nothing (NOMEM, nothing submitted, if the pool or the slot count cannot take them all;
 * with several threads submitting at once a later tensor can still meet NOMEM, and the earlier
 * ones stay prefetched); the producer's stream is marked once.  hzp_sched_acquire_params makes
 * `consumer` wait for all of them with one stream operation (the gathers run in order on the
 * scheduler's gather stream) and returns the tensors' addresses in bucket order (`tensors`: HOST
 * array of n_tensors of the bucket).  hzp_sched_release_params gives the regions back behind one
 * event on `consumer` (two where the ring wrapped inside the layer).  They work on the same regions
 * as the _tensor calls and may be mixed with them.
 *   shard_ptrs : HOST array [Z3] of device pointers to the layer's ZeRO-3 shards, all non-NULL
 * Errors: as hzp_sched_prefetch_tensor / _acquire_tensor / _release_tensor. */
hzp_status_t hzp_sched_prefetch_params(hzp_sched_t *sched, uint32_t layer, const void *const *shard_ptrs,
                                       uint32_t n_shards, hipStream_t producer);
hzp_status_t hzp_sched_acquire_params(hzp_sched_t *sched, uint32_t layer, hipStream_t consumer, void **tensors);
hzp_status_t hzp_sched_release_params(hzp_sched_t *sched, uint32_t layer, hipStream_t consumer);
/* Queue hzp_reduce_shard(layer, level, rank, ...) on the reduction stream, to run after the work
 * already enqueued on `producer` (which wrote the gradients).  Arguments are checked now, as by
 * hzp_reduce_shard; the pointer array is copied.  Returns at once. */
hzp_status_t hzp_sched_reduce(hzp_sched_t *sched, uint32_t layer, int level, uint32_t rank,
                              const void *const *grad_slices, uint32_t R, uint32_t grad_dtype, float scale,
                              int accumulate, float *out_f32, hipStream_t producer);
/* Make `consumer` wait for everything queued before this call (both side streams).  Blocks the
 * host until those commands have been launched. */
hzp_status_t hzp_sched_join(hzp_sched_t *sched, hipStream_t consumer);
/* Block the host until everything queued so far has been launched and has finished. */
hzp_status_t hzp_sched_drain(hzp_sched_t *sched);
hzp_status_t hzp_sched_stats(hzp_sched_t *sched, hzp_sched_stats_t *out);

/* Text of the calling thread's last non-OK status ("" if none).  Valid until that thread's next
 * failing call. */
const char *hzp_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* HZP_H */
