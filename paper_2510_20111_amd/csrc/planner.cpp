// Layout planner of libhzp: layers -> padded flat buckets -> ZeRO-3 / ZeRO-1 shard ranges.
// Host-only 64-bit integer code; it makes no HIP call, so a plan can be built without a GPU.
//
// Group sizes follow the memory model of Section 4.1.1 (M_hzp = 12N/Z1 + 4N/Z2 + 2N/Z3):
// Z1 shards the optimizer states, Z2 the gradients, Z3 the parameters, each chosen freely.  The
// bucket rule (A-aligned tensor starts, zero padding up to a multiple of A*lcm(Z1,Z2,Z3)) and the
// rank map (nested wherever one group size divides the next; with Z2 = Z3 | Z1 it is
// j = r mod Z3, k = r div Z3, i = j*K + k) are this library's own choices; the paper only asks
// that parameters and gradients live in a small group and optimizer states in a larger one
// (Figure 1, Section 3.1).
#include <cstdarg>
#include <cstdio>
#include <new>

#include "hzp_internal.hpp"

namespace hzp {

static thread_local char g_err[512] = "";

hzp_status_t fail(hzp_status_t st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

const BucketRec *find_bucket(const hzp_plan_t *plan, uint32_t layer, uint32_t cls)
{
    if (layer >= plan->n_layers || cls > 1) return nullptr;
    int32_t b = plan->bucket_of[layer * 2 + cls];
    return b < 0 ? nullptr : &plan->buckets[b];
}

uint32_t level_index(const hzp_plan_t *plan, int level, uint32_t rank)
{
    const uint32_t z1 = plan->z1, z2 = plan->z2, z3 = plan->z3;
    const uint32_t j3 = rank % z3;
    if (level == 3) return j3;
    const bool up32 = z2 % z3 == 0;
    const uint32_t j2 = up32 ? j3 * (z2 / z3) + rank / z3 % (z2 / z3) : rank % z2;
    if (level == 2) return j2;
    const bool chain = up32 && z1 % z2 == 0;
    if (z1 % z3 == 0 && !chain) return j3 * (z1 / z3) + rank / z3 % (z1 / z3);
    if (z1 % z2 == 0) return j2 * (z1 / z2) + rank / z2 % (z1 / z2);
    return rank % z1;
}

static uint64_t gcd64(uint64_t a, uint64_t b)
{
    while (b) {
        const uint64_t t = a % b;
        a = b;
        b = t;
    }
    return a;
}

static bool round_up(uint64_t x, uint64_t q, uint64_t *out)
{
    uint64_t t;
    if (__builtin_add_overflow(x, q - 1, &t)) return false;
    *out = t / q * q;
    return true;
}

// Split every tensor of the bucket at ZeRO-3 shard boundaries and number the chunks.
static bool build_pieces(const hzp_plan_t *plan, BucketRec &b)
{
    uint64_t chunks = 0;
    for (uint32_t s = 0; s < b.n_tensors; ++s) {
        const TensorRec &t = plan->tensors[b.tensor_ids[s]];
        uint64_t pos = t.offset, end = t.offset + t.numel;
        while (pos < end) {
            uint64_t j = pos / b.S3;
            uint64_t stop = (j + 1) * b.S3 < end ? (j + 1) * b.S3 : end;
            Piece p{};
            p.src_off = pos - j * b.S3;
            p.dst_off = pos - t.offset;
            p.len = stop - pos;
            p.shard = (uint32_t)j;
            p.tensor = s;
            if (chunks > 0xFFFFFFFFull) return false;
            p.chunk_begin = (uint32_t)chunks;
            chunks += (p.len + kUnpackChunk - 1) / kUnpackChunk;
            b.pieces.push_back(p);
            pos = stop;
        }
    }
    if (chunks > 0x7FFFFFFFull) return false;
    b.n_chunks = (uint32_t)chunks;
    return true;
}

}  // namespace hzp

using namespace hzp;

extern "C" const char *hzp_last_error(void) { return g_err; }

extern "C" hzp_status_t hzp_plan(const hzp_plan_desc_t *d, hzp_plan_t **out)
{
    if (!d || !out) return fail(HZP_ERR_INVALID_ARG, "hzp_plan: NULL descriptor or output");
    *out = nullptr;
    if (d->n_layers == 0 || !d->tensors_per_layer || !d->tensor_numel)
        return fail(HZP_ERR_INVALID_ARG, "hzp_plan: need at least one layer and its tensor arrays");
    const uint32_t A = d->align_elems;
    if (A < 8 || (A & (A - 1)) != 0)
        return fail(HZP_ERR_INVALID_ARG, "hzp_plan: align_elems=%u must be a power of two >= 8", A);
    if (d->z3 == 0 || d->z1 == 0)
        return fail(HZP_ERR_INVALID_ARG, "hzp_plan: group sizes must be positive");
    const uint32_t z2 = d->z2 ? d->z2 : d->z3;
    uint64_t world = (uint64_t)d->z1 / gcd64(d->z1, z2) * z2;          // < 2^64: both factors < 2^32
    if (world > 0xFFFFFFFFull || (world = world / gcd64(world, d->z3) * d->z3) > 0xFFFFFFFFull)
        return fail(HZP_ERR_UNSUPPORTED, "hzp_plan: lcm(z1=%u, z2=%u, z3=%u) exceeds 32 bits", d->z1, z2, d->z3);
    uint64_t n_tensors = 0;
    for (uint32_t l = 0; l < d->n_layers; ++l) {
        if (d->tensors_per_layer[l] == 0)
            return fail(HZP_ERR_INVALID_ARG, "hzp_plan: layer %u has no tensor", l);
        n_tensors += d->tensors_per_layer[l];
    }
    if (n_tensors > 0x7FFFFFFFull) return fail(HZP_ERR_UNSUPPORTED, "hzp_plan: too many tensors");
    for (uint64_t t = 0; t < n_tensors; ++t) {
        if (d->tensor_numel[t] == 0)
            return fail(HZP_ERR_INVALID_ARG, "hzp_plan: tensor %llu is empty", (unsigned long long)t);
        if (d->tensor_class && d->tensor_class[t] > 1)
            return fail(HZP_ERR_INVALID_ARG, "hzp_plan: tensor %llu has unknown class %u",
                        (unsigned long long)t, d->tensor_class[t]);
    }

    hzp_plan_t *p = new (std::nothrow) hzp_plan_t;
    if (!p) return fail(HZP_ERR_NOMEM, "hzp_plan: out of host memory");
    try {
        p->n_layers = d->n_layers;
        p->align = A;
        p->z3 = d->z3;
        p->z2 = z2;
        p->z1 = d->z1;
        p->K = d->z1 % d->z3 == 0 ? d->z1 / d->z3 : 0;
        p->world = (uint32_t)world;
        p->uniform_wd = true;
        p->tensors.resize(n_tensors);
        p->bucket_of.assign((size_t)d->n_layers * 2, -1);
        const uint64_t quantum = (uint64_t)A * world;     // every level's shard is a multiple of A
        uint64_t base = 0;
        uint32_t tid0 = 0, slot = 0, piece_slot = 0;
        for (uint32_t l = 0; l < d->n_layers; ++l) {
            const uint32_t cnt = d->tensors_per_layer[l];
            for (uint32_t cls = 0; cls < 2; ++cls) {
                BucketRec b{};
                b.layer = l;
                b.cls = cls;
                b.first_slot = slot;
                uint64_t off = 0, payload_end = 0;
                for (uint32_t t = tid0; t < tid0 + cnt; ++t) {
                    const uint32_t c = d->tensor_class ? d->tensor_class[t] : 0u;
                    if (c != cls) continue;
                    TensorRec &r = p->tensors[t];
                    r.layer = l;
                    r.cls = cls;
                    r.bucket = (uint32_t)p->buckets.size();
                    r.index_in_bucket = (uint32_t)b.tensor_ids.size();
                    r.offset = off;
                    r.numel = d->tensor_numel[t];
                    r.wd_mult = d->tensor_wd_mult ? d->tensor_wd_mult[t] : 1.0f;
                    if (r.wd_mult != 1.0f) p->uniform_wd = false;
                    if (__builtin_add_overflow(off, r.numel, &payload_end) ||
                        !round_up(payload_end, A, &off)) {
                        delete p;
                        return fail(HZP_ERR_INVALID_ARG, "hzp_plan: layer %u overflows 64 bits", l);
                    }
                    b.tensor_ids.push_back(t);
                }
                if (b.tensor_ids.empty()) continue;     // no tensor of this class: no bucket
                b.n_tensors = (uint32_t)b.tensor_ids.size();
                b.payload_end = payload_end;
                if (!round_up(payload_end, quantum, &b.P) || __builtin_add_overflow(base, b.P, &base)) {
                    delete p;
                    return fail(HZP_ERR_INVALID_ARG, "hzp_plan: layer %u overflows 64 bits", l);
                }
                b.base = base - b.P;
                b.S3 = b.P / d->z3;
                b.S2 = b.P / z2;
                b.S1 = b.P / d->z1;
                b.piece_slot = piece_slot;
                if (!build_pieces(p, b)) {
                    delete p;
                    return fail(HZP_ERR_UNSUPPORTED, "hzp_plan: layer %u is too large to unpack", l);
                }
                piece_slot += (uint32_t)b.pieces.size();
                for (uint32_t t : b.tensor_ids) {
                    p->slot_off.push_back(p->tensors[t].offset);
                    p->slot_wd.push_back(p->tensors[t].wd_mult);
                }
                slot += b.n_tensors;
                p->bucket_of[(size_t)l * 2 + cls] = (int32_t)p->buckets.size();
                p->buckets.push_back(std::move(b));
            }
            tid0 += cnt;
        }
        p->total_padded = base;
    } catch (const std::bad_alloc &) {
        delete p;
        return fail(HZP_ERR_NOMEM, "hzp_plan: out of host memory");
    }
    *out = p;
    return HZP_OK;
}

extern "C" void hzp_plan_free(hzp_plan_t *plan)
{
    if (!plan) return;
    free_device_tables(plan);
    delete plan;
}

extern "C" hzp_status_t hzp_plan_info(const hzp_plan_t *plan, hzp_plan_info_t *o)
{
    if (!plan || !o) return fail(HZP_ERR_INVALID_ARG, "hzp_plan_info: NULL argument");
    o->n_layers = plan->n_layers;
    o->n_buckets = (uint32_t)plan->buckets.size();
    o->n_tensors = (uint32_t)plan->tensors.size();
    o->align_elems = plan->align;
    o->z3 = plan->z3;
    o->z2 = plan->z2;
    o->z1 = plan->z1;
    o->k = plan->K;
    o->world = plan->world;
    o->total_padded = plan->total_padded;
    return HZP_OK;
}

extern "C" hzp_status_t hzp_plan_bucket(const hzp_plan_t *plan, uint32_t layer, uint32_t cls,
                                        hzp_bucket_info_t *o)
{
    if (!plan || !o) return fail(HZP_ERR_INVALID_ARG, "hzp_plan_bucket: NULL argument");
    const BucketRec *b = find_bucket(plan, layer, cls);
    if (!b) return fail(HZP_ERR_RANGE, "hzp_plan_bucket: no bucket (layer %u, class %u)", layer, cls);
    o->layer = b->layer;
    o->cls = b->cls;
    o->n_tensors = b->n_tensors;
    o->bucket_index = (uint32_t)(b - plan->buckets.data());
    o->payload_end = b->payload_end;
    o->padded = b->P;
    o->s3 = b->S3;
    o->s1 = b->S1;
    o->base = b->base;
    o->s2 = b->S2;
    return HZP_OK;
}

extern "C" hzp_status_t hzp_plan_tensor(const hzp_plan_t *plan, uint32_t tensor_id, hzp_tensor_info_t *o)
{
    if (!plan || !o) return fail(HZP_ERR_INVALID_ARG, "hzp_plan_tensor: NULL argument");
    if (tensor_id >= plan->tensors.size())
        return fail(HZP_ERR_RANGE, "hzp_plan_tensor: tensor %u of %zu", tensor_id, plan->tensors.size());
    const TensorRec &t = plan->tensors[tensor_id];
    o->layer = t.layer;
    o->cls = t.cls;
    o->bucket_index = t.bucket;
    o->index_in_bucket = t.index_in_bucket;
    o->offset = t.offset;
    o->numel = t.numel;
    o->wd_mult = t.wd_mult;
    return HZP_OK;
}

extern "C" hzp_status_t hzp_plan_rank(const hzp_plan_t *plan, uint32_t rank, uint32_t *j, uint32_t *k,
                                      uint32_t *i)
{
    if (!plan) return fail(HZP_ERR_INVALID_ARG, "hzp_plan_rank: NULL plan");
    if (rank >= plan->world) return fail(HZP_ERR_RANGE, "hzp_plan_rank: rank %u of %u", rank, plan->world);
    const uint32_t jj = level_index(plan, 3, rank), ii = level_index(plan, 1, rank);
    if (j) *j = jj;
    if (k) *k = plan->K ? ii - jj * plan->K : 0;
    if (i) *i = ii;
    return HZP_OK;
}

extern "C" hzp_status_t hzp_plan_index(const hzp_plan_t *plan, int level, uint32_t rank, uint32_t *index)
{
    if (!plan || !index) return fail(HZP_ERR_INVALID_ARG, "hzp_plan_index: NULL argument");
    if (level < 1 || level > 3) return fail(HZP_ERR_RANGE, "hzp_plan_index: level %d is not 1, 2 or 3", level);
    if (rank >= plan->world) return fail(HZP_ERR_RANGE, "hzp_plan_index: rank %u of %u", rank, plan->world);
    *index = level_index(plan, level, rank);
    return HZP_OK;
}

extern "C" hzp_status_t hzp_plan_shard(const hzp_plan_t *plan, uint32_t layer, uint32_t cls, int level,
                                       uint32_t rank, uint64_t *begin, uint64_t *len)
{
    if (!plan || !begin || !len) return fail(HZP_ERR_INVALID_ARG, "hzp_plan_shard: NULL argument");
    const BucketRec *b = find_bucket(plan, layer, cls);
    if (!b) return fail(HZP_ERR_RANGE, "hzp_plan_shard: no bucket (layer %u, class %u)", layer, cls);
    if (rank >= plan->world) return fail(HZP_ERR_RANGE, "hzp_plan_shard: rank %u of %u", rank, plan->world);
    if (level < 1 || level > 3) return fail(HZP_ERR_RANGE, "hzp_plan_shard: level %d is not 1, 2 or 3", level);
    const uint64_t s = level == 1 ? b->S1 : level == 2 ? b->S2 : b->S3;
    *begin = level_index(plan, level, rank) * s;
    *len = s;
    return HZP_OK;
}

extern "C" hzp_status_t hzp_plan_cover(const hzp_plan_t *plan, uint32_t layer, uint32_t cls, uint32_t j,
                                       uint32_t *first_owner, uint32_t *n_owners)
{
    if (!plan || !first_owner || !n_owners) return fail(HZP_ERR_INVALID_ARG, "hzp_plan_cover: NULL argument");
    const BucketRec *b = find_bucket(plan, layer, cls);
    if (!b) return fail(HZP_ERR_RANGE, "hzp_plan_cover: no bucket (layer %u, class %u)", layer, cls);
    if (j >= plan->z3) return fail(HZP_ERR_RANGE, "hzp_plan_cover: shard %u of %u", j, plan->z3);
    const uint64_t lo = j * b->S3, hi = lo + b->S3;             // S1, S3 >= A > 0
    *first_owner = (uint32_t)(lo / b->S1);
    *n_owners = (uint32_t)((hi + b->S1 - 1) / b->S1 - lo / b->S1);
    return HZP_OK;
}

// ---------------------------------------------------------------------------------------------
// One arena for a rank's persistent buffers of one class.
// ---------------------------------------------------------------------------------------------
namespace {

// Where a stream's first slice starts and what a slice of it measures.
struct ArenaWalk {
    uint64_t total = 0;             // bytes of the whole arena
    uint64_t stream_base = 0;       // of the stream asked for
    uint32_t stream_level = 0;      // 1: ZeRO-1 slices, 3: ZeRO-3 slices
    uint32_t stream_elem = 0;       // bytes per element
    bool found = false;
};

// Lays the streams out one after the other (each on a multiple of HZP_ARENA_ALIGN) and notes the one
// asked for.  s1_bytes / s3_bytes: the class's ZeRO-1 / ZeRO-3 slices of all buckets, in elements.
// Spacing rule of each layout variant: the distance between the starts of consecutive streams, in
// units of HZP_ARENA_ALIGN, is the smallest one that holds the earlier stream and is congruent to
// `residue` modulo `modulus`.
struct ArenaRule {
    uint32_t modulus, residue;
};
const ArenaRule kArenaRules[HZP_ARENA_VARIANTS] = {{2, 1}, {1, 0}, {2, 0}, {16, 3}, {16, 13}, {64, 21}, {64, 35}, {64, 59}};

ArenaWalk walk_arena(const hzp_plan_t *plan, uint32_t cls, uint32_t R, uint32_t grad_bytes, uint32_t variant,
                     uint64_t s1_total, uint64_t s3_total, uint32_t want_stream, uint32_t want_index)
{
    const ArenaRule rule = kArenaRules[variant];
    const uint32_t eb = cls == HZP_CLASS_F32 ? 4u : 2u;
    struct Kind {
        uint32_t stream, count, level, elem;
    };
    const Kind kinds[] = {
        {HZP_STREAM_GRAD, R, 1, grad_bytes},          {HZP_STREAM_MASTER, 1, 1, 4},
        {HZP_STREAM_M, 1, 1, 4},                      {HZP_STREAM_V, 1, 1, 4},
        {HZP_STREAM_PARAM_OUT, 1, 1, eb},             {HZP_STREAM_RECV1, plan->K ? plan->K - 1 : 0, 1, eb},
        {HZP_STREAM_SHARD3, 1, 3, eb},                {HZP_STREAM_RECV3, plan->z3 - 1, 3, eb},
    };
    ArenaWalk w;
    uint64_t end = 0;               // end of the data placed so far
    uint64_t last_start = 0;
    bool first = true;
    for (const Kind &k : kinds)
        for (uint32_t i = 0; i < k.count; ++i) {
            uint64_t start = (end + HZP_ARENA_ALIGN - 1) / HZP_ARENA_ALIGN * HZP_ARENA_ALIGN;
            if (!first) {
                const uint64_t units = (start - last_start) / HZP_ARENA_ALIGN;
                start += (rule.residue + rule.modulus - units % rule.modulus) % rule.modulus * HZP_ARENA_ALIGN;
            }
            first = false;
            last_start = start;
            if (k.stream == want_stream && i == want_index) {
                w.stream_base = start;
                w.stream_level = k.level;
                w.stream_elem = k.elem;
                w.found = true;
            }
            end = start + (k.level == 1 ? s1_total : s3_total) * k.elem;
        }
    w.total = end;
    return w;
}

hzp_status_t arena_args(const char *who, const hzp_plan_t *plan, uint32_t cls, uint32_t R, uint32_t grad_dtype,
                        uint32_t variant, uint32_t *grad_bytes, uint64_t *s1_total, uint64_t *s3_total)
{
    if (!plan) return fail(HZP_ERR_INVALID_ARG, "%s: NULL plan", who);
    if (variant >= HZP_ARENA_VARIANTS)
        return fail(HZP_ERR_RANGE, "%s: layout variant %u of %u", who, variant, HZP_ARENA_VARIANTS);
    if (cls > 1) return fail(HZP_ERR_RANGE, "%s: class %u", who, cls);
    if (grad_dtype > HZP_GRAD_F32) return fail(HZP_ERR_INVALID_ARG, "%s: unknown gradient type %u", who, grad_dtype);
    if (R > HZP_MAX_REPLICAS) return fail(HZP_ERR_UNSUPPORTED, "%s: R=%u exceeds %u", who, R, HZP_MAX_REPLICAS);
    *grad_bytes = grad_dtype == HZP_GRAD_DEFAULT ? (cls == HZP_CLASS_F32 ? 4u : 2u) : grad_dtype == HZP_GRAD_F32 ? 4u : 2u;
    uint64_t a = 0, c = 0;
    bool any = false;
    for (const BucketRec &b : plan->buckets)
        if (b.cls == cls) {
            a += b.S1;
            c += b.S3;
            any = true;
        }
    if (!any) return fail(HZP_ERR_RANGE, "%s: the plan has no bucket of class %u", who, cls);
    // at most R + 4 + K + Z3 streams of at most 4 bytes x (a or c) each, plus the gaps (under 65 units each)
    const unsigned __int128 bound = ((unsigned __int128)R + 4 + plan->K + plan->z3) *
                                    (4 * (unsigned __int128)(a > c ? a : c) + 65ull * HZP_ARENA_ALIGN);
    if (bound >> 63) return fail(HZP_ERR_UNSUPPORTED, "%s: the arena would exceed 2^63 bytes", who);
    *s1_total = a;
    *s3_total = c;
    return HZP_OK;
}

}  // namespace

extern "C" hzp_status_t hzp_plan_arena(const hzp_plan_t *plan, uint32_t cls, uint32_t R, uint32_t grad_dtype,
                                       uint32_t variant, uint64_t *total_bytes)
{
    if (!total_bytes) return fail(HZP_ERR_INVALID_ARG, "hzp_plan_arena: NULL output");
    uint32_t gb = 0;
    uint64_t s1 = 0, s3 = 0;
    hzp_status_t st = arena_args("hzp_plan_arena", plan, cls, R, grad_dtype, variant, &gb, &s1, &s3);
    if (st != HZP_OK) return st;
    *total_bytes = walk_arena(plan, cls, R, gb, variant, s1, s3, ~0u, 0).total;
    return HZP_OK;
}

extern "C" hzp_status_t hzp_plan_arena_slice(const hzp_plan_t *plan, uint32_t cls, uint32_t R, uint32_t grad_dtype,
                                             uint32_t variant, uint32_t stream, uint32_t index, uint32_t layer,
                                             uint64_t *byte_offset, uint64_t *bytes)
{
    if (!byte_offset || !bytes) return fail(HZP_ERR_INVALID_ARG, "hzp_plan_arena_slice: NULL output");
    uint32_t gb = 0;
    uint64_t s1 = 0, s3 = 0;
    hzp_status_t st = arena_args("hzp_plan_arena_slice", plan, cls, R, grad_dtype, variant, &gb, &s1, &s3);
    if (st != HZP_OK) return st;
    const BucketRec *b = find_bucket(plan, layer, cls);
    if (!b) return fail(HZP_ERR_RANGE, "hzp_plan_arena_slice: no bucket (layer %u, class %u)", layer, cls);
    if (stream > HZP_STREAM_RECV3) return fail(HZP_ERR_RANGE, "hzp_plan_arena_slice: unknown stream %u", stream);
    if (stream == HZP_STREAM_RECV1 && plan->K == 0)
        return fail(HZP_ERR_UNSUPPORTED, "hzp_plan_arena_slice: z3=%u does not divide z1=%u: a ZeRO-3 shard has no "
                                         "whole ZeRO-1 owners", plan->z3, plan->z1);
    const ArenaWalk w = walk_arena(plan, cls, R, gb, variant, s1, s3, stream, index);
    if (!w.found) return fail(HZP_ERR_RANGE, "hzp_plan_arena_slice: stream %u has no index %u", stream, index);
    // the slices of the class's earlier buckets lie in front of this bucket's
    uint64_t before = 0;
    for (const BucketRec &x : plan->buckets) {
        if (&x == b) break;
        if (x.cls == cls) before += w.stream_level == 1 ? x.S1 : x.S3;
    }
    *byte_offset = w.stream_base + before * w.stream_elem;
    *bytes = (w.stream_level == 1 ? b->S1 : b->S3) * w.stream_elem;
    return HZP_OK;
}

extern "C" hzp_status_t hzp_plan_bytes(const hzp_plan_t *plan, uint64_t *opt, uint64_t *grad, uint64_t *par)
{
    if (!plan) return fail(HZP_ERR_INVALID_ARG, "hzp_plan_bytes: NULL plan");
    uint64_t o = 0, g = 0, q = 0;
    for (const BucketRec &b : plan->buckets) {
        o += 12 * b.S1;
        g += 4 * (b.P / plan->z2);
        q += (b.cls == HZP_CLASS_F32 ? 4 : 2) * b.S3;
    }
    if (opt) *opt = o;
    if (grad) *grad = g;
    if (par) *par = q;
    return HZP_OK;
}

extern "C" hzp_status_t hzp_memory_model(uint64_t n, uint32_t z1, uint32_t z2, uint32_t z3, uint64_t *bytes)
{
    if (!bytes) return fail(HZP_ERR_INVALID_ARG, "hzp_memory_model: NULL output");
    if (z1 == 0 || z2 == 0 || z3 == 0) return fail(HZP_ERR_INVALID_ARG, "hzp_memory_model: group size 0");
    // (12 n z2 z3 + 4 n z1 z3 + 2 n z1 z2) / (z1 z2 z3), exactly, in 128-bit integers:
    // n < 2^64 and each group size < 2^32 keep the numerator below 2^(64+4+64) only if
    // checked, so every product is tested for overflow.
    typedef unsigned __int128 u128;
    const u128 a = (u128)z2 * z3, b = (u128)z1 * z3, c = (u128)z1 * z2;    // each < 2^64
    const u128 den = a * z1;                                               // < 2^96
    u128 num = 0;
    const u128 terms[3] = {12 * a, 4 * b, 2 * c};                          // each < 2^68
    for (const u128 t : terms) {
        if (n != 0 && t > (~(u128)0) / n) return fail(HZP_ERR_UNSUPPORTED, "hzp_memory_model: overflow");
        const u128 add = t * n;
        if (num + add < num) return fail(HZP_ERR_UNSUPPORTED, "hzp_memory_model: overflow");
        num += add;
    }
    const u128 q = num / den + (num % den != 0);
    if (q >> 64) return fail(HZP_ERR_UNSUPPORTED, "hzp_memory_model: result exceeds 64 bits");
    *bytes = (uint64_t)q;
    return HZP_OK;
}

extern "C" hzp_status_t hzp_choose_groups(uint64_t n, uint32_t dp, uint32_t node, uint64_t budget,
                                          uint32_t *z1, uint32_t *z2, uint32_t *z3)
{
    if (!z1 || !z2 || !z3) return fail(HZP_ERR_INVALID_ARG, "hzp_choose_groups: NULL output");
    if (dp == 0 || node == 0) return fail(HZP_ERR_INVALID_ARG, "hzp_choose_groups: dp and node must be positive");
    if (dp > (1u << 20)) return fail(HZP_ERR_UNSUPPORTED, "hzp_choose_groups: dp=%u exceeds 2^20", dp);
    uint32_t last3 = 1, last1 = 1;
    for (uint32_t c3 = 1; c3 <= node && c3 <= dp; ++c3) {       // ascending Z3, then ascending Z1
        if (node % c3 || dp % c3) continue;
        for (uint64_t c1 = c3; c1 <= dp; c1 += c3) {
            if (dp % c1) continue;
            uint64_t bytes;
            const hzp_status_t st = hzp_memory_model(n, (uint32_t)c1, c3, c3, &bytes);
            if (st != HZP_OK) return st;
            last3 = c3;
            last1 = (uint32_t)c1;
            if (bytes <= budget) {          // ceil(M) <= budget  <=>  M <= budget for an integer budget
                *z1 = (uint32_t)c1;
                *z2 = *z3 = c3;
                return HZP_OK;
            }
        }
    }
    *z1 = last1;
    *z2 = *z3 = last3;
    return fail(HZP_ERR_NOMEM, "hzp_choose_groups: even Z1=%u, Z2=Z3=%u exceeds %llu bytes", last1, last3,
                (unsigned long long)budget);
}
