/*
 * Numeric oracle for the shard-update path of hierarchical ZeRO parallelism.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain scalar C, one element at a time, no
 * blocking, no fusion, no vector intrinsics.  Nothing here is shared with
 * the GPU library: no header, helper, table or constant comes from it or
 * goes to it.  Build:  gcc -O2 -fno-fast-math -ffp-contract=off -fopenmp
 * (the OpenMP pragma only splits the independent element loop over host
 * threads; it does not change any element's arithmetic).
 *
 * What the paper fixes:
 *   - state arrays and their types (Section 4.1.1, Table 1): bf16
 *     parameters, fp32 gradient, fp32 master copy, fp32 momentum, fp32
 *     variance;
 *   - gradient reduction is carried out in float32 (Section 4.1.2,
 *     "Backward Pass"), followed by a reduction across the replicas of the
 *     model states (Section 4.1.2, "Optimizer Step");
 *   - the optimizer is Adam under mixed precision, applied by each rank to
 *     its local ZeRO-1 shard with the aggregated gradient slice
 *     (Section 4.1.1 first paragraph; Section 4.1.2, "Optimizer Step");
 *   - afterwards the bf16 parameter shards of the ZeRO-3 group are rebuilt
 *     from the optimizer shards by an all-gather, and before a layer is used
 *     its full parameters are rebuilt by an all-gather in the ZeRO-3 group
 *     (Section 4.1.2) -- on one device these are plain copies.
 * The paper prints no update equations; the AdamW form below (decoupled
 * decay, bias correction, eps added after the square root) is this build's
 * stated reading.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int hzp_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* bf16 is the upper half of an IEEE binary32: widening puts the 16 bits in
 * the high half and zero-fills the low half (exact). */
float hzp_oracle_bf16_to_f32(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* Narrowing: round to nearest, ties to even, on the 16 discarded bits.
 * Infinity stays infinity, a NaN becomes a quiet NaN of the same sign,
 * a finite value whose rounding carries out of the largest exponent becomes
 * infinity (the carry does that by itself). */
uint16_t hzp_oracle_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t exponent = (u >> 23) & 0xFFu;
    uint32_t mantissa = u & 0x7FFFFFu;
    if (exponent == 0xFFu && mantissa != 0)          /* NaN */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t kept = u >> 16;
    uint32_t dropped = u & 0xFFFFu;
    if (dropped > 0x8000u)
        kept += 1;                                   /* above half: up   */
    else if (dropped == 0x8000u && (kept & 1u))
        kept += 1;                                   /* tie: to even     */
    return (uint16_t)kept;
}

/* The same cast over an array: out[x] = hzp_oracle_f32_to_bf16(in[x]). */
void hzp_oracle_f32_to_bf16_array(const float *in, uint64_t n, uint16_t *out)
{
    for (uint64_t x = 0; x < n; ++x) out[x] = hzp_oracle_f32_to_bf16(in[x]);
}

/*
 * Gradient reduction over R contributions for one slice of n elements
 * (arithmetic half of the reduce-scatter plus the cross-replica reduction).
 *   s = ((G_0[x] + G_1[x]) + G_2[x]) + ...     each + one fp32 RNE add,
 *                                              strictly in the order r = 0..R-1
 *   t = scale * s                              one fp32 multiply
 *   out[x] = accumulate ? out[x] + t : t       one fp32 add when accumulating
 * is_f32 = 0: contributions are bf16 bit patterns; 1: they are fp32.
 */
void hzp_oracle_reduce(const void *const *slices, uint32_t R, int is_f32,
                       uint64_t n, float scale, int accumulate, float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t x = 0; x < (int64_t)n; ++x) {
        float s = 0.0f;
        for (uint32_t r = 0; r < R; ++r) {
            float gr = is_f32 ? ((const float *)slices[r])[x]
                              : hzp_oracle_bf16_to_f32(((const uint16_t *)slices[r])[x]);
            if (r == 0)
                s = gr;
            else
                s = s + gr;
        }
        float t = scale * s;
        if (accumulate)
            out[x] = out[x] + t;
        else
            out[x] = t;
    }
}

typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    uint32_t step;              /* 1-based */
} hzp_oracle_adamw_t;

/*
 * AdamW on n elements, double-precision evaluation from fp32 inputs.
 *   m' = b1*m + (1-b1)*g
 *   v' = b2*v + (1-b2)*g*g
 *   u  = (m'/(1-b1^t)) / (sqrt(v'/(1-b2^t)) + eps)
 *   p' = p - lr*(u + wd*wd_mult[x]*p)          decay uses p before the update
 * m', v', p' are rounded to fp32 when stored (state between steps is fp32).
 * g is the already reduced and scaled fp32 gradient.  wd_mult may be NULL
 * (all ones).  p16 (nullable) receives bf16(p' as stored); p32out (nullable)
 * receives the stored fp32 p' (the fp32 parameter class has no cast).
 */
void hzp_oracle_adamw_f64(const hzp_oracle_adamw_t *h, uint64_t n, const float *g,
                          const float *wd_mult, float *p, float *m, float *v,
                          uint16_t *p16, float *p32out)
{
    const double b1 = h->beta1, b2 = h->beta2, lr = h->lr, eps = h->eps, wd = h->weight_decay;
    const double bc1 = 1.0 - pow(b1, (double)h->step);
    const double bc2 = 1.0 - pow(b2, (double)h->step);
#pragma omp parallel for schedule(static)
    for (int64_t x = 0; x < (int64_t)n; ++x) {
        double gx = g[x];
        double mn = b1 * (double)m[x] + (1.0 - b1) * gx;
        double vn = b2 * (double)v[x] + (1.0 - b2) * gx * gx;
        double u = (mn / bc1) / (sqrt(vn / bc2) + eps);
        double mult = wd_mult ? (double)wd_mult[x] : 1.0;
        double pn = (double)p[x] - lr * (u + wd * mult * (double)p[x]);
        m[x] = (float)mn;
        v[x] = (float)vn;
        p[x] = (float)pn;
        if (p16)
            p16[x] = hzp_oracle_f32_to_bf16(p[x]);
        if (p32out)
            p32out[x] = p[x];
    }
}

/*
 * The same update in fp32, one rounding per operation (this file is built
 * with contraction off, so no fused multiply-add is formed).  It exists to
 * show that the stated tolerance is reachable in fp32; the GPU path is
 * compared with the fp64 evaluation above.
 */
void hzp_oracle_adamw_f32(const hzp_oracle_adamw_t *h, uint64_t n, const float *g,
                          const float *wd_mult, float *p, float *m, float *v,
                          uint16_t *p16, float *p32out)
{
    const float b1 = h->beta1, b2 = h->beta2, lr = h->lr, eps = h->eps, wd = h->weight_decay;
    const float bc1 = (float)(1.0 - pow((double)b1, (double)h->step));
    const float bc2 = (float)(1.0 - pow((double)b2, (double)h->step));
#pragma omp parallel for schedule(static)
    for (int64_t x = 0; x < (int64_t)n; ++x) {
        float gx = g[x];
        float mn = b1 * m[x] + (1.0f - b1) * gx;
        float vn = b2 * v[x] + (1.0f - b2) * gx * gx;
        float u = (mn / bc1) / (sqrtf(vn / bc2) + eps);
        float mult = wd_mult ? wd_mult[x] : 1.0f;
        float pn = p[x] - lr * (u + wd * mult * p[x]);
        m[x] = mn;
        v[x] = vn;
        p[x] = pn;
        if (p16)
            p16[x] = hzp_oracle_f32_to_bf16(pn);
        if (p32out)
            p32out[x] = pn;
    }
}

/*
 * Gather, either level: n_shards equal pieces of `len` elements each are
 * placed one after another:  dst[s*len + x] = src_s[x].  Bit copies of
 * elem_bytes-wide elements (2 for bf16, 4 for fp32).
 *   level 1->3: the K ZeRO-1 owners' outputs form one ZeRO-3 shard;
 *   level 3->layer: the Z3 ZeRO-3 shards form the padded layer bucket.
 */
void hzp_oracle_gather_concat(const void *const *srcs, uint32_t n_shards, uint64_t len,
                              uint32_t elem_bytes, void *dst)
{
    for (uint32_t s = 0; s < n_shards; ++s)
        for (uint64_t x = 0; x < len; ++x)
            for (uint32_t b = 0; b < elem_bytes; ++b)
                ((uint8_t *)dst)[(s * len + x) * elem_bytes + b] =
                    ((const uint8_t *)srcs[s])[x * elem_bytes + b];
}

/*
 * Unpack one tensor out of Z3 shards of `S3` elements each: element y of the
 * tensor sits at bucket position offset+y, i.e. in shard (offset+y) div S3 at
 * (offset+y) mod S3.  Padding is dropped simply by never being addressed.
 */
void hzp_oracle_unpack_tensor(const void *const *shards, uint64_t S3, uint32_t elem_bytes,
                              uint64_t offset, uint64_t numel, void *dst)
{
    for (uint64_t y = 0; y < numel; ++y) {
        uint64_t pos = offset + y;
        uint64_t j = pos / S3, x = pos % S3;
        for (uint32_t b = 0; b < elem_bytes; ++b)
            ((uint8_t *)dst)[y * elem_bytes + b] =
                ((const uint8_t *)shards[j])[x * elem_bytes + b];
    }
}
