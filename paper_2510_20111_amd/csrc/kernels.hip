// HIP kernels of libhzp for CDNA4 (gfx950) and their launchers.
//
// Every kernel here streams: each byte is read once and written once, there is no reuse and
// no contraction, so the bound is HBM bandwidth (26+2R bytes per element for the fused update
// with bf16 gradients, against some tens of fp32 operations).  The design therefore is
//   - one 16-byte load per lane per stream and 8 elements per lane, so a wavefront covers
//     1 KiB of each bf16 stream and 2 KiB of each fp32 stream, fully coalesced;
//   - all R+3 input streams of a lane are requested before the first use, which keeps
//     (R+6) x 16 B per lane in flight;
//   - non-temporal loads and stores: nothing is touched twice, so no line should be kept;
//   - many layers per launch: shards of one layer are only a few MB, so the per-layer
//     pointers travel in the kernel-argument block and one grid covers all of them;
//   - consecutive workgroups take consecutive tiles.  The hardware deals workgroups to the
//     8 XCDs round-robin; with no reuse there is nothing for an XCD-local L2 to keep, and the
//     tiles of any window of workgroups still spread over all memory channels.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>

#include "hzp_internal.hpp"

namespace hzp {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
// Same vector with element alignment only, for sources that follow an unaligned destination.
typedef uint32_t u32x4_a2 __attribute__((ext_vector_type(4), aligned(2)));
typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));

constexpr int kThreads = 256;

template <class T>
__device__ __forceinline__ T ld_stream(const T *p)
{
    return __builtin_nontemporal_load(p);
}
template <class T>
__device__ __forceinline__ void st_stream(T *p, T v)
{
    __builtin_nontemporal_store(v, p);
}

// bf16 pair packed in one 32-bit word (element 0 in the low half) -> two fp32 values.
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// fp32 -> bf16, round to nearest even on the 16 dropped bits; NaN stays a (quiet) NaN.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    const uint32_t u = __float_as_uint(f);
    const uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    const uint32_t quiet = (u >> 16) | 0x40u;
    return (u & 0x7FFFFFFFu) > 0x7F800000u ? quiet : rounded;
}

// Load 8 gradient elements of one contribution as fp32.
template <bool G32>
struct GradVec;
template <>
struct GradVec<false> {
    u32x4 w;
    __device__ __forceinline__ void load(const void *base, uint32_t vec)
    {
        w = ld_stream(reinterpret_cast<const u32x4 *>(base) + vec);
    }
    __device__ __forceinline__ float get(int e) const
    {
        const uint32_t word = w[e >> 1];
        return (e & 1) ? bf16_hi(word) : bf16_lo(word);
    }
};
template <>
struct GradVec<true> {
    f32x4 a, b;
    __device__ __forceinline__ void load(const void *base, uint32_t vec)
    {
        const f32x4 *p = reinterpret_cast<const f32x4 *>(base) + 2 * (size_t)vec;
        a = ld_stream(p);
        b = ld_stream(p + 1);
    }
    __device__ __forceinline__ float get(int e) const { return e < 4 ? a[e] : b[e - 4]; }
};

// ---------------------------------------------------------------------------------------
// Standalone reduction (bit-exact with the scalar definition: fixed order, no contraction).
// ---------------------------------------------------------------------------------------
struct ReduceArgs {
    const void *g[HZP_MAX_REPLICAS];
    float *out;
    uint32_t R;
    uint32_t nvec;      // 8-element vectors in the slice
    float scale;
    int accumulate;
};

template <bool G32, int R_T>
__global__ __launch_bounds__(kThreads) void reduce_kernel(const ReduceArgs a)
{
#pragma clang fp contract(off)
    const uint32_t vec = blockIdx.x * kThreads + threadIdx.x;
    if (vec >= a.nvec) return;
    const uint32_t R = R_T ? (uint32_t)R_T : a.R;
    float s[8];
    if constexpr (R_T != 0) {
        GradVec<G32> g[R_T];
#pragma unroll
        for (int r = 0; r < R_T; ++r) g[r].load(a.g[r], vec);
#pragma unroll
        for (int e = 0; e < 8; ++e) s[e] = g[0].get(e);
#pragma unroll
        for (int r = 1; r < R_T; ++r)
#pragma unroll
            for (int e = 0; e < 8; ++e) s[e] = s[e] + g[r].get(e);
    } else {
        GradVec<G32> g0;
        g0.load(a.g[0], vec);
#pragma unroll
        for (int e = 0; e < 8; ++e) s[e] = g0.get(e);
        for (uint32_t r = 1; r < R; ++r) {
            GradVec<G32> gr;
            gr.load(a.g[r], vec);
#pragma unroll
            for (int e = 0; e < 8; ++e) s[e] = s[e] + gr.get(e);
        }
    }
    f32x4 *o = reinterpret_cast<f32x4 *>(a.out) + 2 * (size_t)vec;
    f32x4 lo, hi;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        lo[e] = a.scale * s[e];
        hi[e] = a.scale * s[e + 4];
    }
    if (a.accumulate) {
        const f32x4 olo = ld_stream(o), ohi = ld_stream(o + 1);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            lo[e] = olo[e] + lo[e];
            hi[e] = ohi[e] + hi[e];
        }
    }
    st_stream(o, lo);
    st_stream(o + 1, hi);
}

// ---------------------------------------------------------------------------------------
// Fused reduce + scale + AdamW + cast over many shard segments (one per layer bucket).
// ---------------------------------------------------------------------------------------
struct AdamScalars {
    float lr, beta1, beta2, one_minus_beta1, one_minus_beta2, eps, weight_decay, grad_scale;
    float inv_bc1, inv_bc2;     // 1/(1-beta1^t), 1/(1-beta2^t), computed in double on the host
};

// Segment table in the kernel-argument block.  Segment s owns workgroups
// [blk_end[s-1], blk_end[s]) and the pointers ptr[s*(R+4) ...]: R gradient slices, master,
// momentum, variance, parameter output (may be null).
template <int MAXSEG, int PTRCAP>
struct SegTable {
    static constexpr int kMaxSeg = MAXSEG;
    static constexpr int kPtrCap = PTRCAP;
    uint32_t nseg;
    uint32_t R;
    uint32_t blk_end[MAXSEG];
    uint32_t nvec[MAXSEG];
    const void *ptr[PTRCAP];
};
typedef SegTable<34, 408> SegTableWide;      // 3544 bytes: 34 layer buckets at R = 8 in one launch
typedef SegTable<20, 280> SegTableNarrow;    // leaves room for the weight-decay lookup arguments

struct WdLookup {
    const uint64_t *tensor_off;     // device: bucket-relative tensor offsets, bucket after bucket
    const float *tensor_wd;         // device: multipliers, same order
    uint32_t first_slot[SegTableNarrow::kMaxSeg];
    uint32_t n_tensors[SegTableNarrow::kMaxSeg];
    uint64_t shard_begin[SegTableNarrow::kMaxSeg];
};
struct NoLookup {};

constexpr int kFusedVecPerThread = 1;
constexpr uint32_t kFusedTile = kThreads * kFusedVecPerThread;      // vectors per workgroup

template <int R_T, bool G32, bool O32, class Seg, class Wd>
__global__ __launch_bounds__(kThreads) void fused_adamw_kernel(const Seg a, const AdamScalars h, const Wd w)
{
    // Which segment does this workgroup belong to?  Uniform binary search in the argument block.
    const uint32_t blk = blockIdx.x;
    uint32_t lo = 0, hi = a.nseg - 1;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (blk < a.blk_end[mid])
            hi = mid;
        else
            lo = mid + 1;
    }
    const uint32_t seg = lo;
    const uint32_t blk0 = seg ? a.blk_end[seg - 1] : 0u;
    const uint32_t R = R_T ? (uint32_t)R_T : a.R;
    const void *const *sp = a.ptr + (size_t)seg * (R + 4);
    const uint32_t nvec = a.nvec[seg];
    f32x4 *const P = reinterpret_cast<f32x4 *>(const_cast<void *>(sp[R]));
    f32x4 *const M = reinterpret_cast<f32x4 *>(const_cast<void *>(sp[R + 1]));
    f32x4 *const V = reinterpret_cast<f32x4 *>(const_cast<void *>(sp[R + 2]));
    void *const OUT = const_cast<void *>(sp[R + 3]);

#pragma unroll
    for (int it = 0; it < kFusedVecPerThread; ++it) {
        const uint32_t vec = (blk - blk0) * kFusedTile + it * kThreads + threadIdx.x;
        if (vec >= nvec) continue;

        // Request every input stream of this lane before using any.
        float g[8];
        f32x4 p0, p1, m0, m1, v0, v1;
        if constexpr (R_T != 0) {
            GradVec<G32> gv[R_T];
#pragma unroll
            for (int r = 0; r < R_T; ++r) gv[r].load(sp[r], vec);
            p0 = ld_stream(P + 2 * (size_t)vec);
            p1 = ld_stream(P + 2 * (size_t)vec + 1);
            m0 = ld_stream(M + 2 * (size_t)vec);
            m1 = ld_stream(M + 2 * (size_t)vec + 1);
            v0 = ld_stream(V + 2 * (size_t)vec);
            v1 = ld_stream(V + 2 * (size_t)vec + 1);
#pragma unroll
            for (int e = 0; e < 8; ++e) g[e] = gv[0].get(e);
#pragma unroll
            for (int r = 1; r < R_T; ++r)
#pragma unroll
                for (int e = 0; e < 8; ++e) g[e] += gv[r].get(e);
        } else {
            p0 = ld_stream(P + 2 * (size_t)vec);
            p1 = ld_stream(P + 2 * (size_t)vec + 1);
            m0 = ld_stream(M + 2 * (size_t)vec);
            m1 = ld_stream(M + 2 * (size_t)vec + 1);
            v0 = ld_stream(V + 2 * (size_t)vec);
            v1 = ld_stream(V + 2 * (size_t)vec + 1);
            GradVec<G32> g0;
            g0.load(sp[0], vec);
#pragma unroll
            for (int e = 0; e < 8; ++e) g[e] = g0.get(e);
            uint32_t r = 1;
            for (; r + 1 < R; r += 2) {     // two contributions in flight, summed in order
                GradVec<G32> ga, gb;
                ga.load(sp[r], vec);
                gb.load(sp[r + 1], vec);
#pragma unroll
                for (int e = 0; e < 8; ++e) g[e] += ga.get(e);
#pragma unroll
                for (int e = 0; e < 8; ++e) g[e] += gb.get(e);
            }
            if (r < R) {
                GradVec<G32> ga;
                ga.load(sp[r], vec);
#pragma unroll
                for (int e = 0; e < 8; ++e) g[e] += ga.get(e);
            }
        }

        float wd = h.weight_decay;
        if constexpr (!std::is_same<Wd, NoLookup>::value) {
            // Every tensor starts on a multiple of A >= 8 elements, so the 8 elements of a
            // vector belong to one tensor: the last one whose offset is <= the position.
            const uint64_t pos = w.shard_begin[seg] + 8ull * vec;
            const uint64_t *off = w.tensor_off + w.first_slot[seg];
            uint32_t tl = 0, th = w.n_tensors[seg] - 1;
            while (tl < th) {
                const uint32_t mid = (tl + th + 1) >> 1;
                if (off[mid] <= pos)
                    tl = mid;
                else
                    th = mid - 1;
            }
            wd *= w.tensor_wd[w.first_slot[seg] + tl];
        }

        float p[8], m[8], v[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            p[e] = p0[e]; p[e + 4] = p1[e];
            m[e] = m0[e]; m[e + 4] = m1[e];
            v[e] = v0[e]; v[e + 4] = v1[e];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float ge = h.grad_scale * g[e];
            m[e] = h.beta1 * m[e] + h.one_minus_beta1 * ge;
            v[e] = h.beta2 * v[e] + h.one_minus_beta2 * ge * ge;
            const float denom = sqrtf(v[e] * h.inv_bc2) + h.eps;
            const float u = (m[e] * h.inv_bc1) / denom;
            p[e] = p[e] - h.lr * (u + wd * p[e]);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            p0[e] = p[e]; p1[e] = p[e + 4];
            m0[e] = m[e]; m1[e] = m[e + 4];
            v0[e] = v[e]; v1[e] = v[e + 4];
        }
        st_stream(P + 2 * (size_t)vec, p0);
        st_stream(P + 2 * (size_t)vec + 1, p1);
        st_stream(M + 2 * (size_t)vec, m0);
        st_stream(M + 2 * (size_t)vec + 1, m1);
        st_stream(V + 2 * (size_t)vec, v0);
        st_stream(V + 2 * (size_t)vec + 1, v1);
        if (OUT) {
            if constexpr (O32) {
                f32x4 *o = reinterpret_cast<f32x4 *>(OUT) + 2 * (size_t)vec;
                st_stream(o, p0);
                st_stream(o + 1, p1);
            } else {
                u32x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    o[e] = f32_to_bf16_bits(p[2 * e]) | (f32_to_bf16_bits(p[2 * e + 1]) << 16);
                st_stream(reinterpret_cast<u32x4 *>(OUT) + vec, o);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Gather: concatenation of equal shards (16-byte vectors; everything is aligned).
// grid = (tiles per shard, number of shards).
// ---------------------------------------------------------------------------------------
struct ConcatArgs {
    const void *src[HZP_MAX_GROUP];
    u32x4 *dst;
    uint32_t vec_per_shard;
};
constexpr int kConcatVecPerThread = 4;

__global__ __launch_bounds__(kThreads) void concat_kernel(const ConcatArgs a)
{
    const uint32_t s = blockIdx.y;
    const u32x4 *src = reinterpret_cast<const u32x4 *>(a.src[s]);
    u32x4 *dst = a.dst + (size_t)s * a.vec_per_shard;
    const uint32_t base = blockIdx.x * (kThreads * kConcatVecPerThread) + threadIdx.x;
    u32x4 val[kConcatVecPerThread];
#pragma unroll
    for (int i = 0; i < kConcatVecPerThread; ++i) {
        const uint32_t vec = base + i * kThreads;
        if (vec < a.vec_per_shard) val[i] = ld_stream(src + vec);
    }
#pragma unroll
    for (int i = 0; i < kConcatVecPerThread; ++i) {
        const uint32_t vec = base + i * kThreads;
        if (vec < a.vec_per_shard) st_stream(dst + vec, val[i]);
    }
}

// ---------------------------------------------------------------------------------------
// Gather + unpack: ZeRO-3 shards -> separate, unpadded tensor buffers.
// One wavefront per chunk of at most kUnpackChunk elements of one piece (a run of one tensor
// inside one shard).  Sources are 16-byte aligned; a destination is only element-aligned, so a
// chunk is written as: up to 15 bytes of single elements to reach a 16-byte boundary of the
// destination, whole 16-byte vectors (whose source is then read unaligned), single elements.
// ---------------------------------------------------------------------------------------
constexpr int kUnpackTensorCap = 400;
struct UnpackArgs {
    const void *shard[HZP_MAX_GROUP];
    void *tensor[kUnpackTensorCap];     // tensor[t - tensor0]
    const Piece *pieces;                // device table of the bucket, pieces [0, n_pieces)
    uint32_t n_pieces;
    uint32_t chunk0, chunk_end;         // chunks handled by this launch
    uint32_t tensor0;
};

template <int ES>   // element size in bytes: 2 or 4
__global__ __launch_bounds__(kThreads) void unpack_kernel(const UnpackArgs a)
{
    constexpr uint32_t VE = 16 / ES;    // elements per vector
    typedef typename std::conditional<ES == 2, uint16_t, uint32_t>::type elem_t;
    typedef typename std::conditional<ES == 2, u32x4_a2, u32x4_a4>::type vec_unaligned_t;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6));
    const uint32_t chunk = a.chunk0 + wave;
    if (chunk >= a.chunk_end) return;
    // last piece whose chunk_begin <= chunk
    uint32_t lo = 0, hi = a.n_pieces - 1;
    while (lo < hi) {
        const uint32_t mid = (lo + hi + 1) >> 1;
        if (a.pieces[mid].chunk_begin <= chunk)
            lo = mid;
        else
            hi = mid - 1;
    }
    const Piece pc = a.pieces[lo];
    const uint64_t first = (uint64_t)(chunk - pc.chunk_begin) * kUnpackChunk;
    const uint64_t left = pc.len - first;
    const uint32_t n = left < kUnpackChunk ? (uint32_t)left : kUnpackChunk;
    const elem_t *src = reinterpret_cast<const elem_t *>(a.shard[pc.shard]) + pc.src_off + first;
    elem_t *dst = reinterpret_cast<elem_t *>(a.tensor[pc.tensor - a.tensor0]) + pc.dst_off + first;

    uint32_t head = (uint32_t)((16u - (uint32_t)(reinterpret_cast<uintptr_t>(dst) & 15u)) & 15u) / ES;
    if (head > n) head = n;
    const uint32_t nbody = (n - head) / VE;
    const uint32_t tail0 = head + nbody * VE;
    if (lane < head) dst[lane] = src[lane];
    if (lane < n - tail0) dst[tail0 + lane] = src[tail0 + lane];

    const elem_t *bsrc = src + head;
    u32x4 *bdst = reinterpret_cast<u32x4 *>(dst + head);
    constexpr int U = 4;
    for (uint32_t q0 = 0; q0 < nbody; q0 += 64 * U) {
        u32x4 val[U];
#pragma unroll
        for (int i = 0; i < U; ++i) {
            const uint32_t q = q0 + i * 64 + lane;
            if (q < nbody) val[i] = __builtin_nontemporal_load(reinterpret_cast<const vec_unaligned_t *>(bsrc + (size_t)q * VE));
        }
#pragma unroll
        for (int i = 0; i < U; ++i) {
            const uint32_t q = q0 + i * 64 + lane;
            if (q < nbody) st_stream(bdst + q, val[i]);
        }
    }
}

// ---------------------------------------------------------------------------------------
// Launchers (host).  Arguments were validated by the callers in api.cpp.
// ---------------------------------------------------------------------------------------
static hzp_status_t check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(HZP_ERR_HIP, "%s: launch failed: %s", what, hipGetErrorString(e));
    return HZP_OK;
}

hzp_status_t launch_reduce(bool g32, const void *const *slices, uint32_t R, uint64_t n, float scale,
                           int accumulate, float *out, hipStream_t stream)
{
    if (n == 0) return HZP_OK;
    ReduceArgs a{};
    for (uint32_t r = 0; r < R; ++r) a.g[r] = slices[r];
    a.out = out;
    a.R = R;
    a.nvec = (uint32_t)(n / 8);
    a.scale = scale;
    a.accumulate = accumulate;
    const dim3 grid((a.nvec + kThreads - 1) / kThreads), block(kThreads);
#define HZP_REDUCE_CASE(G, RT) hipLaunchKernelGGL((reduce_kernel<G, RT>), grid, block, 0, stream, a)
    if (!g32) {
        switch (R) {
        case 4: HZP_REDUCE_CASE(false, 4); break;
        case 8: HZP_REDUCE_CASE(false, 8); break;
        case 16: HZP_REDUCE_CASE(false, 16); break;
        default: HZP_REDUCE_CASE(false, 0); break;
        }
    } else {
        switch (R) {
        case 4: HZP_REDUCE_CASE(true, 4); break;
        case 8: HZP_REDUCE_CASE(true, 8); break;
        default: HZP_REDUCE_CASE(true, 0); break;
        }
    }
#undef HZP_REDUCE_CASE
    return check_launch("hzp_reduce_shard");
}

template <class Seg, class Wd>
static void launch_fused_variant(bool g32, bool o32, uint32_t R, const Seg &a, const AdamScalars &h,
                                 const Wd &w, uint32_t blocks, hipStream_t stream)
{
    const dim3 grid(blocks), block(kThreads);
#define HZP_FUSED_CASE(RT, G, O) \
    hipLaunchKernelGGL((fused_adamw_kernel<RT, G, O, Seg, Wd>), grid, block, 0, stream, a, h, w)
    if (!g32 && !o32) {
        switch (R) {
        case 4: HZP_FUSED_CASE(4, false, false); break;
        case 8: HZP_FUSED_CASE(8, false, false); break;
        case 16: HZP_FUSED_CASE(16, false, false); break;
        default: HZP_FUSED_CASE(0, false, false); break;
        }
    } else if (g32 && o32) {
        HZP_FUSED_CASE(0, true, true);
    } else if (g32 && !o32) {
        HZP_FUSED_CASE(0, true, false);
    } else {
        HZP_FUSED_CASE(0, false, true);
    }
#undef HZP_FUSED_CASE
}

template <class Seg>
static hzp_status_t launch_fused_table(const hzp_plan_t *plan, bool use_wd, bool g32, bool o32, uint32_t R,
                                       const FusedSegment *segs, size_t nseg, const AdamScalars &h,
                                       hipStream_t stream)
{
    const DeviceTables *tab = nullptr;
    if (use_wd) {
        hzp_status_t st = device_tables(plan, &tab);
        if (st != HZP_OK) return st;
    }
    const uint32_t per_seg = R + 4;
    const size_t cap = std::min<size_t>(Seg::kMaxSeg, Seg::kPtrCap / per_seg);
    size_t s0 = 0;
    while (s0 < nseg) {
        Seg a{};
        WdLookup w{};
        uint32_t blocks = 0;
        uint32_t cnt = 0;
        for (; s0 + cnt < nseg && cnt < cap; ++cnt) {
            const FusedSegment &f = segs[s0 + cnt];
            const uint32_t nvec = (uint32_t)(f.n / 8);
            const uint32_t nb = (nvec + kFusedTile - 1) / kFusedTile;
            if (blocks + nb < blocks || blocks + nb > 0x7FFFFFFFu) break;   // start another launch
            blocks += nb;
            a.blk_end[cnt] = blocks;
            a.nvec[cnt] = nvec;
            const void **sp = a.ptr + (size_t)cnt * per_seg;
            for (uint32_t r = 0; r < R; ++r) sp[r] = f.grads[r];
            sp[R] = f.master;
            sp[R + 1] = f.m;
            sp[R + 2] = f.v;
            sp[R + 3] = f.out;
            if constexpr (std::is_same<Seg, SegTableNarrow>::value) {
                w.first_slot[cnt] = f.first_slot;
                w.n_tensors[cnt] = f.n_tensors;
                w.shard_begin[cnt] = f.shard_begin;
            }
        }
        if (cnt == 0) return fail(HZP_ERR_UNSUPPORTED, "hzp_adamw_shard: shard too large for one launch");
        a.nseg = cnt;
        a.R = R;
        if (blocks > 0) {
            if constexpr (std::is_same<Seg, SegTableNarrow>::value) {
                w.tensor_off = tab->tensor_off;
                w.tensor_wd = tab->tensor_wd;
                launch_fused_variant(g32, o32, R, a, h, w, blocks, stream);
            } else {
                launch_fused_variant(g32, o32, R, a, h, NoLookup{}, blocks, stream);
            }
            hzp_status_t st = check_launch("hzp_adamw_shard");
            if (st != HZP_OK) return st;
        }
        s0 += cnt;
    }
    return HZP_OK;
}

hzp_status_t launch_fused(const hzp_plan_t *plan, bool g32, bool o32, uint32_t R, const FusedSegment *segs,
                          size_t nseg, const hzp_adamw_t &hy, hipStream_t stream)
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
    if (plan->uniform_wd)
        return launch_fused_table<SegTableWide>(plan, false, g32, o32, R, segs, nseg, h, stream);
    return launch_fused_table<SegTableNarrow>(plan, true, g32, o32, R, segs, nseg, h, stream);
}

hzp_status_t launch_concat(const void *const *srcs, uint32_t n_shards, uint64_t bytes_per_shard, void *dst,
                           hipStream_t stream)
{
    if (bytes_per_shard == 0) return HZP_OK;
    const uint64_t nvec = bytes_per_shard / 16;
    if (nvec > 0xFFFFFFFFull) return fail(HZP_ERR_UNSUPPORTED, "hzp_gather_layer: shard larger than 64 GiB");
    ConcatArgs a{};
    for (uint32_t s = 0; s < n_shards; ++s) a.src[s] = srcs[s];
    a.dst = reinterpret_cast<u32x4 *>(dst);
    a.vec_per_shard = (uint32_t)nvec;
    const uint32_t per_block = kThreads * kConcatVecPerThread;
    const dim3 grid((uint32_t)((nvec + per_block - 1) / per_block), n_shards), block(kThreads);
    hipLaunchKernelGGL(concat_kernel, grid, block, 0, stream, a);
    return check_launch("hzp_gather_layer");
}

hzp_status_t launch_unpack(const hzp_plan_t *plan, const BucketRec &b, const void *const *shards,
                           uint32_t n_shards, void *const *tensors, hipStream_t stream)
{
    const DeviceTables *tab = nullptr;
    hzp_status_t st = device_tables(plan, &tab);
    if (st != HZP_OK) return st;
    const uint32_t waves_per_block = kThreads / 64;
    // Tensors travel in the argument block, kUnpackTensorCap at a time; pieces are sorted by tensor.
    size_t p0 = 0;
    for (uint32_t t0 = 0; t0 < b.n_tensors; t0 += kUnpackTensorCap) {
        const uint32_t t1 = std::min<uint32_t>(b.n_tensors, t0 + kUnpackTensorCap);
        size_t p1 = p0;
        while (p1 < b.pieces.size() && b.pieces[p1].tensor < t1) ++p1;
        UnpackArgs a{};
        for (uint32_t s = 0; s < n_shards; ++s) a.shard[s] = shards[s];
        for (uint32_t t = t0; t < t1; ++t) a.tensor[t - t0] = tensors[t];
        a.pieces = tab->pieces + b.piece_slot;
        a.n_pieces = (uint32_t)b.pieces.size();
        a.chunk0 = b.pieces[p0].chunk_begin;
        a.chunk_end = p1 < b.pieces.size() ? b.pieces[p1].chunk_begin : b.n_chunks;
        a.tensor0 = t0;
        const uint32_t chunks = a.chunk_end - a.chunk0;
        const dim3 grid((chunks + waves_per_block - 1) / waves_per_block), block(kThreads);
        if (b.cls == HZP_CLASS_F32)
            hipLaunchKernelGGL(unpack_kernel<4>, grid, block, 0, stream, a);
        else
            hipLaunchKernelGGL(unpack_kernel<2>, grid, block, 0, stream, a);
        st = check_launch("hzp_gather_layer");
        if (st != HZP_OK) return st;
        p0 = p1;
    }
    return HZP_OK;
}

// ---------------------------------------------------------------------------------------
// Per-plan, per-device lookup tables.
// ---------------------------------------------------------------------------------------
hzp_status_t device_tables(const hzp_plan_t *plan, const DeviceTables **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(HZP_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    std::lock_guard<std::mutex> lock(plan->mu);
    for (const DeviceTables &t : plan->dev)
        if (t.device == dev) {
            *out = &t;
            return HZP_OK;
        }
    DeviceTables t;
    t.device = dev;
    std::vector<Piece> all;
    for (const BucketRec &b : plan->buckets) all.insert(all.end(), b.pieces.begin(), b.pieces.end());
    const size_t nt = plan->slot_off.size();
    auto upload = [&](void **dptr, const void *src, size_t bytes) -> hipError_t {
        hipError_t err = hipMalloc(dptr, bytes ? bytes : 16);
        if (err != hipSuccess) return err;
        return bytes ? hipMemcpy(*dptr, src, bytes, hipMemcpyHostToDevice) : hipSuccess;
    };
    e = upload((void **)&t.tensor_off, plan->slot_off.data(), nt * sizeof(uint64_t));
    if (e == hipSuccess) e = upload((void **)&t.tensor_wd, plan->slot_wd.data(), nt * sizeof(float));
    if (e == hipSuccess) e = upload((void **)&t.pieces, all.data(), all.size() * sizeof(Piece));
    if (e != hipSuccess) {
        (void)hipFree(t.tensor_off);
        (void)hipFree(t.tensor_wd);
        (void)hipFree(t.pieces);
        return fail(e == hipErrorOutOfMemory ? HZP_ERR_NOMEM : HZP_ERR_HIP, "device tables: %s",
                    hipGetErrorString(e));
    }
    // The vector may only grow while no reader holds a pointer into it: reserve once.
    if (plan->dev.capacity() == 0) plan->dev.reserve(64);
    if (plan->dev.size() == plan->dev.capacity())
        return fail(HZP_ERR_UNSUPPORTED, "plan used on more than 64 devices");
    plan->dev.push_back(t);
    *out = &plan->dev.back();
    return HZP_OK;
}

void free_device_tables(hzp_plan_t *plan)
{
    for (DeviceTables &t : plan->dev) {
        int cur = -1;
        if (hipGetDevice(&cur) == hipSuccess && cur != t.device) (void)hipSetDevice(t.device);
        (void)hipFree(t.tensor_off);
        (void)hipFree(t.tensor_wd);
        (void)hipFree(t.pieces);
        if (cur >= 0 && cur != t.device) (void)hipSetDevice(cur);
    }
    plan->dev.clear();
}

}  // namespace hzp
