// HIP kernels of libhzp for CDNA4 (gfx950) and their launchers.
//
// Every kernel here streams: each byte is read once and written once, there is no reuse and
// no contraction, so the bound is HBM bandwidth (26+2R bytes per element for the fused update
// with bf16 gradients, against about 30 fp32 operations).  The design therefore is
//   - every load/store instruction of a wavefront covers one contiguous run of memory, and a
//     lane requests all of its (R+3) x 2 input vectors before it uses the first one;
//   - single-wavefront workgroups, dispatched in address order, and for the many-stream fused
//     update only about 5 of them resident per CU: a small, coherent front of in-flight
//     groups serves the memory controllers better than full occupancy;
//   - non-temporal loads, and stores that are written through to memory with the streaming
//     hint: nothing is touched twice, so no line should be kept;
//   - many layers per launch: shards of one layer are only a few MB, so the per-layer
//     pointers travel in the kernel-argument block and one grid covers all of them;
//   - consecutive workgroups take consecutive tiles.  The hardware deals workgroups to the
//     8 XCDs round-robin; with no reuse there is nothing for an XCD-local L2 to keep, the
//     tiles of any window of workgroups still spread over all memory channels, and a remap
//     that gives each XCD its own contiguous eighth measured 5 % slower.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <vector>

#include "hzp_internal.hpp"

namespace hzp {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
// Same vector with element alignment only, for sources that follow an unaligned destination.
typedef uint32_t u32x4_a2 __attribute__((ext_vector_type(4), aligned(2)));
typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));

template <class T>
__device__ __forceinline__ T ld_stream(const T *p)
{
    return __builtin_nontemporal_load(p);
}

// Element (vector) `idx` of a stream whose base is uniform: base + 32-bit byte offset, so that the
// access uses a scalar base register and one VGPR offset.  Callers keep streams below 4 GiB.
template <class T>
__device__ __forceinline__ const T *at(const void *base, uint32_t idx)
{
    return reinterpret_cast<const T *>(reinterpret_cast<const char *>(base) + idx * (uint32_t)sizeof(T));
}
template <class T>
__device__ __forceinline__ T *at(void *base, uint32_t idx)
{
    return reinterpret_cast<T *>(reinterpret_cast<char *>(base) + idx * (uint32_t)sizeof(T));
}

// Streaming store with write-through to memory: system scope plus the non-temporal hint.  Measured
// on MI355X, the many concurrent write streams of the fused update drain 1-4 % faster with these
// cache-policy bits than with the non-temporal hint alone.  The compiler has no source-level way
// to ask for this combination on a 16-byte store, hence the instruction is written out.  The
// trailing s_nop keeps the two wait states this hardware generation needs between a store of more
// than 8 bytes and an overwrite of its data registers (the compiler cannot see inside the asm to
// add them; with one wait state the first dword of some lanes was stored from the next value
// when the store pipeline was under pressure).
__device__ __forceinline__ void st_writethrough(void *base, uint32_t byte_off, f32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, %2 sc0 sc1 nt\n\ts_nop 1" ::"v"(byte_off), "v"(v), "s"(base) : "memory");
}
// The same store for a full 64-bit address in a VGPR pair (copy kernels, whose lanes compute their
// own destination).
__device__ __forceinline__ void st_writethrough(u32x4 *dst, u32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_nop 1" ::"v"(dst), "v"(v) : "memory");
}
__device__ __forceinline__ void st_writethrough(void *base, uint32_t byte_off, u32x2 v)
{
    asm volatile("global_store_dwordx2 %0, %1, %2 sc0 sc1 nt" ::"v"(byte_off), "v"(v), "s"(base) : "memory");
}

// bf16 pair packed in one 32-bit word (element 0 in the low half) -> two fp32 values.
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Two fp32 -> packed bf16 pair (first value in the low half), round to nearest even, NaN stays a
// quiet NaN: gfx950's packed conversion instruction.
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    const f32x2 x = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

// ---------------------------------------------------------------------------------------
// Work decomposition of the element-wise kernels.
//
// A workgroup is ONE wavefront and owns one group of 512 consecutive elements.  Lane l works on
// two quads of 4 elements: [4l, 4l+4) and [256+4l, 256+4l+4) of the group.  With that mapping
// every load/store instruction of the wavefront covers one contiguous run (1 KiB of an fp32
// stream, 512 B of a bf16 stream), and the fp32 and bf16 streams give each lane the same
// elements.  Measured on MI355X, single-wavefront workgroups with whole-instruction contiguity
// stream the 15-19 concurrent address streams of the fused update about 10 % faster than
// 256-thread workgroups whose lanes read 32 contiguous bytes of the fp32 streams.
// Shards are multiples of 8 elements, so a quad is never split; only the last group of a
// segment can be partly filled, and its lanes are predicated per quad.
// ---------------------------------------------------------------------------------------
constexpr int kWave = 64;
constexpr uint32_t kGroupQuads = 128;       // quads per group (512 elements)

// Four gradient elements of one contribution, widened to fp32 on access.
template <bool G32>
struct GradQuad;
template <>
struct GradQuad<false> {
    u32x2 w;
    __device__ __forceinline__ void load(const void *base, uint32_t quad) { w = ld_stream(at<u32x2>(base, quad)); }
    __device__ __forceinline__ float get(int e) const
    {
        const uint32_t word = w[e >> 1];
        return (e & 1) ? bf16_hi(word) : bf16_lo(word);
    }
};
template <>
struct GradQuad<true> {
    f32x4 a;
    __device__ __forceinline__ void load(const void *base, uint32_t quad) { a = ld_stream(at<f32x4>(base, quad)); }
    __device__ __forceinline__ float get(int e) const { return a[e]; }
};

// Issue the loads of R_T contributions for the lane's two quads (valid[h]: quad h exists).
template <int R_T, bool G32, bool FULL>
__device__ __forceinline__ void load_contributions(GradQuad<G32> (&g)[R_T][2], const void *const *slices,
                                                   const uint32_t quad[2], const bool valid[2])
{
#pragma unroll
    for (int r = 0; r < R_T; ++r)
#pragma unroll
        for (int h = 0; h < 2; ++h)
            if (FULL || valid[h]) g[r][h].load(slices[r], quad[h]);
}

// Left-to-right fp32 sum of loaded contributions: ((g0 + g1) + g2) + ...
template <int R_T, bool G32>
__device__ __forceinline__ void sum_loaded(const GradQuad<G32> (&g)[R_T][2], float s[2][4])
{
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int e = 0; e < 4; ++e) s[h][e] = g[0][h].get(e);
#pragma unroll
    for (int r = 1; r < R_T; ++r)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int e = 0; e < 4; ++e) s[h][e] = s[h][e] + g[r][h].get(e);
}

// The same sum for a run-time R: two contributions in flight, still added in order.
template <bool G32, bool FULL>
__device__ __forceinline__ void sum_contributions_loop(const void *const *slices, uint32_t R, const uint32_t quad[2],
                                                       const bool valid[2], float s[2][4])
{
    GradQuad<G32> g0[2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
        if (FULL || valid[h]) g0[h].load(slices[0], quad[h]);
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int e = 0; e < 4; ++e) s[h][e] = g0[h].get(e);
    uint32_t r = 1;
    for (; r + 1 < R; r += 2) {
        GradQuad<G32> ga[2], gb[2];
#pragma unroll
        for (int h = 0; h < 2; ++h)
            if (FULL || valid[h]) {
                ga[h].load(slices[r], quad[h]);
                gb[h].load(slices[r + 1], quad[h]);
            }
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int e = 0; e < 4; ++e) s[h][e] = s[h][e] + ga[h].get(e);
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int e = 0; e < 4; ++e) s[h][e] = s[h][e] + gb[h].get(e);
    }
    if (r < R) {
        GradQuad<G32> ga[2];
#pragma unroll
        for (int h = 0; h < 2; ++h)
            if (FULL || valid[h]) ga[h].load(slices[r], quad[h]);
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int e = 0; e < 4; ++e) s[h][e] = s[h][e] + ga[h].get(e);
    }
}

// ---------------------------------------------------------------------------------------
// Standalone reduction (bit-exact with the scalar definition: fixed order, no contraction).
// ---------------------------------------------------------------------------------------
struct ReduceArgs {
    const void *g[HZP_MAX_REPLICAS];
    float *out;
    uint32_t R;
    uint32_t nquad;     // 4-element quads in the slice
    float scale;
    int accumulate;
};

template <bool G32, int R_T, bool FULL>
__device__ __forceinline__ void reduce_group(const ReduceArgs &a, const uint32_t quad[2], const bool valid[2])
{
#pragma clang fp contract(off)
    float s[2][4];
    f32x4 prev[2];
    if (a.accumulate) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
            if (FULL || valid[h]) prev[h] = ld_stream(at<f32x4>((const void *)a.out, quad[h]));
    }
    if constexpr (R_T != 0) {
        GradQuad<G32> g[R_T][2];
        load_contributions<R_T, G32, FULL>(g, a.g, quad, valid);
        __builtin_amdgcn_sched_barrier(0);      // every load is issued before the first add
        sum_loaded<R_T, G32>(g, s);
    } else {
        sum_contributions_loop<G32, FULL>(a.g, a.R, quad, valid, s);
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        f32x4 t;
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] = a.scale * s[h][e];
        if (a.accumulate) {
#pragma unroll
            for (int e = 0; e < 4; ++e) t[e] = prev[h][e] + t[e];
        }
        if (FULL || valid[h]) st_writethrough((void *)a.out, quad[h] * 16u, t);
    }
}

template <bool G32, int R_T>
__global__ __launch_bounds__(kWave) void reduce_kernel(const ReduceArgs a)
{
    const uint32_t q0 = blockIdx.x * kGroupQuads + threadIdx.x;
    const uint32_t quad[2] = {q0, q0 + kWave};
    const bool valid[2] = {quad[0] < a.nquad, quad[1] < a.nquad};
    if ((uint64_t)(blockIdx.x + 1) * kGroupQuads <= a.nquad)
        reduce_group<G32, R_T, true>(a, quad, valid);
    else
        reduce_group<G32, R_T, false>(a, quad, valid);
}

// ---------------------------------------------------------------------------------------
// Fused reduce + scale + AdamW + cast over many shard segments (one per layer bucket).
// ---------------------------------------------------------------------------------------
// Where a launch finds the step's scalars: in its argument block, or in device memory (a captured
// launch then takes each replay's values from there).
struct ScalarsInMemory {
    const AdamScalars *p;
};
__device__ __forceinline__ const AdamScalars &scalars_of(const AdamScalars &h) { return h; }
__device__ __forceinline__ AdamScalars scalars_of(const ScalarsInMemory &h) { return *h.p; }

// Segment table in the kernel-argument block.  Segment s owns workgroups
// [blk_end[s-1], blk_end[s]) and the pointers ptr[s*(R+4) ...]: R gradient slices, master,
// momentum, variance, parameter output (may be null).
template <int MAXSEG, int PTRCAP>
struct SegTable {
    static constexpr int kMaxSeg = MAXSEG;
    static constexpr int kPtrCap = PTRCAP;
    uint32_t nseg;
    uint32_t R;
    uint32_t grid2d;            // 1: grid is (groups, segments) and blk_end[s] is segment s's group count
    uint32_t pad_;
    uint32_t blk_end[MAXSEG];   // flat grid: running total of groups up to and including segment s
    uint32_t nquad[MAXSEG];
    const void *ptr[PTRCAP];
};
typedef SegTable<34, 408> SegTableWide;      // 3552 bytes: 34 layer buckets at R = 8 in one launch
typedef SegTable<20, 280> SegTableNarrow;    // leaves room for the weight-decay lookup arguments

struct WdLookup {
    const uint64_t *tensor_off;     // device: bucket-relative tensor offsets, bucket after bucket
    const float *tensor_wd;         // device: multipliers, same order
    uint32_t first_slot[SegTableNarrow::kMaxSeg];
    uint32_t n_tensors[SegTableNarrow::kMaxSeg];
    uint64_t shard_begin[SegTableNarrow::kMaxSeg];
};
struct NoLookup {};

template <int R_T, bool G32, bool O32, bool FULL, class Wd>
__device__ __forceinline__ void fused_group(const void *const *sp, uint32_t R, const AdamScalars &h, const Wd &w,
                                            uint32_t seg, const uint32_t quad[2], const bool valid[2])
{
    void *const P = const_cast<void *>(sp[R]);
    void *const M = const_cast<void *>(sp[R + 1]);
    void *const V = const_cast<void *>(sp[R + 2]);
    void *const OUT = const_cast<void *>(sp[R + 3]);

    // Request the R gradient streams (used first), then the state streams; a scheduling barrier
    // keeps all of the lane's (R+3) x 2 loads above the first use, otherwise the scheduler sinks
    // the loads that are needed last and the wavefront pays two memory round trips.
    f32x4 p[2], m[2], v[2];
    float g[2][4];
    auto load_state = [&]() {
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
            if (FULL || valid[hh]) {
                p[hh] = ld_stream(at<f32x4>((const void *)P, quad[hh]));
                m[hh] = ld_stream(at<f32x4>((const void *)M, quad[hh]));
                v[hh] = ld_stream(at<f32x4>((const void *)V, quad[hh]));
            }
    };
    if constexpr (R_T != 0) {
        GradQuad<G32> gq[R_T][2];
        load_contributions<R_T, G32, FULL>(gq, sp, quad, valid);
        load_state();
        __builtin_amdgcn_sched_barrier(0);
        sum_loaded<R_T, G32>(gq, g);
    } else {
        load_state();
        sum_contributions_loop<G32, FULL>(sp, R, quad, valid, g);
    }

    float wd[2] = {h.weight_decay, h.weight_decay};
    if constexpr (!std::is_same<Wd, NoLookup>::value) {
        // Every tensor starts on a multiple of A >= 8 elements, so the 4 elements of a quad
        // belong to one tensor: the last one whose offset is <= the quad's bucket position.
        const uint64_t *off = w.tensor_off + w.first_slot[seg];
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const uint64_t pos = w.shard_begin[seg] + 4ull * quad[hh];
            uint32_t tl = 0, th = w.n_tensors[seg] - 1;
            while (tl < th) {
                const uint32_t mid = (tl + th + 1) >> 1;
                if (off[mid] <= pos)
                    tl = mid;
                else
                    th = mid - 1;
            }
            wd[hh] *= w.tensor_wd[w.first_slot[seg] + tl];
        }
    }

    // The arithmetic is not hidden behind other wavefronts (few are resident by design), so it is
    // kept short: hardware square root and reciprocal (1 ulp each) instead of the correctly
    // rounded expansions.  Their error enters p only through lr*u, far below the tolerance.
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float ge = h.grad_scale * g[hh][e];
            const float mn = h.beta1 * m[hh][e] + h.one_minus_beta1 * ge;
            const float vn = h.beta2 * v[hh][e] + (h.one_minus_beta2 * ge) * ge;
            const float denom = __builtin_amdgcn_sqrtf(vn * h.inv_bc2) + h.eps;
            const float u = (mn * h.inv_bc1) * __builtin_amdgcn_rcpf(denom);
            const float pe = p[hh][e];
            m[hh][e] = mn;
            v[hh][e] = vn;
            p[hh][e] = pe - h.lr * (u + wd[hh] * pe);
        }
    }
#pragma unroll
    for (int hh = 0; hh < 2; ++hh)
        if (FULL || valid[hh]) {
            st_writethrough(P, quad[hh] * 16u, p[hh]);
            st_writethrough(M, quad[hh] * 16u, m[hh]);
            st_writethrough(V, quad[hh] * 16u, v[hh]);
        }
    if (OUT) {
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
            if (FULL || valid[hh]) {
                if constexpr (O32) {
                    st_writethrough(OUT, quad[hh] * 16u, p[hh]);
                } else {
                    u32x2 o;
                    o[0] = pack_bf16(p[hh][0], p[hh][1]);
                    o[1] = pack_bf16(p[hh][2], p[hh][3]);
                    st_writethrough(OUT, quad[hh] * 8u, o);
                }
            }
    }
}

// Unused LDS requested at launch so that at most 5 single-wavefront workgroups are resident per
// CU.  With 15-19 address streams, a smaller, more coherent front of in-flight groups serves the
// memory controllers better than full occupancy; each wavefront already keeps (R+3) x 2 loads
// in flight.  Measured optimum on MI355X: 4-6 wavefronts per CU.
constexpr unsigned kFusedLdsBytes = 32768;

template <int R_T, bool G32, bool O32, class Seg, class H, class Wd>
__global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(1, 2))) void fused_adamw_kernel(const Seg a, const H h, const Wd w)
{
    // Which segment and which group of it?  When the segments are of similar length the grid is
    // two-dimensional (y = segment, x = group; surplus workgroups of shorter segments leave at
    // once) and nothing is looked up; otherwise the grid is flat and a uniform binary search over
    // the table in the argument block finds the segment.  With few wavefronts resident, the
    // search's chain of dependent scalar loads would delay every wavefront's first memory request.
    uint32_t seg, grp;
    if (a.grid2d) {
        seg = blockIdx.y;
        grp = blockIdx.x;
        if (grp >= a.blk_end[seg]) return;      // holds the segment's own group count in this mode
    } else {
        const uint32_t blk = blockIdx.x;
        uint32_t lo = 0, hi = a.nseg - 1;
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if (blk < a.blk_end[mid])
                hi = mid;
            else
                lo = mid + 1;
        }
        seg = lo;
        grp = blk - (seg ? a.blk_end[seg - 1] : 0u);
    }
    const uint32_t R = R_T ? (uint32_t)R_T : a.R;
    const void *const *sp = a.ptr + (size_t)seg * (R + 4);
    const uint32_t nquad = a.nquad[seg];
    const uint32_t q0 = grp * kGroupQuads + threadIdx.x;
    const uint32_t quad[2] = {q0, q0 + kWave};
    const bool valid[2] = {quad[0] < nquad, quad[1] < nquad};
    if ((uint64_t)(grp + 1) * kGroupQuads <= nquad)
        fused_group<R_T, G32, O32, true>(sp, R, scalars_of(h), w, seg, quad, valid);
    else
        fused_group<R_T, G32, O32, false>(sp, R, scalars_of(h), w, seg, quad, valid);
}

// ---------------------------------------------------------------------------------------
// Gather: concatenation of equal shards (16-byte vectors; everything is aligned).
// grid = (wavefront tiles per shard, number of shards).
// ---------------------------------------------------------------------------------------
struct ConcatArgs {
    const void *src[HZP_MAX_GROUP];     // the pieces that are copied (one that already lies in place is left out)
    uint8_t slot[HZP_MAX_GROUP];        // position of each of them in the output
    u32x4 *dst;
    uint32_t vec_per_shard;
};
// One wavefront per workgroup, one 16-byte vector per lane: of the shapes measured (1-8 vectors
// per lane, 64- and 256-thread workgroups, with and without an occupancy cap) this one copies
// fastest on MI355X (6.8 TB/s on the 8 x 51 MB -> 405 MB layer gather); a plain copy keeps few
// bytes in flight per wavefront and wants every wave slot filled.
__global__ __launch_bounds__(kWave) void concat_kernel(const ConcatArgs a)
{
    const uint32_t s = blockIdx.y;
    const uint32_t vec = blockIdx.x * kWave + threadIdx.x;
    if (vec >= a.vec_per_shard) return;
    const u32x4 val = ld_stream(reinterpret_cast<const u32x4 *>(a.src[s]) + vec);
    u32x4 *dst = a.dst + (size_t)a.slot[s] * a.vec_per_shard + vec;
    st_writethrough(dst, val);
}

// The same copy for the buckets of many layers in one launch (the post-step gather runs for all
// layers at once; 34 launches of 16 us each leave the memory system idle between them).
// grid = (tiles of the longest piece, pieces to copy of all layers); a piece that already lies in
// place is left out of the list.  Everything a workgroup needs is indexed by its piece alone (one
// round of scalar loads before the first vector load).
constexpr int kLayersPieceCap = 192;
struct ConcatLayersArgs {
    const void *src[kLayersPieceCap];
    u32x4 *dst[kLayersPieceCap];            // where the piece goes
    uint32_t nvec[kLayersPieceCap];         // its length in 16-byte vectors
};
static_assert(sizeof(ConcatLayersArgs) <= 4096, "kernel arguments");
__global__ __launch_bounds__(kWave) void concat_layers_kernel(const ConcatLayersArgs a)
{
    const uint32_t s = blockIdx.y;
    const uint32_t vec = blockIdx.x * kWave + threadIdx.x;
    if (vec >= a.nvec[s]) return;
    const u32x4 val = ld_stream(reinterpret_cast<const u32x4 *>(a.src[s]) + vec);
    st_writethrough(a.dst[s] + vec, val);
}

// The same copy for pieces of different lengths (a ZeRO-3 shard rebuilt from whole and partial
// ZeRO-1 shards when the group sizes do not nest).  One-dimensional grid over the 64-vector tiles
// of all pieces; a workgroup finds its piece by scanning the tile prefix (at most HZP_MAX_GROUP
// uniform compares), so no workgroup is launched for nothing.
struct ConcatRangesArgs {
    const void *src[HZP_MAX_GROUP];         // first vector to read of each piece
    uint32_t dst_vec[HZP_MAX_GROUP];        // where it goes, in 16-byte vectors from dst
    uint32_t nvec[HZP_MAX_GROUP];
    uint32_t tile_end[HZP_MAX_GROUP];       // running count of tiles up to and including the piece
    u32x4 *dst;
    uint32_t n;
};
__global__ __launch_bounds__(kWave) void concat_ranges_kernel(const ConcatRangesArgs a)
{
    uint32_t s = 0;
    while (s + 1 < a.n && blockIdx.x >= a.tile_end[s]) ++s;
    const uint32_t tile = blockIdx.x - (s ? a.tile_end[s - 1] : 0u);
    const uint32_t vec = tile * kWave + threadIdx.x;
    if (vec >= a.nvec[s]) return;
    const u32x4 val = ld_stream(reinterpret_cast<const u32x4 *>(a.src[s]) + vec);
    st_writethrough(a.dst + (size_t)a.dst_vec[s] + vec, val);
}

// ---------------------------------------------------------------------------------------
// Gather + unpack: ZeRO-3 shards -> separate, unpadded tensor buffers.
// One single-wavefront workgroup per chunk of at most kUnpackChunk elements of one piece (a run of
// one tensor inside one shard).  1024-element chunks measured fastest on MI355X (6.5-6.6 TB/s on
// dense and MoE layers; 4096: 6.0, 16384: 5.4, 512: 5.3-6.0): like the plain copy, this kernel
// wants little work per wavefront and every wave slot filled.  Sources are 16-byte aligned; a
// destination is only element-aligned, so a chunk is written as: up to 15 bytes of single
// elements to reach a 16-byte boundary of the destination, whole 16-byte vectors (whose source is
// then read unaligned), single elements.
// ---------------------------------------------------------------------------------------
constexpr int kUnpackTensorCap = 400;
struct UnpackArgs {
    const void *shard[HZP_MAX_GROUP];
    void *tensor[kUnpackTensorCap];     // tensor[t - tensor0]
    const Piece *pieces;                // device table of the bucket, pieces [0, n_pieces)
    const uint32_t *piece_chunk;        // device: chunk_begin of the same pieces, densely packed
    uint32_t n_pieces;
    uint32_t chunk0, chunk_end;         // chunks handled by this launch
    uint32_t tensor0;
};

template <int ES>   // element size in bytes: 2 or 4
__global__ __launch_bounds__(kWave) void unpack_kernel(const UnpackArgs a)
{
    constexpr uint32_t VE = 16 / ES;    // elements per vector
    typedef typename std::conditional<ES == 2, uint16_t, uint32_t>::type elem_t;
    typedef typename std::conditional<ES == 2, u32x4_a2, u32x4_a4>::type vec_unaligned_t;
    const uint32_t lane = threadIdx.x;
    const uint32_t chunk = a.chunk0 + blockIdx.x;
    // Last piece whose chunk_begin <= chunk, by a 64-ary search: every lane probes one pivot and
    // a ballot counts the pivots at or below the chunk.  One round covers 64 pieces, two 4096.
    uint32_t lo = 0, n = a.n_pieces;
    while (n > kWave) {
        const uint32_t stride = (n + kWave - 1) / kWave;
        const uint32_t off = lane * stride;
        const bool le = off < n && a.piece_chunk[lo + off] <= chunk;
        const uint32_t c = (uint32_t)__popcll(__ballot(le));       // >= 1: piece lo is at or below
        const uint32_t step = (c - 1) * stride;
        n = n - step < stride ? n - step : stride;
        lo += step;
    }
    const bool le = lane < n && a.piece_chunk[lo + lane] <= chunk;
    const uint32_t piece = __builtin_amdgcn_readfirstlane(lo + (uint32_t)__popcll(__ballot(le)) - 1u);
    const Piece pc = a.pieces[piece];
    const uint64_t first = (uint64_t)(chunk - pc.chunk_begin) * kUnpackChunk;
    const uint64_t left = pc.len - first;
    const uint32_t n_el = left < kUnpackChunk ? (uint32_t)left : kUnpackChunk;
    const elem_t *src = reinterpret_cast<const elem_t *>(a.shard[pc.shard]) + pc.src_off + first;
    elem_t *dst = reinterpret_cast<elem_t *>(a.tensor[pc.tensor - a.tensor0]) + pc.dst_off + first;

    uint32_t head = (uint32_t)((16u - (uint32_t)(reinterpret_cast<uintptr_t>(dst) & 15u)) & 15u) / ES;
    if (head > n_el) head = n_el;
    const uint32_t nbody = (n_el - head) / VE;
    const uint32_t tail0 = head + nbody * VE;
    if (lane < head) dst[lane] = src[lane];
    if (lane < n_el - tail0) dst[tail0 + lane] = src[tail0 + lane];

    const elem_t *bsrc = src + head;
    u32x4 *bdst = reinterpret_cast<u32x4 *>(dst + head);
    constexpr int U = 4;
    for (uint32_t q0 = 0; q0 < nbody; q0 += kWave * U) {
        u32x4 val[U];
#pragma unroll
        for (int i = 0; i < U; ++i) {
            const uint32_t q = q0 + i * kWave + lane;
            if (q < nbody) val[i] = __builtin_nontemporal_load(reinterpret_cast<const vec_unaligned_t *>(bsrc + (size_t)q * VE));
        }
#pragma unroll
        for (int i = 0; i < U; ++i) {
            const uint32_t q = q0 + i * kWave + lane;
            if (q < nbody) st_writethrough(bdst + q, val[i]);
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
    a.nquad = (uint32_t)(n / 4);
    a.scale = scale;
    a.accumulate = accumulate;
    const dim3 grid((a.nquad + kGroupQuads - 1) / kGroupQuads), block(kWave);
    // Unused LDS per workgroup caps the resident wavefronts, as in the fused update.  For the
    // reduction it pays only with many bf16 streams (measured on MI355X: R = 8, 8 wavefronts per CU:
    // 6.23 -> 6.37 TB/s; R = 16, 6 per CU: 6.03 -> 6.18; nothing at R = 4 or with fp32 inputs).
#define HZP_REDUCE_CASE(G, RT, LDS) hipLaunchKernelGGL((reduce_kernel<G, RT>), grid, block, LDS, stream, a)
    if (!g32) {
        switch (R) {
        case 4: HZP_REDUCE_CASE(false, 4, 0); break;
        case 8: HZP_REDUCE_CASE(false, 8, 20480); break;
        case 16: HZP_REDUCE_CASE(false, 16, 27136); break;
        default: HZP_REDUCE_CASE(false, 0, 0); break;
        }
    } else {
        switch (R) {
        case 4: HZP_REDUCE_CASE(true, 4, 0); break;
        case 8: HZP_REDUCE_CASE(true, 8, 0); break;
        default: HZP_REDUCE_CASE(true, 0, 0); break;
        }
    }
#undef HZP_REDUCE_CASE
    return check_launch("hzp_reduce_shard");
}

template <class Seg, class H, class Wd>
static void launch_fused_variant(bool g32, bool o32, uint32_t R, const Seg &a, const H &h,
                                 const Wd &w, dim3 grid, hipStream_t stream)
{
    const dim3 block(kWave);
    // The occupancy cap pays off only where every load is issued up front (compile-time R);
    // the run-time-R loop keeps two contributions in flight and needs the resident wavefronts.
    const unsigned lds = kFusedLdsBytes;
#define HZP_FUSED_CASE(RT, G, O) \
    hipLaunchKernelGGL((fused_adamw_kernel<RT, G, O, Seg, H, Wd>), grid, block, (RT) ? lds : 0u, stream, a, h, w)
    if (!g32 && !o32) {
        switch (R) {
        case 1: HZP_FUSED_CASE(1, false, false); break;
        case 2: HZP_FUSED_CASE(2, false, false); break;
        case 4: HZP_FUSED_CASE(4, false, false); break;
        case 8: HZP_FUSED_CASE(8, false, false); break;
        case 16: HZP_FUSED_CASE(16, false, false); break;
        default: HZP_FUSED_CASE(0, false, false); break;
        }
    } else if (g32 && o32) {
        switch (R) {
        case 4: HZP_FUSED_CASE(4, true, true); break;
        case 8: HZP_FUSED_CASE(8, true, true); break;
        case 16: HZP_FUSED_CASE(16, true, true); break;
        default: HZP_FUSED_CASE(0, true, true); break;
        }
    } else if (g32 && !o32) {
        if (R == 1) {
            HZP_FUSED_CASE(1, true, false);     // the pre-reduced form
        } else {
            HZP_FUSED_CASE(0, true, false);
        }
    } else {
        HZP_FUSED_CASE(0, false, true);
    }
#undef HZP_FUSED_CASE
}

// Most groups one launch of the fused update covers (about 150 M elements, 0.6-1.3 ms of work).
// Workgroups go to the 8 XCDs round-robin, so each XCD owns a fixed eighth of the groups of a
// launch; the XCDs do not run at exactly the same speed, and over a long launch they drift apart
// (measured on MI355X: by 5-10 % of the grid after 3 ms), which spreads the addresses in flight and
// leaves the slowest XCD to finish alone.  A launch boundary lines them up again for a few
// microseconds: at R = 16 on 72 M-element shards, launches of 140-280 k groups stream 2-6 % faster
// than one launch over everything, and shorter ones lose to the gaps between launches.
constexpr uint32_t kMaxGroupsPerLaunch = 300000;

// A run of one segment handled by one launch: elements [first, first + n) of segment `seg`.
struct SegRun {
    uint32_t seg;
    uint64_t first, n;
};

template <class Seg, class H>
static hzp_status_t launch_fused_table(const hzp_plan_t *plan, bool use_wd, bool g32, bool o32, uint32_t R,
                                       const FusedSegment *segs, size_t nseg, const H &h,
                                       hipStream_t stream)
{
    const DeviceTables *tab = nullptr;
    if (use_wd) {
        hzp_status_t st = device_tables(plan, &tab);
        if (st != HZP_OK) return st;
    }
    const uint32_t per_seg = R + 4;
    const size_t cap = std::min<size_t>(Seg::kMaxSeg, Seg::kPtrCap / per_seg);
    const uint32_t gsz = g32 ? 4u : 2u, osz = o32 ? 4u : 2u;
    constexpr uint64_t kGroupElems = 4ull * kGroupQuads;
    // Cut the segments into runs of at most kMaxGroupsPerLaunch groups (a shard longer than that is
    // covered by several launches), then fill launches with whole runs.
    std::vector<SegRun> runs;
    try {
        for (size_t s = 0; s < nseg; ++s)
            for (uint64_t first = 0; first < segs[s].n; first += kMaxGroupsPerLaunch * kGroupElems)
                runs.push_back(SegRun{(uint32_t)s, first, std::min<uint64_t>(segs[s].n - first, kMaxGroupsPerLaunch * kGroupElems)});
    } catch (const std::bad_alloc &) {
        return fail(HZP_ERR_NOMEM, "hzp_adamw_shard: out of host memory");
    }
    size_t r0 = 0;
    while (r0 < runs.size()) {
        Seg a{};
        WdLookup w{};
        uint32_t blocks = 0;
        uint32_t cnt = 0;
        for (; r0 + cnt < runs.size() && cnt < cap; ++cnt) {
            const SegRun &run = runs[r0 + cnt];
            const FusedSegment &f = segs[run.seg];
            const uint32_t nquad = (uint32_t)(run.n / 4);
            const uint32_t nb = (nquad + kGroupQuads - 1) / kGroupQuads;
            if (cnt > 0 && blocks + nb > kMaxGroupsPerLaunch) break;    // start another launch
            blocks += nb;
            a.blk_end[cnt] = blocks;
            a.nquad[cnt] = nquad;
            const void **sp = a.ptr + (size_t)cnt * per_seg;
            for (uint32_t r = 0; r < R; ++r) sp[r] = static_cast<const char *>(f.grads[r]) + run.first * gsz;
            sp[R] = f.master + run.first;
            sp[R + 1] = f.m + run.first;
            sp[R + 2] = f.v + run.first;
            sp[R + 3] = f.out ? static_cast<char *>(f.out) + run.first * osz : nullptr;
            if constexpr (std::is_same<Seg, SegTableNarrow>::value) {
                w.first_slot[cnt] = f.first_slot;
                w.n_tensors[cnt] = f.n_tensors;
                w.shard_begin[cnt] = f.shard_begin + run.first;
            }
        }
        a.nseg = cnt;
        a.R = R;
        // Two-dimensional grid unless the segments differ so much in length that more than an
        // eighth of its workgroups would be surplus.
        uint32_t max_groups = 0;
        for (uint32_t c = 0; c < cnt; ++c) {
            const uint32_t groups = a.blk_end[c] - (c ? a.blk_end[c - 1] : 0u);
            max_groups = std::max(max_groups, groups);
        }
        dim3 grid(blocks);
        const bool two_d = (uint64_t)max_groups * cnt - blocks <= blocks / 8 && cnt <= 65535;
        if (two_d) {
            for (uint32_t c = cnt; c-- > 0;) a.blk_end[c] -= c ? a.blk_end[c - 1] : 0u;
            a.grid2d = 1;
            grid = dim3(max_groups, cnt);
        }
        if (blocks > 0) {
            if constexpr (std::is_same<Seg, SegTableNarrow>::value) {
                w.tensor_off = tab->tensor_off;
                w.tensor_wd = tab->tensor_wd;
                launch_fused_variant(g32, o32, R, a, h, w, grid, stream);
            } else {
                launch_fused_variant(g32, o32, R, a, h, NoLookup{}, grid, stream);
            }
            hzp_status_t st = check_launch("hzp_adamw_shard");
            if (st != HZP_OK) return st;
        }
        r0 += cnt;
    }
    return HZP_OK;
}

hzp_status_t launch_fused(const hzp_plan_t *plan, bool g32, bool o32, uint32_t R, const FusedSegment *segs,
                          size_t nseg, const AdamScalars &h, hipStream_t stream)
{
    if (plan->uniform_wd)
        return launch_fused_table<SegTableWide>(plan, false, g32, o32, R, segs, nseg, h, stream);
    return launch_fused_table<SegTableNarrow>(plan, true, g32, o32, R, segs, nseg, h, stream);
}

hzp_status_t launch_fused_dev(const hzp_plan_t *plan, bool g32, bool o32, uint32_t R, const FusedSegment *segs,
                              size_t nseg, const AdamScalars *scalars_dev, hipStream_t stream)
{
    const ScalarsInMemory h{scalars_dev};
    if (plan->uniform_wd)
        return launch_fused_table<SegTableWide>(plan, false, g32, o32, R, segs, nseg, h, stream);
    return launch_fused_table<SegTableNarrow>(plan, true, g32, o32, R, segs, nseg, h, stream);
}

hzp_status_t launch_concat(const void *const *srcs, uint32_t n_shards, uint64_t bytes_per_shard, void *dst,
                           hipStream_t stream)
{
    if (bytes_per_shard == 0) return HZP_OK;
    const uint64_t nvec = bytes_per_shard / 16;
    // (a grid holds fewer than 2^32 threads per dimension: one thread per vector, rounded up to whole wavefronts)
    if (nvec > 0xFFFFFFFFull - kWave) return fail(HZP_ERR_UNSUPPORTED, "hzp_gather_layer: shard of 64 GiB or more");
    ConcatArgs a{};
    uint32_t listed = 0;
    for (uint32_t s = 0; s < n_shards; ++s) {
        if (srcs[s] == static_cast<const char *>(dst) + (size_t)s * bytes_per_shard) continue;     // in place
        a.src[listed] = srcs[s];
        a.slot[listed++] = (uint8_t)s;
    }
    if (listed == 0) return HZP_OK;
    a.dst = reinterpret_cast<u32x4 *>(dst);
    a.vec_per_shard = (uint32_t)nvec;
    const dim3 grid((uint32_t)((nvec + kWave - 1) / kWave), listed), block(kWave);
    hipLaunchKernelGGL(concat_kernel, grid, block, 0, stream, a);
    return check_launch("hzp_gather_layer");
}

hzp_status_t launch_concat_layers(const void *const *srcs, uint32_t per_layer, const uint64_t *bytes_per_piece,
                                  void *const *dsts, uint32_t n_layers, hipStream_t stream)
{
    // the pieces that have to move, layer after layer
    struct Item {
        const void *src;
        char *dst;
        uint64_t nvec;
    };
    std::vector<Item> items;
    try {
        items.reserve((size_t)n_layers * per_layer);
    } catch (const std::bad_alloc &) {
        return fail(HZP_ERR_NOMEM, "hzp_gather_layers: out of host memory");
    }
    for (uint32_t l = 0; l < n_layers; ++l) {
        const uint64_t bytes = bytes_per_piece[l];
        if (bytes / 16 > 0xFFFFFFFFull - kWave) return fail(HZP_ERR_UNSUPPORTED, "hzp_gather_layers: shard of 64 GiB or more");
        if (bytes == 0) continue;
        for (uint32_t k = 0; k < per_layer; ++k) {
            const void *src = srcs[(size_t)l * per_layer + k];
            char *dst = static_cast<char *>(dsts[l]) + (size_t)k * bytes;
            if (src != dst) items.push_back({src, dst, bytes / 16});      // else the piece lies in place
        }
    }
    // launches of equal numbers of pieces
    const size_t launches = (items.size() + kLayersPieceCap - 1) / kLayersPieceCap;
    for (size_t i = 0, done = 0; i < launches; ++i) {
        const size_t cnt = (items.size() - done + (launches - i) - 1) / (launches - i);
        ConcatLayersArgs a{};
        uint64_t longest = 0;
        for (size_t s = 0; s < cnt; ++s) {
            const Item &it = items[done + s];
            a.src[s] = it.src;
            a.dst[s] = reinterpret_cast<u32x4 *>(it.dst);
            a.nvec[s] = (uint32_t)it.nvec;
            longest = std::max(longest, it.nvec);
        }
        done += cnt;
        const dim3 grid((uint32_t)((longest + kWave - 1) / kWave), (uint32_t)cnt), block(kWave);
        hipLaunchKernelGGL(concat_layers_kernel, grid, block, 0, stream, a);
        hzp_status_t st = check_launch("hzp_gather_layers");
        if (st != HZP_OK) return st;
    }
    return HZP_OK;
}

hzp_status_t launch_concat_ranges(const void *const *srcs, const uint64_t *dst_off, const uint64_t *bytes,
                                  uint32_t n, void *dst, hipStream_t stream)
{
    ConcatRangesArgs a{};
    uint64_t tiles = 0, total = 0;
    bool uniform = true;
    for (uint32_t s = 0; s < n; ++s) {
        if (bytes[s] / 16 > 0xFFFFFFFFull - kWave || dst_off[s] / 16 > 0xFFFFFFFFull)
            return fail(HZP_ERR_UNSUPPORTED, "hzp_gather_shard: shard larger than 64 GiB");
        a.src[s] = srcs[s];
        a.dst_vec[s] = (uint32_t)(dst_off[s] / 16);
        a.nvec[s] = (uint32_t)(bytes[s] / 16);
        tiles += (bytes[s] / 16 + kWave - 1) / kWave;
        a.tile_end[s] = (uint32_t)tiles;           // checked below
        uniform = uniform && bytes[s] == bytes[0] && dst_off[s] == s * bytes[0];
        total += bytes[s];
    }
    if (total == 0) return HZP_OK;
    if (uniform) return launch_concat(srcs, n, bytes[0], dst, stream);     // equal whole pieces
    if (tiles > 0x7FFFFFFFull) return fail(HZP_ERR_UNSUPPORTED, "hzp_gather_shard: shard too large for one launch");
    a.dst = reinterpret_cast<u32x4 *>(dst);
    a.n = n;
    const dim3 grid((uint32_t)tiles), block(kWave);
    hipLaunchKernelGGL(concat_ranges_kernel, grid, block, 0, stream, a);
    return check_launch("hzp_gather_shard");
}

// Launches of the unpack kernel for tensors [t_begin, t_end) of a bucket; `pieces` and `piece_chunk`
// are device tables that hold the bucket's pieces from entry 0.
static hzp_status_t launch_unpack_with(const Piece *pieces, const uint32_t *piece_chunk, const BucketRec &b,
                                       const void *const *shards, uint32_t n_shards, void *const *tensors,
                                       uint32_t t_begin, uint32_t t_end, hipStream_t stream, const char *who)
{
    // Tensors travel in the argument block, kUnpackTensorCap at a time; pieces are sorted by tensor.
    size_t p0 = 0;
    while (p0 < b.pieces.size() && b.pieces[p0].tensor < t_begin) ++p0;
    for (uint32_t t0 = t_begin; t0 < t_end; t0 += kUnpackTensorCap) {
        const uint32_t t1 = std::min<uint32_t>(t_end, t0 + kUnpackTensorCap);
        size_t p1 = p0;
        while (p1 < b.pieces.size() && b.pieces[p1].tensor < t1) ++p1;
        UnpackArgs a{};
        for (uint32_t s = 0; s < n_shards; ++s) a.shard[s] = shards[s];
        for (uint32_t t = t0; t < t1; ++t) a.tensor[t - t0] = tensors[t - t_begin];
        a.pieces = pieces;
        a.piece_chunk = piece_chunk;
        a.n_pieces = (uint32_t)b.pieces.size();
        a.chunk0 = b.pieces[p0].chunk_begin;
        a.chunk_end = p1 < b.pieces.size() ? b.pieces[p1].chunk_begin : b.n_chunks;
        a.tensor0 = t0;
        const uint32_t chunks = a.chunk_end - a.chunk0;
        const dim3 grid(chunks), block(kWave);
        if (b.cls == HZP_CLASS_F32)
            hipLaunchKernelGGL(unpack_kernel<4>, grid, block, 0, stream, a);
        else
            hipLaunchKernelGGL(unpack_kernel<2>, grid, block, 0, stream, a);
        hzp_status_t st = check_launch(who);
        if (st != HZP_OK) return st;
        p0 = p1;
    }
    return HZP_OK;
}

hzp_status_t launch_unpack(const hzp_plan_t *plan, const BucketRec &b, const void *const *shards,
                           uint32_t n_shards, void *const *tensors, uint32_t t_begin, uint32_t t_end,
                           hipStream_t stream)
{
    const DeviceTables *tab = nullptr;
    hzp_status_t st = device_tables(plan, &tab);
    if (st != HZP_OK) return st;
    return launch_unpack_with(tab->pieces + b.piece_slot, tab->piece_chunk + b.piece_slot, b, shards, n_shards,
                              tensors, t_begin, t_end, stream, "hzp_gather_layer");
}

// ---------------------------------------------------------------------------------------
// The same unpack for callers that must not allocate: the bucket's piece table is written, by a
// small kernel that carries it in its arguments, into a fixed array in device memory instead of
// the per-plan tables that device_tables() allocates on first use.
// ---------------------------------------------------------------------------------------
struct StaticTables {
    Piece pieces[HZP_STATIC_MAX_PIECES];
    uint32_t piece_chunk[HZP_STATIC_MAX_PIECES];
};
// One copy per GPU, at an address of its own, held until the process ends.  In host code this
// name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[sizeof(StaticTables)];

constexpr uint32_t kFillWords = 896;    // 3584 bytes of table per launch, in the argument block
struct FillArgs {
    uint32_t word[kFillWords];
    uint32_t *dst;
    uint32_t n;
};
__global__ __launch_bounds__(256) void table_fill_kernel(const FillArgs a)
{
    for (uint32_t i = threadIdx.x; i < a.n; i += 256) a.dst[i] = a.word[i];
}

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up once per device).
static hzp_status_t scratch_address(StaticTables **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(HZP_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(HZP_ERR_UNSUPPORTED, "device %d: more than %d devices", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(HZP_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = ptr;
    }
    *out = static_cast<StaticTables *>(g_scratch_ptr[dev]);
    return HZP_OK;
}

// Enqueue the copy of `bytes` (a multiple of 4) of host data to device memory at `dst`.
static hzp_status_t fill_table(void *dst, const void *src, size_t bytes, hipStream_t stream)
{
    const uint32_t *w = static_cast<const uint32_t *>(src);
    size_t left = bytes / 4;
    uint32_t *d = static_cast<uint32_t *>(dst);
    while (left) {
        FillArgs a;
        a.n = (uint32_t)std::min<size_t>(left, kFillWords);
        std::memcpy(a.word, w, (size_t)a.n * 4);
        a.dst = d;
        hipLaunchKernelGGL(table_fill_kernel, dim3(1), dim3(256), 0, stream, a);
        hzp_status_t st = check_launch("hzp_gather_layer_static");
        if (st != HZP_OK) return st;
        w += a.n;
        d += a.n;
        left -= a.n;
    }
    return HZP_OK;
}

hzp_status_t launch_unpack_static(const BucketRec &b, const void *const *shards, uint32_t n_shards,
                                  void *const *tensors, hipStream_t stream)
{
    if (b.pieces.size() > HZP_STATIC_MAX_PIECES)        // refused by the entry point; the table below has this many rows
        return fail(HZP_ERR_UNSUPPORTED, "hzp_gather_layer_static: more tensor pieces than the fixed table holds");
    StaticTables *tab = nullptr;
    hzp_status_t st = scratch_address(&tab);
    if (st != HZP_OK) return st;
    uint32_t chunk_begin[HZP_STATIC_MAX_PIECES];
    for (size_t i = 0; i < b.pieces.size(); ++i) chunk_begin[i] = b.pieces[i].chunk_begin;
    static_assert(sizeof(Piece) % 4 == 0, "tables are copied in 32-bit words");
    st = fill_table(tab->pieces, b.pieces.data(), b.pieces.size() * sizeof(Piece), stream);
    if (st == HZP_OK) st = fill_table(tab->piece_chunk, chunk_begin, b.pieces.size() * sizeof(uint32_t), stream);
    if (st != HZP_OK) return st;
    return launch_unpack_with(tab->pieces, tab->piece_chunk, b, shards, n_shards, tensors, 0, b.n_tensors, stream,
                              "hzp_gather_layer_static");
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
    std::vector<uint32_t> chunk_begin(all.size());
    for (size_t i = 0; i < all.size(); ++i) chunk_begin[i] = all[i].chunk_begin;
    if (e == hipSuccess) e = upload((void **)&t.piece_chunk, chunk_begin.data(), chunk_begin.size() * sizeof(uint32_t));
    if (e != hipSuccess) {
        (void)hipFree(t.piece_chunk);
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

}  // namespace hzp

extern "C" hzp_status_t hzp_plan_prepare(const hzp_plan_t *plan, hipStream_t stream)
{
    if (!plan) return hzp::fail(HZP_ERR_INVALID_ARG, "hzp_plan_prepare: NULL plan");
    const hzp::DeviceTables *tab = nullptr;
    hzp_status_t st = hzp::device_tables(plan, &tab);       // allocates and copies (blocking) on first use
    if (st != HZP_OK) return st;
    // The copies above were blocking host-to-device copies on the null stream; a stream created
    // as non-blocking is not ordered behind them by itself, so wait for them once here.
    hipError_t e = hipStreamSynchronize(stream);
    if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
    if (e != hipSuccess) return hzp::fail(HZP_ERR_HIP, "hzp_plan_prepare: %s", hipGetErrorString(e));
    return HZP_OK;
}

namespace hzp {

void free_device_tables(hzp_plan_t *plan)
{
    for (DeviceTables &t : plan->dev) {
        int cur = -1;
        if (hipGetDevice(&cur) == hipSuccess && cur != t.device) (void)hipSetDevice(t.device);
        (void)hipFree(t.tensor_off);
        (void)hipFree(t.tensor_wd);
        (void)hipFree(t.pieces);
        (void)hipFree(t.piece_chunk);
        if (cur >= 0 && cur != t.device) (void)hipSetDevice(cur);
    }
    plan->dev.clear();
}

}  // namespace hzp
