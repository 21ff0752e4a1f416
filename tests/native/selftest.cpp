// Stand-alone check of libhzp.so from C++: no Python and no PyTorch in the process, device memory
// from the HIP runtime, results compared with the plain C oracle (oracle/numeric.c).  Test
// infrastructure: built by tests/native/build.py, run by tests/test_gpu_native.py.
//
// Covers one pass of the path on a small plan: fused reduce + AdamW + cast on a rank's ZeRO-1
// shards of two layers in one call, the level-1 gather of both layers in one call, the level-3
// gather with unpack, and the stand-alone reduction.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "hzp.h"

extern "C" {
typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    uint32_t step;
} hzp_oracle_adamw_t;
uint16_t hzp_oracle_f32_to_bf16(float f);
float hzp_oracle_bf16_to_f32(uint16_t h);
void hzp_oracle_reduce(const void *const *slices, uint32_t R, int is_f32, uint64_t n, float scale, int accumulate,
                       float *out);
void hzp_oracle_adamw_f64(const hzp_oracle_adamw_t *h, uint64_t n, const float *g, const float *wd_mult, float *p,
                          float *m, float *v, uint16_t *p16, float *p32out);
void hzp_oracle_gather_concat(const void *const *srcs, uint32_t n_shards, uint64_t len, uint32_t elem_bytes, void *dst);
void hzp_oracle_unpack_tensor(const void *const *shards, uint64_t S3, uint32_t elem_bytes, uint64_t offset,
                              uint64_t numel, void *dst);
}

#define HIP(x)                                                                              \
    do {                                                                                    \
        hipError_t e_ = (x);                                                                \
        if (e_ != hipSuccess) {                                                             \
            printf("selftest: %s failed: %s\n", #x, hipGetErrorString(e_));                 \
            return 2;                                                                       \
        }                                                                                   \
    } while (0)
#define HZP(x)                                                                              \
    do {                                                                                    \
        if ((x) != HZP_OK) {                                                                \
            printf("selftest: %s failed: %s\n", #x, hzp_last_error());                      \
            return 2;                                                                       \
        }                                                                                   \
    } while (0)

static uint32_t g_state = 12345u;
static float uniform() { g_state = g_state * 1664525u + 1013904223u; return (float)(g_state >> 8) / 16777216.0f; }
static float gaussian_ish(float sigma) { return sigma * 2.0f * (uniform() + uniform() + uniform() - 1.5f); }

template <class T>
static T *to_device(const std::vector<T> &h)
{
    T *d = nullptr;
    if (hipMalloc((void **)&d, h.size() * sizeof(T)) != hipSuccess) return nullptr;
    if (hipMemcpy(d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) return nullptr;
    return d;
}
template <class T>
static bool to_host(std::vector<T> &h, const T *d)
{
    return hipMemcpy(h.data(), d, h.size() * sizeof(T), hipMemcpyDeviceToHost) == hipSuccess;
}

static int bad = 0;
static void check_f32(const char *what, const std::vector<float> &got, const std::vector<float> &want)
{
    double ss = 0;
    for (float w : want) ss += (double)w * w;
    const double rms = std::sqrt(ss / (want.empty() ? 1 : want.size()));
    for (size_t x = 0; x < want.size(); ++x) {
        const double a = got[x], b = want[x];
        const double scale = std::fmax(std::fmax(std::fabs(a), std::fabs(b)), rms);
        if (!(std::fabs(a - b) <= 2e-6 * scale)) {
            if (bad++ < 5) printf("selftest: %s[%zu] = %.9g, oracle %.9g\n", what, x, a, b);
        }
    }
}

int main()
{
    int ndev = 0;
    HIP(hipGetDeviceCount(&ndev));
    if (ndev < 1) {
        printf("selftest: no GPU\n");
        return 3;
    }
    HIP(hipSetDevice(0));
    hipStream_t stream;
    HIP(hipStreamCreateWithFlags(&stream, hipStreamNonBlocking));

    // two layers, three tensors, A = 8, Z3 = Z2 = 2, Z1 = 4 (K = 2); rank 3 -> j = 1, k = 1, i = 3
    const uint32_t per_layer[2] = {2, 1};
    const uint64_t numel[3] = {3001, 517, 7000};
    hzp_plan_desc_t desc = {2, per_layer, numel, nullptr, nullptr, 8, 2, 0, 4};
    hzp_plan_t *plan = nullptr;
    HZP(hzp_plan(&desc, &plan));
    const uint32_t rank = 3, R = 4, Z3 = 2, K = 2;
    uint32_t j, k, i;
    HZP(hzp_plan_rank(plan, rank, &j, &k, &i));
    hzp_bucket_info_t b[2];
    for (uint32_t l = 0; l < 2; ++l) HZP(hzp_plan_bucket(plan, l, HZP_CLASS_BF16, &b[l]));

    const hzp_adamw_t hyper = {1e-4f, 0.9f, 0.95f, 1e-8f, 0.1f, 1.0f / R, 3};
    const hzp_oracle_adamw_t ohyper = {1e-4f, 0.9f, 0.95f, 1e-8f, 0.1f, 3};

    std::vector<uint16_t> hg[2][4], hout[2], hshard3[2];
    std::vector<float> hp[2], hm[2], hv[2];
    std::vector<float> hp0[2], hm0[2], hv0[2];      // the inputs as they were (the oracle updates hp, hm, hv in place)
    const void *dgrad[8];
    float *dp[2], *dm[2], *dv[2];
    void *dout[2];
    for (uint32_t l = 0; l < 2; ++l) {
        const uint64_t n = b[l].s1;
        // payload mask of the rank's ZeRO-1 shard: padding elements are zero in every array
        uint64_t begin, len;
        HZP(hzp_plan_shard(plan, l, HZP_CLASS_BF16, 1, rank, &begin, &len));
        std::vector<char> payload(n, 0);
        for (uint32_t t = 0; t < 3; ++t) {
            hzp_tensor_info_t ti;
            HZP(hzp_plan_tensor(plan, t, &ti));
            if (ti.layer != l) continue;
            for (uint64_t x = 0; x < n; ++x)
                if (begin + x >= ti.offset && begin + x < ti.offset + ti.numel) payload[x] = 1;
        }
        hp[l].resize(n);
        hm[l].resize(n);
        hv[l].resize(n);
        for (uint64_t x = 0; x < n; ++x) {
            hp[l][x] = payload[x] ? gaussian_ish(0.02f) : 0.0f;
            hm[l][x] = payload[x] ? gaussian_ish(1e-3f) : 0.0f;
            hv[l][x] = payload[x] ? 1e-6f * uniform() : 0.0f;
        }
        for (uint32_t r = 0; r < R; ++r) {
            hg[l][r].resize(n);
            for (uint64_t x = 0; x < n; ++x) hg[l][r][x] = hzp_oracle_f32_to_bf16(payload[x] ? gaussian_ish(1e-3f) : 0.0f);
            dgrad[l * R + r] = to_device(hg[l][r]);
            if (!dgrad[l * R + r]) return 2;
        }
        hp0[l] = hp[l];
        hm0[l] = hm[l];
        hv0[l] = hv[l];
        dp[l] = to_device(hp[l]);
        dm[l] = to_device(hm[l]);
        dv[l] = to_device(hv[l]);
        hout[l].assign(n, 0);
        dout[l] = to_device(hout[l]);
        if (!dp[l] || !dm[l] || !dv[l] || !dout[l]) return 2;
    }

    // fused update of both layers in one call
    HZP(hzp_adamw_shard(plan, 0, 2, HZP_CLASS_BF16, rank, &hyper, dgrad, R, dp, dm, dv, dout, stream));
    HIP(hipStreamSynchronize(stream));
    for (uint32_t l = 0; l < 2; ++l) {
        const uint64_t n = b[l].s1;
        std::vector<float> g(n), gp(n), gm(n), gv(n);
        std::vector<uint16_t> want16(n), got16(n);
        const void *slices[4] = {hg[l][0].data(), hg[l][1].data(), hg[l][2].data(), hg[l][3].data()};
        hzp_oracle_reduce(slices, R, 0, n, 1.0f / R, 0, g.data());
        hzp_oracle_adamw_f64(&ohyper, n, g.data(), nullptr, hp[l].data(), hm[l].data(), hv[l].data(), want16.data(), nullptr);
        if (!to_host(gp, dp[l]) || !to_host(gm, dm[l]) || !to_host(gv, dv[l]) || !to_host(got16, (const uint16_t *)dout[l]))
            return 2;
        check_f32("master", gp, hp[l]);
        check_f32("momentum", gm, hm[l]);
        check_f32("variance", gv, hv[l]);
        double ss = 0;
        for (float w : hp[l]) ss += (double)w * w;
        const double floor_ = 2e-6 * std::sqrt(ss / n);
        for (uint64_t x = 0; x < n; ++x) {
            const int d = std::abs((int)(got16[x] & 0x7FFF) - (int)(want16[x] & 0x7FFF));
            const bool same_sign = ((got16[x] ^ want16[x]) & 0x8000) == 0 || ((got16[x] | want16[x]) & 0x7FFF) == 0;
            const double gotv = hzp_oracle_bf16_to_f32(got16[x]), wantv = hzp_oracle_bf16_to_f32(want16[x]);
            const double ulp = std::fabs(hzp_oracle_bf16_to_f32((uint16_t)(want16[x] + 1)) - wantv);
            if (!((same_sign && d <= 1) || std::fabs(gotv - wantv) <= ulp + floor_)) {
                if (bad++ < 5) printf("selftest: bf16 layer %u [%llu]: %04x, oracle %04x\n", l, (unsigned long long)x, got16[x], want16[x]);
            }
        }
        hout[l] = got16;
    }

    // level-1 gather of both layers in one call: piece k is this rank's output, the other is "received"
    std::vector<uint16_t> hpeer[2];
    const void *dpieces[4];
    void *dshard3[2];
    for (uint32_t l = 0; l < 2; ++l) {
        hpeer[l].resize(b[l].s1);
        for (auto &x : hpeer[l]) x = (uint16_t)(g_state = g_state * 1664525u + 1013904223u);
        void *dpeer = to_device(hpeer[l]);
        if (!dpeer) return 2;
        for (uint32_t kk = 0; kk < K; ++kk) dpieces[l * K + kk] = kk == k ? dout[l] : dpeer;
        HIP(hipMalloc(&dshard3[l], b[l].s3 * 2));
    }
    HZP(hzp_gather_layers(plan, 0, 2, HZP_CLASS_BF16, 1, dpieces, K, dshard3, stream));
    HIP(hipStreamSynchronize(stream));
    for (uint32_t l = 0; l < 2; ++l) {
        hshard3[l].resize(b[l].s3);
        if (!to_host(hshard3[l], (const uint16_t *)dshard3[l])) return 2;
        std::vector<uint16_t> want(b[l].s3);
        const void *pieces[2] = {k == 0 ? hout[l].data() : hpeer[l].data(), k == 1 ? hout[l].data() : hpeer[l].data()};
        hzp_oracle_gather_concat(pieces, K, b[l].s1, 2, want.data());
        if (memcmp(want.data(), hshard3[l].data(), want.size() * 2) != 0) {
            bad++;
            printf("selftest: level-1 gather of layer %u differs\n", l);
        }
    }

    // level-3 gather of layer 0 with unpack into its two tensors (the second one element-aligned only)
    {
        std::vector<uint16_t> hother(b[0].s3);
        for (auto &x : hother) x = (uint16_t)(g_state = g_state * 1664525u + 1013904223u);
        void *dother = to_device(hother);
        if (!dother) return 2;
        const void *dshards[2] = {j == 0 ? dshard3[0] : dother, j == 1 ? dshard3[0] : dother};
        const void *hshards[2] = {j == 0 ? (const void *)hshard3[0].data() : hother.data(),
                                  j == 1 ? (const void *)hshard3[0].data() : hother.data()};
        void *dbucket, *dt0, *dt1raw;
        HIP(hipMalloc(&dbucket, b[0].padded * 2));
        HIP(hipMalloc(&dt0, numel[0] * 2));
        HIP(hipMalloc(&dt1raw, numel[1] * 2 + 16));
        void *tensors[2] = {dt0, (char *)dt1raw + 6};
        HZP(hzp_gather_layer(plan, 0, HZP_CLASS_BF16, 3, dshards, Z3, dbucket, tensors, stream));
        HIP(hipStreamSynchronize(stream));
        std::vector<uint16_t> gotb(b[0].padded), wantb(b[0].padded);
        if (!to_host(gotb, (const uint16_t *)dbucket)) return 2;
        hzp_oracle_gather_concat(hshards, Z3, b[0].s3, 2, wantb.data());
        if (memcmp(gotb.data(), wantb.data(), gotb.size() * 2) != 0) {
            bad++;
            printf("selftest: level-3 gather differs\n");
        }
        for (uint32_t t = 0; t < 2; ++t) {
            hzp_tensor_info_t ti;
            HZP(hzp_plan_tensor(plan, t, &ti));
            std::vector<uint16_t> got(ti.numel), want(ti.numel);
            if (!to_host(got, (const uint16_t *)tensors[t])) return 2;
            hzp_oracle_unpack_tensor(hshards, b[0].s3, 2, ti.offset, ti.numel, want.data());
            if (memcmp(got.data(), want.data(), got.size() * 2) != 0) {
                bad++;
                printf("selftest: unpacked tensor %u differs\n", t);
            }
        }
    }

    // stand-alone reduction with accumulation, bit for bit
    {
        const uint64_t n = b[1].s1;
        std::vector<float> acc(n, 0.25f), got(n);
        float *dacc = to_device(acc);
        if (!dacc) return 2;
        HZP(hzp_reduce_shard(plan, 1, HZP_CLASS_BF16, 1, rank, dgrad + R, R, HZP_GRAD_DEFAULT, 0.5f, 1, dacc, stream));
        HIP(hipStreamSynchronize(stream));
        const void *slices[4] = {hg[1][0].data(), hg[1][1].data(), hg[1][2].data(), hg[1][3].data()};
        hzp_oracle_reduce(slices, R, 0, n, 0.5f, 1, acc.data());
        if (!to_host(got, dacc)) return 2;
        if (memcmp(got.data(), acc.data(), n * 4) != 0) {
            bad++;
            printf("selftest: accumulated reduction differs\n");
        }
    }

    // the arena layout, the tuner's choice of a variant, and the update on slices carved from the arena
    {
        uint64_t total[HZP_ARENA_VARIANTS], largest = 0;
        for (uint32_t v = 0; v < HZP_ARENA_VARIANTS; ++v) {
            HZP(hzp_plan_arena(plan, HZP_CLASS_BF16, R, HZP_GRAD_DEFAULT, v, &total[v]));
            if (total[v] > largest) largest = total[v];
        }
        char *raw = nullptr;
        HIP(hipMalloc((void **)&raw, largest + HZP_ARENA_ALIGN));
        char *arena = raw + (HZP_ARENA_ALIGN - (uintptr_t)raw % HZP_ARENA_ALIGN) % HZP_ARENA_ALIGN;
        uint32_t variant = 99;
        double seconds[HZP_ARENA_VARIANTS];
        HZP(hzp_arena_tune(plan, HZP_CLASS_BF16, rank, R, arena, largest, stream, &variant, seconds));
        if (variant >= HZP_ARENA_VARIANTS || !(seconds[variant] > 0.0)) {
            bad++;
            printf("selftest: the tuner chose variant %u\n", variant);
            variant = 0;
        }
        std::vector<unsigned char> zeros(largest, 1);
        HIP(hipMemcpy(zeros.data(), arena, largest, hipMemcpyDeviceToHost));
        for (uint64_t x = 0; x < largest; ++x)
            if (zeros[x]) {
                bad++;
                printf("selftest: the arena is not clear after tuning (byte %llu)\n", (unsigned long long)x);
                break;
            }
        // the same update as above, this time from the arena: inputs in, one call, outputs against the first run's
        const void *ag[8];
        float *ap[2], *am[2], *av[2];
        void *ao[2];
        for (uint32_t l = 0; l < 2; ++l) {
            uint64_t off, nb;
            for (uint32_t r = 0; r < R; ++r) {
                HZP(hzp_plan_arena_slice(plan, HZP_CLASS_BF16, R, HZP_GRAD_DEFAULT, variant, HZP_STREAM_GRAD, r, l, &off, &nb));
                HIP(hipMemcpy(arena + off, hg[l][r].data(), nb, hipMemcpyHostToDevice));
                ag[l * R + r] = arena + off;
            }
            HZP(hzp_plan_arena_slice(plan, HZP_CLASS_BF16, R, HZP_GRAD_DEFAULT, variant, HZP_STREAM_MASTER, 0, l, &off, &nb));
            HIP(hipMemcpy(arena + off, hp0[l].data(), nb, hipMemcpyHostToDevice));
            ap[l] = (float *)(arena + off);
            HZP(hzp_plan_arena_slice(plan, HZP_CLASS_BF16, R, HZP_GRAD_DEFAULT, variant, HZP_STREAM_M, 0, l, &off, &nb));
            HIP(hipMemcpy(arena + off, hm0[l].data(), nb, hipMemcpyHostToDevice));
            am[l] = (float *)(arena + off);
            HZP(hzp_plan_arena_slice(plan, HZP_CLASS_BF16, R, HZP_GRAD_DEFAULT, variant, HZP_STREAM_V, 0, l, &off, &nb));
            HIP(hipMemcpy(arena + off, hv0[l].data(), nb, hipMemcpyHostToDevice));
            av[l] = (float *)(arena + off);
            HZP(hzp_plan_arena_slice(plan, HZP_CLASS_BF16, R, HZP_GRAD_DEFAULT, variant, HZP_STREAM_PARAM_OUT, 0, l, &off, &nb));
            ao[l] = arena + off;
        }
        // ... through the form that reads the step's scalars from device memory
        hzp_adamw_scalars_t hscal;
        HZP(hzp_adamw_scalars(&hyper, &hscal));
        hzp_adamw_scalars_t *dscal = nullptr;
        HIP(hipMalloc((void **)&dscal, sizeof hscal));
        HIP(hipMemcpy(dscal, &hscal, sizeof hscal, hipMemcpyHostToDevice));
        HZP(hzp_adamw_shard_dev(plan, 0, 2, HZP_CLASS_BF16, rank, dscal, ag, R, ap, am, av, ao, stream));
        HIP(hipStreamSynchronize(stream));
        HIP(hipFree(dscal));
        for (uint32_t l = 0; l < 2; ++l) {
            std::vector<float> got(b[l].s1), first(b[l].s1), gotv(b[l].s1), firstv(b[l].s1);
            if (!to_host(got, ap[l]) || !to_host(first, dp[l]) || !to_host(gotv, av[l]) || !to_host(firstv, dv[l])) return 2;
            if (memcmp(got.data(), first.data(), got.size() * 4) != 0 || memcmp(gotv.data(), firstv.data(), got.size() * 4) != 0) {
                bad++;
                printf("selftest: the update on arena slices differs from the update on separate buffers (layer %u)\n", l);
            }
        }
        HIP(hipFree(raw));
    }

    hzp_plan_free(plan);
    if (bad) {
        printf("selftest: %d mismatches\n", bad);
        return 1;
    }
    printf("selftest ok: fused update of 2 layers (rank %u: j=%u k=%u i=%u), gathers, unpack, reduction, arena and tuner, scalars in device memory\n", rank, j, k, i);
    return 0;
}
