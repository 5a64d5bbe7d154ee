// Host-side sanitizer run of the C ABI's argument and life-cycle paths: this program and api.hip's host code are
// compiled with AddressSanitizer and UndefinedBehaviorSanitizer (the GPU code is not instrumented), and every call
// below is checked against the status the header promises.  Exit status 0 = all as promised and no report.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
#include <hip/hip_runtime.h>
#include "gelo.h"

static int failures = 0;
#define EXPECT(call, want) do { gelo_status got_ = (call); if (got_ != (want)) { \
    std::printf("line %d: %s -> %s, expected %s\n", __LINE__, #call, gelo_status_string(got_), gelo_status_string(want)); ++failures; } } while (0)
#define HIP_OK(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { std::printf("line %d: %s\n", __LINE__, hipGetErrorString(e_)); return 2; } } while (0)

int main() {
    gelo_ctx* ctx = nullptr;
    EXPECT(gelo_create(nullptr, 0, 1, 0), GELO_EINVAL);
    EXPECT(gelo_create(&ctx, 99, 1, 0), GELO_EINVAL);
    EXPECT(gelo_create(&ctx, 0, 0xC0FFEEull, 0), GELO_OK);
    if (!ctx) { std::printf("no context\n"); return 2; }
    EXPECT(gelo_destroy(nullptr), GELO_EINVAL);
    if (std::strlen(gelo_last_error(ctx)) != 0) { std::printf("fresh context has an error text\n"); ++failures; }

    const int nd = 20, k = 2, d = 64, p = 32, n = nd + k;
    gelo_mixing* m = nullptr;
    gelo_mixing* none = nullptr;                                  // a failing draw resets its out argument
    // argument checks: nothing is enqueued, the context stays usable
    EXPECT(gelo_sample_mixing(ctx, GELO_ORTHOGONAL, 0, k, d, GELO_F32, 0.0, 1, 1, &m, nullptr), GELO_EINVAL);
    EXPECT(gelo_sample_mixing(ctx, GELO_ORTHOGONAL, nd, -1, d, GELO_F32, 0.0, 1, 1, &m, nullptr), GELO_EINVAL);
    EXPECT(gelo_sample_mixing(ctx, GELO_ORTHOGONAL, nd, k, 60, GELO_F32, 0.0, 1, 1, &m, nullptr), GELO_EALIGN);
    EXPECT(gelo_sample_mixing(ctx, GELO_ORTHOGONAL, nd, k, d, GELO_F32, 0.0, 1, 1, nullptr, nullptr), GELO_EINVAL);
    EXPECT(gelo_sample_mixing(ctx, GELO_ORTHOGONAL, GELO_MAX_N, 1, d, GELO_F32, 0.0, 1, 1, &m, nullptr), GELO_ESHAPE);
    EXPECT(gelo_sample_mixing(ctx, GELO_GAUSSIAN, nd, k, d, GELO_F32, 1e3, 0, 1, &m, nullptr), GELO_EINVAL);
    EXPECT(gelo_reserve(ctx, GELO_ORTHOGONAL, GELO_F32, nd, k, d, p, 1, 3), GELO_OK);
    EXPECT(gelo_reserve(ctx, GELO_ORTHOGONAL, GELO_F32, nd, k, d, -1, 1, 3), GELO_EINVAL);

    float *H = nullptr, *W = nullptr, *U = nullptr, *Y = nullptr, *Z = nullptr;
    HIP_OK(hipMalloc(&H, sizeof(float) * nd * d)); HIP_OK(hipMalloc(&W, sizeof(float) * d * p));
    HIP_OK(hipMalloc(&U, sizeof(float) * n * d)); HIP_OK(hipMalloc(&Y, sizeof(float) * n * p)); HIP_OK(hipMalloc(&Z, sizeof(float) * nd * p));
    std::vector<float> h((size_t)nd * d), w((size_t)d * p);
    for (size_t i = 0; i < h.size(); ++i) h[i] = (float)((int)(i * 37 % 101) - 50) / 50.f;
    for (size_t i = 0; i < w.size(); ++i) w[i] = (float)((int)(i * 53 % 97) - 48) / 2400.f;
    HIP_OK(hipMemcpy(H, h.data(), sizeof(float) * h.size(), hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(W, w.data(), sizeof(float) * w.size(), hipMemcpyHostToDevice));

    // one whole batch through the four calls, then every misuse of the object
    EXPECT(gelo_sample_mixing(ctx, GELO_ORTHOGONAL, nd, k, d, GELO_F32, 0.0, 1, 7, &m, nullptr), GELO_OK);
    EXPECT(gelo_sample_mixing(ctx, GELO_ORTHOGONAL, nd, k, d, GELO_F32, 0.0, 1, 7, &none, nullptr), GELO_EREUSE);   // batch id twice
    if (none != nullptr) { std::printf("a failing draw left its out argument set\n"); ++failures; }
    int i_nd = 0, i_k = 0, i_d = 0; gelo_dtype i_t = GELO_BF16; gelo_kind i_kind = GELO_GAUSSIAN;
    EXPECT(gelo_mixing_info(ctx, m, &i_nd, &i_k, &i_d, &i_t, &i_kind), GELO_OK);
    if (i_nd != nd || i_k != k || i_d != d || i_t != GELO_F32 || i_kind != GELO_ORTHOGONAL) { std::printf("gelo_mixing_info reports another object\n"); ++failures; }
    EXPECT(gelo_unmix(ctx, m, GELO_F32, p, Y, p, Z, p, nullptr), GELO_ESTATE);                                       // before mix
    EXPECT(gelo_mix(ctx, m, GELO_BF16, H, d, 10.f, GELO_NORM_MEDIAN, U, d, nullptr), GELO_EDTYPE);
    EXPECT(gelo_mix(ctx, m, GELO_F32, nullptr, d, 10.f, GELO_NORM_MEDIAN, U, d, nullptr), GELO_EINVAL);
    EXPECT(gelo_mix(ctx, m, GELO_F32, H, d - 8, 10.f, GELO_NORM_MEDIAN, U, d, nullptr), GELO_EINVAL);                 // ld < width
    EXPECT(gelo_mix(ctx, m, GELO_F32, H, d, 10.f, GELO_NORM_MEDIAN, U, d, nullptr), GELO_OK);
    EXPECT(gelo_mix(ctx, m, GELO_F32, H, d, 10.f, GELO_NORM_MEDIAN, U, d, nullptr), GELO_EREUSE);                     // mixes once
    EXPECT(gelo_project(ctx, GELO_F32, n, d, p, U, d, W, p, Y, p, nullptr), GELO_OK);
    EXPECT(gelo_project(ctx, GELO_F32, n, d, p, U, d, W, p - 8, Y, p, nullptr), GELO_EINVAL);
    EXPECT(gelo_unmix(ctx, m, GELO_BF16, p, Y, p, Z, p, nullptr), GELO_EDTYPE);
    EXPECT(gelo_unmix(ctx, m, GELO_F32, p, Y, p, Z, p, nullptr), GELO_OK);
    EXPECT(gelo_unmix(ctx, m, GELO_F32, p, Y, p, Z, p, nullptr), GELO_EREUSE);
    EXPECT(gelo_mixing_free(ctx, m), GELO_OK);
    EXPECT(gelo_mixing_free(ctx, m), GELO_EINVAL);                                                                   // already freed
    EXPECT(gelo_mixing_free(ctx, nullptr), GELO_EINVAL);
    HIP_OK(hipDeviceSynchronize());
    // Z = H W within the float contract
    std::vector<float> z((size_t)nd * p);
    HIP_OK(hipMemcpy(z.data(), Z, sizeof(float) * z.size(), hipMemcpyDeviceToHost));
    double err = 0.0, ref = 0.0;
    for (int i = 0; i < nd; ++i)
        for (int j = 0; j < p; ++j) {
            double s = 0.0;
            for (int t = 0; t < d; ++t) s += (double)h[(size_t)i * d + t] * (double)w[(size_t)t * p + j];
            const double e = s - (double)z[(size_t)i * p + j];
            err += e * e; ref += s * s;
        }
    if (!(err <= 1e-8 * ref)) { std::printf("Z differs from H W: relative error %g\n", std::sqrt(err / ref)); ++failures; }

    // batched draw, the id window and the floor
    gelo_mixing* many[GELO_MAX_BATCH_DRAW + 1];
    EXPECT(gelo_sample_mixing_batch(ctx, GELO_ORTHOGONAL, nd, k, d, GELO_F32, 100, 0, many, nullptr), GELO_EINVAL);
    EXPECT(gelo_sample_mixing_batch(ctx, GELO_ORTHOGONAL, nd, k, d, GELO_F32, 100, GELO_MAX_BATCH_DRAW + 1, many, nullptr), GELO_EINVAL);
    EXPECT(gelo_sample_mixing_batch(ctx, GELO_GAUSSIAN, nd, k, d, GELO_F32, 100, 2, many, nullptr), GELO_EINVAL);
    EXPECT(gelo_sample_mixing_batch(ctx, GELO_ORTHOGONAL, nd, k, d, GELO_F32, 100, 3, many, nullptr), GELO_OK);
    EXPECT(gelo_sample_mixing_batch(ctx, GELO_ORTHOGONAL, nd, k, d, GELO_F32, 102, 2, many + 3, nullptr), GELO_EREUSE);
    for (int i = 0; i < 3; ++i) EXPECT(gelo_mixing_free(ctx, many[i]), GELO_OK);
    uint64_t floor_id = 0;
    EXPECT(gelo_get_batch_floor(ctx, &floor_id), GELO_OK);
    if (floor_id != 103) { std::printf("first unused id %llu, expected 103\n", (unsigned long long)floor_id); ++failures; }
    EXPECT(gelo_set_batch_floor(ctx, 5000), GELO_OK);
    EXPECT(gelo_set_batch_floor(ctx, 10), GELO_EINVAL);
    EXPECT(gelo_sample_mixing(ctx, GELO_ORTHOGONAL, nd, k, d, GELO_F32, 0.0, 1, 4999, &none, nullptr), GELO_EREUSE);
    EXPECT(gelo_sample_mixing(ctx, GELO_ORTHOGONAL, nd, k, d, GELO_F32, 0.0, 1, 5000 + 2 * (uint64_t)GELO_BATCH_WINDOW, &m, nullptr), GELO_OK);
    EXPECT(gelo_mixing_free(ctx, m), GELO_OK);
    EXPECT(gelo_sample_mixing(ctx, GELO_ORTHOGONAL, nd, k, d, GELO_F32, 0.0, 1, 5001, &none, nullptr), GELO_EREUSE);   // fell out of the window

    // the block-diagonal kind through the same life cycle, with more rows than one block holds (its host code: the block
    // layout, one workspace per block, per-block launches, the dense export)
    {
        const int bnd = 280, bk = 14, bn = bnd + bk;
        float *BH = nullptr, *BU = nullptr, *BY = nullptr, *BZ = nullptr, *BA = nullptr;
        HIP_OK(hipMalloc(&BH, sizeof(float) * bnd * d)); HIP_OK(hipMalloc(&BU, sizeof(float) * bn * d));
        HIP_OK(hipMalloc(&BY, sizeof(float) * bn * p)); HIP_OK(hipMalloc(&BZ, sizeof(float) * bnd * p));
        HIP_OK(hipMalloc(&BA, sizeof(float) * bn * bn));
        HIP_OK(hipMemset(BH, 0, sizeof(float) * bnd * d));
        const uint64_t bid = 5000 + 3 * (uint64_t)GELO_BATCH_WINDOW;
        EXPECT(gelo_sample_mixing(ctx, GELO_BLOCK_ORTHOGONAL, bnd, bk, d, GELO_F32, 0.0, 1, bid, &m, nullptr), GELO_OK);
        EXPECT(gelo_mix(ctx, m, GELO_F32, BH, d, 10.f, GELO_NORM_MEDIAN, BU, d, nullptr), GELO_OK);
        EXPECT(gelo_project(ctx, GELO_F32, bn, d, p, BU, d, W, p, BY, p, nullptr), GELO_OK);
        EXPECT(gelo_unmix(ctx, m, GELO_F32, p, BY, p, BZ, p, nullptr), GELO_OK);
        EXPECT(gelo_mixing_export(ctx, m, BA, nullptr, nullptr, nullptr, nullptr, nullptr), GELO_OK);
        EXPECT(gelo_mixing_free(ctx, m), GELO_OK);
        EXPECT(gelo_sample_mixing_batch(ctx, GELO_BLOCK_ORTHOGONAL, bnd, bk, d, GELO_F32, bid + 1, 3, many, nullptr), GELO_OK);
        for (int i = 0; i < 3; ++i) EXPECT(gelo_mixing_free(ctx, many[i]), GELO_OK);
        // the product of directly drawn reflectors: the host path of the QR kind with the factorisation left out
        EXPECT(gelo_sample_mixing(ctx, GELO_REFLECTOR_PRODUCT, bnd, bk, d, GELO_F32, 0.0, 1, bid + 8, &m, nullptr), GELO_OK);
        EXPECT(gelo_mix(ctx, m, GELO_F32, BH, d, 10.f, GELO_NORM_MEDIAN, BU, d, nullptr), GELO_OK);
        EXPECT(gelo_project(ctx, GELO_F32, bn, d, p, BU, d, W, p, BY, p, nullptr), GELO_OK);
        EXPECT(gelo_unmix(ctx, m, GELO_F32, p, BY, p, BZ, p, nullptr), GELO_OK);
        EXPECT(gelo_mixing_export(ctx, m, BA, nullptr, nullptr, nullptr, nullptr, nullptr), GELO_OK);
        EXPECT(gelo_mixing_free(ctx, m), GELO_OK);
        EXPECT(gelo_sample_mixing_batch(ctx, GELO_REFLECTOR_PRODUCT, bnd, bk, d, GELO_F32, bid + 9, 3, many, nullptr), GELO_OK);
        for (int i = 0; i < 3; ++i) EXPECT(gelo_mixing_free(ctx, many[i]), GELO_OK);
        HIP_OK(hipDeviceSynchronize());
        HIP_OK(hipFree(BH)); HIP_OK(hipFree(BU)); HIP_OK(hipFree(BY)); HIP_OK(hipFree(BZ)); HIP_OK(hipFree(BA));
    }

    size_t bytes = 0;
    EXPECT(gelo_fp8_weight_bytes(128, 64, &bytes), GELO_OK);
    EXPECT(gelo_fp8_weight_bytes(128, 64, nullptr), GELO_EINVAL);

    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipFree(H)); HIP_OK(hipFree(W)); HIP_OK(hipFree(U)); HIP_OK(hipFree(Y)); HIP_OK(hipFree(Z));
    EXPECT(gelo_destroy(ctx), GELO_OK);
    std::printf(failures ? "%d expectation(s) failed\n" : "lifecycle: all statuses as promised\n", failures);
    return failures ? 1 : 0;
}
