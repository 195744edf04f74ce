// Host-only driver for the AddressSanitizer / UBSan build of the library: walks the argument-validation and
// host-side paths of the C ABI (status strings, every entry point's error returns, the grouped-launch plan built
// into heap buffers of exactly the advertised size, workspace queries, the refresh policy).  No GPU is needed or
// used: every call below returns before its first HIP call.  Prints "sanitizer driver ok" and exits 0 when every
// return code is the expected one; a sanitizer report ends the process with a non-zero status.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "qgalore.h"

static int failures = 0;
#define EXPECT(call, want)                                                              \
    do {                                                                                \
        const long long got_ = (long long)(call);                                       \
        if (got_ != (long long)(want)) {                                                \
            std::printf("line %d: %s = %lld, expected %lld\n", __LINE__, #call, got_, (long long)(want)); \
            ++failures;                                                                 \
        }                                                                               \
    } while (0)

int main() {
    // non-null, 16-byte aligned, never dereferenced on the error paths
    uint8_t* const F8 = reinterpret_cast<uint8_t*>(0x10000);
    float* const FF = reinterpret_cast<float*>(0x10000);
    uint16_t* const F16 = reinterpret_cast<uint16_t*>(0x10000);
    int8_t* const FI8 = reinterpret_cast<int8_t*>(0x10000);
    int32_t* const FI32 = reinterpret_cast<int32_t*>(0x10000);
    float* const FF4 = reinterpret_cast<float*>(0x10004);
    const qg_hparams hp = {0.9f, 0.999f, 1e-8f, 1e-3f, 0.25f};

    for (int code = 0; code <= 7; ++code) EXPECT(std::strlen(qg_status_string(code)) > 0, 1);
    EXPECT(qg_last_hip_error() >= 0, 1);

    EXPECT(qg_quant_int8(nullptr, 4, 256, 256, FI8, FF, nullptr), QG_ERR_NULL);
    EXPECT(qg_quant_int8(FF, 0, 256, 256, FI8, FF, nullptr), QG_ERR_SHAPE);
    EXPECT(qg_quant_int8(FF, 4, 256, 128, FI8, FF, nullptr), QG_ERR_GROUP);
    EXPECT(qg_quant_int8(FF4, 4, 256, 256, FI8, FF, nullptr), QG_ERR_ALIGN);
    EXPECT(qg_quant_int4(FF, 4, 256, 256, nullptr, FF, nullptr), QG_ERR_NULL);
    EXPECT(qg_dequant_int8(FI8, nullptr, 4, 256, 256, FF, nullptr), QG_ERR_NULL);
    EXPECT(qg_dequant_int4(F8, FF, 4, 256, 256, FF4, nullptr), QG_ERR_ALIGN);
    EXPECT(qg_quant_int8_zp(FF, 4, 256, 256, FI8, FF, nullptr, nullptr), QG_ERR_NULL);
    EXPECT(qg_dequant_int8_zp(FI8, FF, nullptr, 4, 256, 256, FF, nullptr), QG_ERR_NULL);

    EXPECT(qg_project(nullptr, FF, F16, 512, 512, 128, 256, FF, nullptr, 0, nullptr), QG_ERR_NULL);
    EXPECT(qg_project(F8, FF, F16, 512, 512, 127, 256, FF, nullptr, 0, nullptr), QG_ERR_SHAPE);
    EXPECT(qg_project(F8, FF, F16, (int64_t)1 << 17, (int64_t)1 << 17, 128, 256, FF, nullptr, 0, nullptr), QG_ERR_SHAPE);
    EXPECT(qg_project(F8, FF, F16, INT64_MAX, INT64_MAX, 128, 256, FF, nullptr, 0, nullptr), QG_ERR_SHAPE);
    EXPECT(qg_workspace_bytes(512, 512, 128), 0);
    EXPECT(qg_lowrank_adam(FF, FF, FF, F16, 100, 0, &hp, nullptr), QG_ERR_SHAPE);
    EXPECT(qg_lowrank_adam(FF, FF, FF, F16, 100, 1, nullptr, nullptr), QG_ERR_NULL);
    EXPECT(qg_project_adam(F8, FF, F16, nullptr, FF, FF, F16, 512, 512, 128, 256, 0, &hp, nullptr), QG_ERR_SHAPE);
    EXPECT(qg_backproject_update_sr(F8, FF, F16, FI8, nullptr, 512, 512, 128, 256, 0.25f, 1e-3f, 0, 1, nullptr, nullptr), QG_ERR_NULL);
    EXPECT(qg_backproject_update_sr(F8, FF, F16, FI8, FF, 512, 512, 128, 256, 0.25f, 1e-3f, 0, 1, FF4, nullptr), QG_ERR_ALIGN);
    EXPECT(qg_backproject_update_sr_zp(F8, FF, F16, FI8, FF, nullptr, 512, 512, 128, 256, 0.25f, 1e-3f, 0, 1, nullptr), QG_ERR_NULL);
    EXPECT(qg_step(F8, FF, F16, FI8, FF, FF, FF, FF, F16, 512, 512, 128, 256, nullptr, 0, 1, nullptr, 0, nullptr), QG_ERR_NULL);
    EXPECT(qg_step(F8, FF, F16, FI8, FF, FF, FF, FF, F16, 512, 512, 128, 256, &hp, 0, 0, nullptr, 0, nullptr), QG_ERR_SHAPE);
    EXPECT(qg_step_zp(F8, FF, F16, FI8, FF, nullptr, FF, FF, nullptr, F16, 512, 512, 128, 256, &hp, 0, 1, nullptr), QG_ERR_NULL);
    EXPECT(qg_step8(F8, FF, F16, FI8, FF, F8, FF, F8, FF, FF, F16, 512, 512, 128, 64, &hp, 0, 1, nullptr), QG_ERR_GROUP);
    EXPECT(qg_sr_uniform(0, 1, 0, 0, FF, nullptr), QG_ERR_SHAPE);
    EXPECT(qg_diag_clock_probe(0, reinterpret_cast<int64_t*>(0x10000), nullptr), QG_ERR_SHAPE);
    EXPECT(qg_diag_mfma_loop(0, 0, FF, nullptr), QG_ERR_SHAPE);
    EXPECT(qg_diag_mfma_f64_loop(10, 0, FF, nullptr), QG_ERR_SHAPE);

    EXPECT(qg_cossim_workspace_bytes(512, 128), (8 * 3 * 128 + 2 * 2) * 4);
    EXPECT(qg_cossim_workspace_bytes(-5, 128), 0);
    EXPECT(qg_subspace_cossim(F8, FF, F8, FF, 512, 128, 256, FF, nullptr, 0, nullptr), QG_ERR_WORKSPACE);
    EXPECT(qg_subspace_cossim(F8, FF, F8, FF, 512, 130, 256, FF, FF, 1 << 20, nullptr), QG_ERR_SHAPE);
    EXPECT(qg_subspace_cossim_weighted(F8, FF, F8, FF, FF, 512, 128, 256, FF, nullptr, 0, nullptr), QG_ERR_WORKSPACE);
    EXPECT(qg_subspace_cossim_weighted(F8, FF, F8, FF, reinterpret_cast<float*>(0x10002), 512, 128, 256, FF, FF, 1 << 20, nullptr), QG_ERR_ALIGN);
    EXPECT(qg_step_ld(F8, FF, F16, FI8, FF, FF, FF, nullptr, F16, 2048, 5461, 5464, 512, 256, &hp, 0, 1, nullptr), QG_ERR_SHAPE);
    EXPECT(qg_step_ld(F8, FF, F16, FI8, FF, FF, FF, nullptr, F16, 2048, 5461, 5472, 512, 256, nullptr, 0, 1, nullptr), QG_ERR_NULL);
    EXPECT(qg_subspace_cossim_static(F8, FF, F8, nullptr, 512, 128, 256, FF, nullptr), QG_ERR_NULL);
    EXPECT(qg_subspace_cossim_static(F8, FF, F8, FF, 65536, 2048, 256, FF, nullptr), QG_ERR_WORKSPACE);
    EXPECT(qg_subspace_cossim_static(F8, FF, F8, FF, 512, 128, 256, FF4 + 0, nullptr) == QG_ERR_HIP ||
               qg_subspace_cossim_static(F8, FF, F8, FF, 512, 128, 128, FF, nullptr) == QG_ERR_GROUP, 1);

    EXPECT(qg_state8_quant(nullptr, 256, 1, F8, FF, nullptr), QG_ERR_NULL);
    EXPECT(qg_state8_quant(FF, 258, 1, F8, FF, nullptr), QG_ERR_SHAPE);
    EXPECT(qg_state8_dequant(F8, nullptr, 256, 0, FF, nullptr), QG_ERR_NULL);
    EXPECT(qg_lowrank_adam8(FF, F8, FF, F8, FF, F16, 256, 0, &hp, nullptr), QG_ERR_SHAPE);

    EXPECT(qg_int8_linear_forward(nullptr, FI8, FF, nullptr, 16, 512, 512, 256, F16, nullptr), QG_ERR_NULL);
    EXPECT(qg_int8_linear_forward(F16, FI8, FF, nullptr, (int64_t)1 << 20, (int64_t)1 << 12, 512, 256, F16, nullptr), QG_ERR_SHAPE);
    EXPECT(qg_int8_linear_backward(F16, F16, FI8, FF, 16, 512, 512, 256, nullptr, nullptr, nullptr), QG_ERR_NULL);
    EXPECT(qg_int8_linear_forward_ld(F16, FI8, FF, nullptr, 16, 512, 500, 504, 512, 256, F16, nullptr), QG_ERR_SHAPE);
    EXPECT(qg_int8_linear_forward_ld(F16, FI8, FF, nullptr, 16, 512, 500, 512, 512, 256, nullptr, nullptr), QG_ERR_NULL);
    EXPECT(qg_int8_linear_backward_ld(F16, F16, FI8, FF, 16, 500, 512, 512, 496, 256, F16, F16, nullptr), QG_ERR_SHAPE);
    EXPECT(qg_int8_linear_t_forward(F16, nullptr, FF, nullptr, 16, 512, 512, 256, F16, nullptr), QG_ERR_NULL);
    EXPECT(qg_int8_linear_t_backward(F16, F16, FI8, FF, 16, 512, 512, 256, nullptr, nullptr, nullptr), QG_ERR_NULL);
    EXPECT(qg_int8_linear_zp_forward(F16, FI8, FF, nullptr, nullptr, 16, 512, 512, 256, F16, nullptr), QG_ERR_NULL);
    EXPECT(qg_int8_linear_zp_backward(F16, F16, FI8, FF, nullptr, 16, 512, 512, 256, F16, F16, nullptr), QG_ERR_NULL);
    EXPECT(qg_int8_linear_t_zp_forward(F16, FI8, FF, nullptr, nullptr, 16, 512, 512, 256, F16, nullptr), QG_ERR_NULL);
    EXPECT(qg_int8_linear_t_zp_backward(F16, F16, FI8, FF, FF, 0, 512, 512, 256, F16, F16, nullptr), QG_ERR_SHAPE);

    // refresh: workspace queries (64-bit size arithmetic) and the host-side descriptor checks
    EXPECT(qg_range_apply(nullptr, F16, 512, 512, 128, FF, nullptr), QG_ERR_NULL);
    EXPECT(qg_orthonormalize_workspace_bytes(64, 128), 0);
    const size_t ob = qg_orthonormalize_workspace_bytes(512, 128);
    EXPECT(ob > 0 && ob % 256 == 0, 1);
    EXPECT(qg_orthonormalize(FF, 512, 128, FF + 4096, FI32, FF, ob - 1, nullptr), QG_ERR_WORKSPACE);
    EXPECT(qg_orthonormalize(FF, (int64_t)1 << 22, 1024, FF + 4096, FI32, FF, (size_t)1 << 40, nullptr), QG_ERR_SHAPE);
    EXPECT(qg_refresh_workspace_bytes(0, 512, 512, 128), 0);
    const size_t rb = qg_refresh_workspace_bytes(4, 512, 512, 128);
    EXPECT(rb > qg_refresh_workspace_bytes(1, 512, 512, 128), 1);
    EXPECT(qg_refresh_workspace_bytes(224, 11008, 4096, 1024) > qg_refresh_workspace_bytes(1, 11008, 4096, 1024), 1);
    {
        std::vector<qg_refresh_desc> rd(2);
        rd[0] = {F8, FF, F16, F8 + 4096, FF + 4096};
        rd[1] = {F8, FF, F16, F8 + 4096, nullptr};
        EXPECT(qg_subspace_refresh_many(2, rd.data(), 512, 512, 128, 256, 1, FF, FI32, FF, rb, nullptr), QG_ERR_NULL);
        EXPECT(qg_subspace_refresh_many(0, rd.data(), 512, 512, 128, 256, 1, FF, FI32, FF, rb, nullptr), QG_ERR_SHAPE);
        EXPECT(qg_subspace_refresh_many_ld(1, rd.data(), 512, 500, 504, 128, 256, 1, FF, FI32, FF, rb, nullptr), QG_ERR_SHAPE);
        EXPECT(qg_subspace_refresh_many_ld(1, rd.data(), 512, 500, 512, 128, 256, 1, FF, FI32, nullptr, 0, nullptr), QG_ERR_WORKSPACE);
        EXPECT(qg_subspace_refresh_many(1, rd.data(), 512, 512, 128, 256, 65, FF, FI32, FF, rb, nullptr), QG_ERR_SHAPE);
        EXPECT(qg_subspace_refresh(F8, FF, F16, 512, 512, 128, 256, 1, F8, FF + 4096, FF, FI32, FF, rb, nullptr), QG_ERR_SHAPE);
    }

    // the grouped-launch plan: built on the host into a heap buffer of exactly qg_plan_bytes
    {
        const int count = 7;
        const int64_t shapes[7][3] = {{4096, 4096, 1024}, {4096, 4096, 1024}, {11008, 4096, 1024}, {4096, 11008, 1024},
                                      {2048, 5461, 512},  {1024, 2736, 256},  {300, 700, 40}};
        std::vector<qg_matrix_desc> d(count);
        for (int i = 0; i < count; ++i) {
            std::memset(&d[i], 0, sizeof d[i]);
            d[i].m = shapes[i][0]; d[i].n = shapes[i][1]; d[i].r = shapes[i][2];
            d[i].Pq = F8; d[i].Ps = FF; d[i].G = F16; d[i].Wq = FI8; d[i].Ws = FF;
            d[i].M = FF; d[i].V = FF; d[i].R = FF; d[i].N = F16;
        }
        const size_t nb = qg_plan_bytes(count, d.data());
        EXPECT(nb > 0, 1);
        EXPECT(qg_plan_bytes(0, d.data()), 0);
        char* host = static_cast<char*>(std::malloc(nb));
        EXPECT(qg_plan_build(count, d.data(), host, nb - 1), QG_ERR_WORKSPACE);
        EXPECT(qg_plan_build(count, d.data(), host, nb), QG_OK);
        uint32_t hdr[16];
        std::memcpy(hdr, host, sizeof hdr);
        EXPECT(hdr[1], count);
        EXPECT(hdr[4] + hdr[5] + hdr[6], count);             // every matrix in exactly one class
        EXPECT(hdr[4], 4);
        d[4].ld = 5472;                                      // the odd row length with a pitch: aligned rows
        EXPECT(qg_plan_build(count, d.data(), host, nb), QG_OK);
        d[4].ld = 5464;
        EXPECT(qg_plan_build(count, d.data(), host, nb), QG_ERR_SHAPE);
        d[4].ld = 0;
        d[2].Wz = FF;                                        // zero points for some matrices only
        EXPECT(qg_plan_build(count, d.data(), host, nb), QG_ERR_NULL);
        d[2].Wz = nullptr;
        d[6].R = nullptr;                                    // no R buffer: the unfused phases must refuse the plan
        EXPECT(qg_plan_build(count, d.data(), host, nb), QG_OK);
        EXPECT(qg_project_many(count, host, FF, nb, nullptr), QG_ERR_NULL);
        EXPECT(qg_lowrank_adam_many(count, host, FF, nb, &hp, 1, nullptr), QG_ERR_NULL);
        EXPECT(qg_project_adam_many(count, host, FF, nb, &hp, 1, 1, nullptr), QG_ERR_NULL);
        EXPECT(qg_step_many(count, nullptr, FF, nb, &hp, 0, 1, nullptr), QG_ERR_NULL);
        EXPECT(qg_step_many(count + 1, host, FF, nb, &hp, 0, 1, nullptr), QG_ERR_WORKSPACE);
        EXPECT(qg_backproject_update_sr_many(count, host, FF, nb, &hp, 0, 0, nullptr), QG_ERR_SHAPE);
        EXPECT(qg_step_many(count, host, FF4, nb, &hp, 0, 1, nullptr), QG_ERR_ALIGN);
        std::free(host);
    }

    // the refresh policy (host only)
    {
        qg_policy p = {200, 0, 2, 200, 0.4f, 0.0f};
        EXPECT(qg_policy_update(&p, 0.9f), 0);
        EXPECT(qg_policy_update(&p, 0.9f), 1);
        EXPECT(p.interval, 400);
        EXPECT(p.next_refresh, 200 + 200 + 400);
        EXPECT(qg_policy_update(&p, 0.1f), 0);
        EXPECT(p.streak, 0);
        EXPECT(qg_policy_update(nullptr, 0.5f), -1);
    }

    if (failures) {
        std::printf("%d unexpected return codes\n", failures);
        return 1;
    }
    std::printf("sanitizer driver ok\n");
    return 0;
}
