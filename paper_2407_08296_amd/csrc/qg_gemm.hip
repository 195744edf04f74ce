// Host dispatch of the projection and back-projection kernels (see qg_gemm_kernels.h).
#include "qg_gemm_kernels.h"

namespace qg {

// ---------------------------------------------------------------------------
// Host dispatch
// ---------------------------------------------------------------------------
static inline unsigned grid8(uint32_t tiles) { return ((tiles + 7u) / 8u) * 8u; }

template <int BM, int BN, int BK, int WGM, int WGN, int MINWG>
static int launch_project_cfg(const uint8_t* Pq, const float* Ps, const uint16_t* G, float* R, int m, int n, int r,
                              hipStream_t stream) {
    const uint32_t tiles_r = (uint32_t)((r + BM - 1) / BM), tiles_n = (uint32_t)((n + BN - 1) / BN);
    const uint32_t tiles = tiles_r * tiles_n;
    const bool ragged = (r % BM) || (n % BN) || (m % BK);
    if (ragged)
        hipLaunchKernelGGL((k_project<BM, BN, BK, WGM, WGN, true, MINWG>), dim3(grid8(tiles)), dim3(WGM * WGN * 64), 0,
                           stream, Pq, Ps, G, R, m, n, r, tiles_r, tiles);
    else
        hipLaunchKernelGGL((k_project<BM, BN, BK, WGM, WGN, false, MINWG>), dim3(grid8(tiles)), dim3(WGM * WGN * 64), 0,
                           stream, Pq, Ps, G, R, m, n, r, tiles_r, tiles);
    return check_launch();
}

template <int BM, int BN, int BK, int WGM, int WGN, int MINWG>
static int launch_project_adam_cfg(const uint8_t* Pq, const float* Ps, const uint16_t* G, float* R, float* M, float* V,
                                   uint16_t* N, int m, int n, int r, const AdamCoef& coef, hipStream_t stream) {
    const uint32_t tiles_r = (uint32_t)((r + BM - 1) / BM), tiles_n = (uint32_t)((n + BN - 1) / BN);
    const uint32_t tiles = tiles_r * tiles_n;
    const bool ragged = (r % BM) || (n % BN) || (m % BK);
    if (ragged)
        hipLaunchKernelGGL((k_project_adam<BM, BN, BK, WGM, WGN, true, MINWG>), dim3(grid8(tiles)),
                           dim3(WGM * WGN * 64), 0, stream, Pq, Ps, G, R, M, V, N, m, n, r, tiles_r, tiles, coef);
    else
        hipLaunchKernelGGL((k_project_adam<BM, BN, BK, WGM, WGN, false, MINWG>), dim3(grid8(tiles)),
                           dim3(WGM * WGN * 64), 0, stream, Pq, Ps, G, R, M, V, N, m, n, r, tiles_r, tiles, coef);
    return check_launch();
}

int launch_project_adam(const uint8_t* Pq, const float* Ps, const uint16_t* G, float* R, float* M, float* V,
                        uint16_t* N, int64_t m, int64_t n, int64_t r, int64_t step, const qg_hparams* hp,
                        hipStream_t stream) {
    const AdamCoef coef = make_adam_coef(hp, step);
    const int64_t big_tiles = ((r + 127) / 128) * ((n + 255) / 256);
    if (big_tiles >= 384)
        return launch_project_adam_cfg<128, 256, 32, 2, 2, 2>(Pq, Ps, G, R, M, V, N, (int)m, (int)n, (int)r, coef, stream);
    return launch_project_adam_cfg<128, 128, 32, 2, 2, 2>(Pq, Ps, G, R, M, V, N, (int)m, (int)n, (int)r, coef, stream);
}

// Grouped launches: class 0 = matrices [0, n_fast) with the unguarded kernels, class 1 = the rest, guarded.
static inline int class_first(const PlanHeader* h, int cls) { return cls == 0 ? 0 : h->n_fast; }
static inline int class_count(const PlanHeader* h, int cls) { return cls == 0 ? h->n_fast : h->count - h->n_fast; }

int launch_project_adam_many(const PlanHeader* plan_host, const PlanHeader* plan_dev, int write_R, int64_t step,
                             const qg_hparams* hp, hipStream_t stream) {
    const AdamCoef coef = make_adam_coef(hp, step);
    for (int cls = 0; cls < 2; ++cls) {
        const int cnt = class_count(plan_host, cls);
        const uint32_t tiles = plan_host->proj_tiles[cls];
        if (cnt == 0 || tiles == 0) continue;
        if (cls == 0)
            hipLaunchKernelGGL((k_project_adam_many<kManyProjBM, kManyProjBN, 32, 2, 2, false, 2>), dim3(grid8(tiles)),
                               dim3(256), 0, stream, plan_dev, class_first(plan_host, cls), cnt, tiles, write_R, coef);
        else
            hipLaunchKernelGGL((k_project_adam_many<kManyProjBM, kManyProjBN, 32, 2, 2, true, 2>), dim3(grid8(tiles)),
                               dim3(256), 0, stream, plan_dev, class_first(plan_host, cls), cnt, tiles, write_R, coef);
        if (int e = check_launch()) return e;
    }
    return QG_OK;
}

// Tile choice: 128 x 256 tiles of R with two workgroups resident per CU (one's staging and epilogue overlap the
// other's MFMA work) when that still yields enough workgroups to fill 256 CUs twice; 128 x 128 tiles otherwise.
int launch_project(const uint8_t* Pq, const float* Ps, const uint16_t* G, float* R, int64_t m, int64_t n, int64_t r,
                   hipStream_t stream) {
    const int64_t big_tiles = ((r + 127) / 128) * ((n + 255) / 256);
    if (big_tiles >= 384)
        return launch_project_cfg<128, 256, 32, 2, 2, 2>(Pq, Ps, G, R, (int)m, (int)n, (int)r, stream);
    return launch_project_cfg<128, 128, 32, 2, 2, 2>(Pq, Ps, G, R, (int)m, (int)n, (int)r, stream);
}

template <int BMm, int BK, int WGn, int WGm, bool PREF, int MINWG>
static int launch_backproject_cfg(const uint8_t* Pq, const float* Ps, const uint16_t* N, int8_t* Wq, float* Ws,
                                  float* Udbg, int m, int n, int r, float alpha, float lr, uint32_t key,
                                  hipStream_t stream) {
    const uint32_t tiles_m = (uint32_t)((m + BMm - 1) / BMm), tiles_n = (uint32_t)((n + kGroup - 1) / kGroup);
    const uint32_t tiles = tiles_m * tiles_n;
    const bool ragged = (m % BMm) || (n % kGroup) || (r % BK);
    const dim3 grid(grid8(tiles)), block(WGn * WGm * 64);
    // the bounds-checked kernels need more registers: one workgroup fewer per CU
#define QG_LAUNCH_BP(RAG, DUMP)                                                                                     \
    hipLaunchKernelGGL((k_backproject<BMm, BK, WGn, WGm, RAG, DUMP, PREF, (RAG ? MINWG - 1 : MINWG)>), grid, block, 0,    \
                       stream, Pq, Ps, N, Wq, Ws, Udbg, m, n, r, alpha, lr, key, tiles_m, tiles)
    if (ragged) {
        if (Udbg) QG_LAUNCH_BP(true, true); else QG_LAUNCH_BP(true, false);
    } else {
        if (Udbg) QG_LAUNCH_BP(false, true); else QG_LAUNCH_BP(false, false);
    }
#undef QG_LAUNCH_BP
    return check_launch();
}

int launch_backproject(const uint8_t* Pq, const float* Ps, const uint16_t* N, int8_t* Wq, float* Ws, float* Udbg,
                       int64_t m, int64_t n, int64_t r, float alpha, float lr, uint64_t seed, int64_t step,
                       hipStream_t stream) {
    const uint32_t key = sr_key(seed, (uint64_t)step, 0u);
    // 128-row tiles, weight tile sharing the staging LDS, three workgroups per CU: the VALU-heavy update epilogue of
    // one workgroup overlaps the MFMA main loops of the others.
    return launch_backproject_cfg<128, 32, 2, 2, false, 3>(Pq, Ps, N, Wq, Ws, Udbg, (int)m, (int)n, (int)r, alpha, lr,
                                                           key, stream);
}

int launch_project_many(const PlanHeader* plan_host, const PlanHeader* plan_dev, hipStream_t stream) {
    for (int cls = 0; cls < 2; ++cls) {
        const int cnt = class_count(plan_host, cls);
        const uint32_t tiles = plan_host->proj_tiles[cls];
        if (cnt == 0 || tiles == 0) continue;
        if (cls == 0)
            hipLaunchKernelGGL((k_project_many<kManyProjBM, kManyProjBN, 32, 2, 2, false, 2>), dim3(grid8(tiles)),
                               dim3(256), 0, stream, plan_dev, class_first(plan_host, cls), cnt, tiles);
        else
            hipLaunchKernelGGL((k_project_many<kManyProjBM, kManyProjBN, 32, 2, 2, true, 2>), dim3(grid8(tiles)),
                               dim3(256), 0, stream, plan_dev, class_first(plan_host, cls), cnt, tiles);
        if (int e = check_launch()) return e;
    }
    return QG_OK;
}

int launch_backproject_many(const PlanHeader* plan_host, const PlanHeader* plan_dev, float alpha, float lr,
                            uint64_t seed, int64_t step, hipStream_t stream) {
    for (int cls = 0; cls < 2; ++cls) {
        const int cnt = class_count(plan_host, cls);
        const uint32_t tiles = plan_host->bp_tiles[cls];
        if (cnt == 0 || tiles == 0) continue;
        if (cls == 0)
            hipLaunchKernelGGL((k_backproject_many<kManyBpBM, 32, 2, 2, false, false, 3>), dim3(grid8(tiles)), dim3(256),
                               0, stream, plan_dev, class_first(plan_host, cls), cnt, tiles, alpha, lr, seed,
                               (uint64_t)step);
        else
            hipLaunchKernelGGL((k_backproject_many<kManyBpBM, 32, 2, 2, true, false, 2>), dim3(grid8(tiles)), dim3(256),
                               0, stream, plan_dev, class_first(plan_host, cls), cnt, tiles, alpha, lr, seed,
                               (uint64_t)step);
        if (int e = check_launch()) return e;
    }
    return QG_OK;
}

}  // namespace qg
