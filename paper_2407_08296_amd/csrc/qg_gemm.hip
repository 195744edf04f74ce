// Host dispatch of the projection and back-projection kernels (see qg_gemm_kernels.h).
#include "qg_gemm_kernels.h"

namespace qg {

// ---------------------------------------------------------------------------
// Host dispatch
// ---------------------------------------------------------------------------
static inline unsigned grid8(uint32_t tiles) { return ((tiles + 7u) / 8u) * 8u; }

// Edge mode of a matrix for tiles of TM (along r for the projection, along m for the back-projection) x TN and K
// steps of BK over `kdim`; ld is the row pitch of the n-wide arrays.  The direct loads need 16-byte aligned rows
// (ld % 8, and r % 16 for the 8-byte P fetches) and 32-bit per-lane offsets.
static inline int edge_mode(int64_t tiled, int TM, int64_t n, int64_t ld, int TN, int64_t kdim, int BK, int64_t r) {
    if (ld > (int64_t(1) << 24) || (ld % 8) != 0 || (r % 16) != 0) return kUnaligned;
    if ((tiled % TM) == 0 && (n % TN) == 0 && (kdim % BK) == 0) return kExact;
    return kMasked;
}
int project_mode(int64_t m, int64_t n, int64_t ld, int64_t r) { return edge_mode(r, kManyProjBM, n, ld, kManyProjBN, m, 32, r); }
int backproject_mode(int64_t m, int64_t n, int64_t ld, int64_t r) {
    return edge_mode(m, kManyBpBM, n, ld, kManyBpBN, r, 32, r);
}

template <int BM, int BN, int BK, int WGM, int WGN, int MINWG>
static int launch_project_cfg(const uint8_t* Pq, const float* Ps, const uint16_t* G, float* R, int m, int n, int ld,
                              int r, hipStream_t stream) {
    const uint32_t tiles_r = (uint32_t)((r + BM - 1) / BM), tiles_n = (uint32_t)((n + BN - 1) / BN);
    const uint32_t tiles = tiles_r * tiles_n;
    const dim3 grid(grid8(tiles)), block(WGM * WGN * 64);
    switch (edge_mode(r, BM, n, ld, BN, m, BK, r)) {
        case kExact:
            hipLaunchKernelGGL((k_project<BM, BN, BK, WGM, WGN, kExact, MINWG>), grid, block, 0, stream, Pq, Ps, G, R, m,
                               n, ld, r, tiles_r, tiles);
            break;
        case kMasked:
            hipLaunchKernelGGL((k_project<BM, BN, BK, WGM, WGN, kMasked, MINWG>), grid, block, 0, stream, Pq, Ps, G, R,
                               m, n, ld, r, tiles_r, tiles);
            break;
        default:
            hipLaunchKernelGGL((k_project<BM, BN, BK, WGM, WGN, kUnaligned, MINWG>), grid, block, 0, stream, Pq, Ps, G,
                               R, m, n, ld, r, tiles_r, tiles);
    }
    return check_launch();
}

template <int BM, int BN, int BK, int WGM, int WGN, int MINWG>
static int launch_project_adam_cfg(const uint8_t* Pq, const float* Ps, const uint16_t* G, float* R, float* M, float* V,
                                   uint16_t* N, int m, int n, int ld, int r, const AdamCoef& coef, hipStream_t stream) {
    const uint32_t tiles_r = (uint32_t)((r + BM - 1) / BM), tiles_n = (uint32_t)((n + BN - 1) / BN);
    const uint32_t tiles = tiles_r * tiles_n;
    const dim3 grid(grid8(tiles)), block(WGM * WGN * 64);
    switch (edge_mode(r, BM, n, ld, BN, m, BK, r)) {
        case kExact:
            hipLaunchKernelGGL((k_project_adam<BM, BN, BK, WGM, WGN, kExact, MINWG>), grid, block, 0, stream, Pq, Ps, G,
                               R, M, V, N, m, n, ld, r, tiles_r, tiles, coef);
            break;
        case kMasked:
            hipLaunchKernelGGL((k_project_adam<BM, BN, BK, WGM, WGN, kMasked, MINWG>), grid, block, 0, stream, Pq, Ps,
                               G, R, M, V, N, m, n, ld, r, tiles_r, tiles, coef);
            break;
        default:
            hipLaunchKernelGGL((k_project_adam<BM, BN, BK, WGM, WGN, kUnaligned, MINWG>), grid, block, 0, stream, Pq,
                               Ps, G, R, M, V, N, m, n, ld, r, tiles_r, tiles, coef);
    }
    return check_launch();
}

// ld: row pitch in elements of G, R, M, V, N (n for dense rows).
int launch_project_adam(const uint8_t* Pq, const float* Ps, const uint16_t* G, float* R, float* M, float* V,
                        uint16_t* N, int64_t m, int64_t n, int64_t ld, int64_t r, int64_t step, const qg_hparams* hp,
                        hipStream_t stream) {
    const AdamCoef coef = make_adam_coef(hp, step);
    const int64_t big_tiles = ((r + 127) / 128) * ((n + 255) / 256);
    if (big_tiles >= 384)
        return launch_project_adam_cfg<128, 256, 32, 2, 2, 2>(Pq, Ps, G, R, M, V, N, (int)m, (int)n, (int)ld, (int)r, coef,
                                                              stream);
    return launch_project_adam_cfg<128, 128, 32, 2, 2, 2>(Pq, Ps, G, R, M, V, N, (int)m, (int)n, (int)ld, (int)r, coef,
                                                          stream);
}

// Grouped launches: the plan stores the matrices class by class (kExact, kMasked, kUnaligned); each class that is
// not empty gets a launch of its own kernel instance.
static inline int class_first(const PlanHeader* h, int cls) {
    int first = 0;
    for (int c = 0; c < cls; ++c) first += h->class_count[c];
    return first;
}
static inline int class_count(const PlanHeader* h, int cls) { return h->class_count[cls]; }

int launch_project_adam_many(const PlanHeader* plan_host, const PlanHeader* plan_dev, int write_R, int64_t step,
                             const qg_hparams* hp, hipStream_t stream) {
    const AdamCoef coef = make_adam_coef(hp, step);
    for (int cls = 0; cls < kPlanClasses; ++cls) {
        const int cnt = class_count(plan_host, cls), first = class_first(plan_host, cls);
        const uint32_t tiles = plan_host->proj_tiles[cls];
        if (cnt == 0 || tiles == 0) continue;
        const dim3 grid(grid8(tiles)), block(256);
        if (cls == kExact)
            hipLaunchKernelGGL((k_project_adam_many<kManyProjBM, kManyProjBN, 32, 2, 2, kExact, 2>), grid, block, 0,
                               stream, plan_dev, first, cnt, tiles, write_R, coef);
        else if (cls == kMasked)
            hipLaunchKernelGGL((k_project_adam_many<kManyProjBM, kManyProjBN, 32, 2, 2, kMasked, 2>), grid, block, 0,
                               stream, plan_dev, first, cnt, tiles, write_R, coef);
        else
            hipLaunchKernelGGL((k_project_adam_many<kManyProjBM, kManyProjBN, 32, 2, 2, kUnaligned, 2>), grid, block, 0,
                               stream, plan_dev, first, cnt, tiles, write_R, coef);
        if (int e = check_launch()) return e;
    }
    return QG_OK;
}

// Tile choice: 128 x 256 tiles of R with two workgroups resident per CU (one's staging and epilogue overlap the
// other's MFMA work) when that still yields enough workgroups to fill 256 CUs twice; 128 x 128 tiles otherwise.
int launch_project(const uint8_t* Pq, const float* Ps, const uint16_t* G, float* R, int64_t m, int64_t n, int64_t ld,
                   int64_t r, hipStream_t stream) {
    const int64_t big_tiles = ((r + 127) / 128) * ((n + 255) / 256);
    if (big_tiles >= 384)
        return launch_project_cfg<128, 256, 32, 2, 2, 2>(Pq, Ps, G, R, (int)m, (int)n, (int)ld, (int)r, stream);
    return launch_project_cfg<128, 128, 32, 2, 2, 2>(Pq, Ps, G, R, (int)m, (int)n, (int)ld, (int)r, stream);
}

// R_z = dequant(P_z)^T G_z for `count` (<= kProjBatchMax) matrices of one shape in one launch, with the tiles of the
// grouped step (same arithmetic per element as launch_project: the order of the sum over m does not depend on the
// tile shape).
int launch_project_batch(const ProjBatch& batch, int count, float* R, int64_t strideR, int64_t m, int64_t n, int64_t ld,
                         int64_t r, hipStream_t stream) {
    constexpr int BM = kManyProjBM, BN = kManyProjBN;
    const uint32_t tiles_r = (uint32_t)((r + BM - 1) / BM), tiles_n = (uint32_t)((n + BN - 1) / BN);
    const uint32_t tiles_per = tiles_r * tiles_n, tiles = tiles_per * (uint32_t)count;
    const dim3 grid(grid8(tiles)), block(256);
    switch (edge_mode(r, BM, n, ld, BN, m, 32, r)) {
        case kExact:
            hipLaunchKernelGGL((k_project_batch<BM, BN, 32, 2, 2, kExact, 2>), grid, block, 0, stream, batch, R, strideR,
                               (int)m, (int)n, (int)ld, (int)r, tiles_r, tiles_per, tiles);
            break;
        case kMasked:
            hipLaunchKernelGGL((k_project_batch<BM, BN, 32, 2, 2, kMasked, 2>), grid, block, 0, stream, batch, R, strideR,
                               (int)m, (int)n, (int)ld, (int)r, tiles_r, tiles_per, tiles);
            break;
        default:
            hipLaunchKernelGGL((k_project_batch<BM, BN, 32, 2, 2, kUnaligned, 2>), grid, block, 0, stream, batch, R,
                               strideR, (int)m, (int)n, (int)ld, (int)r, tiles_r, tiles_per, tiles);
    }
    return check_launch();
}

// Workgroups per CU the back-projection instances are compiled for (the checked variants need more registers).
static constexpr int kBpWgPerCu[3] = {3, 3, 2};

template <int BMm, int BK, int WGn, int WGm, bool PREF>
static int launch_backproject_cfg(const uint8_t* Pq, const float* Ps, const uint16_t* N, int8_t* Wq, float* Ws,
                                  float* Wz, float* Udbg, int m, int n, int ld, int r, float alpha, float lr,
                                  uint32_t key, hipStream_t stream) {
    const uint32_t tiles_m = (uint32_t)((m + BMm - 1) / BMm), tiles_n = (uint32_t)((n + kGroup - 1) / kGroup);
    const uint32_t tiles = tiles_m * tiles_n;
    const dim3 grid(grid8(tiles)), block(WGn * WGm * 64);
#define QG_LAUNCH_BP(MODE, DUMP)                                                                                    \
    hipLaunchKernelGGL((k_backproject<BMm, BK, WGn, WGm, MODE, DUMP, PREF, kBpWgPerCu[MODE]>), grid, block, 0, stream, \
                       Pq, Ps, N, Wq, Ws, nullptr, Udbg, m, n, ld, r, alpha, lr, key, tiles_m, tiles)
#define QG_LAUNCH_BP_ZP(MODE)                                                                                        \
    hipLaunchKernelGGL((k_backproject<BMm, BK, WGn, WGm, MODE, false, PREF, kBpWgPerCu[MODE], true>), grid, block, 0, \
                       stream, Pq, Ps, N, Wq, Ws, Wz, nullptr, m, n, ld, r, alpha, lr, key, tiles_m, tiles)
    const int mode = edge_mode(m, BMm, n, ld, kGroup, r, BK, r);
    if (Wz != nullptr) {   // zero-point weights (no U dump)
        if (mode == kExact) QG_LAUNCH_BP_ZP(kExact);
        else if (mode == kMasked) QG_LAUNCH_BP_ZP(kMasked);
        else QG_LAUNCH_BP_ZP(kUnaligned);
        return check_launch();
    }
    switch (mode) {
        case kExact:
            if (Udbg) QG_LAUNCH_BP(kExact, true); else QG_LAUNCH_BP(kExact, false);
            break;
        case kMasked:
            if (Udbg) QG_LAUNCH_BP(kMasked, true); else QG_LAUNCH_BP(kMasked, false);
            break;
        default:
            if (Udbg) QG_LAUNCH_BP(kUnaligned, true); else QG_LAUNCH_BP(kUnaligned, false);
    }
#undef QG_LAUNCH_BP
#undef QG_LAUNCH_BP_ZP
    return check_launch();
}

// ld: row pitch in elements of N and Wq (n for dense rows); the U dump, if asked for, is dense.
int launch_backproject(const uint8_t* Pq, const float* Ps, const uint16_t* N, int8_t* Wq, float* Ws, float* Wz,
                       float* Udbg, int64_t m, int64_t n, int64_t ld, int64_t r, float alpha, float lr, uint64_t seed,
                       int64_t step, hipStream_t stream) {
    const uint32_t key = sr_key(seed, (uint64_t)step, 0u);
    // 128-row tiles, weight tile sharing the staging LDS, several workgroups per CU: the VALU-heavy update epilogue
    // of one workgroup overlaps the MFMA main loops of the others.
    return launch_backproject_cfg<128, 32, 2, 2, false>(Pq, Ps, N, Wq, Ws, Wz, Udbg, (int)m, (int)n, (int)ld, (int)r, alpha,
                                                           lr, key, stream);
}

int launch_project_many(const PlanHeader* plan_host, const PlanHeader* plan_dev, hipStream_t stream) {
    for (int cls = 0; cls < kPlanClasses; ++cls) {
        const int cnt = class_count(plan_host, cls), first = class_first(plan_host, cls);
        const uint32_t tiles = plan_host->proj_tiles[cls];
        if (cnt == 0 || tiles == 0) continue;
        const dim3 grid(grid8(tiles)), block(256);
        if (cls == kExact)
            hipLaunchKernelGGL((k_project_many<kManyProjBM, kManyProjBN, 32, 2, 2, kExact, 2>), grid, block, 0, stream,
                               plan_dev, first, cnt, tiles);
        else if (cls == kMasked)
            hipLaunchKernelGGL((k_project_many<kManyProjBM, kManyProjBN, 32, 2, 2, kMasked, 2>), grid, block, 0, stream,
                               plan_dev, first, cnt, tiles);
        else
            hipLaunchKernelGGL((k_project_many<kManyProjBM, kManyProjBN, 32, 2, 2, kUnaligned, 2>), grid, block, 0,
                               stream, plan_dev, first, cnt, tiles);
        if (int e = check_launch()) return e;
    }
    return QG_OK;
}

int launch_backproject_many(const PlanHeader* plan_host, const PlanHeader* plan_dev, float alpha, float lr,
                            uint64_t seed, int64_t step, hipStream_t stream) {
    for (int cls = 0; cls < kPlanClasses; ++cls) {
        const int cnt = class_count(plan_host, cls), first = class_first(plan_host, cls);
        const uint32_t tiles = plan_host->bp_tiles[cls];
        if (cnt == 0 || tiles == 0) continue;
        const dim3 grid(grid8(tiles)), block(256);
        if (plan_host->zero_points) {
            if (cls == kExact)
                hipLaunchKernelGGL((k_backproject_many<kManyBpBM, 32, 2, 2, kExact, false, kBpWgPerCu[kExact], true>), grid,
                                   block, 0, stream, plan_dev, first, cnt, tiles, alpha, lr, seed, (uint64_t)step);
            else if (cls == kMasked)
                hipLaunchKernelGGL((k_backproject_many<kManyBpBM, 32, 2, 2, kMasked, false, kBpWgPerCu[kMasked], true>), grid,
                                   block, 0, stream, plan_dev, first, cnt, tiles, alpha, lr, seed, (uint64_t)step);
            else
                hipLaunchKernelGGL((k_backproject_many<kManyBpBM, 32, 2, 2, kUnaligned, false, kBpWgPerCu[kUnaligned], true>),
                                   grid, block, 0, stream, plan_dev, first, cnt, tiles, alpha, lr, seed, (uint64_t)step);
        } else if (cls == kExact)
            hipLaunchKernelGGL((k_backproject_many<kManyBpBM, 32, 2, 2, kExact, false, kBpWgPerCu[kExact]>), grid, block,
                               0, stream, plan_dev, first, cnt, tiles, alpha, lr, seed, (uint64_t)step);
        else if (cls == kMasked)
            hipLaunchKernelGGL((k_backproject_many<kManyBpBM, 32, 2, 2, kMasked, false, kBpWgPerCu[kMasked]>), grid,
                               block, 0, stream, plan_dev, first, cnt, tiles, alpha, lr, seed, (uint64_t)step);
        else
            hipLaunchKernelGGL((k_backproject_many<kManyBpBM, 32, 2, 2, kUnaligned, false, kBpWgPerCu[kUnaligned]>),
                               grid, block, 0, stream, plan_dev, first, cnt, tiles, alpha, lr, seed, (uint64_t)step);
        if (int e = check_launch()) return e;
    }
    return QG_OK;
}

}  // namespace qg
