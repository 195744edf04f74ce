// C-ABI entry points that validate arguments and chain the kernels of one step
// (Sec. 3.5), the grouped-launch plan, and the host-side refresh policy (Sec. 3.2).
#include <atomic>
#include <cstring>

#include "qg_common.h"
#include "qg_plan.h"

namespace qg {

static std::atomic<int> g_last_hip_error{0};

void set_hip_error(hipError_t e) { g_last_hip_error.store((int)e); }

int check_launch() {
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_hip_error(e);
        return QG_ERR_HIP;
    }
    return QG_OK;
}

// defined in qg_gemm.hip / qg_adam.hip
int launch_project(const uint8_t*, const float*, const uint16_t*, float*, int64_t, int64_t, int64_t, int64_t, hipStream_t);
int launch_backproject(const uint8_t*, const float*, const uint16_t*, int8_t*, float*, float*, float*, int64_t, int64_t,
                       int64_t, int64_t, float, float, uint64_t, int64_t, hipStream_t);   // ..., Ws, Wz (or null), U dump (or null); m, n, ld, r
int launch_adam(const float*, float*, float*, uint16_t*, int64_t, int64_t, const qg_hparams*, hipStream_t);
int launch_project_many(const PlanHeader*, const PlanHeader*, hipStream_t);
int launch_backproject_many(const PlanHeader*, const PlanHeader*, float, float, uint64_t, int64_t, hipStream_t);
int launch_adam_many(const PlanHeader*, const PlanHeader*, int64_t, const qg_hparams*, hipStream_t);
int launch_project_adam(const uint8_t*, const float*, const uint16_t*, float*, float*, float*, uint16_t*, int64_t, int64_t,
                        int64_t, int64_t, int64_t, const qg_hparams*, hipStream_t);   // m, n, ld, r, step
int launch_project_adam_many(const PlanHeader*, const PlanHeader*, int, int64_t, const qg_hparams*, hipStream_t);
int project_mode(int64_t m, int64_t n, int64_t ld, int64_t r);       // edge class the grouped projection needs for a matrix
int backproject_mode(int64_t m, int64_t n, int64_t ld, int64_t r);   // ... and the grouped back-projection
constexpr int kAdamChunkElems = 256 * 4 * 4;  // must equal kAdamChunk of qg_adam.hip

static int check_mnr(int64_t m, int64_t n, int64_t r, int group) {
    if (m <= 0 || n <= 0 || r <= 0 || (r & 7) || r > m) return QG_ERR_SHAPE;
    if (m > (int64_t(1) << 32) / n || m * n >= (int64_t(1) << 32)) return QG_ERR_SHAPE;
    if (group != kGroup) return QG_ERR_GROUP;
    return QG_OK;
}

}  // namespace qg

using namespace qg;

extern "C" const char* qg_status_string(int status) {
    switch (status) {
        case QG_OK: return "ok";
        case QG_ERR_NULL: return "null pointer";
        case QG_ERR_SHAPE: return "shape or step out of range";
        case QG_ERR_GROUP: return "unsupported quantization block size (only 256)";
        case QG_ERR_ALIGN: return "pointer not 16-byte aligned";
        case QG_ERR_WORKSPACE: return "workspace missing or too small";
        case QG_ERR_HIP: return "HIP error (see qg_last_hip_error)";
        default: return "unknown status";
    }
}

extern "C" int qg_last_hip_error(void) { return g_last_hip_error.load(); }

extern "C" size_t qg_workspace_bytes(int64_t, int64_t, int64_t) { return 0; }

extern "C" int qg_project(const uint8_t* Pq, const float* Ps, const uint16_t* G_bf16, int64_t m, int64_t n, int64_t r,
                          int group, float* R, void* workspace, size_t workspace_bytes, void* stream) {
    (void)workspace;
    (void)workspace_bytes;
    if (!Pq || !Ps || !G_bf16 || !R) return QG_ERR_NULL;
    if (int e = check_mnr(m, n, r, group)) return e;
    if (!aligned16(Pq) || !aligned16(Ps) || !aligned16(G_bf16) || !aligned16(R)) return QG_ERR_ALIGN;
    return launch_project(Pq, Ps, G_bf16, R, m, n, n, r, (hipStream_t)stream);
}

extern "C" int qg_backproject_update_sr(const uint8_t* Pq, const float* Ps, const uint16_t* N_bf16, int8_t* Wq,
                                        float* Ws, int64_t m, int64_t n, int64_t r, int group, float alpha, float lr,
                                        uint64_t seed, int64_t step, float* U_debug, void* stream) {
    if (!Pq || !Ps || !N_bf16 || !Wq || !Ws) return QG_ERR_NULL;
    if (int e = check_mnr(m, n, r, group)) return e;
    if (step < 1) return QG_ERR_SHAPE;
    if (!aligned16(Pq) || !aligned16(Ps) || !aligned16(N_bf16) || !aligned16(Wq) || !aligned16(Ws) ||
        (U_debug && !aligned16(U_debug)))
        return QG_ERR_ALIGN;
    return launch_backproject(Pq, Ps, N_bf16, Wq, Ws, nullptr, U_debug, m, n, n, r, alpha, lr, seed, step, (hipStream_t)stream);
}

extern "C" int qg_backproject_update_sr_zp(const uint8_t* Pq, const float* Ps, const uint16_t* N_bf16, int8_t* Wq,
                                           float* Ws, float* Wz, int64_t m, int64_t n, int64_t r, int group, float alpha,
                                           float lr, uint64_t seed, int64_t step, void* stream) {
    if (!Pq || !Ps || !N_bf16 || !Wq || !Ws || !Wz) return QG_ERR_NULL;
    if (int e = check_mnr(m, n, r, group)) return e;
    if (step < 1) return QG_ERR_SHAPE;
    if (!aligned16(Pq) || !aligned16(Ps) || !aligned16(N_bf16) || !aligned16(Wq) || !aligned16(Ws) || !aligned16(Wz))
        return QG_ERR_ALIGN;
    return launch_backproject(Pq, Ps, N_bf16, Wq, Ws, Wz, nullptr, m, n, n, r, alpha, lr, seed, step, (hipStream_t)stream);
}

extern "C" int qg_step_zp(const uint8_t* Pq, const float* Ps, const uint16_t* G_bf16, int8_t* Wq, float* Ws, float* Wz,
                          float* M, float* V, float* R, uint16_t* N_bf16, int64_t m, int64_t n, int64_t r, int group,
                          const qg_hparams* hp, uint64_t seed, int64_t step, void* stream) {
    if (!Pq || !Ps || !G_bf16 || !Wq || !Ws || !Wz || !M || !V || !N_bf16 || !hp) return QG_ERR_NULL;
    if (int e = check_mnr(m, n, r, group)) return e;
    if (step < 1) return QG_ERR_SHAPE;
    if (!aligned16(Pq) || !aligned16(Ps) || !aligned16(G_bf16) || !aligned16(Wq) || !aligned16(Ws) || !aligned16(Wz) ||
        !aligned16(M) || !aligned16(V) || (R && !aligned16(R)) || !aligned16(N_bf16))
        return QG_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    if (int e = launch_project_adam(Pq, Ps, G_bf16, R, M, V, N_bf16, m, n, n, r, step, hp, s)) return e;
    return launch_backproject(Pq, Ps, N_bf16, Wq, Ws, Wz, nullptr, m, n, n, r, hp->alpha, hp->lr, seed, step, s);
}

extern "C" int qg_step(const uint8_t* Pq, const float* Ps, const uint16_t* G_bf16, int8_t* Wq, float* Ws, float* M,
                       float* V, float* R, uint16_t* N_bf16, int64_t m, int64_t n, int64_t r, int group,
                       const qg_hparams* hp, uint64_t seed, int64_t step, void* workspace, size_t workspace_bytes,
                       void* stream) {
    (void)workspace;
    (void)workspace_bytes;
    if (!Pq || !Ps || !G_bf16 || !Wq || !Ws || !M || !V || !N_bf16 || !hp) return QG_ERR_NULL;
    if (int e = check_mnr(m, n, r, group)) return e;
    if (step < 1) return QG_ERR_SHAPE;
    if (!aligned16(Pq) || !aligned16(Ps) || !aligned16(G_bf16) || !aligned16(Wq) || !aligned16(Ws) || !aligned16(M) ||
        !aligned16(V) || (R && !aligned16(R)) || !aligned16(N_bf16))
        return QG_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    if (int e = launch_project_adam(Pq, Ps, G_bf16, R, M, V, N_bf16, m, n, n, r, step, hp, s)) return e;
    return launch_backproject(Pq, Ps, N_bf16, Wq, Ws, nullptr, nullptr, m, n, n, r, hp->alpha, hp->lr, seed, step, s);
}

extern "C" int qg_step_ld(const uint8_t* Pq, const float* Ps, const uint16_t* G_bf16, int8_t* Wq, float* Ws, float* M,
                          float* V, float* R, uint16_t* N_bf16, int64_t m, int64_t n, int64_t ld, int64_t r, int group,
                          const qg_hparams* hp, uint64_t seed, int64_t step, void* stream) {
    if (!Pq || !Ps || !G_bf16 || !Wq || !Ws || !M || !V || !N_bf16 || !hp) return QG_ERR_NULL;
    if (int e = check_mnr(m, n, r, group)) return e;
    if (step < 1) return QG_ERR_SHAPE;
    if (ld == 0) ld = n;
    if (ld != n && (ld < n || (ld & 15) || m * ld >= (int64_t(1) << 32))) return QG_ERR_SHAPE;
    if (!aligned16(Pq) || !aligned16(Ps) || !aligned16(G_bf16) || !aligned16(Wq) || !aligned16(Ws) || !aligned16(M) ||
        !aligned16(V) || (R && !aligned16(R)) || !aligned16(N_bf16))
        return QG_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    if (int e = launch_project_adam(Pq, Ps, G_bf16, R, M, V, N_bf16, m, n, ld, r, step, hp, s)) return e;
    return launch_backproject(Pq, Ps, N_bf16, Wq, Ws, nullptr, nullptr, m, n, ld, r, hp->alpha, hp->lr, seed, step, s);
}

extern "C" int qg_policy_update(qg_policy* p, float cos) {
    if (!p) return -1;
    p->last_cos = cos;
    p->streak = (cos >= p->threshold) ? p->streak + 1 : 0;
    int doubled = 0;
    if (p->streak >= p->k) {
        p->interval *= 2;
        p->streak = 0;
        doubled = 1;
    }
    p->next_refresh += p->interval;
    return doubled;
}

extern "C" size_t qg_plan_bytes(int count, const qg_matrix_desc* descs) {
    (void)descs;
    if (count <= 0) return 0;
    return sizeof(PlanHeader) + (size_t)count * sizeof(PlanMatrix);
}

extern "C" int qg_plan_build(int count, const qg_matrix_desc* descs, void* plan_host, size_t plan_bytes) {
    if (!descs || !plan_host) return QG_ERR_NULL;
    if (count <= 0) return QG_ERR_SHAPE;
    if (plan_bytes < qg_plan_bytes(count, descs)) return QG_ERR_WORKSPACE;
    PlanHeader h;
    std::memset(&h, 0, sizeof h);
    h.magic = kPlanMagic;
    h.count = count;
    PlanMatrix* mats = reinterpret_cast<PlanMatrix*>(reinterpret_cast<char*>(plan_host) + sizeof(PlanHeader));
    for (int i = 0; i < count; ++i) {
        const qg_matrix_desc& d = descs[i];
        if (!d.Pq || !d.Ps || !d.G || !d.Wq || !d.Ws || !d.M || !d.V || !d.N) return QG_ERR_NULL;
        if (!d.R) h.no_R = 1;   // the unfused phases cannot run on this plan
        if (int e = check_mnr(d.m, d.n, d.r, kGroup)) return e;
        // a row pitch other than n: at least n, rows 16-byte aligned in every array, m * ld inside the 32-bit range
        if (d.ld != 0 && d.ld != d.n && (d.ld < d.n || (d.ld & 15) || d.m * d.ld >= (int64_t(1) << 32))) return QG_ERR_SHAPE;
        if (!aligned16(d.Pq) || !aligned16(d.Ps) || !aligned16(d.G) || !aligned16(d.Wq) || !aligned16(d.Ws) ||
            !aligned16(d.M) || !aligned16(d.V) || (d.R && !aligned16(d.R)) || !aligned16(d.N) ||
            (d.Wz && !aligned16(d.Wz)))
            return QG_ERR_ALIGN;
        if ((d.Wz != nullptr) != (descs[0].Wz != nullptr)) return QG_ERR_NULL;   // zero points: all matrices or none
    }
    h.zero_points = descs[0].Wz != nullptr ? 1u : 0u;
    auto matrix_class = [](const qg_matrix_desc& d) {
        const int64_t ld = d.ld ? d.ld : d.n;
        const int a = project_mode(d.m, d.n, ld, d.r), b = backproject_mode(d.m, d.n, ld, d.r);
        return a > b ? a : b;
    };
    uint64_t adam = 0, proj[kPlanClasses] = {0, 0, 0}, bp[kPlanClasses] = {0, 0, 0};
    int out = 0;
    for (int cls = 0; cls < kPlanClasses; ++cls) {
        for (int i = 0; i < count; ++i) {
            const qg_matrix_desc& d = descs[i];
            if (matrix_class(d) != cls) continue;
            PlanMatrix pm;
            std::memset(&pm, 0, sizeof pm);
            pm.m = d.m; pm.n = d.n; pm.r = d.r;
            pm.ld = d.ld ? d.ld : d.n;
            pm.Pq = d.Pq; pm.Ps = d.Ps; pm.G = d.G; pm.Wq = d.Wq; pm.Ws = d.Ws;
            pm.M = d.M; pm.V = d.V; pm.R = d.R; pm.N = d.N; pm.Wz = d.Wz;
            pm.index = (uint32_t)i;
            pm.adam_chunk0 = (uint32_t)adam;
            pm.proj_tile0 = (uint32_t)proj[cls];
            pm.bp_tile0 = (uint32_t)bp[cls];
            pm.proj_tiles_r = (uint32_t)((d.r + kManyProjBM - 1) / kManyProjBM);
            pm.bp_tiles_m = (uint32_t)((d.m + kManyBpBM - 1) / kManyBpBM);
            adam += (uint64_t)((d.r * pm.ld + kAdamChunkElems - 1) / kAdamChunkElems);
            proj[cls] += (uint64_t)pm.proj_tiles_r * (uint64_t)((d.n + kManyProjBN - 1) / kManyProjBN);
            bp[cls] += (uint64_t)pm.bp_tiles_m * (uint64_t)((d.n + kManyBpBN - 1) / kManyBpBN);
            mats[out++] = pm;
            ++h.class_count[cls];
        }
    }
    if (adam > 0x7FFFFFF0ull) return QG_ERR_SHAPE;
    h.adam_chunks = (uint32_t)adam;
    for (int cls = 0; cls < kPlanClasses; ++cls) {
        if (proj[cls] > 0x7FFFFFF0ull || bp[cls] > 0x7FFFFFF0ull) return QG_ERR_SHAPE;
        h.proj_tiles[cls] = (uint32_t)proj[cls];
        h.bp_tiles[cls] = (uint32_t)bp[cls];
    }
    std::memcpy(plan_host, &h, sizeof h);
    return QG_OK;
}

static int check_plan(int count, const void* plan_host, const void* plan_dev, size_t plan_bytes) {
    if (!plan_host || !plan_dev) return QG_ERR_NULL;
    if (count <= 0) return QG_ERR_SHAPE;
    if (plan_bytes < sizeof(PlanHeader) + (size_t)count * sizeof(PlanMatrix)) return QG_ERR_WORKSPACE;
    const PlanHeader* h = reinterpret_cast<const PlanHeader*>(plan_host);
    if (h->magic != kPlanMagic || h->count != count) return QG_ERR_WORKSPACE;
    if (!aligned16(plan_dev)) return QG_ERR_ALIGN;
    return QG_OK;
}

extern "C" int qg_project_many(int count, const void* plan_host, const void* plan_dev, size_t plan_bytes,
                               void* stream) {
    if (int e = check_plan(count, plan_host, plan_dev, plan_bytes)) return e;
    if (reinterpret_cast<const PlanHeader*>(plan_host)->no_R) return QG_ERR_NULL;   // needs every R buffer
    return launch_project_many(reinterpret_cast<const PlanHeader*>(plan_host),
                               reinterpret_cast<const PlanHeader*>(plan_dev), (hipStream_t)stream);
}

extern "C" int qg_lowrank_adam_many(int count, const void* plan_host, const void* plan_dev, size_t plan_bytes,
                                    const qg_hparams* hp, int64_t step, void* stream) {
    if (int e = check_plan(count, plan_host, plan_dev, plan_bytes)) return e;
    if (!hp) return QG_ERR_NULL;
    if (step < 1) return QG_ERR_SHAPE;
    if (reinterpret_cast<const PlanHeader*>(plan_host)->no_R) return QG_ERR_NULL;   // needs every R buffer
    return launch_adam_many(reinterpret_cast<const PlanHeader*>(plan_host),
                            reinterpret_cast<const PlanHeader*>(plan_dev), step, hp, (hipStream_t)stream);
}

extern "C" int qg_backproject_update_sr_many(int count, const void* plan_host, const void* plan_dev,
                                             size_t plan_bytes, const qg_hparams* hp, uint64_t seed, int64_t step,
                                             void* stream) {
    if (int e = check_plan(count, plan_host, plan_dev, plan_bytes)) return e;
    if (!hp) return QG_ERR_NULL;
    if (step < 1) return QG_ERR_SHAPE;
    return launch_backproject_many(reinterpret_cast<const PlanHeader*>(plan_host),
                                   reinterpret_cast<const PlanHeader*>(plan_dev), hp->alpha, hp->lr, seed, step,
                                   (hipStream_t)stream);
}

extern "C" int qg_project_adam(const uint8_t* Pq, const float* Ps, const uint16_t* G_bf16, float* R, float* M,
                              float* V, uint16_t* N_bf16, int64_t m, int64_t n, int64_t r, int group, int64_t step,
                              const qg_hparams* hp, void* stream) {
    if (!Pq || !Ps || !G_bf16 || !M || !V || !N_bf16 || !hp) return QG_ERR_NULL;
    if (int e = check_mnr(m, n, r, group)) return e;
    if (step < 1) return QG_ERR_SHAPE;
    if (!aligned16(Pq) || !aligned16(Ps) || !aligned16(G_bf16) || (R && !aligned16(R)) || !aligned16(M) ||
        !aligned16(V) || !aligned16(N_bf16))
        return QG_ERR_ALIGN;
    return launch_project_adam(Pq, Ps, G_bf16, R, M, V, N_bf16, m, n, n, r, step, hp, (hipStream_t)stream);
}

extern "C" int qg_project_adam_many(int count, const void* plan_host, const void* plan_dev, size_t plan_bytes,
                                    const qg_hparams* hp, int64_t step, int write_R, void* stream) {
    if (int e = check_plan(count, plan_host, plan_dev, plan_bytes)) return e;
    if (!hp) return QG_ERR_NULL;
    if (step < 1) return QG_ERR_SHAPE;
    const PlanHeader* h = reinterpret_cast<const PlanHeader*>(plan_host);
    if (write_R && h->no_R) return QG_ERR_NULL;
    return launch_project_adam_many(h, reinterpret_cast<const PlanHeader*>(plan_dev), write_R ? 1 : 0, step, hp,
                                    (hipStream_t)stream);
}

extern "C" int qg_step_many(int count, const void* plan_host, const void* plan_dev, size_t plan_bytes,
                            const qg_hparams* hp, uint64_t seed, int64_t step, void* stream) {
    if (int e = check_plan(count, plan_host, plan_dev, plan_bytes)) return e;
    // R is written only if every descriptor supplies a buffer for it
    const int write_R = reinterpret_cast<const PlanHeader*>(plan_host)->no_R ? 0 : 1;
    if (int e = qg_project_adam_many(count, plan_host, plan_dev, plan_bytes, hp, step, write_R, stream)) return e;
    return qg_backproject_update_sr_many(count, plan_host, plan_dev, plan_bytes, hp, seed, step, stream);
}
