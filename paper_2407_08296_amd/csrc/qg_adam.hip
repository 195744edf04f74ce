// Adam on the low-rank gradient (Sec. 3.5; Adam as cited in Sec. 4.1).
// Element-wise and HBM-bound: 22 B per element (R read; M, V read+write; N bf16 write).
#include "qg_common.h"
#include <cmath>

#include "qg_plan.h"

namespace qg {

constexpr int kAdamVec = 4;                              // float4 per thread per array
constexpr int kAdamChunk = 256 * 4 * kAdamVec;           // elements per workgroup chunk

// One chunk of kAdamChunk elements starting at `base` (multiple of 4) of one matrix.
__device__ inline void adam_chunk(const float* __restrict__ R, float* __restrict__ M, float* __restrict__ V,
                                  uint16_t* __restrict__ N, int64_t count, int64_t base, const AdamCoef& c) {
    const int t = threadIdx.x;
    if (base + kAdamChunk <= count) {
        // every access is streaming (nothing here is re-read before it has left the caches): non-temporal loads and
        // stores throughout, one array at a time
        f32x4 r[kAdamVec], m[kAdamVec], v[kAdamVec];
#pragma unroll
        for (int k = 0; k < kAdamVec; ++k)
            r[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(R + base + (int64_t)(k * 256 + t) * 4));
#pragma unroll
        for (int k = 0; k < kAdamVec; ++k)
            m[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(M + base + (int64_t)(k * 256 + t) * 4));
#pragma unroll
        for (int k = 0; k < kAdamVec; ++k)
            v[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(V + base + (int64_t)(k * 256 + t) * 4));
#pragma unroll
        for (int k = 0; k < kAdamVec; ++k) {
            const int64_t e = base + (int64_t)(k * 256 + t) * 4;
            float nn[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float mj = m[k][j], vj = v[k][j];
                nn[j] = adam_one(r[k][j], mj, vj, c);
                m[k][j] = mj;
                v[k][j] = vj;
            }
            __builtin_nontemporal_store(m[k], reinterpret_cast<f32x4*>(M + e));
            __builtin_nontemporal_store(v[k], reinterpret_cast<f32x4*>(V + e));
            typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
            const u32x2 nb = {pack_bf16x2(nn[0], nn[1]), pack_bf16x2(nn[2], nn[3])};
            __builtin_nontemporal_store(nb, reinterpret_cast<u32x2*>(N + e));
        }
    } else {
        for (int64_t e = base + t; e < count && e < base + kAdamChunk; e += 256) {
            float m = M[e], v = V[e];
            const float nv = adam_one(R[e], m, v, c);
            M[e] = m;
            V[e] = v;
            N[e] = to_bf16(nv);
        }
    }
}

__global__ __launch_bounds__(256) void k_lowrank_adam(const float* __restrict__ R, float* __restrict__ M,
                                                      float* __restrict__ V, uint16_t* __restrict__ N,
                                                      int64_t count, AdamCoef c) {
    adam_chunk(R, M, V, N, count, (int64_t)blockIdx.x * kAdamChunk, c);
}

// Grouped: block b works on chunk (b - chunk_prefix[i]) of matrix i.
__global__ __launch_bounds__(256) void k_lowrank_adam_many(const PlanHeader* __restrict__ plan, AdamCoef c) {
    const PlanMatrix* mats = plan_matrices(plan);
    int lo = 0, hi = plan->count - 1;
    const uint32_t b = blockIdx.x;
    while (lo < hi) {                       // last matrix whose first chunk is <= b
        const int mid = (lo + hi + 1) >> 1;
        if (mats[mid].adam_chunk0 <= b) lo = mid; else hi = mid - 1;
    }
    const PlanMatrix& d = mats[lo];
    adam_chunk(d.R, d.M, d.V, d.N, d.r * d.ld, (int64_t)(b - d.adam_chunk0) * kAdamChunk, c);   // padding included
}

AdamCoef make_adam_coef(const qg_hparams* hp, int64_t step) {
    AdamCoef c;
    c.b1 = hp->beta1;
    c.b2 = hp->beta2;
    c.omb1 = 1.0f - hp->beta1;
    c.omb2 = 1.0f - hp->beta2;
    c.rc1 = (float)(1.0 / (1.0 - pow((double)hp->beta1, (double)step)));
    c.rc2 = (float)(1.0 / (1.0 - pow((double)hp->beta2, (double)step)));
    c.eps = hp->eps;
    c.sqrt_rc2 = (float)sqrt(1.0 / (1.0 - pow((double)hp->beta2, (double)step)));
    return c;
}

int launch_adam(const float* R, float* M, float* V, uint16_t* N, int64_t count, int64_t step, const qg_hparams* hp,
                hipStream_t stream) {
    const int64_t blocks = (count + kAdamChunk - 1) / kAdamChunk;
    hipLaunchKernelGGL(k_lowrank_adam, dim3((unsigned)blocks), dim3(256), 0, stream, R, M, V, N, count,
                       make_adam_coef(hp, step));
    return check_launch();
}

int launch_adam_many(const PlanHeader* plan_host, const PlanHeader* plan_dev, int64_t step, const qg_hparams* hp,
                     hipStream_t stream) {
    hipLaunchKernelGGL(k_lowrank_adam_many, dim3(plan_host->adam_chunks), dim3(256), 0, stream, plan_dev,
                       make_adam_coef(hp, step));
    return check_launch();
}

}  // namespace qg

using namespace qg;

extern "C" int qg_lowrank_adam(const float* R, float* M, float* V, uint16_t* N_bf16, int64_t count, int64_t step,
                               const qg_hparams* hp, void* stream) {
    if (!R || !M || !V || !N_bf16 || !hp) return QG_ERR_NULL;
    if (count <= 0 || step < 1 || count > (int64_t(1) << 40)) return QG_ERR_SHAPE;
    if (!aligned16(R) || !aligned16(M) || !aligned16(V) || !aligned16(N_bf16)) return QG_ERR_ALIGN;
    return launch_adam(R, M, V, N_bf16, count, step, hp, (hipStream_t)stream);
}
