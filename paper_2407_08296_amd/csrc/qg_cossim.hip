// Subspace convergence check (Sec. 3.2, Fig. 2): mean over the r columns of the
// cosine between corresponding columns of two INT4 projection matrices.
// Two deterministic passes: per-row-chunk partial sums, then a fixed-order finish.
#include "qg_common.h"

namespace qg {

constexpr int kCosRows = 64;  // rows per partial-sum chunk

// partial[chunk][3][r]: dot, |a|^2, |b|^2 of each column over the chunk's rows.
__global__ __launch_bounds__(256) void k_cossim_partial(const uint8_t* __restrict__ PqA, const float* __restrict__ PsA,
                                                        const uint8_t* __restrict__ PqB, const float* __restrict__ PsB,
                                                        int m, int r, int wpr, int lanes_rows, int chunks,
                                                        float* __restrict__ partial) {
    const int t = threadIdx.x;
    const int rl = t / wpr, wc0 = t % wpr;
    if (rl >= lanes_rows) return;
    const int chunk = blockIdx.x * lanes_rows + rl;
    if (chunk >= chunks) return;
    const int W = r >> 3;
    const int i0 = chunk * kCosRows, i1 = min(m, i0 + kCosRows);
    for (int wc = wc0; wc < W; wc += wpr) {
        float dot[8], na[8], nb[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) dot[j] = na[j] = nb[j] = 0.f;
        for (int i = i0; i < i1; ++i) {
            const int64_t e = (int64_t)i * r + wc * 8;
            const uint32_t wa = *reinterpret_cast<const uint32_t*>(PqA + (e >> 1));
            const uint32_t wb = *reinterpret_cast<const uint32_t*>(PqB + (e >> 1));
            const float sa = PsA[e >> 8], sb = PsB[e >> 8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float a = (float)((int)((wa >> (4 * j)) & 0xFu) - 8) * sa;
                const float b = (float)((int)((wb >> (4 * j)) & 0xFu) - 8) * sb;
                dot[j] = __builtin_fmaf(a, b, dot[j]);
                na[j] = __builtin_fmaf(a, a, na[j]);
                nb[j] = __builtin_fmaf(b, b, nb[j]);
            }
        }
        float* out = partial + (int64_t)chunk * 3 * r + wc * 8;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            out[j] = dot[j];
            out[r + j] = na[j];
            out[2 * r + j] = nb[j];
        }
    }
}

__global__ __launch_bounds__(256) void k_cossim_finish(const float* __restrict__ partial, int r, int chunks,
                                                       float* __restrict__ cos_out) {
    __shared__ float red[256];
    const int t = threadIdx.x;
    float acc = 0.f;
    for (int k = t; k < r; k += 256) {
        float dot = 0.f, na = 0.f, nb = 0.f;
        for (int c = 0; c < chunks; ++c) {
            const float* p = partial + (int64_t)c * 3 * r + k;
            dot += p[0];
            na += p[r];
            nb += p[2 * r];
        }
        acc += dot / fmaxf(sqrtf(na) * sqrtf(nb), 1e-8f);
    }
    red[t] = acc;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (t < s) red[t] += red[t + s];
        __syncthreads();
    }
    if (t == 0) cos_out[0] = red[0] / (float)r;
}

}  // namespace qg

using namespace qg;

extern "C" size_t qg_cossim_workspace_bytes(int64_t m, int64_t r) {
    if (m <= 0 || r <= 0) return 0;
    const int64_t chunks = (m + kCosRows - 1) / kCosRows;
    return (size_t)(chunks * 3 * r * (int64_t)sizeof(float));
}

extern "C" int qg_subspace_cossim(const uint8_t* PqA, const float* PsA, const uint8_t* PqB, const float* PsB, int64_t m,
                                  int64_t r, int group, float* cos_out, void* workspace, size_t workspace_bytes,
                                  void* stream) {
    if (!PqA || !PsA || !PqB || !PsB || !cos_out) return QG_ERR_NULL;
    if (m <= 0 || r <= 0 || (r & 7) || r > m || m * r >= (int64_t(1) << 32)) return QG_ERR_SHAPE;
    if (group != kGroup) return QG_ERR_GROUP;
    if (!aligned16(PqA) || !aligned16(PsA) || !aligned16(PqB) || !aligned16(PsB)) return QG_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(cos_out) & 3u) != 0) return QG_ERR_ALIGN;
    if (!workspace || workspace_bytes < qg_cossim_workspace_bytes(m, r) || !aligned16(workspace))
        return QG_ERR_WORKSPACE;
    const int W = (int)(r >> 3);
    const int wpr = W < 256 ? W : 256;
    const int lanes_rows = 256 / wpr;
    const int chunks = (int)((m + kCosRows - 1) / kCosRows);
    const int blocks = (chunks + lanes_rows - 1) / lanes_rows;
    hipLaunchKernelGGL(k_cossim_partial, dim3(blocks), dim3(256), 0, (hipStream_t)stream, PqA, PsA, PqB, PsB, (int)m,
                       (int)r, wpr, lanes_rows, chunks, (float*)workspace);
    if (int e = check_launch()) return e;
    hipLaunchKernelGGL(k_cossim_finish, dim3(1), dim3(256), 0, (hipStream_t)stream, (const float*)workspace, (int)r,
                       chunks, cos_out);
    return check_launch();
}
