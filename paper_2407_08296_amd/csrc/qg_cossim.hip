// Subspace convergence check (Sec. 3.2, Fig. 2): mean over the r columns of the
// cosine between corresponding columns of two INT4 projection matrices.
// Deterministic: per-row-chunk partial sums, then per-column cosines and their mean, all in fixed orders.
#include <atomic>

#include "qg_common.h"
#include "qg_cossim.h"

namespace qg {

constexpr int kCosRows = 64;  // rows per partial-sum chunk

// Up to kCosBatchMax pairs of one shape per launch (gridDim.y of them), pointers by value (CosBatch); pair z uses the
// workspace slice at z * ws_stride floats and writes cos_out[z].
// partial[chunk][3][r]: dot, |a|^2, |b|^2 of each column over the chunk's rows.
__global__ __launch_bounds__(256) void k_cossim_partial(CosBatch batch, int m, int r, int wpr, int lanes_rows, int chunks,
                                                        float* __restrict__ partial, int64_t ws_stride) {
    const uint8_t* __restrict__ PqA = batch.PqA[blockIdx.y];
    const float* __restrict__ PsA = batch.PsA[blockIdx.y];
    const uint8_t* __restrict__ PqB = batch.PqB[blockIdx.y];
    const float* __restrict__ PsB = batch.PsB[blockIdx.y];
    partial += ws_stride * blockIdx.y;
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

// Columns of one 64-wide group per workgroup: four threads per column add the chunks' partial sums (thread p takes
// chunks p, p + 4, ...), the four are combined in a fixed order, the column's cosine is formed and the group's 64
// cosines are added by a fixed tree -> group_sum[blockIdx.x].
constexpr int kCosGroup = 64;

// With `weights` (one float per column, batch entry z at weights + z * w_stride) the column cosines are weighted:
// group_sum holds sum w_k cos_k and group_sum[groups + g] the weights' sum of group g.
__global__ __launch_bounds__(256) void k_cossim_columns(const float* __restrict__ partial, int r, int chunks,
                                                        float* __restrict__ group_sum, int64_t ws_stride,
                                                        const float* __restrict__ weights, int64_t w_stride) {
    partial += ws_stride * blockIdx.y;
    group_sum += ws_stride * blockIdx.y;
    if (weights != nullptr) weights += w_stride * blockIdx.y;
    __shared__ float sh[3][4][kCosGroup];
    __shared__ float cosv[kCosGroup];
    __shared__ float wv[kCosGroup];
    const int t = threadIdx.x, cl = t & 63, part = t >> 6;
    const int k = blockIdx.x * kCosGroup + cl;
    float dot = 0.f, na = 0.f, nb = 0.f;
    if (k < r) {
#pragma unroll 4
        for (int c = part; c < chunks; c += 4) {
            const float* p = partial + (int64_t)c * 3 * r + k;
            dot += p[0];
            na += p[r];
            nb += p[2 * r];
        }
    }
    sh[0][part][cl] = dot;
    sh[1][part][cl] = na;
    sh[2][part][cl] = nb;
    __syncthreads();
    if (part == 0) {
        float v[3];
#pragma unroll
        for (int q = 0; q < 3; ++q) v[q] = ((sh[q][0][cl] + sh[q][1][cl]) + sh[q][2][cl]) + sh[q][3][cl];
        const float c = k < r ? v[0] / fmaxf(sqrtf(v[1]) * sqrtf(v[2]), 1e-8f) : 0.f;
        const float w = (weights != nullptr && k < r) ? weights[k] : 1.f;
        cosv[cl] = weights != nullptr ? w * c : c;
        wv[cl] = k < r ? w : 0.f;
    }
    __syncthreads();
    for (int s = kCosGroup / 2; s > 0; s >>= 1) {
        if (t < s) {
            cosv[t] += cosv[t + s];
            wv[t] += wv[t + s];
        }
        __syncthreads();
    }
    if (t == 0) {
        group_sum[blockIdx.x] = cosv[0];
        group_sum[gridDim.x + blockIdx.x] = wv[0];
    }
}

// cos_out = sum of the groups' (weighted) cosine sums over the sum of the weights (r when unweighted).
__global__ void k_cossim_mean(const float* __restrict__ group_sum, int groups, int r, float* __restrict__ cos_out,
                              int64_t ws_stride, int weighted) {
    group_sum += ws_stride * blockIdx.x;
    float acc = 0.f, wsum = 0.f;
    for (int g = 0; g < groups; ++g) {
        acc += group_sum[g];
        wsum += group_sum[groups + g];
    }
    cos_out[blockIdx.x] = weighted ? (wsum > 0.f ? acc / wsum : 0.f) : acc / (float)r;
}

static size_t cossim_ws_floats(int64_t m, int64_t r) {
    const int64_t chunks = (m + kCosRows - 1) / kCosRows;
    const int64_t groups = (r + kCosGroup - 1) / kCosGroup;
    return (size_t)((chunks * 3 * r + 2 * groups + 63) / 64 * 64);   // partial sums, then two sums per column group; padded
}

// `count` <= kCosBatchMax pairs; workspace: count slices of cossim_ws_floats(m, r) floats.
int launch_cossim_batch(const CosBatch& batch, int count, int64_t m, int64_t r, float* cos_out, float* ws,
                        hipStream_t stream, const float* weights, int64_t w_stride) {
    const int W = (int)(r >> 3);
    const int wpr = W < 256 ? W : 256;
    const int lanes_rows = 256 / wpr;
    const int chunks = (int)((m + kCosRows - 1) / kCosRows);
    const int blocks = (chunks + lanes_rows - 1) / lanes_rows;
    const int64_t stride = (int64_t)cossim_ws_floats(m, r);
    hipLaunchKernelGGL(k_cossim_partial, dim3(blocks, count), dim3(256), 0, stream, batch, (int)m, (int)r, wpr, lanes_rows,
                       chunks, ws, stride);
    if (int e = check_launch()) return e;
    const int groups = (int)((r + kCosGroup - 1) / kCosGroup);
    float* group_sum = ws + (int64_t)chunks * 3 * r;
    hipLaunchKernelGGL(k_cossim_columns, dim3(groups, count), dim3(256), 0, stream, (const float*)ws, (int)r, chunks,
                       group_sum, stride, weights, w_stride);
    hipLaunchKernelGGL(k_cossim_mean, dim3(count), dim3(1), 0, stream, (const float*)group_sum, groups, (int)r, cos_out,
                       stride, weights != nullptr ? 1 : 0);
    return check_launch();
}

size_t cossim_batch_workspace_bytes(int64_t m, int64_t r, int count) { return cossim_ws_floats(m, r) * 4 * (size_t)count; }

}  // namespace qg

using namespace qg;

extern "C" size_t qg_cossim_workspace_bytes(int64_t m, int64_t r) {
    if (m <= 0 || r <= 0) return 0;
    const int64_t chunks = (m + kCosRows - 1) / kCosRows;
    const int64_t groups = (r + kCosGroup - 1) / kCosGroup;
    return (size_t)((chunks * 3 * r + 2 * groups) * (int64_t)sizeof(float));   // partial sums, then two sums per column group
}

extern "C" int qg_subspace_cossim_weighted(const uint8_t* PqA, const float* PsA, const uint8_t* PqB, const float* PsB,
                                           const float* weights, int64_t m, int64_t r, int group, float* cos_out,
                                           void* workspace, size_t workspace_bytes, void* stream);

extern "C" int qg_subspace_cossim(const uint8_t* PqA, const float* PsA, const uint8_t* PqB, const float* PsB, int64_t m,
                                  int64_t r, int group, float* cos_out, void* workspace, size_t workspace_bytes,
                                  void* stream) {
    return qg_subspace_cossim_weighted(PqA, PsA, PqB, PsB, nullptr, m, r, group, cos_out, workspace, workspace_bytes, stream);
}

extern "C" int qg_subspace_cossim_weighted(const uint8_t* PqA, const float* PsA, const uint8_t* PqB, const float* PsB,
                                           const float* weights, int64_t m, int64_t r, int group, float* cos_out,
                                           void* workspace, size_t workspace_bytes, void* stream) {
    if (!PqA || !PsA || !PqB || !PsB || !cos_out) return QG_ERR_NULL;
    if (weights && (reinterpret_cast<uintptr_t>(weights) & 3u) != 0) return QG_ERR_ALIGN;
    if (m <= 0 || r <= 0 || (r & 7) || r > m || m * r >= (int64_t(1) << 32)) return QG_ERR_SHAPE;
    if (group != kGroup) return QG_ERR_GROUP;
    if (!aligned16(PqA) || !aligned16(PsA) || !aligned16(PqB) || !aligned16(PsB)) return QG_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(cos_out) & 3u) != 0) return QG_ERR_ALIGN;
    if (!workspace || workspace_bytes < qg_cossim_workspace_bytes(m, r) || !aligned16(workspace))
        return QG_ERR_WORKSPACE;
    CosBatch batch;
    for (int i = 0; i < kCosBatchMax; ++i) {
        batch.PqA[i] = PqA; batch.PsA[i] = PsA; batch.PqB[i] = PqB; batch.PsB[i] = PsB;
    }
    return launch_cossim_batch(batch, 1, m, r, cos_out, (float*)workspace, (hipStream_t)stream, weights, 0);
}

// ---- The same check for callers that may not allocate: the partial sums live in a file-scope device array.
// Every device that loads the library holds its own copy of the array at its own address; the address is looked up
// once per device (hipGetSymbolAddress, with that device current) and only that pointer is ever handed to kernels.
namespace qg {
constexpr size_t kStaticScratchFloats = size_t(1) << 20;   // 4 MiB per device
static __device__ __align__(256) float scratch[kStaticScratchFloats];
constexpr int kMaxDevices = 64;
static std::atomic<float*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (nullptr + QG_ERR_HIP on failure).
static int static_scratch(float** out) {
    int devid = -1;
    hipError_t e = hipGetDevice(&devid);
    if (e != hipSuccess || devid < 0 || devid >= kMaxDevices) {
        set_hip_error(e != hipSuccess ? e : hipErrorInvalidDevice);
        return QG_ERR_HIP;
    }
    float* p = g_scratch_ptr[devid].load(std::memory_order_acquire);
    if (p == nullptr) {
        void* sym = nullptr;
        e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
        if (e != hipSuccess || sym == nullptr) {
            set_hip_error(e != hipSuccess ? e : hipErrorInvalidSymbol);
            return QG_ERR_HIP;
        }
        p = static_cast<float*>(sym);
        g_scratch_ptr[devid].store(p, std::memory_order_release);   // racing first calls store the same address
    }
    *out = p;
    return QG_OK;
}
}  // namespace qg

extern "C" int qg_subspace_cossim_static(const uint8_t* PqA, const float* PsA, const uint8_t* PqB, const float* PsB,
                                         int64_t m, int64_t r, int group, float* cos_out, void* stream) {
    if (!PqA || !PsA || !PqB || !PsB || !cos_out) return QG_ERR_NULL;
    if (m <= 0 || r <= 0 || (r & 7) || r > m || m * r >= (int64_t(1) << 32)) return QG_ERR_SHAPE;
    if (group != kGroup) return QG_ERR_GROUP;
    if (!aligned16(PqA) || !aligned16(PsA) || !aligned16(PqB) || !aligned16(PsB)) return QG_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(cos_out) & 3u) != 0) return QG_ERR_ALIGN;
    if (qg_cossim_workspace_bytes(m, r) > kStaticScratchFloats * sizeof(float)) return QG_ERR_WORKSPACE;
    float* ws = nullptr;
    if (int e = static_scratch(&ws)) return e;
    CosBatch batch;
    for (int i = 0; i < kCosBatchMax; ++i) {
        batch.PqA[i] = PqA; batch.PsA[i] = PsA; batch.PqB[i] = PqB; batch.PsB[i] = PsB;
    }
    // every partial sum the later kernels read is written by the first one: nothing has to start at zero
    return launch_cossim_batch(batch, 1, m, r, cos_out, ws, (hipStream_t)stream, nullptr, 0);
}
