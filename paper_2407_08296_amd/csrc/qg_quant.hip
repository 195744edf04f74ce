// Block-wise uniform quantization Quant_n (Sec. 3.1) and its inverse (Appendix A,
// zeros = 0), plus the test helper that exposes the SR generator's draws.
#include "qg_common.h"

namespace qg {

// One wave per block of 256 elements; each lane owns 4 consecutive elements.
// INT8: blocks live inside a row (row-major [rows][cols], short last block).
// ZP: the quantizer with a zero point (Sec. 3.1 eq.): range [min(0, min x), max(0, max x)] over 255 steps,
// z = -128 - round(lo / s), code = clamp(round(x / s) + z).
template <bool ZP>
__global__ __launch_bounds__(256) void k_quant_int8(const float* __restrict__ x, int64_t rows, int64_t cols,
                                                    int64_t ng, int8_t* __restrict__ q,
                                                    float* __restrict__ scales, float* __restrict__ zeros) {
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wave >= rows * ng) return;
    const int lane = threadIdx.x & 63;
    const int64_t row = wave / ng, g = wave % ng;
    const int64_t c0 = g * kGroup + 4 * lane;
    const float* xr = x + row * cols;
    const bool vec = (cols & 3) == 0;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    if (vec) {
        if (c0 < cols) {
            const float4 t = *reinterpret_cast<const float4*>(xr + c0);
            v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (c0 + j < cols) v[j] = xr[c0 + j];
    }
    float s, inv, z = 0.f;
    if constexpr (ZP) {
        // elements past the row's end hold 0, which the range contains anyway
        const float hi = wave_max(fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), 0.f));
        const float lo = -wave_max(fmaxf(fmaxf(fmaxf(-v[0], -v[1]), fmaxf(-v[2], -v[3])), 0.f));
        const float rng = hi - lo;
        s = rng > 0.f ? rng / 255.0f : 0.f;
        inv = rng > 0.f ? 255.0f / rng : 0.f;
        z = rng > 0.f ? fminf(fmaxf(-128.f - rintf(lo * inv), -128.f), 127.f) : 0.f;
        if (lane == 0) zeros[row * ng + g] = z;
    } else {
        float a = fmaxf(fmaxf(fabsf(v[0]), fabsf(v[1])), fmaxf(fabsf(v[2]), fabsf(v[3])));
        a = wave_max(a);
        s = a > 0.f ? a / 127.0f : 0.f;
        inv = a > 0.f ? 127.0f / a : 0.f;
    }
    if (lane == 0) scales[row * ng + g] = s;
    int c[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) c[j] = (int)fminf(fmaxf(rintf(v[j] * inv) + z, -128.f), 127.f);
    int8_t* qr = q + row * cols;
    if (vec) {
        if (c0 < cols) {
            const uint32_t pk = (uint32_t)(c[0] & 0xFF) | ((uint32_t)(c[1] & 0xFF) << 8) |
                                ((uint32_t)(c[2] & 0xFF) << 16) | ((uint32_t)(c[3] & 0xFF) << 24);
            *reinterpret_cast<uint32_t*>(qr + c0) = pk;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (c0 + j < cols) qr[c0 + j] = (int8_t)c[j];
    }
}

// INT4: blocks of 256 of the flattened array; nibble = code + 8, two per byte.
__global__ __launch_bounds__(256) void k_quant_int4(const float* __restrict__ x, int64_t total, int64_t nblocks,
                                                    uint8_t* __restrict__ q, float* __restrict__ scales) {
    const int64_t blk = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (blk >= nblocks) return;
    const int lane = threadIdx.x & 63;
    const int64_t e0 = blk * kGroup + 4 * lane;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    if (e0 + 3 < total) {
        const float4 t = *reinterpret_cast<const float4*>(x + e0);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (e0 + j < total) v[j] = x[e0 + j];
    }
    float a = fmaxf(fmaxf(fabsf(v[0]), fabsf(v[1])), fmaxf(fabsf(v[2]), fabsf(v[3])));
    a = wave_max(a);
    const float s = a > 0.f ? a / 7.0f : 0.f;
    const float inv = a > 0.f ? 7.0f / a : 0.f;
    if (lane == 0) scales[blk] = s;
    uint32_t nib[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) nib[j] = (uint32_t)((int)fminf(fmaxf(rintf(v[j] * inv), -8.f), 7.f) + 8);
    const uint32_t b0 = nib[0] | (nib[1] << 4), b1 = nib[2] | (nib[3] << 4);
    if (e0 + 3 < total) {
        *reinterpret_cast<uint16_t*>(q + (e0 >> 1)) = (uint16_t)(b0 | (b1 << 8));
    } else {
        if (e0 < total) q[e0 >> 1] = (uint8_t)b0;
        if (e0 + 2 < total) q[(e0 >> 1) + 1] = (uint8_t)b1;
    }
}

__global__ __launch_bounds__(256) void k_dequant_int8(const int8_t* __restrict__ q, const float* __restrict__ scales,
                                                      const float* __restrict__ zeros, int64_t rows, int64_t cols,
                                                      int64_t ng, float* __restrict__ x) {
    const int64_t total = rows * cols;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = e / cols, c = e % cols;
        const float z = zeros != nullptr ? zeros[row * ng + c / kGroup] : 0.f;
        x[e] = ((float)q[e] - z) * scales[row * ng + c / kGroup];
    }
}

__global__ __launch_bounds__(256) void k_dequant_int4(const uint8_t* __restrict__ q, const float* __restrict__ scales,
                                                      int64_t total, float* __restrict__ x) {
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t byte = q[e >> 1];
        const int code = (int)((e & 1) ? (byte >> 4) : (byte & 0xFu)) - 8;
        x[e] = (float)code * scales[e / kGroup];
    }
}

__global__ __launch_bounds__(256) void k_sr_uniform(uint32_t key_lo, uint64_t seed, uint64_t step, uint64_t idx0,
                                                    int64_t count, float* __restrict__ out) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x) {
        const uint64_t idx = idx0 + (uint64_t)i;
        const uint32_t hi = (uint32_t)(idx >> 32);
        const uint32_t key = hi == 0 ? key_lo : sr_key(seed, step, hi);
        out[i] = sr_uniform(key, (uint32_t)idx);
    }
}

static inline unsigned grid_for(int64_t work_items, int per_block, int64_t cap = 1 << 20) {
    int64_t g = (work_items + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (unsigned)g;
}

}  // namespace qg

using namespace qg;

static int check_quant_args(const void* a, const void* b, const void* c, int64_t rows, int64_t cols, int group) {
    if (!a || !b || !c) return QG_ERR_NULL;
    if (rows <= 0 || cols <= 0 || rows > (int64_t(1) << 40) / cols) return QG_ERR_SHAPE;
    if (group != kGroup) return QG_ERR_GROUP;
    if (!aligned16(a) || !aligned16(b) || !aligned16(c)) return QG_ERR_ALIGN;
    return QG_OK;
}

extern "C" int qg_quant_int8(const float* x, int64_t rows, int64_t cols, int group, int8_t* q, float* scales,
                             void* stream) {
    if (int e = check_quant_args(x, q, scales, rows, cols, group)) return e;
    const int64_t ng = (cols + kGroup - 1) / kGroup;
    const int64_t waves = rows * ng;
    if ((waves + 3) / 4 > 0x7FFFFFFF) return QG_ERR_SHAPE;
    hipLaunchKernelGGL(k_quant_int8<false>, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, (hipStream_t)stream, x, rows,
                       cols, ng, q, scales, (float*)nullptr);
    return check_launch();
}

extern "C" int qg_quant_int8_zp(const float* x, int64_t rows, int64_t cols, int group, int8_t* q, float* scales,
                                float* zeros, void* stream) {
    if (!zeros) return QG_ERR_NULL;
    if (int e = check_quant_args(x, q, scales, rows, cols, group)) return e;
    if (!aligned16(zeros)) return QG_ERR_ALIGN;
    const int64_t ng = (cols + kGroup - 1) / kGroup;
    const int64_t waves = rows * ng;
    if ((waves + 3) / 4 > 0x7FFFFFFF) return QG_ERR_SHAPE;
    hipLaunchKernelGGL(k_quant_int8<true>, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, (hipStream_t)stream, x, rows,
                       cols, ng, q, scales, zeros);
    return check_launch();
}

extern "C" int qg_dequant_int8_zp(const int8_t* q, const float* scales, const float* zeros, int64_t rows, int64_t cols,
                                  int group, float* x, void* stream) {
    if (!zeros) return QG_ERR_NULL;
    if (int e = check_quant_args(q, scales, x, rows, cols, group)) return e;
    if (!aligned16(zeros)) return QG_ERR_ALIGN;
    const int64_t ng = (cols + kGroup - 1) / kGroup;
    hipLaunchKernelGGL(k_dequant_int8, dim3(grid_for(rows * cols, 256, 65536)), dim3(256), 0, (hipStream_t)stream, q,
                       scales, zeros, rows, cols, ng, x);
    return check_launch();
}

extern "C" int qg_quant_int4(const float* x, int64_t rows, int64_t cols, int group, uint8_t* q_packed, float* scales,
                             void* stream) {
    if (int e = check_quant_args(x, q_packed, scales, rows, cols, group)) return e;
    const int64_t total = rows * cols;
    const int64_t nblocks = (total + kGroup - 1) / kGroup;
    if ((nblocks + 3) / 4 > 0x7FFFFFFF) return QG_ERR_SHAPE;
    hipLaunchKernelGGL(k_quant_int4, dim3((unsigned)((nblocks + 3) / 4)), dim3(256), 0, (hipStream_t)stream, x, total,
                       nblocks, q_packed, scales);
    return check_launch();
}

extern "C" int qg_dequant_int8(const int8_t* q, const float* scales, int64_t rows, int64_t cols, int group, float* x,
                               void* stream) {
    if (int e = check_quant_args(q, scales, x, rows, cols, group)) return e;
    const int64_t ng = (cols + kGroup - 1) / kGroup;
    hipLaunchKernelGGL(k_dequant_int8, dim3(grid_for(rows * cols, 256, 65536)), dim3(256), 0, (hipStream_t)stream, q,
                       scales, (const float*)nullptr, rows, cols, ng, x);
    return check_launch();
}

extern "C" int qg_dequant_int4(const uint8_t* q_packed, const float* scales, int64_t rows, int64_t cols, int group,
                               float* x, void* stream) {
    if (int e = check_quant_args(q_packed, scales, x, rows, cols, group)) return e;
    hipLaunchKernelGGL(k_dequant_int4, dim3(grid_for(rows * cols, 256, 65536)), dim3(256), 0, (hipStream_t)stream,
                       q_packed, scales, rows * cols, x);
    return check_launch();
}

extern "C" int qg_sr_uniform(uint64_t seed, int64_t step, uint64_t idx0, int64_t count, float* out, void* stream) {
    if (!out) return QG_ERR_NULL;
    if (count <= 0) return QG_ERR_SHAPE;
    if (!aligned16(out)) return QG_ERR_ALIGN;
    const uint32_t key_lo = sr_key(seed, (uint64_t)step, 0u);
    hipLaunchKernelGGL(k_sr_uniform, dim3(grid_for(count, 256, 65536)), dim3(256), 0, (hipStream_t)stream, key_lo, seed,
                       (uint64_t)step, idx0, count, out);
    return check_launch();
}
