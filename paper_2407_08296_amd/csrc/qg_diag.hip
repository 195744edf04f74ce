// Measurement helpers: what the machine sustains while the step's kernels run (shader clock) and the ceilings the
// roofline fractions are read against (a register-only MFMA loop).  Not part of the method.
#include "qg_common.h"

namespace qg {
int check_launch();

// One wave spins until `ticks` of the constant 100 MHz counter have passed and reports how many shader clock cycles
// went by in that time; launched on a second stream beside the kernel under test.  The loop always ends: the counter
// is free-running and `ticks` is capped by the caller.
__global__ void k_clock_probe(long long ticks, long long* out) {
    const long long c0 = clock64(), w0 = wall_clock64();
    long long w = w0;
    while (w - w0 < ticks) {
        __builtin_amdgcn_s_sleep(32);
        w = wall_clock64();
    }
    if (threadIdx.x == 0) {
        out[0] = clock64() - c0;
        out[1] = w - w0;
    }
}

// 8 waves per workgroup (two per SIMD), each issuing `iters` rounds of 16 independent v_mfma_f32_32x32x16_bf16 on
// register operands: the matrix pipe with nothing else to do.  RANDOM fills the operands with varied finite bit
// patterns (data-dependent power draw lowers the clock the chip sustains); otherwise small constants.
template <bool RANDOM>
__global__ __launch_bounds__(512) void k_mfma_loop(long long iters, float* sink) {
    f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    bf16x8 a[2], b[4];
    uint32_t h = mix32(threadIdx.x * 2654435761u + blockIdx.x);
#pragma unroll
    for (int q = 0; q < 6; ++q) {
        u32x4 w;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            h = mix32(h + 0x9E3779B9u);
            // two bf16 in [-2, 2): sign and mantissa random, exponent 0x3F80 or below
            const uint32_t lo = RANDOM ? ((h & 0x807Fu) | 0x3F00u) : 0x3C00u;
            const uint32_t hi = RANDOM ? (((h >> 16) & 0x807Fu) | 0x3F00u) : 0x3C00u;
            w[j] = lo | (hi << 16);
        }
        if (q < 2) a[q] = __builtin_bit_cast(bf16x8, w); else b[q - 2] = __builtin_bit_cast(bf16x8, w);
    }
    for (long long it = 0; it < iters; ++it) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int i = 0; i < 8; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i >> 2], b[i & 3], acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    sink[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// The same for the fp64 matrix cores: rounds of 8 independent v_mfma_f64_16x16x4 on register operands, 256-thread
// workgroups (the shape of the refresh's fp64 kernels; three of them per CU are resident there).
typedef double diag_f64x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void k_mfma_f64_loop(long long iters, float* sink) {
    diag_f64x4 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = diag_f64x4{0.0, 0.0, 0.0, 0.0};
    const double a = 1.0 + threadIdx.x * 0x1p-10, b = 2.0 - threadIdx.x * 0x1p-10;
    for (long long it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[i], 0, 0, 0);
    }
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += (acc[i][0] + acc[i][1]) + (acc[i][2] + acc[i][3]);
    sink[blockIdx.x * blockDim.x + threadIdx.x] = (float)s;
}

}  // namespace qg

using namespace qg;

extern "C" int qg_diag_clock_probe(int64_t ticks_100mhz, int64_t* out2, void* stream) {
    if (!out2) return QG_ERR_NULL;
    if (ticks_100mhz < 1 || ticks_100mhz > 100000000) return QG_ERR_SHAPE;   // at most one second
    hipLaunchKernelGGL(k_clock_probe, dim3(1), dim3(64), 0, (hipStream_t)stream, (long long)ticks_100mhz,
                       reinterpret_cast<long long*>(out2));
    return check_launch();
}

extern "C" int qg_diag_mfma_loop(int64_t iters, int random_operands, float* sink, void* stream) {
    if (!sink) return QG_ERR_NULL;
    if (iters < 1 || iters > (int64_t(1) << 24)) return QG_ERR_SHAPE;
    if (random_operands)
        hipLaunchKernelGGL(k_mfma_loop<true>, dim3(QG_DIAG_MFMA_WORKGROUPS), dim3(512), 0, (hipStream_t)stream,
                           (long long)iters, sink);
    else
        hipLaunchKernelGGL(k_mfma_loop<false>, dim3(QG_DIAG_MFMA_WORKGROUPS), dim3(512), 0, (hipStream_t)stream,
                           (long long)iters, sink);
    return check_launch();
}

extern "C" int qg_diag_mfma_f64_loop(int64_t iters, int workgroups, float* sink, void* stream) {
    if (!sink) return QG_ERR_NULL;
    if (iters < 1 || iters > (int64_t(1) << 24) || workgroups < 1 || workgroups > 65536) return QG_ERR_SHAPE;
    hipLaunchKernelGGL(k_mfma_f64_loop, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)stream, (long long)iters, sink);
    return check_launch();
}
