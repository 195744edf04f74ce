// Adam on the low-rank gradient with 8-bit states (Sec. 3.5: an 8-bit Adam is the inner optimizer).  The paper takes
// the state format from a third-party library and does not define it; this one is designed here after the published
// idea of block-wise dynamic quantization:
//   block   256 consecutive elements of the flattened r x n state, one fp32 scale = the block's absolute maximum
//   code    index of the entry nearest to x / scale (ties to the lower index) in a sorted table of 8-bit values with
//           relative resolution: entry p >= 1 of the unsigned table (second moment) has level L = floor(log2 p),
//           k = p - 2^L and value 10^-(7-L) * (0.1 + 0.9 (k+1) / 2^L), entry 0 is 0: 2^L values spaced linearly over
//           each decade from 1e-7 to 1.  The signed table (first moment) has levels 0..6 (1e-6 to 1): indices 0..126
//           the negatives from -1 up, 127 zero, 128..254 the positives; index 255 is not used.
// One step: states are dequantized (table[code] * scale), updated exactly like the fp32 states, and quantized again;
// 10 bytes of HBM traffic per element instead of 22.  A wave owns a block: a lane holds four consecutive elements,
// the block maximum is a wave reduction; the nearest entry is estimated arithmetically (the table is linear inside a
// decade) and settled against the four midpoints around the estimate in LDS.
#include "qg_common.h"

namespace qg {

typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kS8Block = kGroup;      // elements per block
constexpr int kS8SignedZero = 127;    // index of 0 in the signed table

struct S8Tables {
    float uval[256];    // unsigned table
    float umid[256];    // midpoints of neighbouring entries, padded with +inf
    float sval[256];    // signed table (255 entries, the last one repeated)
    float smid[256];
    float pw[8];        // 10^-j
    float ipw[8];       // 10^j
};

// Entry p >= 1 of the positive half of a table with levels 0..top.
__device__ inline double s8_positive(int p, int top) {
    const double pow10neg[8] = {1e0, 1e-1, 1e-2, 1e-3, 1e-4, 1e-5, 1e-6, 1e-7};
    const int L = 31 - __clz(p), k = p - (1 << L);
    return pow10neg[top - L] * (0.1 + 0.9 * (double)(k + 1) / (double)(1 << L));
}

// Every workgroup (256 threads) builds the tables from the definition; thread p makes entry p.
__device__ inline void s8_build(S8Tables& T) {
    const int p = threadIdx.x;
    T.uval[p] = p == 0 ? 0.f : (float)s8_positive(p, 7);
    float s;
    if (p < kS8SignedZero) s = -(float)s8_positive(kS8SignedZero - p, 6);
    else if (p == kS8SignedZero) s = 0.f;
    else s = (float)s8_positive((p < 255 ? p : 254) - kS8SignedZero, 6);
    T.sval[p] = s;
    if (p < 8) {
        const double pow10[8] = {1e0, 1e1, 1e2, 1e3, 1e4, 1e5, 1e6, 1e7};
        T.pw[p] = (float)(1.0 / pow10[p]);
        T.ipw[p] = (float)pow10[p];
    }
    __syncthreads();
    T.umid[p] = p < 255 ? (float)(0.5 * ((double)T.uval[p] + (double)T.uval[p + 1])) : INFINITY;
    T.smid[p] = p < 254 ? (float)(0.5 * ((double)T.sval[p] + (double)T.sval[p + 1])) : INFINITY;
    __syncthreads();
}

// Index, to within one entry, of the entry nearest to the magnitude ax >= 0 in the positive half of a table with
// levels 0..TOP (index 0 = the zero entry).  The decade comes from the binary exponent (floor(e2 log10 2), one low at
// most, put right by one comparison with the decade's top); inside a decade the entries are linear.  Checked on the
// host against a sorted search for every entry and midpoint +- 4 ulps and 10^7 random values: never off by more
// than one.
template <int TOP>
__device__ inline int s8_estimate(const S8Tables& T, float ax) {
    const int e2 = (int)(__builtin_bit_cast(uint32_t, ax) >> 23) - 127;
    int L = min(max(TOP + 1 + ((e2 * 1233) >> 12), 0), TOP);
    if (L < TOP && ax > T.pw[TOP - L]) ++L;
    const float t = ax * T.ipw[TOP - L];
    const float c = (float)(1 << L) * (1.0f / 0.9f);
    const int k = (int)rintf(t * c - 0.1f * c - 1.0f);
    return (1 << L) + min(max(k, -1), 1 << L);
}

// Index of the nearest table entry, ties to the lower index = the number of midpoints below x: the estimate is
// within one entry, so counting the four midpoints around it settles it exactly.
__device__ inline uint32_t s8_nearest4(const float* mid, int est, float x) {
    const float* m = mid + est - 2;
    return (uint32_t)(est - 2 + (m[0] < x) + (m[1] < x) + (m[2] < x) + (m[3] < x));
}

// Codes of the lane's four values of a block whose absolute maximum is amax; returns them packed, low byte first.
template <bool SIGNED>
__device__ inline uint32_t s8_encode4(const S8Tables& T, const float (&x)[4], float amax) {
    const float inv = amax > 0.f ? 1.0f / amax : 0.f;
    uint32_t pk = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float xn = x[j] * inv;
        uint32_t code;
        if constexpr (SIGNED) {
            const int pm = min(max(s8_estimate<6>(T, fabsf(xn)), 0), kS8SignedZero);
            const int est = xn < 0.f ? kS8SignedZero - pm : kS8SignedZero + pm;
            code = s8_nearest4(T.smid, min(max(est, 2), 252), xn);
        } else {
            code = s8_nearest4(T.umid, min(max(s8_estimate<7>(T, xn), 2), 253), xn);
        }
        pk |= code << (8 * j);
    }
    return pk;
}

// blocks of 256 elements, one per wave; count is a multiple of 4, so a lane's four elements are all in or all out
template <typename F>
__device__ inline void for_each_block(int64_t count, F f) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t blocks = (count + kS8Block - 1) / kS8Block;
    for (int64_t b = (int64_t)blockIdx.x * 4 + wave; b < blocks; b += (int64_t)gridDim.x * 4) {
        const int64_t e = b * kS8Block + lane * 4;
        f(b, e, e < count, lane);
    }
}

__global__ __launch_bounds__(256) void k_state8_quant(const float* __restrict__ x, int64_t count, int is_signed,
                                                      uint8_t* __restrict__ codes, float* __restrict__ scales) {
    __shared__ S8Tables T;
    s8_build(T);
    for_each_block(count, [&](int64_t b, int64_t e, bool in, int lane) {
        const f32x4 v = in ? *reinterpret_cast<const f32x4*>(x + e) : f32x4{0.f, 0.f, 0.f, 0.f};
        const float xs[4] = {v[0], v[1], v[2], v[3]};
        const float amax = wave_max(fmaxf(fmaxf(fabsf(xs[0]), fabsf(xs[1])), fmaxf(fabsf(xs[2]), fabsf(xs[3]))));
        const uint32_t pk = is_signed ? s8_encode4<true>(T, xs, amax) : s8_encode4<false>(T, xs, amax);
        if (in) *reinterpret_cast<uint32_t*>(codes + e) = pk;
        if (lane == 0) scales[b] = amax;
    });
}

__global__ __launch_bounds__(256) void k_state8_dequant(const uint8_t* __restrict__ codes, const float* __restrict__ scales,
                                                        int64_t count, int is_signed, float* __restrict__ x) {
    __shared__ S8Tables T;
    s8_build(T);
    const float* val = is_signed ? T.sval : T.uval;
    for_each_block(count, [&](int64_t b, int64_t e, bool in, int lane) {
        if (!in) return;
        const uint32_t pk = *reinterpret_cast<const uint32_t*>(codes + e);
        const float s = scales[b];
        f32x4 v;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = val[(pk >> (8 * j)) & 0xFFu] * s;
        *reinterpret_cast<f32x4*>(x + e) = v;
    });
}

__global__ __launch_bounds__(256) void k_lowrank_adam8(const float* __restrict__ R, uint8_t* __restrict__ Mq,
                                                       float* __restrict__ Ms, uint8_t* __restrict__ Vq,
                                                       float* __restrict__ Vs, uint16_t* __restrict__ N, int64_t count,
                                                       AdamCoef c) {
    __shared__ S8Tables T;
    s8_build(T);
    for_each_block(count, [&](int64_t b, int64_t e, bool in, int lane) {
        f32x4 r = {0.f, 0.f, 0.f, 0.f};
        uint32_t mq = 0x7F7F7F7Fu, vq = 0;              // zeros of the two tables
        if (in) {
            r = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(R + e));
            mq = *reinterpret_cast<const uint32_t*>(Mq + e);
            vq = *reinterpret_cast<const uint32_t*>(Vq + e);
        }
        const float ms = Ms[b], vs = Vs[b];
        float m[4], v[4], nn[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            m[j] = T.sval[(mq >> (8 * j)) & 0xFFu] * ms;
            v[j] = T.uval[(vq >> (8 * j)) & 0xFFu] * vs;
            nn[j] = adam_one(r[j], m[j], v[j], c);
        }
        const float am = wave_max(fmaxf(fmaxf(fabsf(m[0]), fabsf(m[1])), fmaxf(fabsf(m[2]), fabsf(m[3]))));
        const float av = wave_max(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])));
        const uint32_t mq1 = s8_encode4<true>(T, m, am), vq1 = s8_encode4<false>(T, v, av);
        if (in) {
            *reinterpret_cast<uint32_t*>(Mq + e) = mq1;
            *reinterpret_cast<uint32_t*>(Vq + e) = vq1;
            const u32x2 nb = {pack_bf16x2(nn[0], nn[1]), pack_bf16x2(nn[2], nn[3])};
            __builtin_nontemporal_store(nb, reinterpret_cast<u32x2*>(N + e));
        }
        if (lane == 0) {
            Ms[b] = am;
            Vs[b] = av;
        }
    });
}

static unsigned s8_grid(int64_t count) {
    const int64_t blocks = (count + kS8Block - 1) / kS8Block, wgs = (blocks + 3) / 4;
    return (unsigned)(wgs < 8192 ? wgs : 8192);          // 32 waves per CU at most; the rest is a grid-stride loop
}

static int check_state8(int64_t count) {
    if (count <= 0 || (count & 3) || count >= (int64_t(1) << 40)) return QG_ERR_SHAPE;
    return QG_OK;
}

}  // namespace qg

using namespace qg;

extern "C" int qg_state8_quant(const float* x, int64_t count, int is_signed, uint8_t* codes, float* scales, void* stream) {
    if (!x || !codes || !scales) return QG_ERR_NULL;
    if (int e = check_state8(count)) return e;
    if (!aligned16(x) || !aligned16(codes) || !aligned16(scales)) return QG_ERR_ALIGN;
    hipLaunchKernelGGL(k_state8_quant, dim3(s8_grid(count)), dim3(256), 0, (hipStream_t)stream, x, count, is_signed != 0, codes,
                       scales);
    return check_launch();
}

extern "C" int qg_state8_dequant(const uint8_t* codes, const float* scales, int64_t count, int is_signed, float* x,
                                 void* stream) {
    if (!x || !codes || !scales) return QG_ERR_NULL;
    if (int e = check_state8(count)) return e;
    if (!aligned16(x) || !aligned16(codes) || !aligned16(scales)) return QG_ERR_ALIGN;
    hipLaunchKernelGGL(k_state8_dequant, dim3(s8_grid(count)), dim3(256), 0, (hipStream_t)stream, codes, scales, count,
                       is_signed != 0, x);
    return check_launch();
}

extern "C" int qg_lowrank_adam8(const float* R, uint8_t* Mq, float* Ms, uint8_t* Vq, float* Vs, uint16_t* N_bf16,
                                int64_t count, int64_t step, const qg_hparams* hp, void* stream) {
    if (!R || !Mq || !Ms || !Vq || !Vs || !N_bf16 || !hp) return QG_ERR_NULL;
    if (int e = check_state8(count)) return e;
    if (step < 1) return QG_ERR_SHAPE;
    if (!aligned16(R) || !aligned16(Mq) || !aligned16(Ms) || !aligned16(Vq) || !aligned16(Vs) || !aligned16(N_bf16))
        return QG_ERR_ALIGN;
    hipLaunchKernelGGL(k_lowrank_adam8, dim3(s8_grid(count)), dim3(256), 0, (hipStream_t)stream, R, Mq, Ms, Vq, Vs, N_bf16,
                       count, make_adam_coef(hp, step));
    return check_launch();
}

extern "C" int qg_step8(const uint8_t* Pq, const float* Ps, const uint16_t* G_bf16, int8_t* Wq, float* Ws, uint8_t* Mq,
                        float* Ms, uint8_t* Vq, float* Vs, float* R, uint16_t* N_bf16, int64_t m, int64_t n, int64_t r,
                        int group, const qg_hparams* hp, uint64_t seed, int64_t step, void* stream) {
    if (!R || !hp) return QG_ERR_NULL;
    if (int e = qg_project(Pq, Ps, G_bf16, m, n, r, group, R, nullptr, 0, stream)) return e;
    if (int e = qg_lowrank_adam8(R, Mq, Ms, Vq, Vs, N_bf16, r * n, step, hp, stream)) return e;
    return qg_backproject_update_sr(Pq, Ps, N_bf16, Wq, Ws, m, n, r, group, hp->alpha, hp->lr, seed, step, nullptr, stream);
}
