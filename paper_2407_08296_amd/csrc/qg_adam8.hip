// Adam on the low-rank gradient with 8-bit states (Sec. 3.5: an 8-bit Adam is the inner optimizer).  The paper takes
// the state format from a third-party library and does not define it; this one is designed here after the published
// idea of block-wise dynamic quantization:
//   block   256 consecutive elements of the flattened r x n state, one fp32 scale = the block's absolute maximum
//   code    index of the entry nearest to x / scale (ties to the lower index) in a sorted table of 8-bit values with
//           relative resolution: entry p >= 1 of the unsigned table (second moment) has level L = floor(log2 p),
//           k = p - 2^L and value 10^-(7-L) * (0.1 + 0.9 (k+1) / 2^L), entry 0 is 0: 2^L values spaced linearly over
//           each decade from 1e-7 to 1.  The signed table (first moment) has levels 0..6 (1e-6 to 1): indices 0..126
//           the negatives from -1 up, 127 zero, 128..254 the positives; index 255 is not used.  One exception to
//           "nearest": a positive second moment takes code 1 at least.
// One step: states are dequantized (table[code] * scale), updated exactly like the fp32 states, and quantized again;
// 10 bytes of HBM traffic per element instead of 22.  A wave owns a block: a lane holds four consecutive elements,
// the block maximum is a wave reduction; the nearest entry comes from a bucket table indexed by the value's top
// float bits plus one comparison with a midpoint.
#include "qg_common.h"

namespace qg {

typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kS8Block = kGroup;      // elements per block
constexpr int kS8SignedZero = 127;    // index of 0 in the signed table

// Bucket table of the encoder: the positive floats up to 1 are cut into buckets by their top 15 bits (exponent and 7
// mantissa bits); lut[bucket] = number of midpoints below the bucket's lower edge.  Buckets are narrower than the
// spacing of the midpoints everywhere (at most one midpoint per bucket, which s8_build relies on and the bit-exact
// tests of the quantizer cover), so the code of a value is lut[bucket] plus one comparison with the next midpoint.
constexpr int kS8KeyShift = 16;
constexpr int kS8KeyOne = 0x3F800000 >> kS8KeyShift;     // bucket of 1.0
constexpr int kS8UKey0 = 0x33560000 >> kS8KeyShift;      // bucket of the first midpoint of the unsigned table, 5e-8
constexpr int kS8SKey0 = 0x35060000 >> kS8KeyShift;      // ... of the positive half of the signed table, 5e-7
constexpr int kS8ULut = kS8KeyOne - kS8UKey0 + 1, kS8SLut = kS8KeyOne - kS8SKey0 + 1;

struct S8Tables {
    float uval[256];    // unsigned table
    float umid[256];    // midpoints of neighbouring entries, padded with +inf
    float sval[256];    // signed table (255 entries, the last one repeated)
    float smid[256];
    uint8_t ulut[(kS8ULut + 15) / 16 * 16];
    uint8_t slut[(kS8SLut + 15) / 16 * 16];   // over the midpoints of the positive half, smid[127 + j]
};

// Entry p >= 1 of the positive half of a table with levels 0..top.
__device__ inline double s8_positive(int p, int top) {
    const double pow10neg[8] = {1e0, 1e-1, 1e-2, 1e-3, 1e-4, 1e-5, 1e-6, 1e-7};
    const int L = 31 - __clz(p), k = p - (1 << L);
    return pow10neg[top - L] * (0.1 + 0.9 * (double)(k + 1) / (double)(1 << L));
}

// Number of the `count` ascending midpoints mid[0..count) that lie below x.
__device__ inline int s8_count_below(const float* mid, int count, float x) {
    int lo = 0, hi = count;   // answer in [lo, hi]
    while (lo < hi) {
        const int m = (lo + hi) >> 1;
        if (mid[m] < x) lo = m + 1; else hi = m;
    }
    return lo;
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
    __syncthreads();
    T.umid[p] = p < 255 ? (float)(0.5 * ((double)T.uval[p] + (double)T.uval[p + 1])) : INFINITY;
    T.smid[p] = p < 254 ? (float)(0.5 * ((double)T.sval[p] + (double)T.sval[p + 1])) : INFINITY;
    __syncthreads();
    for (int i = p; i < kS8ULut; i += 256)
        T.ulut[i] = (uint8_t)s8_count_below(T.umid, 255, __builtin_bit_cast(float, (uint32_t)(kS8UKey0 + i) << kS8KeyShift));
    for (int i = p; i < kS8SLut; i += 256)
        T.slut[i] = (uint8_t)s8_count_below(T.smid + kS8SignedZero, 127,
                                            __builtin_bit_cast(float, (uint32_t)(kS8SKey0 + i) << kS8KeyShift));
    __syncthreads();
}

// Bucket of the magnitude ax >= 0 (values above 1 by a rounding error share the bucket of 1).
template <int KEY0, int SIZE>
__device__ inline int s8_bucket(float ax) {
    const int key = (int)(__builtin_bit_cast(uint32_t, ax) >> kS8KeyShift);
    return min(max(key - KEY0, 0), SIZE - 1);
}

// Codes of the lane's four values of a block whose absolute maximum is amax; returns them packed, low byte first.
// A code is the index of the nearest table entry, ties to the lower index = the number of midpoints below the value.
template <bool SIGNED>
__device__ inline uint32_t s8_encode4(const S8Tables& T, const float (&x)[4], float amax) {
    const float inv = amax > 0.f ? 1.0f / amax : 0.f;
    uint32_t pk = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float xn = x[j] * inv;
        uint32_t code;
        if constexpr (SIGNED) {
            // the table is symmetric: midpoints below a negative value -a = 127 - (positive midpoints <= a)
            const float a = fabsf(xn);
            const int c = T.slut[s8_bucket<kS8SKey0, kS8SLut>(a)];
            const float mid = T.smid[kS8SignedZero + c];
            code = xn < 0.f ? (uint32_t)(kS8SignedZero - c - (mid <= a)) : (uint32_t)(kS8SignedZero + c + (mid < a));
        } else {
            const int c = T.ulut[s8_bucket<kS8UKey0, kS8ULut>(fmaxf(xn, 0.f))];   // nothing lies below a negative value
            code = (uint32_t)(c + (T.umid[c] < xn));
            // a positive second moment never rounds to zero (the first moment's table reaches ten times further down:
            // with V flushed and M kept, Adam's quotient would come from the newest gradient alone)
            code = xn > 0.f ? max(code, 1u) : code;
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
                                                         // (2048 workgroups, one resident set, measured slower)
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
