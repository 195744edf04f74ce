// The two dense contractions of the step (Sec. 3.5) as bf16 MFMA GEMMs with the
// INT4 -> bf16 dequantization of P fused into LDS tile staging:
//   project:      R = dequant(P)^T G                      (K = m)
//   back-project: U = alpha dequant(P) N, followed in registers by the INT8
//                 stochastic-rounding weight update (Sec. 3.4).
//
// MFMA: v_mfma_f32_32x32x16_bf16.  Operand lane l holds row/column (l % 32) and
// the 8 consecutive k values 8*(l/32)..+7; accumulator register v of lane l is
// D[8*(v/4) + 4*(l/32) + v%4][l % 32].
//
// Operands whose K index is the slow (row) index in memory (P^T and G in the
// projection, N in the back-projection) are staged K-major in LDS exactly as
// they sit in HBM and fetched with the LDS transpose read ds_read_b64_tr_b16:
// inside a group of 16 lanes, lane i receives element (i % 4) of the four lanes
// 4j + i/4 (j = 0..3); lanes 4j..4j+3 point at 16 consecutive elements of tile
// row k+j, so lane i ends up with column i of rows k..k+3.
#pragma once

#include "qg_common.h"
#include "qg_plan.h"

namespace qg {

constexpr int kPadK = 32;  // bf16 of padding per row of a K-major tile (64 B: rows k..k+3 hit distinct bank groups)
// Cache policy of the R stores: non-temporal.  R is written once and read by a later kernel; kept out of the L2 it
// leaves the operand panels there for the tiles that share them (+13 % on one large matrix alone, neutral inside
// the full 7B step).
constexpr int kAuxStream = 2;
constexpr int kMfmaPrio = 1;   // wave priority during the MFMA phase of a K step (0 outside)
constexpr int kPadX = 8;   // bf16 of padding per row of a K-contiguous tile (16 B)

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

// Element offset (inside a K-major tile of `pitch` elements per row) of the first
// transpose read of this lane for the 32-wide operand block at column x0, k-step k0.
__device__ __forceinline__ int kmajor_lane_offset(int pitch, int lane) {
    const int g = lane >> 4, s = lane & 15;
    return (8 * (g >> 1) + (s >> 2)) * pitch + 16 * (g & 1) + 4 * (s & 3);
}

__device__ __forceinline__ bf16x8 read_kmajor_frag(const uint16_t* p, int pitch) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * pitch));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

// Vector types with the alignment of their elements only: rows of a matrix with an odd (or merely not 8-aligned)
// row length start at arbitrary element offsets.  Global memory accesses need no natural alignment on this target,
// so these still compile to single wide loads and stores.
typedef u32x4 __attribute__((aligned(2))) u32x4_align2;
typedef u32x4 __attribute__((aligned(1))) u32x4_align1;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef u32x2 __attribute__((aligned(4))) u32x2_align4;
typedef u32x4 __attribute__((aligned(4))) u32x4_align4;

// How a kernel instance treats the matrix edges.
//   kExact:     every tile lies inside the matrix and the K extent is a whole number of steps: no checks at all.
//   kMasked:    any m and r, rows 16-byte aligned (n a multiple of 8, r of 16).  Loads are the same wide buffer and
//               direct-to-LDS loads as kExact, bounded by the end of the matrix: what lies past the end reads as
//               zero, which is all the K tail needs; columns past a row's end read the next row (finite values that
//               only reach output elements the masked epilogue never stores).
//   kUnaligned: rows start at arbitrary element offsets (n not a multiple of 8): operands go through registers with
//               per-chunk checks.
enum : int { kExact = 0, kMasked = 1, kUnaligned = 2 };

// Number of bytes a bounded buffer resource may cover: `bytes` (not negative, a multiple of 4, below 2^34) clamped
// to what the 32-bit field holds; per-lane offsets stay far below that clamp.  Written with a shift and a 32-bit
// minimum so that it stays on the scalar unit (which has no 64-bit ordered compare).
__device__ __forceinline__ int bound_bytes(int64_t bytes) {
    const uint32_t words = (uint32_t)((uint64_t)bytes >> 2);
    return (int)((words < 0x1FFFFFFFu ? words : 0x1FFFFFFFu) << 2);
}

// Buffer resource over memory starting at `base`: loads through it take a scalar base, a scalar offset and a 32-bit
// per-thread byte offset, so a loop that only moves the base spends no vector instructions on addresses.
// Offsets at or past `bytes` read as zero.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, int bytes = 0x7FFFFFFF) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

// One wave-wide 16-byte-per-lane load straight into LDS: lane i's bytes land at lds + 16*i (lds is wave-uniform).
// `byte_off` is per lane, `uniform_off` wave-uniform (a scalar register).
__device__ __forceinline__ void buffer_load_lds16(__amdgpu_buffer_rsrc_t rs, void* lds, uint32_t byte_off,
                                                  uint32_t uniform_off) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void*)lds, 16, byte_off,
                                             uniform_off, 0, 0);
}

template <int WPT>
__device__ __forceinline__ void buffer_load_words(__amdgpu_buffer_rsrc_t rs, uint32_t byte_off, uint32_t (&w)[WPT]) {
    if constexpr (WPT == 4) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, byte_off, 0, 0);
        w[0] = v[0]; w[1] = v[1]; w[2] = v[2]; w[3] = v[3];
    } else if constexpr (WPT == 2) {
        const auto v = __builtin_amdgcn_raw_buffer_load_b64(rs, byte_off, 0, 0);
        w[0] = v[0]; w[1] = v[1];
    } else {
        w[0] = __builtin_amdgcn_raw_buffer_load_b32(rs, byte_off, 0, 0);
    }
}

// bf16 [K][X] operand tile of BK x BX elements whose rows are NOT padded: the kExact and kMasked kernels fill it with direct
// global -> LDS loads (no registers, no LDS write instructions), and one wave-wide 16-byte load deposits 1 KB of
// consecutive LDS.  Bank spreading comes from a swizzle instead: the 16-byte chunk c of row k sits at chunk position
// c ^ ((k & 3) << 2), so the four rows a transpose read touches fall into four different 64-byte bank groups.  For a
// transpose-read lane, k & 3 is a per-lane constant, and the swizzle is one xor on the (32-aligned) fragment column.
template <int BX, int BK, int NT>
struct KMajorSwizzled {
    static constexpr int STAGE = BK * BX;        // uint16 elements per stage
    static constexpr int CPR = BX / 8;           // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;         // rows per wave-wide load
    static constexpr int PER = BK / (RPI * (NT / 64));   // loads per wave per stage
    static_assert(CPR >= 16 && 64 % CPR == 0 && BK % (RPI * (NT / 64)) == 0 && PER >= 1, "tile shape");

    // element offset of 16-byte chunk c of row k
    __device__ static __forceinline__ int chunk_offset(int k, int c) { return k * BX + ((c ^ ((k & 3) << 2)) << 3); }
    // A wave's i-th load fills tile rows load_row0(wave, i) .. +RPI-1.  Lane `lane` fetches the chunk at byte offset
    // lane_src_bytes(lane, ld, v) + load_row0(wave, i) * ld * 2 from the tile's first element (row length ld).  The
    // second summand is wave-uniform; the first depends on the load only through the residue v = load_row0 & 3 in
    // the swizzle, which takes 4 / RPI values (at most two for the tiles used here): that many per-lane offsets
    // serve all loads.
    static constexpr int VARIANTS = RPI >= 4 ? 1 : 4 / RPI;
    static_assert(PER % VARIANTS == 0, "every wave starts at a row that is a multiple of 4");
    __device__ static __forceinline__ int load_row0(int wave, int i) { return (wave * PER + i) * RPI; }
    __device__ static __forceinline__ uint32_t lane_src_bytes(int lane, int ld, int v) {
        const int row = lane / CPR;   // row inside the load
        const int c = (lane % CPR) ^ (((v * RPI + row) & 3) << 2);
        return 2u * (uint32_t)(row * ld + c * 8);
    }
    // transpose-read lane offset and swizzle term (elements)
    __device__ static __forceinline__ int lane_offset(int lane) { return kmajor_lane_offset(BX, lane); }
    __device__ static __forceinline__ int lane_swizzle(int lane) { return ((lane & 15) >> 2) << 5; }
};

// 8 consecutive bf16 starting at `src`, of which the first `valid` lie inside the matrix (ragged shapes): one
// 16-byte load when all do, element by element for the chunk that straddles the edge, zeros outside.
__device__ __forceinline__ u32x4 load8_bf16_guarded(const uint16_t* src, int valid) {
    if (valid >= 8) return *reinterpret_cast<const u32x4_align2*>(src);
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 8; ++j)
        if (j < valid) w[j >> 1] |= (uint32_t)src[j] << (16 * (j & 1));
    const u32x4 o = {w[0], w[1], w[2], w[3]};
    return o;
}

// Guarded fetch of WPT words of INT4 codes starting at flat element index e (a multiple of 8), of which the first
// `valid` codes lie inside the matrix.  Every word carries the scale of its own block: with r not a multiple of
// 8*WPT the words of one fetch can fall into two blocks of 256.  Words outside read as code 0, scale 0.
template <int WPT>
__device__ __forceinline__ void load_p_guarded(const uint8_t* Pq, const float* Ps, uint32_t e, int valid,
                                               uint32_t (&w)[WPT], float (&sc)[WPT]) {
    const uint8_t* p = Pq + (e >> 1);
    if (valid >= 8 * WPT) {
        if constexpr (WPT == 4) {
            const u32x4 v = *reinterpret_cast<const u32x4_align4*>(p);
            w[0] = v[0]; w[1] = v[1]; w[2] = v[2]; w[3] = v[3];
        } else if constexpr (WPT == 2) {
            const u32x2 v = *reinterpret_cast<const u32x2_align4*>(p);
            w[0] = v[0]; w[1] = v[1];
        } else {
            w[0] = *reinterpret_cast<const uint32_t*>(p);
        }
#pragma unroll
        for (int j = 0; j < WPT; ++j) sc[j] = Ps[(e + 8 * j) >> 8];
    } else {
#pragma unroll
        for (int j = 0; j < WPT; ++j) {
            const bool ok = valid > 8 * j;
            w[j] = ok ? *reinterpret_cast<const uint32_t*>(p + 4 * j) : 0x88888888u;
            sc[j] = ok ? Ps[(e + 8 * j) >> 8] : 0.f;
        }
    }
}

// Words of INT4 codes a thread fetches with one load when staging a P tile: as wide as the tile allows.  Where r is
// a multiple of 8*WPT a fetch starts at a multiple of 8*WPT codes and never straddles a block of 256, so one scale
// serves it; the kernels for unaligned shapes (r only a multiple of 8) keep a scale per word.
template <int WORDS, int NT, bool PER_WORD_SCALES>
struct P_Task {
    static constexpr int WPT = WORDS / NT >= 4 ? 4 : (WORDS / NT >= 2 ? 2 : 1);
    static constexpr int PER = WORDS / (NT * WPT);
    static constexpr int NSC = PER_WORD_SCALES ? WPT : 1;   // scales kept per fetch
    static_assert(WORDS % (NT * WPT) == 0 && PER >= 1, "staging must divide evenly");
};

// XCD-aware tile order: consecutive workgroup ids go round-robin over the 8 XCDs
// (each with its own L2), so XCD x is handed the contiguous range of tiles
// [x*per, (x+1)*per), and neighbouring tiles (which share operand panels) meet in
// one L2.  gridDim.x is a multiple of 8.
__device__ __forceinline__ uint32_t xcd_tile(uint32_t wg, uint32_t grid) {
    const uint32_t per = grid >> 3;
    return (wg & 7u) * per + (wg >> 3);
}

// ============================================================================
// Projection: R[r0.., n0..] tile of BM x BN, K loop over m in steps of BK.
// ============================================================================
template <int BM, int BN, int BK, int WGM, int WGN>
struct ProjShape {
    static constexpr int NT = WGM * WGN * 64;
    static constexpr int PA = BM + kPadK, PB = BN;   // P tile padded, G tile swizzled (KMajorSwizzled)
    static constexpr int A_STAGE = BK * PA, B_STAGE = BK * PB;
    static constexpr int SMEM = 2 * (A_STAGE + B_STAGE);  // uint16 elements
};

// With FUSE_ADAM the epilogue runs Adam on the tile while R is still in the accumulators: M and V are read and
// written in place, N is stored as bf16 and R goes to memory only if the caller asked for it (R != nullptr), which
// saves the 8 bytes per element of writing R and reading it back in a separate pass.
template <int BM, int BN, int BK, int WGM, int WGN, int MODE, bool FUSE_ADAM = false>
__device__ __forceinline__ void project_tile(const uint8_t* __restrict__ Pq, const float* __restrict__ Ps,
                                             const uint16_t* __restrict__ G, float* __restrict__ R, int m, int n,
                                             int ld, int r, int r0, int n0, uint16_t* smem, float* __restrict__ Mo = nullptr,
                                             float* __restrict__ Vo = nullptr, uint16_t* __restrict__ No = nullptr,
                                             const AdamCoef* coef = nullptr) {
    constexpr bool RAGGED = MODE != kExact;      // masked epilogue
    constexpr bool DIRECT = MODE != kUnaligned;  // buffer / direct-to-LDS loads; a P fetch (8*WPT codes) starts at a
                                                 // multiple of 8*WPT codes, so it lies in one block of 256
    using S = ProjShape<BM, BN, BK, WGM, WGN>;
    constexpr int NT = S::NT;
    constexpr int WM = BM / WGM, WN = BN / WGN, MB = WM / 32, NB = WN / 32;
    constexpr int PA = S::PA;
    constexpr int A_WORDS = BK * BM / 8;
    using AT = P_Task<A_WORDS, NT, !DIRECT>;
    constexpr int A_PER = AT::PER, WPT = AT::WPT, A_TPR = BM / (8 * WPT);   // tasks per tile row
    using BD = KMajorSwizzled<BN, BK, NT>;
    constexpr int B_PER = BD::PER;
    static_assert(B_PER * NT * 8 == BK * BN, "staging must divide evenly");
    static_assert(BK % 16 == 0 && WM % 32 == 0 && WN % 32 == 0, "tile shape");
    uint16_t* As = smem;
    uint16_t* Bs = smem + 2 * S::A_STAGE;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);   // wave-uniform: keeps everything derived from it scalar
    const int wm = wave / WGN, wn = wave % WGN;
    uint32_t aw[A_PER][WPT];
    float asc[A_PER][AT::NSC];
    u32x4 bv[DIRECT ? 1 : B_PER];   // the unaligned kernels stage G through registers

    // Addresses are split into a part that is uniform over the workgroup and advances with the K step (scalar
    // registers, scalar arithmetic) and a 32-bit per-thread offset fixed for the whole loop; the kExact and kMasked kernels
    // load through buffer resources based at the uniform part, so their loop spends no vector instructions on
    // address arithmetic.  A K step covers BK rows of P, i.e. BK*r codes: a multiple of 256 (r is a multiple of 8),
    // so code bytes and block scales split the same way.
    static_assert(BK % 32 == 0, "a K step must cover whole blocks of 256 codes");
    constexpr int B_OFFS = DIRECT ? BD::VARIANTS : B_PER;
    uint32_t a_el[A_PER], b_byte[B_OFFS];   // P: element offset; G: byte offset
#pragma unroll
    for (int p = 0; p < A_PER; ++p) {
        const int ti = t + p * NT;
        a_el[p] = (uint32_t)((ti / A_TPR) * r + r0 + (ti % A_TPR) * (8 * WPT));
    }
#pragma unroll
    for (int p = 0; p < B_OFFS; ++p) {
        if constexpr (DIRECT) {
            b_byte[p] = BD::lane_src_bytes(lane, ld, p);
        } else {
            const int ci = t + p * NT;
            b_byte[p] = 2u * (uint32_t)((ci / BD::CPR) * ld + (ci % BD::CPR) * 8);
        }
    }

    // Tile kt: P codes and scales into registers; G straight into LDS stage `stage` (kExact, kMasked) or into
    // registers (kUnaligned, stored by sstore).
    auto gload = [&](int kt, int stage) {
        const int i0 = kt * BK;
        const int64_t e0 = (int64_t)i0 * r;
        const uint8_t* pq = Pq + (e0 >> 1);
        const float* ps = Ps + (e0 >> 8);
        const uint8_t* g = reinterpret_cast<const uint8_t*>(G + (int64_t)i0 * ld + n0);
        if constexpr (DIRECT) {
            __amdgpu_buffer_rsrc_t rq, rs, rg;
            if constexpr (MODE == kExact) {
                rq = make_rsrc(pq); rs = make_rsrc(ps); rg = make_rsrc(g);
            } else {   // bounded by the end of each array: rows at or past m read as zero
                const int64_t mr = (int64_t)m * r;
                rq = make_rsrc(pq, bound_bytes((mr - e0) >> 1));
                rs = make_rsrc(ps, bound_bytes((((mr + kGroup - 1) >> 8) - (e0 >> 8)) * 4));
                rg = make_rsrc(g, bound_bytes(((int64_t)(m - i0) * ld - n0) * 2));
            }
#pragma unroll
            for (int p = 0; p < B_PER; ++p)
                buffer_load_lds16(rg, Bs + stage * S::B_STAGE + BD::load_row0(wave, p) * BN, b_byte[p % BD::VARIANTS],
                                  2u * (uint32_t)(BD::load_row0(wave, p) * ld));
#pragma unroll
            for (int p = 0; p < A_PER; ++p) {
                buffer_load_words<WPT>(rq, a_el[p] >> 1, aw[p]);
#pragma unroll
                for (int j = 0; j < AT::NSC; ++j)
                    asc[p][j] = __builtin_bit_cast(
                        float, __builtin_amdgcn_raw_buffer_load_b32(rs, ((a_el[p] + 8 * j) >> 8) << 2, 0, 0));
            }
        } else {
#pragma unroll
            for (int p = 0; p < A_PER; ++p) {
                const int ti = t + p * NT;
                const int row = ti / A_TPR, c = (ti % A_TPR) * (8 * WPT);
                load_p_guarded<WPT>(pq, ps, a_el[p], i0 + row < m ? r - (r0 + c) : 0, aw[p], asc[p]);
            }
#pragma unroll
            for (int p = 0; p < B_PER; ++p) {
                const int ci = t + p * NT;
                const int row = ci / BD::CPR, c8 = ci % BD::CPR;
                const int valid = (i0 + row < m) ? (n - (n0 + c8 * 8)) : 0;
                bv[p] = load8_bf16_guarded(reinterpret_cast<const uint16_t*>(g + b_byte[p]), valid);
            }
        }
    };
    // Dequantized P tile (and, in the kUnaligned kernels, the G tile) into LDS stage `stage`; returns once the stage's
    // direct loads have landed too, so that the barrier that follows publishes the whole stage.
    auto sstore = [&](int stage) {
#pragma unroll
        for (int p = 0; p < A_PER; ++p) {
            const int ti = t + p * NT;
            const int row = ti / A_TPR, c = (ti % A_TPR) * (8 * WPT);
#pragma unroll
            for (int j = 0; j < WPT; ++j)
                *reinterpret_cast<u32x4*>(As + stage * S::A_STAGE + row * PA + c + 8 * j) =
                    dequant8_bf16(aw[p][j], asc[p][DIRECT ? 0 : j]);
        }
        if constexpr (!DIRECT) {
#pragma unroll
            for (int p = 0; p < B_PER; ++p) {
                const int ci = t + p * NT;
                *reinterpret_cast<u32x4*>(Bs + stage * S::B_STAGE + BD::chunk_offset(ci / BD::CPR, ci % BD::CPR)) = bv[p];
            }
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // direct loads are counted like any other load
        }
    };

    f32x16 acc[MB][NB];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    const int a_lane = kmajor_lane_offset(PA, lane) + wm * WM;
    int b_lane[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) b_lane[b] = BD::lane_offset(lane) + ((wn * WN + b * 32) ^ BD::lane_swizzle(lane));
    const int KT = (m + BK - 1) / BK;

    auto mfma_step = [&](int stage) {
        const uint16_t* Ac = As + stage * S::A_STAGE + a_lane;
        const uint16_t* Bc = Bs + stage * S::B_STAGE;
        // With several workgroups per CU a SIMD holds several waves; the one in its MFMA phase gets issue priority so the
        // matrix pipe stays fed while the other waves' staging instructions fill the gaps.
        __builtin_amdgcn_s_setprio(kMfmaPrio);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 af[MB], bf[NB];
#pragma unroll
            for (int a = 0; a < MB; ++a) af[a] = read_kmajor_frag(Ac + kk * 16 * PA + a * 32, PA);
#pragma unroll
            for (int b = 0; b < NB; ++b) bf[b] = read_kmajor_frag(Bc + kk * 16 * BN + b_lane[b], BN);
#pragma unroll
            for (int a = 0; a < MB; ++a)
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bf[b], acc[a][b], 0, 0, 0);
            // fragments of one 16-wide sub-step at a time (keeps the register count within three workgroups per CU)
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_s_setprio(0);
    };

    // Unrolled by two so that the LDS stage of every access is a compile-time constant (no per-step address
    // arithmetic).  Loads past the end re-read the last K slab (in bounds, never consumed), which keeps every load
    // and store unconditional.
    gload(0, 0);
    sstore(0);
    __syncthreads();
    for (int kt = 0; kt < KT; kt += 2) {
        gload(min(kt + 1, KT - 1), 1);
        mfma_step(0);
        sstore(1);
        __syncthreads();
        gload(min(kt + 2, KT - 1), 0);
        if (kt + 1 < KT) mfma_step(1);
        sstore(0);
        __syncthreads();
    }

    const int lcol = lane & 31, lhalf = lane >> 5;
    if (!FUSE_ADAM) {
        // R through buffer stores: the base of each 32-row block and the row inside it are scalars, the lane supplies
        // one byte offset per 32-column block, and stores past the resource's end are dropped by the hardware.  That
        // is the whole row mask (rows at or past r lie past the end of R); a column at or past n gets an offset no
        // resource covers.
        uint32_t voff[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int col = wn * WN + b * 32 + lcol;   // inside the tile
            voff[b] = (!RAGGED || n0 + col < n) ? 4u * (uint32_t)(4 * lhalf * ld + col) : 0x80000000u;
        }
#pragma unroll
        for (int a = 0; a < MB; ++a) {
            const int row0 = r0 + wm * WM + a * 32;
            float* base = R + (int64_t)row0 * ld + n0;
            const __amdgpu_buffer_rsrc_t rr =
                RAGGED ? make_rsrc(base, row0 < r ? bound_bytes(((int64_t)(r - row0) * ld - n0) * 4) : 0) : make_rsrc(base);
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float x = acc[a][b][v];   // (a copy: bit_cast of a vector element lvalue reads element 0)
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, x), rr, voff[b],
                                                          4u * (uint32_t)((8 * (v >> 2) + (v & 3)) * ld), kAuxStream);
                }
        }
    } else if constexpr (DIRECT) {
        // Adam on the tile while R is still in the accumulators.  M, V (and R, N) go through buffer resources like
        // the R stores above: scalar base per 32-row block, scalar row offset, one per-lane offset per 32-column
        // block; rows at or past r lie past the end of every array (loads return 0, stores are dropped), columns at
        // or past n get an offset no resource covers.  Loads are issued eight rows at a time ahead of the
        // arithmetic.  N: registers v and v+1 of a lane are rows i and i+1 of one column; even lanes store row i,
        // odd lanes row i+1, each as one 4-byte bf16 pair with the value of the neighbouring column from lane ^ 1.
        const AdamCoef c = *coef;
        const bool odd = (lane & 1) != 0;
        // v_perm_b32 selector over {nbr (bytes 4..7), own (bytes 0..3)}: even lanes (own.lo, nbr.lo), odd (nbr.hi, own.hi)
        const uint32_t pair_sel = odd ? 0x03020706u : 0x05040100u;
        uint32_t voff[NB], voffn[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int col = wn * WN + b * 32 + lcol;   // inside the tile
            const bool ok = !RAGGED || n0 + col < n;
            voff[b] = ok ? 4u * (uint32_t)(4 * lhalf * ld + col) : 0x80000000u;
            // a pair is stored if its first (even) column is a real one: with an odd n (possible only with a row pitch
            // ld > n) the pair of column n - 1 also covers the first padding column
            const bool okn = !RAGGED || n0 + (col & ~1) < n;
            voffn[b] = okn ? 2u * (uint32_t)(4 * lhalf * ld + col + (odd ? ld - 1 : 0)) : 0x80000000u;
        }
#pragma unroll
        for (int a = 0; a < MB; ++a) {
            const int row0 = r0 + wm * WM + a * 32;
            const int64_t e0 = (int64_t)row0 * ld + n0;
            const int left4 = RAGGED ? (row0 < r ? bound_bytes(((int64_t)(r - row0) * ld - n0) * 4) : 0) : 0x7FFFFFFF;
            const __amdgpu_buffer_rsrc_t rm = make_rsrc(Mo + e0, left4), rv = make_rsrc(Vo + e0, left4);
            const bool write_R = R != nullptr;
            const __amdgpu_buffer_rsrc_t rr = make_rsrc(write_R ? R + e0 : Mo + e0, write_R ? left4 : 0);
            const __amdgpu_buffer_rsrc_t rn = make_rsrc(No + e0, RAGGED ? left4 / 2 : 0x7FFFFFFF);
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    float mm[8], vv[8];
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        const int v = 8 * h + q;
                        const uint32_t so = 4u * (uint32_t)((8 * (v >> 2) + (v & 3)) * ld);
                        mm[q] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rm, voff[b], so, kAuxStream));
                        vv[q] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rv, voff[b], so, kAuxStream));
                    }
#pragma unroll
                    for (int q = 0; q < 8; q += 2) {
                        float nn[2];
#pragma unroll
                        for (int e = 0; e < 2; ++e) {
                            const int v = 8 * h + q + e;
                            const uint32_t so = 4u * (uint32_t)((8 * (v >> 2) + (v & 3)) * ld);
                            const float rr_ = acc[a][b][v];
                            nn[e] = adam_one(rr_, mm[q + e], vv[q + e], c);
                            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, mm[q + e]), rm, voff[b], so, kAuxStream);
                            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, vv[q + e]), rv, voff[b], so, kAuxStream);
                            if (write_R)
                                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, rr_), rr, voff[b], so, kAuxStream);
                        }
                        const int v = 8 * h + q;   // rows i (v) and i + 1 (v + 1)
                        // own column as (row i, row i+1), the neighbour lane's the same way (one DPP move), then one
                        // byte permute picks (own row i, neighbour row i) in even lanes and (neighbour row i+1, own
                        // row i+1) in odd lanes
                        const uint32_t own = pack_bf16x2(nn[0], nn[1]);
                        const uint32_t nbr = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)own, 0xB1, 0xF, 0xF, true);
                        const uint32_t pk = __builtin_amdgcn_perm(nbr, own, pair_sel);
                        __builtin_amdgcn_raw_buffer_store_b32(pk, rn, voffn[b],
                                                              2u * (uint32_t)((8 * (v >> 2) + (v & 3)) * ld), kAuxStream);
                    }
                }
        }
    } else {
        const AdamCoef c = *coef;
#pragma unroll
        for (int a = 0; a < MB; ++a)
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int col = n0 + wn * WN + b * 32 + lcol;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = r0 + wm * WM + a * 32 + 8 * (v >> 2) + 4 * lhalf + (v & 3);
                    const int64_t off = (int64_t)row * ld + col;
                    if (row < r && col < n) {
                        const float rr_ = acc[a][b][v];
                        float mm = Mo[off], vv = Vo[off];
                        const float nn = adam_one(rr_, mm, vv, c);
                        if (R != nullptr) R[off] = rr_;
                        Mo[off] = mm;
                        Vo[off] = vv;
                        No[off] = to_bf16(nn);
                    }
                }
            }
    }
}

template <int BM, int BN, int BK, int WGM, int WGN, int MODE, int MIN_WG_PER_CU = 1>
__global__ __launch_bounds__(WGM* WGN * 64, MIN_WG_PER_CU) void k_project(const uint8_t* __restrict__ Pq,
                                                           const float* __restrict__ Ps,
                                                           const uint16_t* __restrict__ G, float* __restrict__ R,
                                                           int m, int n, int ld, int r, uint32_t tiles_r, uint32_t tiles) {
    __shared__ __attribute__((aligned(16))) uint16_t smem[ProjShape<BM, BN, BK, WGM, WGN>::SMEM];
    const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x);
    if (tile >= tiles) return;
    project_tile<BM, BN, BK, WGM, WGN, MODE>(Pq, Ps, G, R, m, n, ld, r, (int)(tile % tiles_r) * BM,
                                               (int)(tile / tiles_r) * BN, smem);
}

template <int BM, int BN, int BK, int WGM, int WGN, int MODE, int MIN_WG_PER_CU = 1>
__global__ __launch_bounds__(WGM* WGN * 64, MIN_WG_PER_CU) void k_project_adam(
    const uint8_t* __restrict__ Pq, const float* __restrict__ Ps, const uint16_t* __restrict__ G,
    float* __restrict__ R, float* __restrict__ M, float* __restrict__ V, uint16_t* __restrict__ N, int m, int n, int ld,
    int r, uint32_t tiles_r, uint32_t tiles, AdamCoef coef) {
    __shared__ __attribute__((aligned(16))) uint16_t smem[ProjShape<BM, BN, BK, WGM, WGN>::SMEM];
    const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x);
    if (tile >= tiles) return;
    project_tile<BM, BN, BK, WGM, WGN, MODE, true>(Pq, Ps, G, R, m, n, ld, r, (int)(tile % tiles_r) * BM,
                                                     (int)(tile / tiles_r) * BN, smem, M, V, N, &coef);
}

template <typename F>
__device__ __forceinline__ int plan_find(const PlanMatrix* mats, int count, uint32_t tile, F first_tile) {
    int lo = 0, hi = count - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (first_tile(mats[mid]) <= tile) lo = mid; else hi = mid - 1;
    }
    return lo;
}

template <int BM, int BN, int BK, int WGM, int WGN, int MODE, int MIN_WG_PER_CU = 1>
__global__ __launch_bounds__(WGM* WGN * 64, MIN_WG_PER_CU) void k_project_many(const PlanHeader* __restrict__ plan, int first,
                                                                               int count, uint32_t tiles) {
    __shared__ __attribute__((aligned(16))) uint16_t smem[ProjShape<BM, BN, BK, WGM, WGN>::SMEM];
    const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x);
    if (tile >= tiles) return;
    const PlanMatrix* mats = plan_matrices(plan) + first;
    const PlanMatrix& d = mats[plan_find(mats, count, tile, [](const PlanMatrix& x) { return x.proj_tile0; })];
    const uint32_t local = tile - d.proj_tile0;
    project_tile<BM, BN, BK, WGM, WGN, MODE>(d.Pq, d.Ps, d.G, d.R, (int)d.m, (int)d.n, (int)d.ld, (int)d.r,
                                               (int)(local % d.proj_tiles_r) * BM,
                                               (int)(local / d.proj_tiles_r) * BN, smem);
}

// Up to kProjBatchMax matrices of one shape in one launch, their pointers passed by value (no plan in device memory:
// what the subspace refresh needs, which owns no device buffer beyond its workspace and may run under graph capture).
// R of matrix z goes to R + z * strideR, with the row pitch ld of the gradients.
constexpr int kProjBatchMax = 16;
struct ProjBatch {
    const uint8_t* Pq[kProjBatchMax];
    const float* Ps[kProjBatchMax];
    const uint16_t* G[kProjBatchMax];
};

template <int BM, int BN, int BK, int WGM, int WGN, int MODE, int MIN_WG_PER_CU = 1>
__global__ __launch_bounds__(WGM* WGN * 64, MIN_WG_PER_CU) void k_project_batch(ProjBatch batch, float* __restrict__ R,
                                                                                int64_t strideR, int m, int n, int ld,
                                                                                int r, uint32_t tiles_r,
                                                                                uint32_t tiles_per, uint32_t tiles) {
    __shared__ __attribute__((aligned(16))) uint16_t smem[ProjShape<BM, BN, BK, WGM, WGN>::SMEM];
    const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x);
    if (tile >= tiles) return;
    const uint32_t z = tile / tiles_per, local = tile % tiles_per;
    project_tile<BM, BN, BK, WGM, WGN, MODE>(batch.Pq[z], batch.Ps[z], batch.G[z], R + (int64_t)z * strideR, m, n, ld, r,
                                               (int)(local % tiles_r) * BM, (int)(local / tiles_r) * BN, smem);
}

template <int BM, int BN, int BK, int WGM, int WGN, int MODE, int MIN_WG_PER_CU = 1>
__global__ __launch_bounds__(WGM* WGN * 64, MIN_WG_PER_CU) void k_project_adam_many(const PlanHeader* __restrict__ plan,
                                                                                     int first, int count,
                                                                                     uint32_t tiles, int write_R,
                                                                                     AdamCoef coef) {
    __shared__ __attribute__((aligned(16))) uint16_t smem[ProjShape<BM, BN, BK, WGM, WGN>::SMEM];
    const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x);
    if (tile >= tiles) return;
    const PlanMatrix* mats = plan_matrices(plan) + first;
    const PlanMatrix& d = mats[plan_find(mats, count, tile, [](const PlanMatrix& x) { return x.proj_tile0; })];
    const uint32_t local = tile - d.proj_tile0;
    project_tile<BM, BN, BK, WGM, WGN, MODE, true>(d.Pq, d.Ps, d.G, write_R ? d.R : nullptr, (int)d.m, (int)d.n,
                                                     (int)d.ld, (int)d.r, (int)(local % d.proj_tiles_r) * BM,
                                                     (int)(local / d.proj_tiles_r) * BN, smem, d.M, d.V, d.N, &coef);
}

// ============================================================================
// Back-projection + INT8 stochastic-rounding update.
// The MFMA computes the TRANSPOSED tile D = N^T-block x P^T-block, i.e.
// D[row = n index][col = m index], so that one lane owns ONE weight row (m) and
// 4-element runs of consecutive columns (n): the per-row block absmax is an
// in-lane reduction plus one cross-half shuffle and one LDS exchange.
// Tile: 256 columns of W (exactly one quantization block per row) x BMm rows.
// ============================================================================
// W_PREFETCH: the weight tile has LDS of its own and is fetched before the main loop (one workgroup per CU);
// otherwise it reuses the staging buffers after the main loop (smaller footprint, two workgroups per CU, whose
// epilogue and main loop then overlap).
template <int BMm, int BK, int WGn, int WGm, bool W_PREFETCH = true, bool ZP = false>
struct BpShape {
    static constexpr int BNn = kGroup;
    static constexpr int NT = WGn * WGm * 64;
    static constexpr int PA = BNn;          // N tile, K-major, swizzled (KMajorSwizzled)
    static constexpr int PB = BK + kPadX;   // P tile, [m][k], padded
    static constexpr int A_STAGE = BK * PA, B_STAGE = BMm * PB;
    static constexpr int STAGING = 2 * (A_STAGE + B_STAGE);   // uint16 elements
    static constexpr int WTILE = BMm * BNn / 2;                // INT8 weight tile, in uint16 elements
    static constexpr int EXCH = (ZP ? 2 : 1) * WGn * BMm * 2;   // row-max (and, with zero points, row-min) exchange
    static constexpr int WOFF = W_PREFETCH ? STAGING : EXCH;    // after the exchange area if aliased
    static constexpr int SMEM = W_PREFETCH ? STAGING + WTILE : (STAGING > WOFF + WTILE ? STAGING : WOFF + WTILE);
};

// Byte offset of weight-tile element (row, col) in LDS.  Rows are 256 bytes (one quantization block); the 16
// 16-byte chunks of a row are stored at chunk ^ (row & 15), so the 32 lanes of an MFMA accumulator column (32
// consecutive rows, same column) spread over 16 bank groups, while every row still fills 256 contiguous bytes
// (direct global->LDS loads deposit whole rows).
__device__ __forceinline__ int wtile_offset(int row, int col) {
    return row * kGroup + ((((col >> 4) ^ row) & 15) << 4) + (col & 15);
}

// A lane's 4-element runs of an accumulator row sit at columns c0 + 32*a + 8*v4 (c0 = the lane's first column, a
// multiple of 4 below 8 plus a multiple of the wave's column span).  Their tile offsets differ from that of c0 only
// in bits that c0 leaves clear, so they are wtile_offset(row, c0) ^ wtile_run_bits(a, v4): one xor with a
// compile-time constant per access instead of the full swizzle.
__device__ __forceinline__ constexpr int wtile_run_bits(int a, int v4) {
    return ((2 * a + (v4 >> 1)) << 4) | ((v4 & 1) << 3);
}

// ZP: the weight carries a zero point per block (Sec. 3.1 eq.; Appendix A's `W_q - zeros`): x = (code - z)*s - lr*U,
// the new block takes s' = (hi - lo)/255 over [min(0, min x), max(0, max x)], z' = -128 - round(lo/s'), and the
// stochastically rounded code is floor(x/s' + u) + z'.
template <int BMm, int BK, int WGn, int WGm, int MODE, bool DUMP_U, bool W_PREFETCH = true, bool ZP = false>
__device__ __forceinline__ void backproject_tile(const uint8_t* __restrict__ Pq, const float* __restrict__ Ps,
                                                 const uint16_t* __restrict__ N, int8_t* __restrict__ Wq,
                                                 float* __restrict__ Ws, float* __restrict__ Wz,
                                                 float* __restrict__ Udbg, int m, int n, int ld,
                                                 int r, int m0, int tile_n, float alpha, float lr, uint32_t key,
                                                 uint16_t* smem) {
    constexpr bool RAGGED = MODE != kExact;      // masked epilogue
    constexpr bool DIRECT = MODE != kUnaligned;  // buffer / direct-to-LDS loads; a P fetch (8*WPT codes) starts at a
                                                 // multiple of 8*WPT codes, so it lies in one block of 256
    using S = BpShape<BMm, BK, WGn, WGm, W_PREFETCH, ZP>;
    constexpr int BNn = S::BNn, NT = S::NT, NW = WGn * WGm;
    constexpr int SN = BNn / WGn, SM = BMm / WGm, IB = SN / 32, JB = SM / 32;
    constexpr int PA = S::PA, PB = S::PB;
    using AD = KMajorSwizzled<BNn, BK, NT>;
    constexpr int A_PER = AD::PER;
    constexpr int B_WORDS = BMm * BK / 8;
    using BT = P_Task<B_WORDS, NT, !DIRECT>;
    constexpr int B_PER = BT::PER, WPT = BT::WPT, B_TPR = BK / (8 * WPT);   // tasks per tile row
    static_assert(BK % (8 * WPT) == 0, "tile shape");
    constexpr int W_ROUNDS = BMm / 4 / NW;   // each wave-wide 16-byte access covers 4 tile rows
    static_assert(A_PER * NT * 8 == BK * BNn, "staging must divide evenly");
    static_assert(S::EXCH <= S::STAGING, "row-max exchange must fit in the staging buffers");
    static_assert((BMm / 4) % NW == 0, "weight tile rows must divide evenly over the waves");
    static_assert(SN % 32 == 0 && (SN & (SN - 1)) == 0, "a wave's column span must be a power of two (wtile_run_bits)");
    uint16_t* As = smem;
    uint16_t* Bs = smem + 2 * S::A_STAGE;
    uint8_t* wt = reinterpret_cast<uint8_t*>(smem + S::WOFF);
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);   // wave-uniform: keeps everything derived from it scalar
    const int wn = wave / WGm, wm = wave % WGm;
    const int n0 = tile_n * BNn;
    const int ng = (n + kGroup - 1) / kGroup;

    // ---- weight tile -> LDS (asynchronous direct loads where shapes allow) ----
    // whole tile inside the matrix and rows 16-byte aligned: the direct loads work in the edge-checking kernels too
    const bool w_fast = !RAGGED || (m0 + BMm <= m && n0 + BNn <= n && (ld & 15) == 0);
    auto load_wtile = [&]() {
    if (w_fast) {
#pragma unroll
        for (int i = 0; i < W_ROUNDS; ++i) {
            const int rb = (wave * W_ROUNDS + i) * 4;             // first of the 4 rows this wave access covers
            const int row = rb + (lane >> 4), chunk = (lane ^ row) & 15;
            const int8_t* src = Wq + (int64_t)(m0 + row) * ld + n0 + chunk * 16;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)(wt + rb * kGroup), 16, 0, 0);
        }
    } else {
        // same lane -> (row, chunk) map through registers: rows may start at any byte offset, and the chunk that
        // straddles the matrix edge is fetched byte by byte
#pragma unroll
        for (int i = 0; i < W_ROUNDS; ++i) {
            const int rb = (wave * W_ROUNDS + i) * 4;
            const int row = rb + (lane >> 4), chunk = (lane ^ row) & 15;
            const int8_t* src = Wq + (int64_t)(m0 + row) * ld + n0 + chunk * 16;
            const int valid = m0 + row < m ? n - (n0 + chunk * 16) : 0;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (valid >= 16) {
                v = *reinterpret_cast<const u32x4_align1*>(src);
            } else {
                uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    if (j < valid) w[j >> 2] |= (uint32_t)(uint8_t)src[j] << (8 * (j & 3));
                v[0] = w[0]; v[1] = w[1]; v[2] = w[2]; v[3] = w[3];
            }
            *reinterpret_cast<u32x4*>(wt + rb * kGroup + lane * 16) = v;
        }
    }
    };
    if (W_PREFETCH) load_wtile();   // lands while the GEMM main loop runs

    u32x4 av[DIRECT ? 1 : A_PER];   // the unaligned kernels stage N through registers
    uint32_t bw[B_PER][WPT];
    float bsc[B_PER][BT::NSC];

    // Uniform bases that advance with the K step plus fixed 32-bit per-thread offsets, as in the projection.  The
    // tile's first code, m0*r, starts a block of 256 (m0 is a multiple of 128, r of 8); the K offset k0 does not,
    // so the index of a code's block scale takes one add and two shifts per step.
    constexpr int A_OFFS = DIRECT ? AD::VARIANTS : A_PER;
    uint32_t a_byte[A_OFFS], b_el[B_PER];   // N: byte offset; P: element offset inside the tile's rows
#pragma unroll
    for (int p = 0; p < A_OFFS; ++p) {
        if constexpr (DIRECT) {
            a_byte[p] = AD::lane_src_bytes(lane, ld, p);
        } else {
            const int ci = t + p * NT;
            a_byte[p] = 2u * (uint32_t)((ci / AD::CPR) * ld + (ci % AD::CPR) * 8);
        }
    }
#pragma unroll
    for (int p = 0; p < B_PER; ++p) {
        const int ti = t + p * NT;
        b_el[p] = (uint32_t)((ti / B_TPR) * r + (ti % B_TPR) * (8 * WPT));
    }
    const int64_t e_tile = (int64_t)m0 * r;

    // Tile kt: N straight into LDS stage `stage` (kExact, kMasked) or into registers (kUnaligned); P codes and scales
    // into registers.
    auto gload = [&](int kt, int stage) {
        const int k0 = kt * BK;
        const uint8_t* nb = reinterpret_cast<const uint8_t*>(N + (int64_t)k0 * ld + n0);
        const uint8_t* pq = Pq + ((e_tile + k0) >> 1);
        const float* ps = Ps + (e_tile >> 8);
        if constexpr (DIRECT) {
            __amdgpu_buffer_rsrc_t rn, rq, rs;
            if constexpr (MODE == kExact) {
                rn = make_rsrc(nb); rq = make_rsrc(pq); rs = make_rsrc(ps);
            } else {   // bounded by the end of each array: rows of N at or past r read as zero (the K tail)
                const int64_t mr = (int64_t)m * r;
                rn = make_rsrc(nb, bound_bytes(((int64_t)(r - k0) * ld - n0) * 2));
                rq = make_rsrc(pq, bound_bytes((mr - e_tile - k0) >> 1));
                rs = make_rsrc(ps, bound_bytes((((mr + kGroup - 1) >> 8) - (e_tile >> 8)) * 4));
            }
#pragma unroll
            for (int p = 0; p < A_PER; ++p)
                buffer_load_lds16(rn, As + stage * S::A_STAGE + AD::load_row0(wave, p) * BNn, a_byte[p % AD::VARIANTS],
                                  2u * (uint32_t)(AD::load_row0(wave, p) * ld));
#pragma unroll
            for (int p = 0; p < B_PER; ++p) {
                buffer_load_words<WPT>(rq, b_el[p] >> 1, bw[p]);
#pragma unroll
                for (int j = 0; j < BT::NSC; ++j)
                    bsc[p][j] = __builtin_bit_cast(
                        float, __builtin_amdgcn_raw_buffer_load_b32(rs, ((b_el[p] + (uint32_t)(k0 + 8 * j)) >> 8) << 2, 0, 0));
            }
        } else {
#pragma unroll
            for (int p = 0; p < A_PER; ++p) {
                const int ci = t + p * NT;
                const int row = ci / AD::CPR, c8 = ci % AD::CPR;
                const int valid = (k0 + row < r) ? (n - (n0 + c8 * 8)) : 0;
                av[p] = load8_bf16_guarded(reinterpret_cast<const uint16_t*>(nb + a_byte[p]), valid);
            }
#pragma unroll
            for (int p = 0; p < B_PER; ++p) {
                const int ti = t + p * NT;
                const int row = ti / B_TPR, c = (ti % B_TPR) * (8 * WPT);
                load_p_guarded<WPT>(Pq + (e_tile >> 1), ps, b_el[p] + (uint32_t)k0, m0 + row < m ? r - (k0 + c) : 0,
                                    bw[p], bsc[p]);
            }
        }
    };
    auto sstore = [&](int stage) {
#pragma unroll
        for (int p = 0; p < B_PER; ++p) {
            const int ti = t + p * NT;
            const int row = ti / B_TPR, c = (ti % B_TPR) * (8 * WPT);
#pragma unroll
            for (int j = 0; j < WPT; ++j)
                *reinterpret_cast<u32x4*>(Bs + stage * S::B_STAGE + row * PB + c + 8 * j) =
                    dequant8_bf16(bw[p][j], bsc[p][DIRECT ? 0 : j]);
        }
        if constexpr (!DIRECT) {
#pragma unroll
            for (int p = 0; p < A_PER; ++p) {
                const int ci = t + p * NT;
                *reinterpret_cast<u32x4*>(As + stage * S::A_STAGE + AD::chunk_offset(ci / AD::CPR, ci % AD::CPR)) = av[p];
            }
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the stage's direct loads have landed
        }
    };

    f32x16 acc[IB][JB];
#pragma unroll
    for (int a = 0; a < IB; ++a)
#pragma unroll
        for (int b = 0; b < JB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    const int lrow = lane & 31, lhalf = lane >> 5;
    int a_lane[IB];
#pragma unroll
    for (int a = 0; a < IB; ++a) a_lane[a] = AD::lane_offset(lane) + ((wn * SN + a * 32) ^ AD::lane_swizzle(lane));
    const int b_lane = (wm * SM + lrow) * PB + 8 * lhalf;
    const int KT = (r + BK - 1) / BK;

    auto mfma_step = [&](int stage) {
        const uint16_t* Ac = As + stage * S::A_STAGE;
        const uint16_t* Bc = Bs + stage * S::B_STAGE + b_lane;
        __builtin_amdgcn_s_setprio(kMfmaPrio);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 af[IB], bf[JB];
#pragma unroll
            for (int a = 0; a < IB; ++a) af[a] = read_kmajor_frag(Ac + kk * 16 * PA + a_lane[a], PA);
#pragma unroll
            for (int b = 0; b < JB; ++b)
                bf[b] = *reinterpret_cast<const bf16x8*>(Bc + b * 32 * PB + kk * 16);
#pragma unroll
            for (int a = 0; a < IB; ++a)
#pragma unroll
                for (int b = 0; b < JB; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bf[b], acc[a][b], 0, 0, 0);
        }
        __builtin_amdgcn_s_setprio(0);
    };

    // unrolled by two (constant LDS stages); loads past the end re-read the last K slab, see the projection
    gload(0, 0);
    sstore(0);
    __syncthreads();
    for (int kt = 0; kt < KT; kt += 2) {
        gload(min(kt + 1, KT - 1), 1);
        mfma_step(0);
        sstore(1);
        __syncthreads();
        gload(min(kt + 2, KT - 1), 0);
        if (kt + 1 < KT) mfma_step(1);
        sstore(0);
        __syncthreads();
    }

    if (!W_PREFETCH) load_wtile();    // the staging buffers are free now (the main loop ends with a barrier)
    // The rows' old scales (and zero points) are fetched together with the weight tile: one wait covers both, where
    // loading them inside the epilogue exposed a second memory latency per tile.
    float s_old_row[JB], z_old_row[ZP ? JB : 1];
#pragma unroll
    for (int b = 0; b < JB; ++b) {
        const int mrow = m0 + wm * SM + b * 32 + (lane & 31);
        const bool row_ok = !RAGGED || mrow < m;
        s_old_row[b] = row_ok ? Ws[(int64_t)mrow * ng + tile_n] : 0.f;
        if constexpr (ZP) z_old_row[b] = row_ok ? Wz[(int64_t)mrow * ng + tile_n] : 0.f;
    }
    // The weight tile's direct loads are counted by vmcnt like any other load.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // ---- epilogue: x = Wq*s - lr*U in place of the accumulators, per-row block absmax ----
    float* smax = reinterpret_cast<float*>(smem);  // [WGn][BMm]; staging buffers are free after the last barrier
    float* smin = smax + WGn * BMm;                // the same for the row minima of the zero-point format
    const float nlra = -(lr * alpha);
    float rowmax[JB];
    float rowmin[ZP ? JB : 1];
#pragma unroll
    for (int b = 0; b < JB; ++b) {
        const int rl = wm * SM + b * 32 + lrow;       // row inside the tile
        const int mrow = m0 + rl;
        const bool row_ok = !RAGGED || mrow < m;
        const float s_old = s_old_row[b];
        float z_old = 0.f;
        if constexpr (ZP) z_old = z_old_row[b];
        float mx = 0.f, mn = 0.f;   // the zero-point range contains zero
        const int wt_lane = wtile_offset(rl, wn * SN + 4 * lhalf);
#pragma unroll
        for (int a = 0; a < IB; ++a)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int col = wn * SN + a * 32 + 8 * v4 + 4 * lhalf;
                const uint32_t w = *reinterpret_cast<const uint32_t*>(wt + (wt_lane ^ wtile_run_bits(a, v4)));
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float code = (float)(int)(int8_t)(w >> (8 * e));
                    const float cw = ZP ? (code - z_old) * s_old : code * s_old;
                    const bool ok = !RAGGED || (row_ok && n0 + col + e < n);
                    if (DUMP_U) {
                        if (ok) Udbg[(int64_t)mrow * n + n0 + col + e] = alpha * acc[a][b][4 * v4 + e];
                    }
                    const float x = ok ? __builtin_fmaf(nlra, acc[a][b][4 * v4 + e], cw) : 0.f;
                    acc[a][b][4 * v4 + e] = x;
                    if constexpr (ZP) {
                        mx = fmaxf(mx, x);
                        mn = fminf(mn, x);
                    } else {
                        mx = fmaxf(mx, fabsf(x));
                    }
                }
            }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        rowmax[b] = mx;
        if (WGn > 1 && lhalf == 0) smax[wn * BMm + rl] = mx;
        if constexpr (ZP) {
            mn = fminf(mn, __shfl_xor(mn, 32, 64));
            rowmin[b] = mn;
            if (WGn > 1 && lhalf == 0) smin[wn * BMm + rl] = mn;
        }
    }
    if (WGn > 1) __syncthreads();

    // ---- new scale, stochastic rounding; the new codes replace the old ones in the LDS tile ----
#pragma unroll
    for (int b = 0; b < JB; ++b) {
        const int rl = wm * SM + b * 32 + lrow;
        const int mrow = m0 + rl;
        const bool row_ok = !RAGGED || mrow < m;
        float amax = rowmax[b];
        if (WGn > 1) {
#pragma unroll
            for (int w = 0; w < WGn; ++w) amax = fmaxf(amax, smax[w * BMm + rl]);
        }
        float s_new, inv, code_bias = 128.0f;   // added to floor(v) before the saturating conversion: 128 (+ z')
        if constexpr (ZP) {
            float amin = rowmin[b];
            if (WGn > 1) {
#pragma unroll
                for (int w = 0; w < WGn; ++w) amin = fminf(amin, smin[w * BMm + rl]);
            }
            const float rng = amax - amin;
            s_new = rng > 0.f ? rng / 255.0f : 0.f;
            inv = rng > 0.f ? 255.0f / rng : 0.f;
            const float z_new = rng > 0.f ? fminf(fmaxf(-128.f - rintf(amin * inv), -128.f), 127.f) : 0.f;
            if (wn == 0 && lhalf == 0 && row_ok) Wz[(int64_t)mrow * ng + tile_n] = z_new;
            code_bias = 128.0f + z_new;
        } else {
            s_new = amax > 0.f ? amax / 127.0f : 0.f;
            inv = amax > 0.f ? 127.0f / amax : 0.f;
        }
        if (wn == 0 && lhalf == 0 && row_ok) Ws[(int64_t)mrow * ng + tile_n] = s_new;
        const uint32_t idx_row = (uint32_t)mrow * (uint32_t)n + (uint32_t)n0;   // m*n < 2^32
        const bool xor_ok = MODE == kExact || (DIRECT && (n & 3) == 0);   // wave-uniform
        const int wt_lane = wtile_offset(rl, wn * SN + 4 * lhalf);
#pragma unroll
        for (int a = 0; a < IB; ++a)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int col = wn * SN + a * 32 + 8 * v4 + 4 * lhalf;
                uint32_t pk = 0;
                // when n is a multiple of 4 the run's first element index is one too: index + e == index | e, and
                // key ^ (index | e) == (key ^ index) ^ e, one xor per element instead of an add and an xor
                const uint32_t run_idx = idx_row + (uint32_t)col;
                const uint32_t run_key = key ^ run_idx;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float tq = acc[a][b][4 * v4 + e] * inv;
                    const uint32_t h = mix32(xor_ok ? run_key ^ (uint32_t)e : key ^ (run_idx + (uint32_t)e));
                    // fl32(tq + u) with u = (h >> 8) * 2^-24: the product is exact, so one fma rounds the same sum
                    const float v = __builtin_fmaf((float)(h >> 8), 0x1p-24f, tq);
                    // clamp(floor(v), -128, 127) as a byte: the saturating float -> u8 conversion of floor(v) + 128
                    // (exact: |v| stays far below 2^23) packs straight into byte e; the bias comes off below
                    pk = __builtin_amdgcn_cvt_pk_u8_f32(floorf(v) + code_bias, e, pk);
                }
                pk ^= 0x80808080u;
                *reinterpret_cast<uint32_t*>(wt + (wt_lane ^ wtile_run_bits(a, v4))) = pk;
            }
    }
    __syncthreads();

    // ---- updated tile -> global, whole 256-byte rows per 16 lanes ----
    if (w_fast) {
#pragma unroll
        for (int i = 0; i < W_ROUNDS; ++i) {
            const int row = (wave * W_ROUNDS + i) * 4 + (lane >> 4), chunk = (lane ^ row) & 15;
            const u32x4 v = *reinterpret_cast<const u32x4*>(wt + row * kGroup + (lane & 15) * 16);
            *reinterpret_cast<u32x4*>(Wq + (int64_t)(m0 + row) * ld + n0 + chunk * 16) = v;
        }
    } else {
#pragma unroll
        for (int i = 0; i < W_ROUNDS; ++i) {
            const int row = (wave * W_ROUNDS + i) * 4 + (lane >> 4), chunk = (lane ^ row) & 15;
            const u32x4 v = *reinterpret_cast<const u32x4*>(wt + row * kGroup + (lane & 15) * 16);
            int8_t* dst = Wq + (int64_t)(m0 + row) * ld + n0 + chunk * 16;
            const int valid = m0 + row < m ? n - (n0 + chunk * 16) : 0;
            if (valid >= 16) {
                *reinterpret_cast<u32x4_align1*>(dst) = v;
            } else {
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    if (j < valid) dst[j] = (int8_t)(v[j >> 2] >> (8 * (j & 3)));
            }
        }
    }
}

template <int BMm, int BK, int WGn, int WGm, int MODE, bool DUMP_U, bool W_PREFETCH = true, int MIN_WG_PER_CU = 1,
          bool ZP = false>
__global__ __launch_bounds__(WGn* WGm * 64, MIN_WG_PER_CU) void k_backproject(const uint8_t* __restrict__ Pq,
                                                               const float* __restrict__ Ps,
                                                               const uint16_t* __restrict__ N,
                                                               int8_t* __restrict__ Wq, float* __restrict__ Ws,
                                                               float* __restrict__ Wz,
                                                               float* __restrict__ Udbg, int m, int n, int ld, int r,
                                                               float alpha, float lr, uint32_t key, uint32_t tiles_m,
                                                               uint32_t tiles) {
    __shared__ __attribute__((aligned(16))) uint16_t smem[BpShape<BMm, BK, WGn, WGm, W_PREFETCH, ZP>::SMEM];
    const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x);
    if (tile >= tiles) return;
    backproject_tile<BMm, BK, WGn, WGm, MODE, DUMP_U, W_PREFETCH, ZP>(Pq, Ps, N, Wq, Ws, Wz, Udbg, m, n, ld, r, (int)(tile % tiles_m) * BMm,
                                                (int)(tile / tiles_m), alpha, lr, key, smem);
}

constexpr int kBpStrip = 16;   // row tiles per strip of the grouped back-projection's tile numbering (8: the same
                               // time; 32: 2 % slower; whole columns of tiles, as before: 1 % slower)

template <int BMm, int BK, int WGn, int WGm, int MODE, bool W_PREFETCH = true, int MIN_WG_PER_CU = 1, bool ZP = false>
__global__ __launch_bounds__(WGn* WGm * 64, MIN_WG_PER_CU) void k_backproject_many(const PlanHeader* __restrict__ plan, int first,
                                                                                   int count, uint32_t tiles,
                                                                                   float alpha, float lr,
                                                                                   uint64_t seed, uint64_t step) {
    __shared__ __attribute__((aligned(16))) uint16_t smem[BpShape<BMm, BK, WGn, WGm, W_PREFETCH, ZP>::SMEM];
    const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x);
    if (tile >= tiles) return;
    const PlanMatrix* mats = plan_matrices(plan) + first;
    const PlanMatrix& d = mats[plan_find(mats, count, tile, [](const PlanMatrix& x) { return x.bp_tile0; })];
    const uint32_t local = tile - d.bp_tile0;
    const uint32_t key = sr_key(seed + (uint64_t)d.index * 0x9E3779B97F4A7C15ull, step, 0u);
    // Tiles are numbered in strips kBpStrip row tiles tall, column tile by column tile inside a strip: the ~100 tiles
    // an XCD has in flight then share the P rows of one strip (1 MB of INT4 at r = 1024) and a few N panels, which
    // fits its 4 MB L2 also when the matrix is tall (86 row tiles at m = 11008: numbered column by column the
    // tiles in flight need all of P, 5.6 MB).
    const uint32_t tiles_n = (uint32_t)((d.n + kGroup - 1) / kGroup);
    const uint32_t strip = local / (kBpStrip * tiles_n), in_strip = local % (kBpStrip * tiles_n);
    const uint32_t strip_rows = min((uint32_t)kBpStrip, d.bp_tiles_m - strip * kBpStrip);
    const uint32_t tile_m = strip * kBpStrip + in_strip % strip_rows, tile_n = in_strip / strip_rows;
    backproject_tile<BMm, BK, WGn, WGm, MODE, false, W_PREFETCH, ZP>(d.Pq, d.Ps, d.N, d.Wq, d.Ws, d.Wz, nullptr, (int)d.m, (int)d.n, (int)d.ld, (int)d.r,
                                                (int)tile_m * BMm, (int)tile_n, alpha, lr, key, smem);
}

}  // namespace qg
