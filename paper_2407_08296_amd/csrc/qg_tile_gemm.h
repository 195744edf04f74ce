// bf16 MFMA GEMM on row-major operands in any of the four orientations, with an INT8 operand dequantized while
// its tile is staged: the kernel of the INT8 linear layer (Appendix A) and of the refresh's Y = G Z^T (Sec. 3.2).
//
// The contraction index of an operand is either its fast (contiguous) index - the operand is then staged as an
// [x][k] tile and read with 16-byte LDS reads - or its slow index - staged as a [k][x] tile and read with the
// transposing LDS reads of the optimizer step's kernels.  Rows may start at any element offset (n = 5461 in the
// LLaMA-1B shapes): chunks are fetched with under-aligned wide loads, element by element only where a chunk
// straddles the edge of the matrix.
#pragma once
#include "qg_common.h"
#include "qg_gemm_kernels.h"

namespace qg {

// (the Z layouts: INT8 with a zero point per block, dequantized as (code - zero) * scale)
enum : int { kBf16KFast = 0, kBf16KSlow = 1, kInt8KFast = 2, kInt8KSlow = 3, kInt8ZKFast = 4, kInt8ZKSlow = 5 };

constexpr int kLinTM = 128;                // output tile: 128 (A's index) x TN (B's index, 256 or 128), 4 waves of 64 x TN/2;
                                           // BK (32 or 64) = contraction depth per step
constexpr int kLinStrip = 8;               // row tiles per strip of the tile numbering

// 16 consecutive INT8 codes starting at `src`, of which the first `valid` lie inside the matrix.
__device__ __forceinline__ u32x4 load16_i8_guarded(const int8_t* src, int valid) {
    if (valid >= 16) return *reinterpret_cast<const u32x4_align1*>(src);
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 16; ++j)
        if (j < valid) w[j >> 2] |= (uint32_t)(uint8_t)src[j] << (8 * (j & 3));
    const u32x4 o = {w[0], w[1], w[2], w[3]};
    return o;
}

// bf16(fl32(code * s)) of the 8 codes in two words; ZP: bf16(fl32((code - z) * s)), the difference being exact
template <bool ZP = false>
__device__ __forceinline__ u32x4 dequant8_i8_bf16(uint32_t c0, uint32_t c1, float s, float z = 0.f) {
    float e[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float a = (float)(int)(int8_t)(c0 >> (8 * j)), b = (float)(int)(int8_t)(c1 >> (8 * j));
        e[j] = ZP ? (a - z) * s : a * s;
        e[4 + j] = ZP ? (b - z) * s : b * s;
    }
    const u32x4 o = {pack_bf16x2(e[0], e[1]), pack_bf16x2(e[2], e[3]), pack_bf16x2(e[4], e[5]), pack_bf16x2(e[6], e[7])};
    return o;
}

// One GEMM operand: a row-major matrix (bf16, or INT8 codes with one fp32 scale per block of 256 elements of a
// row) of which a workgroup needs XT "x" indices starting at x0 (X of them exist) against the contraction index k
// (K of them).  LAYOUT says which of the two is the column (fast) index of the matrix in memory.
struct LinOperand {
    const void* base;
    const float* scales;   // INT8 only: [rows][sgroups]
    int64_t ld;            // row length in elements
    int sgroups;
    const float* zeros = nullptr;   // INT8 with zero points only: [rows][sgroups]
};

// Several GEMMs of one shape in one launch (gridDim.y of them): GEMM z takes its A operand from a[z], its B operand
// strideB_bytes * z past B's base and writes C + strideC * z.  One GEMM: a[0] = A's base, strides 0.
constexpr int kLinBatchMax = 16;
struct LinBatch {
    const void* a[kLinBatchMax];
    int64_t strideB_bytes;
    int64_t strideC;
    int64_t ldc = 0;   // row pitch of C in elements (0: N, dense rows)
};

// Staging of one operand tile: global -> registers (fetch) -> LDS (commit; INT8 is dequantized here).  EXACT: the
// tile lies inside the matrix, K is a whole number of steps and rows are 16-byte aligned - no checks.
template <int LAYOUT, int XT, int BK, bool EXACT, int NT = 256>
struct LinStage {
    static constexpr bool kFast = LAYOUT == kBf16KFast || LAYOUT == kInt8KFast || LAYOUT == kInt8ZKFast;
    static constexpr bool kZero = LAYOUT == kInt8ZKFast || LAYOUT == kInt8ZKSlow;
    static constexpr bool kInt8 = LAYOUT == kInt8KFast || LAYOUT == kInt8KSlow || kZero;
    static constexpr int CH = kInt8 ? 16 : 8;                   // elements per 16-byte chunk (one block scale each)
    static constexpr int CPR = (kFast ? BK : XT) / CH;          // chunks per tile row
    static constexpr int PITCH = kFast ? BK + kPadX : XT + kPadK;   // LDS pitch: [x][k] or [k][x]
    static constexpr int ELEMS = (kFast ? XT : BK) * PITCH;
    static constexpr int PER = XT * BK / CH / NT;               // chunks per thread (NT threads in the workgroup)
    static_assert(XT * BK % (CH * NT) == 0, "tile must divide evenly over the threads");
    u32x4 v[PER];
    float s[kInt8 ? PER : 1];
    float z[kZero ? PER : 1];

    __device__ __forceinline__ void fetch(const LinOperand& op, int x0, int X, int k0, int K) {
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int idx = threadIdx.x + NT * q;
            const int tr = idx / CPR, tc = (idx % CPR) * CH;         // row and first column inside the tile
            const int row = kFast ? x0 + tr : k0 + tr;               // ... and inside the matrix
            const int col = kFast ? k0 + tc : x0 + tc;
            const int rows = kFast ? X : K, cols = kFast ? K : X;
            const int valid = EXACT ? CH : (row < rows ? cols - col : 0);
            const int64_t off = (int64_t)row * op.ld + col;
            if constexpr (kInt8) {
                const int8_t* src = static_cast<const int8_t*>(op.base) + off;
                if constexpr (EXACT) v[q] = *reinterpret_cast<const u32x4*>(src); else v[q] = load16_i8_guarded(src, valid);
                s[q] = valid > 0 ? op.scales[(int64_t)row * op.sgroups + (col >> 8)] : 0.f;
                if constexpr (kZero) z[q] = valid > 0 ? op.zeros[(int64_t)row * op.sgroups + (col >> 8)] : 0.f;
            } else {
                const uint16_t* src = static_cast<const uint16_t*>(op.base) + off;
                if constexpr (EXACT) v[q] = *reinterpret_cast<const u32x4*>(src); else v[q] = load8_bf16_guarded(src, valid);
            }
        }
    }
    __device__ __forceinline__ void commit(uint16_t* tile) const {
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int idx = threadIdx.x + NT * q;
            uint16_t* dst = tile + (idx / CPR) * PITCH + (idx % CPR) * CH;
            if constexpr (kInt8) {
                *reinterpret_cast<u32x4*>(dst) = dequant8_i8_bf16<kZero>(v[q][0], v[q][1], s[q], kZero ? z[q] : 0.f);
                *reinterpret_cast<u32x4*>(dst + 8) = dequant8_i8_bf16<kZero>(v[q][2], v[q][3], s[q], kZero ? z[q] : 0.f);
            } else {
                *reinterpret_cast<u32x4*>(dst) = v[q];
            }
        }
    }
    // MFMA operand fragment of the 32 x indices starting at xb for the 16-deep sub-step kk
    __device__ static __forceinline__ bf16x8 frag(const uint16_t* tile, int xb, int kk, int lane) {
        if constexpr (kFast)
            return *reinterpret_cast<const bf16x8*>(tile + (xb + (lane & 31)) * PITCH + kk * 16 + 8 * (lane >> 5));
        else
            return read_kmajor_frag(tile + kk * 16 * PITCH + xb + kmajor_lane_offset(PITCH, lane), PITCH);
    }
};

// C[M][N] (bf16 or fp32) = sum_k A(i, k) B(k, j) (+ bias[j]); A's x index runs over the rows of C, B's over its
// columns.
// Two LDS stages: while the MFMAs of step kt read stage kt & 1, the operands of step kt + 1 (fetched into registers
// before those MFMAs) are written to the other stage; one barrier per step.
// WM: wave rows of the workgroup (2: 128-row tile, 256 threads, two workgroups per CU; 4: 256-row tile, 512 threads,
// one workgroup per CU - the B tile, and with it the dequantization of an INT8 B operand, is then shared by twice as
// many MFMAs).
template <int AL, int BL, bool EXACT, typename OUT, int TN, int BK, int WM = 2>
__global__ __launch_bounds__(WM * 128, WM == 2 ? 2 : 1) void k_tile_gemm(LinOperand A, LinOperand B,
                                                      const uint16_t* __restrict__ bias,
                                                      OUT* __restrict__ C, int M, int N, int K, int tiles_m, int tiles_n,
                                                      LinBatch batch) {
    constexpr int TM = 64 * WM, NT = 128 * WM;
    using SA = LinStage<AL, TM, BK, EXACT, NT>;
    using SB = LinStage<BL, TN, BK, EXACT, NT>;
    A.base = batch.a[blockIdx.y];
    B.base = static_cast<const char*>(B.base) + batch.strideB_bytes * blockIdx.y;
    C += batch.strideC * blockIdx.y;
    const int64_t ldc = batch.ldc ? batch.ldc : N;
    __shared__ __attribute__((aligned(16))) uint16_t At[2][SA::ELEMS];
    __shared__ __attribute__((aligned(16))) uint16_t Bt[2][SB::ELEMS];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), wm = wave >> 1, wn = wave & 1;
    // Each XCD (own L2) takes a contiguous range of tiles, and tiles are numbered in strips eight row tiles tall,
    // column tile by column tile: the tiles in flight on an XCD share eight A panels and a few B panels.
    const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x);
    if (tile >= (uint32_t)(tiles_m * tiles_n)) return;
    const int strip = (int)(tile / (uint32_t)(kLinStrip * tiles_n)), in_strip = (int)(tile % (uint32_t)(kLinStrip * tiles_n));
    const int strip_rows = min(kLinStrip, tiles_m - strip * kLinStrip);
    const int i0 = (strip * kLinStrip + in_strip % strip_rows) * TM, j0 = (in_strip / strip_rows) * TN;
    SA sa;
    SB sb;
    constexpr int MB = 2, NB = TN / 64;        // 32 x 32 blocks of the wave's 64 x TN/2
    f32x16 acc[MB][NB];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    const int KT = (K + BK - 1) / BK;
    sa.fetch(A, i0, M, 0, K);
    sb.fetch(B, j0, N, 0, K);
    sa.commit(At[0]);
    sb.commit(Bt[0]);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < KT;
        if (more) {
            sa.fetch(A, i0, M, (kt + 1) * BK, K);
            sb.fetch(B, j0, N, (kt + 1) * BK, K);
        }
        __builtin_amdgcn_s_setprio(kMfmaPrio);     // the wave in its MFMA phase goes first (two workgroups per CU)
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 af[MB], bf[NB];
#pragma unroll
            for (int a = 0; a < MB; ++a) af[a] = SA::frag(At[cur], wm * 64 + a * 32, kk, lane);
#pragma unroll
            for (int b = 0; b < NB; ++b) bf[b] = SB::frag(Bt[cur], wn * (TN / 2) + b * 32, kk, lane);
#pragma unroll
            for (int a = 0; a < MB; ++a)
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bf[b], acc[a][b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);     // fragments of one sub-step at a time
        }
        __builtin_amdgcn_s_setprio(0);
        if (more) {
            sa.commit(At[cur ^ 1]);
            sb.commit(Bt[cur ^ 1]);
        }
        __syncthreads();
    }
    // register v of a 32 x 32 block: row 8 (v / 4) + 4 (l / 32) + v % 4 (A's index), column l % 32 (B's index)
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int col = j0 + wn * (TN / 2) + b * 32 + (lane & 31);
            const bool col_ok = EXACT || col < N;
            const float bj = (bias != nullptr && col_ok) ? __builtin_bit_cast(float, (uint32_t)bias[col] << 16) : 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = i0 + wm * 64 + a * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const float x = acc[a][b][v];
                if (EXACT || (row < M && col_ok)) {
                    if constexpr (sizeof(OUT) == 4) C[(int64_t)row * ldc + col] = x + bj;
                    else C[(int64_t)row * ldc + col] = to_bf16(x + bj);
                }
            }
        }
}

// Both operands bf16 with the contraction index as their slow index, whole tiles and aligned rows (grad_W at the
// LLaMA shapes): the staging of the optimizer step's projection kernel for its gradient operand, applied to both -
// direct global -> LDS loads into unpadded swizzled [k][x] tiles (no staging registers, no LDS write instructions),
// two stages, the loads of step k+1 issued ahead of the MFMAs of step k, three workgroups per CU.
template <typename OUT>
__global__ __launch_bounds__(256, 3) void k_gemm_kslow_direct(const uint16_t* __restrict__ A, const uint16_t* __restrict__ B,
                                                              OUT* __restrict__ C, int M, int N, int K, int tiles_m,
                                                              int tiles_n) {
    constexpr int TN = 256, BK = 32;
    const int64_t ldc = N;   // dense operands and output only
    using AD = KMajorSwizzled<kLinTM, BK, 256>;
    using BD = KMajorSwizzled<TN, BK, 256>;
    __shared__ __attribute__((aligned(16))) uint16_t As[2][AD::STAGE];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BD::STAGE];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), wm = wave >> 1, wn = wave & 1;
    const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x);
    if (tile >= (uint32_t)(tiles_m * tiles_n)) return;
    const int strip = (int)(tile / (uint32_t)(kLinStrip * tiles_n)), in_strip = (int)(tile % (uint32_t)(kLinStrip * tiles_n));
    const int strip_rows = min(kLinStrip, tiles_m - strip * kLinStrip);
    const int i0 = (strip * kLinStrip + in_strip % strip_rows) * kLinTM, j0 = (in_strip / strip_rows) * TN;
    static_assert(AD::VARIANTS == 1 && BD::VARIANTS == 2, "per-lane source offsets below");
    const uint32_t a_byte = AD::lane_src_bytes(lane, M, 0);
    const uint32_t b_byte[2] = {BD::lane_src_bytes(lane, N, 0), BD::lane_src_bytes(lane, N, 1)};
    auto gload = [&](int kt, int stage) {
        const __amdgpu_buffer_rsrc_t ra = make_rsrc(A + (int64_t)kt * BK * M + i0);
        const __amdgpu_buffer_rsrc_t rb = make_rsrc(B + (int64_t)kt * BK * N + j0);
#pragma unroll
        for (int p = 0; p < AD::PER; ++p)
            buffer_load_lds16(ra, As[stage] + AD::load_row0(wave, p) * kLinTM, a_byte, 2u * (uint32_t)(AD::load_row0(wave, p) * M));
#pragma unroll
        for (int p = 0; p < BD::PER; ++p)
            buffer_load_lds16(rb, Bs[stage] + BD::load_row0(wave, p) * TN, b_byte[p % 2], 2u * (uint32_t)(BD::load_row0(wave, p) * N));
    };
    constexpr int MB = 2, NB = 4;
    f32x16 acc[MB][NB];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    int a_lane[MB], b_lane[NB];
#pragma unroll
    for (int a = 0; a < MB; ++a) a_lane[a] = AD::lane_offset(lane) + ((wm * 64 + a * 32) ^ AD::lane_swizzle(lane));
#pragma unroll
    for (int b = 0; b < NB; ++b) b_lane[b] = BD::lane_offset(lane) + ((wn * 128 + b * 32) ^ BD::lane_swizzle(lane));
    auto mfma_step = [&](int stage) {
        __builtin_amdgcn_s_setprio(kMfmaPrio);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 af[MB], bf[NB];
#pragma unroll
            for (int a = 0; a < MB; ++a) af[a] = read_kmajor_frag(As[stage] + kk * 16 * kLinTM + a_lane[a], kLinTM);
#pragma unroll
            for (int b = 0; b < NB; ++b) bf[b] = read_kmajor_frag(Bs[stage] + kk * 16 * TN + b_lane[b], TN);
#pragma unroll
            for (int a = 0; a < MB; ++a)
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bf[b], acc[a][b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_s_setprio(0);
    };
    auto landed = [] { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };   // direct loads count like any other load
    const int KT = K / BK;
    // unrolled by two: constant LDS stages; loads past the end re-read the last K slab (in bounds, never consumed)
    gload(0, 0);
    landed();
    __syncthreads();
    for (int kt = 0; kt < KT; kt += 2) {
        gload(min(kt + 1, KT - 1), 1);
        mfma_step(0);
        landed();
        __syncthreads();
        gload(min(kt + 2, KT - 1), 0);
        if (kt + 1 < KT) mfma_step(1);
        landed();
        __syncthreads();
    }
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int col = j0 + wn * 128 + b * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = i0 + wm * 64 + a * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const float x = acc[a][b][v];
                if constexpr (sizeof(OUT) == 4) C[(int64_t)row * ldc + col] = x;
                else C[(int64_t)row * ldc + col] = to_bf16(x);
            }
        }
}

// bf16 [X][64] operand tile (rows along the contraction index, 128 bytes each) filled by direct global -> LDS loads:
// one wave-wide 16-byte-per-lane load deposits 1 KB = 8 rows, lane l at row l / 8, chunk position l % 8.  Rows are
// not padded; bank spreading comes from a swizzle on the source side: position p of row x holds the row's chunk
// p ^ (x & 7), so the 8 rows that 8 consecutive lanes of a fragment read touch (same chunk) sit at 8 different
// positions.  X rows over NW waves.
template <int XT, int NW>
struct KFastDirect {
    static constexpr int BK = 64, ROW = BK;                 // elements per tile row
    static constexpr int ELEMS = XT * BK;
    static constexpr int PER = XT / 8 / NW;                 // wave-wide loads per wave
    static_assert(XT % (8 * NW) == 0, "tile rows must divide evenly over the waves");
    // byte offset, from the tile's first element (row pitch ld elements), of the chunk lane `lane` fetches in the
    // load that covers rows [8 q, 8 q + 8): the same for every q
    __device__ static __forceinline__ uint32_t lane_src_bytes(int lane, int64_t ld) {
        const int row = lane >> 3, chunk = (lane & 7) ^ row;
        return (uint32_t)(2 * (row * ld + chunk * 8));
    }
    // element offset of the fragment of lane `lane` for the 32 rows starting at xb (a multiple of 32), sub-step kk
    __device__ static __forceinline__ int frag_offset(int xb, int kk, int lane) {
        const int row = xb + (lane & 31), chunk = (2 * kk + (lane >> 5)) ^ (lane & 7);
        return row * ROW + chunk * 8;
    }
};

// C = A B^T-style product for operands whose contraction index is fast in both: A bf16 through direct loads, B INT8
// dequantized through registers.  256 x 256 tile, 64-deep steps, eight waves (64 x 128 each), whole tiles only:
// M % 256 = N % 256 = K % 64 = 0, rows of A and B 16-byte aligned.  (With a bf16 B through direct loads as well the
// refresh's G Z^T ran 0.5 % slower than through k_tile_gemm: a wave's fragment reads queue behind its own pending
// direct loads, and with both operands direct nothing else is left to overlap them with.  With an INT8 B the direct
// A loads pay: about 4 % on the forward pass of a 7B layer and on grad_input on transposed storage.  With an INT8 B
// whose contraction index is slow, grad_input, they made it 1.5 % slower: that case stays in k_tile_gemm.)
template <int BL, typename OUT>
__global__ __launch_bounds__(512, 1) void k_gemm_kfast_direct(LinOperand A, LinOperand B, const uint16_t* __restrict__ bias,
                                                              OUT* __restrict__ C, int M, int N, int K, int tiles_m,
                                                              int tiles_n, LinBatch batch) {
    constexpr int TM = 256, TN = 256, BK = 64, NW = 8;
    static_assert(BL == kInt8KFast || BL == kInt8ZKFast, "B: INT8 with the contraction index fast");
    using AD = KFastDirect<TM, NW>;
    using SB = LinStage<BL, TN, BK, true, 512>;
    __shared__ __attribute__((aligned(16))) uint16_t As[2][AD::ELEMS];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][SB::ELEMS];
    A.base = batch.a[blockIdx.y];
    B.base = static_cast<const char*>(B.base) + batch.strideB_bytes * blockIdx.y;
    C += batch.strideC * blockIdx.y;
    const int64_t ldc = batch.ldc ? batch.ldc : N;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), wm = wave >> 1, wn = wave & 1;
    const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x);
    if (tile >= (uint32_t)(tiles_m * tiles_n)) return;
    const int strip = (int)(tile / (uint32_t)(kLinStrip * tiles_n)), in_strip = (int)(tile % (uint32_t)(kLinStrip * tiles_n));
    const int strip_rows = min(kLinStrip, tiles_m - strip * kLinStrip);
    const int i0 = (strip * kLinStrip + in_strip % strip_rows) * TM, j0 = (in_strip / strip_rows) * TN;
    const uint16_t* Ag = static_cast<const uint16_t*>(A.base) + (int64_t)i0 * A.ld;
    const uint32_t a_byte = AD::lane_src_bytes(lane, A.ld);
    SB sb;
    auto gload = [&](int kt, int stage) {
        const __amdgpu_buffer_rsrc_t ra = make_rsrc(Ag + kt * BK);
#pragma unroll
        for (int p = 0; p < AD::PER; ++p) {
            const int row0 = (wave * AD::PER + p) * 8;
            buffer_load_lds16(ra, As[stage] + row0 * AD::ROW, a_byte, 2u * (uint32_t)(row0 * A.ld));
        }
        sb.fetch(B, j0, N, kt * BK, K);
    };
    constexpr int MB = 2, NB = 4;
    f32x16 acc[MB][NB];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    auto mfma_step = [&](int stage) {
        __builtin_amdgcn_s_setprio(kMfmaPrio);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 af[MB], bf[NB];
#pragma unroll
            for (int a = 0; a < MB; ++a)
                af[a] = *reinterpret_cast<const bf16x8*>(As[stage] + AD::frag_offset(wm * 64 + a * 32, kk, lane));
#pragma unroll
            for (int b = 0; b < NB; ++b) bf[b] = SB::frag(Bs[stage], wn * 128 + b * 32, kk, lane);
#pragma unroll
            for (int a = 0; a < MB; ++a)
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bf[b], acc[a][b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_s_setprio(0);
    };
    auto landed = [] { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };   // direct loads count like any other load
    const int KT = K / BK;
    // two LDS stages; the loads of step kt + 1 are issued before the MFMAs of step kt and land in the other stage
    gload(0, 0);
    sb.commit(Bs[0]);
    landed();
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < KT;
        if (more) gload(kt + 1, cur ^ 1);
        mfma_step(cur);
        if (more) sb.commit(Bs[cur ^ 1]);
        landed();
        __syncthreads();
    }
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int col = j0 + wn * 128 + b * 32 + (lane & 31);
            const float bj = bias != nullptr ? __builtin_bit_cast(float, (uint32_t)bias[col] << 16) : 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = i0 + wm * 64 + a * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const float x = acc[a][b][v] + bj;
                if constexpr (sizeof(OUT) == 4) C[(int64_t)row * ldc + col] = x;
                else C[(int64_t)row * ldc + col] = to_bf16(x);
            }
        }
}

template <int AL, int BL, typename OUT, int TN, int BK, int WM = 2>
static void launch_tile_gemm_shape(const LinOperand& A, const LinOperand& B, const uint16_t* bias, OUT* C, int64_t M,
                                   int64_t N, int64_t K, hipStream_t st, const LinBatch* many, int count, int64_t ldc) {
    constexpr int TM = 64 * WM;
    const int64_t tiles_m = (M + TM - 1) / TM, tiles_n = (N + TN - 1) / TN;
    const dim3 grid((unsigned)((tiles_m * tiles_n + 7) / 8 * 8), (unsigned)count);   // x: a multiple of the 8 XCDs
    LinBatch batch;
    if (many != nullptr) {
        batch = *many;
    } else {
        batch.a[0] = A.base;
        batch.strideB_bytes = 0;
        batch.strideC = 0;
    }
    batch.ldc = ldc;
    // no checks at all when every tile and every step is whole and rows start 16-byte aligned
    const bool exact = M % TM == 0 && N % TN == 0 && K % BK == 0 && A.ld % 8 == 0 && B.ld % 16 == 0;
    if (exact)
        hipLaunchKernelGGL((k_tile_gemm<AL, BL, true, OUT, TN, BK, WM>), grid, dim3(128 * WM), 0, st, A, B, bias, C, (int)M,
                           (int)N, (int)K, (int)tiles_m, (int)tiles_n, batch);
    else
        hipLaunchKernelGGL((k_tile_gemm<AL, BL, false, OUT, TN, BK, WM>), grid, dim3(128 * WM), 0, st, A, B, bias, C, (int)M,
                           (int)N, (int)K, (int)tiles_m, (int)tiles_n, batch);
}

// Tile shape, from measurements on the linear layer of the LLaMA-7B shapes (ms per decoder layer at 4096 tokens):
//  * large outputs with an INT8 B operand, or with the contraction index fast in both operands: 256 x 256 tiles with
//    64-deep steps, eight waves, one workgroup per CU (144 KB of LDS).  The B tile - and the dequantization of an
//    INT8 B - is shared by twice as many MFMAs as in a 128-row tile, global traffic per MFMA halves, and 64-deep
//    steps fetch whole cache lines of operands whose rows run along k.  Forward pass 2.24 -> 1.87, grad_input
//    1.82 -> 1.66 (256 x 256 x 32 with eight waves: 1.72; 256 x 128 x 64: forward unchanged at 2.24).
//  * otherwise two workgroups of four waves per CU: 128 x 128 x 64 when both operands have k fast (2.28 against 2.37
//    for 128 x 256 x 32 and 2.80 for 128 x 128 x 32 on the forward pass), 128 x 256 x 32 when that fills the chip,
//    128 x 128 x 32 for small outputs.
template <int AL, int BL, typename OUT>
// ldc: row pitch of C in elements (0: N).
static int launch_tile_gemm(const LinOperand& A, const LinOperand& B, const uint16_t* bias, OUT* C, int64_t M, int64_t N,
                            int64_t K, hipStream_t st, const LinBatch* many = nullptr, int count = 1, int64_t ldc = 0) {
    constexpr bool both_fast = (AL == kBf16KFast || AL == kInt8KFast || AL == kInt8ZKFast) &&
                               (BL == kBf16KFast || BL == kInt8KFast || BL == kInt8ZKFast);
    if constexpr (AL == kBf16KSlow && BL == kBf16KSlow) {
        const int64_t tiles_m = M / kLinTM, tiles_n = N / 256;
        if (many == nullptr && M % kLinTM == 0 && N % 256 == 0 && K % 32 == 0 && bias == nullptr &&
            tiles_m * tiles_n >= 512 && K >= 32 && A.ld == M && B.ld == N && (ldc == 0 || ldc == N)) {
            const unsigned grid = (unsigned)((tiles_m * tiles_n + 7) / 8 * 8);
            hipLaunchKernelGGL((k_gemm_kslow_direct<OUT>), dim3(grid), dim3(256), 0, st, static_cast<const uint16_t*>(A.base),
                               static_cast<const uint16_t*>(B.base), C, (int)M, (int)N, (int)K, (int)tiles_m, (int)tiles_n);
            return check_launch();
        }
    }
    constexpr bool int8_b = BL == kInt8KFast || BL == kInt8KSlow || BL == kInt8ZKFast || BL == kInt8ZKSlow;
    if constexpr (int8_b || both_fast) {
        if (M >= 1024 && ((M + 255) / 256) * ((N + 255) / 256) * count >= 256) {   // at least one workgroup per CU
            if constexpr (AL == kBf16KFast && (BL == kInt8KFast || BL == kInt8ZKFast)) {
                // whole tiles and aligned rows: the bf16 operand goes straight into LDS
                if (M % 256 == 0 && N % 256 == 0 && K % 64 == 0 && A.ld % 8 == 0 && B.ld % 16 == 0) {
                    const int64_t tiles_m = M / 256, tiles_n = N / 256;
                    const dim3 grid((unsigned)((tiles_m * tiles_n + 7) / 8 * 8), (unsigned)count);
                    LinBatch batch;
                    if (many != nullptr) {
                        batch = *many;
                    } else {
                        batch.a[0] = A.base;
                        batch.strideB_bytes = 0;
                        batch.strideC = 0;
                    }
                    batch.ldc = ldc;
                    hipLaunchKernelGGL((k_gemm_kfast_direct<BL, OUT>), grid, dim3(512), 0, st, A, B, bias, C, (int)M, (int)N,
                                       (int)K, (int)tiles_m, (int)tiles_n, batch);
                    return check_launch();
                }
            }
            launch_tile_gemm_shape<AL, BL, OUT, 256, 64, 4>(A, B, bias, C, M, N, K, st, many, count, ldc);
            return check_launch();
        }
    }
    if constexpr (both_fast)
        launch_tile_gemm_shape<AL, BL, OUT, 128, 64>(A, B, bias, C, M, N, K, st, many, count, ldc);
    else if (((M + kLinTM - 1) / kLinTM) * ((N + 255) / 256) * count >= 512)
        launch_tile_gemm_shape<AL, BL, OUT, 256, 32>(A, B, bias, C, M, N, K, st, many, count, ldc);
    else
        launch_tile_gemm_shape<AL, BL, OUT, 128, 32>(A, B, bias, C, M, N, K, st, many, count, ldc);
    return check_launch();
}

}  // namespace qg
