// Subspace refresh (Sec. 3.2: the projection matrix is recomputed from the current gradient; the paper takes the
// first r left singular vectors from an SVD).  Here one pass of orthogonal iteration started from the stored INT4
// projection replaces the SVD:
//     R = dequant(P)^T G  (the projection kernel of the optimizer step)      bf16 MFMA
//     Z = bf16(R)
//     Y = G Z^T           (m x r)                                            bf16 MFMA, fp32 accumulation (qg_tile_gemm.h)
//     Q = Y T^-1          with Y = Q T, T upper triangular, diag(T) > 0      fp64 MFMA (Cholesky QR)
//     P <- quant_int4(Q)  (Sec. 3.3)
// followed by the cosine check of Sec. 3.2 between the old and the new P.
//
// The orthonormalisation works on the r x r Gram matrix S = Y^T Y in fp64: S = L L^T (blocked Cholesky, 64-wide
// blocks), X = L^-1, Q = Y X^T, and all of that a second time on the result (Cholesky QR twice): one round leaves
// |Q^T Q - I| ~ 1e-16 * cond(Y)^2, which for the low-rank-plus-noise gradients this is made for (cond(Y) up to 1e7)
// is far from orthonormal; the second round starts from a matrix with cond ~ 1 and lands within fp32 rounding of
// the Gram-Schmidt factor, because multiplying Y from the right by a triangular matrix with a positive diagonal
// does not change that factor.  Each Gram matrix gets a shift of 2^-46 of its trace on the diagonal, which keeps
// the first round's pivots positive for cond(Y) well beyond 1e8 at no cost in the result.  A column that is
// numerically dependent on its predecessors (a last-round pivot no larger than the shift) is reported through
// `info`; every kernel runs to completion whatever the data.
#include <type_traits>

#include "qg_cossim.h"
#include "qg_tile_gemm.h"

namespace qg {

int launch_project_batch(const ProjBatch& batch, int count, float* R, int64_t strideR, int64_t m, int64_t n, int64_t ld,
                         int64_t r, hipStream_t stream);   // qg_gemm.hip
int launch_project(const uint8_t* Pq, const float* Ps, const uint16_t* G, float* R, int64_t m, int64_t n, int64_t ld,
                   int64_t r, hipStream_t stream);        // qg_gemm.hip

typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef double f64x2 __attribute__((ext_vector_type(2)));

constexpr int kNB = 64;               // block size of the fp64 kernels: one workgroup (4 waves) per 64 x 64 block
constexpr int kKC = 16;               // K extent staged in LDS per barrier pair: 20 KB of LDS per workgroup, so that six
                                      // or more are resident per CU (the fp64 matrix pipe sustains more with more waves
                                      // per SIMD; 32 gave three workgroups and 9 % more time, 8 no further gain)
constexpr int kPitchKF = kKC + 1;     // LDS pitch of a [64][k] chunk (k fastest): odd, so that the 16 rows a fragment
                                      // read touches at one k fall on 16 different bank pairs (36 gave 4-way conflicts)
constexpr int kPitchKS = kNB + 16;    // LDS pitch of a [k][64] chunk (k slowest)
constexpr int kPitchT = kNB + 2;      // LDS pitch of a 64 x 64 intermediate

// ROWS x COLS block at (row0, col0) of a row-major matrix (fp32 or fp64) -> registers -> LDS doubles.  Elements
// outside [0, rows) x [0, cols) read as zero.  col0 and cols are even, so an element pair never straddles the edge.
template <int ROWS, int COLS, int PITCH, typename T>
struct BlockStage {
    static constexpr int PER = ROWS * COLS / 2 / 256;
    static_assert(ROWS * COLS % 512 == 0, "256 threads, two elements each");
    double v[PER][2];
    __device__ __forceinline__ void fetch(const T* __restrict__ src, int64_t ld, int row0, int col0, int rows, int cols) {
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int idx = threadIdx.x + 256 * q;
            const int gr = row0 + idx / (COLS / 2), gc = col0 + (idx % (COLS / 2)) * 2;
            v[q][0] = v[q][1] = 0.0;
            if (gr < rows && gc < cols) {
                typedef T pair_t __attribute__((ext_vector_type(2)));
                const pair_t p = *reinterpret_cast<const pair_t*>(src + (int64_t)gr * ld + gc);
                v[q][0] = (double)p[0];
                v[q][1] = (double)p[1];
            }
        }
    }
    __device__ __forceinline__ void commit(double* dst) const {
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int idx = threadIdx.x + 256 * q;
            double* d = dst + (idx / (COLS / 2)) * PITCH + (idx % (COLS / 2)) * 2;
            d[0] = v[q][0];
            d[1] = v[q][1];
        }
    }
};

// One K chunk of the workgroup's 64 x 64 product on the fp64 matrix cores.  Wave (wi, wj) owns the 32 x 32 quadrant
// as 2 x 2 blocks of v_mfma_f64_16x16x4: lane l supplies A[i = l % 16][k = l / 16] and B[k = l / 16][j = l % 16];
// register v of the result is element (i = 4 v + l / 16, j = l % 16).  Operand element (i, k) of A sits at
// At[i * a_pi + k * a_pk], element (k, j) of B at Bt[j * b_pj + k * b_pk].
__device__ __forceinline__ void mma_chunk(const double* At, int a_pi, int a_pk, const double* Bt, int b_pj, int b_pk,
                                          f64x4 (&acc)[2][2], int lane, int wi, int wj) {
    const double* ap = At + (wi * 32 + (lane & 15)) * a_pi + (lane >> 4) * a_pk;
    const double* bp = Bt + (wj * 32 + (lane & 15)) * b_pj + (lane >> 4) * b_pk;
#pragma unroll
    for (int k0 = 0; k0 < kKC; k0 += 4) {
        double af[2], bf[2];
#pragma unroll
        for (int a = 0; a < 2; ++a) af[a] = ap[a * 16 * a_pi + k0 * a_pk];
#pragma unroll
        for (int b = 0; b < 2; ++b) bf[b] = bp[b * 16 * b_pj + k0 * b_pk];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_f64_16x16x4f64(af[a], bf[b], acc[a][b], 0, 0, 0);
    }
}

__device__ __forceinline__ void zero_acc(f64x4 (&acc)[2][2]) {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = f64x4{0.0, 0.0, 0.0, 0.0};
}

// f(row, col, value) for every element of the wave's quadrant, row and col inside the 64 x 64 block.
template <typename F>
__device__ __forceinline__ void for_each_acc(const f64x4 (&acc)[2][2], int lane, int wi, int wj, F f) {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) f(wi * 32 + a * 16 + 4 * v + (lane >> 4), wj * 32 + b * 16 + (lane & 15), acc[a][b][v]);
}

// A batch of matrices with the same m and r runs through the fp64 kernels in one launch each, matrix b =
// blockIdx.z; its pieces sit at these element strides from matrix 0's (all zero for a single matrix).  The in and
// out matrices of a round share the stride Y/Q (both are m x r fp32 arrays of the same batch layout).
struct BatchStride {
    int64_t Y, Q, S, X, D, part, shift;
};

// 1 / sqrt(d) for d > 0 to fp64 accuracy: the hardware estimate and two Newton steps (the correctly rounded sqrt
// and divide of the library cost an order of magnitude more instructions, on the critical path of every column).
__device__ __forceinline__ double rsqrt_f64(double d) {
    double y = __builtin_amdgcn_rsq(d);
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const double e = fma(-d * y, y, 1.0);      // 1 - d y^2
        y = fma(0.5 * y, e, y);
    }
    return y;
}

// (bi, bj) with bi >= bj of the idx-th block of a lower block triangle, rows first.
__device__ __forceinline__ void lower_pair(int idx, int& bi, int& bj) {
    int i = 0;
    while ((i + 1) * (i + 2) / 2 <= idx) ++i;
    bi = i;
    bj = idx - i * (i + 1) / 2;
}

// ---------------------------------------------------------------------------------------------------------------
// Z = bf16(R), round to nearest even
// ---------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_f32_to_bf16(const float* __restrict__ x, uint16_t* __restrict__ y, int64_t quads) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < quads; i += (int64_t)gridDim.x * 256) {
        const f32x4 v = reinterpret_cast<const f32x4*>(x)[i];
        u32x2 o;
        o[0] = pack_bf16x2(v[0], v[1]);
        o[1] = pack_bf16x2(v[2], v[3]);
        reinterpret_cast<u32x2*>(y)[i] = o;
    }
}

// Energy that each column of a projection captures from the gradient: e[z][k] = sum_j R_z[k][j]^2 with
// R_z = P_z^T G_z (r rows of n elements, pitch ld, matrix z at R + z * strideR).  One workgroup per row; every thread
// adds its elements in index order, the 256 partial sums are added by a fixed tree: deterministic.
__global__ __launch_bounds__(256) void k_row_energy(const float* __restrict__ R, int64_t strideR, int n, int ld, int r,
                                                    float* __restrict__ e) {
    __shared__ float sh[256];
    const float* row = R + (int64_t)blockIdx.y * strideR + (int64_t)blockIdx.x * ld;
    float acc = 0.f;
    for (int j = threadIdx.x; j < n; j += 256) acc = __builtin_fmaf(row[j], row[j], acc);
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) e[(int64_t)blockIdx.y * r + blockIdx.x] = sh[0];
}

__global__ void k_set_i32(int32_t* p, int32_t v, int count) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = v;
}

// ---------------------------------------------------------------------------------------------------------------
// S = Y^T Y in fp64, lower block triangle only (Y fp32 m x r; S r x r row-major).  The m rows are cut into
// gridDim.y slices so that the launch fills the chip; slice s writes its partial sums to part + s * r * r and
// k_gram_reduce adds the slices in a fixed order (the result does not depend on scheduling).
// ---------------------------------------------------------------------------------------------------------------
constexpr int kGramMaxSlices = 8;

__global__ __launch_bounds__(256) void k_gram(const float* __restrict__ Y, double* __restrict__ part, int m, int r,
                                              int slice_rows, BatchStride st) {
    Y += blockIdx.z * st.Y;
    part += blockIdx.z * st.part;
    __shared__ double At[kKC * kPitchKS];
    __shared__ double Bt[kKC * kPitchKS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wi = wave >> 1, wj = wave & 1;
    int bi, bj;
    lower_pair(blockIdx.x, bi, bj);
    const bool diag = bi == bj;
    const int k_begin = blockIdx.y * slice_rows, k_end = min(m, k_begin + slice_rows);
    double* S = part + (int64_t)blockIdx.y * r * r;
    BlockStage<kKC, kNB, kPitchKS, float> sa, sb;
    f64x4 acc[2][2];
    zero_acc(acc);
    sa.fetch(Y, r, k_begin, bi * kNB, k_end, r);
    if (!diag) sb.fetch(Y, r, k_begin, bj * kNB, k_end, r);
    for (int k0 = k_begin; k0 < k_end; k0 += kKC) {
        sa.commit(At);
        if (!diag) sb.commit(Bt);
        __syncthreads();
        if (k0 + kKC < k_end) {
            sa.fetch(Y, r, k0 + kKC, bi * kNB, k_end, r);
            if (!diag) sb.fetch(Y, r, k0 + kKC, bj * kNB, k_end, r);
        }
        mma_chunk(At, 1, kPitchKS, diag ? At : Bt, 1, kPitchKS, acc, lane, wi, wj);
        __syncthreads();
    }
    for_each_acc(acc, lane, wi, wj, [&](int row, int col, double x) {
        const int gi = bi * kNB + row, gj = bj * kNB + col;
        if (gi < r && gj < r) S[(int64_t)gi * r + gj] = x;
    });
}

__global__ __launch_bounds__(256) void k_gram_reduce(const double* __restrict__ part, double* __restrict__ S, int r,
                                                     int slices, BatchStride st) {
    part += blockIdx.z * st.part;
    S += blockIdx.z * st.S;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (int64_t)r * r) return;
    const int i = (int)(e / r), j = (int)(e % r);
    if (j / kNB > i / kNB) return;                 // above the lower block triangle: never written, never read
    double sum = 0.0;
    for (int s = 0; s < slices; ++s) sum += part[(int64_t)s * r * r + e];
    S[e] = sum;
}

// S += sigma I with sigma = 2^-46 trace(S) (at least 128 units of fp64 roundoff of the largest eigenvalue): keeps
// the pivots of a Gram matrix with cond(Y) beyond ~1e8 positive.  The shift changes L, not the factor Q in exact
// arithmetic (Y X^T for any triangular X with a positive diagonal has the same Gram-Schmidt factor); the second
// round, on a matrix with a far smaller condition number, removes what it costs in orthogonality.  sigma is kept
// for the pivot check of k_chol_diag.
__global__ __launch_bounds__(256) void k_gram_shift(double* __restrict__ S, int r, double* __restrict__ shift, BatchStride st) {
    __shared__ double red[256];
    S += blockIdx.z * st.S;
    shift += blockIdx.z * st.shift;
    const int t = threadIdx.x;
    double acc = 0.0;
    for (int i = t; i < r; i += 256) acc += S[(int64_t)i * r + i];
    red[t] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (t < w) red[t] += red[t + w];
        __syncthreads();
    }
    const double sigma = red[0] > 0.0 ? 0x1p-46 * red[0] : 0.0;
    for (int i = t; i < r; i += 256) S[(int64_t)i * r + i] += sigma;
    if (t == 0) shift[0] = sigma;
}

// ---------------------------------------------------------------------------------------------------------------
// Blocked Cholesky S = L L^T in place (lower triangle), right-looking, one block column per step kb:
//   k_chol_diag:   L_kk from the diagonal block, and X_kk = L_kk^-1 (to Dinv[kb] and to the diagonal block of X)
//   k_chol_panel:  L_ik = S_ik X_kk^T for the blocks below
//   k_chol_update: S_ij -= L_ik L_jk^T for i >= j > kb
// Rows and columns at or past r (r not a multiple of 64) behave like an identity block.  A pivot that is not positive
// is replaced by 1 so that the factorization runs to completion whatever the data.
// ---------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_chol_diag(double* __restrict__ S, int r, int kb, double* __restrict__ Dinv,
                                                   double* __restrict__ X, int32_t* __restrict__ info,
                                                   const double* __restrict__ shift, double flag_factor, BatchStride st) {
    // a pivot at or below flag_factor * sigma is reported: 0 in the first round (only pivots that are not positive),
    // 16 in the last, where a pivot that small is the shift alone, i.e. a column that is numerically dependent
    const double floor_d = flag_factor * shift[blockIdx.z * st.shift];
    S += blockIdx.z * st.S;
    Dinv += blockIdx.z * st.D;
    X += blockIdx.z * st.X;
    info += blockIdx.z;
    constexpr int P = kNB + 1;
    __shared__ double T[kNB * P];
    __shared__ double dg[kNB], rdg[kNB];
    const int t = threadIdx.x;
    const int base = kb * kNB;
    for (int e = t; e < kNB * kNB; e += 256) {     // consecutive threads along a row
        const int i = e >> 6, c = e & 63;
        const int gi = base + i, gc = base + c;
        T[i * P + c] = (gi < r && gc < r) ? S[(int64_t)gi * r + gc] : (i == c ? 1.0 : 0.0);
    }
    const int i = t & 63, cg = t >> 6;              // row i, columns cg, cg + 4, ...
    for (int j = 0; j < kNB; ++j) {
        __syncthreads();
        double d = T[j * P + j];
        if (!(d > floor_d)) {                       // too small, not positive, or NaN
            if (t == 0 && base + j < r) atomicCAS(info, 0, base + j + 1);
            if (!(d > 0.0)) d = 1.0;
        }
        const double rs = rsqrt_f64(d);             // column j is scaled by 1 / L_jj, kept for the inverse below
        if (cg == 0) {
            if (i > j) T[i * P + j] *= rs;
            if (i == j) {
                dg[j] = d * rs;                     // T[j][j] itself stays until every thread has read it
                rdg[j] = rs;
            }
        }
        __syncthreads();
        // row i loses lij * L[c][j] in its columns c = c0, c0 + 4, ... <= i.  Unrolled to a fixed count that depends
        // on j alone, with every LDS read issued before the first use (clamped addresses, predicated stores): as a
        // loop with a data-dependent trip count each iteration waited out its own LDS round trip.
        const double lij = T[i * P + j];
        const int c0 = j + 1 + ((cg - (j + 1)) & 3);
        auto update = [&](auto qn) {
            constexpr int QN = decltype(qn)::value;
            double a[QN], b[QN];
#pragma unroll
            for (int q = 0; q < QN; ++q) {
                const int cc = min(c0 + 4 * q, kNB - 1);
                a[q] = T[i * P + cc];
                b[q] = T[cc * P + j];
            }
#pragma unroll
            for (int q = 0; q < QN; ++q) {
                const int c = c0 + 4 * q;
                if (c <= i) T[i * P + c] = a[q] - lij * b[q];
            }
        };
        const int need = (kNB - 1 - j + 3) >> 2;    // columns left of the four column groups, rounded up
        if (need > 12) update(std::integral_constant<int, 16>());
        else if (need > 8) update(std::integral_constant<int, 12>());
        else if (need > 4) update(std::integral_constant<int, 8>());
        else update(std::integral_constant<int, 4>());
    }
    __syncthreads();
    if (t < kNB) T[t * P + t] = dg[t];
    __syncthreads();
    for (int e = t; e < kNB * kNB; e += 256) {
        const int ii = e >> 6, c = e & 63;
        if (c <= ii && base + ii < r) S[(int64_t)(base + ii) * r + base + c] = T[ii * P + c];
    }
    // X = L^-1 by forward substitution on all 64 columns of the identity at once, right-looking: once row j of X is
    // final, every later row's residual loses its L[i][j] X[j][.] term.  The residuals (and then X) live transposed
    // in the strict upper triangle of T, which the factor does not use: X[i][c] at T[c][i] for c < i; the diagonal
    // of X is 1 / L_jj (rdg).
    for (int e = t; e < kNB * kNB; e += 256) {
        const int ii = e >> 6, c = e & 63;
        if (c > ii) T[ii * P + c] = 0.0;
    }
    for (int j = 0; j < kNB; ++j) {
        __syncthreads();
        const double xjj = rdg[j];
        if (t < j) T[t * P + j] *= xjj;             // row j of X: residual / L_jj
        __syncthreads();
        if (i > j) {
            const double lij = T[i * P + j];
            auto update = [&](auto qn) {            // rows c = cg, cg + 4, ... <= j of X^T, as in the factorization
                constexpr int QN = decltype(qn)::value;
                double a[QN], b[QN];
#pragma unroll
                for (int q = 0; q < QN; ++q) {
                    const int cc = min(cg + 4 * q, kNB - 1);
                    a[q] = T[cc * P + i];
                    b[q] = T[cc * P + j];
                }
#pragma unroll
                for (int q = 0; q < QN; ++q) {
                    const int c = cg + 4 * q;
                    if (c <= j) T[c * P + i] = a[q] - lij * (c < j ? b[q] : xjj);
                }
            };
            const int need = (j >> 2) + 1;
            if (need > 12) update(std::integral_constant<int, 16>());
            else if (need > 8) update(std::integral_constant<int, 12>());
            else if (need > 4) update(std::integral_constant<int, 8>());
            else update(std::integral_constant<int, 4>());
        }
    }
    __syncthreads();
    for (int e = t; e < kNB * kNB; e += 256) {
        const int ii = e >> 6, c = e & 63;
        const double x = c < ii ? T[c * P + ii] : (c == ii ? rdg[ii] : 0.0);
        Dinv[(int64_t)kb * kNB * kNB + e] = x;
        if (base + ii < r && base + c < r) X[(int64_t)(base + ii) * r + base + c] = x;
    }
}

__global__ __launch_bounds__(256) void k_chol_panel(double* __restrict__ S, int r, int kb, const double* __restrict__ Dinv,
                                                    BatchStride st) {
    S += blockIdx.z * st.S;
    Dinv += blockIdx.z * st.D;
    __shared__ double At[kNB * kPitchKF];
    __shared__ double Bt[kNB * kPitchKF];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wi = wave >> 1, wj = wave & 1;
    const int ib = kb + 1 + blockIdx.x;
    const double* D = Dinv + (int64_t)kb * kNB * kNB;
    BlockStage<kNB, kKC, kPitchKF, double> sa, sb;
    f64x4 acc[2][2];
    zero_acc(acc);
    sa.fetch(S, r, ib * kNB, kb * kNB, r, r);
    sb.fetch(D, kNB, 0, 0, kNB, kNB);
    for (int kc = 0; kc < kNB; kc += kKC) {
        sa.commit(At);
        sb.commit(Bt);
        __syncthreads();
        if (kc + kKC < kNB) {
            sa.fetch(S, r, ib * kNB, kb * kNB + kc + kKC, r, r);
            sb.fetch(D, kNB, 0, kc + kKC, kNB, kNB);
        }
        mma_chunk(At, kPitchKF, 1, Bt, kPitchKF, 1, acc, lane, wi, wj);
        __syncthreads();
    }
    for_each_acc(acc, lane, wi, wj, [&](int row, int col, double x) {
        const int gi = ib * kNB + row, gj = kb * kNB + col;
        if (gi < r && gj < r) S[(int64_t)gi * r + gj] = x;
    });
}

__global__ __launch_bounds__(256) void k_chol_update(double* __restrict__ S, int r, int kb, BatchStride st) {
    S += blockIdx.z * st.S;
    __shared__ double At[kNB * kPitchKF];
    __shared__ double Bt[kNB * kPitchKF];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wi = wave >> 1, wj = wave & 1;
    int pi, pj;
    lower_pair(blockIdx.x, pi, pj);
    const int ib = kb + 1 + pi, jb = kb + 1 + pj;
    BlockStage<kNB, kKC, kPitchKF, double> sa, sb;
    f64x4 acc[2][2];
    zero_acc(acc);
    sa.fetch(S, r, ib * kNB, kb * kNB, r, r);
    sb.fetch(S, r, jb * kNB, kb * kNB, r, r);
    for (int kc = 0; kc < kNB; kc += kKC) {
        sa.commit(At);
        sb.commit(Bt);
        __syncthreads();
        if (kc + kKC < kNB) {
            sa.fetch(S, r, ib * kNB, kb * kNB + kc + kKC, r, r);
            sb.fetch(S, r, jb * kNB, kb * kNB + kc + kKC, r, r);
        }
        mma_chunk(At, kPitchKF, 1, Bt, kPitchKF, 1, acc, lane, wi, wj);
        __syncthreads();
    }
    for_each_acc(acc, lane, wi, wj, [&](int row, int col, double x) {
        const int gi = ib * kNB + row, gj = jb * kNB + col;
        if (gi < r && gj < r) S[(int64_t)gi * r + gj] -= x;
    });
}

// ---------------------------------------------------------------------------------------------------------------
// X = L^-1, block row ib (all block rows above are complete):  X_ik = -X_ii (sum_{j=k}^{i-1} L_ij X_jk),  k < i
// ---------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_trinv_row(const double* __restrict__ S, double* __restrict__ X,
                                                   const double* __restrict__ Dinv, int r, int ib, BatchStride st) {
    S += blockIdx.z * st.S;
    X += blockIdx.z * st.X;
    Dinv += blockIdx.z * st.D;
    // phase 1: At (L chunk, k fast) and Bt (X chunk, k slow); phase 2: Tm (the sum) and At (X_ii chunk)
    __shared__ double At[kNB * kPitchKF];
    __shared__ double Bt[kNB * kPitchT];
    static_assert(kNB * kPitchT >= kKC * kPitchKS, "the intermediate reuses the X chunk's buffer");
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wi = wave >> 1, wj = wave & 1;
    const int kb = blockIdx.x;
    f64x4 acc[2][2];
    zero_acc(acc);
    BlockStage<kNB, kKC, kPitchKF, double> sa;
    BlockStage<kKC, kNB, kPitchKS, double> sb;
    const double* D = Dinv + (int64_t)ib * kNB * kNB;
    const int k_end = ib * kNB;
    sa.fetch(S, r, ib * kNB, kb * kNB, r, r);
    sb.fetch(X, r, kb * kNB, kb * kNB, r, r);
    for (int kc = kb * kNB; kc < k_end; kc += kKC) {
        sa.commit(At);
        sb.commit(Bt);
        __syncthreads();
        if (kc + kKC < k_end) {
            sa.fetch(S, r, ib * kNB, kc + kKC, r, r);
            sb.fetch(X, r, kc + kKC, kb * kNB, r, r);
        } else {
            sa.fetch(D, kNB, 0, 0, kNB, kNB);     // first chunk of the second product
        }
        mma_chunk(At, kPitchKF, 1, Bt, 1, kPitchKS, acc, lane, wi, wj);
        __syncthreads();
    }
    double* Tm = Bt;
    for_each_acc(acc, lane, wi, wj, [&](int row, int col, double x) { Tm[row * kPitchT + col] = x; });
    zero_acc(acc);
    for (int kc = 0; kc < kNB; kc += kKC) {
        sa.commit(At);
        __syncthreads();       // also publishes Tm on the first pass
        if (kc + kKC < kNB) sa.fetch(D, kNB, 0, kc + kKC, kNB, kNB);
        mma_chunk(At, kPitchKF, 1, Tm + kc * kPitchT, 1, kPitchT, acc, lane, wi, wj);
        __syncthreads();
    }
    for_each_acc(acc, lane, wi, wj, [&](int row, int col, double x) {
        const int gi = ib * kNB + row, gj = kb * kNB + col;
        if (gi < r && gj < r) X[(int64_t)gi * r + gj] = -x;
    });
}

// ---------------------------------------------------------------------------------------------------------------
// Q = Y X^T (X lower triangular: column block jb needs the contraction index up to the end of that block only)
// ---------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_apply(const float* __restrict__ Y, const double* __restrict__ X,
                                               float* __restrict__ Q, int m, int r, BatchStride st) {
    Y += blockIdx.z * st.Y;
    X += blockIdx.z * st.X;
    Q += blockIdx.z * st.Q;
    __shared__ double At[kNB * kPitchKF];
    __shared__ double Bt[kNB * kPitchKF];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wi = wave >> 1, wj = wave & 1;
    const int a0 = blockIdx.x * kNB, jb = blockIdx.y;
    const int kend = min(r, (jb + 1) * kNB);
    BlockStage<kNB, kKC, kPitchKF, float> sa;
    BlockStage<kNB, kKC, kPitchKF, double> sb;
    f64x4 acc[2][2];
    zero_acc(acc);
    sa.fetch(Y, r, a0, 0, m, r);
    sb.fetch(X, r, jb * kNB, 0, r, r);
    for (int kc = 0; kc < kend; kc += kKC) {
        sa.commit(At);
        sb.commit(Bt);
        __syncthreads();
        if (kc + kKC < kend) {
            sa.fetch(Y, r, a0, kc + kKC, m, r);
            sb.fetch(X, r, jb * kNB, kc + kKC, r, r);
        }
        mma_chunk(At, kPitchKF, 1, Bt, kPitchKF, 1, acc, lane, wi, wj);
        __syncthreads();
    }
    for_each_acc(acc, lane, wi, wj, [&](int row, int col, double x) {
        const int gi = a0 + row, gj = jb * kNB + col;
        if (gi < m && gj < r) Q[(int64_t)gi * r + gj] = (float)x;
    });
}

static size_t align256(size_t b) { return (b + 255) & ~size_t(255); }

// Number of row slices of the Gram kernel: a function of the shape only (never of the batch size), so that a
// matrix gets bit-identical results alone and inside a batch.  About two workgroups per CU for a single matrix,
// at least 256 rows per slice.
static int gram_slices(int64_t m, int64_t r, int* slice_rows) {
    const int nt = (int)((r + kNB - 1) / kNB);
    const int pairs = nt * (nt + 1) / 2;
    int slices = (512 + pairs - 1) / pairs;
    const int by_rows = (int)((m + 255) / 256);
    slices = slices < by_rows ? slices : by_rows;
    slices = slices < kGramMaxSlices ? slices : kGramMaxSlices;
    *slice_rows = (int)(((m + slices - 1) / slices + kKC - 1) / kKC) * kKC;
    return (int)((m + *slice_rows - 1) / *slice_rows);
}

// Workspace of the orthonormalisation of `batch` matrices of one shape: per matrix S and X (r x r fp64), the
// inverted diagonal blocks, the result of the first round T (fp32 m x r) and the Gram slices.
struct OrthLayout {
    size_t S, X, Dinv, T, part, shift, total;
    BatchStride st;   // element strides between consecutive matrices; st.Y = st.Q = stride of T
};
static OrthLayout orth_layout(int64_t m, int64_t r, int64_t batch) {
    const int64_t nt = (r + kNB - 1) / kNB;
    int slice_rows;
    const int slices = gram_slices(m, r, &slice_rows);
    const size_t bS = align256((size_t)r * r * 8), bD = align256((size_t)nt * kNB * kNB * 8),
                 bT = align256((size_t)m * r * 4), bP = align256((size_t)slices * r * r * 8);
    OrthLayout L;
    L.S = 0;
    L.X = L.S + bS * batch;
    L.Dinv = L.X + bS * batch;
    L.T = L.Dinv + bD * batch;
    L.part = L.T + bT * batch;
    L.shift = L.part + bP * batch;
    L.total = L.shift + 256 * (size_t)batch;     // one double per matrix, 256 bytes apart
    L.st = BatchStride{(int64_t)(bT / 4), (int64_t)(bT / 4), (int64_t)(bS / 8), (int64_t)(bS / 8), (int64_t)(bD / 8),
                       (int64_t)(bP / 8), 256 / 8};
    return L;
}

// Workspace of the refresh of `batch` matrices of one shape: R and Z of the matrix in flight (shared: the
// per-matrix launches are ordered on the stream), per matrix Y (which also receives Q), then the orthonormalisation's
// and the cosine check's.
// The two GEMMs that precede the orthonormalisation (R = P^T G, Y = G Z^T) run over groups of up to kRefreshGroup
// matrices per launch, so R and Z are held for that many matrices; Y, Q and the Cholesky QR for the whole batch.
constexpr int kRefreshGroup = 16;
static_assert(kRefreshGroup <= kProjBatchMax && kRefreshGroup <= kLinBatchMax && kRefreshGroup <= kCosBatchMax, "group size");
struct RefreshLayout {
    size_t R, Z, Y, orth, cos, wts, total;
    size_t y_bytes;   // per matrix
    size_t r_bytes, z_bytes;
    int group;        // matrices per GEMM launch
};
// n: elements per row of R and Z as stored, i.e. the row pitch of the gradients.
static RefreshLayout refresh_layout(int64_t m, int64_t n, int64_t r, int64_t batch) {
    RefreshLayout L;
    L.group = (int)(batch < kRefreshGroup ? batch : kRefreshGroup);
    L.y_bytes = align256((size_t)m * r * 4);
    const size_t slice = ((size_t)r * n + 127) / 128 * 128;   // elements per matrix of R and of Z: the same count, so
    L.r_bytes = slice * 4;                                     // that one conversion launch maps R onto Z slice by slice
    L.z_bytes = slice * 2;
    L.R = 0;
    L.Z = L.R + L.r_bytes * L.group;
    L.Y = L.Z + L.z_bytes * L.group;
    L.orth = L.Y + 2 * L.y_bytes * batch;        // Y and Q of every matrix
    L.cos = L.orth + orth_layout(m, r, batch).total;
    L.wts = L.cos + align256(cossim_batch_workspace_bytes(m, r, L.group));
    L.total = L.wts + align256((size_t)L.group * r * 4);   // the columns' captured energies, one group at a time
    return L;
}

static int check_mr(int64_t m, int64_t r) {
    if (m <= 0 || r <= 0 || (r & 7) || r > m || m >= (int64_t(1) << 31) / r) return QG_ERR_SHAPE;
    return QG_OK;
}

// Y = G Z^T: G m x n and Z r x n, both bf16 with the contraction index n as their fast index; Y fp32 m x r.
// ldg, ldz: row pitches of G and Z in elements.
static int launch_range(const uint16_t* G, const uint16_t* Z, float* Y, int64_t m, int64_t n, int64_t ldg, int64_t ldz,
                        int64_t r, hipStream_t st) {
    const LinOperand A = {G, nullptr, ldg, 0}, B = {Z, nullptr, ldz, 0};
    return launch_tile_gemm<kBf16KFast, kBf16KFast, float>(A, B, nullptr, Y, m, r, n, st);
}

// One round on `batch` matrices (matrix b at Y + b * sYin, result at Q + b * sQout): Q = Y L^-T with L the Cholesky
// factor of Y^T Y.
static void launch_cholqr(const float* Y, int64_t sYin, float* Q, int64_t sQout, int64_t m, int64_t r, int batch,
                          int32_t* info, double flag_factor, char* ws, const OrthLayout& L, hipStream_t stream) {
    double* S = reinterpret_cast<double*>(ws + L.S);
    double* X = reinterpret_cast<double*>(ws + L.X);
    double* Dinv = reinterpret_cast<double*>(ws + L.Dinv);
    double* part = reinterpret_cast<double*>(ws + L.part);
    double* shift = reinterpret_cast<double*>(ws + L.shift);
    BatchStride st = L.st;
    st.Y = sYin;
    st.Q = sQout;
    const int nt = (int)((r + kNB - 1) / kNB);
    const int pairs = nt * (nt + 1) / 2;
    int slice_rows;
    const int slices = gram_slices(m, r, &slice_rows);
    const dim3 blk(256);
    const unsigned B = (unsigned)batch;
    hipLaunchKernelGGL(k_gram, dim3(pairs, slices, B), blk, 0, stream, Y, part, (int)m, (int)r, slice_rows, st);
    hipLaunchKernelGGL(k_gram_reduce, dim3((unsigned)((r * r + 255) / 256), 1, B), blk, 0, stream, part, S, (int)r, slices, st);
    hipLaunchKernelGGL(k_gram_shift, dim3(1, 1, B), blk, 0, stream, S, (int)r, shift, st);
    for (int kb = 0; kb < nt; ++kb) {
        hipLaunchKernelGGL(k_chol_diag, dim3(1, 1, B), blk, 0, stream, S, (int)r, kb, Dinv, X, info, shift, flag_factor, st);
        const int below = nt - kb - 1;
        if (below > 0) {
            hipLaunchKernelGGL(k_chol_panel, dim3(below, 1, B), blk, 0, stream, S, (int)r, kb, Dinv, st);
            hipLaunchKernelGGL(k_chol_update, dim3(below * (below + 1) / 2, 1, B), blk, 0, stream, S, (int)r, kb, st);
        }
    }
    for (int ib = 1; ib < nt; ++ib)
        hipLaunchKernelGGL(k_trinv_row, dim3(ib, 1, B), blk, 0, stream, S, X, Dinv, (int)r, ib, st);
    hipLaunchKernelGGL(k_apply, dim3((unsigned)((m + kNB - 1) / kNB), nt, B), blk, 0, stream, Y, X, Q, (int)m, (int)r, st);
}

// Cholesky QR twice: Y -> T -> Q.  info: `batch` consecutive device ints.
static int launch_orth(const float* Y, int64_t sY, float* Q, int64_t sQ, int64_t m, int64_t r, int batch, int32_t* info,
                       bool reset_info, char* ws, hipStream_t stream) {
    const OrthLayout L = orth_layout(m, r, batch);
    float* T = reinterpret_cast<float*>(ws + L.T);
    if (reset_info)
        hipLaunchKernelGGL(k_set_i32, dim3((batch + 255) / 256), dim3(256), 0, stream, info, 0, batch);
    launch_cholqr(Y, sY, T, L.st.Y, m, r, batch, info, 0.0, ws, L, stream);
    launch_cholqr(T, L.st.Y, Q, sQ, m, r, batch, info, 16.0, ws, L, stream);
    return check_launch();
}

static int launch_to_bf16(const float* R, uint16_t* Z, int64_t count, hipStream_t st) {
    const int64_t quads = count / 4, blocks = (quads + 255) / 256;
    hipLaunchKernelGGL(k_f32_to_bf16, dim3((unsigned)(blocks < 65536 ? blocks : 65536)), dim3(256), 0, st, R, Z, quads);
    return check_launch();
}

}  // namespace qg

using namespace qg;

extern "C" int qg_range_apply(const uint16_t* G_bf16, const uint16_t* Z_bf16, int64_t m, int64_t n, int64_t r, float* Y,
                              void* stream) {
    if (!G_bf16 || !Z_bf16 || !Y) return QG_ERR_NULL;
    if (int e = check_mr(m, r)) return e;
    if (n <= 0 || m * n >= (int64_t(1) << 32) || r * n >= (int64_t(1) << 32)) return QG_ERR_SHAPE;
    if (!aligned16(G_bf16) || !aligned16(Z_bf16) || !aligned16(Y)) return QG_ERR_ALIGN;
    return launch_range(G_bf16, Z_bf16, Y, m, n, n, n, r, (hipStream_t)stream);
}

extern "C" size_t qg_orthonormalize_workspace_bytes(int64_t m, int64_t r) {
    if (check_mr(m, r) != QG_OK) return 0;
    return orth_layout(m, r, 1).total;
}

extern "C" int qg_orthonormalize(const float* Y, int64_t m, int64_t r, float* Q, int32_t* info, void* workspace,
                                 size_t workspace_bytes, void* stream) {
    if (!Y || !Q || !info) return QG_ERR_NULL;
    if (int e = check_mr(m, r)) return e;
    if (!aligned16(Y) || !aligned16(Q) || !aligned16(workspace) || (reinterpret_cast<uintptr_t>(info) & 3)) return QG_ERR_ALIGN;
    if (Y == Q) return QG_ERR_SHAPE;
    if (!workspace || workspace_bytes < orth_layout(m, r, 1).total) return QG_ERR_WORKSPACE;
    return launch_orth(Y, 0, Q, 0, m, r, 1, info, true, static_cast<char*>(workspace), (hipStream_t)stream);
}

static int check_ld(int64_t m, int64_t n, int64_t r, int64_t ld) {
    if (n <= 0 || ld < n || (ld != n && (ld & 15))) return QG_ERR_SHAPE;
    if (m * ld >= (int64_t(1) << 32) || r * ld >= (int64_t(1) << 32)) return QG_ERR_SHAPE;
    return QG_OK;
}

extern "C" size_t qg_refresh_workspace_bytes(int count, int64_t m, int64_t n, int64_t r) {
    if (count < 1 || check_mr(m, r) != QG_OK || check_ld(m, n, r, n) != QG_OK) return 0;
    return refresh_layout(m, n, r, count).total;
}

extern "C" int qg_subspace_refresh_many_ld(int count, const qg_refresh_desc* descs, int64_t m, int64_t n, int64_t ld,
                                           int64_t r, int group, int passes, float* cos_out, int32_t* info,
                                           void* workspace, size_t workspace_bytes, void* stream) {
    if (!descs || !cos_out || !info) return QG_ERR_NULL;
    if (count < 1 || passes < 1 || passes > 64) return QG_ERR_SHAPE;
    if (int e = check_mr(m, r)) return e;
    if (ld == 0) ld = n;
    if (int e = check_ld(m, n, r, ld)) return e;
    if (group != kGroup) return QG_ERR_GROUP;
    if (!aligned16(workspace) || (reinterpret_cast<uintptr_t>(cos_out) & 3) || (reinterpret_cast<uintptr_t>(info) & 3))
        return QG_ERR_ALIGN;
    for (int i = 0; i < count; ++i) {
        const qg_refresh_desc& d = descs[i];
        if (!d.Pq || !d.Ps || !d.G || !d.Pq_new || !d.Ps_new) return QG_ERR_NULL;
        if (!aligned16(d.Pq) || !aligned16(d.Ps) || !aligned16(d.G) || !aligned16(d.Pq_new) || !aligned16(d.Ps_new))
            return QG_ERR_ALIGN;
        if (d.Pq == d.Pq_new || d.Ps == d.Ps_new) return QG_ERR_SHAPE;   // the cosine check needs the old P intact
    }
    if (!workspace) return QG_ERR_WORKSPACE;
    // as many matrices per batch as the workspace holds; R and Z are stored with the gradients' row pitch
    int batch = count < 32768 ? count : 32768;   // the batch index is a grid dimension
    while (batch > 1 && refresh_layout(m, ld, r, batch).total > workspace_bytes) batch = (batch + 1) / 2;
    const RefreshLayout L = refresh_layout(m, ld, r, batch);
    if (L.total > workspace_bytes) return QG_ERR_WORKSPACE;
    char* ws = static_cast<char*>(workspace);
    float* R = reinterpret_cast<float*>(ws + L.R);
    uint16_t* Z = reinterpret_cast<uint16_t*>(ws + L.Z);
    float* Y = reinterpret_cast<float*>(ws + L.Y);
    float* Q = reinterpret_cast<float*>(ws + L.Y + L.y_bytes * batch);
    float* wts = reinterpret_cast<float*>(ws + L.wts);
    const int64_t sY = (int64_t)(L.y_bytes / 4);
    hipStream_t st = (hipStream_t)stream;
    const int64_t sR = (int64_t)(L.r_bytes / 4);
    // R_b = dequant(P_b)^T G_b for the `ng` matrices from descriptor `d0` on, into the R slices
    auto project_group = [&](const qg_refresh_desc* d0, int ng, bool new_p) -> int {
        if (ng == 1) {   // one matrix: the single-matrix launch (smaller tiles, lower latency)
            return launch_project(new_p ? d0->Pq_new : d0->Pq, new_p ? d0->Ps_new : d0->Ps, d0->G, R, m, n, ld, r, st);
        }
        ProjBatch pb;
        for (int b = 0; b < kRefreshGroup; ++b) {   // unused slots: valid pointers, never dereferenced
            const qg_refresh_desc& d = d0[b < ng ? b : 0];
            pb.Pq[b] = new_p ? d.Pq_new : d.Pq;
            pb.Ps[b] = new_p ? d.Ps_new : d.Ps;
            pb.G[b] = d.G;
        }
        return launch_project_batch(pb, ng, R, sR, m, n, ld, r, st);
    };
    for (int first = 0; first < count; first += batch) {
        const int nb = count - first < batch ? count - first : batch;
        for (int pass = 0; pass < passes; ++pass) {
            for (int g0 = 0; g0 < nb; g0 += L.group) {
                const int ng = nb - g0 < L.group ? nb - g0 : L.group;
                const qg_refresh_desc* d0 = descs + first + g0;
                if (int e = project_group(d0, ng, pass > 0)) return e;
                // the slices of R and of Z hold the same number of elements
                if (int e = launch_to_bf16(R, Z, sR * (ng - 1) + r * ld, st)) return e;
                if (ng == 1) {
                    if (int e = launch_range(d0->G, Z, Y + g0 * sY, m, n, ld, ld, r, st)) return e;
                    continue;
                }
                LinBatch lb;
                for (int b = 0; b < kRefreshGroup; ++b) lb.a[b] = d0[b < ng ? b : 0].G;
                lb.strideB_bytes = (int64_t)L.z_bytes;
                lb.strideC = sY;
                const LinOperand A = {d0->G, nullptr, ld, 0}, B = {Z, nullptr, ld, 0};
                if (int e = launch_tile_gemm<kBf16KFast, kBf16KFast, float>(A, B, nullptr, Y + g0 * sY, m, r, n, st, &lb, ng))
                    return e;
            }
            if (int e = launch_orth(Y, sY, Q, sY, m, r, nb, info + first, pass == 0, ws + L.orth, st)) return e;
            for (int b = 0; b < nb; ++b) {
                const qg_refresh_desc& d = descs[first + b];
                if (int e = qg_quant_int4(Q + b * sY, m, r, group, d.Pq_new, d.Ps_new, stream)) return e;
            }
        }
        // the convergence check: column cosines of the old and the new projection, each weighted with the energy of
        // the gradient that the new column captures (squared row norms of R_new = dequant(P_new)^T G)
        for (int g0 = 0; g0 < nb; g0 += L.group) {
            const int ng = nb - g0 < L.group ? nb - g0 : L.group;
            const qg_refresh_desc* d0 = descs + first + g0;
            if (int e = project_group(d0, ng, true)) return e;
            hipLaunchKernelGGL(k_row_energy, dim3((unsigned)r, (unsigned)ng), dim3(256), 0, st, (const float*)R, sR, (int)n,
                               (int)ld, (int)r, wts);
            if (int e = check_launch()) return e;
            CosBatch cb;
            for (int b = 0; b < kCosBatchMax; ++b) {   // unused slots repeat the first pair
                const qg_refresh_desc& d = d0[b < ng ? b : 0];
                cb.PqA[b] = d.Pq; cb.PsA[b] = d.Ps; cb.PqB[b] = d.Pq_new; cb.PsB[b] = d.Ps_new;
            }
            if (int e = launch_cossim_batch(cb, ng, m, r, cos_out + first + g0, reinterpret_cast<float*>(ws + L.cos), st,
                                            wts, r))
                return e;
        }
    }
    return QG_OK;
}

extern "C" int qg_subspace_refresh_many(int count, const qg_refresh_desc* descs, int64_t m, int64_t n, int64_t r, int group,
                                        int passes, float* cos_out, int32_t* info, void* workspace,
                                        size_t workspace_bytes, void* stream) {
    return qg_subspace_refresh_many_ld(count, descs, m, n, n, r, group, passes, cos_out, info, workspace, workspace_bytes,
                                       stream);
}

extern "C" int qg_subspace_refresh(const uint8_t* Pq, const float* Ps, const uint16_t* G_bf16, int64_t m, int64_t n,
                                   int64_t r, int group, int passes, uint8_t* Pq_new, float* Ps_new, float* cos_out,
                                   int32_t* info, void* workspace, size_t workspace_bytes, void* stream) {
    const qg_refresh_desc d = {Pq, Ps, G_bf16, Pq_new, Ps_new};
    return qg_subspace_refresh_many(1, &d, m, n, r, group, passes, cos_out, info, workspace, workspace_bytes, stream);
}
