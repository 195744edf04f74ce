/*
 * libqgalore - the per-weight-matrix Q-GaLore optimizer step for AMD MI355X (gfx950).
 *
 * C ABI.  Conventions that hold for every entry point unless stated otherwise:
 *
 *  - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *    never allocates, frees or retains device memory; scratch space is passed
 *    in as `workspace` (size from the matching *_workspace_bytes query).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls enqueue work and return WITHOUT synchronising.
 *  - All matrices are dense row-major with leading dimension = row length
 *    (the *_ld entry points and the grouped descriptors take a row pitch).
 *    Base pointers must be 16-byte aligned (QG_ERR_ALIGN otherwise).
 *  - Notation (the paper's): W is the m x n weight, G the m x n gradient,
 *    P the m x r projection matrix, R = P^T G (r x n), M and V the Adam moments
 *    (r x n), N the Adam direction (r x n), U = alpha P N (m x n), t the 1-based
 *    step count.
 *  - `group` is the quantization block size; only 256 (the paper's value,
 *    Sec. 3.1) is accepted, anything else returns QG_ERR_GROUP.
 *  - INT8 weight format: codes int8 [m][n]; one fp32 scale per block of 256
 *    consecutive elements OF A ROW, scales [m][ceil(n/256)] (a row's last block
 *    is short when n % 256 != 0).  Symmetric: zero point 0, scale = absmax/127.
 *  - INT4 projection format: block = 256 consecutive elements of the FLATTENED
 *    row-major m x r array, scales [ceil(m*r/256)], scale = absmax/7.  Two
 *    codes per byte, flat element 2b in the low nibble of byte b, stored
 *    nibble = code + 8.
 *  - bf16 tensors are passed as uint16_t bit patterns.
 *  - Sizes are positive: an empty tensor (m, n, r or an element count of 0) is
 *    an argument error (QG_ERR_SHAPE), not a no-op; m * n must stay below 2^32
 *    (the stochastic-rounding stream and the kernels index elements with 32
 *    bits), r is a multiple of 8 and at most m.
 *  - Return value: QG_OK or a QG_ERR_* code.  Arguments are validated before
 *    any HIP call, so argument errors are reported even with no GPU present.
 *    After QG_ERR_HIP, qg_last_hip_error() returns the hipError_t value.
 */
#ifndef QGALORE_H
#define QGALORE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    QG_OK = 0,
    QG_ERR_NULL = 1,       /* a required pointer is NULL */
    QG_ERR_SHAPE = 2,      /* m, n, r, count, step out of range (see each call) */
    QG_ERR_GROUP = 3,      /* group != 256 */
    QG_ERR_ALIGN = 4,      /* a base pointer is not 16-byte aligned */
    QG_ERR_WORKSPACE = 5,  /* workspace missing or too small */
    QG_ERR_HIP = 6         /* a HIP call or kernel launch failed */
};

/* Adam and GaLore hyper-parameters (Sec. 4.1: Adam as the inner optimizer,
 * scale factor alpha = 0.25). */
typedef struct {
    float beta1, beta2, eps, lr, alpha;
} qg_hparams;

/* Per-layer state of the adaptive lazy subspace update (Sec. 3.2). */
typedef struct {
    int interval;      /* current refresh interval t (steps) */
    int streak;        /* consecutive checks with cos >= threshold */
    int k;             /* checks in a row required before the interval doubles */
    int next_refresh;  /* step at which the next refresh is due */
    float threshold;   /* 0.4 in the paper */
    float last_cos;
} qg_policy;

/* One matrix of a grouped step (qg_step_many).  All pointers are device
 * pointers with the layouts of the single-matrix calls, except for the optional row pitch `ld`. */
typedef struct {
    int64_t m, n, r;
    const uint8_t*  Pq;   /* INT4 P, packed            */
    const float*    Ps;   /* INT4 P block scales        */
    const uint16_t* G;    /* bf16 gradient m x n        */
    int8_t*         Wq;   /* INT8 weight codes, in/out  */
    float*          Ws;   /* INT8 weight scales, in/out */
    float*          M;    /* first moment r x n, in/out */
    float*          V;    /* second moment r x n, in/out*/
    float*          R;    /* projected gradient r x n, out; may be NULL (not written then) */
    uint16_t*       N;    /* bf16 Adam direction r x n, out */
    int64_t         ld;   /* row pitch, in elements, of EVERY n-wide array above (G, Wq: m rows; M, V, R, N: r rows).
                             0 or n: dense rows.  Otherwise >= n and a multiple of 16: rows then start 16-byte aligned
                             whatever n is, which takes a matrix with n % 8 != 0 (n = 5461 in the LLaMA-1B shapes) off
                             the slow under-aligned path.  Every array holds rows * ld elements.  Padding columns are never read for a
                             result; they are not written either, with two exceptions: N goes out as pairs of columns (an
                             odd n overwrites the first padding column of N), and the unfused qg_lowrank_adam_many runs
                             over the padding of M, V, N as well. */
    float*          Wz;   /* zero points of W, [m][ceil(n/256)], in/out, or NULL: the symmetric format.  Either every
                             matrix of a plan has them or none (QG_ERR_NULL otherwise). */
} qg_matrix_desc;

const char* qg_status_string(int status);
int qg_last_hip_error(void);

/* ---- Block-wise uniform quantization, Quant_n of Sec. 3.1 (z = 0, s = absmax/qmax,
 * code = clamp(round_half_even(fl32(x * fl32(qmax/absmax))), -2^(n-1), 2^(n-1)-1)).
 * A block whose absmax is 0 gets scale 0 and codes 0.
 * qg_quant_int8: x fp32 [rows][cols] -> q int8 [rows][cols], scales [rows][ceil(cols/256)].
 * qg_quant_int4: x fp32 [rows][cols] -> q_packed uint8 [ceil(rows*cols/2)], scales [ceil(rows*cols/256)].
 * Errors: NULL pointer, rows/cols <= 0 (or rows*cols >= 2^40), group, alignment. */
int qg_quant_int8(const float* x, int64_t rows, int64_t cols, int group,
                  int8_t* q, float* scales, void* stream);
int qg_quant_int4(const float* x, int64_t rows, int64_t cols, int group,
                  uint8_t* q_packed, float* scales, void* stream);

/* ---- Dequantization, W = W_q * s (Appendix A with zeros = 0); fp32 out [rows][cols]. */
int qg_dequant_int8(const int8_t* q, const float* scales, int64_t rows, int64_t cols, int group,
                    float* x, void* stream);
int qg_dequant_int4(const uint8_t* q_packed, const float* scales, int64_t rows, int64_t cols, int group,
                    float* x, void* stream);

/* ---- Gradient projection (Sec. 3.5): R = dequant(P)^T G.
 * P is dequantized inside the GEMM: code*scale in fp32, rounded once to bf16;
 * bf16 MFMA with fp32 accumulation; R fp32 [r][n] is overwritten.
 * Requires 1 <= r <= m, r % 8 == 0, m*n < 2^32.  `workspace` / `workspace_bytes`
 * are reserved: no kernel of this call uses scratch memory, the arguments are
 * not read and may be NULL / 0 (qg_workspace_bytes returns 0). */
int qg_project(const uint8_t* Pq, const float* Ps, const uint16_t* G_bf16,
               int64_t m, int64_t n, int64_t r, int group,
               float* R, void* workspace, size_t workspace_bytes, void* stream);

/* ---- Adam on the low-rank gradient (Sec. 3.5; Adam of Sec. 4.1), element-wise over
 * count = r*n elements:  M <- b1 M + (1-b1) R;  V <- b2 V + (1-b2) R^2;
 * N = bf16( (M/(1-b1^t)) / (sqrt(V/(1-b2^t)) + eps) ).  M, V updated in place (fp32).
 * step = t >= 1.  R may not alias M, V or N. */
int qg_lowrank_adam(const float* R, float* M, float* V, uint16_t* N_bf16,
                    int64_t count, int64_t step, const qg_hparams* hp, void* stream);

/* ---- Adam with 8-bit states (Sec. 3.5: an 8-bit Adam is the paper's inner optimizer; it takes the state format from
 * a third-party library and does not define it - this format is this library's own design).
 * State format: block = 256 consecutive elements of the flattened r x n state; scales [ceil(count/256)] fp32 = the
 * block's absolute maximum; codes uint8 [count] = index of the entry nearest to x/scale (ties to the lower index) in
 * a sorted table with relative resolution.  Unsigned table (second moment): entry 0 is 0, entry p >= 1 has level
 * L = floor(log2 p), k = p - 2^L and value 10^-(7-L) * (0.1 + 0.9 (k+1) / 2^L) (2^L values spaced linearly over each
 * decade from 1e-7 to 1).  Signed table (first moment): levels 0..6 (1e-6 to 1), indices 0..126 the negatives from
 * -1 up, 127 zero, 128..254 the positives, 255 unused.  A positive second moment takes code 1 at least (it never
 * rounds to zero while the first moment, whose table reaches ten times further down, survives).
 * qg_state8_quant / qg_state8_dequant: fp32 [count] <-> (codes, scales); is_signed selects the table.
 * qg_lowrank_adam8: as qg_lowrank_adam, with M and V held in this format (Mq/Ms signed, Vq/Vs unsigned, updated in
 * place): dequantize (table[code] * scale), the same update and direction N, quantize again.
 * count >= 1, a multiple of 4, below 2^40; step >= 1. */
int qg_state8_quant(const float* x, int64_t count, int is_signed, uint8_t* codes, float* scales, void* stream);
int qg_state8_dequant(const uint8_t* codes, const float* scales, int64_t count, int is_signed, float* x, void* stream);
int qg_lowrank_adam8(const float* R, uint8_t* Mq, float* Ms, uint8_t* Vq, float* Vs, uint16_t* N_bf16,
                     int64_t count, int64_t step, const qg_hparams* hp, void* stream);
/* qg_step8: one full step on one matrix with 8-bit Adam states, the paper's default configuration (Sec. 3.5): qg_project
 * -> qg_lowrank_adam8 -> qg_backproject_update_sr on `stream`, with exactly their results.  R (fp32 r x n) and N are
 * caller-provided scratch outputs and both required. */
int qg_step8(const uint8_t* Pq, const float* Ps, const uint16_t* G_bf16, int8_t* Wq, float* Ws,
             uint8_t* Mq, float* Ms, uint8_t* Vq, float* Vs, float* R, uint16_t* N_bf16,
             int64_t m, int64_t n, int64_t r, int group, const qg_hparams* hp, uint64_t seed, int64_t step, void* stream);

/* ---- Projection and Adam fused (Sec. 3.5): the same arithmetic as qg_project followed by qg_lowrank_adam, with
 * Adam applied in the GEMM epilogue while R is still in registers.  M, V in/out, N out; R (nullable) receives the
 * projected gradient only if the caller wants to inspect it - leaving it NULL saves writing and re-reading
 * 8 bytes per low-rank element.  Results are bit-identical to the two separate calls.  This is the form qg_step
 * and qg_step_many run. */
int qg_project_adam(const uint8_t* Pq, const float* Ps, const uint16_t* G_bf16,
                    float* R /* nullable */, float* M, float* V, uint16_t* N_bf16,
                    int64_t m, int64_t n, int64_t r, int group, int64_t step, const qg_hparams* hp, void* stream);

/* ---- Back-projection and INT8 weight update with stochastic rounding
 * (Sec. 3.4, Sec. 3.5):  U = alpha * dequant(P) * N;  x = W_q*s - lr*U;  per block
 * of 256 of each row a = max|x|, s' = a/127, code' = clamp(floor(x*(127/a) + u), -128, 127)
 * with u = 2^-24 * (hash32(seed, step, i*n+j) >> 8).  Wq and Ws are updated in
 * place.  U_debug (nullable) receives U as fp32 [m][n] for parity checks.
 * Requires r % 8 == 0, r <= m, m*n < 2^32. */
int qg_backproject_update_sr(const uint8_t* Pq, const float* Ps, const uint16_t* N_bf16,
                             int8_t* Wq, float* Ws, int64_t m, int64_t n, int64_t r, int group,
                             float alpha, float lr, uint64_t seed, int64_t step,
                             float* U_debug, void* stream);

/* ---- Subspace convergence check (Sec. 3.2, Fig. 2): mean over the r columns of
 * the cosine between column k of dequant(PA) and of dequant(PB).  cos_out is one
 * device float.  workspace: at least qg_cossim_workspace_bytes(m, r) bytes. */
size_t qg_cossim_workspace_bytes(int64_t m, int64_t r);
int qg_subspace_cossim(const uint8_t* PqA, const float* PsA, const uint8_t* PqB, const float* PsB,
                       int64_t m, int64_t r, int group, float* cos_out,
                       void* workspace, size_t workspace_bytes, void* stream);

/* qg_subspace_cossim_weighted: sum_k w_k cos_k / sum_k w_k over the same column cosines, with non-negative weights
 * w (device, fp32 [r], 4-byte aligned; NULL = the plain mean above).  The subspace refresh below reports this form,
 * with the gradient energy each new column captures as the weights.  Same workspace and errors. */
int qg_subspace_cossim_weighted(const uint8_t* PqA, const float* PsA, const uint8_t* PqB, const float* PsB,
                                const float* weights, int64_t m, int64_t r, int group, float* cos_out,
                                void* workspace, size_t workspace_bytes, void* stream);

/* ---- qg_subspace_cossim for callers that cannot allocate device memory or carry a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels and the same result, with the
 * partial sums in a 4 MiB device array that is part of the library image (each GPU that loads the library holds its
 * own copy until the process ends).  Limit: qg_cossim_workspace_bytes(m, r) <= 4 MiB, i.e. about
 * ceil(m/64) * 3 * r <= 2^20 (m = 11008 with r = 1024 fits); larger shapes return QG_ERR_WORKSPACE.  The call
 * allocates nothing and frees nothing; its first call on a device looks the array's address up (make that call
 * outside graph capture).  All calls on one GPU share the array: calls that overlap on one GPU (different streams
 * or threads) race; calls on one stream are ordered and safe.  Other errors as qg_subspace_cossim. */
int qg_subspace_cossim_static(const uint8_t* PqA, const float* PsA, const uint8_t* PqB, const float* PsB,
                              int64_t m, int64_t r, int group, float* cos_out, void* stream);

/* ---- Subspace refresh (Sec. 3.2: every `interval` steps the projection is recomputed from the current gradient;
 * the paper takes the first r left singular vectors of G).  One pass of orthogonal iteration started from the stored
 * projection stands in for the SVD; it converges to the same singular vectors, in the same order, at the rate
 * (sigma_{r+1} / sigma_r)^2 per pass:
 *     R = dequant(P)^T G (qg_project);  Z = bf16(R);  Y = G Z^T;  Q = orthonormalize(Y);  P_new = quant_int4(Q)
 * and, after the last pass, the convergence check of Sec. 3.2 between P and P_new:
 *     *cos_out = qg_subspace_cossim_weighted(P, P_new, e),   e_k = sum_j (dequant(P_new)^T G)[k][j]^2,
 * the column cosines weighted with the gradient energy each new column captures.  (The iteration starts from the old
 * projection, so columns that capture next to no energy come back much as they went in whatever the gradient does;
 * unweighted they would dominate the mean.  With comparable energies in all columns it is the plain mean.)
 *
 * qg_range_apply: Y (fp32 [m][r], overwritten) = G (bf16 [m][n]) * Z^T (Z bf16 [r][n]); bf16 MFMA, fp32 accumulation.
 *
 * qg_orthonormalize: Q (fp32 [m][r]) = the orthonormal factor of Y = Q T with T upper triangular and a positive
 * diagonal (Gram-Schmidt on the columns of Y in order), computed in fp64 as Q = Y L^-T from the Cholesky factor
 * of Y^T Y, twice in a row (the second round removes the cond(Y)^2 loss of orthogonality of the first; accurate to
 * fp32 rounding of what Householder QR gives for cond(Y) up to several 1e8; a shift of 2^-46 trace(Y^T Y) on the
 * Gram diagonal keeps the pivots positive).  *info (device int32) receives 0, or 1 + the index of the first column
 * found numerically dependent on its predecessors (Y rank deficient: that column of Q and the later ones are then
 * meaningless, but every kernel still completes).  Y and Q may not alias.
 * workspace: qg_orthonormalize_workspace_bytes(m, r) bytes, 16-byte aligned.
 *
 * qg_subspace_refresh_many: `passes` (1 .. 64) passes as above on `count` matrices of ONE shape (m, n, r).  descs
 * is a HOST array; Pq/Ps hold each matrix's old projection (unchanged), Pq_new/Ps_new (same sizes, distinct
 * buffers) receive the new one.  cos_out and info are device arrays of `count` elements (info as for
 * qg_orthonormalize, first failure over all passes).  The fp64 stages run batched over the matrices, as many at a
 * time as the workspace holds: qg_refresh_workspace_bytes(count, m, n, r) bytes let all of them run in one batch,
 * qg_refresh_workspace_bytes(1, m, n, r) is the minimum; results do not depend on the batch size.  workspace is
 * 16-byte aligned; after the call it starts with dequant(P_new)^T G (fp32 [r][n]) of the last matrix.
 * qg_subspace_refresh: the same for one matrix.
 * qg_subspace_refresh_many_ld: the same with gradients stored at a row pitch of ld elements (ld >= n, a multiple of
 * 16, or ld == n / 0 for dense rows; m*ld and r*ld below 2^32): rows then start 16-byte aligned whatever n is (the
 * 2048 x 5461 matrices of the LLaMA-1B shapes).  Size the workspace with qg_refresh_workspace_bytes(count, m, ld, r).
 *
 * All require r % 8 == 0, r <= m, m*r < 2^31 and m*n < 2^32 (QG_ERR_SHAPE otherwise). */
typedef struct {
    const uint8_t*  Pq;      /* old projection, INT4 packed  */
    const float*    Ps;      /* old projection, block scales */
    const uint16_t* G;       /* bf16 gradient m x n          */
    uint8_t*        Pq_new;  /* out */
    float*          Ps_new;  /* out */
} qg_refresh_desc;
int qg_range_apply(const uint16_t* G_bf16, const uint16_t* Z_bf16, int64_t m, int64_t n, int64_t r, float* Y,
                   void* stream);
size_t qg_orthonormalize_workspace_bytes(int64_t m, int64_t r);
int qg_orthonormalize(const float* Y, int64_t m, int64_t r, float* Q, int32_t* info,
                      void* workspace, size_t workspace_bytes, void* stream);
size_t qg_refresh_workspace_bytes(int count, int64_t m, int64_t n, int64_t r);
int qg_subspace_refresh_many(int count, const qg_refresh_desc* descs, int64_t m, int64_t n, int64_t r, int group,
                             int passes, float* cos_out, int32_t* info,
                             void* workspace, size_t workspace_bytes, void* stream);
int qg_subspace_refresh_many_ld(int count, const qg_refresh_desc* descs, int64_t m, int64_t n, int64_t ld, int64_t r,
                                int group, int passes, float* cos_out, int32_t* info,
                                void* workspace, size_t workspace_bytes, void* stream);
int qg_subspace_refresh(const uint8_t* Pq, const float* Ps, const uint16_t* G_bf16,
                        int64_t m, int64_t n, int64_t r, int group, int passes,
                        uint8_t* Pq_new, float* Ps_new, float* cos_out, int32_t* info,
                        void* workspace, size_t workspace_bytes, void* stream);

/* ---- INT8 linear layer (Appendix A): the layer whose weight the step updates; its backward pass produces the
 * gradient G the step consumes.  W is the m x n INT8 weight (codes + block scales as above, zero point 0),
 * dequantized inside the GEMMs as bf16(fl32(code * scale)); bf16 MFMA, fp32 accumulation, outputs rounded once
 * to bf16 (activations and gradients are BFloat16, Sec. 3.1).
 * qg_int8_linear_forward:  y [tokens][m] = x [tokens][n] * W^T (+ bias [m], bf16, nullable).
 * qg_int8_linear_backward: dx [tokens][n] = dy [tokens][m] * W and G [m][n] = dy^T * x; either output may be NULL
 *   (then it is not computed, and the inputs only it needs - Wq/Ws for dx, x for G - may be NULL too).
 * Any tokens, m, n >= 1 with tokens*m, tokens*n and m*n below 2^31; base pointers 16-byte aligned (rows need not
 * be).  Outputs may not alias inputs. */
int qg_int8_linear_forward(const uint16_t* x_bf16, const int8_t* Wq, const float* Ws, const uint16_t* bias_bf16,
                           int64_t tokens, int64_t m, int64_t n, int group, uint16_t* y_bf16, void* stream);
int qg_int8_linear_backward(const uint16_t* dy_bf16, const uint16_t* x_bf16, const int8_t* Wq, const float* Ws,
                            int64_t tokens, int64_t m, int64_t n, int group,
                            uint16_t* dx_bf16, uint16_t* G_bf16, void* stream);

/* The same two calls on arrays stored at a row pitch: ld_n is the pitch of the arrays with n elements per row (x, dx,
 * Wq, G), ld_m that of the arrays with m (y, dy); each is the row length itself (or 0), or at least it and a multiple
 * of 16 elements, with rows * pitch below 2^31.  Rows then start 16-byte aligned whatever m and n are (n = 5461 in the
 * LLaMA-1B shapes); G comes out in the layout qg_step_ld and the `ld` of qg_matrix_desc take.  Scales stay
 * [m][ceil(n/256)].  Padding is never read for a result and never written. */
int qg_int8_linear_forward_ld(const uint16_t* x_bf16, const int8_t* Wq, const float* Ws, const uint16_t* bias_bf16,
                              int64_t tokens, int64_t m, int64_t n, int64_t ld_n, int64_t ld_m, int group,
                              uint16_t* y_bf16, void* stream);
int qg_int8_linear_backward_ld(const uint16_t* dy_bf16, const uint16_t* x_bf16, const int8_t* Wq, const float* Ws,
                               int64_t tokens, int64_t m, int64_t n, int64_t ld_n, int64_t ld_m, int group,
                               uint16_t* dx_bf16, uint16_t* G_bf16, void* stream);

/* ---- Right-side projection (GaLore's second form, which Sec. 3.5 inherits: R = G Q with Q the n x r matrix of right
 * singular vectors, moments m x r, update alpha N Q^T; used where a weight has more rows than columns).  A weight
 * that is projected from the right is kept TRANSPOSED, S = W^T: n x m INT8 codes, blocks of 256 along each row of S,
 * scales [n][ceil(m/256)].  Its optimizer step, subspace refresh and cosine check are then the left-side calls above
 * on the n x m matrix S with P = Q (n x r) and the gradient in S's layout: qg_step(Qq, Qs, G_S, Sq, Ss, M, V, R, N,
 * n, m, r, ...) with moments r x m (the transposes of GaLore's m x r; Adam is element-wise).  The two calls below are
 * the linear layer on that storage; its backward pass writes the gradient directly in S's layout, so nothing is ever
 * transposed in memory.
 * qg_int8_linear_t_forward:  y [tokens][m] = x [tokens][n] * S (+ bias [m], bf16, nullable)      (= x W^T)
 * qg_int8_linear_t_backward: dx [tokens][n] = dy [tokens][m] * S^T                                (= dy W)
 *                            G_S [n][m] = x^T * dy                                               (= (dy^T x)^T)
 * Arguments, limits, NULL outputs and alignment as for the two calls above. */
int qg_int8_linear_t_forward(const uint16_t* x_bf16, const int8_t* Sq, const float* Ss, const uint16_t* bias_bf16,
                             int64_t tokens, int64_t m, int64_t n, int group, uint16_t* y_bf16, void* stream);
int qg_int8_linear_t_backward(const uint16_t* dy_bf16, const uint16_t* x_bf16, const int8_t* Sq, const float* Ss,
                              int64_t tokens, int64_t m, int64_t n, int group,
                              uint16_t* dx_bf16, uint16_t* GS_bf16, void* stream);

/* ---- Zero-point (asymmetric) INT8 weights: the quantizer as Sec. 3.1 writes it, W_q = clamp(round(W/s) + z), and
 * Appendix A's dequantization W = (W_q - zeros) * scales.  Per block of 256 elements of a row: lo = min(0, min x),
 * hi = max(0, max x), s = (hi - lo)/255, z = clamp(-128 - round(lo * (255/(hi - lo))), -128, 127), code =
 * clamp(round(x * (255/(hi - lo))) + z, -128, 127), all in fp32; an all-zero block has s = 0, z = 0.  Zero points are
 * whole numbers kept as fp32 [rows][ceil(cols/256)], next to the scales.  Zero itself is always a code (z).
 * qg_quant_int8_zp / qg_dequant_int8_zp: as qg_quant_int8 / qg_dequant_int8, with the zero points.
 * qg_backproject_update_sr_zp: as qg_backproject_update_sr on such a weight: x = (W_q - z)*s - lr*U, new (s', z')
 *   from the block's min and max as above, code' = clamp(floor(x*(255/(hi - lo)) + u) + z', -128, 127) with the same
 *   uniform draw u; Wq, Ws, Wz updated in place.
 * qg_step_zp: qg_step on such a weight (qg_project_adam, then qg_backproject_update_sr_zp); in a grouped plan give
 *   every descriptor its Wz.
 * qg_int8_linear_zp_forward / _backward: the linear layer on such a weight (W dequantized inside the GEMMs as
 *   bf16(fl32((code - zero) * scale))).
 * qg_int8_linear_t_zp_forward / _backward: the same on a zero-point weight stored transposed (S = W^T: codes
 *   [n][m], scales and zero points [n][ceil(m/256)]), the layer of a right-projected matrix in this format; its
 *   step is qg_step_zp on S as for the symmetric format.
 * Shapes, limits, alignment and NULL rules as for the calls they mirror; Wz may never be NULL. */
int qg_quant_int8_zp(const float* x, int64_t rows, int64_t cols, int group, int8_t* q, float* scales, float* zeros,
                     void* stream);
int qg_dequant_int8_zp(const int8_t* q, const float* scales, const float* zeros, int64_t rows, int64_t cols, int group,
                       float* x, void* stream);
int qg_backproject_update_sr_zp(const uint8_t* Pq, const float* Ps, const uint16_t* N_bf16,
                                int8_t* Wq, float* Ws, float* Wz, int64_t m, int64_t n, int64_t r, int group,
                                float alpha, float lr, uint64_t seed, int64_t step, void* stream);
int qg_step_zp(const uint8_t* Pq, const float* Ps, const uint16_t* G_bf16,
               int8_t* Wq, float* Ws, float* Wz, float* M, float* V, float* R, uint16_t* N_bf16,
               int64_t m, int64_t n, int64_t r, int group,
               const qg_hparams* hp, uint64_t seed, int64_t step, void* stream);
int qg_int8_linear_zp_forward(const uint16_t* x_bf16, const int8_t* Wq, const float* Ws, const float* Wz,
                              const uint16_t* bias_bf16, int64_t tokens, int64_t m, int64_t n, int group,
                              uint16_t* y_bf16, void* stream);
int qg_int8_linear_zp_backward(const uint16_t* dy_bf16, const uint16_t* x_bf16, const int8_t* Wq, const float* Ws,
                               const float* Wz, int64_t tokens, int64_t m, int64_t n, int group,
                               uint16_t* dx_bf16, uint16_t* G_bf16, void* stream);
int qg_int8_linear_t_zp_forward(const uint16_t* x_bf16, const int8_t* Sq, const float* Ss, const float* Sz,
                                const uint16_t* bias_bf16, int64_t tokens, int64_t m, int64_t n, int group,
                                uint16_t* y_bf16, void* stream);
int qg_int8_linear_t_zp_backward(const uint16_t* dy_bf16, const uint16_t* x_bf16, const int8_t* Sq, const float* Ss,
                                 const float* Sz, int64_t tokens, int64_t m, int64_t n, int group,
                                 uint16_t* dx_bf16, uint16_t* GS_bf16, void* stream);

/* ---- Adaptive lazy update policy (Sec. 3.2), HOST ONLY (p is a host pointer):
 * streak counts consecutive checks with cos >= threshold; at k in a row the
 * interval doubles and the streak restarts; next_refresh advances by the
 * (possibly doubled) interval.  Returns 1 if the interval doubled, 0 if not,
 * -1 if p is NULL. */
int qg_policy_update(qg_policy* p, float cos);

/* ---- One full step on one matrix (Sec. 3.5): project -> Adam -> back-project +
 * SR update, as two kernels on `stream` (qg_project_adam, then
 * qg_backproject_update_sr): the same results as the three separate calls.
 * N is a caller-provided output (r x n bf16); R (r x n fp32) is written only
 * if it is not NULL.  No subspace refresh happens inside.
 * qg_workspace_bytes: scratch bytes qg_project and qg_step need for a matrix of
 * this shape: always 0 (both run out of registers and LDS); their `workspace`
 * and `workspace_bytes` arguments are reserved, never read, and may be NULL / 0. */
size_t qg_workspace_bytes(int64_t m, int64_t n, int64_t r);
int qg_step(const uint8_t* Pq, const float* Ps, const uint16_t* G_bf16,
            int8_t* Wq, float* Ws, float* M, float* V, float* R, uint16_t* N_bf16,
            int64_t m, int64_t n, int64_t r, int group,
            const qg_hparams* hp, uint64_t seed, int64_t step,
            void* workspace, size_t workspace_bytes, void* stream);

/* qg_step_ld: qg_step on arrays stored at a row pitch: G, Wq (m rows) and M, V, R, N (r rows) all have rows ld
 * elements apart (ld >= n and a multiple of 16, or ld == n / 0 for dense rows; m*ld < 2^32), as in the `ld` field of
 * qg_matrix_desc: a matrix whose n is not a multiple of 8 then runs in the kernels for 16-byte aligned rows.  Scales
 * stay [m][ceil(n/256)]; the stochastic-rounding index stays i*n + j, so the n real columns get the dense layout's
 * result.  Padding is never read for a result and not written, except that N is stored in pairs of columns. */
int qg_step_ld(const uint8_t* Pq, const float* Ps, const uint16_t* G_bf16,
               int8_t* Wq, float* Ws, float* M, float* V, float* R, uint16_t* N_bf16,
               int64_t m, int64_t n, int64_t ld, int64_t r, int group,
               const qg_hparams* hp, uint64_t seed, int64_t step, void* stream);

/* ---- Grouped step over many matrices (the whole model's linear weights) in
 * two grouped launches per edge class (projection with Adam in its epilogue,
 * back-projection + update).  R is written only if every descriptor supplies
 * a buffer for it; qg_project_many and qg_lowrank_adam_many need every R.
 * `descs` is a HOST array of `count` descriptors.
 * The library needs a device-resident launch plan: the caller provides
 * `plan_host` (host scratch) and `plan_dev` (device memory), each of
 * qg_plan_bytes(count, descs) bytes; qg_plan_build fills plan_host, the
 * caller copies it to plan_dev (any memcpy), and qg_step_many uses both.
 * Matrix i draws its SR numbers with seed + i * 0x9E3779B97F4A7C15 (mod 2^64). */
size_t qg_plan_bytes(int count, const qg_matrix_desc* descs);
int qg_plan_build(int count, const qg_matrix_desc* descs, void* plan_host, size_t plan_bytes);
int qg_step_many(int count, const void* plan_host, const void* plan_dev, size_t plan_bytes,
                 const qg_hparams* hp, uint64_t seed, int64_t step, void* stream);

/* The grouped launches one by one (same plan arguments): projection of every matrix, Adam over every matrix
 * (these two need every descriptor's R), their fusion (write_R != 0 also stores R), and back-projection + SR update
 * of every matrix.  qg_step_many(...) == qg_project_adam_many, qg_backproject_update_sr_many; the unfused pair
 * qg_project_many, qg_lowrank_adam_many gives bit-identical M, V, N (and R). */
int qg_project_many(int count, const void* plan_host, const void* plan_dev, size_t plan_bytes, void* stream);
int qg_lowrank_adam_many(int count, const void* plan_host, const void* plan_dev, size_t plan_bytes,
                         const qg_hparams* hp, int64_t step, void* stream);
int qg_project_adam_many(int count, const void* plan_host, const void* plan_dev, size_t plan_bytes,
                         const qg_hparams* hp, int64_t step, int write_R, void* stream);
int qg_backproject_update_sr_many(int count, const void* plan_host, const void* plan_dev, size_t plan_bytes,
                                  const qg_hparams* hp, uint64_t seed, int64_t step, void* stream);

/* ---- Measurement helpers (no part of the method; used by the benchmark to state what the machine sustains).
 *
 * qg_diag_clock_probe: enqueues a one-wave kernel that waits ticks_100mhz ticks (1 .. 10^8) of the constant
 * 100 MHz counter and writes {shader clock cycles elapsed, ticks elapsed} to out2 (device, 2 x int64).  Launched
 * on a second stream beside a kernel under test it gives the shader clock that kernel runs at.
 *
 * qg_diag_mfma_loop: QG_DIAG_MFMA_WORKGROUPS workgroups of 512 threads (8 waves, two per SIMD); each wave issues
 * iters (1 .. 2^24) rounds of 16 independent bf16 32x32x16 MFMAs on register operands, i.e.
 * QG_DIAG_MFMA_WORKGROUPS * 8 * iters * 16 * 32768 flop per launch: the ceiling of the matrix pipe with nothing else
 * running.  random_operands != 0 fills the operands with varied finite bit patterns (the sustained clock depends on
 * the data), 0 with constants.  sink: device, QG_DIAG_MFMA_WORKGROUPS * 512 floats (written so the loop is live).
 *
 * qg_diag_mfma_f64_loop: `workgroups` (1 .. 65536) workgroups of 256 threads; each wave issues iters rounds of 8
 * independent v_mfma_f64_16x16x4 on register operands: workgroups * 4 * iters * 8 * 2048 flop per launch, the
 * ceiling of the fp64 matrix pipe for the kernels of the subspace refresh.  sink: workgroups * 256 floats. */
#define QG_DIAG_MFMA_WORKGROUPS 512
int qg_diag_clock_probe(int64_t ticks_100mhz, int64_t* out2, void* stream);
int qg_diag_mfma_loop(int64_t iters, int random_operands, float* sink, void* stream);
int qg_diag_mfma_f64_loop(int64_t iters, int workgroups, float* sink, void* stream);

/* ---- Test helper: out[i] = u(seed, step, idx0 + i) for i < count, the uniform
 * draws of the stochastic-rounding generator, as fp32. */
int qg_sr_uniform(uint64_t seed, int64_t step, uint64_t idx0, int64_t count, float* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* QGALORE_H */
