// INT8 linear layer (Appendix A): the layer whose weight the optimizer step updates, and whose backward pass
// produces the gradient G that the step consumes.
//     forward:   y  = x W^T (+ bias)       x bf16 [tokens][n], W INT8 [m][n] + block scales, y bf16 [tokens][m]
//     backward:  dx = dy W                 dy bf16 [tokens][m], dx bf16 [tokens][n]
//                G  = dy^T x               bf16 [m][n]
// W is dequantized while its tile is staged into LDS (code * scale in fp32, rounded once to bf16: the operand the
// projection GEMM of the step sees for P); all three products are bf16 MFMA GEMMs with fp32 accumulation and one
// rounding to bf16 at the store.
//
// The three products are instances of the tile GEMM of qg_tile_gemm.h: the contraction index is the fast one of x and
// W in the forward pass, of dy only in grad_input, of neither in grad_W.
#include "qg_tile_gemm.h"

namespace qg {

static int check_linear(int64_t tokens, int64_t m, int64_t n, int group) {
    const int64_t lim = int64_t(1) << 31;
    if (tokens <= 0 || m <= 0 || n <= 0 || tokens >= lim / m || tokens >= lim / n || m >= lim / n) return QG_ERR_SHAPE;
    if (group != kGroup) return QG_ERR_GROUP;
    return QG_OK;
}

// Row pitches of the pitched entry points: ld_n for the arrays with n elements per row (x, dx, Wq, G), ld_m for those
// with m (y, dy).  Each is the row length itself, or at least it and a multiple of 16 elements.
static int check_pitch(int64_t rows_limit, int64_t len, int64_t& ld) {
    if (ld == 0) ld = len;
    if (ld != len && (ld < len || (ld & 15))) return QG_ERR_SHAPE;
    if (rows_limit >= (int64_t(1) << 31) / ld) return QG_ERR_SHAPE;
    return QG_OK;
}

}  // namespace qg

using namespace qg;

extern "C" int qg_int8_linear_forward_ld(const uint16_t* x_bf16, const int8_t* Wq, const float* Ws,
                                         const uint16_t* bias_bf16, int64_t tokens, int64_t m, int64_t n, int64_t ld_n,
                                         int64_t ld_m, int group, uint16_t* y_bf16, void* stream) {
    if (!x_bf16 || !Wq || !Ws || !y_bf16) return QG_ERR_NULL;
    if (int e = check_linear(tokens, m, n, group)) return e;
    if (int e = check_pitch(tokens > m ? tokens : m, n, ld_n)) return e;
    if (int e = check_pitch(tokens, m, ld_m)) return e;
    if (!aligned16(x_bf16) || !aligned16(Wq) || !aligned16(Ws) || !aligned16(y_bf16) || (bias_bf16 && !aligned16(bias_bf16)))
        return QG_ERR_ALIGN;
    const int sg = (int)((n + kGroup - 1) / kGroup);
    const LinOperand A = {x_bf16, nullptr, ld_n, 0}, B = {Wq, Ws, ld_n, sg};
    return launch_tile_gemm<kBf16KFast, kInt8KFast, uint16_t>(A, B, bias_bf16, y_bf16, tokens, m, n, (hipStream_t)stream,
                                                              nullptr, 1, ld_m);
}

extern "C" int qg_int8_linear_forward(const uint16_t* x_bf16, const int8_t* Wq, const float* Ws, const uint16_t* bias_bf16,
                                      int64_t tokens, int64_t m, int64_t n, int group, uint16_t* y_bf16, void* stream) {
    return qg_int8_linear_forward_ld(x_bf16, Wq, Ws, bias_bf16, tokens, m, n, n, m, group, y_bf16, stream);
}

extern "C" int qg_int8_linear_backward_ld(const uint16_t* dy_bf16, const uint16_t* x_bf16, const int8_t* Wq,
                                          const float* Ws, int64_t tokens, int64_t m, int64_t n, int64_t ld_n,
                                          int64_t ld_m, int group, uint16_t* dx_bf16, uint16_t* G_bf16, void* stream) {
    if (!dy_bf16 || (!dx_bf16 && !G_bf16)) return QG_ERR_NULL;
    if ((dx_bf16 && (!Wq || !Ws)) || (G_bf16 && !x_bf16)) return QG_ERR_NULL;
    if (int e = check_linear(tokens, m, n, group)) return e;
    if (int e = check_pitch(tokens > m ? tokens : m, n, ld_n)) return e;
    if (int e = check_pitch(tokens, m, ld_m)) return e;
    if (!aligned16(dy_bf16) || (x_bf16 && !aligned16(x_bf16)) || (Wq && !aligned16(Wq)) || (Ws && !aligned16(Ws)) ||
        (dx_bf16 && !aligned16(dx_bf16)) || (G_bf16 && !aligned16(G_bf16)))
        return QG_ERR_ALIGN;
    const int sg = (int)((n + kGroup - 1) / kGroup);
    if (dx_bf16) {   // dx[t][i] = sum_o dy[t][o] W[o][i]
        const LinOperand A = {dy_bf16, nullptr, ld_m, 0}, B = {Wq, Ws, ld_n, sg};
        if (int e = launch_tile_gemm<kBf16KFast, kInt8KSlow, uint16_t>(A, B, nullptr, dx_bf16, tokens, n, m, (hipStream_t)stream,
                                                                       nullptr, 1, ld_n))
            return e;
    }
    if (G_bf16) {    // G[o][i] = sum_t dy[t][o] x[t][i]
        const LinOperand A = {dy_bf16, nullptr, ld_m, 0}, B = {x_bf16, nullptr, ld_n, 0};
        if (int e = launch_tile_gemm<kBf16KSlow, kBf16KSlow, uint16_t>(A, B, nullptr, G_bf16, m, n, tokens, (hipStream_t)stream,
                                                                       nullptr, 1, ld_n))
            return e;
    }
    return QG_OK;
}

extern "C" int qg_int8_linear_backward(const uint16_t* dy_bf16, const uint16_t* x_bf16, const int8_t* Wq, const float* Ws,
                                       int64_t tokens, int64_t m, int64_t n, int group, uint16_t* dx_bf16,
                                       uint16_t* G_bf16, void* stream) {
    return qg_int8_linear_backward_ld(dy_bf16, x_bf16, Wq, Ws, tokens, m, n, n, m, group, dx_bf16, G_bf16, stream);
}

// The same layer on a weight stored transposed, S = W^T (n x m, blocks along m): the storage of a matrix whose
// gradient is projected from the right.  The three products are the ones above with the operand roles exchanged: the
// forward pass has the layout of grad_input, grad_input that of the forward pass, and the weight gradient comes out
// in S's layout.
extern "C" int qg_int8_linear_t_forward(const uint16_t* x_bf16, const int8_t* Sq, const float* Ss,
                                        const uint16_t* bias_bf16, int64_t tokens, int64_t m, int64_t n, int group,
                                        uint16_t* y_bf16, void* stream) {
    if (!x_bf16 || !Sq || !Ss || !y_bf16) return QG_ERR_NULL;
    if (int e = check_linear(tokens, m, n, group)) return e;
    if (!aligned16(x_bf16) || !aligned16(Sq) || !aligned16(Ss) || !aligned16(y_bf16) || (bias_bf16 && !aligned16(bias_bf16)))
        return QG_ERR_ALIGN;
    const int sg = (int)((m + kGroup - 1) / kGroup);
    // y[t][o] = sum_i x[t][i] S[i][o]
    const LinOperand A = {x_bf16, nullptr, n, 0}, B = {Sq, Ss, m, sg};
    return launch_tile_gemm<kBf16KFast, kInt8KSlow, uint16_t>(A, B, bias_bf16, y_bf16, tokens, m, n, (hipStream_t)stream);
}

extern "C" int qg_int8_linear_t_backward(const uint16_t* dy_bf16, const uint16_t* x_bf16, const int8_t* Sq, const float* Ss,
                                         int64_t tokens, int64_t m, int64_t n, int group, uint16_t* dx_bf16,
                                         uint16_t* GS_bf16, void* stream) {
    if (!dy_bf16 || (!dx_bf16 && !GS_bf16)) return QG_ERR_NULL;
    if ((dx_bf16 && (!Sq || !Ss)) || (GS_bf16 && !x_bf16)) return QG_ERR_NULL;
    if (int e = check_linear(tokens, m, n, group)) return e;
    if (!aligned16(dy_bf16) || (x_bf16 && !aligned16(x_bf16)) || (Sq && !aligned16(Sq)) || (Ss && !aligned16(Ss)) ||
        (dx_bf16 && !aligned16(dx_bf16)) || (GS_bf16 && !aligned16(GS_bf16)))
        return QG_ERR_ALIGN;
    const int sg = (int)((m + kGroup - 1) / kGroup);
    if (dx_bf16) {   // dx[t][i] = sum_o dy[t][o] S[i][o]
        const LinOperand A = {dy_bf16, nullptr, m, 0}, B = {Sq, Ss, m, sg};
        if (int e = launch_tile_gemm<kBf16KFast, kInt8KFast, uint16_t>(A, B, nullptr, dx_bf16, tokens, n, m, (hipStream_t)stream)) return e;
    }
    if (GS_bf16) {   // G_S[i][o] = sum_t x[t][i] dy[t][o]
        const LinOperand A = {x_bf16, nullptr, n, 0}, B = {dy_bf16, nullptr, m, 0};
        if (int e = launch_tile_gemm<kBf16KSlow, kBf16KSlow, uint16_t>(A, B, nullptr, GS_bf16, n, m, tokens, (hipStream_t)stream)) return e;
    }
    return QG_OK;
}

// The layer on a zero-point weight (Sec. 3.1 eq. with z; Appendix A: W = (W_q - zeros) * scales): the same products,
// the weight operand dequantized as bf16(fl32((code - zero) * scale)).  grad_W does not read the weight.
extern "C" int qg_int8_linear_zp_forward(const uint16_t* x_bf16, const int8_t* Wq, const float* Ws, const float* Wz,
                                         const uint16_t* bias_bf16, int64_t tokens, int64_t m, int64_t n, int group,
                                         uint16_t* y_bf16, void* stream) {
    if (!x_bf16 || !Wq || !Ws || !Wz || !y_bf16) return QG_ERR_NULL;
    if (int e = check_linear(tokens, m, n, group)) return e;
    if (!aligned16(x_bf16) || !aligned16(Wq) || !aligned16(Ws) || !aligned16(Wz) || !aligned16(y_bf16) ||
        (bias_bf16 && !aligned16(bias_bf16)))
        return QG_ERR_ALIGN;
    const int sg = (int)((n + kGroup - 1) / kGroup);
    const LinOperand A = {x_bf16, nullptr, n, 0}, B = {Wq, Ws, n, sg, Wz};
    return launch_tile_gemm<kBf16KFast, kInt8ZKFast, uint16_t>(A, B, bias_bf16, y_bf16, tokens, m, n, (hipStream_t)stream);
}

extern "C" int qg_int8_linear_zp_backward(const uint16_t* dy_bf16, const uint16_t* x_bf16, const int8_t* Wq,
                                          const float* Ws, const float* Wz, int64_t tokens, int64_t m, int64_t n,
                                          int group, uint16_t* dx_bf16, uint16_t* G_bf16, void* stream) {
    if (!dy_bf16 || (!dx_bf16 && !G_bf16)) return QG_ERR_NULL;
    if ((dx_bf16 && (!Wq || !Ws || !Wz)) || (G_bf16 && !x_bf16)) return QG_ERR_NULL;
    if (int e = check_linear(tokens, m, n, group)) return e;
    if (!aligned16(dy_bf16) || (x_bf16 && !aligned16(x_bf16)) || (Wq && !aligned16(Wq)) || (Ws && !aligned16(Ws)) ||
        (Wz && !aligned16(Wz)) || (dx_bf16 && !aligned16(dx_bf16)) || (G_bf16 && !aligned16(G_bf16)))
        return QG_ERR_ALIGN;
    const int sg = (int)((n + kGroup - 1) / kGroup);
    if (dx_bf16) {
        const LinOperand A = {dy_bf16, nullptr, m, 0}, B = {Wq, Ws, n, sg, Wz};
        if (int e = launch_tile_gemm<kBf16KFast, kInt8ZKSlow, uint16_t>(A, B, nullptr, dx_bf16, tokens, n, m, (hipStream_t)stream)) return e;
    }
    if (G_bf16) {
        const LinOperand A = {dy_bf16, nullptr, m, 0}, B = {x_bf16, nullptr, n, 0};
        if (int e = launch_tile_gemm<kBf16KSlow, kBf16KSlow, uint16_t>(A, B, nullptr, G_bf16, m, n, tokens, (hipStream_t)stream)) return e;
    }
    return QG_OK;
}

// Zero-point weight stored transposed (S = W^T with zero points along each row of S): the two variants combined.
extern "C" int qg_int8_linear_t_zp_forward(const uint16_t* x_bf16, const int8_t* Sq, const float* Ss, const float* Sz,
                                           const uint16_t* bias_bf16, int64_t tokens, int64_t m, int64_t n, int group,
                                           uint16_t* y_bf16, void* stream) {
    if (!x_bf16 || !Sq || !Ss || !Sz || !y_bf16) return QG_ERR_NULL;
    if (int e = check_linear(tokens, m, n, group)) return e;
    if (!aligned16(x_bf16) || !aligned16(Sq) || !aligned16(Ss) || !aligned16(Sz) || !aligned16(y_bf16) ||
        (bias_bf16 && !aligned16(bias_bf16)))
        return QG_ERR_ALIGN;
    const int sg = (int)((m + kGroup - 1) / kGroup);
    const LinOperand A = {x_bf16, nullptr, n, 0}, B = {Sq, Ss, m, sg, Sz};
    return launch_tile_gemm<kBf16KFast, kInt8ZKSlow, uint16_t>(A, B, bias_bf16, y_bf16, tokens, m, n, (hipStream_t)stream);
}

extern "C" int qg_int8_linear_t_zp_backward(const uint16_t* dy_bf16, const uint16_t* x_bf16, const int8_t* Sq,
                                            const float* Ss, const float* Sz, int64_t tokens, int64_t m, int64_t n,
                                            int group, uint16_t* dx_bf16, uint16_t* GS_bf16, void* stream) {
    if (!dy_bf16 || (!dx_bf16 && !GS_bf16)) return QG_ERR_NULL;
    if ((dx_bf16 && (!Sq || !Ss || !Sz)) || (GS_bf16 && !x_bf16)) return QG_ERR_NULL;
    if (int e = check_linear(tokens, m, n, group)) return e;
    if (!aligned16(dy_bf16) || (x_bf16 && !aligned16(x_bf16)) || (Sq && !aligned16(Sq)) || (Ss && !aligned16(Ss)) ||
        (Sz && !aligned16(Sz)) || (dx_bf16 && !aligned16(dx_bf16)) || (GS_bf16 && !aligned16(GS_bf16)))
        return QG_ERR_ALIGN;
    const int sg = (int)((m + kGroup - 1) / kGroup);
    if (dx_bf16) {
        const LinOperand A = {dy_bf16, nullptr, m, 0}, B = {Sq, Ss, m, sg, Sz};
        if (int e = launch_tile_gemm<kBf16KFast, kInt8ZKFast, uint16_t>(A, B, nullptr, dx_bf16, tokens, n, m, (hipStream_t)stream)) return e;
    }
    if (GS_bf16) {
        const LinOperand A = {x_bf16, nullptr, n, 0}, B = {dy_bf16, nullptr, m, 0};
        if (int e = launch_tile_gemm<kBf16KSlow, kBf16KSlow, uint16_t>(A, B, nullptr, GS_bf16, n, m, tokens, (hipStream_t)stream)) return e;
    }
    return QG_OK;
}
