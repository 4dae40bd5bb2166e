// Host-side evaluation of the variance-increment indicator from tensor statistics (no GPU work).
//
// Paper, Indicator section.  Prop. 2 (tensor quantization variance): a tensor of D elements quantized
// with stochastic rounding carries a variance of q^2 D / 6 on a fixed-point grid of step q and of
// (2^e eps)^2 D / 6 on a floating-point grid whose spacing in the tensor's top binade 2^e is 2^e eps,
// eps = 2^-k.  Prop. 3 (variance increment): the forward term of a linear or convolution operator weighs
// each operand's quantization variance with the squared norm of the other operand, the backward term does
// the same for the activation gradient and the saved activation, and
//     Omega = gamma^2 d_o sigma_fp + (d_L - d_o) sigma_bp.
// In the backward pass of a fixed-point operator the gradient is kept in floating point (second summand
// of the fixed-point case of the backward equation), the saved activation on its fixed-point grid.
#include "../../include/qsync.h"

#include <cmath>

namespace {

// spacing of the quantization grid seen by a tensor: a fixed-point step, or 2^(e - k) with 2^e <= amax < 2^(e+1)
double fixed_step(double q) { return q; }
double float_step(double amax, int k)
{
    const int e = amax > 0.0 ? std::ilogb(amax) : -126;       // all-zero tensor: smallest normal binade of binary32
    return std::ldexp(1.0, e - k);
}
// Prop. 2: variance a stochastic-rounding grid of that spacing adds to a tensor of D elements
double grid_variance(double step, int64_t D) { return step * step * static_cast<double>(D) / 6.0; }

bool stats_ok(const qsync_tensor_stats_t* t)
{
    return t->D >= 0 && t->sumsq >= 0.0 && t->amax >= 0.0 && std::isfinite(t->sumsq) && std::isfinite(t->amax);
}

}  // namespace

extern "C" int qsync_variance_increment(int kind, const qsync_tensor_stats_t* x, const qsync_tensor_stats_t* v,
                                        const qsync_tensor_stats_t* grad_v, double q_x, double q_v, int k,
                                        double gamma, int64_t d_o, int64_t d_L, double* sigma_fp, double* sigma_bp,
                                        double* omega)
{
    if(!x || !v || !grad_v || !omega) return QSYNC_ERR_NULL;
    if(kind != QSYNC_QUANT_FIXED && kind != QSYNC_QUANT_FLOAT) return QSYNC_ERR_BAD_ENUM;
    if(!stats_ok(x) || !stats_ok(v) || !stats_ok(grad_v) || d_o < 0 || d_L < d_o) return QSYNC_ERR_BAD_SHAPE;
    if(k < 1 || k > 52 || !std::isfinite(gamma)) return QSYNC_ERR_UNSUPPORTED;
    if(kind == QSYNC_QUANT_FIXED && !(q_x >= 0.0 && q_v >= 0.0 && std::isfinite(q_x) && std::isfinite(q_v)))
        return QSYNC_ERR_UNSUPPORTED;
    const bool   fixed  = kind == QSYNC_QUANT_FIXED;
    // grids of the forward pass: parameter x and activation v in the operator's own format
    const double var_x  = grid_variance(fixed ? fixed_step(q_x) : float_step(x->amax, k), x->D);
    const double var_v  = grid_variance(fixed ? fixed_step(q_v) : float_step(v->amax, k), v->D);
    // the activation gradient travels in floating point in both cases
    const double var_gv = grid_variance(float_step(grad_v->amax, k), grad_v->D);
    const double fp     = x->sumsq * var_v + v->sumsq * var_x;
    const double bp     = grad_v->sumsq * var_v + v->sumsq * var_gv;
    if(sigma_fp) *sigma_fp = fp;
    if(sigma_bp) *sigma_bp = bp;
    *omega = gamma * gamma * static_cast<double>(d_o) * fp + static_cast<double>(d_L - d_o) * bp;
    return QSYNC_OK;
}
