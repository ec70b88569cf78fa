// The per-parameter arithmetic of the LSGD update (supplement B.1 / Eq. 3 of arXiv 1905.10395,
// with the optional momentum, Nesterov and weight-decay forms of Section 4.1), shared by the
// streaming update kernels and by the gradient kernels that apply the update in their epilogue.
#pragma once

namespace lsgd {

struct Coef {
    float eta, cL, cG, mu, wd;
    int nesterov, grad_only;
};

// One parameter (V = float) or four (V = a 4-wide vector), element-wise.  Written with plain
// operators so that the compiler forms the fused multiply-adds itself.
// KIND 0: gradient step, 1: gradient step with momentum, 2: Algorithm 1's communication pull
// (x <- x - cL (x - zl), then x <- x - cG (x - zg); no gradient, momentum untouched).
template <int KIND, class V>
__device__ __forceinline__ void update_vec(V& x, const V g, V& m, const V zl, const V zg, const Coef& c)
{
    constexpr bool MOM = KIND == 1;
    if (KIND == 2) {
        const V y = x - c.cL * (x - zl);
        x = y - c.cG * (y - zg);
        return;
    }
    V d = g + c.wd * x;
    const V pull = c.cL * (x - zl) + c.cG * (x - zg);
    V step;
    if (MOM) {
        if (c.grad_only) {
            m = c.mu * m + d;
            step = (c.nesterov ? d + c.mu * m : m) + pull;
        } else {
            d += pull;
            m = c.mu * m + d;
            step = c.nesterov ? d + c.mu * m : m;
        }
    } else {
        step = d + pull;
    }
    x = x - c.eta * step;
}

} // namespace lsgd
