// Device-side pieces shared by the epoch kernels: the per-nonzero terms of the two inner products
// and the scalar step of one coordinate update (Section 3.1).
#pragma once
#include "common.h"

namespace snap {

struct StepParams {
    double lambda;
    double lambda1;   // weight of the l1 term (primal forms)
    double inv_n;     // 1/n
    double lam_n;     // lambda * n
    double damping;   // in (0,1]: the step is scaled by it (Section 3.1, adaptive damping)
};

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int off = WAVE / 2; off > 0; off >>= 1) x += __shfl_xor(x, off, WAVE);
    return x;
}

__device__ __forceinline__ float load_shared(const float* v, uint32_t r) {
    // relaxed device-scope load: sees the other compute dies' atomic updates of v
    return __hip_atomic_load(v + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Contribution of one nonzero (value a, shared entry vv, label yy) to the two sums of the step.
template <int KIND>
__device__ __forceinline__ void accumulate(float a, float vv, float yy, float& g, float& h) {
    if (KIND == K_PRIMAL_RIDGE) {
        g += a * (vv - yy);                       // loss' = v - y ; loss'' = 1 (h comes from the norm)
    } else if (KIND == K_PRIMAL_LOGISTIC) {
        const float e = __expf(yy * vv);          // p = sigmoid(-y v) = 1/(1+e)
        const float p = __builtin_amdgcn_rcpf(1.0f + e);   // hardware reciprocal (1 ulp); e = inf gives p = 0
        g -= a * yy * p;                          // loss'  = -y p
        h += a * a * (p - p * p);                 // loss'' = p (1 - p)
    } else {
        g += a * vv;                              // x_i . v
    }
}

// The scalar step.  Returns the new value of the coordinate; `mult` receives the multiplier of a_j
// that is added to v: the change actually applied to the fp32 coordinate (times y_i in the hinge
// dual), so that v keeps tracking A x as closely as fp32 allows.
template <int KIND>
__device__ __forceinline__ float take_step(double g, double h, float xc, float norm, float yc,
                                           const StepParams& sp, float& mult) {
    float xn;
    if (KIND == K_PRIMAL_RIDGE || KIND == K_PRIMAL_LOGISTIC) {
        const double Gf = g * sp.inv_n;                                       // loss part of the gradient
        const double Hf = (KIND == K_PRIMAL_RIDGE ? (double)norm : h) * sp.inv_n;
        double step;
        if (sp.lambda1 == 0.0) {
            step = -(Gf + sp.lambda * (double)xc) / (Hf + sp.lambda);
        } else {
            // minimiser of Gf d + (Hf/2) d^2 + (lambda/2)(x+d)^2 + lambda1 |x+d|: soft threshold
            const double t = Hf * (double)xc - Gf;
            const double s = t > sp.lambda1 ? t - sp.lambda1 : (t < -sp.lambda1 ? t + sp.lambda1 : 0.0);
            step = s / (Hf + sp.lambda) - (double)xc;
        }
        xn = (float)((double)xc + sp.damping * step);
        mult = (float)((double)xn - (double)xc);
    } else {
        double anew;
        if (norm == 0.0f) {
            anew = 1.0;                                   // empty row: dD/dalpha = 1/n > 0
        } else {
            const double m = (double)yc * g / sp.lam_n;   // y_i x_i.w
            const double q = (double)norm / sp.lam_n;
            anew = (double)xc + (1.0 - m) / q;
            anew = anew < 0.0 ? 0.0 : (anew > 1.0 ? 1.0 : anew);
        }
        anew = (double)xc + sp.damping * (anew - (double)xc);   // stays inside the box
        xn = (float)anew;
        mult = (float)(((double)xn - (double)xc) * (double)yc);
    }
    return xn;
}

template <int KIND>
__device__ __forceinline__ void decode(uint32_t raw, uint32_t& r, float& yy, const float* __restrict__ y) {
    if (KIND == K_PRIMAL_LOGISTIC) {
        r = raw & ~LABEL_BIT;
        yy = (raw & LABEL_BIT) ? -1.0f : 1.0f;
    } else if (KIND == K_PRIMAL_RIDGE) {
        r = raw;
        yy = y[r];
    } else {
        r = raw;
        yy = 0.0f;
    }
}


inline StepParams make_step_params(const snap_handle* h) {
    StepParams sp;
    sp.lambda = h->lambda;
    sp.lambda1 = h->lambda1;
    sp.inv_n = 1.0 / (double)h->n;
    sp.lam_n = h->lambda * (double)h->n;
    sp.damping = (double)h->damping;
    return sp;
}

}  // namespace snap
