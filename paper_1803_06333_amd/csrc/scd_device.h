// Device-side pieces shared by the epoch kernels: the per-nonzero terms of the two inner products
// and the scalar step of one coordinate update (Section 3.1).
#pragma once
#include "common.h"

namespace snap {

struct StepParams {
    double lambda;
    double lambda1;   // weight of the l1 term (primal forms)
    int dual_logistic; // dual form: 1 = logistic loss (Newton step on the entropy), 0 = hinge
    double inv_n;     // 1/n
    double lam_n;     // lambda * n
    double inv_lam_n; // 1 / (lambda * n)
    double damping;   // in (0,1]: the step is scaled by it (Section 3.1, adaptive damping)
};

// Sum over the wavefront through the data-parallel-primitive lane moves of the vector ALU (no LDS
// traffic, unlike shuffles): all-reduce inside each row of 16 lanes (swap neighbours, swap pairs,
// rotate by 4, rotate by 8), then the four row sums are read as scalars.  The result is uniform over
// the wavefront; lanes that are switched off contribute 0.
__device__ __forceinline__ float row_sum(float x);
__device__ __forceinline__ float wave_sum(float x) {
    const int xi = __float_as_int(row_sum(x));
    return __int_as_float(__builtin_amdgcn_readlane(xi, 0)) + __int_as_float(__builtin_amdgcn_readlane(xi, 16)) +
           __int_as_float(__builtin_amdgcn_readlane(xi, 32)) + __int_as_float(__builtin_amdgcn_readlane(xi, 48));
}

// The first part alone: every lane gets the sum over its row of 16 lanes.
__device__ __forceinline__ float row_sum(float x) {
    constexpr int QUAD_SWAP_1 = 0xB1;    // quad_perm [1,0,3,2]
    constexpr int QUAD_SWAP_2 = 0x4E;    // quad_perm [2,3,0,1]
    constexpr int ROW_ROR_4 = 0x124, ROW_ROR_8 = 0x128;
    int xi = __float_as_int(x);
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, xi, QUAD_SWAP_1, 0xF, 0xF, false));
    xi = __float_as_int(x);
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, xi, QUAD_SWAP_2, 0xF, 0xF, false));
    xi = __float_as_int(x);
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, xi, ROW_ROR_4, 0xF, 0xF, false));
    xi = __float_as_int(x);
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, xi, ROW_ROR_8, 0xF, 0xF, false));
    return x;
}

__device__ __forceinline__ float load_shared(const float* v, uint32_t r) {
    // relaxed device-scope load: sees the other compute dies' atomic updates of v
    return __hip_atomic_load(v + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// log(1 + exp(t)) in fp32 with the fast exponential, overflow safe: the logistic loss of a margin -t as
// the accept check of the epoch sums it (Section 3.1).  One definition for every place that takes this
// sum, so that values from different kernels can be compared.
__device__ __forceinline__ float logistic_loss_f32(float t) {
    // max(t, 0) + log(1 + exp(-|t|)) with the hardware exponential and logarithm (a few instructions;
    // absolute error of a term about 1e-7, the same in every place that uses it)
    return fmaxf(t, 0.0f) + __logf(1.0f + __expf(-fabsf(t)));
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

// Step of a primal coordinate from the loss part of the gradient Gf = (1/n) sum a loss', the curvature
// Hf = (1/n) sum a^2 loss'' and rinv = 1/(Hf + lambda) (constant per coordinate for the ridge loss).
__device__ __forceinline__ float primal_step(double Gf, double Hf, double rinv, float xc, const StepParams& sp,
                                             float& mult) {
    double step;
    if (sp.lambda1 == 0.0) {
        step = -(Gf + sp.lambda * (double)xc) * rinv;
    } else {
        // minimiser of Gf d + (Hf/2) d^2 + (lambda/2)(x+d)^2 + lambda1 |x+d|: soft threshold
        const double t = Hf * (double)xc - Gf;
        const double s = t - fmax(-sp.lambda1, fmin(t, sp.lambda1));       // t minus its clamp to [-lambda1, lambda1]
        step = s * rinv - (double)xc;
    }
    const float xn = (float)((double)xc + sp.damping * step);
    mult = (float)((double)xn - (double)xc);
    return xn;
}

// The scalar step.  Returns the new value of the coordinate; `mult` receives the multiplier of a_j
// that is added to v: the change actually applied to the fp32 coordinate (times y_i in the hinge
// dual), so that v keeps tracking A x as closely as fp32 allows.
template <int KIND>
__device__ __forceinline__ float take_step(double g, double h, float xc, float norm, float yc,
                                           const StepParams& sp, float& mult) {
    float xn;
    if (KIND == K_PRIMAL_RIDGE || KIND == K_PRIMAL_LOGISTIC) {
        const double Hf = (KIND == K_PRIMAL_RIDGE ? (double)norm : h) * sp.inv_n;
        xn = primal_step(g * sp.inv_n, Hf, 1.0 / (Hf + sp.lambda), xc, sp, mult);
    } else {
        double anew;
        if (sp.dual_logistic) {
            // -n dD/da = ln(a/(1-a)) + m,  -n d2D/da2 = 1/(a(1-a)) + q: one Newton step, kept inside (0,1)
            const double a = (double)xc;
            const double m = (double)yc * g * sp.inv_lam_n, q = (double)norm * sp.inv_lam_n;
            anew = a - (log(a) - log1p(-a) + m) / (1.0 / (a * (1.0 - a)) + q);
            anew = anew < ALPHA_EPS ? ALPHA_EPS : (anew > 1.0 - ALPHA_EPS ? 1.0 - ALPHA_EPS : anew);
        } else if (norm == 0.0f) {
            anew = 1.0;                                   // empty row: dD/dalpha = 1/n > 0
        } else {
            // (fp64 divisions are long instruction sequences on the one lane that takes the step, and
            // with few rows in flight the step is on the critical path: one is left)
            const double m = (double)yc * g * sp.inv_lam_n;   // y_i x_i.w
            anew = (double)xc + (1.0 - m) * sp.lam_n / (double)norm;
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
    sp.dual_logistic = (h->form == SNAP_DUAL && h->loss == SNAP_LOGISTIC) ? 1 : 0;
    sp.inv_n = 1.0 / (double)h->n;
    sp.lam_n = h->lambda * (double)h->n;
    sp.inv_lam_n = 1.0 / sp.lam_n;
    sp.damping = (double)h->damping;
    return sp;
}

}  // namespace snap
