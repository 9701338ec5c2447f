// Pure host pieces shared by the GPU path's host side and the host-CPU step: error reporting,
// argument checks and the per-step scalars.  No HIP types here, so the host compiler can use it.
#pragma once

#include <cmath>
#include <cstddef>
#include <cstdint>

#include "zi.h"

namespace zi {

// Per-step constants of the update, every one already rounded to fp32 on the host.
struct StepConsts {
    float beta1, beta2, omb1, omb2, eps, step_size, inv_sqrt_bc2, decay, weight_decay;
    float loss_scale;      // as given by the caller
    float max_grad_norm;   // <= 0: no clipping
    float host_gscale;     // 1 / loss_scale: the gradient factor of a step that does not clip
    uint32_t scale_is_pow2;     // loss_scale is a power of two: dividing by it is multiplying by its inverse, exactly
    uint32_t max_norm_is_pow2;  // max_grad_norm is a power of two: max_grad_norm / x is max_grad_norm * (1 / x), exactly
    double inv_loss_scale;      // 1 / loss_scale in double (exact when scale_is_pow2)
};

namespace host {

// Stores the calling thread's error text (returned by zi_last_error) and passes the status through.
zi_status fail(zi_status st, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
const char* last_error();

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline zi_status check_dtype(int dt)
{
    if (dt != ZI_BF16 && dt != ZI_FP16) return fail(ZI_ERR_INVALID_ARG, "unknown low-precision dtype %d", dt);
    return ZI_OK;
}

inline zi_status check_config(const zi_adamw_config* c)
{
    if (!c) return fail(ZI_ERR_INVALID_ARG, "cfg is NULL");
    if (c->step < 1) return fail(ZI_ERR_INVALID_ARG, "step must be >= 1 (got %lld)", (long long)c->step);
    if (!(c->beta1 >= 0.0f && c->beta1 < 1.0f)) return fail(ZI_ERR_INVALID_ARG, "beta1 must be in [0,1)");
    if (!(c->beta2 >= 0.0f && c->beta2 < 1.0f)) return fail(ZI_ERR_INVALID_ARG, "beta2 must be in [0,1)");
    if (!(c->eps >= 0.0f) || std::isinf(c->eps)) return fail(ZI_ERR_INVALID_ARG, "eps must be finite and >= 0");
    if (!std::isfinite(c->lr)) return fail(ZI_ERR_INVALID_ARG, "lr must be finite");
    if (!std::isfinite(c->weight_decay)) return fail(ZI_ERR_INVALID_ARG, "weight_decay must be finite");
    if (!(c->loss_scale > 0.0f) || std::isinf(c->loss_scale))
        return fail(ZI_ERR_INVALID_ARG, "loss_scale must be finite and > 0");
    if (std::isnan(c->max_grad_norm)) return fail(ZI_ERR_INVALID_ARG, "max_grad_norm is NaN");
    if (c->mode != ZI_MODE_ADAMW && c->mode != ZI_MODE_ADAM_L2)
        return fail(ZI_ERR_INVALID_ARG, "unknown mode %d", c->mode);
    return ZI_OK;
}

// Tensor list of a step: pointers present and aligned to their element size.
inline zi_status check_step_tensors(const zi_tensor* t, int32_t n)
{
    if (n < 0) return fail(ZI_ERR_INVALID_ARG, "n_tensors < 0");
    if (n > 0 && !t) return fail(ZI_ERR_INVALID_ARG, "tensor list is NULL");
    for (int32_t i = 0; i < n; ++i) {
        if (t[i].numel < 0) return fail(ZI_ERR_INVALID_ARG, "tensor %d: numel < 0", i);
        if (t[i].numel == 0) continue;
        if (!t[i].p || !t[i].m || !t[i].v || !t[i].g)
            return fail(ZI_ERR_INVALID_ARG, "tensor %d: p, m, v and g must not be NULL", i);
        if (!aligned(t[i].p, 4) || !aligned(t[i].m, 4) || !aligned(t[i].v, 4))
            return fail(ZI_ERR_ALIGNMENT, "tensor %d: p, m, v must be 4-byte aligned", i);
        if (!aligned(t[i].g, 2) || !aligned(t[i].p_lp, 2))
            return fail(ZI_ERR_ALIGNMENT, "tensor %d: g and p_lp must be 2-byte aligned", i);
        // the five byte ranges of a tensor must be pairwise disjoint (views that overlap in part included)
        const uintptr_t n = (uintptr_t)t[i].numel;
        const uintptr_t lo[5] = {(uintptr_t)t[i].p, (uintptr_t)t[i].m, (uintptr_t)t[i].v, (uintptr_t)t[i].g,
                                 (uintptr_t)t[i].p_lp};
        const uintptr_t len[5] = {4 * n, 4 * n, 4 * n, 2 * n, t[i].p_lp ? 2 * n : 0};
        static const char* const name[5] = {"p", "m", "v", "g", "p_lp"};
        for (int a = 0; a < 5; ++a)
            for (int b = a + 1; b < 5; ++b)
                if (len[a] && len[b] && lo[a] < lo[b] + len[b] && lo[b] < lo[a] + len[a])
                    return fail(ZI_ERR_INVALID_ARG, "tensor %d: %s and %s overlap", i, name[a], name[b]);
    }
    return ZI_OK;
}

// Per-step constants, in double, each rounded once to fp32.
inline zi::StepConsts make_consts(const zi_adamw_config& c)
{
    zi::StepConsts k{};
    const double b1 = (double)c.beta1, b2 = (double)c.beta2;
    const double bc1 = 1.0 - std::pow(b1, (double)c.step);
    const double bc2 = 1.0 - std::pow(b2, (double)c.step);
    k.beta1 = c.beta1;
    k.beta2 = c.beta2;
    k.omb1 = (float)(1.0 - b1);
    k.omb2 = (float)(1.0 - b2);
    k.eps = c.eps;
    k.step_size = (float)((double)c.lr / bc1);
    k.inv_sqrt_bc2 = (float)(1.0 / std::sqrt(bc2));
    k.decay = c.mode == ZI_MODE_ADAMW ? (float)((double)c.lr * (double)c.weight_decay) : 0.0f;
    k.weight_decay = c.weight_decay;
    k.loss_scale = c.loss_scale;
    k.max_grad_norm = c.max_grad_norm;
    k.host_gscale = (float)(1.0 / (double)c.loss_scale);
    int exponent = 0;
    k.scale_is_pow2 = std::frexp((double)c.loss_scale, &exponent) == 0.5 ? 1u : 0u;
    k.inv_loss_scale = 1.0 / (double)c.loss_scale;
    k.max_norm_is_pow2 = c.max_grad_norm > 0.0f && std::frexp((double)c.max_grad_norm, &exponent) == 0.5 ? 1u : 0u;
    return k;
}

// Gradient factor of a step that has a norm result (host-side twin of the kernels' prologue, same
// expressions in double): norm = sqrt(sumsq) / loss_scale, clip = max_norm / (norm + 1e-6) when that
// is below 1, factor = clip / loss_scale rounded once to fp32.
inline float gradient_factor(double sumsq, const zi::StepConsts& c)
{
    const double norm = std::sqrt(sumsq) / (double)c.loss_scale;
    const double mx = (double)c.max_grad_norm;
    double clip = 1.0;
    if (c.max_grad_norm > 0.0f && norm + 1e-6 > mx) clip = mx / (norm + 1e-6);
    return (float)(clip / (double)c.loss_scale);
}

// Gradient list of a reduction: only g and numel of each tensor are looked at.
inline zi_status check_grad_list(const zi_tensor* t, int32_t n_tensors, float loss_scale)
{
    if (n_tensors < 0) return fail(ZI_ERR_INVALID_ARG, "n_tensors < 0");
    if (n_tensors > 0 && !t) return fail(ZI_ERR_INVALID_ARG, "tensor list is NULL");
    if (!(loss_scale > 0.0f) || std::isinf(loss_scale))
        return fail(ZI_ERR_INVALID_ARG, "loss_scale must be finite and > 0");
    for (int32_t i = 0; i < n_tensors; ++i) {
        if (t[i].numel < 0) return fail(ZI_ERR_INVALID_ARG, "tensor %d: numel < 0", i);
        if (t[i].numel > 0 && !t[i].g) return fail(ZI_ERR_INVALID_ARG, "tensor %d: g is NULL", i);
        if (!aligned(t[i].g, 2)) return fail(ZI_ERR_ALIGNMENT, "tensor %d: g must be 2-byte aligned", i);
    }
    return ZI_OK;
}

// The host-CPU step over elements [lo, hi) of one tensor (zi_cpu_step.cpp; AVX2 / FMA / F16C): the
// routine behind zi_host_adamw_step, also used by the engine when the step runs on the CPUs while
// gradients and the copy cross the link.  g / lp are indexed like p, m, v.  lp may be null.
void host_step_range(const zi::StepConsts& c, float gscale, int dt, bool l2, float* p, float* m, float* v,
                     const uint16_t* g, uint16_t* lp, int64_t lo, int64_t hi);
bool host_step_supported();     // the CPU has the vector instructions the routine is written with

}  // namespace host
}  // namespace zi
