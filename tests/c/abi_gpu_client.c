/*
 * A plain C99 caller of the GPU entry points: built as a small shared object by the test, loaded into
 * the test's process, and handed device buffers as plain addresses.  Everything it knows about the
 * library comes from include/zi.h.  It runs the resident path (zi_grad_norm, then zi_adamw_step reading
 * that result on the device) and the no-allocation variant of the reduction, and returns the status
 * codes; the test checks the arrays against the oracle.
 */
#include <stdint.h>
#include <string.h>

#include "zi.h"

struct client_args {
    uint64_t p, m, v, g, p_lp;        /* device addresses */
    int64_t numel;
    uint64_t d_norm, d_norm2;         /* device, sizeof(zi_norm_result) each */
    uint64_t d_workspace;
    uint64_t workspace_bytes;
    uint64_t hip_stream;
    int32_t lp_dtype;
    int32_t step;
    float loss_scale, max_grad_norm;
};

/* Returns 0 if every call returned ZI_OK; otherwise 100 * (index of the failing call) - status. */
int zi_c_client_run(const struct client_args* a, char* err, size_t err_len)
{
    zi_tensor t;
    zi_adamw_config cfg;
    zi_status st;

    memset(&t, 0, sizeof t);
    t.p = (void*)(uintptr_t)a->p;
    t.m = (void*)(uintptr_t)a->m;
    t.v = (void*)(uintptr_t)a->v;
    t.g = (const void*)(uintptr_t)a->g;
    t.p_lp = (void*)(uintptr_t)a->p_lp;
    t.numel = a->numel;

    memset(&cfg, 0, sizeof cfg);
    cfg.lr = 1e-3f; cfg.beta1 = 0.9f; cfg.beta2 = 0.999f; cfg.eps = 1e-8f; cfg.weight_decay = 0.01f;
    cfg.step = a->step; cfg.loss_scale = a->loss_scale; cfg.max_grad_norm = a->max_grad_norm;
    cfg.mode = ZI_MODE_ADAMW;

    if (a->workspace_bytes < zi_norm_workspace_bytes(a->numel, 1)) return 1;
    st = zi_grad_norm(&t, 1, (zi_lp_dtype)a->lp_dtype, a->loss_scale, (zi_norm_result*)(uintptr_t)a->d_norm,
                      (void*)(uintptr_t)a->d_workspace, (size_t)a->workspace_bytes, (void*)(uintptr_t)a->hip_stream);
    if (st != ZI_OK) { strncpy(err, zi_last_error(), err_len - 1); return 100 - (int)st; }
    st = zi_grad_norm_noalloc(&t, 1, (zi_lp_dtype)a->lp_dtype, a->loss_scale, (zi_norm_result*)(uintptr_t)a->d_norm2,
                              (void*)(uintptr_t)a->hip_stream);
    if (st != ZI_OK) { strncpy(err, zi_last_error(), err_len - 1); return 200 - (int)st; }
    st = zi_adamw_step(&t, 1, (zi_lp_dtype)a->lp_dtype, &cfg, (const zi_norm_result*)(uintptr_t)a->d_norm,
                       (void*)(uintptr_t)a->hip_stream);
    if (st != ZI_OK) { strncpy(err, zi_last_error(), err_len - 1); return 300 - (int)st; }
    /* a host pointer where device memory is required comes back as a code, not as a fault */
    t.p = (void*)&cfg;
    t.numel = 1;
    st = zi_adamw_step(&t, 1, (zi_lp_dtype)a->lp_dtype, &cfg, NULL, (void*)(uintptr_t)a->hip_stream);
    if (st != ZI_ERR_INVALID_ARG) return 400 - (int)st;
    return 0;
}
