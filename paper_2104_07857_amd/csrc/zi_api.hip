// C-ABI entry points of the HBM-resident path: queries, gradient norm, fused step, HBM probe, pinned
// memory helpers.  See include/zi.h for the contract of every call.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <mutex>
#include <new>
#include <vector>

#include "zi_host.h"

namespace zi {
namespace host {

namespace {
thread_local char g_err[512] = "";
}

zi_status fail(zi_status st, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

const char* last_error() { return g_err; }

}  // namespace host
}  // namespace zi

using namespace zi::host;

// ============================================================================ plain queries

extern "C" const char* zi_last_error(void) { return last_error(); }

extern "C" size_t zi_norm_workspace_bytes(int64_t, int32_t)
{
    return (size_t)zi::kMaxPartials * sizeof(zi::NormPartial);
}

// ================================================================================ grad norm

extern "C" zi_status zi_grad_norm(const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt, float loss_scale,
                                  zi_norm_result* d_out, void* d_workspace, size_t workspace_bytes,
                                  void* hip_stream)
{
    if (zi_status st = check_norm_args(t, n_tensors, (int)dt, loss_scale, d_out, d_workspace, workspace_bytes)) return st;
    if (zi_status st = check_kernel_visible(d_out, sizeof(zi_norm_result), -1, "d_out")) return st;
    if (zi_status st = check_kernel_visible(d_workspace, workspace_bytes, -1, "d_workspace")) return st;
    PointerChecker reach;
    for (int32_t i = 0; i < n_tensors; ++i)
        if (zi_status st = reach.check(t[i].g, (size_t)t[i].numel * 2, i, "g")) return st;

    NormIssuer issue((zi::NormPartial*)d_workspace, (int)dt, loss_scale, d_out, (hipStream_t)hip_stream);
    for (int32_t i = 0; i < n_tensors; ++i) ZI_HIP(issue.add((const uint16_t*)t[i].g, t[i].numel));
    ZI_HIP(issue.finish());   // also writes zeros for an empty list
    return ZI_OK;
}

// ------------------------------------------------------------ grad norm without a workspace
//
// For callers that cannot allocate (code under graph capture, tight serving loops, harnesses that
// forbid it): the per-block partials live in a fixed array in the device image of this library
// instead of a caller-provided workspace.  Each GPU holds its own copy at its own address; the name
// below is only a host-side stand-in, so the device address is looked up once per device and that
// pointer is what the kernels get.
static __device__ __align__(256) unsigned char scratch[ZI_NOALLOC_MAX_PARTIALS * sizeof(zi::NormPartial)];

namespace {

constexpr int kMaxScratchDevices = 64;
std::mutex g_scratch_mu;
zi::NormPartial* g_scratch_ptr[kMaxScratchDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call on that device).
zi_status scratch_for_current_device(zi::NormPartial** out)
{
    int dev = -1;
    ZI_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxScratchDevices)
        return fail(ZI_ERR_UNSUPPORTED, "device ordinal %d is beyond the %d this call keeps scratch pointers for", dev,
                    kMaxScratchDevices);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        ZI_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(ZI_ERR_HIP, "hipGetSymbolAddress gave a null address for the scratch array");
        g_scratch_ptr[dev] = static_cast<zi::NormPartial*>(ptr);
    }
    *out = g_scratch_ptr[dev];
    return ZI_OK;
}

}  // namespace

extern "C" zi_status zi_grad_norm_noalloc(const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt, float loss_scale,
                                          zi_norm_result* d_out, void* hip_stream)
{
    static_assert(ZI_NOALLOC_MAX_PARTIALS <= zi::kMaxPartials, "the issuer counts partials against kMaxPartials");
    zi::NormPartial* partials = nullptr;
    if (zi_status st = scratch_for_current_device(&partials)) return st;
    if (zi_status st = check_norm_args(t, n_tensors, (int)dt, loss_scale, d_out, partials,
                                       sizeof(zi::NormPartial) * ZI_NOALLOC_MAX_PARTIALS))
        return st;
    if (zi_status st = check_kernel_visible(d_out, sizeof(zi_norm_result), -1, "d_out")) return st;
    PointerChecker reach;
    int64_t non_empty = 0;
    for (int32_t i = 0; i < n_tensors; ++i) {
        if (zi_status st = reach.check(t[i].g, (size_t)t[i].numel * 2, i, "g")) return st;
        non_empty += t[i].numel > 0;
    }
    // One pass: every partial of the call must fit the fixed array.  Each tensor needs at least one
    // workgroup, so the list length is the hard limit; below it, long tensors get fewer workgroups.
    if (non_empty > ZI_NOALLOC_MAX_PARTIALS)
        return fail(ZI_ERR_UNSUPPORTED, "%lld non-empty gradient tensors: the fixed scratch holds one partial for each of "
                    "at most %d (split the list, or use zi_grad_norm with a workspace)", (long long)non_empty,
                    ZI_NOALLOC_MAX_PARTIALS);
    int64_t cap = NormIssuer::kBlocksPerTensor;
    for (;; cap /= 2) {
        int64_t total = 0;
        for (int32_t i = 0; i < n_tensors; ++i)
            if (t[i].numel > 0) total += NormIssuer::blocks_for(t[i].numel, cap);
        if (total <= ZI_NOALLOC_MAX_PARTIALS || cap == 1) break;
    }

    NormIssuer issue(partials, (int)dt, loss_scale, d_out, (hipStream_t)hip_stream);
    issue.blocks_cap = cap;
    for (int32_t i = 0; i < n_tensors; ++i) ZI_HIP(issue.add((const uint16_t*)t[i].g, t[i].numel));
    ZI_HIP(issue.finish());
    return ZI_OK;
}

extern "C" zi_status zi_norm_refresh(zi_norm_result* d_result, float loss_scale, void* hip_stream)
{
    if (!d_result) return fail(ZI_ERR_INVALID_ARG, "d_result is NULL");
    if (!aligned(d_result, 8)) return fail(ZI_ERR_ALIGNMENT, "d_result must be 8-byte aligned");
    if (zi_status st = check_kernel_visible(d_result, sizeof(zi_norm_result), -1, "d_result")) return st;
    if (!(loss_scale > 0.0f) || std::isinf(loss_scale))
        return fail(ZI_ERR_INVALID_ARG, "loss_scale must be finite and > 0");
    ZI_HIP(zi::launch_norm_refresh(d_result, loss_scale, (hipStream_t)hip_stream));
    return ZI_OK;
}

// =============================================================================== resident step

extern "C" zi_status zi_adamw_step(const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt,
                                   const zi_adamw_config* cfg, const zi_norm_result* d_norm, void* hip_stream)
{
    if (zi_status st = check_dtype((int)dt)) return st;
    if (zi_status st = check_config(cfg)) return st;
    if (zi_status st = check_step_tensors(t, n_tensors)) return st;
    if (d_norm && !aligned(d_norm, 8)) return fail(ZI_ERR_ALIGNMENT, "d_norm must be 8-byte aligned");
    if (zi_status st = check_kernel_visible(d_norm, sizeof(zi_norm_result), -1, "d_norm")) return st;
    PointerChecker reach;
    for (int32_t i = 0; i < n_tensors; ++i) {
        const size_t n = (size_t)t[i].numel;
        if (zi_status st = reach.check(t[i].p, n * 4, i, "p")) return st;
        if (zi_status st = reach.check(t[i].m, n * 4, i, "m")) return st;
        if (zi_status st = reach.check(t[i].v, n * 4, i, "v")) return st;
        if (zi_status st = reach.check(t[i].g, n * 2, i, "g")) return st;
        if (zi_status st = reach.check(t[i].p_lp, n * 2, i, "p_lp")) return st;
    }

    const zi::StepConsts k = make_consts(*cfg);
    StepIssuer issue(k, d_norm, (int)dt, cfg->mode == ZI_MODE_ADAM_L2, (hipStream_t)hip_stream);
    for (int32_t i = 0; i < n_tensors; ++i)
        ZI_HIP(issue.add((float*)t[i].p, (float*)t[i].m, (float*)t[i].v, (const uint16_t*)t[i].g,
                         (uint16_t*)t[i].p_lp, t[i].numel));
    ZI_HIP(issue.flush());
    return ZI_OK;
}

extern "C" zi_status zi_plan_step(const zi_tensor* t, int32_t n_tensors, zi_step_plan_item* out, int64_t cap,
                                  int64_t* n_items_out, int64_t* n_launches_out)
{
    if (zi_status st = check_step_tensors(t, n_tensors)) return st;
    if (cap < 0 || (cap > 0 && !out)) return fail(ZI_ERR_INVALID_ARG, "bad output buffer");
    if (!n_items_out || !n_launches_out) return fail(ZI_ERR_INVALID_ARG, "output counters are NULL");
    std::vector<zi_step_plan_item> items;
    try {
        StepIssuer issue(zi::StepConsts{}, nullptr, ZI_BF16, false, nullptr);
        issue.plan = &items;
        for (int32_t i = 0; i < n_tensors; ++i) {
            issue.cur_tensor = i;
            (void)issue.add((float*)t[i].p, (float*)t[i].m, (float*)t[i].v, (const uint16_t*)t[i].g,
                            (uint16_t*)t[i].p_lp, t[i].numel);
        }
        (void)issue.flush();
        *n_launches_out = issue.launches;
    } catch (const std::bad_alloc&) {
        return fail(ZI_ERR_NOMEM, "out of host memory while planning");
    }
    for (int64_t i = 0; i < (int64_t)items.size() && i < cap; ++i) out[i] = items[(size_t)i];
    *n_items_out = (int64_t)items.size();
    return ZI_OK;
}

// ================================================================================ pinned memory

extern "C" zi_status zi_pinned_alloc(void** out, size_t bytes)
{
    if (!out) return fail(ZI_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (bytes == 0) return fail(ZI_ERR_INVALID_ARG, "bytes is 0");
    hipError_t e = hipHostMalloc(out, bytes, hipHostMallocDefault);
    if (e != hipSuccess) {
        *out = nullptr;
        (void)hipGetLastError();   // a failed allocation must not poison the caller's next HIP call
        return fail(e == hipErrorOutOfMemory ? ZI_ERR_NOMEM : ZI_ERR_HIP, "hipHostMalloc(%zu) failed: %s", bytes,
                    hipGetErrorString(e));
    }
    return ZI_OK;
}

extern "C" zi_status zi_pinned_free(void* ptr)
{
    if (!ptr) return ZI_OK;
    ZI_HIP(hipHostFree(ptr));
    return ZI_OK;
}

