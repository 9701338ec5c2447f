// Entry points around the streamed step that move the 2-byte arrays rather than the state:
//   zi_grad_offload / zi_grad_offload_wait / zi_grad_offload_order   freshly produced gradient partitions
//       leave for host memory on the engine's device-to-host stream while their producer keeps running;
//   zi_adamw_step_cpu   the step itself on the host CPUs over host-resident state, with only gradients
//       coming down the link and the low-precision copy going up, the three stages overlapped
//       through the engine's pinned ring.
// See include/zi.h for the contract of every call.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstring>

#include "zi_engine_internal.h"

using namespace zi::host;

// ============================================================================ gradient offload

extern "C" zi_status zi_grad_offload(zi_engine* e, const void* d_src, void* h_dst, size_t bytes,
                                     void* producer_stream)
{
    if (zi_status st = check_engine(e)) return st;
    if (bytes == 0) return ZI_OK;
    if (!d_src || !h_dst) return fail(ZI_ERR_INVALID_ARG, "d_src and h_dst must not be NULL");
    PointerChecker reach;
    if (memory_kind(d_src) != 0) return fail(ZI_ERR_INVALID_ARG, "d_src must be device memory");
    if (zi_status st = reach.check(d_src, bytes, -1, "d_src")) return st;
    if (memory_kind(h_dst) != 1 || memory_kind(static_cast<const char*>(h_dst) + bytes - 1) != 1)
        return fail(ZI_ERR_INVALID_ARG, "h_dst (%zu bytes) must be page-locked host memory", bytes);
    ZI_HIP(hipSetDevice(e->device));

    // One event per call orders the copy after everything the producer has enqueued so far.  The
    // events are reused round-robin; before a reuse, the copy that waited on the event is long
    // done (64 offloads ago), which the host makes sure of.
    const int idx = (int)(e->n_offloads % kOffloadEvents);
    if (e->n_offloads >= (uint64_t)kOffloadEvents) ZI_HIP(hipEventSynchronize(e->ev_offload[idx]));
    ZI_HIP(hipEventRecord(e->ev_offload[idx], (hipStream_t)producer_stream));
    ZI_HIP(hipStreamWaitEvent(e->s_d2h, e->ev_offload[idx], 0));
    ZI_HIP(hipMemcpyAsync(h_dst, d_src, bytes, hipMemcpyDeviceToHost, e->s_d2h));
    ZI_HIP(hipEventRecord(e->ev_offload_done, e->s_d2h));
    ++e->n_offloads;
    e->offload_pending = true;
    return ZI_OK;
}

extern "C" zi_status zi_grad_offload_wait(zi_engine* e)
{
    if (zi_status st = check_engine(e)) return st;
    if (!e->offload_pending) return ZI_OK;
    ZI_HIP(hipSetDevice(e->device));
    ZI_HIP(hipEventSynchronize(e->ev_offload_done));
    e->offload_pending = false;
    return ZI_OK;
}

extern "C" zi_status zi_grad_offload_order(zi_engine* e, void* consumer_stream)
{
    if (zi_status st = check_engine(e)) return st;
    ZI_HIP(hipSetDevice(e->device));
    ZI_HIP(order_after_offloads(e, (hipStream_t)consumer_stream));
    return ZI_OK;
}

// ====================================================================== the step on the host CPUs

namespace {

// One block of one segment for the host step's thread pool.
struct CpuBlock {
    float *p, *m, *v;
    const uint16_t* g;
    uint16_t* lp;
    int64_t n;
};

struct CpuJob {
    const CpuBlock* blocks;
    zi::StepConsts c;
    float gscale;
    int dt;
    bool l2;
};

int run_cpu_block(void* ctx, size_t index, int)
{
    const CpuJob& job = *static_cast<const CpuJob*>(ctx);
    const CpuBlock& b = job.blocks[index];
    host_step_range(job.c, job.gscale, job.dt, job.l2, b.p, b.m, b.v, b.g, b.lp, 0, b.n);
    return 0;
}

// Elements per task of the thread pool: 64 KiB of each fp32 array.  A chunk of 2^24 elements is 1024
// tasks, so the barrier at the end of every chunk finds the threads within one short task of each
// other (2^18-element tasks measured 4% slower, 2^16 2% slower).
constexpr int64_t kCpuBlockElems = (int64_t)1 << 14;

}  // namespace

extern "C" zi_status zi_adamw_step_cpu(zi_engine* e, const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt,
                                       const zi_adamw_config* cfg, const zi_norm_result* d_norm,
                                       int32_t n_threads, void* hip_stream)
{
    ZI_GUARD_BEGIN
    if (zi_status st = check_engine(e)) return st;
    if (!host_step_supported()) return fail(ZI_ERR_UNSUPPORTED, "the host step needs a CPU with AVX2, FMA and F16C");
    if (n_threads < 1 || n_threads > 256) return fail(ZI_ERR_INVALID_ARG, "n_threads must be in 1..256");
    if (zi_status st = check_dtype((int)dt)) return st;
    if (zi_status st = check_config(cfg)) return st;
    if (zi_status st = check_step_tensors(t, n_tensors)) return st;
    if (d_norm && !aligned(d_norm, 8)) return fail(ZI_ERR_ALIGNMENT, "d_norm must be 8-byte aligned");
    if (zi_status st = check_kernel_visible(d_norm, sizeof(zi_norm_result), -1, "d_norm")) return st;
    ZI_HIP(hipSetDevice(e->device));
    hipStream_t user = (hipStream_t)hip_stream;
    e->stats = zi_stream_stats{};

    // p, m, v: host memory of any kind (the CPUs work on them in place).  g, p_lp: device memory
    // (staged through the pinned ring, chunk by chunk) or host memory (used in place).
    bool any_device = false;
    PointerChecker reach;
    e->src.resize((size_t)n_tensors);
    for (int32_t i = 0; i < n_tensors; ++i) {
        StateSrc& S = e->src[(size_t)i];
        S = StateSrc{};
        S.ptr[0] = (char*)t[i].p; S.ptr[1] = (char*)t[i].m; S.ptr[2] = (char*)t[i].v;
        S.g = t[i].g; S.p_lp = t[i].p_lp; S.numel = t[i].numel;
        S.g_host = S.lp_host = true;
        if (t[i].numel == 0) continue;
        const size_t n = (size_t)t[i].numel;
        for (int w = 0; w < 3; ++w) {
            const int k0 = memory_kind(S.ptr[w]), k1 = memory_kind(S.ptr[w] + n * 4 - 1);
            if (k0 == -2) return fail(ZI_ERR_HIP, "no usable HIP device (pointer query failed)");
            if ((k0 != 1 && k0 != 2) || k1 != k0)
                return fail(ZI_ERR_INVALID_ARG, "tensor %d: p, m, v must be host memory", i);
        }
        const int gk = memory_kind(S.g);
        if (gk < 0) return fail(ZI_ERR_INVALID_ARG, "tensor %d: g is neither device nor host memory", i);
        if (gk == 0) {
            if (zi_status st = reach.check(S.g, n * 2, i, "g")) return st;
            S.g_host = false;
            any_device = true;
        }
        if (S.p_lp) {
            const int lk = memory_kind(S.p_lp);
            if (lk < 0) return fail(ZI_ERR_INVALID_ARG, "tensor %d: p_lp is neither device nor host memory", i);
            if (lk == 0) {
                if (zi_status st = reach.check(S.p_lp, n * 2, i, "p_lp")) return st;
                S.lp_host = false;
                any_device = true;
            }
        }
    }
    const int n_h = e->n_hslots;
    if (any_device && n_h < 3)
        return fail(ZI_ERR_INVALID_ARG, "device-resident gradients or copy need a pinned ring of at least 3 slots "
                                        "(ZI_OPT_HOST_RING_SLOTS)");
    if (!e->pool_step || e->pool_step->threads() != n_threads) {
        delete e->pool_step;
        e->pool_step = new TaskPool(n_threads);
    }

    e->plan_numel.resize((size_t)n_tensors);
    for (int32_t i = 0; i < n_tensors; ++i) e->plan_numel[(size_t)i] = t[i].numel;
    int64_t n_uses = 0;
    plan_chunks(e->plan_numel.data(), n_tensors, e->chunk_elems, e->segs, n_uses);
    index_uses(e->segs, n_uses, e->use_begin);
    const std::vector<Segment>& segs = e->segs;
    const std::vector<size_t>& use_begin = e->use_begin;

    // The flag and the sum of squares come to the host first: a skipped step touches nothing.
    zi::StepConsts k = make_consts(*cfg);
    float gscale = k.host_gscale;
    if (d_norm) {
        ZI_HIP(hipMemcpyAsync(e->h_norm, d_norm, sizeof(zi_norm_result), hipMemcpyDeviceToHost, user));
        ZI_HIP(hipStreamSynchronize(user));
        if (e->h_norm->found_inf) return ZI_SKIPPED_OVERFLOW;
        gscale = gradient_factor(e->h_norm->sumsq, k);
    }
    // Gradients produced on the caller's stream are complete before they are fetched; gradient
    // offloads on their way to host memory are complete before the CPUs read them.
    ZI_HIP(hipEventRecord(e->ev_in, user));
    ZI_HIP(hipStreamWaitEvent(e->s_d2h, e->ev_in, 0));
    ZI_HIP(hipStreamWaitEvent(e->s_h2d, e->ev_in, 0));
    if (e->offload_pending) {
        ZI_HIP(hipEventSynchronize(e->ev_offload_done));
        e->offload_pending = false;
    }

    const auto t0 = std::chrono::steady_clock::now();
    // Ring slot u mod n_h carries slot use u: its gradient half is filled by a device-to-host copy,
    // the CPUs step the use (reading that half, writing the copy half), a host-to-device copy ships
    // the copy half.  Fetches run `ahead` uses in front of the CPUs; a slot is fetched into again
    // only after the upload of its previous use has left it, which by then is two steps old.
    const int ahead = n_h >= 3 ? n_h - 2 : 1;
    auto fetch = [&](int64_t u) -> zi_status {
        const int h = n_h > 0 ? (int)(u % n_h) : 0;
        bool any = false;
        for (size_t j = use_begin[(size_t)u]; j < use_begin[(size_t)u + 1]; ++j) {
            const Segment& sg = segs[j];
            const StateSrc& S = e->src[(size_t)sg.tensor];
            if (S.g_host) continue;
            if (!any && u >= n_h) ZI_HIP(hipEventSynchronize(e->ev_back[h]));
            any = true;
            ZI_HIP(hipMemcpyAsync(e->hslot_g(h) + sg.slot_offset, (const uint16_t*)S.g + sg.elem_offset,
                                  (size_t)sg.count * 2, hipMemcpyDeviceToHost, e->s_d2h));
            e->stats.bytes_d2h += (size_t)sg.count * 2;
            e->stats.n_copies += 1;
        }
        if (any) ZI_HIP(hipEventRecord(e->ev_fill[h], e->s_d2h));
        return ZI_OK;
    };
    auto pipeline = [&]() -> zi_status {
        std::vector<CpuBlock> blocks;
        for (int64_t u = 0; u < n_uses && u < ahead; ++u)
            if (zi_status st = fetch(u)) return st;
        for (int64_t u = 0; u < n_uses; ++u) {
            if (u + ahead < n_uses)
                if (zi_status st = fetch(u + ahead)) return st;
            const int h = n_h > 0 ? (int)(u % n_h) : 0;
            blocks.clear();
            bool fetched = false, upload = false;
            for (size_t j = use_begin[(size_t)u]; j < use_begin[(size_t)u + 1]; ++j) {
                const Segment& sg = segs[j];
                const StateSrc& S = e->src[(size_t)sg.tensor];
                fetched = fetched || !S.g_host;
                upload = upload || (S.p_lp && !S.lp_host);
                const uint16_t* g = S.g_host ? (const uint16_t*)S.g + sg.elem_offset : e->hslot_g(h) + sg.slot_offset;
                uint16_t* lp = !S.p_lp ? nullptr
                               : S.lp_host ? (uint16_t*)S.p_lp + sg.elem_offset : e->hslot_lp(h) + sg.slot_offset;
                for (int64_t o = 0; o < sg.count; o += kCpuBlockElems) {
                    const int64_t nb = sg.count - o < kCpuBlockElems ? sg.count - o : kCpuBlockElems;
                    const int64_t at = sg.elem_offset + o;
                    blocks.push_back({(float*)S.ptr[0] + at, (float*)S.ptr[1] + at, (float*)S.ptr[2] + at, g + o,
                                      lp ? lp + o : nullptr, nb});
                }
            }
            // A ring slot whose upload of `n_h` uses ago is still leaving must not be written yet
            // (uses with host-resident gradients skip the fetch that would have waited for it).
            if (upload && !fetched && u >= n_h) ZI_HIP(hipEventSynchronize(e->ev_back[h]));
            if (fetched) ZI_HIP(hipEventSynchronize(e->ev_fill[h]));
            CpuJob job{blocks.data(), k, gscale, (int)dt, cfg->mode == ZI_MODE_ADAM_L2};
            (void)e->pool_step->run(blocks.size(), run_cpu_block, &job);
            for (size_t j = use_begin[(size_t)u]; j < use_begin[(size_t)u + 1]; ++j) {
                const Segment& sg = segs[j];
                const StateSrc& S = e->src[(size_t)sg.tensor];
                if (!S.p_lp || S.lp_host) continue;
                ZI_HIP(hipMemcpyAsync((uint16_t*)S.p_lp + sg.elem_offset, e->hslot_lp(h) + sg.slot_offset,
                                      (size_t)sg.count * 2, hipMemcpyHostToDevice, e->s_h2d));
                e->stats.bytes_h2d += (size_t)sg.count * 2;
                e->stats.n_copies += 1;
            }
            if (upload || fetched) ZI_HIP(hipEventRecord(e->ev_back[h], e->s_h2d));
            ++e->stats.n_slot_uses;
        }
        // The copy is complete on return, and later work on the caller's stream sees it.
        ZI_HIP(hipEventRecord(e->ev_out, e->s_h2d));
        ZI_HIP(hipStreamWaitEvent(user, e->ev_out, 0));
        ZI_HIP(hipStreamSynchronize(e->s_h2d));
        ZI_HIP(hipStreamSynchronize(e->s_d2h));
        return ZI_OK;
    };
    const zi_status st = pipeline();
    if (st != ZI_OK) drain_streams(e);
    e->stats.seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    return st;
    ZI_GUARD_END
}
