// The streaming engine: staging slots in HBM, three streams, event-ordered slot reuse, the pinned
// ring for state that is not page-locked (ordinary memory or files), and the entry points built on it.
// See include/zi.h for the contract of every call.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdio>
#include <cstring>
#include <new>

#include "zi_engine_internal.h"

using namespace zi::host;

namespace {

// A pool of `n` parked threads / one parked stage thread, or null if memory or threads cannot be had.
TaskPool* make_pool(int n)
{
    try {
        return new TaskPool(n);
    } catch (const std::exception&) {
        return nullptr;
    }
}

StageThread* make_stage()
{
    try {
        return new StageThread();
    } catch (const std::exception&) {
        return nullptr;
    }
}

void ring_release(zi_engine* e)
{
    delete e->stage_in;
    delete e->stage_out;
    e->stage_in = e->stage_out = nullptr;
    delete e->pool_in;
    delete e->pool_out;
    e->pool_in = e->pool_out = nullptr;
    for (int i = 0; i < kMaxHostSlots; ++i) {
        if (e->ev_back[i]) (void)hipEventDestroy(e->ev_back[i]);
        if (e->ev_fill[i]) (void)hipEventDestroy(e->ev_fill[i]);
        e->ev_back[i] = e->ev_fill[i] = nullptr;
    }
    if (e->hring) (void)hipHostFree(e->hring);
    e->hring = nullptr;
    e->n_hslots = 0;
}

void engine_release(zi_engine* e)
{
    for (int i = 0; i < 8; ++i) {
        if (e->ev_h2d[i]) (void)hipEventDestroy(e->ev_h2d[i]);
        if (e->ev_k[i]) (void)hipEventDestroy(e->ev_k[i]);
        if (e->ev_d2h[i]) (void)hipEventDestroy(e->ev_d2h[i]);
        if (e->ev_out_start[i]) (void)hipEventDestroy(e->ev_out_start[i]);
    }
    for (int i = 0; i < kOffloadEvents; ++i)
        if (e->ev_offload[i]) (void)hipEventDestroy(e->ev_offload[i]);
    if (e->ev_offload_done) (void)hipEventDestroy(e->ev_offload_done);
    if (e->ev_in) (void)hipEventDestroy(e->ev_in);
    if (e->ev_out) (void)hipEventDestroy(e->ev_out);
    if (e->s_h2d) (void)hipStreamDestroy(e->s_h2d);
    if (e->s_k) (void)hipStreamDestroy(e->s_k);
    if (e->s_d2h) (void)hipStreamDestroy(e->s_d2h);
    if (e->staging) (void)hipFree(e->staging);
    if (e->h_norm) (void)hipHostFree(e->h_norm);
    ring_release(e);
    delete e->pool_step;
    e->pool_step = nullptr;
    e->magic = 0;
    delete e;
}

}  // namespace

extern "C" zi_status zi_engine_create(zi_engine** out, int32_t device, size_t chunk_bytes_per_array,
                                      int32_t n_slots)
{
    if (!out) return fail(ZI_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (device < 0) return fail(ZI_ERR_INVALID_ARG, "device < 0");
    if (chunk_bytes_per_array == 0 || chunk_bytes_per_array % 4096)
        return fail(ZI_ERR_INVALID_ARG, "chunk_bytes_per_array must be a positive multiple of 4096");
    if (chunk_bytes_per_array > ((size_t)1 << 34))
        return fail(ZI_ERR_INVALID_ARG, "chunk_bytes_per_array above 16 GiB");
    if (n_slots < 2 || n_slots > 8) return fail(ZI_ERR_INVALID_ARG, "n_slots must be in 2..8");

    int count = 0;
    ZI_HIP(hipGetDeviceCount(&count));
    if (device >= count) return fail(ZI_ERR_INVALID_ARG, "device %d does not exist (%d devices)", device, count);
    ZI_HIP(hipSetDevice(device));

    zi_engine* e = new (std::nothrow) zi_engine();
    if (!e) return fail(ZI_ERR_NOMEM, "out of host memory");
    e->device = device;
    e->chunk_bytes = chunk_bytes_per_array;
    e->chunk_elems = (int64_t)(chunk_bytes_per_array / 4);
    e->n_slots = n_slots;
    e->array_bytes = chunk_bytes_per_array + 4096;   // room for lead-in elements and a rounded-up last block

#define ZI_HIP_E(call)                                                                           \
    do {                                                                                         \
        hipError_t e_ = (call);                                                                  \
        if (e_ != hipSuccess) {                                                                  \
            (void)hipGetLastError();                                                             \
            engine_release(e);                                                                   \
            return fail(e_ == hipErrorOutOfMemory ? ZI_ERR_NOMEM : ZI_ERR_HIP, "%s failed: %s",   \
                        #call, hipGetErrorString(e_));                                           \
        }                                                                                        \
    } while (0)

    ZI_HIP_E(hipMalloc((void**)&e->staging, (size_t)n_slots * kSlotArrays * e->array_bytes));
    ZI_HIP_E(hipHostMalloc((void**)&e->h_norm, sizeof(zi_norm_result), hipHostMallocDefault));
    ZI_HIP_E(hipStreamCreateWithFlags(&e->s_h2d, hipStreamNonBlocking));
    ZI_HIP_E(hipStreamCreateWithFlags(&e->s_k, hipStreamNonBlocking));
    ZI_HIP_E(hipStreamCreateWithFlags(&e->s_d2h, hipStreamNonBlocking));
    for (int i = 0; i < 8; ++i) {      // all eight: the link probe paces up to eight pieces per direction
        ZI_HIP_E(hipEventCreateWithFlags(&e->ev_h2d[i], hipEventDisableTiming));
        ZI_HIP_E(hipEventCreateWithFlags(&e->ev_k[i], hipEventDisableTiming));
        ZI_HIP_E(hipEventCreateWithFlags(&e->ev_d2h[i], hipEventDisableTiming));
        ZI_HIP_E(hipEventCreateWithFlags(&e->ev_out_start[i], hipEventDisableTiming));
    }
    ZI_HIP_E(hipEventCreateWithFlags(&e->ev_in, hipEventDisableTiming));
    ZI_HIP_E(hipEventCreateWithFlags(&e->ev_out, hipEventDisableTiming));
    for (int i = 0; i < kOffloadEvents; ++i) ZI_HIP_E(hipEventCreateWithFlags(&e->ev_offload[i], hipEventDisableTiming));
    ZI_HIP_E(hipEventCreateWithFlags(&e->ev_offload_done, hipEventDisableTiming));
#undef ZI_HIP_E
    e->magic = kEngineMagic;
    *out = e;
    return ZI_OK;
}

extern "C" zi_status zi_engine_destroy(zi_engine* e)
{
    if (!e) return ZI_OK;
    if (zi_status st = check_engine(e)) return st;
    (void)hipSetDevice(e->device);
    (void)hipStreamSynchronize(e->s_h2d);
    (void)hipStreamSynchronize(e->s_k);
    (void)hipStreamSynchronize(e->s_d2h);
    engine_release(e);
    return ZI_OK;
}

extern "C" zi_status zi_engine_last_stats(const zi_engine* e, zi_stream_stats* out)
{
    if (zi_status st = check_engine(e)) return st;
    if (!out) return fail(ZI_ERR_INVALID_ARG, "out is NULL");
    *out = e->stats;
    return ZI_OK;
}

extern "C" zi_status zi_engine_set_option(zi_engine* e, int32_t option, int64_t value)
{
    if (zi_status st = check_engine(e)) return st;
    if (option == ZI_OPT_SKIP_KERNEL) {
        e->skip_kernel = value != 0;
        return ZI_OK;
    }
    if (option == ZI_OPT_MAX_INFLIGHT) {
        if (value < 0 || value > e->n_slots)
            return fail(ZI_ERR_INVALID_ARG, "slot uses in flight must be in 0..n_slots (0 = the default pacing)");
        e->max_inflight = (int)value;
        return ZI_OK;
    }
    if (option == ZI_OPT_HOST_COPY_THREADS) {
        if (value < 1 || value > 64) return fail(ZI_ERR_INVALID_ARG, "host copy threads must be in 1..64");
        e->copy_threads = (int)value;
        if (e->pool_in) {
            delete e->pool_in;
            delete e->pool_out;
            e->pool_in = make_pool(e->copy_threads);
            e->pool_out = make_pool(e->copy_threads);
            if (!e->pool_in || !e->pool_out) {
                ring_release(e);          // the engine is left without a ring rather than with half of one
                return fail(ZI_ERR_NOMEM, "could not start the copy threads; the pinned ring was released");
            }
        }
        return ZI_OK;
    }
    if (option == ZI_OPT_HOST_RING_SLOTS) {
        if (value != 0 && (value < 2 || value > kMaxHostSlots))
            return fail(ZI_ERR_INVALID_ARG, "host ring slots must be 0 or in 2..%d", kMaxHostSlots);
        ZI_HIP(hipSetDevice(e->device));
        ring_release(e);
        if (value == 0) return ZI_OK;
        hipError_t he = hipHostMalloc((void**)&e->hring, (size_t)value * kSlotArrays * e->array_bytes, hipHostMallocDefault);
        if (he != hipSuccess) {
            e->hring = nullptr;
            (void)hipGetLastError();
            return fail(he == hipErrorOutOfMemory ? ZI_ERR_NOMEM : ZI_ERR_HIP, "pinned ring of %lld slots: %s",
                        (long long)value, hipGetErrorString(he));
        }
        for (int i = 0; i < (int)value; ++i) {
            he = hipEventCreateWithFlags(&e->ev_back[i], hipEventDisableTiming);
            if (he == hipSuccess) he = hipEventCreateWithFlags(&e->ev_fill[i], hipEventDisableTiming);
            if (he != hipSuccess) {
                (void)hipGetLastError();
                ring_release(e);
                return fail(ZI_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(he));
            }
        }
        e->pool_in = make_pool(e->copy_threads);
        e->pool_out = make_pool(e->copy_threads);
        e->stage_in = make_stage();
        e->stage_out = make_stage();
        if (!e->pool_in || !e->pool_out || !e->stage_in || !e->stage_out) {
            ring_release(e);
            return fail(ZI_ERR_NOMEM, "could not start the copy threads");
        }
        e->n_hslots = (int)value;
        return ZI_OK;
    }
    return fail(ZI_ERR_INVALID_ARG, "unknown engine option %d", option);
}

namespace {

// Every array a kernel or a copy engine will touch is looked at before anything is issued: a
// device-resident array over its whole byte range, a host array at its first and last byte.
// Returns the memory kind of the array (0 device, 1 page-locked host, 2 ordinary host).
zi_status classify_array(PointerChecker& reach, const void* p, size_t bytes, int tensor, const char* name, int& kind)
{
    kind = memory_kind(p);
    if (kind == -2) return fail(ZI_ERR_HIP, "no usable HIP device (pointer query failed)");
    if (kind < 0) return fail(ZI_ERR_INVALID_ARG, "tensor %d: %s is neither device nor host memory", tensor, name);
    if (kind == 0) return reach.check(p, bytes, tensor, name);
    const int last = memory_kind(static_cast<const char*>(p) + bytes - 1);
    if (last != kind)
        return fail(ZI_ERR_INVALID_ARG, "tensor %d: %s (%zu bytes) does not lie in one kind of host memory", tensor,
                    name, bytes);
    return ZI_OK;
}

// The chunk pipeline.  `staged` = the state is not page-locked memory and travels through the
// engine's pinned ring (CPU threads fill and empty the ring slots).
struct StreamedRun {
    zi_engine* e;
    const std::vector<StateSrc>& src;
    const std::vector<Segment>& segs;
    const std::vector<size_t>& use_begin;
    int64_t n_uses;
    int n_h;

    // Progress shared by the three actors of the ring path (gather thread, the caller's thread,
    // scatter thread), under one mutex.
    std::mutex mu;
    std::condition_variable cv;
    int64_t gathered = 0, issued = 0, scattered = 0;
    bool abort = false;
    bool io_error = false;
    char err_text[160] = "";

    StreamedRun(zi_engine* e_, int64_t n_uses_)
        : e(e_), src(e_->src), segs(e_->segs), use_begin(e_->use_begin), n_uses(n_uses_), n_h(e_->n_hslots)
    {
    }

    // Where a segment sits inside a slot (HBM slot and pinned-ring slot share one layout).
    int64_t slot_off(const Segment& sg) const
    {
        // Lead-in elements that give the staged arrays the alignment phase of the device-resident
        // 2-byte array the kernel will see beside them (gradients, else the low-precision copy).
        const StateSrc& S = src[(size_t)sg.tensor];
        const uint16_t* ref = nullptr;
        if (!S.g_host) ref = (const uint16_t*)S.g + sg.elem_offset;
        else if (S.p_lp && !S.lp_host) ref = (const uint16_t*)S.p_lp + sg.elem_offset;
        return sg.slot_offset + (ref ? (int64_t)((reinterpret_cast<uintptr_t>(ref) / 2) % 4) : 0);
    }

    // Transfer lists between the caller's state (ordinary memory or files) and ring slot h for one
    // slot use.  Direct-I/O files move whole 4096-byte blocks: the rounded-up tail of a region is read
    // and written back unchanged (the update only touches `count` elements of the slot).
    void ring_pieces(int64_t use, int h, bool inbound, std::vector<Piece>& out) const
    {
        out.clear();
        auto mem_pieces = [&](char* ring, char* user_mem, size_t bytes) {
            for (size_t o = 0; o < bytes; o += kCopyPieceBytes) {
                const size_t nb = bytes - o < kCopyPieceBytes ? bytes - o : kCopyPieceBytes;
                if (inbound) out.push_back({0, ring + o, user_mem + o, -1, 0, nb, nb, false});
                else         out.push_back({0, user_mem + o, ring + o, -1, 0, nb, nb, false});
            }
        };
        for (size_t j = use_begin[(size_t)use]; j < use_begin[(size_t)use + 1]; ++j) {
            const Segment& sg = segs[j];
            const StateSrc& S = src[(size_t)sg.tensor];
            const int64_t so = slot_off(sg);
            if (inbound && S.g_host)
                mem_pieces((char*)(e->hslot_g(h) + so), (char*)S.g + sg.elem_offset * 2, (size_t)sg.count * 2);
            if (!inbound && S.lp_host && S.p_lp)
                mem_pieces((char*)(e->hslot_lp(h) + so), (char*)S.p_lp + sg.elem_offset * 2, (size_t)sg.count * 2);
            for (int w = 0; w < 3; ++w) {
                char* rp = (char*)(e->hslot_array(h, w) + so);
                const size_t need = (size_t)sg.count * 4;
                if (S.kind == kSrcFile) {
                    const size_t total = S.direct[w] ? (need + 4095) / 4096 * 4096 : need;
                    const int64_t fo = S.off[w] + sg.elem_offset * 4;
                    for (size_t o = 0; o < total; o += kCopyPieceBytes) {
                        const size_t nb = total - o < kCopyPieceBytes ? total - o : kCopyPieceBytes;
                        const size_t nd = o >= need ? 0 : (need - o < nb ? need - o : nb);
                        out.push_back({inbound ? 1 : 2, rp + o, nullptr, S.fd[w], fo + (int64_t)o, nb, nd, S.direct[w]});
                    }
                } else {
                    mem_pieces(rp, S.ptr[w] + sg.elem_offset * 4, need);
                }
            }
        }
    }

    void fail_stage(const char* what, const char* detail, bool io)
    {
        std::lock_guard<std::mutex> lk(mu);
        if (!abort) snprintf(err_text, sizeof err_text, "%s: %s", what, detail);
        abort = true;
        io_error = io_error || io;
    }

    // Stage thread: fills ring slot u mod n_h with the state of slot use u, as soon as the slot's
    // previous contents have been written back.
    static void gather_main(void* ctx)
    {
        StreamedRun& r = *static_cast<StreamedRun*>(ctx);
        try {
            for (int64_t u = 0; u < r.n_uses; ++u) {
                {
                    std::unique_lock<std::mutex> lk(r.mu);
                    r.cv.wait(lk, [&] { return r.abort || r.scattered >= u - r.n_h + 1; });
                    if (r.abort) return;
                }
                r.ring_pieces(u, (int)(u % r.n_h), true, r.e->pieces_in);
                const int err = run_pieces(*r.e->pool_in, r.e->pieces_in);
                if (err) {
                    r.fail_stage("reading state", strerror(err), true);
                    r.cv.notify_all();
                    return;
                }
                {
                    std::lock_guard<std::mutex> lk(r.mu);
                    r.gathered = u + 1;
                }
                r.cv.notify_all();
            }
        } catch (const std::exception& ex) {
            r.fail_stage("reading state", ex.what(), false);
            r.cv.notify_all();
        }
    }

    // Stage thread: once the device-to-host copies of slot use u have landed in its ring slot, writes
    // the slot back to the caller's state.
    static void scatter_main(void* ctx)
    {
        StreamedRun& r = *static_cast<StreamedRun*>(ctx);
        try {
            (void)hipSetDevice(r.e->device);
            for (int64_t u = 0; u < r.n_uses; ++u) {
                {
                    std::unique_lock<std::mutex> lk(r.mu);
                    r.cv.wait(lk, [&] { return r.abort || r.issued > u; });
                    if (r.abort) return;
                }
                const int h = (int)(u % r.n_h);
                const hipError_t he = hipEventSynchronize(r.e->ev_back[h]);
                if (he != hipSuccess) {
                    (void)hipGetLastError();
                    r.fail_stage("hipEventSynchronize", hipGetErrorString(he), false);
                    r.cv.notify_all();
                    return;
                }
                r.ring_pieces(u, h, false, r.e->pieces_out);
                const int err = run_pieces(*r.e->pool_out, r.e->pieces_out);
                if (err) {
                    r.fail_stage("writing state", strerror(err), true);
                    r.cv.notify_all();
                    return;
                }
                {
                    std::lock_guard<std::mutex> lk(r.mu);
                    r.scattered = u + 1;
                }
                r.cv.notify_all();
            }
        } catch (const std::exception& ex) {
            r.fail_stage("writing state", ex.what(), false);
            r.cv.notify_all();
        }
    }
};

zi_status run_streamed(zi_engine* e, bool staged, zi_lp_dtype dt, const zi_adamw_config* cfg,
                       const zi_norm_result* d_norm, hipStream_t user)
{
    const std::vector<StateSrc>& src = e->src;
    const int32_t n_tensors = (int32_t)src.size();
    e->plan_numel.resize((size_t)n_tensors);
    for (int32_t i = 0; i < n_tensors; ++i) e->plan_numel[(size_t)i] = src[(size_t)i].numel;
    int64_t n_uses = 0;
    plan_chunks(e->plan_numel.data(), n_tensors, e->chunk_elems, e->segs, n_uses);
    index_uses(e->segs, n_uses, e->use_begin);
    const std::vector<Segment>& segs = e->segs;
    const std::vector<size_t>& use_begin = e->use_begin;

    // Overflow flag first: a skipped step moves nothing (4 bytes decide about gigabytes of traffic).
    if (d_norm) {
        ZI_HIP(hipMemcpyAsync(e->h_norm, d_norm, sizeof(zi_norm_result), hipMemcpyDeviceToHost, user));
        ZI_HIP(hipStreamSynchronize(user));
        if (e->h_norm->found_inf) return ZI_SKIPPED_OVERFLOW;
    }

    // Everything already enqueued on the caller's stream (gradients, norm) happens before our work,
    // and so do gradient offloads still on their way to host memory.
    ZI_HIP(hipEventRecord(e->ev_in, user));
    ZI_HIP(hipStreamWaitEvent(e->s_h2d, e->ev_in, 0));
    ZI_HIP(hipStreamWaitEvent(e->s_k, e->ev_in, 0));
    ZI_HIP(order_after_offloads(e, e->s_h2d));
    if (staged && e->offload_pending) ZI_HIP(hipEventSynchronize(e->ev_offload_done));   // CPU threads read host memory

    const zi::StepConsts k = make_consts(*cfg);
    const bool l2 = cfg->mode == ZI_MODE_ADAM_L2;
    const int n_h = e->n_hslots;

    StreamedRun run(e, n_uses);
    uint64_t staged_bytes = 0;
    if (staged) {
        e->stage_in->start(&StreamedRun::gather_main, &run);
        e->stage_out->start(&StreamedRun::scatter_main, &run);
    }

    const auto t0 = std::chrono::steady_clock::now();

    auto pipeline = [&]() -> zi_status {
        for (int64_t use = 0; use < n_uses; ++use) {
            const int slot = (int)(use % e->n_slots);
            const int h = staged ? (int)(use % n_h) : 0;
            if (staged) {
                std::unique_lock<std::mutex> lk(run.mu);
                run.cv.wait(lk, [&] { return run.abort || run.gathered > use; });
                if (run.abort) return fail(run.io_error ? ZI_ERR_IO : ZI_ERR_HIP, "%s", run.err_text);
            }
            // Pacing.  A slot is refilled only after the device-to-host copies of its previous use have
            // finished; beyond that the host decides how far the copy-in stream may run ahead.
            // Default (n_slots >= 3): use u is issued when the copy-out of use u - 2 STARTS, i.e. when
            // that use's update is done.  The copy-out stream works in order, so this implies that the
            // slot's previous occupant (n_slots >= 3 uses back) has left.  Both directions then run
            // side by side, one chunk apart, and the update of the chunk in between runs while both
            // links are busy: its time is hidden (measured: 265 ms for 12.9 GB each way with and
            // without the kernel).  Pacing by the END of the use two back (ZI_OPT_MAX_INFLIGHT = 2)
            // keeps the directions in lockstep too but exposes the update once per chunk (266-271 ms);
            // letting the copy-in stream run further ahead makes the directions take turns (3 uses:
            // 441 ms; a whole slot ring: up to 2.2x slower).
            if (e->max_inflight == 0 && e->n_slots >= 3) {
                if (use >= 2) ZI_HIP(hipEventSynchronize(e->ev_out_start[(int)((use - 2) % e->n_slots)]));
            } else {
                const int want = e->max_inflight == 0 ? 2 : e->max_inflight;
                const int depth = want < e->n_slots ? want : e->n_slots;
                if (use >= depth) ZI_HIP(hipEventSynchronize(e->ev_d2h[(int)((use - depth) % e->n_slots)]));
            }

            struct Placed { float *dp, *dm, *dv; char *hp, *hm, *hv; size_t bytes;
                            const uint16_t* g; uint16_t* lp; char* lp_host; size_t lp_bytes; };
            Placed placed[zi::kMaxStepDesc];
            StepIssuer issue(k, d_norm, (int)dt, l2, e->s_k);
            int np = 0;
            for (size_t j = use_begin[(size_t)use]; j < use_begin[(size_t)use + 1]; ++j, ++np) {
                const Segment& sg = segs[j];
                const StateSrc& T = src[(size_t)sg.tensor];
                const int64_t so = run.slot_off(sg);
                Placed& P = placed[np];
                P.dp = e->slot_array(slot, 0) + so;
                P.dm = e->slot_array(slot, 1) + so;
                P.dv = e->slot_array(slot, 2) + so;
                if (staged) {          // the link sees the pinned ring, not the caller's memory
                    P.hp = (char*)(e->hslot_array(h, 0) + so);
                    P.hm = (char*)(e->hslot_array(h, 1) + so);
                    P.hv = (char*)(e->hslot_array(h, 2) + so);
                } else {
                    P.hp = T.ptr[0] + sg.elem_offset * 4;
                    P.hm = T.ptr[1] + sg.elem_offset * 4;
                    P.hv = T.ptr[2] + sg.elem_offset * 4;
                }
                P.bytes = (size_t)sg.count * 4;
                // 2-byte arrays: used in place when device-resident, staged in the slot otherwise
                P.g = (const uint16_t*)T.g + sg.elem_offset;
                if (T.g_host) {
                    const char* hg = staged ? (const char*)(e->hslot_g(h) + so) : (const char*)T.g + sg.elem_offset * 2;
                    ZI_HIP(hipMemcpyAsync(e->slot_g(slot) + so, hg, (size_t)sg.count * 2, hipMemcpyHostToDevice,
                                          e->s_h2d));
                    P.g = e->slot_g(slot) + so;
                    e->stats.bytes_h2d += (size_t)sg.count * 2;
                    e->stats.n_copies += 1;
                    if (staged) staged_bytes += (size_t)sg.count * 2;
                }
                P.lp = T.p_lp ? (uint16_t*)T.p_lp + sg.elem_offset : nullptr;
                P.lp_host = nullptr;
                P.lp_bytes = 0;
                if (T.p_lp && T.lp_host) {
                    P.lp = e->slot_lp(slot) + so;
                    P.lp_host = staged ? (char*)(e->hslot_lp(h) + so) : (char*)T.p_lp + sg.elem_offset * 2;
                    P.lp_bytes = (size_t)sg.count * 2;
                }
                ZI_HIP(hipMemcpyAsync(P.dp, P.hp, P.bytes, hipMemcpyHostToDevice, e->s_h2d));
                ZI_HIP(hipMemcpyAsync(P.dm, P.hm, P.bytes, hipMemcpyHostToDevice, e->s_h2d));
                ZI_HIP(hipMemcpyAsync(P.dv, P.hv, P.bytes, hipMemcpyHostToDevice, e->s_h2d));
                e->stats.bytes_h2d += 3 * P.bytes;
                e->stats.n_copies += 3;
                if (staged) staged_bytes += 6 * P.bytes;
            }
            ZI_HIP(hipEventRecord(e->ev_h2d[slot], e->s_h2d));

            ZI_HIP(hipStreamWaitEvent(e->s_k, e->ev_h2d[slot], 0));
            if (!e->skip_kernel) {
                np = 0;
                for (size_t j = use_begin[(size_t)use]; j < use_begin[(size_t)use + 1]; ++j, ++np) {
                    const Segment& sg = segs[j];
                    ZI_HIP(issue.add(placed[np].dp, placed[np].dm, placed[np].dv, placed[np].g, placed[np].lp,
                                     sg.count));
                }
                ZI_HIP(issue.flush());
                e->stats.n_kernels += issue.launches;
            }
            ZI_HIP(hipEventRecord(e->ev_k[slot], e->s_k));

            ZI_HIP(hipStreamWaitEvent(e->s_d2h, e->ev_k[slot], 0));
            ZI_HIP(hipEventRecord(e->ev_out_start[slot], e->s_d2h));
            for (int q = 0; q < np; ++q) {
                const Placed& P = placed[q];
                ZI_HIP(hipMemcpyAsync(P.hp, P.dp, P.bytes, hipMemcpyDeviceToHost, e->s_d2h));
                ZI_HIP(hipMemcpyAsync(P.hm, P.dm, P.bytes, hipMemcpyDeviceToHost, e->s_d2h));
                ZI_HIP(hipMemcpyAsync(P.hv, P.dv, P.bytes, hipMemcpyDeviceToHost, e->s_d2h));
                e->stats.bytes_d2h += 3 * P.bytes;
                e->stats.n_copies += 3;
                if (P.lp_host) {
                    ZI_HIP(hipMemcpyAsync(P.lp_host, P.lp, P.lp_bytes, hipMemcpyDeviceToHost, e->s_d2h));
                    e->stats.bytes_d2h += P.lp_bytes;
                    e->stats.n_copies += 1;
                    if (staged) staged_bytes += P.lp_bytes;
                }
            }
            ZI_HIP(hipEventRecord(e->ev_d2h[slot], e->s_d2h));
            if (staged) {
                ZI_HIP(hipEventRecord(e->ev_back[h], e->s_d2h));
                {
                    std::lock_guard<std::mutex> lk(run.mu);
                    run.issued = use + 1;
                }
                run.cv.notify_all();
            }
            ++e->stats.n_slot_uses;
        }
        // Host arrays are valid on return; later work on the caller's stream sees the finished p_lp.
        ZI_HIP(hipStreamSynchronize(e->s_d2h));
        ZI_HIP(hipEventRecord(e->ev_out, e->s_k));
        ZI_HIP(hipStreamWaitEvent(user, e->ev_out, 0));
        ZI_HIP(hipStreamSynchronize(e->s_k));
        return ZI_OK;
    };

    zi_status st = pipeline();
    if (st != ZI_OK) drain_streams(e);     // nothing of ours still touches the caller's memory on return
    if (staged) {
        if (st != ZI_OK) {
            std::lock_guard<std::mutex> lk(run.mu);
            run.abort = true;
        }
        run.cv.notify_all();
        e->stage_in->wait();
        e->stage_out->wait();
        if (st == ZI_OK && run.abort) st = fail(run.io_error ? ZI_ERR_IO : ZI_ERR_HIP, "%s", run.err_text);
    }
    if (st == ZI_OK) e->offload_pending = false;      // every stream that carried an offload has been drained
    e->stats.bytes_staged_host = staged_bytes;
    e->stats.seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    return st;
}

}  // namespace

extern "C" zi_status zi_adamw_step_streamed(zi_engine* e, const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt,
                                            const zi_adamw_config* cfg, const zi_norm_result* d_norm,
                                            void* hip_stream)
{
    ZI_GUARD_BEGIN
    if (zi_status st = check_engine(e)) return st;
    if (zi_status st = check_dtype((int)dt)) return st;
    if (zi_status st = check_config(cfg)) return st;
    if (zi_status st = check_step_tensors(t, n_tensors)) return st;
    if (d_norm && !aligned(d_norm, 8)) return fail(ZI_ERR_ALIGNMENT, "d_norm must be 8-byte aligned");
    if (zi_status st = check_kernel_visible(d_norm, sizeof(zi_norm_result), -1, "d_norm")) return st;

    ZI_HIP(hipSetDevice(e->device));
    hipStream_t user = (hipStream_t)hip_stream;
    e->stats = zi_stream_stats{};

    // State that is not page-locked cannot feed the copy engines directly (a pageable source turns
    // every copy into a staged, synchronous one).  It goes through the engine's pinned ring if one
    // has been set up, otherwise it is refused.  Gradients and the low-precision copy may live on
    // the device (used in place) or in host memory (staged with the state, chunk by chunk).
    bool pageable = false;
    PointerChecker reach;
    e->src.resize((size_t)n_tensors);
    for (int32_t i = 0; i < n_tensors; ++i) {
        StateSrc& S = e->src[(size_t)i];
        S.kind = kSrcPinned;
        S.ptr[0] = (char*)t[i].p; S.ptr[1] = (char*)t[i].m; S.ptr[2] = (char*)t[i].v;
        S.fd[0] = S.fd[1] = S.fd[2] = -1;
        S.off[0] = S.off[1] = S.off[2] = 0;
        S.direct[0] = S.direct[1] = S.direct[2] = false;
        S.g = t[i].g; S.p_lp = t[i].p_lp; S.numel = t[i].numel;
        S.g_host = S.lp_host = false;
        if (t[i].numel == 0) continue;
        const size_t n = (size_t)t[i].numel;
        static const char* const names[3] = {"p", "m", "v"};
        for (int w = 0; w < 3; ++w) {
            int kind = 0;
            if (zi_status st = classify_array(reach, S.ptr[w], n * 4, i, names[w], kind)) return st;
            if (kind == 0) return fail(ZI_ERR_INVALID_ARG, "tensor %d: p, m, v must be host memory", i);
            if (kind == 2) pageable = true;
        }
        int gk = 0, lk = 0;
        if (zi_status st = classify_array(reach, S.g, n * 2, i, "g", gk)) return st;
        S.g_host = gk != 0;
        if (gk == 2) pageable = true;
        if (S.p_lp) {
            if (zi_status st = classify_array(reach, S.p_lp, n * 2, i, "p_lp", lk)) return st;
            S.lp_host = lk != 0;
            if (lk == 2) pageable = true;
        }
    }
    if (pageable) {
        if (e->n_hslots == 0)
            return fail(ZI_ERR_INVALID_ARG, "host arrays must be pinned host memory (or give the engine a pinned "
                                            "ring with ZI_OPT_HOST_RING_SLOTS)");
        for (auto& S : e->src) S.kind = kSrcPageable;   // one path per call: everything host-side rides the ring
    }
    return run_streamed(e, pageable, dt, cfg, d_norm, user);
    ZI_GUARD_END
}

namespace {

// Shared state of zi_grad_norm_streamed's ring path: one stage thread fills ring slots with chunks
// of host-resident gradients, the caller's thread ships them to HBM and reduces them.
struct NormRun {
    zi_engine* e;
    const zi_tensor* t;
    int64_t n_uses;
    int n_h;
    std::mutex mu;
    std::condition_variable cv;
    int64_t gathered = 0, issued = 0;
    bool abort = false;
    char err_text[160] = "";

    void fail_stage(const char* what, const char* detail)
    {
        {
            std::lock_guard<std::mutex> lk(mu);
            if (!abort) snprintf(err_text, sizeof err_text, "%s: %s", what, detail);
            abort = true;
        }
        cv.notify_all();
    }

    static void gather_main(void* ctx)
    {
        NormRun& r = *static_cast<NormRun*>(ctx);
        zi_engine* e = r.e;
        try {
            (void)hipSetDevice(e->device);
            for (int64_t u = 0; u < r.n_uses; ++u) {
                const int h = (int)(u % r.n_h);
                if (u >= r.n_h) {      // the ring slot is free once its previous host-to-device copies are done
                    {
                        std::unique_lock<std::mutex> lk(r.mu);
                        r.cv.wait(lk, [&] { return r.abort || r.issued > u - r.n_h; });
                        if (r.abort) return;
                    }
                    const hipError_t he = hipEventSynchronize(e->ev_back[h]);
                    if (he != hipSuccess) {
                        (void)hipGetLastError();
                        r.fail_stage("hipEventSynchronize", hipGetErrorString(he));
                        return;
                    }
                }
                std::vector<Piece>& pieces = e->pieces_in;
                pieces.clear();
                for (size_t j = e->use_begin[(size_t)u]; j < e->use_begin[(size_t)u + 1]; ++j) {
                    const Segment& sg = e->segs[j];
                    char* ring = (char*)(e->hslot_g(h) + sg.slot_offset);
                    const char* um = (const char*)r.t[e->host_idx[(size_t)sg.tensor]].g + sg.elem_offset * 2;
                    const size_t bytes = (size_t)sg.count * 2;
                    for (size_t o = 0; o < bytes; o += kCopyPieceBytes) {
                        const size_t nb = bytes - o < kCopyPieceBytes ? bytes - o : kCopyPieceBytes;
                        pieces.push_back({0, ring + o, um + o, -1, 0, nb, nb, false});
                    }
                }
                const int err = run_pieces(*e->pool_in, pieces);
                if (err) {
                    r.fail_stage("copying gradients into the pinned ring", strerror(err));
                    return;
                }
                {
                    std::lock_guard<std::mutex> lk(r.mu);
                    r.gathered = u + 1;
                }
                r.cv.notify_all();
            }
        } catch (const std::exception& ex) {
            r.fail_stage("copying gradients into the pinned ring", ex.what());
        }
    }
};

}  // namespace

extern "C" zi_status zi_grad_norm_streamed(zi_engine* e, const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt,
                                           float loss_scale, zi_norm_result* d_out, void* d_workspace,
                                           size_t workspace_bytes, void* hip_stream)
{
    ZI_GUARD_BEGIN
    if (zi_status st = check_engine(e)) return st;
    if (zi_status st = check_norm_args(t, n_tensors, (int)dt, loss_scale, d_out, d_workspace, workspace_bytes)) return st;
    if (zi_status st = check_kernel_visible(d_out, sizeof(zi_norm_result), -1, "d_out")) return st;
    if (zi_status st = check_kernel_visible(d_workspace, workspace_bytes, -1, "d_workspace")) return st;
    ZI_HIP(hipSetDevice(e->device));
    hipStream_t user = (hipStream_t)hip_stream;
    e->stats = zi_stream_stats{};

    // Device-resident gradients are reduced in place; host-resident ones are staged chunk by chunk.
    e->host_idx.clear();
    e->plan_numel.clear();
    bool pageable = false;
    PointerChecker reach;
    for (int32_t i = 0; i < n_tensors; ++i) {
        if (t[i].numel == 0) continue;
        int k = 0;
        if (zi_status st = classify_array(reach, t[i].g, (size_t)t[i].numel * 2, i, "g", k)) return st;
        if (k == 0) continue;
        if (k == 2) pageable = true;
        e->host_idx.push_back(i);
        e->plan_numel.push_back(t[i].numel);
    }
    if (pageable && e->n_hslots == 0)
        return fail(ZI_ERR_INVALID_ARG, "host gradients must be pinned host memory (or give the engine a pinned "
                                        "ring with ZI_OPT_HOST_RING_SLOTS)");
    int64_t n_uses = 0;
    plan_chunks(e->plan_numel.data(), (int32_t)e->plan_numel.size(), e->chunk_elems, e->segs, n_uses);
    index_uses(e->segs, n_uses, e->use_begin);
    const std::vector<Segment>& segs = e->segs;
    const std::vector<size_t>& use_begin = e->use_begin;

    ZI_HIP(hipEventRecord(e->ev_in, user));
    ZI_HIP(hipStreamWaitEvent(e->s_h2d, e->ev_in, 0));
    ZI_HIP(hipStreamWaitEvent(e->s_k, e->ev_in, 0));
    ZI_HIP(order_after_offloads(e, e->s_h2d));
    if (pageable && e->offload_pending) ZI_HIP(hipEventSynchronize(e->ev_offload_done));

    const int n_h = e->n_hslots;
    NormRun run;
    run.e = e;
    run.t = t;
    run.n_uses = n_uses;
    run.n_h = n_h;
    if (pageable) e->stage_in->start(&NormRun::gather_main, &run);

    const auto t0 = std::chrono::steady_clock::now();
    uint64_t staged_bytes = 0;
    auto pipeline = [&]() -> zi_status {
        NormIssuer issue((zi::NormPartial*)d_workspace, (int)dt, loss_scale, d_out, e->s_k);
        for (int32_t i = 0; i < n_tensors; ++i)
            if (t[i].numel > 0 && memory_kind(t[i].g) == 0) ZI_HIP(issue.add((const uint16_t*)t[i].g, t[i].numel));
        for (int64_t use = 0; use < n_uses; ++use) {
            const int slot = (int)(use % e->n_slots);
            const int h = pageable ? (int)(use % n_h) : 0;
            if (pageable) {
                std::unique_lock<std::mutex> lk(run.mu);
                run.cv.wait(lk, [&] { return run.abort || run.gathered > use; });
                if (run.abort) return fail(ZI_ERR_HIP, "%s", run.err_text);
            }
            // the slot's staged gradients are free once the reduction that last read them is done
            if (use >= e->n_slots) ZI_HIP(hipEventSynchronize(e->ev_k[slot]));
            for (size_t j = use_begin[(size_t)use]; j < use_begin[(size_t)use + 1]; ++j) {
                const Segment& sg = segs[j];
                const char* hg = pageable ? (const char*)(e->hslot_g(h) + sg.slot_offset)
                                          : (const char*)t[e->host_idx[(size_t)sg.tensor]].g + sg.elem_offset * 2;
                ZI_HIP(hipMemcpyAsync(e->slot_g(slot) + sg.slot_offset, hg, (size_t)sg.count * 2,
                                      hipMemcpyHostToDevice, e->s_h2d));
                e->stats.bytes_h2d += (size_t)sg.count * 2;
                e->stats.n_copies += 1;
                if (pageable) staged_bytes += (size_t)sg.count * 2;
            }
            ZI_HIP(hipEventRecord(e->ev_h2d[slot], e->s_h2d));
            if (pageable) {
                ZI_HIP(hipEventRecord(e->ev_back[h], e->s_h2d));
                {
                    std::lock_guard<std::mutex> lk(run.mu);
                    run.issued = use + 1;
                }
                run.cv.notify_all();
            }
            ZI_HIP(hipStreamWaitEvent(e->s_k, e->ev_h2d[slot], 0));
            for (size_t j = use_begin[(size_t)use]; j < use_begin[(size_t)use + 1]; ++j)
                ZI_HIP(issue.add(e->slot_g(slot) + segs[j].slot_offset, segs[j].count));
            ZI_HIP(issue.finish());      // the staged chunk is consumed before its slot is reused
            e->stats.n_kernels += 2;
            ZI_HIP(hipEventRecord(e->ev_k[slot], e->s_k));
            ++e->stats.n_slot_uses;
        }
        if (n_uses == 0) ZI_HIP(issue.finish());
        ZI_HIP(hipEventRecord(e->ev_out, e->s_k));
        ZI_HIP(hipStreamWaitEvent(user, e->ev_out, 0));
        ZI_HIP(hipStreamSynchronize(e->s_k));
        return ZI_OK;
    };
    zi_status st = pipeline();
    if (st != ZI_OK) drain_streams(e);
    if (pageable) {
        if (st != ZI_OK) {
            std::lock_guard<std::mutex> lk(run.mu);
            run.abort = true;
        }
        run.cv.notify_all();
        e->stage_in->wait();
        if (st == ZI_OK && run.abort) st = fail(ZI_ERR_HIP, "%s", run.err_text);
    }
    e->stats.bytes_staged_host = staged_bytes;
    e->stats.seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    return st;
    ZI_GUARD_END
}

extern "C" zi_status zi_adamw_step_files(zi_engine* e, const zi_file_tensor* t, int32_t n_tensors, zi_lp_dtype dt,
                                         const zi_adamw_config* cfg, const zi_norm_result* d_norm,
                                         void* hip_stream)
{
    ZI_GUARD_BEGIN
    if (zi_status st = check_engine(e)) return st;
    if (zi_status st = check_dtype((int)dt)) return st;
    if (zi_status st = check_config(cfg)) return st;
    if (n_tensors < 0) return fail(ZI_ERR_INVALID_ARG, "n_tensors < 0");
    if (n_tensors > 0 && !t) return fail(ZI_ERR_INVALID_ARG, "tensor list is NULL");
    if (d_norm && !aligned(d_norm, 8)) return fail(ZI_ERR_ALIGNMENT, "d_norm must be 8-byte aligned");
    if (zi_status st = check_kernel_visible(d_norm, sizeof(zi_norm_result), -1, "d_norm")) return st;
    if (e->n_hslots == 0)
        return fail(ZI_ERR_INVALID_ARG, "file-resident state needs a pinned ring (ZI_OPT_HOST_RING_SLOTS)");

    PointerChecker reach;
    e->src.resize((size_t)n_tensors);
    for (int32_t i = 0; i < n_tensors; ++i) {
        StateSrc& S = e->src[(size_t)i];
        S.kind = kSrcFile;
        S.ptr[0] = S.ptr[1] = S.ptr[2] = nullptr;
        S.fd[0] = t[i].fd_p; S.fd[1] = t[i].fd_m; S.fd[2] = t[i].fd_v;
        S.off[0] = t[i].off_p; S.off[1] = t[i].off_m; S.off[2] = t[i].off_v;
        S.g = t[i].g; S.p_lp = t[i].p_lp; S.numel = t[i].numel;
        S.g_host = S.lp_host = false;
        if (S.numel < 0) return fail(ZI_ERR_INVALID_ARG, "tensor %d: numel < 0", i);
        if (S.numel == 0) continue;
        if (!S.g) return fail(ZI_ERR_INVALID_ARG, "tensor %d: g is NULL", i);
        if (!aligned(S.g, 2) || !aligned(S.p_lp, 2))
            return fail(ZI_ERR_ALIGNMENT, "tensor %d: g and p_lp must be 2-byte aligned", i);
        int gk = 0, lk = 0;
        if (zi_status st = classify_array(reach, S.g, (size_t)S.numel * 2, i, "g", gk)) return st;
        if (S.p_lp)
            if (zi_status st = classify_array(reach, S.p_lp, (size_t)S.numel * 2, i, "p_lp", lk)) return st;
        S.g_host = gk != 0;
        S.lp_host = S.p_lp && lk != 0;
        // the device-resident 2-byte array that sets the alignment phase of the staged arrays, if any
        const void* phase_ref = !S.g_host ? S.g : (S.p_lp && !S.lp_host ? S.p_lp : nullptr);
        for (int w = 0; w < 3; ++w) {
            const int fl = S.fd[w] >= 0 ? fcntl(S.fd[w], F_GETFL) : -1;
            if (fl < 0) return fail(ZI_ERR_INVALID_ARG, "tensor %d: bad file descriptor", i);
            if ((fl & O_ACCMODE) != O_RDWR)
                return fail(ZI_ERR_INVALID_ARG, "tensor %d: descriptors must be open for reading and writing", i);
            if (S.off[w] < 0 || S.off[w] % 4) return fail(ZI_ERR_ALIGNMENT, "tensor %d: offsets must be multiples of 4", i);
            S.direct[w] = (fl & O_DIRECT) != 0;
            if (S.direct[w]) {
                if (S.off[w] % 4096)
                    return fail(ZI_ERR_ALIGNMENT, "tensor %d: with O_DIRECT, offsets must be multiples of 4096", i);
                if (!aligned(phase_ref, 8))
                    return fail(ZI_ERR_ALIGNMENT, "tensor %d: with O_DIRECT, g (p_lp if g is host memory) must be "
                                                  "8-byte aligned", i);
            }
        }
    }
    ZI_HIP(hipSetDevice(e->device));
    e->stats = zi_stream_stats{};
    return run_streamed(e, true, dt, cfg, d_norm, (hipStream_t)hip_stream);
    ZI_GUARD_END
}
