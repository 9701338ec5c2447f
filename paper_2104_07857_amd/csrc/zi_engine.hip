// The streaming engine: staging slots in HBM, three streams, event-ordered slot reuse, the pinned
// ring for state that is not page-locked (ordinary memory or files), and the entry points built on it.
// See include/zi.h for the contract of every call.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdio>
#include <cstring>
#include <new>

#include "zi_host.h"
#include "zi_io_pool.h"

using namespace zi::host;

namespace {

constexpr int kMaxHostSlots = 16;
// A slot holds p, m, v and a fourth array whose first half stages host-resident gradients and whose
// second half stages a host-resident low-precision copy.
constexpr int kSlotArrays = 4;

}  // namespace

struct zi_engine {
    int device = 0;
    size_t chunk_bytes = 0;            // per state array
    int64_t chunk_elems = 0;
    size_t array_bytes = 0;            // chunk_bytes + room for lead-in elements and a rounded-up last block
    uint32_t magic = 0;

    // HBM staging: n_slots slots of kSlotArrays arrays, three streams, events that order slot reuse.
    int n_slots = 0;
    char* staging = nullptr;
    hipStream_t s_h2d = nullptr, s_k = nullptr, s_d2h = nullptr;
    hipEvent_t ev_h2d[8] = {}, ev_k[8] = {}, ev_d2h[8] = {};
    hipEvent_t ev_in = nullptr, ev_out = nullptr;
    zi_norm_result* h_norm = nullptr;  // pinned landing place of the norm result

    // Pinned ring for state that is not page-locked (ordinary memory, files): n_hslots slots shaped
    // like the HBM slots, filled and emptied by two small thread pools.
    int n_hslots = 0;
    char* hring = nullptr;
    hipEvent_t ev_back[kMaxHostSlots] = {};
    int copy_threads = 6;
    CopyPool* pool_in = nullptr;
    CopyPool* pool_out = nullptr;

    // options and figures
    int64_t skip_kernel = 0;
    int max_inflight = 2;              // slot uses the host keeps in flight (<= n_slots)
    zi_stream_stats stats{};

    float* slot_array(int slot, int which) const
    {
        return reinterpret_cast<float*>(staging + ((size_t)slot * kSlotArrays + which) * array_bytes);
    }
    uint16_t* slot_g(int slot) const { return reinterpret_cast<uint16_t*>(slot_array(slot, 3)); }
    uint16_t* slot_lp(int slot) const
    {
        return reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(slot_array(slot, 3)) + array_bytes / 2);
    }
    float* hslot_array(int hslot, int which) const
    {
        return reinterpret_cast<float*>(hring + ((size_t)hslot * kSlotArrays + which) * array_bytes);
    }
    uint16_t* hslot_g(int h) const { return reinterpret_cast<uint16_t*>(hslot_array(h, 3)); }
    uint16_t* hslot_lp(int h) const
    {
        return reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(hslot_array(h, 3)) + array_bytes / 2);
    }
};

namespace {

constexpr uint32_t kEngineMagic = 0x5A49454Eu;

zi_status check_engine(const zi_engine* e)
{
    if (!e) return fail(ZI_ERR_INVALID_ARG, "engine is NULL");
    if (e->magic != kEngineMagic) return fail(ZI_ERR_INVALID_ARG, "engine is not valid (destroyed?)");
    return ZI_OK;
}

// A pool of `n` copy threads, or null if memory or threads cannot be had.
CopyPool* make_pool(int n)
{
    try {
        return new CopyPool(n);
    } catch (const std::exception&) {
        return nullptr;
    }
}

void ring_release(zi_engine* e)
{
    delete e->pool_in;
    delete e->pool_out;
    e->pool_in = e->pool_out = nullptr;
    for (int i = 0; i < kMaxHostSlots; ++i) {
        if (e->ev_back[i]) (void)hipEventDestroy(e->ev_back[i]);
        e->ev_back[i] = nullptr;
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
    }
    if (e->ev_in) (void)hipEventDestroy(e->ev_in);
    if (e->ev_out) (void)hipEventDestroy(e->ev_out);
    if (e->s_h2d) (void)hipStreamDestroy(e->s_h2d);
    if (e->s_k) (void)hipStreamDestroy(e->s_k);
    if (e->s_d2h) (void)hipStreamDestroy(e->s_d2h);
    if (e->staging) (void)hipFree(e->staging);
    if (e->h_norm) (void)hipHostFree(e->h_norm);
    ring_release(e);
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
    for (int i = 0; i < n_slots; ++i) {
        ZI_HIP_E(hipEventCreateWithFlags(&e->ev_h2d[i], hipEventDisableTiming));
        ZI_HIP_E(hipEventCreateWithFlags(&e->ev_k[i], hipEventDisableTiming));
        ZI_HIP_E(hipEventCreateWithFlags(&e->ev_d2h[i], hipEventDisableTiming));
    }
    ZI_HIP_E(hipEventCreateWithFlags(&e->ev_in, hipEventDisableTiming));
    ZI_HIP_E(hipEventCreateWithFlags(&e->ev_out, hipEventDisableTiming));
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
        if (value < 1 || value > e->n_slots)
            return fail(ZI_ERR_INVALID_ARG, "slot uses in flight must be in 1..n_slots");
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
            if (he != hipSuccess) {
                (void)hipGetLastError();
                ring_release(e);
                return fail(ZI_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(he));
            }
        }
        e->pool_in = make_pool(e->copy_threads);
        e->pool_out = make_pool(e->copy_threads);
        if (!e->pool_in || !e->pool_out) {
            ring_release(e);
            return fail(ZI_ERR_NOMEM, "could not start the copy threads");
        }
        e->n_hslots = (int)value;
        return ZI_OK;
    }
    return fail(ZI_ERR_INVALID_ARG, "unknown engine option %d", option);
}

namespace {

enum { kSrcPinned = 0, kSrcPageable = 1, kSrcFile = 2 };

// Where the fp32 state of one tensor lives for the streamed step.
struct StateSrc {
    int kind;
    char* ptr[3];        // p, m, v (memory kinds)
    int fd[3];           // file kind
    int64_t off[3];
    bool direct[3];      // descriptor was opened with O_DIRECT
    const void* g;       // device, or host when g_host
    void* p_lp;          // device, or host when lp_host; may be null
    bool g_host;         // gradients live in host memory and are staged chunk by chunk
    bool lp_host;        // the low-precision copy is written back to host memory
    int64_t numel;
};

// After a failed call: wait for whatever the engine's streams still hold, keeping the first error.
void drain_streams(zi_engine* e)
{
    (void)hipStreamSynchronize(e->s_h2d);
    (void)hipStreamSynchronize(e->s_k);
    (void)hipStreamSynchronize(e->s_d2h);
    (void)hipGetLastError();
}

// The chunk pipeline.  `staged` = the state is not page-locked memory and travels through the
// engine's pinned ring (CPU threads fill and empty the ring slots).
zi_status run_streamed(zi_engine* e, const std::vector<StateSrc>& src, bool staged, zi_lp_dtype dt,
                       const zi_adamw_config* cfg, const zi_norm_result* d_norm, hipStream_t user)
{
    const int32_t n_tensors = (int32_t)src.size();
    std::vector<int64_t> numel((size_t)n_tensors);
    for (int32_t i = 0; i < n_tensors; ++i) numel[(size_t)i] = src[(size_t)i].numel;
    std::vector<Segment> segs;
    int64_t n_uses = 0;
    try {
        plan_chunks(numel.data(), n_tensors, e->chunk_elems, segs, n_uses);
    } catch (const std::bad_alloc&) {
        return fail(ZI_ERR_NOMEM, "out of host memory while planning");
    }

    // Overflow flag first: a skipped step moves nothing (4 bytes decide about gigabytes of traffic).
    if (d_norm) {
        ZI_HIP(hipMemcpyAsync(e->h_norm, d_norm, sizeof(zi_norm_result), hipMemcpyDeviceToHost, user));
        ZI_HIP(hipStreamSynchronize(user));
        if (e->h_norm->found_inf) return ZI_SKIPPED_OVERFLOW;
    }

    // Everything already enqueued on the caller's stream (gradients, norm) happens before our work.
    ZI_HIP(hipEventRecord(e->ev_in, user));
    ZI_HIP(hipStreamWaitEvent(e->s_h2d, e->ev_in, 0));
    ZI_HIP(hipStreamWaitEvent(e->s_k, e->ev_in, 0));

    const zi::StepConsts k = make_consts(*cfg);
    const bool l2 = cfg->mode == ZI_MODE_ADAM_L2;
    const int n_h = e->n_hslots;

    // First segment of every slot use.
    std::vector<size_t> use_begin((size_t)n_uses + 1, segs.size());
    for (size_t j = segs.size(); j-- > 0;) use_begin[(size_t)segs[j].slot_use] = j;
    for (int64_t u = n_uses - 1; u >= 0; --u)
        if (use_begin[(size_t)u] > use_begin[(size_t)u + 1]) use_begin[(size_t)u] = use_begin[(size_t)u + 1];

    // Where a segment sits inside a slot (HBM slot and pinned-ring slot share one layout).
    auto slot_off = [&](const Segment& sg) -> int64_t {
        // Lead-in elements that give the staged arrays the alignment phase of the device-resident
        // 2-byte array the kernel will see beside them (gradients, else the low-precision copy).
        const StateSrc& S = src[(size_t)sg.tensor];
        const uint16_t* ref = nullptr;
        if (!S.g_host) ref = (const uint16_t*)S.g + sg.elem_offset;
        else if (S.p_lp && !S.lp_host) ref = (const uint16_t*)S.p_lp + sg.elem_offset;
        return sg.slot_offset + (ref ? (int64_t)((reinterpret_cast<uintptr_t>(ref) / 2) % 4) : 0);
    };
    // Transfer lists between the caller's state (ordinary memory or files) and ring slot h for one
    // slot use.  Direct-I/O files move whole 4096-byte blocks: the rounded-up tail of a region is read
    // and written back unchanged (the update only touches `count` elements of the slot).
    auto ring_pieces = [&](int64_t use, int h, bool inbound, std::vector<CopyPool::Piece>& out) {
        out.clear();
        for (size_t j = use_begin[(size_t)use]; j < use_begin[(size_t)use + 1]; ++j) {
            const Segment& sg = segs[j];
            const StateSrc& S = src[(size_t)sg.tensor];
            auto mem_pieces = [&](char* ring, char* user_mem, size_t bytes) {
                for (size_t o = 0; o < bytes; o += kCopyPieceBytes) {
                    const size_t nb = bytes - o < kCopyPieceBytes ? bytes - o : kCopyPieceBytes;
                    if (inbound) out.push_back({0, ring + o, user_mem + o, -1, 0, nb, nb, false});
                    else         out.push_back({0, user_mem + o, ring + o, -1, 0, nb, nb, false});
                }
            };
            if (inbound && S.g_host)
                mem_pieces((char*)(e->hslot_g(h) + slot_off(sg)), (char*)S.g + sg.elem_offset * 2,
                           (size_t)sg.count * 2);
            if (!inbound && S.lp_host && S.p_lp)
                mem_pieces((char*)(e->hslot_lp(h) + slot_off(sg)), (char*)S.p_lp + sg.elem_offset * 2,
                           (size_t)sg.count * 2);
            for (int w = 0; w < 3; ++w) {
                char* rp = (char*)(e->hslot_array(h, w) + slot_off(sg));
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
                    char* up = S.ptr[w] + sg.elem_offset * 4;
                    for (size_t o = 0; o < need; o += kCopyPieceBytes) {
                        const size_t nb = need - o < kCopyPieceBytes ? need - o : kCopyPieceBytes;
                        if (inbound) out.push_back({0, rp + o, up + o, -1, 0, nb, nb, false});
                        else         out.push_back({0, up + o, rp + o, -1, 0, nb, nb, false});
                    }
                }
            }
        }
    };

    // Progress shared by the three actors of the ring path (gather thread, this thread, scatter thread).
    struct {
        std::mutex mu;
        std::condition_variable cv;
        int64_t gathered = 0, issued = 0, scattered = 0;
        bool abort = false;
        bool io_error = false;
        char scatter_err[160] = "";
    } sync;
    uint64_t staged_bytes = 0;
    std::thread gather_thread, scatter_thread;
    auto stop_threads = [&] {
        {
            std::lock_guard<std::mutex> lk(sync.mu);
            sync.abort = true;
        }
        sync.cv.notify_all();
        if (gather_thread.joinable()) gather_thread.join();
        if (scatter_thread.joinable()) scatter_thread.join();
    };
    if (staged) try {
        gather_thread = std::thread([&] {
            std::vector<CopyPool::Piece> pieces;
            for (int64_t u = 0; u < n_uses; ++u) {
                {
                    std::unique_lock<std::mutex> lk(sync.mu);
                    sync.cv.wait(lk, [&] { return sync.abort || sync.scattered >= u - n_h + 1; });
                    if (sync.abort) return;
                }
                ring_pieces(u, (int)(u % n_h), true, pieces);
                const int err = e->pool_in->run(pieces);
                {
                    std::lock_guard<std::mutex> lk(sync.mu);
                    if (err) {
                        snprintf(sync.scatter_err, sizeof sync.scatter_err, "reading state: %s", strerror(err));
                        sync.abort = sync.io_error = true;
                    } else {
                        sync.gathered = u + 1;
                    }
                }
                sync.cv.notify_all();
                if (err) return;
            }
        });
        scatter_thread = std::thread([&] {
            (void)hipSetDevice(e->device);
            std::vector<CopyPool::Piece> pieces;
            for (int64_t u = 0; u < n_uses; ++u) {
                {
                    std::unique_lock<std::mutex> lk(sync.mu);
                    sync.cv.wait(lk, [&] { return sync.abort || sync.issued > u; });
                    if (sync.abort) return;
                }
                const int h = (int)(u % n_h);
                hipError_t he = hipEventSynchronize(e->ev_back[h]);
                if (he != hipSuccess) {
                    (void)hipGetLastError();
                    std::lock_guard<std::mutex> lk(sync.mu);
                    snprintf(sync.scatter_err, sizeof sync.scatter_err, "hipEventSynchronize: %s",
                             hipGetErrorString(he));
                    sync.abort = true;
                    sync.cv.notify_all();
                    return;
                }
                ring_pieces(u, h, false, pieces);
                const int err = e->pool_out->run(pieces);
                {
                    std::lock_guard<std::mutex> lk(sync.mu);
                    if (err) {
                        snprintf(sync.scatter_err, sizeof sync.scatter_err, "writing state: %s", strerror(err));
                        sync.abort = sync.io_error = true;
                    } else {
                        sync.scattered = u + 1;
                    }
                }
                sync.cv.notify_all();
                if (err) return;
            }
        });
    } catch (const std::exception& ex) {
        stop_threads();
        return fail(ZI_ERR_NOMEM, "could not start the ring's copy threads: %s", ex.what());
    }

    const auto t0 = std::chrono::steady_clock::now();

    auto pipeline = [&]() -> zi_status {
        for (int64_t use = 0; use < n_uses; ++use) {
            const int slot = (int)(use % e->n_slots);
            const int h = staged ? (int)(use % n_h) : 0;
            if (staged) {
                std::unique_lock<std::mutex> lk(sync.mu);
                sync.cv.wait(lk, [&] { return sync.abort || sync.gathered > use; });
                if (sync.abort) return fail(sync.io_error ? ZI_ERR_IO : ZI_ERR_HIP, "%s", sync.scatter_err);
            }
            // Slot reuse is ordered by the event of the device-to-host copies that last emptied it.
            // The host waits for the use `depth` positions back before it issues this one.  Depth 2
            // keeps the two directions of the link in lockstep: measured at the link's two-way peak
            // with no jitter, where deeper queues let the copy-in stream run ahead and the directions
            // take turns (3 in flight: 3-25% slower, 6: 2.2x slower).
            const int depth = e->max_inflight < e->n_slots ? e->max_inflight : e->n_slots;
            if (use >= depth) ZI_HIP(hipEventSynchronize(e->ev_d2h[(int)((use - depth) % e->n_slots)]));

            struct Placed { float *dp, *dm, *dv; char *hp, *hm, *hv; size_t bytes;
                            const uint16_t* g; uint16_t* lp; char* lp_host; size_t lp_bytes; };
            Placed placed[zi::kMaxStepDesc];
            StepIssuer issue(k, d_norm, (int)dt, l2, e->s_k);
            int np = 0;
            for (size_t j = use_begin[(size_t)use]; j < use_begin[(size_t)use + 1]; ++j, ++np) {
                const Segment& sg = segs[j];
                const StateSrc& T = src[(size_t)sg.tensor];
                const int64_t so = slot_off(sg);
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
                    std::lock_guard<std::mutex> lk(sync.mu);
                    sync.issued = use + 1;
                }
                sync.cv.notify_all();
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
            std::lock_guard<std::mutex> lk(sync.mu);
            sync.abort = true;
        }
        sync.cv.notify_all();
        gather_thread.join();
        scatter_thread.join();
        if (st == ZI_OK && sync.abort) st = fail(sync.io_error ? ZI_ERR_IO : ZI_ERR_HIP, "%s", sync.scatter_err);
    }
    e->stats.bytes_staged_host = staged_bytes;
    e->stats.seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    return st;
}

}  // namespace

extern "C" zi_status zi_adamw_step_streamed(zi_engine* e, const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt,
                                            const zi_adamw_config* cfg, const zi_norm_result* d_norm,
                                            void* hip_stream)
{
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
    std::vector<StateSrc> src((size_t)n_tensors);
    for (int32_t i = 0; i < n_tensors; ++i) {
        StateSrc& S = src[(size_t)i];
        S.kind = kSrcPinned;
        S.ptr[0] = (char*)t[i].p; S.ptr[1] = (char*)t[i].m; S.ptr[2] = (char*)t[i].v;
        S.fd[0] = S.fd[1] = S.fd[2] = -1;
        S.off[0] = S.off[1] = S.off[2] = 0;
        S.direct[0] = S.direct[1] = S.direct[2] = false;
        S.g = t[i].g; S.p_lp = t[i].p_lp; S.numel = t[i].numel;
        S.g_host = S.lp_host = false;
        if (t[i].numel == 0) continue;
        for (int w = 0; w < 3; ++w) {
            const int kind = memory_kind(S.ptr[w]);
            if (kind != 1 && kind != 2) return fail(ZI_ERR_INVALID_ARG, "tensor %d: p, m, v must be host memory", i);
            if (kind == 2) pageable = true;
        }
        const int gk = memory_kind(S.g);
        if (gk < 0) return fail(ZI_ERR_INVALID_ARG, "tensor %d: g is neither device nor host memory", i);
        S.g_host = gk != 0;
        if (gk == 2) pageable = true;
        if (S.p_lp) {
            const int lk = memory_kind(S.p_lp);
            if (lk < 0) return fail(ZI_ERR_INVALID_ARG, "tensor %d: p_lp is neither device nor host memory", i);
            S.lp_host = lk != 0;
            if (lk == 2) pageable = true;
        }
    }
    if (pageable) {
        if (e->n_hslots == 0)
            return fail(ZI_ERR_INVALID_ARG, "host arrays must be pinned host memory (or give the engine a pinned "
                                            "ring with ZI_OPT_HOST_RING_SLOTS)");
        for (auto& S : src) S.kind = kSrcPageable;   // one path per call: everything host-side rides the ring
    }
    return run_streamed(e, src, pageable, dt, cfg, d_norm, user);
}

extern "C" zi_status zi_grad_norm_streamed(zi_engine* e, const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt,
                                           float loss_scale, zi_norm_result* d_out, void* d_workspace,
                                           size_t workspace_bytes, void* hip_stream)
{
    if (zi_status st = check_engine(e)) return st;
    if (zi_status st = check_norm_args(t, n_tensors, (int)dt, loss_scale, d_out, d_workspace, workspace_bytes)) return st;
    if (zi_status st = check_kernel_visible(d_out, sizeof(zi_norm_result), -1, "d_out")) return st;
    if (zi_status st = check_kernel_visible(d_workspace, workspace_bytes, -1, "d_workspace")) return st;
    ZI_HIP(hipSetDevice(e->device));
    hipStream_t user = (hipStream_t)hip_stream;
    e->stats = zi_stream_stats{};

    // Device-resident gradients are reduced in place; host-resident ones are staged chunk by chunk.
    std::vector<int32_t> host_idx;
    std::vector<int64_t> host_numel;
    bool pageable = false;
    for (int32_t i = 0; i < n_tensors; ++i) {
        if (t[i].numel == 0) continue;
        const int k = memory_kind(t[i].g);
        if (k < 0) return fail(ZI_ERR_INVALID_ARG, "tensor %d: g is neither device nor host memory", i);
        if (k == 0) continue;
        if (k == 2) pageable = true;
        host_idx.push_back(i);
        host_numel.push_back(t[i].numel);
    }
    if (pageable && e->n_hslots == 0)
        return fail(ZI_ERR_INVALID_ARG, "host gradients must be pinned host memory (or give the engine a pinned "
                                        "ring with ZI_OPT_HOST_RING_SLOTS)");
    std::vector<Segment> segs;
    int64_t n_uses = 0;
    try {
        plan_chunks(host_numel.data(), (int32_t)host_numel.size(), e->chunk_elems, segs, n_uses);
    } catch (const std::bad_alloc&) {
        return fail(ZI_ERR_NOMEM, "out of host memory while planning");
    }
    std::vector<size_t> use_begin((size_t)n_uses + 1, segs.size());
    for (size_t j = segs.size(); j-- > 0;) use_begin[(size_t)segs[j].slot_use] = j;
    for (int64_t u = n_uses - 1; u >= 0; --u)
        if (use_begin[(size_t)u] > use_begin[(size_t)u + 1]) use_begin[(size_t)u] = use_begin[(size_t)u + 1];

    ZI_HIP(hipEventRecord(e->ev_in, user));
    ZI_HIP(hipStreamWaitEvent(e->s_h2d, e->ev_in, 0));
    ZI_HIP(hipStreamWaitEvent(e->s_k, e->ev_in, 0));

    const int n_h = e->n_hslots;
    struct {
        std::mutex mu;
        std::condition_variable cv;
        int64_t gathered = 0, issued = 0;
        bool abort = false;
    } sync;
    std::thread gather_thread;
    if (pageable) try {
        gather_thread = std::thread([&] {
            (void)hipSetDevice(e->device);
            std::vector<CopyPool::Piece> pieces;
            for (int64_t u = 0; u < n_uses; ++u) {
                const int h = (int)(u % n_h);
                if (u >= n_h) {      // the ring slot is free once its previous host-to-device copies are done
                    std::unique_lock<std::mutex> lk(sync.mu);
                    sync.cv.wait(lk, [&] { return sync.abort || sync.issued > u - n_h; });
                    if (sync.abort) return;
                    lk.unlock();
                    if (hipEventSynchronize(e->ev_back[h]) != hipSuccess) {
                        (void)hipGetLastError();
                        std::lock_guard<std::mutex> lk2(sync.mu);
                        sync.abort = true;
                        sync.cv.notify_all();
                        return;
                    }
                }
                pieces.clear();
                for (size_t j = use_begin[(size_t)u]; j < use_begin[(size_t)u + 1]; ++j) {
                    const Segment& sg = segs[j];
                    char* ring = (char*)(e->hslot_g(h) + sg.slot_offset);
                    const char* um = (const char*)t[host_idx[(size_t)sg.tensor]].g + sg.elem_offset * 2;
                    const size_t bytes = (size_t)sg.count * 2;
                    for (size_t o = 0; o < bytes; o += kCopyPieceBytes) {
                        const size_t nb = bytes - o < kCopyPieceBytes ? bytes - o : kCopyPieceBytes;
                        pieces.push_back({0, ring + o, um + o, -1, 0, nb, nb, false});
                    }
                }
                e->pool_in->run(pieces);
                {
                    std::lock_guard<std::mutex> lk(sync.mu);
                    sync.gathered = u + 1;
                }
                sync.cv.notify_all();
            }
        });
    } catch (const std::exception& ex) {
        return fail(ZI_ERR_NOMEM, "could not start the ring's copy thread: %s", ex.what());
    }

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
                std::unique_lock<std::mutex> lk(sync.mu);
                sync.cv.wait(lk, [&] { return sync.abort || sync.gathered > use; });
                if (sync.abort) return fail(ZI_ERR_HIP, "waiting for the pinned ring failed");
            }
            // the slot's staged gradients are free once the reduction that last read them is done
            if (use >= e->n_slots) ZI_HIP(hipEventSynchronize(e->ev_k[slot]));
            for (size_t j = use_begin[(size_t)use]; j < use_begin[(size_t)use + 1]; ++j) {
                const Segment& sg = segs[j];
                const char* hg = pageable ? (const char*)(e->hslot_g(h) + sg.slot_offset)
                                          : (const char*)t[host_idx[(size_t)sg.tensor]].g + sg.elem_offset * 2;
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
                    std::lock_guard<std::mutex> lk(sync.mu);
                    sync.issued = use + 1;
                }
                sync.cv.notify_all();
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
            std::lock_guard<std::mutex> lk(sync.mu);
            sync.abort = true;
        }
        sync.cv.notify_all();
        gather_thread.join();
        if (st == ZI_OK && sync.abort) st = fail(ZI_ERR_HIP, "the pinned ring's copy thread failed");
    }
    e->stats.bytes_staged_host = staged_bytes;
    e->stats.seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    return st;
}

extern "C" zi_status zi_adamw_step_files(zi_engine* e, const zi_file_tensor* t, int32_t n_tensors, zi_lp_dtype dt,
                                         const zi_adamw_config* cfg, const zi_norm_result* d_norm,
                                         void* hip_stream)
{
    if (zi_status st = check_engine(e)) return st;
    if (zi_status st = check_dtype((int)dt)) return st;
    if (zi_status st = check_config(cfg)) return st;
    if (n_tensors < 0) return fail(ZI_ERR_INVALID_ARG, "n_tensors < 0");
    if (n_tensors > 0 && !t) return fail(ZI_ERR_INVALID_ARG, "tensor list is NULL");
    if (d_norm && !aligned(d_norm, 8)) return fail(ZI_ERR_ALIGNMENT, "d_norm must be 8-byte aligned");
    if (zi_status st = check_kernel_visible(d_norm, sizeof(zi_norm_result), -1, "d_norm")) return st;
    if (e->n_hslots == 0)
        return fail(ZI_ERR_INVALID_ARG, "file-resident state needs a pinned ring (ZI_OPT_HOST_RING_SLOTS)");

    std::vector<StateSrc> src((size_t)n_tensors);
    for (int32_t i = 0; i < n_tensors; ++i) {
        StateSrc& S = src[(size_t)i];
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
        const int gk = memory_kind(S.g), lk = S.p_lp ? memory_kind(S.p_lp) : 0;
        if (gk < 0 || lk < 0) return fail(ZI_ERR_INVALID_ARG, "tensor %d: g / p_lp is neither device nor host memory", i);
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
    return run_streamed(e, src, true, dt, cfg, d_norm, (hipStream_t)hip_stream);
}

extern "C" zi_status zi_engine_file_probe(zi_engine* e, int32_t fd_read, int32_t fd_write, size_t bytes,
                                          double* seconds_out)
{
    if (zi_status st = check_engine(e)) return st;
    if (!seconds_out) return fail(ZI_ERR_INVALID_ARG, "seconds_out is NULL");
    if (e->n_hslots == 0) return fail(ZI_ERR_INVALID_ARG, "the probe needs a pinned ring (ZI_OPT_HOST_RING_SLOTS)");
    if (fd_read < 0 && fd_write < 0) return fail(ZI_ERR_INVALID_ARG, "no file descriptor given");
    if (bytes == 0 || bytes % 4096) return fail(ZI_ERR_INVALID_ARG, "bytes must be a positive multiple of 4096");
    if (e->n_hslots < 2) return fail(ZI_ERR_INVALID_ARG, "ring too small");
    // Reads land in the first half of the ring, writes leave from the second half.
    const size_t half = (size_t)(e->n_hslots / 2) * kSlotArrays * e->array_bytes / 4096 * 4096;
    auto pieces_for = [&](int fd, int op, char* base, std::vector<CopyPool::Piece>& out) {
        const int fl = fcntl(fd, F_GETFL);
        const bool direct = fl >= 0 && (fl & O_DIRECT);
        size_t ring_o = 0;
        for (size_t o = 0; o < bytes; o += kCopyPieceBytes) {
            const size_t nb = bytes - o < kCopyPieceBytes ? bytes - o : kCopyPieceBytes;
            if (ring_o + nb > half) ring_o = 0;
            out.push_back({op, base + ring_o, nullptr, fd, (int64_t)o, nb, nb, direct});
            ring_o += nb;
        }
    };
    std::vector<CopyPool::Piece> rd, wr;
    if (fd_read >= 0) pieces_for(fd_read, 1, e->hring, rd);
    if (fd_write >= 0) pieces_for(fd_write, 2, e->hring + half, wr);
    int err_r = 0, err_w = 0;
    const auto t0 = std::chrono::steady_clock::now();
    std::thread tw;
    if (!wr.empty()) tw = std::thread([&] { err_w = e->pool_out->run(wr); });
    if (!rd.empty()) err_r = e->pool_in->run(rd);
    if (tw.joinable()) tw.join();
    *seconds_out = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    if (err_r) return fail(ZI_ERR_IO, "reading: %s", strerror(err_r));
    if (err_w) return fail(ZI_ERR_IO, "writing: %s", strerror(err_w));
    return ZI_OK;
}

extern "C" zi_status zi_engine_link_probe(zi_engine* e, const void* host_src, void* host_dst, size_t bytes,
                                          int32_t mode, int32_t repeats, double* seconds_out)
{
    if (zi_status st = check_engine(e)) return st;
    if (mode < 0 || mode > 2) return fail(ZI_ERR_INVALID_ARG, "mode must be 0, 1 or 2");
    if (repeats < 1) return fail(ZI_ERR_INVALID_ARG, "repeats < 1");
    if (!seconds_out) return fail(ZI_ERR_INVALID_ARG, "seconds_out is NULL");
    if ((mode == 0 || mode == 2) && !host_src) return fail(ZI_ERR_INVALID_ARG, "host_src is NULL");
    if ((mode == 1 || mode == 2) && !host_dst) return fail(ZI_ERR_INVALID_ARG, "host_dst is NULL");
    if (bytes == 0) return fail(ZI_ERR_INVALID_ARG, "bytes is 0");
    ZI_HIP(hipSetDevice(e->device));
    ZI_HIP(hipStreamSynchronize(e->s_h2d));
    ZI_HIP(hipStreamSynchronize(e->s_d2h));

    // Host-to-device pieces land in the p arrays of the slots, device-to-host pieces leave from
    // the m arrays, so the two directions never touch the same staging bytes.  In the two-way mode
    // the host keeps the same number of pieces in flight as the streamed step does (a deep queue
    // lets one direction run ahead and measures a lower two-way rate).
    const int depth = e->max_inflight < e->n_slots ? e->max_inflight : e->n_slots;
    const auto t0 = std::chrono::steady_clock::now();
    for (int r = 0; r < repeats; ++r) {
        int64_t piece = 0;
        for (size_t off = 0; off < bytes; off += e->chunk_bytes, ++piece) {
            const size_t nb = bytes - off < e->chunk_bytes ? bytes - off : e->chunk_bytes;
            const int slot = (int)(piece % e->n_slots);
            if (mode == 2 && piece >= depth) {
                const int old_slot = (int)((piece - depth) % e->n_slots);
                ZI_HIP(hipEventSynchronize(e->ev_h2d[old_slot]));
                ZI_HIP(hipEventSynchronize(e->ev_d2h[old_slot]));
            }
            if (mode == 0 || mode == 2)
                ZI_HIP(hipMemcpyAsync(e->slot_array(slot, 0), (const char*)host_src + off, nb,
                                      hipMemcpyHostToDevice, e->s_h2d));
            if (mode == 1 || mode == 2)
                ZI_HIP(hipMemcpyAsync((char*)host_dst + off, e->slot_array(slot, 1), nb, hipMemcpyDeviceToHost,
                                      e->s_d2h));
            if (mode == 2) {
                ZI_HIP(hipEventRecord(e->ev_h2d[slot], e->s_h2d));
                ZI_HIP(hipEventRecord(e->ev_d2h[slot], e->s_d2h));
            }
        }
        if (mode == 2) {     // the next repeat starts with an empty pipeline
            ZI_HIP(hipStreamSynchronize(e->s_h2d));
            ZI_HIP(hipStreamSynchronize(e->s_d2h));
        }
    }
    ZI_HIP(hipStreamSynchronize(e->s_h2d));
    ZI_HIP(hipStreamSynchronize(e->s_d2h));
    *seconds_out = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    return ZI_OK;
}

