// The streaming engine's state, shared by the translation units that implement its entry points.
#pragma once

#include <hip/hip_runtime.h>

#include <vector>

#include "zi_host.h"
#include "zi_io_pool.h"

namespace zi {
namespace host {

constexpr int kMaxHostSlots = 16;
// A slot holds p, m, v and a fourth array whose first half stages host-resident gradients and whose
// second half stages a host-resident low-precision copy.
constexpr int kSlotArrays = 4;
constexpr int kOffloadEvents = 64;       // events that order gradient offloads after their producers
constexpr uint32_t kEngineMagic = 0x5A49454Eu;

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

}  // namespace host
}  // namespace zi

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
    hipEvent_t ev_out_start[8] = {};   // the slot's device-to-host copies are about to start (its update is done)
    hipEvent_t ev_in = nullptr, ev_out = nullptr;
    zi_norm_result* h_norm = nullptr;  // pinned landing place of the norm result

    // Pinned ring for state that is not page-locked (ordinary memory, files): n_hslots slots shaped
    // like the HBM slots, filled and emptied by two small thread pools, each driven by one parked
    // stage thread.  All of these threads are created with the ring and parked between calls.
    int n_hslots = 0;
    char* hring = nullptr;
    hipEvent_t ev_back[zi::host::kMaxHostSlots] = {};   // the slot's outbound traffic has left / its inbound copy is done
    hipEvent_t ev_fill[zi::host::kMaxHostSlots] = {};   // the slot's device-to-host fill has landed
    int copy_threads = 6;
    zi::host::TaskPool* pool_in = nullptr;
    zi::host::TaskPool* pool_out = nullptr;
    zi::host::StageThread* stage_in = nullptr;
    zi::host::StageThread* stage_out = nullptr;
    zi::host::TaskPool* pool_step = nullptr;            // blocks of the host-CPU step (created on first use)

    // Gradient offload: copies in flight on the device-to-host stream, ordered after their producers.
    hipEvent_t ev_offload[zi::host::kOffloadEvents] = {};
    hipEvent_t ev_offload_done = nullptr;               // recorded after the last offload copy issued
    uint64_t n_offloads = 0;
    bool offload_pending = false;

    // Per-call plans.  The vectors keep their capacity between calls, so once a list of a given size
    // has been seen, later calls allocate no host memory either.
    std::vector<zi::host::StateSrc> src;
    std::vector<int64_t> plan_numel;
    std::vector<zi::host::Segment> segs;
    std::vector<size_t> use_begin;
    std::vector<zi::host::Piece> pieces_in, pieces_out;
    std::vector<int32_t> host_idx;

    // options and figures
    int64_t skip_kernel = 0;
    int max_inflight = 0;              // 0: paced by the start of the copy-out two uses back; k: by the end of use - k
    zi_stream_stats stats{};

    float* slot_array(int slot, int which) const
    {
        return reinterpret_cast<float*>(staging + ((size_t)slot * zi::host::kSlotArrays + which) * array_bytes);
    }
    uint16_t* slot_g(int slot) const { return reinterpret_cast<uint16_t*>(slot_array(slot, 3)); }
    uint16_t* slot_lp(int slot) const
    {
        return reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(slot_array(slot, 3)) + array_bytes / 2);
    }
    float* hslot_array(int hslot, int which) const
    {
        return reinterpret_cast<float*>(hring + ((size_t)hslot * zi::host::kSlotArrays + which) * array_bytes);
    }
    uint16_t* hslot_g(int h) const { return reinterpret_cast<uint16_t*>(hslot_array(h, 3)); }
    uint16_t* hslot_lp(int h) const
    {
        return reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(hslot_array(h, 3)) + array_bytes / 2);
    }
};

namespace zi {
namespace host {

inline zi_status check_engine(const zi_engine* e)
{
    if (!e) return fail(ZI_ERR_INVALID_ARG, "engine is NULL");
    if (e->magic != kEngineMagic) return fail(ZI_ERR_INVALID_ARG, "engine is not valid (destroyed?)");
    return ZI_OK;
}

// After a failed call: wait for whatever the engine's streams still hold, dropping the errors.
inline void drain_streams(zi_engine* e)
{
    (void)hipStreamSynchronize(e->s_h2d);
    (void)hipStreamSynchronize(e->s_k);
    (void)hipStreamSynchronize(e->s_d2h);
    (void)hipGetLastError();
}

// First segment of every slot use (segments are sorted by slot use within each planning pass).
inline void index_uses(const std::vector<Segment>& segs, int64_t n_uses, std::vector<size_t>& use_begin)
{
    use_begin.assign((size_t)n_uses + 1, segs.size());
    for (size_t j = segs.size(); j-- > 0;) use_begin[(size_t)segs[j].slot_use] = j;
    for (int64_t u = n_uses - 1; u >= 0; --u)
        if (use_begin[(size_t)u] > use_begin[(size_t)u + 1]) use_begin[(size_t)u] = use_begin[(size_t)u + 1];
}

// Work already enqueued on the device-to-host stream by zi_grad_offload happens before anything a
// streamed call reads from host memory: its copy-in stream waits for the last offload.
inline hipError_t order_after_offloads(zi_engine* e, hipStream_t consumer)
{
    if (!e->offload_pending) return hipSuccess;
    return hipStreamWaitEvent(consumer, e->ev_offload_done, 0);
}

// Maps a C++ exception that reached an entry point to a status (nothing may cross the C ABI).
#define ZI_GUARD_BEGIN try {
#define ZI_GUARD_END                                                                              \
    }                                                                                             \
    catch (const std::bad_alloc&) { return ::zi::host::fail(ZI_ERR_NOMEM, "out of host memory"); } \
    catch (const std::exception& ex_) { return ::zi::host::fail(ZI_ERR_NOMEM, "%s", ex_.what()); }

}  // namespace host
}  // namespace zi
