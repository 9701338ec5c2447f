// Chunk plan of the streamed step: how a tensor list maps onto slot uses (pure host code).
#include <new>

#include "zi_host.h"

using namespace zi::host;

extern "C" zi_status zi_plan_chunks(const int64_t* numel, int32_t n_tensors, int64_t chunk_elems,
                                    zi_chunk_segment* out, int64_t cap, int64_t* n_segments_out,
                                    int64_t* n_slot_uses_out)
{
    if (n_tensors < 0) return fail(ZI_ERR_INVALID_ARG, "n_tensors < 0");
    if (n_tensors > 0 && !numel) return fail(ZI_ERR_INVALID_ARG, "numel is NULL");
    if (chunk_elems < kPackAlign || chunk_elems % kPackAlign)
        return fail(ZI_ERR_INVALID_ARG, "chunk_elems must be a positive multiple of %lld", (long long)kPackAlign);
    if (cap < 0 || (cap > 0 && !out)) return fail(ZI_ERR_INVALID_ARG, "bad output buffer");
    if (!n_segments_out || !n_slot_uses_out) return fail(ZI_ERR_INVALID_ARG, "output counters are NULL");
    for (int32_t i = 0; i < n_tensors; ++i)
        if (numel[i] < 0) return fail(ZI_ERR_INVALID_ARG, "tensor %d: numel < 0", i);
    std::vector<Segment> segs;
    int64_t uses = 0;
    try {
        plan_chunks(numel, n_tensors, chunk_elems, segs, uses);
    } catch (const std::bad_alloc&) {
        return fail(ZI_ERR_NOMEM, "out of host memory while planning");
    }
    for (int64_t i = 0; i < (int64_t)segs.size() && i < cap; ++i) {
        out[i].tensor = segs[i].tensor;
        out[i].reserved = 0;
        out[i].elem_offset = segs[i].elem_offset;
        out[i].count = segs[i].count;
        out[i].slot_use = segs[i].slot_use;
        out[i].slot_offset = segs[i].slot_offset;
    }
    *n_segments_out = (int64_t)segs.size();
    *n_slot_uses_out = uses;
    return ZI_OK;
}

