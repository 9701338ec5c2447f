// Chunk plan of the streamed step: how a tensor list maps onto slot uses.  Pure host code with no HIP
// types, so it can be compiled and checked by the host compiler alone.
#pragma once

#include <cstdint>
#include <vector>

namespace zi {
namespace host {

constexpr int kPlanMaxSegmentsPerUse = 32;   // = tensors (or segments) one fused-step launch takes
constexpr int64_t kPackAlign = 1024; // packed segments start on 4096-byte boundaries of the slot arrays (direct file I/O)
constexpr int64_t kPhasePad = 8;     // room for lead-in elements that keep alignment phases equal

struct Segment {
    int32_t tensor;
    int64_t elem_offset, count, slot_use, slot_offset;
};

// Pass 1: every whole chunk of every tensor takes a slot use of its own, in list order.
// Pass 2: what is left (tensors shorter than a chunk and the remainders of long ones) is packed
// first-fit, in list order, into shared slot uses of at most kPlanMaxSegmentsPerUse segments each, so a
// list with many tiny tensors between giant ones costs one extra slot use, not one per tensor.
inline void plan_chunks(const int64_t* numel, int32_t n_tensors, int64_t chunk_elems, std::vector<Segment>& out,
                 int64_t& n_uses)
{
    out.clear();
    int64_t use = 0;
    for (int32_t i = 0; i < n_tensors; ++i) {
        const int64_t whole = numel[i] / chunk_elems;
        for (int64_t c = 0; c < whole; ++c) out.push_back({i, c * chunk_elems, chunk_elems, use++, 0});
    }
    int64_t fill = 0;          // next free element of the open packed slot use
    int packed = 0;            // segments in the open packed slot use
    bool open = false;
    for (int32_t i = 0; i < n_tensors; ++i) {
        const int64_t off = numel[i] / chunk_elems * chunk_elems;
        const int64_t left = numel[i] - off;
        if (left == 0) continue;
        if (open && (fill + left + kPhasePad > chunk_elems || packed == kPlanMaxSegmentsPerUse)) {
            ++use;
            open = false;
        }
        if (!open) { open = true; fill = 0; packed = 0; }
        out.push_back({i, off, left, use, fill});
        ++packed;
        fill = (fill + left + kPhasePad + kPackAlign - 1) / kPackAlign * kPackAlign;
    }
    if (open) ++use;
    n_uses = use;
}

}  // namespace host
}  // namespace zi
