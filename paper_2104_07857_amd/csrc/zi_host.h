// Host-side helpers shared by the C-ABI translation units: error reporting, argument checks,
// per-step scalars, and the objects that assemble kernel launches over tensor lists.
#pragma once

#include <hip/hip_runtime.h>

#include <cmath>
#include <initializer_list>
#include <cstdint>
#include <vector>

#include "zi_internal.h"
#include "zi_checks.h"
#include "zi_plan.h"

static_assert(zi::host::kPlanMaxSegmentsPerUse == zi::kMaxStepDesc, "a packed slot use must fit one fused-step launch");

namespace zi {
namespace host {

#define ZI_HIP(call)                                                                                  \
    do {                                                                                              \
        hipError_t e_ = (call);                                                                       \
        if (e_ != hipSuccess) {                                                                       \
            (void)hipGetLastError(); /* do not leave a sticky error for the caller's next HIP call */ \
            return ::zi::host::fail(ZI_ERR_HIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
        }                                                                                             \
    } while (0)

// What kind of memory an address is: 0 device, 1 page-locked host, 2 ordinary host, -1 anything else,
// -2 if the HIP runtime cannot answer (no usable device).
inline int memory_kind(const void* p)
{
    hipPointerAttribute_t attr{};
    const hipError_t pe = hipPointerGetAttributes(&attr, p);
    if (pe != hipSuccess) {
        (void)hipGetLastError();
        return pe == hipErrorInvalidValue ? 2 : -2;      // older runtimes report unregistered memory this way
    }
    if (attr.type == hipMemoryTypeDevice) return 0;
    if (attr.type == hipMemoryTypeHost) return 1;
    if (attr.type == hipMemoryTypeUnregistered) return 2;
    return -1;
}

// A kernel is about to read or write `bytes` at p: both ends must be memory the GPU can reach (device
// or page-locked host).  An ordinary host pointer here would be a GPU memory fault, not an error code.
// Device allocations that have been looked up are remembered for the rest of the call, so a list of
// thousands of views into a few allocations costs a few queries, not thousands.
struct PointerChecker {
    struct Range { uintptr_t lo, hi; };
    Range known[8] = {};
    int n_known = 0, next = 0;

    zi_status check(const void* p, size_t bytes, int tensor, const char* name)
    {
        if (!p || bytes == 0) return ZI_OK;
        const uintptr_t lo = reinterpret_cast<uintptr_t>(p), hi = lo + bytes;
        for (int i = 0; i < n_known; ++i)
            if (lo >= known[i].lo && hi <= known[i].hi) return ZI_OK;
        const void* ends[2] = {p, static_cast<const char*>(p) + bytes - 1};
        for (const void* e : ends) {
            const int k = memory_kind(e);
            if (k == -2) return fail(ZI_ERR_HIP, "no usable HIP device (pointer query failed)");
            if (k != 0 && k != 1)
                return fail(ZI_ERR_INVALID_ARG, "tensor %d: %s (%zu bytes) is not device or page-locked host memory",
                            tensor, name, bytes);
        }
        hipDeviceptr_t base = nullptr;
        size_t size = 0;
        if (hipMemGetAddressRange(&base, &size, const_cast<void*>(p)) == hipSuccess && size > 0) {
            const uintptr_t blo = reinterpret_cast<uintptr_t>(base);
            if (lo >= blo && hi <= blo + size) {
                known[next] = {blo, blo + size};
                next = (next + 1) % 8;
                if (n_known < 8) ++n_known;
            }
        } else {
            (void)hipGetLastError();
        }
        return ZI_OK;
    }
};

inline zi_status check_kernel_visible(const void* p, size_t bytes, int tensor, const char* name)
{
    PointerChecker c;
    return c.check(p, bytes, tensor, name);
}

// Number of leading elements (0..63) the step handles one by one before its vector body.  Any value
// is legal: the body's vector accesses need only element alignment.  The choice decides how much of
// the body's traffic starts on a 128-byte line (a wavefront's run then covers whole lines) and,
// failing that, on a lane-vector boundary (16 bytes for fp32, 8 for the 2-byte arrays); arrays are
// weighted by the bytes they move per element (p, m, v: 8; g, p_lp: 2).
inline int choose_head(const void* p, const void* m, const void* v, const void* g, const void* p_lp)
{
    int best_h = 0, best = -1;
    for (int h = 0; h < 64; ++h) {
        int score = 0;
        for (const void* x : {p, m, v}) {
            const uintptr_t i = reinterpret_cast<uintptr_t>(x) / 4 + (uintptr_t)h;
            score += 8 * (i % 32 == 0 ? 4 : i % 4 == 0 ? 1 : 0);
        }
        for (const void* x : {g, (const void*)p_lp}) {
            if (!x) continue;
            const uintptr_t i = reinterpret_cast<uintptr_t>(x) / 2 + (uintptr_t)h;
            score += 2 * (i % 64 == 0 ? 4 : i % 4 == 0 ? 1 : 0);
        }
        if (score > best) { best = score; best_h = h; }
    }
    return best_h;
}

// Tensors of at least this many tiles (2^22 elements, some 20 microseconds of HBM time) are launched
// alone; shorter ones share launches of up to kMaxStepDesc tensors.
#ifndef ZI_SOLO_TILES
#define ZI_SOLO_TILES 8192
#endif
constexpr int64_t kSoloTiles = ZI_SOLO_TILES;

// Issues the fused step over a list of device-resident segments.
struct StepIssuer {
    zi::StepArgs args{};
    uint32_t tiles = 0;
    int dt;
    bool l2;
    hipStream_t stream;
    int64_t launches = 0;
    // Planning mode (zi_plan_step): with a sink set nothing is launched; every descriptor of every
    // launch is recorded instead.  `cur_tensor` is the caller's index of the tensor being added.
    std::vector<zi_step_plan_item>* plan = nullptr;
    int32_t cur_tensor = -1;
    int32_t tensor_of[zi::kMaxStepDesc] = {};

    StepIssuer(const zi::StepConsts& c, const zi_norm_result* d_norm, int dt_, bool l2_, hipStream_t s)
        : dt(dt_), l2(l2_), stream(s)
    {
        args.c = c;
        args.d_norm = d_norm;
        reset();
    }

    void reset()
    {
        args.n_desc = 0;
        tiles = 0;
        for (uint32_t& f : args.first_tile) f = 0xFFFFFFFFu;
    }

    hipError_t launch(const zi::StepArgs& a, uint32_t n_tiles, const int32_t* tensors)
    {
        const int64_t index = launches++;
        if (!plan) return zi::launch_step_wide(a, n_tiles, dt, l2, stream);
        for (int32_t i = 0; i < a.n_desc; ++i) {
            const int64_t end = i + 1 < a.n_desc ? a.t[i + 1].first_tile : n_tiles;
            plan->push_back({tensors[i], a.t[i].head, end - (int64_t)a.t[i].first_tile, (int64_t)a.t[i].first_tile,
                             (int32_t)index, a.n_desc == 1 ? 1 : 0});
        }
        return hipSuccess;
    }

    hipError_t flush()
    {
        hipError_t e = hipSuccess;
        if (args.n_desc > 0) e = launch(args, tiles, tensor_of);
        reset();
        return e;
    }

    hipError_t add(float* p, float* m, float* v, const uint16_t* g, uint16_t* p_lp, int64_t numel)
    {
        if (numel <= 0) return hipSuccess;
        zi::StepDesc d{};
        const int h = choose_head(p, m, v, g, p_lp);
        d.head = (int32_t)(h < numel ? h : numel);
        d.p_body = p + d.head; d.m_body = m + d.head; d.v_body = v + d.head; d.g_body = g + d.head;
        d.lp_body = p_lp ? p_lp + d.head : nullptr;
        d.numel = numel;
        const int64_t nquad = (numel - d.head) / zi::kQuad;
        int64_t nt = (nquad + zi::kStepTileQuads - 1) / zi::kStepTileQuads;
        if (nt < 1) nt = 1;                       // the first tile also owns the unaligned ends
        if (nt > 0x7FFFFFFF) return hipErrorInvalidValue;
        d.nquad = nquad;
        d.n_tiles = (uint32_t)nt;
        if (nt >= kSoloTiles) {                   // a launch of its own: no tensor lookup in the kernel
            zi::StepArgs solo{};
            solo.c = args.c;
            solo.d_norm = args.d_norm;
            solo.n_desc = 1;
            for (uint32_t& f : solo.first_tile) f = 0xFFFFFFFFu;
            d.first_tile = 0;
            solo.first_tile[0] = 0;
            solo.t[0] = d;
            return launch(solo, (uint32_t)nt, &cur_tensor);
        }
        if (args.n_desc == zi::kMaxStepDesc || (uint64_t)tiles + (uint64_t)nt > 0x7FFFFFFFull) {
            hipError_t e = flush();
            if (e != hipSuccess) return e;
        }
        d.first_tile = tiles;
        args.first_tile[args.n_desc] = tiles;
        tensor_of[args.n_desc] = cur_tensor;
        args.t[args.n_desc++] = d;
        tiles += (uint32_t)nt;
        return hipSuccess;
    }
};

inline zi_status check_norm_args(const zi_tensor* t, int32_t n_tensors, int dt, float loss_scale, zi_norm_result* d_out,
                          void* d_workspace, size_t workspace_bytes)
{
    if (zi_status st = check_dtype(dt)) return st;
    if (zi_status st = check_grad_list(t, n_tensors, loss_scale)) return st;
    if (!d_out) return fail(ZI_ERR_INVALID_ARG, "d_out is NULL");
    if (!aligned(d_out, 8)) return fail(ZI_ERR_ALIGNMENT, "d_out must be 8-byte aligned");
    if (!d_workspace) return fail(ZI_ERR_INVALID_ARG, "d_workspace is NULL");
    if (!aligned(d_workspace, 16)) return fail(ZI_ERR_ALIGNMENT, "d_workspace must be 16-byte aligned");
    if (workspace_bytes < (size_t)zi::kMaxPartials * sizeof(zi::NormPartial))
        return fail(ZI_ERR_INVALID_ARG, "workspace too small: %zu < %zu", workspace_bytes,
                    (size_t)zi::kMaxPartials * sizeof(zi::NormPartial));
    return ZI_OK;
}

// Issues the gradient reduction over a list of device-resident gradient arrays: partial-sum launches
// of up to kMaxNormDesc tensors, and a finalize pass whenever the workspace's partial slots run out
// and at finish().  After the first finalize the later ones add to the result already in d_out.
struct NormIssuer {
    // A workgroup covers at least four tile iterations of its tensor; at most kBlocksPerTensor
    // workgroups walk one tensor, so the partial count stays small whatever the size.
    static constexpr int64_t kMinElemsPerBlock = 4 * zi::kNormTileElems;
    static constexpr int64_t kBlocksPerTensor = 4096;

    zi::NormArgs a{};
    int64_t blocks_cap = kBlocksPerTensor;   // workgroups one tensor may get (lowered by callers with a tight budget)
    uint32_t blocks = 0;       // blocks of the launch being assembled
    uint32_t used = 0;         // partials written since the last finalize
    int finalized = 0;
    int dt;
    float loss_scale;
    zi_norm_result* d_out;
    hipStream_t s;

    NormIssuer(zi::NormPartial* partials, int dt_, float ls, zi_norm_result* out, hipStream_t st)
        : dt(dt_), loss_scale(ls), d_out(out), s(st)
    {
        a.partials = partials;
        a.partial_base = 0;
        clear_table();
    }
    static int64_t blocks_for(int64_t n, int64_t cap)
    {
        const int64_t nb = (n + kMinElemsPerBlock - 1) / kMinElemsPerBlock;
        return nb > cap ? cap : nb;
    }
    void clear_table()
    {
        a.n_desc = 0;
        for (uint32_t& f : a.first_block) f = 0xFFFFFFFFu;
    }
    hipError_t flush_launch()
    {
        hipError_t e = hipSuccess;
        if (a.n_desc > 0) e = zi::launch_norm_partials(a, blocks, dt, s);
        used += blocks;
        a.partial_base = used;
        clear_table();
        blocks = 0;
        return e;
    }
    hipError_t flush_partials()
    {
        hipError_t e = zi::launch_norm_finalize(a.partials, used, loss_scale, finalized, d_out, s);
        finalized = 1;
        used = 0;
        a.partial_base = 0;
        return e;
    }
    hipError_t add(const uint16_t* g, int64_t n)
    {
        if (n <= 0) return hipSuccess;
        int64_t nb = blocks_for(n, blocks_cap);
        hipError_t e = hipSuccess;
        if (a.n_desc == zi::kMaxNormDesc && (e = flush_launch()) != hipSuccess) return e;
        if ((uint64_t)used + blocks + (uint64_t)nb > zi::kMaxPartials) {
            if ((e = flush_launch()) != hipSuccess) return e;
            if ((e = flush_partials()) != hipSuccess) return e;
        }
        zi::NormDesc d{};
        d.g = g;
        d.numel = n;
        const int h = (int)((8 - (reinterpret_cast<uintptr_t>(g) / 2) % 8) % 8);
        d.head = (int32_t)(h < n ? h : n);
        d.first_block = blocks;
        d.n_blocks = (uint32_t)nb;
        a.first_block[a.n_desc] = blocks;
        a.t[a.n_desc++] = d;
        blocks += (uint32_t)nb;
        return hipSuccess;
    }
    hipError_t finish()
    {
        hipError_t e = flush_launch();
        if (e != hipSuccess) return e;
        return flush_partials();
    }
};


}  // namespace host
}  // namespace zi
