// Internal interface between the C-ABI layer (host) and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "zi.h"
#include "zi_checks.h"

namespace zi {

constexpr int kThreads = 256;        // 4 wavefronts of 64 lanes per workgroup
constexpr int kVec = 8;              // elements per 16-byte vector of a 2-byte array (norm pass)
// Fused step: a lane owns quads of 4 consecutive elements = one 16-byte vector of each fp32 array and
// one 8-byte vector of each 2-byte array, so every wavefront-wide access is one contiguous run.
constexpr int kQuad = 4;
constexpr int kStepThreads = 64;     // one wavefront per workgroup
constexpr int kStepUnroll = 2;       // quads per thread per tile
constexpr int kStepTileQuads = kStepThreads * kStepUnroll;
constexpr int64_t kStepTileElems = (int64_t)kStepTileQuads * kQuad;   // 512 elements per tile
constexpr int kMaxStepDesc = 32;     // tensors (or segments) per fused-step launch
// Dynamic LDS requested (never touched) by the fused step: caps residency at six single-wavefront
// workgroups per compute unit.  On this 1:1 read/write stream few, short-lived wavefronts measured
// 4-8% faster than full occupancy (sweeps over workgroup size, unroll and residency).
#ifndef ZI_STEP_LDS
#define ZI_STEP_LDS (26 * 1024)
#endif
// Workgroup ids are dealt round-robin to the 8 XCDs.  Tiles are renumbered so that, inside every run
// of 8 * kStepXcdRun tiles, each XCD owns kStepXcdRun consecutive tiles (256 KiB of each fp32 array)
// instead of every eighth one: measured +4% on top of the residency cap.
constexpr int kXcds = 8;
#ifndef ZI_STEP_XCD_RUN
#define ZI_STEP_XCD_RUN 128
#endif
constexpr int64_t kStepXcdRun = ZI_STEP_XCD_RUN;
constexpr unsigned kStepOccupancyLds = ZI_STEP_LDS;

constexpr int kNormUnroll = 8;
constexpr int kNormTileVecs = kThreads * kNormUnroll;
constexpr int64_t kNormTileElems = (int64_t)kNormTileVecs * kVec;   // 16384 elements per block iteration
constexpr int kMaxNormDesc = 64;     // gradient tensors per partial-sum launch
constexpr uint32_t kMaxPartials = 16384;   // per-block partial results the workspace holds

// One per-block partial of the gradient reduction (device workspace element).
struct NormPartial {
    double sumsq;
    uint32_t found_inf;
    uint32_t pad;
};

// One tensor (or one segment of one) as the fused step sees it.  All pointers are device memory.
// The first `head` elements are handled one by one; the 4-element lane vectors (the body) start
// after them (the host picks `head` so that as much of the traffic as possible starts on a 128-byte
// line).  Everything a workgroup would otherwise derive from numel and head is worked out once on
// the host: a wavefront lives for a few microseconds, and every scalar instruction in front of its
// first load is time with nothing in flight.
struct StepDesc {
    float* p_body;         // p + head
    float* m_body;
    float* v_body;
    const uint16_t* g_body;
    uint16_t* lp_body;     // p_lp + head, null if there is no copy
    int64_t numel;
    int64_t nquad;         // whole quads of the body: (numel - head) / 4
    int32_t head;          // 0..63
    uint32_t first_tile;   // index of this tensor's first tile within the launch
    uint32_t n_tiles;      // tiles of this tensor: max(1, ceil(nquad / kStepTileQuads))
    uint32_t reserved;
};

struct StepArgs {
    StepDesc t[kMaxStepDesc];
    int32_t n_desc;
    StepConsts c;
    const zi_norm_result* d_norm;   // device, may be null
    // first_tile of every descriptor once more, packed, 0xFFFFFFFF beyond n_desc: a workgroup finds its
    // tensor by counting the entries <= its id (a few wide scalar loads, no dependent chain).
    uint32_t first_tile[kMaxStepDesc];
};

struct NormDesc {
    const uint16_t* g;
    int64_t numel;
    int32_t head;          // 0..7 elements before the first 16-byte aligned one
    uint32_t first_block;
    uint32_t n_blocks;
    uint32_t pad;
};

struct NormArgs {
    NormDesc t[kMaxNormDesc];
    uint32_t first_block[kMaxNormDesc];   // packed copy of the descriptors' first_block, 0xFFFFFFFF beyond n_desc
    int32_t n_desc;
    uint32_t partial_base;          // index of this launch's first partial
    NormPartial* partials;
};

// Launchers (zi_kernels.hip).  Each returns the hipError_t of the launch.
hipError_t launch_step_wide(const StepArgs& a, uint32_t n_tiles, int dt, bool l2, hipStream_t s);
hipError_t launch_norm_partials(const NormArgs& a, uint32_t n_blocks, int dt, hipStream_t s);
hipError_t launch_norm_finalize(const NormPartial* partials, uint32_t count, float loss_scale, int accumulate,
                                zi_norm_result* d_out, hipStream_t s);

hipError_t launch_norm_refresh(zi_norm_result* d_result, float loss_scale, hipStream_t s);
hipError_t launch_hbm_probe(void* a, void* b, int64_t n4, int mode, float* sink, hipStream_t s);

}  // namespace zi
