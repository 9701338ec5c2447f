// gfx950 kernels of the optimizer hot path: gradient sum of squares + overflow flag,
// and the fused AdamW read-modify-write pass.
//
// Both are pure HBM streams (Section 4.1, "AIT w.r.t. Optimizer States": the step reads every
// state once and writes it once), so the design is about bytes, not flops: each wavefront-wide
// access is one contiguous run of 16-byte (fp32 arrays) or 8-byte (2-byte arrays) lanes, marked
// non-temporal because nothing is reused, a thread has all loads of a tile in flight before the
// first use, nothing goes through LDS except the block reduction of the norm, and no matrix core
// is involved because there is no contraction.
//
// Arithmetic order of the update: see include/zi.h.  Compile with -ffp-contract=off so that the
// only fused multiply-adds are the ones written as fma below.
#include <hip/hip_runtime.h>

#include "zi_internal.h"

namespace zi {

// ---------------------------------------------------------------------------------- casts

template <int DT>
__device__ __forceinline__ float widen16(uint32_t h);

template <>
__device__ __forceinline__ float widen16<ZI_BF16>(uint32_t h)
{
    return __uint_as_float(h << 16);
}

template <>
__device__ __forceinline__ float widen16<ZI_FP16>(uint32_t h)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)h);   // exact, fp16 subnormals included
}

// low and high half of a packed pair
template <int DT>
__device__ __forceinline__ void widen_pair(uint32_t w, float& lo, float& hi)
{
    if constexpr (DT == ZI_BF16) {
        lo = __uint_as_float(w << 16);
        hi = __uint_as_float(w & 0xFFFF0000u);
    } else {
        lo = widen16<ZI_FP16>(w & 0xFFFFu);
        hi = widen16<ZI_FP16>(w >> 16);
    }
}

// fp32 -> low precision, round to nearest even (the hardware converters of gfx950 in the default
// rounding mode; fp16 subnormals are produced, NaN stays NaN, overflow gives inf).
template <int DT>
__device__ __forceinline__ uint32_t narrow16(float x)
{
    if constexpr (DT == ZI_BF16) {
        return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)x);
    } else {
        return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)x);
    }
}

template <int DT>
__device__ __forceinline__ uint32_t narrow_pair(float lo, float hi)
{
    return narrow16<DT>(lo) | (narrow16<DT>(hi) << 16);
}

// ------------------------------------------------------------------------- the update itself

template <bool L2>
__device__ __forceinline__ void adamw_element(float& p, float& m, float& v, float g, float gscale,
                                              const StepConsts& c)
{
    g = g * gscale;
    if constexpr (L2) g = __builtin_fmaf(c.weight_decay, p, g);
    const float m1 = __builtin_fmaf(c.beta1, m, c.omb1 * g);
    const float v1 = __builtin_fmaf(c.beta2, v, c.omb2 * (g * g));
    const float d = __builtin_fmaf(__builtin_sqrtf(v1), c.inv_sqrt_bc2, c.eps);
    const float q = m1 / d;
    const float pd = __builtin_fmaf(-c.decay, p, p);
    p = __builtin_fmaf(-c.step_size, q, pd);
    m = m1;
    v = v1;
}

// Skip decision and gradient factor, from the device-resident norm result: norm = sqrt(sumsq) /
// loss_scale, clip = max_norm / (norm + 1e-6) where that is below 1, factor = clip / loss_scale, in
// double, rounded once to fp32.  Returns false if the step must be skipped.
//
// Every wavefront runs this before it issues its first load and lives for a few microseconds, so
// the dependent chain is kept short (an fp64 square root and three divisions cost 5 points of
// bandwidth on some devices); each shortcut gives the same bits as the full expression:
//   - a step that does not clip uses the factor the host prepared, (float)(1 / loss_scale);
//   - the result's `norm` is used when its `scale_bits` say it was divided by this step's loss scale
//     (the reduction wrote both); with any other scale the norm is derived from the sum of squares,
//     so a reduction called with a different scale cannot make the step clip wrongly;
//   - dividing by a loss scale that is a power of two is multiplying by its inverse, which is exact;
//   - with a maximum norm that is a power of two (1 is the usual value) the quotient max_norm /
//     (norm + 1e-6) is the reduction's 1 / (norm + 1e-6) times that power, again exactly.
// What is left in the usual case is a comparison and two multiplications.
//
// The result is read through the constant address space, which makes the reads scalar loads: they
// are served by the scalar cache in a few hundred cycles.  As ordinary global loads they would
// join the vector memory pipeline behind the streaming traffic of the other wavefronts, and every
// wavefront would spend a full loaded-memory round trip (as long as its real loads take) before it
// issues anything, which costs 4 to 9 points of bandwidth.  The result was written by an earlier
// kernel on the stream and nothing writes it while the step runs, which is what that address space asks.
// All 32 bytes are fetched by one load in front of the first branch: field-by-field reads would be
// sunk into the branches that use them, one dependent round trip to the scalar cache each.
typedef uint32_t u32x8_k __attribute__((ext_vector_type(8), aligned(8)));
static_assert(sizeof(zi_norm_result) == 32, "the prologue reads the result as eight dwords");
__device__ __forceinline__ double dwords_as_double(uint32_t lo, uint32_t hi)
{
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ bool step_prologue(const zi_norm_result* d_norm, const StepConsts& c, float& gscale)
{
    gscale = c.host_gscale;
    if (d_norm) {
        const u32x8_k raw = *(const __attribute__((address_space(4))) u32x8_k*)(uintptr_t)d_norm;
        const double sumsq = dwords_as_double(raw[0], raw[1]);
        const double r_norm = dwords_as_double(raw[2], raw[3]);
        const uint32_t found_inf = raw[4], scale_bits = raw[5];
        const double r_inv_norm = dwords_as_double(raw[6], raw[7]);
        if (found_inf) return false;
        if (c.max_grad_norm > 0.0f) {
            const double ls = (double)c.loss_scale;
            const bool same_scale = scale_bits == __float_as_uint(c.loss_scale);
            const double norm = same_scale ? r_norm : __builtin_sqrt(sumsq) / ls;
            const double mx = (double)c.max_grad_norm;
            if (norm + 1e-6 > mx) {
                const double clip = same_scale && c.max_norm_is_pow2 ? mx * r_inv_norm : mx / (norm + 1e-6);
                gscale = (float)(c.scale_is_pow2 ? clip * c.inv_loss_scale : clip / ls);
            }
        }
    }
    return true;
}

// One element of the unaligned ends, addressed relative to the body (i may be negative: the head).
template <int DT, bool L2>
__device__ __forceinline__ void step_scalar_at(const StepDesc& T, int64_t i, float gscale, const StepConsts& c)
{
    float p = T.p_body[i], m = T.m_body[i], v = T.v_body[i];
    const float g = widen16<DT>(T.g_body[i]);
    adamw_element<L2>(p, m, v, g, gscale, c);
    T.p_body[i] = p;
    T.m_body[i] = m;
    T.v_body[i] = v;
    if (T.lp_body) T.lp_body[i] = (uint16_t)narrow16<DT>(p);
}

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// The fused step's lane vectors as they sit in memory: only element alignment is promised (gfx950
// runs global loads and stores of any alignment as one instruction; the host picks the body's
// start so that as many arrays as possible are line-aligned anyway).
typedef f32x4 f32x4_mem __attribute__((aligned(4)));
typedef u32x2 u32x2_mem __attribute__((aligned(2)));

// Streaming accesses: the data is touched once, so it should not displace anything in the caches.
// (The two switches exist for tuning builds; the defaults are the measured best.)
#ifndef ZI_NT_LOAD
#define ZI_NT_LOAD 1
#endif
#ifndef ZI_NT_STORE
#define ZI_NT_STORE 1
#endif
template <typename V>
__device__ __forceinline__ V load_stream(const V* a)
{
#if ZI_NT_LOAD
    return __builtin_nontemporal_load(a);
#else
    return *a;
#endif
}
template <typename V>
__device__ __forceinline__ void store_stream(V* a, V x)
{
#if ZI_NT_STORE
    __builtin_nontemporal_store(x, a);
#else
    *a = x;
#endif
}
// The same for the element-aligned lane vectors of the fused step (written out: an alignment attribute
// on a typedef does not survive template argument deduction).  The pointers carry the global address
// space in their type, so the accesses stay global_load / global_store wherever the pointer value
// has been through (a pointer of unknown provenance would make them flat accesses, which also tie up
// the scalar-memory counter and force the compiler to wait for all loads at once).
#define ZI_GLOBAL __attribute__((address_space(1)))
typedef ZI_GLOBAL f32x4_mem* GlobalF4;
typedef ZI_GLOBAL u32x2_mem* GlobalU2;
typedef const ZI_GLOBAL u32x2_mem* GlobalConstU2;
__device__ __forceinline__ f32x4 load_stream_any(const ZI_GLOBAL f32x4_mem* a)
{
#if ZI_NT_LOAD
    return __builtin_nontemporal_load(a);
#else
    return *a;
#endif
}
__device__ __forceinline__ u32x2 load_stream_any(const ZI_GLOBAL u32x2_mem* a)
{
#if ZI_NT_LOAD
    return __builtin_nontemporal_load(a);
#else
    return *a;
#endif
}
__device__ __forceinline__ void store_stream_any(ZI_GLOBAL f32x4_mem* a, f32x4 x)
{
#if ZI_NT_STORE
    __builtin_nontemporal_store(x, a);
#else
    *a = x;
#endif
}
__device__ __forceinline__ void store_stream_any(ZI_GLOBAL u32x2_mem* a, u32x2 x)
{
#if ZI_NT_STORE
    __builtin_nontemporal_store(x, a);
#else
    *a = x;
#endif
}

// Four consecutive elements: one 16-byte vector of p, m, v and one 8-byte vector of g.
template <int DT, bool L2>
__device__ __forceinline__ u32x2 step_quad(f32x4& p, f32x4& m, f32x4& v, const u32x2 g, float gscale,
                                           const StepConsts& c)
{
    float g0, g1, g2, g3;
    widen_pair<DT>(g.x, g0, g1);
    widen_pair<DT>(g.y, g2, g3);
    float px = p.x, py = p.y, pz = p.z, pw = p.w;
    float mx = m.x, my = m.y, mz = m.z, mw = m.w;
    float vx = v.x, vy = v.y, vz = v.z, vw = v.w;
    adamw_element<L2>(px, mx, vx, g0, gscale, c);
    adamw_element<L2>(py, my, vy, g1, gscale, c);
    adamw_element<L2>(pz, mz, vz, g2, gscale, c);
    adamw_element<L2>(pw, mw, vw, g3, gscale, c);
    p = f32x4{px, py, pz, pw};
    m = f32x4{mx, my, mz, mw};
    v = f32x4{vx, vy, vz, vw};
    u32x2 lp;
    lp.x = narrow_pair<DT>(px, py);
    lp.y = narrow_pair<DT>(pz, pw);
    return lp;
}

// One workgroup = one tile of kStepTileElems elements of one tensor.  blockIdx.x counts tiles over
// all tensors of the launch; first_tile locates the tensor.
// SINGLE: the launch covers one tensor (every long tensor gets such a launch: a workgroup lives for a few
// microseconds, so even a short search for its tensor costs bandwidth).  Otherwise the workgroup counts
// the table entries <= its id: a few wide scalar loads and no dependent chain.
template <int DT, bool L2, bool SINGLE>
__global__ __launch_bounds__(kStepThreads) __attribute__((amdgpu_waves_per_eu(1, 2)))
void adamw_wide_kernel(const StepArgs a)
{
    const uint32_t block = blockIdx.x;
    int d = 0;
    if constexpr (!SINGLE) {
        d = -1;                           // first_tile[0] is 0, so the count is at least 1
#pragma unroll
        for (int i = 0; i < kMaxStepDesc; ++i) d += block >= a.first_tile[i] ? 1 : 0;
    }
    const StepDesc& T = a.t[d];

    const int64_t nquad = T.nquad;

    // XCD-aware renumbering.  Workgroup ids of the launch go round-robin to the XCDs, so the runs are
    // counted in launch-wide ids (a tensor that does not start on a run boundary keeps the XCD <->
    // contiguous-tiles correspondence); it is a bijection on every run of 8 * kStepXcdRun workgroups
    // that lies inside one tensor, and the workgroups of incomplete runs keep their tiles.
    uint32_t tile;
    {
        constexpr uint32_t run = kXcds * kStepXcdRun;
        const uint32_t r = block % run;
        const uint32_t base = block - r;
        uint32_t nb = block;
        if (base >= T.first_tile && T.n_tiles >= run && base - T.first_tile <= T.n_tiles - run)
            nb = base + (r % kXcds) * (uint32_t)kStepXcdRun + r / kXcds;
        tile = nb - T.first_tile;
    }
    const int64_t ti = tile;

    GlobalF4 __restrict__ p4 = (GlobalF4)(uintptr_t)T.p_body;
    GlobalF4 __restrict__ m4 = (GlobalF4)(uintptr_t)T.m_body;
    GlobalF4 __restrict__ v4 = (GlobalF4)(uintptr_t)T.v_body;
    GlobalConstU2 __restrict__ g2 = (GlobalConstU2)(uintptr_t)T.g_body;
    GlobalU2 __restrict__ lp2 = (GlobalU2)(uintptr_t)T.lp_body;
    // Everything the tile needs from the kernel arguments is made to exist here, in front of the
    // prologue: otherwise the compiler sinks the argument loads of the five pointers below the
    // prologue's early exit, and a wavefront pays a third dependent round trip to the scalar cache
    // (arguments, norm result, arguments again) before its first load.
    asm volatile("" : "+s"(p4), "+s"(m4), "+s"(v4), "+s"(g2), "+s"(lp2));

    // The norm result is looked at only now, so that its scalar load (whose address is itself a kernel
    // argument) is not in front of the work above.
    float gscale;
    if (!step_prologue(a.d_norm, a.c, gscale)) return;

    // Elements before the vector body (at most 63) and after it (at most 3), by the tensor's first tile.
    if (tile == 0) {
        const int64_t t = threadIdx.x;
        const int64_t head = T.head;
        if (t < head) step_scalar_at<DT, L2>(T, t - head, gscale, a.c);
        const int64_t body = nquad * kQuad;
        const int64_t tail = T.numel - head - body;
        if (t >= 4 && t - 4 < tail) step_scalar_at<DT, L2>(T, body + (t - 4), gscale, a.c);
    }

    const int64_t q0 = ti * kStepTileQuads + threadIdx.x;

    if ((ti + 1) * kStepTileQuads <= nquad) {
        // full tile: every load is issued before the first result is needed
        f32x4 p[kStepUnroll], m[kStepUnroll], v[kStepUnroll];
        u32x2 g[kStepUnroll];
#pragma unroll
        for (int u = 0; u < kStepUnroll; ++u) {
            const int64_t i = q0 + (int64_t)u * kStepThreads;
            g[u] = load_stream_any(g2 + i);
            p[u] = load_stream_any(p4 + i);
            m[u] = load_stream_any(m4 + i);
            v[u] = load_stream_any(v4 + i);
        }
#pragma unroll
        for (int u = 0; u < kStepUnroll; ++u) {
            const int64_t i = q0 + (int64_t)u * kStepThreads;
            const u32x2 lp = step_quad<DT, L2>(p[u], m[u], v[u], g[u], gscale, a.c);
            store_stream_any(p4 + i, p[u]);
            store_stream_any(m4 + i, m[u]);
            store_stream_any(v4 + i, v[u]);
            if (lp2) store_stream_any(lp2 + i, lp);
        }
    } else {
        for (int u = 0; u < kStepUnroll; ++u) {
            const int64_t i = q0 + (int64_t)u * kStepThreads;
            if (i < nquad) {
                const u32x2 g = load_stream_any(g2 + i);
                f32x4 p = load_stream_any(p4 + i), m = load_stream_any(m4 + i), v = load_stream_any(v4 + i);
                const u32x2 lp = step_quad<DT, L2>(p, m, v, g, gscale, a.c);
                store_stream_any(p4 + i, p);
                store_stream_any(m4 + i, m);
                store_stream_any(v4 + i, v);
                if (lp2) store_stream_any(lp2 + i, lp);
            }
        }
    }
}

hipError_t launch_step_wide(const StepArgs& a, uint32_t n_tiles, int dt, bool l2, hipStream_t s)
{
    if (n_tiles == 0) return hipSuccess;
    const dim3 grid(n_tiles), block(kStepThreads);
    const bool single = a.n_desc == 1;
#define ZI_LAUNCH_STEP(DT, L2, SINGLE) \
    hipLaunchKernelGGL((adamw_wide_kernel<DT, L2, SINGLE>), grid, block, kStepOccupancyLds, s, a)
    if (dt == ZI_BF16) {
        if (l2) { if (single) ZI_LAUNCH_STEP(ZI_BF16, true, true); else ZI_LAUNCH_STEP(ZI_BF16, true, false); }
        else    { if (single) ZI_LAUNCH_STEP(ZI_BF16, false, true); else ZI_LAUNCH_STEP(ZI_BF16, false, false); }
    } else {
        if (l2) { if (single) ZI_LAUNCH_STEP(ZI_FP16, true, true); else ZI_LAUNCH_STEP(ZI_FP16, true, false); }
        else    { if (single) ZI_LAUNCH_STEP(ZI_FP16, false, true); else ZI_LAUNCH_STEP(ZI_FP16, false, false); }
    }
#undef ZI_LAUNCH_STEP
    return hipGetLastError();
}

// ------------------------------------------------------- gradient sum of squares + overflow flag

// Bit 15 / bit 31 of the result is set iff the exponent field of the low / high half is all ones.
template <int DT>
__device__ __forceinline__ uint32_t nonfinite_bits(uint32_t w)
{
    constexpr uint32_t mask = DT == ZI_BF16 ? 0x7F807F80u : 0x7C007C00u;
    constexpr uint32_t one = DT == ZI_BF16 ? 0x00800080u : 0x04000400u;
    return ((w & mask) + one) & 0x80008000u;
}

template <int DT>
__device__ __forceinline__ void sumsq_word(uint32_t w, double& acc0, double& acc1, uint32_t& flag)
{
    flag |= nonfinite_bits<DT>(w);
    float lo, hi;
    widen_pair<DT>(w, lo, hi);
    const double dlo = (double)lo, dhi = (double)hi;
    acc0 = __builtin_fma(dlo, dlo, acc0);
    acc1 = __builtin_fma(dhi, dhi, acc1);
}

template <int DT>
__device__ __forceinline__ void sumsq_vec(const u32x4 g, double& acc0, double& acc1, uint32_t& flag)
{
    sumsq_word<DT>(g.x, acc0, acc1, flag);
    sumsq_word<DT>(g.y, acc0, acc1, flag);
    sumsq_word<DT>(g.z, acc0, acc1, flag);
    sumsq_word<DT>(g.w, acc0, acc1, flag);
}

__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

__device__ __forceinline__ uint32_t wave_or(uint32_t x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x |= __shfl_xor(x, off, 64);
    return x;
}

// Two-level reduction: wavefront shuffles, then one LDS slot per wavefront.  Result valid in thread 0.
template <int NWAVES>
__device__ __forceinline__ void block_reduce(double& sum, uint32_t& flag)
{
    __shared__ double s_sum[NWAVES];
    __shared__ uint32_t s_flag[NWAVES];
    sum = wave_sum(sum);
    flag = wave_or(flag);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) {
        s_sum[wave] = sum;
        s_flag[wave] = flag;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        uint32_t f = 0;
#pragma unroll
        for (int w = 0; w < NWAVES; ++w) {
            t += s_sum[w];
            f |= s_flag[w];
        }
        sum = t;
        flag = f;
    }
}

// Each workgroup walks its tensor with a stride of n_blocks tiles and leaves one partial.
// Squares are accumulated in double: exact products, and a finite gradient whose square would
// overflow fp32 still gives a finite sum.
template <int DT>
__global__ __launch_bounds__(kThreads) void sumsq_partial_kernel(const NormArgs a)
{
    uint32_t b = blockIdx.x;
    int d = -1;                               // first_block[0] is 0: the count is at least 1
#pragma unroll
    for (int i = 0; i < kMaxNormDesc; ++i) d += b >= a.first_block[i] ? 1 : 0;
    const NormDesc& T = a.t[d];
    b -= T.first_block;

    const int64_t head = T.head;
    const int64_t nvec = (T.numel - head) / kVec;
    const int64_t body_end = head + nvec * kVec;
    const u32x4* __restrict__ g4 = reinterpret_cast<const u32x4*>(T.g + head);

    double acc0 = 0.0, acc1 = 0.0;
    uint32_t flag = 0;

    if (b == 0) {
        const int64_t t = threadIdx.x;
        const int64_t tail = T.numel - body_end;
        int64_t idx = -1;
        if (t < head) idx = t;
        else if (t >= 8 && t - 8 < tail) idx = body_end + (t - 8);
        if (idx >= 0) {
            const uint32_t h = T.g[idx];
            flag |= nonfinite_bits<DT>(h);
            const double x = (double)widen16<DT>(h);
            acc0 = __builtin_fma(x, x, acc0);
        }
    }

    const int64_t stride = (int64_t)T.n_blocks * kNormTileVecs;
    for (int64_t base = (int64_t)b * kNormTileVecs; base < nvec; base += stride) {
        const int64_t iv = base + threadIdx.x;
        if (base + kNormTileVecs <= nvec) {
            u32x4 g[kNormUnroll];
#pragma unroll
            for (int u = 0; u < kNormUnroll; ++u) g[u] = load_stream(g4 + iv + (int64_t)u * kThreads);
#pragma unroll
            for (int u = 0; u < kNormUnroll; ++u) sumsq_vec<DT>(g[u], acc0, acc1, flag);
        } else {
            for (int u = 0; u < kNormUnroll; ++u) {
                const int64_t j = iv + (int64_t)u * kThreads;
                if (j < nvec) sumsq_vec<DT>(load_stream(g4 + j), acc0, acc1, flag);
            }
        }
    }

    double sum = acc0 + acc1;
    block_reduce<kThreads / 64>(sum, flag);
    if (threadIdx.x == 0) {
        NormPartial out;
        out.sumsq = sum;
        out.found_inf = flag ? 1u : 0u;
        out.pad = 0;
        a.partials[a.partial_base + blockIdx.x] = out;
    }
}

constexpr int kFinalThreads = 1024;

// One workgroup adds the partials in a fixed order (so the result does not depend on scheduling)
// and writes the device-resident result.
__global__ __launch_bounds__(kFinalThreads) void norm_finalize_kernel(const NormPartial* __restrict__ partials,
                                                                      uint32_t count, float loss_scale,
                                                                      int accumulate, zi_norm_result* out)
{
    double sum = 0.0;
    uint32_t flag = 0;
    for (uint32_t i = threadIdx.x; i < count; i += kFinalThreads) {
        sum += partials[i].sumsq;
        flag |= partials[i].found_inf;
    }
    block_reduce<kFinalThreads / 64>(sum, flag);
    if (threadIdx.x == 0) {
        if (accumulate) {
            sum += out->sumsq;
            flag |= out->found_inf;
        }
        zi_norm_result r;
        r.sumsq = sum;
        r.norm = __builtin_sqrt(sum) / (double)loss_scale;
        r.found_inf = flag ? 1u : 0u;
        r.scale_bits = __float_as_uint(loss_scale);
        r.inv_norm = 1.0 / (r.norm + 1e-6);
        *out = r;
    }
}

// After the sum of squares and the flag have been combined across ranks (sum and max), the norm
// field is recomputed from the combined sum.
__global__ void norm_refresh_kernel(zi_norm_result* r, float loss_scale)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        r->norm = __builtin_sqrt(r->sumsq) / (double)loss_scale;
        r->found_inf = r->found_inf ? 1u : 0u;
        r->scale_bits = __float_as_uint(loss_scale);
        r->inv_norm = 1.0 / (r->norm + 1e-6);
    }
}

hipError_t launch_norm_refresh(zi_norm_result* d_result, float loss_scale, hipStream_t s)
{
    hipLaunchKernelGGL(norm_refresh_kernel, dim3(1), dim3(64), 0, s, d_result, loss_scale);
    return hipGetLastError();
}

hipError_t launch_norm_partials(const NormArgs& a, uint32_t n_blocks, int dt, hipStream_t s)
{
    if (n_blocks == 0) return hipSuccess;
    const dim3 grid(n_blocks), block(kThreads);
    if (dt == ZI_BF16) hipLaunchKernelGGL((sumsq_partial_kernel<ZI_BF16>), grid, block, 0, s, a);
    else               hipLaunchKernelGGL((sumsq_partial_kernel<ZI_FP16>), grid, block, 0, s, a);
    return hipGetLastError();
}

hipError_t launch_norm_finalize(const NormPartial* partials, uint32_t count, float loss_scale, int accumulate,
                                zi_norm_result* d_out, hipStream_t s)
{
    hipLaunchKernelGGL(norm_finalize_kernel, dim3(1), dim3(kFinalThreads), 0, s, partials, count, loss_scale,
                       accumulate, d_out);
    return hipGetLastError();
}

// -------------------------------------------------------------- plain streams (measurement aid)

// What the memory system gives a pure read, a 1:1 copy and an in-place read-modify-write of one
// array, launched the way that measured best for such streams on this device: single-wavefront
// workgroups, four 16-byte vectors per lane (4 KiB contiguous per wavefront), non-temporal accesses,
// residency capped at six wavefronts per compute unit by unused dynamic LDS, and the same XCD-aware
// tile renumbering as the fused step.  These are the ceilings the fused step is compared with.
constexpr int kProbeUnroll = 4;
constexpr int kProbeTileVecs = 64 * kProbeUnroll;

template <int MODE>
__global__ __launch_bounds__(64) void hbm_probe_kernel(f32x4* __restrict__ a, f32x4* __restrict__ b, int64_t n4,
                                                       float* sink)
{
    const int64_t ntiles = (n4 + kProbeTileVecs - 1) / kProbeTileVecs;
    constexpr uint32_t run = kXcds * (uint32_t)kStepXcdRun;
    const uint32_t block = blockIdx.x;
    const uint32_t r = block % run, base = block - r;
    uint32_t nb = block;
    if ((int64_t)base + run <= ntiles) nb = base + (r % kXcds) * (uint32_t)kStepXcdRun + r / kXcds;
    const int64_t i0 = (int64_t)nb * kProbeTileVecs + threadIdx.x;
    f32x4 x[kProbeUnroll];
    if ((int64_t)(nb + 1) * kProbeTileVecs <= n4) {
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) x[u] = load_stream(a + i0 + u * 64);
        if constexpr (MODE == 0) {
            float s = 0.0f;
#pragma unroll
            for (int u = 0; u < kProbeUnroll; ++u) s += x[u].x + x[u].y + x[u].z + x[u].w;
            if (s == 1.2345678e-30f) *sink = 1.0f;   // keeps the loads alive
        } else if constexpr (MODE == 1) {
#pragma unroll
            for (int u = 0; u < kProbeUnroll; ++u) store_stream(b + i0 + u * 64, x[u]);
        } else {
#pragma unroll
            for (int u = 0; u < kProbeUnroll; ++u) store_stream(a + i0 + u * 64, x[u] + 1.0f);
        }
    } else {
        for (int u = 0; u < kProbeUnroll; ++u) {
            const int64_t i = i0 + u * 64;
            if (i >= n4) break;
            const f32x4 y = load_stream(a + i);
            if constexpr (MODE == 0) {
                if (y.x + y.y + y.z + y.w == 1.2345678e-30f) *sink = 1.0f;
            } else if constexpr (MODE == 1) {
                store_stream(b + i, y);
            } else {
                store_stream(a + i, y + 1.0f);
            }
        }
    }
}

hipError_t launch_hbm_probe(void* a, void* b, int64_t n4, int mode, float* sink, hipStream_t s)
{
    if (n4 <= 0) return hipSuccess;
    const dim3 grid((uint32_t)((n4 + kProbeTileVecs - 1) / kProbeTileVecs)), block(64);
    const unsigned lds = kStepOccupancyLds;
    if (mode == 0) hipLaunchKernelGGL(hbm_probe_kernel<0>, grid, block, lds, s, (f32x4*)a, (f32x4*)b, n4, sink);
    else if (mode == 1) hipLaunchKernelGGL(hbm_probe_kernel<1>, grid, block, lds, s, (f32x4*)a, (f32x4*)b, n4, sink);
    else hipLaunchKernelGGL(hbm_probe_kernel<2>, grid, block, lds, s, (f32x4*)a, (f32x4*)b, n4, sink);
    return hipGetLastError();
}

}  // namespace zi
