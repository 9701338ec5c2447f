// The optimizer step on the host CPUs, for state that lives in host memory.
//
// This is the paper's own placement of the offloaded step (Section 5.2.2: with optimizer states in CPU
// memory the step uses the aggregate CPU compute and memory bandwidth; only gradients come down and the
// low-precision parameters go up over the link, 2 + 2 bytes per element instead of 12 + 12).  It is a
// separate entry point that a caller chooses explicitly; no GPU entry point ever falls back to it.
//
// Same arithmetic, in the same binary32 order, as the HIP kernels (see include/zi.h), written with
// AVX2 / FMA / F16C intrinsics: vector sqrt and divide are IEEE-correct, fmadd / fnmadd round once, and
// the default MXCSR keeps denormals.  Compiled by the host compiler with -ffp-contract=off.
#include <immintrin.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <exception>
#include <thread>
#include <vector>

#include "zi.h"

namespace zi {
namespace host {
zi_status fail(zi_status st, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
}
}  // namespace zi

using zi::host::fail;

namespace {

struct Consts {
    float beta1, beta2, omb1, omb2, eps, step_size, inv_sqrt_bc2, decay, weight_decay, gscale;
    bool l2;
};

inline float widen_scalar(uint16_t h, int dt)
{
    if (dt == ZI_BF16) {
        const uint32_t b = (uint32_t)h << 16;
        float f;
        std::memcpy(&f, &b, 4);
        return f;
    }
    return _cvtsh_ss(h);
}

inline uint16_t narrow_scalar(float x, int dt)
{
    if (dt == ZI_BF16) {
        uint32_t b;
        std::memcpy(&b, &x, 4);
        if ((b & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((b >> 16) | 0x0040u);
        b += 0x7FFFu + ((b >> 16) & 1u);
        return (uint16_t)(b >> 16);
    }
    return (uint16_t)_cvtss_sh(x, _MM_FROUND_TO_NEAREST_INT | _MM_FROUND_NO_EXC);
}

inline void step_scalar(float* p, float* m, float* v, const uint16_t* g, uint16_t* lp, int64_t i, int dt,
                        const Consts& c)
{
    float gi = widen_scalar(g[i], dt) * c.gscale;
    if (c.l2) gi = std::fmaf(c.weight_decay, p[i], gi);
    const float m1 = std::fmaf(c.beta1, m[i], c.omb1 * gi);
    const float v1 = std::fmaf(c.beta2, v[i], c.omb2 * (gi * gi));
    const float d = std::fmaf(std::sqrt(v1), c.inv_sqrt_bc2, c.eps);
    const float q = m1 / d;
    const float pd = std::fmaf(-c.decay, p[i], p[i]);
    const float p1 = std::fmaf(-c.step_size, q, pd);
    m[i] = m1;
    v[i] = v1;
    p[i] = p1;
    if (lp) lp[i] = narrow_scalar(p1, dt);
}

template <int DT>
inline __m256 widen8(const uint16_t* g)
{
    const __m128i h = _mm_loadu_si128((const __m128i*)g);
    if (DT == ZI_BF16) return _mm256_castsi256_ps(_mm256_slli_epi32(_mm256_cvtepu16_epi32(h), 16));
    return _mm256_cvtph_ps(h);
}

template <int DT>
inline void narrow8(__m256 x, uint16_t* out)
{
    if (DT == ZI_FP16) {
        _mm_storeu_si128((__m128i*)out, _mm256_cvtps_ph(x, _MM_FROUND_TO_NEAREST_INT | _MM_FROUND_NO_EXC));
        return;
    }
    // bf16, round to nearest even: add 0x7FFF + lsb, keep the upper half; NaN is quieted instead
    const __m256i b = _mm256_castps_si256(x);
    const __m256i lsb = _mm256_and_si256(_mm256_srli_epi32(b, 16), _mm256_set1_epi32(1));
    const __m256i rounded = _mm256_srli_epi32(_mm256_add_epi32(b, _mm256_add_epi32(lsb, _mm256_set1_epi32(0x7FFF))), 16);
    const __m256i quiet = _mm256_or_si256(_mm256_srli_epi32(b, 16), _mm256_set1_epi32(0x0040));
    const __m256 isnan = _mm256_cmp_ps(x, x, _CMP_UNORD_Q);
    const __m256i r = _mm256_blendv_epi8(rounded, quiet, _mm256_castps_si256(isnan));
    const __m256i packed = _mm256_packus_epi32(r, r);                         // per 128-bit lane
    const __m256i ordered = _mm256_permute4x64_epi64(packed, 0x08);           // lanes 0 and 2
    _mm_storeu_si128((__m128i*)out, _mm256_castsi256_si128(ordered));
}

template <int DT, bool L2>
void step_range(float* p, float* m, float* v, const uint16_t* g, uint16_t* lp, int64_t lo, int64_t hi,
                const Consts& c)
{
    const __m256 beta1 = _mm256_set1_ps(c.beta1), beta2 = _mm256_set1_ps(c.beta2);
    const __m256 omb1 = _mm256_set1_ps(c.omb1), omb2 = _mm256_set1_ps(c.omb2), eps = _mm256_set1_ps(c.eps);
    const __m256 step = _mm256_set1_ps(c.step_size), isb = _mm256_set1_ps(c.inv_sqrt_bc2);
    const __m256 decay = _mm256_set1_ps(c.decay), wd = _mm256_set1_ps(c.weight_decay);
    const __m256 gscale = _mm256_set1_ps(c.gscale);
    int64_t i = lo;
    for (; i + 8 <= hi; i += 8) {
        __m256 gi = _mm256_mul_ps(widen8<DT>(g + i), gscale);
        const __m256 pi = _mm256_loadu_ps(p + i);
        if (L2) gi = _mm256_fmadd_ps(wd, pi, gi);
        const __m256 m1 = _mm256_fmadd_ps(beta1, _mm256_loadu_ps(m + i), _mm256_mul_ps(omb1, gi));
        const __m256 v1 = _mm256_fmadd_ps(beta2, _mm256_loadu_ps(v + i), _mm256_mul_ps(omb2, _mm256_mul_ps(gi, gi)));
        const __m256 d = _mm256_fmadd_ps(_mm256_sqrt_ps(v1), isb, eps);
        const __m256 q = _mm256_div_ps(m1, d);
        const __m256 pd = _mm256_fnmadd_ps(decay, pi, pi);
        const __m256 p1 = _mm256_fnmadd_ps(step, q, pd);
        _mm256_storeu_ps(m + i, m1);
        _mm256_storeu_ps(v + i, v1);
        _mm256_storeu_ps(p + i, p1);
        if (lp) narrow8<DT>(p1, lp + i);
    }
    for (; i < hi; ++i) step_scalar(p, m, v, g, lp, i, DT, c);
}

// Runs fn(block) for block = 0..n_blocks-1 on n_threads threads (the caller's included).
template <class F>
void parallel_blocks(int64_t n_blocks, int n_threads, F fn)
{
    std::atomic<int64_t> next{0};
    auto work = [&] {
        for (int64_t b = next.fetch_add(1); b < n_blocks; b = next.fetch_add(1)) fn(b);
    };
    std::vector<std::thread> th;
    const int extra = (int)std::min<int64_t>(n_threads - 1, n_blocks - 1);
    for (int i = 0; i < extra; ++i) {
        try {
            th.emplace_back(work);
        } catch (const std::exception&) {
            break;          // fewer threads than asked for; the result does not depend on the count
        }
    }
    work();
    for (auto& t : th) t.join();
}

constexpr int64_t kBlockElems = 1 << 18;   // 1 MiB of each fp32 array per block

bool cpu_ok()
{
    return __builtin_cpu_supports("avx2") && __builtin_cpu_supports("fma") && __builtin_cpu_supports("f16c");
}

zi_status check_common(const zi_tensor* t, int32_t n_tensors, int dt, int32_t n_threads)
{
    if (!cpu_ok()) return fail(ZI_ERR_UNSUPPORTED, "the host step needs a CPU with AVX2, FMA and F16C");
    if (dt != ZI_BF16 && dt != ZI_FP16) return fail(ZI_ERR_INVALID_ARG, "unknown low-precision dtype %d", dt);
    if (n_tensors < 0) return fail(ZI_ERR_INVALID_ARG, "n_tensors < 0");
    if (n_tensors > 0 && !t) return fail(ZI_ERR_INVALID_ARG, "tensor list is NULL");
    if (n_threads < 1 || n_threads > 256) return fail(ZI_ERR_INVALID_ARG, "n_threads must be in 1..256");
    return ZI_OK;
}

}  // namespace

extern "C" zi_status zi_host_grad_norm(const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt, float loss_scale,
                                       zi_norm_result* h_out, int32_t n_threads)
{
    try {
        if (zi_status st = check_common(t, n_tensors, (int)dt, n_threads)) return st;
        if (!(loss_scale > 0.0f) || std::isinf(loss_scale))
            return fail(ZI_ERR_INVALID_ARG, "loss_scale must be finite and > 0");
        if (!h_out) return fail(ZI_ERR_INVALID_ARG, "h_out is NULL");
        for (int32_t i = 0; i < n_tensors; ++i) {
            if (t[i].numel < 0) return fail(ZI_ERR_INVALID_ARG, "tensor %d: numel < 0", i);
            if (t[i].numel > 0 && !t[i].g) return fail(ZI_ERR_INVALID_ARG, "tensor %d: g is NULL", i);
            if (reinterpret_cast<uintptr_t>(t[i].g) % 2) return fail(ZI_ERR_ALIGNMENT, "tensor %d: g must be 2-byte aligned", i);
        }
        // One partial per block, summed in block order afterwards: the result does not depend on the
        // number of threads.
        struct Block { int32_t tensor; int64_t lo, hi; };
        std::vector<Block> blocks;
        for (int32_t i = 0; i < n_tensors; ++i)
            for (int64_t lo = 0; lo < t[i].numel; lo += kBlockElems)
                blocks.push_back({i, lo, std::min(lo + kBlockElems, t[i].numel)});
        std::vector<double> part(blocks.size(), 0.0);
        std::vector<uint8_t> flag(blocks.size(), 0);
        const uint16_t expmask = dt == ZI_BF16 ? 0x7F80u : 0x7C00u;
        parallel_blocks((int64_t)blocks.size(), n_threads, [&](int64_t b) {
            const Block& B = blocks[(size_t)b];
            const uint16_t* g = (const uint16_t*)t[B.tensor].g;
            __m256d acc0 = _mm256_setzero_pd(), acc1 = _mm256_setzero_pd();
            __m128i bad = _mm_setzero_si128();
            const __m128i em = _mm_set1_epi16((short)expmask);
            int64_t i = B.lo;
            for (; i + 8 <= B.hi; i += 8) {
                const __m128i h = _mm_loadu_si128((const __m128i*)(g + i));
                bad = _mm_or_si128(bad, _mm_cmpeq_epi16(_mm_and_si128(h, em), em));
                const __m256 f = dt == ZI_BF16 ? widen8<ZI_BF16>(g + i) : widen8<ZI_FP16>(g + i);
                const __m256d lo = _mm256_cvtps_pd(_mm256_castps256_ps128(f));
                const __m256d hi = _mm256_cvtps_pd(_mm256_extractf128_ps(f, 1));
                acc0 = _mm256_fmadd_pd(lo, lo, acc0);
                acc1 = _mm256_fmadd_pd(hi, hi, acc1);
            }
            double lanes[4];
            _mm256_storeu_pd(lanes, _mm256_add_pd(acc0, acc1));
            double s = (lanes[0] + lanes[1]) + (lanes[2] + lanes[3]);
            bool f = !_mm_testz_si128(bad, bad);
            for (; i < B.hi; ++i) {
                if ((g[i] & expmask) == expmask) f = true;
                const double x = (double)widen_scalar(g[i], (int)dt);
                s = std::fma(x, x, s);
            }
            part[(size_t)b] = s;
            flag[(size_t)b] = f;
        });
        double sum = 0.0;
        uint32_t found = 0;
        for (size_t b = 0; b < blocks.size(); ++b) {
            sum += part[b];
            found |= flag[b];
        }
        h_out->sumsq = sum;
        h_out->norm = std::sqrt(sum) / (double)loss_scale;
        h_out->found_inf = found ? 1u : 0u;
        h_out->reserved = 0;
        return ZI_OK;
    } catch (const std::exception& ex) {
        return fail(ZI_ERR_NOMEM, "host step: %s", ex.what());
    }
}

extern "C" zi_status zi_host_adamw_step(const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt,
                                        const zi_adamw_config* cfg, const zi_norm_result* h_norm,
                                        int32_t n_threads)
{
    try {
        if (zi_status st = check_common(t, n_tensors, (int)dt, n_threads)) return st;
        if (!cfg) return fail(ZI_ERR_INVALID_ARG, "cfg is NULL");
        if (cfg->step < 1) return fail(ZI_ERR_INVALID_ARG, "step must be >= 1");
        if (!(cfg->beta1 >= 0.0f && cfg->beta1 < 1.0f) || !(cfg->beta2 >= 0.0f && cfg->beta2 < 1.0f))
            return fail(ZI_ERR_INVALID_ARG, "betas must be in [0,1)");
        if (!(cfg->eps >= 0.0f) || std::isinf(cfg->eps)) return fail(ZI_ERR_INVALID_ARG, "eps must be finite and >= 0");
        if (!std::isfinite(cfg->lr) || !std::isfinite(cfg->weight_decay))
            return fail(ZI_ERR_INVALID_ARG, "lr and weight_decay must be finite");
        if (!(cfg->loss_scale > 0.0f) || std::isinf(cfg->loss_scale))
            return fail(ZI_ERR_INVALID_ARG, "loss_scale must be finite and > 0");
        if (std::isnan(cfg->max_grad_norm)) return fail(ZI_ERR_INVALID_ARG, "max_grad_norm is NaN");
        if (cfg->mode != ZI_MODE_ADAMW && cfg->mode != ZI_MODE_ADAM_L2) return fail(ZI_ERR_INVALID_ARG, "unknown mode");
        for (int32_t i = 0; i < n_tensors; ++i) {
            if (t[i].numel < 0) return fail(ZI_ERR_INVALID_ARG, "tensor %d: numel < 0", i);
            if (t[i].numel == 0) continue;
            if (!t[i].p || !t[i].m || !t[i].v || !t[i].g)
                return fail(ZI_ERR_INVALID_ARG, "tensor %d: p, m, v and g must not be NULL", i);
            if (reinterpret_cast<uintptr_t>(t[i].p) % 4 || reinterpret_cast<uintptr_t>(t[i].m) % 4 ||
                reinterpret_cast<uintptr_t>(t[i].v) % 4)
                return fail(ZI_ERR_ALIGNMENT, "tensor %d: p, m, v must be 4-byte aligned", i);
            if (reinterpret_cast<uintptr_t>(t[i].g) % 2 || reinterpret_cast<uintptr_t>(t[i].p_lp) % 2)
                return fail(ZI_ERR_ALIGNMENT, "tensor %d: g and p_lp must be 2-byte aligned", i);
        }
        if (h_norm && h_norm->found_inf) return ZI_SKIPPED_OVERFLOW;

        // per-step scalars: double, each rounded once to fp32 (same expressions as the GPU path's host side)
        Consts c{};
        const double b1 = (double)cfg->beta1, b2 = (double)cfg->beta2;
        const double bc1 = 1.0 - std::pow(b1, (double)cfg->step);
        const double bc2 = 1.0 - std::pow(b2, (double)cfg->step);
        c.beta1 = cfg->beta1;
        c.beta2 = cfg->beta2;
        c.omb1 = (float)(1.0 - b1);
        c.omb2 = (float)(1.0 - b2);
        c.eps = cfg->eps;
        c.step_size = (float)((double)cfg->lr / bc1);
        c.inv_sqrt_bc2 = (float)(1.0 / std::sqrt(bc2));
        c.l2 = cfg->mode == ZI_MODE_ADAM_L2;
        c.decay = c.l2 ? 0.0f : (float)((double)cfg->lr * (double)cfg->weight_decay);
        c.weight_decay = cfg->weight_decay;
        double clip = 1.0;
        if (h_norm) {
            const double mx = (double)cfg->max_grad_norm;
            if (cfg->max_grad_norm > 0.0f && h_norm->norm + 1e-6 > mx) clip = mx / (h_norm->norm + 1e-6);
        }
        c.gscale = (float)(clip / (double)cfg->loss_scale);

        struct Block { int32_t tensor; int64_t lo, hi; };
        std::vector<Block> blocks;
        for (int32_t i = 0; i < n_tensors; ++i)
            for (int64_t lo = 0; lo < t[i].numel; lo += kBlockElems)
                blocks.push_back({i, lo, std::min(lo + kBlockElems, t[i].numel)});
        parallel_blocks((int64_t)blocks.size(), n_threads, [&](int64_t b) {
            const Block& B = blocks[(size_t)b];
            const zi_tensor& T = t[B.tensor];
            float *p = (float*)T.p, *m = (float*)T.m, *v = (float*)T.v;
            const uint16_t* g = (const uint16_t*)T.g;
            uint16_t* lp = (uint16_t*)T.p_lp;
            if (dt == ZI_BF16) {
                if (c.l2) step_range<ZI_BF16, true>(p, m, v, g, lp, B.lo, B.hi, c);
                else      step_range<ZI_BF16, false>(p, m, v, g, lp, B.lo, B.hi, c);
            } else {
                if (c.l2) step_range<ZI_FP16, true>(p, m, v, g, lp, B.lo, B.hi, c);
                else      step_range<ZI_FP16, false>(p, m, v, g, lp, B.lo, B.hi, c);
            }
        });
        return ZI_OK;
    } catch (const std::exception& ex) {
        return fail(ZI_ERR_NOMEM, "host step: %s", ex.what());
    }
}
