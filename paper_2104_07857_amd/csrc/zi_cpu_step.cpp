// The optimizer step on the host CPUs, for state that lives in host memory.
//
// This is the paper's own placement of the offloaded step (Section 5.2.2: with optimizer states in CPU
// memory the step uses the aggregate CPU compute and memory bandwidth; only gradients come down and the
// low-precision parameters go up over the link, 2 + 2 bytes per element instead of 12 + 12).  It is a
// separate entry point that a caller chooses explicitly; no GPU entry point ever falls back to it.
//
// Same arithmetic, in the same binary32 order, as the HIP kernels (see include/zi.h).  There is ONE
// arithmetic routine: eight lanes of AVX2 / FMA / F16C (vector sqrt and divide are IEEE-correct,
// fmadd / fnmadd round once, the default MXCSR keeps denormals).  A range that is not a multiple of
// eight ends in one more pass of the same routine over a padded group: the fp32 arrays are read and
// written through lane masks, the 2-byte arrays through an 8-element stack copy, so no element is
// ever computed by different code than its neighbours.  Compiled by the host compiler with
// -ffp-contract=off.
#include <immintrin.h>

#include <algorithm>
#include <atomic>
#include <cstring>
#include <exception>
#include <thread>
#include <vector>

#include "zi_checks.h"

using namespace zi::host;

namespace {

// ------------------------------------------------------------------------------- 16-bit formats

template <int DT>
inline __m256 widen8(__m128i h)
{
    if (DT == ZI_BF16) return _mm256_castsi256_ps(_mm256_slli_epi32(_mm256_cvtepu16_epi32(h), 16));
    return _mm256_cvtph_ps(h);
}

// Eight fp32 values to eight 16-bit patterns, round to nearest even.
template <int DT>
inline __m128i narrow8(__m256 x)
{
    if (DT == ZI_FP16) return _mm256_cvtps_ph(x, _MM_FROUND_TO_NEAREST_INT | _MM_FROUND_NO_EXC);
    // bf16 keeps the upper half of the fp32 pattern.  The dropped half decides: above one half of the
    // kept unit the upper half goes up by one, exactly one half goes to the even neighbour, below
    // stays.  (Signed compares are fine: the dropped half is at most 0xFFFF.)  A NaN keeps its upper
    // half with the quiet bit set, so it can neither become an infinity nor carry into the sign.
    const __m256i bits = _mm256_castps_si256(x);
    const __m256i upper = _mm256_srli_epi32(bits, 16);
    const __m256i dropped = _mm256_and_si256(bits, _mm256_set1_epi32(0xFFFF));
    const __m256i half = _mm256_set1_epi32(0x8000);
    const __m256i above = _mm256_cmpgt_epi32(dropped, half);
    const __m256i tie = _mm256_cmpeq_epi32(dropped, half);
    const __m256i odd = _mm256_cmpeq_epi32(_mm256_and_si256(upper, _mm256_set1_epi32(1)), _mm256_set1_epi32(1));
    const __m256i up = _mm256_or_si256(above, _mm256_and_si256(tie, odd));           // all ones where rounding up
    const __m256i rounded = _mm256_sub_epi32(upper, up);                               // minus (-1) = plus one
    const __m256i nan = _mm256_castps_si256(_mm256_cmp_ps(x, x, _CMP_UNORD_Q));
    const __m256i quiet = _mm256_or_si256(upper, _mm256_set1_epi32(0x0040));
    const __m256i r = _mm256_blendv_epi8(rounded, quiet, nan);
    const __m256i packed = _mm256_packus_epi32(r, r);                                  // per 128-bit half
    return _mm256_castsi256_si128(_mm256_permute4x64_epi64(packed, 0x08));            // halves 0 and 2
}

// Lane mask with the first k of eight lanes set (k in 0..8).
inline __m256i first_lanes(int k)
{
    alignas(32) static const int32_t ramp[8] = {0, 1, 2, 3, 4, 5, 6, 7};
    return _mm256_cmpgt_epi32(_mm256_set1_epi32(k), _mm256_load_si256((const __m256i*)ramp));
}

// ------------------------------------------------------------------------------------ the update

template <int DT, bool L2>
struct Updater {
    __m256 beta1, beta2, omb1, omb2, eps, step_size, inv_sqrt_bc2, decay, wd, gscale;

    Updater(const zi::StepConsts& c, float gs)
        : beta1(_mm256_set1_ps(c.beta1)), beta2(_mm256_set1_ps(c.beta2)), omb1(_mm256_set1_ps(c.omb1)),
          omb2(_mm256_set1_ps(c.omb2)), eps(_mm256_set1_ps(c.eps)), step_size(_mm256_set1_ps(c.step_size)),
          inv_sqrt_bc2(_mm256_set1_ps(c.inv_sqrt_bc2)), decay(_mm256_set1_ps(c.decay)),
          wd(_mm256_set1_ps(c.weight_decay)), gscale(_mm256_set1_ps(gs))
    {
    }

    // Eight elements: state in, state out (in place in the arguments), low-precision copy returned.
    inline __m128i eight(__m256& p, __m256& m, __m256& v, __m128i g16) const
    {
        __m256 g = _mm256_mul_ps(widen8<DT>(g16), gscale);
        if (L2) g = _mm256_fmadd_ps(wd, p, g);
        m = _mm256_fmadd_ps(beta1, m, _mm256_mul_ps(omb1, g));
        v = _mm256_fmadd_ps(beta2, v, _mm256_mul_ps(omb2, _mm256_mul_ps(g, g)));
        const __m256 denom = _mm256_fmadd_ps(_mm256_sqrt_ps(v), inv_sqrt_bc2, eps);
        const __m256 ratio = _mm256_div_ps(m, denom);
        p = _mm256_fnmadd_ps(step_size, ratio, _mm256_fnmadd_ps(decay, p, p));
        return narrow8<DT>(p);
    }

    // Elements [lo, hi) of one tensor.
    void range(float* p, float* m, float* v, const uint16_t* g, uint16_t* lp, int64_t lo, int64_t hi) const
    {
        int64_t i = lo;
        for (; i + 8 <= hi; i += 8) {
            __m256 pi = _mm256_loadu_ps(p + i), mi = _mm256_loadu_ps(m + i), vi = _mm256_loadu_ps(v + i);
            const __m128i out = eight(pi, mi, vi, _mm_loadu_si128((const __m128i*)(g + i)));
            _mm256_storeu_ps(p + i, pi);
            _mm256_storeu_ps(m + i, mi);
            _mm256_storeu_ps(v + i, vi);
            if (lp) _mm_storeu_si128((__m128i*)(lp + i), out);
        }
        const int k = (int)(hi - i);
        if (k > 0) {
            // The same routine over a padded group: lanes beyond k hold zeros and are never stored.
            const __m256i mask = first_lanes(k);
            __m256 pi = _mm256_maskload_ps(p + i, mask), mi = _mm256_maskload_ps(m + i, mask),
                   vi = _mm256_maskload_ps(v + i, mask);
            alignas(16) uint16_t g8[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            std::memcpy(g8, g + i, (size_t)k * 2);
            const __m128i out = eight(pi, mi, vi, _mm_load_si128((const __m128i*)g8));
            _mm256_maskstore_ps(p + i, mask, pi);
            _mm256_maskstore_ps(m + i, mask, mi);
            _mm256_maskstore_ps(v + i, mask, vi);
            if (lp) {
                alignas(16) uint16_t o8[8];
                _mm_store_si128((__m128i*)o8, out);
                std::memcpy(lp + i, o8, (size_t)k * 2);
            }
        }
    }
};

// Sum of squares (in double) and non-finite test of elements [lo, hi); a short end goes through the
// same eight-lane code on a zero-padded copy (zeros add nothing and are finite).
template <int DT>
void sumsq_range(const uint16_t* g, int64_t lo, int64_t hi, double& sum_out, bool& bad_out)
{
    const __m128i expmask = _mm_set1_epi16((short)(DT == ZI_BF16 ? 0x7F80 : 0x7C00));
    __m256d acc_lo = _mm256_setzero_pd(), acc_hi = _mm256_setzero_pd();
    __m128i bad = _mm_setzero_si128();
    auto eight = [&](__m128i h) {
        bad = _mm_or_si128(bad, _mm_cmpeq_epi16(_mm_and_si128(h, expmask), expmask));
        const __m256 f = widen8<DT>(h);
        const __m256d a = _mm256_cvtps_pd(_mm256_castps256_ps128(f));
        const __m256d b = _mm256_cvtps_pd(_mm256_extractf128_ps(f, 1));
        acc_lo = _mm256_fmadd_pd(a, a, acc_lo);
        acc_hi = _mm256_fmadd_pd(b, b, acc_hi);
    };
    int64_t i = lo;
    for (; i + 8 <= hi; i += 8) eight(_mm_loadu_si128((const __m128i*)(g + i)));
    if (i < hi) {
        alignas(16) uint16_t g8[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        std::memcpy(g8, g + i, (size_t)(hi - i) * 2);
        eight(_mm_load_si128((const __m128i*)g8));
    }
    alignas(32) double lanes[4];
    _mm256_store_pd(lanes, _mm256_add_pd(acc_lo, acc_hi));
    sum_out = (lanes[0] + lanes[1]) + (lanes[2] + lanes[3]);
    bad_out = !_mm_testz_si128(bad, bad);
}

// ------------------------------------------------------------------------------------ threading

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

struct Block {
    int32_t tensor;
    int64_t lo, hi;
};

std::vector<Block> blocks_of(const zi_tensor* t, int32_t n_tensors)
{
    std::vector<Block> blocks;
    for (int32_t i = 0; i < n_tensors; ++i)
        for (int64_t lo = 0; lo < t[i].numel; lo += kBlockElems)
            blocks.push_back({i, lo, std::min(lo + kBlockElems, t[i].numel)});
    return blocks;
}

zi_status check_cpu_and_threads(int32_t n_threads)
{
    if (!host_step_supported())
        return fail(ZI_ERR_UNSUPPORTED, "the host step needs a CPU with AVX2, FMA and F16C");
    if (n_threads < 1 || n_threads > 256) return fail(ZI_ERR_INVALID_ARG, "n_threads must be in 1..256");
    return ZI_OK;
}

}  // namespace

namespace zi {
namespace host {

bool host_step_supported()
{
    return __builtin_cpu_supports("avx2") && __builtin_cpu_supports("fma") && __builtin_cpu_supports("f16c");
}

void host_step_range(const zi::StepConsts& c, float gscale, int dt, bool l2, float* p, float* m, float* v,
                     const uint16_t* g, uint16_t* lp, int64_t lo, int64_t hi)
{
    if (dt == ZI_BF16) {
        if (l2) Updater<ZI_BF16, true>(c, gscale).range(p, m, v, g, lp, lo, hi);
        else    Updater<ZI_BF16, false>(c, gscale).range(p, m, v, g, lp, lo, hi);
    } else {
        if (l2) Updater<ZI_FP16, true>(c, gscale).range(p, m, v, g, lp, lo, hi);
        else    Updater<ZI_FP16, false>(c, gscale).range(p, m, v, g, lp, lo, hi);
    }
}

}  // namespace host
}  // namespace zi

extern "C" zi_status zi_host_grad_norm(const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt, float loss_scale,
                                       zi_norm_result* h_out, int32_t n_threads)
{
    try {
        if (zi_status st = check_cpu_and_threads(n_threads)) return st;
        if (zi_status st = check_dtype((int)dt)) return st;
        if (zi_status st = check_grad_list(t, n_tensors, loss_scale)) return st;
        if (!h_out) return fail(ZI_ERR_INVALID_ARG, "h_out is NULL");
        // One partial per block, summed in block order afterwards: the result does not depend on the
        // number of threads.
        const std::vector<Block> blocks = blocks_of(t, n_tensors);
        std::vector<double> part(blocks.size(), 0.0);
        std::vector<uint8_t> flag(blocks.size(), 0);
        parallel_blocks((int64_t)blocks.size(), n_threads, [&](int64_t b) {
            const Block& B = blocks[(size_t)b];
            const uint16_t* g = (const uint16_t*)t[B.tensor].g;
            bool bad = false;
            if (dt == ZI_BF16) sumsq_range<ZI_BF16>(g, B.lo, B.hi, part[(size_t)b], bad);
            else               sumsq_range<ZI_FP16>(g, B.lo, B.hi, part[(size_t)b], bad);
            flag[(size_t)b] = bad;
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
        uint32_t bits;
        std::memcpy(&bits, &loss_scale, sizeof bits);
        h_out->scale_bits = bits;
        h_out->inv_norm = 1.0 / (h_out->norm + 1e-6);
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
        if (zi_status st = check_cpu_and_threads(n_threads)) return st;
        if (zi_status st = check_dtype((int)dt)) return st;
        if (zi_status st = check_config(cfg)) return st;
        if (zi_status st = check_step_tensors(t, n_tensors)) return st;
        if (h_norm && h_norm->found_inf) return ZI_SKIPPED_OVERFLOW;

        const zi::StepConsts c = make_consts(*cfg);
        const float gs = h_norm ? gradient_factor(h_norm->sumsq, c) : c.host_gscale;
        const bool l2 = cfg->mode == ZI_MODE_ADAM_L2;
        const std::vector<Block> blocks = blocks_of(t, n_tensors);
        parallel_blocks((int64_t)blocks.size(), n_threads, [&](int64_t b) {
            const Block& B = blocks[(size_t)b];
            const zi_tensor& T = t[B.tensor];
            host_step_range(c, gs, (int)dt, l2, (float*)T.p, (float*)T.m, (float*)T.v, (const uint16_t*)T.g,
                            (uint16_t*)T.p_lp, B.lo, B.hi);
        });
        return ZI_OK;
    } catch (const std::exception& ex) {
        return fail(ZI_ERR_NOMEM, "host step: %s", ex.what());
    }
}
