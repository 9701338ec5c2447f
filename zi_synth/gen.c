/*
 * zi_synth — seeded, counter-based generators for synthetic optimizer state.
 *
 * This module holds NONE of the optimizer's arithmetic.  It only produces
 * inputs: normally distributed fp32 arrays (master parameters, first and
 * second moments) and low-precision gradient arrays, shaped like the model
 * states of mixed-precision Adam training (Section 3, "Memory for Model
 * States": fp16 parameters/gradients, fp32 momentum, variance, parameters).
 *
 * Every value is a pure function of (seed, stream, tensor, element index), so
 * any sub-range of a very large array can be regenerated on demand and filled
 * by many threads at once.
 *
 *   pair j = index >> 1 draws two 64-bit hashes -> two uniforms -> one
 *   Box-Muller pair (cos branch for even indices, sin branch for odd ones).
 *
 * Low-precision gradients are quantised by the generator's own rule, which is
 * deliberately not the optimizer's rounding rule:
 *   bf16: keep the upper 16 bits of the fp32 pattern (truncation);
 *   fp16: the CPU's hardware converter (F16C, round to nearest even).
 */
#define _GNU_SOURCE
#include <immintrin.h>
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ZS_BF16 0
#define ZS_FP16 1

static inline uint64_t zs_mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* Key of one (seed, stream, tensor) triple. */
uint64_t zs_key(uint64_t seed, uint32_t stream, uint32_t tensor)
{
    uint64_t k = zs_mix64(seed);
    k = zs_mix64(k ^ ((uint64_t)stream << 32 | (uint64_t)tensor));
    return k;
}

/* Standard normal deviates for the pair that contains elements 2j and 2j+1. */
static inline void zs_pair(uint64_t key, uint64_t j, double* z0, double* z1)
{
    uint64_t a = zs_mix64(key + 2u * j);
    uint64_t b = zs_mix64(key + 2u * j + 1u);
    double u1 = (double)((a >> 11) + 1u) * 0x1.0p-53; /* (0, 1] */
    double u2 = (double)(b >> 11) * 0x1.0p-53;        /* [0, 1) */
    double r = sqrt(-2.0 * log(u1));
    float s, c;
    sincosf((float)(6.283185307179586476925 * u2), &s, &c);
    *z0 = r * (double)c;
    *z1 = r * (double)s;
}

static inline double zs_normal(uint64_t key, uint64_t index)
{
    double z0, z1;
    zs_pair(key, index >> 1, &z0, &z1);
    return (index & 1u) ? z1 : z0;
}


/* z[0..count) = standard normals for indices first..first+count-1; count <= 4096.
 * Each Box-Muller pair is evaluated once. */
static void zs_block(uint64_t key, uint64_t first, int count, double* z)
{
    int k = 0;
    if (count > 0 && (first & 1u)) {
        z[k++] = zs_normal(key, first);
    }
    for (; k + 1 < count; k += 2) {
        zs_pair(key, (first + (uint64_t)k) >> 1, &z[k], &z[k + 1]);
    }
    if (k < count) {
        z[k] = zs_normal(key, first + (uint64_t)k);
    }
}

/* One standard-normal deviate, for spot checks from Python. */
double zs_normal_at(uint64_t seed, uint32_t stream, uint32_t tensor, uint64_t index)
{
    return zs_normal(zs_key(seed, stream, tensor), index);
}

/* A seeded index in [0, n): used to choose where a test plants a value. */
uint64_t zs_pick_index(uint64_t seed, uint64_t tag, uint64_t n)
{
    if (n == 0) return 0;
    return zs_mix64(zs_mix64(seed) ^ tag) % n;
}

int zs_cpu_ok(void)
{
    return __builtin_cpu_supports("f16c") ? 1 : 0;
}

static int zs_threads(int nthreads, int64_t n)
{
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
    if (n < 65536) nthreads = 1;
    return nthreads;
#else
    (void)nthreads; (void)n;
    return 1;
#endif
}

/*
 * out[i] = (float)(mean + std * z(first_index + i)), optionally |.|.
 * Returns 0, or -1 on a bad argument.
 */
int zs_fill_normal_f32(float* out, int64_t n, uint64_t seed, uint32_t stream, uint32_t tensor,
                       int64_t first_index, double mean, double std, int take_abs, int nthreads)
{
    if (n < 0 || first_index < 0 || (n > 0 && !out)) return -1;
    const uint64_t key = zs_key(seed, stream, tensor);
    const int nt = zs_threads(nthreads, n);
    (void)nt;
#pragma omp parallel for num_threads(nt) schedule(static)
    for (int64_t blk = 0; blk < (n + 4095) / 4096; ++blk) {
        int64_t lo = blk * 4096, hi = lo + 4096 < n ? lo + 4096 : n;
        double z[4096];
        zs_block(key, (uint64_t)(first_index + lo), (int)(hi - lo), z);
        for (int64_t i = lo; i < hi; ++i) {
            float f = (float)(mean + std * z[i - lo]);
            out[i] = take_abs ? fabsf(f) : f;
        }
    }
    return 0;
}

static inline uint16_t zs_quantise(float f, int dtype)
{
    if (dtype == ZS_BF16) {
        uint32_t b;
        memcpy(&b, &f, 4);
        return (uint16_t)(b >> 16);
    }
    return (uint16_t)_cvtss_sh(f, _MM_FROUND_TO_NEAREST_INT | _MM_FROUND_NO_EXC);
}

/*
 * Low-precision gradients: out[i] = quantise((float)(mean + std * z)).
 * dtype: 0 = bf16, 1 = fp16.  Returns 0, or -1 on a bad argument.
 */
int zs_fill_normal_lp(uint16_t* out, int64_t n, uint64_t seed, uint32_t stream, uint32_t tensor,
                      int64_t first_index, double mean, double std, int dtype, int nthreads)
{
    if (n < 0 || first_index < 0 || (n > 0 && !out)) return -1;
    if (dtype != ZS_BF16 && dtype != ZS_FP16) return -1;
    if (dtype == ZS_FP16 && !zs_cpu_ok()) return -2;
    const uint64_t key = zs_key(seed, stream, tensor);
    const int nt = zs_threads(nthreads, n);
    (void)nt;
#pragma omp parallel for num_threads(nt) schedule(static)
    for (int64_t blk = 0; blk < (n + 4095) / 4096; ++blk) {
        int64_t lo = blk * 4096, hi = lo + 4096 < n ? lo + 4096 : n;
        double z[4096];
        zs_block(key, (uint64_t)(first_index + lo), (int)(hi - lo), z);
        for (int64_t i = lo; i < hi; ++i) {
            out[i] = zs_quantise((float)(mean + std * z[i - lo]), dtype);
        }
    }
    return 0;
}
