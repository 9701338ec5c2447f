/*
 * zi_oracle.h — interface of the CPU reference (test infrastructure only).
 * Deliberately separate from the product's header: the two share nothing.
 */
#ifndef ZI_ORACLE_H
#define ZI_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ZIO_BF16 = 0, ZIO_FP16 = 1 };
enum { ZIO_MODE_ADAMW = 0, ZIO_MODE_ADAM_L2 = 1 };

typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    int64_t step;          /* 1-based index of the step being taken */
    float loss_scale;      /* 1 = none; raw gradients are divided by it */
    float max_grad_norm;   /* <= 0: no clipping */
    int32_t mode;
} zio_config;

typedef struct {
    double bc1, bc2, norm, clip;
    float omb1, omb2, step_size, inv_sqrt_bc2, decay, gscale;
} zio_scalars_out;

typedef struct {
    double sum, comp;
    uint32_t found_inf;
} zio_sumsq_state;

float zio_bf16_to_f32(uint16_t h);
float zio_f16_to_f32(uint16_t h);
uint16_t zio_f32_to_bf16(float x);
uint16_t zio_f32_to_f16(float x);
void zio_cast_array(const float* x, uint16_t* out, int64_t n, int dtype);
void zio_widen_array(const uint16_t* x, float* out, int64_t n, int dtype);

void zio_sumsq_init(zio_sumsq_state* st);
void zio_sumsq_accumulate(zio_sumsq_state* st, const uint16_t* g, int64_t n, int dtype);
double zio_sumsq_value(const zio_sumsq_state* st);

int zio_scalars(const zio_config* c, int have_norm, double sumsq, zio_scalars_out* o);

/* returns 0 = updated, 1 = skipped (found_inf), -1 = bad argument */
int zio_adamw(float* p, float* m, float* v, const uint16_t* g, uint16_t* p_lp, int64_t n, int dtype,
              const zio_config* c, int have_norm, double sumsq, int found_inf);

int zio_cpu_ok(void);

#ifdef __cplusplus
}
#endif
#endif
