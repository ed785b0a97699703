/*
 * Seeded, counter-based input generators shared by the CPU oracle's tests and
 * the GPU harness.  This file holds no arithmetic of the verification method:
 * it only turns (seed, stream, index) into reproducible pseudo-random values,
 * so both sides can be fed bit-identical weights, caches and token ids.
 *
 * Every value is a pure function of (seed, stream, index): any sub-range of a
 * tensor can be regenerated on demand, in any order, on any number of threads.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ULL;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebULL;
    return z ^ (z >> 31);
}

static inline uint64_t counter_hash(uint64_t seed, uint64_t stream, uint64_t idx) {
    uint64_t a = mix64(seed + 0x9e3779b97f4a7c15ULL);
    uint64_t b = mix64(a ^ (stream * 0xd1342543de82ef95ULL + 0x632be59bd9b4e019ULL));
    return mix64(b + idx * 0x9e3779b97f4a7c15ULL);
}

/* Standard normal for counter idx.  Indices 2j and 2j+1 share one hash and are
 * the cosine and sine branches of one Box-Muller pair. */
static inline double normal_at(uint64_t seed, uint64_t stream, uint64_t idx) {
    uint64_t h = counter_hash(seed, stream, idx >> 1);
    double u1 = ((double)(h >> 32) + 1.0) * (1.0 / 4294967296.0);        /* (0,1] */
    double u2 = (double)(h & 0xffffffffULL) * (1.0 / 4294967296.0);      /* [0,1) */
    double r = sqrt(-2.0 * log(u1));
    double t = 6.283185307179586476925286766559 * u2;
    return (idx & 1) ? r * sin(t) : r * cos(t);
}

static inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

void synth_normal_f32(uint64_t seed, uint64_t stream, uint64_t offset, uint64_t n,
                      double scale, float *out) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i)
        out[i] = (float)(scale * normal_at(seed, stream, offset + (uint64_t)i));
}

/* Same values as synth_normal_f32, rounded to nearest-even bfloat16 bit patterns. */
void synth_normal_bf16(uint64_t seed, uint64_t stream, uint64_t offset, uint64_t n,
                       double scale, uint16_t *out) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i)
        out[i] = f32_to_bf16_rne((float)(scale * normal_at(seed, stream, offset + (uint64_t)i)));
}

/* Uniform integers in [lo, hi). */
void synth_uniform_i32(uint64_t seed, uint64_t stream, uint64_t offset, uint64_t n,
                       int32_t lo, int32_t hi, int32_t *out) {
    uint64_t span = (uint64_t)((int64_t)hi - (int64_t)lo);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i) {
        uint64_t h = counter_hash(seed, stream, offset + (uint64_t)i);
        out[i] = (int32_t)((int64_t)lo + (int64_t)(((h >> 32) * span) >> 32));
    }
}

/* Uniform doubles in [0, 1). */
void synth_uniform_f64(uint64_t seed, uint64_t stream, uint64_t offset, uint64_t n,
                       double *out) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i) {
        uint64_t h = counter_hash(seed, stream, offset + (uint64_t)i);
        out[i] = (double)(h >> 11) * (1.0 / 9007199254740992.0);
    }
}
