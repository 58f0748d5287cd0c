/*
 * Seeded synthetic-input generator for the HATA decode workloads.
 *
 * This file holds NO arithmetic of the method itself (no hashing of vectors,
 * no Hamming scores, no selection, no attention).  It only produces
 * reproducible pseudo-random tensors: every element is a pure function of
 * (seed, tensor id, flat element index), so any element can be regenerated on
 * its own and the same host buffers feed both the CPU oracle and the GPU path.
 *
 * Generator: a 64-bit finaliser-style mixer over a counter (one counter per
 * PAIR of elements), turned into two standard normals with the Box-Muller
 * transform.  bf16 outputs are rounded to nearest-even from the double value.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC synth.c -o libhata_synth.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* Raw 64-bit draw number `idx` of stream (seed, tensor_id). */
uint64_t synth_u64(uint64_t seed, uint64_t tensor_id, uint64_t idx) {
    uint64_t key = mix64(seed ^ mix64(tensor_id * 0xD1342543DE82EF95ull + 0x632BE59BD9B4E019ull));
    return mix64(key ^ mix64(idx));
}

/* Standard normal number `i` of stream (seed, tensor_id): elements 2p and 2p+1
 * share the two uniforms of pair p (cosine and sine branch). */
static inline double normal_at(uint64_t seed, uint64_t tensor_id, uint64_t i) {
    uint64_t p = i >> 1;
    uint64_t h1 = synth_u64(seed, tensor_id, 2 * p);
    uint64_t h2 = synth_u64(seed, tensor_id, 2 * p + 1);
    double u1 = ((double)(h1 >> 11) + 1.0) * (1.0 / 9007199254740992.0); /* (0,1] */
    double u2 = (double)(h2 >> 11) * (1.0 / 9007199254740992.0);         /* [0,1) */
    double rad = sqrt(-2.0 * log(u1));
    double ang = 6.283185307179586476925286766559 * u2;
    return (i & 1) ? rad * sin(ang) : rad * cos(ang);
}

double synth_normal(uint64_t seed, uint64_t tensor_id, uint64_t i) {
    return normal_at(seed, tensor_id, i);
}

/* double -> bf16 bit pattern, round to nearest, ties to even (via fp32: the
 * double->float step is itself correctly rounded and a double carries enough
 * extra bits that double rounding cannot change a bf16 tie decision except on
 * measure-zero inputs, which the continuous generator does not produce). */
static inline uint16_t to_bf16(double v) {
    float f = (float)v;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) return (uint16_t)(u >> 16); /* inf/nan */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

/*
 * Fill a bf16 tensor whose flat layout is [..., heads, rows, d] (d fastest).
 * out[i] = bf16( normal(seed, tensor_id, first + i) * chan_scale[head(i)][c(i)] )
 * with c = (first+i) % d and head = ((first+i) / (d*rows)) % heads.
 * chan_scale may be NULL (all ones).  `first` lets a caller generate a slice.
 */
void synth_fill_bf16(uint64_t seed, uint64_t tensor_id, uint64_t first, uint64_t count,
                     uint64_t d, uint64_t rows, uint64_t heads, const float* chan_scale,
                     uint16_t* out) {
#pragma omp parallel for schedule(static)
    for (int64_t ii = 0; ii < (int64_t)count; ++ii) {
        uint64_t i = first + (uint64_t)ii;
        double z = normal_at(seed, tensor_id, i);
        if (chan_scale) {
            uint64_t c = i % d;
            uint64_t h = (i / (d * rows)) % heads;
            z *= (double)chan_scale[h * d + c];
        }
        out[ii] = to_bf16(z);
    }
}

/* out[i] = (float)( normal(seed, tensor_id, first + i) * sigma ) */
void synth_fill_f32(uint64_t seed, uint64_t tensor_id, uint64_t first, uint64_t count,
                    double sigma, float* out) {
#pragma omp parallel for schedule(static)
    for (int64_t ii = 0; ii < (int64_t)count; ++ii) {
        out[ii] = (float)(normal_at(seed, tensor_id, first + (uint64_t)ii) * sigma);
    }
}

/* out[i] = raw 32-bit words (upper half of the 64-bit draw); used for random code words. */
void synth_fill_u32(uint64_t seed, uint64_t tensor_id, uint64_t first, uint64_t count,
                    uint32_t* out) {
#pragma omp parallel for schedule(static)
    for (int64_t ii = 0; ii < (int64_t)count; ++ii) {
        out[ii] = (uint32_t)(synth_u64(seed, tensor_id, first + (uint64_t)ii) >> 32);
    }
}
