/*
 * Seeded, counter-based synthetic input generator.
 *
 * Every element is a pure function of (seed, tensor_id, linear index), so any
 * slice of any tensor can be regenerated independently and both the CPU oracle
 * and the GPU path are handed byte-identical inputs.  This file holds no
 * attention or layout arithmetic: it only draws numbers.
 *
 *   bits   = mix64(mix64(seed ^ (tensor_id+1)*C) + index)
 *   u1,u2  = upper / lower 32 bits mapped to (0,1] and [0,1)
 *   z      = sqrt(-2 ln u1) * cos(2 pi u2)             (Box-Muller, one branch)
 *   out    = bf16_rne( (float)z * mult )                (mult applied in fp32, then rounded)
 */
#include <math.h>
#include <stdint.h>

static inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static inline uint16_t f32_to_bf16_rne(float f) {
    union { float f; uint32_t u; } v = { f };
    if ((v.u & 0x7F800000u) == 0x7F800000u) {           /* inf / nan: truncate, keep nan a nan */
        uint16_t hi = (uint16_t)(v.u >> 16);
        if ((v.u & 0x007FFFFFu) && !(hi & 0x007F)) hi |= 0x0040;
        return hi;
    }
    uint32_t lsb = (v.u >> 16) & 1u;
    v.u += 0x7FFFu + lsb;
    return (uint16_t)(v.u >> 16);
}

/* out[i] for i in [0, count) is element (start + i) of the tensor. */
void synth_normal_bf16(uint16_t* out, int64_t count, int64_t start,
                       uint64_t seed, uint32_t tensor_id, float mult) {
    const uint64_t key = mix64(seed ^ ((uint64_t)(tensor_id + 1u) * 0xD1B54A32D192ED03ull));
    const double two_pi = 6.283185307179586476925286766559;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        uint64_t bits = mix64(key + (uint64_t)(start + i));
        double u1 = ((double)(uint32_t)(bits >> 32) + 1.0) * (1.0 / 4294967296.0);
        double u2 = (double)(uint32_t)(bits & 0xFFFFFFFFu) * (1.0 / 4294967296.0);
        double z = sqrt(-2.0 * log(u1)) * cos(two_pi * u2);
        out[i] = f32_to_bf16_rne((float)z * mult);
    }
}

/* Uniform 16-bit payloads (for the bit-exact layout kernels: every bit pattern is legal). */
void synth_bits_u16(uint16_t* out, int64_t count, int64_t start, uint64_t seed, uint32_t tensor_id) {
    const uint64_t key = mix64(seed ^ ((uint64_t)(tensor_id + 1u) * 0xD1B54A32D192ED03ull));
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i)
        out[i] = (uint16_t)(mix64(key + (uint64_t)(start + i)) >> 24);
}
