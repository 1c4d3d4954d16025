/*
 * Seeded synthetic input generator shared by the tests, the benchmark, the CPU
 * oracle's callers and the GPU path's callers.  It holds none of the attention
 * arithmetic: it only turns (seed, stream, element index) into a bf16 bit
 * pattern of an i.i.d. N(0,1) draw.
 *
 * Counter-based: element i of a stream depends on (seed, stream, i) only, so any
 * sub-range can be generated independently and in parallel, and host and device
 * consumers see identical bytes.
 *
 *   h(seed, stream, c, lane) : 64-bit mix (splitmix64 finaliser applied to a
 *                              running combination of the four words)
 *   u1 in (0,1], u2 in [0,1) : top 53 bits of two hashes
 *   z = sqrt(-2 ln u1) * (cos | sin)(2 pi u2)     Box-Muller; element i uses
 *       counter c = i / 2 and the cos branch when i is even, sin when odd
 *   bf16 = round-to-nearest-even of (float) z
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static inline uint64_t mix64(uint64_t x) {
    x += 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}

static inline uint64_t hash4(uint64_t seed, uint64_t stream, uint64_t c, uint64_t lane) {
    uint64_t h = mix64(seed);
    h = mix64(h ^ stream);
    h = mix64(h ^ c);
    return mix64(h ^ lane);
}

static inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u); /* NaN stays NaN */
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* Exported so Python-side tests can check single values. */
double wl_normal_f64(uint64_t seed, uint64_t stream, uint64_t i) {
    const uint64_t c = i >> 1;
    const double u1 = (double)((hash4(seed, stream, c, 0) >> 11) + 1) * 0x1.0p-53; /* (0,1] */
    const double u2 = (double)(hash4(seed, stream, c, 1) >> 11) * 0x1.0p-53;       /* [0,1) */
    const double r = sqrt(-2.0 * log(u1));
    const double a = 6.283185307179586476925286766559 * u2;
    return (i & 1) ? r * sin(a) : r * cos(a);
}

/* out[j] = bf16(N(0,1)) for element index offset + j of (seed, stream), j in [0, n). */
void wl_normal_bf16(uint64_t seed, uint64_t stream, uint64_t offset, uint64_t n, uint16_t* out) {
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < (int64_t)n; ++j)
        out[j] = f32_to_bf16_rne((float)wl_normal_f64(seed, stream, offset + (uint64_t)j));
}

/* Uniform 64-bit words for the length samplers: out[j] = h(seed, stream, offset + j, 2). */
void wl_uniform_u64(uint64_t seed, uint64_t stream, uint64_t offset, uint64_t n, uint64_t* out) {
    for (uint64_t j = 0; j < n; ++j) out[j] = hash4(seed, stream, offset + j, 2);
}
