/* Seeded, counter-based input generators shared by the CPU oracle's tests and the
 * GPU path's tests/bench.  This file holds NO arithmetic of the decoding method:
 * only pseudo-random numbers (token ids, Gaussian weights, Gaussian KV fill).
 *
 * Generator: element i of stream s under seed z is a pure function of (z, s, i):
 *   key  = mix64(z ^ mix64(s + 0x632BE59BD9B4E019))
 *   word = mix64(key + (i+1) * 0x9E3779B97F4A7C15)          (splitmix64 finaliser)
 * Gaussians use Box-Muller on the pair index p = i/2 with
 *   u1 = (hi32(word)+1) / 2^32  in (0,1],  u2 = lo32(word) / 2^32 in [0,1)
 *   z0 = sqrt(-2 ln u1) cos(2 pi u2)   (element 2p)
 *   z1 = sqrt(-2 ln u1) sin(2 pi u2)   (element 2p+1)
 * evaluated in double, scaled by sigma, rounded to float, and (for bf16 outputs)
 * rounded once more to bfloat16 with round-to-nearest-even.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

static inline uint64_t mix64(uint64_t x) {
    x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27; x *= 0x94D049BB133111EBull;
    x ^= x >> 31; return x;
}
static inline uint64_t stream_key(uint64_t seed, uint64_t stream) {
    return mix64(seed ^ mix64(stream + 0x632BE59BD9B4E019ull));
}
static inline uint64_t word_at(uint64_t key, uint64_t i) {
    return mix64(key + (i + 1) * 0x9E3779B97F4A7C15ull);
}
static inline void gauss_pair(uint64_t key, uint64_t p, double *z0, double *z1) {
    uint64_t w = word_at(key, p);
    double u1 = ((double)(uint32_t)(w >> 32) + 1.0) * (1.0 / 4294967296.0);
    double u2 = (double)(uint32_t)(w & 0xFFFFFFFFu) * (1.0 / 4294967296.0);
    double r = sqrt(-2.0 * log(u1));
    double a = 6.283185307179586476925286766559 * u2;
    *z0 = r * cos(a);
    *z1 = r * sin(a);
}
static inline uint16_t f32_to_bf16_rne(float f) {
    union { float f; uint32_t u; } v; v.f = f;
    uint32_t u = v.u;
    if ((u & 0x7F800000u) == 0x7F800000u) return (uint16_t)(u >> 16); /* inf/nan: truncate */
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* out[i] = float(sigma * z_i), i in [0,n) */
void synth_normal_f32(uint64_t seed, uint64_t stream, double sigma, float *out, size_t n) {
    uint64_t key = stream_key(seed, stream);
    size_t pairs = (n + 1) / 2;
    #pragma omp parallel for schedule(static)
    for (size_t p = 0; p < pairs; ++p) {
        double z0, z1; gauss_pair(key, p, &z0, &z1);
        out[2 * p] = (float)(sigma * z0);
        if (2 * p + 1 < n) out[2 * p + 1] = (float)(sigma * z1);
    }
}
/* out[i] = bf16(float(sigma * z_i)) as raw 16-bit patterns */
void synth_normal_bf16(uint64_t seed, uint64_t stream, double sigma, uint16_t *out, size_t n) {
    uint64_t key = stream_key(seed, stream);
    size_t pairs = (n + 1) / 2;
    #pragma omp parallel for schedule(static)
    for (size_t p = 0; p < pairs; ++p) {
        double z0, z1; gauss_pair(key, p, &z0, &z1);
        out[2 * p] = f32_to_bf16_rne((float)(sigma * z0));
        if (2 * p + 1 < n) out[2 * p + 1] = f32_to_bf16_rne((float)(sigma * z1));
    }
}
/* out[i] uniform on [0, bound): high 32 bits of the word, multiply-shift */
void synth_uniform_i32(uint64_t seed, uint64_t stream, int32_t bound, int32_t *out, size_t n) {
    uint64_t key = stream_key(seed, stream);
    #pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        uint64_t w = word_at(key, i);
        out[i] = (int32_t)(((w >> 32) * (uint64_t)(uint32_t)bound) >> 32);
    }
}
/* out[i] uniform double on [0,1) with 53 bits */
void synth_uniform_f64(uint64_t seed, uint64_t stream, double *out, size_t n) {
    uint64_t key = stream_key(seed, stream);
    for (size_t i = 0; i < n; ++i)
        out[i] = (double)(word_at(key, i) >> 11) * (1.0 / 9007199254740992.0);
}
