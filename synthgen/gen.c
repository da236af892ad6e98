/* Seeded synthetic-input generators shared by the CPU oracle's tests and the GPU
 * library's tests and benchmark.  This file holds no arithmetic of the decoding
 * method: it only produces token ids and weight values from (seed, stream, index)
 * with integer hashing, so any consumer gets bit-identical inputs.
 *
 * Counter-based: value i of stream s under a seed never depends on any other value.
 *   base   = mix64(seed ^ stream * 0xD6E8FEB86659FD93)
 *   h(i,r) = mix64(base + 2*i + r)                 (mix64 = the splitmix64 output function)
 * Token ids:  h(i,0) mod vocab.
 * "Normal" weights: the eight 16-bit lanes of h(i,0), h(i,1) are summed and centred
 * (an Irwin-Hall sum: bell-shaped, support clipped at about +-4.9 sigma), converted to
 * fp32 exactly (|sum| < 2^19) and multiplied once by an fp32 scale = std / sigma_sum.
 * Optionally the result is rounded to the nearest bf16 (ties to even).
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>

static inline uint64_t mix64(uint64_t x) {
    x += 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}

static inline uint64_t stream_base(uint64_t seed, uint64_t stream) {
    return mix64(seed ^ (stream * 0xD6E8FEB86659FD93ull));
}

static inline int32_t lane_sum(uint64_t h) {
    return (int32_t)(h & 0xFFFF) + (int32_t)((h >> 16) & 0xFFFF) +
           (int32_t)((h >> 32) & 0xFFFF) + (int32_t)(h >> 48);
}

static inline float normal_at(uint64_t base, uint64_t i, float scale) {
    int32_t s = lane_sum(mix64(base + 2 * i)) + lane_sum(mix64(base + 2 * i + 1)) - 262140;
    return (float)s * scale;
}

static inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);      /* finite inputs only */
    return (uint16_t)(u >> 16);
}

/* standard deviation of the centred 8-lane sum: sqrt(8 * (2^32 - 1) / 12) */
double synth_sigma_sum(void) { return 53509.920855032404; }

void synth_tokens(int32_t* dst, size_t count, uint64_t seed, uint64_t stream, int32_t vocab) {
    const uint64_t base = stream_base(seed, stream);
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < count; ++i)
        dst[i] = (int32_t)(mix64(base + 2 * (uint64_t)i) % (uint64_t)vocab);
}

/* fp32 output; if round_bf16 != 0 every value is exactly representable in bf16 */
void synth_normal_f32(float* dst, size_t count, uint64_t seed, uint64_t stream, float scale,
                      int round_bf16) {
    const uint64_t base = stream_base(seed, stream);
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < count; ++i) {
        float v = normal_at(base, (uint64_t)i, scale);
        if (round_bf16) {
            uint32_t u = (uint32_t)f32_to_bf16_rne(v) << 16;
            memcpy(&v, &u, 4);
        }
        dst[i] = v;
    }
}

/* bf16 bit patterns (uint16) of the same values synth_normal_f32(..., round_bf16=1) gives */
void synth_normal_bf16(uint16_t* dst, size_t count, uint64_t seed, uint64_t stream, float scale) {
    const uint64_t base = stream_base(seed, stream);
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < count; ++i)
        dst[i] = f32_to_bf16_rne(normal_at(base, (uint64_t)i, scale));
}
