/*
 * Seeded synthetic-input generator (weights, per-sublayer output scales, prompts).
 *
 * This file holds no arithmetic of the decoding method.  It only defines a
 * counter-based stream of numbers so that any element of any tensor can be
 * produced anywhere (host or device) from (seed, tensor id, layer, element index):
 *
 *   stream = mix64(mix64(seed + GOLD) ^ (tensor << 32 | layer))
 *   draw(c) = mix64(stream + (c + 1) * GOLD)          (splitmix64 finaliser)
 *   element i uses draws 2i and 2i+1; the sum S of their eight 16-bit fields is
 *   an Irwin-Hall variable with mean 262140 and sigma 65536*sqrt(8/12);
 *   value = float(S - 262140) * cst, one fp32 multiply, then (for bf16 storage)
 *   one round-to-nearest-even to bf16.  Only integer ops and a single exact
 *   IEEE multiply are involved, so every platform yields the same bits.
 *
 * The distribution is a central-limit approximation of N(0, std^2) truncated
 * near +-4.9 sigma.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

#define GOLD 0x9E3779B97F4A7C15ULL

static inline uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27; z *= 0x94D049BB133111EBULL;
    z ^= z >> 31; return z;
}

uint64_t synth_stream(uint64_t seed, uint32_t tensor, uint32_t layer) {
    return mix64(mix64(seed + GOLD) ^ (((uint64_t)tensor << 32) | (uint64_t)layer));
}

static inline uint64_t draw(uint64_t stream, uint64_t c) {
    return mix64(stream + (c + 1) * GOLD);
}

static inline int32_t field_sum(uint64_t r) {
    return (int32_t)(r & 0xFFFF) + (int32_t)((r >> 16) & 0xFFFF) +
           (int32_t)((r >> 32) & 0xFFFF) + (int32_t)(r >> 48);
}

static inline int32_t centred_sum(uint64_t stream, uint64_t i) {
    return field_sum(draw(stream, 2 * i)) + field_sum(draw(stream, 2 * i + 1)) - 262140;
}

/* fp32 constant that turns the centred integer sum into a sample of std `std`. */
float synth_constant(double std) {
    return (float)(std / (65536.0 * sqrt(8.0 / 12.0)));
}

static inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u; memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* out[i] = value of element first+i of the tensor, fp32 storage. */
void synth_fill_f32(float* out, uint64_t first, uint64_t n, uint64_t seed,
                    uint32_t tensor, uint32_t layer, float cst) {
    uint64_t s = synth_stream(seed, tensor, layer);
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i)
        out[i] = (float)centred_sum(s, first + (uint64_t)i) * cst;
}

/* Same values rounded once to bf16 (raw 16-bit patterns). */
void synth_fill_bf16(uint16_t* out, uint64_t first, uint64_t n, uint64_t seed,
                     uint32_t tensor, uint32_t layer, float cst) {
    uint64_t s = synth_stream(seed, tensor, layer);
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i)
        out[i] = f32_to_bf16_rne((float)centred_sum(s, first + (uint64_t)i) * cst);
}

/* Uniform in [0,1) with 53 bits from draw c of a stream. */
double synth_uniform(uint64_t seed, uint32_t tensor, uint32_t layer, uint64_t c) {
    return (double)(draw(synth_stream(seed, tensor, layer), c) >> 11) * (1.0 / 9007199254740992.0);
}

/* Per-sublayer output scale: log-uniform on [1e-3, 1]; index 2l = attention, 2l+1 = MLP. */
void synth_sublayer_scales(uint64_t seed, int32_t n_layers, double* out /*[2L]*/) {
    for (int32_t j = 0; j < 2 * n_layers; ++j)
        out[j] = pow(10.0, -3.0 * synth_uniform(seed, 101u, 0u, (uint64_t)j));
}

/* Uniform-random prompt token ids in [0, vocab). */
void synth_prompt(uint64_t seed, int32_t n, int32_t vocab, int32_t* out) {
    uint64_t s = synth_stream(seed, 100u, 0u);
    for (int32_t i = 0; i < n; ++i)
        out[i] = (int32_t)(draw(s, (uint64_t)i) % (uint64_t)vocab);
}
