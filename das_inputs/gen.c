/*
 * Seeded synthetic input generators shared by the tests, the bench and the
 * oracle-vs-GPU parity harness.  This file holds NO arithmetic of the method
 * (no norm, projection, attention, acceptance): it only produces inputs --
 * random-init weights, synthetic KV contents and a bf16->f32 widening helper.
 *
 * Canonical weight blob (the "model file" both sides read; every matrix is
 * [out_features][in_features] row-major, bf16):
 *   embed[V][d]
 *   for each layer: g1[d] Wq[Hq*D][d] Wk[Hkv*D][d] Wv[Hkv*D][d] Wo[d][Hq*D]
 *                   g2[d] Wg[F][d] Wu[F][d] Wd[d][F]
 *   gf[d] Wlm[V][d]
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>
#include <omp.h>

static inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static inline uint16_t f32_to_bf16_rne(float f) {
    union { float f; uint32_t u; } c; c.f = f;
    uint32_t u = c.u;
    uint32_t r = 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)((u + r) >> 16);
}

/* standard normal from a 64-bit counter hash (Box-Muller, cosine branch) */
static inline double normal_from_bits(uint64_t h) {
    double u1 = ((double)(uint32_t)(h >> 32) + 1.0) * (1.0 / 4294967296.0); /* (0,1] */
    double u2 = (double)(uint32_t)h * (1.0 / 4294967296.0);
    return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
}

static void fill_normal(uint16_t *dst, size_t n, uint64_t seed, uint64_t tensor_id, double sigma) {
    const uint64_t base = mix64(mix64(seed ^ 0x5745494748545321ull) ^ tensor_id);
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i)
        dst[i] = f32_to_bf16_rne((float)(sigma * normal_from_bits(mix64(base ^ (uint64_t)i))));
}

static void fill_gain(uint16_t *dst, size_t n, uint64_t seed, uint64_t tensor_id, double gain_sigma) {
    const uint64_t base = mix64(mix64(seed ^ 0x4741494E53212121ull) ^ tensor_id);
    for (size_t i = 0; i < n; ++i)
        dst[i] = f32_to_bf16_rne((float)(1.0 + gain_sigma * normal_from_bits(mix64(base ^ (uint64_t)i))));
}

int64_t dasin_weight_count(int32_t L, int32_t d, int32_t Hq, int32_t Hkv, int32_t D, int32_t F, int32_t V) {
    int64_t per_layer = (int64_t)d + (int64_t)(Hq + 2 * Hkv) * D * d + (int64_t)d * Hq * D
                      + d + 3ll * F * d;
    return (int64_t)V * d + L * per_layer + d + (int64_t)V * d;
}

/* Fill the canonical blob: matrices ~ N(0, sigma^2), gains = 1 + N(0, gain_sigma^2). */
void dasin_weights_bf16(int32_t L, int32_t d, int32_t Hq, int32_t Hkv, int32_t D, int32_t F, int32_t V,
                        uint64_t seed, double sigma, double gain_sigma, uint16_t *out) {
    uint16_t *p = out;
    uint64_t id = 0;
    fill_normal(p, (size_t)V * d, seed, id++, sigma); p += (size_t)V * d;
    for (int l = 0; l < L; ++l) {
        fill_gain(p, d, seed, id++, gain_sigma); p += d;
        fill_normal(p, (size_t)Hq * D * d, seed, id++, sigma); p += (size_t)Hq * D * d;
        fill_normal(p, (size_t)Hkv * D * d, seed, id++, sigma); p += (size_t)Hkv * D * d;
        fill_normal(p, (size_t)Hkv * D * d, seed, id++, sigma); p += (size_t)Hkv * D * d;
        fill_normal(p, (size_t)d * Hq * D, seed, id++, sigma); p += (size_t)d * Hq * D;
        fill_gain(p, d, seed, id++, gain_sigma); p += d;
        fill_normal(p, (size_t)F * d, seed, id++, sigma); p += (size_t)F * d;
        fill_normal(p, (size_t)F * d, seed, id++, sigma); p += (size_t)F * d;
        fill_normal(p, (size_t)d * F, seed, id++, sigma); p += (size_t)d * F;
    }
    fill_gain(p, d, seed, id++, gain_sigma); p += d;
    fill_normal(p, (size_t)V * d, seed, id++, sigma);
}

void dasin_bf16_to_f32(const uint16_t *src, float *dst, int64_t n) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        union { float f; uint32_t u; } c; c.u = (uint32_t)src[i] << 16; dst[i] = c.f;
    }
}

void dasin_f32_to_bf16(const float *src, uint16_t *dst, int64_t n) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) dst[i] = f32_to_bf16_rne(src[i]);
}

/*
 * Synthetic KV contents, reproducible with integer operations only so that a
 * device-side filler can regenerate the same bits: element e of the
 * [token][kv_head][dim] tensor is the centred sum of the four 16-bit fields of
 * a 64-bit hash, scaled by 2^-15 (std ~= 1.155), rounded to bf16.
 *   which = 0 for K, 1 for V.
 */
void dasin_kv_synth(uint64_t seed, uint64_t seq_key, int32_t layer, int32_t which,
                    int64_t first_token, int64_t n_tokens, int32_t Hkv, int32_t D, uint16_t *out) {
    const uint64_t base = mix64(mix64(mix64(seed ^ 0x4B5653594E544821ull) ^ seq_key)
                                ^ ((uint64_t)layer * 2u + (uint64_t)which));
    const int64_t per_tok = (int64_t)Hkv * D;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n_tokens; ++t)
        for (int64_t e = 0; e < per_tok; ++e) {
            uint64_t h = mix64(base ^ (uint64_t)((first_token + t) * per_tok + e));
            int32_t s = (int32_t)(h & 0xFFFF) + (int32_t)((h >> 16) & 0xFFFF)
                      + (int32_t)((h >> 32) & 0xFFFF) + (int32_t)(h >> 48) - 131070;
            out[t * per_tok + e] = f32_to_bf16_rne((float)s * (1.0f / 32768.0f));
        }
}

/* uniform in [0,1) with 24 bits, keyed by (seed, seq, absolute position, stream) */
void dasin_uniforms(uint64_t seed, int64_t n, const int64_t *seq_key, const int64_t *pos, int32_t stream, float *out) {
    for (int64_t i = 0; i < n; ++i) {
        uint64_t h = mix64(mix64(mix64(mix64(seed ^ 0x554E49464F524D21ull) ^ (uint64_t)seq_key[i])
                                 ^ (uint64_t)pos[i]) ^ (uint64_t)stream);
        out[i] = (float)(h >> 40) * (1.0f / 16777216.0f);
    }
}

int32_t dasin_num_threads(void) { return omp_get_max_threads(); }
