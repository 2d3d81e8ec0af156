/* Seeded synthetic-input helpers (no cache logic, no embedding arithmetic).
 *
 * w0(seed, id, c) is a counter-based value in (-0.05, 0.05): any element of the
 * initial embedding table can be regenerated from its coordinates alone, so two
 * independent consumers can each build their own copy of the same table.
 * The Python module next to this file implements the same function in numpy;
 * the two are checked against each other in the CPU tests.
 */
#include <stdint.h>
#include <stddef.h>

static inline uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27; z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

static inline float w0(uint64_t seed, uint64_t id, uint64_t c) {
    uint64_t key = (seed + 1) * 0x9E3779B97F4A7C15ULL + id * 0xD1B54A32D192ED03ULL + c * 0x8CB92BA72F3D8DD7ULL;
    uint64_t bits = mix64(key) >> 40;               /* 24 bits */
    float u = (float)bits * (1.0f / 16777216.0f);   /* exact in fp32 */
    return (u - 0.5f) * 0.1f;
}

/* out[r*dim + c] = w0(seed, row_id[r], c) for r in [0, rows). row_id may be NULL (identity). */
void fc_fill_table(float* out, const int32_t* row_id, int64_t rows, int32_t dim, uint64_t seed) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        uint64_t id = row_id ? (uint64_t)row_id[r] : (uint64_t)r;
        float* o = out + (size_t)r * dim;
        for (int32_t c = 0; c < dim; ++c) o[c] = w0(seed, id, (uint64_t)c);
    }
}

/* Standard-normal-ish gradients from the same counter hash (Box-Muller on two 24-bit uniforms). */
#include <math.h>
void fc_fill_normal(float* out, int64_t count, uint64_t seed) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; i += 2) {
        uint64_t a = mix64((seed + 1) * 0x9E3779B97F4A7C15ULL + (uint64_t)i * 0xD1B54A32D192ED03ULL);
        double u1 = ((double)(a >> 40) + 0.5) * (1.0 / 16777216.0);
        double u2 = ((double)((a >> 16) & 0xFFFFFF) + 0.5) * (1.0 / 16777216.0);
        double rad = sqrt(-2.0 * log(u1));
        out[i] = (float)(rad * cos(6.283185307179586 * u2));
        if (i + 1 < count) out[i + 1] = (float)(rad * sin(6.283185307179586 * u2));
    }
}
